"""Plain CPU oracle for one worker's Kimad+ compression step.

TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute;
it is deliberately slow and literal.  Only the test-suite, the smoke check and
the benchmark's ``cpu_baseline`` leg may import it.  It shares no code with the
HIP path and imports nothing from the product package.

What is computed, per training round, for one worker (Kimad paper, Algorithm 1,
worker lines "Select compressor" and "Upload the compressed vector"; Section 3.2):

    x_i       = u_i - u_hat_i                          the vector that is compressed
    K_ij      = candidate sizes from the ratio grid    (Section 3.2, the discrete set)
    E_ij      = || x_i - TopK_{K_ij}(x_i) ||^2         (Section 3.2, Eq. norm decomposition)
    j_i       = argmin sum_i E_{i j_i}  s.t.  sum_i b_{i j_i} <= c   (Eq. optimisation; Appendix C)
    payload_i = (index, value) pairs of TopK_{K_i}(x_i)            (Algorithm 1, upload line)
    u_hat_i  += TopK_{K_i}(x_i)                        (Section 3.3, Eq. EF21-2; Algorithm 1, aggregate line)

In the code below g = u (fresh update), h = u_hat (estimator), x = g - h.

And, per round, for the server (Algorithm 1, server lines "Aggregate all update estimators"
and "Updates the model"):

    u_hat_m  += C_m(u_m - u_hat_m)                     decode worker m's payload into its estimator
    x_model  -= gamma * sum_m w_m u_hat_m              model step from the M estimators

Parts that are plain definitions (written out as such): the operand, TopK by a
full sort, the error as the sum of squares of what TopK drops, the payload and
the estimator update.  The part that is an algorithm (followed step by step, in
the paper's order): the knapsack dynamic programme of Appendix C.

Readings taken where the paper is silent or inconsistent (each also listed in
the design notes of this repository):
  R1  "K largest absolute values" (Section 2.2): magnitudes are compared by the
      IEEE-754 bit pattern with the sign cleared, as an unsigned integer; equal
      magnitudes are kept in order of lower index first.
  R2  Ratio -> size: K = ceil(r * d_i) in fp64, clamped to [1, d_i]
      (Omega = {TopK | K > 0}, Section 4.2).
  R3  Size of a compressed layer (the Costs matrix of Appendix C): K * pair_bytes,
      pair_bytes = 8 for a u32 index plus an fp32 value.
  R4  The error is the squared l2 norm of Eq. norm decomposition, in fp64, not
      discretised; measured on x (equal to ||u_hat_new - u||^2 in exact arithmetic).
  R5  Appendix C indexes its table by cost and stores the least error; the
      undefined index e_i of its inner update is read as cost_i.  The
      discretisation factor D divides the budget: unit = ceil(P / D) pairs with
      P = floor(c / pair_bytes); costs round up to units, capacity rounds down,
      so the result never exceeds the budget.  D = 0 means unit = 1 pair (exact).
  R6  The first layer is treated like every other one, starting from a virtual
      row that is 0 at cost 0 and +inf elsewhere (the listing's separate first-
      layer loop would let a worse candidate overwrite a better one).
  R7  Ties: strict "<" while candidates are visited in ascending j keeps the
      lowest j; the final argmin takes the smallest cost among equal minima.
  R8  A budget below the cheapest allocation is reported as INFEASIBLE; a table
      with a non-finite entry as NONFINITE.
  R9  Payload layout: per layer, pairs in ascending layer-local index; layer i
      occupies [offsets[i], offsets[i+1]) with offsets the exclusive scan of K.
  R13 Server model step: the paper fixes no precision.  The weighted sum over
      workers is taken in fp64, workers in order m = 0..M-1, each term the fp64
      product w_m * u_hat_m; the model is fp32 and gets fl32(x - gamma * sum),
      the subtraction and the product with gamma in fp64.

  R14 Budget rule (Section 3.1, Eq. budget): the paper prints c = B (t - T_comp) / 2, which is
      its time split t = c/B + T_comp + alpha c/B solved for c at alpha = 1; for another alpha the
      same equation gives c = B (t - T_comp) / (1 + alpha).  B in bits per second, c in bits;
      the byte budget is floor(c / 8); a step with t <= T_comp has no budget.

  R15 Dense fallback (Section 4.2, "Communication adaptivity": the sent size levels off at the
      uncompressed size).  A layer never costs more than its bare values: K pairs cost
      min(K * pair_bytes, n * value_bytes) bytes.  A grid point at or beyond the break-even
      (K * pair_bytes >= n * value_bytes) therefore stands for sending the layer whole: K = n,
      error 0, charged ceil(n * value_bytes / pair_bytes) pairs.  Optional (`dense_sizes`).
  R16 Half-precision values (Section 2.2 names quantisation beside sparsification; a 6-byte pair).
      A kept value v travels as binary16, round to nearest even, saturated to +-65504, NaN kept;
      worker and server both add the decoded value: h[idx] = fl32(h[idx] + fl32(q16(v))), so the
      two estimator copies stay equal and what the rounding lost stays in g - h for the next
      round.  The error table remains that of TopK (the rounding of kept values is not charged).

Pins (tests/test_oracle_*.py): brute force over all subsets / all assignments on
tiny inputs, closed forms for constant vectors, numpy partition on distinct
magnitudes, the contraction bound of the paper's compressor class, monotonicity,
the worker/server estimator round trip; for the server step, exact rational
arithmetic on tiny inputs and closed forms.  No function here is unpinned.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np

OK = 0
ERR_INFEASIBLE = -6
ERR_NONFINITE = -7


# --------------------------------------------------------------------------- operand / order

def operand(g: np.ndarray, h: np.ndarray) -> np.ndarray:
    """x = fl32(g - h): the vector handed to the compressor (Algorithm 1, upload line)."""
    g = np.asarray(g, dtype=np.float32)
    h = np.asarray(h, dtype=np.float32)
    return np.subtract(g, h, dtype=np.float32)


def magnitude_key(x: np.ndarray) -> np.ndarray:
    """|x| as an unsigned integer: the binary32 pattern with the sign bit cleared (reading R1)."""
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) & np.uint32(0x7FFFFFFF)


def magnitude_order(x: np.ndarray) -> np.ndarray:
    """Indices of x sorted by magnitude descending, equal magnitudes by index ascending."""
    key = magnitude_key(x).astype(np.int64)
    # A stable sort of the negated key keeps equal keys in index order.
    return np.argsort(-key, kind="stable")


# --------------------------------------------------------------------------- grid

def grid_sizes(ratios: Sequence[float], n: int) -> np.ndarray:
    """K_j = min(n, max(1, ceil(r_j * n))) for every grid ratio (reading R2)."""
    out = np.empty(len(ratios), dtype=np.int64)
    for j, r in enumerate(ratios):
        k = int(math.ceil(float(r) * float(n)))
        out[j] = min(int(n), max(1, k))
    return out


# --------------------------------------------------------------------------- TopK, error, payload, EF

def topk_support(x: np.ndarray, K: int) -> np.ndarray:
    """The K positions TopK keeps (Section 2.2), as the first K entries of the magnitude order."""
    return magnitude_order(x)[:K]


def topk_error_profile(x: np.ndarray, Ks: Sequence[int]) -> np.ndarray:
    """E(K) = sum of squares of the entries TopK_K drops, for each K (Section 3.2, Eq. norm decomposition).

    Squares are taken and added in fp64, from the smallest magnitude upward.  E(n) is exactly 0.
    """
    n = x.shape[0]
    pi = magnitude_order(x)
    sq = x[pi[::-1]].astype(np.float64) ** 2          # smallest magnitude first
    running = np.cumsum(sq)                            # running[m-1] = sum of the m smallest squares
    out = np.empty(len(Ks), dtype=np.float64)
    for j, K in enumerate(Ks):
        dropped = n - int(K)
        out[j] = 0.0 if dropped == 0 else running[dropped - 1]
    return out


def profile(g_layers: Sequence[np.ndarray], h_layers: Sequence[np.ndarray],
            ratios: Sequence[float]) -> Tuple[np.ndarray, np.ndarray]:
    """The Errors matrix of Appendix C (L x J, fp64) and the matching sizes K_ij (L x J)."""
    L, J = len(g_layers), len(ratios)
    E = np.empty((L, J), dtype=np.float64)
    Kt = np.empty((L, J), dtype=np.int64)
    for i in range(L):
        x = operand(g_layers[i], h_layers[i])
        Kt[i] = grid_sizes(ratios, x.shape[0])
        E[i] = topk_error_profile(x, Kt[i])
    return E, Kt


def quantise_f16(v: np.ndarray) -> np.ndarray:
    """binary16 bit patterns of fp32 values: round to nearest even, saturated to +-65504, NaN kept (reading R16)."""
    v = np.asarray(v, dtype=np.float32)
    with np.errstate(invalid="ignore", over="ignore"):
        clipped = np.clip(v, np.float32(-65504.0), np.float32(65504.0))      # (NaN passes through a clip)
        return clipped.astype(np.float16).view(np.uint16)


def dequantise_f16(bits: np.ndarray) -> np.ndarray:
    """fp32 values of binary16 bit patterns (exact)."""
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float32)


def compress_ef_layer(g: np.ndarray, h: np.ndarray, K: int, value_format: str = "f32"):
    """One layer: payload (ascending index, value) of TopK_K(g - h), and the updated estimator.

    h_new[t] = fl32(h[t] + c[t]) on the support, h[t] elsewhere (Section 3.3, Eq. EF21-2), where c is what the
    receiver decodes: x itself for fp32 values, fl32(q16(x)) for half-precision values (reading R16; the
    returned values are then uint16 bit patterns).
    """
    x = operand(g, h)
    idx = np.sort(topk_support(x, int(K))).astype(np.uint32)
    val = x[idx]
    h_new = np.array(h, dtype=np.float32, copy=True)
    if value_format == "f16":
        bits = quantise_f16(val)
        h_new[idx] = np.add(h_new[idx], dequantise_f16(bits), dtype=np.float32)
        return idx, bits, h_new
    assert value_format == "f32"
    h_new[idx] = np.add(h_new[idx], val, dtype=np.float32)
    return idx, val, h_new


def compress_ef(g_layers: Sequence[np.ndarray], h_layers: Sequence[np.ndarray],
                K: Sequence[int]):
    """All layers: (offsets[L+1], idx[sum K], val[sum K], list of updated h)."""
    L = len(g_layers)
    offsets = np.zeros(L + 1, dtype=np.uint64)
    for i in range(L):
        offsets[i + 1] = offsets[i] + np.uint64(int(K[i]))
    total = int(offsets[L])
    idx = np.empty(total, dtype=np.uint32)
    val = np.empty(total, dtype=np.float32)
    h_out: List[np.ndarray] = []
    for i in range(L):
        a, b = int(offsets[i]), int(offsets[i + 1])
        idx[a:b], val[a:b], hn = compress_ef_layer(g_layers[i], h_layers[i], int(K[i]))
        h_out.append(hn)
    return offsets, idx, val, h_out


# --------------------------------------------------------------------------- allocation (Appendix C)

def cost_units(K_table: np.ndarray, budget_bytes: int, pair_bytes: int, D: int):
    """Budget and candidate sizes in knapsack units (reading R5): returns (unit, capacity, w_ij)."""
    P = int(budget_bytes) // int(pair_bytes)
    unit = 1 if (D == 0 or P <= D) else -(-P // int(D))
    cap = P // unit
    w = -(-np.asarray(K_table, dtype=np.int64) // unit)
    return unit, cap, w


def dense_view(E: np.ndarray, K_table: np.ndarray, sizes: Sequence[int], pair_bytes: int, value_bytes: int = 4):
    """The tables as the allocation sees them with the dense fallback (reading R15): per grid point the error,
    the pairs charged and the size actually sent.  A point with K * pair_bytes >= n * value_bytes becomes
    (error 0, ceil(n * value_bytes / pair_bytes) pairs charged, K = n sent)."""
    E = np.asarray(E, dtype=np.float64)
    K_table = np.asarray(K_table, dtype=np.int64)
    n = np.asarray(sizes, dtype=np.int64)[:, None]
    dense = K_table * int(pair_bytes) >= n * int(value_bytes)
    dense_pairs = -(-(n * int(value_bytes)) // int(pair_bytes))
    return (np.where(dense, 0.0, E), np.where(dense, dense_pairs, K_table), np.where(dense, n, K_table))


def allocate(E: np.ndarray, K_table: np.ndarray, budget_bytes: int,
             pair_bytes: int = 8, D: int = 0, dense_sizes: Sequence[int] = None):
    """Knapsack dynamic programme of Appendix C with readings R5-R8.

    Returns (status, j[L], K[L], offsets[L+1]).  On a non-zero status the arrays are empty.
    `dense_sizes` (the layers' element counts) switches the dense fallback of reading R15 on: the
    programme then runs on `dense_view` of the tables and K is the size actually sent.
    """
    E = np.asarray(E, dtype=np.float64)
    K_table = np.asarray(K_table, dtype=np.int64)
    K_sent = K_table
    if dense_sizes is not None:
        E, K_table, K_sent = dense_view(E, K_table, dense_sizes, pair_bytes)
    L, J = E.shape
    empty = (np.empty(0, np.int32), np.empty(0, np.uint64), np.empty(0, np.uint64))
    if not np.all(np.isfinite(E)):
        return (ERR_NONFINITE,) + empty
    unit, cap, w = cost_units(K_table, budget_bytes, pair_bytes, D)

    inf = np.inf
    prev = np.full(cap + 1, inf, dtype=np.float64)       # DP row of the layers seen so far
    prev[0] = 0.0
    choice = np.full((L, cap + 1), -1, dtype=np.int32)   # the PD matrix of the listing
    for i in range(L):
        cur = np.full(cap + 1, inf, dtype=np.float64)
        for j in range(J):
            wij = int(w[i, j])
            if wij > cap:
                continue
            # for cost = wij .. cap:  t = DP[i-1][cost - wij] + Errors[i][j];  if t < DP[i][cost]: take it
            t = prev[0:cap + 1 - wij] + E[i, j]
            better = t < cur[wij:]
            cur[wij:][better] = t[better]
            choice[i, wij:][better] = j
        prev = cur

    best = prev.min()
    if not np.isfinite(best):
        return (ERR_INFEASIBLE,) + empty
    c = int(np.argmax(prev == best))                      # smallest cost attaining the minimum
    j_out = np.empty(L, dtype=np.int32)
    for i in range(L - 1, -1, -1):
        j_out[i] = choice[i, c]
        c -= int(w[i, j_out[i]])
    K_out = K_sent[np.arange(L), j_out].astype(np.uint64)
    offsets = np.zeros(L + 1, dtype=np.uint64)
    np.cumsum(K_out, out=offsets[1:])
    return OK, j_out, K_out, offsets


# --------------------------------------------------------------------------- whole step

def step(g_layers, h_layers, ratios, budget_bytes, pair_bytes: int = 8, D: int = 0):
    """profile -> allocate -> compress with error feedback, as one worker does once per round."""
    E, Kt = profile(g_layers, h_layers, ratios)
    status, j, K, offsets = allocate(E, Kt, budget_bytes, pair_bytes, D)
    if status != OK:
        return dict(status=status, E=E, K_table=Kt)
    offsets2, idx, val, h_new = compress_ef(g_layers, h_layers, K)
    assert np.array_equal(offsets, offsets2)
    return dict(status=OK, E=E, K_table=Kt, j=j, K=K, offsets=offsets, idx=idx, val=val, h=h_new)


# --------------------------------------------------------------------------- server side
def server_apply(payloads, u_hats: Sequence[np.ndarray], weights: Sequence[float], x_model,
                 gamma: float, layer_starts: Sequence[int]):
    """Algorithm 1, server lines "Aggregate all update estimators" and "Updates the model".

    payloads[m] = (offsets, idx, val) of worker m as produced by `compress_ef` (layer-local
    indices); u_hats[m] is the server's flat fp32 copy of worker m's estimator, layer i at
    [layer_starts[i], layer_starts[i+1]).  Returns (new u_hats, new model); `x_model` may be None
    (aggregate only).  Decoding adds each value to its entry in fp32, which is exactly what the
    worker did to its own estimator; the model step follows reading R13."""
    M = len(u_hats)
    assert len(payloads) == M and len(weights) == M
    L = len(layer_starts) - 1
    new_hats = []
    for m in range(M):
        offsets, idx, val = payloads[m]
        u = np.array(u_hats[m], dtype=np.float32, copy=True)
        for i in range(L):
            a, b = int(offsets[i]), int(offsets[i + 1])
            where = int(layer_starts[i]) + idx[a:b].astype(np.int64)
            v = dequantise_f16(val[a:b]) if val.dtype == np.uint16 else val[a:b].astype(np.float32)   # reading R16
            u[where] = u[where] + v                                  # fp32 add; indices of a layer are distinct
        new_hats.append(u)
    if x_model is None:
        return new_hats, None
    acc = np.zeros(len(x_model), dtype=np.float64)
    for m in range(M):
        acc = acc + np.float64(weights[m]) * new_hats[m].astype(np.float64)
    x_new = (np.asarray(x_model, dtype=np.float32).astype(np.float64) - np.float64(gamma) * acc).astype(np.float32)
    return new_hats, x_new


# --------------------------------------------------------------------------- baseline allocators (Section 4.3)
def uniform_sizes(sizes: Sequence[int], budget_bytes: int, pair_bytes: int = 8) -> np.ndarray:
    """Kimad without the layer-wise allocation (Section 4.3): one ratio rho = P / d for every layer,
    K_i = ceil(rho * d_i) clamped to [1, d_i] as for any grid ratio (reading R2); rho is capped at 1."""
    d = int(sum(int(n) for n in sizes))
    P = int(budget_bytes) // int(pair_bytes)
    rho = min(1.0, P / d)
    return np.array([int(grid_sizes([rho], int(n))[0]) for n in sizes], dtype=np.int64)


def whole_model_sizes(g_layers, h_layers, budget_bytes: int, pair_bytes: int = 8) -> np.ndarray:
    """TopK over the whole model (the paper's "optimal baseline ... with the whole model information"):
    the P = min(floor(budget / pair_bytes), d) entries of largest magnitude of the concatenation, equal
    magnitudes by lower position; returned as the number kept in every layer.  Within a layer the kept
    entries are its own TopK of that size, so its error is `topk_error_profile` at that size."""
    x = np.concatenate([operand(g, h) for g, h in zip(g_layers, h_layers)])
    P = min(int(budget_bytes) // int(pair_bytes), x.shape[0])
    kept = np.zeros(x.shape[0], dtype=bool)
    kept[magnitude_order(x)[:P]] = True
    out, pos = [], 0
    for g in g_layers:
        out.append(int(kept[pos:pos + len(g)].sum()))
        pos += len(g)
    return np.array(out, dtype=np.int64)


def errors_at(g_layers, h_layers, K: Sequence[int]) -> np.ndarray:
    """Per-layer error of TopK at the given sizes (Section 3.2, Eq. norm decomposition), any 0 <= K_i <= d_i."""
    return np.array([topk_error_profile(operand(g, h), [int(k)])[0] for g, h, k in zip(g_layers, h_layers, K)])


def budget_bytes(bandwidth_bits_per_s: float, t: float, t_comp: float, alpha: float = 1.0,
                 cap_bytes: int = 0) -> int:
    """Compression budget of one round (Section 3.1, Eq. budget; reading R14): the bytes that fit
    into the up-link share of the time budget t at the monitored bandwidth.  cap_bytes > 0 limits
    the result (the uncompressed size: the plateau of the communication-size figure, Section 4.2)."""
    B, t, t_comp, alpha = float(bandwidth_bits_per_s), float(t), float(t_comp), float(alpha)
    if not (B > 0.0) or not (t > t_comp) or not (alpha >= 0.0) or B == np.inf or t == np.inf:
        return 0
    c_bits = B * (t - t_comp) / (1.0 + alpha)
    nbytes = int(np.floor(c_bits / 8.0))
    if cap_bytes > 0:
        nbytes = min(nbytes, int(cap_bytes))
    return nbytes
