"""ctypes binding with the names of include/kimad.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkimad.so")

KIMAD_REUSE_PROFILE = 1
KIMAD_CFG_CLASSIC_PROFILE = 1
KIMAD_CFG_FULL_DP = 2
KIMAD_CFG_BAND_DP = 4
KIMAD_CFG_DENSE_FALLBACK = 8
KIMAD_CFG_SAMPLE_ALWAYS = 16
KIMAD_VALUES_F32 = 0
KIMAD_VALUES_F16 = 1
KIMAD_MAX_J = 64

EXPORTED_SYMBOLS = [
    "kimad_workspace_bytes", "kimad_plan_create", "kimad_plan_destroy", "kimad_plan_grid_sizes",
    "kimad_profile", "kimad_allocate", "kimad_allocate_static", "kimad_compress_ef", "kimad_step",
    "kimad_error_at", "kimad_uniform_sizes", "kimad_payload_layer_counts",
    "kimad_profile_diagnostics", "kimad_allocate_diagnostics", "kimad_plan_layer_states", "kimad_plan_set_timing", "kimad_plan_get_timings",
    "kimad_server_apply", "kimad_selftest_wave_primitives", "kimad_budget_bytes", "kimad_strerror", "kimad_version",
]


class KimadError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {kimad_strerror(code)} ({code})")


class _Layer(C.Structure):
    _fields_ = [("g", C.c_void_p), ("h", C.c_void_p), ("n", C.c_uint64)]


class _Payload(C.Structure):
    _fields_ = [("idx", C.c_void_p), ("val", C.c_void_p), ("offsets", C.c_void_p), ("capacity_pairs", C.c_uint64),
                ("value_format", C.c_uint32), ("pad", C.c_uint32)]


class _Config(C.Structure):
    _fields_ = [("pair_bytes", C.c_uint32), ("cost_units_D", C.c_uint32),
                ("max_budget_bytes", C.c_uint64), ("flags", C.c_uint64),
                ("max_workgroups", C.c_uint32), ("value_format", C.c_uint32)]


_lib = None


def lib() -> C.CDLL:
    """Load libkimad.so (built by paper_2312_08053_amd.build).  Fails loudly when it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: run `python -m paper_2312_08053_amd.build` (there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, u32, u64, i32p = C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p
    L.kimad_workspace_bytes.argtypes = [C.POINTER(C.c_uint64), u32, u32, C.POINTER(_Config), C.POINTER(C.c_uint64)]
    L.kimad_plan_create.argtypes = [C.POINTER(_Layer), u32, C.POINTER(C.c_double), u32, C.POINTER(_Config),
                                    vp, u64, vp, C.POINTER(vp)]
    L.kimad_plan_destroy.argtypes = [vp]
    L.kimad_plan_grid_sizes.argtypes = [vp, C.POINTER(C.c_uint64)]
    L.kimad_profile.argtypes = [vp, vp, u64, vp]
    L.kimad_allocate.argtypes = [vp, vp, u64, vp, vp, vp, i32p, vp]
    L.kimad_allocate_static.argtypes = [vp, vp, u64, vp, vp, vp, i32p, vp]
    L.kimad_compress_ef.argtypes = [vp, vp, vp, vp, vp, u64, u32, i32p, vp]
    L.kimad_step.argtypes = [vp, u64, vp, vp, vp, vp, vp, vp, u64, i32p, vp]
    L.kimad_error_at.argtypes = [vp, vp, vp, vp]
    L.kimad_uniform_sizes.argtypes = [C.POINTER(C.c_uint64), u32, u64, u32, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
    L.kimad_payload_layer_counts.argtypes = [vp, u64, vp, u32, vp, vp]
    L.kimad_profile_diagnostics.argtypes = [vp, C.POINTER(C.c_uint32), vp]
    L.kimad_allocate_diagnostics.argtypes = [vp, C.POINTER(C.c_uint32), vp]
    L.kimad_plan_layer_states.argtypes = [vp, C.POINTER(C.c_uint32), u32, C.POINTER(C.c_uint32), vp]
    L.kimad_plan_set_timing.argtypes = [vp, C.c_int]
    L.kimad_plan_get_timings.argtypes = [vp, C.c_char_p, u32, C.POINTER(C.c_float), u32, C.POINTER(C.c_uint32)]
    L.kimad_server_apply.argtypes = [C.POINTER(_Payload), C.POINTER(C.c_void_p), C.POINTER(C.c_double), u32, vp, u32, u64,
                                     vp, C.c_double, vp, vp]
    L.kimad_selftest_wave_primitives.argtypes = [vp, vp, vp, vp, vp]
    L.kimad_strerror.argtypes = [C.c_int]
    L.kimad_strerror.restype = C.c_char_p
    L.kimad_version.restype = C.c_char_p
    for name in EXPORTED_SYMBOLS:
        if name not in ("kimad_strerror", "kimad_version", "kimad_budget_bytes"):
            getattr(L, name).restype = C.c_int
    L.kimad_budget_bytes.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double, C.c_uint64]
    L.kimad_budget_bytes.restype = C.c_uint64
    _lib = L
    return L


def kimad_strerror(code: int) -> str:
    return lib().kimad_strerror(int(code)).decode()


def kimad_budget_bytes(bandwidth_bits_per_s: float, t_seconds: float, t_comp_seconds: float, alpha: float = 1.0,
                       cap_bytes: int = 0) -> int:
    return int(lib().kimad_budget_bytes(float(bandwidth_bits_per_s), float(t_seconds), float(t_comp_seconds),
                                        float(alpha), int(cap_bytes)))


def kimad_version() -> str:
    return lib().kimad_version().decode()


def _cfg(pair_bytes=8, D=0, max_budget_bytes=0, cfg_flags=0, max_workgroups=0, value_format=0) -> _Config:
    return _Config(int(pair_bytes), int(D), int(max_budget_bytes), int(cfg_flags), int(max_workgroups), int(value_format))


def _check(code: int, where: str) -> None:
    if code != 0:
        raise KimadError(code, where)


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    return int(getattr(stream, "cuda_stream", stream))


def kimad_workspace_bytes(sizes: Sequence[int], J: int, pair_bytes=8, D=0, max_budget_bytes=0,
                          cfg_flags=0, max_workgroups=0, value_format=0) -> int:
    n = (C.c_uint64 * len(sizes))(*[int(s) for s in sizes])
    out = C.c_uint64(0)
    cfg = _cfg(pair_bytes, D, max_budget_bytes, cfg_flags, max_workgroups, value_format)
    _check(lib().kimad_workspace_bytes(n, len(sizes), int(J), C.byref(cfg), C.byref(out)), "kimad_workspace_bytes")
    return int(out.value)


def kimad_plan_create(g_ptrs: Sequence[int], h_ptrs: Sequence[int], sizes: Sequence[int], ratios: Sequence[float],
                      workspace_ptr: int, workspace_bytes: int, stream=None, pair_bytes=8, D=0,
                      max_budget_bytes=0, cfg_flags=0, max_workgroups=0, value_format=0) -> int:
    L = len(sizes)
    layers = (_Layer * L)()
    for i in range(L):
        layers[i].g, layers[i].h, layers[i].n = int(g_ptrs[i]), int(h_ptrs[i]), int(sizes[i])
    r = (C.c_double * len(ratios))(*[float(x) for x in ratios])
    cfg = _cfg(pair_bytes, D, max_budget_bytes, cfg_flags, max_workgroups, value_format)
    plan = C.c_void_p(0)
    _check(lib().kimad_plan_create(layers, L, r, len(ratios), C.byref(cfg), C.c_void_p(int(workspace_ptr)),
                                   int(workspace_bytes), C.c_void_p(_stream(stream)), C.byref(plan)),
           "kimad_plan_create")
    return int(plan.value)


def kimad_plan_destroy(plan: int) -> None:
    _check(lib().kimad_plan_destroy(C.c_void_p(plan)), "kimad_plan_destroy")


def kimad_profile(plan: int, err_table, budget_hint_bytes: int = 0, stream=None) -> None:
    _check(lib().kimad_profile(C.c_void_p(plan), C.c_void_p(_ptr(err_table)), int(budget_hint_bytes),
                               C.c_void_p(_stream(stream))), "kimad_profile")


def kimad_allocate(plan: int, err_table, budget_bytes: int, j_out, K_out, offsets_out, status_out,
                   stream=None) -> None:
    _check(lib().kimad_allocate(C.c_void_p(plan), C.c_void_p(_ptr(err_table)), int(budget_bytes),
                                C.c_void_p(_ptr(j_out)), C.c_void_p(_ptr(K_out)), C.c_void_p(_ptr(offsets_out)),
                                C.c_void_p(_ptr(status_out)), C.c_void_p(_stream(stream))), "kimad_allocate")


def kimad_allocate_static(plan: int, err_table, budget_bytes: int, j_out, K_out, offsets_out, status_out,
                          stream=None) -> None:
    _check(lib().kimad_allocate_static(C.c_void_p(plan), C.c_void_p(_ptr(err_table)), int(budget_bytes),
                                       C.c_void_p(_ptr(j_out)), C.c_void_p(_ptr(K_out)), C.c_void_p(_ptr(offsets_out)),
                                       C.c_void_p(_ptr(status_out)), C.c_void_p(_stream(stream))), "kimad_allocate_static")


def kimad_compress_ef(plan: int, K, offsets, idx_out, val_out, capacity_pairs: int, flags: int, status_out,
                      stream=None) -> None:
    _check(lib().kimad_compress_ef(C.c_void_p(plan), C.c_void_p(_ptr(K)), C.c_void_p(_ptr(offsets)),
                                   C.c_void_p(_ptr(idx_out)), C.c_void_p(_ptr(val_out)), int(capacity_pairs),
                                   int(flags), C.c_void_p(_ptr(status_out)), C.c_void_p(_stream(stream))),
           "kimad_compress_ef")


def kimad_step(plan: int, budget_bytes: int, err_table, j_out, K_out, offsets_out, idx_out, val_out,
               capacity_pairs: int, status_out, stream=None) -> None:
    _check(lib().kimad_step(C.c_void_p(plan), int(budget_bytes), C.c_void_p(_ptr(err_table)),
                            C.c_void_p(_ptr(j_out)), C.c_void_p(_ptr(K_out)), C.c_void_p(_ptr(offsets_out)),
                            C.c_void_p(_ptr(idx_out)), C.c_void_p(_ptr(val_out)), int(capacity_pairs),
                            C.c_void_p(_ptr(status_out)), C.c_void_p(_stream(stream))), "kimad_step")


def kimad_error_at(plan: int, K, err_out, stream=None) -> None:
    _check(lib().kimad_error_at(C.c_void_p(plan), C.c_void_p(_ptr(K)), C.c_void_p(_ptr(err_out)),
                                C.c_void_p(_stream(stream))), "kimad_error_at")


def kimad_uniform_sizes(sizes: Sequence[int], budget_bytes: int, pair_bytes: int = 8):
    """([K_i], pairs of the whole-model TopK of the same budget): host arithmetic of the library."""
    L = len(sizes)
    n = (C.c_uint64 * L)(*[int(s) for s in sizes])
    out = (C.c_uint64 * L)()
    pairs = C.c_uint64(0)
    _check(lib().kimad_uniform_sizes(n, L, int(budget_bytes), int(pair_bytes), out, C.byref(pairs)), "kimad_uniform_sizes")
    return [int(v) for v in out], int(pairs.value)


def kimad_payload_layer_counts(idx, pairs: int, layer_start, counts_out, stream=None) -> None:
    _check(lib().kimad_payload_layer_counts(C.c_void_p(_ptr(idx)), int(pairs), C.c_void_p(_ptr(layer_start)),
                                            int(layer_start.numel()) - 1, C.c_void_p(_ptr(counts_out)),
                                            C.c_void_p(_stream(stream))), "kimad_payload_layer_counts")


def kimad_server_apply(payloads, u_hats, weights, layer_start, d: int, x=None, gamma: float = 0.0, stream=None,
                       status_out=None):
    """payloads: list of (idx, val, offsets) device tensors, one per worker; u_hats: list of flat fp32
    device tensors (updated in place); layer_start: device uint64/int64 tensor [L+1]; x: flat fp32 model
    or None; status_out: device int32[M] (allocated here if None).  Returns status_out."""
    M = len(u_hats)
    def cap(i, v):
        return 0 if i is None or v is None else min(int(i.numel()), int(v.numel()))

    def fmt(v):                                           # half-precision payloads are torch.float16 tensors
        return KIMAD_VALUES_F16 if v is not None and v.element_size() == 2 else KIMAD_VALUES_F32
    pl = (_Payload * M)(*[_Payload(_ptr(i), _ptr(v), _ptr(o), cap(i, v), fmt(v), 0) for (i, v, o) in payloads])
    uh = (C.c_void_p * M)(*[_ptr(u) for u in u_hats])
    w = (C.c_double * M)(*[float(t) for t in weights])
    if status_out is None:
        import torch
        status_out = torch.empty(M, dtype=torch.int32, device=u_hats[0].device)
    _check(lib().kimad_server_apply(pl, uh, w, M, C.c_void_p(_ptr(layer_start)), int(layer_start.numel()) - 1, int(d),
                                    C.c_void_p(_ptr(x) if x is not None else 0), float(gamma),
                                    C.c_void_p(_ptr(status_out)), C.c_void_p(_stream(stream))), "kimad_server_apply")
    return status_out


def kimad_selftest_wave_primitives(in_u32, in_f64, out_u32, out_f64, stream=None) -> None:
    _check(lib().kimad_selftest_wave_primitives(C.c_void_p(_ptr(in_u32)), C.c_void_p(_ptr(in_f64)), C.c_void_p(_ptr(out_u32)),
                                                C.c_void_p(_ptr(out_f64)), C.c_void_p(_stream(stream))),
           "kimad_selftest_wave_primitives")


class Plan:
    """Owns the torch tensors a plan needs (workspace, outputs) and forwards to the C calls.

    ``g`` and ``h`` are flat fp32 CUDA tensors holding the layers back to back in the order of
    ``sizes`` (or lists of per-layer tensors).
    """

    def __init__(self, g, h, sizes: Sequence[int], ratios: Sequence[float], pair_bytes: int = 0, D: int = 0,
                 max_budget_bytes: int = 0, cfg_flags: int = 0, capacity_pairs: Optional[int] = None,
                 max_workgroups: int = 0, value_format: int = 0):
        import torch
        self.torch = torch
        self.sizes = [int(s) for s in sizes]
        self.L, self.J = len(self.sizes), len(ratios)
        self.ratios = [float(r) for r in ratios]
        if isinstance(g, (list, tuple)):
            g_ptrs = [int(t.data_ptr()) for t in g]
            h_ptrs = [int(t.data_ptr()) for t in h]
            dev = g[0].device
        else:
            starts = np.concatenate([[0], np.cumsum(self.sizes)])
            g_ptrs = [int(g.data_ptr()) + 4 * int(s) for s in starts[:-1]]
            h_ptrs = [int(h.data_ptr()) + 4 * int(s) for s in starts[:-1]]
            dev = g.device
        self._keep = (g, h)
        self.device = dev
        self.value_format = int(value_format)
        self.pair_bytes = int(pair_bytes) if pair_bytes else (6 if value_format == KIMAD_VALUES_F16 else 8)
        nbytes = kimad_workspace_bytes(self.sizes, self.J, pair_bytes, D, max_budget_bytes, cfg_flags, max_workgroups,
                                       value_format)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        base = int(self.workspace.data_ptr())
        self._ws_ptr = (base + 255) // 256 * 256
        self.workspace_bytes = nbytes
        self.handle = kimad_plan_create(g_ptrs, h_ptrs, self.sizes, self.ratios, self._ws_ptr, nbytes,
                                        None, pair_bytes, D, max_budget_bytes, cfg_flags, max_workgroups, value_format)
        d = int(sum(self.sizes))
        self.capacity_pairs = int(capacity_pairs) if capacity_pairs is not None else d
        self.err_table = torch.empty(self.L * self.J, dtype=torch.float64, device=dev)
        self.j = torch.empty(self.L, dtype=torch.int32, device=dev)
        self.K = torch.empty(self.L, dtype=torch.int64, device=dev)
        self.offsets = torch.empty(self.L + 1, dtype=torch.int64, device=dev)
        self.status = torch.zeros(2, dtype=torch.int32, device=dev)
        self.idx = torch.empty(self.capacity_pairs, dtype=torch.int32, device=dev)
        self.val = torch.empty(self.capacity_pairs, device=dev,
                               dtype=torch.float16 if value_format == KIMAD_VALUES_F16 else torch.float32)

    def grid_sizes(self) -> np.ndarray:
        out = (C.c_uint64 * (self.L * self.J))()
        _check(lib().kimad_plan_grid_sizes(C.c_void_p(self.handle), out), "kimad_plan_grid_sizes")
        return np.array(out[:], dtype=np.int64).reshape(self.L, self.J)

    def profile(self, err_table=None, budget_hint_bytes: int = 0):
        t = self.err_table if err_table is None else err_table
        kimad_profile(self.handle, t, budget_hint_bytes)
        return t

    def allocate(self, budget_bytes: int, err_table=None):
        t = self.err_table if err_table is None else err_table
        kimad_allocate(self.handle, t, budget_bytes, self.j, self.K, self.offsets, self.status[0:1])
        return self.j, self.K, self.offsets, self.status[0:1]

    def compress_ef(self, K=None, offsets=None, reuse_profile: bool = False):
        K = self.K if K is None else K
        offsets = self.offsets if offsets is None else offsets
        kimad_compress_ef(self.handle, K, offsets, self.idx, self.val, self.capacity_pairs,
                          KIMAD_REUSE_PROFILE if reuse_profile else 0, self.status[1:2])
        return self.idx, self.val, self.status[1:2]

    def step(self, budget_bytes: int):
        kimad_step(self.handle, budget_bytes, self.err_table, self.j, self.K, self.offsets, self.idx, self.val,
                   self.capacity_pairs, self.status)
        return self.status

    def error_at(self, K, err_out=None):
        """Per-layer TopK error at the sizes K (device int64[L]); returns a device float64[L]."""
        if err_out is None:
            err_out = self.torch.empty(self.L, dtype=self.torch.float64, device=self.device)
        kimad_error_at(self.handle, K, err_out)
        return err_out

    def diagnostics(self):
        out = (C.c_uint32 * 4)()
        _check(lib().kimad_profile_diagnostics(C.c_void_p(self.handle), out, C.c_void_p(_stream(None))),
               "kimad_profile_diagnostics")
        return dict(uncertified=int(out[0]), recomputed=int(out[1]), pool_entries=int(out[2]),
                    redo_layers=int(out[3]))

    def allocate_diagnostics(self):
        out = (C.c_uint32 * 4)()
        _check(lib().kimad_allocate_diagnostics(C.c_void_p(self.handle), out, C.c_void_p(_stream(None))),
               "kimad_allocate_diagnostics")
        return dict(max_band=int(out[0]), sum_bands=int(out[1]), whole_rows=int(out[2]), upgrades=int(out[3]))

    def layer_states(self):
        """Per tiled layer: dict(layer, spill_bin, slots_pre, slots_cand, redo, spill_cnt, spill_valid, mode)."""
        out = (C.c_uint32 * (8 * self.L))()
        cnt = C.c_uint32(0)
        _check(lib().kimad_plan_layer_states(C.c_void_p(self.handle), out, self.L, C.byref(cnt),
                                             C.c_void_p(_stream(None))), "kimad_plan_layer_states")
        names = ("layer", "spill_bin", "slots_pre", "slots_cand", "redo", "spill_cnt", "spill_valid", "mode")
        return [dict(zip(names, out[8 * b:8 * b + 8])) for b in range(cnt.value)]

    def set_timing(self, enable: bool) -> None:
        _check(lib().kimad_plan_set_timing(C.c_void_p(self.handle), int(bool(enable))), "kimad_plan_set_timing")

    def get_timings(self):
        """[(kernel name, milliseconds)] for every launch since the last call (timing must be on)."""
        names = C.create_string_buffer(65536)
        ms = (C.c_float * 1024)()
        cnt = C.c_uint32(0)
        _check(lib().kimad_plan_get_timings(C.c_void_p(self.handle), names, 65536, ms, 1024, C.byref(cnt)),
               "kimad_plan_get_timings")
        nm = names.value.decode().split("\n")[:cnt.value]
        return [(nm[k], float(ms[k])) for k in range(cnt.value)]

    def close(self):
        if getattr(self, "handle", 0):
            kimad_plan_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
