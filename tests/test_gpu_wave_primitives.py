"""The DPP-based wave primitives of the kernels, lane by lane against host-computed values.  They are written as
inline assembly with explicit wait states (the hardware needs two cycles between a vector write and a DPP read of
the same register, and the compiler does not see through the assembly): an edit or a compiler that loses one
shows here as a wrong lane instead of as a wrong rank, and a memory fault, inside the streaming pass."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_every_lane_of_the_dpp_primitives(seed):
    import torch
    import paper_2312_08053_amd.binding as b
    rng = np.random.default_rng(seed)
    if seed == 0:
        u = np.arange(128, dtype=np.uint32) * 3 + 1          # distinct per lane: a shifted or swapped lane shows
        f = np.arange(128, dtype=np.float64) * 1.25 - 17.0
    else:
        u = rng.integers(0, 1 << 20, size=128).astype(np.uint32)
        f = rng.standard_normal(128) * 10.0 ** rng.uniform(-3, 3, size=128)
    if seed == 3:
        f[:64] = np.round(f[:64] / np.abs(f[:64]).max() * 3.0)     # few distinct values: the pair minimum must break ties by the record
    u[64:] = (0 - u[64:].astype(np.int64)).astype(np.uint32) if seed == 2 else u[64:]   # negated costs, as the recurrence passes them
    in_u = torch.from_numpy(u.view(np.int32).copy()).cuda()
    in_f = torch.from_numpy(f.copy()).cuda()
    out_u = torch.full((64 + 1024 + 256,), -1, dtype=torch.int32, device="cuda")
    out_f = torch.full((1024 + 192 + 256,), float("nan"), dtype=torch.float64, device="cuda")
    b.kimad_selftest_wave_primitives(in_u, in_f, out_u, out_f)
    torch.cuda.synchronize()
    got_u = out_u.cpu().numpy().view(np.uint32)
    got_f = out_f.cpu().numpy()
    lanes = np.arange(64)
    assert np.array_equal(got_u[:64], np.cumsum(u[:64].astype(np.uint64)).astype(np.uint32))
    for k in range(4):
        for t in range(4):
            src = 64 + 16 * (lanes // 16) + 4 * k + t
            want_u = (u[:64].astype(np.uint64) + u[src].astype(np.uint64)).astype(np.uint32)
            assert np.array_equal(got_u[64 + (4 * k + t) * 64:][:64], want_u), (k, t)
            want_f = f[:64] + f[src]
            assert np.array_equal(got_f[(4 * k + t) * 64:][:64], want_f), (k, t)
    for t, width in enumerate((2, 4, 8)):
        want = f[:64].reshape(-1, width).max(axis=1).repeat(width)
        assert np.array_equal(got_f[1024 + 64 * t:][:64], want), width
    rec = u[64:] & 255
    for t, width in enumerate((2, 4, 8, 16)):
        v = f[:64].reshape(-1, width)
        r = rec.reshape(-1, width)
        vmin = v.min(axis=1)
        rmin = np.where(v == vmin[:, None], r, 256).min(axis=1)
        assert np.array_equal(got_f[1216 + 64 * t:][:64], vmin.repeat(width)), width
        assert np.array_equal(got_u[1088 + 64 * t:][:64], rmin.repeat(width).astype(np.uint32)), width
