"""Helpers shared by the GPU parity tests (marshalling between numpy inputs and the two sides)."""
import numpy as np

TOL = 1e-5  # |Y_gpu - Y_oracle| <= TOL * (|A^| |X|), element by element


def to_gpu_snapshots(torch, snaps, ts, device="cuda:0"):
    return [(torch.from_numpy(np.ascontiguousarray(snaps.rowptr[t])).to(device),
             torch.from_numpy(np.ascontiguousarray(snaps.col[t])).to(device)) for t in ts]


def csr_to_coo(n, rowptr, col):
    rows = np.repeat(np.arange(n, dtype=np.int32), np.diff(rowptr))
    return rows, col


def check_overlap(frame, oracle_parts):
    """Bit-exact comparison of the frame's CSRs with the oracle's."""
    (c_rp, c_col), excl = oracle_parts
    g_rp, g_col = frame.common()
    assert np.array_equal(g_rp.cpu().numpy(), c_rp), "common rowptr"
    assert np.array_equal(g_col.cpu().numpy(), c_col), "common colidx"
    for t, (e_rp, e_col) in enumerate(excl):
        d_rp, d_col = frame.delta(t)
        assert np.array_equal(d_rp.cpu().numpy(), e_rp), f"delta {t} rowptr"
        assert np.array_equal(d_col.cpu().numpy(), e_col), f"delta {t} colidx"


def check_y(y_gpu, yd, bound, what=""):
    """The parity bar for fp32 outputs."""
    err = np.abs(y_gpu.astype(np.float64) - yd)
    lim = TOL * bound
    bad = err > lim
    if bad.any():
        idx = np.argwhere(bad)[0]
        worst = np.max(err / np.maximum(bound, 1e-300))
        raise AssertionError(f"{what}: {bad.sum()} elements beyond {TOL}*B, first at {tuple(idx)}: "
                             f"err {err[tuple(idx)]:.3e} lim {lim[tuple(idx)]:.3e}; worst ratio {worst:.3e}")
    return float(np.max(err / np.maximum(bound, 1e-300)))
