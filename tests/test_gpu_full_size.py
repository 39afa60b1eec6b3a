"""Full-size parity of the entry points beyond pipad_frame_aggregate, on the frame bench.py times
(large: N = 1M R-MAT, k = 8), with default options, element by element against the CPU oracle:

  pipad_frame_aggregate_update   F = Fo = 64, all 8 snapshots (fused update, Section 4.2 weight reuse)
  the coalescent kernel          concatenated operand at the paper's widths F = 2 and F = 16 (Section 5.1)
  pipad_frame_transpose          on a directed variant of the frame (one direction of a random half of
                                 the edges dropped): parts bit-exact, aggregation checked through the
                                 adjoint identity and on sampled rows computed from the definition
"""
import numpy as np
import pytest

import oracle
import synth
from _util import check_y, to_gpu_snapshots

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def pipad():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2301_00391_amd as p
    p.load_library()
    return p


@pytest.fixture(scope="module")
def large():
    cfg = synth.CONFIGS["large"]
    s = synth.graphs(cfg.n, cfg.edges, cfg.k, cfg.churn, cfg.model, cfg.params, cfg.seed)
    return cfg, s


def update_tolerance(F):
    """The aggregation's 1e-5, plus one float32 rounding per term of the F-term dot product and one
    for the bias (unit roundoff 2^-24), relative to B2 = (|A^||X|)|W| + |bias|."""
    return 1e-5 + (F + 2) * 2.0 ** -24


def test_fused_update_on_the_large_frame(pipad, large):
    cfg, s = large
    n, k, F, Fo = cfg.n, cfg.k, 64, 64
    dev = "cuda:0"
    frame = pipad.frame_build_overlap(to_gpu_snapshots(torch, s, range(k)))
    stride = pipad.padded_row_stride(F)
    rng = np.random.default_rng(64)
    W = (rng.standard_normal((F, Fo)) / np.sqrt(F)).astype(np.float32)
    b = rng.standard_normal(Fo).astype(np.float32)
    X, xs = [], []
    for t in range(k):
        X.append(synth.features(cfg.seed, t, n, F))
        buf = torch.zeros((n, stride), dtype=torch.float32, device=dev)
        buf[:, :F] = torch.from_numpy(X[t]).to(dev)
        xs.append(buf[:, :F])
    H = pipad.frame_aggregate_update(frame, xs, torch.from_numpy(W).to(dev), torch.from_numpy(b).to(dev))
    torch.cuda.synchronize()
    threads = oracle.hardware_threads()
    for t in range(k):
        rows, cols = s.coo(t)
        Hd, B2 = oracle.aggregate_update(n, rows, cols, X[t], W, b, threads=threads)
        err = np.abs(H[t].cpu().numpy().astype(np.float64) - Hd)
        ratio = float(np.max(err / np.maximum(B2, 1e-300)))
        print(f"large, fused update, snapshot {t}: worst error ratio {ratio:.3e} "
              f"(budget {update_tolerance(F):.3e})", flush=True)
        assert ratio <= update_tolerance(F), f"snapshot {t}"
    frame.close()


def test_entry_point_without_allocation_on_the_large_frame(pipad, large):
    """The large frame's partial sums (133 MB for 8 snapshots) do not fit the fixed 64 MiB array at
    once: pipad_frame_aggregate_static takes the snapshots in groups of three and must give the
    bits of pipad_frame_aggregate."""
    cfg, s = large
    n, k, F = cfg.n, cfg.k, cfg.feat
    dev = "cuda:0"
    frame = pipad.frame_build_overlap(to_gpu_snapshots(torch, s, range(k)))
    xs = [torch.from_numpy(synth.features(cfg.seed, t, n, F)).to(dev) for t in range(k)]
    y_alloc = [y.clone() for y in pipad.frame_aggregate(frame, xs)]
    y_static = pipad.frame_aggregate(frame, xs, static_scratch=True)
    torch.cuda.synchronize()
    for t in range(k):
        assert torch.equal(y_alloc[t], y_static[t]), f"snapshot {t}"
    frame.close()


@pytest.mark.parametrize("F", [2, 16])
def test_coalescent_kernel_on_the_large_frame(pipad, large, F):
    """Default options: the concatenated [N, k, F] operand of 64 / 512 MB takes the coalescent
    kernel by the automatic rule."""
    cfg, s = large
    n, k = cfg.n, cfg.k
    dev = "cuda:0"
    assert pipad.get_option("agg_coalescent") == 1
    frame = pipad.frame_build_overlap(to_gpu_snapshots(torch, s, range(k)))
    X = [synth.features(cfg.seed + 50, t, n, F) for t in range(k)]
    xw = torch.from_numpy(np.stack(X, axis=1)).to(dev)
    yw = pipad.frame_aggregate(frame, xw)
    torch.cuda.synchronize()
    threads = oracle.hardware_threads()
    for t in range(k):
        rows, cols = s.coo(t)
        _, yd, bound, _ = oracle.aggregate(n, rows, cols, X[t], threads=threads)
        worst = check_y(yw[:, t, :].cpu().numpy(), yd, bound, f"coalescent F={F}, snapshot {t}")
        print(f"large, coalescent F={F}, snapshot {t}: worst error ratio {worst:.3e}", flush=True)
    frame.close()


def directed_variant(n, rowptr, col):
    """Drops one direction of about half of the undirected edges; which edges, and which direction,
    depends only on the edge, so an edge shared by several snapshots meets the same fate in all."""
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    c = col.astype(np.int64)
    lo, hi = np.minimum(rows, c), np.maximum(rows, c)
    h = ((lo * 2654435761 + hi * 40503) ^ ((lo + 7) * (hi + 13))) >> 7  # some bits of a hash of the edge
    drop_edge = (h & 1) == 1
    drop_upper = ((h >> 1) & 1) == 1
    keep = ~(drop_edge & (drop_upper == (rows < c)))
    new_rowptr = np.concatenate([[0], np.cumsum(np.bincount(rows[keep], minlength=n))]).astype(np.int32)
    return new_rowptr, col[keep]


def transpose_csr(n, rowptr, col):
    rows = np.repeat(np.arange(n, dtype=np.int32), np.diff(rowptr))
    order = np.lexsort((rows, col))
    t_rowptr = np.concatenate([[0], np.cumsum(np.bincount(col, minlength=n))]).astype(np.int32)
    return t_rowptr, rows[order]


def test_transposed_frame_of_a_directed_variant_of_the_large_frame(pipad, large):
    cfg, s = large
    n, k, F = cfg.n, cfg.k, 64
    dev = "cuda:0"
    lists = [directed_variant(n, s.rowptr[t], s.col[t]) for t in range(k)]
    snaps = [(torch.from_numpy(rp).to(dev), torch.from_numpy(c).to(dev)) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps)
    tframe = pipad.frame_transpose(frame)
    # parts: bit-exact transposes (overlap part and two exclusive parts compared entry by entry)
    for part in (None, 0, k - 1):
        rp, col = frame.common() if part is None else frame.delta(part)
        trp, tcol = tframe.common() if part is None else tframe.delta(part)
        want_rp, want_col = transpose_csr(n, rp.cpu().numpy(), col.cpu().numpy())
        assert np.array_equal(trp.cpu().numpy(), want_rp), f"rowptr of part {part}"
        assert np.array_equal(tcol.cpu().numpy(), want_col), f"columns of part {part}"
    assert torch.equal(frame.dinv(), tframe.dinv())
    frame.close()
    stride = pipad.padded_row_stride(F)
    G, gs = [], []
    for t in range(k):
        G.append(synth.features(cfg.seed + 9, t, n, F))
        buf = torch.zeros((n, stride), dtype=torch.float32, device=dev)
        buf[:, :F] = torch.from_numpy(G[t]).to(dev)
        gs.append(buf[:, :F])
    Z = pipad.frame_aggregate(tframe, gs)
    torch.cuda.synchronize()
    threads = oracle.hardware_threads()
    rng = np.random.default_rng(5)
    for t in (0, 3, k - 1):
        rp, col = lists[t]
        rows = np.repeat(np.arange(n, dtype=np.int32), np.diff(rp))
        z = Z[t].cpu().numpy().astype(np.float64)
        # (1) adjoint identity against the pinned forward oracle: <A^ X, G> = <X, A^T G>
        X = synth.features(cfg.seed + 77, t, n, F)
        _, yd, bound, _ = oracle.aggregate(n, rows, col, X, threads=threads)
        lhs = float(np.sum(yd * G[t]))
        rhs = float(np.sum(X.astype(np.float64) * z))
        scale = float(np.sum(bound * np.abs(G[t])))
        assert abs(lhs - rhs) <= 1e-5 * scale, f"adjoint identity, snapshot {t}: {lhs} vs {rhs}"
        # (2) sampled rows from the definition: Z[j] = sum over i with (i, j) in A + I of X[i] / sqrt(d_i d_j)
        trp, trow = transpose_csr(n, rp, col)
        d = (np.diff(rp) + 1).astype(np.float64)
        heavy = np.argsort(-np.diff(trp))[:20]
        for j in np.concatenate([heavy, rng.choice(n, 2000, replace=False)]):
            src = np.concatenate([trow[trp[j]:trp[j + 1]], [j]]).astype(np.int64)
            wgt = 1.0 / np.sqrt(d[src] * d[j])
            g64 = G[t][src].astype(np.float64)
            want = (wgt[:, None] * g64).sum(axis=0)
            lim = 1e-5 * (wgt[:, None] * np.abs(g64)).sum(axis=0)
            assert np.all(np.abs(z[j] - want) <= lim), f"snapshot {t}, row {j}"
        print(f"large directed variant, transposed aggregation, snapshot {t}: ok", flush=True)
    tframe.close()
