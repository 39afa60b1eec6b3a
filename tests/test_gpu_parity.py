"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Integer outputs (overlap and exclusive CSRs) must be bit-exact; fp32 outputs must satisfy
|dY| <= 1e-5 * (|A^| |X|) per element.  Inputs are the seeded synthetic frames of ``synth``.
"""
import numpy as np
import pytest

import oracle
import synth
from _util import check_overlap, check_y, csr_to_coo, to_gpu_snapshots

pytestmark = pytest.mark.gpu

DEFAULT_OPTIONS = {"short_max": 64, "mid_max": 512, "hub_threshold": 2048, "hub_segment": 2048,
                   "sub_classes": 1, "agg_order": 2, "agg_nt": 1, "agg_generic": 0, "agg_coalescent": 1, "slice_cols": 0}

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def pipad():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2301_00391_amd as p
    p.load_library()
    return p


@pytest.fixture(autouse=True)
def _reset_options(pipad):
    yield
    for key, val in DEFAULT_OPTIONS.items():
        pipad.set_option(key, val)


def run_case(pipad, n, lists, F, seed, layout="list", allocator="torch", validate=True,
             check_csr=True):
    """lists: k (rowptr, col) numpy CSR pairs.  Returns the worst error ratio."""
    k = len(lists)
    dev = "cuda:0"
    snaps = [(torch.from_numpy(np.ascontiguousarray(rp)).to(dev),
              torch.from_numpy(np.ascontiguousarray(c)).to(dev)) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps, validate=validate, allocator=allocator)
    coo = [csr_to_coo(n, rp, c) for rp, c in lists]
    if check_csr:
        check_overlap(frame, oracle.overlap(n, coo))
    X = [synth.features(seed, t, n, F) for t in range(k)]
    if layout == "wide":
        xw = torch.from_numpy(np.stack(X, axis=1)).to(dev)  # [n, k, F]
        yw = pipad.frame_aggregate(frame, xw)
        torch.cuda.synchronize()
        ys = [yw[:, t, :].cpu().numpy() for t in range(k)]
    else:
        xs = [torch.from_numpy(x).to(dev) for x in X]
        yl = pipad.frame_aggregate(frame, xs)
        torch.cuda.synchronize()
        ys = [y.cpu().numpy() for y in yl]
    worst = 0.0
    for t in range(k):
        _, yd, bound, _ = oracle.aggregate(n, coo[t][0], coo[t][1], X[t], threads=8)
        worst = max(worst, check_y(ys[t], yd, bound, f"snapshot {t}"))
    frame.close()
    return worst


def rand_csr(rng, n, p, symmetric=True):
    M = rng.random((n, n)) < p
    if symmetric:
        M = np.triu(M, 1)
        M = M | M.T
    np.fill_diagonal(M, False)
    rowptr = np.concatenate([[0], np.cumsum(M.sum(axis=1))]).astype(np.int32)
    col = np.nonzero(M)[1].astype(np.int32)
    return rowptr, col


def churned(rng, n, k, p, keep, symmetric=True):
    base = rng.random((n, n)) < p
    out = []
    for _ in range(k):
        M = base & (rng.random((n, n)) < keep) | (rng.random((n, n)) < p * (1 - keep))
        if symmetric:
            M = np.triu(M, 1)
            M = M | M.T
        np.fill_diagonal(M, False)
        rowptr = np.concatenate([[0], np.cumsum(M.sum(axis=1))]).astype(np.int32)
        out.append((rowptr, np.nonzero(M)[1].astype(np.int32)))
    return out


@pytest.mark.parametrize("nt,coalescent,mid_max,order", [(0, 1, 256, 2), (3, 2, 40, 1), (0, 0, 10, 0)])
@pytest.mark.parametrize("layout", ["list", "wide"])
def test_tiny_config(pipad, nt, coalescent, mid_max, order, layout):
    pipad.set_option("agg_nt", nt)
    pipad.set_option("agg_order", order)
    pipad.set_option("agg_coalescent", coalescent)
    pipad.set_option("mid_max", mid_max)
    cfg = synth.CONFIGS["tiny"]
    s = synth.make(cfg)
    lists = [(s.rowptr[t], s.col[t]) for t in range(cfg.k)]
    run_case(pipad, cfg.n, lists, cfg.feat, cfg.seed, layout=layout)


@pytest.mark.parametrize("first", [0, 7, 12])
def test_small_config_sliding_frames(pipad, first):
    cfg = synth.CONFIGS["small"]
    s = synth.make(cfg)
    lists = [(s.rowptr[t], s.col[t]) for t in range(first, first + cfg.k)]
    run_case(pipad, cfg.n, lists, cfg.feat, cfg.seed + first, layout="wide")


@pytest.mark.parametrize("k,F", [(1, 1), (2, 2), (3, 6), (4, 16), (5, 20), (8, 64), (8, 128),
                                 (2, 130), (16, 32), (3, 260), (32, 4), (8, 256), (7, 12)])
@pytest.mark.parametrize("short_max,generic,mid_max", [(32, 0, 256), (4, 0, 12), (4, 1, 12), (2, 0, 2)])
def test_shapes_and_feature_widths(pipad, k, F, short_max, generic, mid_max):
    pipad.set_option("short_max", short_max)
    pipad.set_option("agg_generic", generic)
    pipad.set_option("mid_max", mid_max)
    rng = np.random.default_rng(1000 * k + F)
    n = 333  # several workgroups and a ragged tail
    lists = churned(rng, n, k, 0.03, 0.8)
    run_case(pipad, n, lists, F, seed=k * 7 + F, layout="wide" if F % 2 == 0 else "list")


@pytest.mark.parametrize("sub_classes", [1, 2, 4])
@pytest.mark.parametrize("short_max,mid_max,threshold,segment",
                         [(2, 8, 14, 4), (0, 0, 1, 1), (5, 5, 5, 3), (0, 20, 9, 70), (3, 1000, 6, 4)])
def test_row_classes_short_mid_hub(pipad, short_max, mid_max, threshold, segment, sub_classes):
    """Low thresholds push rows through all three paths (whole short rows walked by lane teams,
    whole mid rows by a wave, class parts of hub rows by a wave each, with one or several
    classes per XCD); very long rows are cut into units; the partial sums of a row are added in
    a fixed order."""
    pipad.set_option("short_max", short_max)
    pipad.set_option("mid_max", mid_max)
    pipad.set_option("hub_threshold", threshold)
    pipad.set_option("hub_segment", segment)
    pipad.set_option("sub_classes", sub_classes)
    rng = np.random.default_rng(77)
    n = 500
    lists = churned(rng, n, 4, 0.04, 0.7)
    run_case(pipad, n, lists, 130, seed=4)
    run_case(pipad, n, lists, 64, seed=4, layout="wide")
    run_case(pipad, n, lists, 16, seed=5)
    run_case(pipad, n, lists, 9, seed=6)
    run_case(pipad, n, lists, 64, seed=7, layout="wide")
    # concatenated operand with small F: the coalescent kernel (snapshot groups side by side)
    pipad.set_option("agg_coalescent", 2)
    run_case(pipad, n, lists, 16, seed=8, layout="wide")
    run_case(pipad, n, lists, 6, seed=9, layout="wide")
    run_case(pipad, n, lists, 3, seed=10, layout="wide")


@pytest.mark.parametrize("keep", [0.95, 0.3])
def test_column_arrays_that_are_only_4_byte_aligned(pipad, keep):
    """The ABI asks for int32 alignment only: column arrays that start in the middle of a 16-byte
    piece are valid input (little overlap: the lane-per-entry scatter of the exclusive parts; much
    overlap: the expand)."""
    rng = np.random.default_rng(int(keep * 100))
    n, k, F = 800, 4, 32
    lists = churned(rng, n, k, 0.03, keep)
    dev = "cuda:0"
    snaps, hold = [], []
    for rp, c in lists:
        store = torch.zeros(c.size + 3, dtype=torch.int32, device=dev)
        for shift in (1, 2, 3):
            if (store.data_ptr() + 4 * shift) % 16 != 0:
                break
        view = store[shift:shift + c.size]
        view.copy_(torch.from_numpy(c).to(dev))
        assert view.data_ptr() % 16 != 0 and view.is_contiguous()
        hold.append(store)
        snaps.append((torch.from_numpy(rp).to(dev), view))
    frame = pipad.frame_build_overlap(snaps)
    coo = [csr_to_coo(n, rp, c) for rp, c in lists]
    check_overlap(frame, oracle.overlap(n, coo))
    X = [synth.features(5, t, n, F) for t in range(k)]
    ys = pipad.frame_aggregate(frame, [torch.from_numpy(x).to(dev) for x in X])
    torch.cuda.synchronize()
    for t in range(k):
        _, yd, bound, _ = oracle.aggregate(n, coo[t][0], coo[t][1], X[t], threads=4)
        check_y(ys[t].cpu().numpy(), yd, bound, f"snapshot {t}")
    frame.close()


def test_a_frame_keeps_the_options_it_was_built_with(pipad):
    """Options are copied into the frame by the build: changing them afterwards must not change a
    bit of what the frame computes, while a frame built afterwards takes the new values (here: all
    rows become hub rows cut into small units, which sums in another order)."""
    rng = np.random.default_rng(99)
    n, k, F = 600, 3, 64
    lists = churned(rng, n, k, 0.05, 0.8)
    dev = "cuda:0"
    snaps = [(torch.from_numpy(rp).to(dev), torch.from_numpy(c).to(dev)) for rp, c in lists]
    xs = [torch.from_numpy(synth.features(3, t, n, F)).to(dev) for t in range(k)]
    frame = pipad.frame_build_overlap(snaps)
    before = [y.clone() for y in pipad.frame_aggregate(frame, xs)]
    for key, val in (("short_max", 0), ("mid_max", 0), ("hub_threshold", 4), ("hub_segment", 4),
                     ("sub_classes", 4), ("agg_generic", 1)):
        pipad.set_option(key, val)
    after = pipad.frame_aggregate(frame, xs)
    other = pipad.frame_build_overlap(snaps)
    different = pipad.frame_aggregate(other, xs)
    torch.cuda.synchronize()
    for t in range(k):
        assert torch.equal(before[t], after[t]), f"snapshot {t}"
    assert any(not torch.equal(before[t], different[t]) for t in range(k)), \
        "the new options did not reach the frame built after them"
    for t in range(k):
        assert torch.allclose(before[t], different[t], rtol=1e-4, atol=1e-5)
    frame.close()
    other.close()


@pytest.mark.parametrize("k,F", [(8, 2), (8, 6), (4, 16), (8, 16), (2, 30), (32, 2), (3, 5)])
@pytest.mark.parametrize("coalescent", [2, 0])
def test_small_feature_widths_on_the_concatenated_operand(pipad, k, F, coalescent):
    """The paper's own regime (F = 2 / 6 / 16, Section 5.1): with the concatenated operand the
    coalescent kernel runs; switched off, the per-snapshot slices must give the same answer."""
    pipad.set_option("agg_coalescent", coalescent)
    rng = np.random.default_rng(500 + 10 * k + F)
    n = 700
    lists = churned(rng, n, k, 0.02, 0.85)
    run_case(pipad, n, lists, F, seed=k + F, layout="wide", check_csr=False)


@pytest.mark.parametrize("k,keep", [(3, 0.97), (8, 0.9), (12, 0.97), (20, 0.5)])
def test_long_rows_whose_entries_shift_between_snapshots(pipad, k, keep):
    """Rows of thousands of entries next to short ones: a changed entry moves everything behind
    it, so the matches of a wave's 64 entries sit at other offsets in the other snapshots (by a
    few places at keep = 0.97, by hundreds at 0.5, beyond what a wave stages on chip)."""
    rng = np.random.default_rng(31 * k + int(100 * keep))
    n = 2500
    dens = np.full((n, 1), 0.004)
    dens[rng.choice(n, 6, replace=False)] = 0.8
    base = rng.random((n, n)) < dens
    lists = []
    for _ in range(k):
        M = base & (rng.random((n, n)) < keep) | (rng.random((n, n)) < dens * (1 - keep))
        np.fill_diagonal(M, False)
        rowptr = np.concatenate([[0], np.cumsum(M.sum(axis=1))]).astype(np.int32)
        lists.append((rowptr, np.nonzero(M)[1].astype(np.int32)))
    run_case(pipad, n, lists, 4, seed=k)


def test_directed_patterns(pipad):
    rng = np.random.default_rng(5)
    lists = churned(rng, 257, 3, 0.05, 0.6, symmetric=False)
    run_case(pipad, 257, lists, 24, seed=11)


def test_degenerate_frames(pipad):
    rng = np.random.default_rng(6)
    n = 130
    a = rand_csr(rng, n, 0.05)
    empty = (np.zeros(n + 1, np.int32), np.zeros(0, np.int32))
    # k = 1: all common; identical snapshots: no exclusive edges
    run_case(pipad, n, [a], 8, seed=1)
    run_case(pipad, n, [a, a, a], 8, seed=2)
    # one empty snapshot: empty overlap, everything exclusive; all empty: Y = X
    run_case(pipad, n, [a, empty], 8, seed=3)
    run_case(pipad, n, [empty, a], 8, seed=3)
    run_case(pipad, n, [empty, empty], 8, seed=4)
    # a single node, and two nodes joined by an edge
    run_case(pipad, 1, [(np.zeros(2, np.int32), np.zeros(0, np.int32))], 4, seed=5)
    two = (np.array([0, 1, 2], np.int32), np.array([1, 0], np.int32))
    run_case(pipad, 2, [two, two], 4, seed=6)


def test_no_nodes(pipad):
    rp = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    col = torch.zeros(0, dtype=torch.int32, device="cuda:0")
    frame = pipad.frame_build_overlap([(rp, col), (rp, col)])
    c_rp, c_col = frame.common()
    assert c_rp.tolist() == [0] and c_col.numel() == 0
    x = torch.zeros((0, 2, 4), device="cuda:0")
    y = pipad.frame_aggregate(frame, x)
    assert y.shape == (0, 2, 4)


def test_library_allocator_and_determinism(pipad):
    rng = np.random.default_rng(8)
    n = 400
    lists = churned(rng, n, 4, 0.03, 0.8)
    run_case(pipad, n, lists, 32, seed=9, allocator="library")
    pipad.set_option("short_max", 3)
    pipad.set_option("mid_max", 6)
    pipad.set_option("hub_threshold", 8)
    pipad.set_option("hub_segment", 8)
    snaps = [(torch.from_numpy(rp).cuda(), torch.from_numpy(c).cuda()) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps)
    x = torch.rand((n, 4, 32), device="cuda:0") * 2 - 1
    y1 = pipad.frame_aggregate(frame, x).clone()
    y2 = pipad.frame_aggregate(frame, x)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2), "same inputs must give the same bits"


def test_aggregate_replayed_from_a_hip_graph(pipad):
    """pipad_frame_aggregate only enqueues kernels (after one eager call has sized the hub
    scratch), so a training loop can capture it once and replay it.  Every replay, with eager work
    and synchronisations in between, must reproduce the eager result bit for bit."""
    pipad.set_option("short_max", 2)
    pipad.set_option("mid_max", 5)
    pipad.set_option("hub_threshold", 6)
    pipad.set_option("hub_segment", 4)
    rng = np.random.default_rng(99)
    n, k, F = 900, 4, 48
    lists = churned(rng, n, k, 0.03, 0.8)
    dev = "cuda:0"
    snaps = [(torch.from_numpy(rp).to(dev), torch.from_numpy(c).to(dev)) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps)
    X = [torch.from_numpy(synth.features(3, t, n, F)).to(dev) for t in range(k)]
    Y = [torch.empty_like(x) for x in X]
    Y_eager = [torch.empty_like(x) for x in X]
    pipad.frame_aggregate(frame, X, Y)  # eager: sizes the scratch of the hub rows
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pipad.frame_aggregate(frame, X, Y)
    for replay in range(4):
        for t in range(k):
            X[t].copy_(torch.from_numpy(synth.features(100 + replay, t, n, F)))
        pipad.frame_aggregate(frame, X, Y_eager)
        torch.cuda.synchronize()
        for y in Y:
            y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for t in range(k):
            assert torch.equal(Y[t], Y_eager[t]), f"replay {replay}, snapshot {t}"
    # and the replayed result is the right one
    coo = csr_to_coo(n, *lists[0])
    x0 = synth.features(103, 0, n, F)
    _, yd, bound, _ = oracle.aggregate(n, coo[0], coo[1], x0, threads=4)
    check_y(Y[0].cpu().numpy(), yd, bound, "replayed snapshot 0")
    frame.close()


def test_padded_rows_are_left_alone(pipad):
    """ldy > F: the columns beyond F of Y keep their contents."""
    rng = np.random.default_rng(10)
    n, k, F, pad = 200, 2, 12, 20
    lists = churned(rng, n, k, 0.05, 0.8)
    snaps = [(torch.from_numpy(rp).cuda(), torch.from_numpy(c).cuda()) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps)
    xb = [torch.rand((n, pad), device="cuda:0") for _ in range(k)]
    yb = [torch.full((n, pad), 7.0, device="cuda:0") for _ in range(k)]
    pipad.frame_aggregate(frame, [x[:, :F] for x in xb], [y[:, :F] for y in yb])
    torch.cuda.synchronize()
    for t in range(k):
        assert torch.all(yb[t][:, F:] == 7.0)
        rows, cols = csr_to_coo(n, *lists[t])
        xnp = np.ascontiguousarray(xb[t][:, :F].cpu().numpy())
        _, yd, bound, _ = oracle.aggregate(n, rows, cols, xnp)
        check_y(yb[t][:, :F].cpu().numpy(), yd, bound, f"padded {t}")


def test_validation_rejects_non_canonical_input(pipad):
    n = 50
    good = rand_csr(np.random.default_rng(12), n, 0.1)

    def build(rp, col):
        snaps = [(torch.from_numpy(np.asarray(rp, np.int32)).cuda(),
                  torch.from_numpy(np.asarray(col, np.int32)).cuda())]
        return pipad.frame_build_overlap(snaps, validate=True)

    build(*good).close()
    rp, col = good
    row = int(np.argmax(np.diff(rp) >= 2))
    a = rp[row]
    bad_sets = []
    c = col.copy(); c[a], c[a + 1] = c[a + 1], c[a]; bad_sets.append((rp, c))        # unsorted
    c = col.copy(); c[a + 1] = c[a]; bad_sets.append((rp, c))                         # duplicate
    c = col.copy(); c[a] = row; bad_sets.append((rp, c))                              # diagonal
    c = col.copy(); c[a] = n; bad_sets.append((rp, c))                                # out of range
    r = rp.copy(); r[3] = r[4] + 1; bad_sets.append((r, col))                         # decreasing
    r = rp.copy(); r[-1] -= 1; bad_sets.append((r, col))                              # rowptr[n] != nnz
    for rp_b, col_b in bad_sets:
        with pytest.raises(pipad.PipadError) as info:
            build(rp_b, col_b)
        assert info.value.status == -2


def test_allocator_failure_is_reported_not_fatal(pipad):
    """A caller allocator that runs dry at any of its calls must give PIPAD_ERR_ALLOC (-3) from
    build or aggregate, leave no frame behind, and leave the library usable."""
    import ctypes
    from paper_2301_00391_amd import binding
    lib = pipad.load_library()
    rng = np.random.default_rng(21)
    n, k = 300, 3
    lists = churned(rng, n, k, 0.05, 0.8)
    pipad.set_option("short_max", 2)
    pipad.set_option("mid_max", 4)
    pipad.set_option("hub_threshold", 6)   # split rows exist, so aggregate needs scratch
    pipad.set_option("hub_segment", 4)
    snaps = [(torch.from_numpy(rp).cuda(), torch.from_numpy(c).cuda()) for rp, c in lists]
    arr = (binding._Csr * k)()
    for t, (rp, col) in enumerate(snaps):
        arr[t].n, arr[t].nnz = n, col.numel()
        arr[t].rowptr, arr[t].colidx = rp.data_ptr(), col.data_ptr()
    stream = torch.cuda.current_stream().cuda_stream
    x = torch.rand((n, k, 8), device="cuda:0")
    y = torch.empty_like(x)
    xp = (ctypes.c_void_p * k)(*[x[:, t, :].data_ptr() for t in range(k)])
    yp = (ctypes.c_void_p * k)(*[y[:, t, :].data_ptr() for t in range(k)])
    statuses = []
    for fail_at in range(1, 6):
        keep, calls = [], [0]

        def alloc(nbytes, _ctx):
            calls[0] += 1
            if calls[0] == fail_at:
                return None
            buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda:0")
            keep.append(buf)
            return buf.data_ptr()

        cb = binding.ALLOC_FN(alloc)
        out = ctypes.c_void_p()
        rc = lib.pipad_frame_build_overlap(n, k, arr, 0, ctypes.cast(cb, ctypes.c_void_p), None,
                                           stream, ctypes.byref(out))
        if rc == 0:
            rc = lib.pipad_frame_aggregate(out, 8, xp, k * 8, yp, k * 8, stream)
            torch.cuda.synchronize()
            lib.pipad_frame_destroy(out)
        else:
            assert out.value is None, "no frame may be handed out on failure"
        statuses.append(rc)
    assert statuses[:4] == [-3, -3, -3, -3], statuses  # 3 calls in build, the 4th in aggregate
    assert statuses[4] == 0
    # and the library still works afterwards
    run_case(pipad, n, lists, 8, seed=3)


def test_invalid_arguments(pipad):
    rp = torch.zeros(5, dtype=torch.int32, device="cuda:0")
    col = torch.zeros(0, dtype=torch.int32, device="cuda:0")
    frame = pipad.frame_build_overlap([(rp, col)])
    x = torch.zeros((4, 1, 8), device="cuda:0")
    with pytest.raises(ValueError):
        pipad.frame_aggregate(frame, torch.zeros((4, 2, 8), device="cuda:0"))
    with pytest.raises(pipad.PipadError):
        pipad.frame_build_overlap([(rp, col), (torch.zeros(7, dtype=torch.int32, device="cuda:0"), col)])
    pipad.frame_aggregate(frame, x)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name,check_snapshots", [("large", (0, 3, 7)), ("low-overlap", (0, 7))])
def test_full_size_frames_in_the_benchmark_configuration(pipad, name, check_snapshots):
    """The frames bench.py times (N = 1M R-MAT, k = 8, F = 64; N = 500k, F = 128, 40 % churn), in
    the layout it uses (k separate [N, F] matrices whose rows are padded to an odd number of
    128-byte lines, default options): every CSR entry is compared,
    and every output element of the listed snapshots."""
    cfg = synth.CONFIGS[name]
    s = synth.graphs(cfg.n, cfg.edges, cfg.k, cfg.churn, cfg.model, cfg.params, cfg.seed)
    dev = "cuda:0"
    snaps = [(torch.from_numpy(s.rowptr[t]).to(dev), torch.from_numpy(s.col[t]).to(dev))
             for t in range(cfg.k)]
    frame = pipad.frame_build_overlap(snaps)
    coo = [s.coo(t) for t in range(cfg.k)]
    check_overlap(frame, oracle.overlap(cfg.n, coo))
    stride = pipad.padded_row_stride(cfg.feat)  # bench.py pads the rows of X the same way
    xs = []
    for t in range(cfg.k):
        buf = torch.zeros((cfg.n, stride), dtype=torch.float32, device=dev)
        buf[:, :cfg.feat] = torch.from_numpy(synth.features(cfg.seed, t, cfg.n, cfg.feat)).to(dev)
        xs.append(buf[:, :cfg.feat])
    ys = pipad.frame_aggregate(frame, xs)
    torch.cuda.synchronize()
    for t in check_snapshots:
        _, yd, bound, _ = oracle.aggregate(cfg.n, coo[t][0], coo[t][1],
                                           np.ascontiguousarray(xs[t].cpu().numpy()),
                                           threads=oracle.hardware_threads())
        worst = check_y(ys[t].cpu().numpy(), yd, bound, f"{name} snapshot {t}")
        print(f"{name} snapshot {t}: worst error ratio {worst:.3e} of the 1e-5 budget")
    frame.close()


def test_medium_frame_full_check(pipad):
    """One frame of the medium workload (N = 200k, k = 8, F = 64), every element checked."""
    cfg = synth.CONFIGS["medium"]
    s = synth.graphs(cfg.n, cfg.edges, cfg.k, cfg.churn, cfg.model, cfg.params, cfg.seed)
    lists = [(s.rowptr[t], s.col[t]) for t in range(cfg.k)]
    worst = run_case(pipad, cfg.n, lists, cfg.feat, cfg.seed, layout="wide", validate=False)
    print(f"medium worst error ratio {worst:.3e} of the 1e-5 budget")


# ---- aggregation followed by the fully connected update (one GCN layer, Eq. 1) ------------------
def update_tolerance(F):
    """Per-element budget relative to B2 = (|A^||X|)|W| + |bias|: the aggregation's 1e-5, plus one
    float32 rounding per term of the F-term dot product and one for the bias (unit roundoff 2^-24)."""
    return 1e-5 + (F + 2) * 2.0 ** -24


def run_update_case(pipad, n, lists, F, Fo, seed, with_bias=True, with_a=True, x_stride=None):
    k = len(lists)
    dev = "cuda:0"
    rng = np.random.default_rng(seed)
    snaps = [(torch.from_numpy(np.ascontiguousarray(rp)).to(dev),
              torch.from_numpy(np.ascontiguousarray(c)).to(dev)) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps)
    X = [synth.features(seed, t, n, F) for t in range(k)]
    W = (rng.standard_normal((F, Fo)) / np.sqrt(F)).astype(np.float32)
    b = rng.standard_normal(Fo).astype(np.float32) if with_bias else None
    xs = []
    for x in X:
        buf = torch.zeros((n, x_stride or F), dtype=torch.float32, device=dev)
        buf[:, :F] = torch.from_numpy(x).to(dev)
        xs.append(buf[:, :F])
    A = [torch.full((n, F), float("nan"), device=dev) for _ in range(k)] if with_a else None
    H = [torch.full((n, Fo), float("nan"), device=dev) for _ in range(k)]
    pipad.frame_aggregate_update(frame, xs, torch.from_numpy(W).to(dev),
                                 torch.from_numpy(b).to(dev) if with_bias else None, H=H, A=A)
    torch.cuda.synchronize()
    worst = 0.0
    for t in range(k):
        rows, cols = csr_to_coo(n, *lists[t])
        Hd, B2 = oracle.aggregate_update(n, rows, cols, X[t], W, b, threads=4)
        err = np.abs(H[t].cpu().numpy().astype(np.float64) - Hd)
        ratio = float(np.max(err / np.maximum(B2, 1e-300)))
        assert ratio <= update_tolerance(F), f"H, snapshot {t}: {ratio:.3e}"
        worst = max(worst, ratio)
        if with_a:
            _, yd, bound, _ = oracle.aggregate(n, rows, cols, X[t], threads=4)
            check_y(A[t].cpu().numpy(), yd, bound, f"A, snapshot {t}")
    frame.close()
    return worst


@pytest.mark.parametrize("k,F,Fo", [(4, 64, 64), (8, 32, 16), (3, 16, 48), (2, 48, 32), (5, 64, 16),
                                    (1, 64, 64)])
@pytest.mark.parametrize("with_bias,with_a", [(True, True), (False, False)])
def test_update_fused_into_the_aggregation(pipad, k, F, Fo, with_bias, with_a):
    rng = np.random.default_rng(40 + k + F + Fo)
    n = 1111  # many 16-row tiles per wave and a ragged last one
    lists = churned(rng, n, k, 0.02, 0.8)
    run_update_case(pipad, n, lists, F, Fo, seed=k + F, with_bias=with_bias, with_a=with_a)


def test_update_fused_with_mid_and_hub_rows_and_padded_input_rows(pipad):
    pipad.set_option("short_max", 3)
    pipad.set_option("mid_max", 7)
    pipad.set_option("hub_threshold", 9)
    pipad.set_option("hub_segment", 4)
    rng = np.random.default_rng(4)
    n = 700
    lists = churned(rng, n, 4, 0.03, 0.7)
    run_update_case(pipad, n, lists, 64, 32, seed=1, x_stride=96)
    run_update_case(pipad, n, lists, 32, 64, seed=2, with_a=False)


@pytest.mark.parametrize("k,F,Fo", [(2, 128, 64), (3, 20, 10), (2, 64, 80), (1, 6, 3), (2, 8, 16),
                                    (2, 260, 33), (2, 128, 200), (1, 800, 8)])
def test_update_as_a_second_step_for_other_shapes(pipad, k, F, Fo):
    rng = np.random.default_rng(60 + k + F + Fo)
    n = 530
    lists = churned(rng, n, k, 0.03, 0.8)
    run_update_case(pipad, n, lists, F, Fo, seed=F + Fo)


def test_update_without_workspace_is_refused_for_shapes_that_need_it(pipad):
    rng = np.random.default_rng(8)
    n = 100
    lists = churned(rng, n, 2, 0.05, 0.8)
    dev = "cuda:0"
    snaps = [(torch.from_numpy(rp).to(dev), torch.from_numpy(c).to(dev)) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps)
    xs = [torch.zeros((n, 128), device=dev) for _ in range(2)]
    with pytest.raises(pipad.PipadError) as e:
        pipad.frame_aggregate_update(frame, xs, torch.zeros((128, 16), device=dev))
    assert e.value.status == -1
    frame.close()


def test_symmetric_frames_take_their_backward_pass_through_the_same_entry_point(pipad):
    """For symmetric patterns A^_t is symmetric, so the gradient of the layer H_t = (A^_t X_t) W
    with respect to X_t is A^_t (G_t W^T) = (A^_t G_t) W^T: the same call with W transposed.
    Checked through the adjoint identity <H(X), G> = <X, dX(G)> and against the oracle."""
    rng = np.random.default_rng(17)
    n, k, F, Fo = 640, 3, 32, 48
    lists = churned(rng, n, k, 0.02, 0.8, symmetric=True)
    dev = "cuda:0"
    snaps = [(torch.from_numpy(rp).to(dev), torch.from_numpy(c).to(dev)) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps)
    X = [synth.features(1, t, n, F) for t in range(k)]
    G = [synth.features(2, t, n, Fo) for t in range(k)]
    W = (rng.standard_normal((F, Fo)) / np.sqrt(F)).astype(np.float32)
    Wd = torch.from_numpy(W).to(dev)
    H = pipad.frame_aggregate_update(frame, [torch.from_numpy(x).to(dev) for x in X], Wd)
    dX = pipad.frame_aggregate_update(frame, [torch.from_numpy(g).to(dev) for g in G],
                                      Wd.t().contiguous())
    torch.cuda.synchronize()
    for t in range(k):
        rows, cols = csr_to_coo(n, *lists[t])
        dXd, B2 = oracle.aggregate_update(n, rows, cols, G[t], np.ascontiguousarray(W.T))
        err = np.abs(dX[t].cpu().numpy().astype(np.float64) - dXd)
        assert float(np.max(err / np.maximum(B2, 1e-300))) <= update_tolerance(Fo)
        lhs = float(np.sum(H[t].cpu().numpy().astype(np.float64) * G[t]))
        rhs = float(np.sum(X[t].astype(np.float64) * dX[t].cpu().numpy()))
        scale = float(np.sum(np.abs(X[t].astype(np.float64)) * B2))
        assert abs(lhs - rhs) <= 2 * update_tolerance(max(F, Fo)) * scale
    frame.close()


# ---- transposed frames (the backward operator for directed patterns) ----------------------------
def transpose_csr(n, rowptr, col):
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    order = np.lexsort((rows, col))  # by column, then by row: the transposed CSR's order
    t_rowptr = np.concatenate([[0], np.cumsum(np.bincount(col, minlength=n))]).astype(np.int32)
    return t_rowptr, rows[order].astype(np.int32)


@pytest.mark.parametrize("k,n,p,keep,F,classes", [(3, 300, 0.05, 0.7, 24, None), (1, 64, 0.2, 1.0, 4, None),
                                                  (8, 1500, 0.01, 0.9, 64, None),
                                                  (4, 400, 0.05, 0.7, 16, (2, 8, 4)),
                                                  (4, 400, 0.05, 0.7, 16, (2, 2, 4))])
def test_transposed_frame_of_directed_patterns(pipad, k, n, p, keep, F, classes):
    if classes:
        pipad.set_option("short_max", classes[0])
        pipad.set_option("mid_max", classes[1])
        pipad.set_option("hub_threshold", 12)
        pipad.set_option("hub_segment", classes[2])
    rng = np.random.default_rng(1000 + k + n)
    lists = churned(rng, n, k, p, keep, symmetric=False)
    dev = "cuda:0"
    snaps = [(torch.from_numpy(rp).to(dev), torch.from_numpy(c).to(dev)) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps)
    tframe = pipad.frame_transpose(frame)
    # the parts: bit-exact transposes of the forward frame's parts; D^-1/2 unchanged
    for part in [None] + list(range(k)):
        rp, col = (frame.common() if part is None else frame.delta(part))
        trp, tcol = (tframe.common() if part is None else tframe.delta(part))
        want_rp, want_col = transpose_csr(n, rp.cpu().numpy(), col.cpu().numpy())
        assert np.array_equal(trp.cpu().numpy(), want_rp), f"rowptr of part {part}"
        assert np.array_equal(tcol.cpu().numpy(), want_col), f"columns of part {part}"
    assert torch.equal(frame.dinv(), tframe.dinv())
    frame.close()  # the transposed frame stands on its own
    G = [synth.features(9, t, n, F) for t in range(k)]
    Z = pipad.frame_aggregate(tframe, [torch.from_numpy(g).to(dev) for g in G])
    torch.cuda.synchronize()
    for t in range(k):
        rows, cols = csr_to_coo(n, *lists[t])
        Zd, B = oracle.aggregate_transposed(n, rows, cols, G[t])
        check_y(Z[t].cpu().numpy(), Zd, B, f"transposed snapshot {t}")
    tframe.close()


def test_transposing_a_symmetric_frame_changes_nothing_and_library_allocator_works(pipad):
    rng = np.random.default_rng(3)
    n, k = 500, 3
    lists = churned(rng, n, k, 0.03, 0.8, symmetric=True)
    dev = "cuda:0"
    snaps = [(torch.from_numpy(rp).to(dev), torch.from_numpy(c).to(dev)) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps, allocator="library")
    tframe = pipad.frame_transpose(frame, allocator="library")
    for part in [None] + list(range(k)):
        a = frame.common() if part is None else frame.delta(part)
        b = tframe.common() if part is None else tframe.delta(part)
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    X = [torch.from_numpy(synth.features(4, t, n, 32)).to(dev) for t in range(k)]
    Y1 = pipad.frame_aggregate(frame, X)
    Y2 = pipad.frame_aggregate(tframe, X)
    torch.cuda.synchronize()
    for t in range(k):
        assert torch.equal(Y1[t], Y2[t])
    frame.close()
    tframe.close()


@pytest.mark.parametrize("seed", range(24))
def test_randomised_frames(pipad, seed):
    """Seeded random frames over the whole parameter space of the extraction: node counts from 1 up,
    1 to 32 snapshots, rows from empty to thousands of entries, churn from none to total, directed
    and symmetric patterns, random row-class thresholds.  CSRs bit-exact, aggregation in tolerance."""
    rng = np.random.default_rng(7000 + seed)
    n = int(rng.choice([1, 2, 63, 64, 65, 200, 777, 1500, 2600]))
    k = int(rng.choice([1, 2, 3, 5, 8, 9, 16, 17, 32]))
    if n * n * k > 40_000_000:
        k = max(1, 40_000_000 // (n * n))
    symmetric = bool(rng.integers(2))
    keep = float(rng.choice([0.0, 0.5, 0.9, 0.99, 1.0]))
    dens = np.full((n, 1), float(rng.choice([0.0, 0.002, 0.02, 0.2])))
    hubs = rng.choice(n, min(n, int(rng.integers(0, 4))), replace=False)
    dens[hubs] = float(rng.choice([0.5, 0.95]))
    base = rng.random((n, n)) < dens
    lists = []
    for _ in range(k):
        M = base & (rng.random((n, n)) < keep) | (rng.random((n, n)) < dens * (1 - keep))
        if symmetric:
            M = np.triu(M, 1)
            M = M | M.T
        np.fill_diagonal(M, False)
        rowptr = np.concatenate([[0], np.cumsum(M.sum(axis=1))]).astype(np.int32)
        lists.append((rowptr, np.nonzero(M)[1].astype(np.int32)))
    pipad.set_option("short_max", int(rng.choice([0, 4, 32])))
    pipad.set_option("mid_max", int(rng.choice([0, 16, 256])))
    pipad.set_option("hub_threshold", int(rng.choice([8, 100, 8192])))
    pipad.set_option("hub_segment", int(rng.choice([3, 64, 8192])))
    pipad.set_option("sub_classes", int(rng.choice([1, 2, 4])))
    F = int(rng.choice([1, 4, 7, 16, 64, 96]))
    run_case(pipad, n, lists, F, seed=seed, layout="list" if seed % 2 else "wide")


# ---- sliding frames: inter-frame reuse of first-layer aggregation results ---------------------
@pytest.mark.parametrize("name", ["small", "medium"])
def test_sliding_frames_with_cached_results(pipad, name):
    """Section 3.3 / 4.4: when the frame slides by one snapshot, the first layer's aggregation of
    the k - 1 kept snapshots is unchanged.  Every slid frame of the workload is built; the entering
    snapshot alone is aggregated (pipad_frame_aggregate_subset) into a cache of per-snapshot
    results.  What the subset call writes must equal, bit for bit, what a full aggregation of the
    same frame gives for that snapshot; the results kept from earlier frames were summed in another
    order (an entry may sit in the overlap part of one frame and in an exclusive part of the next),
    so they agree with the full aggregation within twice the parity bound, and every cached result
    is checked against the oracle itself."""
    cfg = synth.CONFIGS[name]
    s = synth.make(cfg)
    n, k, F = cfg.n, cfg.k, cfg.feat
    dev = "cuda:0"
    gs = to_gpu_snapshots(torch, s, range(cfg.snapshots))
    Xh = [synth.features(cfg.seed, t, n, F) for t in range(cfg.snapshots)]
    X = [torch.from_numpy(x).to(dev) for x in Xh]
    cache = [None] * cfg.snapshots
    for f in range(cfg.frames):
        frame = pipad.frame_build_overlap(gs[f:f + k])
        if f < 2:  # the decomposition of a slid frame is as exact as any other
            check_overlap(frame, oracle.overlap(n, [s.coo(t) for t in range(f, f + k)]))
        new = list(range(k)) if f == 0 else [k - 1]
        ys = [None] * k
        for j in new:
            cache[f + j] = torch.full((n, F), float("nan"), device=dev)
            ys[j] = cache[f + j]
        pipad.frame_aggregate_subset(frame, new, [X[f + j] if j in new else None for j in range(k)], ys)
        full = pipad.frame_aggregate(frame, X[f:f + k])
        torch.cuda.synchronize()
        for j in new:
            assert torch.equal(full[j], cache[f + j]), f"frame {f}, snapshot {f + j}"
        kept = [j for j in range(k) if j not in new]
        if kept:
            worst = max(float((full[j] - cache[f + j]).abs().max()) for j in kept)
            assert worst < 1e-4, f"frame {f}: kept results drifted by {worst}"
        frame.close()
    for t in range(cfg.snapshots):
        rows, cols = s.coo(t)
        _, yd, bound, _ = oracle.aggregate(n, rows, cols, Xh[t], threads=8)
        check_y(cache[t].cpu().numpy(), yd, bound, f"cached snapshot {t}")


def test_subset_arguments(pipad):
    import ctypes
    rng = np.random.default_rng(3)
    n, k, F = 120, 4, 8
    lists = churned(rng, n, k, 0.05, 0.8)
    snaps = [(torch.from_numpy(rp).cuda(), torch.from_numpy(c).cuda()) for rp, c in lists]
    frame = pipad.frame_build_overlap(snaps)
    X = [torch.rand((n, F), device="cuda:0") for _ in range(k)]
    Y = [torch.full((n, F), 5.0, device="cuda:0") for _ in range(k)]
    lib = pipad.load_library()
    xp = (ctypes.c_void_p * k)(*[x.data_ptr() for x in X])
    yp = (ctypes.c_void_p * k)(*[y.data_ptr() for y in Y])
    st = torch.cuda.current_stream().cuda_stream
    for bad in ([0, 0], [4], [-1], [0, 1, 2, 3, 0]):
        arr = (ctypes.c_int32 * len(bad))(*bad)
        assert lib.pipad_frame_aggregate_subset(frame._h, len(bad), arr, F, xp, F, yp, F, st) == -1
    # snapshots 2 and 0, in that order; 1 and 3 are left alone
    pipad.frame_aggregate_subset(frame, [2, 0], X, Y)
    full = pipad.frame_aggregate(frame, X)
    torch.cuda.synchronize()
    assert torch.equal(Y[2], full[2]) and torch.equal(Y[0], full[0])
    assert torch.all(Y[1] == 5.0) and torch.all(Y[3] == 5.0)
    frame.close()
