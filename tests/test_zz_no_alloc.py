"""pipad_frame_aggregate_static (the entry point for callers that cannot allocate) against
pipad_frame_aggregate, through the C ABI: same kernels, so the outputs must agree bit for bit (which
is inside the 1e-5 * |A^||X| parity bar), on two calls in a row that share the GPU's fixed scratch
array, the second with a smaller input; and against the CPU oracle."""
import ctypes

import numpy as np
import pytest

import oracle
import synth
from _util import check_y, csr_to_coo

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def pipad():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2301_00391_amd as p
    p.load_library()
    return p


def churned(rng, n, k, p, keep):
    base = rng.random((n, n)) < p
    out = []
    for _ in range(k):
        M = base & (rng.random((n, n)) < keep) | (rng.random((n, n)) < p * (1 - keep))
        M = np.triu(M, 1)
        M = M | M.T
        rowptr = np.concatenate([[0], np.cumsum(M.sum(axis=1))]).astype(np.int32)
        out.append((rowptr, np.nonzero(M)[1].astype(np.int32)))
    return out


def build_frame_abi(lib, binding, lists, n):
    """pipad_frame_build_overlap through ctypes with the library's own allocator."""
    k = len(lists)
    snaps = [(torch.from_numpy(rp).cuda(), torch.from_numpy(c).cuda()) for rp, c in lists]
    arr = (binding._Csr * k)()
    for t, (rp, col) in enumerate(snaps):
        arr[t].n, arr[t].nnz = n, col.numel()
        arr[t].rowptr, arr[t].colidx = rp.data_ptr(), col.data_ptr() if col.numel() else None
    out = ctypes.c_void_p()
    stream = torch.cuda.current_stream().cuda_stream
    rc = lib.pipad_frame_build_overlap(n, k, arr, 0, None, None, stream, ctypes.byref(out))
    assert rc == 0, rc
    torch.cuda.synchronize()
    return out, snaps


def both_entry_points(lib, frame, X, n, k, F):
    """(Y of pipad_frame_aggregate, Y of pipad_frame_aggregate_static), k matrices each."""
    stream = torch.cuda.current_stream().cuda_stream
    xp = (ctypes.c_void_p * k)(*[x.data_ptr() for x in X])
    outs = []
    for fn in (lib.pipad_frame_aggregate, lib.pipad_frame_aggregate_static):
        Y = [torch.full((n, F), float("nan"), device="cuda:0") for _ in range(k)]
        yp = (ctypes.c_void_p * k)(*[y.data_ptr() for y in Y])
        rc = fn(frame, F, xp, F, yp, F, stream)
        assert rc == 0, (fn.__name__, rc)
        torch.cuda.synchronize()
        outs.append(Y)
    return outs


def test_static_scratch_entry_point_matches_the_allocating_one(pipad):
    from paper_2301_00391_amd import binding
    lib = pipad.load_library()
    saved = {key: pipad.get_option(key) for key in ("short_max", "mid_max", "hub_threshold", "hub_segment")}
    try:
        # low thresholds: most rows are split (mid rows, hub rows, hub rows cut into units), so
        # the scratch array is really used
        pipad.set_option("short_max", 8)
        pipad.set_option("mid_max", 20)
        pipad.set_option("hub_threshold", 24)
        pipad.set_option("hub_segment", 16)
        rng = np.random.default_rng(2024)
        # two calls in a row on the same GPU: the second, smaller one finds the first one's partial
        # sums still in the array
        for n, k, F, p in ((900, 4, 32, 0.03), (310, 3, 16, 0.05)):
            lists = churned(rng, n, k, p, 0.8)
            frame, _snaps = build_frame_abi(lib, binding, lists, n)
            Xh = [synth.features(11, t, n, F) for t in range(k)]
            X = [torch.from_numpy(x).cuda() for x in Xh]
            y_alloc, y_static = both_entry_points(lib, frame, X, n, k, F)
            for t in range(k):
                assert torch.equal(y_alloc[t], y_static[t]), f"n={n}: snapshot {t} differs"
                rows, cols = csr_to_coo(n, *lists[t])
                _, yd, bound, _ = oracle.aggregate(n, rows, cols, Xh[t], threads=4)
                check_y(y_static[t].cpu().numpy(), yd, bound, f"static, n={n}, snapshot {t}")
            lib.pipad_frame_destroy(frame)
    finally:
        for key, val in saved.items():
            pipad.set_option(key, val)


def test_static_scratch_entry_point_takes_the_snapshots_in_groups(pipad):
    """A frame whose partial sums fit the fixed array for one snapshot (about 5 k units x 8 classes
    x 128 floats = 20 MB) but not for all 8: the call goes through the snapshots in groups of
    three, one launch after the other, and still gives the bits of the allocating entry point."""
    from paper_2301_00391_amd import binding
    lib = pipad.load_library()
    saved = {key: pipad.get_option(key) for key in ("short_max", "mid_max", "hub_threshold", "hub_segment")}
    try:
        pipad.set_option("short_max", 0)
        pipad.set_option("mid_max", 0)
        pipad.set_option("hub_threshold", 1)
        pipad.set_option("hub_segment", 1)
        rng = np.random.default_rng(6)
        n, k, F = 1000, 8, 128
        lists = churned(rng, n, k, 0.005, 0.9)
        frame, _snaps = build_frame_abi(lib, binding, lists, n)
        Xh = [synth.features(12, t, n, F) for t in range(k)]
        X = [torch.from_numpy(x).cuda() for x in Xh]
        y_alloc, y_static = both_entry_points(lib, frame, X, n, k, F)
        for t in range(k):
            assert torch.equal(y_alloc[t], y_static[t]), f"snapshot {t} differs"
        for t in (0, k - 1):
            rows, cols = csr_to_coo(n, *lists[t])
            _, yd, bound, _ = oracle.aggregate(n, rows, cols, Xh[t], threads=4)
            check_y(y_static[t].cpu().numpy(), yd, bound, f"static in groups, snapshot {t}")
        lib.pipad_frame_destroy(frame)
    finally:
        for key, val in saved.items():
            pipad.set_option(key, val)


def test_static_scratch_entry_point_recorded_into_a_hip_graph_without_an_eager_call(pipad):
    """What the entry point is for: a fresh frame (its own scratch buffer was never sized) goes
    straight into a stream capture; every replay, with eager work and synchronisations in between,
    must give the bits of the eager allocating call."""
    saved = {key: pipad.get_option(key) for key in ("short_max", "mid_max", "hub_threshold", "hub_segment")}
    try:
        pipad.set_option("short_max", 2)
        pipad.set_option("mid_max", 5)
        pipad.set_option("hub_threshold", 6)
        pipad.set_option("hub_segment", 4)
        rng = np.random.default_rng(123)
        n, k, F = 700, 3, 64
        lists = churned(rng, n, k, 0.03, 0.8)
        dev = "cuda:0"
        snaps = [(torch.from_numpy(rp).to(dev), torch.from_numpy(c).to(dev)) for rp, c in lists]
        frame = pipad.frame_build_overlap(snaps)
        other = pipad.frame_build_overlap(snaps)  # for the eager reference
        X = [torch.from_numpy(synth.features(7, t, n, F)).to(dev) for t in range(k)]
        Y = [torch.empty_like(x) for x in X]
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            pipad.frame_aggregate(frame, X, Y, static_scratch=True)
        for replay in range(3):
            for t in range(k):
                X[t].copy_(torch.from_numpy(synth.features(200 + replay, t, n, F)))
            want = [y.clone() for y in pipad.frame_aggregate(other, X)]
            torch.cuda.synchronize()
            for y in Y:
                y.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            for t in range(k):
                assert torch.equal(Y[t], want[t]), f"replay {replay}, snapshot {t}"
        frame.close()
        other.close()
    finally:
        for key, val in saved.items():
            pipad.set_option(key, val)


def test_static_scratch_entry_point_rejects_what_does_not_fit(pipad):
    from paper_2301_00391_amd import binding
    lib = pipad.load_library()
    saved = {key: pipad.get_option(key) for key in ("short_max", "mid_max", "hub_threshold", "hub_segment")}
    try:
        # every entry a unit of its own: about 20 k units x 8 classes x F = 128 floats for ONE
        # snapshot > 64 MiB
        pipad.set_option("short_max", 0)
        pipad.set_option("mid_max", 0)
        pipad.set_option("hub_threshold", 1)
        pipad.set_option("hub_segment", 1)
        rng = np.random.default_rng(5)
        n, k, F = 2000, 8, 128
        lists = churned(rng, n, k, 0.005, 1.0)
        frame, _snaps = build_frame_abi(lib, binding, lists, n)
        X = [torch.zeros((n, F), device="cuda:0") for _ in range(k)]
        Y = [torch.full((n, F), 3.0, device="cuda:0") for _ in range(k)]
        xp = (ctypes.c_void_p * k)(*[x.data_ptr() for x in X])
        yp = (ctypes.c_void_p * k)(*[y.data_ptr() for y in Y])
        stream = torch.cuda.current_stream().cuda_stream
        rc = lib.pipad_frame_aggregate_static(frame, F, xp, F, yp, F, stream)
        torch.cuda.synchronize()
        assert rc == -6, rc
        assert lib.pipad_strerror(rc).startswith(b"the fixed scratch")
        assert all(torch.all(y == 3.0) for y in Y), "nothing may be enqueued on rejection"
        # the allocating entry point still takes the same frame
        assert lib.pipad_frame_aggregate(frame, F, xp, F, yp, F, stream) == 0
        torch.cuda.synchronize()
        lib.pipad_frame_destroy(frame)
    finally:
        for key, val in saved.items():
            pipad.set_option(key, val)
