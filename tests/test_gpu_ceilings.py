"""The measurement kernels of include/pipad_ceilings.h through the C ABI: the copy copies, the
gather gathers what the index says (its sink sums are recomputed on the host), bad arguments are
refused before anything is enqueued."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def lib():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2301_00391_amd as p
    return p.load_library()


def stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def test_stream_copy_and_read(lib):
    gen = torch.Generator(device="cpu").manual_seed(1)
    for floats in (4, 1 << 20, (1 << 22) + 4 * 37):  # one piece, whole strides, a ragged tail
        src = torch.randn(floats, generator=gen).cuda()
        dst = torch.zeros_like(src)
        assert lib.pipad_ceiling_stream_copy(src.data_ptr(), dst.data_ptr(), floats * 4, stream()) == 0
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
    sink = torch.zeros(lib.pipad_ceiling_sink_floats(), device="cuda:0")
    ones = torch.ones(1 << 20, device="cuda:0")
    assert lib.pipad_ceiling_stream_read(ones.data_ptr(), ones.numel() * 4, sink.data_ptr(), stream()) == 0
    torch.cuda.synchronize()
    assert float(sink.sum()) == ones.numel()  # every float was read exactly once
    # refused: odd size, misaligned pointer, overlapping buffers, null
    a = torch.zeros(1024, device="cuda:0")
    assert lib.pipad_ceiling_stream_copy(a.data_ptr(), a.data_ptr() + 2048, 2052, stream()) == -1
    assert lib.pipad_ceiling_stream_copy(a.data_ptr() + 4, a.data_ptr() + 2048, 1024, stream()) == -1
    assert lib.pipad_ceiling_stream_copy(a.data_ptr(), a.data_ptr() + 1024, 2048, stream()) == -1
    assert lib.pipad_ceiling_stream_copy(None, a.data_ptr(), 16, stream()) == -1
    assert lib.pipad_ceiling_stream_read(a.data_ptr(), 20, sink.data_ptr(), stream()) == -1


@pytest.mark.parametrize("row_floats,stride", [(64, 64), (64, 96), (32, 32), (16, 16)])
@pytest.mark.parametrize("classes", [0, 8])
def test_gather_sums_what_the_index_names(lib, row_floats, stride, classes):
    rng = np.random.default_rng(row_floats + classes)
    rows, count = 5000, 8 * 4096 * 2
    table = rng.integers(-8, 8, size=(rows, stride)).astype(np.float32)  # small integers: exact sums
    index = rng.integers(0, rows, size=count).astype(np.int32)
    t = torch.from_numpy(table).cuda()
    idx = torch.from_numpy(index).cuda()
    sink = torch.zeros(lib.pipad_ceiling_sink_floats(), device="cuda:0")
    rc = lib.pipad_ceiling_gather(t.data_ptr(), rows, row_floats, stride, idx.data_ptr(), count, classes,
                                  sink.data_ptr(), stream())
    assert rc == 0
    torch.cuda.synchronize()
    # the lane that reports holds the first four floats of the rows its lane team gathered: the
    # entries at positions 0, NT, 2 NT, ... of every 64-entry chunk (NT = 64 / lanes per row)
    nt = 64 // (row_floats // 4)
    mine = index.reshape(-1, 64)[:, ::nt].reshape(-1)
    want = float(table[mine, :4].sum())
    waves = count // 1024
    assert float(sink[:waves].sum()) == want
    assert float(sink[waves:].abs().sum()) == 0.0


def test_gather_refuses_bad_arguments(lib):
    t = torch.zeros((64, 64), device="cuda:0")
    idx = torch.zeros(8 * 4096, dtype=torch.int32, device="cuda:0")
    sink = torch.zeros(lib.pipad_ceiling_sink_floats(), device="cuda:0")
    ok = dict(rows=64, row_floats=64, stride=64, count=8 * 4096, classes=8)

    def call(**kw):
        a = {**ok, **kw}
        return lib.pipad_ceiling_gather(t.data_ptr(), a["rows"], a["row_floats"], a["stride"], idx.data_ptr(),
                                        a["count"], a["classes"], sink.data_ptr(), stream())
    assert call() == 0
    assert call(row_floats=48) == -1      # 16, 32 or 64 only
    assert call(stride=32) == -1          # shorter than a row
    assert call(count=4096) == -1         # not a multiple of 8 workgroups with classes
    assert call(count=4096, classes=0) == 0
    assert call(count=1000, classes=0) == -1
    assert call(classes=4) == -1
    assert call(rows=0) == -1
    torch.cuda.synchronize()
