"""redux_sum_static, the entry point that allocates nothing (its block partials and ticket live in a static array in
device memory): called through the C ABI and compared with redux_sum on the same input -- bit for bit for int8, and
for the floating-point types too, since both run the same kernels with the same launch shape -- and against the CPU
oracle; two calls in a row, the second on a smaller input, so that what the first call left in the array is there
when the second one starts."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_1903_03640_amd import redux, workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available()
    redux.load()
    torch.cuda.set_device(0)
    yield torch.device("cuda:0")
    redux.set_variant("auto")


@pytest.fixture(autouse=True)
def reset():
    yield
    for name, val in (("max_grid", 16384), ("blocks_per_cu", 1), ("finish", -1), ("unroll", 0)):
        redux.set_param(name, val)
    redux.set_variant("auto")


def both(x, dtype_code, out_dtype, dev):
    """(redux_sum_static, redux_sum) results of one input as 0-d host arrays"""
    stream = torch.cuda.current_stream().cuda_stream
    a = torch.full((1,), -77, dtype=out_dtype, device=dev)
    b = torch.full((1,), -77, dtype=out_dtype, device=dev)
    lib = redux.load()
    assert lib.redux_sum_static(x.data_ptr(), x.numel(), dtype_code, a.data_ptr(), stream) == 0
    assert lib.redux_sum(x.data_ptr(), x.numel(), dtype_code, b.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    return a.cpu().numpy()[0], b.cpu().numpy()[0]


@pytest.mark.parametrize("variant", ("auto", "mfma", "classic"))
@pytest.mark.parametrize("finish", (-1, 1, 2, 3, 4, 5, 6, 7, 8))
def test_static_matches_redux_sum_two_calls_in_a_row(dev, variant, finish):
    redux.set_variant(variant)
    redux.set_param("finish", finish)
    # the first, larger input leaves 256 block partials (and a used ticket) behind; the second uses fewer blocks
    sizes = ((1 << 24) + 12345, (1 << 18) + 77, 1000, (1 << 22) + 1, 5)
    for k, n in enumerate(sizes):
        xh = workloads.normal_f16(100 + k, n)
        x = torch.from_numpy(xh).to(dev)
        got, ref = both(x, redux.F16, torch.float32, dev)
        want, want_abs = oracle.sum_f16(xh)
        assert abs(float(got) - want) <= TOL * want_abs, (n, got, want)
        if finish != 3:                                          # atomic additions: the order of arrival decides the last bits
            assert got.view(np.uint32) == ref.view(np.uint32), (n, got, ref)
        ih = workloads.uniform_i8(200 + k, n)
        xi = torch.from_numpy(ih).to(dev)
        goti, refi = both(xi, redux.I8, torch.int64, dev)
        assert int(goti) == int(refi) == oracle.sum_i8(ih)[0], (n, goti, refi)


def test_static_alternating_inputs_and_other_dtypes(dev):
    """Back-to-back calls on one stream, alternating between two arrays of different size: every call must see its own
    partials, not what the previous call left in the array."""
    a, b = workloads.uniform_i8(31, (1 << 23) + 5), workloads.uniform_i8(32, (1 << 20) + 3)
    wa, wb = oracle.sum_i8(a)[0], oracle.sum_i8(b)[0]
    xa, xb = torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev)
    outs = torch.zeros(100, dtype=torch.int64, device=dev)
    lib, stream = redux.load(), torch.cuda.current_stream().cuda_stream
    for k in range(100):
        x = xa if k % 2 == 0 else xb
        assert lib.redux_sum_static(x.data_ptr(), x.numel(), redux.I8, outs[k:].data_ptr(), stream) == 0
    torch.cuda.synchronize()
    got = outs.cpu().numpy()
    assert np.all(got[0::2] == wa) and np.all(got[1::2] == wb)
    for code, tdt in ((redux.BF16, torch.bfloat16), (redux.F32, torch.float32), (redux.F8E4M3, torch.float8_e4m3fn)):
        x = (torch.randn((1 << 21) + 9, device=dev) * 0.5).to(tdt)
        g, r = both(x, code, torch.float32, dev)
        assert g.view(np.uint32) == r.view(np.uint32)


def test_static_limits_and_errors(dev):
    lib = redux.load()
    x = torch.zeros(1 << 24, dtype=torch.int8, device=dev)
    out = torch.zeros(1, dtype=torch.int64, device=dev)
    # more block partials than the static array holds: refused, nothing launched, out untouched
    redux.set_param("blocks_per_cu", 16)
    redux.set_param("unroll", 1)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    want_grid = min((1 << 24) // 16 // 256, cus * 16)
    out.fill_(123)
    rc = lib.redux_sum_static(x.data_ptr(), x.numel(), redux.I8, out.data_ptr(), 0)
    torch.cuda.synchronize()
    if want_grid > 2048:
        assert rc == -9 and out.item() == 123
        assert b"static" in lib.redux_strerror(rc)
        assert lib.redux_sum(x.data_ptr(), x.numel(), redux.I8, out.data_ptr(), 0) == 0     # the allocating entry point takes it
    else:
        assert rc == 0 and out.item() == 0
    redux.set_param("max_grid", 2048)                            # exactly at the limit: accepted
    assert lib.redux_sum_static(x.data_ptr(), x.numel(), redux.I8, out.data_ptr(), 0) == 0
    torch.cuda.synchronize()
    assert out.item() == 0
    # the usual argument checks, and the empty sum
    assert lib.redux_sum_static(None, 5, redux.I8, out.data_ptr(), 0) == -1
    assert lib.redux_sum_static(x.data_ptr(), 5, 17, out.data_ptr(), 0) == -2
    assert lib.redux_sum_static(x.data_ptr(), 5, redux.I8, x.data_ptr() + 1, 0) in (-4, -7)
    out.fill_(9)
    assert lib.redux_sum_static(None, 0, redux.I8, out.data_ptr(), 0) == 0
    torch.cuda.synchronize()
    assert out.item() == 0


def test_static_replays_from_a_graph(dev):
    """The entry point allocates nothing, so after one eager call on the device (which looks up the array's address)
    it can be captured without a warm-up on the capture stream; replays match the eager result."""
    n = (1 << 22) + 321
    xh = workloads.normal_f16(55, n)
    x = torch.from_numpy(xh).to(dev)
    out = torch.zeros(1, dtype=torch.float32, device=dev)
    lib = redux.load()
    assert lib.redux_sum_static(x.data_ptr(), n, redux.F16, out.data_ptr(), torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    eager = out.clone()
    stream = torch.cuda.Stream()                                 # never used by the library before
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        assert lib.redux_sum_static(x.data_ptr(), n, redux.F16, out.data_ptr(), torch.cuda.current_stream().cuda_stream) == 0
    for rep in range(4):
        out.fill_(-1)
        redux.sum(x)                                             # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
    want, want_abs = oracle.sum_f16(xh)
    assert abs(eager.item() - want) <= TOL * want_abs
