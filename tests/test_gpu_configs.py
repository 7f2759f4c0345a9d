"""The five benchmark configurations at full size, in the launch configuration bench.py times
(library defaults), against the CPU oracle run over the whole array (about a second each)."""
import numpy as np
import pytest

import oracle
from paper_1903_03640_amd import redux, workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4
_cache = {}


def config_data(name):
    """(host array, device tensor, oracle result) for one configuration; kept for both variants."""
    if name not in _cache:
        _cache.clear()                                   # one configuration resident at a time
        cfg = workloads.CONFIGS[name]
        host = workloads.make(cfg)
        if cfg.segmented:
            want = oracle.sum_segmented_f16(host, cfg.nseg, cfg.seglen)
        elif cfg.dtype == "f16":
            want = oracle.sum_f16(host)
            exact = oracle.sum_f16_exact(host)
            assert abs(want[0] - exact[0]) <= 1e-12 * exact[1]     # the oracle's own cross-check at full size
        else:
            want = oracle.sum_i8(host)
        _cache[name] = (cfg, host, torch.from_numpy(host).to("cuda:0"), want)
    return _cache[name]


@pytest.fixture(scope="module", autouse=True)
def _setup():
    assert torch.cuda.is_available()
    redux.load()
    torch.cuda.set_device(0)
    yield
    _cache.clear()
    redux.set_variant("auto")


@pytest.mark.parametrize("variant", ["auto", "mfma", "classic"])
@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_f16_configs(name, variant):
    cfg, host, x, (want, want_abs) = config_data(name)
    redux.set_variant(variant)
    got = redux.sum(x)
    torch.cuda.synchronize()
    got = float(got.item())
    print("%s %s: gpu %.6f oracle %.6f sum|x| %.6g err/sum|x| %.3g" % (name, variant, got, want, want_abs, abs(got - want) / want_abs))
    assert abs(got - want) <= TOL * want_abs
    if name in ("C1", "C3"):                             # non-negative data: the relative form of the bar
        assert abs(got - want) <= TOL * abs(want)


@pytest.mark.parametrize("variant", ["auto", "mfma", "classic"])
def test_i8_config(variant):
    cfg, host, x, (want, _) = config_data("C4")
    redux.set_variant(variant)
    got = redux.sum(x)
    torch.cuda.synchronize()
    assert int(got.item()) == want


@pytest.mark.parametrize("variant", ["auto", "mfma", "classic"])
def test_segmented_config(variant):
    cfg, host, x, (want, want_abs) = config_data("C5")
    redux.set_variant(variant)
    got = redux.sum_segmented(x, cfg.nseg, cfg.seglen)
    torch.cuda.synchronize()
    got = got.cpu().numpy().astype(np.float64)
    assert got.shape == (cfg.nseg,)
    assert np.all(np.abs(got - want) <= TOL * want_abs)
    print("C5 %s: worst err/sum|x| %.3g" % (variant, np.max(np.abs(got - want) / want_abs)))


@pytest.mark.parametrize("variant", ["auto", "mfma", "classic"])
def test_full_size_arrays_as_a_few_long_segments(variant):
    """The arrays of C5 and C4 at full size, read as a handful of long segments: every segment is cut into pieces, one
    block each, whose totals meet in the same kernel (the library's choice: a block for every piece) or, when asked
    for, in a second one."""
    redux.set_variant(variant)
    try:
        cfg, host, x, _ = config_data("C5")
        n = cfg.nseg * cfg.seglen
        for nseg in (16, 128, 1):
            seglen = n // nseg
            want, want_abs = oracle.sum_segmented_f16(host, nseg, seglen)
            for seg_finish, finish in ((-1, 6), (0, 2)):
                redux.set_param("seg_finish", seg_finish)
                plan = redux.plan_sum_segmented(nseg, seglen, redux.F16, x.data_ptr(), 256)
                assert plan.kernel == redux.KERNEL_BLOCK and plan.parts > 1 and plan.finish == finish, (nseg, plan.parts, plan.finish)
                got = redux.sum_segmented(x, nseg, seglen)
                torch.cuda.synchronize()
                assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - want) <= TOL * want_abs), (nseg, seg_finish)
        cfg, host, x, _ = config_data("C4")
        for nseg in (64, 4):
            seglen = cfg.n // nseg
            want = oracle.sum_segmented_i8(host, nseg, seglen)[0]
            for seg_finish, finish in ((-1, 5), (0, 2)):
                redux.set_param("seg_finish", seg_finish)
                plan = redux.plan_sum_segmented(nseg, seglen, redux.I8, x.data_ptr(), 256)
                assert plan.kernel == redux.KERNEL_BLOCK and plan.parts > 1 and plan.finish == finish, (nseg, plan.parts, plan.finish)
                got = redux.sum_segmented(x, nseg, seglen)
                torch.cuda.synchronize()
                assert np.array_equal(got.cpu().numpy(), want), (nseg, seg_finish)
    finally:
        redux.set_param("seg_finish", -1)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
def test_multipass_configs(name):
    """The level-by-level form at full size: result and number of launches."""
    from oracle import mma_reduction as mr
    cfg, host, x, want = config_data(name)
    out, levels = redux.sum_multipass(x)
    torch.cuda.synchronize()
    if cfg.dtype == "i8":
        assert int(out.item()) == want[0]
        assert levels == 1 + mr.expected_levels(-(-cfg.n // 512), 256)
    else:
        assert abs(float(out.item()) - want[0]) <= TOL * want[1]
        assert levels == mr.expected_levels(cfg.n, 256)
        print("%s multipass: levels %d err/sum|x| %.3g" % (name, levels, abs(float(out.item()) - want[0]) / want[1]))


@pytest.mark.parametrize("variant", ["mfma", "classic"])
def test_more_than_2_to_32_elements(variant):
    """64-bit indexing: closed forms on arrays longer than 2^32 elements (int8) and 2^32 bytes (binary16)."""
    _cache.clear()
    redux.set_variant(variant)
    n = (1 << 32) + 12345
    x = torch.ones(n, dtype=torch.int8, device="cuda:0")
    x[n - 1] = -100
    x[1 << 32] = 7
    got = redux.sum(x)
    nseg = 3
    seg = redux.sum_segmented(x[: nseg * ((1 << 30) + 5)], nseg, (1 << 30) + 5)      # three segments of 2^30 + 5
    torch.cuda.synchronize()
    assert int(got.item()) == n - 2 + 7 - 100
    assert seg.cpu().tolist() == [(1 << 30) + 5] * 3
    del x
    h = torch.full(((1 << 31) + 7,), 0.5, dtype=torch.float16, device="cuda:0")       # 4 GiB + 14 B
    h[-1] = 1024.0
    got = redux.sum(h)
    torch.cuda.synchronize()
    want = 0.5 * ((1 << 31) + 6) + 1024.0
    assert abs(float(got.item()) - want) <= 1e-4 * want
    del h
