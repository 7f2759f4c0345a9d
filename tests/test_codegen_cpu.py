"""What the compiler made of the kernels, checked without a GPU: the device code is compiled to gfx950 assembly
and a few properties that decide the speed of the memory-bound loops are read off it.

Each of these was once broken by an innocent-looking source change and cost 30-50 % of a kernel's bandwidth:

  * no flat loads or stores: an address built by integer arithmetic loses its address space, the load becomes a
    flat load, a flat load counts as an LDS operation too, and every wait for an LDS read then waits for all
    loads in flight;
  * no scratch memory (register spills) in any kernel;
  * the software-pipelined kernels wait for the oldest of eight loads in flight (`s_waitcnt vmcnt(7)`): a load
    under a branch, or loads issued in another order than they are consumed in, turns that into vmcnt(0);
  * register counts stay where several blocks fit a compute unit.
"""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import __graft_entry__ as entry  # noqa: E402


@pytest.fixture(scope="module")
def kernels(tmp_path_factory):
    """{demangled-ish kernel name: (assembly text, vgpr count, scratch bytes)}"""
    if not os.path.exists(entry.HIPCC):
        pytest.skip("hipcc not found")
    out = tmp_path_factory.mktemp("asm") / "redux_api.s"
    flags = [f for f in entry.HIP_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [entry.HIPCC] + flags + ["--cuda-device-only", "-S", "-I", os.path.join(ROOT, "include"), "-o", str(out),
                                   os.path.join(entry.PKG, "csrc", "redux_api.hip")]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = out.read_text()
    bodies = {}
    for m in re.finditer(r"^(_ZN5redux\w+):.*?^\.Lfunc_end\d+:", text, re.S | re.M):
        bodies[m.group(1)] = m.group(0)
    meta = {}
    for m in re.finditer(r"\.name:\s+(_ZN5redux\w+)\n(.*?)(?=\n  - \.a|\namdhsa\.target|\Z)", text, re.S):
        block = m.group(2)
        vg = re.search(r"\.vgpr_count:\s+(\d+)", block)
        sc = re.search(r"\.private_segment_fixed_size:\s+(\d+)", block)
        if vg and sc:
            meta[m.group(1)] = (int(vg.group(1)), int(sc.group(1)))
    assert len(bodies) > 100 and set(bodies) <= set(meta) | set(bodies)
    return {k: (bodies[k],) + meta.get(k, (None, None)) for k in bodies}


def pick(kernels, *parts):
    hit = [k for k in kernels if all(p in k for p in parts)]
    assert hit, parts
    return hit


def test_no_flat_memory_instructions_and_no_scratch(kernels):
    for name, (body, vgprs, scratch) in kernels.items():
        assert "flat_load" not in body and "flat_store" not in body and "flat_atomic" not in body, name
        assert "scratch_" not in body, name
        if scratch is not None:
            assert scratch == 0, (name, scratch)


def test_pipelined_kernels_wait_for_the_oldest_load_only(kernels):
    # the short-segment kernels of the MMA family (aligned and ragged form, every element type) refill a register as
    # soon as it is consumed: eight uses per loop trip, each behind a wait that leaves the seven newer loads outstanding
    # (the classic family's stores sit under a branch between the loads, so the compiler cannot count as finely there)
    for name in pick(kernels, "sum_short_mfma_kernel"):
        body = kernels[name][0]
        waits = len(re.findall(r"s_waitcnt vmcnt\((7|8)\)", body))       # 8: one result store is outstanding as well
        assert waits >= 8, (name, waits)


def test_streaming_loops_issue_all_loads_before_the_first_wait(kernels):
    # flat sum, eight loads per lane: the loop body has eight global loads in a row with no wait between them
    for name in pick(kernels, "sum_flat_kernel", "Li8ELb1E"):
        body = kernels[name][0]
        runs = re.findall(r"(?:\s+global_load_dwordx4[^\n]*\n(?:\s+(?:v_|s_(?!waitcnt))[^\n]*\n)*){8}", body)
        assert runs, name


def test_run_kernels_wait_for_the_oldest_load_first(kernels):
    # run-of-segments kernels: U loads per iteration, and the first use waits for the oldest of them only
    # (vmcnt(U - 1)): everything about a run is wavefront-uniform, so no load sits under a lane-dependent branch
    for u in (4, 8):
        for name in pick(kernels, "sum_segment_runs_mfma_kernel", "Li%dELb1E" % u):
            body = kernels[name][0]
            assert re.search(r"s_waitcnt vmcnt\(%d\)" % (u - 1), body), name
            # the boundaries are walked in scalar registers: scalar branches outnumber the lane-mask ones (the classic
            # family's "lane 0 stores" among them) by far
            assert body.count("s_cbranch_scc") > 2 * body.count("s_cbranch_exec"), name


def test_rolling_run_kernel_keeps_its_loads_in_flight(kernels):
    # the rolling form reloads every register right after its use: inside its main loop every wait in front of a use
    # leaves the U - 1 younger loads in flight (vmcnt(U - 1), at least once per register), and a reload follows each use
    for u in (4, 8):
        for name in pick(kernels, "sum_segment_runs_mfma_stream_kernel", "Li%dELb1E" % u) + pick(kernels, "sum_segment_runs_classic_stream_kernel", "Li%dELb1E" % u):
            body = kernels[name][0]
            loop = body[body.index("Loop Header: Depth=1"):]
            first_reloads = loop[:loop.index("global_store")]            # the main loop up to the store at the end of a pass
            assert len(re.findall(r"s_waitcnt vmcnt\(%d\)" % (u - 1), first_reloads)) >= u, name
            assert len(re.findall(r"global_load_dwordx4", first_reloads)) == u, name
            assert not re.search(r"s_waitcnt vmcnt\(0\)", first_reloads), name
            assert body.count("s_cbranch_scc") > 2 * body.count("s_cbranch_exec"), name


def test_register_counts(kernels):
    for name in pick(kernels, "sum_segment_runs_"):
        assert kernels[name][1] <= 128, (name, kernels[name][1])       # four blocks per compute unit fit

    for name in pick(kernels, "sum_flat_kernel"):
        assert kernels[name][1] <= 128, (name, kernels[name][1])
    for name in pick(kernels, "sum_short_classic_kernel"):
        assert kernels[name][1] <= 128, (name, kernels[name][1])       # at least four blocks per compute unit
    for name in pick(kernels, "sum_short_mfma_kernel"):
        assert kernels[name][1] <= 160, (name, kernels[name][1])
    for name in pick(kernels, "sum_segmented_kernel"):
        assert kernels[name][1] <= 128, (name, kernels[name][1])
