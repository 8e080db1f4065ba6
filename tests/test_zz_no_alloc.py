"""The allocation-free fused step (sdl_fragment_outer_step_plan_static) against the entry point it
is a variant of (sdl_fragment_outer_step_plan_ex with caller-provided scale words): same results
bit for bit, on two calls in a row that share the library's device array, the second on a smaller
fragment; and against the oracle to the usual bars."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_18512_amd as sdl
import workloads
from gpu_util import HostCopy, assert_bf16_within_ulp, assert_f32_close, host_bits, host_f32

DEV = "cuda"


def _plan(numel, n_blocks, P):
    block = [i % n_blocks for i in range(len(numel))]
    return sdl.sdl_fragment_plan(numel, block, n_blocks, P, sdl.PATTERN_STRIDED, 100, 1)


def _run_pair(plan, p, M, fmt, seed):
    """One fragment through both entry points on identical copies of the same state."""
    total = plan.total_numel
    g, mom, w_send, w_now = workloads.make_span(total, M, tau=1, delta="student_t3", base_seed=seed, device=DEV)
    mom.copy_(torch.randn(total, device=DEV, generator=torch.Generator(DEV).manual_seed(seed)) * 1e-4)
    host = HostCopy(g, mom, w_send, w_now)
    g2, mom2, w_now2 = g.clone(), mom.clone(), [w.clone() for w in w_now]
    words = None
    if fmt == sdl.FMT_E3M0_SPAN:
        sb = sdl.sdl_plan_message_bytes(plan, p, fmt)[1]
        # poison: the existing entry point clears its scale words itself
        words = [torch.full((max(sb, 4),), 0xff, dtype=torch.uint8, device=DEV) for _ in range(M)]
    sdl.sdl_fragment_outer_step_plan_ex(plan, p, g, mom, w_send, w_now, fmt, 0.7, 0.9, 0.5, None, words)
    sdl.sdl_fragment_outer_step_plan_static(plan, p, g2, mom2, w_send, w_now2, fmt, 0.7, 0.9, 0.5)
    torch.cuda.synchronize()
    assert torch.equal(g.view(torch.int32), g2.view(torch.int32)), "g differs between the two entry points"
    assert torch.equal(mom.view(torch.int32), mom2.view(torch.int32)), "mom differs between the two entry points"
    for a, b in zip(w_now, w_now2):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "a replica differs between the two entry points"
    # and both against the oracle, span by span (one scale per span)
    for off, n, _ in sdl.sdl_plan_fragment_spans(plan, p):
        sl = slice(off, off + n)
        oracle.fragment_outer_step(host.g[sl], host.mom[sl], [w[sl] for w in host.w_send],
                                   [w[sl] for w in host.w_now], fmt, 0.7, 0.9, 0.5)
    assert_f32_close(host_f32(g2), host.g, "static g")
    assert_f32_close(host_f32(mom2), host.mom, "static mom")
    for m in range(M):
        assert_bf16_within_ulp(host_bits(w_now2[m]), host.w_now[m], f"static w_now[{m}]")


@pytest.mark.gpu
def test_static_entry_point_matches_workspace_entry_point_twice():
    rng = np.random.default_rng(11)
    # first call: 3 fragments over 7 blocks, 40 ragged spans, 4 replicas -- many spans per fragment,
    # tiles of several runs, ragged tails
    big = _plan([int(x) for x in rng.integers(1, 90000, 36)] + [262144, 4096, 33, 513], 7, 3)
    _run_pair(big, 0, 4, sdl.FMT_E3M0_SPAN, seed=1)
    # second call right after it, smaller in every respect (fewer spans, fewer replicas, fewer
    # parameters): the device array still holds the first call's maxima
    small = _plan([5000, 77, 1024, 300], 2, 2)
    _run_pair(small, 1, 2, sdl.FMT_E3M0_SPAN, seed=2)
    # a third, again larger, and a format that uses no scratch at all
    _run_pair(big, 2, 3, sdl.FMT_E3M0_SPAN, seed=3)
    _run_pair(small, 0, 2, sdl.FMT_E3M0, seed=4)


def test_static_entry_point_size_check_needs_no_gpu():
    """The capacity check comes before anything touches the device (made-up addresses, never used)."""
    plan = _plan([64] * (sdl.STATIC_MAX_SPANS + 1), 1, 1)
    fake = [0x1000, 0x2000]
    with pytest.raises(sdl.SdlError) as err:
        sdl.sdl_fragment_outer_step_plan_static(plan, 0, 0x3000, 0x4000, fake, fake, sdl.FMT_E3M0_SPAN, 0.7, 0.9, 0.5,
                                                stream=0)
    assert err.value.status == -6


@pytest.mark.gpu
def test_static_entry_point_rejects_more_spans_than_it_holds():
    n_units = sdl.STATIC_MAX_SPANS + 1
    plan = _plan([64] * n_units, 1, 1)                      # one fragment of 1025 spans
    total = plan.total_numel
    g, mom, w_send, w_now = workloads.make_span(total, 2, tau=1, device=DEV)
    before = g.clone()
    with pytest.raises(sdl.SdlError) as err:
        sdl.sdl_fragment_outer_step_plan_static(plan, 0, g, mom, w_send, w_now, sdl.FMT_E3M0_SPAN, 0.7, 0.9, 0.5)
    assert err.value.status == -6 and "capacity" in str(err.value)
    torch.cuda.synchronize()
    assert torch.equal(before, g)                            # nothing was launched
    # the formats without scratch have no such limit
    sdl.sdl_fragment_outer_step_plan_static(plan, 0, g, mom, w_send, w_now, sdl.FMT_E3M0, 0.7, 0.9, 0.5)
    torch.cuda.synchronize()
    assert not torch.equal(before, g)


@pytest.mark.gpu
def test_static_entry_point_under_graph_capture():
    """What the entry point is for: captured into a HIP graph (after one eager call, which looks the device
    array's address up) and replayed several times with eager work in between; every replay must reproduce
    the eager result of the same inputs bit for bit (the scale words are cleared by a fill kernel, not by a
    memset node)."""
    rng = np.random.default_rng(5)
    plan = _plan([int(x) for x in rng.integers(1, 60000, 20)] + [131072, 77], 5, 2)
    M, fmt, p = 3, sdl.FMT_E3M0_SPAN, 1
    total = plan.total_numel
    g0, mom0, w_send, wn0 = workloads.make_span(total, M, tau=1, delta="outliers", base_seed=9, device=DEV)
    # eager reference through the workspace entry point
    ge, me, we = g0.clone(), mom0.clone(), [w.clone() for w in wn0]
    words = [torch.zeros(max(sdl.sdl_plan_message_bytes(plan, p, fmt)[1], 4), dtype=torch.uint8, device=DEV) for _ in range(M)]
    sdl.sdl_fragment_outer_step_plan_ex(plan, p, ge, me, w_send, we, fmt, 0.7, 0.9, 0.5, None, words)
    # the arrays the graph works on
    g, mom, wn = g0.clone(), mom0.clone(), [w.clone() for w in wn0]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sdl.sdl_fragment_outer_step_plan_static(plan, p, g, mom, w_send, wn, fmt, 0.7, 0.9, 0.5)   # eager, on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sdl.sdl_fragment_outer_step_plan_static(plan, p, g, mom, w_send, wn, fmt, 0.7, 0.9, 0.5)
    for replay in range(4):
        # restore the inputs with eager copies, dirty the device array with an eager call on another plan in between
        g.copy_(g0), mom.copy_(mom0)
        for a, b in zip(wn, wn0):
            a.copy_(b)
        if replay % 2:
            small = _plan([5000, 77, 1024, 300], 2, 2)
            sg, sm, sws, swn = workloads.make_span(small.total_numel, 2, tau=1, base_seed=replay, device=DEV)
            sdl.sdl_fragment_outer_step_plan_static(small, 0, sg, sm, sws, swn, fmt, 0.7, 0.9, 0.5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g.view(torch.int32), ge.view(torch.int32)), f"replay {replay}: g"
        assert torch.equal(mom.view(torch.int32), me.view(torch.int32)), f"replay {replay}: mom"
        for a, b in zip(wn, we):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {replay}: replica"
