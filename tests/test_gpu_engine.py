"""Algorithm 2 end to end on the GPU: the schedule driver walks T inner steps of a small
synthetic model (inner updates are seeded noise, identical on both sides) and must leave the
global parameters, the momentum and every replica where the oracle's walk leaves them."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_18512_amd as sdl
import workloads
from gpu_util import assert_bf16_within_ulp, assert_f32_close, host_bits, host_f32

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _small_model(seed=0):
    """7 blocks of 4 parameter groups with assorted (also ragged) sizes + embedding + head."""
    rng = np.random.default_rng(seed)
    numel, block = [4096], [sdl.UNIT_PRE]
    for b in range(7):
        for k in range(4):
            numel.append(int(rng.choice([512, 1024, 2048 + 32, 640, 100, 33, 4096])))
            block.append(b)
    numel += [64, 4096]
    block += [sdl.UNIT_POST, sdl.UNIT_POST]
    return numel, block, 7


@pytest.mark.parametrize("taus,P,pattern,fmt", [
    ((0, 0), 3, sdl.PATTERN_STRIDED, sdl.FMT_E3M0),        # no overlap: fused at the send step
    ((1, 1), 3, sdl.PATTERN_STRIDED, sdl.FMT_E3M0),        # the paper's main setting
    ((5, 5, 5, 5), 4, sdl.PATTERN_STRIDED, sdl.FMT_E3M0),  # tau larger than the spacing of fragments
    ((1, 4), 2, sdl.PATTERN_SEQUENTIAL, sdl.FMT_E4M3),     # slack between workers
    ((0, 3, 2), 7, sdl.PATTERN_STRIDED, sdl.FMT_BF16),
    ((2, 2), 1, sdl.PATTERN_STRIDED, sdl.FMT_FP32),        # P = 1: DiLoCo with overlap
    ((1, 1), 3, sdl.PATTERN_STRIDED, sdl.FMT_E3M0_SPAN),   # one scale per tensor (4.0 bits / parameter)
    ((0, 0), 2, sdl.PATTERN_STRIDED, sdl.FMT_E3M0_SPAN),
    ((1, 2), 2, sdl.PATTERN_STRIDED, sdl.FMT_E3M0_B128),
])
def test_engine_matches_oracle_walk(taus, P, pattern, fmt):
    H, T, M = 12, 3 * 12 + 9, len(taus)
    lr, mu, alpha = 0.7, 0.9, 0.5
    numel, block, L = _small_model()
    plan = sdl.sdl_fragment_plan(numel, block, L, P, pattern, H, min(taus))
    ref_plan = oracle.fragment_plan(numel, block, L, P, pattern, H, min(taus))
    total = plan.total_numel
    g, mom, w, _ = workloads.make_span(total, M, tau=0, delta="normal", device=DEV)
    ref = oracle.RefEngine(ref_plan, taus, fmt, lr, mu, alpha, host_f32(g), host_f32(mom), [host_bits(x) for x in w])
    eng = sdl.sdl_engine_create(plan, H, taus, fmt, lr, mu, alpha)
    codes, scales = [], []
    for p in range(P):
        cb, sb = sdl.sdl_plan_message_bytes(plan, p, fmt)
        for m in range(M):
            codes.append(torch.zeros(max(cb, 16), dtype=torch.uint8, device=DEV))
            scales.append(torch.zeros(max(sb, 16), dtype=torch.uint8, device=DEV))
    sdl.sdl_engine_bind(eng, g, mom, w, codes, scales)
    gen = torch.Generator(DEV).manual_seed(7)
    events = 0
    for t in range(1, T + 1):
        # inner step: the same seeded noise moves every replica on both sides
        for m in range(M):
            noise = torch.randn(total, device=DEV, generator=gen) * 3e-4
            w[m].copy_((w[m].float() + noise).bfloat16())
            hn = torch.from_numpy(ref.w[m].view(np.int16)).view(torch.bfloat16).float() + noise.cpu()
            ref.w[m][:] = host_bits(hn.bfloat16())
        got = sdl.sdl_engine_step(eng, t)
        want = ref.step(t)
        assert got == want, (t, got, want)
        assert got[0] == len(sdl.sdl_plan_events(plan, t)[0])
        events += got[0]
    torch.cuda.synchronize()
    assert events >= 2 * P
    assert_f32_close(host_f32(g), ref.g, "engine g")
    assert_f32_close(host_f32(mom), ref.mom, "engine mom")
    for m in range(M):
        assert_bf16_within_ulp(host_bits(w[m]), ref.w[m], f"engine w[{m}]")
    assert float(np.abs(ref.mom).max()) > 0


def test_fragment_level_calls_match_span_level_calls():
    """quantize / reduce / merge on a whole fragment = the same calls span by span."""
    numel, block, L = _small_model(seed=1)
    P, M, fmt = 2, 2, sdl.FMT_E3M0
    plan = sdl.sdl_fragment_plan(numel, block, L, P, sdl.PATTERN_STRIDED, 10, 1)
    total = plan.total_numel
    g, mom, w_send, w_now = workloads.make_span(total, M, tau=1, device=DEV)
    g2, mom2, wn2 = g.clone(), mom.clone(), [x.clone() for x in w_now]
    for p in range(P):
        cb, sb = sdl.sdl_plan_message_bytes(plan, p, fmt)
        codes = [torch.zeros(cb, dtype=torch.uint8, device=DEV) for _ in range(M)]
        scales = [torch.zeros(sb, dtype=torch.uint8, device=DEV) for _ in range(M)]
        sdl.sdl_quantize_outer_grad_plan(plan, p, g, w_send, fmt, codes, scales)
        sdl.sdl_dequant_reduce_nesterov_plan(plan, p, g, mom, codes, scales, fmt, 0.7, 0.9)
        sdl.sdl_merge_overlap_plan(plan, p, g, w_now, 0.5)
        for off, n, _ in sdl.sdl_plan_fragment_spans(plan, p):
            sl = slice(off, off + n)
            c, s = sdl.alloc_exchange(fmt, n, M)
            sdl.sdl_quantize_outer_grad(g2[sl], [x[sl] for x in w_send], n, fmt, c, s)
            sdl.sdl_dequant_reduce_nesterov(g2[sl], mom2[sl], c, s, n, fmt, 0.7, 0.9)
            sdl.sdl_merge_overlap(g2[sl], [x[sl] for x in wn2], n, 0.5)
    torch.cuda.synchronize()
    assert torch.equal(g, g2) and torch.equal(mom, mom2)
    for a, b in zip(w_now, wn2):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("fmt", [sdl.FMT_E3M0, sdl.FMT_E4M3, sdl.FMT_E3M0_B128, sdl.FMT_E3M0_SPAN])
@pytest.mark.parametrize("tau", [0, 1])
def test_fused_fragment_call_with_messages(fmt, tau):
    """The fused call of a whole fragment, messages written out: the messages are those of the
    fragment-level send side, the state that of the three fragment-level calls; also for the
    whole-span scale, whose scale words the call needs as workspace."""
    numel, block, L = _small_model(seed=2)
    P, M = 2, 3
    plan = sdl.sdl_fragment_plan(numel, block, L, P, sdl.PATTERN_STRIDED, 10, tau)
    total = plan.total_numel
    g, mom, w_send, w_now = workloads.make_span(total, M, tau=tau, delta="student_t3", device=DEV)
    g2, mom2 = g.clone(), mom.clone()
    ws2 = [x.clone() for x in w_send]
    wn2 = ws2 if tau == 0 else [x.clone() for x in w_now]
    g3, mom3 = g.clone(), mom.clone()
    ws3 = [x.clone() for x in w_send]
    wn3 = ws3 if tau == 0 else [x.clone() for x in w_now]
    for p in range(P):
        cb, sb = sdl.sdl_plan_message_bytes(plan, p, fmt)
        codes = [torch.zeros(cb, dtype=torch.uint8, device=DEV) for _ in range(M)]
        scales = [torch.zeros(max(sb, 4), dtype=torch.uint8, device=DEV) for _ in range(M)]
        sdl.sdl_fragment_outer_step_plan_ex(plan, p, g, mom, w_send, w_now, fmt, 0.7, 0.9, 0.5, codes, scales)
        codes2 = [torch.zeros(cb, dtype=torch.uint8, device=DEV) for _ in range(M)]
        scales2 = [torch.zeros(max(sb, 4), dtype=torch.uint8, device=DEV) for _ in range(M)]
        sdl.sdl_quantize_outer_grad_plan(plan, p, g2, ws2, fmt, codes2, scales2)
        sdl.sdl_dequant_reduce_nesterov_plan(plan, p, g2, mom2, codes2, scales2, fmt, 0.7, 0.9)
        sdl.sdl_merge_overlap_plan(plan, p, g2, wn2, 0.5)
        # without messages: scale words only where the format needs them as workspace
        work = [torch.zeros(max(sb, 4), dtype=torch.uint8, device=DEV) for _ in range(M)]
        sdl.sdl_fragment_outer_step_plan_ex(plan, p, g3, mom3, ws3, wn3, fmt, 0.7, 0.9, 0.5, None,
                                            work if fmt == sdl.FMT_E3M0_SPAN else None)
        torch.cuda.synchronize()
        for m in range(M):
            assert torch.equal(codes[m], codes2[m]), f"fragment {p} codes[{m}]"
            assert torch.equal(scales[m][:sb], scales2[m][:sb]), f"fragment {p} scales[{m}]"
    for a, b, what in ((g, g2, "g"), (mom, mom2, "mom"), (g3, g2, "g, no messages"), (mom3, mom2, "mom, no messages")):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32)), what
    for a, b, c in zip(w_now, wn2, wn3):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
        assert torch.equal(c.view(torch.int16), b.view(torch.int16))
    if fmt == sdl.FMT_E3M0_SPAN:
        with pytest.raises(sdl.SdlError) as e:
            sdl.sdl_fragment_outer_step_plan(plan, 0, g, mom, w_send, w_now, fmt, 0.7, 0.9, 0.5)
        assert e.value.status == -2


@pytest.mark.parametrize("taus,P,fmt,n_slots,lookahead", [
    ((0, 0), 2, sdl.FMT_E3M0_SPAN, 1, 1),     # whole-span scale without overlap: staged fused call
    ((1, 1), 3, sdl.FMT_E3M0, 3, 1),          # the paper's setting, everything prefetched one step ahead
    ((0, 0), 3, sdl.FMT_E3M0, 1, 0),          # no overlap, a single slot, fetched on demand
    ((5, 5, 5, 5), 4, sdl.FMT_E3M0, 4, 2),    # several fragments in flight at once
    ((1, 4), 2, sdl.FMT_E4M3, 2, 3),
    # a tight pool and a long look-ahead: one fragment is in flight while later senders are prefetched
    # early; the fragment that is due next must still find a slot (a prefetched, unused copy gives way)
    ((2, 2), 4, sdl.FMT_E3M0, 2, 8),
    ((2, 2), 4, sdl.FMT_E3M0, 1, 11),
    ((5, 5), 4, sdl.FMT_E3M0, 2, 11),         # two in flight at once, exactly two slots, everything else on demand
])
def test_engine_with_outer_state_in_host_memory(taus, P, fmt, n_slots, lookahead):
    """Section 2.5: outer parameters and momentum live in (pinned) host memory; fragments are
    staged through a small pool of device slots on a copy stream.  Same walk, same result."""
    H, T, M = 12, 3 * 12 + 9, len(taus)
    lr, mu, alpha = 0.7, 0.9, 0.5
    numel, block, L = _small_model()
    plan = sdl.sdl_fragment_plan(numel, block, L, P, sdl.PATTERN_STRIDED, H, min(taus))
    ref_plan = oracle.fragment_plan(numel, block, L, P, sdl.PATTERN_STRIDED, H, min(taus))
    total = plan.total_numel
    g, mom, w, _ = workloads.make_span(total, M, tau=0, delta="normal", device=DEV)
    ref = oracle.RefEngine(ref_plan, taus, fmt, lr, mu, alpha, host_f32(g), host_f32(mom), [host_bits(x) for x in w])
    g_host = g.cpu().pin_memory()
    mom_host = mom.cpu().pin_memory()
    del g, mom                                     # no flat device copy of the outer state exists
    pool = sdl.sdl_offload_create(plan, n_slots)
    assert pool.slot_numel == max(sdl.sdl_plan_staged_numel(plan, p) for p in range(P))
    slot_g = [torch.full((pool.slot_numel,), float("nan"), device=DEV) for _ in range(n_slots)]
    slot_mom = [torch.full((pool.slot_numel,), float("nan"), device=DEV) for _ in range(n_slots)]
    sdl.sdl_offload_bind(pool, g_host, mom_host, slot_g, slot_mom)
    eng = sdl.sdl_engine_create(plan, H, taus, fmt, lr, mu, alpha)
    codes, scales = [], []
    for p in range(P):
        cb, sb = sdl.sdl_plan_message_bytes(plan, p, fmt)
        for m in range(M):
            codes.append(torch.zeros(max(cb, 16), dtype=torch.uint8, device=DEV))
            scales.append(torch.zeros(max(sb, 16), dtype=torch.uint8, device=DEV))
    copy_stream = torch.cuda.Stream()
    sdl.sdl_engine_bind_offload(eng, pool, w, codes, scales, copy_stream=copy_stream, lookahead=lookahead)
    gen = torch.Generator(DEV).manual_seed(7)
    prefetched = 0
    for t in range(1, T + 1):
        for m in range(M):
            noise = torch.randn(total, device=DEV, generator=gen) * 3e-4
            w[m].copy_((w[m].float() + noise).bfloat16())
            hn = torch.from_numpy(ref.w[m].view(np.int16)).view(torch.bfloat16).float() + noise.cpu()
            ref.w[m][:] = host_bits(hn.bfloat16())
        due_next = sdl.sdl_plan_events(plan, t + 1)[0] if lookahead else []
        assert sdl.sdl_engine_step(eng, t) == ref.step(t)
        prefetched += sum(sdl.sdl_offload_resident(pool, p) for p in due_next)
    if lookahead:
        assert prefetched > 0
    sdl.sdl_offload_flush(pool, copy_stream)
    copy_stream.synchronize()
    torch.cuda.synchronize()
    assert_f32_close(g_host.numpy(), ref.g, "offloaded g")
    assert_f32_close(mom_host.numpy(), ref.mom, "offloaded mom")
    for m in range(M):
        assert_bf16_within_ulp(host_bits(w[m]), ref.w[m], f"offloaded w[{m}]")


def test_engine_refuses_a_pool_with_too_few_slots():
    """With a delay of 5 of every 12 steps and 4 staggered fragments, two fragments are between send and merge at
    the same time: a pool of one slot is refused when it is bound, not half way through a step."""
    numel, block, L = _small_model()
    plan = sdl.sdl_fragment_plan(numel, block, L, 4, sdl.PATTERN_STRIDED, 12, 5)
    total, M, fmt = plan.total_numel, 2, sdl.FMT_E3M0
    g, mom, w, _ = workloads.make_span(total, M, tau=0, device=DEV)
    g_host, mom_host = g.cpu().pin_memory(), mom.cpu().pin_memory()
    codes, scales = [], []
    for p in range(4):
        cb, sb = sdl.sdl_plan_message_bytes(plan, p, fmt)
        for m in range(M):
            codes.append(torch.zeros(max(cb, 16), dtype=torch.uint8, device=DEV))
            scales.append(torch.zeros(max(sb, 16), dtype=torch.uint8, device=DEV))
    for n_slots, ok in ((1, False), (2, True)):
        pool = sdl.sdl_offload_create(plan, n_slots)
        slot_g = [torch.zeros(pool.slot_numel, device=DEV) for _ in range(n_slots)]
        slot_mom = [torch.zeros(pool.slot_numel, device=DEV) for _ in range(n_slots)]
        sdl.sdl_offload_bind(pool, g_host, mom_host, slot_g, slot_mom)
        eng = sdl.sdl_engine_create(plan, 12, (5, 5), fmt, 0.7, 0.9, 0.5)
        if ok:
            sdl.sdl_engine_bind_offload(eng, pool, w, codes, scales, copy_stream=torch.cuda.Stream(), lookahead=3)
        else:
            with pytest.raises(sdl.SdlError) as e:
                sdl.sdl_engine_bind_offload(eng, pool, w, codes, scales, copy_stream=torch.cuda.Stream(), lookahead=3)
            assert e.value.status == -1


@pytest.mark.parametrize("taus", [(0, 0, 0), (2, 2, 2)])
def test_engine_tracks_cosine_similarity_at_every_send(taus):
    """Appendix: the similarity between the replicas' outer gradients, recorded when they are sent."""
    from oracle import cosine as ref_cosine
    H, M, P = 8, len(taus), 3
    numel, block, L = _small_model(seed=3)
    plan = sdl.sdl_fragment_plan(numel, block, L, P, sdl.PATTERN_STRIDED, H, min(taus))
    total = plan.total_numel
    g, mom, w, _ = workloads.make_span(total, M, tau=0, delta="shared10", device=DEV)
    eng = sdl.sdl_engine_create(plan, H, taus, sdl.FMT_E3M0, 0.7, 0.9, 0.5)
    codes, scales = [], []
    for p in range(P):
        cb, sb = sdl.sdl_plan_message_bytes(plan, p, sdl.FMT_E3M0)
        for m in range(M):
            codes.append(torch.zeros(max(cb, 16), dtype=torch.uint8, device=DEV))
            scales.append(torch.zeros(max(sb, 16), dtype=torch.uint8, device=DEV))
    sdl.sdl_engine_bind(eng, g, mom, w, codes, scales)
    R = sdl.cosine_result_doubles(M)
    spans = [sdl.sdl_plan_fragment_spans(plan, p) for p in range(P)]
    frag_results = torch.full((P, R), float("nan"), dtype=torch.float64, device=DEV)
    span_results = [torch.full((len(spans[p]), R), float("nan"), dtype=torch.float64, device=DEV) if p != 1 else None
                    for p in range(P)]
    work = torch.empty(max(sdl.sdl_cosine_workspace_bytes(M, len(sp)) for sp in spans), dtype=torch.uint8, device=DEV)
    with pytest.raises(sdl.SdlError):
        sdl.sdl_engine_track_cosine(eng, span_results, frag_results, work[:1024])
    sdl.sdl_engine_track_cosine(eng, span_results, frag_results, work)
    gen = torch.Generator(DEV).manual_seed(11)
    checked = 0
    for t in range(1, 3 * H + 1):
        for m in range(M):
            w[m].copy_((w[m].float() + torch.randn(total, device=DEV, generator=gen) * 3e-4).bfloat16())
        sending = sdl.sdl_plan_events(plan, t)[0]
        hg, hw = host_f32(g), [host_bits(x) for x in w]          # the state the sends of this step see
        sdl.sdl_engine_step(eng, t)
        torch.cuda.synchronize()
        for p in sending:
            grams = []
            for i, (off, n, _) in enumerate(spans[p]):
                G, cos, mean = ref_cosine.outer_grad_cosine(hg[off:off + n], [x[off:off + n] for x in hw])
                grams.append(G)
                if span_results[p] is not None:
                    got = sdl.split_cosine_result(span_results[p][i], M)
                    assert np.all(np.abs(got[1].cpu().numpy() - cos) <= 1e-11)
            G, cos, mean = ref_cosine.combine(grams)
            got_G, got_cos, got_mean = (x.cpu().numpy() for x in sdl.split_cosine_result(frag_results[p], M))
            assert np.all(np.abs(got_G - G) <= 1e-11 * np.sqrt(np.outer(np.diag(G), np.diag(G))))
            assert np.all(np.abs(got_cos - cos) <= 1e-11) and abs(float(got_mean) - mean) <= 1e-11
            checked += 1
    assert checked == 2 * P + sum(1 for p in range(P) if sdl.sdl_plan_offset(plan, p) == 0)
    # switched off again: nothing is written any more
    sdl.sdl_engine_track_cosine(eng, None, None, None)
    frag_results.fill_(7.0)
    for t in range(3 * H + 1, 4 * H + 1):
        sdl.sdl_engine_step(eng, t)
    torch.cuda.synchronize()
    assert torch.all(frag_results == 7.0)


def test_fragment_step_can_be_captured_in_a_graph():
    """The calls only enqueue kernels (no allocation, no synchronisation, no memset node), so a
    caller may capture them in a HIP graph.  Three replays, with eager work and synchronisations
    between them, each checked against the eager result from the same starting state."""
    wl = workloads.WORKLOADS["tiny"]
    n, M, fmt = 1 << 18, 2, sdl.FMT_E3M0
    g, mom, w_send, w_now = workloads.make_span(n, M, tau=1, delta="student_t3", device=DEV)
    plan = sdl.sdl_fragment_plan([n // 2, n // 2 - 96, 96], [0, 1, 1], 2, 1, sdl.PATTERN_STRIDED, 10, 1)
    span_scales = sdl.alloc_exchange(sdl.FMT_E3M0_SPAN, n, M)[1]
    # eager reference: three consecutive steps, state saved after each
    eg, em, ew = g.clone(), mom.clone(), [x.clone() for x in w_now]
    want = []
    for _ in range(3):
        sdl.sdl_fragment_outer_step_plan(plan, 0, eg, em, w_send, ew, fmt, wl.lr, wl.mu, wl.alpha)
        sdl.sdl_fragment_outer_step(eg, em, w_send, ew, n, sdl.FMT_E3M0_SPAN, wl.lr, wl.mu, wl.alpha, scales=span_scales)
        torch.cuda.synchronize()
        want.append((eg.clone(), em.clone(), [x.clone() for x in ew]))
    # captured: the same two calls in one graph
    cg, cm, cw = g.clone(), mom.clone(), [x.clone() for x in w_now]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up outside the capture
        sdl.sdl_copy_bytes(cm, cm, 0)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sdl.sdl_fragment_outer_step_plan(plan, 0, cg, cm, w_send, cw, fmt, wl.lr, wl.mu, wl.alpha)
        sdl.sdl_fragment_outer_step(cg, cm, w_send, cw, n, sdl.FMT_E3M0_SPAN, wl.lr, wl.mu, wl.alpha, scales=span_scales)
    # the capture itself does not execute: state still at the start
    assert torch.equal(cg, g)
    scratch = torch.zeros(1 << 20, device=DEV)
    for k in range(3):
        graph.replay()
        scratch.add_(1.0).sum().item()                  # eager work and a synchronisation between replays
        torch.cuda.synchronize()
        eg_k, em_k, ew_k = want[k]
        assert torch.equal(cg, eg_k) and torch.equal(cm, em_k), f"replay {k}"
        for a, b in zip(cw, ew_k):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {k}"
