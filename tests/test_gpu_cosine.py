"""GPU parity of the outer-gradient cosine similarity (Appendix) against the CPU oracle.

Tolerance.  Both sides form the same fp32 outer gradients and add their exact fp64 products;
only the order of the fp64 additions differs.  A sum of n terms carries a relative rounding
error of at most n * 2^-53 of the sum of absolute values, which is itself at most
sqrt(G[a][a] * G[b][b]); the kernel's lanes add at most a few thousand terms each and the
tree above them 2^17 more, the oracle's library routine blocks its sum too, so 1e-11 of
sqrt(G[a][a] * G[b][b]) for the Gram matrix and 1e-11 absolute for cos and the mean hold
with orders of magnitude to spare at every size used here."""
import numpy as np
import pytest
import torch

import paper_2501_18512_amd as sdl
import workloads
from gpu_util import FlatModel, host_bits, host_f32
from oracle import cosine as ref

pytestmark = pytest.mark.gpu
DEV = "cuda"
TOL = 1e-11


def _compare(result, M, G, cos, mean, what):
    got_G, got_cos, got_mean = (x.cpu().numpy() for x in sdl.split_cosine_result(result, M))
    scale = np.sqrt(np.outer(np.diag(G), np.diag(G)))
    assert np.all(np.abs(got_G - G) <= TOL * scale), f"{what}: Gram matrix\n{got_G}\n{G}"
    assert np.array_equal(got_G, got_G.T), f"{what}: Gram matrix not symmetric"
    assert np.all(np.abs(got_cos - cos) <= TOL), f"{what}: cos\n{got_cos}\n{cos}"
    assert abs(float(got_mean) - mean) <= TOL, f"{what}: mean {got_mean} vs {mean}"


def _span(n, M, delta="shared10", seed=0):
    g, _, w, _ = workloads.make_span(n, M, tau=0, delta=delta, unit=n % 89, base_seed=seed, device=DEV)
    return g, w


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 9, 12, 16])
def test_span_level_matches_oracle(M):
    # ragged tails, fewer tiles than workgroups, and more than one tile per workgroup
    for n in [1, 7, 8, 511, 512, 513, 20000 + 13, 2048 * 512 * 2 + 777]:
        if M > 8 and n > 20013 and n < 2048 * 512:
            continue
        print(f"cosine M={M} n={n}", flush=True)
        g, w = _span(n, M)
        result, work = sdl.alloc_cosine(M)
        sdl.sdl_outer_grad_cosine(g, w, n, result[0], work)
        torch.cuda.synchronize()
        G, cos, mean = ref.outer_grad_cosine(host_f32(g), [host_bits(x) for x in w])
        _compare(result[0], M, G, cos, mean, f"M={M} n={n}")


def test_reproducible_bit_for_bit():
    n, M = 3_000_017, 4
    g, w = _span(n, M)
    r1, work = sdl.alloc_cosine(M)
    r2, _ = sdl.alloc_cosine(M)
    sdl.sdl_outer_grad_cosine(g, w, n, r1[0], work)
    work.fill_(0xff)
    sdl.sdl_outer_grad_cosine(g, w, n, r2[0], work)
    torch.cuda.synchronize()
    assert torch.equal(r1.view(torch.int64), r2.view(torch.int64))


def test_unaligned_pointers_and_empty_set():
    n, M = 5000, 3
    g, w = _span(n + 3, M)
    gu, wu = g[1:], [x[3:] for x in w]                       # 4-byte and 6-byte offsets
    m = n - 2
    result, work = sdl.alloc_cosine(M)
    sdl.sdl_outer_grad_cosine(gu, wu, m, result[0], work)
    torch.cuda.synchronize()
    G, cos, mean = ref.outer_grad_cosine(host_f32(gu[:m]), [host_bits(x[:m]) for x in wu])
    _compare(result[0], M, G, cos, mean, "unaligned")
    sdl.sdl_outer_grad_cosine(g, w, 0, result[0], work)
    torch.cuda.synchronize()
    assert torch.count_nonzero(result[0]).item() == 0


def test_closed_forms_on_gpu():
    n = 1 << 20
    g = torch.zeros(n, dtype=torch.float32, device=DEV)
    idx = torch.arange(n, device=DEV)
    base = torch.where(idx % 2 == 0, 0.5, -0.25).to(torch.bfloat16)
    half = (idx < n // 2).to(torch.bfloat16)
    w = [-base, -2 * base, base, -half, -(1 - half), g.to(torch.bfloat16)]        # last: zero outer gradient
    M = len(w)
    result, work = sdl.alloc_cosine(M)
    sdl.sdl_outer_grad_cosine(g, w, n, result[0], work)
    torch.cuda.synchronize()
    G, cos, mean = (x.cpu().numpy() for x in sdl.split_cosine_result(result[0], M))
    assert G[0, 0] == n / 2 * (0.25 + 0.0625) and G[0, 1] == 2 * G[0, 0] and G[0, 2] == -G[0, 0]
    assert abs(cos[0, 1] - 1) < 1e-15 and abs(cos[0, 2] + 1) < 1e-15 and cos[3, 4] == 0
    assert G[3, 3] == n / 2 and G[3, 4] == 0
    assert np.all(cos[5] == 0) and np.all(cos[:, 5] == 0) and G[5, 5] == 0


def _small_model(seed=0, groups_per_block=3):
    rng = np.random.default_rng(seed)
    numel, block = [4096 * 3], [sdl.UNIT_PRE]
    for b in range(6):
        for _ in range(groups_per_block):
            numel.append(int(rng.choice([512, 1024, 2048 + 32, 640, 96, 32, 4096, 70000 + 64])))
            block.append(b)
    numel += [64, 4096]
    block += [sdl.UNIT_POST, sdl.UNIT_POST]
    return numel, block, 6


@pytest.mark.parametrize("M,P,pre_own,groups", [(2, 3, False, 3), (4, 2, True, 3), (9, 1, False, 3),
                                                 (3, 1, False, 20)])      # last: more spans than one launch takes
def test_plan_level_per_layer_fragment_and_union(M, P, pre_own, groups):
    numel, block, L = _small_model(groups_per_block=groups)
    flags = sdl.PLAN_PRE_OWN_FRAGMENT if pre_own else 0
    plan = sdl.sdl_fragment_plan_ex(numel, block, L, P, sdl.PATTERN_STRIDED, 100, 1, flags=flags)
    total = plan.total_numel
    g, w = _span(total, M, delta="shared10", seed=4)
    hg, hw = host_f32(g), [host_bits(x) for x in w]
    n_frag = plan.num_fragments
    frag_results = torch.empty((n_frag, sdl.cosine_result_doubles(M)), dtype=torch.float64, device=DEV)
    ref_grams = []
    for p in range(n_frag):
        spans = sdl.sdl_plan_fragment_spans(plan, p)
        span_results, work = sdl.alloc_cosine(M, len(spans))
        sdl.sdl_outer_grad_cosine_plan(plan, p, g, w, span_results, frag_results[p], work)
        torch.cuda.synchronize()
        grams = []
        for i, (off, n, unit) in enumerate(spans):
            G, cos, mean = ref.outer_grad_cosine(hg[off:off + n], [x[off:off + n] for x in hw])
            _compare(span_results[i], M, G, cos, mean, f"fragment {p} span {i} (unit {unit})")
            grams.append(G)
        G, cos, mean = ref.combine(grams)
        _compare(frag_results[p], M, G, cos, mean, f"fragment {p}")
        ref_grams.append(G)
        # the per-span results are optional
        again = torch.empty_like(frag_results[p])
        sdl.sdl_outer_grad_cosine_plan(plan, p, g, w, None, again, work)
        torch.cuda.synchronize()
        assert torch.equal(again.view(torch.int64), frag_results[p].view(torch.int64))
    # union of all fragments = the whole model; union of all but the first = "all but the embedding"
    whole = torch.empty(sdl.cosine_result_doubles(M), dtype=torch.float64, device=DEV)
    sdl.sdl_cosine_combine(frag_results, n_frag, M, whole)
    torch.cuda.synchronize()
    G, cos, mean = ref.outer_grad_cosine(hg, hw)
    _compare(whole, M, G, cos, mean, "whole model")
    if n_frag > 1:
        sdl.sdl_cosine_combine(frag_results[1:], n_frag - 1, M, whole)
        torch.cuda.synchronize()
        G, cos, mean = ref.combine(ref_grams[1:])
        _compare(whole, M, G, cos, mean, "all fragments but the first")


def test_full_size_1b_fragment():
    """The configuration the benchmark times: fragment 1 of the 1B shape, M = 4.  The oracle takes
    a sample of spans one by one (largest, smallest, first, last); the rest is covered by the
    identity fragment = sum of spans, checked against the oracle's own combination rule."""
    import dataclasses
    wl = dataclasses.replace(workloads.WORKLOADS["1b"], delta="shared10", tau=0)
    model = FlatModel(wl, fill_fragments=[1])
    M, p = wl.M, 1
    spans = sdl.sdl_plan_fragment_spans(model.plan, p)
    span_results, work = sdl.alloc_cosine(M, len(spans))
    frag = torch.empty(sdl.cosine_result_doubles(M), dtype=torch.float64, device=DEV)
    sdl.sdl_outer_grad_cosine_plan(model.plan, p, model.g, model.w_send, span_results, frag, work)
    torch.cuda.synchronize()
    order = sorted(range(len(spans)), key=lambda i: spans[i][1])
    for i in sorted({order[0], order[-1], 0, len(spans) - 1}):
        off, n, unit = spans[i]
        print(f"1b fragment 1 span {i}: unit {unit}, {n} parameters", flush=True)
        G, cos, mean = ref.outer_grad_cosine(host_f32(model.g[off:off + n]),
                                             [host_bits(w[off:off + n]) for w in model.w_send])
        _compare(span_results[i], M, G, cos, mean, f"1b span {i}")
        assert abs(mean - 0.1) < 0.01                        # the recipe's correlation comes back
    grams = [sdl.split_cosine_result(span_results[i], M)[0].cpu().numpy() for i in range(len(spans))]
    G, cos, mean = ref.combine(grams)
    _compare(frag, M, G, cos, mean, "1b fragment 1 from its spans")


def test_more_than_2_to_the_31_parameters():
    """The 4B shape as one set of 4,273,695,744 parameters (element indices beyond 2^31, byte offsets
    beyond 2^34): the single call must agree with the sum of the per-span results of the plan-level
    call, and the oracle checks the spans at the far end of the arrays one by one."""
    import dataclasses
    wl = dataclasses.replace(workloads.WORKLOADS["4b_p1"], delta="shared10", tau=0)
    model = FlatModel(wl)
    M, total = wl.M, model.plan.total_numel
    assert total > 2 ** 31
    whole, work = sdl.alloc_cosine(M)
    sdl.sdl_outer_grad_cosine(model.g, model.w_send, total, whole[0], work)
    spans = sdl.sdl_plan_fragment_spans(model.plan, 0)
    span_results, work2 = sdl.alloc_cosine(M, len(spans))
    frag = torch.empty(sdl.cosine_result_doubles(M), dtype=torch.float64, device=DEV)
    sdl.sdl_outer_grad_cosine_plan(model.plan, 0, model.g, model.w_send, span_results, frag, work2)
    torch.cuda.synchronize()
    G1, cos1, mean1 = (x.cpu().numpy() for x in sdl.split_cosine_result(whole[0], M))
    _compare(frag, M, G1, cos1, float(mean1), "4B: one set against the sum of its spans")
    assert abs(float(mean1) - 0.1) < 0.01
    for i in (len(spans) - 1, len(spans) - 2, len(spans) - 3):
        off, n, unit = spans[i]
        print(f"4B span {i}: unit {unit}, offset {off}, {n} parameters", flush=True)
        G, cos, mean = ref.outer_grad_cosine(host_f32(model.g[off:off + n]),
                                             [host_bits(w[off:off + n]) for w in model.w_send])
        _compare(span_results[i], M, G, cos, mean, f"4B span {i}")


def test_stream_argument_and_graph_replay():
    """The calls run on the caller's stream, allocate nothing and use no memset, so they can be
    captured; every replay must give the eager result."""
    n, M = 700_001, 3
    g, w = _span(n, M)
    eager, work = sdl.alloc_cosine(M)
    sdl.sdl_outer_grad_cosine(g, w, n, eager[0], work)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    got, work2 = sdl.alloc_cosine(M)
    sdl.sdl_outer_grad_cosine(g, w, n, got[0], work2, stream=side)
    side.synchronize()
    assert torch.equal(got.view(torch.int64), eager.view(torch.int64))
    graph = torch.cuda.CUDAGraph()
    captured, work3 = sdl.alloc_cosine(M)
    with torch.cuda.graph(graph):
        sdl.sdl_outer_grad_cosine(g, w, n, captured[0], work3)
    for replay in range(3):
        captured.zero_()
        work3.fill_(replay)                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(captured.view(torch.int64), eager.view(torch.int64)), f"replay {replay}"


def test_argument_errors():
    g, w = _span(1024, 2)
    result, work = sdl.alloc_cosine(2)
    with pytest.raises(sdl.SdlError):
        sdl.sdl_outer_grad_cosine(g, w, 1024, result[0], work[:64])              # workspace too small
    with pytest.raises(sdl.SdlError):
        sdl.sdl_outer_grad_cosine(g, w, 1024, result[0].view(torch.uint8)[4:].view(torch.uint8), work)
    with pytest.raises(sdl.SdlError):
        sdl.sdl_outer_grad_cosine(g, [], 1024, result[0], work)
