"""GPU parity at the three large benchmark configurations, every element: the 1B fragment (M = 4,
heavy-tailed deltas), the stress fragment (M = 8, outliers) and the whole 4B model (P = 1 and P = 6),
in the launch configuration bench.py times and in the other paths that reach the same result
(messages written, send side then receive side).  The oracle is streamed over the fragment span by
span; nothing is sampled."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_18512_amd as sdl
import workloads
from gpu_stream_check import Variant, message_positions, stream_check
from gpu_util import FlatModel, HostCopy, assert_bf16_within_ulp, assert_bytes_equal, assert_f32_close, host_bits, host_f32

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _messages(plan, p, fmt, M):
    cb, sb = sdl.sdl_plan_message_bytes(plan, p, fmt)
    # poisoned: every byte that is compared has to be written by the call
    return ([torch.full((max(cb, 16),), 0xa5, dtype=torch.uint8, device=DEV) for _ in range(M)],
            [torch.full((max(sb, 16),), 0xa5, dtype=torch.uint8, device=DEV) for _ in range(M)])


def _progress(capsys):
    def say(line):
        with capsys.disabled():
            print("\n    " + line, end="", flush=True)
    return say


def _three_paths(model, p, fmt, capsys, what):
    """Fused, fused with messages, and send side followed by the one-pass receive side, each from the
    same inputs; all three compared in full with one pass of the oracle."""
    wl = model.wl
    M = wl.M
    g0, mom0, wn0 = model.g.clone(), model.mom.clone(), [w.clone() for w in model.w_now]
    variants = []
    # (a) what bench.py times: one fused launch, messages in registers (the whole-span scale needs its words)
    words = _messages(model.plan, p, fmt, M)[1] if fmt == sdl.FMT_E3M0_SPAN else None
    sdl.sdl_fragment_outer_step_plan_ex(model.plan, p, model.g, model.mom, model.w_send, model.w_now, fmt, wl.lr,
                                        wl.mu, wl.alpha, None, words)
    variants.append(Variant("fused", model.g, model.mom, model.w_now))
    # (b) the same with the messages written
    gb, mb, wb = g0.clone(), mom0.clone(), [w.clone() for w in wn0]
    cb_, sb_ = _messages(model.plan, p, fmt, M)
    sdl.sdl_fragment_outer_step_plan_ex(model.plan, p, gb, mb, model.w_send, wb, fmt, wl.lr, wl.mu, wl.alpha, cb_, sb_)
    variants.append(Variant("fused, messages written", gb, mb, wb, cb_, sb_))
    # (c) what the schedule driver issues when tau > 0: send side, then the one-pass receive side
    gc, mc, wc = g0.clone(), mom0.clone(), [w.clone() for w in wn0]
    cc, sc = _messages(model.plan, p, fmt, M)
    sdl.sdl_quantize_outer_grad_plan(model.plan, p, gc, model.w_send, fmt, cc, sc)
    sdl.sdl_receive_outer_step_plan(model.plan, p, gc, mc, cc, sc, wc, fmt, wl.lr, wl.mu, wl.alpha)
    variants.append(Variant("send, one-pass receive", gc, mc, wc, cc, sc))
    torch.cuda.synchronize()
    return stream_check(model.plan, p, fmt, wl.lr, wl.mu, wl.alpha, g0=g0, mom0=mom0, w_send=model.w_send,
                        w_now0=wn0, variants=variants, what=what, progress=_progress(capsys))


@pytest.mark.parametrize("fmt", ["e3m0", "e3m0_span", "e3m0_b64", "e3m0_b128", "e3m0_rn"])
def test_config_1b_fragment_every_element(fmt, capsys):
    wl = workloads.WORKLOADS["1b"]
    model = FlatModel(wl, fill_fragments=[1])
    assert sum(n for _, n, _ in sdl.sdl_plan_fragment_runs(model.plan, 1)) == 302014464
    counts = _three_paths(model, 1, sdl.FORMATS[fmt], capsys, f"1b f1 {fmt}")
    assert counts["elements"] == 302014464
    assert counts["code_bytes"] == 2 * wl.M * 302014464 // 2          # two message-writing paths, 4 replicas
    block = {"e3m0": 32, "e3m0_rn": 32, "e3m0_b64": 64, "e3m0_b128": 128}.get(fmt)
    assert counts["scale_bytes"] == (2 * wl.M * 302014464 // block if block else 2 * wl.M * 4 * 48)


@pytest.mark.parametrize("fmt_name", ["e3m0", "e4m3", "bf16"])
def test_config_stress_m8_every_element(fmt_name, capsys):
    """Config 5 in full for each of its three formats at alpha = 0.5: the fused step, and the three separate calls
    (send side, receive side alone -- the call the configuration is named after --, merge), whose
    intermediate results are compared as well."""
    wl = workloads.WORKLOADS["stress"]
    fmt, M, p = sdl.FORMATS[fmt_name], wl.M, 1
    model = FlatModel(wl, fill_fragments=[p])
    g0, mom0, wn0 = model.g.clone(), model.mom.clone(), [w.clone() for w in model.w_now]
    # three separate calls on a copy; g', mom' right after the receive side are kept for a comparison of their own
    gu, mu_, wu = g0.clone(), mom0.clone(), [w.clone() for w in wn0]
    cu, su = _messages(model.plan, p, fmt, M)
    sdl.sdl_quantize_outer_grad_plan(model.plan, p, gu, model.w_send, fmt, cu, su)
    sdl.sdl_dequant_reduce_nesterov_plan(model.plan, p, gu, mu_, cu, su, fmt, wl.lr, wl.mu)
    g_mid, mom_mid = gu.clone(), mu_.clone()
    sdl.sdl_merge_overlap_plan(model.plan, p, gu, wu, wl.alpha)
    model.step(p, fmt=fmt, alpha=wl.alpha)
    torch.cuda.synchronize()
    say = _progress(capsys)
    counts = stream_check(model.plan, p, fmt, wl.lr, wl.mu, wl.alpha, g0=g0, mom0=mom0, w_send=model.w_send,
                          w_now0=wn0, what=f"stress M=8 {fmt_name}", progress=say,
                          variants=[Variant("fused", model.g, model.mom, model.w_now),
                                    Variant("send, receive, merge", gu, mu_, wu, cu, su)])
    assert counts["elements"] == 302014464
    assert counts["code_bytes"] == M * sdl.sdl_exchange_bytes(fmt, 302014464)[0]
    # the receive side alone: g', mom' before the merge touched anything (the merge does not write them,
    # so this is the same check from the other side: the arrays did not change after the receive side)
    assert torch.equal(g_mid.view(torch.int32), gu.view(torch.int32))
    assert torch.equal(mom_mid.view(torch.int32), mu_.view(torch.int32))


@pytest.mark.parametrize("fmt", ["e3m0", "fp32"])
def test_config_4b_every_element(fmt, capsys):
    """Config 4: the whole 4B model synchronised as one fragment (P = 1), every element against the oracle;
    the same seed as six strided fragments gives the same model bit for bit; for the 4-bit format the
    send-side messages of P = 1 are compared with the oracle byte for byte and with those of P = 6."""
    say = _progress(capsys)
    f = sdl.FORMATS[fmt]
    wl = workloads.WORKLOADS["4b_p1"]
    one = FlatModel(wl)
    total = one.plan.total_numel
    assert total == 4273695744 > 2 ** 31
    M = wl.M
    shape = workloads.SHAPES["4b"]
    numel, block, _ = shape.units()
    wl6 = workloads.WORKLOADS["4b_p6"]
    p6 = sdl.sdl_fragment_plan(numel, block, shape.n_layers, wl6.P, sdl.PATTERN_STRIDED, wl6.H, wl6.tau)
    assert [sdl.sdl_plan_offset(p6, p) for p in range(6)] == [0, 16, 33, 50, 66, 83]
    g0, mom0, wn0 = one.g.clone(), one.mom.clone(), [w.clone() for w in one.w_now]
    variants = []
    if fmt == "e3m0":
        # send side of both partitions, before anything is updated
        c1, s1 = _messages(one.plan, 0, f, M)
        sdl.sdl_quantize_outer_grad_plan(one.plan, 0, one.g, one.w_send, f, c1, s1)
        pos1 = message_positions(one.plan, 0, f)
        for p in range(6):
            c6, s6 = _messages(p6, p, f, M)
            sdl.sdl_quantize_outer_grad_plan(p6, p, one.g, one.w_send, f, c6, s6)
            torch.cuda.synchronize()
            pos6 = message_positions(p6, p, f)
            for off, n, _ in sdl.sdl_plan_fragment_spans(p6, p):
                a1, a6 = pos1[off], pos6[off]
                for m in range(M):
                    assert torch.equal(c1[m][a1 // 2:(a1 + n) // 2], c6[m][a6 // 2:(a6 + n) // 2]), (p, off, m)
                    assert torch.equal(s1[m][a1 // 32:(a1 + n) // 32], s6[m][a6 // 32:(a6 + n) // 32]), (p, off, m)
            del c6, s6
        say(f"4b {fmt}: messages of P=1 and P=6 are the same bytes")
        variants.append(Variant("send side P=1 (messages only)", None, None, None, c1, s1))
    # P = 6 on a copy of the state, P = 1 in place
    g6, m6, w6 = g0.clone(), mom0.clone(), [w.clone() for w in wn0]
    for p in range(6):
        sdl.sdl_fragment_outer_step_plan(p6, p, g6, m6, one.w_send, w6, f, wl.lr, wl.mu, wl.alpha)
    one.step(0, fmt=f)
    torch.cuda.synchronize()
    assert torch.equal(one.g.view(torch.int32), g6.view(torch.int32))
    assert torch.equal(one.mom.view(torch.int32), m6.view(torch.int32))
    for a, b in zip(one.w_now, w6):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    del g6, m6, w6
    say(f"4b {fmt}: P=1 and P=6 give the same model")
    variants.append(Variant("fused P=1", one.g, one.mom, one.w_now))
    counts = stream_check(one.plan, 0, f, wl.lr, wl.mu, wl.alpha, g0=g0, mom0=mom0, w_send=one.w_send, w_now0=wn0,
                          variants=variants, what=f"4b P=1 {fmt}", progress=say)
    assert counts["elements"] == total
    if fmt == "e3m0":
        assert counts["code_bytes"] == M * total // 2 and counts["scale_bytes"] == M * total // 32


@pytest.mark.parametrize("M,n_spans", [(9, 7), (2, 150), (9, 70)])
def test_whole_span_scale_prepass_batches(M, n_spans):
    """The pre-pass of the whole-span scale takes 64 spans and 8 replicas per launch: more spans and
    more replicas than that, deterministically (ragged spans, one fragment)."""
    rng = np.random.default_rng(100 * M + n_spans)
    numel = [int(x) for x in rng.integers(1, 3000, n_spans - 2)] + [40000, 1]
    plan = sdl.sdl_fragment_plan(numel, [0] * n_spans, 1, 1, sdl.PATTERN_STRIDED, 100, 1)
    fmt = sdl.FMT_E3M0_SPAN
    total = plan.total_numel
    g, mom, w_send, w_now = workloads.make_span(total, M, tau=1, delta="outliers", base_seed=n_spans, device=DEV)
    host = HostCopy(g, mom, w_send, w_now)
    codes, scales = _messages(plan, 0, fmt, M)
    sdl.sdl_fragment_outer_step_plan_ex(plan, 0, g, mom, w_send, w_now, fmt, 0.7, 0.9, 0.5, codes, scales)
    torch.cuda.synchronize()
    pos = message_positions(plan, 0, fmt)
    for i, (off, n, _) in enumerate(sdl.sdl_plan_fragment_spans(plan, 0)):
        sl = slice(off, off + n)
        rc, rs = oracle.fragment_outer_step(host.g[sl], host.mom[sl], [w[sl] for w in host.w_send],
                                            [w[sl] for w in host.w_now], fmt, 0.7, 0.9, 0.5, want_codes=True)
        for m in range(M):
            a = pos[off] // 2
            assert_bytes_equal(codes[m][a:a + rc[m].size].cpu().numpy(), rc[m], f"codes[{m}] span {i}")
            assert_bytes_equal(scales[m][4 * i:4 * i + 4].cpu().numpy(), rs[m], f"scale word[{m}] span {i}")
    assert_f32_close(host_f32(g), host.g, "g")
    assert_f32_close(host_f32(mom), host.mom, "mom")
    for m in range(M):
        assert_bf16_within_ulp(host_bits(w_now[m]), host.w_now[m], f"w_now[{m}]")
