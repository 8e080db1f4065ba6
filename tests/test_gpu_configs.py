"""GPU parity at the benchmark configurations, in the launch configuration bench.py times
(sdl_fragment_outer_step_plan on flat model arrays).  The two small configurations are compared
in full here; the three large ones (1B fragment, 4B model, stress fragment) are compared in full,
every element and every message byte, in test_gpu_configs_full.py.  What remains sampled here are
the variations around the stress configuration (three formats x three values of alpha), on
block-aligned windows, plus size-independent properties."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_18512_amd as sdl
import workloads
from gpu_util import (FlatModel, HostCopy, assert_bf16_within_ulp, assert_bytes_equal, assert_f32_close,
                      check_fused_against_oracle, host_bits, host_f32)

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_config_tiny():
    wl = workloads.WORKLOADS["tiny"]
    n = wl.flat_numel
    g, mom, w_send, w_now = workloads.make_span(n, wl.M, tau=wl.tau, delta=wl.delta, base_seed=wl.seed,
                                                device=DEV)
    ref = check_fused_against_oracle(g, mom, w_send, w_now, sdl.FORMATS[wl.fmt], wl.lr, wl.mu, wl.alpha,
                                     emit=True, what="tiny, first outer step")
    # second round: the replicas move on, the momentum is no longer zero
    for w in w_now:
        w.copy_((w.float() + torch.randn(n, device=DEV) * 1e-3).bfloat16())
    check_fused_against_oracle(g, mom, w_now, w_now, sdl.FORMATS[wl.fmt], wl.lr, wl.mu, wl.alpha,
                               emit=True, what="tiny, second outer step")
    assert float(mom.abs().max()) > 0


def test_config_100m_all_fragments_two_rounds():
    wl = workloads.WORKLOADS["100m"]
    model = FlatModel(wl)
    assert [sdl.sdl_plan_offset(model.plan, p) for p in range(3)] == [0, 33, 66]
    host = HostCopy(model.g, model.mom, model.w_send, model.w_now)
    gen = torch.Generator(DEV).manual_seed(1)
    for rnd in (1, 2):
        for p in range(wl.P):
            print(f"100m round {rnd} fragment {p}", flush=True)
            model.step(p)
        torch.cuda.synchronize()
        # the oracle walks the spans (one per parameter group), not the joined runs
        for p in range(wl.P):
            for off, n, _ in sdl.sdl_plan_fragment_spans(model.plan, p):
                sl = slice(off, off + n)
                oracle.fragment_outer_step_chunked(host.g[sl], host.mom[sl], [w[sl] for w in host.w_send],
                                                   [w[sl] for w in host.w_now], sdl.FORMATS[wl.fmt],
                                                   wl.lr, wl.mu, wl.alpha, threads=8)
        assert_f32_close(host_f32(model.g), host.g, f"100m round {rnd} g")
        assert_f32_close(host_f32(model.mom), host.mom, f"100m round {rnd} mom")
        for m in range(wl.M):
            assert_bf16_within_ulp(host_bits(model.w_now[m]), host.w_now[m], f"100m round {rnd} w_now[{m}]")
        if rnd == 1:
            # next outer round: replicas continue from the merged state (input generation only)
            for m in range(wl.M):
                model.w_send[m].copy_((model.w_now[m].float() + torch.randn(
                    model.g.numel(), device=DEV, generator=gen) * 1e-3).bfloat16())
                model.w_now[m].copy_((model.w_send[m].float() + torch.randn(
                    model.g.numel(), device=DEV, generator=gen) * 1e-4).bfloat16())
            host = HostCopy(model.g, model.mom, model.w_send, model.w_now)
    assert float(np.abs(host.mom).max()) > 0


def test_config_1b_fragment_touches_nothing_else():
    """Size-independent property of the plan-level call: a step of fragment 1 leaves every other
    fragment's parameters bit for bit as they were."""
    wl = workloads.WORKLOADS["1b"]
    model = FlatModel(wl, fill_fragments=[0, 1])
    runs = sdl.sdl_plan_fragment_runs(model.plan, 1)
    assert sum(n for _, n, _ in runs) == 302014464 and len(runs) == 6
    others = [(o, n) for o, n, _ in sdl.sdl_plan_fragment_spans(model.plan, 0)]
    before = [(model.g[o:o + n].clone(), model.mom[o:o + n].clone(), [w[o:o + n].clone() for w in model.w_now])
              for o, n in others]
    model.step(1)
    torch.cuda.synchronize()
    for (o, n), (g0, m0, w0) in zip(others, before):
        assert torch.equal(g0.view(torch.int32), model.g[o:o + n].view(torch.int32))
        assert torch.equal(m0.view(torch.int32), model.mom[o:o + n].view(torch.int32))
        for a, b in zip(w0, model.w_now):
            assert torch.equal(a.view(torch.int16), b[o:o + n].view(torch.int16))


@pytest.mark.parametrize("fmt", ["e3m0", "e4m3", "bf16"])
def test_config_stress_m8_variations_sampled(fmt):
    wl = workloads.WORKLOADS["stress"]
    f = sdl.FORMATS[fmt]
    model = FlatModel(wl, fill_fragments=[1])
    wins = model.windows(1, n_random=4, width=1 << 14, seed=5)
    for alpha in (0.0, 0.5, 1.0):
        print(f"stress fmt={fmt} alpha={alpha}", flush=True)
        snaps = model.snapshot(wins)
        model.step(1, fmt=f, alpha=alpha)
        torch.cuda.synchronize()
        model.verify(wins, snaps, fmt=f, alpha=alpha, what=f"stress {fmt} alpha={alpha}")
    # receive side alone on one run of the fragment: messages from the GPU send side,
    # checked against the oracle's on a sampled window
    off, n, _ = sdl.sdl_plan_fragment_runs(model.plan, 1)[0]
    sl = slice(off, off + n)
    codes, scales = sdl.alloc_exchange(f, n, wl.M)
    sdl.sdl_quantize_outer_grad(model.g[sl], [w[sl] for w in model.w_send], n, f, codes, scales)
    lo, width = 32 * 1000, 1 << 14
    ref = HostCopy(model.g[sl][lo:lo + width], model.mom[sl][lo:lo + width],
                   [w[sl][lo:lo + width] for w in model.w_send], [w[sl][lo:lo + width] for w in model.w_now])
    sdl.sdl_dequant_reduce_nesterov(model.g[sl], model.mom[sl], codes, scales, n, f, wl.lr, wl.mu)
    torch.cuda.synchronize()
    rc, rs = oracle.quantize_outer_grad(ref.g, ref.w_send, f)
    cb, sb = sdl.sdl_exchange_bytes(f, width)
    c0 = sdl.sdl_exchange_bytes(f, lo)[0]
    for m in range(wl.M):
        assert_bytes_equal(codes[m][c0:c0 + cb].cpu().numpy(), rc[m], f"stress codes[{m}]")
        if sb:
            assert_bytes_equal(scales[m][lo // 32:lo // 32 + sb].cpu().numpy(), rs[m], f"stress scales[{m}]")
    oracle.dequant_reduce_nesterov(ref.g, ref.mom, rc, rs, f, wl.lr, wl.mu)
    assert_f32_close(host_f32(model.g[sl][lo:lo + width]), ref.g, "stress reduce g")
    assert_f32_close(host_f32(model.mom[sl][lo:lo + width]), ref.mom, "stress reduce mom")


def test_plan_call_with_many_ragged_runs():
    """More runs than one launch holds (16), ragged and partly unaligned: spans whose lengths are
    not multiples of 128 end their run, so nearly every span is its own run, with its own block grid."""
    rng = np.random.default_rng(3)
    numel = [int(x) for x in rng.integers(1, 5000, 45)] + [4096, 512, 33, 2048 * 3]
    block = [i % 7 for i in range(len(numel))]
    P, M, fmt = 3, 3, sdl.FMT_E3M0
    plan = sdl.sdl_fragment_plan(numel, block, 7, P, sdl.PATTERN_STRIDED, 100, 1)
    total = plan.total_numel
    g, mom, w_send, w_now = workloads.make_span(total, M, tau=1, delta="student_t3", device=DEV)
    host = HostCopy(g, mom, w_send, w_now)
    for p in range(P):
        runs = sdl.sdl_plan_fragment_runs(plan, p)
        assert len(runs) > 16 or p > 0
        sdl.sdl_fragment_outer_step_plan(plan, p, g, mom, w_send, w_now, fmt, 0.7, 0.9, 0.5)
        for off, n, _ in sdl.sdl_plan_fragment_spans(plan, p):
            sl = slice(off, off + n)
            oracle.fragment_outer_step(host.g[sl], host.mom[sl], [w[sl] for w in host.w_send],
                                       [w[sl] for w in host.w_now], fmt, 0.7, 0.9, 0.5)
    torch.cuda.synchronize()
    assert_f32_close(host_f32(g), host.g, "ragged plan g")
    assert_f32_close(host_f32(mom), host.mom, "ragged plan mom")
    for m in range(M):
        assert_bf16_within_ulp(host_bits(w_now[m]), host.w_now[m], f"ragged plan w_now[{m}]")


@pytest.mark.parametrize("M", [6, 16])
def test_generic_replica_count_large_span(M):
    """Replica counts without a compile-time variant, on a span of several thousand tiles."""
    n = 3_000_000 + 77
    g, mom, w_send, w_now = workloads.make_span(n, M, tau=1, delta="outliers", device=DEV)
    check_fused_against_oracle(g, mom, w_send, w_now, sdl.FMT_E3M0, 0.7, 0.9, 0.5, emit=False,
                               what=f"generic M={M}")
