"""Seeded random sweep of the fragment-level fused call against the oracle: random models
(number and sizes of parameter groups, ragged and block-aligned, blocks, embedding/head groups),
fragment count and pattern, layout with or without padding, format, replica count, aliasing, flat
or staged outer state, messages written or not.  The oracle walks the parameter groups of its own
plan one by one."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2501_18512_amd as sdl
import workloads
from gpu_util import (HostCopy, assert_bf16_within_ulp, assert_bytes_equal, assert_f32_close, host_bits,
                      host_f32)

pytestmark = pytest.mark.gpu
DEV = "cuda"
FMTS = [sdl.FMT_E3M0, sdl.FMT_E4M3, sdl.FMT_BF16, sdl.FMT_FP32, sdl.FMT_E3M0_B64, sdl.FMT_E3M0_B128,
        sdl.FMT_E3M0_SPAN, sdl.FMT_E3M0_RN]
PAD = 512        # message and staging layouts pad every piece to a multiple of 512 elements


def _model(rng):
    L = int(rng.integers(1, 10))
    numel, block = [], []
    if rng.integers(0, 2):
        numel.append(int(rng.choice([4096, 1000, 128 * 37])))
        block.append(sdl.UNIT_PRE)
    for b in range(L):
        for _ in range(int(rng.integers(1, 12))):
            kind = int(rng.integers(0, 5))
            if kind == 0:
                n = 128 * int(rng.integers(1, 40))          # joins with its neighbours
            elif kind == 1:
                n = 512 * int(rng.integers(1, 24))
            elif kind == 2:
                n = int(rng.integers(1, 3000))               # ragged: ends a run
            elif kind == 3:
                n = 32 * int(rng.integers(1, 64))            # whole 32-blocks, not whole 128-blocks
            else:
                n = int(rng.integers(20000, 60000))
            numel.append(n)
            block.append(b)
    for _ in range(int(rng.integers(0, 3))):
        numel.append(int(rng.choice([64, 2048, 777])))
        block.append(sdl.UNIT_POST)
    return numel, block, L


def _padded(n):
    return (n + PAD - 1) // PAD * PAD


N_CHUNKS = int(os.environ.get("SDL_TEST_RANDOM_CHUNKS", "6"))


@pytest.mark.parametrize("chunk", range(N_CHUNKS))
def test_random_fragment_level_fused_calls(chunk):
    rng = np.random.default_rng(5000 + chunk)
    for i in range(6):
        numel, block, L = _model(rng)
        P = int(rng.integers(1, L + 1))
        pattern = int(rng.choice([sdl.PATTERN_STRIDED, sdl.PATTERN_SEQUENTIAL]))
        own = bool(rng.integers(0, 2)) and block[0] == sdl.UNIT_PRE
        fmt = FMTS[int(rng.integers(len(FMTS)))]
        M = int(rng.choice([1, 2, 3, 4, 8, 9]))
        tau = int(rng.integers(0, 2))
        emit, staged = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        padded = bool(rng.integers(0, 2))            # groups laid out on 64-element boundaries
        lr, mu, alpha = float(rng.choice([0.4, 0.7])), float(rng.choice([0.0, 0.9])), float(rng.choice([0.0, 0.5, 1.0]))
        seed = int(rng.integers(1 << 30))
        print(f"random plan case {chunk}.{i}: units={len(numel)} L={L} P={P} pattern={pattern} own={own} "
              f"fmt={fmt} M={M} tau={tau} emit={emit} staged={staged} padded={padded} seed={seed}", flush=True)
        plan = sdl.sdl_fragment_plan_ex(numel, block, L, P, pattern, 10, tau,
                                        flags=(sdl.PLAN_PRE_OWN_FRAGMENT if own else 0)
                                        | (sdl.PLAN_ALIGN_GROUPS if padded else 0))
        ref_plan = oracle.fragment_plan(numel, block, L, P, pattern, 10, tau, pre_own_fragment=own,
                                        align=sdl.PLAN_GROUP_ALIGN if padded else 1)
        total = plan.total_numel
        assert total == ref_plan.total
        g, mom, w_send, w_now = workloads.make_span(total, M, tau=tau, delta="student_t3", base_seed=seed,
                                                    device=DEV)
        mom.copy_(torch.randn(total, device=DEV, generator=torch.Generator(DEV).manual_seed(seed)) * 1e-3)
        host = HostCopy(g, mom, w_send, w_now)
        for p in range(ref_plan.P):
            spans = [s for s in ref_plan.spans[p] if s[1] > 0]
            runs = sdl.sdl_plan_fragment_runs(plan, p)
            assert [(o, n, u) for o, n, u in sdl.sdl_plan_fragment_spans(plan, p) if n > 0] == spans
            pieces = spans if fmt == sdl.FMT_E3M0_SPAN else runs
            cb, sb = sdl.sdl_plan_message_bytes(plan, p, fmt)
            codes = [torch.zeros(max(cb, 16), dtype=torch.uint8, device=DEV) for _ in range(M)]
            scales = [torch.zeros(max(sb, 16), dtype=torch.uint8, device=DEV) for _ in range(M)]
            need_scales = emit or fmt == sdl.FMT_E3M0_SPAN
            args = (fmt, lr, mu, alpha, codes if emit else None, scales if need_scales else None)
            if staged:
                ns = sdl.sdl_plan_staged_numel(plan, p)
                assert ns == sum(_padded(n) for _, n, _ in runs)
                gf = torch.zeros(max(ns, 1), dtype=torch.float32, device=DEV)
                mf = torch.zeros(max(ns, 1), dtype=torch.float32, device=DEV)
                pos = 0
                for o, n, _ in runs:
                    gf[pos:pos + n].copy_(g[o:o + n])
                    mf[pos:pos + n].copy_(mom[o:o + n])
                    pos += _padded(n)
                sdl.sdl_fragment_outer_step_staged_ex(plan, p, gf, mf, w_send, w_now, *args)
                pos = 0
                for o, n, _ in runs:
                    g[o:o + n].copy_(gf[pos:pos + n])
                    mom[o:o + n].copy_(mf[pos:pos + n])
                    pos += _padded(n)
            else:
                sdl.sdl_fragment_outer_step_plan_ex(plan, p, g, mom, w_send, w_now, *args)
            torch.cuda.synchronize()
            # the oracle, group by group; its messages go where the layout puts that group
            start = {}
            pos = 0
            for o, n, _ in pieces:
                start[o] = pos
                pos += _padded(n)
            got_c = [c.cpu().numpy() for c in codes]
            got_s = [s.cpu().numpy() for s in scales]
            for k, (o, n, _) in enumerate(spans):
                sl = slice(o, o + n)
                rc, rs = oracle.fragment_outer_step(host.g[sl], host.mom[sl], [w[sl] for w in host.w_send],
                                                    [w[sl] for w in host.w_now], fmt, lr, mu, alpha,
                                                    want_codes=True)
                if not emit:
                    continue
                po = max(q for q in start if q <= o)          # the piece this group lies in
                rel = start[po] + (o - po)                    # element position inside the message
                assert (o - po) % 128 == 0
                c0 = sdl.sdl_exchange_bytes(fmt, rel)[0]
                nb = sdl.sdl_exchange_bytes(fmt, n)[0]
                for m in range(M):
                    assert_bytes_equal(got_c[m][c0:c0 + nb], rc[m], f"fragment {p} group {k} codes[{m}]")
                    if fmt == sdl.FMT_E3M0_SPAN:
                        assert_bytes_equal(got_s[m][4 * k:4 * k + 4], rs[m], f"fragment {p} group {k} scale word[{m}]")
                    elif len(rs[m]):
                        s0 = sdl.sdl_exchange_bytes(fmt, rel)[1]
                        assert_bytes_equal(got_s[m][s0:s0 + len(rs[m])], rs[m], f"fragment {p} group {k} scales[{m}]")
        assert_f32_close(host_f32(g), host.g, "g")
        assert_f32_close(host_f32(mom), host.mom, "mom")
        for m in range(M):
            assert_bf16_within_ulp(host_bits(w_now[m]), host.w_now[m], f"w_now[{m}]")
