"""Seeded random sweep of the span-level calls against the oracle: format, replica count, size,
element offsets of every array (so that 16-byte alignment comes and goes independently per
array), hyper-parameters, delta distribution, aliasing and whether messages are written."""
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
DELTAS = ["normal", "student_t3", "outliers", "shared10"]


def _case(rng):
    fmt = FMTS[int(rng.integers(len(FMTS)))]
    M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 11, 16]))
    n = int(rng.choice([int(rng.integers(1, 600)), int(rng.integers(600, 5000)), int(rng.integers(5000, 70000))]))
    return dict(fmt=fmt, M=M, n=n, tau=int(rng.integers(0, 3)), delta=DELTAS[int(rng.integers(len(DELTAS)))],
                lr=float(rng.choice([0.4, 0.7, 1.0])), mu=float(rng.choice([0.0, 0.9, 0.5])),
                alpha=float(rng.choice([0.0, 0.5, 1.0, 0.25, 0.8])),
                off_g=int(rng.integers(0, 4)), off_mom=int(rng.integers(0, 4)),
                off_w=[int(rng.integers(0, 8)) for _ in range(M)], emit=bool(rng.integers(0, 2)),
                seed=int(rng.integers(1 << 30)))


def _make(c):
    """Arrays with independent element offsets into slightly larger allocations."""
    n, M = c["n"], c["M"]
    g0, mom0, ws0, wn0 = workloads.make_span(n + 8, M, tau=c["tau"], delta=c["delta"], unit=c["seed"] % 101,
                                             base_seed=c["seed"], device=DEV)
    mom0.copy_(torch.randn(n + 8, device=DEV, generator=torch.Generator(DEV).manual_seed(c["seed"])) * 1e-3)
    g = g0[c["off_g"]:c["off_g"] + n]
    mom = mom0[c["off_mom"]:c["off_mom"] + n]
    w_send = [w[o:o + n] for w, o in zip(ws0, c["off_w"])]
    for w, o in zip(w_send, c["off_w"]):
        # keep the recipe's small deltas: re-pair the shifted replica with the shifted g
        w.copy_((g - (g0[o:o + n] - w.float())).bfloat16())
    if c["tau"] == 0:
        w_now = w_send
    else:
        w_now = [w[o:o + n] for w, o in zip(wn0, c["off_w"])]
        for a, b in zip(w_now, w_send):
            a.copy_((b.float() + torch.randn(n, device=DEV, generator=torch.Generator(DEV).manual_seed(
                c["seed"] + 1)) * 1e-4 * c["tau"]).bfloat16())
    return g, mom, w_send, w_now


# more seeds on request (a soak of the same sweep): SDL_TEST_RANDOM_CHUNKS=100 python -m pytest ...
N_CHUNKS = int(os.environ.get("SDL_TEST_RANDOM_CHUNKS", "8"))


@pytest.mark.parametrize("chunk", range(N_CHUNKS))
def test_random_fused_and_unfused_cases(chunk):
    rng = np.random.default_rng(1000 + chunk)
    for i in range(24):
        c = _case(rng)
        print(f"random case {chunk}.{i}: {c}", flush=True)
        n, M, fmt = c["n"], c["M"], c["fmt"]
        g, mom, w_send, w_now = _make(c)
        ref = HostCopy(g, mom, w_send, w_now)
        cb, sb = sdl.sdl_exchange_bytes(fmt, n)
        if i % 2 == 0:
            # fused call
            codes, scales = sdl.alloc_exchange(fmt, n, M)
            need_scales = c["emit"] or fmt == sdl.FMT_E3M0_SPAN
            sdl.sdl_fragment_outer_step(g, mom, w_send, w_now, n, fmt, c["lr"], c["mu"], c["alpha"],
                                        codes if c["emit"] else None, scales if need_scales else None)
            torch.cuda.synchronize()
            rc, rs = oracle.fragment_outer_step(ref.g, ref.mom, ref.w_send, ref.w_now, fmt, c["lr"], c["mu"],
                                                c["alpha"], want_codes=True)
            if c["emit"]:
                for m in range(M):
                    assert_bytes_equal(codes[m][:cb].cpu().numpy(), rc[m], f"codes[{m}]")
                    if sb:
                        assert_bytes_equal(scales[m][:sb].cpu().numpy(), rs[m], f"scales[{m}]")
        else:
            # send side, then either the one-pass receive side or its two halves
            codes, scales = sdl.alloc_exchange(fmt, n, M)
            sdl.sdl_quantize_outer_grad(g, w_send, n, fmt, codes, scales)
            if c["emit"]:
                sdl.sdl_receive_outer_step(g, mom, codes, scales, w_now, n, fmt, c["lr"], c["mu"], c["alpha"])
            else:
                sdl.sdl_dequant_reduce_nesterov(g, mom, codes, scales, n, fmt, c["lr"], c["mu"])
                sdl.sdl_merge_overlap(g, w_now, n, c["alpha"])
            torch.cuda.synchronize()
            rc, rs = oracle.quantize_outer_grad(ref.g, ref.w_send, fmt)
            for m in range(M):
                assert_bytes_equal(codes[m][:cb].cpu().numpy(), rc[m], f"codes[{m}]")
                if sb:
                    assert_bytes_equal(scales[m][:sb].cpu().numpy(), rs[m], f"scales[{m}]")
            oracle.dequant_reduce_nesterov(ref.g, ref.mom, rc, rs, fmt, c["lr"], c["mu"])
            oracle.merge_overlap(ref.g, ref.w_now, c["alpha"])
        assert_f32_close(host_f32(g), ref.g, "g")
        assert_f32_close(host_f32(mom), ref.mom, "mom")
        for m in range(M):
            assert_bf16_within_ulp(host_bits(w_now[m]), ref.w_now[m], f"w_now[{m}]")
