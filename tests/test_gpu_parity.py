"""GPU parity: every C-ABI device call against the CPU oracle on the same seeded bits,
element by element, at sizes that span several workgroup tiles (2048 elements) and end in
ragged tails, for every exchange format and replica count, plus the degenerate cases."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_18512_amd as sdl
import workloads
from gpu_util import (HostCopy, assert_bf16_within_ulp, assert_bytes_equal, assert_f32_close,
                      check_fused_against_oracle, host_bits, host_f32)

pytestmark = pytest.mark.gpu
DEV = "cuda"
LR, MU = 0.7, 0.9
SIZES = [1, 7, 8, 31, 32, 33, 255, 2047, 2048, 2049, 3 * 2048 + 77, 20000 + 13]
FMTS = [sdl.FMT_E3M0, sdl.FMT_E4M3, sdl.FMT_BF16, sdl.FMT_FP32, sdl.FMT_E3M0_B64, sdl.FMT_E3M0_B128,
        sdl.FMT_E3M0_SPAN, sdl.FMT_E3M0_RN]


def _span(n, M, tau=1, delta="normal", seed=0):
    return workloads.make_span(n, M, tau=tau, delta=delta, unit=n % 97, base_seed=seed, device=DEV)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M", [1, 2, 3, 4, 8])
def test_quantize_bit_exact(fmt, M):
    for n in SIZES:
        print(f"quantize fmt={fmt} M={M} n={n}", flush=True)
        g, mom, w_send, _ = _span(n, M, delta="student_t3")
        codes, scales = sdl.alloc_exchange(fmt, n, M)
        sdl.sdl_quantize_outer_grad(g, w_send, n, fmt, codes, scales)
        torch.cuda.synchronize()
        rc, rs = oracle.quantize_outer_grad(host_f32(g), [host_bits(w) for w in w_send], fmt)
        cb, sb = sdl.sdl_exchange_bytes(fmt, n)
        for m in range(M):
            assert_bytes_equal(codes[m][:cb].cpu().numpy(), rc[m], f"codes[{m}] n={n}")
            if sb:
                assert_bytes_equal(scales[m][:sb].cpu().numpy(), rs[m], f"scales[{m}] n={n}")


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M", [1, 2, 3, 4, 8])
def test_dequant_reduce_nesterov(fmt, M):
    for n in SIZES:
        print(f"reduce fmt={fmt} M={M} n={n}", flush=True)
        g, mom, w_send, _ = _span(n, M, delta="outliers")
        mom.copy_(torch.randn(n, device=DEV, generator=torch.Generator(DEV).manual_seed(n)) * 1e-3)
        hg, hmom = host_f32(g), host_f32(mom)
        rc, rs = oracle.quantize_outer_grad(hg, [host_bits(w) for w in w_send], fmt)
        # the messages come from the oracle: this isolates the receive side
        codes, scales = sdl.alloc_exchange(fmt, n, M)
        for m in range(M):
            codes[m][:rc[m].size].copy_(torch.from_numpy(rc[m]))
            scales[m][:rs[m].size].copy_(torch.from_numpy(rs[m]))
        sdl.sdl_dequant_reduce_nesterov(g, mom, codes, scales, n, fmt, LR, MU)
        torch.cuda.synchronize()
        oracle.dequant_reduce_nesterov(hg, hmom, rc, rs, fmt, LR, MU)
        assert_f32_close(host_f32(g), hg, f"g n={n}")
        assert_f32_close(host_f32(mom), hmom, f"mom n={n}")


@pytest.mark.parametrize("fmt", [sdl.FMT_E3M0, sdl.FMT_E4M3, sdl.FMT_E3M0_B64, sdl.FMT_E3M0_B128, sdl.FMT_E3M0_RN])
@pytest.mark.parametrize("M", [1, 3])
def test_receive_side_decodes_every_code_and_scale(fmt, M):
    """Messages are plain bytes: whatever a peer sends is decoded like the oracle decodes it,
    including the codes the encoder never produces and the extreme scale bytes."""
    n = 4 * 2048 + 96
    rng = np.random.default_rng(1234 + fmt)
    cb, sb = sdl.sdl_exchange_bytes(fmt, n)
    rc, rs = [], []
    for m in range(M):
        c = rng.integers(0, 256, cb, dtype=np.uint8)
        c[:256] = np.arange(256, dtype=np.uint8)                 # every byte value at least once
        s = rng.integers(100, 150, sb, dtype=np.uint8)
        s[:8] = [0, 1, 2, 127, 253, 254, 255, 126]
        rc.append(c), rs.append(s)
    hg = rng.standard_normal(n).astype(np.float32)
    hmom = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g, mom = torch.from_numpy(hg).to(DEV), torch.from_numpy(hmom).to(DEV)
    codes, scales = sdl.alloc_exchange(fmt, n, M)
    for m in range(M):
        codes[m][:cb].copy_(torch.from_numpy(rc[m]))
        scales[m][:sb].copy_(torch.from_numpy(rs[m]))
    sdl.sdl_dequant_reduce_nesterov(g, mom, codes, scales, n, fmt, LR, MU)
    torch.cuda.synchronize()
    oracle.dequant_reduce_nesterov(hg, hmom, rc, rs, fmt, LR, MU)
    assert np.isnan(hg).any() and np.isfinite(hg).any()
    assert_f32_close(host_f32(g), hg, "g")
    assert_f32_close(host_f32(mom), hmom, "mom")


@pytest.mark.parametrize("alpha", [0.0, 0.5, 1.0, 0.3])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 8])
def test_merge_overlap(alpha, M):
    for n in SIZES:
        print(f"merge alpha={alpha} M={M} n={n}", flush=True)
        g, _, _, w_now = _span(n, M)
        hg, hw = host_f32(g), [host_bits(w) for w in w_now]
        sdl.sdl_merge_overlap(g, w_now, n, alpha)
        torch.cuda.synchronize()
        oracle.merge_overlap(hg, hw, alpha)
        for m in range(M):
            assert_bf16_within_ulp(host_bits(w_now[m]), hw[m], f"w_now[{m}] n={n}")
        assert np.array_equal(host_f32(g), hg)          # g_new is read-only


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 16])
@pytest.mark.parametrize("tau", [0, 1])
def test_fused_step(fmt, M, tau):
    for n in SIZES:
        print(f"fused fmt={fmt} M={M} tau={tau} n={n}", flush=True)
        g, mom, w_send, w_now = _span(n, M, tau=tau, delta="student_t3")
        mom.copy_(torch.randn(n, device=DEV, generator=torch.Generator(DEV).manual_seed(n + 1)) * 1e-3)
        check_fused_against_oracle(g, mom, w_send, w_now, fmt, LR, MU, 0.5, emit=(n % 2 == 1),
                                   what=f"fmt={fmt} M={M} tau={tau} n={n}")


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("M", [1, 3, 4, 8])
def test_receive_outer_step(fmt, M):
    """Mean + Nesterov + merge of all replicas in one pass, against the oracle's two steps."""
    for n in SIZES:
        print(f"receive fmt={fmt} M={M} n={n}", flush=True)
        g, mom, w_send, w_now = _span(n, M, tau=1, delta="student_t3")
        mom.copy_(torch.randn(n, device=DEV, generator=torch.Generator(DEV).manual_seed(n + 2)) * 1e-3)
        ref = HostCopy(g, mom, w_send, w_now)
        rc, rs = oracle.quantize_outer_grad(ref.g, ref.w_send, fmt)
        codes, scales = sdl.alloc_exchange(fmt, n, M)
        for m in range(M):
            codes[m][:rc[m].size].copy_(torch.from_numpy(rc[m]))
            scales[m][:rs[m].size].copy_(torch.from_numpy(rs[m]))
        sdl.sdl_receive_outer_step(g, mom, codes, scales, w_now, n, fmt, LR, MU, 0.5)
        torch.cuda.synchronize()
        oracle.dequant_reduce_nesterov(ref.g, ref.mom, rc, rs, fmt, LR, MU)
        oracle.merge_overlap(ref.g, ref.w_now, 0.5)
        assert_f32_close(host_f32(g), ref.g, f"g n={n}")
        assert_f32_close(host_f32(mom), ref.mom, f"mom n={n}")
        for m in range(M):
            assert_bf16_within_ulp(host_bits(w_now[m]), ref.w_now[m], f"w_now[{m}] n={n}")


@pytest.mark.parametrize("fmt", FMTS)
def test_fused_equals_three_calls_on_gpu(fmt):
    n, M = 5 * 2048 + 19, 4
    g, mom, w_send, w_now = _span(n, M, tau=1)
    g2, mom2 = g.clone(), mom.clone()
    ws2, wn2 = [w.clone() for w in w_send], [w.clone() for w in w_now]
    codes, scales = sdl.alloc_exchange(fmt, n, M)
    # (the whole-span scale needs its scale words as workspace even when no message is written)
    work = sdl.alloc_exchange(fmt, n, M)[1] if fmt == sdl.FMT_E3M0_SPAN else None
    sdl.sdl_fragment_outer_step(g, mom, w_send, w_now, n, fmt, LR, MU, 0.5, scales=work)
    sdl.sdl_quantize_outer_grad(g2, ws2, n, fmt, codes, scales)
    sdl.sdl_dequant_reduce_nesterov(g2, mom2, codes, scales, n, fmt, LR, MU)
    sdl.sdl_merge_overlap(g2, wn2, n, 0.5)
    torch.cuda.synchronize()
    assert torch.equal(g, g2) and torch.equal(mom, mom2)
    for a, b in zip(w_now, wn2):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("fmt", FMTS)
def test_unaligned_model_arrays(fmt):
    """Model arrays that start at odd element offsets (4-byte / 2-byte aligned only): whole tiles
    go through element-aligned vectors, the ragged last tile element by element."""
    n, M = 2 * 2048 + 5, 2
    g, mom, w_send, w_now = _span(n + 3, M, tau=1)
    views = (g[1:1 + n], mom[3:3 + n], [w[1:1 + n] for w in w_send], [w[3:3 + n] for w in w_now])
    assert views[0].data_ptr() % 16 != 0 and views[2][0].data_ptr() % 16 != 0
    check_fused_against_oracle(*views, fmt, LR, MU, 0.5, emit=True, what=f"unaligned fmt={fmt}")


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("model_offset", [0, 1])
def test_unaligned_message_arrays(fmt, model_offset):
    """Message arrays at the smallest alignment their element type allows (1 byte for the 4- and
    8-bit codes, 2 / 4 bytes for bf16 / fp32): every tile goes element by element."""
    n, M = 3 * 512 + 77, 2
    g0, mom0, ws0, wn0 = _span(n + 1, M, tau=1, delta="student_t3")
    o = model_offset
    g, mom = g0[o:o + n], mom0[o:o + n]
    w_send, w_now = [w[o:o + n] for w in ws0], [w[o:o + n] for w in wn0]
    ref = HostCopy(g, mom, w_send, w_now)
    cb, sb = sdl.sdl_exchange_bytes(fmt, n)
    step = {sdl.FMT_FP32: 4, sdl.FMT_BF16: 2}.get(fmt, 1)
    code_bufs = [torch.zeros(cb + 16, dtype=torch.uint8, device=DEV) for _ in range(M)]
    codes = [b[step:] for b in code_bufs]
    assert codes[0].data_ptr() % 16 == step
    scales = sdl.alloc_exchange(fmt, n, M)[1]
    sdl.sdl_quantize_outer_grad(g, w_send, n, fmt, codes, scales)
    sdl.sdl_receive_outer_step(g, mom, codes, scales, w_now, n, fmt, LR, MU, 0.5)
    torch.cuda.synchronize()
    rc, rs = oracle.fragment_outer_step(ref.g, ref.mom, ref.w_send, ref.w_now, fmt, LR, MU, 0.5, want_codes=True)
    for m in range(M):
        assert_bytes_equal(codes[m][:cb].cpu().numpy(), rc[m], f"codes[{m}]")
        if sb:
            assert_bytes_equal(scales[m][:sb].cpu().numpy(), rs[m], f"scales[{m}]")
        assert code_bufs[m][:step].sum() == 0 and code_bufs[m][step + cb:].sum() == 0
    assert_f32_close(host_f32(g), ref.g, "g")
    assert_f32_close(host_f32(mom), ref.mom, "mom")
    for m in range(M):
        assert_bf16_within_ulp(host_bits(w_now[m]), ref.w_now[m], f"w_now[{m}]")


def _from_host(g, mom, w_send, w_now):
    return (torch.from_numpy(g).to(DEV), torch.from_numpy(mom).to(DEV),
            [workloads.bits_bf16(w, DEV) for w in w_send], [workloads.bits_bf16(w, DEV) for w in w_now])


@pytest.mark.parametrize("fmt", FMTS)
def test_degenerate_blocks(fmt):
    """Zero blocks, fp32-subnormal maxima, scale-byte clamp at 0, huge values, Inf and NaN."""
    n = 32 * 12
    g = np.zeros(n, np.float32)
    w = np.zeros(n, np.float32)
    g[32:64] = np.float32(1e-40) * np.arange(32)                # subnormal block maximum
    g[64:96] = np.float32(2.0 ** -123) * np.linspace(-1, 1, 32).astype(np.float32)   # sb clamps to 0
    g[96:128] = np.float32(3e38) * np.linspace(-1, 1, 32).astype(np.float32)         # largest binade
    g[128:160] = np.linspace(-1, 1, 32)
    g[130] = np.inf
    g[160:192] = np.linspace(-1, 1, 32)
    g[170] = np.nan
    g[192:224] = -np.float32(0.0)
    w[224:256] = np.linspace(-2, 2, 32)                         # delta = -w
    g[256:288] = np.linspace(-1, 1, 32)
    g[260] = -np.inf
    g[288:320] = [16.0, 12.0, 6.0, 3.0, 1.5, 0.75, 0.375, 0.125] * 4   # every tie of the E3M0 grid
    g[320:352] = [-24.0, 448.0 / 16, 480.0 / 16, 20.0, 0.0, -0.0, 2.0 ** -9, 2.0 ** -10] * 4
    g[352:384] = np.float32(1.0)
    M = 2
    w_bits = [workloads.bf16_bits(torch.from_numpy(w)), workloads.bf16_bits(torch.from_numpy(-w))]
    mom = np.zeros(n, np.float32)
    dev = _from_host(g, mom, w_bits, [b.copy() for b in w_bits])
    with np.errstate(all="ignore"):
        check_fused_against_oracle(*dev, fmt, LR, MU, 0.5, emit=True, what=f"degenerate fmt={fmt}")
    # unfused send side on the same input
    dev = _from_host(g, mom, w_bits, w_bits)
    codes, scales = sdl.alloc_exchange(fmt, n, M)
    sdl.sdl_quantize_outer_grad(dev[0], dev[2], n, fmt, codes, scales)
    torch.cuda.synchronize()
    rc, rs = oracle.quantize_outer_grad(g, w_bits, fmt)
    for m in range(M):
        if fmt in (sdl.FMT_FP32, sdl.FMT_BF16):
            # NaN payloads are not part of the contract: compare everything but NaN bit patterns
            width = 4 if fmt == sdl.FMT_FP32 else 2
            got = codes[m][:rc[m].size].cpu().numpy().reshape(-1, width)
            want = rc[m].reshape(-1, width)
            keep = ~np.isnan(g - (w if m == 0 else -w))
            assert np.array_equal(got[keep], want[keep])
        else:
            assert_bytes_equal(codes[m][:rc[m].size].cpu().numpy(), rc[m], f"codes[{m}]")
            if fmt == sdl.FMT_E3M0_SPAN:
                # the span holds Inf and NaN: the scale word is the largest bit pattern seen, which
                # is a NaN's; only its exponent field (255) is part of the contract
                assert int(scales[m][:4].cpu().numpy().view(np.uint32)[0] >> 23) == 255 == int(rs[m].view(np.uint32)[0] >> 23)
            else:
                assert_bytes_equal(scales[m][:rs[m].size].cpu().numpy(), rs[m], f"scales[{m}]")


def test_paper_special_cases_on_gpu():
    """The special cases the method reduces to (Sections 2.1-2.3), on the GPU path itself."""
    n = 4096 + 40
    # alpha = 1: no communication, replicas untouched (bit-exact)
    g, mom, w_send, w_now = _span(n, 2, tau=1)
    keep = [w.clone() for w in w_now]
    sdl.sdl_fragment_outer_step(g, mom, w_send, w_now, n, sdl.FMT_E3M0, LR, MU, 1.0)
    torch.cuda.synchronize()
    for a, b in zip(w_now, keep):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    # alpha = 0, tau = 0, no quantisation, P = 1: DiLoCo -- every replica becomes bf16(g')
    g, mom, w_send, _ = _span(n, 2, tau=0)
    sdl.sdl_fragment_outer_step(g, mom, w_send, w_send, n, sdl.FMT_FP32, LR, MU, 0.0)
    torch.cuda.synchronize()
    for w in w_send:
        assert torch.equal(w.view(torch.int16), g.to(torch.bfloat16).view(torch.int16))
    # identical workers average to themselves (M = 8 against M = 1)
    g, mom, w_send, _ = _span(n, 1, tau=0)
    g1, m1 = g.clone(), mom.clone()
    w8 = [w_send[0].clone() for _ in range(8)]
    w1 = [w_send[0].clone()]
    sdl.sdl_fragment_outer_step(g, mom, w8, w8, n, sdl.FMT_E3M0, LR, MU, 0.5)
    sdl.sdl_fragment_outer_step(g1, m1, w1, w1, n, sdl.FMT_E3M0, LR, MU, 0.5)
    torch.cuda.synchronize()
    assert torch.equal(g, g1) and torch.equal(mom, m1)
    # M = 1, lr = 1, mu = 0, alpha = 1 reproduces the local parameters
    g, mom, w_send, w_now = _span(n, 1, tau=1)
    keep = w_now[0].clone()
    sdl.sdl_fragment_outer_step(g, mom, w_send, w_now, n, sdl.FMT_FP32, 1.0, 0.0, 1.0)
    torch.cuda.synchronize()
    assert torch.equal(w_now[0].view(torch.int16), keep.view(torch.int16))
    assert (g == w_send[0].float()).float().mean() > 0.95


def test_stream_argument_is_honoured():
    n, M = 1 << 20, 2
    g, mom, w_send, w_now = _span(n, M)
    ref = HostCopy(g, mom, w_send, w_now)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    sdl.sdl_fragment_outer_step(g, mom, w_send, w_now, n, sdl.FMT_E3M0, LR, MU, 0.5, stream=s)
    s.synchronize()
    oracle.fragment_outer_step_chunked(ref.g, ref.mom, ref.w_send, ref.w_now, sdl.FMT_E3M0, LR, MU, 0.5, 8)
    assert_f32_close(host_f32(g), ref.g, "g on side stream")
