"""Pins of the oracle's reduce / Nesterov / merge / whole step against library routines,
closed forms and the special cases the paper states."""
import numpy as np
import pytest
import torch

import oracle
from oracle import FMT_BF16, FMT_E3M0, FMT_E4M3, FMT_FP32


def _bits(t):
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()


def _f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _make(n, M, seed=0, tau=1):
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal(n) * 0.02).astype(np.float32)
    w_send = [_bits(torch.from_numpy(g - (rng.standard_normal(n) * 1e-3).astype(np.float32)))
              for _ in range(M)]
    w_now = [_bits(torch.from_numpy(_f32(w) + (rng.standard_normal(n) * 1e-4 * tau).astype(np.float32)))
             for w in w_send]
    return g, np.zeros(n, np.float32), w_send, w_now


def test_nesterov_against_torch_sgd_three_rounds():
    """Section 2.1: OuterOpt is SGD with Nesterov momentum; the averaged outer gradient
    plays the role of the gradient."""
    n, M, lr, mu = 4096, 2, 0.7, 0.9
    g, mom, _, _ = _make(n, M, seed=1)
    p = torch.nn.Parameter(torch.from_numpy(g.copy()))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, nesterov=True)
    rng = np.random.default_rng(2)
    for rnd in range(3):
        deltas = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(M)]
        codes = [d.view(np.uint8) for d in deltas]
        oracle.dequant_reduce_nesterov(g, mom, codes, codes, FMT_FP32, lr, mu)
        p.grad = torch.from_numpy(((deltas[0] + deltas[1]) / np.float32(M)).astype(np.float32))
        opt.step()
        np.testing.assert_allclose(g, p.detach().numpy(), rtol=1e-6, atol=1e-8)
        buf = opt.state[p]["momentum_buffer"].numpy()
        np.testing.assert_allclose(mom, buf, rtol=1e-6, atol=1e-9)
    assert np.abs(mom).max() > 0


def test_constant_gradient_momentum_closed_form():
    n, lr, mu = 64, 0.4, 0.9
    d = np.full(n, 0.5, np.float32)
    g = np.zeros(n, np.float32)
    mom = np.zeros(n, np.float32)
    codes = [d.view(np.uint8)]
    for k in range(1, 8):
        oracle.dequant_reduce_nesterov(g, mom, codes, codes, FMT_FP32, lr, mu)
        np.testing.assert_allclose(mom, 0.5 * (1 - mu ** k) / (1 - mu), rtol=1e-6)


def test_fedavg_closed_form():
    """mu = 0, lr = 1, no quantisation: the outer step is plain parameter averaging."""
    n, M = 5000, 4
    g, mom, w_send, _ = _make(n, M, seed=3)
    w_now = [w.copy() for w in w_send]
    g0 = g.copy()
    oracle.fragment_outer_step(g, mom, w_send, w_now, FMT_FP32, 1.0, 0.0, 0.0)
    mean = np.mean([_f32(w).astype(np.float64) for w in w_send], axis=0)
    np.testing.assert_allclose(g, mean, rtol=0, atol=4e-9)
    assert np.abs(g - g0).max() > 1e-4
    # alpha = 0: every replica is the rounded new global model
    for w in w_now:
        assert np.array_equal(w, _bits(torch.from_numpy(g)))


@pytest.mark.parametrize("M", [1, 2, 4, 8])
@pytest.mark.parametrize("fmt", [FMT_E3M0, FMT_E4M3, FMT_BF16, FMT_FP32])
def test_identical_workers_average_to_themselves(M, fmt):
    n = 1000
    g, mom, w_send, _ = _make(n, 1, seed=4)
    ws = [w_send[0]] * M
    codes, scales = oracle.quantize_outer_grad(g, ws, fmt)
    codes1, scales1 = oracle.quantize_outer_grad(g, ws[:1], fmt)
    # lr = 1, mu = 0  =>  g' = g - mean, so the mean can be read back
    gM, g1 = g.copy(), g.copy()
    oracle.dequant_reduce_nesterov(gM, mom.copy(), codes, scales, fmt, 1.0, 0.0)
    oracle.dequant_reduce_nesterov(g1, mom.copy(), codes1, scales1, fmt, 1.0, 0.0)
    if fmt == FMT_FP32 and M > 2:
        # partial sums 3x, 5x, ... of a full 24-bit value round in fp32: equal only to tolerance
        np.testing.assert_allclose(gM, g1, rtol=1e-6, atol=1e-9)
    else:
        # <= 8 significant bits per value: every partial sum k*x is exact in fp32
        assert np.array_equal(gM, g1)


def test_reduction_is_fp32_in_replica_order():
    # three values whose fp32 sum depends on the order: (1e8 + 1) - 1e8 = 0 in fp32
    vals = [np.array([1e8], np.float32), np.array([1.0], np.float32), np.array([-1e8], np.float32)]
    g, mom = np.zeros(1, np.float32), np.zeros(1, np.float32)
    codes = [v.view(np.uint8) for v in vals]
    oracle.dequant_reduce_nesterov(g, mom, codes, codes, FMT_FP32, 1.0, 0.0)
    assert mom[0] == 0.0
    order2 = [codes[0], codes[2], codes[1]]
    g[:] = 0
    mom[:] = 0
    oracle.dequant_reduce_nesterov(g, mom, order2, order2, FMT_FP32, 1.0, 0.0)
    assert mom[0] == np.float32(1.0) / np.float32(3.0)
    # against a float64 shadow on ordinary data
    rng = np.random.default_rng(5)
    n, M = 2000, 8
    ds = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(M)]
    g, mom = np.zeros(n, np.float32), np.zeros(n, np.float32)
    cs = [d.view(np.uint8) for d in ds]
    oracle.dequant_reduce_nesterov(g, mom, cs, cs, FMT_FP32, 1.0, 0.0)
    shadow = np.mean(np.stack(ds).astype(np.float64), axis=0)
    np.testing.assert_allclose(mom, shadow, rtol=0, atol=M * 2.0 ** -24 * 4e-3)


def test_merge_alpha_semantics():
    """Section 2.3: alpha = 1 is no communication, alpha = 0 discards the local tau steps,
    alpha = 0.5 is the uniform average."""
    n, M = 3000, 3
    g, _, _, w_now = _make(n, M, seed=6)
    keep = [w.copy() for w in w_now]
    oracle.merge_overlap(g, w_now, 1.0)
    for a, b in zip(w_now, keep):
        assert np.array_equal(a, b)
    oracle.merge_overlap(g, w_now, 0.0)
    for a in w_now:
        assert np.array_equal(a, _bits(torch.from_numpy(g)))
    # fixed point: replicas equal to bf16(g) exactly representable => unchanged by alpha = 0.5
    gb = _f32(_bits(torch.from_numpy(g)))
    w = [_bits(torch.from_numpy(gb))]
    oracle.merge_overlap(gb, w, 0.5)
    assert np.array_equal(w[0], _bits(torch.from_numpy(gb)))
    # uniform average against torch
    g, _, _, w_now = _make(n, 1, seed=7)
    want = (0.5 * torch.from_numpy(_f32(w_now[0])) + 0.5 * torch.from_numpy(g)).to(torch.bfloat16)
    oracle.merge_overlap(g, w_now, 0.5)
    assert np.array_equal(w_now[0], _bits(want))
    # a generic alpha against a float64 evaluation, within one bf16 ulp
    g, _, _, w_now = _make(n, 1, seed=8)
    before = _f32(w_now[0]).astype(np.float64)
    oracle.merge_overlap(g, w_now, 0.3)
    exact = 0.3 * before + 0.7 * g.astype(np.float64)
    err = np.abs(_f32(w_now[0]).astype(np.float64) - exact)
    assert np.all(err <= np.abs(exact) * 2.0 ** -8 + 1e-12)


def test_single_worker_identity():
    """M = 1, lr = 1, mu = 0, alpha = 1 reproduces the local parameters; with no
    quantisation the global model becomes the local model."""
    n = 4096
    g, mom, w_send, w_now = _make(n, 1, seed=9)
    keep_now = w_now[0].copy()
    oracle.fragment_outer_step(g, mom, w_send, w_now, FMT_FP32, 1.0, 0.0, 1.0)
    assert np.array_equal(w_now[0], keep_now)
    local = _f32(w_send[0])
    np.testing.assert_allclose(g, local, rtol=0, atol=2e-9)
    assert np.mean(g == local) > 0.95      # exact wherever g - w is exact (Sterbenz)


def test_whole_model_no_overlap_is_diloco():
    """P = 1, tau = 0, alpha = 0, no quantisation: Algorithm 1 (every replica restarts from
    OuterOpt(theta_global, mean of outer gradients))."""
    n, M, lr, mu = 2048, 2, 0.7, 0.9
    g, mom, w_send, _ = _make(n, M, seed=10)
    mom[:] = np.random.default_rng(11).standard_normal(n).astype(np.float32) * 1e-3
    g0, mom0 = g.copy(), mom.copy()
    oracle.fragment_outer_step(g, mom, w_send, w_send, FMT_FP32, lr, mu, 0.0)
    p = torch.nn.Parameter(torch.from_numpy(g0.copy()))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, nesterov=True)
    opt.state[p]["momentum_buffer"] = torch.from_numpy(mom0.copy())
    deltas = [torch.from_numpy(g0) - torch.from_numpy(_f32(w)) for w in
              _make(n, M, seed=10)[2]]
    p.grad = (deltas[0] + deltas[1]) / 2
    opt.step()
    np.testing.assert_allclose(g, p.detach().numpy(), rtol=1e-6, atol=1e-8)
    for w in w_send:
        assert np.array_equal(w, _bits(torch.from_numpy(g)))


@pytest.mark.parametrize("fmt", [FMT_E3M0, FMT_E4M3, FMT_BF16, FMT_FP32])
@pytest.mark.parametrize("tau", [0, 1])
def test_fused_equals_three_calls(fmt, tau):
    n, M = 1000 + 13, 3
    g, mom, w_send, w_now = _make(n, M, seed=12, tau=tau)
    if tau == 0:
        w_now = w_send
    g2, mom2 = g.copy(), mom.copy()
    ws2 = [w.copy() for w in w_send]
    wn2 = ws2 if tau == 0 else [w.copy() for w in w_now]
    codes, scales = oracle.fragment_outer_step(g, mom, w_send, w_now, fmt, 0.7, 0.9, 0.5,
                                               want_codes=True)
    c2, s2 = oracle.quantize_outer_grad(g2, ws2, fmt)
    oracle.dequant_reduce_nesterov(g2, mom2, c2, s2, fmt, 0.7, 0.9)
    oracle.merge_overlap(g2, wn2, 0.5)
    assert np.array_equal(g, g2) and np.array_equal(mom, mom2)
    for a, b in zip(w_now, wn2):
        assert np.array_equal(a, b)
    for a, b in zip(codes + scales, c2 + s2):
        assert np.array_equal(a, b)


def test_brute_force_tiny_e3m0_step():
    """n <= 64, M <= 3: the whole step re-derived with python floats (binary64 holds every
    intermediate of the codec exactly) and explicit fp32 roundings."""
    f32 = np.float32
    n, M, lr, mu, alpha = 45, 3, f32(0.7), f32(0.9), f32(0.5)
    g, mom, w_send, w_now = _make(n, M, seed=13)
    mom[:] = (np.random.default_rng(14).standard_normal(n) * 1e-3).astype(np.float32)
    g0, mom0 = g.copy(), mom.copy()
    ws0, wn0 = [w.copy() for w in w_send], [w.copy() for w in w_now]
    oracle.fragment_outer_step(g, mom, w_send, w_now, FMT_E3M0, float(lr), float(mu), float(alpha))
    mags = [0.0] + [2.0 ** (E - 3) for E in range(1, 8)]
    dec = np.zeros((M, n), np.float32)
    for m in range(M):
        delta = g0 - _f32(ws0[m])
        for b0 in range(0, n, 32):
            blk = delta[b0:b0 + 32]
            a = float(np.abs(blk).max())
            scale = 2.0 ** (int(np.floor(np.log2(a))) - 4)
            for i, x in enumerate(blk):
                y = abs(float(x)) / scale
                E = min(range(8), key=lambda e: (abs(y - mags[e]), e & 1))
                dec[m, b0 + i] = f32(np.copysign(mags[E] * scale, x))
    for i in range(n):
        acc = f32(0)
        for m in range(M):
            acc = f32(acc + dec[m, i])
        dbar = f32(acc / f32(M))
        mnew = f32(f32(mu * mom0[i]) + dbar)
        gnew = f32(g0[i] - f32(lr * f32(dbar + f32(mu * mnew))))
        assert mnew == mom[i] and gnew == g[i]
        for m in range(M):
            mix = f32(f32(alpha * _f32(wn0[m][i:i + 1])[0]) + f32(f32(1 - alpha) * gnew))
            assert _bits(torch.tensor([mix]))[0] == w_now[m][i]


def test_chunked_threads_same_result():
    n, M = 32 * 50 + 7, 2
    g, mom, w_send, w_now = _make(n, M, seed=15)
    g2, mom2 = g.copy(), mom.copy()
    ws2, wn2 = [w.copy() for w in w_send], [w.copy() for w in w_now]
    oracle.fragment_outer_step(g, mom, w_send, w_now, FMT_E3M0, 0.7, 0.9, 0.5)
    oracle.fragment_outer_step_chunked(g2, mom2, ws2, wn2, FMT_E3M0, 0.7, 0.9, 0.5, threads=4)
    assert np.array_equal(g, g2) and np.array_equal(mom, mom2)
    for a, b in zip(w_now, wn2):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("kind,log2n,span_zero_min,span_bulk_min", [("student_t3", 22, 0.5, 0.45),
                                                                     ("outliers", 18, 0.3, 0.27)])
def test_scale_granularity_under_heavy_tails(kind, log2n, span_zero_min, span_bulk_min):
    """Why the default scale covers 32 elements (Section 2.4 fixes only the 4-bit element): with one
    scale per tensor, the few large entries of a heavy-tailed outer gradient set the scale and a
    large share of the ordinary entries falls below half the smallest magnitude and is sent as
    zero; with block scales the error of the ordinary entries stays at the format's own level
    (mean relative error of nearest-power-of-two rounding, about 0.2)."""
    import workloads
    from oracle import FMT_E3M0_B128, FMT_E3M0_SPAN, cosine
    n, M = 1 << log2n, 4                               # the largest entry of t(3) noise grows with the tensor
    g, _, w, _ = workloads.make_span(n, M, tau=0, delta=kind, unit=5)
    hg, hw = g.numpy(), [workloads.bf16_bits(x) for x in w]
    d = cosine.outer_grads(hg, hw)
    mean = d.astype(np.float64).mean(0)
    bulk = np.abs(d).max(0) < 4e-3                      # entries where no replica has an outlier
    assert bulk.mean() > 0.85
    out = {}
    for fmt in (FMT_E3M0, FMT_E3M0_B128, FMT_E3M0_SPAN):
        codes, scales = oracle.quantize_outer_grad(hg, hw, fmt)
        zero = float(np.mean((oracle.unpack_e3m0(codes[0], n) & 7) == 0))
        got, unused = np.zeros(n, np.float32), np.zeros(n, np.float32)
        oracle.dequant_reduce_nesterov(unused, got, codes, scales, fmt, 1.0, 0.0)    # mom' = mean of the decoded
        err = np.linalg.norm((got - mean)[bulk]) / np.linalg.norm(mean[bulk])
        out[fmt] = (zero, err)
    assert out[FMT_E3M0][0] < 0.05 and out[FMT_E3M0][1] < 0.26
    assert out[FMT_E3M0_B128][0] < 0.08 and out[FMT_E3M0_B128][1] < 0.26
    assert out[FMT_E3M0_SPAN][0] > span_zero_min and out[FMT_E3M0_SPAN][1] > span_bulk_min
