"""Pins of the cosine-similarity oracle (Appendix, cosine similarity of the outer gradients)
against exact rational arithmetic, closed forms, an independent library routine and the
invariants of a Gram matrix."""
from fractions import Fraction

import numpy as np
import pytest
import torch
from scipy.spatial.distance import cosine as scipy_cosine_distance

import workloads
from oracle import cosine


def _bf16_bits(x):
    return workloads.bf16_bits(torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16))


def _case(n, M, seed=0, rho=0.0):
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal(n) * 0.02).astype(np.float32)
    s = rng.standard_normal(n)
    w = [_bf16_bits(g - 1e-3 * (np.sqrt(rho) * s + np.sqrt(1 - rho) * rng.standard_normal(n)).astype(np.float32))
         for _ in range(M)]
    return g, w


def test_exact_rational_brute_force():
    """Tiny case in exact arithmetic: the fp32 subtraction is the only rounding of the Gram matrix."""
    g, w = _case(37, 3, seed=5)
    G, cos, _ = cosine.outer_grad_cosine(g, w)
    d = []
    for m in range(3):
        wf = (w[m].astype(np.uint32) << 16).view(np.float32)
        d.append([Fraction(float(np.float32(g[i]) - np.float32(wf[i]))) for i in range(37)])
    for a in range(3):
        for b in range(3):
            exact = sum(x * y for x, y in zip(d[a], d[b]))
            assert abs(Fraction(float(G[a, b])) - exact) <= abs(exact) * Fraction(1, 10 ** 14) + Fraction(1, 10 ** 30)
    exact01 = float(sum(x * y for x, y in zip(d[0], d[1]))) / np.sqrt(float(sum(x * x for x in d[0]))
                                                                  * float(sum(y * y for y in d[1])))
    assert abs(cos[0, 1] - exact01) < 1e-14


def test_closed_forms():
    n = 4096
    g = np.zeros(n, np.float32)
    base = np.where(np.arange(n) % 2 == 0, 0.5, -0.25).astype(np.float32)       # exact in bf16
    half = np.where(np.arange(n) < n // 2, 1.0, 0.0).astype(np.float32)
    w = [_bf16_bits(-base), _bf16_bits(-2 * base), _bf16_bits(base),           # delta = base, 2 base, -base
         _bf16_bits(-half), _bf16_bits(-(1 - half)),                            # disjoint supports
         _bf16_bits(-np.ones(n, np.float32))]                                   # 45 degrees to either half
    G, cos, mean = cosine.outer_grad_cosine(g, w)
    assert abs(cos[0, 1] - 1.0) < 1e-15 and abs(cos[0, 2] + 1.0) < 1e-15 and abs(cos[1, 2] + 1.0) < 1e-15
    assert cos[3, 4] == 0.0
    assert abs(cos[3, 5] - np.sqrt(0.5)) < 1e-15 and abs(cos[4, 5] - np.sqrt(0.5)) < 1e-15
    assert G[0, 0] == n / 2 * (0.25 + 0.0625) and G[3, 3] == n / 2 and G[5, 5] == n
    assert G[0, 1] == 2 * G[0, 0] and G[0, 2] == -G[0, 0]
    pairs = [cos[a, b] for a in range(6) for b in range(a + 1, 6)]
    assert abs(mean - sum(pairs) / 15) < 1e-15


def test_outer_gradient_sign_and_operands():
    """Delta = g - w (Algorithm 2), not w - g and not w alone: a case where each mistake shows."""
    g = np.array([1.0, 2.0, 3.0, 4.0], np.float32)
    w = [_bf16_bits([0.0, 2.0, 3.0, 4.0]), _bf16_bits([1.0, 2.0, 3.0, 2.0]), _bf16_bits([0.5, 2.0, 3.0, 3.0])]
    d = cosine.outer_grads(g, w)
    assert np.array_equal(d, np.array([[1, 0, 0, 0], [0, 0, 0, 2], [0.5, 0, 0, 1]], np.float32))
    G, cos, _ = cosine.outer_grad_cosine(g, w)
    assert np.array_equal(G, np.array([[1, 0, 0.5], [0, 4, 2], [0.5, 2, 1.25]]))
    assert cos[0, 1] == 0.0
    assert abs(cos[0, 2] - 0.5 / np.sqrt(1.25)) < 1e-15
    assert abs(cos[1, 2] - 2 / (2 * np.sqrt(1.25))) < 1e-15


@pytest.mark.parametrize("M", [2, 4, 7])
def test_against_scipy_and_numpy_routines(M):
    g, w = _case(10007, M, seed=M, rho=0.3)
    G, cos, _ = cosine.outer_grad_cosine(g, w)
    d = cosine.outer_grads(g, w).astype(np.float64)
    for a in range(M):
        for b in range(M):
            if a != b:
                assert abs(cos[a, b] - (1.0 - scipy_cosine_distance(d[a], d[b]))) < 1e-12
            assert abs(G[a, b] - np.vdot(d[a], d[b])) <= 1e-12 * np.sqrt(G[a, a] * G[b, b])
    # uncentred correlation = Pearson correlation once the mean is taken out
    dc = d - d.mean(1, keepdims=True)
    Gc = dc @ dc.T
    assert np.allclose(cosine.cosine_from_gram(Gc)[0], np.corrcoef(d), atol=1e-12)


@pytest.mark.parametrize("M", [1, 2, 5, 16])
def test_gram_invariants(M):
    g, w = _case(5000, M, seed=10 + M, rho=0.2)
    G, cos, mean = cosine.outer_grad_cosine(g, w)
    assert G.shape == (M, M) and np.array_equal(G, G.T) and np.array_equal(cos, cos.T)
    assert np.all(np.diag(cos) == 1.0) or np.allclose(np.diag(cos), 1.0, atol=1e-15)
    assert np.all(np.abs(cos) <= 1.0 + 1e-15)
    assert np.linalg.eigvalsh(G).min() >= -1e-12 * np.trace(G)                  # positive semi-definite
    if M == 1:
        assert mean == 0.0
    # a permutation of the replicas permutes rows and columns
    perm = list(reversed(range(M)))
    G2, cos2, mean2 = cosine.outer_grad_cosine(g, [w[i] for i in perm])
    assert np.allclose(G2, G[np.ix_(perm, perm)], rtol=1e-14) and abs(mean2 - mean) < 1e-14
    # the Gram matrix of a concatenation is the sum of the parts' Gram matrices
    cut = 1234
    Ga = cosine.gram(g[:cut], [x[:cut] for x in w])
    Gb = cosine.gram(g[cut:], [x[cut:] for x in w])
    Gu, cosu, meanu = cosine.combine([Ga, Gb])
    assert np.allclose(Gu, G, rtol=1e-13, atol=1e-30) and np.allclose(cosu, cos, atol=1e-13)
    assert abs(meanu - mean) < 1e-13


def test_scale_invariance_is_exact_for_powers_of_two():
    n = 2048
    rng = np.random.default_rng(3)
    g = np.zeros(n, np.float32)
    d0 = workloads.bits_bf16(_bf16_bits(rng.standard_normal(n))).to(torch.float32).numpy()
    d1 = workloads.bits_bf16(_bf16_bits(rng.standard_normal(n))).to(torch.float32).numpy()
    _, cos_a, _ = cosine.outer_grad_cosine(g, [_bf16_bits(-d0), _bf16_bits(-d1)])
    _, cos_b, _ = cosine.outer_grad_cosine(g, [_bf16_bits(-8 * d0), _bf16_bits(-0.25 * d1)])
    assert cos_a[0, 1] == cos_b[0, 1]


def test_zero_outer_gradient_reads_as_zero_similarity():
    g = np.linspace(-1, 1, 64).astype(np.float32)
    gb = _bf16_bits(g)
    g = workloads.bits_bf16(gb).to(torch.float32).numpy()                        # replica 0 equals g
    w1 = _bf16_bits(g + 0.5)
    G, cos, mean = cosine.outer_grad_cosine(g, [gb, w1])
    assert G[0, 0] == 0 and cos[0, 0] == 0 and cos[0, 1] == 0 and cos[1, 1] == 1 and mean == 0


@pytest.mark.parametrize("rho", [0.0, 0.1, 0.5])
def test_statistics_of_the_synthetic_workload(rho):
    """Replicas that share a fraction rho of their outer gradient's variance have cosine rho
    (the paper's curves move between about +0.1 and -0.1)."""
    n, M = 1 << 18, 4
    kind = "normal" if rho == 0 else f"shared{int(rho * 100)}"
    g, _, w_send, _ = workloads.make_span(n, M, tau=0, delta=kind, unit=3)
    _, cos, mean = cosine.outer_grad_cosine(g.numpy(), [workloads.bf16_bits(x) for x in w_send])
    off = cos[~np.eye(M, dtype=bool)]
    assert np.all(np.abs(off - rho) < 6 / np.sqrt(n) + 0.002)                   # bf16 rounding adds a little noise
    assert abs(mean - rho) < 6 / np.sqrt(n) + 0.002
