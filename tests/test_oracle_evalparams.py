"""Pins of the evaluation-parameter oracle (Appendix, "Which parameters to evaluate")."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import workloads
from oracle import evalparams as ep


def _bits(x):
    return workloads.bf16_bits(torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16))


def _f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def test_bf16_rounding_against_torch_and_by_hand():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * s for s in (1e-30, 1e-3, 1.0, 1e30)])
    special = np.array([0.0, -0.0, np.inf, -np.inf, 1.0, 1.00390625, 1.01171875, 1.005859375, 3.3895314e38],
                       np.float32)          # 1 + 2^-8 (tie -> even, down), 1 + 3*2^-8 (tie -> up), just above a tie, near max
    x = np.concatenate([x, special])
    want = workloads.bf16_bits(torch.from_numpy(x).to(torch.bfloat16))
    assert np.array_equal(ep.bf16_round(x), want)
    assert ep.bf16_round(np.array([1.00390625], np.float32))[0] == 0x3f80          # tie to even: down
    assert ep.bf16_round(np.array([1.01171875], np.float32))[0] == 0x3f82          # tie to even: up
    assert ep.bf16_round(np.array([3.3961775e38], np.float32))[0] == 0x7f80        # rounds up to infinity
    # NaN stays NaN, also one whose payload sits only in the bits that are rounded away
    for pattern in (0x7fc00000, 0x7f800001, 0xff80ffff):
        nan = ep.bf16_round(np.array([pattern], np.uint32).view(np.float32))[0]
        assert (nan & 0x7f80) == 0x7f80 and (nan & 0x7f) != 0 and (nan >> 15) == (pattern >> 31)


def test_three_candidates_on_a_hand_case():
    g = np.array([1.0, 2.0, -3.0, 0.1], np.float32)
    w = [_bits([1.0, 4.0, -2.0, 0.0]), _bits([3.0, 0.0, -4.0, 0.0]), _bits([2.0, -1.0, -3.0, 3.0])]
    assert np.array_equal(ep.evaluation_params(ep.FIRST_REPLICA, g, w), w[0])
    assert np.array_equal(_f32(ep.evaluation_params(ep.REPLICA_MEAN, g, w)), np.array([2.0, 1.0, -3.0, 1.0], np.float32))
    assert np.array_equal(ep.evaluation_params(ep.OUTER, g, w), _bits(g))
    assert _f32(ep.evaluation_params(ep.OUTER, g, w))[3] == np.float32(0.10009765625)   # bf16(0.1)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 7, 8, 16])
def test_mean_properties(M):
    rng = np.random.default_rng(M)
    n = 4096
    w = [_bits(rng.standard_normal(n) * 0.02) for _ in range(M)]
    g = np.zeros(n, np.float32)
    out = ep.evaluation_params(ep.REPLICA_MEAN, g, w)
    # within half a bf16 ulp (plus the fp32 sum's rounding) of the exact rational mean
    exact = [sum(Fraction(float(_f32(x)[i])) for x in w) / M for i in range(64)]
    for i in range(64):
        got = Fraction(float(_f32(out)[i]))
        ulp = Fraction(2) ** (int(np.floor(np.log2(max(abs(float(exact[i])), 1e-30)))) - 7)
        assert abs(got - exact[i]) <= ulp * Fraction(501, 1000) + Fraction(1, 10 ** 12)
    # identical replicas average to themselves when the sum is exact (M a power of two)
    if M & (M - 1) == 0:
        same = ep.evaluation_params(ep.REPLICA_MEAN, g, [w[0]] * M)
        assert np.array_equal(same, w[0])
    # one replica: the mean is that replica
    assert np.array_equal(ep.evaluation_params(ep.REPLICA_MEAN, g, [w[0]]), w[0])
    # the order of summation is the replica order (fp32 addition is not associative)
    if M >= 3:
        # 1 + 2^-24 is a tie that rounds back to 1, so the small terms vanish one by one when
        # they come after the 1, and survive when they meet its cancellation first
        seq = [_bits(np.full(8, 1.0))] + [_bits(np.full(8, 2.0 ** -24))] * (M - 2) + [_bits(np.full(8, -1.0))]
        fwd = _f32(ep.evaluation_params(ep.REPLICA_MEAN, g[:8], seq))
        rev = _f32(ep.evaluation_params(ep.REPLICA_MEAN, g[:8], seq[::-1]))
        assert np.all(fwd == 0) and np.all(rev > 0)


def test_accumulates_in_fp32_not_in_bf16():
    # 1 + 2^-8 is a tie between bf16 neighbours that rounds back to 1: a bf16 accumulator would
    # lose both small terms and give 0.25
    w = [_bits([1.0]), _bits([2.0 ** -8]), _bits([2.0 ** -8]), _bits([0.0])]
    out = _f32(ep.evaluation_params(ep.REPLICA_MEAN, np.zeros(1, np.float32), w))
    assert out[0] == np.float32(0.251953125)      # (1 + 2^-7) / 4, exact in bf16
