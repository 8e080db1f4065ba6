"""Pins of the oracle's exchange-format codec against things other than itself.

E3M0 (Section 2.4: 1 sign, 3 exponent, 0 mantissa bits) has no worked example in the
paper, so it is pinned by: the hand-derived midpoint table (tests/golden), an exact
rational nearest-value search, the closed form for powers of two, exact round trips,
sign symmetry, scale invariance, idempotence and the 1/3 relative-error bound.
E4M3 and BF16 are pinned against PyTorch's CPU casts.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import FMT_BF16, FMT_E3M0, FMT_E4M3, FMT_FP32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(1234)


def _e3m0_of_y(y32: np.ndarray, pad=16.0):
    """E codes of scaled magnitudes y: put them in a block whose maximum is `pad`
    (scale byte 127, scale 1) so that delta == y."""
    out = []
    for lo in range(0, len(y32), 31):
        blk = np.concatenate([[np.float32(pad)], y32[lo:lo + 31]]).astype(np.float32)
        codes, sb = oracle.encode_block(blk, FMT_E3M0)
        assert sb == 127
        out.append(codes[1:])
    return np.concatenate(out)


def test_scale_of_one_when_max_in_16_32():
    for a in (16.0, 17.5, 31.999998):
        codes, sb = oracle.encode_block(np.array([a, 1.0], np.float32), FMT_E3M0)
        assert sb == 127 and codes[0] == 7 and codes[1] == 3


def test_threshold_table_golden():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "e3m0_thresholds.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 7
    for mid, below, above, tie in rows:
        mid = np.float32(float(mid))
        lo = np.nextafter(mid, np.float32(0), dtype=np.float32)
        hi = np.nextafter(mid, np.float32(100), dtype=np.float32)
        got = _e3m0_of_y(np.array([lo, mid, hi], np.float32))
        assert list(got) == [int(below), int(tie), int(above)], (mid, got)
        # negative values: same exponent code, sign bit set
        blk = np.array([16.0, -lo, -mid, -hi], np.float32)
        codes, _ = oracle.encode_block(blk, FMT_E3M0)
        assert list(codes[1:]) == [8 | int(below), 8 | int(tie), 8 | int(above)]


def _exact_e3m0(y: Fraction) -> int:
    mags = [Fraction(0)] + [Fraction(2) ** (E - 3) for E in range(1, 8)]
    best = min(range(8), key=lambda E: (abs(y - mags[E]), E & 1))
    return best


def test_exact_rational_search():
    # dense sweep of fp32 values around every midpoint and random ones elsewhere
    ys = []
    for mid in (0.125, 0.375, 0.75, 1.5, 3.0, 6.0, 12.0):
        v = np.float32(mid)
        down = up = v
        for _ in range(40):
            down = np.nextafter(down, np.float32(0), dtype=np.float32)
            up = np.nextafter(up, np.float32(100), dtype=np.float32)
            ys += [down, up]
        ys.append(v)
    ys += list(np.exp(RNG.uniform(np.log(1e-4), np.log(15.99), 2000)).astype(np.float32))
    ys += [np.float32(0.0), np.float32(1e-30), np.float32(15.999999)]
    ys = np.array(ys, np.float32)
    got = _e3m0_of_y(ys)
    want = [_exact_e3m0(Fraction(float(y))) for y in ys]
    assert list(got) == want


def test_closed_form_nearest_power_of_two():
    # away from ties and above the zero threshold: E = 4 + floor(log2(y / 1.5)), clipped to [1, 7]
    y = np.exp(RNG.uniform(np.log(0.126), np.log(15.9), 20000)).astype(np.float32)
    frac = np.abs(np.log2(y.astype(np.float64) / 1.5) % 1.0)
    keep = (frac > 1e-6) & (frac < 1 - 1e-6)
    y = y[keep]
    want = np.clip(4 + np.floor(np.log2(y.astype(np.float64) / 1.5)), 1, 7).astype(int)
    assert np.array_equal(_e3m0_of_y(y), want)
    small = np.float32(RNG.uniform(0, 0.125, 1000))
    assert np.all(_e3m0_of_y(small) == 0)


def test_block_maximum_sets_scale_byte():
    for a in (1e-3, 3.7e-5, 0.02, 1.0, 123.4, 2.0 ** -100, 2.0 ** 100):
        a32 = np.float32(a)
        m, e = math.frexp(float(a32))           # a = m * 2^e, m in [0.5, 1)
        floor_log2 = e - 1
        for fmt, emax in ((FMT_E3M0, 4), (FMT_E4M3, 8)):
            blk = np.zeros(32, np.float32)
            blk[7] = -a32
            codes, sb = oracle.encode_block(blk, fmt)
            assert sb == floor_log2 - emax + 127
            dec = oracle.decode_code(int(codes[7]), sb, fmt)
            if fmt == FMT_E3M0:
                assert dec == -(2.0 ** floor_log2)      # block max saturates to 2^floor(log2 a)
            assert all(c == 0 for i, c in enumerate(codes) if i != 7)


def test_round_trip_powers_of_two():
    # 0 and +-2^k within 7 binades of the block maximum survive encode/decode unchanged
    for top in (-10, 0, 5):
        vals = [0.0] + [s * 2.0 ** (top - j) for j in range(7) for s in (1, -1)]
        blk = np.array(vals, np.float32)
        codes, sb = oracle.encode_block(blk, FMT_E3M0)
        dec = np.array([oracle.decode_code(int(c), sb, FMT_E3M0) for c in codes], np.float32)
        assert np.array_equal(dec, blk)
        # an eighth binade falls below the smallest magnitude and flushes to zero
        blk2 = np.array([2.0 ** top, 2.0 ** (top - 7)], np.float32)
        codes2, _ = oracle.encode_block(blk2, FMT_E3M0)
        assert codes2[1] == 0


@pytest.mark.parametrize("fmt", [FMT_E3M0, FMT_E4M3])
def test_idempotent_symmetric_scale_invariant(fmt):
    for trial in range(50):
        blk = (RNG.standard_normal(32) * 10.0 ** RNG.uniform(-6, 2)).astype(np.float32)
        codes, sb = oracle.encode_block(blk, fmt)
        dec = np.array([oracle.decode_code(int(c), sb, fmt) for c in codes], np.float32)
        # idempotence: the decoded block encodes to the same codes and scale
        codes2, sb2 = oracle.encode_block(dec, fmt)
        assert sb2 == sb and np.array_equal(codes2, codes)
        # sign symmetry
        sign = 8 if fmt == FMT_E3M0 else 0x80
        codes3, sb3 = oracle.encode_block(-blk, fmt)
        assert sb3 == sb and np.array_equal(codes3, codes ^ sign)
        # scale invariance: multiplying by 2^k only moves the scale byte
        k = int(RNG.integers(-20, 20))
        codes4, sb4 = oracle.encode_block(np.ldexp(blk, k).astype(np.float32), fmt)
        assert sb4 == sb + k and np.array_equal(codes4, codes)


def test_e3m0_relative_error_bound():
    worst = 0.0
    for trial in range(200):
        blk = (RNG.standard_normal(32) * 1e-3).astype(np.float32)
        codes, sb = oracle.encode_block(blk, FMT_E3M0)
        scale = 2.0 ** (sb - 127)
        for x, c in zip(blk, codes):
            y = abs(float(x)) / scale
            dec = oracle.decode_code(int(c), sb, FMT_E3M0)
            if 0.25 <= y < 24:
                worst = max(worst, abs(dec - float(x)) / abs(float(x)))
            if y <= 0.125:
                assert dec == 0.0
    assert worst <= 1.0 / 3.0 + 1e-12
    # the worst case is reached at y = 1.5 * 2^k
    codes, sb = oracle.encode_block(np.array([16.0, 1.5], np.float32), FMT_E3M0)
    assert oracle.decode_code(int(codes[1]), sb, FMT_E3M0) == 2.0


def test_e4m3_against_torch_cast():
    for trial in range(100):
        blk = (RNG.standard_normal(32) * 10.0 ** RNG.uniform(-5, 1)).astype(np.float32)
        codes, sb = oracle.encode_block(blk, FMT_E4M3)
        y = np.ldexp(blk, 127 - sb).astype(np.float32)          # exact power-of-two scaling
        assert 256 <= np.abs(y).max() < 512
        inside = np.abs(y) <= 448
        want = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(codes[inside], want[inside])
        # above the largest finite value the encoder saturates instead of producing NaN
        assert np.all((codes[~inside] & 0x7f) == 0x7e)
        assert np.array_equal(codes[~inside] >> 7, (y[~inside] < 0).astype(np.uint8))
    # decode against torch's widening cast
    allc = np.arange(256, dtype=np.uint8)
    ref = torch.from_numpy(allc).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for c in allc:
        if (c & 0x7f) == 0x7f:
            continue
        assert oracle.decode_code(int(c), 127, FMT_E4M3) == ref[c]
        assert oracle.decode_code(int(c), 120, FMT_E4M3) == ref[c] * 2.0 ** -7


def test_e4m3_subnormal_grid_against_torch():
    # small elements next to a large block maximum land on the m * 2^-9 grid
    blk = np.zeros(32, np.float32)
    blk[0] = 300.0
    blk[1:] = RNG.uniform(-0.02, 0.02, 31).astype(np.float32)
    codes, sb = oracle.encode_block(blk, FMT_E4M3)
    assert sb == 127
    want = torch.from_numpy(blk).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(codes, want)


def _make(n, M, seed=0, scale=1e-3):
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal(n) * 0.02).astype(np.float32)
    w = []
    for m in range(M):
        t = torch.from_numpy(g - (rng.standard_normal(n) * scale).astype(np.float32))
        w.append(t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy())
    return g, w


def _bf16_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def test_bf16_and_fp32_formats_against_torch():
    g, w = _make(1000, 2, seed=3)
    codes, _ = oracle.quantize_outer_grad(g, w, FMT_FP32)
    for m in range(2):
        delta = g - _bf16_f32(w[m])
        assert np.array_equal(codes[m].view(np.float32), delta)
    codes, _ = oracle.quantize_outer_grad(g, w, FMT_BF16)
    for m in range(2):
        delta = torch.from_numpy(g - _bf16_f32(w[m]))
        want = delta.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(codes[m].view(np.uint16), want)


def test_packing_nibble_order_and_ragged_tail():
    # g = 0, w = -v  =>  delta = v exactly; choose v so that the codes are known
    v = np.array([16.0, -8.0, 4.0, -2.0, 1.0, -0.5, 0.25, 0.0, -0.0625], np.float32)   # n = 9 (odd)
    # (the last one underflows to zero and keeps its sign bit: code 0x8)
    want_codes = [7, 8 | 6, 5, 8 | 4, 3, 8 | 2, 1, 0, 8]
    g = np.zeros(9, np.float32)
    w = [torch.from_numpy(-v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()]
    codes, scales = oracle.quantize_outer_grad(g, w, FMT_E3M0)
    assert codes[0].size == 5 and scales[0].size == 1 and scales[0][0] == 127
    packed = [want_codes[0] | want_codes[1] << 4, want_codes[2] | want_codes[3] << 4,
              want_codes[4] | want_codes[5] << 4, want_codes[6] | want_codes[7] << 4,
              want_codes[8]]                        # last high nibble is padding = 0
    assert list(codes[0]) == packed
    assert list(oracle.unpack_e3m0(codes[0], 9)) == want_codes
    assert oracle.exchange_bytes(FMT_E3M0, 33) == (17, 2)
    assert oracle.exchange_bytes(FMT_E4M3, 33) == (33, 2)
    assert oracle.exchange_bytes(FMT_BF16, 33) == (66, 0)
    assert oracle.exchange_bytes(FMT_FP32, 33) == (132, 0)
    assert oracle.exchange_bytes(FMT_E3M0, 0) == (0, 0)


def test_blocks_are_independent_and_32_wide():
    # changing one element only changes codes of its own 32-element block
    g, w = _make(200, 1, seed=5)
    c0, s0 = oracle.quantize_outer_grad(g, w, FMT_E3M0)
    g2 = g.copy()
    g2[70] += 1.0                                   # block 2 = elements 64..95
    c1, s1 = oracle.quantize_outer_grad(g2, w, FMT_E3M0)
    diff_bytes = np.nonzero(c0[0] != c1[0])[0]
    assert diff_bytes.size > 0 and diff_bytes.min() >= 32 and diff_bytes.max() < 48
    assert list(np.nonzero(s0[0] != s1[0])[0]) == [2]
    assert s0[0].size == 7                           # ceil(200 / 32), last block partial


def test_degenerate_blocks():
    # all zero / fp32-subnormal maximum: scale byte 0, all exponent codes 0, signs kept
    blk = np.array([0.0, -0.0, 1e-40, -1e-41], np.float32)
    codes, sb = oracle.encode_block(blk, FMT_E3M0)
    assert sb == 0 and list(codes) == [0, 8, 0, 8]
    # tiny normal maximum: scale byte clamps at 0, values still resolved against 2^-127
    blk = np.array([2.0 ** -123, 2.0 ** -126, 2.0 ** -131], np.float32)
    codes, sb = oracle.encode_block(blk, FMT_E3M0)
    assert sb == 0 and list(codes) == [7, 4, 0]
    assert oracle.decode_code(7, 0, FMT_E3M0) == 2.0 ** -123
    assert oracle.decode_code(1, 0, FMT_E3M0) == 2.0 ** -129      # fp32 subnormal, exact
    # Inf / NaN anywhere in the block: scale byte 0xff, block decodes to NaN
    for bad in (np.inf, -np.inf, np.nan):
        blk = np.array([1.0, bad, -2.0], np.float32)
        for fmt in (FMT_E3M0, FMT_E4M3):
            codes, sb = oracle.encode_block(blk, fmt)
            assert sb == 0xff
            assert math.isnan(oracle.decode_code(int(codes[0]), sb, fmt))
    # huge finite maximum
    blk = np.array([3.0e38, 1.0], np.float32)
    codes, sb = oracle.encode_block(blk, FMT_E3M0)
    assert sb == 127 + 127 - 4 and codes[0] == 7 and codes[1] == 0
    assert oracle.decode_code(7, sb, FMT_E3M0) == 2.0 ** 127


# ------------------------------------------------------------------ other scale granularities

from oracle import FMT_E3M0_B64, FMT_E3M0_B128, FMT_E3M0_SPAN   # noqa: E402


def _delta_of(g, w):
    return g - _bf16_f32(w)


@pytest.mark.parametrize("fmt,block", [(FMT_E3M0_B64, 64), (FMT_E3M0_B128, 128), (FMT_E3M0_SPAN, 0)])
def test_wider_scale_blocks(fmt, block):
    n = 1000
    g, w = _make(n, 2, seed=21, scale=3e-3)
    g[500] += 0.5                       # one large outer gradient
    codes, scales = oracle.quantize_outer_grad(g, w, fmt)
    c32, s32 = oracle.quantize_outer_grad(g, w, FMT_E3M0)
    B = block or n
    for m in range(2):
        d = _delta_of(g, w[m])
        got = oracle.unpack_e3m0(codes[m], n)
        for b0 in range(0, n, B):
            blk = d[b0:b0 + B]
            a = np.abs(blk).max()
            e_a = int(np.float32(a).view(np.uint32) >> 23)
            sb = max(e_a - 4, 0)
            if block:
                assert scales[m][b0 // B] == sb
                # the wide block's scale is the largest of its 32-element blocks' scales
                assert sb == s32[m][b0 // 32:(b0 + B + 31) // 32].max()
            else:
                assert scales[m].size == 4 and scales[m].view(np.uint32)[0] == np.float32(a).view(np.uint32)
            # element codes: the exact nearest-magnitude rule under that scale
            for i in range(0, len(blk), 7):
                y = Fraction(abs(float(blk[i]))) / Fraction(2) ** (sb - 127)
                assert got[b0 + i] & 7 == _exact_e3m0(y), (m, b0, i)
                assert got[b0 + i] >> 3 == int(np.signbit(blk[i]))
    assert oracle.exchange_bytes(fmt, n) == (500, -(-n // B) if block else 4)


def test_span_scale_equals_block_scale_on_one_block():
    g, w = _make(32, 1, seed=22)
    c_blk, s_blk = oracle.quantize_outer_grad(g, w, FMT_E3M0)
    c_span, s_span = oracle.quantize_outer_grad(g, w, FMT_E3M0_SPAN)
    assert np.array_equal(c_blk[0], c_span[0])
    assert max(int(s_span[0].view(np.uint32)[0] >> 23) - 4, 0) == s_blk[0][0]
    # and the receive side decodes them alike
    ga, gb = g.copy(), g.copy()
    oracle.dequant_reduce_nesterov(ga, np.zeros(32, np.float32), c_blk, s_blk, FMT_E3M0, 1.0, 0.0)
    oracle.dequant_reduce_nesterov(gb, np.zeros(32, np.float32), c_span, s_span, FMT_E3M0_SPAN, 1.0, 0.0)
    assert np.array_equal(ga, gb)


def test_per_tensor_scale_is_four_bits_per_parameter():
    """The table of exchanged data (Section 3.2.2) implies exactly 4 bits per parameter: the ratio
    Data-Parallel / Streaming DiLoCo FP4 is H x 16 / 4 = 400.  With one scale word per tensor the
    encoded 1B model costs 4.0000x bits per parameter; with one scale byte per 32 elements 4.25."""
    import workloads
    numel, _, _ = workloads.SHAPES["1b"].units()
    total = sum(numel)
    span_bits = 8 * sum(sum(oracle.exchange_bytes(FMT_E3M0_SPAN, n)) for n in numel) / total
    block_bits = 8 * sum(sum(oracle.exchange_bytes(FMT_E3M0, n)) for n in numel) / total
    assert abs(span_bits - 4.0) < 1e-4 and abs(block_bits - 4.25) < 1e-9
    for budget, dp_tb, ours_tb in [l.split() for l in open(os.path.join(GOLDEN, "exchanged_data.txt"))
                                   if l.strip() and not l.startswith("#")]:
        ratio = float(dp_tb) / float(ours_tb)
        assert abs(ratio - 100 * 16 / span_bits) / ratio < 0.01          # H = 100 inner steps, 16-bit baseline
        assert abs(ratio - 100 * 16 / block_bits) / ratio > 0.05         # block scaling would not add up


# ------------------------------------------------------------------ block maximum rounded to nearest

from oracle import FMT_E3M0_RN   # noqa: E402


def test_round_to_nearest_maximum_variant():
    """E3M0_RN: same codes, same packing, the scale one binade higher (max / scale in [8, 16)).  Pins: the
    scale byte from the definition, every element by the exact-rational nearest search under that scale,
    the block maximum decodes to 2^e or 2^(e+1) whichever is nearer (tie at 1.5 * 2^e -> the even code, 8),
    nothing saturates, and a block whose maximum is doubled by a pilot element has the same codes in the
    default format (the two conventions differ by that factor of two and nothing else)."""
    n = 32 * 40
    g, w = _make(n, 2, seed=31, scale=2e-3)
    g[7] += 0.25
    codes, scales = oracle.quantize_outer_grad(g, w, FMT_E3M0_RN)
    assert oracle.exchange_bytes(FMT_E3M0_RN, n) == oracle.exchange_bytes(FMT_E3M0, n) == (n // 2, n // 32)
    for m in range(2):
        d = _delta_of(g, w[m])
        got = oracle.unpack_e3m0(codes[m], n)
        for b0 in range(0, n, 32):
            blk = d[b0:b0 + 32]
            a = np.abs(blk).max()
            e_a = int(np.float32(a).view(np.uint32) >> 23)
            sb = max(e_a - 3, 0)
            assert scales[m][b0 // 32] == sb
            top = Fraction(float(a)) / Fraction(2) ** (sb - 127)
            assert 8 <= top < 16
            for i in range(32):
                y = Fraction(abs(float(blk[i]))) / Fraction(2) ** (sb - 127)
                assert got[b0 + i] & 7 == _exact_e3m0(y), (m, b0, i)
                assert got[b0 + i] >> 3 == int(np.signbit(blk[i]))
            i_top = int(np.abs(blk).argmax())
            dec = abs(oracle.decode_code(int(got[b0 + i_top]), sb, FMT_E3M0_RN))
            lo = 2.0 ** (e_a - 127)
            assert dec == (lo if top <= 12 else 2 * lo)
            # the same block with a pilot element of twice the maximum, in the default format: the
            # scale is the same, so are the codes of the original elements
            pilot = np.concatenate([blk[:31], np.float32([2 * a])]).astype(np.float32)
            c_def, sb_def = oracle.encode_block(pilot, FMT_E3M0)
            assert sb_def == sb
            assert np.array_equal(c_def[:31], got[b0:b0 + 31])
    # decode is the default format's decode
    for code in range(16):
        for sb in (0, 1, 100, 127, 254, 255):
            a, b = oracle.decode_code(code, sb, FMT_E3M0_RN), oracle.decode_code(code, sb, FMT_E3M0)
            assert (a == b) or (a != a and b != b)


def test_round_to_nearest_maximum_tie_and_powers_of_two():
    # a block whose maximum is exactly 1.5 * 2^k: tie between 8 and 16 -> even code 6 (value 8)
    blk = np.zeros(32, np.float32)
    blk[3] = 1.5 * 2.0 ** -9
    blk[4] = -(2.0 ** -9)
    blk[5] = 2.0 ** -14           # 5 binades below the maximum's binade: the smallest magnitude, 1/4 of the scale
    blk[6] = 2.0 ** -15           # exactly half of it: tie with zero -> even code 0
    blk[8] = 2.0 ** -15 * 1.0000001
    c, sb = oracle.encode_block(blk, FMT_E3M0_RN)
    assert sb == (127 - 9) - 3
    assert list(c[[3, 4, 5, 6, 8]]) == [6, 8 | 6, 1, 0, 1]
    for i in (4, 5):
        assert oracle.decode_code(int(c[i]), sb, FMT_E3M0_RN) == blk[i]
    # the whole step accepts the format and the fused step equals the three calls
    g, w = _make(4096 + 37, 3, seed=33)
    wn = [x.copy() for x in w]
    g2, m2 = g.copy(), np.zeros_like(g)
    g3, m3, w3 = g.copy(), np.zeros_like(g), [x.copy() for x in w]
    oracle.fragment_outer_step(g2, m2, w, wn, FMT_E3M0_RN, 0.7, 0.9, 0.5)
    rc, rs = oracle.quantize_outer_grad(g3, w, FMT_E3M0_RN)
    oracle.dequant_reduce_nesterov(g3, m3, rc, rs, FMT_E3M0_RN, 0.7, 0.9)
    oracle.merge_overlap(g3, w3, 0.5)
    assert np.array_equal(g2, g3) and np.array_equal(m2, m3)
    assert all(np.array_equal(a, b) for a, b in zip(wn, w3))
