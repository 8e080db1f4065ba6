/*
 * sdl_ref.c -- CPU oracle for the Streaming DiLoCo per-fragment outer step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * statement of what the fragment outer step computes.  It exists so that the
 * GPU library can be checked against it.  It shares no code, header, table or
 * constant with the GPU library, and the GPU library never calls it.
 *
 * What it follows (Streaming DiLoCo paper):
 *   - Algorithm 2, send branch: each replica m forms its outer gradient for
 *     fragment p, Delta_m = theta_global - theta_m   (global minus local).
 *   - Section 2.4 (low-precision outer gradients): every replica's *unreduced*
 *     outer gradient is compressed before it is exchanged, down to a 4-bit
 *     float with 1 sign bit, 3 exponent bits and no mantissa bit (E3M0);
 *     after receipt the accumulation over replicas happens in FP32.
 *   - Algorithm 2, receive branch: the averaged outer gradient (1/M sum) is
 *     given to OuterOpt, which Section 2.1 fixes as SGD with Nesterov
 *     momentum, applied to the previously synchronised (global) parameters.
 *   - Algorithm 2, last statement, and Section 2.3: the result is mixed into
 *     each replica's locally advanced copy,
 *     theta_m <- alpha * theta_m + (1 - alpha) * theta_tilde.
 *
 * Points the paper leaves open, and the reading taken here (each one is also
 * listed in the design notes of the repository):
 *   - E3M0 value set: code = s<<3 | E; E == 0 is zero, otherwise the
 *     magnitude is 2^(E-3) (bias 3, no Inf/NaN), i.e. {0, 1/4, 1/2, 1, 2, 4,
 *     8, 16}.  s is always the sign bit of the fp32 outer gradient.
 *   - Scaling: blocks of 32 consecutive elements share one power-of-two scale
 *     byte sb (value 2^(sb-127)), chosen from the block's absolute maximum a
 *     so that a / scale lies in [16, 32) for E3M0 (largest element magnitude
 *     exponent 4) and in [256, 512) for E4M3 (largest exponent 8).  Variants of
 *     E3M0 use blocks of 64 or 128 elements, or the whole span (one scale per
 *     tensor, the 4.0 bits per parameter that the paper's table of exchanged
 *     data implies).  One more variant (E3M0_RN) places a / scale in [8, 16)
 *     instead, so that the block maximum is rounded to nearest rather than
 *     saturated; which of the two the paper's own encoder does is unknown.
 *   - Rounding: nearest representable magnitude measured in the linear
 *     domain, ties to the even code, saturating at the largest magnitude.
 *   - Nibble order: element 2j in the low nibble of byte j, 2j+1 in the high.
 *   - Nesterov form: mom' = mu*mom + d ; g' = g - lr*(d + mu*mom').
 *   - All arithmetic on values is IEEE binary32 with one rounding per
 *     operation, in the order written (compile with -ffp-contract=off); the
 *     sum over replicas runs m = 0, 1, ..., M-1 starting from +0.
 *
 * Parity status: no passage of the paper prints a worked E3M0 example, so the
 * E3M0 encoder is pinned only by mathematical properties (threshold table
 * derived by hand from the value set, closed form, exact round trips,
 * symmetry, scale invariance, error bound).  E3M0 versus the paper's own
 * encoder (either placement of the block maximum): parity unpinned.  E4M3,
 * BF16, Nesterov and the merge are pinned
 * against library routines and closed forms in the CPU test-suite.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Exchange formats.  Numbering is this file's own.  Formats 4 to 6 are E3M0 with
 * another scale granularity: blocks of 64 or 128 elements, or one scale for the whole span
 * (per tensor), which is what the paper's accounting of exactly 4 bits per parameter
 * suggests.  A whole-span scale is stored as a 4-byte word: the fp32 bit pattern of the
 * span's absolute maximum (the scale byte follows from its exponent field as for blocks).
 * Format 7 is E3M0 in 32-element blocks with the scale one binade higher, so that the block
 * maximum a falls into [8, 16) of the code grid and is rounded to nearest like every other
 * element (2^floor(log2 a) or twice that), instead of into [16, 32) where it always
 * saturates downwards.  Section 2.4 of the paper says nothing on scaling; both are readings. */
enum { REF_FMT_FP32 = 0, REF_FMT_BF16 = 1, REF_FMT_E4M3 = 2, REF_FMT_E3M0 = 3,
       REF_FMT_E3M0_B64 = 4, REF_FMT_E3M0_B128 = 5, REF_FMT_E3M0_SPAN = 6, REF_FMT_E3M0_RN = 7,
       REF_FMT_COUNT = 8 };

#define REF_BLOCK 32u /* elements that share one scale byte in the default formats */

static int is_e3m0(int fmt) { return fmt == REF_FMT_E3M0 || fmt >= REF_FMT_E3M0_B64; }
static int is_scaled(int fmt) { return fmt == REF_FMT_E4M3 || is_e3m0(fmt); }
/* exponent of the code grid that the block maximum's binade is mapped to */
static unsigned elem_emax(int fmt) { return fmt == REF_FMT_E4M3 ? 8u : fmt == REF_FMT_E3M0_RN ? 3u : 4u; }
/* elements per scale; 0 = the whole span */
static uint64_t block_of(int fmt)
{
    switch (fmt) {
    case REF_FMT_E3M0_B64: return 64;
    case REF_FMT_E3M0_B128: return 128;
    case REF_FMT_E3M0_SPAN: return 0;
    default: return REF_BLOCK;
    }
}

/* ---------------------------------------------------------------- helpers */

static uint32_t f32_bits(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }
static float bits_f32(uint32_t u) { float x; memcpy(&x, &u, 4); return x; }

/* bf16 is the upper half of a binary32: widening is exact. */
static float bf16_to_f32(uint16_t h) { return bits_f32((uint32_t)h << 16); }

/* Round a binary32 to bf16, nearest, ties to even; NaN stays a quiet NaN. */
static uint16_t f32_to_bf16_rne(float x)
{
    uint32_t u = f32_bits(x);
    if ((u & 0x7fffffffu) > 0x7f800000u)            /* NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* Magnitude of an E3M0 exponent code (bias 3, E == 0 is zero). */
static double e3m0_magnitude(unsigned E) { return E == 0 ? 0.0 : ldexp(1.0, (int)E - 3); }

/* Magnitude of an E4M3 code without its sign bit (OCP FP8 E4M3: bias 7,
 * subnormals m * 2^-9, largest finite 448 = code 0x7e, code 0x7f is NaN). */
static double e4m3_magnitude(unsigned c)
{
    unsigned e = (c >> 3) & 15u, m = c & 7u;
    if (e == 0) return ldexp((double)m, -9);
    return ldexp(1.0 + (double)m / 8.0, (int)e - 7);
}

/* Nearest code in the linear domain among codes 0..last whose magnitudes
 * increase with the code; a tie between two neighbours goes to the even
 * code; anything above the largest magnitude saturates to it.  y >= 0 and
 * finite.  y is held in double, where fp32 * 2^k and the distances that can
 * tie are exact. */
static unsigned nearest_code(double y, unsigned last, double (*mag)(unsigned))
{
    unsigned best = 0;
    double best_d = fabs(y - mag(0));
    for (unsigned c = 1; c <= last; ++c) {
        double d = fabs(y - mag(c));
        if (d < best_d || (d == best_d && (c & 1u) == 0u)) { best = c; best_d = d; }
    }
    return best;
}

/* Absolute maximum of one block: the fp32 bit pattern (sign cleared) of the largest
 * magnitude, where any Inf / NaN counts as larger than every finite value. */
static uint32_t block_max_bits(const float* d, uint64_t len)
{
    uint32_t a = 0;
    for (uint64_t i = 0; i < len; ++i) {
        uint32_t m = f32_bits(d[i]) & 0x7fffffffu;
        if (m > a) a = m;
    }
    return a;
}

/* Scale byte for a block whose largest magnitude has biased exponent e_a and
 * whose binade is mapped to exponent emax of the code grid (4 for E3M0, the grid's largest
 * value; 3 for the round-to-nearest variant; 8 for E4M3):
 * 2^(sb-127) = 2^(floor(log2 a) - emax), clamped at sb = 0; a zero or
 * fp32-subnormal maximum gives sb = 0; Inf/NaN gives 0xff. */
static unsigned scale_byte(unsigned e_a, unsigned emax)
{
    if (e_a == 255u) return 0xffu;
    if (e_a <= emax) return 0u;
    return e_a - emax;
}

/* Element code (sign and magnitude code) of one outer gradient in a block whose largest
 * magnitude has biased exponent e_a. */
static unsigned encode_element(float x, unsigned e_a, int fmt)
{
    const unsigned emax = elem_emax(fmt);
    const unsigned sign_shift = is_e3m0(fmt) ? 3u : 7u;
    const unsigned sb = scale_byte(e_a, emax);
    unsigned s = f32_bits(x) >> 31;
    unsigned mag_code = 0;
    if (e_a != 0u && e_a != 255u) {
        double y = ldexp(fabs((double)x), 127 - (int)sb);
        mag_code = is_e3m0(fmt) ? nearest_code(y, 7u, e3m0_magnitude) : nearest_code(y, 0x7eu, e4m3_magnitude);
    }
    return (s << sign_shift) | mag_code;
}

/* Encode one block of up to 32 outer gradients into unpacked element codes
 * (one per byte, E3M0 in the low 4 bits / E4M3 in all 8) and its scale byte. */
static unsigned encode_block(const float* d, unsigned len, int fmt, uint8_t* code)
{
    const unsigned emax = elem_emax(fmt);
    unsigned e_a = block_max_bits(d, len) >> 23;
    for (unsigned i = 0; i < len; ++i) code[i] = (uint8_t)encode_element(d[i], e_a, fmt);
    return scale_byte(e_a, emax);
}

/* Decode one element of a scaled format.  A block whose scale byte is 0xff
 * decodes to NaN in every element. */
static float decode_scaled(unsigned code, unsigned sb, int fmt)
{
    if (sb == 0xffu) return bits_f32(0x7fc00000u);
    double mag;
    unsigned s;
    if (is_e3m0(fmt)) { mag = e3m0_magnitude(code & 7u); s = (code >> 3) & 1u; }
    else                     { mag = e4m3_magnitude(code & 0x7fu); s = (code >> 7) & 1u; }
    /* at most 4 significant bits times a power of two no smaller than
     * 2^-136: exactly representable in binary32, subnormals included */
    float v = (float)ldexp(mag, (int)sb - 127);
    return s ? -v : v;
}

static size_t ceil_div(uint64_t a, uint64_t b) { return (size_t)((a + b - 1) / b); }

/* ------------------------------------------------------------- public API */

/* Bytes of the code array and of the scale array of one replica for n
 * elements.  Returns their sum. */
size_t sdl_ref_exchange_bytes(int fmt, uint64_t n, size_t* code_bytes, size_t* scale_bytes)
{
    size_t c = 0, s = 0;
    switch (fmt) {
    case REF_FMT_FP32: c = (size_t)n * 4; break;
    case REF_FMT_BF16: c = (size_t)n * 2; break;
    case REF_FMT_E4M3: c = (size_t)n; s = ceil_div(n, REF_BLOCK); break;
    case REF_FMT_E3M0: case REF_FMT_E3M0_B64: case REF_FMT_E3M0_B128: case REF_FMT_E3M0_RN:
        c = ceil_div(n, 2); s = ceil_div(n, block_of(fmt)); break;
    case REF_FMT_E3M0_SPAN: c = ceil_div(n, 2); s = n ? 4 : 0; break;
    default: break;
    }
    if (code_bytes) *code_bytes = c;
    if (scale_bytes) *scale_bytes = s;
    return c + s;
}

/* Algorithm 2 send branch + Section 2.4: for every replica m, the outer
 * gradient g - w_send[m] of n elements, encoded in the exchange format.
 * w_send[m]: bf16 bit patterns.  codes[m], scales[m]: sized as
 * sdl_ref_exchange_bytes says (scales unused for FP32/BF16). */
int sdl_ref_quantize_outer_grad(const float* g, const uint16_t* const* w_send, uint32_t M,
                                uint64_t n, int fmt, uint8_t* const* codes, uint8_t* const* scales)
{
    if (fmt < 0 || fmt >= REF_FMT_COUNT) return -1;
    for (uint32_t m = 0; m < M; ++m) {
        const uint16_t* w = w_send[m];
        if (fmt == REF_FMT_FP32) {
            float* out = (float*)codes[m];
            for (uint64_t i = 0; i < n; ++i) out[i] = g[i] - bf16_to_f32(w[i]);
            continue;
        }
        if (fmt == REF_FMT_BF16) {
            uint16_t* out = (uint16_t*)codes[m];
            for (uint64_t i = 0; i < n; ++i) out[i] = f32_to_bf16_rne(g[i] - bf16_to_f32(w[i]));
            continue;
        }
        if (is_e3m0(fmt)) memset(codes[m], 0, ceil_div(n, 2));
        const uint64_t block = block_of(fmt) ? block_of(fmt) : (n ? n : 1);
        const unsigned emax = elem_emax(fmt);
        float* d = (float*)malloc((size_t)(block < n ? block : n) * sizeof(float) + 4);
        if (!d) return -5;
        for (uint64_t b0 = 0; b0 < n; b0 += block) {
            uint64_t len = (n - b0 < block) ? (n - b0) : block;
            for (uint64_t i = 0; i < len; ++i) d[i] = g[b0 + i] - bf16_to_f32(w[b0 + i]);
            const uint32_t amax = block_max_bits(d, len);
            const unsigned e_a = amax >> 23;
            if (fmt == REF_FMT_E3M0_SPAN) memcpy(scales[m], &amax, 4);
            else scales[m][b0 / block] = (uint8_t)scale_byte(e_a, emax);
            for (uint64_t i = 0; i < len; ++i) {
                uint64_t k = b0 + i;
                unsigned c = encode_element(d[i], e_a, fmt);
                if (fmt == REF_FMT_E4M3) codes[m][k] = (uint8_t)c;
                else codes[m][k >> 1] |= (uint8_t)((c & 15u) << ((k & 1u) * 4u));
            }
        }
        free(d);
    }
    return 0;
}

/* Scale byte that governs element i of a scaled message. */
static unsigned scale_of(const uint8_t* scale, uint64_t i, int fmt)
{
    if (fmt == REF_FMT_E3M0_SPAN) {
        uint32_t amax;
        memcpy(&amax, scale, 4);
        return scale_byte(amax >> 23, 4u);
    }
    return scale[i / block_of(fmt)];
}

/* Value that replica m's message holds for element i. */
static float decode_element(const uint8_t* code, const uint8_t* scale, uint64_t i, int fmt)
{
    switch (fmt) {
    case REF_FMT_FP32: return ((const float*)code)[i];
    case REF_FMT_BF16: return bf16_to_f32(((const uint16_t*)code)[i]);
    case REF_FMT_E4M3: return decode_scaled(code[i], scale_of(scale, i, fmt), fmt);
    default:           return decode_scaled((code[i >> 1] >> ((i & 1u) * 4u)) & 15u, scale_of(scale, i, fmt), fmt);
    }
}

/* Section 2.4 (FP32 accumulation) + Algorithm 2 receive branch: decode the M
 * messages, average them in fp32, and apply SGD with Nesterov momentum to the
 * global parameters g and the momentum mom, both updated in place. */
int sdl_ref_dequant_reduce_nesterov(float* g, float* mom, const uint8_t* const* codes,
                                    const uint8_t* const* scales, uint32_t M, uint64_t n, int fmt,
                                    float lr, float mu)
{
    if (fmt < 0 || fmt >= REF_FMT_COUNT || M == 0) return -1;
    for (uint64_t i = 0; i < n; ++i) {
        float acc = 0.0f;
        for (uint32_t m = 0; m < M; ++m) {
            float v = decode_element(codes[m], scales ? scales[m] : NULL, i, fmt);
            acc = acc + v;
        }
        float dbar = acc / (float)M;
        float mu_mom = mu * mom[i];
        float mom_new = mu_mom + dbar;
        float mu_mom_new = mu * mom_new;
        float look = dbar + mu_mom_new;
        float step = lr * look;
        mom[i] = mom_new;
        g[i] = g[i] - step;
    }
    return 0;
}

/* Algorithm 2 last statement / Section 2.3: every replica's current bf16
 * parameters are replaced by alpha * local + (1 - alpha) * g_new, computed in
 * fp32 (1 - alpha is formed once in fp32) and rounded to bf16. */
int sdl_ref_merge_overlap(const float* g_new, uint16_t* const* w_now, uint32_t M, uint64_t n,
                          float alpha)
{
    const float one_minus_alpha = 1.0f - alpha;
    for (uint32_t m = 0; m < M; ++m) {
        uint16_t* w = w_now[m];
        for (uint64_t i = 0; i < n; ++i) {
            float local_part = alpha * bf16_to_f32(w[i]);
            float global_part = one_minus_alpha * g_new[i];
            float mixed = local_part + global_part;
            w[i] = f32_to_bf16_rne(mixed);
        }
    }
    return 0;
}

/* The whole outer step of one span: quantize -> (exchange) -> dequantize,
 * average, Nesterov -> merge.  w_send[m] may be the same array as w_now[m]
 * (no overlap, tau = 0).  If codes_out / scales_out are not NULL they receive
 * the exchanged messages. */
int sdl_ref_fragment_outer_step(float* g, float* mom, const uint16_t* const* w_send,
                                uint16_t* const* w_now, uint32_t M, uint64_t n, int fmt, float lr,
                                float mu, float alpha, uint8_t* const* codes_out,
                                uint8_t* const* scales_out)
{
    if (fmt < 0 || fmt >= REF_FMT_COUNT || M == 0) return -1;
    size_t cb, sb;
    sdl_ref_exchange_bytes(fmt, n, &cb, &sb);
    uint8_t** codes = (uint8_t**)calloc(M, sizeof(uint8_t*));
    uint8_t** scales = (uint8_t**)calloc(M, sizeof(uint8_t*));
    if (!codes || !scales) { free(codes); free(scales); return -5; }
    int rc = 0;
    for (uint32_t m = 0; m < M; ++m) {
        codes[m] = (uint8_t*)malloc(cb ? cb : 1);
        scales[m] = (uint8_t*)malloc(sb ? sb : 1);
        if (!codes[m] || !scales[m]) rc = -5;
    }
    if (rc == 0) rc = sdl_ref_quantize_outer_grad(g, w_send, M, n, fmt, codes, scales);
    if (rc == 0) {
        for (uint32_t m = 0; m < M; ++m) {
            if (codes_out && codes_out[m]) memcpy(codes_out[m], codes[m], cb);
            if (scales_out && scales_out[m]) memcpy(scales_out[m], scales[m], sb);
        }
        rc = sdl_ref_dequant_reduce_nesterov(g, mom, (const uint8_t* const*)codes,
                                             (const uint8_t* const*)scales, M, n, fmt, lr, mu);
    }
    if (rc == 0) rc = sdl_ref_merge_overlap(g, w_now, M, n, alpha);
    for (uint32_t m = 0; m < M; ++m) { free(codes[m]); free(scales[m]); }
    free(codes);
    free(scales);
    return rc;
}

/* ------------------------------------------- element-level entry points
 * (used by the CPU pin tests to probe the encoder without building replicas) */

/* Encode len <= 32 fp32 values as one block; code_out gets one unpacked
 * element code per byte; returns the scale byte. */
int sdl_ref_encode_block(const float* delta, uint32_t len, int fmt, uint8_t* code_out)
{
    if (len == 0 || len > REF_BLOCK || !is_scaled(fmt)) return -1;
    return (int)encode_block(delta, len, fmt, code_out);
}

/* Decode one unpacked element code under scale byte sb. */
float sdl_ref_decode_code(uint32_t code, uint32_t sb, int fmt)
{
    return decode_scaled(code, sb, fmt);
}
