// Device side of the library: the streaming kernels of the fragment outer step for
// gfx950 (MI355X), and the C entry points that launch them.
//
// One templated kernel serves every call: send side (quantize), receive side (decode + mean +
// Nesterov, with or without the merge), merge alone, and the fused outer step; the
// absolute-maximum pre-pass of the whole-span scale is a kernel of its own.
//
// Work decomposition (all modes).  A workgroup is one 64-lane wavefront and owns a
// tile of one or two rows of 256 consecutive parameters (the height is chosen per call and
// replica count, see tile_rows).  Lane l owns the four parameters [4l, 4l+4) of each row, so
//   - every memory instruction of the wavefront touches one contiguous piece of an
//     array (1 KiB of fp32 through 128-bit accesses, 512 B of bf16 through 64-bit
//     accesses): whole cache lines, nothing strided;
//   - eight neighbouring lanes own one 32-element scale block, and the block maximum
//     is three DPP exchanges (two inside the quad, one across the half row); wider
//     blocks add a row mirror and ds_bpermute exchanges.  No LDS storage is used.
// Full, 16-byte aligned tiles use buffer instructions with non-temporal cache policy
// (every byte is touched once); full tiles of runs whose model arrays start at some other
// element use vector accesses of element alignment in the same lane layout; ragged tails
// and calls with unaligned message arrays use guarded element-wise accesses.  A launch covers up to kMaxRuns contiguous runs of the flat
// model; every workgroup belongs to exactly one run, so scale blocks never straddle
// runs.
//
// Arithmetic contract (Algorithm 2 and Sections 2.1, 2.3, 2.4 of the paper, with the
// exchange formats documented in sdl.h): every fp32 operation is a single IEEE
// operation in the documented order; this file must be compiled with
// -ffp-contract=off and with fp32 denormals enabled (the hipcc default).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <mutex>

#include "sdl.h"
#include "sdl_device.h"

// Scale words of the allocation-free fused step (sdl_fragment_outer_step_plan_static): for the
// whole-span scale, one 4-byte word per span and replica, replica m's words at
// scratch + m * SDL_STATIC_MAX_SPANS.  Every GPU the library runs on holds its own copy of the
// array at its own address until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress: kernels and fills always get the per-device address kept below.
static __device__ __align__(256) uint32_t scratch[SDL_STATIC_MAX_SPANS * SDL_MAX_WORKERS];

namespace {

using namespace sdl_device;

constexpr int kVec = 4;                       // consecutive parameters a lane owns in one row
constexpr int kMaxRows = 2;                   // rows of the tallest tile
constexpr int kRow = kVec * kWave;            // parameters per row (256); a workgroup is one wavefront
constexpr int kPad = kRow * kMaxRows;          // message and staging layouts pad every piece to this many
                                              // parameters (512): a whole number of tiles of either height
constexpr int kMaxRuns = 16;                  // runs per launch

enum Mode { kQuantize = 0, kReduce = 1, kMerge = 2, kFused = 3, kReceive = 5 };   // kReceive = kReduce + kMerge

// Rows of a workgroup's tile, by call and compile-time replica count (0 = any M at run time).
// Rows are independent of each other (a scale block never leaves its row), so the height is a
// pure scheduling choice.  Measured on MI355X over 302 M parameters: one row instead of two gains
// 3-5 % on the fused kernel and the one-pass receive at M = 1, 2 and 4, 2-9 % on the receive side
// without the merge and 7 % on the merge at M = 1, and loses 2 % on the first two at M = 8, 1-3 % on
// the merge at M >= 2 and 3-12 % on the send side.  The whole-span scale keeps two rows: every tile reads its span's scale words, all
// tiles of a span the same few bytes, and twice the tiles cost it 8-14 %.
constexpr int tile_rows(int mode, int mt, int fmt)
{
    if (fmt == SDL_FMT_E3M0_SPAN) return 2;
    if (mode == kReduce) return mt > 0 ? 1 : 2;
    if (mode == kFused || mode == kReceive) return (mt == 1 || mt == 2 || mt == 4) ? 1 : 2;
    if (mode == kMerge) return mt == 1 ? 1 : 2;
    return 2;
}
// The compile-time replica count a call runs with: the kernels are built for 1, 2, 4 and 8 replicas
// plus one variant that takes any M; the message-writing fused kernel is a verification aid, for
// which the any-M variant is enough.
constexpr uint32_t variant_mt(int mode, uint32_t M, bool emit)
{
    const uint32_t mt = (mode == kFused && emit) ? 0u : M;
    return (mt == 1 || mt == 2 || mt == 4 || mt == 8) ? mt : 0u;
}

constexpr bool is_e3m0(int f) { return f == SDL_FMT_E3M0 || f >= SDL_FMT_E3M0_B64; }
constexpr bool is_scaled(int f) { return f == SDL_FMT_E4M3 || is_e3m0(f); }
constexpr bool is_span_scaled(int f) { return f == SDL_FMT_E3M0_SPAN; }
// elements that share a scale (0: the whole span)
constexpr int block_elems(int f)
{
    return f == SDL_FMT_E3M0_B64 ? 64 : f == SDL_FMT_E3M0_B128 ? 128 : f == SDL_FMT_E3M0_SPAN ? 0 : SDL_BLOCK;
}

// How the whole tiles of a run reach memory (a ragged last tile always takes the guarded path).
enum TilePath : uint32_t {
    kPathGuarded = 0,   // element by element: some message array is not 16-byte aligned
    kPathBuffer = 1,    // every array of the call is 16-byte aligned at the run's first element
    kPathVector = 2,    // the message arrays are, the model arrays start at some other element
};

struct Run {
    uint64_t offset;     // first element of the run in the flat arrays
    uint64_t numel;
    uint64_t msg;        // where the run starts in the message arrays, in elements (a multiple of 512)
    uint64_t soff;       // where the run starts in staged g / mom arrays, in elements (staged state only)
    uint32_t first_wg;   // first workgroup of the launch that works on this run
    uint32_t path;       // TilePath of the run's whole tiles
    uint32_t sidx;       // whole-span scale: index of the run's 4-byte scale word
    uint32_t pad_;
};

struct Args {
    float* g;
    float* mom;
    const uint16_t* w_send[SDL_MAX_WORKERS];
    uint16_t* w_now[SDL_MAX_WORKERS];
    uint8_t* codes[SDL_MAX_WORKERS];
    uint8_t* scales[SDL_MAX_WORKERS];
    Run runs[kMaxRuns];
    uint32_t n_runs;
    uint32_t M;
    float lr, mu, alpha, one_minus_alpha;
    uint32_t aliased;    // w_send[m] == w_now[m]
    uint32_t emit;       // fused kernel: also write the messages
    uint32_t staged;     // g / mom point at a staging buffer that holds only this fragment
};

// Cache policy bits of the buffer instructions on gfx950: 1 = sc0, 2 = nt, 16 = sc1.
constexpr int kAuxLoad = 2;      // loads: non-temporal (every byte is touched once)
constexpr int kAuxStore = 2;     // stores: non-temporal
constexpr int kAuxScale = 0;     // scale bytes: 16 per tile, 8 tiles per cache line -> let L2 combine them
constexpr int kWavesPerEu = 2;   // register budget: at least this many wavefronts per SIMD

// ------------------------------------------------------------------ bit helpers

// bf16 pair packed in one dword: element 0 in the low half.
__device__ __forceinline__ float bf16_lo(uint32_t u) { return u2f(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return u2f(u & 0xffff0000u); }

// Two fp32 -> packed bf16, round to nearest even, NaN stays a quiet NaN (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t bf16_pack(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ void unpack_bf16(const uint32_t (&u)[2], float (&v)[kVec])
{
    v[0] = bf16_lo(u[0]); v[1] = bf16_hi(u[0]); v[2] = bf16_lo(u[1]); v[3] = bf16_hi(u[1]);
}

// Maximum over the LANES consecutive lanes that share a scale block (8, 16, 32 or all 64).
template <int LANES>
__device__ __forceinline__ uint32_t lanes_max(uint32_t v)
{
    uint32_t t = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);    // quad_perm 1,0,3,2
    v = v > t ? v : t;
    t = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);             // quad_perm 2,3,0,1
    v = v > t ? v : t;
    t = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x141, 0xF, 0xF, true);            // row_half_mirror: 7-i
    v = v > t ? v : t;
    if constexpr (LANES >= 16) {
        t = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x140, 0xF, 0xF, true);        // row_mirror: 15-i
        v = v > t ? v : t;
    }
    if constexpr (LANES >= 32) {
        t = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(((threadIdx.x ^ 16u) & 63u) << 2), (int)v);   // lane ^ 16
        v = v > t ? v : t;
    }
    if constexpr (LANES >= 64) {
        t = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(((threadIdx.x ^ 32u) & 63u) << 2), (int)v);   // lane ^ 32
        v = v > t ? v : t;
    }
    return v;
}

// ------------------------------------------------------------------ exchange formats
// A message element is produced in two forms: its decoded fp32 value dq (what the
// receiver accumulates) and, when asked for, its code.

struct BlockScale {
    uint32_t sb;      // scale byte
    float inv;        // 2^(127-sb), or 0 for a degenerate block
    float scale;      // 2^(sb-127), NaN for a block that holds Inf/NaN
    bool degenerate;  // block maximum is zero, subnormal, Inf or NaN
};

template <int FMT>
__device__ __forceinline__ BlockScale block_scale_from_exponent(uint32_t e_a)
{
    // written with single comparisons and selects: this runs once per scale block and replica,
    // and as control flow it cost more than the codec of the block's elements
    // exponent of the code grid that the block maximum's binade is mapped to
    constexpr uint32_t emax = FMT == SDL_FMT_E4M3 ? 8u : FMT == SDL_FMT_E3M0_RN ? 3u : 4u;
    BlockScale b;
    const uint32_t sb = e_a > emax ? e_a - emax : 0u;
    const bool nan_block = e_a == 255u;
    b.degenerate = (e_a - 1u) >= 254u;                          // 0 (zero / subnormal maximum) or 255 (Inf / NaN)
    b.inv = b.degenerate ? 0.0f : u2f((254u - sb) << 23);
    const uint32_t scale_bits = (sb << 23) > 0x00400000u ? (sb << 23) : 0x00400000u;   // 2^-127 is an fp32 subnormal
    b.scale = u2f(nan_block ? 0x7fc00000u : scale_bits);
    b.sb = nan_block ? 255u : sb;
    return b;
}

__device__ __forceinline__ float scale_from_byte(uint32_t sb)
{
    float s = sb ? u2f(sb << 23) : u2f(0x00400000u);
    return sb == 255u ? u2f(0x7fc00000u) : s;
}

// Encode the lane's 4 outer gradients d of one row and one replica.  dq = decoded
// values.  Codes: E3M0 -> c[0] holds 4 nibbles (16 bits); E4M3 -> c[0] holds 4 bytes;
// BF16 -> c[0..1]; FP32 -> the bits of d.  sb = scale byte of the lane's block.
// span_amax: for the whole-span scale, the bit pattern of the span's absolute maximum.
template <int FMT>
__device__ __forceinline__ void encode(const float (&d)[kVec], float (&dq)[kVec], uint32_t (&c)[kVec],
                                       uint32_t& sb, bool want_codes, uint32_t span_amax)
{
    if constexpr (FMT == SDL_FMT_FP32) {
#pragma unroll
        for (int j = 0; j < kVec; ++j) { dq[j] = d[j]; c[j] = f2u(d[j]); }
        sb = 0;
    } else if constexpr (FMT == SDL_FMT_BF16) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            c[k] = bf16_pack(d[2 * k], d[2 * k + 1]);
            dq[2 * k] = bf16_lo(c[k]);
            dq[2 * k + 1] = bf16_hi(c[k]);
        }
        sb = 0;
    } else {
        uint32_t amax = 0;
#pragma unroll
        for (int j = 0; j < kVec; ++j) {
            const uint32_t m = f2u(d[j]) & 0x7fffffffu;
            amax = m > amax ? m : amax;
        }
        if constexpr (is_span_scaled(FMT)) amax = span_amax;
        else amax = lanes_max<block_elems(FMT) / kVec>(amax);
        const BlockScale b = block_scale_from_exponent<FMT>(amax >> 23);
        sb = b.sb;
        uint32_t packed = 0;
        if constexpr (FMT == SDL_FMT_E4M3) {
            // OCP FP8 E4M3 through the conversion instructions of gfx950 (round to nearest even,
            // subnormals, signed zero); they do not saturate, so clamp to +-448 first
            float y[kVec];
#pragma unroll
            for (int j = 0; j < kVec; ++j) y[j] = __builtin_amdgcn_fmed3f(d[j] * b.inv, 448.0f, -448.0f);
            packed = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], 0, false);
            packed = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], (int)packed, true);
            if (b.sb == 255u) {
                // a block that holds Inf / NaN keeps only the signs (0 * Inf made NaN codes above)
                packed = 0;
#pragma unroll
                for (int j = 0; j < kVec; ++j) packed |= ((f2u(d[j]) >> 24) & 0x80u) << (8 * j);
            }
            const f32x2_t lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)packed, false);
            const f32x2_t hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)packed, true);
            dq[0] = lo.x * b.scale; dq[1] = lo.y * b.scale; dq[2] = hi.x * b.scale; dq[3] = hi.y * b.scale;
        } else {
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                const float y = __builtin_fabsf(d[j]) * b.inv;     // exact power-of-two scaling
                const uint32_t yb = f2u(y);
                const uint32_t sign = f2u(d[j]) & 0x80000000u;
                // nearest power of two in the linear domain; a tie (mantissa exactly
                // 1.5) goes to the even exponent code, whose parity is that of the
                // biased fp32 exponent because the re-bias (124) is even
                const uint32_t rr = yb + 0x3fffffu + ((yb >> 23) & 1u);
                const float pw = __builtin_amdgcn_fmed3f(u2f(rr & 0x7f800000u), 0.25f, 16.0f);
                const float val = y > 0.125f ? pw : 0.0f;          // half of the smallest magnitude
                dq[j] = u2f(sign | f2u(val * b.scale));
                if (want_codes) {
                    // the code comes straight from a rounded bit pattern, not from val, so that a
                    // kernel that only writes messages does not carry the decode arithmetic: clamp
                    // to [1/4, 16] first (exact: everything below rounds up to 1/4 or is the zero
                    // code, everything above saturates), round as above with 4 added to the
                    // exponent field, and the three low bits of the field are the code
                    // (fields 125..131 -> 129..135 -> 1..7)
                    const uint32_t cb = f2u(__builtin_amdgcn_fmed3f(y, 0.25f, 16.0f));
                    const uint32_t rc = cb + 0x023fffffu + ((cb >> 23) & 1u);
                    const uint32_t E = y > 0.125f ? (rc >> 23) & 7u : 0u;
                    packed |= ((sign >> 28) | E) << (4 * j);
                }
            }
        }
        c[0] = packed;
    }
}

// Decode 4 E3M0 nibbles / 4 E4M3 bytes under the block scale.
__device__ __forceinline__ void decode_e3m0(uint32_t c0, float scale, float (&dq)[kVec])
{
#pragma unroll
    for (int j = 0; j < kVec; ++j) {
        const uint32_t nib = (c0 >> (4 * j)) & 15u;
        const uint32_t E = nib & 7u;
        const float val = E ? u2f((E + 124u) << 23) : 0.0f;
        dq[j] = u2f(((nib & 8u) << 28) | f2u(val * scale));
    }
}
// EXACT = false: the conversion instruction alone, which reads the byte values 0x7f / 0xff as
// NaN; the caller then repeats the decode with EXACT = true wherever a NaN shows up in the sum.
template <bool EXACT>
__device__ __forceinline__ void decode_e4m3(uint32_t c0, float scale, float (&dq)[kVec])
{
    // codes 0x7f / 0xff never come out of the encoder; read as a number (480) like every other
    // code rather than as the NaN the conversion instruction makes of them
    if (EXACT && (((c0 & 0x7f7f7f7fu) + 0x01010101u) & 0x80808080u)) {
#pragma unroll
        for (int j = 0; j < kVec; ++j) {
            const uint32_t byte = (c0 >> (8 * j)) & 255u;
            const uint32_t mag = byte & 0x7fu;
            const float val = mag >= 8u ? u2f((mag + 960u) << 20) : (float)mag * 0.001953125f;
            dq[j] = u2f(((byte & 0x80u) << 24) | f2u(val * scale));
        }
    } else {
        const f32x2_t lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)c0, false);
        const f32x2_t hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)c0, true);
        dq[0] = lo.x * scale; dq[1] = lo.y * scale; dq[2] = hi.x * scale; dq[3] = hi.y * scale;
    }
}

// ------------------------------------------------------------------ tile I/O policies
// The arithmetic is written once against an I/O policy that moves a lane's 4 elements
// of row `row` of each array.
//   TileIO     a whole, 16-byte aligned tile: buffer loads / stores through one resource
//              per array (scalar base, 32-bit lane offset) with explicit cache policy
//   TileIOT<false>  a whole tile whose model arrays start at any element (a run behind a
//              parameter group of odd length): the same lane layout through plain vector
//              loads / stores of element alignment; the message arrays as in TileIO
//   GuardedIO  any alignment, any tail: per-element global loads / stores under a
//              per-row count of valid elements

template <bool ALIGNED, int ROWS>
struct TileIOT {
    static constexpr int kTile = ROWS * kRow;   // parameters of the tile
    const Args& a;
    uint64_t t0;      // tile's first element in the flat arrays (workgroup uniform)
    uint64_t tb;      // tile's first element in the message arrays (a multiple of 512)
    uint32_t lane;
    uint32_t sidx;    // whole-span scale: index of the run's scale word
    uint64_t s0;      // tile's first element in g / mom (= t0 unless the state is staged)

    // bit pattern of the span's absolute maximum (whole-span scale)
    __device__ __forceinline__ uint32_t span_amax(uint32_t m) const
    {
        return reinterpret_cast<const uint32_t*>(a.scales[m])[sidx];
    }
    template <int FMT> __device__ __forceinline__ float load_scale(uint32_t m, int row) const
    {
        if constexpr (is_span_scaled(FMT)) {
            return block_scale_from_exponent<FMT>(span_amax(m) >> 23).scale;
        } else {
            constexpr int B = block_elems(FMT);
            const uint32_t sb = __builtin_amdgcn_raw_buffer_load_b8(
                rsrc(a.scales[m] + tb / B, kTile / B), (int)(row * (kRow / B) + lane / (B / kVec)), 0, kAuxScale);
            return scale_from_byte(sb);
        }
    }
    template <int FMT> __device__ __forceinline__ void store_scale(uint32_t m, int row, uint32_t sb) const
    {
        if constexpr (!is_span_scaled(FMT)) {
            constexpr int B = block_elems(FMT);
            if ((lane % (B / kVec)) == 0u)
                __builtin_amdgcn_raw_buffer_store_b8((uint8_t)sb, rsrc(a.scales[m] + tb / B, kTile / B),
                                                     (int)(row * (kRow / B) + lane / (B / kVec)), 0, kAuxScale);
        }
    }
    // p = address of the tile's first element in the array
    __device__ __forceinline__ void ld_f32(const float* p, int row, float (&v)[kVec]) const
    {
        const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(rsrc(p, kTile * 4),
                                                              (int)(row * kRow * 4 + lane * 16), 0, kAuxLoad);
        v[0] = u2f(x.x); v[1] = u2f(x.y); v[2] = u2f(x.z); v[3] = u2f(x.w);
    }
    __device__ __forceinline__ void st_f32(float* p, int row, const float (&v)[kVec]) const
    {
        const u32x4 x = {f2u(v[0]), f2u(v[1]), f2u(v[2]), f2u(v[3])};
        __builtin_amdgcn_raw_buffer_store_b128(x, rsrc(p, kTile * 4), (int)(row * kRow * 4 + lane * 16), 0,
                                               kAuxStore);
    }
    __device__ __forceinline__ void ld_bf16(const uint16_t* p, int row, uint32_t (&u)[2]) const
    {
        const u32x2 x = __builtin_amdgcn_raw_buffer_load_b64(rsrc(p, kTile * 2),
                                                             (int)(row * kRow * 2 + lane * 8), 0, kAuxLoad);
        u[0] = x.x; u[1] = x.y;
    }
    __device__ __forceinline__ void st_bf16(uint16_t* p, int row, const uint32_t (&u)[2]) const
    {
        const u32x2 x = {u[0], u[1]};
        __builtin_amdgcn_raw_buffer_store_b64(x, rsrc(p, kTile * 2), (int)(row * kRow * 2 + lane * 8), 0,
                                              kAuxStore);
    }

    // the model arrays: the buffer path above when the tile is 16-byte aligned in all of them,
    // element-aligned vectors (non-temporal as well) otherwise
    __device__ __forceinline__ void model_ld_f32(const float* p, int row, float (&v)[kVec]) const
    {
        if constexpr (ALIGNED) {
            ld_f32(p, row, v);
        } else {
            const f32x4_elem x =
                __builtin_nontemporal_load(reinterpret_cast<const f32x4_elem*>(p + row * kRow + lane * kVec));
            v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
        }
    }
    __device__ __forceinline__ void model_st_f32(float* p, int row, const float (&v)[kVec]) const
    {
        if constexpr (ALIGNED) {
            st_f32(p, row, v);
        } else {
            const f32x4_elem x = {v[0], v[1], v[2], v[3]};
            __builtin_nontemporal_store(x, reinterpret_cast<f32x4_elem*>(p + row * kRow + lane * kVec));
        }
    }
    __device__ __forceinline__ void model_ld_bf16(const uint16_t* p, int row, uint32_t (&u)[2]) const
    {
        if constexpr (ALIGNED) {
            ld_bf16(p, row, u);
        } else {
            const u32x2_elem x =
                __builtin_nontemporal_load(reinterpret_cast<const u32x2_elem*>(p + row * kRow + lane * kVec));
            u[0] = x.x; u[1] = x.y;
        }
    }
    __device__ __forceinline__ void model_st_bf16(uint16_t* p, int row, const uint32_t (&u)[2]) const
    {
        if constexpr (ALIGNED) {
            st_bf16(p, row, u);
        } else {
            const u32x2_elem x = {u[0], u[1]};
            __builtin_nontemporal_store(x, reinterpret_cast<u32x2_elem*>(p + row * kRow + lane * kVec));
        }
    }
    __device__ __forceinline__ void load_g(int row, float (&v)[kVec]) const { model_ld_f32(a.g + s0, row, v); }
    __device__ __forceinline__ void load_mom(int row, float (&v)[kVec]) const { model_ld_f32(a.mom + s0, row, v); }
    __device__ __forceinline__ void store_g(int row, const float (&v)[kVec]) const { model_st_f32(a.g + s0, row, v); }
    __device__ __forceinline__ void store_mom(int row, const float (&v)[kVec]) const { model_st_f32(a.mom + s0, row, v); }
    __device__ __forceinline__ void load_ws(uint32_t m, int row, uint32_t (&u)[2]) const { model_ld_bf16(a.w_send[m] + t0, row, u); }
    __device__ __forceinline__ void load_wn(uint32_t m, int row, uint32_t (&u)[2]) const { model_ld_bf16(a.w_now[m] + t0, row, u); }
    __device__ __forceinline__ void store_wn(uint32_t m, int row, const uint32_t (&u)[2]) const { model_st_bf16(a.w_now[m] + t0, row, u); }

    // E4M3 only: with EXACT = false the two byte values the encoder never writes decode to NaN
    static constexpr bool kHasInexactDecode = true;
    // whole tiles: a run-time replica count is taken in groups whose loads are issued together
    static constexpr bool kGroupReplicas = true;
    template <int FMT, bool EXACT = true>
    __device__ __forceinline__ void load_message(uint32_t m, int row, float (&dq)[kVec]) const
    {
        const uint8_t* codes = a.codes[m];
        if constexpr (FMT == SDL_FMT_FP32) {
            ld_f32(reinterpret_cast<const float*>(codes) + tb, row, dq);
        } else if constexpr (FMT == SDL_FMT_BF16) {
            uint32_t u[2];
            ld_bf16(reinterpret_cast<const uint16_t*>(codes) + tb, row, u);
            unpack_bf16(u, dq);
        } else {
            const float scale = load_scale<FMT>(m, row);
            if constexpr (is_e3m0(FMT)) {
                const uint32_t c0 = __builtin_amdgcn_raw_buffer_load_b16(rsrc(codes + tb / 2, kTile / 2),
                                                                         (int)(row * (kRow / 2) + lane * 2), 0,
                                                                         kAuxLoad);
                decode_e3m0(c0, scale, dq);
            } else {
                const uint32_t c0 = __builtin_amdgcn_raw_buffer_load_b32(rsrc(codes + tb, kTile),
                                                                         (int)(row * kRow + lane * 4), 0, kAuxLoad);
                decode_e4m3<EXACT>(c0, scale, dq);
            }
        }
    }
    template <int FMT>
    __device__ __forceinline__ void store_message(uint32_t m, int row, const uint32_t (&c)[kVec], uint32_t sb) const
    {
        uint8_t* codes = a.codes[m];
        if constexpr (FMT == SDL_FMT_FP32) {
            const u32x4 x = {c[0], c[1], c[2], c[3]};
            __builtin_amdgcn_raw_buffer_store_b128(x, rsrc(codes + tb * 4, kTile * 4),
                                                   (int)(row * kRow * 4 + lane * 16), 0, kAuxStore);
        } else if constexpr (FMT == SDL_FMT_BF16) {
            const u32x2 x = {c[0], c[1]};
            __builtin_amdgcn_raw_buffer_store_b64(x, rsrc(codes + tb * 2, kTile * 2),
                                                  (int)(row * kRow * 2 + lane * 8), 0, kAuxStore);
        } else {
            store_scale<FMT>(m, row, sb);
            if constexpr (is_e3m0(FMT)) {
                __builtin_amdgcn_raw_buffer_store_b16((uint16_t)c[0], rsrc(codes + tb / 2, kTile / 2),
                                                      (int)(row * (kRow / 2) + lane * 2), 0, kAuxStore);
            } else {
                __builtin_amdgcn_raw_buffer_store_b32(c[0], rsrc(codes + tb, kTile), (int)(row * kRow + lane * 4), 0,
                                                      kAuxStore);
            }
        }
    }
};

struct GuardedIO {
    const Args& a;
    uint64_t t0;           // tile's first element in the flat arrays
    uint64_t tb;           // tile's first element counted from the run start
    uint64_t mb;           // tile's first element in the message arrays
    uint64_t run_n;        // elements of the run
    uint32_t lane;
    uint32_t sidx;         // whole-span scale: index of the run's scale word
    uint64_t s0;           // tile's first element in g / mom (= t0 unless the state is staged)

    __device__ __forceinline__ uint32_t span_amax(uint32_t m) const
    {
        return reinterpret_cast<const uint32_t*>(a.scales[m])[sidx];
    }

    // lane's first element of a row, counted from the run start, and how many of its 4 exist
    __device__ __forceinline__ uint64_t first(int row) const { return tb + (uint64_t)(row * kRow) + lane * kVec; }
    __device__ __forceinline__ int valid(int row) const
    {
        const uint64_t b = first(row);
        return b >= run_n ? 0 : (run_n - b >= (uint64_t)kVec ? kVec : (int)(run_n - b));
    }
    __device__ __forceinline__ uint64_t flat(int row) const { return t0 + (uint64_t)(row * kRow) + lane * kVec; }
    __device__ __forceinline__ uint64_t msg(int row) const { return mb + (uint64_t)(row * kRow) + lane * kVec; }
    __device__ __forceinline__ uint64_t state(int row) const { return s0 + (uint64_t)(row * kRow) + lane * kVec; }

    __device__ __forceinline__ void ld_f32(const float* p, int n, float (&v)[kVec]) const
    {
#pragma unroll
        for (int j = 0; j < kVec; ++j) v[j] = j < n ? p[j] : 0.0f;
    }
    __device__ __forceinline__ void st_f32(float* p, int n, const float (&v)[kVec]) const
    {
#pragma unroll
        for (int j = 0; j < kVec; ++j)
            if (j < n) p[j] = v[j];
    }
    __device__ __forceinline__ void ld_bf16(const uint16_t* p, int n, uint32_t (&u)[2]) const
    {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const uint32_t lo = 2 * k < n ? p[2 * k] : 0u;
            const uint32_t hi = 2 * k + 1 < n ? p[2 * k + 1] : 0u;
            u[k] = lo | (hi << 16);
        }
    }
    __device__ __forceinline__ void st_bf16(uint16_t* p, int n, const uint32_t (&u)[2]) const
    {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            if (2 * k < n) p[2 * k] = (uint16_t)(u[k] & 0xffffu);
            if (2 * k + 1 < n) p[2 * k + 1] = (uint16_t)(u[k] >> 16);
        }
    }

    __device__ __forceinline__ void load_g(int row, float (&v)[kVec]) const { ld_f32(a.g + state(row), valid(row), v); }
    __device__ __forceinline__ void load_mom(int row, float (&v)[kVec]) const { ld_f32(a.mom + state(row), valid(row), v); }
    __device__ __forceinline__ void store_g(int row, const float (&v)[kVec]) const { st_f32(a.g + state(row), valid(row), v); }
    __device__ __forceinline__ void store_mom(int row, const float (&v)[kVec]) const { st_f32(a.mom + state(row), valid(row), v); }
    __device__ __forceinline__ void load_ws(uint32_t m, int row, uint32_t (&u)[2]) const { ld_bf16(a.w_send[m] + flat(row), valid(row), u); }
    __device__ __forceinline__ void load_wn(uint32_t m, int row, uint32_t (&u)[2]) const { ld_bf16(a.w_now[m] + flat(row), valid(row), u); }
    __device__ __forceinline__ void store_wn(uint32_t m, int row, const uint32_t (&u)[2]) const { st_bf16(a.w_now[m] + flat(row), valid(row), u); }

    static constexpr bool kHasInexactDecode = false;
    static constexpr bool kGroupReplicas = false;    // ragged tails: one replica at a time, small code
    template <int FMT, bool EXACT = true>
    __device__ __forceinline__ void load_message(uint32_t m, int row, float (&dq)[kVec]) const
    {
        const uint8_t* codes = a.codes[m];
        const uint64_t b = msg(row);
        const int n = valid(row);
        if constexpr (FMT == SDL_FMT_FP32) {
            ld_f32(reinterpret_cast<const float*>(codes) + b, n, dq);
        } else if constexpr (FMT == SDL_FMT_BF16) {
            uint32_t u[2];
            ld_bf16(reinterpret_cast<const uint16_t*>(codes) + b, n, u);
            unpack_bf16(u, dq);
        } else {
            float scale;
            if constexpr (is_span_scaled(FMT)) scale = block_scale_from_exponent<FMT>(span_amax(m) >> 23).scale;
            else scale = scale_from_byte(n > 0 ? a.scales[m][b / block_elems(FMT)] : 127u);
            uint32_t c0 = 0;
            if constexpr (is_e3m0(FMT)) {
#pragma unroll
                for (int k = 0; k < 2; ++k)
                    if (2 * k < n) c0 |= (uint32_t)codes[b / 2 + k] << (8 * k);
                decode_e3m0(c0, scale, dq);
            } else {
#pragma unroll
                for (int j = 0; j < kVec; ++j)
                    if (j < n) c0 |= (uint32_t)codes[b + j] << (8 * j);
                decode_e4m3<true>(c0, scale, dq);
            }
        }
    }
    template <int FMT>
    __device__ __forceinline__ void store_message(uint32_t m, int row, const uint32_t (&c)[kVec], uint32_t sb) const
    {
        uint8_t* codes = a.codes[m];
        const uint64_t b = msg(row);
        const int n = valid(row);
        if constexpr (FMT == SDL_FMT_FP32) {
            float v[kVec];
#pragma unroll
            for (int j = 0; j < kVec; ++j) v[j] = u2f(c[j]);
            st_f32(reinterpret_cast<float*>(codes) + b, n, v);
        } else if constexpr (FMT == SDL_FMT_BF16) {
            const uint32_t u[2] = {c[0], c[1]};
            st_bf16(reinterpret_cast<uint16_t*>(codes) + b, n, u);
        } else {
            if constexpr (!is_span_scaled(FMT)) {
                constexpr int B = block_elems(FMT);
                if ((lane % (B / kVec)) == 0u && n > 0) a.scales[m][b / B] = (uint8_t)sb;
            }
            if constexpr (is_e3m0(FMT)) {
                // elements beyond the end are zero outer gradients: their nibbles are 0
#pragma unroll
                for (int k = 0; k < 2; ++k)
                    if (2 * k < n) codes[b / 2 + k] = (uint8_t)(c[0] >> (8 * k));
            } else {
#pragma unroll
                for (int j = 0; j < kVec; ++j)
                    if (j < n) codes[b + j] = (uint8_t)(c[0] >> (8 * j));
            }
        }
    }
};

// ------------------------------------------------------------------ the arithmetic of one lane
// MT > 0: number of replicas known at compile time; the replicas' words are loaded up
// front so that many loads are in flight.  MT == 0: any M at run time, taken in groups of four,
// two and one replicas whose loads are issued together (one replica at a time costs 6-8 %).

// One replica's contribution to the sum of one row: its message decoded (receive side), or its
// outer gradient encoded (send side and fused; ws = the replica's words at the send step).
template <int MODE, int FMT, bool EMIT, class IO>
__device__ __forceinline__ void add_replica(const IO& io, uint32_t m, int r, const uint32_t (&ws)[2],
                                            const float (&g)[kVec], float (&acc)[kVec])
{
    float dq[kVec];
    if constexpr (MODE == kReduce || MODE == kReceive) {
        io.template load_message<FMT, !(FMT == SDL_FMT_E4M3 && IO::kHasInexactDecode)>(m, r, dq);
    } else {
        float w[kVec], d[kVec];
        uint32_t c[kVec], sb;
        unpack_bf16(ws, w);
#pragma unroll
        for (int j = 0; j < kVec; ++j) d[j] = g[j] - w[j];
        constexpr bool want = MODE == kQuantize || EMIT;
        uint32_t samax = 0;
        if constexpr (is_span_scaled(FMT)) samax = io.span_amax(m);
        encode<FMT>(d, dq, c, sb, want, samax);
        if constexpr (want) io.template store_message<FMT>(m, r, c, sb);
    }
#pragma unroll
    for (int j = 0; j < kVec; ++j) acc[j] = acc[j] + dq[j];
}

// G replicas starting at m0, in ascending order, their loads issued before the first is consumed.
template <int MODE, int FMT, bool EMIT, int kRows, int G, class IO>
__device__ __forceinline__ void add_replica_group(const IO& io, uint32_t m0, const float (&g)[kRows][kVec],
                                                  float (&acc)[kRows][kVec])
{
    uint32_t ws[G][kRows][2] = {};
    if constexpr (MODE == kQuantize || MODE == kFused) {
#pragma unroll
        for (int k = 0; k < G; ++k)
#pragma unroll
            for (int r = 0; r < kRows; ++r) io.load_ws(m0 + k, r, ws[k][r]);
    }
#pragma unroll
    for (int k = 0; k < G; ++k)
#pragma unroll
        for (int r = 0; r < kRows; ++r) add_replica<MODE, FMT, EMIT>(io, m0 + k, r, ws[k][r], g[r], acc[r]);
}

// alpha-merge of the new global parameters into one row of one replica (wn = its words now).
template <class IO>
__device__ __forceinline__ void merge_replica(const Args& a, const IO& io, uint32_t m, int r, const uint32_t (&wn)[2],
                                              const float (&g)[kVec])
{
    float w[kVec];
    unpack_bf16(wn, w);
    uint32_t out[2];
#pragma unroll
    for (int k = 0; k < 2; ++k)
        out[k] = bf16_pack(a.alpha * w[2 * k] + a.one_minus_alpha * g[2 * k],
                           a.alpha * w[2 * k + 1] + a.one_minus_alpha * g[2 * k + 1]);
    io.store_wn(m, r, out);
}

template <int kRows, int G, class IO>
__device__ __forceinline__ void merge_replica_group(const Args& a, const IO& io, uint32_t m0, const float (&g)[kRows][kVec])
{
    uint32_t wn[G][kRows][2];
#pragma unroll
    for (int k = 0; k < G; ++k)
#pragma unroll
        for (int r = 0; r < kRows; ++r) io.load_wn(m0 + k, r, wn[k][r]);
#pragma unroll
    for (int k = 0; k < G; ++k)
#pragma unroll
        for (int r = 0; r < kRows; ++r) merge_replica(a, io, m0 + k, r, wn[k][r], g[r]);
}

// ALIASED: w_send[m] and w_now[m] are the same array (no overlap delay).  EMIT: the fused
// kernel also writes the messages.
template <int MODE, int FMT, int MT, bool ALIASED, bool EMIT, int kRows, class IO>
__device__ __forceinline__ void process(const Args& a, const IO& io)
{
    const uint32_t M = MT > 0 ? (uint32_t)MT : a.M;
    constexpr int MU = MT > 0 ? MT : 1;

    float g[kRows][kVec], mom[kRows][kVec], acc[kRows][kVec];
    uint32_t ws[MU][kRows][2] = {}, wn[MU][kRows][2];

    // ---- loads that do not depend on anything
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        io.load_g(r, g[r]);
        if constexpr (MODE == kReduce || MODE == kFused || MODE == kReceive) io.load_mom(r, mom[r]);
    }
    if constexpr (MT > 0) {
        if constexpr (MODE == kQuantize || MODE == kFused) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int r = 0; r < kRows; ++r) io.load_ws(m, r, ws[m][r]);
        }
        if constexpr (MODE == kMerge || MODE == kReceive) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int r = 0; r < kRows; ++r) io.load_wn(m, r, wn[m][r]);
        }
        if constexpr (MODE == kFused && !ALIASED) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int r = 0; r < kRows; ++r) io.load_wn(m, r, wn[m][r]);
        }
    }

    // ---- outer gradients, messages, fp32 sum over replicas in ascending order
    if constexpr (MODE != kMerge) {
#pragma unroll
        for (int r = 0; r < kRows; ++r)
#pragma unroll
            for (int j = 0; j < kVec; ++j) acc[r][j] = 0.0f;
        if constexpr (MT > 0) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int r = 0; r < kRows; ++r) add_replica<MODE, FMT, EMIT>(io, (uint32_t)m, r, ws[m][r], g[r], acc[r]);
        } else {
            uint32_t m = 0;
            if constexpr (IO::kGroupReplicas) {
                for (; m + 4u <= M; m += 4u) add_replica_group<MODE, FMT, EMIT, kRows, 4>(io, m, g, acc);
                if (M - m >= 2u) { add_replica_group<MODE, FMT, EMIT, kRows, 2>(io, m, g, acc); m += 2u; }
            }
            for (; m < M; ++m) add_replica_group<MODE, FMT, EMIT, kRows, 1>(io, m, g, acc);
        }
    }

    // E4M3 messages were decoded by the conversion instruction alone.  It turns the two byte
    // values that the encoder never writes into NaN, which survives the sum: where any lane of
    // the wavefront sees a NaN (rare: a foreign message, or a block that really holds NaN), the
    // row is decoded again, exactly, from the messages in memory.
    if constexpr ((MODE == kReduce || MODE == kReceive) && FMT == SDL_FMT_E4M3 && IO::kHasInexactDecode) {
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const float t = (acc[r][0] + acc[r][1]) + (acc[r][2] + acc[r][3]);
            if (__builtin_amdgcn_ballot_w64(t != t) != 0ull) {
#pragma unroll
                for (int j = 0; j < kVec; ++j) acc[r][j] = 0.0f;
                for (uint32_t m = 0; m < M; ++m) {
                    float dq[kVec];
                    io.template load_message<FMT, true>(m, r, dq);
#pragma unroll
                    for (int j = 0; j < kVec; ++j) acc[r][j] = acc[r][j] + dq[j];
                }
            }
        }
    }

    // ---- mean and Nesterov outer step
    if constexpr (MODE == kReduce || MODE == kFused || MODE == kReceive) {
        const float fm = (float)M;
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                const float dbar = acc[r][j] / fm;
                const float m_new = a.mu * mom[r][j] + dbar;
                const float look = dbar + a.mu * m_new;
                mom[r][j] = m_new;
                g[r][j] = g[r][j] - a.lr * look;
            }
            io.store_g(r, g[r]);
            io.store_mom(r, mom[r]);
        }
    }

    // ---- alpha-merge into every replica
    if constexpr (MODE == kMerge || MODE == kFused || MODE == kReceive) {
        if constexpr (MT > 0) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
#pragma unroll
                for (int r = 0; r < kRows; ++r) {
                    if constexpr (MODE == kFused && ALIASED) {
                        // same words as at the send step; hide that from the optimizer so that it
                        // re-expands the two packed registers instead of keeping four floats alive
                        uint32_t u[2] = {ws[m][r][0], ws[m][r][1]};
                        asm volatile("" : "+v"(u[0]), "+v"(u[1]));
                        merge_replica(a, io, (uint32_t)m, r, u, g[r]);
                    } else {
                        merge_replica(a, io, (uint32_t)m, r, wn[m][r], g[r]);
                    }
                }
            }
        } else {
            // (with w_send aliasing w_now these are the same words as at the send step, read again)
            uint32_t m = 0;
            if constexpr (IO::kGroupReplicas) {
                for (; m + 4u <= M; m += 4u) merge_replica_group<kRows, 4>(a, io, m, g);
                if (M - m >= 2u) { merge_replica_group<kRows, 2>(a, io, m, g); m += 2u; }
            }
            for (; m < M; ++m) merge_replica_group<kRows, 1>(a, io, m, g);
        }
    }
}

// ------------------------------------------------------------------ the kernel

template <int MODE, int FMT, int MT, bool ALIASED, bool EMIT>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(kWavesPerEu)))
void sdl_kernel(const Args a)
{
    // which run does this workgroup work on (uniform scan of at most kMaxRuns entries)
    const uint32_t wg = blockIdx.x;
    uint32_t r = 0;
    for (uint32_t i = 1; i < a.n_runs; ++i)
        if (wg >= a.runs[i].first_wg) r = i;
    const uint64_t run_off = a.runs[r].offset;
    const uint64_t run_n = a.runs[r].numel;
    constexpr int ROWS = tile_rows(MODE, MT, FMT);
    constexpr int kTile = ROWS * kRow;
    const uint64_t tile = (uint64_t)(wg - a.runs[r].first_wg) * kTile;   // first element of the tile in the run
    const bool whole = run_n - tile >= (uint64_t)kTile;
    if (whole && a.runs[r].path == kPathBuffer) {
        const TileIOT<true, ROWS> io{a, run_off + tile, a.runs[r].msg + tile, threadIdx.x, a.runs[r].sidx,
                                     a.staged ? a.runs[r].soff + tile : run_off + tile};
        process<MODE, FMT, MT, ALIASED, EMIT, ROWS>(a, io);
    } else if (whole && a.runs[r].path == kPathVector) {
        const TileIOT<false, ROWS> io{a, run_off + tile, a.runs[r].msg + tile, threadIdx.x, a.runs[r].sidx,
                                      a.staged ? a.runs[r].soff + tile : run_off + tile};
        process<MODE, FMT, MT, ALIASED, EMIT, ROWS>(a, io);
    } else {
        const GuardedIO io{a, run_off + tile, tile, a.runs[r].msg + tile, run_n, threadIdx.x, a.runs[r].sidx,
                           a.staged ? a.runs[r].soff + tile : run_off + tile};
        process<MODE, FMT, 0, ALIASED, EMIT, ROWS>(a, io);
    }
}

// Pre-pass of the whole-span scale: the absolute maximum of every replica's outer gradient over
// each run, folded into the run's scale word with an integer atomic maximum (the words hold fp32
// bit patterns of non-negative values, which order like the values).  It has an argument block of
// its own, so that one launch covers up to 64 runs (a whole fragment as a rule).  A fixed number of
// wavefronts is shared out among the runs; wavefront k of a run walks the run's tiles k, k + G, ...
// with 8 consecutive parameters per lane (128-bit loads, the next tile's loads issued before the
// current tile is consumed), keeps the running maxima in registers, and the scale words are touched
// once at the very end -- one atomic per workgroup (4 wavefronts) and replica instead of one per
// tile: atomics on one cache line are served one after the other, and the scale words of a launch
// share a few lines.
constexpr int kAbsmaxMaxRuns = 64;
constexpr int kAbsmaxWaves = 4;       // wavefronts per workgroup (50 to 113 VGPRs)
constexpr int kAbsmaxTile = 512;      // parameters a wavefront takes at a time: 8 per lane

struct AbsmaxRun {
    uint64_t offset;     // first element of the run in the flat arrays
    uint64_t numel;
    uint64_t soff;       // where the run starts in staged g (staged state only)
    uint32_t vec;        // g and every w_send are 16-byte aligned at the run start
    uint32_t sidx;       // index of the run's scale word
    uint32_t first;      // first workgroup of the launch that works on this run
    uint32_t G;          // workgroups of this run (>= 1)
};

struct AbsmaxArgs {
    const float* g;
    const uint16_t* w_send[SDL_MAX_WORKERS];
    uint8_t* scales[SDL_MAX_WORKERS];
    uint32_t M;
    uint32_t m0;         // first replica handled by this launch
    uint32_t staged;
    uint32_t n_runs;
    AbsmaxRun runs[kAbsmaxMaxRuns];
};

template <int MB>
struct AbsmaxTile {
    u32x4 g0, g1;
    u32x4 w[MB];
};

template <int MB>
__device__ __forceinline__ void absmax_load(AbsmaxTile<MB>& t, const AbsmaxArgs& a, uint64_t ge, uint64_t we,
                                            uint32_t valid, bool fast, uint32_t lane)
{
    if (fast && valid == (uint32_t)kAbsmaxTile) {
        const __amdgpu_buffer_rsrc_t rg = rsrc(a.g + ge, kAbsmaxTile * 4);
        t.g0 = __builtin_amdgcn_raw_buffer_load_b128(rg, (int)(lane * 32), 0, kAuxLoad);
        t.g1 = __builtin_amdgcn_raw_buffer_load_b128(rg, (int)(lane * 32 + 16), 0, kAuxLoad);
#pragma unroll
        for (int m = 0; m < MB; ++m)
            t.w[m] = __builtin_amdgcn_raw_buffer_load_b128(rsrc(a.w_send[a.m0 + m] + we, kAbsmaxTile * 2),
                                                           (int)(lane * 16), 0, kAuxLoad);
    } else if (valid == (uint32_t)kAbsmaxTile) {
        // a whole tile of a run that starts at some other element: vectors of element alignment
        const u32x4_f32elem* pg = reinterpret_cast<const u32x4_f32elem*>(a.g + ge + lane * 8);
        t.g0 = __builtin_nontemporal_load(pg);
        t.g1 = __builtin_nontemporal_load(pg + 1);
#pragma unroll
        for (int m = 0; m < MB; ++m)
            t.w[m] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4_bf16elem*>(a.w_send[a.m0 + m] + we + lane * 8));
    } else {
        // ragged tail: element by element under the buffer range check, which returns 0 past the
        // end (g = 0 and w = 0 give an outer gradient of 0: no effect on a maximum)
        const __amdgpu_buffer_rsrc_t rg = rsrc(a.g + ge, valid * 4);
        uint32_t x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = __builtin_amdgcn_raw_buffer_load_b32(rg, (int)((lane * 8 + j) * 4), 0, 0);
        t.g0 = u32x4{x[0], x[1], x[2], x[3]};
        t.g1 = u32x4{x[4], x[5], x[6], x[7]};
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            const __amdgpu_buffer_rsrc_t rw = rsrc(a.w_send[a.m0 + m] + we, valid * 2);
            uint32_t h[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                h[j] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rw, (int)((lane * 8 + j) * 2), 0, 0) & 0xffffu;
            t.w[m] = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        }
    }
}

template <int MB>
__global__ __launch_bounds__(kWave * kAbsmaxWaves) void sdl_span_absmax_kernel(const AbsmaxArgs a)
{
    __shared__ uint32_t wave_max[kAbsmaxWaves][MB];
    // the wavefront's number is the same in all of its lanes: say so, or every address derived from it
    // is treated as different per lane and every buffer access is wrapped in a loop over lanes
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    uint32_t r = 0;
    for (uint32_t i = 1; i < a.n_runs; ++i)
        if (blockIdx.x >= a.runs[i].first) r = i;
    const AbsmaxRun run = a.runs[r];
    // every wavefront of the run's workgroups walks its own tiles: k, k + G, ...; neighbouring
    // tiles go to neighbouring workgroups (which the dispatcher deals to different XCDs), not to
    // the wavefronts of one workgroup
    const uint32_t k = wave * run.G + (blockIdx.x - run.first), G = run.G * kAbsmaxWaves;
    const uint64_t n_tiles = (run.numel + kAbsmaxTile - 1) / kAbsmaxTile;
    const bool fast = run.vec != 0u;
    auto valid_of = [&](uint64_t t) -> uint32_t {
        const uint64_t rem = run.numel - t * kAbsmaxTile;
        return rem < (uint64_t)kAbsmaxTile ? (uint32_t)rem : (uint32_t)kAbsmaxTile;
    };
    auto g_elem = [&](uint64_t t) -> uint64_t { return (a.staged ? run.soff : run.offset) + t * kAbsmaxTile; };

    uint32_t amax[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) amax[m] = 0u;

    AbsmaxTile<MB> cur;
    if (k < n_tiles) absmax_load<MB>(cur, a, g_elem(k), run.offset + (uint64_t)k * kAbsmaxTile, valid_of(k), fast, lane);
    for (uint64_t t = k; t < n_tiles; t += G) {
        AbsmaxTile<MB> nxt = cur;
        const uint64_t tn = t + G;
        if (tn < n_tiles) absmax_load<MB>(nxt, a, g_elem(tn), run.offset + tn * kAbsmaxTile, valid_of(tn), fast, lane);
        const uint32_t gb[8] = {cur.g0.x, cur.g0.y, cur.g0.z, cur.g0.w, cur.g1.x, cur.g1.y, cur.g1.z, cur.g1.w};
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            const uint32_t wb[4] = {cur.w[m].x, cur.w[m].y, cur.w[m].z, cur.w[m].w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float d = u2f(gb[j]) - ((j & 1) ? bf16_hi(wb[j / 2]) : bf16_lo(wb[j / 2]));
                const uint32_t mag = f2u(d) & 0x7fffffffu;
                amax[m] = mag > amax[m] ? mag : amax[m];
            }
        }
        cur = nxt;
    }
    // wavefront, then workgroup (all of whose wavefronts work on the same run), then one atomic
    // per workgroup and replica
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const uint32_t v = lanes_max<kWave>(amax[m]);
        if (lane == 0u) wave_max[wave][m] = v;
    }
    __syncthreads();
    if (threadIdx.x < (uint32_t)MB) {
        uint32_t v = 0u;
        for (int w = 0; w < kAbsmaxWaves; ++w) v = wave_max[w][threadIdx.x] > v ? wave_max[w][threadIdx.x] : v;
        // look before the atomic: reads of one cache line are served in parallel, atomics on it one
        // after the other, and by the time most workgroups finish the word already holds a larger value
        uint32_t* word = reinterpret_cast<uint32_t*>(a.scales[a.m0 + threadIdx.x]) + run.sidx;
        if (v > __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            __hip_atomic_fetch_max(word, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Clears the scale words of a pre-pass launch's runs before the maximum is accumulated
// (thread = run * 16 + replica).
__global__ __launch_bounds__(SDL_MAX_WORKERS * kAbsmaxMaxRuns) void sdl_zero_span_scales(const AbsmaxArgs a)
{
    const uint32_t r = threadIdx.x / SDL_MAX_WORKERS, m = threadIdx.x % SDL_MAX_WORKERS;
    if (m < a.M && r < a.n_runs) reinterpret_cast<uint32_t*>(a.scales[m])[a.runs[r].sidx] = 0u;
}

// Streaming yardsticks for the HBM roofline, 16 bytes per lane: a plain copy, and the same copy, a
// read-only pass and a write-only pass with the non-temporal policy the method's kernels use.
constexpr int kCopyThreads = 256;
__global__ __launch_bounds__(kCopyThreads) void sdl_copy_kernel(uint4* __restrict__ dst,
                                                            const uint4* __restrict__ src, uint64_t n16)
{
    const uint64_t i = (uint64_t)blockIdx.x * kCopyThreads + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}
template <int KIND>
__global__ __launch_bounds__(kCopyThreads) void sdl_probe_kernel(u32x4* __restrict__ dst,
                                                             const u32x4* __restrict__ src, uint64_t n16)
{
    const uint64_t i = (uint64_t)blockIdx.x * kCopyThreads + threadIdx.x;
    if (i >= n16) return;
    if constexpr (KIND == SDL_PROBE_COPY_NT) {
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
    } else if constexpr (KIND == SDL_PROBE_READ_NT) {
        // the data has to be used for the load to stay: one word of dst is written if the 16 bytes spell a
        // value that seeded or zeroed buffers never hold
        const u32x4 x = __builtin_nontemporal_load(src + i);
        if ((x.x ^ x.y ^ x.z ^ x.w) == 0x9e3779b9u && x.x == 0x7f4a7c15u) dst[0] = x;
    } else {
        const u32x4 x = {(uint32_t)i, 0u, 0u, 0u};
        __builtin_nontemporal_store(x, dst + i);
    }
}

// ------------------------------------------------------------------ host side

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

size_t code_align(sdl_format_t fmt)
{
    return fmt == SDL_FMT_FP32 ? 4 : fmt == SDL_FMT_BF16 ? 2 : 1;
}
size_t scale_align(sdl_format_t fmt) { return is_span_scaled(fmt) ? 4 : 1; }
// bytes of code per element (x2 for E3M0, which holds half a byte)
size_t code_bytes_at(sdl_format_t fmt, uint64_t elem)
{
    switch (fmt) {
    case SDL_FMT_FP32: return (size_t)elem * 4;
    case SDL_FMT_BF16: return (size_t)elem * 2;
    case SDL_FMT_E4M3: return (size_t)elem;
    default: return (size_t)(elem / 2);
    }
}

// Dynamic LDS requested per workgroup.  The kernels use no LDS; the request only caps how
// many wavefronts share a CU (160 KiB of LDS per CU: 20480 B -> 8, 13653 B -> 12, 10240 B -> 16),
// which is the knob that matters for a streaming kernel: enough loads in flight, not so many
// that the access window in each array grows and DRAM page locality is lost.  Measured on
// MI355X (medians of three runs over 302 M parameters, replica counts 2 / 4 / 8): the kernels
// that write the replicas back want few wavefronts -- fused 12 / 8 / 8 (12 when w_send aliases
// w_now), one-pass receive 12 / 8 / 8, merge 16 / 12 / 8 --, the receive side without the merge
// all / 16 / all (measured again with the arrays in one allocation: 16 cost it 3 % at two replicas),
// and the send side every wavefront it can get.  A single replica: 16 for the fused
// kernel and the one-pass receive, no cap otherwise.
uint32_t lds_cap_bytes(int mode, uint32_t mt, bool aliased)
{
    if (mt == 0) return 0u;
    if (mode == kFused) return mt == 1 ? 10240u : ((aliased || mt == 2) ? 13653u : 20480u);
    if (mode == kReceive) return mt == 1 ? 10240u : (mt == 2 ? 13653u : 20480u);
    if (mode == kMerge) return mt == 1 ? 0u : (mt == 2 ? 10240u : (mt == 4 ? 13653u : 20480u));
    if (mode == kReduce) return mt == 4 ? 10240u : 0u;
    return 0u;
}

template <int MODE, int FMT, bool ALIASED, bool EMIT>
hipError_t launch_m(const Args& a, uint32_t n_wg, hipStream_t s)
{
    const dim3 grid(n_wg), block(kWave);
    const uint32_t mt = variant_mt(MODE, a.M, EMIT);   // the grid was sized for this variant's tile
    const uint32_t lds = lds_cap_bytes(MODE, mt, ALIASED);
    switch (mt) {
    case 1: if constexpr (!EMIT) hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 1, ALIASED, EMIT>), grid, block, lds, s, a); break;
    case 2: if constexpr (!EMIT) hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 2, ALIASED, EMIT>), grid, block, lds, s, a); break;
    case 4: if constexpr (!EMIT) hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 4, ALIASED, EMIT>), grid, block, lds, s, a); break;
    case 8: if constexpr (!EMIT) hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 8, ALIASED, EMIT>), grid, block, lds, s, a); break;
    default: hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 0, ALIASED, EMIT>), grid, block, lds, s, a); break;
    }
    return hipGetLastError();
}

template <int MODE, int FMT>
hipError_t launch_f(const Args& a, uint32_t n_wg, hipStream_t s)
{
    if constexpr (MODE == kFused) {
        if (a.emit) return a.aliased ? launch_m<MODE, FMT, true, true>(a, n_wg, s) : launch_m<MODE, FMT, false, true>(a, n_wg, s);
        return a.aliased ? launch_m<MODE, FMT, true, false>(a, n_wg, s) : launch_m<MODE, FMT, false, false>(a, n_wg, s);
    } else {
        return launch_m<MODE, FMT, false, false>(a, n_wg, s);
    }
}

// Whole-span scale words of a list of runs: cleared, then the maximum of every replica's outer
// gradient over each run.  kAbsmaxGroups wavefronts per launch are shared out among the runs in
// proportion to their tiles (whole workgroups, at least one each); up to 8 replicas per pass over g.
constexpr uint32_t kAbsmaxGroups = 8192;

struct SpanRun { uint64_t offset, numel, soff; bool vec; uint32_t sidx; };

hipError_t launch_span_prepass(const Args& a, const SpanRun* runs, uint32_t n_runs, hipStream_t s)
{
    for (uint32_t r0 = 0; r0 < n_runs; r0 += kAbsmaxMaxRuns) {
        AbsmaxArgs b{};
        b.g = a.g;
        b.M = a.M;
        b.staged = a.staged;
        for (uint32_t m = 0; m < a.M; ++m) { b.w_send[m] = a.w_send[m]; b.scales[m] = a.scales[m]; }
        const uint32_t n = n_runs - r0 < (uint32_t)kAbsmaxMaxRuns ? n_runs - r0 : (uint32_t)kAbsmaxMaxRuns;
        uint64_t total_tiles = 0;
        for (uint32_t r = 0; r < n; ++r) total_tiles += (runs[r0 + r].numel + kAbsmaxTile - 1) / kAbsmaxTile;
        uint32_t next = 0;
        for (uint32_t r = 0; r < n; ++r) {
            const SpanRun& in = runs[r0 + r];
            const uint64_t tiles = (in.numel + kAbsmaxTile - 1) / kAbsmaxTile;
            uint64_t waves = total_tiles ? (tiles * kAbsmaxGroups + total_tiles - 1) / total_tiles : 1;
            if (waves > tiles) waves = tiles;
            uint64_t G = (waves + kAbsmaxWaves - 1) / kAbsmaxWaves;
            if (G < 1) G = 1;
            b.runs[r] = AbsmaxRun{in.offset, in.numel, in.soff, in.vec ? 1u : 0u, in.sidx, next, (uint32_t)G};
            next += (uint32_t)G;
        }
        b.n_runs = n;
        hipLaunchKernelGGL(sdl_zero_span_scales, dim3(1), dim3(SDL_MAX_WORKERS * kAbsmaxMaxRuns), 0, s, b);
        const dim3 grid(next), block(kWave * kAbsmaxWaves);
        for (uint32_t m0 = 0; m0 < a.M;) {
            const uint32_t left = a.M - m0;
            const uint32_t mb = left < 8u ? left : 8u;
            b.m0 = m0;
            switch (mb) {
            case 8: hipLaunchKernelGGL((sdl_span_absmax_kernel<8>), grid, block, 0, s, b); break;
            case 7: hipLaunchKernelGGL((sdl_span_absmax_kernel<7>), grid, block, 0, s, b); break;
            case 6: hipLaunchKernelGGL((sdl_span_absmax_kernel<6>), grid, block, 0, s, b); break;
            case 5: hipLaunchKernelGGL((sdl_span_absmax_kernel<5>), grid, block, 0, s, b); break;
            case 4: hipLaunchKernelGGL((sdl_span_absmax_kernel<4>), grid, block, 0, s, b); break;
            case 3: hipLaunchKernelGGL((sdl_span_absmax_kernel<3>), grid, block, 0, s, b); break;
            case 2: hipLaunchKernelGGL((sdl_span_absmax_kernel<2>), grid, block, 0, s, b); break;
            default: hipLaunchKernelGGL((sdl_span_absmax_kernel<1>), grid, block, 0, s, b); break;
            }
            m0 += mb;
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

template <int MODE>
hipError_t launch(const Args& a, sdl_format_t fmt, uint32_t n_wg, hipStream_t s)
{
    if constexpr (MODE == kMerge) return launch_f<MODE, SDL_FMT_FP32>(a, n_wg, s);
    switch (fmt) {
    case SDL_FMT_FP32: return launch_f<MODE, SDL_FMT_FP32>(a, n_wg, s);
    case SDL_FMT_BF16: return launch_f<MODE, SDL_FMT_BF16>(a, n_wg, s);
    case SDL_FMT_E4M3: return launch_f<MODE, SDL_FMT_E4M3>(a, n_wg, s);
    case SDL_FMT_E3M0_B64: return launch_f<MODE, SDL_FMT_E3M0_B64>(a, n_wg, s);
    case SDL_FMT_E3M0_B128: return launch_f<MODE, SDL_FMT_E3M0_B128>(a, n_wg, s);
    case SDL_FMT_E3M0_SPAN: return launch_f<MODE, SDL_FMT_E3M0_SPAN>(a, n_wg, s);
    case SDL_FMT_E3M0_RN: return launch_f<MODE, SDL_FMT_E3M0_RN>(a, n_wg, s);
    default: return launch_f<MODE, SDL_FMT_E3M0>(a, n_wg, s);
    }
}

bool valid_format(sdl_format_t fmt) { return fmt >= SDL_FMT_FP32 && fmt <= SDL_FMT_E3M0_RN; }

// 16-byte alignment of a call's pointers: model = g, mom and the replicas; msg = codes (scale
// bytes need none).
struct Align16 {
    bool model = true, msg = true;
    TilePath path() const { return !msg ? kPathGuarded : model ? kPathBuffer : kPathVector; }
    Align16 at(bool run_start_aligned) const { return Align16{model && run_start_aligned, msg}; }
};

// Parameters per workgroup of the kernel variant that a call in this mode will run.
uint32_t tile_elems(int mode, const Args& a, sdl_format_t fmt)
{
    return (uint32_t)(tile_rows(mode, (int)variant_mt(mode, a.M, a.emit != 0u), (int)fmt) * kRow);
}

// Fill a.runs from a list of (offset, numel); returns the number of workgroups.
struct RunBuilder {
    Args* a;
    uint64_t tile;       // parameters per workgroup
    uint64_t n_wg = 0;
    RunBuilder(Args* args, uint32_t tile_elems) : a(args), tile(tile_elems) { a->n_runs = 0; }
    bool full() const { return a->n_runs == kMaxRuns; }
    void add(uint64_t offset, uint64_t numel, TilePath path, uint64_t msg = 0, uint32_t sidx = 0, uint64_t soff = 0)
    {
        Run& r = a->runs[a->n_runs++];
        r.offset = offset; r.numel = numel; r.msg = msg; r.soff = soff; r.first_wg = (uint32_t)n_wg;
        r.path = path; r.sidx = sidx; r.pad_ = 0;
        n_wg += (numel + tile - 1) / tile;
    }
};

// The aliasing rule of the interface, checked: an array that a call writes must not overlap any other
// array of the call (w_send[m] being the very same pointer as w_now[m] is the one exception, and then
// only w_now[m] is listed).  model_elems / state_elems: elements of the replicas and of g / mom that the
// call may touch; code_bytes / scale_bytes: size of one replica's message arrays.
template <int MODE>
bool arrays_clash(const Args& a, sdl_format_t fmt, uint64_t model_elems, uint64_t state_elems, size_t code_bytes,
                  size_t scale_bytes)
{
    struct Range { uintptr_t lo, hi; bool written; };
    Range r[2 + 4 * SDL_MAX_WORKERS];
    int n = 0;
    auto add = [&](const void* p, uint64_t bytes, bool written) {
        if (p && bytes) { r[n].lo = reinterpret_cast<uintptr_t>(p); r[n].hi = r[n].lo + bytes; r[n].written = written; ++n; }
    };
    constexpr bool state_written = MODE == kReduce || MODE == kFused || MODE == kReceive;
    add(a.g, state_elems * 4, state_written);
    if constexpr (state_written) add(a.mom, state_elems * 4, true);
    const bool msg_written = MODE == kQuantize || (MODE == kFused && a.emit);
    const bool msg_used = msg_written || MODE == kReduce || MODE == kReceive;
    for (uint32_t m = 0; m < a.M; ++m) {
        if (MODE == kQuantize || (MODE == kFused && !a.aliased)) add(a.w_send[m], model_elems * 2, false);
        if (MODE == kMerge || MODE == kFused || MODE == kReceive) add(a.w_now[m], model_elems * 2, true);
        if (msg_used) add(a.codes[m], code_bytes, msg_written);
        if (msg_used || (MODE == kFused && is_span_scaled(fmt))) add(a.scales[m], scale_bytes, msg_written || MODE == kFused);
    }
    for (int i = 0; i < n; ++i)
        for (int j = i + 1; j < n; ++j)
            if ((r[i].written || r[j].written) && r[i].lo < r[j].hi && r[j].lo < r[i].hi) return true;
    return false;
}

// One span starting at the given pointers (offset 0).
template <int MODE>
int run_single_span(Args& a, uint64_t n, sdl_format_t fmt, Align16 al, void* stream)
{
    if (n == 0) return SDL_OK;
    const uint32_t tile = tile_elems(MODE, a, fmt);
    if (n > (uint64_t)0x7fffffff * (uint64_t)tile) return SDL_ERR_UNSUPPORTED;
    {
        size_t cb = 0, sb = 0;
        sdl_exchange_bytes(fmt, n, &cb, &sb);
        if (arrays_clash<MODE>(a, fmt, n, n, cb, sb)) return SDL_ERR_INVALID_ARG;
    }
    RunBuilder rb(&a, tile);
    rb.add(0, n, al.path());
    if constexpr (MODE == kQuantize || MODE == kFused) {
        if (is_span_scaled(fmt)) {
            // whole-span scale: clear the scale word, take the grid-wide maximum, then encode
            const SpanRun one{0, n, 0, al.model, 0};
            if (launch_span_prepass(a, &one, 1, (hipStream_t)stream) != hipSuccess) return SDL_ERR_DEVICE;
        }
    }
    hipError_t e = launch<MODE>(a, fmt, (uint32_t)rb.n_wg, (hipStream_t)stream);
    return e == hipSuccess ? SDL_OK : SDL_ERR_DEVICE;
}

}  // namespace

extern "C" {

int sdl_quantize_outer_grad(const float* g, const void* const* w_send, uint32_t M, uint64_t n,
                            sdl_format_t fmt, void* const* codes, void* const* scales, void* stream)
{
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    const bool scaled = is_scaled(fmt);
    if (n && (!g || !w_send || !codes || (scaled && !scales))) return SDL_ERR_INVALID_ARG;
    if (n == 0) return SDL_OK;
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.g = const_cast<float*>(g);
    a.M = M;
    Align16 al;
    al.model = aligned(g, 16);
    if (!aligned(g, 4)) return SDL_ERR_ALIGNMENT;
    for (uint32_t m = 0; m < M; ++m) {
        if (!w_send[m] || !codes[m] || (scaled && !scales[m])) return SDL_ERR_INVALID_ARG;
        if (!aligned(w_send[m], 2) || !aligned(codes[m], code_align(fmt))) return SDL_ERR_ALIGNMENT;
        if (scaled && !aligned(scales[m], scale_align(fmt))) return SDL_ERR_ALIGNMENT;
        al.model = al.model && aligned(w_send[m], 16);
        al.msg = al.msg && aligned(codes[m], 16);
        a.w_send[m] = static_cast<const uint16_t*>(w_send[m]);
        a.codes[m] = static_cast<uint8_t*>(codes[m]);
        a.scales[m] = scaled ? static_cast<uint8_t*>(scales[m]) : nullptr;
    }
    return run_single_span<kQuantize>(a, n, fmt, al, stream);
}

int sdl_dequant_reduce_nesterov(float* g, float* mom, const void* const* codes,
                                const void* const* scales, uint32_t M, uint64_t n, sdl_format_t fmt,
                                float lr, float mu, void* stream)
{
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    const bool scaled = is_scaled(fmt);
    if (n && (!g || !mom || !codes || (scaled && !scales))) return SDL_ERR_INVALID_ARG;
    if (n == 0) return SDL_OK;
    if (!aligned(g, 4) || !aligned(mom, 4)) return SDL_ERR_ALIGNMENT;
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.g = g; a.mom = mom; a.M = M; a.lr = lr; a.mu = mu;
    Align16 al;
    al.model = aligned(g, 16) && aligned(mom, 16);
    for (uint32_t m = 0; m < M; ++m) {
        if (!codes[m] || (scaled && !scales[m])) return SDL_ERR_INVALID_ARG;
        if (!aligned(codes[m], code_align(fmt))) return SDL_ERR_ALIGNMENT;
        if (scaled && !aligned(scales[m], scale_align(fmt))) return SDL_ERR_ALIGNMENT;
        al.msg = al.msg && aligned(codes[m], 16);
        a.codes[m] = static_cast<uint8_t*>(const_cast<void*>(codes[m]));
        a.scales[m] = scaled ? static_cast<uint8_t*>(const_cast<void*>(scales[m])) : nullptr;
    }
    return run_single_span<kReduce>(a, n, fmt, al, stream);
}

// Argument marshalling shared by the receive-side calls that also merge.
static int fill_receive_args(Args& a, float* g, float* mom, const void* const* codes, const void* const* scales,
                             void* const* w_now, uint32_t M, sdl_format_t fmt, float lr, float mu, float alpha,
                             Align16* al)
{
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    const bool scaled = is_scaled(fmt);
    if (!g || !mom || !codes || !w_now || (scaled && !scales)) return SDL_ERR_INVALID_ARG;
    if (!aligned(g, 4) || !aligned(mom, 4)) return SDL_ERR_ALIGNMENT;
    std::memset(&a, 0, sizeof(a));
    a.g = g; a.mom = mom; a.M = M; a.lr = lr; a.mu = mu; a.alpha = alpha; a.one_minus_alpha = 1.0f - alpha;
    *al = Align16{aligned(g, 16) && aligned(mom, 16), true};
    for (uint32_t m = 0; m < M; ++m) {
        if (!codes[m] || !w_now[m] || (scaled && !scales[m])) return SDL_ERR_INVALID_ARG;
        if (!aligned(codes[m], code_align(fmt)) || !aligned(w_now[m], 2)) return SDL_ERR_ALIGNMENT;
        if (scaled && !aligned(scales[m], scale_align(fmt))) return SDL_ERR_ALIGNMENT;
        al->model = al->model && aligned(w_now[m], 16);
        al->msg = al->msg && aligned(codes[m], 16);
        a.codes[m] = static_cast<uint8_t*>(const_cast<void*>(codes[m]));
        a.scales[m] = scaled ? static_cast<uint8_t*>(const_cast<void*>(scales[m])) : nullptr;
        a.w_now[m] = static_cast<uint16_t*>(w_now[m]);
    }
    return SDL_OK;
}

int sdl_receive_outer_step(float* g, float* mom, const void* const* codes, const void* const* scales,
                           void* const* w_now, uint32_t M, uint64_t n, sdl_format_t fmt, float lr, float mu,
                           float alpha, void* stream)
{
    if (n == 0) return (valid_format(fmt) && M >= 1 && M <= SDL_MAX_WORKERS) ? SDL_OK : SDL_ERR_INVALID_ARG;
    Args a;
    Align16 al;
    int rc = fill_receive_args(a, g, mom, codes, scales, w_now, M, fmt, lr, mu, alpha, &al);
    if (rc != SDL_OK) return rc;
    return run_single_span<kReceive>(a, n, fmt, al, stream);
}

int sdl_merge_overlap(const float* g_new, void* const* w_now, uint32_t M, uint64_t n, float alpha,
                      void* stream)
{
    if (M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    if (n && (!g_new || !w_now)) return SDL_ERR_INVALID_ARG;
    if (n == 0) return SDL_OK;
    if (!aligned(g_new, 4)) return SDL_ERR_ALIGNMENT;
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.g = const_cast<float*>(g_new); a.M = M; a.alpha = alpha; a.one_minus_alpha = 1.0f - alpha;
    Align16 al;
    al.model = aligned(g_new, 16);
    for (uint32_t m = 0; m < M; ++m) {
        if (!w_now[m]) return SDL_ERR_INVALID_ARG;
        if (!aligned(w_now[m], 2)) return SDL_ERR_ALIGNMENT;
        al.model = al.model && aligned(w_now[m], 16);
        a.w_now[m] = static_cast<uint16_t*>(w_now[m]);
    }
    return run_single_span<kMerge>(a, n, SDL_FMT_FP32, al, stream);
}

// Shared argument marshalling of the two fused entry points.
static int fill_fused_args(Args& a, float* g, float* mom, const void* const* w_send, void* const* w_now,
                           uint32_t M, sdl_format_t fmt, float lr, float mu, float alpha, Align16* al)
{
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    if (!g || !mom || !w_send || !w_now) return SDL_ERR_INVALID_ARG;
    if (!aligned(g, 4) || !aligned(mom, 4)) return SDL_ERR_ALIGNMENT;
    std::memset(&a, 0, sizeof(a));
    a.g = g; a.mom = mom; a.M = M; a.lr = lr; a.mu = mu; a.alpha = alpha;
    a.one_minus_alpha = 1.0f - alpha;
    *al = Align16{aligned(g, 16) && aligned(mom, 16), true};
    uint32_t same = 0;
    for (uint32_t m = 0; m < M; ++m) {
        if (!w_send[m] || !w_now[m]) return SDL_ERR_INVALID_ARG;
        if (!aligned(w_send[m], 2) || !aligned(w_now[m], 2)) return SDL_ERR_ALIGNMENT;
        al->model = al->model && aligned(w_send[m], 16) && aligned(w_now[m], 16);
        same += (w_send[m] == w_now[m]);
        a.w_send[m] = static_cast<const uint16_t*>(w_send[m]);
        a.w_now[m] = static_cast<uint16_t*>(w_now[m]);
    }
    if (same != 0 && same != M) return SDL_ERR_INVALID_ARG;   // alias all replicas or none
    a.aliased = same == M;
    return SDL_OK;
}

// Optional message outputs of a fused call; the whole-span scale needs its scale words as
// workspace even when no message is written.
static int attach_fused_messages(Args& a, uint32_t M, sdl_format_t fmt, void* const* codes_or_null,
                                 void* const* scales_or_null, Align16* al)
{
    if (codes_or_null) {
        const bool scaled = is_scaled(fmt);
        if (scaled && !scales_or_null) return SDL_ERR_INVALID_ARG;
        for (uint32_t m = 0; m < M; ++m) {
            if (!codes_or_null[m] || (scaled && !scales_or_null[m])) return SDL_ERR_INVALID_ARG;
            if (!aligned(codes_or_null[m], code_align(fmt))) return SDL_ERR_ALIGNMENT;
            al->msg = al->msg && aligned(codes_or_null[m], 16);
            a.codes[m] = static_cast<uint8_t*>(codes_or_null[m]);
            a.scales[m] = scaled ? static_cast<uint8_t*>(scales_or_null[m]) : nullptr;
        }
        a.emit = 1;
    }
    if (is_span_scaled(fmt)) {
        if (!scales_or_null) return SDL_ERR_INVALID_ARG;
        for (uint32_t m = 0; m < M; ++m) {
            if (!scales_or_null[m]) return SDL_ERR_INVALID_ARG;
            if (!aligned(scales_or_null[m], 4)) return SDL_ERR_ALIGNMENT;
            a.scales[m] = static_cast<uint8_t*>(scales_or_null[m]);
        }
    }
    return SDL_OK;
}

int sdl_fragment_outer_step(float* g, float* mom, const void* const* w_send, void* const* w_now,
                            uint32_t M, uint64_t n, sdl_format_t fmt, float lr, float mu, float alpha,
                            void* const* codes_or_null, void* const* scales_or_null, void* stream)
{
    if (n == 0) return (valid_format(fmt) && M >= 1 && M <= SDL_MAX_WORKERS) ? SDL_OK : SDL_ERR_INVALID_ARG;
    Args a;
    Align16 al;
    int rc = fill_fused_args(a, g, mom, w_send, w_now, M, fmt, lr, mu, alpha, &al);
    if (rc != SDL_OK) return rc;
    rc = attach_fused_messages(a, M, fmt, codes_or_null, scales_or_null, &al);
    if (rc != SDL_OK) return rc;
    return run_single_span<kFused>(a, n, fmt, al, stream);
}

}  // extern "C"

// The pieces of fragment p that one call processes, in model order: the joined runs, or, for the
// whole-span scale, the spans themselves (one scale word per parameter group).  Yields, for every
// non-empty piece, where it lies in the flat arrays, in the message arrays (pieces back to back,
// each padded to whole tiles) and in staged g / mom (the fragment's runs back to back, each padded
// to whole tiles).  Holds no storage of its own: the callers walk it once per pass.
struct PieceWalk {
    struct Piece { uint64_t offset, numel, msg, soff; Align16 al; uint32_t sidx; };
    const sdl_span_t* runs;
    const sdl_span_t* pieces;
    uint32_t n_runs, n_pieces;
    Align16 al;
    bool staged;
    uint32_t i = 0, run_i = 0;
    uint64_t msg = 0, run_start = 0;

    bool next(Piece* out)
    {
        for (; i < n_pieces; ++i) {
            if (pieces[i].numel == 0) continue;
            // the run that contains this piece, and where that run starts in the staged arrays
            while (run_i < n_runs && pieces[i].offset >= runs[run_i].offset + runs[run_i].numel) {
                run_start += (runs[run_i].numel + kPad - 1) / kPad * kPad;
                ++run_i;
            }
            const uint64_t soff = run_i < n_runs ? run_start + (pieces[i].offset - runs[run_i].offset) : 0;
            // a piece keeps the 16-byte alignment of the bases when it starts on a multiple of 8 elements
            const Align16 piece_al = al.at((pieces[i].offset % 8 == 0) && (!staged || soff % 8 == 0));
            *out = Piece{pieces[i].offset, pieces[i].numel, msg, soff, piece_al, i};
            msg += (pieces[i].numel + kPad - 1) / kPad * kPad;
            ++i;
            return true;
        }
        return false;
    }
};

// One mode over all runs of fragment p, on flat model arrays; the fragment's messages are
// the concatenation of its runs, each padded to a multiple of 512 elements.  No host or device
// memory is allocated on the way.
template <int MODE>
static int launch_fragment(Args& a, const sdl_plan_t* plan, uint32_t p, Align16 al, sdl_format_t fmt, void* stream)
{
    const sdl_span_t* runs = nullptr;
    const sdl_span_t* pieces = nullptr;
    uint32_t n_runs = 0, n_pieces = 0;
    int rc = sdl_plan_fragment_runs(plan, p, &runs, &n_runs);
    if (rc != SDL_OK) return rc;
    if (is_span_scaled(fmt) && MODE != kMerge) rc = sdl_plan_fragment_spans(plan, p, &pieces, &n_pieces);
    else { pieces = runs; n_pieces = n_runs; }
    if (rc != SDL_OK) return rc;
    const PieceWalk start{runs, pieces, n_runs, n_pieces, al, a.staged != 0u};
    PieceWalk::Piece pc;
    const uint32_t tile = tile_elems(MODE, a, fmt);
    {
        // sizes are checked for every launch of the call before the first one is made
        PieceWalk walk = start;
        uint64_t n_wg = 0;
        for (uint32_t in_group = 0; walk.next(&pc);) {
            n_wg += (pc.numel + tile - 1) / tile;
            if (n_wg > 0x7fffffffull) return SDL_ERR_UNSUPPORTED;
            if (++in_group == (uint32_t)kMaxRuns) { in_group = 0; n_wg = 0; }
        }
    }
    {
        // the replicas are flat model arrays; g / mom too, unless they are a staging buffer of this fragment
        size_t cb = 0, sb = 0;
        if (MODE != kMerge) {
            rc = sdl_plan_message_bytes(plan, p, fmt, &cb, &sb);
            if (rc != SDL_OK) return rc;
        }
        const uint64_t model = sdl_plan_total_numel(plan);
        if (arrays_clash<MODE>(a, fmt, model, a.staged ? sdl_plan_staged_numel(plan, p) : model, cb, sb))
            return SDL_ERR_INVALID_ARG;
    }
    if (is_span_scaled(fmt) && (MODE == kQuantize || MODE == kFused)) {
        // whole-span scale: clear the scale words, take the grid-wide maxima, then encode
        SpanRun batch[kAbsmaxMaxRuns];
        uint32_t nb = 0;
        PieceWalk walk = start;
        for (bool more = walk.next(&pc); more || nb;) {
            if (more) batch[nb++] = SpanRun{pc.offset, pc.numel, pc.soff, pc.al.model, pc.sidx};
            more = more && walk.next(&pc);
            if (nb == (uint32_t)kAbsmaxMaxRuns || !more) {
                if (launch_span_prepass(a, batch, nb, (hipStream_t)stream) != hipSuccess) return SDL_ERR_DEVICE;
                nb = 0;
            }
        }
    }
    RunBuilder rb(&a, tile);
    PieceWalk walk = start;
    for (bool more = walk.next(&pc); more || a.n_runs;) {
        if (more) rb.add(pc.offset, pc.numel, pc.al.path(), pc.msg, pc.sidx, pc.soff);
        more = more && walk.next(&pc);
        if (rb.full() || !more) {
            if (launch<MODE>(a, fmt, (uint32_t)rb.n_wg, (hipStream_t)stream) != hipSuccess) return SDL_ERR_DEVICE;
            rb = RunBuilder(&a, tile);
        }
    }
    return SDL_OK;
}

extern "C" {

int sdl_plan_message_bytes(const sdl_plan_t* plan, uint32_t p, sdl_format_t fmt, size_t* code_bytes,
                           size_t* scale_bytes)
{
    if (!valid_format(fmt)) return SDL_ERR_INVALID_ARG;
    const sdl_span_t* runs = nullptr;
    uint32_t n_runs = 0;
    int rc = is_span_scaled(fmt) ? sdl_plan_fragment_spans(plan, p, &runs, &n_runs)
                                 : sdl_plan_fragment_runs(plan, p, &runs, &n_runs);
    if (rc != SDL_OK) return rc;
    uint64_t padded = 0;
    for (uint32_t i = 0; i < n_runs; ++i) padded += (runs[i].numel + kPad - 1) / kPad * kPad;
    sdl_exchange_bytes(fmt, padded, code_bytes, scale_bytes);
    if (is_span_scaled(fmt) && scale_bytes) *scale_bytes = (size_t)n_runs * 4;   // one word per span
    return SDL_OK;
}

static int fused_fragment(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                          const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                          sdl_format_t fmt, float lr, float mu, float alpha, void* const* codes_or_null,
                          void* const* scales_or_null, void* stream, bool staged)
{
    if (!plan || p >= sdl_plan_num_fragments(plan)) return SDL_ERR_INVALID_ARG;
    // the whole-span scale needs scale words as workspace: only the calls that take them support it
    if (valid_format(fmt) && is_span_scaled(fmt) && !scales_or_null) return SDL_ERR_UNSUPPORTED;
    Args a;
    Align16 al;
    int rc = fill_fused_args(a, g_base, mom_base, w_send_base, w_now_base, M, fmt, lr, mu, alpha, &al);
    if (rc != SDL_OK) return rc;
    rc = attach_fused_messages(a, M, fmt, codes_or_null, scales_or_null, &al);
    if (rc != SDL_OK) return rc;
    a.staged = staged ? 1u : 0u;
    return launch_fragment<kFused>(a, plan, p, al, fmt, stream);
}

static int quantize_fragment(const sdl_plan_t* plan, uint32_t p, const float* g_base,
                             const void* const* w_send_base, uint32_t M, sdl_format_t fmt,
                             void* const* codes, void* const* scales, void* stream, bool staged)
{
    if (!plan || p >= sdl_plan_num_fragments(plan)) return SDL_ERR_INVALID_ARG;
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    const bool scaled = is_scaled(fmt);
    if (!g_base || !w_send_base || !codes || (scaled && !scales)) return SDL_ERR_INVALID_ARG;
    if (!aligned(g_base, 4)) return SDL_ERR_ALIGNMENT;
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.g = const_cast<float*>(g_base);
    a.M = M;
    Align16 al;
    al.model = aligned(g_base, 16);
    for (uint32_t m = 0; m < M; ++m) {
        if (!w_send_base[m] || !codes[m] || (scaled && !scales[m])) return SDL_ERR_INVALID_ARG;
        if (!aligned(w_send_base[m], 2) || !aligned(codes[m], code_align(fmt))) return SDL_ERR_ALIGNMENT;
        if (scaled && !aligned(scales[m], scale_align(fmt))) return SDL_ERR_ALIGNMENT;
        al.model = al.model && aligned(w_send_base[m], 16);
        al.msg = al.msg && aligned(codes[m], 16);
        a.w_send[m] = static_cast<const uint16_t*>(w_send_base[m]);
        a.codes[m] = static_cast<uint8_t*>(codes[m]);
        a.scales[m] = scaled ? static_cast<uint8_t*>(scales[m]) : nullptr;
    }
    a.staged = staged ? 1u : 0u;
    return launch_fragment<kQuantize>(a, plan, p, al, fmt, stream);
}

static int reduce_fragment(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                           const void* const* codes, const void* const* scales, uint32_t M,
                           sdl_format_t fmt, float lr, float mu, void* stream, bool staged)
{
    if (!plan || p >= sdl_plan_num_fragments(plan)) return SDL_ERR_INVALID_ARG;
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    const bool scaled = is_scaled(fmt);
    if (!g_base || !mom_base || !codes || (scaled && !scales)) return SDL_ERR_INVALID_ARG;
    if (!aligned(g_base, 4) || !aligned(mom_base, 4)) return SDL_ERR_ALIGNMENT;
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.g = g_base; a.mom = mom_base; a.M = M; a.lr = lr; a.mu = mu;
    Align16 al;
    al.model = aligned(g_base, 16) && aligned(mom_base, 16);
    for (uint32_t m = 0; m < M; ++m) {
        if (!codes[m] || (scaled && !scales[m])) return SDL_ERR_INVALID_ARG;
        if (!aligned(codes[m], code_align(fmt))) return SDL_ERR_ALIGNMENT;
        if (scaled && !aligned(scales[m], scale_align(fmt))) return SDL_ERR_ALIGNMENT;
        al.msg = al.msg && aligned(codes[m], 16);
        a.codes[m] = static_cast<uint8_t*>(const_cast<void*>(codes[m]));
        a.scales[m] = scaled ? static_cast<uint8_t*>(const_cast<void*>(scales[m])) : nullptr;
    }
    a.staged = staged ? 1u : 0u;
    return launch_fragment<kReduce>(a, plan, p, al, fmt, stream);
}

static int receive_fragment(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                            const void* const* codes, const void* const* scales, void* const* w_now_base,
                            uint32_t M, sdl_format_t fmt, float lr, float mu, float alpha, void* stream, bool staged)
{
    if (!plan || p >= sdl_plan_num_fragments(plan)) return SDL_ERR_INVALID_ARG;
    Args a;
    Align16 al;
    int rc = fill_receive_args(a, g_base, mom_base, codes, scales, w_now_base, M, fmt, lr, mu, alpha, &al);
    if (rc != SDL_OK) return rc;
    a.staged = staged ? 1u : 0u;
    return launch_fragment<kReceive>(a, plan, p, al, fmt, stream);
}

static int merge_fragment(const sdl_plan_t* plan, uint32_t p, const float* g_new_base, void* const* w_now_base,
                          uint32_t M, float alpha, void* stream, bool staged)
{
    if (!plan || p >= sdl_plan_num_fragments(plan)) return SDL_ERR_INVALID_ARG;
    if (M == 0 || M > SDL_MAX_WORKERS || !g_new_base || !w_now_base) return SDL_ERR_INVALID_ARG;
    if (!aligned(g_new_base, 4)) return SDL_ERR_ALIGNMENT;
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.g = const_cast<float*>(g_new_base); a.M = M; a.alpha = alpha; a.one_minus_alpha = 1.0f - alpha;
    Align16 al;
    al.model = aligned(g_new_base, 16);
    for (uint32_t m = 0; m < M; ++m) {
        if (!w_now_base[m]) return SDL_ERR_INVALID_ARG;
        if (!aligned(w_now_base[m], 2)) return SDL_ERR_ALIGNMENT;
        al.model = al.model && aligned(w_now_base[m], 16);
        a.w_now[m] = static_cast<uint16_t*>(w_now_base[m]);
    }
    a.staged = staged ? 1u : 0u;
    return launch_fragment<kMerge>(a, plan, p, al, SDL_FMT_FP32, stream);
}


int sdl_fragment_outer_step_plan(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                 const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                 sdl_format_t fmt, float lr, float mu, float alpha, void* stream)
{
    return fused_fragment(plan, p, g_base, mom_base, w_send_base, w_now_base, M, fmt, lr, mu, alpha, nullptr, nullptr,
                          stream, false);
}
int sdl_fragment_outer_step_plan_ex(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                    const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                    sdl_format_t fmt, float lr, float mu, float alpha, void* const* codes_or_null,
                                    void* const* scales_or_null, void* stream)
{
    return fused_fragment(plan, p, g_base, mom_base, w_send_base, w_now_base, M, fmt, lr, mu, alpha, codes_or_null,
                          scales_or_null, stream, false);
}

// Device address of `scratch` on the current device, looked up once per device.
static int static_scratch(uint32_t** out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mutex;
    static uint32_t* address[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SDL_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(mutex);
    if (!address[dev]) {
        uint32_t* ptr = nullptr;
        if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SDL_ERR_DEVICE;
        address[dev] = ptr;
    }
    *out = address[dev];
    return SDL_OK;
}

int sdl_fragment_outer_step_plan_static(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                        const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                        sdl_format_t fmt, float lr, float mu, float alpha, void* stream)
{
    if (!plan || p >= sdl_plan_num_fragments(plan)) return SDL_ERR_INVALID_ARG;
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    if (!is_span_scaled(fmt))   // no other format needs memory beyond the model arrays
        return fused_fragment(plan, p, g_base, mom_base, w_send_base, w_now_base, M, fmt, lr, mu, alpha, nullptr,
                              nullptr, stream, false);
    const sdl_span_t* spans = nullptr;
    uint32_t n_spans = 0;
    int rc = sdl_plan_fragment_spans(plan, p, &spans, &n_spans);
    if (rc != SDL_OK) return rc;
    if (n_spans > SDL_STATIC_MAX_SPANS) return SDL_ERR_TOO_LARGE;
    uint32_t* base = nullptr;
    rc = static_scratch(&base);
    if (rc != SDL_OK) return rc;
    void* words[SDL_MAX_WORKERS];
    for (uint32_t m = 0; m < M; ++m) words[m] = base + (size_t)m * SDL_STATIC_MAX_SPANS;
    // the pre-pass clears the words of the fragment's spans with a fill kernel before it takes the
    // maxima, so what an earlier call left in the array does not matter
    return fused_fragment(plan, p, g_base, mom_base, w_send_base, w_now_base, M, fmt, lr, mu, alpha, nullptr, words,
                          stream, false);
}

int sdl_quantize_outer_grad_plan(const sdl_plan_t* plan, uint32_t p, const float* g_base,
                                 const void* const* w_send_base, uint32_t M, sdl_format_t fmt,
                                 void* const* codes, void* const* scales, void* stream)
{
    return quantize_fragment(plan, p, g_base, w_send_base, M, fmt, codes, scales, stream, false);
}
int sdl_dequant_reduce_nesterov_plan(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                     const void* const* codes, const void* const* scales, uint32_t M,
                                     sdl_format_t fmt, float lr, float mu, void* stream)
{
    return reduce_fragment(plan, p, g_base, mom_base, codes, scales, M, fmt, lr, mu, stream, false);
}
int sdl_merge_overlap_plan(const sdl_plan_t* plan, uint32_t p, const float* g_new_base, void* const* w_now_base,
                           uint32_t M, float alpha, void* stream)
{
    return merge_fragment(plan, p, g_new_base, w_now_base, M, alpha, stream, false);
}

int sdl_receive_outer_step_plan(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                const void* const* codes, const void* const* scales, void* const* w_now_base,
                                uint32_t M, sdl_format_t fmt, float lr, float mu, float alpha, void* stream)
{
    return receive_fragment(plan, p, g_base, mom_base, codes, scales, w_now_base, M, fmt, lr, mu, alpha, stream, false);
}
int sdl_receive_outer_step_staged(const sdl_plan_t* plan, uint32_t p, float* g_frag, float* mom_frag,
                                  const void* const* codes, const void* const* scales, void* const* w_now_base,
                                  uint32_t M, sdl_format_t fmt, float lr, float mu, float alpha, void* stream)
{
    return receive_fragment(plan, p, g_frag, mom_frag, codes, scales, w_now_base, M, fmt, lr, mu, alpha, stream, true);
}

uint64_t sdl_plan_staged_numel(const sdl_plan_t* plan, uint32_t p)
{
    const sdl_span_t* runs = nullptr;
    uint32_t n_runs = 0;
    if (sdl_plan_fragment_runs(plan, p, &runs, &n_runs) != SDL_OK) return 0;
    uint64_t padded = 0;
    for (uint32_t i = 0; i < n_runs; ++i) padded += (runs[i].numel + kPad - 1) / kPad * kPad;
    return padded;
}
int sdl_fragment_outer_step_staged(const sdl_plan_t* plan, uint32_t p, float* g_frag, float* mom_frag,
                                   const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                   sdl_format_t fmt, float lr, float mu, float alpha, void* stream)
{
    return fused_fragment(plan, p, g_frag, mom_frag, w_send_base, w_now_base, M, fmt, lr, mu, alpha, nullptr, nullptr,
                          stream, true);
}
int sdl_fragment_outer_step_staged_ex(const sdl_plan_t* plan, uint32_t p, float* g_frag, float* mom_frag,
                                      const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                      sdl_format_t fmt, float lr, float mu, float alpha, void* const* codes_or_null,
                                      void* const* scales_or_null, void* stream)
{
    return fused_fragment(plan, p, g_frag, mom_frag, w_send_base, w_now_base, M, fmt, lr, mu, alpha, codes_or_null,
                          scales_or_null, stream, true);
}
int sdl_quantize_outer_grad_staged(const sdl_plan_t* plan, uint32_t p, const float* g_frag,
                                   const void* const* w_send_base, uint32_t M, sdl_format_t fmt,
                                   void* const* codes, void* const* scales, void* stream)
{
    return quantize_fragment(plan, p, g_frag, w_send_base, M, fmt, codes, scales, stream, true);
}
int sdl_dequant_reduce_nesterov_staged(const sdl_plan_t* plan, uint32_t p, float* g_frag, float* mom_frag,
                                       const void* const* codes, const void* const* scales, uint32_t M,
                                       sdl_format_t fmt, float lr, float mu, void* stream)
{
    return reduce_fragment(plan, p, g_frag, mom_frag, codes, scales, M, fmt, lr, mu, stream, true);
}
int sdl_merge_overlap_staged(const sdl_plan_t* plan, uint32_t p, const float* g_new_frag, void* const* w_now_base,
                             uint32_t M, float alpha, void* stream)
{
    return merge_fragment(plan, p, g_new_frag, w_now_base, M, alpha, stream, true);
}

int sdl_memory_probe(sdl_probe_t kind, void* dst, const void* src, uint64_t nbytes, void* stream)
{
    if (kind < SDL_PROBE_COPY || kind > SDL_PROBE_FILL_NT) return SDL_ERR_INVALID_ARG;
    if (nbytes == 0) return SDL_OK;
    if (!dst || (!src && kind != SDL_PROBE_FILL_NT) || nbytes % 16 != 0) return SDL_ERR_INVALID_ARG;
    if (!aligned(dst, 16) || !aligned(src, 16)) return SDL_ERR_ALIGNMENT;
    const uint64_t n16 = nbytes / 16, n_wg = (n16 + kCopyThreads - 1) / kCopyThreads;
    if (n_wg > 0x7fffffffull) return SDL_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)n_wg), block(kCopyThreads);
    hipStream_t s = (hipStream_t)stream;
    u32x4* d = static_cast<u32x4*>(dst);
    const u32x4* r = static_cast<const u32x4*>(src);
    switch (kind) {
    case SDL_PROBE_COPY:
        hipLaunchKernelGGL(sdl_copy_kernel, grid, block, 0, s, static_cast<uint4*>(dst), static_cast<const uint4*>(src), n16);
        break;
    case SDL_PROBE_COPY_NT: hipLaunchKernelGGL((sdl_probe_kernel<SDL_PROBE_COPY_NT>), grid, block, 0, s, d, r, n16); break;
    case SDL_PROBE_READ_NT: hipLaunchKernelGGL((sdl_probe_kernel<SDL_PROBE_READ_NT>), grid, block, 0, s, d, r, n16); break;
    default: hipLaunchKernelGGL((sdl_probe_kernel<SDL_PROBE_FILL_NT>), grid, block, 0, s, d, r, n16); break;
    }
    return hipGetLastError() == hipSuccess ? SDL_OK : SDL_ERR_DEVICE;
}

int sdl_copy_bytes(void* dst, const void* src, uint64_t nbytes, void* stream)
{
    return sdl_memory_probe(SDL_PROBE_COPY, dst, src, nbytes, stream);
}

}  // extern "C"
