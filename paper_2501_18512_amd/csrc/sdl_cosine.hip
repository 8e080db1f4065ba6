// Cosine similarity between the replicas' outer gradients (Appendix of the paper, paragraph on
// the outer gradients' cosine similarity) for gfx950 (MI355X).
//
// Two kernels.
//   sdl_gram_kernel   streams g and the M replicas once and accumulates the Gram matrix of
//                     the outer gradients Delta_m = g - float(w_m).  A workgroup is one
//                     64-lane wavefront; a set of parameters gets a share G of the launch's
//                     workgroups in proportion to its size, and workgroup k of the set walks
//                     the set's tiles of 512 consecutive parameters with a fixed stride
//                     (tile k, k + G, k + 2G, ...), lane l owning the eight
//                     parameters [8l, 8l+8) of a tile, so every load instruction of the
//                     wavefront covers one contiguous piece of an array (2 x 1 KiB of fp32,
//                     1 KiB of bf16 through 128-bit accesses).  Each lane keeps its M(M+1)/2
//                     sums in fp64 registers (products of fp32 values are exact in fp64); at
//                     the end the wavefront folds them with a butterfly of lane exchanges and
//                     lane 0 writes one partial Gram matrix.  The next tile's loads are issued
//                     before the current tile is consumed.
//   sdl_gram_finalize adds the partial matrices of a set in a fixed order (lane-strided, then
//                     the same butterfly; a set with more than 128 partial matrices in two
//                     launches, chunks of 64 first) and derives cos and the mean over pairs.
//                     The same kernel adds the Gram matrices of several sets (fragment from
//                     spans, unions of fragments).
// No atomics: the order of every sum depends on the sizes alone, so results are reproducible.
// More than 8 replicas are handled as 8 x 8 blocks of the matrix, one launch per block.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "sdl.h"
#include "sdl_device.h"

namespace {

using namespace sdl_device;

constexpr int kLaneElems = 8;                   // consecutive parameters a lane owns in a tile
constexpr int kTile = kLaneElems * kWave;       // 512
constexpr int kBlockM = 8;                      // replicas per side of one launch's block of the matrix
constexpr int kMaxSets = 48;                    // parameter sets per launch
constexpr int kWindows = 48;                    // windows per launch: a set holding a share of 4/48 or more is cut
constexpr int kMaxPieces = kMaxSets + kWindows;
constexpr uint32_t kGroups = 8192;              // workgroups per launch, shared out among the sets (32 per compute unit)
constexpr uint32_t kMaxGroups = 8192;           // what the workspace is sized for


struct Set {
    uint64_t offset;     // first element in the flat arrays
    uint64_t numel;
    uint32_t first_wg;   // first workgroup of the launch that works on this set
    uint32_t G;          // workgroups of this set (>= 1)
};

// What the kernel walks: a set, or a window of a large set (tile aligned), with its own
// share of the set's workgroups.
struct Piece {
    uint64_t offset;
    uint64_t numel;
    uint32_t first_wg;
    uint32_t G;
    uint32_t fast;       // every array is 16-byte aligned at the piece's start
    uint32_t pad_;
};

struct GramArgs {
    const float* g;
    const uint16_t* wr[kBlockM];   // replicas of the block's rows
    const uint16_t* wc[kBlockM];   // replicas of the block's columns (unused for a diagonal block)
    double* partial;               // [workgroup of the launch][M*M]
    uint32_t M;                    // side of the whole matrix
    uint32_t r0, c0;               // first row / column of this block
    uint32_t n_pieces;
    Piece pieces[kMaxPieces];
};

// Raw bits of one tile as a lane holds them: 8 fp32 of g, 8 bf16 of each replica.
template <int NW>
struct TileRegs {
    u32x4 g0, g1;
    u32x4 w[NW];
};

// valid = parameters of the tile that exist (512 except in a set's last tile).  Full tiles of
// aligned sets use 128-bit buffer loads, full tiles of sets that start at some other element
// 128-bit loads of element alignment; a ragged last tile goes element by element under the buffer
// range check, which returns 0 past the end (g = 0 and w = 0 give Delta = 0: no contribution).
template <int NW>
__device__ __forceinline__ void load_tile(TileRegs<NW>& t, const float* g, const uint16_t* (&w)[NW],
                                          uint64_t e0, uint32_t valid, bool fast, uint32_t lane)
{
    if (fast && valid == (uint32_t)kTile) {
        const __amdgpu_buffer_rsrc_t rg = rsrc(g + e0, kTile * 4);
        t.g0 = __builtin_amdgcn_raw_buffer_load_b128(rg, (int)(lane * 32), 0, 2);
        t.g1 = __builtin_amdgcn_raw_buffer_load_b128(rg, (int)(lane * 32 + 16), 0, 2);
#pragma unroll
        for (int m = 0; m < NW; ++m)
            t.w[m] = __builtin_amdgcn_raw_buffer_load_b128(rsrc(w[m] + e0, kTile * 2), (int)(lane * 16), 0, 2);
    } else if (valid == (uint32_t)kTile) {
        const u32x4_f32elem* pg = reinterpret_cast<const u32x4_f32elem*>(g + e0 + lane * kLaneElems);
        t.g0 = __builtin_nontemporal_load(pg);
        t.g1 = __builtin_nontemporal_load(pg + 1);
#pragma unroll
        for (int m = 0; m < NW; ++m)
            t.w[m] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_bf16elem*>(w[m] + e0 + lane * kLaneElems));
    } else {
        const __amdgpu_buffer_rsrc_t rg = rsrc(g + e0, valid * 4);
        uint32_t x[kLaneElems];
#pragma unroll
        for (int j = 0; j < kLaneElems; ++j)
            x[j] = __builtin_amdgcn_raw_buffer_load_b32(rg, (int)((lane * kLaneElems + j) * 4), 0, 0);
        t.g0 = u32x4{x[0], x[1], x[2], x[3]};
        t.g1 = u32x4{x[4], x[5], x[6], x[7]};
#pragma unroll
        for (int m = 0; m < NW; ++m) {
            const __amdgpu_buffer_rsrc_t rw = rsrc(w[m] + e0, valid * 2);
            uint32_t h[kLaneElems];
#pragma unroll
            for (int j = 0; j < kLaneElems; ++j)
                h[j] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rw, (int)((lane * kLaneElems + j) * 2), 0, 0)
                       & 0xffffu;
            t.w[m] = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        }
    }
}

// Outer gradients of one replica for the lane's 8 parameters: one fp32 subtraction each.
__device__ __forceinline__ void deltas(const u32x4& g0, const u32x4& g1, const u32x4& w, float (&d)[kLaneElems])
{
    const uint32_t gb[kLaneElems] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
    const uint32_t wb[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int j = 0; j < kLaneElems; ++j) {
        const uint32_t bits = (j & 1) ? (wb[j / 2] & 0xffff0000u) : (wb[j / 2] << 16);
        d[j] = u2f(gb[j]) - u2f(bits);
    }
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// MR x MC block of the Gram matrix; DIAG: rows and columns are the same replicas (upper
// triangle only, MC == MR).
template <int MR, int MC, bool DIAG>
__global__ void __launch_bounds__(kWave) sdl_gram_kernel(const GramArgs a)
{
    constexpr int NW = DIAG ? MR : MR + MC;
    const uint32_t lane = threadIdx.x;
    uint32_t s = 0;
    while (s + 1 < a.n_pieces && blockIdx.x >= a.pieces[s + 1].first_wg) ++s;
    const Piece set = a.pieces[s];
    const uint32_t k = blockIdx.x - set.first_wg;
    const bool fast = set.fast != 0u;
    const uint64_t n_tiles = (set.numel + kTile - 1) / kTile;

    const uint16_t* w[NW];
#pragma unroll
    for (int m = 0; m < MR; ++m) w[m] = a.wr[m];
    if constexpr (!DIAG) {
#pragma unroll
        for (int m = 0; m < MC; ++m) w[MR + m] = a.wc[m];
    }

    double acc[MR][MC];
#pragma unroll
    for (int r = 0; r < MR; ++r)
#pragma unroll
        for (int c = 0; c < MC; ++c) acc[r][c] = 0.0;

    auto valid_of = [&](uint64_t t) -> uint32_t {
        const uint64_t rem = set.numel - t * kTile;
        return rem < (uint64_t)kTile ? (uint32_t)rem : (uint32_t)kTile;
    };

    auto consume = [&](const TileRegs<NW>& t) {
        float f[NW][kLaneElems];
#pragma unroll
        for (int m = 0; m < NW; ++m) deltas(t.g0, t.g1, t.w[m], f[m]);
#pragma unroll
        for (int j = 0; j < kLaneElems; ++j) {
            double d[NW];
#pragma unroll
            for (int m = 0; m < NW; ++m) d[m] = (double)f[m][j];
#pragma unroll
            for (int r = 0; r < MR; ++r)
#pragma unroll
                for (int c = DIAG ? r : 0; c < MC; ++c)
                    acc[r][c] = __builtin_fma(d[r], d[DIAG ? c : MR + c], acc[r][c]);
        }
    };

    // workgroup k's tiles: first, first + step, ... below end; the next tile's loads are issued before the
    // current tile is consumed
    const uint64_t first = k, step = set.G, end = n_tiles;
    TileRegs<NW> cur;
    if (first < end) load_tile<NW>(cur, a.g, w, set.offset + first * kTile, valid_of(first), fast, lane);
    for (uint64_t t = first; t < end; t += step) {
        TileRegs<NW> nxt = cur;
        const uint64_t tn = t + step;
        if (tn < end) load_tile<NW>(nxt, a.g, w, set.offset + tn * kTile, valid_of(tn), fast, lane);
        consume(cur);
        cur = nxt;
    }

    double* out = a.partial + (uint64_t)blockIdx.x * a.M * a.M;
#pragma unroll
    for (int r = 0; r < MR; ++r)
#pragma unroll
        for (int c = DIAG ? r : 0; c < MC; ++c) {
            const double v = wave_sum(acc[r][c]);
            if (lane == 0) out[(a.r0 + r) * a.M + (a.c0 + c)] = v;
        }
}

// What each output of the finalize kernel adds up.
constexpr uint32_t kFinChunk = 64;                                        // matrices one first-level output adds
constexpr int kMaxFin = kMaxGroups / kFinChunk + 2 * kMaxSets + 2;        // outputs per finalize launch

struct FinArgs {
    const double* in;              // matrices of M*M doubles (only a <= b is read), stride_k doubles apart
    double* out;                   // output o at out + o * out_stride
    uint64_t stride_k;
    uint64_t out_stride;
    uint32_t M;
    uint32_t emit;                 // 1: G, cos, mean (2*M*M + 1 doubles); 0: G only (M*M doubles)
    uint32_t first[kMaxFin];       // output o adds the matrices first[o] .. first[o] + count[o] - 1
    uint32_t count[kMaxFin];
};

// One workgroup per output.  A lane adds every 64th matrix of its output's range, so a range
// should be short: long ranges go through a first level of kFinChunk matrices per output.
__global__ void __launch_bounds__(256) sdl_gram_finalize(const FinArgs f)
{
    __shared__ double G[SDL_MAX_WORKERS * SDL_MAX_WORKERS];
    __shared__ double C[SDL_MAX_WORKERS * SDL_MAX_WORKERS];
    const uint32_t M = f.M, count = f.count[blockIdx.x];
    const double* base = f.in + (uint64_t)f.first[blockIdx.x] * f.stride_k;
    const uint32_t wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    uint32_t pair = 0;
    for (uint32_t a = 0; a < M; ++a)
        for (uint32_t b = a; b < M; ++b, ++pair) {
            if (pair % 4u != wave) continue;
            double s = 0.0;
            for (uint32_t k = lane; k < count; k += kWave) s += base[(uint64_t)k * f.stride_k + a * M + b];
            s = wave_sum(s);
            if (lane == 0) { G[a * M + b] = s; G[b * M + a] = s; }
        }
    __syncthreads();
    double* o = f.out + (uint64_t)blockIdx.x * f.out_stride;
    if (!f.emit) {
        for (uint32_t i = threadIdx.x; i < M * M; i += 256) o[i] = G[i];
        return;
    }
    for (uint32_t i = threadIdx.x; i < M * M; i += 256) {
        const uint32_t a = i / M, b = i % M;
        const double den = __builtin_sqrt(G[a * M + a]) * __builtin_sqrt(G[b * M + b]);
        const double c = den > 0.0 ? G[i] / den : 0.0;
        C[i] = c;
        o[i] = G[i];
        o[M * M + i] = c;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        uint32_t n = 0;
        for (uint32_t a = 0; a < M; ++a)
            for (uint32_t b = a + 1; b < M; ++b, ++n) s += C[a * M + b];
        o[2 * M * M] = n ? s / (double)n : 0.0;
    }
}

// ------------------------------------------------------------------ host side

uint32_t windows_per_launch() { return kWindows; }
uint32_t groups_per_launch() { return kGroups; }

template <int MR, bool DIAG>
int launch_block_c(int mc, const GramArgs& a, hipStream_t st)
{
    const dim3 grid(a.pieces[a.n_pieces - 1].first_wg + a.pieces[a.n_pieces - 1].G), block(kWave);
    if constexpr (DIAG) {
        hipLaunchKernelGGL((sdl_gram_kernel<MR, MR, true>), grid, block, 0, st, a);
    } else {
        switch (mc) {
        case 1: hipLaunchKernelGGL((sdl_gram_kernel<MR, 1, false>), grid, block, 0, st, a); break;
        case 2: hipLaunchKernelGGL((sdl_gram_kernel<MR, 2, false>), grid, block, 0, st, a); break;
        case 3: hipLaunchKernelGGL((sdl_gram_kernel<MR, 3, false>), grid, block, 0, st, a); break;
        case 4: hipLaunchKernelGGL((sdl_gram_kernel<MR, 4, false>), grid, block, 0, st, a); break;
        case 5: hipLaunchKernelGGL((sdl_gram_kernel<MR, 5, false>), grid, block, 0, st, a); break;
        case 6: hipLaunchKernelGGL((sdl_gram_kernel<MR, 6, false>), grid, block, 0, st, a); break;
        case 7: hipLaunchKernelGGL((sdl_gram_kernel<MR, 7, false>), grid, block, 0, st, a); break;
        case 8: hipLaunchKernelGGL((sdl_gram_kernel<MR, 8, false>), grid, block, 0, st, a); break;
        default: return SDL_ERR_INVALID_ARG;
        }
    }
    return hipGetLastError() == hipSuccess ? SDL_OK : SDL_ERR_DEVICE;
}

int launch_diag(int m, const GramArgs& a, hipStream_t st)
{
    switch (m) {
    case 1: return launch_block_c<1, true>(1, a, st);
    case 2: return launch_block_c<2, true>(2, a, st);
    case 3: return launch_block_c<3, true>(3, a, st);
    case 4: return launch_block_c<4, true>(4, a, st);
    case 5: return launch_block_c<5, true>(5, a, st);
    case 6: return launch_block_c<6, true>(6, a, st);
    case 7: return launch_block_c<7, true>(7, a, st);
    case 8: return launch_block_c<8, true>(8, a, st);
    default: return SDL_ERR_INVALID_ARG;
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shares the launch's workgroups out among the sets in proportion to their tiles (at least
// one each); returns the total, at most groups + n_sets.
uint32_t share_groups(Set* sets, uint32_t n_sets, uint32_t groups)
{
    uint64_t total_tiles = 0;
    for (uint32_t s = 0; s < n_sets; ++s) total_tiles += (sets[s].numel + kTile - 1) / kTile;
    uint32_t next = 0;
    for (uint32_t s = 0; s < n_sets; ++s) {
        const uint64_t tiles = (sets[s].numel + kTile - 1) / kTile;
        uint64_t G = total_tiles ? (tiles * groups + total_tiles - 1) / total_tiles : 1;
        if (G > tiles) G = tiles;
        if (G < 1) G = 1;
        sets[s].first_wg = next;
        sets[s].G = (uint32_t)G;
        next += (uint32_t)G;
    }
    return next;
}

// Partial Gram matrices of up to kMaxSets sets (already given their workgroups) into
// `partial`, one M x M matrix per workgroup of the launch.
int launch_gram(const float* g, const void* const* w, uint32_t M, const Set* sets, uint32_t n_sets, double* partial,
                hipStream_t st)
{
    GramArgs a{};
    a.g = g;
    a.partial = partial;
    a.M = M;
    // cut the sets into windows: about `windows` pieces per launch, shared out like the workgroups
    const uint32_t windows = windows_per_launch();
    uint64_t total_G = 0;
    for (uint32_t s = 0; s < n_sets; ++s) total_G += sets[s].G;
    for (uint32_t s = 0; s < n_sets; ++s) {
        const uint64_t tiles = (sets[s].numel + kTile - 1) / kTile;
        // only a set that holds a large share of the launch is cut (measured: cutting the spans
        // of a many-span fragment in two or three costs a few per cent, one large span gains 10 %)
        uint64_t nsub = total_G ? (uint64_t)windows * sets[s].G / total_G : 1;
        if (nsub < 4) nsub = 1;
        if (nsub > sets[s].G) nsub = sets[s].G;
        if (nsub > tiles) nsub = tiles;
        if (nsub < 1) nsub = 1;
        const uint64_t tiles_per = (tiles + nsub - 1) / nsub;
        for (uint64_t j = 0; j < nsub; ++j) {
            Piece& pc = a.pieces[a.n_pieces++];
            const uint64_t e0 = j * tiles_per * kTile;
            const uint64_t e1 = (j + 1) * tiles_per * kTile < sets[s].numel ? (j + 1) * tiles_per * kTile : sets[s].numel;
            pc.offset = sets[s].offset + (e0 < sets[s].numel ? e0 : sets[s].numel);
            pc.numel = e1 > e0 ? e1 - e0 : 0;
            const uint32_t w0 = (uint32_t)((uint64_t)sets[s].G * j / nsub), w1 = (uint32_t)((uint64_t)sets[s].G * (j + 1) / nsub);
            pc.first_wg = sets[s].first_wg + w0;
            pc.G = w1 - w0;
            bool fast = aligned16(g + pc.offset);
            for (uint32_t m = 0; m < M; ++m)
                fast = fast && aligned16(static_cast<const uint16_t*>(w[m]) + pc.offset);
            pc.fast = fast ? 1u : 0u;
        }
    }
    // the matrix in blocks of up to 8 x 8 replicas: diagonal blocks, then the blocks above them
    for (uint32_t r0 = 0; r0 < M; r0 += kBlockM) {
        const uint32_t mr = M - r0 < (uint32_t)kBlockM ? M - r0 : (uint32_t)kBlockM;
        for (uint32_t c0 = r0; c0 < M; c0 += kBlockM) {
            const uint32_t mc = M - c0 < (uint32_t)kBlockM ? M - c0 : (uint32_t)kBlockM;
            a.r0 = r0;
            a.c0 = c0;
            for (uint32_t m = 0; m < mr; ++m) a.wr[m] = static_cast<const uint16_t*>(w[r0 + m]);
            for (uint32_t m = 0; m < mc; ++m) a.wc[m] = static_cast<const uint16_t*>(w[c0 + m]);
            int rc;
            if (c0 == r0) rc = launch_diag((int)mr, a, st);
            else rc = launch_block_c<kBlockM, false>((int)mc, a, st);   // rows of an off-diagonal block are always full
            if (rc != SDL_OK) return rc;
        }
    }
    return SDL_OK;
}

int launch_finalize(const FinArgs& f, uint32_t n_out, hipStream_t st)
{
    hipLaunchKernelGGL(sdl_gram_finalize, dim3(n_out), dim3(256), 0, st, f);
    return hipGetLastError() == hipSuccess ? SDL_OK : SDL_ERR_DEVICE;
}

// One result per set from the partial matrices of its workgroups.  Sets with many workgroups
// are first added up in chunks of kFinChunk matrices (into tmp), so that no lane of the
// finalize kernel walks a long range.
int finalize_sets(const double* partial, const Set* sets, uint32_t n_sets, uint32_t M, double* out, double* tmp,
                  hipStream_t st)
{
    const uint64_t mm = (uint64_t)M * M;
    bool two_level = false;
    for (uint32_t s = 0; s < n_sets; ++s) two_level = two_level || sets[s].G > 2 * kFinChunk;
    FinArgs last{};
    last.out = out;
    last.stride_k = mm;
    last.out_stride = SDL_COSINE_RESULT_DOUBLES(M);
    last.M = M;
    last.emit = 1;
    if (!two_level) {
        last.in = partial;
        for (uint32_t s = 0; s < n_sets; ++s) { last.first[s] = sets[s].first_wg; last.count[s] = sets[s].G; }
        return launch_finalize(last, n_sets, st);
    }
    FinArgs lvl1{};
    lvl1.in = partial;
    lvl1.out = tmp;
    lvl1.stride_k = mm;
    lvl1.out_stride = mm;
    lvl1.M = M;
    lvl1.emit = 0;
    uint32_t n = 0;
    for (uint32_t s = 0; s < n_sets; ++s) {
        last.first[s] = n;
        for (uint32_t c = 0; c < sets[s].G; c += kFinChunk) {
            lvl1.first[n] = sets[s].first_wg + c;
            lvl1.count[n] = sets[s].G - c < kFinChunk ? sets[s].G - c : kFinChunk;
            ++n;
        }
        last.count[s] = n - last.first[s];
    }
    int rc = launch_finalize(lvl1, n, st);
    if (rc != SDL_OK) return rc;
    last.in = tmp;
    return launch_finalize(last, n_sets, st);
}

// One result from the Gram matrices of `count` results that lie stride doubles apart.
int finalize_union(const double* results, uint64_t stride, uint32_t count, uint32_t M, double* out, hipStream_t st)
{
    FinArgs f{};
    f.in = results;
    f.out = out;
    f.stride_k = stride;
    f.out_stride = SDL_COSINE_RESULT_DOUBLES(M);
    f.M = M;
    f.emit = 1;
    f.first[0] = 0;
    f.count[0] = count;
    return launch_finalize(f, 1, st);
}

// Workspace layout, in M x M matrices: the partial matrices of every launch, then the
// first-level sums of the finalize step; then (plan-level call without span_results) one
// result per set.
size_t partial_mats(size_t n_sets)
{
    const size_t launches = (n_sets + kMaxSets - 1) / kMaxSets;
    return launches * kMaxGroups + n_sets;
}
size_t tmp_mats(size_t n_sets)
{
    const size_t launches = (n_sets + kMaxSets - 1) / kMaxSets;
    return launches * (kMaxGroups / kFinChunk + 2) + 2 * n_sets;
}

int check_common(const void* g, const void* const* w, uint32_t M, const void* workspace)
{
    if (!g || !w || M == 0 || M > SDL_MAX_WORKERS || !workspace) return SDL_ERR_INVALID_ARG;
    for (uint32_t m = 0; m < M; ++m)
        if (!w[m]) return SDL_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) & 7u) return SDL_ERR_ALIGNMENT;
    return SDL_OK;
}

}  // namespace

extern "C" {

size_t sdl_cosine_workspace_bytes(uint32_t M, uint32_t n_sets)
{
    if (M == 0 || M > SDL_MAX_WORKERS) return 0;
    return ((partial_mats(n_sets) + tmp_mats(n_sets)) * M * M + (size_t)n_sets * SDL_COSINE_RESULT_DOUBLES(M))
           * sizeof(double);
}

int sdl_outer_grad_cosine(const float* g, const void* const* w, uint32_t M, uint64_t numel, double* result,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_common(g, w, M, workspace);
    if (rc != SDL_OK) return rc;
    if (!result) return SDL_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(result) & 7u) return SDL_ERR_ALIGNMENT;
    if (workspace_bytes < sdl_cosine_workspace_bytes(M, 1)) return SDL_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Set set{0, numel, 0, 0};
    share_groups(&set, 1, groups_per_launch());
    double* partial = static_cast<double*>(workspace);
    double* tmp = partial + partial_mats(1) * M * M;
    rc = launch_gram(g, w, M, &set, 1, partial, st);
    if (rc != SDL_OK) return rc;
    return finalize_sets(partial, &set, 1, M, result, tmp, st);
}

int sdl_outer_grad_cosine_plan(const sdl_plan_t* plan, uint32_t p, const float* g_base, const void* const* w_base,
                               uint32_t M, double* span_results, double* fragment_result, void* workspace,
                               size_t workspace_bytes, void* stream)
{
    int rc = check_common(g_base, w_base, M, workspace);
    if (rc != SDL_OK) return rc;
    if (!plan || !fragment_result) return SDL_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(fragment_result) & 7u) || (reinterpret_cast<uintptr_t>(span_results) & 7u))
        return SDL_ERR_ALIGNMENT;
    const sdl_span_t* spans = nullptr;
    uint32_t n_spans = 0;
    rc = sdl_plan_fragment_spans(plan, p, &spans, &n_spans);
    if (rc != SDL_OK) return rc;
    if (workspace_bytes < sdl_cosine_workspace_bytes(M, n_spans)) return SDL_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t groups = groups_per_launch();
    const uint64_t mm = (uint64_t)M * M, R = SDL_COSINE_RESULT_DOUBLES(M);
    double* partial = static_cast<double*>(workspace);
    double* tmp = partial + partial_mats(n_spans) * mm;
    double* per_span = span_results ? span_results : tmp + tmp_mats(n_spans) * mm;
    uint64_t used = 0, used_tmp = 0;   // matrices handed out so far
    for (uint32_t s0 = 0; s0 < n_spans; s0 += kMaxSets) {
        const uint32_t ns = n_spans - s0 < (uint32_t)kMaxSets ? n_spans - s0 : (uint32_t)kMaxSets;
        Set sets[kMaxSets];
        for (uint32_t s = 0; s < ns; ++s) sets[s] = Set{spans[s0 + s].offset, spans[s0 + s].numel, 0, 0};
        const uint32_t n_wg = share_groups(sets, ns, groups);
        double* part = partial + used * mm;
        rc = launch_gram(g_base, w_base, M, sets, ns, part, st);
        if (rc != SDL_OK) return rc;
        rc = finalize_sets(part, sets, ns, M, per_span + (uint64_t)s0 * R, tmp + used_tmp * mm, st);
        if (rc != SDL_OK) return rc;
        used += n_wg;
        used_tmp += n_wg / kFinChunk + ns;
    }
    // the fragment: Gram matrices of its spans added in span order
    return finalize_union(per_span, R, n_spans, M, fragment_result, st);
}

int sdl_cosine_combine(const double* results, uint64_t stride_doubles, uint32_t n_sets, uint32_t M, double* result,
                       void* stream)
{
    if (!results || !result || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    if (n_sets && stride_doubles < SDL_COSINE_RESULT_DOUBLES(M)) return SDL_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(results) & 7u) || (reinterpret_cast<uintptr_t>(result) & 7u))
        return SDL_ERR_ALIGNMENT;
    return finalize_union(results, stride_doubles, n_sets, M, result, static_cast<hipStream_t>(stream));
}

}  // extern "C"
