/*
 * sdl.h -- C ABI of the Streaming DiLoCo fragment outer step for AMD MI355X (gfx950).
 *
 * One fragment of the model is synchronised per call sequence:
 *
 *   send side      sdl_quantize_outer_grad       outer gradient of every replica,
 *                                                encoded in the exchange format
 *   receive side   sdl_dequant_reduce_nesterov   decode, fp32 mean over replicas,
 *                                                Nesterov outer optimizer
 *                  sdl_merge_overlap             alpha-mix into every replica
 *   or fused       sdl_fragment_outer_step       all of the above in one pass
 *
 * and sdl_fragment_plan builds the fragment map and the send/receive schedule on
 * the host; the *_plan forms of the calls work on whole fragments of a plan, and
 * sdl_engine_step drives them along the schedule.  sdl_offload_* keep the outer state
 * in host memory; sdl_outer_grad_cosine* and sdl_evaluation_params are the appendix's
 * diagnostics on the same arrays.  sdl_fragment_outer_step_plan_static is the fused step
 * for callers that cannot allocate; sdl_flat_layout says where to put the flat arrays and
 * sdl_memory_probe measures what the memory system gives (neither is part of the method).
 * The M replicas ("workers") are M parameter arrays
 * resident in one GPU's memory; no call communicates with another device.
 *
 * Conventions for every call
 *   - Returns an sdl_status_t (0 = SDL_OK, negative = error).  Never throws, never
 *     aborts.  On error nothing has been launched and no output was touched.
 *   - Argument checks run synchronously on the host.  Kernels are enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and the
 *     call returns without waiting for them.
 *   - "device" pointers are HIP device addresses owned by the caller; the library
 *     allocates and frees no device memory.  Arrays of pointers (w_send, w_now,
 *     codes, scales) are HOST arrays of M DEVICE pointers, read during the call.
 *   - n is the number of parameters of one contiguous span; any n >= 0 is
 *     accepted (n == 0 is a no-op).  Scale blocks are the 32-element groups
 *     [32k, 32k+32) counted from the start of the span; the last may be partial.
 *   - fp32 arrays must be 4-byte aligned, bf16 arrays 2-byte aligned, code and
 *     scale arrays as the format needs (4 / 2 / 1 / 1 bytes for FP32 / BF16 /
 *     E4M3 / E3M0); anything less gives SDL_ERR_ALIGNMENT.  Results do not depend
 *     on alignment, speed does: full speed needs every array to start on a 128-byte
 *     boundary (a cache line); model arrays (g, mom, replicas) that start elsewhere,
 *     at any element, cost up to a fifth (lines shared between neighbouring tiles
 *     are fetched twice); code arrays that are not 16-byte aligned put the whole
 *     call on an element-by-element path at a quarter of the speed.
 *   - 1 <= M <= SDL_MAX_WORKERS.
 *   - An array that a call writes must not overlap any other array of the call, except that
 *     w_send[m] may be the very same pointer as w_now[m] for every m (no overlap delay,
 *     tau = 0).  The span-level and fragment-level calls check this from the sizes they are
 *     given (n, or the plan's model size) and return SDL_ERR_INVALID_ARG; arrays that are
 *     only read may coincide.
 *   - Non-finite inputs: a block that contains Inf or NaN gets scale byte 0xff and
 *     decodes to NaN in every element (E3M0 / E4M3); BF16 / FP32 carry them through.
 */
#ifndef SDL_H
#define SDL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SDL_MAX_WORKERS 16
#define SDL_BLOCK 32           /* elements per scale byte (default formats) */
#define SDL_MAX_BLOCK 128      /* largest block of the block-scaled formats */
#define SDL_UNIT_PRE  (-1)     /* parameter group before the first block (embedding) */
#define SDL_UNIT_POST (-2)     /* parameter group after the last block (final norm, head) */

typedef enum {
    SDL_OK = 0,
    SDL_ERR_INVALID_ARG = -1,  /* NULL where not allowed, M out of range, bad enum, tau >= H ... */
    SDL_ERR_UNSUPPORTED = -2,
    SDL_ERR_ALIGNMENT = -3,    /* pointer not aligned to its element type */
    SDL_ERR_DEVICE = -4,       /* HIP reported an error at launch */
    SDL_ERR_NOMEM = -5,        /* host allocation failed (plan, engine); no free staging slot (offload) */
    SDL_ERR_TOO_LARGE = -6     /* input exceeds the fixed capacity of an allocation-free entry point */
} sdl_status_t;

/* Exchange format of the outer gradients (Section 2.4: lower precision for the
 * exchanged outer gradients, down to a 4-bit float with 1 sign, 3 exponent and 0
 * mantissa bits; Section 3.3.3 ablates float32 down to float4).
 *   SDL_FMT_FP32  no quantisation, 4 bytes / element, no scales
 *   SDL_FMT_BF16  round-to-nearest-even bfloat16, 2 bytes / element, no scales
 *   SDL_FMT_E4M3  OCP FP8 E4M3 (bias 7, max 448, saturating), 1 byte / element,
 *                 plus one power-of-two scale byte per 32 elements
 *   SDL_FMT_E3M0  code = s<<3 | E, magnitude 0 for E = 0 else 2^(E-3); two codes per
 *                 byte (element 2j in the low nibble of byte j); plus one scale byte
 *                 per 32 elements
 * Scale byte sb means 2^(sb-127); it is chosen from the block's absolute maximum a
 * as sb = max(0, biased_exponent(a) - emax) with emax = 4 (E3M0) or 8 (E4M3), 0 if
 * a is zero or subnormal.  Elements are rounded to the nearest representable
 * magnitude of |x| / 2^(sb-127) in the linear domain, ties to the even code,
 * saturating at the largest magnitude.
 *
 * E3M0 with another scale granularity (the element codes and their packing are the same):
 *   SDL_FMT_E3M0_B64 / _B128   one scale byte per 64 / 128 elements
 *   SDL_FMT_E3M0_SPAN          one scale for the whole span (per tensor): exactly the 4 bits
 *                              per parameter of the paper's accounting of exchanged data.  The
 *                              scale array of a span is one 4-byte word (4-byte aligned): the
 *                              fp32 bit pattern of the span's absolute maximum, from whose
 *                              exponent field the scale byte follows as above.  It is produced
 *                              by an extra pass over g and w_send (a grid-wide maximum).
 * E3M0 with the other choice of scale (Section 2.4 is silent on scaling; codes, packing and 32-element
 * blocks as SDL_FMT_E3M0):
 *   SDL_FMT_E3M0_RN            emax = 3: the scale is one binade higher, so the block maximum a falls
 *                              into [8, 16) of the code grid and is rounded to nearest like every other
 *                              element (to 2^floor(log2 a) or twice that) instead of always saturating
 *                              downwards; one binade less at the small end.  The smaller error of the
 *                              decoded mean on heavy-tailed outer gradients. */
typedef enum { SDL_FMT_FP32 = 0, SDL_FMT_BF16 = 1, SDL_FMT_E4M3 = 2, SDL_FMT_E3M0 = 3,
               SDL_FMT_E3M0_B64 = 4, SDL_FMT_E3M0_B128 = 5, SDL_FMT_E3M0_SPAN = 6, SDL_FMT_E3M0_RN = 7 } sdl_format_t;

/* Fragment patterns of Section 2.2: interleaved blocks (default) or consecutive blocks. */
typedef enum { SDL_PATTERN_STRIDED = 0, SDL_PATTERN_SEQUENTIAL = 1 } sdl_pattern_t;

/* A contiguous piece of the flat model that belongs to one fragment.
 * unit = index of its (first) parameter group in the caller's unit list. */
typedef struct { uint64_t offset; uint64_t numel; int32_t unit; } sdl_span_t;

typedef struct sdl_plan sdl_plan_t;   /* opaque, host memory, immutable after creation */

/* ------------------------------------------------------------------ plan (host only)
 *
 * Section 2.2 and the Require list of Algorithm 2: the model's transformer blocks
 * are partitioned into P fragments; fragment p has a synchronisation offset t_p; the
 * overlap delay tau is smaller than H.
 *
 * The model is a flat array made of n_units parameter groups in the given order;
 * unit u has unit_numel[u] elements and belongs to block unit_block[u] in
 * [0, n_blocks), or to SDL_UNIT_PRE / SDL_UNIT_POST, which travel with the fragment
 * of block 0 / block n_blocks-1.  Strided: block i -> fragment i mod P.  Sequential:
 * fragment p owns blocks [floor(p*L/P), floor((p+1)*L/P)).  t_p == NULL selects
 * t_p = floor(p*H/P); otherwise t_p[p] < H is required.
 *
 * Schedule (Algorithm 2's two conditions, with Section 2.2's rule that a fragment
 * always does H inner steps first): fragment p sends at t = t_p + k*H and receives
 * at t = t_p + k*H + tau, k = 1, 2, ...
 *
 * Errors: SDL_ERR_INVALID_ARG for P == 0, P > n_blocks, H == 0, tau >= H, a block
 * index out of range, an offset >= H, NULL arrays; SDL_ERR_NOMEM.  *out is set only
 * on success and must be released with sdl_plan_destroy. */
int sdl_fragment_plan(const uint64_t* unit_numel, const int32_t* unit_block, uint32_t n_units,
                      uint32_t n_blocks, uint32_t P, sdl_pattern_t pattern, uint32_t H, uint32_t tau,
                      const uint32_t* t_p, sdl_plan_t** out);
/* The same with options.  SDL_PLAN_PRE_OWN_FRAGMENT: the SDL_UNIT_PRE groups (the embedding)
 * form fragment 0 by themselves and the blocks are partitioned into fragments 1..P, so the
 * plan has P + 1 fragments (t_p, if given, has P + 1 entries; the default is
 * floor(p*H/(P+1))).  This is the layout the appendix's fragment counts imply (three layers
 * per fragment give 8 / 16 / 36 block fragments and a synchronisation every 11 / 5 / 2 steps,
 * i.e. H / (fragments + 1)). */
#define SDL_PLAN_PRE_OWN_FRAGMENT 1u
/* SDL_PLAN_ALIGN_GROUPS (a memory-layout option, not part of the method): every parameter group
 * starts at the next multiple of SDL_PLAN_GROUP_ALIGN elements of the flat arrays, i.e. on a
 * 128-byte boundary of the bf16 replicas when their bases are 128-byte aligned, which is what
 * the kernels need for full speed whatever the group sizes are.  The spans' offsets and
 * sdl_plan_total_numel then include the padding; padding elements belong to no fragment and
 * are never read or written.  The caller lays its flat arrays out by the spans' offsets. */
#define SDL_PLAN_ALIGN_GROUPS 2u
#define SDL_PLAN_GROUP_ALIGN 64u
int sdl_fragment_plan_ex(const uint64_t* unit_numel, const int32_t* unit_block, uint32_t n_units,
                         uint32_t n_blocks, uint32_t P, sdl_pattern_t pattern, uint32_t H, uint32_t tau,
                         const uint32_t* t_p, uint32_t flags, sdl_plan_t** out);
void sdl_plan_destroy(sdl_plan_t* plan);

uint32_t sdl_plan_num_fragments(const sdl_plan_t* plan);
uint64_t sdl_plan_total_numel(const sdl_plan_t* plan);
/* Fragment that owns transformer block `block`; negative status on bad arguments. */
int sdl_plan_block_fragment(const sdl_plan_t* plan, uint32_t block);
/* One span per parameter group of fragment p, in model order.  The array belongs to
 * the plan. */
int sdl_plan_fragment_spans(const sdl_plan_t* plan, uint32_t p, const sdl_span_t** spans,
                            uint32_t* n_spans);
/* The same elements as maximal contiguous runs: neighbouring spans are joined when
 * that leaves every 32-element scale block where it was (all joined spans but the
 * last have a multiple of 128 elements).  Processing the runs instead of the spans
 * gives identical results with fewer launches.  (Joining happens at multiples of 128
 * elements, the largest scale block, so it is valid for every block-scaled format.) */
int sdl_plan_fragment_runs(const sdl_plan_t* plan, uint32_t p, const sdl_span_t** runs,
                           uint32_t* n_runs);
int sdl_plan_offset(const sdl_plan_t* plan, uint32_t p, uint32_t* t_p);
/* Fragments that send / receive at inner step t >= 1, ascending p.  send and recv are
 * caller arrays of capacity P (either may be NULL together with its counter). */
int sdl_plan_events(const sdl_plan_t* plan, uint64_t t, uint32_t* send, uint32_t* n_send,
                    uint32_t* recv, uint32_t* n_recv);

/* Bytes of one replica's message for numel elements: returns code_bytes + scale_bytes
 * and stores the two parts when the pointers are not NULL (0 for an unknown format). */
size_t sdl_exchange_bytes(sdl_format_t fmt, uint64_t numel, size_t* code_bytes, size_t* scale_bytes);

/* ------------------------------------------------------------------ device calls */

/* Send side (Algorithm 2, the first conditional: the step at which fragment p is due; Section 2.4): for every
 * replica m, delta_m[i] = g[i] - float(w_send[m][i]) (one fp32 subtraction), encoded
 * in fmt into codes[m] (and scales[m] for E4M3 / E3M0).
 *   g        device, fp32[n], read
 *   w_send   host array of M device pointers to bf16[n], read
 *   codes    host array of M device pointers, code_bytes each, written
 *   scales   host array of M device pointers, scale_bytes each, written; may be
 *            NULL for FP32 / BF16 */
int sdl_quantize_outer_grad(const float* g, const void* const* w_send, uint32_t M, uint64_t n,
                            sdl_format_t fmt, void* const* codes, void* const* scales, void* stream);

/* Receive side (Algorithm 2, the second conditional: tau steps after the send; Section 2.4:
 * FP32 accumulation of the received outer gradients; Section 2.1: OuterOpt is SGD with Nesterov
 * momentum):
 *   d[i]   = (sum over m = 0..M-1, in that order, starting from +0, of decode_m[i]) / M
 *   mom[i] = mu * mom[i] + d[i]
 *   g[i]   = g[i] - lr * (d[i] + mu * mom[i])          (new mom)
 * each operation rounded once to fp32.  g and mom (device, fp32[n]) are updated in
 * place. */
int sdl_dequant_reduce_nesterov(float* g, float* mom, const void* const* codes,
                                const void* const* scales, uint32_t M, uint64_t n, sdl_format_t fmt,
                                float lr, float mu, void* stream);

/* Merge (last statement of Algorithm 2; Section 2.3): for every replica m,
 *   w_now[m][i] = bf16_rne(alpha * float(w_now[m][i]) + (1 - alpha) * g_new[i])
 * with 1 - alpha formed once in fp32.  alpha = 1 keeps the replica, alpha = 0
 * replaces it by the new global parameters.  w_now[m]: device bf16[n], in place. */
int sdl_merge_overlap(const float* g_new, void* const* w_now, uint32_t M, uint64_t n, float alpha,
                      void* stream);

/* Receive side in one pass (Algorithm 2, everything under the second conditional: receive, OuterOpt
 * and the mixing statement; Section 2.3): sdl_dequant_reduce_nesterov followed by sdl_merge_overlap of all
 * M replicas, without re-reading the new global parameters (16 + 4M + M*c bytes per parameter
 * instead of 20 + 4M + M*c).  Use it when every worker merges at the step the mean is taken
 * (one common delay tau); results are identical to the two separate calls. */
int sdl_receive_outer_step(float* g, float* mom, const void* const* codes, const void* const* scales,
                           void* const* w_now, uint32_t M, uint64_t n, sdl_format_t fmt, float lr, float mu,
                           float alpha, void* stream);

/* Fused outer step of one span: the three calls above in a single pass over memory,
 * with the messages kept in registers.  g, mom and w_now[m] are updated in place;
 * w_send[m] (the replica as it was at the send step) is only read and may be the same
 * pointer as w_now[m] for all m.  If codes_or_null is not NULL the messages are also
 * written out exactly as sdl_quantize_outer_grad would (scales_or_null then must be
 * given for the scaled formats).  SDL_FMT_E3M0_SPAN always needs scales_or_null: M device
 * pointers to one 4-byte scale word each, used as workspace even when no message is written. */
int sdl_fragment_outer_step(float* g, float* mom, const void* const* w_send, void* const* w_now,
                            uint32_t M, uint64_t n, sdl_format_t fmt, float lr, float mu, float alpha,
                            void* const* codes_or_null, void* const* scales_or_null, void* stream);

/* Fused outer step of a whole fragment of a plan: every run of fragment p, in one
 * kernel launch per group of up to 16 runs.  The pointers are the bases of the flat model arrays
 * (element 0 of the model); run r is processed at element offset runs[r].offset.
 * Messages are not written.  SDL_FMT_E3M0_SPAN is not supported here (SDL_ERR_UNSUPPORTED): it needs the
 * scale words that the _ex form below takes. */
int sdl_fragment_outer_step_plan(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                 const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                 sdl_format_t fmt, float lr, float mu, float alpha, void* stream);

/* The same with the optional outputs of sdl_fragment_outer_step: if codes_or_null is given the
 * fragment's messages are also written, laid out as sdl_quantize_outer_grad_plan writes them
 * (sdl_plan_message_bytes per replica); SDL_FMT_E3M0_SPAN is supported when scales_or_null is
 * given (M device pointers, one 4-byte word per span of the fragment each: workspace, and the
 * scale part of the messages). */
int sdl_fragment_outer_step_plan_ex(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                    const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                    sdl_format_t fmt, float lr, float mu, float alpha, void* const* codes_or_null,
                                    void* const* scales_or_null, void* stream);

/* sdl_fragment_outer_step_plan for callers that can neither allocate device memory nor hand over
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid allocation.
 * Same arguments, arithmetic and results as sdl_fragment_outer_step_plan_ex without message output;
 * unlike sdl_fragment_outer_step_plan it also takes SDL_FMT_E3M0_SPAN, whose scale words (one per
 * span and replica, the grid-wide maxima of the pre-pass) then live in a device array that is part
 * of the library image: SDL_STATIC_MAX_SPANS * SDL_MAX_WORKERS 4-byte words (64 KiB) per GPU, held
 * until the process ends.  The call allocates and frees nothing, on the host or on the device.
 *   - A fragment with more than SDL_STATIC_MAX_SPANS spans gives SDL_ERR_TOO_LARGE for
 *     SDL_FMT_E3M0_SPAN (the other formats use no scratch and have no limit); nothing is launched.
 *   - The array keeps the previous call's contents; every call clears the words it uses with a
 *     fill kernel (no memset node) before the maxima are taken.
 *   - All calls on one GPU share the array: two calls with SDL_FMT_E3M0_SPAN that overlap in time
 *     on the same GPU (different streams, or graphs replayed concurrently) race.  Calls on one
 *     stream are ordered and safe.
 *   - The array's device address is looked up at the first call on each device (current device =
 *     the device of `stream`); make that first call outside graph capture. */
#define SDL_STATIC_MAX_SPANS 1024
int sdl_fragment_outer_step_plan_static(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                        const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                        sdl_format_t fmt, float lr, float mu, float alpha, void* stream);

/* Fragment-level forms of the send-side and receive-side calls (Section 2.2: what is synchronised at a
 * step is a fragment, a subset of the transformer blocks, not the whole model): every run of fragment p
 * of a plan, on the flat model arrays (bases = element 0 of the model).  The messages of a
 * fragment are laid out as the concatenation of its runs, each run padded to a multiple
 * of 512 elements; sdl_plan_message_bytes gives the size of codes[m] / scales[m] for that
 * layout.  For SDL_FMT_E3M0_SPAN the pieces are the fragment's spans (parameter groups)
 * instead of the joined runs, and scales[m] holds one 4-byte word per span.  Argument
 * meaning, arithmetic and errors as in the span-level calls above. */
int sdl_plan_message_bytes(const sdl_plan_t* plan, uint32_t p, sdl_format_t fmt, size_t* code_bytes,
                           size_t* scale_bytes);
int sdl_quantize_outer_grad_plan(const sdl_plan_t* plan, uint32_t p, const float* g_base,
                                 const void* const* w_send_base, uint32_t M, sdl_format_t fmt,
                                 void* const* codes, void* const* scales, void* stream);
int sdl_dequant_reduce_nesterov_plan(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                     const void* const* codes, const void* const* scales, uint32_t M,
                                     sdl_format_t fmt, float lr, float mu, void* stream);
int sdl_merge_overlap_plan(const sdl_plan_t* plan, uint32_t p, const float* g_new_base, void* const* w_now_base,
                           uint32_t M, float alpha, void* stream);
int sdl_receive_outer_step_plan(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                const void* const* codes, const void* const* scales, void* const* w_now_base,
                                uint32_t M, sdl_format_t fmt, float lr, float mu, float alpha, void* stream);

/* ------------------------------------------------------------------ schedule driver
 *
 * Algorithm 2 as a whole, seen from the outer optimizer: the caller runs the inner steps
 * (its own training code updates the M replicas in place) and calls sdl_engine_step(t)
 * after the inner update of step t = 1, 2, ...  The engine issues, on `stream`,
 *   - for every fragment that sends at t (t = t_p + k*H): sdl_quantize_outer_grad_plan into
 *     that fragment's message buffers (the exchange between workers would happen here);
 *   - tau steps later: sdl_dequant_reduce_nesterov_plan, then sdl_merge_overlap_plan into
 *     the replicas as they are then (Section 2.3) -- as the single pass
 *     sdl_receive_outer_step_plan when all workers share one delay;
 *   - with tau = 0 for every worker: sdl_fragment_outer_step_plan_ex at the send step.
 * tau_m[m] < H is worker m's delay (Section 3.3.2: workers may receive the same update at
 * different steps); the mean and the Nesterov update happen once, at the smallest delay,
 * and each worker merges when its own delay expires.
 * The plan must outlive the engine.  H must be the H the plan was built with.  Steps must
 * be fed in order without gaps: a step that finds a send, receive or merge of an earlier step
 * undone is refused with SDL_ERR_INVALID_ARG before anything is launched.  SDL_ERR_DEVICE (a launch
 * or copy failed) can come after earlier fragments of the same step were launched; the engine's
 * state is then undefined and it must be destroyed.
 * sdl_engine_bind: g_base, mom_base, w_base[M] = flat device arrays (the live replicas);
 * codes / scales = host arrays of P*M device pointers, entry p*M + m sized by
 * sdl_plan_message_bytes(plan, p, ...); both may be NULL when every delay is 0 (except that
 * SDL_FMT_E3M0_SPAN always needs scales: its scale words are workspace of the fused call).
 * n_sent / n_received (optional) count the fragments whose send / mean+Nesterov ran. */
typedef struct sdl_engine sdl_engine_t;
int sdl_engine_create(const sdl_plan_t* plan, uint32_t H, uint32_t M, const uint32_t* tau_m, sdl_format_t fmt,
                      float lr, float mu, float alpha, sdl_engine_t** out);
void sdl_engine_destroy(sdl_engine_t* engine);
int sdl_engine_bind(sdl_engine_t* engine, float* g_base, float* mom_base, void* const* w_base,
                    void* const* codes, void* const* scales);
int sdl_engine_step(sdl_engine_t* engine, uint64_t t, void* stream, uint32_t* n_sent, uint32_t* n_received);

/* ------------------------------------------------------------------ outer state in host memory
 *
 * Section 2.5: only the fragment being synchronised needs its outer parameters and Nesterov
 * state in HBM (two words per parameter of the fragment); the rest can live in host memory,
 * and because the schedule is known in advance a fragment can be copied in ahead of time.
 *
 * "Staged" forms of the fragment-level calls: g_frag / mom_frag point at a device buffer that
 * holds only fragment p, its runs back to back, each padded to a multiple of 512 elements
 * (sdl_plan_staged_numel elements in all); the replicas stay flat model arrays. */
uint64_t sdl_plan_staged_numel(const sdl_plan_t* plan, uint32_t p);
int sdl_fragment_outer_step_staged(const sdl_plan_t* plan, uint32_t p, float* g_frag, float* mom_frag,
                                   const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                   sdl_format_t fmt, float lr, float mu, float alpha, void* stream);
int sdl_fragment_outer_step_staged_ex(const sdl_plan_t* plan, uint32_t p, float* g_frag, float* mom_frag,
                                      const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                      sdl_format_t fmt, float lr, float mu, float alpha, void* const* codes_or_null,
                                      void* const* scales_or_null, void* stream);
int sdl_quantize_outer_grad_staged(const sdl_plan_t* plan, uint32_t p, const float* g_frag,
                                   const void* const* w_send_base, uint32_t M, sdl_format_t fmt,
                                   void* const* codes, void* const* scales, void* stream);
int sdl_dequant_reduce_nesterov_staged(const sdl_plan_t* plan, uint32_t p, float* g_frag, float* mom_frag,
                                       const void* const* codes, const void* const* scales, uint32_t M,
                                       sdl_format_t fmt, float lr, float mu, void* stream);
int sdl_merge_overlap_staged(const sdl_plan_t* plan, uint32_t p, const float* g_new_frag, void* const* w_now_base,
                             uint32_t M, float alpha, void* stream);
int sdl_receive_outer_step_staged(const sdl_plan_t* plan, uint32_t p, float* g_frag, float* mom_frag,
                                  const void* const* codes, const void* const* scales, void* const* w_now_base,
                                  uint32_t M, sdl_format_t fmt, float lr, float mu, float alpha, void* stream);

/* The staging pool.  g_host / mom_host: the whole model's outer parameters and momentum in
 * host memory (flat layout; pinned memory makes the copies asynchronous).  slot_g / slot_mom:
 * n_slots device buffers of sdl_offload_slot_numel() floats each, 16-byte aligned.  All
 * memory is the caller's.
 *   prefetch  starts the host-to-device copy of fragment p into a free slot on copy_stream
 *             (SDL_ERR_NOMEM if every slot is taken; no-op if p is already staged)
 *   acquire   make compute_stream wait for the copy and return the slot; a fragment that is not staged
 *             yet is copied into a free slot, else into the slot of a fragment that was prefetched but
 *             never acquired (that copy is dropped: it holds nothing the host arrays do not);
 *             SDL_ERR_NOMEM only if every slot is held by an acquired fragment
 *   release   after the work queued on compute_stream: copy the fragment back to the host
 *             arrays on copy_stream and free the slot
 *   flush     write every staged fragment back without freeing its slot (checkpointing)
 * The same copy_stream must be used for all calls on one pool (write-back and the next
 * copy-in of a slot are ordered by it).  Host arrays are valid after the copy stream has
 * been synchronised.  sdl_engine_bind_offload makes an engine take g / mom from the pool
 * instead of flat device arrays; it prefetches the fragments that send within `lookahead`
 * steps, in the order of their send steps.  The pool needs one slot for every fragment that can be
 * between its send step and its last merge at the same time (offsets, H and the largest delay decide;
 * one slot when no worker has a delay); fewer give SDL_ERR_INVALID_ARG here, so that a step never
 * runs out of slots half way. */
typedef struct sdl_offload sdl_offload_t;
int sdl_offload_create(const sdl_plan_t* plan, uint32_t n_slots, sdl_offload_t** out);
void sdl_offload_destroy(sdl_offload_t* pool);
uint64_t sdl_offload_slot_numel(const sdl_offload_t* pool);
uint32_t sdl_offload_num_slots(const sdl_offload_t* pool);
int sdl_offload_bind(sdl_offload_t* pool, float* g_host, float* mom_host, float* const* slot_g,
                     float* const* slot_mom);
int sdl_offload_resident(const sdl_offload_t* pool, uint32_t p);
int sdl_offload_prefetch(sdl_offload_t* pool, uint32_t p, void* copy_stream);
int sdl_offload_acquire(sdl_offload_t* pool, uint32_t p, void* compute_stream, void* copy_stream,
                        float** g_frag, float** mom_frag);
int sdl_offload_release(sdl_offload_t* pool, uint32_t p, void* compute_stream, void* copy_stream);
int sdl_offload_flush(sdl_offload_t* pool, void* compute_stream, void* copy_stream);
int sdl_engine_bind_offload(sdl_engine_t* engine, sdl_offload_t* pool, void* const* w_base, void* const* codes,
                            void* const* scales, void* copy_stream, uint32_t lookahead);

/* ---- Diagnostics: cosine similarity between the replicas' outer gradients ----------
 *
 * Appendix, paragraph on the outer gradients' cosine similarity (figures per model scale, for
 * the embedding, for everything else, and per transformer layer).  For one set of parameters
 * and M replicas:
 *     Delta_m   = g - float(w[m])                  fp32, Algorithm 2's outer gradient
 *     G[a][b]   = sum_i Delta_a[i] * Delta_b[i]    fp64 products and sums
 *     cos[a][b] = G[a][b] / (sqrt(G[a][a]) * sqrt(G[b][b])),  0 when either norm is 0
 *     mean      = average of cos[a][b] over the pairs a < b (0 when M == 1)
 * A result is SDL_COSINE_RESULT_DOUBLES(M) = 2*M*M + 1 doubles in device memory: G (row
 * major), then cos (row major), then mean.  Summation order is fixed by the sizes alone, so a
 * call is reproducible bit for bit; it differs from a sequential sum by fp64 rounding only.
 * Reads 4 + 2*M bytes per parameter and writes nothing but the result.
 *
 * workspace: device memory of at least sdl_cosine_workspace_bytes(M, n_sets) bytes, 8-byte
 * aligned, owned by the caller, contents irrelevant before and after the call.
 * Errors: SDL_ERR_INVALID_ARG (null pointer, M == 0 or > SDL_MAX_WORKERS, workspace too
 * small, p out of range), SDL_ERR_ALIGNMENT (result or workspace not 8-byte aligned),
 * SDL_ERR_DEVICE (launch failure).  numel == 0 gives G = 0, cos = 0, mean = 0. */
#define SDL_COSINE_RESULT_DOUBLES(M) (2u * (M) * (M) + 1u)
size_t sdl_cosine_workspace_bytes(uint32_t M, uint32_t n_sets);

/* One set: the numel parameters at g, w[m] (device pointers; w[m] bf16). */
int sdl_outer_grad_cosine(const float* g, const void* const* w, uint32_t M, uint64_t numel, double* result,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Fragment p of a plan, on the flat model at g_base / w_base[m]: one result per span of the
 * fragment (= per transformer layer, embedding or head; order and units as
 * sdl_plan_fragment_spans reports them) in span_results[n_spans][2*M*M+1], and the result of
 * the whole fragment in fragment_result[2*M*M+1].  span_results may be null. */
int sdl_outer_grad_cosine_plan(const sdl_plan_t* plan, uint32_t p, const float* g_base, const void* const* w_base,
                               uint32_t M, double* span_results, double* fragment_result, void* workspace,
                               size_t workspace_bytes, void* stream);

/* Result of the union of n_sets disjoint parameter sets from their results (device memory,
 * results[k] at results + k * stride_doubles): the Gram matrices add, cos and mean follow.
 * This is how the result for all fragments but the embedding is formed from per-fragment or per-span
 * results.  Needs no workspace. */
int sdl_cosine_combine(const double* results, uint64_t stride_doubles, uint32_t n_sets, uint32_t M, double* result,
                       void* stream);

/* Cosine similarity inside the schedule driver: after this call, every send of fragment p
 * first runs sdl_outer_grad_cosine_plan on the outer gradients that are about to be sent (the
 * curves of the appendix are this, recorded over training).  fragment_results: device memory,
 * P results of 2*M*M + 1 doubles, result p rewritten at every send of fragment p;
 * span_results: NULL, or a host array of P device pointers (entries may be NULL) to
 * n_spans(p) results each; workspace: device memory, at least the largest
 * sdl_cosine_workspace_bytes(M, n_spans(p)) over the fragments, shared by all sends (they run
 * on one stream).  fragment_results == NULL switches the diagnostics off.  Not available while
 * the outer state is offloaded (sdl_engine_step then returns SDL_ERR_UNSUPPORTED). */
int sdl_engine_track_cosine(sdl_engine_t* engine, double* const* span_results, double* fragment_results,
                            void* workspace, size_t workspace_bytes);

/* ---- Parameters handed to evaluation -------------------------------------------------
 *
 * Appendix, paragraph "Which parameters to evaluate": the first replica, the average of all
 * replicas, or the outer parameters (whose fragments were synchronised at different steps).
 * out_bf16[i], in the model's storage type, is
 *     SDL_EVAL_FIRST_REPLICA   w[0][i]
 *     SDL_EVAL_REPLICA_MEAN    bf16( (((0 + float(w[0][i])) + float(w[1][i])) + ...) / float(M) ), fp32, RNE
 *     SDL_EVAL_OUTER           bf16( g[i] ), RNE
 * g (device, fp32) is only read for SDL_EVAL_OUTER and may be NULL otherwise; w (host array of
 * M device pointers, bf16) is only read for the other two and may be NULL for SDL_EVAL_OUTER.
 * out_bf16: device memory, numel bf16 values, owned by the caller; it must not overlap an input
 * it is not identical to.  Any numel and 2-/4-byte alignment (full speed from 128-byte aligned
 * arrays).  Errors: SDL_ERR_INVALID_ARG (bad selector, M out of range, missing pointer),
 * SDL_ERR_ALIGNMENT, SDL_ERR_UNSUPPORTED (numel above 2^40), SDL_ERR_DEVICE. */
typedef enum { SDL_EVAL_FIRST_REPLICA = 0, SDL_EVAL_REPLICA_MEAN = 1, SDL_EVAL_OUTER = 2 } sdl_eval_params_t;
int sdl_evaluation_params(sdl_eval_params_t which, const float* g, const void* const* w, uint32_t M, uint64_t numel,
                          void* out_bf16, void* stream);

/* Where to put the flat model arrays (a memory-layout aid, not part of the method).  The calls take
 * any pointers, but their speed depends on how the arrays lie relative to each other: on MI355X the
 * fused step over 2 + 2M arrays that were allocated one by one (every base on its own 2 MiB-aligned
 * allocation) was measured 2-6 % slower than over the same arrays carved from ONE allocation, and
 * another 1-2 % is gained when successive bases are staggered by 32 KiB on top of their 2 MiB-aligned
 * slots (the effect repeats with a period of 64 KiB).  sdl_flat_layout gives such a carving:
 * offsets[k], in bytes from a 2 MiB-aligned base, for k = g, mom, w_send[0..M), then, if
 * separate_w_now is not 0, w_now[0..M); total_bytes = size of the allocation.  fp32 arrays hold
 * total_numel * 4 bytes, bf16 arrays total_numel * 2.  offsets must have room for 2 + M (or 2 + 2M)
 * entries.  Errors: SDL_ERR_INVALID_ARG (NULL, M out of range). */
#define SDL_LAYOUT_SLOT_ALIGN 2097152u
#define SDL_LAYOUT_STAGGER 32768u
int sdl_flat_layout(uint64_t total_numel, uint32_t M, int separate_w_now, uint64_t* offsets, uint64_t* total_bytes);

/* Memory-system yardsticks.  Not part of the method: they are what the achieved bandwidth of the
 * calls above is judged against.  nbytes is a multiple of 16, both pointers are 16-byte aligned.
 *   SDL_PROBE_COPY      plain device-to-device copy (2 * nbytes of traffic); also the kernel of known
 *                       size that the profiler's HBM counters are calibrated with
 *   SDL_PROBE_COPY_NT   the same copy with the non-temporal policy the method's kernels use
 *   SDL_PROBE_READ_NT   reads src and writes nothing (nbytes of traffic); dst must still point at 16
 *                       valid bytes (written only if the data spell one particular value)
 *   SDL_PROBE_FILL_NT   writes dst and reads nothing (nbytes of traffic); src is ignored
 * sdl_copy_bytes(dst, src, n, s) is sdl_memory_probe(SDL_PROBE_COPY, dst, src, n, s). */
typedef enum { SDL_PROBE_COPY = 0, SDL_PROBE_COPY_NT = 1, SDL_PROBE_READ_NT = 2, SDL_PROBE_FILL_NT = 3 } sdl_probe_t;
int sdl_memory_probe(sdl_probe_t kind, void* dst, const void* src, uint64_t nbytes, void* stream);
int sdl_copy_bytes(void* dst, const void* src, uint64_t nbytes, void* stream);

const char* sdl_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SDL_H */
