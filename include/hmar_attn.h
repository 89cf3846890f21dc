/* hmar_attn.h -- C ABI of the MI355X (gfx950) Markovian next-scale attention library.
 *
 * The operation is softmax attention under the mask of HMAR's Markovian next-scale
 * prediction (paper Sec. "Efficient Markovian Next-Scale Prediction", Eq. 4; appendix
 * "Attention Patterns"): the sequence is the concatenation, coarse to fine, of K scales with
 * n_k = side_k^2 tokens each; a query of scale k attends to the keys of scale k
 * (bidirectionally) and of its immediate predecessor k-1, and to nothing else.  Scale 1
 * attends to itself only.  The library evaluates it exactly, in the FlashAttention manner the
 * paper describes (same section, IO-aware windowed attention; appendix "Efficient Attention
 * Performance"): tiles of the masked score matrix that hold no allowed pair are never loaded.
 *
 * Conventions shared by every entry point
 *  - Tensors are DEVICE pointers, bf16, contiguous, layout [B, H, L, D] with D fastest,
 *    L = sum_k side_k^2, scales laid coarse to fine along L.  LSE is fp32 [B, H, L].
 *  - side_lens is a HOST pointer to num_scales int32 values.
 *  - D must be 64 (the only head dimension the paper uses, appendix "Efficient Attention
 *    Performance").
 *  - sm_scale multiplies the raw scores q.k; a value <= 0 selects 1/sqrt(D).
 *  - The caller owns every buffer.  Inputs are not modified.  Outputs are fully
 *    overwritten and need no initialisation.  Buffers must not overlap.
 *  - Calls enqueue work on `stream` (a hipStream_t, may be null for the default stream)
 *    and return without synchronising.  For the training-shape entry points (hmar_attn_fwd*,
 *    hmar_attn_bwd*) a small per-schedule device table is built on the first use of a schedule
 *    on a device and cached for the life of the process (the cache is thread-safe; a later call
 *    with the same sizes costs one look-up).  That first use allocates and copies
 *    synchronously: make it outside a HIP stream capture; later calls with the same schedule
 *    only launch kernels and may be captured into a graph.  The inference-step entry points
 *    (hmar_attn_step*) never allocate, nor does hmar_attn_bwd_noalloc.
 *  - Errors are return codes.  Argument checks happen before any device work.
 *  - Inputs must be finite.  Rounding: products accumulate in fp32; the softmax
 *    probabilities (and, in the backward, dS) are rounded to bf16 before the second
 *    contraction, results are rounded to bf16 once at the end (round to nearest even).
 *  - Results are deterministic: no atomics, a fixed summation order per schedule.
 */
#ifndef HMAR_ATTN_H
#define HMAR_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HMAR_OK = 0,
    HMAR_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, misaligned pointer, unknown flag  */
    HMAR_ERR_UNSUPPORTED = 2, /* D != 64; num_scales, L, B*H or a step count beyond the HMAR_MAX_*
                                 limits (L includes every value that would not fit 32 bits)        */
    HMAR_ERR_WORKSPACE = 3,   /* workspace null or smaller than hmar_attn_bwd_workspace_bytes       */
    HMAR_ERR_HIP = 4          /* a HIP runtime call or kernel launch failed                         */
} hmar_status;

#define HMAR_MAX_SCALES 64
#define HMAR_MAX_SEQ_LEN (1 << 20)
#define HMAR_MAX_STEPS 1024          /* inference steps per hmar_attn_steps_fwd call */

/* Human-readable name of a status code (static storage, never null). */
const char* hmar_status_string(hmar_status s);

/* Forward pass (paper Sec. "Efficient Markovian Next-Scale Prediction"; appendix "Efficient
 * Attention Performance", forward benchmark).
 *   O[b,h,i,:]  = sum_j P_ij V[b,h,j,:],  P = softmax over the allowed keys j of
 *                 sm_scale * Q[b,h,i,:].K[b,h,j,:]
 *   LSE[b,h,i]  = natural log of sum_j exp(sm_scale * q_i.k_j) over the allowed keys
 * Q, K, V: device bf16 [B,H,L,D] (in).  O: device bf16 [B,H,L,D] (out).
 * LSE: device fp32 [B,H,L] (out).  All device pointers 16-byte aligned. */
hmar_status hmar_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                          const int32_t* side_lens, int32_t num_scales,
                          int32_t B, int32_t H, int32_t D, float sm_scale, void* stream);

/* The same forward under a chosen mask.  HMAR_MASK_MARKOV is the mask above;
 * HMAR_MASK_BLOCK_CAUSAL is VAR's block-causal mask (paper Sec. "Background", appendix
 * "Attention Patterns": scale k attends to every scale <= k, bidirectionally inside a scale),
 * the pattern the paper's micro-benchmark (appendix "Efficient Attention Performance")
 * compares against.  Everything else as hmar_attn_fwd. */
typedef enum { HMAR_MASK_MARKOV = 0, HMAR_MASK_BLOCK_CAUSAL = 1 } hmar_mask_kind;
/* May be OR-ed into the mask_kind argument of the *_masked entry points: side_lens then holds
 * the token count n_k of each scale itself instead of a side length, for token maps that are
 * not square (the paper's scales are H_k x W_k maps, Sec. "Background": n_k = H_k * W_k).
 * Row order inside a scale is the caller's business: attention inside a scale is
 * bidirectional. */
#define HMAR_SCALE_COUNTS 0x100
hmar_status hmar_attn_fwd_masked(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                 const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                                 int32_t B, int32_t H, int32_t D, float sm_scale, void* stream);

/* One KV-cache-free inference step (paper Sec. "Efficient Markovian Next-Scale Prediction",
 * last paragraph; Sec. "Efficiency"): the n_cur tokens of the scale being generated attend to
 * the n_prev tokens that stand for everything before it and to themselves; nothing is cached
 * between steps.
 * Q, O: device bf16 [B,H,n_cur,D]; K, V: device bf16 [B,H,n_prev+n_cur,D], predecessor block
 * first; LSE: device fp32 [B,H,n_cur].  n_prev >= 0 (0 for the first scale), n_cur >= 1.
 * Equals rows of hmar_attn_fwd restricted to one scale.  Allocates nothing, keeps no state. */
hmar_status hmar_attn_step_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                               int32_t n_prev, int32_t n_cur, int32_t B, int32_t H, int32_t D,
                               float sm_scale, void* stream);

/* Several independent inference steps in one launch (same passages): step i is
 * hmar_attn_step_fwd(Q[i], K[i], V[i], O[i], LSE[i], n_prev[i], n_cur[i], B, H, D, ...).
 * The coarse steps of a schedule hold a handful of tokens each and cost a launch apiece when
 * issued one by one; batched, the work of all steps is walked heaviest first by one grid.
 * Meant for requests that sit at different scales (continuous batching) and for timing a whole
 * schedule; the steps of ONE image depend on each other and cannot share a launch.
 * Q, K, V, O, LSE, n_prev, n_cur: HOST arrays of n_steps entries (device pointers / sizes as
 * above; every step has the same B, H, D).  1 <= n_steps <= HMAR_MAX_STEPS; up to 16 steps
 * share a kernel launch.  The buffers of different steps must not overlap. */
hmar_status hmar_attn_steps_fwd(const void* const* Q, const void* const* K, const void* const* V,
                                void* const* O, float* const* LSE,
                                const int32_t* n_prev, const int32_t* n_cur, int32_t n_steps,
                                int32_t B, int32_t H, int32_t D, float sm_scale, void* stream);

/* One refinement pass of the masked sampling inside a scale (paper Sec. "Hierarchical
 * Multi-Step Masked Generation", Eq. 6; appendix "Masked Sampling"): of the n_cur tokens of
 * the scale only the re-masked ones are predicted again, conditioned on the predecessor block
 * and on all tokens of the scale.  Only the n_rows query rows listed in `rows` are computed:
 *   for r in rows:  O[b,h,r,:], LSE[b,h,r] = attention of Q[b,h,r,:] over all n_prev+n_cur keys
 * Q, O, LSE keep their full step shapes ([B,H,n_cur,D], [B,H,n_cur]); rows of O and LSE that
 * are not listed are left untouched; K and V as in hmar_attn_step_fwd (the predecessor block's
 * n_prev rows are the same in every pass of a scale and stay where they are).
 * rows: DEVICE pointer, int32, n_rows distinct values in [0, n_cur), 4-byte aligned, shared by
 * all heads.  1 <= n_rows <= n_cur.  The values are device data and not checked: one outside
 * the range is clamped into it (no access leaves the buffers; what is written for such an
 * entry is unspecified).  Allocates nothing. */
hmar_status hmar_attn_step_fwd_rows(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                    const int32_t* rows, int32_t n_rows,
                                    int32_t n_prev, int32_t n_cur, int32_t B, int32_t H, int32_t D,
                                    float sm_scale, void* stream);

/* Bytes of device workspace hmar_attn_bwd needs for this problem (0 on invalid arguments).
 * The workspace holds two fp32 [B,H,L] arrays: -Delta_i = -sum_d dO_id O_id and -LSE_i*log2(e). */
size_t hmar_attn_bwd_workspace_bytes(const int32_t* side_lens, int32_t num_scales,
                                     int32_t B, int32_t H, int32_t D);

/* Backward pass (paper Sec. "Efficient Markovian Next-Scale Prediction"; appendix "Efficient
 * Attention Performance", backward benchmark): gradients of sum(O * dO) with respect to Q, K,
 * V, recomputing P from Q, K and LSE:
 *   dV = P^T dO;  dP = dO V^T;  dS = P o (dP - Delta);  dQ = sm_scale dS K;  dK = sm_scale dS^T Q
 * Q, K, V, O, dO: device bf16 [B,H,L,D] (in); LSE: device fp32 [B,H,L] (in, from the
 * forward).  dQ, dK, dV: device bf16 [B,H,L,D] (out).  workspace: device, 16-byte
 * aligned, at least hmar_attn_bwd_workspace_bytes(...) bytes, contents undefined after. */
hmar_status hmar_attn_bwd(const void* Q, const void* K, const void* V, const void* O,
                          const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                          const int32_t* side_lens, int32_t num_scales,
                          int32_t B, int32_t H, int32_t D, float sm_scale,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Workspace size for hmar_attn_bwd_masked with the same side_lens / mask_kind arguments (the
 * mask does not change it, HMAR_SCALE_COUNTS does: L = sum_k n_k).  0 on invalid arguments. */
size_t hmar_attn_bwd_workspace_bytes_masked(const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                                            int32_t B, int32_t H, int32_t D);

/* The same backward under a chosen mask (see hmar_attn_fwd_masked); workspace of at least
 * hmar_attn_bwd_workspace_bytes_masked(...) bytes. */
hmar_status hmar_attn_bwd_masked(const void* Q, const void* K, const void* V, const void* O,
                                 const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                                 const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                                 int32_t B, int32_t H, int32_t D, float sm_scale,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* hmar_attn_bwd for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments without the workspace, same results bit for bit.  The two fp32 [B,H,L] arrays and
 * the schedule tables live in a fixed array in the library's device image (about 8.2 MiB on
 * every GPU the library runs on, held until the process ends); the call makes no hipMalloc,
 * hipFree, memcpy or other allocating call: it only launches kernels.  Limits, beyond those of hmar_attn_bwd:
 *   B*H*L <= HMAR_NOALLOC_MAX_ROWS and L <= HMAR_NOALLOC_MAX_SEQ_LEN, else HMAR_ERR_UNSUPPORTED.
 * Every call on a GPU uses that GPU's one array, which keeps the last call's contents: calls
 * that overlap in time on one GPU (two streams, two threads) race; calls on one stream, or
 * ordered by events, are safe.  When the schedule differs from the previous call's on that GPU
 * its tables (a few KB) are first written to the array by small kernels on `stream`, their
 * contents carried in the kernel arguments.  A call made while `stream` is being captured into
 * a graph always records those writes, so that every replay brings its own tables; from then on
 * calls outside graphs write theirs every time as well (a replay may have changed the array).
 * The first call on a GPU looks up the array's address and must be made outside a capture.
 * Markovian mask, scales given by side lengths. */
#define HMAR_NOALLOC_MAX_ROWS (1 << 20)
#define HMAR_NOALLOC_MAX_SEQ_LEN 8192
hmar_status hmar_attn_bwd_noalloc(const void* Q, const void* K, const void* V, const void* O,
                                  const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                                  const int32_t* side_lens, int32_t num_scales,
                                  int32_t B, int32_t H, int32_t D, float sm_scale, void* stream);

/* Host-only description of a schedule (no device work): prefix sums off[0..num_scales]
 * of side^2 and the number of unmasked (query, key) pairs per head.  Either output
 * pointer may be null. */
hmar_status hmar_schedule_describe(const int32_t* side_lens, int32_t num_scales,
                                   int32_t* offsets_out, int64_t* allowed_pairs_out);

/* Host-only export of the tile work lists the kernels walk, for inspection and tests.
 *   which = 0: forward / dQ list (query-row ranges), 1: dK/dV list (key-row ranges);
 *   add 2 for the block-causal mask instead of the Markovian one, add 4 when side_lens holds
 *   token counts (see HMAR_SCALE_COUNTS).
 * Each item is 4 int32: {own_begin, own_end, other_begin, other_end}: the rows the
 * workgroup owns and the contiguous range of the other operand's rows it visits.
 * Writes up to max_items items to items_out (may be null) and the item count to
 * n_items_out.  row_lo_out / row_hi_out (each L int32, may be null) receive, per owned
 * row, the half-open range of the other operand's rows it may pair with. */
hmar_status hmar_schedule_tiles(const int32_t* side_lens, int32_t num_scales, int32_t which,
                                int32_t* items_out, int32_t max_items, int32_t* n_items_out,
                                int32_t* row_lo_out, int32_t* row_hi_out);

/* Measurement aid (not an operation of the paper): between hmar_profile_begin() and
 * hmar_profile_end() every kernel the library launches is bracketed by a pair of HIP events
 * recorded on the launch stream.  hmar_profile_end() waits for those events and adds up, per
 * kernel, the elapsed milliseconds and the number of launches.  Kernel ids: 0 forward (and
 * inference steps), 1 dK/dV, 2 dQ.  total_ms_out and launches_out are HOST arrays of
 * HMAR_NUM_KERNELS entries (either may be null).  One stream at a time: the first launch
 * after hmar_profile_begin() fixes the stream; launches on any other stream are not
 * recorded and make hmar_profile_end() return HMAR_ERR_INVALID_ARG.  Launches must not be
 * issued from several threads while profiling is on. */
#define HMAR_NUM_KERNELS 3
hmar_status hmar_profile_begin(void);
hmar_status hmar_profile_end(double* total_ms_out, int64_t* launches_out);

/* Measurement aid: a plain device-to-device copy kernel of `bytes` bytes (a multiple of 16;
 * dst and src device pointers, 16-byte aligned, not overlapping) on `stream`.  Its known
 * traffic (bytes read + bytes written) calibrates the HBM byte counters read with
 * rocprofv3 for the attention kernels. */
hmar_status hmar_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HMAR_ATTN_H */
