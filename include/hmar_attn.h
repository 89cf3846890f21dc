/* hmar_attn.h -- C ABI of the MI355X (gfx950) Markovian next-scale attention library.
 *
 * The operation is softmax attention under the mask of HMAR's Markovian next-scale
 * prediction (paper Sec. 3.1, Eq. 4; App. B.2): the sequence is the concatenation, coarse
 * to fine, of K scales with n_k = side_k^2 tokens each; a query of scale k attends to the
 * keys of scale k (bidirectionally) and of its immediate predecessor k-1, and to nothing
 * else.  Scale 1 attends to itself only.  The library evaluates it exactly, in the
 * FlashAttention manner the paper describes (Sec. 3.1 "I/O-aware windowed attention",
 * App. B.4): tiles of the masked score matrix that hold no allowed pair are never loaded.
 *
 * Conventions shared by every entry point
 *  - Tensors are DEVICE pointers, bf16, contiguous, layout [B, H, L, D] with D fastest,
 *    L = sum_k side_k^2, scales laid coarse to fine along L.  LSE is fp32 [B, H, L].
 *  - side_lens is a HOST pointer to num_scales int32 values.
 *  - D must be 64 (the only head dimension the paper uses, App. B.4).
 *  - sm_scale multiplies the raw scores q.k; a value <= 0 selects 1/sqrt(D).
 *  - The caller owns every buffer.  Inputs are not modified.  Outputs are fully
 *    overwritten and need no initialisation.  Buffers must not overlap.
 *  - Calls enqueue work on `stream` (a hipStream_t, may be null for the default stream)
 *    and return without synchronising.  A small per-schedule device table is built on the
 *    first use of a schedule on a device and cached for the life of the process (this is
 *    the only allocation the library makes; the cache is thread-safe).  That first use
 *    allocates and copies synchronously: make it outside a HIP stream capture; later calls
 *    with the same schedule only launch kernels and may be captured into a graph.
 *  - Errors are return codes.  Argument checks happen before any device work.
 *  - Inputs must be finite.  Rounding: products accumulate in fp32; the softmax
 *    probabilities (and, in the backward, dS) are rounded to bf16 before the second
 *    contraction, results are rounded to bf16 once at the end (round to nearest even).
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
    HMAR_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, misaligned pointer, L overflow */
    HMAR_ERR_UNSUPPORTED = 2, /* D != 64, num_scales or L beyond HMAR_MAX_*                  */
    HMAR_ERR_WORKSPACE = 3,   /* workspace null or smaller than hmar_attn_bwd_workspace_bytes */
    HMAR_ERR_HIP = 4          /* a HIP runtime call or kernel launch failed                   */
} hmar_status;

#define HMAR_MAX_SCALES 64
#define HMAR_MAX_SEQ_LEN (1 << 20)

/* Human-readable name of a status code (static storage, never null). */
const char* hmar_status_string(hmar_status s);

/* Forward pass (paper Sec. 3.1; App. B.4 forward benchmark).
 *   O[b,h,i,:]  = sum_j P_ij V[b,h,j,:],  P = softmax over the allowed keys j of
 *                 sm_scale * Q[b,h,i,:].K[b,h,j,:]
 *   LSE[b,h,i]  = natural log of sum_j exp(sm_scale * q_i.k_j) over the allowed keys
 * Q, K, V: device bf16 [B,H,L,D] (in).  O: device bf16 [B,H,L,D] (out).
 * LSE: device fp32 [B,H,L] (out).  All device pointers 16-byte aligned. */
hmar_status hmar_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                          const int32_t* side_lens, int32_t num_scales,
                          int32_t B, int32_t H, int32_t D, float sm_scale, void* stream);

/* The same forward under a chosen mask.  HMAR_MASK_MARKOV is the mask above;
 * HMAR_MASK_BLOCK_CAUSAL is VAR's block-causal mask (paper Sec. 2, App. B.2: scale k attends
 * to every scale <= k, bidirectionally inside a scale), the pattern the paper's
 * micro-benchmark (App. B.4) compares against.  Everything else as hmar_attn_fwd. */
typedef enum { HMAR_MASK_MARKOV = 0, HMAR_MASK_BLOCK_CAUSAL = 1 } hmar_mask_kind;
/* May be OR-ed into the mask_kind argument of the *_masked entry points: side_lens then holds
 * the token count n_k of each scale itself instead of a side length, for token maps that are
 * not square (the paper's scales are H_k x W_k maps, Sec. 2: n_k = H_k * W_k).  Row order
 * inside a scale is the caller's business: attention inside a scale is bidirectional. */
#define HMAR_SCALE_COUNTS 0x100
hmar_status hmar_attn_fwd_masked(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                 const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                                 int32_t B, int32_t H, int32_t D, float sm_scale, void* stream);

/* One KV-cache-free inference step (paper Sec. 3.1, last paragraph; Sec. 5.2): the n_cur
 * tokens of the scale being generated attend to the n_prev tokens that stand for everything
 * before it and to themselves; nothing is cached between steps.
 * Q, O: device bf16 [B,H,n_cur,D]; K, V: device bf16 [B,H,n_prev+n_cur,D], predecessor block
 * first; LSE: device fp32 [B,H,n_cur].  n_prev >= 0 (0 for the first scale), n_cur >= 1.
 * Equals rows of hmar_attn_fwd restricted to one scale. */
hmar_status hmar_attn_step_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                               int32_t n_prev, int32_t n_cur, int32_t B, int32_t H, int32_t D,
                               float sm_scale, void* stream);

/* Bytes of device workspace hmar_attn_bwd needs for this problem (0 on invalid arguments).
 * The workspace holds two fp32 [B,H,L] arrays: -Delta_i = -sum_d dO_id O_id and -LSE_i*log2(e). */
size_t hmar_attn_bwd_workspace_bytes(const int32_t* side_lens, int32_t num_scales,
                                     int32_t B, int32_t H, int32_t D);

/* Backward pass (paper Sec. 3.1; App. B.4 backward benchmark): gradients of
 * sum(O * dO) with respect to Q, K, V, recomputing P from Q, K and LSE:
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

/* Measurement aid (used by the benchmark for the per-kernel roofline figures of paper
 * App. B.4-style timing): between hmar_profile_begin() and hmar_profile_end() every kernel
 * the library launches is bracketed by a pair of HIP events recorded on the launch stream.
 * hmar_profile_end() waits for those events and adds up, per kernel, the elapsed
 * milliseconds and the number of launches.  Kernel ids: 0 forward, 1 dK/dV, 2 dQ.
 * total_ms_out and launches_out are HOST arrays of HMAR_NUM_KERNELS entries (either may be
 * null).  Not thread-safe against concurrent launches; adds two event records per kernel. */
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
