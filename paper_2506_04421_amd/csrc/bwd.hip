// Backward kernels of the Markovian next-scale attention (paper Sec. "Efficient Markovian Next-Scale Prediction", appendix "Efficient Attention Performance") for gfx950.
//
//   hmar_dq_kernel    : query-stationary, same walk as the forward but over the heads in reverse
//                       order (the forward before it and the dK/dV kernel after it both walk
//                       forwards, so each kernel begins where its predecessor ended).  First
//                       forms, for its own rows, -Delta_i = -sum_d dO_id O_id and
//                       -LSE_i * log2(e) and leaves them in the workspace for the dK/dV kernel
//                       (launched after it).  Recomputes P^T = exp(S^T - LSE), dP^T = V dO^T,
//                       dS^T = P^T o (dP^T - Delta) and accumulates dQ^T += K^T dS^T.
//   hmar_dkdv_kernel  : key-stationary, walks the transposed schedule (a key of scale k is
//                       seen by the queries of scales k and k+1).  Recomputes P and dS with
//                       the keys in the lane dimension and accumulates dV^T += dO^T P,
//                       dK^T += Q^T dS.
// Both main kernels recompute the probabilities, so no gradient is accumulated across
// workgroups: results are deterministic and nothing needs zero-initialising.  Streamed
// tiles are row-major in LDS and serve both as row-wise operands (S, dP) and, through the
// LDS transpose load, as transposed operands (dQ, dK, dV).
#include <algorithm>
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace hmar {

struct BwdParams {
    const __bf16* Q; const __bf16* K; const __bf16* V; const __bf16* dO;
    const __bf16* O; const float* LSE;
    float* neg_lse2;         // -LSE * log2(e): written by the dQ kernel, read by the dK/dV kernel
    float* neg_delta;        // -Delta: likewise
    __bf16* dQ; __bf16* dK; __bf16* dV;
    const Item* items; const int32_t* row_lo; const int32_t* row_hi;
    int n_items, n_heads, L;
    int tail_groups;  // see map_workgroup
    float c;          // sm_scale * log2(e)
    float sm_scale;
};

// ------------------------------------------------------------------------------------- dQ
#ifndef HMAR_DQ_MIN_WAVES
#define HMAR_DQ_MIN_WAVES 4
#endif
// -Delta of a row from the lane's half of it: each half-wave holds 32 of the row's 64 dO values
__device__ __forceinline__ float neg_delta_of_row(const __bf16* o_row, const bf16x8 (&dob)[4], int h) {
    float acc = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const bf16x8 ov = HMAR_ROW_LOAD(reinterpret_cast<const bf16x8*>(o_row + 16 * t + 8 * h));
        const bf16x8 gv = dob[t];
        // two products per instruction (v_dot2c_f32_bf16), fp32 accumulation
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(ov, ov, 0, 1), __builtin_shufflevector(gv, gv, 0, 1), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(ov, ov, 2, 3), __builtin_shufflevector(gv, gv, 2, 3), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(ov, ov, 4, 5), __builtin_shufflevector(gv, gv, 4, 5), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(ov, ov, 6, 7), __builtin_shufflevector(gv, gv, 6, 7), acc, false);
    }
    return -half_sum(acc);
}

// The work of one dQ item.  smem: ring of 2 stages, each a K tile followed by a V tile.
// OWN_STATS: form the row statistics here and leave them in the workspace (the shipped kernel);
// otherwise they are read from the workspace.
template <bool OWN_STATS>
__device__ __forceinline__ void dq_body(const BwdParams& p, const Item it, const int32_t* row_lo, const int32_t* row_hi,
                                        int head, int item_id, char* smem) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, h = lane >> 5;
    const size_t head_off = (size_t)head * p.L * kD;
    const size_t head_in = (size_t)HMAR_INPUT_HEAD(head) * p.L * kD;     // == head_off outside measurements
    const __bf16* Kh = p.K + head_in;
    const __bf16* Vh = p.V + head_in;
    const LaneOffsets lo_ = make_lane_offsets(lane, wave);
    const uint32_t smem_base = lds_address(smem);

    const int k_begin = it.other_begin, k_end = it.other_end, kmax = k_end - 1;
    const int ntiles = (k_end - k_begin + kTile - 1) / kTile;

    auto issue = [&](int ti, int st) {       // 4 DMA loads per lane and tile
        const uint32_t stage = smem_base + st * (2 * kTileBytes);
        dma_tile(Kh, k_begin + ti * kTile, kmax, stage, lo_, lane, wave);
        dma_tile(Vh, k_begin + ti * kTile, kmax, stage + kTileBytes, lo_, lane, wave);
    };
    issue(0, 0);

    const int wq0 = it.own_begin + wave * kRowsPerWave;
    const bool wave_active = wq0 < it.own_end;
    const int qrow = min(wq0 + lr, it.own_end - 1);
    const int lo = row_lo[qrow], hi = row_hi[qrow];
    // pair ranges never decrease along the rows: the wavefront's extremes are at its first and last row
    const int rfirst = min(wq0, it.own_end - 1), rlast = min(wq0 + kRowsPerWave - 1, it.own_end - 1);
    const int wlo = row_lo[rfirst], whi = row_hi[rlast];        // union of the wavefront's ranges
    const int full_lo = row_lo[rlast], full_hi = row_hi[rfirst];  // what every one of its rows pairs with

    bf16x8 q[4], dob[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        q[t] = HMAR_ROW_LOAD(reinterpret_cast<const bf16x8*>(p.Q + head_in + (size_t)qrow * kD + 16 * t + 8 * h));
        dob[t] = HMAR_ROW_LOAD(reinterpret_cast<const bf16x8*>(p.dO + head_in + (size_t)qrow * kD + 16 * t + 8 * h));
    }
    float nl2, ndelta;
    if constexpr (OWN_STATS) {
        nl2 = -p.LSE[(size_t)HMAR_INPUT_HEAD(head) * p.L + qrow] * kLog2e;
        ndelta = neg_delta_of_row(p.O + head_in + (size_t)qrow * kD, dob, h);
        if (wq0 + lr < it.own_end && h == 0) {
            p.neg_lse2[(size_t)head * p.L + qrow] = nl2;
            p.neg_delta[(size_t)head * p.L + qrow] = ndelta;
        }
    } else {
        nl2 = p.neg_lse2[(size_t)head * p.L + qrow];
        ndelta = p.neg_delta[(size_t)head * p.L + qrow];
    }

    f32x16 dq[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[mb][i] = 0.f;

    // make the compiler wait for these registers here, not inside the loop (see the forward);
    // loads complete in order, so tile 0 has landed as well
    asm volatile("" :: "v"(q[0]), "v"(q[1]), "v"(q[2]), "v"(q[3]), "v"(dob[0]), "v"(dob[1]), "v"(dob[2]),
                 "v"(dob[3]), "v"(nl2), "v"(ndelta));
    HMAR_WAIT_DMA_AND_BARRIER(0);

    // one tile: request the next one, compute, wait for the request; the stage is a template
    // constant so that every LDS address of the step is a per-lane register plus an immediate
    auto tile_step = [&](const int ti, auto stage_c) {
        constexpr int ST = decltype(stage_c)::value;
        const int kt = k_begin + ti * kTile;
        if (ti + 1 < ntiles) issue(ti + 1, ST ^ 1);
#ifdef HMAR_TUNE_NO_COMPUTE_DQ
        if (false) {
#else
        if (wave_active && kt < whi && kt + kTile > wlo) {
#endif
            const uint32_t Kt = smem_base + ST * (2 * kTileBytes);
            const uint32_t Vt = Kt + kTileBytes;
            const bool need_lo = kt < full_lo, need_hi = kt + kTile > full_hi;
            const int lim_lo = lo - kt - 4 * h, lim_hi = hi - kt - 4 * h;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                // (no explicit operand staging here: at 4 wavefronts per SIMD the extra
                // registers cost more in occupancy than the batched LDS reads gain)
                f32x16 s, dp;
#pragma unroll
                for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    s = mfma32(lds_a_row(Kt, lo_, kb, t), q[t], s);
                    dp = mfma32(lds_a_row(Vt, lo_, kb, t), dob[t], dp);
                }
                mask_block(s, 32 * kb, lim_lo, lim_hi, need_lo, need_hi);     // exp2(-inf) = 0
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], p.c, nl2));
                    s[i] = pv * (dp[i] + ndelta);
                }
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) {
                    const int e0 = 8 * sub, tp = 2 * kb + sub;
                    const bf16x8 dsb = pack8(s[e0 + 0], s[e0 + 1], s[e0 + 2], s[e0 + 3],
                                             s[e0 + 4], s[e0 + 5], s[e0 + 6], s[e0 + 7]);
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
                        dq[mb] = mfma32(lds_a_tr(Kt, lo_, mb, tp), dsb, dq[mb]);
                }
            }
        }
        HMAR_WAIT_DMA_AND_BARRIER(0);     // the tile requested above has landed and this one is free
    };
    for (int ti = 0; ti < ntiles; ti += 2) {
        tile_step(ti, std::integral_constant<int, 0>{});
        if (ti + 1 >= ntiles) break;
        tile_step(ti + 1, std::integral_constant<int, 1>{});
    }

    if (wave_active)
        store_block_rows(smem_base + wave * kPatchBytes, dq, p.sm_scale, p.dQ + head_off, wq0, it.own_end - wq0, lane, nullptr, HMAR_NT_GRADS != 0);
}

__global__ __launch_bounds__(kThreads, HMAR_DQ_MIN_WAVES) void hmar_dq_kernel(BwdParams p) {
    __shared__ __attribute__((aligned(1024))) char smem[2 * 2 * kTileBytes];
#ifdef HMAR_TUNE_LDS_PAD_DQ
    HMAR_TUNE_LDS_PAD(HMAR_TUNE_LDS_PAD_DQ)
#endif
    int head, item_id;
    if (!map_workgroup(p.n_items, p.n_heads, p.tail_groups, &head, &item_id, true)) return;
    dq_body<true>(p, p.items[item_id], p.row_lo, p.row_hi, head, item_id, smem);
}

// ---------------------------------------------------------------------------------- dK, dV
// Register budget: the two result accumulators, the own K and V rows, both blocks' scores and
// the batched LDS operands need about 250 VGPRs, which means two wavefronts per SIMD (two
// workgroups per CU); the leanest form of the kernel would still need about 190, more than
// the 168 that three wavefronts allow.
#ifndef HMAR_DKDV_MIN_WAVES
#define HMAR_DKDV_MIN_WAVES 2
#endif
// One tile of the dK/dV computation: the wavefront's 32 keys (rows kreg, vreg) against the 64
// query rows of the tile at LDS addresses Qt (Q) and Gt (dO), whose statistics are at nl2_t and
// delta_t.  lim_lo, lim_hi: the lane's key pairs with tile rows [lim_lo + 4h, lim_hi + 4h).
__device__ __forceinline__ void dkdv_tile(uint32_t Qt, uint32_t Gt, uint32_t nl2_t, uint32_t delta_t,
                                          const bf16x8 (&kreg)[4], const bf16x8 (&vreg)[4], f32x16 (&dk)[2], f32x16 (&dv)[2],
                                          int lim_lo, int lim_hi, bool need_lo, bool need_hi, float c,
                                          const LaneOffsets& lo_) {
    // Operands are fetched from LDS in batches ahead of the contractions that use them
    // (the scheduling barriers keep the compiler from sinking each read next to its use,
    // which would expose the LDS latency once per matrix instruction).  The score and dP
    // contractions of both 32-query blocks are issued first, so that the matrix pipe works
    // on the second block while the vector units form the first block's probabilities.
    f32x16 s[2], dp[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        bf16x8 aq[4], ag[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            aq[t] = lds_a_row(Qt, lo_, qb, t);
            ag[t] = lds_a_row(Gt, lo_, qb, t);
        }
        // statistics of the block's query rows 32qb + 8j + 4h + r (register 4j + r):
        // -Delta seeds the dP accumulator, so dP - Delta costs no vector instruction
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const f32x4 d4 = *(lds_f32x4*)(delta_t + (32 * qb + 8 * j) * 4);
#pragma unroll
            for (int r = 0; r < 4; ++r) { s[qb][4 * j + r] = 0.f; dp[qb][4 * j + r] = d4[r]; }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            s[qb] = mfma32(aq[t], kreg[t], s[qb]);
            dp[qb] = mfma32(ag[t], vreg[t], dp[qb]);
        }
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        // transposed operands of the second pair of contractions and the row statistics,
        // requested before the exponentials so that their latency hides behind them
        bf16x8 tg[2][2], tq[2][2];
        f32x4 l4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) l4[j] = *(lds_f32x4*)(nl2_t + (32 * qb + 8 * j) * 4);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                tg[sub][mb] = lds_a_tr(Gt, lo_, mb, 2 * qb + sub);
                tq[sub][mb] = lds_a_tr(Qt, lo_, mb, 2 * qb + sub);
            }
        __builtin_amdgcn_sched_barrier(0);
        mask_block(s[qb], 32 * qb, lim_lo, lim_hi, need_lo, need_hi);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = 4 * j + r;
                const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qb][i], c, l4[j][r]));
                s[qb][i] = pv;
                dp[qb][i] = pv * dp[qb][i];
            }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int e0 = 8 * sub;
            const bf16x8 pb = pack8(s[qb][e0 + 0], s[qb][e0 + 1], s[qb][e0 + 2], s[qb][e0 + 3],
                                    s[qb][e0 + 4], s[qb][e0 + 5], s[qb][e0 + 6], s[qb][e0 + 7]);
            const bf16x8 dsb = pack8(dp[qb][e0 + 0], dp[qb][e0 + 1], dp[qb][e0 + 2], dp[qb][e0 + 3],
                                     dp[qb][e0 + 4], dp[qb][e0 + 5], dp[qb][e0 + 6], dp[qb][e0 + 7]);
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                dv[mb] = mfma32(tg[sub][mb], pb, dv[mb]);
                dk[mb] = mfma32(tq[sub][mb], dsb, dk[mb]);
            }
        }
    }
}

// The work of one dK/dV item.  smem: ring of 2 stages, each a Q tile followed by a dO tile;
// nl2_s, delta_s: the per-row statistics of the two stages.
__device__ __forceinline__ void dkdv_body(const BwdParams& p, const Item it, const int32_t* row_lo, const int32_t* row_hi,
                                          int head, int item_id, char* smem, float (*nl2_s)[kTile], float (*delta_s)[kTile]) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, h = lane >> 5;
    const size_t head_off = (size_t)head * p.L * kD;
    const size_t head_in = (size_t)HMAR_INPUT_HEAD(head) * p.L * kD;     // == head_off outside measurements
    const __bf16* Qh = p.Q + head_in;
    const __bf16* Gh = p.dO + head_in;
    const float* NLh = p.neg_lse2 + (size_t)head * p.L;
    const float* Dh = p.neg_delta + (size_t)head * p.L;
    const LaneOffsets lo_ = make_lane_offsets(lane, wave);
    const uint32_t smem_base = lds_address(smem);
    const uint32_t nl2_base = lds_address(nl2_s), delta_base = lds_address(delta_s);

    const int q_begin = it.other_begin, q_end = it.other_end, qmax = q_end - 1;
    const int ntiles = (q_end - q_begin + kTile - 1) / kTile;

    // per lane and tile: 4 DMA loads, plus one for wavefronts 0 (-LSE*log2e) and 1 (Delta)
    auto issue = [&](int ti, int st) {
        const uint32_t stage = smem_base + st * (2 * kTileBytes);
        const int qt = q_begin + ti * kTile;
        dma_tile(Qh, qt, qmax, stage, lo_, lane, wave);
        dma_tile(Gh, qt, qmax, stage + kTileBytes, lo_, lane, wave);
        if (wave == 0) dma_floats(NLh, qt, qmax, nl2_base + st * (kTile * 4), lane);
        else if (wave == 1) dma_floats(Dh, qt, qmax, delta_base + st * (kTile * 4), lane);
    };
    issue(0, 0);

    const int wk0 = it.own_begin + wave * kRowsPerWave;
    const bool wave_active = wk0 < it.own_end;
    const int krow = min(wk0 + lr, it.own_end - 1);
    const int lo = row_lo[krow], hi = row_hi[krow];       // queries that see this key
    // pair ranges never decrease along the rows: the wavefront's extremes are at its first and last row
    const int rfirst = min(wk0, it.own_end - 1), rlast = min(wk0 + kRowsPerWave - 1, it.own_end - 1);
    const int wlo = row_lo[rfirst], whi = row_hi[rlast];        // union of the wavefront's ranges
    const int full_lo = row_lo[rlast], full_hi = row_hi[rfirst];  // what every one of its rows pairs with

    bf16x8 kreg[4], vreg[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        kreg[t] = HMAR_ROW_LOAD(reinterpret_cast<const bf16x8*>(p.K + head_in + (size_t)krow * kD + 16 * t + 8 * h));
        vreg[t] = HMAR_ROW_LOAD(reinterpret_cast<const bf16x8*>(p.V + head_in + (size_t)krow * kD + 16 * t + 8 * h));
    }

    f32x16 dk[2], dv[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) { dk[mb][i] = 0.f; dv[mb][i] = 0.f; }

    asm volatile("" :: "v"(kreg[0]), "v"(kreg[1]), "v"(kreg[2]), "v"(kreg[3]), "v"(vreg[0]), "v"(vreg[1]),
                 "v"(vreg[2]), "v"(vreg[3]));
    HMAR_WAIT_DMA_AND_BARRIER(0);

    auto tile_step = [&](const int ti, auto stage_c) {     // see the dQ kernel
        constexpr int ST = decltype(stage_c)::value;
        const int qt = q_begin + ti * kTile;
        if (ti + 1 < ntiles) issue(ti + 1, ST ^ 1);
#ifdef HMAR_TUNE_NO_COMPUTE_DKDV
        if (false) {
#else
        if (wave_active && qt < whi && qt + kTile > wlo) {
#endif
            const uint32_t Qt = smem_base + ST * (2 * kTileBytes);
            const uint32_t nl2_t = nl2_base + ST * (kTile * 4) + 16 * h;
            const uint32_t delta_t = delta_base + ST * (kTile * 4) + 16 * h;
            dkdv_tile(Qt, Qt + kTileBytes, nl2_t, delta_t, kreg, vreg, dk, dv, lo - qt - 4 * h, hi - qt - 4 * h,
                      qt < full_lo, qt + kTile > full_hi, p.c, lo_);
        }
        HMAR_WAIT_DMA_AND_BARRIER(0);
    };
    for (int ti = 0; ti < ntiles; ti += 2) {
        tile_step(ti, std::integral_constant<int, 0>{});
        if (ti + 1 >= ntiles) break;
        tile_step(ti + 1, std::integral_constant<int, 1>{});
    }

    if (wave_active) {
        const uint32_t patch = smem_base + wave * kPatchBytes;
        store_block_rows(patch, dk, p.sm_scale, p.dK + head_off, wk0, it.own_end - wk0, lane, nullptr, HMAR_NT_GRADS != 0);
        store_block_rows(patch, dv, 1.0f, p.dV + head_off, wk0, it.own_end - wk0, lane, nullptr, HMAR_NT_GRADS != 0);
    }
}

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(HMAR_DKDV_MIN_WAVES, HMAR_DKDV_MIN_WAVES))) void hmar_dkdv_kernel(BwdParams p) {
    __shared__ __attribute__((aligned(1024))) char smem[2 * 2 * kTileBytes];
    __shared__ __attribute__((aligned(256))) float nl2_s[2][kTile];
    __shared__ __attribute__((aligned(256))) float delta_s[2][kTile];
#ifdef HMAR_TUNE_LDS_PAD_DKDV
    HMAR_TUNE_LDS_PAD(HMAR_TUNE_LDS_PAD_DKDV)
#endif
    int head, item_id;
    if (!map_workgroup(p.n_items, p.n_heads, p.tail_groups, &head, &item_id)) return;
    dkdv_body(p, p.items[item_id], p.row_lo, p.row_hi, head, item_id, smem, nl2_s, delta_s);
}

#if defined(HMAR_BWD_MERGED)
#include "../tuning/bwd_merged.inc"
#endif
#if defined(HMAR_DKDV_PERSIST)
#include "../tuning/dkdv_persist.inc"
#endif

#if defined(HMAR_DKDV_PIPE) || (defined(HMAR_DKDV_KEYS_PER_WAVE) && HMAR_DKDV_KEYS_PER_WAVE == 16)
#include "../tuning/dkdv_variants.inc"
#endif

// Plain copy, 16 bytes per lane, grid-stride: calibration of the HBM traffic counters.
__global__ __launch_bounds__(256) void hmar_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                        size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t want = (n16 + 255) / 256;
    const unsigned groups = (unsigned)(want < 256 * 64 ? want : 256 * 64);
    hipLaunchKernelGGL(hmar_copy_kernel, dim3(groups), dim3(256), 0, stream, static_cast<u32x4*>(dst),
                       static_cast<const u32x4*>(src), n16);
    return hipGetLastError();
}

#ifndef HMAR_DKDV_KEYS_PER_WAVE
#define HMAR_DKDV_KEYS_PER_WAVE 32
#endif

hipError_t launch_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                      const float* LSE, void* dQ, void* dK, void* dV, float* workspace,
                      const DeviceSchedule& s, int n_heads, float sm_scale, hipStream_t stream) {
    const long long n_rows = (long long)n_heads * s.L;
    BwdParams p;
    p.Q = static_cast<const __bf16*>(Q);
    p.K = static_cast<const __bf16*>(K);
    p.V = static_cast<const __bf16*>(V);
    p.dO = static_cast<const __bf16*>(dO);
    p.O = static_cast<const __bf16*>(O);
    p.LSE = LSE;
    p.neg_delta = workspace;
    p.neg_lse2 = workspace + n_rows;
    p.dQ = static_cast<__bf16*>(dQ);
    p.dK = static_cast<__bf16*>(dK);
    p.dV = static_cast<__bf16*>(dV);
    p.n_heads = n_heads;
    p.L = s.L;
    p.c = sm_scale * kLog2e;
    p.sm_scale = sm_scale;

#if defined(HMAR_BWD_MERGED)
    return launch_bwd_merged(p, s, n_heads, stream);
#endif
    // dQ first: it also produces the per-row statistics the dK/dV kernel streams
    for (int dir = 0; dir < 2; ++dir) {
        p.items = static_cast<const Item*>(s.items[dir]);
        p.row_lo = s.row_lo[dir];
        p.row_hi = s.row_hi[dir];
        p.n_items = s.n_items[dir];
        p.tail_groups = tail_groups_for(s.num_cus, s.n_items[dir]);
        const long long groups = 8LL * ((n_heads + 7) / 8) * s.n_items[dir];
        if (groups <= 0 || groups > 0x7fffffffLL) return hipErrorInvalidValue;
        const int kid = dir == 1 ? kKernelDkDv : kKernelDq;
        profile_before(kid, stream);
#if HMAR_DKDV_KEYS_PER_WAVE == 16
        if (dir == 1) hipLaunchKernelGGL(hmar_dkdv16_kernel, dim3((unsigned)groups), dim3(kThreads16), 0, stream, p);
#elif defined(HMAR_DKDV_PIPE)
        if (dir == 1) hipLaunchKernelGGL(hmar_dkdv_pipe_kernel, dim3((unsigned)groups), dim3(kThreads), 0, stream, p);
#elif defined(HMAR_DKDV_PERSIST)
        if (dir == 1) {
            const long long resident = 2LL * s.num_cus / 8 * 8;       // two workgroups per CU, a multiple of 8
            hipLaunchKernelGGL(hmar_dkdv_persist_kernel, dim3((unsigned)std::min(groups, resident)), dim3(kThreads), 0, stream,
                               p, (int)groups);
        }
#else
        if (dir == 1) hipLaunchKernelGGL(hmar_dkdv_kernel, dim3((unsigned)groups), dim3(kThreads), 0, stream, p);
#endif
        else          hipLaunchKernelGGL(hmar_dq_kernel, dim3((unsigned)groups), dim3(kThreads), 0, stream, p);
        const hipError_t e = hipGetLastError();
        profile_after(kid, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace hmar
