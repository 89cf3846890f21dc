// Forward kernel of the Markovian next-scale attention (paper Sec. "Efficient Markovian
// Next-Scale Prediction"; appendix "Efficient Attention Performance") for gfx950.
//
// One workgroup (4 wavefronts) owns up to 128 consecutive query rows, 32 per wavefront,
// and streams the key/value rows of their two-scale windows through a two-stage ring of LDS
// tiles (64 rows each) filled by global->LDS DMA loads that run one tile ahead.
// Scores are computed transposed (S^T = K Q^T) so that a lane holds one query column:
// the row maximum and sum are then lane-local apart from one exchange between the two
// half-waves, and the probability tile is already laid out as the B operand of the
// second contraction O^T += V^T P^T, whose A operand comes from the row-major V tile
// through the LDS transpose load.
#include <type_traits>
#include <utility>

#include "device_common.h"
#include "kernels.h"

namespace hmar {

struct FwdParams {
    const __bf16* Q; const __bf16* K; const __bf16* V;
    __bf16* O; float* LSE;
    const Item* items; const int32_t* row_lo; const int32_t* row_hi;
    int n_items, n_heads;
    int tail_groups;   // see map_workgroup
    int L, Lk;   // rows per head of Q/O/LSE and of K/V
    float c;   // sm_scale * log2(e): scores are exponentiated in base 2
};

// Inference steps (paper Sec. "Efficient Markovian Next-Scale Prediction", last paragraph): a
// launch covers up to kMaxSteps independent steps, each with its own buffers; every query row
// of a step pairs with all of the step's key rows, so no table is needed: item i of a step owns
// query rows [128 i, 128 (i+1)) and visits keys [0, Lk).  The descriptors travel by value in
// the kernel arguments, sorted by decreasing work (the launch then ends on the lightest step).
struct StepDesc {
    const __bf16* Q; const __bf16* K; const __bf16* V;
    __bf16* O; float* LSE;
    const int32_t* rows;   // optional: row r of the step is row rows[r] of Q, O and LSE (a subset of a scale)
    int n_q;               // query rows of the step
    int q_stride;          // rows per head of the Q, O and LSE buffers (n_q unless `rows` is given)
    int Lk;                // key rows
    int first_item;        // index of the step's first item in the launch
};
// Steps whose keys fit one tile (Lk <= 64; the first scales of a schedule) are too small to fill a
// workgroup: they come last in `step` and share ONE item per head, the launch's last, in which
// every wavefront works on its own: unit u of the pack is the 32-row block pack_unit[u] % 2 of step
// pack_unit[u] / 2, taken by wavefront u % 4 (see small_steps_pack).
constexpr int kMaxPackUnits = 2 * kMaxSteps;
struct StepParams {
    StepDesc step[kMaxSteps];   // the n_tiled steps that get items of their own, then the packed ones
    int n_tiled, n_items, n_heads, tail_groups;
    int n_pack;                 // units of the pack (0: the launch has no pack item)
    int pack_unit[kMaxPackUnits];
    float c;
};

// The running reference maximum of a row is only raised when a tile exceeds it by more
// than this many binades; until then probabilities are at most 2^8, which fp32 sums and
// bf16 operands hold without loss.  The final division by the row sum makes the result
// independent of the reference.
constexpr float kRescaleThreshold = 8.0f;

#ifndef HMAR_FWD_MIN_WAVES
#define HMAR_FWD_MIN_WAVES 4
#endif
// Stages of the K/V ring (each 16 KB); the loads run HMAR_FWD_STAGES - 1 tiles ahead.  Two is what
// ships (see device_common.h); 3 and 4 exist for the measurement that decided it.
#ifndef HMAR_FWD_STAGES
#define HMAR_FWD_STAGES 2
#endif
constexpr int kFwdStages = HMAR_FWD_STAGES;
static_assert(kFwdStages >= 2 && kFwdStages <= 4, "ring depth");

// The pack item of a steps launch: inference steps with at most 64 keys.  A wavefront takes the
// units u = wave, wave + 4, ... and computes each alone, without the workgroup: the unit's 32 query
// rows and the step's key rows go from global memory straight into registers (both are row-wise
// operands), the value rows go by DMA into the wavefront's own quarter of the ring (8 KB, one
// tile), from where the transpose load feeds the second contraction; the same quarter then
// serves as the patch of the result.  One tile holds all keys, so the softmax is the plain
// one: row maximum, exponentials, row sum.  No barrier: nothing is shared between wavefronts.
__device__ __forceinline__ void small_steps_pack(const StepParams& p, int head, char* smem) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, h = lane >> 5;
    const LaneOffsets lo_ = make_lane_offsets(lane, 0);
    const uint32_t Vt = __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * kTileBytes);
    static_assert(kPatchBytes <= kTileBytes, "the result patch reuses the value tile");

    for (int u = wave; u < p.n_pack; u += 4) {
        const int unit = p.pack_unit[u];
        const StepDesc& sd = p.step[unit >> 1];
        const int n_q = sd.n_q, Lk = sd.Lk;                 // Lk <= 64, no row map
        const int row0 = 32 * (unit & 1);                   // < n_q
        const size_t in_head = (size_t)HMAR_INPUT_HEAD(head);
        const __bf16* Qh = sd.Q + in_head * n_q * kD;
        const __bf16* Kh = sd.K + in_head * Lk * kD;
        const __bf16* Vh = sd.V + in_head * Lk * kD;
        const bool two_blocks = Lk > 32;                    // uniform: keys 32..63 exist

        // value rows: this wavefront moves the whole tile, 8 rows per load, rows clamped to the
        // last key (every LDS row the contraction reads must hold finite numbers).  The
        // previous unit's patch reads have been consumed by its stores' operands by now.
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            if (b < 4 || two_blocks) {
                const int r = 8 * b + (lane >> 3);
                const uint32_t voff = min(r, Lk - 1) * kRowBytes + (((lane & 7) ^ swz(r)) << 4);
                dma16(Vh, voff, Vt + b * 1024);
            }
        }
        const int qrow = min(row0 + lr, n_q - 1);
        bf16x8 q[4], ka[2][4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            q[t] = *reinterpret_cast<const bf16x8*>(Qh + (size_t)qrow * kD + 16 * t + 8 * h);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                ka[kb][t] = *reinterpret_cast<const bf16x8*>(Kh + (size_t)min(32 * kb + lr, Lk - 1) * kD + 16 * t + 8 * h);
        }
        // all twelve loads are in flight before the first one is awaited; loads complete in order,
        // so the value tile requested before them has landed as well
        asm volatile("" :: "v"(q[0]), "v"(q[1]), "v"(q[2]), "v"(q[3]), "v"(ka[0][0]), "v"(ka[0][1]), "v"(ka[0][2]),
                     "v"(ka[0][3]), "v"(ka[1][0]), "v"(ka[1][1]), "v"(ka[1][2]), "v"(ka[1][3]));

        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) s[kb] = mfma32(ka[kb][t], q[t], s[kb]);
        }
        // element i of block kb is key 4h + 32kb + 8(i/4) + i%4; keys >= Lk do not exist
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) mask_block(s[kb], 32 * kb, -4 * h, Lk - 4 * h, false, Lk < 64);
        float mt = s[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mt = fmaxf(mt, s[kb][i]);
        const float m_ref = half_max(mt) * p.c;            // key 0 exists: finite
        float lsum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][i], p.c, -m_ref));
                lsum += pv;
                s[kb][i] = pv;
            }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // (already true; the compiler cannot know)
        f32x16 o[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[mb][i] = 0.f;
#pragma unroll
        for (int tp = 0; tp < 4; ++tp) {
            if (tp < 2 || two_blocks) {
                const int kb = tp >> 1, e0 = 8 * (tp & 1);
                const bf16x8 pb = pack8(s[kb][e0 + 0], s[kb][e0 + 1], s[kb][e0 + 2], s[kb][e0 + 3],
                                        s[kb][e0 + 4], s[kb][e0 + 5], s[kb][e0 + 6], s[kb][e0 + 7]);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) o[mb] = mfma32(lds_a_tr(Vt, lo_, mb, tp), pb, o[mb]);
            }
        }
        const float l = half_sum(lsum);
        // LDS operations of a wavefront execute in order: the patch writes follow the tile reads
        store_block_rows(Vt, o, 1.0f / l, sd.O + (size_t)head * n_q * kD, row0, n_q - row0, lane);
        if (row0 + lr < n_q && h == 0) sd.LSE[(size_t)head * n_q + qrow] = (m_ref + log2f(l)) * kLn2;
    }
}
// One body serves both launches: with STEPS the item, its buffers and its (trivial) pair ranges
// come from the step descriptors, otherwise from the schedule tables.
template <bool STEPS, typename Params>
__device__ __forceinline__ void fwd_body(const Params& p, char* smem) {
    int head, item_id;
    if (!map_workgroup(p.n_items, p.n_heads, p.tail_groups, &head, &item_id)) return;
    Item it;
    const __bf16* Qh; const __bf16* Kh; const __bf16* Vh;
    __bf16* Oh; float* LSEh;
    const int32_t* rows = nullptr;    // row map of Q, O, LSE (steps over a subset of rows)
    int q_stride_rows = 0;            // rows per head of those buffers (steps)
    const int32_t* row_lo = nullptr; const int32_t* row_hi = nullptr;
    if constexpr (STEPS) {
        if (p.n_pack > 0 && item_id == p.n_items - 1) {
            small_steps_pack(p, head, smem);
            return;
        }
        int si = 0;
        while (si + 1 < p.n_tiled && item_id >= p.step[si + 1].first_item) ++si;
        const StepDesc& sd = p.step[si];
        const int li = item_id - sd.first_item;
        it.own_begin = li * 128;
        it.own_end = min(sd.n_q, it.own_begin + 128);
        it.other_begin = 0;
        it.other_end = sd.Lk;
        const size_t q_off = (size_t)head * sd.q_stride, q_in = (size_t)HMAR_INPUT_HEAD(head) * sd.q_stride;
        Qh = sd.Q + q_in * kD; Oh = sd.O + q_off * kD; LSEh = sd.LSE + q_off;
        Kh = sd.K + (size_t)HMAR_INPUT_HEAD(head) * sd.Lk * kD;
        Vh = sd.V + (size_t)HMAR_INPUT_HEAD(head) * sd.Lk * kD;
        rows = sd.rows;
        q_stride_rows = sd.q_stride;
    } else {
        it = p.items[item_id];
        const size_t q_off = (size_t)head * p.L, q_in = (size_t)HMAR_INPUT_HEAD(head) * p.L;
        Qh = p.Q + q_in * kD; Oh = p.O + q_off * kD; LSEh = p.LSE + q_off;
        Kh = p.K + (size_t)HMAR_INPUT_HEAD(head) * p.Lk * kD;
        Vh = p.V + (size_t)HMAR_INPUT_HEAD(head) * p.Lk * kD;
        row_lo = p.row_lo; row_hi = p.row_hi;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, h = lane >> 5;
    const LaneOffsets lo_ = make_lane_offsets(lane, wave);
    const uint32_t smem_base = lds_address(smem);

    const int k_begin = it.other_begin, k_end = it.other_end, kmax = k_end - 1;
    const int ntiles = (k_end - k_begin + kTile - 1) / kTile;

    // 4 DMA loads per lane and tile (2 for K, 2 for V); the first tile is requested before
    // anything else so that its latency overlaps the rest of the prologue
    auto issue = [&](int ti, int st) {
        const uint32_t stage = smem_base + st * (2 * kTileBytes);
        dma_tile(Kh, k_begin + ti * kTile, kmax, stage, lo_, lane, wave);
        dma_tile(Vh, k_begin + ti * kTile, kmax, stage + kTileBytes, lo_, lane, wave);
    };
    issue(0, 0);
#pragma unroll
    for (int d = 1; d < kFwdStages - 1; ++d)
        if (d < ntiles) issue(d, d);

    const int wq0 = it.own_begin + wave * kRowsPerWave;
    const bool wave_active = wq0 < it.own_end;               // uniform over the wavefront
    const bool row_valid = wq0 + lr < it.own_end;
    const int qrow = min(wq0 + lr, it.own_end - 1);
    int lo, hi, wlo, whi, full_lo, full_hi;
    if constexpr (STEPS) {
        lo = wlo = full_lo = 0;
        hi = whi = full_hi = k_end;
    } else {
        lo = row_lo[qrow]; hi = row_hi[qrow];
        // pair ranges never decrease along the rows: the wavefront's extremes are at its first and last row
        const int rfirst = min(wq0, it.own_end - 1), rlast = min(wq0 + kRowsPerWave - 1, it.own_end - 1);
        wlo = row_lo[rfirst]; whi = row_hi[rlast];          // union of the wavefront's ranges
        full_lo = row_lo[rlast]; full_hi = row_hi[rfirst];  // what every one of its rows pairs with
    }

    // a listed row outside the buffer is clamped into it: wrong input must not become a wild access
    int q_rows_per_head = 0;
    if constexpr (STEPS) q_rows_per_head = q_stride_rows;
    const int qrow_mem = rows ? min(max(rows[qrow], 0), q_rows_per_head - 1) : qrow;
    bf16x8 q[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
        q[t] = HMAR_ROW_LOAD(reinterpret_cast<const bf16x8*>(Qh + (size_t)qrow_mem * kD + 16 * t + 8 * h));

    f32x16 o[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[mb][i] = 0.f;
    float m_ref = kNegBig, lsum = 0.f;
    bool o_empty = true;              // nothing accumulated yet: the first rescale has nothing to scale

    // The compiler does not see the DMA loads; without this use it would wait for the Q
    // registers inside the loop, where its count would also drain the loads running ahead.
    asm volatile("" :: "v"(q[0]), "v"(q[1]), "v"(q[2]), "v"(q[3]));
    // Loads complete in order: the registers above were requested after tile 0.
    HMAR_WAIT_DMA_AND_BARRIER(0);

    // One tile: request the next one, compute, wait for the request.  The stage is a template
    // constant (the loop below alternates the two instantiations) so that every LDS address of
    // the step is a per-lane register plus an immediate offset.
    auto tile_step = [&](const int ti, auto stage_c) {
        constexpr int ST = decltype(stage_c)::value;
        const int kt = k_begin + ti * kTile;
        // the tile requested now goes into the stage that every wavefront left at the last barrier
        const bool ahead = ti + kFwdStages - 1 < ntiles;
        if (ahead) issue(ti + kFwdStages - 1, (ST + kFwdStages - 1) % kFwdStages);
#ifdef HMAR_TUNE_NO_COMPUTE_FWD
        if (false) {
#else
        if (wave_active && kt < whi && kt + kTile > wlo) {
#endif
            const uint32_t Kt = smem_base + ST * (2 * kTileBytes);
            const uint32_t Vt = Kt + kTileBytes;
            f32x16 s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    s[kb] = mfma32(lds_a_row(Kt, lo_, kb, t), q[t], s[kb]);
            }
            // element i of block kb is key kt + 4h + 32kb + 8(i/4) + i%4; allowed iff lo <= key < hi
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                mask_block(s[kb], 32 * kb, lo - kt - 4 * h, hi - kt - 4 * h, kt < full_lo, kt + kTile > full_hi);
            float mt = s[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mt = fmaxf(mt, s[kb][i]);
            mt = half_max(mt) * p.c;
            if (__builtin_amdgcn_ballot_w64(mt > m_ref + kRescaleThreshold) != 0) {
                const float m_new = fmaxf(m_ref, mt);
                if (!o_empty) {
                    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
                    lsum *= alpha;
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                        for (int i = 0; i < 16; ++i) o[mb][i] *= alpha;
                }
                m_ref = m_new;
            }
            o_empty = false;
            const float neg_m = -m_ref;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][i], p.c, neg_m));
                    lsum += pv;
                    s[kb][i] = pv;
                }
#pragma unroll
            for (int tp = 0; tp < 4; ++tp) {
                const int kb = tp >> 1, e0 = 8 * (tp & 1);
                const bf16x8 pb = pack8(s[kb][e0 + 0], s[kb][e0 + 1], s[kb][e0 + 2], s[kb][e0 + 3],
                                        s[kb][e0 + 4], s[kb][e0 + 5], s[kb][e0 + 6], s[kb][e0 + 7]);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
                    o[mb] = mfma32(lds_a_tr(Vt, lo_, mb, tp), pb, o[mb]);
            }
        }
        // the next tile has landed (4 loads per lane and tile: the younger tiles may still be in
        // flight) and this one is free
        if (kFwdStages > 2 && ahead) { HMAR_WAIT_DMA_AND_BARRIER(4 * (kFwdStages - 2)); }
        else                         { HMAR_WAIT_DMA_AND_BARRIER(0); }
    };
    for (int ti = 0; ti < ntiles; ti += kFwdStages) {
        tile_step(ti, std::integral_constant<int, 0>{});
        if (ti + 1 >= ntiles) break;
        tile_step(ti + 1, std::integral_constant<int, 1>{});
        if constexpr (kFwdStages > 2) {
            if (ti + 2 >= ntiles) break;
            tile_step(ti + 2, std::integral_constant<int, 2>{});
        }
        if constexpr (kFwdStages > 3) {
            if (ti + 3 >= ntiles) break;
            tile_step(ti + 3, std::integral_constant<int, 3>{});
        }
    }

    // every wavefront has passed the last barrier: the ring is free and serves as the patch
    // through which the output block is turned into full rows
    if (wave_active) {
        const float l = half_sum(lsum);
        store_block_rows(smem_base + wave * kPatchBytes, o, 1.0f / l, Oh, wq0, it.own_end - wq0, lane, rows, HMAR_NT_O != 0,
                         q_rows_per_head);
        if (row_valid && h == 0) LSEh[qrow_mem] = (m_ref + log2f(l)) * kLn2;
    }
}

__global__ __launch_bounds__(kThreads, HMAR_FWD_MIN_WAVES) void hmar_fwd_kernel(FwdParams p) {
    // ring of stages, each a K tile followed by a V tile
    __shared__ __attribute__((aligned(1024))) char smem[kFwdStages * 2 * kTileBytes];
#ifdef HMAR_TUNE_LDS_PAD_FWD
    HMAR_TUNE_LDS_PAD(HMAR_TUNE_LDS_PAD_FWD)
#endif
    fwd_body<false>(p, smem);
}

__global__ __launch_bounds__(kThreads, HMAR_FWD_MIN_WAVES) void hmar_fwd_steps_kernel(StepParams p) {
    __shared__ __attribute__((aligned(1024))) char smem[kFwdStages * 2 * kTileBytes];
    fwd_body<true>(p, smem);
}

#ifdef HMAR_TUNE_FWD_STUDY
#include "../tuning/fwd_tile_study.inc"
#ifndef HMAR_STUDY_RB
#define HMAR_STUDY_RB 1
#endif
#ifndef HMAR_STUDY_NW
#define HMAR_STUDY_NW 4
#endif
#ifndef HMAR_STUDY_PIPE
#define HMAR_STUDY_PIPE 0
#endif
#ifndef HMAR_STUDY_MINW
#define HMAR_STUDY_MINW 4
#endif
static_assert(HMAR_STUDY_RB * HMAR_STUDY_NW == 4, "items of the forward list own up to 128 rows");
#endif

hipError_t launch_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                      const DeviceSchedule& s, int n_heads, float sm_scale, hipStream_t stream) {
    FwdParams p;
    p.Q = static_cast<const __bf16*>(Q);
    p.K = static_cast<const __bf16*>(K);
    p.V = static_cast<const __bf16*>(V);
    p.O = static_cast<__bf16*>(O);
    p.LSE = LSE;
    p.items = static_cast<const Item*>(s.items[0]);
    p.row_lo = s.row_lo[0];
    p.row_hi = s.row_hi[0];
    p.n_items = s.n_items[0];
    p.n_heads = n_heads;
    p.tail_groups = tail_groups_for(s.num_cus, s.n_items[0]);
    p.L = s.L;
    p.Lk = s.Lk;
    p.c = sm_scale * kLog2e;
    const long long groups = 8LL * ((n_heads + 7) / 8) * s.n_items[0];
    if (groups <= 0 || groups > 0x7fffffffLL) return hipErrorInvalidValue;
    profile_before(kKernelFwd, stream);
#ifdef HMAR_TUNE_FWD_STUDY
    hipLaunchKernelGGL((hmar_fwd_study_kernel<HMAR_STUDY_RB, HMAR_STUDY_NW, HMAR_STUDY_MINW, HMAR_STUDY_PIPE != 0>),
                       dim3((unsigned)groups), dim3(64 * HMAR_STUDY_NW), 0, stream, p);
#else
    hipLaunchKernelGGL(hmar_fwd_kernel, dim3((unsigned)groups), dim3(kThreads), 0, stream, p);
#endif
    const hipError_t e = hipGetLastError();
    profile_after(kKernelFwd, stream);
    return e;
}

hipError_t launch_fwd_steps(const StepLaunch& L, int n_heads, float sm_scale, int num_cus, hipStream_t stream) {
    if (L.n_steps < 1 || L.n_steps > kMaxSteps) return hipErrorInvalidValue;
    StepParams p;
    // steps with items of their own first (in the given order), then the ones that share the pack
    auto packed = [](const StepLaunch::Step& a) { return a.Lk <= kTile && a.rows == nullptr; };
    int order[kMaxSteps], n = 0;
    for (int i = 0; i < L.n_steps; ++i) if (!packed(L.step[i])) order[n++] = i;
    p.n_tiled = n;
    for (int i = 0; i < L.n_steps; ++i) if (packed(L.step[i])) order[n++] = i;
    int items = 0;
    p.n_pack = 0;
    for (int i = 0; i < L.n_steps; ++i) {
        const StepLaunch::Step& a = L.step[order[i]];
        if (a.n_q < 1 || a.Lk < a.n_q) return hipErrorInvalidValue;
        StepDesc& d = p.step[i];
        d.Q = static_cast<const __bf16*>(a.Q);
        d.K = static_cast<const __bf16*>(a.K);
        d.V = static_cast<const __bf16*>(a.V);
        d.O = static_cast<__bf16*>(a.O);
        d.LSE = a.LSE;
        d.rows = a.rows;
        d.n_q = a.n_q;
        d.q_stride = a.q_stride;
        d.Lk = a.Lk;
        d.first_item = items;
        if (i < p.n_tiled) {
            items += (a.n_q + 127) / 128;
        } else {
            for (int blk = 0; 32 * blk < a.n_q; ++blk)         // at most two: n_q <= Lk <= 64
                p.pack_unit[p.n_pack++] = 2 * i + blk;
        }
    }
    if (p.n_pack > 0) ++items;                                  // the pack is the launch's last item
    for (int i = L.n_steps; i < kMaxSteps; ++i) p.step[i] = p.step[0];
    for (int u = p.n_pack; u < kMaxPackUnits; ++u) p.pack_unit[u] = 0;
    p.n_items = items;
    p.n_heads = n_heads;
    p.tail_groups = tail_groups_for(num_cus, items);
    p.c = sm_scale * kLog2e;
    const long long groups = 8LL * ((n_heads + 7) / 8) * items;
    if (groups <= 0 || groups > 0x7fffffffLL) return hipErrorInvalidValue;
    profile_before(kKernelFwd, stream);
    hipLaunchKernelGGL(hmar_fwd_steps_kernel, dim3((unsigned)groups), dim3(kThreads), 0, stream, p);
    const hipError_t e = hipGetLastError();
    profile_after(kKernelFwd, stream);
    return e;
}

}  // namespace hmar
