// Forward kernel of the Markovian next-scale attention (paper Sec. 3.1, App. B.4) for gfx950.
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

#include "device_common.h"
#include "kernels.h"

namespace hmar {

struct FwdParams {
    const __bf16* Q; const __bf16* K; const __bf16* V;
    __bf16* O; float* LSE;
    const Item* items; const int32_t* row_lo; const int32_t* row_hi;
    int n_items, n_heads;
    int tail_groups;   // see map_workgroup
    int L, Lk;   // rows per head of Q/O/LSE and of K/V (they differ only for an inference step)
    float c;   // sm_scale * log2(e): scores are exponentiated in base 2
};

// The running reference maximum of a row is only raised when a tile exceeds it by more
// than this many binades; until then probabilities are at most 2^8, which fp32 sums and
// bf16 operands hold without loss.  The final division by the row sum makes the result
// independent of the reference.
constexpr float kRescaleThreshold = 8.0f;

#ifndef HMAR_FWD_MIN_WAVES
#define HMAR_FWD_MIN_WAVES 4
#endif
__global__ __launch_bounds__(kThreads, HMAR_FWD_MIN_WAVES) void hmar_fwd_kernel(FwdParams p) {
    // ring of 2 stages, each a K tile followed by a V tile
    __shared__ __attribute__((aligned(1024))) char smem[2 * 2 * kTileBytes];

    int head, item_id;
    if (!map_workgroup(p.n_items, p.n_heads, p.tail_groups, &head, &item_id)) return;
    const Item it = p.items[item_id];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, h = lane >> 5;
    const size_t head_off = (size_t)head * p.L * kD;
    const __bf16* Qh = p.Q + head_off;
    const __bf16* Kh = p.K + (size_t)head * p.Lk * kD;
    const __bf16* Vh = p.V + (size_t)head * p.Lk * kD;
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

    const int wq0 = it.own_begin + wave * kRowsPerWave;
    const bool wave_active = wq0 < it.own_end;               // uniform over the wavefront
    const bool row_valid = wq0 + lr < it.own_end;
    const int qrow = min(wq0 + lr, it.own_end - 1);
    const int lo = p.row_lo[qrow], hi = p.row_hi[qrow];
    // pair ranges never decrease along the rows: the wavefront's extremes are at its first and last row
    const int rfirst = min(wq0, it.own_end - 1), rlast = min(wq0 + kRowsPerWave - 1, it.own_end - 1);
    const int wlo = p.row_lo[rfirst], whi = p.row_hi[rlast];        // union of the wavefront's ranges
    const int full_lo = p.row_lo[rlast], full_hi = p.row_hi[rfirst];  // what every one of its rows pairs with

    bf16x8 q[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
        q[t] = *reinterpret_cast<const bf16x8*>(Qh + (size_t)qrow * kD + 16 * t + 8 * h);

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
        // the next tile goes into the other stage, which every wavefront left at the last barrier
        if (ti + 1 < ntiles) issue(ti + 1, ST ^ 1);
        if (wave_active && kt < whi && kt + kTile > wlo) {
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
        HMAR_WAIT_DMA_AND_BARRIER(0);     // the tile requested above has landed and this one is free
    };
    for (int ti = 0; ti < ntiles; ti += 2) {
        tile_step(ti, std::integral_constant<int, 0>{});
        if (ti + 1 >= ntiles) break;
        tile_step(ti + 1, std::integral_constant<int, 1>{});
    }

    // every wavefront has passed the last barrier: the ring is free and serves as the patch
    // through which the output block is turned into full rows
    if (wave_active) {
        const float l = half_sum(lsum);
        store_block_rows(smem_base + wave * kPatchBytes, o, 1.0f / l, p.O + head_off + (size_t)wq0 * kD,
                         it.own_end - wq0, lane);
        if (row_valid && h == 0) p.LSE[(size_t)head * p.L + wq0 + lr] = (m_ref + log2f(l)) * kLn2;
    }
}

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
    hipLaunchKernelGGL(hmar_fwd_kernel, dim3((unsigned)groups), dim3(kThreads), 0, stream, p);
    const hipError_t e = hipGetLastError();
    profile_after(kKernelFwd, stream);
    return e;
}

}  // namespace hmar
