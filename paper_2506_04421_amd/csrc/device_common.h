// Shared device-side types and helpers of the gfx950 attention kernels.
//
// MFMA register layouts used throughout (v_mfma_f32_32x32x16_bf16, wave64), with
// lr = lane % 32 and h = lane / 32:
//   A operand (M x 16): lane holds row lr, 8 k-values of half h
//   B operand (16 x N): lane holds column lr, the same 8 k-values
//   C/D      (M x N)  : lane holds column lr; register i holds row 8*(i/4) + 4*h + i%4
// The contraction index only has to be enumerated identically by A and B, so a C tile
// can be fed back as a B operand without moving data between lanes: registers 8s..8s+7
// of a C tile (s = 0, 1) are the 8 k-values of half h of a 16-deep step whose rows are
//   16s + 4h + {0,1,2,3}  and  16s + 8 + 4h + {0,1,2,3}
// of the tile.  The matching A operand is fetched with the LDS transpose load
// (ds_read_b64_tr_b16): within a group of 16 lanes, lane i supplies the address of 4
// consecutive elements of row i/4, columns 4*(i%4).., of a 4 x 16 block, and receives
// column i of that block (4 rows).  Two such loads give the 8 k-values above.
//
// LDS tiles are 64 rows x 64 bf16, row-major, 128 bytes per row, no padding.  The eight
// 16-byte chunks of row r are stored permuted: chunk c lives at chunk position
// c ^ swz(r).  The permutation keeps (a) the row-wise 16-byte operand reads of 16
// consecutive rows and (b) the transpose loads of 4 consecutive rows on distinct banks.
// Tiles are filled by global->LDS DMA loads (global_load_lds_dwordx4): a wavefront writes
// 1 KB = 8 rows contiguously, so each lane fetches the global chunk that belongs at its
// own LDS position; the permutation stays inside a 128-byte row, so the global side
// remains fully coalesced.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hmar {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // plain vector types: HIP's uint4/uint2
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;   // structs copy through memory

constexpr int kD = 64;            // head dimension
constexpr int kTile = 64;         // streamed rows per LDS tile
constexpr int kRowBytes = 128;    // one bf16 row of the head dimension
constexpr int kTileBytes = kTile * kRowBytes;   // 8 KB
constexpr int kThreads = 256;     // 4 wavefronts
constexpr int kRowsPerWave = 32;
// Every kernel streams its tiles through a ring of two LDS stages, the DMA loads running one
// tile ahead of the compute.  Two stages (32 KB per workgroup) measured faster than three or
// four on the 256px training shape: the LDS saved lets a fourth workgroup live on each CU, and
// with 3-4 wavefronts per SIMD other workgroups hide the load latency better than a deeper
// ring does.  The kernels unroll their tile loop by two so that the stage is a constant.
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;

struct alignas(16) Item { int32_t own_begin, own_end, other_begin, other_end; };

// ---- build-time knobs for measurements (never set in the library the tests and the benchmark
// load; `python -m paper_2506_04421_amd.build --variant NAME -D...` builds a separate library):
//   HMAR_TUNE_LDS_PAD_FWD / _DQ / _DKDV = bytes   extra LDS per workgroup: caps the workgroups a CU
//                                                 holds, i.e. the wavefronts per SIMD of that kernel
//   HMAR_TUNE_NO_COMPUTE_FWD / _DQ / _DKDV        skip the tile arithmetic: what remains is the
//                                                 kernel's memory skeleton (loads, barriers, stores)
//   HMAR_TUNE_ALIAS_HEADS                         every head reads the inputs of head (head % 8): the
//                                                 loads then hit in L2 and no HBM read remains
//   HMAR_TUNE_FWD_STUDY (+ HMAR_STUDY_*)          the forward of tuning/fwd_tile_study.inc instead: rows
//                                                 per wavefront, key tile, software pipelining
//   HMAR_DKDV_PIPE / HMAR_DKDV_KEYS_PER_WAVE=16   a dK/dV kernel of tuning/dkdv_variants.inc instead: scores
//                                                 formed one block ahead / 16 keys per wavefront on
//                                                 16x16x32 MFMAs at four wavefronts per SIMD
//   HMAR_FWD_STAGES = 2 | 3 | 4                   stages of the forward's K/V ring (csrc/fwd.hip)
//   HMAR_NT_O / HMAR_NT_GRADS / HMAR_NT_ROW_LOADS = 0 | 1   cache policy of result stores and row loads (see below)
//   HMAR_DKDV_PERSIST                             the dK/dV kernel of tuning/dkdv_persist.inc instead: two resident
//                                                 workgroups per CU walk the (head, item) units, the next unit's
//                                                 first tile and key rows requested before the current one's results leave
//   HMAR_BWD_MERGED (+ HMAR_MERGED_*)             the backward of tuning/bwd_merged.inc instead: a row-statistics
//                                                 kernel, then dQ and dK/dV items in one launch
// Cache policy of the accesses no workgroup of the launch repeats (1 = non-temporal: the lines
// are the first to leave the caches).  Result rows are written once and read by nobody in the
// launch: storing them non-temporally keeps the streamed K/V (Q/dO) tiles, which other
// workgroups of the head re-read, in the L2 longer: -1.5 % on a forward+backward step, measured on
// the 256px and 512px training shapes.  Loading the once-read rows (a workgroup's own Q, dO, O
// or K, V rows) non-temporally costs 4-9 % instead.
#ifndef HMAR_NT_O
#define HMAR_NT_O 1          // the forward's O rows
#endif
#ifndef HMAR_NT_GRADS
#define HMAR_NT_GRADS 1      // dQ, dK, dV rows
#endif
#ifndef HMAR_NT_ROW_LOADS
#define HMAR_NT_ROW_LOADS 0  // a workgroup's own rows
#endif
#if HMAR_NT_ROW_LOADS
#define HMAR_ROW_LOAD(ptr) __builtin_nontemporal_load(ptr)
#else
#define HMAR_ROW_LOAD(ptr) (*(ptr))
#endif
#if defined(HMAR_TUNE_ALIAS_HEADS)
#define HMAR_INPUT_HEAD(h) ((h) & 7)
#else
#define HMAR_INPUT_HEAD(h) (h)
#endif
// extra LDS, kept allocated by an address use the compiler cannot remove
#define HMAR_TUNE_LDS_PAD(BYTES)                                                \
    __shared__ char hmar_tune_pad[(BYTES) > 0 ? (BYTES) : 1];                   \
    if ((BYTES) > 0) asm volatile("" :: "v"(lds_address(hmar_tune_pad)));


typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// Workgroup -> (head, item).  Workgroups are handed to the 8 XCDs round-robin, so all
// items of one head are given ids that are congruent mod 8: they then run on one XCD and
// share its L2 for the rows they re-read.  A group is 8 heads, one per XCD.
//  - The ids walk the groups one after the other, a group's items heaviest first, except for
//    the last `tail_groups` groups, which form one batch walked item by item (all their
//    heaviest items, then the next, ...): the launch then ends on the lightest items, and the
//    period in which the device drains is as short as those.  The batch is sized to about one
//    round of resident workgroups, small enough for its heads' K and V to share the L2.
//  - With `reverse` the groups are walked from the last to the first: a kernel that follows
//    another one over the same tensors then starts on the heads that kernel touched last,
//    which are the ones still in the last-level cache.
__device__ __forceinline__ bool map_unit(int wg, int n_items, int n_heads, int tail_groups, int* head, int* item,
                                         bool reverse = false) {
    const int xcd = wg & 7;
    const int slot = wg >> 3;
    const int n_groups = (n_heads + 7) / 8;
    const int tail = min(max(tail_groups, 1), n_groups);
    const int head_major = (n_groups - tail) * n_items;       // slots before the tail batch
    int group, it;
    if (slot < head_major) { group = slot / n_items; it = slot % n_items; }
    else { const int s2 = slot - head_major; it = s2 / tail; group = n_groups - tail + s2 % tail; }
    if (reverse) group = n_groups - 1 - group;
    *head = group * 8 + xcd;
    *item = it;
    return *head < n_heads;
}
__device__ __forceinline__ bool map_workgroup(int n_items, int n_heads, int tail_groups, int* head, int* item,
                                              bool reverse = false) {
    return map_unit(blockIdx.x, n_items, n_heads, tail_groups, head, item, reverse);
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// value of the lane 32 away, combined: max / sum over the two half-waves
__device__ __forceinline__ float half_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2 x = {a, b};
    bf16x2 y = __builtin_convertvector(x, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(uint32_t, y);
}

// 8 fp32 -> one bf16x8 MFMA operand
__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3,
                                        float a4, float a5, float a6, float a7) {
    u32x4 u;
    u.x = pack_bf16(a0, a1);
    u.y = pack_bf16(a2, a3);
    u.z = pack_bf16(a4, a5);
    u.w = pack_bf16(a6, a7);
    return __builtin_bit_cast(bf16x8, u);
}

// ---- LDS tile layout --------------------------------------------------------------------
// chunk permutation of row r: depends on (r >> 1) & 7 only
__device__ __forceinline__ int swz(int r) {
    const int u = (r >> 1) & 7;
    return ((u & 1) << 2) | (u >> 1);
}

// Per-lane byte offsets into a tile, computed once per kernel.
struct LaneOffsets {
    int row0, row1, row2, row3;   // row-wise A operand: row lr (+32 per block), 16-byte chunk 2t + h
    int trA0, trA1;               // transpose load, rows 4h + i/4 of a 16-row step, column block 0 / 1
    int trB0, trB1;               // the same, 8 rows further down
    int dma_src;                  // byte offset, inside its 128-byte global row, of the 16 bytes
                                  // this lane moves (row = lane/8 of the 8 rows a wavefront writes)
    int dma_voff;                 // byte offset of those 16 bytes from the first row of a full tile
};

__device__ __forceinline__ LaneOffsets make_lane_offsets(int lane, int wave) {
    LaneOffsets o;
    const int lr = lane & 31, h = lane >> 5, i = lane & 15, half16 = (lane >> 4) & 1;
    const int s = swz(lr);
    o.row0 = lr * kRowBytes + (((0 + h) ^ s) << 4);
    o.row1 = lr * kRowBytes + (((2 + h) ^ s) << 4);
    o.row2 = lr * kRowBytes + (((4 + h) ^ s) << 4);
    o.row3 = lr * kRowBytes + (((6 + h) ^ s) << 4);
    const int rA = 4 * h + (i >> 2), rB = rA + 8;
    const int chunk = 2 * half16 + ((i & 3) >> 1);
    o.trA0 = rA * kRowBytes + ((chunk ^ swz(rA)) << 4) + 8 * (i & 1);
    o.trA1 = rA * kRowBytes + (((4 + chunk) ^ swz(rA)) << 4) + 8 * (i & 1);
    o.trB0 = rB * kRowBytes + ((chunk ^ swz(rB)) << 4) + 8 * (i & 1);
    o.trB1 = rB * kRowBytes + (((4 + chunk) ^ swz(rB)) << 4) + 8 * (i & 1);
    // DMA: lane p of a wavefront lands at byte 16p of an 8-row block: row p/8, position p%8.
    // The block index is wave + 4j (j = 0, 1); swz of row 8*blk + p/8 depends on
    // (4*blk + p/16) mod 8, i.e. on the parity of blk = parity of wave: one offset serves both j.
    const int r = 8 * wave + (lane >> 3);
    o.dma_src = ((lane & 7) ^ swz(r)) << 4;
    o.dma_voff = r * kRowBytes + o.dma_src;
    return o;
}

// One global->LDS DMA load: every lane moves 16 (or 4) bytes from global address
// sbase + voff (sbase uniform over the wavefront, voff a per-lane byte offset) to LDS address
// lds_base + lane * 16 (or 4); lds_base must be uniform too (it goes through M0).  Written
// as inline assembly so that the compiler does not serialise the LDS reads of the tile being
// computed behind the loads that run ahead into other tiles; completion is awaited
// explicitly (wait_dma_and_barrier) before any wavefront reads the tile.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_base) : "m0", "memory");
}
__device__ __forceinline__ void dma4(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_base) : "m0", "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// Issue the DMA loads of one 64-row tile: rows row0 .. row0+63 of a [rows][64] bf16 matrix
// (clamped to row_max, so a ragged tail re-reads a valid row), into the tile at LDS address
// `tile` (wave-uniform).  Two loads per lane: tile rows 8*wave + lane/8 and 32 further down.
// For a full tile the per-lane offset is a constant of the kernel and only the scalar base
// moves from tile to tile.
__device__ __forceinline__ void dma_tile(const __bf16* base, int row0, int row_max, uint32_t tile,
                                         const LaneOffsets& o, int lane, int wave) {
    const char* sbase = reinterpret_cast<const char*>(base) + (size_t)row0 * kRowBytes;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(tile + wave * 1024);
    if (row0 + kTile - 1 <= row_max) {
        dma16(sbase, o.dma_voff, lds0);
        dma16(sbase + 32 * kRowBytes, o.dma_voff, lds0 + 4096);
    } else {
        const int r = 8 * wave + (lane >> 3), last = row_max - row0;
        dma16(sbase, min(r, last) * kRowBytes + o.dma_src, lds0);
        dma16(sbase, min(r + 32, last) * kRowBytes + o.dma_src, lds0 + 4096);
    }
}

// 64 consecutive fp32 (index clamped to i_max) to LDS address `dst` (wave-uniform): one
// 4-byte DMA load per lane
__device__ __forceinline__ void dma_floats(const float* base, int i0, int i_max, uint32_t dst, int lane) {
    dma4(base + i0, min(lane, i_max - i0) * 4, __builtin_amdgcn_readfirstlane(dst));
}

// Wait until at most N (<= 15) of this wavefront's DMA loads are outstanding and all its LDS
// traffic is done, then meet the workgroup.  (A plain __syncthreads() would wait for every
// outstanding load and so stall the loads running ahead.)  s_waitcnt immediate on gfx9:
// vmcnt in bits 3:0 (and 15:14), expcnt in 6:4 (7 = no wait), lgkmcnt in 11:8.
template <int N>
__device__ __forceinline__ void wait_dma_and_barrier() {
    static_assert(N >= 0 && N <= 15, "vmcnt immediate");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(N | (7 << 4));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
#define HMAR_WAIT_DMA_AND_BARRIER(N) wait_dma_and_barrier<N>()

// LDS is addressed with plain 32-bit byte addresses so that block, step and stage offsets
// fold into the instructions' immediate offset fields.
typedef const __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef const __attribute__((address_space(3))) f32x4 lds_f32x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// A operand, row-wise: row 32*blk + lr of the tile at LDS address `tile`, columns 16t + 8h .. +7
__device__ __forceinline__ bf16x8 lds_a_row(uint32_t tile, const LaneOffsets& o, int blk, int t) {
    const int off = t == 0 ? o.row0 : t == 1 ? o.row1 : t == 2 ? o.row2 : o.row3;
    return *(lds_bf16x8*)(tile + off + blk * (32 * kRowBytes));
}

// A operand, transposed: column 32*mb + lr of the tile, tile rows of 16-deep step tp in the
// enumeration a C tile fed back as B uses
__device__ __forceinline__ bf16x8 lds_a_tr(uint32_t tile, const LaneOffsets& o, int mb, int tp) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + (mb ? o.trA1 : o.trA0) + tp * (16 * kRowBytes)));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + (mb ? o.trB1 : o.trB0) + tp * (16 * kRowBytes)));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// Mask one 32 x 32 score block held in the C layout.  Register i of the lane is the
// streamed row (key in the forward and dQ kernels, query in the dK/dV kernel) with index
// c0 + 8*(i/4) + i%4 relative to the lane's base row; entries whose relative index lies
// outside [lim_lo, lim_hi) become -inf (their probability is then exactly 0).  need_lo and
// need_hi are uniform over the wavefront: only tiles that straddle an edge of some row's
// range pay for the compare-and-select.
__device__ __forceinline__ void mask_block(f32x16& s, int c0, int lim_lo, int lim_hi, bool need_lo, bool need_hi) {
    if (need_hi) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = (c0 + 8 * (i >> 2) + (i & 3)) < lim_hi ? s[i] : -INFINITY;
    }
    if (need_lo) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = (c0 + 8 * (i >> 2) + (i & 3)) >= lim_lo ? s[i] : -INFINITY;
    }
}

// Write a wavefront's result block to global memory as bf16 rows.  The block is the pair of
// fp32 accumulators acc[0], acc[1] in the C layout (lane = result row lr, registers =
// columns 32*mb + 8*(i/4) + 4h + i%4).  Storing it directly would scatter 8-byte pieces over
// 32 rows per instruction; instead it is transposed through a private LDS patch
// (32 rows x kPatchPitch bytes) and leaves as full 128-byte rows, 8 rows per instruction.
// `patch` is the LDS address of this wavefront's patch, `out` points at row 0 of the head, the
// wavefront's rows are row0 .. row0 + nrows - 1 (at most 32; through row_map if given, its
// entries clamped to [0, map_rows) so that a bad index cannot leave the buffer); with
// `streaming` the global stores are non-temporal.  LDS operations of one wavefront execute in
// order, so no barrier is needed between the writes and the reads.
constexpr int kPatchPitch = 144;                     // 128 + 16: keeps 16-byte alignment
constexpr int kPatchBytes = 32 * kPatchPitch;        // per wavefront
__device__ __forceinline__ void store_block_rows(uint32_t patch, const f32x16 (&acc)[2], float scale,
                                                 __bf16* out, int row0, int nrows, int lane,
                                                 const int32_t* row_map = nullptr, bool streaming = false,
                                                 int map_rows = 1) {
    typedef __attribute__((address_space(3))) u32x2 lds_u32x2;
    typedef const __attribute__((address_space(3))) u32x4 lds_u32x4;
    const int lr = lane & 31, h = lane >> 5;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32x2 v = {pack_bf16(acc[mb][4 * j] * scale, acc[mb][4 * j + 1] * scale),
                             pack_bf16(acc[mb][4 * j + 2] * scale, acc[mb][4 * j + 3] * scale)};
            *(lds_u32x2*)(patch + lr * kPatchPitch + (32 * mb + 8 * j + 4 * h) * 2) = v;
        }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 8 * i + (lane >> 3), chunk = lane & 7;
        const u32x4 v = *(lds_u32x4*)(patch + row * kPatchPitch + chunk * 16);
        if (row < nrows) {
            const int r = row_map ? min(max(row_map[row0 + row], 0), map_rows - 1) : row0 + row;
            if (streaming) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out + (size_t)r * kD + chunk * 8));
            else *reinterpret_cast<u32x4*>(out + (size_t)r * kD + chunk * 8) = v;
        }
    }
}

}  // namespace hmar
