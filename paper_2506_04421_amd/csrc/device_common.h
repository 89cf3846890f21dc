// Shared device-side types and helpers of the gfx950 attention kernels.
//
// MFMA register layouts used throughout (v_mfma_f32_32x32x16_bf16, wave64), with
// lr = lane % 32 and h = lane / 32:
//   A operand (M x 16): lane holds row lr, 8 consecutive k of half h (k = 8h .. 8h+7)
//   B operand (16 x N): lane holds column lr, the same 8 k
//   C/D      (M x N)  : lane holds column lr; register i holds row 8*(i/4) + 4*h + i%4
// The contraction index only has to be enumerated identically by A and B, so a C tile
// can be fed back as a B operand without moving data between lanes: registers 8s..8s+7
// of a C tile (s = 0, 1) are "k = 0..7 of half h" of a 16-deep step whose k-th row is
// row 16s + 8*(k/4) + 4h + k%4 of the tile; the A operand is then read from LDS with the
// same row enumeration (two 4-element groups, 8 rows apart).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hmar {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // plain vector types: HIP's uint4/uint2
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;   // structs copy through memory

constexpr int kD = 64;        // head dimension
constexpr int kTile = 64;     // streamed rows per LDS tile
constexpr int kLdRow = 72;    // pitch (bf16) of a row-major [rows][64] tile: 64 + 8 pad, 144 B
constexpr int kLdTr = 68;     // pitch (bf16) of a transposed [64 d][rows] tile: 64 + 4 pad, 136 B
constexpr int kThreads = 256; // 4 wavefronts
constexpr int kRowsPerWave = 32;
constexpr int kRowsPerItem = 128;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;

struct alignas(16) Item { int32_t own_begin, own_end, other_begin, other_end; };

// Workgroup -> (head, item).  Workgroups are handed to the 8 XCDs round-robin, so all
// items of one head are given ids that are congruent mod 8: they then run on one XCD and
// share its L2 for the rows they re-read.
__device__ __forceinline__ bool map_workgroup(int n_items, int n_heads, int* head, int* item) {
    const int wg = blockIdx.x;
    const int xcd = wg & 7;
    const int slot = wg >> 3;
    *head = (slot / n_items) * 8 + xcd;
    *item = slot % n_items;
    return *head < n_heads;
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

__device__ __forceinline__ int wave_min(int x) {
    for (int o = 32; o > 0; o >>= 1) x = min(x, __shfl_xor(x, o));
    return __builtin_amdgcn_readfirstlane(x);
}
__device__ __forceinline__ int wave_max(int x) {
    for (int o = 32; o > 0; o >>= 1) x = max(x, __shfl_xor(x, o));
    return __builtin_amdgcn_readfirstlane(x);
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

// ---- staging of one 64-row tile of a [rows][64] bf16 matrix into LDS --------------------
// row-major copy: thread t moves rows t/8 and 32 + t/8, 16-byte column chunk t%8
struct RowRegs { u32x4 a, b; };
__device__ __forceinline__ void load_rows(RowRegs& r, const __bf16* base, int row0, int row_max, int tid) {
    const int rr = tid >> 3, c = tid & 7;
    const int a = min(row0 + rr, row_max), b = min(row0 + 32 + rr, row_max);
    r.a = *reinterpret_cast<const u32x4*>(base + (size_t)a * kD + c * 8);
    r.b = *reinterpret_cast<const u32x4*>(base + (size_t)b * kD + c * 8);
}
__device__ __forceinline__ void store_rows(const RowRegs& r, __bf16* lds, int tid) {
    const int rr = tid >> 3, c = tid & 7;
    *reinterpret_cast<u32x4*>(lds + rr * kLdRow + c * 8) = r.a;
    *reinterpret_cast<u32x4*>(lds + (rr + 32) * kLdRow + c * 8) = r.b;
}

// transposed copy: thread t moves rows 4*(t/16) .. +3, 4-column chunk t%16, and writes the
// 4x4 block transposed (4 rows of one column packed in 8 bytes) into a [64 col][rows] tile
struct TrRegs { u32x2 v0, v1, v2, v3; };
__device__ __forceinline__ void load_tr(TrRegs& r, const __bf16* base, int row0, int row_max, int tid) {
    const int c = tid & 15, g = tid >> 4;
    const int r0 = row0 + 4 * g;
    r.v0 = *reinterpret_cast<const u32x2*>(base + (size_t)min(r0 + 0, row_max) * kD + c * 4);
    r.v1 = *reinterpret_cast<const u32x2*>(base + (size_t)min(r0 + 1, row_max) * kD + c * 4);
    r.v2 = *reinterpret_cast<const u32x2*>(base + (size_t)min(r0 + 2, row_max) * kD + c * 4);
    r.v3 = *reinterpret_cast<const u32x2*>(base + (size_t)min(r0 + 3, row_max) * kD + c * 4);
}
__device__ __forceinline__ void store_tr(const TrRegs& r, __bf16* lds, int tid) {
    const int c = tid & 15, g = tid >> 4;
    constexpr uint32_t kLo = 0x05040100u, kHi = 0x07060302u;
    u32x2 w;
    __bf16* dst = lds + (4 * c) * kLdTr + 4 * g;
    w.x = __builtin_amdgcn_perm(r.v1.x, r.v0.x, kLo);
    w.y = __builtin_amdgcn_perm(r.v3.x, r.v2.x, kLo);
    *reinterpret_cast<u32x2*>(dst) = w;
    w.x = __builtin_amdgcn_perm(r.v1.x, r.v0.x, kHi);
    w.y = __builtin_amdgcn_perm(r.v3.x, r.v2.x, kHi);
    *reinterpret_cast<u32x2*>(dst + kLdTr) = w;
    w.x = __builtin_amdgcn_perm(r.v1.y, r.v0.y, kLo);
    w.y = __builtin_amdgcn_perm(r.v3.y, r.v2.y, kLo);
    *reinterpret_cast<u32x2*>(dst + 2 * kLdTr) = w;
    w.x = __builtin_amdgcn_perm(r.v1.y, r.v0.y, kHi);
    w.y = __builtin_amdgcn_perm(r.v3.y, r.v2.y, kHi);
    *reinterpret_cast<u32x2*>(dst + 3 * kLdTr) = w;
}

// A operand from a row-major tile: row `row`, columns 16*t + 8*h .. +7
__device__ __forceinline__ bf16x8 lds_a_row(const __bf16* tile, int row, int t, int h) {
    return *reinterpret_cast<const bf16x8*>(tile + row * kLdRow + 16 * t + 8 * h);
}
// A operand from a transposed tile for 16-deep step tp: row `col` of the transposed tile,
// tile rows 16tp+4h..+3 and 16tp+8+4h..+3 (the enumeration a C tile fed back as B uses)
__device__ __forceinline__ bf16x8 lds_a_tr(const __bf16* tile, int col, int tp, int h) {
    const __bf16* p = tile + col * kLdTr + 16 * tp + 4 * h;
    u32x2 lo = *reinterpret_cast<const u32x2*>(p);
    u32x2 hi = *reinterpret_cast<const u32x2*>(p + 8);
    u32x4 u = {lo.x, lo.y, hi.x, hi.y};
    return __builtin_bit_cast(bf16x8, u);
}

// store 4 consecutive fp32 of one output row as bf16 (8 bytes)
__device__ __forceinline__ void store4_bf16(__bf16* dst, float a, float b, float c, float d) {
    u32x2 u = {pack_bf16(a, b), pack_bf16(c, d)};
    *reinterpret_cast<u32x2*>(dst) = u;
}

}  // namespace hmar
