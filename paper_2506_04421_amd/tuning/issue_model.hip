// Instruction-issue microbenchmark for gfx950: what one SIMD sustains when matrix (MFMA), vector,
// transcendental and LDS instructions share it.  It fixes the cost model the kernels are judged
// against: per-instruction issue times, how much of an MFMA's
// duration vector instructions can use, LDS read bandwidth, and the per-block ceilings of the
// instruction mixes of the forward, dQ, dK/dV and a hypothetical fused backward.
//
// Build and run (one GPU, about a second):
//   hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         paper_2506_04421_amd/tuning/issue_model.hip -o issue_model && ./issue_model
// Every kernel touches only its own registers, 16 KB of LDS and one float per lane of output.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

enum Kind { kFma = 0, kExp = 1, kCvt = 2, kLds = 3, kMax3 = 4, kAdd = 5 };

template <int KIND>
__device__ __forceinline__ void one(float& v, float c, f32x4& ld, uint32_t addr) {
    if (KIND == kFma) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(v) : "v"(c));
    if (KIND == kExp) asm volatile("v_exp_f32 %0, %0" : "+v"(v));
    if (KIND == kCvt) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(v) : "v"(c));
    if (KIND == kLds) asm volatile("ds_read_b128 %0, %1" : "=v"(ld) : "v"(addr));
    if (KIND == kMax3) asm volatile("v_max3_f32 %0, %0, %1, %0" : "+v"(v) : "v"(c));
    if (KIND == kAdd) asm volatile("v_add_f32 %0, %0, %1" : "+v"(v) : "v"(c));
}

// NM matrix instructions followed by NV instructions of one kind, four times per iteration.
// SHAPE 0: v_mfma_f32_32x32x16_bf16; 1: two v_mfma_f32_16x16x32_bf16 (the same flops).
template <int NM, int NV, int KIND, int SHAPE>
__global__ __launch_bounds__(256) void pair_kernel(float* out, int iters) {
    __shared__ float4 sm[1024];
    f32x16 acc[4];
    f32x4 acc4[4];
    for (int j = 0; j < 4; ++j) {
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
        for (int i = 0; i < 4; ++i) acc4[j][i] = 0.f;
    }
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x + i); b[i] = (__bf16)1.0f; }
    float v[16];
    for (int i = 0; i < 16; ++i) v[i] = (float)threadIdx.x * 1e-3f + i;
    sm[threadIdx.x] = make_float4(1, 2, 3, 4);
    __syncthreads();
    const float c = 0.9999f;
    const uint32_t addr = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)sm + (threadIdx.x & 63) * 16;
    f32x4 ld[4] = {};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                if (SHAPE == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[(r + m) & 3]) : "v"(a), "v"(b));
                else {
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc4[(r + m) & 3]) : "v"(a), "v"(b));
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc4[(r + m + 2) & 3]) : "v"(a), "v"(b));
                }
            }
#pragma unroll
            for (int q = 0; q < NV; ++q) one<KIND>(v[q % 16], c, ld[q % 4], addr);
        }
        if (KIND == kLds) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    float s = 0;
    for (int j = 0; j < 4; ++j) { for (int i = 0; i < 16; ++i) s += acc[j][i]; s += acc4[j][0] + ld[j][0]; }
    for (int i = 0; i < 16; ++i) s += v[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The instruction mix of one 32 x 32 score block: NM matrix instructions, 16 fma, 16 exp, NADD
// adds, NCVT conversions, NMAX max3, NLDS LDS reads, evenly interleaved, no dependencies.
template <int NM, int NADD, int NCVT, int NMAX, int NLDS>
__global__ __launch_bounds__(256) void block_kernel(float* out, int iters) {
    __shared__ float4 sm[1024];
    f32x16 acc[4];
    for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x + i); b[i] = (__bf16)1.0f; }
    float v[16];
    for (int i = 0; i < 16; ++i) v[i] = (float)threadIdx.x * 1e-3f + i;
    sm[threadIdx.x] = make_float4(1, 2, 3, 4);
    __syncthreads();
    const float c = 0.9999f;
    const uint32_t addr = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)sm + (threadIdx.x & 63) * 16;
    f32x4 ld[4] = {};
    constexpr int NV = 32 + NADD + NCVT + NMAX;
    for (int it = 0; it < iters; ++it) {
        int vi = 0, li = 0;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[m & 3]) : "v"(a), "v"(b));
            const int vend = (NV * (m + 1)) / NM, lend = (NLDS * (m + 1)) / NM;
#pragma unroll
            for (; li < lend; ++li) one<kLds>(v[0], c, ld[li % 4], addr);
#pragma unroll
            for (; vi < vend; ++vi) {
                const int r = (vi * 7) % 16;
                if (vi < 16) one<kFma>(v[r], c, ld[0], addr);
                else if (vi < 32) one<kExp>(v[r], c, ld[0], addr);
                else if (vi < 32 + NADD) one<kAdd>(v[r], c, ld[0], addr);
                else if (vi < 32 + NADD + NCVT) one<kCvt>(v[r], c, ld[0], addr);
                else one<kMax3>(v[r], c, ld[0], addr);
            }
        }
        if (NLDS) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    float s = 0;
    for (int j = 0; j < 4; ++j) { for (int i = 0; i < 16; ++i) s += acc[j][i]; s += ld[j][0]; }
    for (int i = 0; i < 16; ++i) s += v[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

static float* g_out;

template <typename K>
static double time_ns(K kernel, int waves_per_simd, int iters) {
    hipEvent_t e0, e1;
    (void)hipEventCreate(&e0);
    (void)hipEventCreate(&e1);
    const dim3 grid(256 * waves_per_simd), block(256);          // one workgroup = one wavefront per SIMD of a CU
    hipLaunchKernelGGL(kernel, grid, block, 0, 0, g_out, iters / 2);    // warm-up: clocks
    (void)hipEventRecord(e0);
    hipLaunchKernelGGL(kernel, grid, block, 0, 0, g_out, iters);
    (void)hipEventRecord(e1);
    (void)hipEventSynchronize(e1);
    float ms = 0;
    (void)hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return ms * 1e6 / iters;
}

template <int NM, int NV, int KIND, int SHAPE>
static void pair_line(const char* name) {
    printf("%-36s", name);
    for (int w = 1; w <= 4; ++w) printf("  %7.1f", time_ns(pair_kernel<NM, NV, KIND, SHAPE>, w, 4000) / 4.0 / w);
    printf("\n");
    fflush(stdout);
}

template <int NM, int NADD, int NCVT, int NMAX, int NLDS>
static void block_line(const char* name) {
    printf("%-36s", name);
    for (int w = 1; w <= 4; ++w) printf("  %7.1f", time_ns(block_kernel<NM, NADD, NCVT, NMAX, NLDS>, w, 4000) / w);
    printf("   (matrix pipe alone: %5.1f)\n", NM * 15.1);
    fflush(stdout);
}

int main() {
    if (hipMalloc(&g_out, 256 * 4 * 256 * sizeof(float)) != hipSuccess) return 1;
    printf("ns per group and SIMD (all resident wavefronts of the SIMD together), at 1 / 2 / 3 / 4 wavefronts per SIMD\n");
    pair_line<0, 16, kFma, 0>("16 v_fma_f32");
    pair_line<0, 16, kAdd, 0>("16 v_add_f32");
    pair_line<0, 16, kExp, 0>("16 v_exp_f32");
    pair_line<0, 16, kCvt, 0>("16 v_cvt_pk_bf16_f32");
    pair_line<0, 16, kMax3, 0>("16 v_max3_f32");
    pair_line<0, 16, kLds, 0>("16 ds_read_b128 (1 KB each)");
    pair_line<1, 0, kFma, 0>("1 mfma 32x32x16");
    pair_line<1, 0, kFma, 1>("2 mfma 16x16x32");
    pair_line<1, 4, kFma, 0>("1 mfma 32x32x16 + 4 fma");
    pair_line<1, 8, kFma, 0>("1 mfma 32x32x16 + 8 fma");
    pair_line<1, 12, kFma, 0>("1 mfma 32x32x16 + 12 fma");
    pair_line<1, 16, kFma, 0>("1 mfma 32x32x16 + 16 fma");
    pair_line<1, 8, kFma, 1>("2 mfma 16x16x32 + 8 fma");
    pair_line<1, 16, kFma, 1>("2 mfma 16x16x32 + 16 fma");
    pair_line<1, 4, kExp, 0>("1 mfma 32x32x16 + 4 exp");
    pair_line<1, 8, kExp, 0>("1 mfma 32x32x16 + 8 exp");
    pair_line<1, 8, kExp, 1>("2 mfma 16x16x32 + 8 exp");
    pair_line<1, 1, kLds, 0>("1 mfma 32x32x16 + 1 ds_read_b128");
    pair_line<1, 4, kLds, 0>("1 mfma 32x32x16 + 4 ds_read_b128");
    printf("\nns per 32 x 32 score block and SIMD, instruction mix of each kernel, interleaved, no dependencies\n");
    block_line<8, 16, 8, 8, 12>("forward  (8 mfma, 64 valu, 12 lds)");
    block_line<8, 0, 8, 8, 12>("forward without the row-sum adds");
    block_line<12, 16, 8, 0, 12>("dQ       (12 mfma, 72 valu, 12 lds)");
    block_line<16, 16, 16, 0, 17>("dK/dV    (16 mfma, 64 valu, 17 lds)");
    block_line<20, 16, 16, 0, 24>("fused backward (20 mfma, 24 lds)");
    (void)hipFree(g_out);
    return 0;
}
