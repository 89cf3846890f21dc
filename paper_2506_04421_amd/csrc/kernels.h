// Launchers of the gfx950 kernels (internal to the library; the public ABI is hmar_attn.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hmar {

// Device copy of the tile schedule of one (device, scale schedule) pair.
struct DeviceSchedule {
    const void* items[2];      // Item[n_items[dir]]
    int32_t n_items[2];
    const int32_t* row_lo[2];  // L entries
    const int32_t* row_hi[2];
    int32_t L;                 // rows of Q, O, LSE per head
    int32_t Lk;                // rows of K, V per head
    int32_t num_cus;           // compute units of the device the tables live on
};

// Number of head groups (8 heads each) in the batch that ends a launch item by item (see
// map_workgroup): about twice as many (head, item) units as one XCD keeps resident at four
// workgroups per CU.  Measured on the 256px and 512px training shapes (forward+backward step):
// without the batch +1.5 % and +3.8 %; half the size 0 and +1.7 %; twice the size +1.7 % and +1 %;
// batching the whole launch this way instead of its end only loses more in L2 locality than it
// gains.
#ifndef HMAR_TUNE_TAIL_PERCENT
#define HMAR_TUNE_TAIL_PERCENT 100     // measurement builds: size of the batch relative to the shipped one
#endif
inline int tail_groups_for(int num_cus, int n_items) {
    const int g = ((num_cus / 8) * 8) * HMAR_TUNE_TAIL_PERCENT / 100 / (n_items > 0 ? n_items : 1);
    return g < 1 ? 1 : g;
}

// Per-kernel event bracketing for hmar_profile_begin/end (no-ops unless profiling is on).
enum KernelId { kKernelFwd = 0, kKernelDkDv = 1, kKernelDq = 2, kNumKernels = 3 };
void profile_before(int kernel_id, hipStream_t stream);
void profile_after(int kernel_id, hipStream_t stream);

// Up to kMaxSteps independent inference steps in one launch (host view; the launcher turns it
// into kernel arguments).  Steps must be ordered by decreasing work.
constexpr int kMaxSteps = 16;
struct StepLaunch {
    struct Step {
        const void* Q; const void* K; const void* V; void* O; float* LSE;
        const int32_t* rows;    // device, optional: the n_q rows of Q/O/LSE the step covers
        int32_t n_q, q_stride, Lk;
    } step[kMaxSteps];
    int32_t n_steps;
};
hipError_t launch_fwd_steps(const StepLaunch& L, int n_heads, float sm_scale, int num_cus, hipStream_t stream);

hipError_t launch_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                      const DeviceSchedule& s, int n_heads, float sm_scale, hipStream_t stream);

hipError_t launch_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                      const float* LSE, void* dQ, void* dK, void* dV, float* workspace,
                      const DeviceSchedule& s, int n_heads, float sm_scale, hipStream_t stream);

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);

}  // namespace hmar
