// Host-side helpers shared by the entry points of the library (api.cpp, no_alloc.hip).
#pragma once
#include <cstddef>
#include <cstdint>

#include "hmar_attn.h"
#include "kernels.h"
#include "schedule.h"

namespace hmar {

constexpr int kRowsPerItem = 128;   // rows owned by one workgroup: 4 wavefronts x 32

// What the argument checks establish about a training-shape call.
struct Problem {
    int32_t mask_kind;   // HMAR_MASK_* without flags
    bool counts;         // sizes are token counts
    int32_t L;           // sum of the scales' token counts
    int32_t n_heads;     // B * H
};

bool aligned16(const void* p);
float resolve_scale(float sm_scale, int32_t D);
hmar_status check_problem(const int32_t* sizes, int32_t num_scales, int32_t mask_kind, int32_t B, int32_t H,
                          int32_t D, Problem* out);
hmar_status check_bwd_args(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                           const float* LSE, void* dQ, void* dK, void* dV,
                           const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                           int32_t B, int32_t H, int32_t D, float sm_scale, Problem* pb);
bool build_host_schedule(const int32_t* sizes, int32_t num_scales, const Problem& pb, Schedule* out);
size_t table_bytes(const Schedule& s);
void pack_tables(const Schedule& s, unsigned char* staging, unsigned char* base, DeviceSchedule* dev);
int device_cus(int dev);   // compute units of a device (cached), -1 on error

}  // namespace hmar
