// C ABI of the library (see include/hmar_attn.h): argument checks, the per-(device,
// schedule) cache of tile tables, and the kernel launches.
#include "hmar_attn.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <tuple>
#include <utility>
#include <vector>

#include "kernels.h"
#include "schedule.h"

namespace {

constexpr int kRowsPerItem = 128;   // rows owned by one workgroup: 4 wavefronts x 32

struct CachedSchedule {
    hmar::Schedule host;
    hmar::DeviceSchedule dev{};
    void* blob = nullptr;   // one device allocation holding every table
};

std::mutex g_mu;
// key: device, mask kind (+ the counts flag), sizes as given (for an inference step: {n_prev, n_cur})
std::map<std::tuple<int, int32_t, std::vector<int32_t>>, std::unique_ptr<CachedSchedule>> g_cache;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks that need no device.  On success *L is the sequence length.
hmar_status check_problem(const int32_t* side_lens, int32_t num_scales, int32_t mask_kind, int32_t B, int32_t H,
                          int32_t D, hmar::Schedule* sched) {
    if (!side_lens || num_scales < 1 || B < 1 || H < 1 || D < 1) return HMAR_ERR_INVALID_ARG;
    if (mask_kind < 0 || (mask_kind & ~(HMAR_SCALE_COUNTS | 0xFF))) return HMAR_ERR_INVALID_ARG;
    const bool counts = (mask_kind & HMAR_SCALE_COUNTS) != 0;
    mask_kind &= 0xFF;
    if (mask_kind != HMAR_MASK_MARKOV && mask_kind != HMAR_MASK_BLOCK_CAUSAL) return HMAR_ERR_INVALID_ARG;
    for (int32_t k = 0; k < num_scales && k < HMAR_MAX_SCALES; ++k)
        if (side_lens[k] < 1) return HMAR_ERR_INVALID_ARG;
    if (num_scales > HMAR_MAX_SCALES) return HMAR_ERR_UNSUPPORTED;
    if (D != 64) return HMAR_ERR_UNSUPPORTED;
    if (!hmar::build_schedule(side_lens, num_scales, counts, mask_kind, kRowsPerItem, HMAR_MAX_SCALES, HMAR_MAX_SEQ_LEN, sched))
        return HMAR_ERR_UNSUPPORTED;   // only L > HMAR_MAX_SEQ_LEN (or side > 46340) is left
    if ((int64_t)B * H > (1 << 24)) return HMAR_ERR_UNSUPPORTED;
    return HMAR_OK;
}

// Returns the cached device tables of this schedule on the current device, building and
// uploading them on first use.
hmar_status get_device_schedule(hmar::Schedule&& host, hipStream_t stream, const hmar::DeviceSchedule** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return HMAR_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mu);
    auto key = std::make_tuple(dev, host.mask_kind | (host.sizes_are_counts ? HMAR_SCALE_COUNTS : 0), host.sides);
    auto it = g_cache.find(key);
    if (it != g_cache.end()) { *out = &it->second->dev; return HMAR_OK; }

    auto cs = std::make_unique<CachedSchedule>();
    cs->host = std::move(host);
    const hmar::Schedule& s = cs->host;
    const size_t L = (size_t)s.L;
    // layout: items[0] | items[1] | row_lo[0] | row_hi[0] | row_lo[1] | row_hi[1]
    const size_t item_bytes[2] = {s.items[0].size() * sizeof(hmar::TileItem), s.items[1].size() * sizeof(hmar::TileItem)};
    const size_t total = item_bytes[0] + item_bytes[1] + 4 * L * sizeof(int32_t);
    for (int d = 0; d < 2; ++d) {      // an inference-step schedule has no backward direction
        cs->host.row_lo[d].resize(L, 0);
        cs->host.row_hi[d].resize(L, 0);
    }
    std::vector<unsigned char> staging(total);
    size_t o = 0;
    size_t off_items[2], off_lo[2], off_hi[2];
    for (int d = 0; d < 2; ++d) { off_items[d] = o; std::memcpy(&staging[o], s.items[d].data(), item_bytes[d]); o += item_bytes[d]; }
    for (int d = 0; d < 2; ++d) {
        off_lo[d] = o; std::memcpy(&staging[o], s.row_lo[d].data(), L * 4); o += L * 4;
        off_hi[d] = o; std::memcpy(&staging[o], s.row_hi[d].data(), L * 4); o += L * 4;
    }
    if (hipMalloc(&cs->blob, total) != hipSuccess) return HMAR_ERR_HIP;
    // synchronous copy from pageable memory: complete when it returns, so later launches on
    // any stream see the tables
    if (hipMemcpy(cs->blob, staging.data(), total, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(cs->blob);
        return HMAR_ERR_HIP;
    }
    (void)stream;
    unsigned char* base = static_cast<unsigned char*>(cs->blob);
    for (int d = 0; d < 2; ++d) {
        cs->dev.items[d] = base + off_items[d];
        cs->dev.n_items[d] = (int32_t)s.items[d].size();
        cs->dev.row_lo[d] = reinterpret_cast<const int32_t*>(base + off_lo[d]);
        cs->dev.row_hi[d] = reinterpret_cast<const int32_t*>(base + off_hi[d]);
    }
    cs->dev.L = s.L;
    cs->dev.Lk = s.Lk;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
        (void)hipFree(cs->blob);
        return HMAR_ERR_HIP;
    }
    cs->dev.num_cus = cus;
    *out = &cs->dev;
    g_cache.emplace(std::move(key), std::move(cs));
    return HMAR_OK;
}

// ---- per-kernel event profiling (hmar_profile_begin / hmar_profile_end) ----------------
struct ProfRecord { int kernel_id; hipEvent_t start, stop; };
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfRecord> g_prof_records;
hipEvent_t g_prof_pending_start = nullptr;

float resolve_scale(float sm_scale, int32_t D) {
    return sm_scale > 0.f ? sm_scale : 1.0f / std::sqrt((float)D);
}

}  // namespace

namespace hmar {

void profile_before(int kernel_id, hipStream_t stream) {
    (void)kernel_id;
    std::lock_guard<std::mutex> lock(g_prof_mu);
    if (!g_prof_on) return;
    g_prof_pending_start = nullptr;
    hipEvent_t ev;
    if (hipEventCreate(&ev) != hipSuccess) return;
    if (hipEventRecord(ev, stream) != hipSuccess) { (void)hipEventDestroy(ev); return; }
    g_prof_pending_start = ev;
}

void profile_after(int kernel_id, hipStream_t stream) {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    if (!g_prof_on || !g_prof_pending_start) return;
    hipEvent_t ev;
    if (hipEventCreate(&ev) != hipSuccess || hipEventRecord(ev, stream) != hipSuccess) {
        (void)hipEventDestroy(g_prof_pending_start);
        g_prof_pending_start = nullptr;
        return;
    }
    g_prof_records.push_back({kernel_id, g_prof_pending_start, ev});
    g_prof_pending_start = nullptr;
}

}  // namespace hmar

extern "C" {

hmar_status hmar_profile_begin(void) {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    for (auto& r : g_prof_records) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    g_prof_records.clear();
    g_prof_on = true;
    return HMAR_OK;
}

hmar_status hmar_profile_end(double* total_ms_out, int64_t* launches_out) {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    g_prof_on = false;
    double ms[HMAR_NUM_KERNELS] = {0, 0, 0};
    int64_t n[HMAR_NUM_KERNELS] = {0, 0, 0};
    hmar_status st = HMAR_OK;
    for (auto& r : g_prof_records) {
        float t = 0.f;
        if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess)
            st = HMAR_ERR_HIP;
        else if (r.kernel_id >= 0 && r.kernel_id < HMAR_NUM_KERNELS) { ms[r.kernel_id] += t; n[r.kernel_id] += 1; }
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_prof_records.clear();
    for (int i = 0; i < HMAR_NUM_KERNELS; ++i) {
        if (total_ms_out) total_ms_out[i] = ms[i];
        if (launches_out) launches_out[i] = n[i];
    }
    return st;
}

const char* hmar_status_string(hmar_status s) {
    switch (s) {
        case HMAR_OK: return "HMAR_OK";
        case HMAR_ERR_INVALID_ARG: return "HMAR_ERR_INVALID_ARG";
        case HMAR_ERR_UNSUPPORTED: return "HMAR_ERR_UNSUPPORTED";
        case HMAR_ERR_WORKSPACE: return "HMAR_ERR_WORKSPACE";
        case HMAR_ERR_HIP: return "HMAR_ERR_HIP";
    }
    return "HMAR_ERR_UNKNOWN";
}

hmar_status hmar_attn_fwd_masked(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                 const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                                 int32_t B, int32_t H, int32_t D, float sm_scale, void* stream) {
    if (!Q || !K || !V || !O || !LSE) return HMAR_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE)) return HMAR_ERR_INVALID_ARG;
    if (!std::isfinite(sm_scale)) return HMAR_ERR_INVALID_ARG;
    hmar::Schedule host;
    hmar_status st = check_problem(side_lens, num_scales, mask_kind, B, H, D, &host);
    if (st != HMAR_OK) return st;
    const hmar::DeviceSchedule* ds = nullptr;
    st = get_device_schedule(std::move(host), static_cast<hipStream_t>(stream), &ds);
    if (st != HMAR_OK) return st;
    hipError_t e = hmar::launch_fwd(Q, K, V, O, LSE, *ds, B * H, resolve_scale(sm_scale, D),
                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HMAR_OK : HMAR_ERR_HIP;
}

hmar_status hmar_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                          const int32_t* side_lens, int32_t num_scales,
                          int32_t B, int32_t H, int32_t D, float sm_scale, void* stream) {
    return hmar_attn_fwd_masked(Q, K, V, O, LSE, side_lens, num_scales, HMAR_MASK_MARKOV, B, H, D, sm_scale, stream);
}

hmar_status hmar_attn_step_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                               int32_t n_prev, int32_t n_cur, int32_t B, int32_t H, int32_t D,
                               float sm_scale, void* stream) {
    if (!Q || !K || !V || !O || !LSE) return HMAR_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE)) return HMAR_ERR_INVALID_ARG;
    if (!std::isfinite(sm_scale) || n_prev < 0 || n_cur < 1 || B < 1 || H < 1 || D < 1) return HMAR_ERR_INVALID_ARG;
    if (D != 64 || (int64_t)B * H > (1 << 24)) return HMAR_ERR_UNSUPPORTED;
    hmar::Schedule host;
    if (!hmar::build_step_schedule(n_prev, n_cur, kRowsPerItem, HMAR_MAX_SEQ_LEN, &host)) return HMAR_ERR_UNSUPPORTED;
    const hmar::DeviceSchedule* ds = nullptr;
    hmar_status st = get_device_schedule(std::move(host), static_cast<hipStream_t>(stream), &ds);
    if (st != HMAR_OK) return st;
    hipError_t e = hmar::launch_fwd(Q, K, V, O, LSE, *ds, B * H, resolve_scale(sm_scale, D),
                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HMAR_OK : HMAR_ERR_HIP;
}

size_t hmar_attn_bwd_workspace_bytes_masked(const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                                            int32_t B, int32_t H, int32_t D) {
    hmar::Schedule host;
    if (check_problem(side_lens, num_scales, mask_kind, B, H, D, &host) != HMAR_OK) return 0;
    return 2 * (size_t)B * H * host.L * sizeof(float);
}

size_t hmar_attn_bwd_workspace_bytes(const int32_t* side_lens, int32_t num_scales,
                                     int32_t B, int32_t H, int32_t D) {
    return hmar_attn_bwd_workspace_bytes_masked(side_lens, num_scales, HMAR_MASK_MARKOV, B, H, D);
}

hmar_status hmar_attn_bwd_masked(const void* Q, const void* K, const void* V, const void* O,
                                 const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                                 const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                                 int32_t B, int32_t H, int32_t D, float sm_scale,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV) return HMAR_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(dO) || !aligned16(LSE) ||
        !aligned16(dQ) || !aligned16(dK) || !aligned16(dV))
        return HMAR_ERR_INVALID_ARG;
    if (!std::isfinite(sm_scale)) return HMAR_ERR_INVALID_ARG;
    hmar::Schedule host;
    hmar_status st = check_problem(side_lens, num_scales, mask_kind, B, H, D, &host);
    if (st != HMAR_OK) return st;
    const size_t need = 2 * (size_t)B * H * host.L * sizeof(float);
    if (!workspace || workspace_bytes < need) return HMAR_ERR_WORKSPACE;
    if (!aligned16(workspace)) return HMAR_ERR_INVALID_ARG;
    const hmar::DeviceSchedule* ds = nullptr;
    st = get_device_schedule(std::move(host), static_cast<hipStream_t>(stream), &ds);
    if (st != HMAR_OK) return st;
    hipError_t e = hmar::launch_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, static_cast<float*>(workspace), *ds, B * H,
                                    resolve_scale(sm_scale, D), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HMAR_OK : HMAR_ERR_HIP;
}

hmar_status hmar_attn_bwd(const void* Q, const void* K, const void* V, const void* O,
                          const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                          const int32_t* side_lens, int32_t num_scales,
                          int32_t B, int32_t H, int32_t D, float sm_scale,
                          void* workspace, size_t workspace_bytes, void* stream) {
    return hmar_attn_bwd_masked(Q, K, V, O, dO, LSE, dQ, dK, dV, side_lens, num_scales, HMAR_MASK_MARKOV, B, H, D,
                                sm_scale, workspace, workspace_bytes, stream);
}

hmar_status hmar_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || (bytes & 15u) || !aligned16(dst) || !aligned16(src)) return HMAR_ERR_INVALID_ARG;
    return hmar::launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? HMAR_OK : HMAR_ERR_HIP;
}

hmar_status hmar_schedule_describe(const int32_t* side_lens, int32_t num_scales,
                                   int32_t* offsets_out, int64_t* allowed_pairs_out) {
    hmar::Schedule host;
    hmar_status st = check_problem(side_lens, num_scales, HMAR_MASK_MARKOV, 1, 1, 64, &host);
    if (st != HMAR_OK) return st;
    if (offsets_out) std::memcpy(offsets_out, host.off.data(), host.off.size() * sizeof(int32_t));
    if (allowed_pairs_out) *allowed_pairs_out = host.allowed_pairs;
    return HMAR_OK;
}

hmar_status hmar_schedule_tiles(const int32_t* side_lens, int32_t num_scales, int32_t which,
                                int32_t* items_out, int32_t max_items, int32_t* n_items_out,
                                int32_t* row_lo_out, int32_t* row_hi_out) {
    // which: bit 0 = direction, bit 1 = block-causal mask instead of the Markovian one,
    // bit 2 = the sizes are token counts instead of side lengths
    if (which < 0 || which > 7 || !n_items_out || max_items < 0) return HMAR_ERR_INVALID_ARG;
    const int32_t mask_kind = ((which & 2) ? HMAR_MASK_BLOCK_CAUSAL : HMAR_MASK_MARKOV) | ((which & 4) ? HMAR_SCALE_COUNTS : 0);
    which &= 1;
    hmar::Schedule host;
    hmar_status st = check_problem(side_lens, num_scales, mask_kind, 1, 1, 64, &host);
    if (st != HMAR_OK) return st;
    const auto& items = host.items[which];
    *n_items_out = (int32_t)items.size();
    if (items_out) {
        const size_t n = std::min<size_t>(items.size(), (size_t)max_items);
        std::memcpy(items_out, items.data(), n * sizeof(hmar::TileItem));
    }
    if (row_lo_out) std::memcpy(row_lo_out, host.row_lo[which].data(), (size_t)host.L * 4);
    if (row_hi_out) std::memcpy(row_hi_out, host.row_hi[which].data(), (size_t)host.L * 4);
    return HMAR_OK;
}

}  // extern "C"
