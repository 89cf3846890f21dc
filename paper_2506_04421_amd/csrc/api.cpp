// C ABI of the library (see include/hmar_attn.h): argument checks, the per-(device,
// schedule) cache of tile tables, and the kernel launches.
#include "hmar_attn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <tuple>
#include <utility>
#include <vector>

#include "api_internal.h"
#include "kernels.h"
#include "schedule.h"

namespace hmar {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

float resolve_scale(float sm_scale, int32_t D) {
    return sm_scale > 0.f ? sm_scale : 1.0f / std::sqrt((float)D);
}

// Checks that need neither a device nor the tile lists: one pass over the sizes.
hmar_status check_problem(const int32_t* sizes, int32_t num_scales, int32_t mask_kind, int32_t B, int32_t H,
                          int32_t D, Problem* out) {
    if (!sizes || num_scales < 1 || B < 1 || H < 1 || D < 1) return HMAR_ERR_INVALID_ARG;
    if (mask_kind < 0 || (mask_kind & ~(HMAR_SCALE_COUNTS | 0xFF))) return HMAR_ERR_INVALID_ARG;
    const bool counts = (mask_kind & HMAR_SCALE_COUNTS) != 0;
    const int32_t kind = mask_kind & 0xFF;
    if (kind != HMAR_MASK_MARKOV && kind != HMAR_MASK_BLOCK_CAUSAL) return HMAR_ERR_INVALID_ARG;
    for (int32_t k = 0; k < num_scales && k < HMAR_MAX_SCALES; ++k)
        if (sizes[k] < 1) return HMAR_ERR_INVALID_ARG;
    if (num_scales > HMAR_MAX_SCALES) return HMAR_ERR_UNSUPPORTED;
    if (D != 64) return HMAR_ERR_UNSUPPORTED;
    int64_t L = 0;
    for (int32_t k = 0; k < num_scales; ++k) {
        L += counts ? (int64_t)sizes[k] : (int64_t)sizes[k] * sizes[k];
        if (L > HMAR_MAX_SEQ_LEN) return HMAR_ERR_UNSUPPORTED;     // also every L that would not fit 32 bits
    }
    if ((int64_t)B * H > (1 << 24)) return HMAR_ERR_UNSUPPORTED;
    out->mask_kind = kind;
    out->counts = counts;
    out->L = (int32_t)L;
    out->n_heads = B * H;
    return HMAR_OK;
}

hmar_status check_bwd_args(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                           const float* LSE, void* dQ, void* dK, void* dV,
                           const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                           int32_t B, int32_t H, int32_t D, float sm_scale, Problem* pb) {
    if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV) return HMAR_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(dO) || !aligned16(LSE) ||
        !aligned16(dQ) || !aligned16(dK) || !aligned16(dV))
        return HMAR_ERR_INVALID_ARG;
    if (!std::isfinite(sm_scale)) return HMAR_ERR_INVALID_ARG;
    return check_problem(side_lens, num_scales, mask_kind, B, H, D, pb);
}

bool build_host_schedule(const int32_t* sizes, int32_t num_scales, const Problem& pb, Schedule* out) {
    return build_schedule(sizes, num_scales, pb.counts, pb.mask_kind, kRowsPerItem, HMAR_MAX_SCALES, HMAR_MAX_SEQ_LEN, out);
}

size_t table_bytes(const Schedule& s) {
    return (s.items[0].size() + s.items[1].size()) * sizeof(TileItem) + 4 * (size_t)s.L * sizeof(int32_t);
}

// Lays the tables of `s` out in `staging` (table_bytes(s) bytes: items[0] | items[1] | row_lo[0] |
// row_hi[0] | row_lo[1] | row_hi[1]) and fills `dev` with their addresses once copied to `base`.
void pack_tables(const Schedule& s, unsigned char* staging, unsigned char* base, DeviceSchedule* dev) {
    const size_t L = (size_t)s.L;
    size_t o = 0;
    for (int d = 0; d < 2; ++d) {
        const size_t bytes = s.items[d].size() * sizeof(TileItem);
        std::memcpy(staging + o, s.items[d].data(), bytes);
        dev->items[d] = base + o;
        dev->n_items[d] = (int32_t)s.items[d].size();
        o += bytes;
    }
    for (int d = 0; d < 2; ++d) {
        std::memcpy(staging + o, s.row_lo[d].data(), L * 4);
        dev->row_lo[d] = reinterpret_cast<const int32_t*>(base + o);
        o += L * 4;
        std::memcpy(staging + o, s.row_hi[d].data(), L * 4);
        dev->row_hi[d] = reinterpret_cast<const int32_t*>(base + o);
        o += L * 4;
    }
    dev->L = s.L;
    dev->Lk = s.Lk;
}

int device_cus(int dev) {
    static std::mutex mu;
    static std::map<int, int> cus;
    std::lock_guard<std::mutex> lock(mu);
    auto it = cus.find(dev);
    if (it != cus.end()) return it->second;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) return -1;
    cus[dev] = n;
    return n;
}

}  // namespace hmar

namespace {

using hmar::Problem;

struct CachedSchedule {
    hmar::DeviceSchedule dev{};
    void* blob = nullptr;   // one device allocation holding every table
};

std::mutex g_mu;
// key: device, mask kind (+ the counts flag), sizes as given
typedef std::tuple<int, int32_t, std::vector<int32_t>> CacheKey;
std::map<CacheKey, std::unique_ptr<CachedSchedule>> g_cache;

// Returns the cached device tables of this schedule on the current device.  The host tables are
// only built (and uploaded) on the first use of a schedule on a device: a hit costs one map
// lookup on the sizes.
hmar_status get_device_schedule(const int32_t* sizes, int32_t num_scales, const Problem& pb,
                                const hmar::DeviceSchedule** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return HMAR_ERR_HIP;
    CacheKey key(dev, pb.mask_kind | (pb.counts ? HMAR_SCALE_COUNTS : 0), std::vector<int32_t>(sizes, sizes + num_scales));
    std::lock_guard<std::mutex> lock(g_mu);
    auto it = g_cache.find(key);
    if (it != g_cache.end()) { *out = &it->second->dev; return HMAR_OK; }

    hmar::Schedule s;
    if (!hmar::build_host_schedule(sizes, num_scales, pb, &s)) return HMAR_ERR_UNSUPPORTED;
    auto cs = std::make_unique<CachedSchedule>();
    const size_t total = hmar::table_bytes(s);
    std::vector<unsigned char> staging(total);
    const int cus = hmar::device_cus(dev);
    if (cus < 1) return HMAR_ERR_HIP;
    if (hipMalloc(&cs->blob, total) != hipSuccess) return HMAR_ERR_HIP;
    hmar::pack_tables(s, staging.data(), static_cast<unsigned char*>(cs->blob), &cs->dev);
    cs->dev.num_cus = cus;
    // synchronous copy from pageable memory: complete when it returns, so later launches on
    // any stream see the tables
    if (hipMemcpy(cs->blob, staging.data(), total, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(cs->blob);
        return HMAR_ERR_HIP;
    }
    *out = &cs->dev;
    g_cache.emplace(std::move(key), std::move(cs));
    return HMAR_OK;
}

// ---- per-kernel event profiling (hmar_profile_begin / hmar_profile_end) ----------------
struct ProfRecord { int kernel_id; hipEvent_t start, stop; };
std::mutex g_prof_mu;
bool g_prof_on = false;
bool g_prof_stream_set = false;       // the first launch after hmar_profile_begin fixes the stream
bool g_prof_mixed_streams = false;    // a launch on another stream was seen (and not recorded)
hipStream_t g_prof_stream = nullptr;
std::vector<ProfRecord> g_prof_records;
hipEvent_t g_prof_pending_start = nullptr;

hmar_status check_step(const void* Q, const void* K, const void* V, void* O, float* LSE,
                       int32_t n_prev, int32_t n_cur) {
    using hmar::aligned16;
    if (!Q || !K || !V || !O || !LSE) return HMAR_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE)) return HMAR_ERR_INVALID_ARG;
    if (n_prev < 0 || n_cur < 1) return HMAR_ERR_INVALID_ARG;
    if ((int64_t)n_prev + n_cur > HMAR_MAX_SEQ_LEN) return HMAR_ERR_UNSUPPORTED;
    return HMAR_OK;
}

// Inference steps need no tables and no cache: their descriptors travel in the kernel arguments.
hmar_status launch_steps(hmar::StepLaunch::Step* steps, int32_t n_steps, int32_t n_heads, float sm_scale,
                         int32_t D, void* stream) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return HMAR_ERR_HIP;
    const int cus = hmar::device_cus(dev);
    if (cus < 1) return HMAR_ERR_HIP;
    // heaviest steps first, so that the launch ends on its lightest work
    std::stable_sort(steps, steps + n_steps, [](const hmar::StepLaunch::Step& a, const hmar::StepLaunch::Step& b) {
        return (int64_t)a.n_q * a.Lk > (int64_t)b.n_q * b.Lk;
    });
    for (int32_t first = 0; first < n_steps; first += hmar::kMaxSteps) {
        hmar::StepLaunch L;
        L.n_steps = std::min<int32_t>(hmar::kMaxSteps, n_steps - first);
        for (int32_t i = 0; i < L.n_steps; ++i) L.step[i] = steps[first + i];
        if (hmar::launch_fwd_steps(L, n_heads, hmar::resolve_scale(sm_scale, D), cus,
                                   static_cast<hipStream_t>(stream)) != hipSuccess)
            return HMAR_ERR_HIP;
    }
    return HMAR_OK;
}

}  // namespace

namespace hmar {

void profile_before(int kernel_id, hipStream_t stream) {
    (void)kernel_id;
    std::lock_guard<std::mutex> lock(g_prof_mu);
    if (!g_prof_on) return;
    g_prof_pending_start = nullptr;
    if (!g_prof_stream_set) { g_prof_stream = stream; g_prof_stream_set = true; }
    if (stream != g_prof_stream) { g_prof_mixed_streams = true; return; }
    hipEvent_t ev;
    if (hipEventCreate(&ev) != hipSuccess) return;
    if (hipEventRecord(ev, stream) != hipSuccess) { (void)hipEventDestroy(ev); return; }
    g_prof_pending_start = ev;
}

void profile_after(int kernel_id, hipStream_t stream) {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    if (!g_prof_on || !g_prof_pending_start || stream != g_prof_stream) return;
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
    g_prof_stream_set = false;
    g_prof_mixed_streams = false;
    return HMAR_OK;
}

hmar_status hmar_profile_end(double* total_ms_out, int64_t* launches_out) {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    g_prof_on = false;
    double ms[HMAR_NUM_KERNELS] = {0, 0, 0};
    int64_t n[HMAR_NUM_KERNELS] = {0, 0, 0};
    hmar_status st = g_prof_mixed_streams ? HMAR_ERR_INVALID_ARG : HMAR_OK;
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
    using hmar::aligned16;
    if (!Q || !K || !V || !O || !LSE) return HMAR_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE)) return HMAR_ERR_INVALID_ARG;
    if (!std::isfinite(sm_scale)) return HMAR_ERR_INVALID_ARG;
    Problem pb;
    hmar_status st = hmar::check_problem(side_lens, num_scales, mask_kind, B, H, D, &pb);
    if (st != HMAR_OK) return st;
    const hmar::DeviceSchedule* ds = nullptr;
    st = get_device_schedule(side_lens, num_scales, pb, &ds);
    if (st != HMAR_OK) return st;
    hipError_t e = hmar::launch_fwd(Q, K, V, O, LSE, *ds, pb.n_heads, hmar::resolve_scale(sm_scale, D),
                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HMAR_OK : HMAR_ERR_HIP;
}

hmar_status hmar_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                          const int32_t* side_lens, int32_t num_scales,
                          int32_t B, int32_t H, int32_t D, float sm_scale, void* stream) {
    return hmar_attn_fwd_masked(Q, K, V, O, LSE, side_lens, num_scales, HMAR_MASK_MARKOV, B, H, D, sm_scale, stream);
}

hmar_status hmar_attn_steps_fwd(const void* const* Q, const void* const* K, const void* const* V,
                                void* const* O, float* const* LSE,
                                const int32_t* n_prev, const int32_t* n_cur, int32_t n_steps,
                                int32_t B, int32_t H, int32_t D, float sm_scale, void* stream) {
    if (!Q || !K || !V || !O || !LSE || !n_prev || !n_cur || n_steps < 1 || B < 1 || H < 1 || D < 1)
        return HMAR_ERR_INVALID_ARG;
    if (!std::isfinite(sm_scale)) return HMAR_ERR_INVALID_ARG;
    hmar_status worst = HMAR_OK;      // an invalid argument anywhere outranks an unsupported size
    for (int32_t i = 0; i < n_steps && i < HMAR_MAX_STEPS; ++i) {
        const hmar_status st = check_step(Q[i], K[i], V[i], O[i], LSE[i], n_prev[i], n_cur[i]);
        if (st == HMAR_ERR_INVALID_ARG) return st;
        if (st != HMAR_OK) worst = st;
    }
    if (n_steps > HMAR_MAX_STEPS || D != 64 || (int64_t)B * H > (1 << 24)) return HMAR_ERR_UNSUPPORTED;
    if (worst != HMAR_OK) return worst;
    std::vector<hmar::StepLaunch::Step> steps((size_t)n_steps);
    for (int32_t i = 0; i < n_steps; ++i)
        steps[i] = {Q[i], K[i], V[i], O[i], LSE[i], nullptr, n_cur[i], n_cur[i], n_prev[i] + n_cur[i]};
    return launch_steps(steps.data(), n_steps, B * H, sm_scale, D, stream);
}

hmar_status hmar_attn_step_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                               int32_t n_prev, int32_t n_cur, int32_t B, int32_t H, int32_t D,
                               float sm_scale, void* stream) {
    return hmar_attn_steps_fwd(&Q, &K, &V, &O, &LSE, &n_prev, &n_cur, 1, B, H, D, sm_scale, stream);
}

hmar_status hmar_attn_step_fwd_rows(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                    const int32_t* rows, int32_t n_rows,
                                    int32_t n_prev, int32_t n_cur, int32_t B, int32_t H, int32_t D,
                                    float sm_scale, void* stream) {
    if (B < 1 || H < 1 || D < 1 || !std::isfinite(sm_scale)) return HMAR_ERR_INVALID_ARG;
    const hmar_status st = check_step(Q, K, V, O, LSE, n_prev, n_cur);
    if (st == HMAR_ERR_INVALID_ARG) return st;
    if (!rows || (reinterpret_cast<uintptr_t>(rows) & 3u) || n_rows < 1 || n_rows > n_cur) return HMAR_ERR_INVALID_ARG;
    if (st != HMAR_OK) return st;
    if (D != 64 || (int64_t)B * H > (1 << 24)) return HMAR_ERR_UNSUPPORTED;
    hmar::StepLaunch::Step step = {Q, K, V, O, LSE, rows, n_rows, n_cur, n_prev + n_cur};
    return launch_steps(&step, 1, B * H, sm_scale, D, stream);
}

size_t hmar_attn_bwd_workspace_bytes_masked(const int32_t* side_lens, int32_t num_scales, int32_t mask_kind,
                                            int32_t B, int32_t H, int32_t D) {
    Problem pb;
    if (hmar::check_problem(side_lens, num_scales, mask_kind, B, H, D, &pb) != HMAR_OK) return 0;
    return 2 * (size_t)pb.n_heads * pb.L * sizeof(float);
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
    Problem pb;
    hmar_status st = hmar::check_bwd_args(Q, K, V, O, dO, LSE, dQ, dK, dV, side_lens, num_scales, mask_kind, B, H, D,
                                          sm_scale, &pb);
    if (st != HMAR_OK) return st;
    const size_t need = 2 * (size_t)pb.n_heads * pb.L * sizeof(float);
    if (!workspace || workspace_bytes < need) return HMAR_ERR_WORKSPACE;
    if (!hmar::aligned16(workspace)) return HMAR_ERR_INVALID_ARG;
    const hmar::DeviceSchedule* ds = nullptr;
    st = get_device_schedule(side_lens, num_scales, pb, &ds);
    if (st != HMAR_OK) return st;
    hipError_t e = hmar::launch_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, static_cast<float*>(workspace), *ds, pb.n_heads,
                                    hmar::resolve_scale(sm_scale, D), static_cast<hipStream_t>(stream));
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
    if (!dst || !src || (bytes & 15u) || !hmar::aligned16(dst) || !hmar::aligned16(src)) return HMAR_ERR_INVALID_ARG;
    return hmar::launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? HMAR_OK : HMAR_ERR_HIP;
}

hmar_status hmar_schedule_describe(const int32_t* side_lens, int32_t num_scales,
                                   int32_t* offsets_out, int64_t* allowed_pairs_out) {
    Problem pb;
    hmar_status st = hmar::check_problem(side_lens, num_scales, HMAR_MASK_MARKOV, 1, 1, 64, &pb);
    if (st != HMAR_OK) return st;
    hmar::Schedule host;
    if (!hmar::build_host_schedule(side_lens, num_scales, pb, &host)) return HMAR_ERR_UNSUPPORTED;
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
    Problem pb;
    hmar_status st = hmar::check_problem(side_lens, num_scales, mask_kind, 1, 1, 64, &pb);
    if (st != HMAR_OK) return st;
    hmar::Schedule host;
    if (!hmar::build_host_schedule(side_lens, num_scales, pb, &host)) return HMAR_ERR_UNSUPPORTED;
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
