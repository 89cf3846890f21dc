// hmar_attn_bwd_noalloc: the backward for callers that cannot allocate device memory.
//
// Everything the backward keeps on the device besides the caller's tensors -- the two fp32
// [B,H,L] row statistics its two kernels exchange and the tile schedule tables -- lives in one
// fixed array of the library's device image.  Each GPU holds its own copy of that array at its
// own address; the address is looked up once per device with hipGetSymbolAddress while that
// device is current.  The tables reach the array through kernel arguments (a small writer
// kernel, a few KB per launch), so the entry point issues kernel launches only: no hipMalloc,
// no hipFree, no memcpy, nothing a stream capture could not record.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <vector>

#include "api_internal.h"
#include "hmar_attn.h"
#include "kernels.h"
#include "schedule.h"

namespace {

constexpr size_t kStatsBytes = 2ull * HMAR_NOALLOC_MAX_ROWS * sizeof(float);   // -Delta and -LSE*log2(e)
constexpr size_t kTableBytes = 192 * 1024;                                      // items and row ranges
constexpr size_t kScratchBytes = kStatsBytes + kTableBytes;

// In host code this name is a stand-in, not a device address: only the pointer obtained from
// hipGetSymbolAddress below is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
struct DeviceState {
    unsigned char* ptr = nullptr;          // this device's copy of `scratch`
    bool have_tables = false;              // the array holds the tables of (kind, sizes)
    bool graph_seen = false;               // some call was recorded into a graph: its replays rewrite the
                                           // tables at times this code cannot know
    int32_t kind = 0;
    std::vector<int32_t> sizes;
    hmar::DeviceSchedule dev{};
};
std::mutex g_mu;
DeviceState g_state[kMaxDevices];

// One launch moves up to kChunkWords 32-bit words from the kernel arguments to the array.
constexpr int kChunkWords = 768;           // 3 KB of the 4 KB a kernel may take as arguments
struct TableChunk {
    uint32_t n_words;
    uint32_t word[kChunkWords];
};
__global__ __launch_bounds__(256) void hmar_table_writer_kernel(uint32_t* dst, TableChunk c) {
    for (uint32_t i = threadIdx.x; i < c.n_words; i += blockDim.x) dst[i] = c.word[i];
}

}  // namespace

extern "C" hmar_status hmar_attn_bwd_noalloc(const void* Q, const void* K, const void* V, const void* O,
                                             const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                                             const int32_t* side_lens, int32_t num_scales,
                                             int32_t B, int32_t H, int32_t D, float sm_scale, void* stream) {
    hmar::Problem pb;
    hmar_status st = hmar::check_bwd_args(Q, K, V, O, dO, LSE, dQ, dK, dV, side_lens, num_scales, HMAR_MASK_MARKOV,
                                          B, H, D, sm_scale, &pb);
    if (st != HMAR_OK) return st;
    if ((int64_t)pb.n_heads * pb.L > HMAR_NOALLOC_MAX_ROWS || pb.L > HMAR_NOALLOC_MAX_SEQ_LEN)
        return HMAR_ERR_UNSUPPORTED;      // beyond what the fixed array holds
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return HMAR_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return HMAR_ERR_UNSUPPORTED;
    const int cus = hmar::device_cus(dev);
    if (cus < 1) return HMAR_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // A call that is being recorded into a graph must carry its tables with it: the graph is
    // replayed later, when the array may hold another schedule's.
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &capture) != hipSuccess) return HMAR_ERR_HIP;
    if (capture == hipStreamCaptureStatusInvalidated) return HMAR_ERR_HIP;
    const bool capturing = capture == hipStreamCaptureStatusActive;

    hmar::DeviceSchedule ds;
    unsigned char* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        DeviceState& state = g_state[dev];
        if (!state.ptr) {
            // the current device is `dev`: this is the address of ITS copy of the array
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HMAR_ERR_HIP;
            state.ptr = static_cast<unsigned char*>(p);
        }
        base = state.ptr;
        if (capturing) state.graph_seen = true;
        // once graphs exist the array's tables are only known to be this call's if this call writes them
        const bool same = !state.graph_seen && state.have_tables && state.kind == pb.mask_kind &&
                          (int32_t)state.sizes.size() == num_scales &&
                          std::memcmp(state.sizes.data(), side_lens, sizeof(int32_t) * (size_t)num_scales) == 0;
        if (!same) {
            hmar::Schedule host;
            if (!hmar::build_host_schedule(side_lens, num_scales, pb, &host)) return HMAR_ERR_UNSUPPORTED;
            const size_t bytes = hmar::table_bytes(host);          // a multiple of 4
            if (bytes > kTableBytes) return HMAR_ERR_UNSUPPORTED;
            std::vector<unsigned char> staging(bytes);
            unsigned char* tables = base + kStatsBytes;
            hmar::pack_tables(host, staging.data(), tables, &state.dev);
            state.dev.num_cus = cus;
            state.have_tables = false;                              // until every chunk is queued
            const size_t words = bytes / 4;
            for (size_t w0 = 0; w0 < words; w0 += kChunkWords) {
                TableChunk c;
                c.n_words = (uint32_t)std::min<size_t>(kChunkWords, words - w0);
                std::memcpy(c.word, staging.data() + 4 * w0, 4 * (size_t)c.n_words);
                hipLaunchKernelGGL(hmar_table_writer_kernel, dim3(1), dim3(256), 0, s,
                                   reinterpret_cast<uint32_t*>(tables) + w0, c);
                if (hipGetLastError() != hipSuccess) return HMAR_ERR_HIP;
            }
            state.kind = pb.mask_kind;
            state.sizes.assign(side_lens, side_lens + num_scales);
            state.have_tables = true;
        }
        ds = state.dev;
    }
    // The statistics need no clearing: the dQ kernel writes every row before the dK/dV kernel,
    // queued behind it on the same stream, reads it.
    const hipError_t e = hmar::launch_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, reinterpret_cast<float*>(base), ds,
                                          pb.n_heads, hmar::resolve_scale(sm_scale, D), s);
    return e == hipSuccess ? HMAR_OK : HMAR_ERR_HIP;
}
