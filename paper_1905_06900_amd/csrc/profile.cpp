// Optional per-kernel timing: when enabled, every kernel launch of the library is bracketed by
// two HIP events recorded on the stream the kernel is launched on; dcpq_profile_read() waits for
// the pending events and returns accumulated milliseconds and launch counts per stage.
#include <mutex>
#include <vector>

#include "common.h"

namespace dcpq {
namespace prof {

static const char *const kNames[kNumStages] = {
    "small_tables", "scan_hist", "scan_tiecount", "scan_collect", "scan_fast", "select",
    "full_tables",
    "refine_topk", "ivf", "misc",
    "ivf_probe", "ivf_tables", "ivf_scan", "ivf_refine", "plain_scan", "train",
};

struct Pending { int stage; hipEvent_t a, b; };

static std::mutex g_mu;
static bool g_on = false;
static std::vector<Pending> g_pending;
static std::vector<hipEvent_t> g_free;
static double g_ms[kNumStages];
static uint64_t g_count[kNumStages];

bool enabled() { return g_on; }

static hipEvent_t get_event()
{
    if (!g_free.empty()) { hipEvent_t e = g_free.back(); g_free.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void *begin(int stage, hipStream_t st)
{
    if (!g_on) return nullptr;
    std::lock_guard<std::mutex> lk(g_mu);
    Pending p{stage, get_event(), get_event()};
    if (!p.a || !p.b) return nullptr;
    (void)hipEventRecord(p.a, st);
    g_pending.push_back(p);
    return p.b;
}

void end(void *token, hipStream_t st)
{
    if (token) (void)hipEventRecord(static_cast<hipEvent_t>(token), st);
}

static void drain()
{
    for (const Pending &p : g_pending) {
        float ms = 0.f;
        if (hipEventSynchronize(p.b) == hipSuccess && hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
            g_ms[p.stage] += ms;
            g_count[p.stage] += 1;
        }
        g_free.push_back(p.a);
        g_free.push_back(p.b);
    }
    g_pending.clear();
}

}  // namespace prof
}  // namespace dcpq

using namespace dcpq;

extern "C" int dcpq_profile_enable(int on)
{
    std::lock_guard<std::mutex> lk(prof::g_mu);
    prof::drain();
    for (int s = 0; s < kNumStages; ++s) { prof::g_ms[s] = 0.0; prof::g_count[s] = 0; }
    prof::g_on = on != 0;
    return DCPQ_OK;
}

// Plain device-to-device copy of known size: the yardstick the HBM traffic counters are scaled by.
__global__ __launch_bounds__(256) void calibration_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n;
         i += static_cast<size_t>(gridDim.x) * blockDim.x)
        dst[i] = src[i];
}

extern "C" int dcpq_profile_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(src && dst && bytes % 16 == 0, "profile_copy: needs non-null pointers and a multiple of 16 bytes");
    DCPQ_REQUIRE(((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0, "profile_copy: 16-byte alignment");
    if (bytes == 0) return DCPQ_OK;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(8192), dim3(256), 0, as_stream(stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), bytes / 16);
    DCPQ_CHECK_LAUNCH("calibration_copy_kernel");
    return DCPQ_OK;
}

// Read-only stream over `n` 16-byte words: what a kernel that only reads an array once can reach on
// this chip (the yardstick for the HBM-bound scans).  Every thread keeps 8 independent 16-byte loads
// in flight; the XOR of what it read goes to `sink` so that the loads cannot be dropped.
constexpr int kStreamReadBlocks = 256 * 16;
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ src, size_t n, uint32_t *__restrict__ sink)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (; i + 7 * stride < n; i += 8 * stride) {
        uint4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) { acc.x ^= x[u].x; acc.y ^= x[u].y; acc.z ^= x[u].z; acc.w ^= x[u].w; }
    }
    for (; i < n; i += stride) {
        const uint4 x = src[i];
        acc.x ^= x.x; acc.y ^= x.y; acc.z ^= x.z; acc.w ^= x.w;
    }
    sink[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

extern "C" size_t dcpq_profile_stream_read_sink_bytes(void) { return sizeof(uint32_t) * kStreamReadBlocks * 256; }

extern "C" int dcpq_profile_stream_read(const void *src, size_t bytes, void *sink, void *stream)
{
    clear_error();
    DCPQ_REQUIRE(src && sink && bytes % 16 == 0, "profile_stream_read: needs non-null pointers and a multiple of 16 bytes");
    DCPQ_REQUIRE((reinterpret_cast<uintptr_t>(src) & 15) == 0 && (reinterpret_cast<uintptr_t>(sink) & 3) == 0,
                 "profile_stream_read: alignment");
    if (bytes == 0) return DCPQ_OK;
    DCPQ_LAUNCH(kStageMisc, as_stream(stream), stream_read_kernel, dim3(kStreamReadBlocks), dim3(256), 0,
                static_cast<const uint4 *>(src), bytes / 16, static_cast<uint32_t *>(sink));
    DCPQ_CHECK_LAUNCH("stream_read_kernel");
    return DCPQ_OK;
}

extern "C" int dcpq_profile_stage_count(void) { return kNumStages; }

extern "C" const char *dcpq_profile_stage_name(int stage)
{
    return (stage >= 0 && stage < kNumStages) ? prof::kNames[stage] : "";
}

extern "C" int dcpq_profile_read(int stage, double *total_ms, uint64_t *launches)
{
    clear_error();
    DCPQ_REQUIRE(stage >= 0 && stage < kNumStages && total_ms && launches, "profile_read: bad argument");
    std::lock_guard<std::mutex> lk(prof::g_mu);
    prof::drain();
    *total_ms = prof::g_ms[stage];
    *launches = prof::g_count[stage];
    return DCPQ_OK;
}
