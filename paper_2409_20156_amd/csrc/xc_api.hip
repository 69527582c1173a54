// Status strings, per-thread HIP error, and the optional per-kernel event timing
// of the C ABI.
#include <mutex>
#include <vector>

#include "xc_common.h"

namespace xc {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = static_cast<int>(e); }

static const char* const kKernelNames[K_NUM_KERNELS] = {
    "mine_tile", "mine_select", "sample", "gather", "loss_reduce", "radix_count", "radix_scan",
    "radix_scatter", "heads_count", "heads_write", "update"};

struct Pending { int id; hipEvent_t start, stop; };
static std::mutex g_mu;
static bool g_profile = false;
static std::vector<Pending> g_pending;
static std::vector<hipEvent_t> g_free_events;
static double g_total_ms[K_NUM_KERNELS];
static int64_t g_launches[K_NUM_KERNELS];

bool profile_on() { return g_profile; }

static hipEvent_t take_event() {
    if (!g_free_events.empty()) { hipEvent_t e = g_free_events.back(); g_free_events.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void profile_mark(int kernel_id, hipStream_t st, bool begin) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (begin) {
        Pending p{kernel_id, take_event(), take_event()};
        if (p.start) (void)hipEventRecord(p.start, st);
        g_pending.push_back(p);
    } else if (!g_pending.empty()) {
        Pending& p = g_pending.back();
        if (p.stop) (void)hipEventRecord(p.stop, st);
    }
}

// Plain copy, 16 bytes per lane per trip: a kernel whose HBM traffic is known (n16*16 bytes
// read and as many written), used to calibrate hardware traffic counters.
__global__ __launch_bounds__(256) void copy_probe_kernel(uint4* __restrict__ dst,
                                                         const uint4* __restrict__ src, int64_t n16) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}

}  // namespace xc

extern "C" int xc_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || (bytes & 15) || ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15))
        return XC_EINVAL;
    if (bytes == 0) return XC_OK;
    const int64_t n16 = static_cast<int64_t>(bytes / 16);
    const int grid = static_cast<int>(n16 / 256 < 8192 ? (n16 + 255) / 256 : 8192);
    xc::copy_probe_kernel<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<uint4*>(dst), static_cast<const uint4*>(src), n16);
    XC_HIP_CHECK(hipGetLastError());
    return XC_OK;
}

extern "C" const char* xc_strerror(int status) {
    switch (status) {
        case XC_OK: return "ok";
        case XC_EINVAL: return "invalid argument (null or misaligned pointer, bad enum)";
        case XC_ESHAPE: return "unsupported or inconsistent sizes";
        case XC_EWORKSPACE: return "workspace too small";
        case XC_EHIP: return "HIP runtime error (see xc_last_hip_error)";
        default: return "unknown status";
    }
}

extern "C" int xc_last_hip_error(void) { return xc::g_last_hip_error; }

extern "C" int xc_version(void) { return 1; }

extern "C" int xc_profile_enable(int on) {
    std::lock_guard<std::mutex> lock(xc::g_mu);
    xc::g_profile = on != 0;
    return XC_OK;
}

extern "C" int xc_profile_collect(void) {
    using namespace xc;
    std::lock_guard<std::mutex> lock(g_mu);
    for (Pending& p : g_pending) {
        if (p.start && p.stop && hipEventSynchronize(p.stop) == hipSuccess) {
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
                g_total_ms[p.id] += ms;
                g_launches[p.id] += 1;
            }
        }
        if (p.start) g_free_events.push_back(p.start);
        if (p.stop) g_free_events.push_back(p.stop);
    }
    g_pending.clear();
    return K_NUM_KERNELS;
}

extern "C" int xc_profile_get(int i, const char** name, double* total_ms, int64_t* launches) {
    using namespace xc;
    if (i < 0 || i >= K_NUM_KERNELS) return XC_EINVAL;
    std::lock_guard<std::mutex> lock(g_mu);
    if (name) *name = kKernelNames[i];
    if (total_ms) *total_ms = g_total_ms[i];
    if (launches) *launches = g_launches[i];
    return XC_OK;
}

extern "C" int xc_profile_reset(void) {
    using namespace xc;
    std::lock_guard<std::mutex> lock(g_mu);
    for (int i = 0; i < K_NUM_KERNELS; ++i) { g_total_ms[i] = 0.0; g_launches[i] = 0; }
    return XC_OK;
}
