// Status strings, per-thread HIP error, and the optional per-kernel event timing
// of the C ABI.
#include <mutex>
#include <vector>

#include "xc_common.h"

namespace xc {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = static_cast<int>(e); }

static const char* const kKernelNames[K_NUM_KERNELS] = {
    "mine_tile", "mine_select", "sample", "gather", "radix_count", "radix_scan",
    "radix_scatter", "bucket_sort", "heads_count", "heads_write", "update"};

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

// Register-resident MFMA loop: 8 independent 32x32x16 bf16 products per iteration and wave,
// operands either zero or pseudo-random bf16 values in [0.25, 0.5) with random sign.  No memory
// traffic inside the loop; used to measure the MFMA rate the chip sustains (it depends on the
// operand values through the power limit).
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
constexpr int kProbeGrid = 256, kProbeThreads = 512;
__global__ __launch_bounds__(kProbeThreads, 1) void mfma_probe_kernel(float* out, int iters, int random_operands) {
    probe_f32x16 acc[8];
#pragma unroll
    for (int n = 0; n < 8; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[n][i] = 0.0f;
    uint4 fa[4], fb[2];
#pragma unroll
    for (int m = 0; m < 6; ++m) {
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t r = threadIdx.x * 977u + blockIdx.x * 131071u + m * 17u + j;
            r ^= r >> 16; r *= 0x7feb352du; r ^= r >> 15; r *= 0x846ca68bu; r ^= r >> 16;
            const uint32_t lo = 0x3e80u | (r & 0x807fu), hi = 0x3e80u | ((r >> 16) & 0x807fu);
            w[j] = random_operands ? (lo | (hi << 16)) : 0u;
        }
        const uint4 v = make_uint4(w[0], w[1], w[2], w[3]);
        if (m < 4) fa[m] = v; else fb[m - 4] = v;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                probe_bf16x8 av, bv;
                __builtin_memcpy(&av, &fa[mt], 16);
                __builtin_memcpy(&bv, &fb[nt], 16);
                acc[mt * 2 + nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[mt * 2 + nt], 0, 0, 0);
            }
        if (random_operands) { fa[0].x ^= 0x00010001u; fb[1].y ^= 0x00010001u; }   // keep the inputs changing
    }
    float tot = 0.0f;
#pragma unroll
    for (int n = 0; n < 8; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) tot += acc[n][i];
    out[blockIdx.x * kProbeThreads + threadIdx.x] = tot;
}

}  // namespace xc

extern "C" int xc_mfma_probe(float* out, int iters, int random_operands, double* flop, void* stream) {
    if (!out || iters < 1 || iters > (1 << 20)) return XC_EINVAL;
    xc::mfma_probe_kernel<<<xc::kProbeGrid, xc::kProbeThreads, 0, static_cast<hipStream_t>(stream)>>>(
        out, iters, random_operands);
    XC_HIP_CHECK(hipGetLastError());
    if (flop) *flop = 2.0 * 32 * 32 * 16 * 8.0 * iters * (xc::kProbeThreads / 64) * xc::kProbeGrid;
    return XC_OK;
}

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
        case XC_EDTYPE: return "unsupported element type (XC_F32 or XC_BF16 expected)";
        case XC_ESCRATCH: return "the step's temporaries exceed the static scratch array (XC_STATIC_SCRATCH_BYTES)";
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
