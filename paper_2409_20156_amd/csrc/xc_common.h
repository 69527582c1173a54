// Shared host/device helpers of the gfx950 library: status handling, element
// conversion, order-preserving score keys and wave-level primitives.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "astra_xc.h"

namespace xc {

constexpr int kWave = 64;

// ---- status ---------------------------------------------------------------
void set_last_hip_error(hipError_t e);

#define XC_HIP_CHECK(expr)                         \
    do {                                           \
        hipError_t e__ = (expr);                   \
        if (e__ != hipSuccess) {                   \
            ::xc::set_last_hip_error(e__);         \
            return XC_EHIP;                        \
        }                                          \
    } while (0)

// ---- optional per-kernel event timing ----------------------------------------
enum KernelId {
    K_MINE_TILE = 0, K_MINE_SELECT, K_SAMPLE, K_GATHER, K_RADIX_COUNT, K_RADIX_SCAN,
    K_RADIX_SCATTER, K_BUCKET_SORT, K_HEADS_COUNT, K_HEADS_WRITE, K_UPDATE, K_NUM_KERNELS
};
bool profile_on();
void profile_mark(int kernel_id, hipStream_t st, bool begin);

// Launch statement `stmt` for kernel `id` on stream `st`, bracketed by events when
// profiling is enabled.
#define XC_LAUNCH(id, st, stmt)                                   \
    do {                                                          \
        const bool prof__ = ::xc::profile_on();                   \
        if (prof__) ::xc::profile_mark((id), (st), true);         \
        stmt;                                                     \
        if (prof__) ::xc::profile_mark((id), (st), false);        \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- element types ----------------------------------------------------------
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even float -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// unpack 8 bf16 (one 16-byte chunk) into 8 floats
__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

// ---- order-preserving keys --------------------------------------------------
// A candidate (score, id) is packed into one 64-bit key whose ascending order is
// "larger score first, then smaller id": high word = complement of the monotone
// integer image of the float, low word = id.
__device__ __forceinline__ uint32_t float_to_ordered(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_float(uint32_t o) {
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}
__device__ __forceinline__ uint64_t make_key(float score, int32_t id) {
    return (static_cast<uint64_t>(~float_to_ordered(score)) << 32) | static_cast<uint32_t>(id);
}
__device__ __forceinline__ float key_score(uint64_t k) {
    return ordered_to_float(~static_cast<uint32_t>(k >> 32));
}
__device__ __forceinline__ int32_t key_id(uint64_t k) { return static_cast<int32_t>(k & 0xffffffffu); }
constexpr uint64_t kKeySentinel = ~0ull;   // score -NaN pattern never produced, id -1

// ---- wave helpers -----------------------------------------------------------
__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ int wave_incl_scan(int v) {
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        int t = __shfl_up(v, off, kWave);
        if (lane >= off) v += t;
    }
    return v;
}

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        uint64_t t = __shfl_xor(v, off, kWave);
        v = t > v ? t : v;
    }
    return v;
}

// Workgroup barrier for data exchanged through LDS only: waits for this wave's LDS operations, not for
// its global loads and stores (a plain __syncthreads also waits for the stores' acknowledgements).
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
// 16-byte global accesses with the non-temporal hint: the line is marked for early replacement, so data
// that is touched once (rows of a matrix much larger than the caches) does not push out what is reused.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
template <bool STREAM>
__device__ __forceinline__ uint4 load16(const void* p) {
    if (STREAM) {
        const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    }
    return *reinterpret_cast<const uint4*>(p);
}
template <bool STREAM>
__device__ __forceinline__ void store16(void* p, uint4 o) {
    if (STREAM) {
        u32x4_t v;
        v.x = o.x; v.y = o.y; v.z = o.z; v.w = o.w;
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p));
    } else {
        *reinterpret_cast<uint4*>(p) = o;
    }
}
__device__ __forceinline__ uint64_t lanemask_lt() {
    return (1ull << lane_id()) - 1ull;
}

}  // namespace xc
