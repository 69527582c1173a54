// Hard-negative mining: exact top-k inner product of every query against all
// classifier rows (Alg. 1, "ANNS refresh" step, with exact search in place of
// the index; score of Sec. 2.1).
//
// Kernel 1 (mine_tile_kernel) is a tiled MFMA product W_tile x Z_tile^T whose
// accumulators never leave registers as a matrix: labels run along the MFMA M
// dimension and queries along N, so one lane owns one query column and compares
// its 32 partial scores against that query's running threshold tau (the k-th
// best score seen so far in this label slice).  Survivors are appended as
// 64-bit (score,id) keys to a small per-query candidate list; when a list is
// nearly full one wave reduces it to the best k by a radix select and raises
// tau.  Kernel 2 (mine_merge_kernel) merges the per-slice lists of a query and
// emits the k best, ordered by (score descending, id ascending).
#include "xc_common.h"

namespace xc {

constexpr int kBM = 128;            // labels per tile   (MFMA M)
constexpr int kBN = 128;            // queries per tile  (MFMA N)
constexpr int kStageBytes = 128;    // bytes of a row staged in LDS per K step
constexpr int kRowStride = kStageBytes + 16;   // padded LDS row pitch
constexpr int kCandCap = 512;       // keys per (query, slice) candidate list
constexpr int kMineThreads = 256;   // 4 waves: 2 along labels x 2 along queries
constexpr int kMergeMax = 4096;     // keys merged per query

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------
// Reduce a candidate list of n > k keys to its k smallest keys (best scores).
// One wave; n <= kCandCap.  Radix select, most significant byte first, with a
// 256-bin histogram in LDS; stops as soon as every key sharing the prefix is
// needed.  Writes the survivors to buf[0..k), returns the score of the k-th.
// ---------------------------------------------------------------------------
__device__ float wave_select_k(uint64_t* __restrict__ buf, int n, int k, int* hist) {
    const int lane = lane_id();
    constexpr int R = kCandCap / kWave;
    uint64_t key[R];
    bool valid[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int idx = r * kWave + lane;
        valid[r] = idx < n;
        key[r] = valid[r] ? buf[idx] : kKeySentinel;
    }
    uint64_t prefix = 0, pmask = 0;
    int need = k;
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
#pragma unroll
        for (int j = 0; j < 4; ++j) hist[lane * 4 + j] = 0;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (valid[r] && (key[r] & pmask) == prefix)
                atomicAdd(&hist[static_cast<int>((key[r] >> shift) & 255u)], 1);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        int c[4];
        int s = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { c[j] = hist[lane * 4 + j]; s += c[j]; }
        const int incl = wave_incl_scan(s);
        const int excl = incl - s;
        const bool mine = (excl < need) && (need <= incl);
        int dsel = 0, needn = 0, have = 0;
        if (mine) {
            int cum = excl;
            bool done = false;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (!done && need <= cum + c[j]) {
                    dsel = lane * 4 + j; needn = need - cum; have = c[j]; done = true;
                }
                cum += c[j];
            }
        }
        const uint64_t bal = __ballot(mine);
        const int src = __ffsll(static_cast<long long>(bal)) - 1;   // exactly one lane
        dsel = __shfl(dsel, src, kWave);
        needn = __shfl(needn, src, kWave);
        have = __shfl(have, src, kWave);
        prefix |= static_cast<uint64_t>(dsel) << shift;
        pmask |= 0xffull << shift;
        need = needn;
        if (have == need) break;
    }
    const uint64_t bound = prefix | ~pmask;
    uint64_t kmax = 0;
    int base = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool sel = valid[r] && key[r] <= bound;
        const uint64_t m = __ballot(sel);
        const int p = base + __popcll(m & lanemask_lt());
        if (sel && p < k) {
            buf[p] = key[r];
            kmax = key[r] > kmax ? key[r] : kmax;
        }
        base += __popcll(m);
    }
    kmax = wave_max_u64(kmax);
    return key_score(kmax);
}

// ---------------------------------------------------------------------------
// element-type specifics of the tile product
// ---------------------------------------------------------------------------
template <typename T> struct MineTraits;
template <> struct MineTraits<bf16_t> {
    static __device__ __forceinline__ void mma(const uint4& a, const uint4& b, f32x16& c) {
        bf16x8 av, bv;
        __builtin_memcpy(&av, &a, 16);
        __builtin_memcpy(&bv, &b, 16);
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, c, 0, 0, 0);
    }
};
template <> struct MineTraits<float> {
    static __device__ __forceinline__ void mma(const uint4& a, const uint4& b, f32x16& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

// Loads the 16-byte chunks of one K stage of a 128-row tile into registers.
// Rows beyond `nrows` repeat the last row (their results are discarded later);
// bytes beyond the row length read as zero.
__device__ __forceinline__ void load_stage(const unsigned char* __restrict__ base, int64_t row0,
                                           int64_t nrows, int64_t row_bytes, int kbyte0,
                                           uint4 (&r)[4]) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int c = threadIdx.x + kMineThreads * it;
        const int row = c >> 3;
        const int kb = kbyte0 + (c & 7) * 16;
        int64_t gr = row0 + row;
        gr = gr < nrows ? gr : nrows - 1;
        if (kb < row_bytes) {
            r[it] = *reinterpret_cast<const uint4*>(base + gr * row_bytes + kb);
        } else {
            r[it] = make_uint4(0, 0, 0, 0);
        }
    }
}

__device__ __forceinline__ void store_stage(unsigned char* lds, const uint4 (&r)[4]) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int c = threadIdx.x + kMineThreads * it;
        *reinterpret_cast<uint4*>(lds + (c >> 3) * kRowStride + (c & 7) * 16) = r[it];
    }
}

template <typename T>
__global__ __launch_bounds__(kMineThreads, 2)
void mine_tile_kernel(const T* __restrict__ Z, const T* __restrict__ W, int64_t Zq, int64_t L,
                      int d, int k, int kcap, int S, int tiles_per_slice,
                      uint64_t* __restrict__ cand) {
    __shared__ __align__(16) unsigned char ldsW[kBM * kRowStride];
    __shared__ __align__(16) unsigned char ldsZ[kBN * kRowStride];
    __shared__ float tau[kBN];
    __shared__ int cnt[kBN];
    __shared__ int hist[kMineThreads / kWave][256];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave & 1;          // which 64-label half
    const int wn = wave >> 1;         // which 64-query half
    const int slice = blockIdx.x % S;
    const int64_t qtile = blockIdx.x / S;
    const int64_t q0 = qtile * kBN;
    const int64_t row_bytes = static_cast<int64_t>(d) * sizeof(T);
    const int nkb = static_cast<int>((row_bytes + kStageBytes - 1) / kStageBytes);
    const int64_t nLT = (L + kBM - 1) / kBM;
    const int64_t t_begin = static_cast<int64_t>(slice) * tiles_per_slice;
    int64_t t_end = t_begin + tiles_per_slice;
    t_end = t_end < nLT ? t_end : nLT;

    uint64_t* my_cand = cand + static_cast<size_t>(blockIdx.x) * kBN * kCandCap;
    const unsigned char* Zb = reinterpret_cast<const unsigned char*>(Z);
    const unsigned char* Wb = reinterpret_cast<const unsigned char*>(W);

    if (tid < kBN) { tau[tid] = -INFINITY; cnt[tid] = 0; }
    __syncthreads();

    for (int64_t lt = t_begin; lt < t_end; ++lt) {
        const int64_t l0 = lt * kBM;
        f32x16 acc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

        uint4 rw[4], rz[4];
        load_stage(Wb, l0, L, row_bytes, 0, rw);
        load_stage(Zb, q0, Zq, row_bytes, 0, rz);
        for (int kb = 0; kb < nkb; ++kb) {
            __syncthreads();                       // previous stage fully consumed
            store_stage(ldsW, rw);
            store_stage(ldsZ, rz);
            __syncthreads();
            if (kb + 1 < nkb) {                    // next stage in flight during the MFMAs
                load_stage(Wb, l0, L, row_bytes, (kb + 1) * kStageBytes, rw);
                load_stage(Zb, q0, Zq, row_bytes, (kb + 1) * kStageBytes, rz);
            }
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                uint4 a[2], b[2];
                const int koff = kk * 32 + (lane >> 5) * 16;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
                    a[mt] = *reinterpret_cast<const uint4*>(
                        ldsW + (wm * 64 + mt * 32 + (lane & 31)) * kRowStride + koff);
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    b[nt] = *reinterpret_cast<const uint4*>(
                        ldsZ + (wn * 64 + nt * 32 + (lane & 31)) * kRowStride + koff);
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt) MineTraits<T>::mma(a[mt], b[nt], acc[mt][nt]);
            }
        }

        // ---- threshold filter: lane owns query column (lane & 31) of each N tile
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int qloc = wn * 64 + nt * 32 + (lane & 31);
            const float t = tau[qloc];
            const bool qok = (q0 + qloc) < Zq;
            uint64_t* list = my_cand + static_cast<size_t>(qloc) * kCandCap;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int64_t lab = l0 + wm * 64 + mt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                    const float v = acc[mt][nt][i] + 0.0f;     // -0 -> +0
                    if (qok && lab < L && v >= t) {
                        const int slot = atomicAdd(&cnt[qloc], 1);
                        list[slot] = make_key(v, static_cast<int32_t>(lab));
                    }
                }
            }
        }
        __syncthreads();
        // ---- lists that could overflow during the next tile are reduced now
        for (int q = wave; q < kBN; q += kMineThreads / kWave) {
            const int n = cnt[q];
            if (n > kCandCap - kBM) {
                const float t = wave_select_k(my_cand + static_cast<size_t>(q) * kCandCap, n, k, hist[wave]);
                if (lane == 0) { tau[q] = t; cnt[q] = k; }
            }
        }
        // the barrier at the top of the next K loop orders these updates
    }

    __syncthreads();
    // ---- close the slice: at most k keys per query, padded to kcap
    for (int q = wave; q < kBN; q += kMineThreads / kWave) {
        int n = cnt[q];
        uint64_t* list = my_cand + static_cast<size_t>(q) * kCandCap;
        if (n > k) {
            wave_select_k(list, n, k, hist[wave]);
            n = k;
        }
        for (int e = n + lane; e < kcap; e += kWave) list[e] = kKeySentinel;
    }
}

// ---------------------------------------------------------------------------
// Merge the S per-slice lists of one query and write the k best, sorted.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256)
void mine_merge_kernel(const uint64_t* __restrict__ cand, int S, int kcap, int k, int n2,
                       int32_t* __restrict__ shortlist, float* __restrict__ scores) {
    __shared__ uint64_t keys[kMergeMax];
    const int64_t q = blockIdx.x;
    const int64_t qtile = q / kBN;
    const int qloc = static_cast<int>(q % kBN);
    const int total = S * kcap;
    for (int idx = threadIdx.x; idx < n2; idx += blockDim.x) {
        uint64_t v = kKeySentinel;
        if (idx < total) {
            const int s = idx / kcap, e = idx % kcap;
            v = cand[((static_cast<size_t>(qtile) * S + s) * kBN + qloc) * kCandCap + e];
        }
        keys[idx] = v;
    }
    __syncthreads();
    for (int size = 2; size <= n2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = threadIdx.x; t < n2 / 2; t += blockDim.x) {
                const int lo = 2 * t - (t & (stride - 1));
                const int hi = lo + stride;
                const bool up = (lo & size) == 0;
                const uint64_t a = keys[lo], b = keys[hi];
                if ((a > b) == up) { keys[lo] = b; keys[hi] = a; }
            }
            __syncthreads();
        }
    }
    for (int r = threadIdx.x; r < k; r += blockDim.x) {
        const uint64_t v = keys[r];
        const int32_t id = key_id(v);
        shortlist[q * k + r] = id;
        if (scores) scores[q * k + r] = (v == kKeySentinel) ? -INFINITY : key_score(v);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct MinePlan {
    int64_t nQT, nLT;
    int S, tiles_per_slice, kcap, n2;
    size_t ws_bytes;
};

static int plan_mine(int64_t Zq, int64_t L, int d, int k_h, xc_dtype t, MinePlan* p) {
    if (t != XC_F32 && t != XC_BF16) return XC_EINVAL;
    if (Zq < 1 || L < 1 || d < 1 || k_h < 1 || k_h > XC_MAX_K_MINE || k_h > L) return XC_ESHAPE;
    const int64_t row_bytes = static_cast<int64_t>(d) * (t == XC_F32 ? 4 : 2);
    if (row_bytes % 16 != 0) return XC_ESHAPE;
    if (L > 0x7fffffffLL) return XC_ESHAPE;
    int kcap = 8;
    while (kcap < k_h) kcap <<= 1;
    p->kcap = kcap;
    p->nQT = (Zq + kBN - 1) / kBN;
    p->nLT = (L + kBM - 1) / kBM;
    int64_t S = (1024 + p->nQT - 1) / p->nQT;           // aim for >= ~1024 workgroups
    const int64_t s_max = kMergeMax / kcap;
    if (S > s_max) S = s_max;
    if (S > p->nLT) S = p->nLT;
    if (S < 1) S = 1;
    const int64_t tps = (p->nLT + S - 1) / S;
    S = (p->nLT + tps - 1) / tps;                        // no empty slice
    if (tps > 0x7fffffffLL || p->nQT * S > 0x7fffffffLL) return XC_ESHAPE;
    p->S = static_cast<int>(S);
    p->tiles_per_slice = static_cast<int>(tps);
    int n2 = 2;
    while (n2 < p->S * kcap) n2 <<= 1;
    p->n2 = n2;
    p->ws_bytes = static_cast<size_t>(p->nQT) * p->S * kBN * kCandCap * sizeof(uint64_t);
    return XC_OK;
}

}  // namespace xc

extern "C" int xc_mine_workspace(int64_t Zq, int64_t L, int d, int k_h, xc_dtype t, size_t* bytes) {
    if (!bytes) return XC_EINVAL;
    xc::MinePlan p;
    const int rc = xc::plan_mine(Zq, L, d, k_h, t, &p);
    if (rc != XC_OK) return rc;
    *bytes = p.ws_bytes;
    return XC_OK;
}

extern "C" int xc_mine_negatives(const void* Z, const void* W, int64_t Zq, int64_t L, int d, int k_h,
                                 xc_dtype t, int32_t* shortlist, float* scores, void* ws,
                                 size_t ws_bytes, void* stream) {
    using namespace xc;
    MinePlan p;
    const int rc = plan_mine(Zq, L, d, k_h, t, &p);
    if (rc != XC_OK) return rc;
    if (!Z || !W || !shortlist || !ws) return XC_EINVAL;
    if (!aligned16(Z) || !aligned16(W) || !aligned16(ws)) return XC_EINVAL;
    if (ws_bytes < p.ws_bytes) return XC_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(static_cast<unsigned>(p.nQT * p.S));
    uint64_t* cand = static_cast<uint64_t*>(ws);
    if (t == XC_BF16) {
        XC_LAUNCH(K_MINE_TILE, st, (mine_tile_kernel<bf16_t><<<grid, kMineThreads, 0, st>>>(
            static_cast<const bf16_t*>(Z), static_cast<const bf16_t*>(W), Zq, L, d, k_h, p.kcap, p.S,
            p.tiles_per_slice, cand)));
    } else {
        XC_LAUNCH(K_MINE_TILE, st, (mine_tile_kernel<float><<<grid, kMineThreads, 0, st>>>(
            static_cast<const float*>(Z), static_cast<const float*>(W), Zq, L, d, k_h, p.kcap, p.S,
            p.tiles_per_slice, cand)));
    }
    XC_HIP_CHECK(hipGetLastError());
    XC_LAUNCH(K_MINE_MERGE, st, (mine_merge_kernel<<<dim3(static_cast<unsigned>(Zq)), 256, 0, st>>>(
        cand, p.S, p.kcap, k_h, p.n2, shortlist, scores)));
    XC_HIP_CHECK(hipGetLastError());
    return XC_OK;
}
