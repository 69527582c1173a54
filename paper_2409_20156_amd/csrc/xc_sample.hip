// Negative sampling: the stale hard negatives of each query plus uniform draws
// from the remaining labels, with the log-proposal of every slot (Alg. 1,
// hard+random step; Sec. 3.1 Idea 2; p = 1/(L-k_h) under Eq. 2; warm-up phase
// of Alg. 1 when no shortlist is given).  Integer arithmetic only, so the ids
// are a function of (seed, query, draw, shortlist row) and of no launch shape.
#include "xc_common.h"

namespace xc {

constexpr int kSampleThreads = 256;
constexpr uint64_t kQueryMul = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kDrawMul = 0xD1B54A32D192ED03ull;

__device__ __forceinline__ uint64_t fmix64(uint64_t x) {
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

// One workgroup per query.  The shortlist row is sorted in LDS (bitonic, padded
// to a power of two with INT_MAX), reduced to its distinct in-range ids h_0 <
// h_1 < ..., and stored as a_m = h_m - m, which is non-decreasing.  Draw r in
// [0, M) then maps to the r-th label of the complement: r + #{m : a_m <= r}.
__global__ __launch_bounds__(kSampleThreads)
void sample_kernel(const int32_t* __restrict__ shortlist, int k_h, int k_r, int64_t L,
                   uint64_t seed, int n2, int32_t* __restrict__ neg, float* __restrict__ logq) {
    __shared__ int32_t hs[XC_MAX_K_SAMPLE];
    __shared__ int32_t adj[XC_MAX_K_SAMPLE];
    __shared__ int n_unique;
    const int64_t i = blockIdx.x;
    const int n = k_h + k_r;
    int32_t* out = neg + i * n;
    float* lq = logq + i * n;
    int u = 0, n_draw = n, first = 0;

    if (shortlist != nullptr) {
        const int32_t* row = shortlist + i * k_h;
        for (int m = threadIdx.x; m < n2; m += blockDim.x) {
            int32_t v = 0x7fffffff;
            if (m < k_h) {
                const int32_t id = row[m];
                out[m] = id;
                lq[m] = 0.0f;
                if (id >= 0 && id < L) v = id;
            }
            hs[m] = v;
        }
        if (threadIdx.x == 0) n_unique = 0;
        __syncthreads();
        for (int size = 2; size <= n2; size <<= 1) {
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                for (int t = threadIdx.x; t < n2 / 2; t += blockDim.x) {
                    const int lo = 2 * t - (t & (stride - 1));
                    const int hi = lo + stride;
                    const bool up = (lo & size) == 0;
                    const int32_t a = hs[lo], b = hs[hi];
                    if ((a > b) == up) { hs[lo] = b; hs[hi] = a; }
                }
                __syncthreads();
            }
        }
        // distinct valid ids, in order: position = number of distinct ids before m
        for (int m0 = 0; m0 < n2; m0 += blockDim.x) {
            const int m = m0 + threadIdx.x;
            bool head = false;
            int32_t v = 0;
            if (m < n2) {
                v = hs[m];
                head = v != 0x7fffffff && (m == 0 || hs[m - 1] != v);
            }
            // block-wide exclusive count of heads below m within this chunk
            const uint64_t bal = __ballot(head);
            __shared__ int wave_cnt[kSampleThreads / kWave];
            const int w = threadIdx.x >> 6;
            if (lane_id() == 0) wave_cnt[w] = __popcll(bal);
            __syncthreads();
            int before = n_unique;
            for (int ww = 0; ww < w; ++ww) before += wave_cnt[ww];
            const int p = before + __popcll(bal & lanemask_lt());
            int chunk_total = 0;
            for (int ww = 0; ww < kSampleThreads / kWave; ++ww) chunk_total += wave_cnt[ww];
            __syncthreads();
            if (head) adj[p] = v - p;
            if (threadIdx.x == 0) n_unique += chunk_total;
            __syncthreads();
        }
        u = n_unique;
        n_draw = k_r;
        first = k_h;
    }

    const uint64_t M = static_cast<uint64_t>(L) - static_cast<uint64_t>(u);
    const uint64_t qstate = fmix64(seed ^ (kQueryMul * static_cast<uint64_t>(i + 1)));
    // log of the expected number of copies of a label among the draws
    const float lq_rand = static_cast<float>(log(static_cast<double>(n_draw) / static_cast<double>(M)));
    for (int j = threadIdx.x; j < n_draw; j += blockDim.x) {
        const uint64_t w = fmix64(qstate + kDrawMul * static_cast<uint64_t>(j + 1));
        const uint64_t r = __umul64hi(w, M);
        // count of a_m <= r by binary search over the non-decreasing a
        int lo = 0, hi = u;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (static_cast<uint64_t>(adj[mid]) <= r) lo = mid + 1; else hi = mid;
        }
        out[first + j] = static_cast<int32_t>(r + static_cast<uint64_t>(lo));
        lq[first + j] = lq_rand;
    }
}

// ---------------------------------------------------------------------------
// Sampling from the mixture proposal itself (Sec. 3.1, Idea 2): k_h draws from the importance
// part, label of shortlist slot m with probability w_m / T, and k_r uniform draws from [0, L).
// ---------------------------------------------------------------------------

// Integer image of 2^32 * sigmoid(score), fixed point throughout so that the draw is a function
// of the score's bits: t = floor(clamp(score) * 2^16); y = |t| log2(e) in Q16; 2^-y in Q30 from
// a degree-5 polynomial (coefficients ln(2)^k / k! * 2^30) and a shift; sigmoid(-|x|) in Q32 by
// one integer division; mirrored for positive scores.  NaN -> 0, otherwise at least 1.
__device__ __forceinline__ uint64_t sigmoid_weight(float score) {
    if (score != score) return 0ull;
    const float x = fminf(fmaxf(score, -30.0f), 30.0f);
    const int64_t t = static_cast<int64_t>(floor(static_cast<double>(x) * 65536.0));   // exact
    const uint64_t a = static_cast<uint64_t>(t < 0 ? -t : t);
    const uint64_t y = (a * 94548ull) >> 16;
    const uint64_t ip = y >> 16, f = y & 0xffffull;
    uint64_t m = 1ull << 30;
    uint64_t shift = ip;
    if (f != 0) {
        const uint64_t u = 65536ull - f;            // 2^(-f/65536) = 2^(u/65536) / 2
        uint64_t r = 1431680ull;
        r = 10327387ull + ((r * u) >> 16);
        r = 59597083ull + ((r * u) >> 16);
        r = 257941248ull + ((r * u) >> 16);
        r = 744261118ull + ((r * u) >> 16);
        m = (1ull << 30) + ((r * u) >> 16);
        shift = ip + 1;
    }
    const uint64_t e = shift < 62 ? (m >> shift) : 0ull;
    const uint64_t sn = (e << 32) / ((1ull << 30) + e);
    const uint64_t w = t >= 0 ? (1ull << 32) - sn : sn;
    return w ? w : 1ull;
}

// One workgroup per query.  LDS holds, per shortlist slot, the id, the weight, the running sum of
// the weights in slot order (for the draw) and the slots sorted by id (for the total weight of a
// label, which may sit in several slots).
__global__ __launch_bounds__(kSampleThreads)
void sample_mixture_kernel(const int32_t* __restrict__ shortlist, const float* __restrict__ scores, int M,
                           int k_h, int k_r, int64_t L, uint64_t seed, int n2,
                           int32_t* __restrict__ neg, float* __restrict__ logq) {
    __shared__ int32_t ids[XC_MAX_K_SAMPLE];
    __shared__ uint64_t wts[XC_MAX_K_SAMPLE];
    __shared__ uint64_t cum[2][XC_MAX_K_SAMPLE];
    __shared__ uint64_t byid[XC_MAX_K_SAMPLE];
    const int64_t i = blockIdx.x;
    const int n = k_h + k_r;
    const int32_t* row = shortlist + i * M;
    const float* srow = scores + i * M;
    for (int m = threadIdx.x; m < n2; m += blockDim.x) {
        int32_t id = -1;
        uint64_t w = 0;
        if (m < M) {
            id = row[m];
            if (id >= 0 && id < L) w = sigmoid_weight(srow[m]);
        }
        ids[m] = id;
        wts[m] = w;
        cum[0][m] = w;
        byid[m] = w ? ((static_cast<uint64_t>(static_cast<uint32_t>(id)) << 32) | static_cast<uint32_t>(m)) : ~0ull;
    }
    __syncthreads();
    // inclusive running sums (doubling steps between two buffers)
    int cur = 0;
    for (int off = 1; off < n2; off <<= 1) {
        for (int m = threadIdx.x; m < n2; m += blockDim.x)
            cum[cur ^ 1][m] = cum[cur][m] + (m >= off ? cum[cur][m - off] : 0ull);
        cur ^= 1;
        __syncthreads();
    }
    const uint64_t* run = cum[cur];
    // slots ordered by label id (slots without weight last)
    for (int size = 2; size <= n2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = threadIdx.x; t < n2 / 2; t += blockDim.x) {
                const int lo = 2 * t - (t & (stride - 1));
                const int hi = lo + stride;
                const bool up = (lo & size) == 0;
                const uint64_t a = byid[lo], b = byid[hi];
                if ((a > b) == up) { byid[lo] = b; byid[hi] = a; }
            }
            __syncthreads();
        }
    }
    const uint64_t T = run[n2 - 1];
    const int n_imp = T > 0 ? k_h : 0;
    const uint64_t qstate = fmix64(seed ^ (kQueryMul * static_cast<uint64_t>(i + 1)));
    for (int j = threadIdx.x; j < n; j += blockDim.x) {
        const uint64_t u = fmix64(qstate + kDrawMul * static_cast<uint64_t>(j + 1));
        int64_t lab;
        if (j < n_imp) {
            const uint64_t r = __umul64hi(u, T);
            int lo = 0, hi = n2 - 1;                 // first slot whose running sum exceeds r
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (run[mid] > r) hi = mid; else lo = mid + 1;
            }
            lab = ids[lo];
        } else {
            lab = static_cast<int64_t>(__umul64hi(u, static_cast<uint64_t>(L)));
        }
        double c;
        if (T > 0) {
            // total weight of the slots that hold this label
            const uint64_t key = static_cast<uint64_t>(lab) << 32;
            int lo = 0, hi = n2;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (byid[mid] < key) lo = mid + 1; else hi = mid;
            }
            uint64_t wl = 0;
            for (int p = lo; p < n2 && (byid[p] >> 32) == static_cast<uint64_t>(lab); ++p)
                wl += wts[static_cast<uint32_t>(byid[p])];
            c = static_cast<double>(k_h) * static_cast<double>(wl) / static_cast<double>(T) +
                static_cast<double>(k_r) / static_cast<double>(L);
        } else {
            c = static_cast<double>(n) / static_cast<double>(L);
        }
        neg[i * n + j] = static_cast<int32_t>(lab);
        logq[i * n + j] = static_cast<float>(log(c));
    }
}

// ---------------------------------------------------------------------------
// Hard negatives sampled WITHOUT replacement from a wider stale shortlist, slot m with probability
// proportional to w_m = sigmoid_weight(stale score) (Sec. 3.1, Observation 2, inside the mixture of
// Idea 2).  k = min(k_h, slots with weight) slots are chosen:
//   (1) slots with k' w_m >= T' (k' still to choose, T' the remaining weight) are certain; all such
//       slots are taken at once and the test is repeated with the reduced k', T';
//   (2) the rest by systematic sampling: the k' points U + j T' on the axis of the running sums of the
//       remaining weights (slot order) scaled by k', U = floor(u T' / 2^64) from the query's draw 0;
//       a slot is taken when a point falls into its interval (at most one does: k' w_m < T').
// pi_m = 1 resp. k' w_m / T' exactly.  Slots k.. of the output are uniform draws from [0, L), and
// logq = log(sum of pi over the slots holding the label + (k_h + k_r - k) / L).
// One workgroup per query; integer arithmetic for everything that decides an id.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kSampleThreads)
void sample_pps_kernel(const int32_t* __restrict__ shortlist, const float* __restrict__ scores, int M,
                       int k_h, int k_r, int64_t L, uint64_t seed, int n2,
                       int32_t* __restrict__ neg, float* __restrict__ logq) {
    __shared__ int32_t ids[XC_MAX_K_SAMPLE];
    __shared__ uint64_t wts[XC_MAX_K_SAMPLE];
    __shared__ uint64_t cum[2][XC_MAX_K_SAMPLE];
    __shared__ uint64_t byid[XC_MAX_K_SAMPLE];
    __shared__ double pi[XC_MAX_K_SAMPLE];
    __shared__ int32_t sel[XC_MAX_K_SAMPLE];          // taken slots in slot order
    __shared__ unsigned char state[XC_MAX_K_SAMPLE];  // 0 no weight, 1 remaining, 2 certain, 3 taken by a point
    __shared__ uint64_t red_w[kSampleThreads / kWave];
    __shared__ int red_c[kSampleThreads / kWave];
    const int64_t i = blockIdx.x;
    const int n = k_h + k_r;
    const int tid = threadIdx.x;
    const int32_t* row = shortlist + i * M;
    const float* srow = scores + i * M;
    // sum of (count, weight) over the workgroup, fixed order; every thread gets both
    auto block_sum2 = [&](int c, uint64_t w, int& c_out, uint64_t& w_out) {
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) { c += __shfl_xor(c, off, kWave); w += __shfl_xor(w, off, kWave); }
        if ((tid & (kWave - 1)) == 0) { red_c[tid / kWave] = c; red_w[tid / kWave] = w; }
        __syncthreads();
        c_out = 0; w_out = 0;
        for (int q = 0; q < kSampleThreads / kWave; ++q) { c_out += red_c[q]; w_out += red_w[q]; }
        __syncthreads();
    };
    int c_loc = 0;
    uint64_t w_loc = 0;
    for (int m = tid; m < n2; m += blockDim.x) {
        int32_t id = -1;
        uint64_t w = 0;
        if (m < M) {
            id = row[m];
            if (id >= 0 && id < L) w = sigmoid_weight(srow[m]);
        }
        ids[m] = id;
        wts[m] = w;
        state[m] = w ? 1 : 0;
        byid[m] = w ? ((static_cast<uint64_t>(static_cast<uint32_t>(id)) << 32) | static_cast<uint32_t>(m)) : ~0ull;
        c_loc += w ? 1 : 0;
        w_loc += w;
    }
    int nv;
    uint64_t TT;
    block_sum2(c_loc, w_loc, nv, TT);
    const int k = k_h < nv ? k_h : nv;
    int kk = k;
    // (1) certain slots, round by round (each round takes at least one slot or ends the loop)
    while (kk > 0) {
        c_loc = 0; w_loc = 0;
        for (int m = tid; m < n2; m += blockDim.x) {
            if (state[m] == 1 && static_cast<uint64_t>(kk) * wts[m] >= TT) { state[m] = 2; ++c_loc; w_loc += wts[m]; }
        }
        int c_all;
        uint64_t w_all;
        block_sum2(c_loc, w_loc, c_all, w_all);
        if (c_all == 0) break;
        kk -= c_all;
        TT -= w_all;
    }
    // running sums of the remaining weights in slot order (doubling steps between two buffers)
    for (int m = tid; m < n2; m += blockDim.x) cum[0][m] = state[m] == 1 ? wts[m] : 0ull;
    __syncthreads();
    int cur = 0;
    for (int off = 1; off < n2; off <<= 1) {
        for (int m = tid; m < n2; m += blockDim.x)
            cum[cur ^ 1][m] = cum[cur][m] + (m >= off ? cum[cur][m - off] : 0ull);
        cur ^= 1;
        __syncthreads();
    }
    // (2) systematic sampling of the remaining slots, and pi of every slot
    const uint64_t qstate = fmix64(seed ^ (kQueryMul * static_cast<uint64_t>(i + 1)));
    {
        const uint64_t U = (kk > 0 && TT > 0) ? __umul64hi(fmix64(qstate + kDrawMul), TT) : 0ull;
        auto points_below = [&](uint64_t x) -> uint64_t {        // number of j in [0, kk) with U + j TT < x
            if (x <= U) return 0ull;
            const uint64_t c = (x - U - 1) / TT + 1;
            return c < static_cast<uint64_t>(kk) ? c : static_cast<uint64_t>(kk);
        };
        for (int m = tid; m < n2; m += blockDim.x) {
            double p = state[m] == 2 ? 1.0 : 0.0;
            if (state[m] == 1) {
                p = static_cast<double>(static_cast<uint64_t>(kk) * wts[m]) / static_cast<double>(TT);
                if (kk > 0) {
                    const uint64_t hi = static_cast<uint64_t>(kk) * cum[cur][m];
                    const uint64_t lo = hi - static_cast<uint64_t>(kk) * wts[m];
                    if (points_below(hi) - points_below(lo) == 1ull) state[m] = 3;
                }
            }
            pi[m] = p;
        }
    }
    __syncthreads();
    // taken slots in slot order: positions from a running count (reuses the scan buffers)
    for (int m = tid; m < n2; m += blockDim.x) cum[0][m] = state[m] >= 2 ? 1ull : 0ull;
    __syncthreads();
    cur = 0;
    for (int off = 1; off < n2; off <<= 1) {
        for (int m = tid; m < n2; m += blockDim.x)
            cum[cur ^ 1][m] = cum[cur][m] + (m >= off ? cum[cur][m - off] : 0ull);
        cur ^= 1;
        __syncthreads();
    }
    for (int m = tid; m < n2; m += blockDim.x)
        if (state[m] >= 2) sel[cum[cur][m] - 1] = m;
    // slots ordered by label id (slots without weight last), for the expected count of a label
    for (int size = 2; size <= n2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < n2 / 2; t += blockDim.x) {
                const int lo = 2 * t - (t & (stride - 1));
                const int hi = lo + stride;
                const bool up = (lo & size) == 0;
                const uint64_t a = byid[lo], b = byid[hi];
                if ((a > b) == up) { byid[lo] = b; byid[hi] = a; }
            }
            __syncthreads();
        }
    }
    const double unif = static_cast<double>(n - k) / static_cast<double>(L);
    for (int j = tid; j < n; j += blockDim.x) {
        int64_t lab;
        if (j < k) lab = ids[sel[j]];
        else lab = static_cast<int64_t>(__umul64hi(fmix64(qstate + kDrawMul * static_cast<uint64_t>(j + 1)), static_cast<uint64_t>(L)));
        double c = 0.0;
        if (k > 0) {
            const uint64_t key = static_cast<uint64_t>(lab) << 32;
            int lo = 0, hi = n2;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (byid[mid] < key) lo = mid + 1; else hi = mid;
            }
            for (int p = lo; p < n2 && (byid[p] >> 32) == static_cast<uint64_t>(lab); ++p)
                c += pi[static_cast<uint32_t>(byid[p])];                   // in slot order
        }
        neg[i * n + j] = static_cast<int32_t>(lab);
        logq[i * n + j] = static_cast<float>(log(c + unif));
    }
}

}  // namespace xc

extern "C" int xc_sample_negatives(const int32_t* shortlist, int64_t B, int k_h, int k_r, int64_t L,
                                   uint64_t seed, int32_t* neg, float* logq, void* stream) {
    using namespace xc;
    if (B < 1 || k_h < 0 || k_r < 0 || k_h + k_r < 1 || k_h > XC_MAX_K_SAMPLE) return XC_ESHAPE;
    if (L < 1 || L > 0x7fffffffLL || k_h >= L) return XC_ESHAPE;
    if (B > 0x7fffffffLL) return XC_ESHAPE;
    if (!neg || !logq) return XC_EINVAL;
    int n2 = 2;
    while (n2 < k_h) n2 <<= 1;
    if (k_h == 0) shortlist = nullptr;      // nothing to exclude: same as the warm-up draw
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_SAMPLE, st, (sample_kernel<<<dim3(static_cast<unsigned>(B)), kSampleThreads, 0, st>>>(
        shortlist, k_h, k_r, L, seed, n2, neg, logq)));
    XC_HIP_CHECK(hipGetLastError());
    return XC_OK;
}

extern "C" int xc_sample_negatives_mixture(const int32_t* shortlist, const float* scores, int64_t B, int M,
                                           int k_h, int k_r, int64_t L, uint64_t seed, int32_t* neg,
                                           float* logq, void* stream) {
    using namespace xc;
    if (B < 1 || B > 0x7fffffffLL || M < 1 || M > XC_MAX_K_SAMPLE) return XC_ESHAPE;
    if (k_h < 0 || k_r < 0 || k_h + k_r < 1 || L < 1 || L > 0x7fffffffLL) return XC_ESHAPE;
    if (!shortlist || !scores || !neg || !logq) return XC_EINVAL;
    int n2 = 2;
    while (n2 < M) n2 <<= 1;
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_SAMPLE, st, (sample_mixture_kernel<<<dim3(static_cast<unsigned>(B)), kSampleThreads, 0, st>>>(
        shortlist, scores, M, k_h, k_r, L, seed, n2, neg, logq)));
    XC_HIP_CHECK(hipGetLastError());
    return XC_OK;
}

extern "C" int xc_sample_negatives_pps(const int32_t* shortlist, const float* scores, int64_t B, int M,
                                       int k_h, int k_r, int64_t L, uint64_t seed, int32_t* neg,
                                       float* logq, void* stream) {
    using namespace xc;
    if (B < 1 || B > 0x7fffffffLL || M < 1 || M > XC_MAX_K_SAMPLE) return XC_ESHAPE;
    if (k_h < 0 || k_h > XC_MAX_K_SAMPLE || k_r < 0 || k_h + k_r < 1 || L < 1 || L > 0x7fffffffLL) return XC_ESHAPE;
    if (!shortlist || !scores || !neg || !logq) return XC_EINVAL;
    int n2 = 2;
    while (n2 < M) n2 <<= 1;
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_SAMPLE, st, (sample_pps_kernel<<<dim3(static_cast<unsigned>(B)), kSampleThreads, 0, st>>>(
        shortlist, scores, M, k_h, k_r, L, seed, n2, neg, logq)));
    XC_HIP_CHECK(hipGetLastError());
    return XC_OK;
}
