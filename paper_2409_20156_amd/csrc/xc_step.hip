// One training step of the classifier layer (Alg. 1: scores on positives and
// sampled negatives, the loss of Eq. 2, SGD on W; loss averaged over the batch,
// Sec. 4).  Three kernel groups:
//   gather_kernel   per query: gather the candidate rows of W, scores, loss,
//                   d loss/d score per pair, dZ -- one pass over the rows
//   radix sort      (label, pair index) by label, stable, 8 bits per pass
//   heads + update  segment heads -> touched list; per touched label the summed
//                   gradient over its pairs and the fused SGD row update
#include "xc_common.h"

namespace xc {

constexpr int kStepThreads = 256;
constexpr int kMaxRowFloats = XC_MAX_ROW_BYTES / 2;     // bf16 rows hold the most elements
constexpr int kSortTile = 256;                          // keys ranked together in the scatter
constexpr int kSortMaxBlocks = 512;
constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;

template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
    static constexpr int kPerChunk = 8;
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) { unpack8(v, f); }
    static __device__ __forceinline__ uint4 pack(const float (&f)[8]) {
        uint4 v;
        v.x = float_to_bf16_bits(f[0]) | (float_to_bf16_bits(f[1]) << 16);
        v.y = float_to_bf16_bits(f[2]) | (float_to_bf16_bits(f[3]) << 16);
        v.z = float_to_bf16_bits(f[4]) | (float_to_bf16_bits(f[5]) << 16);
        v.w = float_to_bf16_bits(f[6]) | (float_to_bf16_bits(f[7]) << 16);
        return v;
    }
};
template <> struct Elem<float> {
    static constexpr int kPerChunk = 4;
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&f)[4]) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                          __float_as_uint(f[3]));
    }
};

__device__ __forceinline__ float softplusf(float x) {      // log(1 + e^x), stable
    return fmaxf(x, 0.0f) + log1pf(expf(-fabsf(x)));
}
__device__ __forceinline__ float sigmoidf(float x) {
    const float e = expf(-fabsf(x));
    return x >= 0.0f ? 1.0f / (1.0f + e) : e / (1.0f + e);
}
// factor that rescales a sum kept relative to maximum m to a new maximum mn >= m
__device__ __forceinline__ float rescale(float m, float mn) { return m == mn ? 1.0f : expf(m - mn); }

// ---------------------------------------------------------------------------
// gather + scores + loss + dZ.  One workgroup per query; a "group" of G lanes
// (G = 16, 32 or 64) owns one candidate row at a time, lane gl of the group
// holding the 16-byte chunks gl, gl+G, ... of the row (CPL chunks per lane).
// ---------------------------------------------------------------------------
template <typename T, int CPL, int KIND>
__global__ __launch_bounds__(kStepThreads)
void gather_kernel(const T* __restrict__ Z, const T* __restrict__ W, int64_t L, int d,
                   const int32_t* __restrict__ pos, int k_p, const int32_t* __restrict__ neg,
                   const float* __restrict__ logq, int n_neg, int G, float inv_B,
                   uint32_t* __restrict__ keys, uint32_t* __restrict__ vals,
                   float* __restrict__ gco, float* __restrict__ loss_q, float* __restrict__ dZ) {
    constexpr int EPC = Elem<T>::kPerChunk;
    constexpr int U = 4;                          // candidate rows in flight per group
    __shared__ float red[kStepThreads / kWave][kMaxRowFloats];
    __shared__ float part[kStepThreads];          // per-group partial results
    __shared__ float part2[kStepThreads];
    __shared__ float part3[kStepThreads];
    __shared__ float part4[kStepThreads];

    const int64_t i = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int gl = lane & (G - 1);
    const int NG = kStepThreads / G;
    const int grp = tid / G;
    const int n = k_p + n_neg;
    const int nchunks = d / EPC;
    const int64_t row_bytes = static_cast<int64_t>(d) * sizeof(T);
    const unsigned char* Wb = reinterpret_cast<const unsigned char*>(W);
    const int32_t* pos_i = pos + i * k_p;
    const int32_t* neg_i = neg + i * n_neg;
    const float* lq_i = logq + i * n_neg;
    const int64_t p_base = i * n;

    // query row -> registers
    float zf[CPL][EPC];
    {
        const unsigned char* zrow = reinterpret_cast<const unsigned char*>(Z) + i * row_bytes;
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int ch = gl + j * G;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (ch < nchunks) v = *reinterpret_cast<const uint4*>(zrow + ch * 16);
            Elem<T>::unpack(v, zf[j]);
        }
    }

    float dz[CPL][EPC];            // BCE: sum g w.  soft-max: sum e^{t-m} w
    float pz[CPL][EPC];            // soft-max only: sum over positives of w
#pragma unroll
    for (int j = 0; j < CPL; ++j)
#pragma unroll
        for (int e = 0; e < EPC; ++e) { dz[j][e] = 0.0f; pz[j][e] = 0.0f; }
    float loss_acc = 0.0f;         // BCE: sum of pair losses.  soft-max: sum of positive logits
    float m_run = -INFINITY, s_run = 0.0f;
    int npos = 0;

    for (int c0 = grp; c0 < n; c0 += NG * U) {
        int32_t id[U];
        float lq[U];
        bool ok[U], isp[U];
        uint4 rw[U][CPL];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * NG;
            id[u] = -1; lq[u] = 0.0f; isp[u] = false;
            if (c < n) {
                if (c < k_p) { id[u] = pos_i[c]; isp[u] = true; }
                else { id[u] = neg_i[c - k_p]; lq[u] = lq_i[c - k_p]; }
            }
            ok[u] = id[u] >= 0 && id[u] < L;
            if (ok[u] && !isp[u]) {                 // (1 - y_l): a positive among the negatives
                for (int q = 0; q < k_p; ++q) ok[u] = ok[u] && (pos_i[q] != id[u]);
            }
#pragma unroll
            for (int j = 0; j < CPL; ++j) {
                const int ch = gl + j * G;
                rw[u][j] = make_uint4(0, 0, 0, 0);
                if (ok[u] && ch < nchunks)
                    rw[u][j] = *reinterpret_cast<const uint4*>(Wb + static_cast<int64_t>(id[u]) * row_bytes + ch * 16);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * NG;
            float wf[CPL][EPC];
            float s = 0.0f;
#pragma unroll
            for (int j = 0; j < CPL; ++j) {
                Elem<T>::unpack(rw[u][j], wf[j]);
#pragma unroll
                for (int e = 0; e < EPC; ++e) s = fmaf(wf[j][e], zf[j][e], s);
            }
            for (int off = G >> 1; off > 0; off >>= 1) s += __shfl_xor(s, off, kWave);
            float g = 0.0f;
            if (KIND == XC_LOSS_BCE) {
                if (ok[u]) {
                    if (isp[u]) { loss_acc += softplusf(-s); g = sigmoidf(s) - 1.0f; }
                    else { const float a = expf(-lq[u]); loss_acc += a * softplusf(s); g = a * sigmoidf(s); }
                    g *= inv_B;
#pragma unroll
                    for (int j = 0; j < CPL; ++j)
#pragma unroll
                        for (int e = 0; e < EPC; ++e) dz[j][e] = fmaf(g, wf[j][e], dz[j][e]);
                }
            } else {
                if (ok[u]) {
                    const float t = s - lq[u];
                    g = t;                               // logit parked until the normaliser is known
                    const float mn = fmaxf(m_run, t);
                    const float sc = rescale(m_run, mn);
                    const float w = expf(t - mn);
                    s_run = s_run * sc + w;
                    m_run = mn;
#pragma unroll
                    for (int j = 0; j < CPL; ++j)
#pragma unroll
                        for (int e = 0; e < EPC; ++e) dz[j][e] = fmaf(w, wf[j][e], dz[j][e] * sc);
                    if (isp[u]) {
                        loss_acc += t; ++npos;
#pragma unroll
                        for (int j = 0; j < CPL; ++j)
#pragma unroll
                            for (int e = 0; e < EPC; ++e) pz[j][e] += wf[j][e];
                    }
                }
            }
            if (gl == 0 && c < n) {
                keys[p_base + c] = ok[u] ? static_cast<uint32_t>(id[u]) : static_cast<uint32_t>(L);
                vals[p_base + c] = static_cast<uint32_t>(p_base + c);
                gco[p_base + c] = g;
            }
        }
    }

    // ---- combine the groups of the workgroup -------------------------------
    float lse = 0.0f, inv_sum = 0.0f, inv_npos = 0.0f;
    int npos_all = 0;
    if (KIND == XC_LOSS_BCE) {
        if (gl == 0) part[grp] = loss_acc;
        __syncthreads();
        if (tid == 0) {
            float t = 0.0f;
            for (int g2 = 0; g2 < NG; ++g2) t += part[g2];
            loss_q[i] = t;
        }
    } else {
        if (gl == 0) { part[grp] = m_run; part2[grp] = s_run; part3[grp] = loss_acc; part4[grp] = static_cast<float>(npos); }
        __syncthreads();
        float M = -INFINITY;
        for (int g2 = 0; g2 < NG; ++g2) M = fmaxf(M, part[g2]);
        float tot = 0.0f, tp = 0.0f, np = 0.0f;
        for (int g2 = 0; g2 < NG; ++g2) { tot += part2[g2] * rescale(part[g2], M); tp += part3[g2]; np += part4[g2]; }
        npos_all = static_cast<int>(np);
        if (npos_all > 0) {
            lse = M + logf(tot);
            inv_sum = 1.0f / tot;
            inv_npos = 1.0f / np;
        }
        const float sc = npos_all > 0 ? rescale(m_run, M) * inv_sum : 0.0f;   // own partial -> probabilities
#pragma unroll
        for (int j = 0; j < CPL; ++j)
#pragma unroll
            for (int e = 0; e < EPC; ++e) dz[j][e] = (dz[j][e] * sc - pz[j][e] * inv_npos) * inv_B;
        if (tid == 0) loss_q[i] = npos_all > 0 ? (lse - tp * inv_npos) : 0.0f;
    }

    // dZ: sum over groups of a wave (lanes with equal gl), then over the waves
#pragma unroll
    for (int j = 0; j < CPL; ++j)
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
            float v = dz[j][e];
            for (int off = G; off < kWave; off <<= 1) v += __shfl_xor(v, off, kWave);
            dz[j][e] = v;
        }
    if (lane < G) {
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int ch = gl + j * G;
            if (ch < nchunks) {
#pragma unroll
                for (int e = 0; e < EPC; ++e) red[wave][ch * EPC + e] = dz[j][e];
            }
        }
    }
    __syncthreads();
    for (int c = tid; c < d; c += kStepThreads) {
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < kStepThreads / kWave; ++w) v += red[w][c];
        dZ[i * d + c] = v;
    }

    if (KIND == XC_LOSS_SOFTMAX) {
        // pair coefficients now that the normaliser is known
        for (int c = tid; c < n; c += kStepThreads) {
            const int64_t p = p_base + c;
            if (npos_all == 0) { keys[p] = static_cast<uint32_t>(L); gco[p] = 0.0f; }
            else if (keys[p] != static_cast<uint32_t>(L)) {
                const float t = gco[p];
                gco[p] = (expf(t - lse) - (c < k_p ? inv_npos : 0.0f)) * inv_B;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// loss = (1/B) sum_i loss_q[i], summed in a fixed order by one workgroup
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256)
void loss_reduce_kernel(const float* __restrict__ loss_q, int64_t B, float inv_B, float* __restrict__ loss) {
    __shared__ float sh[256];
    float t = 0.0f;
    for (int64_t i = threadIdx.x; i < B; i += 256) t += loss_q[i];
    sh[threadIdx.x] = t;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = sh[0] * inv_B;
}

// ---------------------------------------------------------------------------
// stable LSD radix sort of (key, value) pairs, 8 bits per pass.
// Block b owns the contiguous chunk [b*chunk, (b+1)*chunk) of the input.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256)
void radix_count_kernel(const uint32_t* __restrict__ keys, int64_t P, int64_t chunk, int shift,
                        int nb, int* __restrict__ counts /* [kRadix][nb] */) {
    __shared__ int hist[kRadix];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t p0 = blockIdx.x * chunk;
    int64_t p1 = p0 + chunk;
    p1 = p1 < P ? p1 : P;
    for (int64_t p = p0 + threadIdx.x; p < p1; p += 256)
        atomicAdd(&hist[(keys[p] >> shift) & (kRadix - 1)], 1);
    __syncthreads();
    counts[threadIdx.x * nb + blockIdx.x] = hist[threadIdx.x];
}

// exclusive scan of `n` ints in place, one workgroup of 1024 threads
__global__ __launch_bounds__(1024)
void scan_kernel(int* __restrict__ data, int n) {
    __shared__ int wsum[16];
    const int tid = threadIdx.x;
    const int per = (n + 1023) / 1024;
    const int b = tid * per;
    int e = b + per;
    e = e < n ? e : n;
    int s = 0;
    for (int x = b; x < e; ++x) s += data[x];
    const int incl = wave_incl_scan(s);
    if ((tid & 63) == 63) wsum[tid >> 6] = incl;
    __syncthreads();
    int off = 0;
    for (int w = 0; w < (tid >> 6); ++w) off += wsum[w];
    int run = off + incl - s;
    for (int x = b; x < e; ++x) { const int v = data[x]; data[x] = run; run += v; }
}

__global__ __launch_bounds__(kSortTile)
void radix_scatter_kernel(const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in,
                          uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out, int64_t P,
                          int64_t chunk, int shift, int nb, const int* __restrict__ offsets) {
    __shared__ int offs[kRadix];
    __shared__ int whist[kSortTile / kWave][kRadix];
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    offs[tid] = offsets[tid * nb + blockIdx.x];
#pragma unroll
    for (int w = 0; w < kSortTile / kWave; ++w) whist[w][tid] = 0;
    __syncthreads();
    const int64_t p0 = blockIdx.x * chunk;
    int64_t p1 = p0 + chunk;
    p1 = p1 < P ? p1 : P;
    for (int64_t t0 = p0; t0 < p1; t0 += kSortTile) {
        const int64_t p = t0 + tid;
        const bool valid = p < p1;
        uint32_t key = 0, val = 0;
        if (valid) { key = keys_in[p]; val = vals_in[p]; }
        const int digit = (key >> shift) & (kRadix - 1);
        // lanes of this wave holding the same digit
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            const bool bit = (digit >> b) & 1;
            const uint64_t bal = __ballot(bit);
            same &= bit ? bal : ~bal;
        }
        const int rank = __popcll(same & lanemask_lt());
        if (valid && rank == 0) whist[wave][digit] = __popcll(same);
        __syncthreads();
        if (valid) {
            int before = offs[digit];
            for (int w = 0; w < wave; ++w) before += whist[w][digit];
            keys_out[before + rank] = key;
            vals_out[before + rank] = val;
        }
        __syncthreads();
        int add = 0;
#pragma unroll
        for (int w = 0; w < kSortTile / kWave; ++w) { add += whist[w][tid]; whist[w][tid] = 0; }
        offs[tid] += add;
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// segment heads of the sorted keys -> touched list and segment starts
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool is_head(const uint32_t* keys, int64_t p, uint32_t Lkey) {
    const uint32_t k = keys[p];
    return k < Lkey && (p == 0 || keys[p - 1] != k);
}

__global__ __launch_bounds__(256)
void heads_count_kernel(const uint32_t* __restrict__ keys, int64_t P, int64_t chunk, uint32_t Lkey,
                        int* __restrict__ head_cnt, int* __restrict__ valid_cnt) {
    __shared__ int sh[2][256];
    const int64_t p0 = blockIdx.x * chunk;
    int64_t p1 = p0 + chunk;
    p1 = p1 < P ? p1 : P;
    int h = 0, v = 0;
    for (int64_t p = p0 + threadIdx.x; p < p1; p += 256) {
        h += is_head(keys, p, Lkey) ? 1 : 0;
        v += keys[p] < Lkey ? 1 : 0;
    }
    sh[0][threadIdx.x] = h; sh[1][threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) { sh[0][threadIdx.x] += sh[0][threadIdx.x + s]; sh[1][threadIdx.x] += sh[1][threadIdx.x + s]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) { head_cnt[blockIdx.x] = sh[0][0]; valid_cnt[blockIdx.x] = sh[1][0]; }
}

__global__ __launch_bounds__(256)
void heads_write_kernel(const uint32_t* __restrict__ keys, int64_t P, int64_t chunk, uint32_t Lkey,
                        int nb, const int* __restrict__ head_cnt, const int* __restrict__ valid_cnt,
                        int32_t* __restrict__ touched, int32_t* __restrict__ seg_start,
                        int32_t* __restrict__ n_touched) {
    __shared__ int sh[256];
    __shared__ int wcnt[4];
    __shared__ int running;
    const int tid = threadIdx.x;
    // heads in the blocks before this one
    int t = 0;
    for (int b = tid; b < static_cast<int>(blockIdx.x); b += 256) t += head_cnt[b];
    sh[tid] = t;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) sh[tid] += sh[tid + s];
        __syncthreads();
    }
    if (tid == 0) running = sh[0];
    __syncthreads();
    if (blockIdx.x == 0) {             // totals: block 0 sums every block's counts
        int th = 0, tv = 0;
        for (int b = tid; b < nb; b += 256) { th += head_cnt[b]; tv += valid_cnt[b]; }
        __shared__ int sh2[2][256];
        sh2[0][tid] = th; sh2[1][tid] = tv;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s) { sh2[0][tid] += sh2[0][tid + s]; sh2[1][tid] += sh2[1][tid + s]; }
            __syncthreads();
        }
        if (tid == 0) { n_touched[0] = sh2[0][0]; seg_start[sh2[0][0]] = sh2[1][0]; }
    }
    const int64_t p0 = blockIdx.x * chunk;
    int64_t p1 = p0 + chunk;
    p1 = p1 < P ? p1 : P;
    for (int64_t t0 = p0; t0 < p1; t0 += 256) {
        const int64_t p = t0 + tid;
        const bool head = p < p1 && is_head(keys, p, Lkey);
        const uint64_t bal = __ballot(head);
        if ((tid & 63) == 0) wcnt[tid >> 6] = __popcll(bal);
        __syncthreads();
        int before = running;
        for (int w = 0; w < (tid >> 6); ++w) before += wcnt[w];
        if (head) {
            const int s = before + __popcll(bal & lanemask_lt());
            touched[s] = static_cast<int32_t>(keys[p]);
            seg_start[s] = static_cast<int32_t>(p);
        }
        __syncthreads();
        if (tid == 0) running += wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// per touched label: dW = sum over its pairs of g * z_i ; w <- w - lr * dW
// One group of G lanes per segment, chunks distributed as in gather_kernel.
// ---------------------------------------------------------------------------
template <typename T, int CPL>
__global__ __launch_bounds__(kStepThreads)
void update_kernel(const T* __restrict__ Z, T* __restrict__ W, int d, int n, int G,
                   const uint32_t* __restrict__ vals, const float* __restrict__ gco,
                   const int32_t* __restrict__ touched, const int32_t* __restrict__ seg_start,
                   const int32_t* __restrict__ n_touched, float lr, T* __restrict__ rows_out) {
    constexpr int EPC = Elem<T>::kPerChunk;
    constexpr int U = 4;
    const int tid = threadIdx.x;
    const int gl = tid & (G - 1);
    const int NG = kStepThreads / G;
    const int64_t s = static_cast<int64_t>(blockIdx.x) * NG + tid / G;
    if (s >= n_touched[0]) return;
    const int nchunks = d / EPC;
    const int64_t row_bytes = static_cast<int64_t>(d) * sizeof(T);
    const unsigned char* Zb = reinterpret_cast<const unsigned char*>(Z);
    const int p0 = seg_start[s], p1 = seg_start[s + 1];
    const int64_t label = touched[s];

    float acc[CPL][EPC];
#pragma unroll
    for (int j = 0; j < CPL; ++j)
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[j][e] = 0.0f;

    for (int p = p0; p < p1; p += U) {
        float g[U];
        uint4 rz[U][CPL];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            g[u] = 0.0f;
            const bool on = p + u < p1;
            uint32_t idx = 0;
            if (on) { idx = vals[p + u]; g[u] = gco[idx]; }
            const int64_t qi = idx / static_cast<uint32_t>(n);
#pragma unroll
            for (int j = 0; j < CPL; ++j) {
                const int ch = gl + j * G;
                rz[u][j] = make_uint4(0, 0, 0, 0);
                if (on && ch < nchunks) rz[u][j] = *reinterpret_cast<const uint4*>(Zb + qi * row_bytes + ch * 16);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int j = 0; j < CPL; ++j) {
                float zf[EPC];
                Elem<T>::unpack(rz[u][j], zf);
#pragma unroll
                for (int e = 0; e < EPC; ++e) acc[j][e] = fmaf(g[u], zf[e], acc[j][e]);
            }
        }
    }
    unsigned char* wrow = reinterpret_cast<unsigned char*>(W) + label * row_bytes;
    unsigned char* orow = rows_out ? reinterpret_cast<unsigned char*>(rows_out) + s * row_bytes : nullptr;
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
        const int ch = gl + j * G;
        if (ch < nchunks) {
            float wf[EPC];
            const uint4 v = *reinterpret_cast<const uint4*>(wrow + ch * 16);
            Elem<T>::unpack(v, wf);
#pragma unroll
            for (int e = 0; e < EPC; ++e) wf[e] = fmaf(-lr, acc[j][e], wf[e]);
            const uint4 o = Elem<T>::pack(wf);
            *reinterpret_cast<uint4*>(wrow + ch * 16) = o;
            if (orow) *reinterpret_cast<uint4*>(orow + ch * 16) = o;
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct StepPlan {
    int64_t P;
    int n, G, cpl, nb, passes, key_bits;
    int64_t chunk;
    size_t off_keys0, off_keys1, off_vals0, off_vals1, off_g, off_lossq, off_counts, off_headcnt,
        off_validcnt, off_segstart, total;
};

static int plan_step(int64_t B, int64_t L, int d, int k_p, int n_neg, xc_dtype t, StepPlan* p) {
    if (t != XC_F32 && t != XC_BF16) return XC_EINVAL;
    if (B < 1 || d < 1 || k_p < 0 || n_neg < 0) return XC_ESHAPE;
    const int64_t n = static_cast<int64_t>(k_p) + n_neg;
    if (n < 1 || n > XC_MAX_CANDIDATES) return XC_ESHAPE;
    const int64_t row_bytes = static_cast<int64_t>(d) * (t == XC_F32 ? 4 : 2);
    if (row_bytes % 16 != 0 || row_bytes > XC_MAX_ROW_BYTES) return XC_ESHAPE;
    if (B * n >= 0x7fffffffLL) return XC_ESHAPE;
    p->P = B * n;
    p->n = static_cast<int>(n);
    const int nchunks = static_cast<int>(row_bytes / 16);
    int G = 16;
    while (G < 64 && G * 4 < nchunks) G <<= 1;     // at most 4 chunks per lane
    if (G < 64 && nchunks % G != 0 && nchunks > G) { /* tail chunks are predicated */ }
    p->G = G;
    p->cpl = (nchunks + G - 1) / G;
    if (p->cpl > 4) return XC_ESHAPE;
    int nb = static_cast<int>((p->P + 2047) / 2048);
    if (nb > kSortMaxBlocks) nb = kSortMaxBlocks;
    if (nb < 1) nb = 1;
    int64_t chunk = (p->P + nb - 1) / nb;
    chunk = (chunk + kSortTile - 1) / kSortTile * kSortTile;
    nb = static_cast<int>((p->P + chunk - 1) / chunk);
    p->nb = nb;
    p->chunk = chunk;
    int bits = 1;
    if (L >= 0) { while ((static_cast<int64_t>(1) << bits) <= L && bits < 32) ++bits; }
    p->key_bits = bits;                                // keys take values 0..L
    p->passes = (bits + kRadixBits - 1) / kRadixBits;
    size_t off = 0;
    auto take = [&off](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
    const size_t P = static_cast<size_t>(p->P);
    p->off_keys0 = take(P * 4); p->off_keys1 = take(P * 4);
    p->off_vals0 = take(P * 4); p->off_vals1 = take(P * 4);
    p->off_g = take(P * 4);
    p->off_lossq = take(static_cast<size_t>(B) * 4);
    p->off_counts = take(static_cast<size_t>(kRadix) * nb * 4);
    p->off_headcnt = take(static_cast<size_t>(nb) * 4);
    p->off_validcnt = take(static_cast<size_t>(nb) * 4);
    p->off_segstart = take((P + 1) * 4);
    p->total = off;
    return XC_OK;
}

template <typename T, int KIND>
static void launch_gather(const StepPlan& pl, hipStream_t st, const void* Z, const void* W, int64_t B,
                          int64_t L, int d, const int32_t* pos, int k_p, const int32_t* neg,
                          const float* logq, int n_neg, uint32_t* keys, uint32_t* vals, float* gco,
                          float* loss_q, float* dZ) {
    const float inv_B = 1.0f / static_cast<float>(B);
    const dim3 grid(static_cast<unsigned>(B));
#define XC_GATHER(CPL)                                                                              \
    XC_LAUNCH(K_GATHER, st, (gather_kernel<T, CPL, KIND><<<grid, kStepThreads, 0, st>>>(            \
        static_cast<const T*>(Z), static_cast<const T*>(W), L, d, pos, k_p, neg, logq, n_neg, pl.G, \
        inv_B, keys, vals, gco, loss_q, dZ)))
    switch (pl.cpl) {
        case 1: XC_GATHER(1); break;
        case 2: XC_GATHER(2); break;
        case 3: XC_GATHER(3); break;
        default: XC_GATHER(4); break;
    }
#undef XC_GATHER
}

template <typename T>
static void launch_update(const StepPlan& pl, hipStream_t st, const void* Z, void* W, int d,
                          const uint32_t* vals, const float* gco, const int32_t* touched,
                          const int32_t* seg_start, const int32_t* n_touched, float lr, void* rows_out) {
    const int NG = kStepThreads / pl.G;
    const dim3 grid(static_cast<unsigned>((pl.P + NG - 1) / NG));
#define XC_UPDATE(CPL)                                                                            \
    XC_LAUNCH(K_UPDATE, st, (update_kernel<T, CPL><<<grid, kStepThreads, 0, st>>>(                \
        static_cast<const T*>(Z), static_cast<T*>(W), d, pl.n, pl.G, vals, gco, touched, seg_start, \
        n_touched, lr, static_cast<T*>(rows_out))))
    switch (pl.cpl) {
        case 1: XC_UPDATE(1); break;
        case 2: XC_UPDATE(2); break;
        case 3: XC_UPDATE(3); break;
        default: XC_UPDATE(4); break;
    }
#undef XC_UPDATE
}

}  // namespace xc

extern "C" int xc_step_workspace(int64_t B, int d, int k_p, int n_neg, xc_dtype t, size_t* bytes) {
    if (!bytes) return XC_EINVAL;
    xc::StepPlan p;
    const int rc = xc::plan_step(B, 0x7ffffffeLL, d, k_p, n_neg, t, &p);
    if (rc != XC_OK) return rc;
    *bytes = p.total;
    return XC_OK;
}

extern "C" int xc_step(const void* Z, void* W, int64_t B, int64_t L, int d, const int32_t* pos, int k_p,
                       const int32_t* neg, const float* logq, int n_neg, float lr, xc_loss kind,
                       xc_dtype t, float* loss, float* dZ, int32_t* touched, int32_t* n_touched,
                       void* W_rows_out, void* ws, size_t ws_bytes, void* stream) {
    using namespace xc;
    if (kind != XC_LOSS_BCE && kind != XC_LOSS_SOFTMAX) return XC_EINVAL;
    if (L < 1 || L > 0x7ffffffeLL) return XC_ESHAPE;
    StepPlan pl;
    const int rc = plan_step(B, L, d, k_p, n_neg, t, &pl);
    if (rc != XC_OK) return rc;
    if (!Z || !W || !loss || !dZ || !touched || !n_touched || !ws) return XC_EINVAL;
    if ((k_p > 0 && !pos) || (n_neg > 0 && (!neg || !logq))) return XC_EINVAL;
    if (!aligned16(Z) || !aligned16(W) || !aligned16(dZ) || !aligned16(ws)) return XC_EINVAL;
    if (W_rows_out && !aligned16(W_rows_out)) return XC_EINVAL;
    if (Z == static_cast<const void*>(dZ)) return XC_EINVAL;
    {   // layout does not depend on L except for the number of sort passes
        StepPlan ref;
        plan_step(B, 0x7ffffffeLL, d, k_p, n_neg, t, &ref);
        if (ws_bytes < ref.total) return XC_EWORKSPACE;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* w8 = static_cast<unsigned char*>(ws);
    uint32_t* keys0 = reinterpret_cast<uint32_t*>(w8 + pl.off_keys0);
    uint32_t* keys1 = reinterpret_cast<uint32_t*>(w8 + pl.off_keys1);
    uint32_t* vals0 = reinterpret_cast<uint32_t*>(w8 + pl.off_vals0);
    uint32_t* vals1 = reinterpret_cast<uint32_t*>(w8 + pl.off_vals1);
    float* gco = reinterpret_cast<float*>(w8 + pl.off_g);
    float* loss_q = reinterpret_cast<float*>(w8 + pl.off_lossq);
    int* counts = reinterpret_cast<int*>(w8 + pl.off_counts);
    int* head_cnt = reinterpret_cast<int*>(w8 + pl.off_headcnt);
    int* valid_cnt = reinterpret_cast<int*>(w8 + pl.off_validcnt);
    int32_t* seg_start = reinterpret_cast<int32_t*>(w8 + pl.off_segstart);

    // S3 + S4
    if (t == XC_BF16) {
        if (kind == XC_LOSS_BCE)
            launch_gather<bf16_t, XC_LOSS_BCE>(pl, st, Z, W, B, L, d, pos, k_p, neg, logq, n_neg, keys0, vals0, gco, loss_q, dZ);
        else
            launch_gather<bf16_t, XC_LOSS_SOFTMAX>(pl, st, Z, W, B, L, d, pos, k_p, neg, logq, n_neg, keys0, vals0, gco, loss_q, dZ);
    } else {
        if (kind == XC_LOSS_BCE)
            launch_gather<float, XC_LOSS_BCE>(pl, st, Z, W, B, L, d, pos, k_p, neg, logq, n_neg, keys0, vals0, gco, loss_q, dZ);
        else
            launch_gather<float, XC_LOSS_SOFTMAX>(pl, st, Z, W, B, L, d, pos, k_p, neg, logq, n_neg, keys0, vals0, gco, loss_q, dZ);
    }
    XC_HIP_CHECK(hipGetLastError());
    XC_LAUNCH(K_LOSS_REDUCE, st, (loss_reduce_kernel<<<1, 256, 0, st>>>(loss_q, B, 1.0f / static_cast<float>(B), loss)));
    XC_HIP_CHECK(hipGetLastError());

    // S5: sort pairs by label
    uint32_t *kin = keys0, *kout = keys1, *vin = vals0, *vout = vals1;
    for (int pass = 0; pass < pl.passes; ++pass) {
        const int shift = pass * kRadixBits;
        XC_LAUNCH(K_RADIX_COUNT, st, (radix_count_kernel<<<pl.nb, 256, 0, st>>>(kin, pl.P, pl.chunk, shift, pl.nb, counts)));
        XC_LAUNCH(K_RADIX_SCAN, st, (scan_kernel<<<1, 1024, 0, st>>>(counts, kRadix * pl.nb)));
        XC_LAUNCH(K_RADIX_SCATTER, st, (radix_scatter_kernel<<<pl.nb, kSortTile, 0, st>>>(kin, vin, kout, vout, pl.P, pl.chunk, shift, pl.nb, counts)));
        XC_HIP_CHECK(hipGetLastError());
        uint32_t* tk = kin; kin = kout; kout = tk;
        uint32_t* tv = vin; vin = vout; vout = tv;
    }
    XC_LAUNCH(K_HEADS_COUNT, st, (heads_count_kernel<<<pl.nb, 256, 0, st>>>(kin, pl.P, pl.chunk, static_cast<uint32_t>(L), head_cnt, valid_cnt)));
    XC_LAUNCH(K_HEADS_WRITE, st, (heads_write_kernel<<<pl.nb, 256, 0, st>>>(kin, pl.P, pl.chunk, static_cast<uint32_t>(L), pl.nb, head_cnt,
                                                                            valid_cnt, touched, seg_start, n_touched)));
    XC_HIP_CHECK(hipGetLastError());
    if (t == XC_BF16) launch_update<bf16_t>(pl, st, Z, W, d, vin, gco, touched, seg_start, n_touched, lr, W_rows_out);
    else launch_update<float>(pl, st, Z, W, d, vin, gco, touched, seg_start, n_touched, lr, W_rows_out);
    XC_HIP_CHECK(hipGetLastError());
    return XC_OK;
}
