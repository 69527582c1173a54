// One training step of the classifier layer (Alg. 1: scores on positives and
// sampled negatives, the loss of Eq. 2, SGD on W; loss averaged over the batch,
// Sec. 4).  Three kernel groups:
//   gather_kernel   per query: gather the candidate rows of W, scores, loss,
//                   d loss/d score per pair, dZ -- one pass over the rows
//   radix sort      (label, pair index) by label, stable, digits of up to 11 bits
//   heads + update  segment heads -> touched list; per touched label the summed
//                   gradient over its pairs and the fused SGD row update
#include <mutex>

#include "xc_common.h"

namespace xc {

constexpr int kStepThreads = 256;
constexpr int kMaxRowFloats = XC_MAX_ROW_BYTES / 2;     // bf16 rows hold the most elements
constexpr int kSortTile = 256;                          // keys ranked together in the scatter
constexpr int kSortMaxBlocks = 2048;
constexpr int kSortCountEntries = 1 << 19;              // digit values x sort blocks at most (2 MiB of counts)
constexpr int kUpdateMaxGrid = 256 * 8;                 // workgroups of the update kernel
constexpr int kMaxRadixBits = 11;
constexpr int kMaxRadix = 1 << kMaxRadixBits;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    bf16x2 x, y;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    return __builtin_amdgcn_fdot2_f32_bf16(x, y, c, false);     // a.lo*b.lo + a.hi*b.hi + c in fp32
}

template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
    static constexpr int kPerChunk = 8;
    // s + <w, z> over the 8 elements of a chunk, both still packed
    static __device__ __forceinline__ float dot(const uint4& w, const uint4& z, float s) {
        s = dot2_bf16(w.x, z.x, s); s = dot2_bf16(w.y, z.y, s);
        s = dot2_bf16(w.z, z.z, s); s = dot2_bf16(w.w, z.w, s);
        return s;
    }
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) { unpack8(v, f); }
    // round to nearest even by the hardware conversion (v_cvt_pk_bf16_f32)
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        const f32x2 v = {lo, hi};
        const bf16x2 r = __builtin_convertvector(v, bf16x2);
        uint32_t u;
        __builtin_memcpy(&u, &r, 4);
        return u;
    }
    static __device__ __forceinline__ uint4 pack(const float (&f)[8]) {
        return make_uint4(pack2(f[0], f[1]), pack2(f[2], f[3]), pack2(f[4], f[5]), pack2(f[6], f[7]));
    }
};
template <> struct Elem<float> {
    static constexpr int kPerChunk = 4;
    static __device__ __forceinline__ float dot(const uint4& w, const uint4& z, float s) {
        s = fmaf(__uint_as_float(w.x), __uint_as_float(z.x), s);
        s = fmaf(__uint_as_float(w.y), __uint_as_float(z.y), s);
        s = fmaf(__uint_as_float(w.z), __uint_as_float(z.z), s);
        s = fmaf(__uint_as_float(w.w), __uint_as_float(z.w), s);
        return s;
    }
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

// ---- fast transcendental pieces (hardware exp2/log2/rcp, about 1 ulp each) ------------------
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
// log(1 + e) for 0 <= e <= 1: series below 2^-6 (where 1 + e would lose the low bits of e)
__device__ __forceinline__ float fast_log1p(float e) {
    const float series = e * (1.0f - e * (0.5f - e * (1.0f / 3.0f)));
    const float direct = __builtin_amdgcn_logf(1.0f + e) * 0.693147180559945309f;
    return e < 0.015625f ? series : direct;
}

// Transposing reduction over a group of G lanes: v[u] holds this lane's partial of row u.
// Returns, in lane gl, the sum over the group of row row_of_lane(gl): U-1 exchanges in the
// halving steps plus log2(G/U) plain ones, instead of U*log2(G).
// Value of lane (addr4 / 4) of the wave: one ds_bpermute.  The callers keep 4 * lane in a register and form
// the address with one XOR or take it from a loop-invariant; __shfl would recompute the lane id, the width
// arithmetic and the address at every call, which in the gather's inner loop was a tenth of all instructions.
__device__ __forceinline__ float lane_read(int addr4, float v) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(addr4, __float_as_int(v)));
}
template <int U>
__device__ __forceinline__ float reduce_rows(float (&v)[U], int G, int gl, int lane4) {
    int off = G >> 1;
#pragma unroll
    for (int cnt = U; cnt > 1; cnt >>= 1) {
        const bool hi = (gl & off) != 0;
#pragma unroll
        for (int j = 0; j < cnt / 2; ++j) {
            const float send = hi ? v[j] : v[j + cnt / 2];
            const float keep = hi ? v[j + cnt / 2] : v[j];
            v[j] = keep + lane_read(lane4 ^ (off << 2), send);
        }
        off >>= 1;
    }
    float y = v[0];
    for (; off > 0; off >>= 1) y += lane_read(lane4 ^ (off << 2), y);
    return y;
}
template <int U>
__device__ __forceinline__ int row_of_lane(int gl, int G) {
    int r = 0, off = G >> 1;
#pragma unroll
    for (int cnt = U; cnt > 1; cnt >>= 1) { r += (gl & off) ? cnt / 2 : 0; off >>= 1; }
    return r;
}
template <int U>
__device__ __forceinline__ int lane_of_row(int u, int G) {      // lowest lane of the group holding row u
    int l = 0, off = G >> 1;
#pragma unroll
    for (int cnt = U; cnt > 1; cnt >>= 1) { l += (u & (cnt / 2)) ? off : 0; off >>= 1; }
    return l;
}

// ---------------------------------------------------------------------------
// gather + scores + loss + dZ.  One workgroup per query; a "group" of G lanes
// (G = 16, 32 or 64) owns one candidate row at a time, lane gl of the group
// holding the 16-byte chunks gl, gl+G, ... of the row (CPL chunks per lane).
// ---------------------------------------------------------------------------
// FULL: every lane's CPL chunks exist (d / kPerChunk == G * CPL), so no load needs a bounds test; a masked
// pair then reads the query's own row (finite, and weighted zero) instead of branching around the loads.
// FUSE (BCE only): the pair sort has run before this kernel and single_slot[pair] says whether the pair's label
// occurs in no other unmasked pair of the batch (then: its position in the touched list, else -1).  Such a row
// is read by this pair alone, its gradient is g z_i with both factors at hand, so it is updated here, while it
// is in registers (w - lr g z, rounded once), and the row update kernel never sees it: one read and one write of
// the row in the whole step instead of two reads, a read of z_i and a write.
template <typename T, int CPL, int KIND, int U, bool FULL, bool STREAM, bool FUSE>
__global__ __launch_bounds__(kStepThreads)
void gather_kernel(const T* __restrict__ Z, T* W, int64_t L, int d,
                   const int32_t* __restrict__ pos, int k_p, const int32_t* __restrict__ neg,
                   const float* __restrict__ logq, int n_neg, int G, int SQ, int64_t B, float inv_B,
                   const int32_t* __restrict__ single_slot, float lr, T* rows_out,
                   float* __restrict__ gco, float* __restrict__ loss_q, float* __restrict__ dZ) {
    constexpr int EPC = Elem<T>::kPerChunk;       // U = candidate rows in flight per group
    __shared__ float red[kStepThreads / kWave][kMaxRowFloats];
    __shared__ int32_t spos[XC_MAX_KP];           // the query's positives, for the (1 - y_l) mask
    __shared__ float part[kStepThreads];          // per-group partial results
    __shared__ float part2[kStepThreads];
    __shared__ float part3[kStepThreads];
    __shared__ float part4[kStepThreads];

    // SQ workgroups share one query (the candidates are dealt out in turn); each writes a
    // partial loss and a partial dZ that a later kernel adds up in a fixed order
    const int64_t i = blockIdx.x / SQ;
    const int sq = blockIdx.x % SQ;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int gl = lane & (G - 1);
    const int NG = (kStepThreads / G) * SQ;               // groups working on this query
    const int grp = sq * (kStepThreads / G) + tid / G;
    const int n = k_p + n_neg;
    const int nchunks = d / EPC;
    const int64_t row_bytes = static_cast<int64_t>(d) * sizeof(T);
    unsigned char* Wb = reinterpret_cast<unsigned char*>(W);
    const int32_t* pos_i = pos + i * k_p;
    const int32_t* neg_i = neg + i * n_neg;
    const float* lq_i = logq + i * n_neg;
    const int64_t p_base = i * n;

    // query row -> registers, kept in storage format for the dot products
    uint4 zp[CPL];
    {
        const unsigned char* zrow = reinterpret_cast<const unsigned char*>(Z) + i * row_bytes;
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int ch = gl + j * G;
            zp[j] = make_uint4(0, 0, 0, 0);
            if (ch < nchunks) zp[j] = *reinterpret_cast<const uint4*>(zrow + ch * 16);
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

    for (int q = tid; q < k_p; q += kStepThreads) spos[q] = pos_i[q];
    __syncthreads();

    // ids and log-proposals of the candidates this group handles in one iteration; those
    // of the next iteration are fetched while the rows of the current one are in flight
    // The loads are unconditional, from a clamped index, and what they return is looked at only when the
    // iteration that uses it begins: nothing waits for them where they are issued, behind the row loads.
    int32_t id_nx[U];
    float lq_nx[U];
    int32_t sl_nx[FUSE ? U : 1];
    auto fetch_ids = [&](int c0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int cn = c0 + u * NG - k_p;
            cn = cn < 0 ? 0 : cn;
            cn = cn < n_neg ? cn : n_neg - 1;
            id_nx[u] = -1; lq_nx[u] = 0.0f;
            if (n_neg > 0) { id_nx[u] = neg_i[cn]; lq_nx[u] = lq_i[cn]; }      // uniform
            if (FUSE) {
                int ca = c0 + u * NG;
                ca = ca < n ? ca : n - 1;
                sl_nx[u] = single_slot[p_base + ca];
            }
        }
    };
    fetch_ids(grp);
    const int lane4 = lane << 2;
    const int grp_lane0 = lane & ~(G - 1);       // first lane of this group within the wave
    const uint64_t grp_mask = (G == kWave ? ~0ull : ((1ull << G) - 1ull)) << grp_lane0;
    const int row_rep = G / U;                   // lanes that end up holding the same row's score
    const int my_row = row_of_lane<U>(gl, G);
    const bool my_rep = (gl & (row_rep - 1)) == 0;
    const int32_t my_pos = gl < k_p ? spos[gl] : -2;      // lane-parallel (1 - y_l) check

    for (int c0 = grp; c0 < n; c0 += NG * U) {
        int32_t id[U];
        float lq[U];
        bool ok[U], isp[U];
        int32_t slot[FUSE ? U : 1];
        uint4 rw[U][CPL];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * NG;
            if (FUSE) slot[u] = sl_nx[u];
            isp[u] = c < k_p;
            const int32_t idp = spos[c & (XC_MAX_KP - 1)];           // read whatever c is, used if c < k_p
            id[u] = isp[u] ? idp : (c < n ? id_nx[u] : -1);
            lq[u] = (!isp[u] && c < n) ? lq_nx[u] : 0.0f;
            ok[u] = id[u] >= 0 && id[u] < L;
            {                                       // (1 - y_l): a positive among the negatives
                bool hit = !isp[u] && my_pos == id[u];
                if (k_p > G) {                      // uniform: more positives than lanes in a group
                    for (int q = G + gl; q < k_p; q += G) hit = hit || (!isp[u] && spos[q] == id[u]);
                }
                ok[u] = ok[u] && (__ballot(hit) & grp_mask) == 0ull;
            }
            if (FULL) {
                const unsigned char* src = ok[u] ? Wb + static_cast<int64_t>(id[u]) * row_bytes
                                                 : reinterpret_cast<const unsigned char*>(Z) + i * row_bytes;
#pragma unroll
                for (int j = 0; j < CPL; ++j)
                    rw[u][j] = load16<STREAM>(src + (gl + j * G) * 16);
            } else {
#pragma unroll
                for (int j = 0; j < CPL; ++j) {
                    const int ch = gl + j * G;
                    rw[u][j] = make_uint4(0, 0, 0, 0);
                    if (ok[u] && ch < nchunks)
                        rw[u][j] = load16<STREAM>(Wb + static_cast<int64_t>(id[u]) * row_bytes + ch * 16);
                }
            }
        }
        fetch_ids(c0 + NG * U);

        // per-lane partial dot products of the U rows, then a transposing reduction: lane gl
        // ends up with the complete score of row my_row (each row replicated in G/U lanes)
        float ps[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float s = 0.0f;
#pragma unroll
            for (int j = 0; j < CPL; ++j) s = Elem<T>::dot(rw[u][j], zp[j], s);
            ps[u] = s;
        }
        const float my_s = reduce_rows<U>(ps, G, gl, lane4);
        float my_lq = 0.0f;
        bool my_ok = false, my_isp = false;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (my_row == u) { my_lq = lq[u]; my_ok = ok[u]; my_isp = isp[u]; }
        }
        float my_g = 0.0f;          // BCE: d loss / d score.  soft-max: weight e^{t - m}
        float my_t = my_ok ? my_s - my_lq : -INFINITY;     // soft-max logit
        if (KIND == XC_LOSS_BCE) {
            if (my_ok) {
                // e = exp(-|s|) serves softplus(+-s) = max(+-s, 0) + log1p(e) and the sigmoid
                const float e = fast_exp(-fabsf(my_s));
                const float l1p = fast_log1p(e);
                const float r = fast_rcp(1.0f + e);
                const float sig = my_s >= 0.0f ? r : e * r;
                float term;
                if (my_isp) { term = fmaxf(-my_s, 0.0f) + l1p; my_g = sig - 1.0f; }
                else { const float a = fast_exp(-my_lq); term = a * (fmaxf(my_s, 0.0f) + l1p); my_g = a * sig; }
                if (my_rep) loss_acc += term;
                my_g *= inv_B;
            }
        } else {
            float mi = my_t;        // maximum logit of the iteration, over the row-selecting lane bits
            for (int off = G >> 1; off >= row_rep; off >>= 1) mi = fmaxf(mi, lane_read(lane4 ^ (off << 2), mi));
            const float mn = fmaxf(m_run, mi);
            const float sc_run = rescale(m_run, mn);
            my_g = my_ok ? expf(my_t - mn) : 0.0f;
            float ws = my_g;
            for (int off = G >> 1; off >= row_rep; off >>= 1) ws += lane_read(lane4 ^ (off << 2), ws);
            s_run = s_run * sc_run + ws;
            m_run = mn;
            if (my_ok && my_isp && my_rep) { loss_acc += my_t; ++npos; }
            if (sc_run != 1.0f) {
#pragma unroll
                for (int j = 0; j < CPL; ++j)
#pragma unroll
                    for (int e = 0; e < EPC; ++e) dz[j][e] *= sc_run;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * NG;
            const int src = grp_lane0 + lane_of_row<U>(u, G);
            const float g = lane_read(src << 2, my_g);   // zero for a masked pair
            if (FULL || ok[u]) {
                float wf[CPL][EPC];
#pragma unroll
                for (int j = 0; j < CPL; ++j) {
                    Elem<T>::unpack(rw[u][j], wf[j]);
#pragma unroll
                    for (int e = 0; e < EPC; ++e) dz[j][e] = fmaf(g, wf[j][e], dz[j][e]);
                }
                if (KIND == XC_LOSS_SOFTMAX && isp[u] && ok[u]) {
#pragma unroll
                    for (int j = 0; j < CPL; ++j)
#pragma unroll
                        for (int e = 0; e < EPC; ++e) pz[j][e] += wf[j][e];
                }
                if (FUSE) {
                    if (ok[u] && slot[u] >= 0) {           // the only pair of its label: the row is updated here
                        const float cg = -lr * g;
                        unsigned char* wrow = Wb + static_cast<int64_t>(id[u]) * row_bytes;
                        unsigned char* orow = rows_out ? reinterpret_cast<unsigned char*>(rows_out) +
                                                             static_cast<int64_t>(slot[u]) * row_bytes : nullptr;
#pragma unroll
                        for (int j = 0; j < CPL; ++j) {
                            const int ch = gl + j * G;
                            if (FULL || ch < nchunks) {
                                // (unpacked here, and hidden from the compiler's hoisting: kept unpacked for the
                                // whole loop the query row costs a wave per SIMD)
                                uint4 zc = zp[j];
                                asm volatile("" : "+v"(zc.x), "+v"(zc.y), "+v"(zc.z), "+v"(zc.w));
                                float zf[EPC];
                                Elem<T>::unpack(zc, zf);
#pragma unroll
                                for (int e = 0; e < EPC; ++e) wf[j][e] = fmaf(cg, zf[e], wf[j][e]);
                                const uint4 o = Elem<T>::pack(wf[j]);
                                store16<STREAM>(wrow + ch * 16, o);
                                if (orow) store16<STREAM>(orow + ch * 16, o);
                            }
                        }
                    }
                }
            }
            float park = g;         // soft-max: the logit is parked until the normaliser is known
            if (KIND == XC_LOSS_SOFTMAX) park = lane_read(src << 2, my_t);
            if (gl == 0 && c < n) gco[p_base + c] = park;
        }
    }
    // per-lane partial sums of the group (one lane per row adds) -> every lane of the group
    for (int off = G >> 1; off > 0; off >>= 1) loss_acc += __shfl_xor(loss_acc, off, kWave);
    if (KIND == XC_LOSS_SOFTMAX) {
        for (int off = G >> 1; off > 0; off >>= 1) npos += __shfl_xor(npos, off, kWave);
    }

    // ---- combine the groups of the workgroup -------------------------------
    float lse = 0.0f, inv_sum = 0.0f, inv_npos = 0.0f;
    int npos_all = 0;
    if (KIND == XC_LOSS_BCE) {
        if (gl == 0) part[tid / G] = loss_acc;
        __syncthreads();
        if (tid == 0) {
            float t = 0.0f;
            for (int g2 = 0; g2 < kStepThreads / G; ++g2) t += part[g2];
            loss_q[sq * B + i] = t;
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
        dZ[(sq * B + i) * d + c] = v;
    }

    if (KIND == XC_LOSS_SOFTMAX) {
        // pair coefficients now that the normaliser is known
        // (a masked pair parked -inf: its coefficient comes out 0 and its key is the masked one, so it is never used;
        // a query without a positive has all its keys masked)
        for (int c = tid; c < n; c += kStepThreads) {
            const int64_t p = p_base + c;
            if (npos_all == 0) gco[p] = 0.0f;
            else {
                const float t = gco[p];
                gco[p] = (expf(t - lse) - (c < k_p ? inv_npos : 0.0f)) * inv_B;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// stable radix sort of (key, value) pairs, at most 11 bits per digit.
// Block b owns the contiguous chunk [b*chunk, (b+1)*chunk) of the input.
//   radix_count    per-block digit histogram -> counts[digit][block]
//   radix_prefix   one wave per digit: exclusive prefix over the blocks, digit total
//   radix_scatter  digit bases by a scan of the totals inside every block, then the
//                  block walks its chunk tile by tile with running digit offsets
//   bucket_sort    one workgroup per value of the high digit: histogram, scan and stable
//                  placement by the low digit inside that bucket, no global counts
// Keys of at most 22 bits take one count/prefix/scatter round on the high digit and then
// bucket_sort (5 launches with the segment heads instead of 8); wider keys take
// least-significant-digit-first rounds of count/prefix/scatter.
// A key >= inv_key (the marker of a masked pair) is given the digit inv_digit.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int digit_of(uint32_t key, int shift, int radix, uint32_t inv_key, int inv_digit) {
    return key >= inv_key ? inv_digit : static_cast<int>((key >> shift) & static_cast<uint32_t>(radix - 1));
}

// Sum of v over a workgroup of NW waves, in a fixed order (lanes by butterfly, then waves in turn);
// every thread gets the total.  `sh` holds NW values and may be reused after the call.
template <typename V, int NW>
__device__ __forceinline__ V block_sum(V v, V* sh) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) sh[threadIdx.x / kWave] = v;
    __syncthreads();
    V t = sh[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) t += sh[w];
    __syncthreads();
    return t;
}

// Where the sort keys come from.  Pair p = i * n + c is candidate c of query i: positive c < k_p, else negative
// c - k_p.  Its key is the label id, or L (the masked key, sorted behind every label and never touched again) if
// the id is outside [0, L), if it is a negative that is one of the query's positives (the (1 - y_l) factor of
// the loss), or, for the soft-max, if the query has no valid positive at all.
struct KeySource {
    const int32_t* pos;
    const int32_t* neg;
    int k_p, n_neg, n, n_shift, softmax;
    uint32_t n_magic;
    int64_t L;
};
__device__ __forceinline__ uint32_t pair_index_to_query(uint32_t idx, uint32_t n_magic, int n_shift) {
    // exact division by n through a multiply-high (constants from the host; valid for every index below 2^31)
    if (n_shift < 0) return idx;                                   // n == 1
    const uint32_t t = __umulhi(idx, n_magic);
    return (t + ((idx - t) >> 1)) >> n_shift;
}
__device__ __forceinline__ uint32_t pair_key(const KeySource& k, uint32_t p) {
    const uint32_t i = pair_index_to_query(p, k.n_magic, k.n_shift);
    const int c = static_cast<int>(p - i * static_cast<uint32_t>(k.n));
    const int32_t* pos_i = k.pos + static_cast<int64_t>(i) * k.k_p;
    const bool isp = c < k.k_p;
    const int32_t id = isp ? pos_i[c] : k.neg[static_cast<int64_t>(i) * k.n_neg + (c - k.k_p)];
    bool ok = id >= 0 && id < k.L;
    if (!isp || k.softmax) {
        bool hit = false, any_pos = false;
        for (int q = 0; q < k.k_p; ++q) {
            const int32_t pq = pos_i[q];
            hit = hit || pq == id;
            any_pos = any_pos || (pq >= 0 && pq < k.L);
        }
        if (!isp && hit) ok = false;
        if (k.softmax && !any_pos) ok = false;
    }
    return ok ? static_cast<uint32_t>(id) : static_cast<uint32_t>(k.L);
}

// MAKE: this is the first kernel of the step; it forms the (key, pair index) pairs, writes them to `pairs_out`
// and counts their digits.  Otherwise the pairs are read.
template <bool MAKE>
__global__ __launch_bounds__(256)
void radix_count_kernel(const uint2* __restrict__ pairs, int64_t P, int64_t chunk, int shift, int rb,
                        int nb, int* __restrict__ counts /* [radix][nb] */, uint32_t inv_key, int inv_digit,
                        const KeySource ks, uint2* __restrict__ pairs_out, int32_t* __restrict__ stats) {
    __shared__ int hist[kMaxRadix];
    const int radix = 1 << rb;
    for (int d = threadIdx.x; d < radix; d += 256) hist[d] = 0;
    if (MAKE && blockIdx.x == 0 && threadIdx.x == 0) stats[0] = 0;      // rows updated inside the gather: counted later
    __syncthreads();
    const int64_t p0 = blockIdx.x * chunk;
    int64_t p1 = p0 + chunk;
    p1 = p1 < P ? p1 : P;
    for (int64_t p = p0 + threadIdx.x; p < p1; p += 256) {
        uint32_t key;
        if (MAKE) {
            key = pair_key(ks, static_cast<uint32_t>(p));
            pairs_out[p] = make_uint2(key, static_cast<uint32_t>(p));
        } else {
            key = pairs[p].x;
        }
        atomicAdd(&hist[digit_of(key, shift, radix, inv_key, inv_digit)], 1);
    }
    __syncthreads();
    for (int d = threadIdx.x; d < radix; d += 256) counts[d * nb + blockIdx.x] = hist[d];
}

__global__ __launch_bounds__(kWave)
void radix_prefix_kernel(int* __restrict__ counts /* [radix][nb], in place */, int nb,
                         int* __restrict__ totals /* [radix] */) {
    int* row = counts + static_cast<size_t>(blockIdx.x) * nb;
    const int lane = threadIdx.x;
    int run = 0;
    for (int b0 = 0; b0 < nb; b0 += kWave) {
        const int b = b0 + lane;
        const int v = b < nb ? row[b] : 0;
        const int incl = wave_incl_scan(v);
        if (b < nb) row[b] = run + incl - v;
        run += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) totals[blockIdx.x] = run;
}

// One tile of kSortTile keys: key/val of thread tid (valid or not) goes to offs[digit] + its rank among
// the tile's keys of the same digit, and offs moves on.  whist must be zero on entry and is zero on exit.
__device__ __forceinline__ void place_tile(bool valid, uint32_t key, uint32_t val, int digit, int rb,
                                           int* offs /* [radix] */, int* whist /* [waves][radix] */,
                                           uint2* __restrict__ out) {
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int radix = 1 << rb;
    // lanes of this wave holding the same digit
    uint64_t same = __ballot(valid);
    for (int b = 0; b < rb; ++b) {
        const bool bit = (digit >> b) & 1;
        const uint64_t bal = __ballot(bit);
        same &= bit ? bal : ~bal;
    }
    const int rank = __popcll(same & lanemask_lt());
    if (valid && rank == 0) whist[wave * radix + digit] = __popcll(same);
    lds_barrier();
    if (valid) {
        int before = offs[digit];
        for (int w = 0; w < wave; ++w) before += whist[w * radix + digit];
        out[before + rank] = make_uint2(key, val);       // one 8-byte store: key and payload share a line
    }
    lds_barrier();
    // only digits present in this tile need their running offset advanced
    if (valid && rank == 0) {
        int add = 0;
#pragma unroll
        for (int w = 0; w < kSortTile / kWave; ++w) add += whist[w * radix + digit];
        // one lane per (wave, digit); the wave holding the lowest index among the waves
        // that saw the digit applies the update
        bool first = true;
        for (int w = 0; w < wave; ++w) first = first && whist[w * radix + digit] == 0;
        if (first) offs[digit] += add;
    }
    lds_barrier();
    if (valid && rank == 0) whist[wave * radix + digit] = 0;
    lds_barrier();
}

__global__ __launch_bounds__(kSortTile)
void radix_scatter_kernel(const uint2* __restrict__ in, uint2* __restrict__ out, int64_t P,
                          int64_t chunk, int shift, int rb, int nb, const int* __restrict__ prefix,
                          const int* __restrict__ totals, uint32_t inv_key, int inv_digit,
                          int* __restrict__ bases_out /* [radix] or null: where each digit's pairs start */) {
    extern __shared__ int sort_lds[];                  // offs[radix], whist[waves][radix]: sized by the launch
    __shared__ int wsum[kSortTile / kWave];
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int radix = 1 << rb;
    int* offs = sort_lds;
    int* whist = sort_lds + radix;
    const int per = (radix + kSortTile - 1) / kSortTile;     // digits per thread, contiguous
    // digit bases: exclusive scan of the totals
    {
        int local = 0;
        for (int j = 0; j < per; ++j) { const int d = tid * per + j; if (d < radix) local += totals[d]; }
        const int incl = wave_incl_scan(local);
        if ((tid & 63) == 63) wsum[wave] = incl;
        __syncthreads();
        int run = incl - local;
        for (int w = 0; w < wave; ++w) run += wsum[w];
        for (int j = 0; j < per; ++j) {
            const int d = tid * per + j;
            if (d < radix) {
                if (bases_out != nullptr && blockIdx.x == 0) bases_out[d] = run;
                offs[d] = run + prefix[d * nb + blockIdx.x];
                run += totals[d];
            }
        }
    }
    for (int d = tid; d < radix; d += kSortTile)
#pragma unroll
        for (int w = 0; w < kSortTile / kWave; ++w) whist[w * radix + d] = 0;
    __syncthreads();
    const int64_t p0 = blockIdx.x * chunk;
    int64_t p1 = p0 + chunk;
    p1 = p1 < P ? p1 : P;
    // the next tile's pairs are fetched while the current tile is placed
    uint32_t key_n = 0, val_n = 0;
    if (p0 + tid < p1) { const uint2 kv = in[p0 + tid]; key_n = kv.x; val_n = kv.y; }
    for (int64_t t0 = p0; t0 < p1; t0 += kSortTile) {
        const bool valid = t0 + tid < p1;
        const uint32_t key = key_n, val = val_n;
        const int64_t pn = t0 + kSortTile + tid;
        if (pn < p1) { const uint2 kv = in[pn]; key_n = kv.x; val_n = kv.y; }
        place_tile(valid, key, val, digit_of(key, shift, radix, inv_key, inv_digit), rb, offs, whist, out);
    }
}

// All pairs whose key has high digit blockIdx.x (they are contiguous after the scatter on that digit,
// in their original order): stable placement by the low `rb` bits.  A bucket of up to
// kBucketRegTiles tiles is read once and kept in registers.  Every non-empty bin is one label, so
// the number of segment heads of the bucket falls out of the histogram.
constexpr int kBucketRegTiles = 8;
#ifndef XC_BUCKET_TARGET
#define XC_BUCKET_TARGET 512
#endif
constexpr int64_t kBucketTarget = XC_BUCKET_TARGET;   // pairs per bucket the digit split aims at

__global__ __launch_bounds__(kSortTile)
void bucket_sort_kernel(const uint2* __restrict__ in, uint2* __restrict__ out,
                        const int* __restrict__ sizes /* [gridDim.x] pairs per bucket */,
                        const int* __restrict__ bases /* [gridDim.x] first pair of each bucket */, int rb,
                        int* __restrict__ head_cnt /* [gridDim.x] */,
                        int* __restrict__ multi_cnt /* [gridDim.x] labels of the bucket with several pairs */) {
    extern __shared__ int sort_lds[];                  // offs[radix], whist[waves][radix]: sized by the launch
    __shared__ int wsum[kSortTile / kWave];
    __shared__ int red[kSortTile / kWave];
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int radix = 1 << rb;
    int* offs = sort_lds;
    int* whist = sort_lds + radix;
    const int b = blockIdx.x;
    const int p0 = bases[b];
    const int p1 = p0 + sizes[b];
    for (int d = tid; d < radix; d += kSortTile) {
        offs[d] = 0;
#pragma unroll
        for (int w = 0; w < kSortTile / kWave; ++w) whist[w * radix + d] = 0;
    }
    __syncthreads();
    const bool in_regs = p1 - p0 <= kBucketRegTiles * kSortTile;        // uniform
    uint32_t rk[kBucketRegTiles], rv[kBucketRegTiles];
    if (in_regs) {
#pragma unroll
        for (int u = 0; u < kBucketRegTiles; ++u) {
            const int p = p0 + u * kSortTile + tid;
            rk[u] = 0; rv[u] = 0;
            if (p < p1) { const uint2 kv = in[p]; rk[u] = kv.x; rv[u] = kv.y; }
        }
#pragma unroll
        for (int u = 0; u < kBucketRegTiles; ++u)
            if (p0 + u * kSortTile + tid < p1) atomicAdd(&offs[rk[u] & static_cast<uint32_t>(radix - 1)], 1);
    } else {
        for (int p = p0 + tid; p < p1; p += kSortTile) atomicAdd(&offs[in[p].x & static_cast<uint32_t>(radix - 1)], 1);
    }
    __syncthreads();
    {   // bins -> start positions (exclusive scan, contiguous bins per thread); heads = non-empty bins
        const int per = (radix + kSortTile - 1) / kSortTile;        // <= 8
        int cnt[kMaxRadix / kSortTile];
        int local = 0, nz = 0, nz2 = 0;
        for (int j = 0; j < per; ++j) {
            const int d = tid * per + j;
            const int c = d < radix ? offs[d] : 0;
            cnt[j] = c; local += c; nz += c > 0 ? 1 : 0; nz2 += c > 1 ? 1 : 0;
        }
        const int incl = wave_incl_scan(local);
        if ((tid & 63) == 63) wsum[wave] = incl;
        __syncthreads();
        int run = p0 + incl - local;
        for (int w = 0; w < wave; ++w) run += wsum[w];
        for (int j = 0; j < per; ++j) {
            const int d = tid * per + j;
            if (d < radix) { offs[d] = run; run += cnt[j]; }
        }
        const int heads = block_sum<int, kSortTile / kWave>(nz, red);
        const int multis = block_sum<int, kSortTile / kWave>(nz2, red);
        if (tid == 0) { head_cnt[b] = heads; multi_cnt[b] = multis; }
    }
    if (in_regs) {
#pragma unroll
        for (int u = 0; u < kBucketRegTiles; ++u) {
            if (p0 + u * kSortTile >= p1) break;                       // uniform
            const bool valid = p0 + u * kSortTile + tid < p1;
            place_tile(valid, rk[u], rv[u], static_cast<int>(rk[u] & static_cast<uint32_t>(radix - 1)), rb, offs, whist,
                       out);
        }
    } else {
        uint32_t key_n = 0, val_n = 0;
        if (p0 + tid < p1) { const uint2 kv = in[p0 + tid]; key_n = kv.x; val_n = kv.y; }
        for (int t0 = p0; t0 < p1; t0 += kSortTile) {
            const bool valid = t0 + tid < p1;
            const uint32_t key = key_n, val = val_n;
            const int pn = t0 + kSortTile + tid;
            if (pn < p1) { const uint2 kv = in[pn]; key_n = kv.x; val_n = kv.y; }
            place_tile(valid, key, val, static_cast<int>(key & static_cast<uint32_t>(radix - 1)), rb, offs, whist,
                       out);
        }
    }
}

// ---------------------------------------------------------------------------
// segment heads of the sorted keys -> touched list and segment starts
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool is_head(const uint2* pairs, int64_t p, uint32_t Lkey) {
    const uint32_t k = pairs[p].x;
    return k < Lkey && (p == 0 || pairs[p - 1].x != k);
}

__global__ __launch_bounds__(256)
void heads_count_kernel(const uint2* __restrict__ pairs, int64_t P, int64_t chunk, uint32_t Lkey,
                        int* __restrict__ head_cnt, int* __restrict__ valid_cnt, int* __restrict__ multi_cnt) {
    __shared__ int sh[4];
    const int64_t p0 = blockIdx.x * chunk;
    int64_t p1 = p0 + chunk;
    p1 = p1 < P ? p1 : P;
    int h = 0, v = 0, m = 0;
    for (int64_t p = p0 + threadIdx.x; p < p1; p += 256) {
        const bool head = is_head(pairs, p, Lkey);
        h += head ? 1 : 0;
        m += (head && p + 1 < P && pairs[p + 1].x == pairs[p].x) ? 1 : 0;      // a label with several pairs
        v += pairs[p].x < Lkey ? 1 : 0;
    }
    h = block_sum<int, 4>(h, sh);
    v = block_sum<int, 4>(v, sh);
    m = block_sum<int, 4>(m, sh);
    if (threadIdx.x == 0) { head_cnt[blockIdx.x] = h; valid_cnt[blockIdx.x] = v; multi_cnt[blockIdx.x] = m; }
}

__global__ __launch_bounds__(256)
void heads_write_kernel(const uint2* __restrict__ pairs, int64_t P, int64_t chunk, uint32_t Lkey,
                        int nb, const int* __restrict__ head_cnt, const int* __restrict__ valid_cnt,
                        int32_t* __restrict__ touched,
                        int32_t* __restrict__ seg_start, uint32_t* __restrict__ seg_idx0,
                        int32_t* __restrict__ n_touched,
                        const int* __restrict__ bucket_sizes /* not null: block b covers bucket b ... */,
                        const int* __restrict__ bucket_bases /* ... which starts at pair bucket_bases[b] */,
                        int32_t* __restrict__ single_slot /* [P] by pair index, or null */,
                        const int* __restrict__ multi_cnt, int32_t* __restrict__ multi_list /* segments with several pairs */,
                        int32_t* __restrict__ stats) {
    __shared__ int sh[4];
    __shared__ int wcnt[4], wcnt_m[4];
    __shared__ int running, running_m;
    const int tid = threadIdx.x;
    if (static_cast<int>(blockIdx.x) == nb) {
        // one workgroup beyond those of the keys: the totals, off the other workgroups' path
        int th = 0, tv = 0, tm = 0;
        for (int b = tid; b < nb; b += 256) { th += head_cnt[b]; tv += valid_cnt[b]; tm += multi_cnt[b]; }
        th = block_sum<int, 4>(th, sh);
        tv = block_sum<int, 4>(tv, sh);
        tm = block_sum<int, 4>(tm, sh);
        if (tid == 0) { n_touched[0] = th; seg_start[th] = tv; stats[1] = tm; }
        return;
    }
    int bucket_p0 = 0, bucket_n = 0;
    if (bucket_sizes) { bucket_p0 = bucket_bases[blockIdx.x]; bucket_n = bucket_sizes[blockIdx.x]; }
    // heads in the blocks before this one
    int t = 0, tm = 0;
    for (int b = tid; b < static_cast<int>(blockIdx.x); b += 256) { t += head_cnt[b]; tm += multi_cnt[b]; }
    t = block_sum<int, 4>(t, sh);
    tm = block_sum<int, 4>(tm, sh);
    if (tid == 0) { running = t; running_m = tm; }
    __syncthreads();
    int64_t p0 = blockIdx.x * chunk;
    int64_t p1 = p0 + chunk;
    if (bucket_sizes) { p0 = bucket_p0; p1 = p0 + bucket_n; }
    p1 = p1 < P ? p1 : P;
    int singles = 0;
    for (int64_t t0 = p0; t0 < p1; t0 += 256) {
        const int64_t p = t0 + tid;
        const bool head = p < p1 && is_head(pairs, p, Lkey);
        uint2 kv = make_uint2(0u, 0u);
        if (p < p1) kv = pairs[p];
        const bool single = head && (p + 1 >= P || pairs[p + 1].x != kv.x);
        const uint64_t bal = __ballot(head);
        const uint64_t bal_m = __ballot(head && !single);
        if ((tid & 63) == 0) { wcnt[tid >> 6] = __popcll(bal); wcnt_m[tid >> 6] = __popcll(bal_m); }
        lds_barrier();
        int before = running, before_m = running_m;
        for (int w = 0; w < (tid >> 6); ++w) { before += wcnt[w]; before_m += wcnt_m[w]; }
        if (p < p1) {
            const int s = before + __popcll(bal & lanemask_lt());
            if (head) {
                touched[s] = static_cast<int32_t>(kv.x);
                seg_start[s] = static_cast<int32_t>(p);
                seg_idx0[s] = kv.y;                  // first pair of the segment, saves the update a hop
            }
            if (single_slot != nullptr) {
                // a label with one pair only: the gather updates its row itself and needs the row's place in the
                // touched list (for the copy of the updated rows); every other pair is told -1.  The other
                // labels are listed for the row update kernel.
                single_slot[kv.y] = single ? s : -1;
                singles += single ? 1 : 0;
                if (head && !single) multi_list[before_m + __popcll(bal_m & lanemask_lt())] = s;
            }
        }
        lds_barrier();
        if (tid == 0) {
            running += wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
            running_m += wcnt_m[0] + wcnt_m[1] + wcnt_m[2] + wcnt_m[3];
        }
        lds_barrier();
    }
    if (single_slot != nullptr) {
        singles = block_sum<int, 4>(singles, sh);
        if (tid == 0 && singles > 0) atomicAdd(&stats[0], singles);      // an integer sum: the same in every run
    }
}

// ---------------------------------------------------------------------------
// per touched label: dW = sum over its pairs of g * z_i ; w <- w - lr * dW
// One group of G lanes per segment, chunks distributed as in gather_kernel.  A label shared by
// more than kLongSeg pairs (a frequent positive, a hard negative of many queries) would make
// its group the last to finish: such segments are queued and afterwards worked on by the whole
// workgroup, group g taking pairs g, g + NG, ... and the partial sums added in group order.
// Which segments are queued depends on the data alone (every group queues the first
// kLongPerGroup long segments it meets, in its own fixed order), never on timing, so the order
// in which a row's terms are added is the same in every run.
// ---------------------------------------------------------------------------
constexpr int kLongSeg = 16;        // pairs above which a segment is shared by the workgroup
constexpr int kLongPerGroup = 8;    // long segments a group may queue (its first ones; later ones are done in place)
constexpr int kMaxGroups = kStepThreads / 16;      // groups of a workgroup at most (G >= 16)

template <typename T, int CPL, bool STREAM>
__global__ __launch_bounds__(kStepThreads)
void update_kernel(const T* __restrict__ Z, T* __restrict__ W, int d, uint32_t n_magic, int n_shift, int G,
                   const uint2* __restrict__ pairs, const float* __restrict__ gco,
                   const int32_t* __restrict__ touched, const int32_t* __restrict__ seg_start,
                   const uint32_t* __restrict__ seg_idx0, const int32_t* __restrict__ n_touched, float lr,
                   T* __restrict__ rows_out,
                   const float* __restrict__ dz_part, int SQ, int64_t BD, float* __restrict__ dZ,
                   const int32_t* __restrict__ multi_list /* not null: labels with one pair were updated by the gather,
                                                             these are the segments left, n_multi[0] of them */,
                   const int32_t* __restrict__ n_multi,
                   const float* __restrict__ loss_q, int64_t n_loss, float inv_B, float* __restrict__ loss) {
    constexpr int EPC = Elem<T>::kPerChunk;
    constexpr int U = 2;
    extern __shared__ float lpart[];              // [NG][CPL][G][EPC] partial sums of a long segment
    __shared__ int long_q[kMaxGroups * kLongPerGroup];   // [group][slot]
    __shared__ int long_n[kMaxGroups];                    // slots filled by each group
    const int tid = threadIdx.x;
    if (blockIdx.x == gridDim.x - 1) {
        // one workgroup beyond those of the rows: loss = (1/B) sum of the gather's partial losses, in a fixed order
        __shared__ float shf[kStepThreads / kWave];
        float t2 = 0.0f;
        for (int64_t i = tid; i < n_loss; i += kStepThreads) t2 += loss_q[i];
        t2 = block_sum<float, kStepThreads / kWave>(t2, shf);
        if (tid == 0) loss[0] = t2 * inv_B;
        return;
    }
    const int n_wg = gridDim.x - 1;                       // workgroups that share the rows
    int my_long = 0;                                      // uniform within the group
    // dZ = sum of the partials written by the workgroups that shared a query, in split order
    // (independent of the row updates below; done here because this grid is large)
    if (SQ > 1) {
        for (int64_t e = static_cast<int64_t>(blockIdx.x) * kStepThreads + tid; e < BD;
             e += static_cast<int64_t>(n_wg) * kStepThreads) {
            float v = dz_part[e];
            for (int q = 1; q < SQ; ++q) v += dz_part[q * BD + e];
            dZ[e] = v;
        }
    }
    const int gl = tid & (G - 1);
    const int NG = kStepThreads / G;
    const int nchunks = d / EPC;
    const int64_t row_bytes = static_cast<int64_t>(d) * sizeof(T);
    const unsigned char* Zb = reinterpret_cast<const unsigned char*>(Z);
    const int64_t n_seg = multi_list != nullptr ? n_multi[0] : n_touched[0];
    // pair index -> query row: exact division by n through a multiply-high (n_magic, n_shift
    // from the host; valid for every index below 2^31)
    auto query_of = [&](uint32_t idx) -> int64_t {
        if (n_shift < 0) return static_cast<int64_t>(idx);           // n == 1
        const uint32_t t = __umulhi(idx, n_magic);
        return static_cast<int64_t>((t + ((idx - t) >> 1)) >> n_shift);
    };
    // A group walks several segments so that waves live long enough to keep the chip full.  The
    // loads run ahead of the arithmetic: hop 1 (what identifies a segment) two segments ahead,
    // hop 2 (the row of W, the coefficient and the query row of the first pair) one ahead.
    struct Hop1 { int p0, p1, label, seg; uint32_t idx0; };
    auto load_hop1 = [&](int64_t sl, Hop1& h) {
        const int64_t sx = multi_list != nullptr ? multi_list[sl] : sl;      // position in the touched list
        h.seg = static_cast<int>(sx);
        h.p0 = seg_start[sx]; h.p1 = seg_start[sx + 1]; h.label = touched[sx]; h.idx0 = seg_idx0[sx];
    };
    auto load_hop2 = [&](const Hop1& h, uint4 (&wv)[CPL], uint4 (&z0)[CPL], float& g0) {
        const unsigned char* wr = reinterpret_cast<const unsigned char*>(W) + static_cast<int64_t>(h.label) * row_bytes;
        g0 = gco[h.idx0];
        const int64_t qi = query_of(h.idx0);
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int ch = gl + j * G;
            wv[j] = make_uint4(0, 0, 0, 0);
            z0[j] = make_uint4(0, 0, 0, 0);
            if (ch < nchunks) {
                wv[j] = load16<STREAM>(wr + ch * 16);
                z0[j] = *reinterpret_cast<const uint4*>(Zb + qi * row_bytes + ch * 16);
            }
        }
    };
    const int64_t s_step = static_cast<int64_t>(n_wg) * NG;
    int64_t s = static_cast<int64_t>(blockIdx.x) * NG + tid / G;
    Hop1 h_n = {0, 0, 0, 0, 0u}, h_nn = {0, 0, 0, 0, 0u};
    uint4 wv_n[CPL], z0_n[CPL];
    float g0_n = 0.0f;
#pragma unroll
    for (int j = 0; j < CPL; ++j) { wv_n[j] = make_uint4(0, 0, 0, 0); z0_n[j] = make_uint4(0, 0, 0, 0); }
    if (s < n_seg) { load_hop1(s, h_n); load_hop2(h_n, wv_n, z0_n, g0_n); }
    if (s + s_step < n_seg) load_hop1(s + s_step, h_nn);
    for (; s < n_seg; s += s_step) {
    const int p0 = h_n.p0, p1 = h_n.p1;
    const int64_t label = h_n.label;
    const float g0 = g0_n;
    uint4 wv[CPL], z0[CPL];
#pragma unroll
    for (int j = 0; j < CPL; ++j) { wv[j] = wv_n[j]; z0[j] = z0_n[j]; }
    const int64_t s_cur = h_n.seg;                // position in the touched list
    if (s + s_step < n_seg) { h_n = h_nn; load_hop2(h_n, wv_n, z0_n, g0_n); }
    if (s + 2 * s_step < n_seg) load_hop1(s + 2 * s_step, h_nn);
    if (p1 - p0 > kLongSeg && my_long < kLongPerGroup) {        // uniform within the group
        if (gl == 0) long_q[(tid / G) * kLongPerGroup + my_long] = static_cast<int>(s_cur);
        ++my_long;
        continue;
    }
    unsigned char* wrow = reinterpret_cast<unsigned char*>(W) + label * row_bytes;

    float acc[CPL][EPC];
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
        float zf[EPC];
        Elem<T>::unpack(z0[j], zf);
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[j][e] = g0 * zf[e];
    }

    // further pairs of the same label, in sorted (= original) order.  A round first fetches the
    // pair index, coefficient and query row of up to G pairs, one per lane of the group, so that a
    // long segment (a label many queries share) pays the two dependent index loads once per G
    // pairs; the rows then follow U at a time.
    for (int pb = p0 + 1; pb < p1; pb += G) {
        const int nb = (p1 - pb) < G ? (p1 - pb) : G;
        float my_g = 0.0f;
        int64_t my_q = 0;
        if (gl < nb) {
            const uint32_t idx = pairs[pb + gl].y;
            my_g = gco[idx];
            my_q = query_of(idx);
        }
        for (int u0 = 0; u0 < nb; u0 += U) {
            float g[U];
            uint4 rz[U][CPL];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                g[u] = __shfl(my_g, u0 + u, G);          // lanes past nb hold 0 and row 0: harmless
                const int64_t qi = __shfl(my_q, u0 + u, G);
#pragma unroll
                for (int j = 0; j < CPL; ++j) {
                    const int ch = gl + j * G;
                    rz[u][j] = make_uint4(0, 0, 0, 0);
                    if (ch < nchunks && u0 + u < nb)
                        rz[u][j] = *reinterpret_cast<const uint4*>(Zb + qi * row_bytes + ch * 16);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (u0 + u < nb) {
#pragma unroll
                    for (int j = 0; j < CPL; ++j) {
                        float zf[EPC];
                        Elem<T>::unpack(rz[u][j], zf);
#pragma unroll
                        for (int e = 0; e < EPC; ++e) acc[j][e] = fmaf(g[u], zf[e], acc[j][e]);
                    }
                }
            }
        }
    }
    unsigned char* orow = rows_out ? reinterpret_cast<unsigned char*>(rows_out) + s_cur * row_bytes : nullptr;
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
        const int ch = gl + j * G;
        if (ch < nchunks) {
            float wf[EPC];
            Elem<T>::unpack(wv[j], wf);
#pragma unroll
            for (int e = 0; e < EPC; ++e) wf[e] = fmaf(-lr, acc[j][e], wf[e]);
            const uint4 o = Elem<T>::pack(wf);
            store16<STREAM>(wrow + ch * 16, o);
            if (orow) store16<STREAM>(orow + ch * 16, o);
        }
    }
    }   // segments of this group

    // ---- queued long segments: the whole workgroup on each, in (group, slot) order
    const int grp = tid / G;
    if (gl == 0) long_n[grp] = my_long;
    __syncthreads();
    int li = -1;
    for (int qg = 0; qg < NG; ++qg)
    for (int qs = 0; qs < long_n[qg]; ++qs) {
        ++li;
        const int64_t sl = long_q[qg * kLongPerGroup + qs];
        const int p0 = seg_start[sl], p1 = seg_start[sl + 1];
        const int64_t label = touched[sl];
        float acc[CPL][EPC];
#pragma unroll
        for (int j = 0; j < CPL; ++j)
#pragma unroll
            for (int e = 0; e < EPC; ++e) acc[j][e] = 0.0f;
        // this group's pairs are p0 + grp + NG * m; a round fetches the metadata of G of them
        for (int m0 = 0; p0 + grp + NG * m0 < p1; m0 += G) {
            const int pm = p0 + grp + NG * (m0 + gl);
            float my_g = 0.0f;
            int64_t my_q = 0;
            if (pm < p1) {
                const uint32_t idx = pairs[pm].y;
                my_g = gco[idx];
                my_q = query_of(idx);
            }
            const int left = (p1 - (p0 + grp + NG * m0) + NG - 1) / NG;      // pairs of this group from m0 on
            const int nb = left < G ? left : G;
            for (int u0 = 0; u0 < nb; u0 += U) {
                float g[U];
                uint4 rz[U][CPL];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    g[u] = __shfl(my_g, u0 + u, G);
                    const int64_t qi = __shfl(my_q, u0 + u, G);
#pragma unroll
                    for (int j = 0; j < CPL; ++j) {
                        const int ch = gl + j * G;
                        rz[u][j] = make_uint4(0, 0, 0, 0);
                        if (ch < nchunks && u0 + u < nb)
                            rz[u][j] = *reinterpret_cast<const uint4*>(Zb + qi * row_bytes + ch * 16);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (u0 + u < nb) {
#pragma unroll
                        for (int j = 0; j < CPL; ++j) {
                            float zf[EPC];
                            Elem<T>::unpack(rz[u][j], zf);
#pragma unroll
                            for (int e = 0; e < EPC; ++e) acc[j][e] = fmaf(g[u], zf[e], acc[j][e]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < CPL; ++j)
#pragma unroll
            for (int e = 0; e < EPC; ++e) lpart[((grp * CPL + j) * G + gl) * EPC + e] = acc[j][e];
        __syncthreads();
        if (grp == li % NG) {                      // one group adds the partial sums in group order
            unsigned char* wrow = reinterpret_cast<unsigned char*>(W) + label * row_bytes;
            unsigned char* orow = rows_out ? reinterpret_cast<unsigned char*>(rows_out) + sl * row_bytes : nullptr;
#pragma unroll
            for (int j = 0; j < CPL; ++j) {
                const int ch = gl + j * G;
                if (ch < nchunks) {
                    const uint4 wv = load16<STREAM>(wrow + ch * 16);
                    float tot[EPC];
#pragma unroll
                    for (int e = 0; e < EPC; ++e) tot[e] = lpart[((0 * CPL + j) * G + gl) * EPC + e];
                    for (int g2 = 1; g2 < NG; ++g2)
#pragma unroll
                        for (int e = 0; e < EPC; ++e) tot[e] += lpart[((g2 * CPL + j) * G + gl) * EPC + e];
                    float wf[EPC];
                    Elem<T>::unpack(wv, wf);
#pragma unroll
                    for (int e = 0; e < EPC; ++e) wf[e] = fmaf(-lr, tot[e], wf[e]);
                    const uint4 o = Elem<T>::pack(wf);
                    store16<STREAM>(wrow + ch * 16, o);
                    if (orow) store16<STREAM>(orow + ch * 16, o);
                }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static size_t sort_lds_bytes(int rb) {      // offs + one histogram per wave, for digits of rb bits
    return (static_cast<size_t>(1) + kSortTile / kWave) * (static_cast<size_t>(1) << rb) * sizeof(int);
}
struct StepPlan {
    int64_t P;
    int n, G, cpl, nb, passes, rb, key_bits, sq, n_shift;
    int low_bits, n_buckets, high_rb;       // n_buckets > 0: one round on the high digit, then bucket_sort
    bool stream_update, stream_gather;      // rows of W go through the caches with the non-temporal hint
    uint32_t n_magic;
    int64_t chunk;
    size_t off_stats, off_single, off_multi, off_multicnt, off_pairs0, off_pairs1, off_g, off_lossq, off_dzpart, off_counts, off_totals, off_bases, off_headcnt,
        off_validcnt, off_segstart, off_segidx0, total;
};

static int plan_step(int64_t B, int64_t L, int d, int k_p, int n_neg, xc_dtype t, StepPlan* p) {
    if (t != XC_F32 && t != XC_BF16) return XC_EDTYPE;
    if (B < 1 || d < 1 || k_p < 0 || k_p > XC_MAX_KP || n_neg < 0) return XC_ESHAPE;
    const int64_t n = static_cast<int64_t>(k_p) + n_neg;
    if (n < 1 || n > XC_MAX_CANDIDATES) return XC_ESHAPE;
    const int64_t row_bytes = static_cast<int64_t>(d) * (t == XC_F32 ? 4 : 2);
    if (row_bytes % 16 != 0 || row_bytes > XC_MAX_ROW_BYTES) return XC_ESHAPE;
    if (B * n >= 0x7fffffffLL) return XC_ESHAPE;
    p->P = B * n;
    // A matrix that fits the 256 MB last-level cache is found there again by the update after the gather and
    // by the next step, so its rows are loaded and stored plainly.  A larger one is streamed by the update
    // (every touched row is read and written once, and the query rows it reads many times stay cached), and,
    // from about six times that size, where a gathered row is unlikely to be found again, by the gather too.
    {
        const int64_t w_bytes = L * row_bytes;
        p->stream_update = w_bytes > (static_cast<int64_t>(256) << 20);
        p->stream_gather = w_bytes > (static_cast<int64_t>(1536) << 20);
    }
    p->n = static_cast<int>(n);
    {   // floor(x / n) = (t + ((x - t) >> 1)) >> n_shift with t = mulhi(x, n_magic), for all 32-bit x
        int sh = 0;
        while ((static_cast<int64_t>(1) << sh) < n) ++sh;
        p->n_magic = static_cast<uint32_t>(((static_cast<uint64_t>(1) << 32) * ((static_cast<uint64_t>(1) << sh) - static_cast<uint64_t>(n))) / static_cast<uint64_t>(n) + 1);
        p->n_shift = sh > 0 ? sh - 1 : 0;
        if (n == 1) { p->n_magic = 0; p->n_shift = -1; }      // identity
    }
    const int nchunks = static_cast<int>(row_bytes / 16);
    int G = 16;
    while (G < 64 && G * 4 < nchunks) G <<= 1;     // at most 4 chunks per lane
    if (G < 64 && nchunks % G != 0 && nchunks > G) { /* tail chunks are predicated */ }
    p->G = G;
    p->cpl = (nchunks + G - 1) / G;
    if (p->cpl > 4) return XC_ESHAPE;
    int bits = 1;
    if (L >= 0) { while ((static_cast<int64_t>(1) << bits) <= L && bits < 32) ++bits; }
    p->key_bits = bits;                                // keys take values 0..L
    p->passes = (bits + kMaxRadixBits - 1) / kMaxRadixBits;
    p->rb = (bits + p->passes - 1) / p->passes;          // digit width, <= 11 bits
    // Keys of up to 22 bits: split so that a bucket of the high digit holds about kBucketTarget pairs (the pairs
    // spread over the labels), within what the kernels hold: low digit <= 11 bits, and the high digit,
    // with one more value for the masked pairs, < 2^11.
    p->n_buckets = 0; p->low_bits = 0; p->high_rb = 0;
    if (L >= 2 && bits <= 2 * kMaxRadixBits) {
        int low = 1;
        while (low < kMaxRadixBits && (L >> low) * kBucketTarget > p->P) ++low;
        while (low < kMaxRadixBits && ((L - 1) >> low) + 2 > kMaxRadix - 1) ++low;
        const int64_t nbk = ((L - 1) >> low) + 1;
        if (nbk + 1 <= kMaxRadix - 1) {
            p->low_bits = low;
            p->n_buckets = static_cast<int>(nbk);
            int hb = 1;
            while ((static_cast<int64_t>(1) << hb) <= nbk) ++hb;       // digits 0..nbk fit
            p->high_rb = hb;
        }
    }
    // blocks of the sort: two 256-key tiles per block at least; the [digit][block] count matrix, which is
    // written and read across its rows, stays within kSortCountEntries
    const int radix_max = 1 << (p->n_buckets > 0 ? p->high_rb : p->rb);
    int nb_cap = kSortCountEntries / radix_max;
    if (nb_cap > kSortMaxBlocks) nb_cap = kSortMaxBlocks;
    int nb = static_cast<int>((p->P + 511) / 512);
    if (nb > nb_cap) nb = nb_cap;
    if (nb < 1) nb = 1;
    int64_t chunk = (p->P + nb - 1) / nb;
    chunk = (chunk + kSortTile - 1) / kSortTile * kSortTile;
    nb = static_cast<int>((p->P + chunk - 1) / chunk);
    p->nb = nb;
    p->chunk = chunk;
    size_t off = 0;
    auto take = [&off](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
    const size_t P = static_cast<size_t>(p->P);
    p->off_stats = take(256);                  // word 0: rows updated inside the gather (labels with one pair)
    p->off_pairs0 = take(P * 8); p->off_pairs1 = take(P * 8);
    p->off_g = take(P * 4);
    // few queries: several workgroups share a query so that the chip is filled
    p->sq = B >= 1536 ? 1 : (B >= 768 ? 2 : 4);
    p->off_lossq = take(static_cast<size_t>(B) * p->sq * 4);
    p->off_dzpart = take(p->sq > 1 ? static_cast<size_t>(B) * p->sq * d * 4 : 0);
    p->off_counts = take(static_cast<size_t>(kSortCountEntries) * 4);      // whatever L: the layout does not depend on it
    p->off_totals = take(static_cast<size_t>(kMaxRadix) * 4);
    p->off_bases = take(static_cast<size_t>(kMaxRadix) * 4);
    p->off_headcnt = take(static_cast<size_t>(kSortMaxBlocks > kMaxRadix ? kSortMaxBlocks : kMaxRadix) * 4);
    p->off_validcnt = take(static_cast<size_t>(kSortMaxBlocks) * 4);
    p->off_segstart = take((P + 1) * 4);
    p->off_segidx0 = take(P * 4);
    p->off_single = take(P * 4);
    p->off_multi = take(P * 4);
    p->off_multicnt = take(static_cast<size_t>(kSortMaxBlocks > kMaxRadix ? kSortMaxBlocks : kMaxRadix) * 4);
    p->total = off;
    return XC_OK;
}

template <typename T, int KIND>
static void launch_gather(const StepPlan& pl, hipStream_t st, const void* Z, void* W, int64_t B,
                          int64_t L, int d, const int32_t* pos, int k_p, const int32_t* neg,
                          const float* logq, int n_neg, const int32_t* single_slot /* null: no row updates here */,
                          float lr, void* rows_out, float* gco, float* loss_q, float* dZ, int SQ) {
    const float inv_B = 1.0f / static_cast<float>(B);
    const dim3 grid(static_cast<unsigned>(B * SQ));
    // (the soft-max coefficient needs the whole query first: no fused row updates there)
    const bool fuse = KIND == XC_LOSS_BCE && single_slot != nullptr;
#define XC_GATHER3(CPL, UU, FF, SS, FU)                                                                \
    XC_LAUNCH(K_GATHER, st, (gather_kernel<T, CPL, KIND, UU, FF, SS, FU><<<grid, kStepThreads, 0, st>>>( \
        static_cast<const T*>(Z), static_cast<T*>(W), L, d, pos, k_p, neg, logq, n_neg,                \
        pl.G, SQ, B, inv_B, single_slot, lr, static_cast<T*>(rows_out), gco, loss_q, dZ)))
#define XC_GATHER2(CPL, UU, FF, SS)                                                                    \
    do {                                                                                               \
        if (KIND == XC_LOSS_BCE && fuse) XC_GATHER3(CPL, UU, FF, SS, (KIND == XC_LOSS_BCE));           \
        else XC_GATHER3(CPL, UU, FF, SS, false);                                                       \
    } while (0)
#define XC_GATHER(CPL)                                                                                 \
    do {                                                                                               \
        const bool full = (d / Elem<T>::kPerChunk) == pl.G * CPL && d % Elem<T>::kPerChunk == 0;       \
        if (B * SQ <= 1024) {   /* few workgroups: more rows in flight per group */                   \
            if (full) XC_GATHER2(CPL, 8, true, false); else XC_GATHER2(CPL, 8, false, false);          \
        } else if (full && pl.stream_gather) {                                                         \
            XC_GATHER2(CPL, 4, true, true);                                                            \
        } else {                                                                                       \
            if (full) XC_GATHER2(CPL, 4, true, false); else XC_GATHER2(CPL, 4, false, false);          \
        }                                                                                              \
    } while (0)
    switch (pl.cpl) {
        case 1: XC_GATHER(1); break;
        case 2: XC_GATHER(2); break;
        case 3: XC_GATHER(3); break;
        default: XC_GATHER(4); break;
    }
#undef XC_GATHER
#undef XC_GATHER2
#undef XC_GATHER3
}

template <typename T>
static void launch_update(const StepPlan& pl, hipStream_t st, const void* Z, void* W, int d,
                          const uint2* pairs, const float* gco, const int32_t* touched,
                          const int32_t* seg_start, const uint32_t* seg_idx0, const int32_t* n_touched,
                          float lr, void* rows_out,
                          const float* dz_part, int SQ, int64_t BD, float* dZ, const int32_t* multi_list,
                          const int32_t* n_multi, const float* loss_q, int64_t n_loss, float inv_B, float* loss) {
    const int NG = kStepThreads / pl.G;
    // a pair per group would need P/NG workgroups; with several segments per group the grid is
    // bounded by what the chip holds at once
    int64_t nwg = (pl.P + NG - 1) / NG;
    if (nwg > kUpdateMaxGrid) nwg = kUpdateMaxGrid;
    const dim3 grid(static_cast<unsigned>(nwg + 1));       // one more for the loss
#define XC_UPDATE2(CPL, SS)                                                                       \
    XC_LAUNCH(K_UPDATE, st, (update_kernel<T, CPL, SS><<<grid, kStepThreads,                      \
        kStepThreads * CPL * Elem<T>::kPerChunk * sizeof(float), st>>>(                             \
        static_cast<const T*>(Z), static_cast<T*>(W), d, pl.n_magic, pl.n_shift, pl.G, pairs, gco, touched, seg_start, \
        seg_idx0, n_touched, lr, static_cast<T*>(rows_out), dz_part, SQ, BD, dZ, multi_list, n_multi, loss_q, n_loss, inv_B, loss)))
#define XC_UPDATE(CPL)                                                                            \
    do { if (pl.stream_update) XC_UPDATE2(CPL, true); else XC_UPDATE2(CPL, false); } while (0)
    switch (pl.cpl) {
        case 1: XC_UPDATE(1); break;
        case 2: XC_UPDATE(2); break;
        case 3: XC_UPDATE(3); break;
        default: XC_UPDATE(4); break;
    }
#undef XC_UPDATE
#undef XC_UPDATE2
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

namespace xc {
// host-side checks of a step's arguments (everything but the workspace); fills the launch plan
static int check_step_args(const void* Z, const void* W, int64_t B, int64_t L, int d, const int32_t* pos, int k_p,
                           const int32_t* neg, const float* logq, int n_neg, xc_loss kind, xc_dtype t,
                           const float* loss, const float* dZ, const int32_t* touched, const int32_t* n_touched,
                           const void* W_rows_out, StepPlan* pl) {
    if (kind != XC_LOSS_BCE && kind != XC_LOSS_SOFTMAX) return XC_EINVAL;
    if (L < 1 || L > 0x7ffffffeLL) return XC_ESHAPE;
    const int rc = plan_step(B, L, d, k_p, n_neg, t, pl);
    if (rc != XC_OK) return rc;
    if (!Z || !W || !loss || !dZ || !touched || !n_touched) return XC_EINVAL;
    if ((k_p > 0 && !pos) || (n_neg > 0 && (!neg || !logq))) return XC_EINVAL;
    if (!aligned16(Z) || !aligned16(W) || !aligned16(dZ)) return XC_EINVAL;
    if (W_rows_out && !aligned16(W_rows_out)) return XC_EINVAL;
    if (Z == static_cast<const void*>(dZ)) return XC_EINVAL;
    return XC_OK;
}

static int step_impl(const void* Z, void* W, int64_t B, int64_t L, int d, const int32_t* pos, int k_p,
                     const int32_t* neg, const float* logq, int n_neg, float lr, xc_loss kind,
                     xc_dtype t, float* loss, float* dZ, int32_t* touched, int32_t* n_touched,
                     void* W_rows_out, void* ws, size_t ws_bytes, void* stream) {
    StepPlan pl;
    const int rc = check_step_args(Z, W, B, L, d, pos, k_p, neg, logq, n_neg, kind, t, loss, dZ, touched,
                                   n_touched, W_rows_out, &pl);
    if (rc != XC_OK) return rc;
    if (!ws || !aligned16(ws)) return XC_EINVAL;
    {   // layout does not depend on L except for the number of sort passes
        StepPlan ref;
        plan_step(B, 0x7ffffffeLL, d, k_p, n_neg, t, &ref);
        if (ws_bytes < ref.total) return XC_EWORKSPACE;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* w8 = static_cast<unsigned char*>(ws);
    uint2* pairs0 = reinterpret_cast<uint2*>(w8 + pl.off_pairs0);
    uint2* pairs1 = reinterpret_cast<uint2*>(w8 + pl.off_pairs1);
    float* gco = reinterpret_cast<float*>(w8 + pl.off_g);
    float* loss_q = reinterpret_cast<float*>(w8 + pl.off_lossq);
    int* counts = reinterpret_cast<int*>(w8 + pl.off_counts);
    int* totals = reinterpret_cast<int*>(w8 + pl.off_totals);
    int* bases = reinterpret_cast<int*>(w8 + pl.off_bases);
    int* head_cnt = reinterpret_cast<int*>(w8 + pl.off_headcnt);
    int* valid_cnt = reinterpret_cast<int*>(w8 + pl.off_validcnt);
    int32_t* seg_start = reinterpret_cast<int32_t*>(w8 + pl.off_segstart);
    uint32_t* seg_idx0 = reinterpret_cast<uint32_t*>(w8 + pl.off_segidx0);

    int32_t* stats = reinterpret_cast<int32_t*>(w8 + pl.off_stats);
    int32_t* single_slot = reinterpret_cast<int32_t*>(w8 + pl.off_single);
    int32_t* multi_list = reinterpret_cast<int32_t*>(w8 + pl.off_multi);
    int* multi_cnt = reinterpret_cast<int*>(w8 + pl.off_multicnt);
    // Labels with one pair are updated inside the gather where they are the rule: with P pairs spread over L
    // labels the share of touched labels that have one pair is about exp(-P/L), and the gather pays for each of
    // them with a row written from a kernel that is bound by instruction issue.  Measured: 2.3 M pairs over
    // 1.3 M labels (a third single) loses 8 % of the step, 8.6 M over 120 M (96 % single) gains 30 %.
    const bool fuse = kind == XC_LOSS_BCE && 2 * pl.P <= L;
    KeySource ks;
    ks.pos = pos; ks.neg = neg; ks.k_p = k_p; ks.n_neg = n_neg; ks.n = pl.n; ks.n_shift = pl.n_shift;
    ks.n_magic = pl.n_magic; ks.softmax = kind == XC_LOSS_SOFTMAX ? 1 : 0; ks.L = L;

    // S5, first half: the pairs sorted by label and the segment heads.  They depend on the ids alone, so they come
    // first, and the gather that follows knows which rows it may update itself.
    uint2 *kin = pairs0, *kout = pairs1;
    if (pl.n_buckets > 0) {
        // one round on the high digit (masked pairs behind every label), then each bucket by its low digit
        const int radix = 1 << pl.high_rb;
        const uint32_t Lk = static_cast<uint32_t>(L);
        XC_LAUNCH(K_RADIX_COUNT, st, (radix_count_kernel<true><<<pl.nb, 256, 0, st>>>(nullptr, pl.P, pl.chunk, pl.low_bits, pl.high_rb, pl.nb, counts, Lk, pl.n_buckets, ks, kin, stats)));
        XC_LAUNCH(K_RADIX_SCAN, st, (radix_prefix_kernel<<<radix, kWave, 0, st>>>(counts, pl.nb, totals)));
        XC_LAUNCH(K_RADIX_SCATTER, st, (radix_scatter_kernel<<<pl.nb, kSortTile, sort_lds_bytes(pl.high_rb), st>>>(kin, kout, pl.P, pl.chunk, pl.low_bits, pl.high_rb, pl.nb, counts, totals, Lk, pl.n_buckets, bases)));
        XC_LAUNCH(K_BUCKET_SORT, st, (bucket_sort_kernel<<<pl.n_buckets, kSortTile, sort_lds_bytes(pl.low_bits), st>>>(kout, kin, totals, bases, pl.low_bits, head_cnt, multi_cnt)));
        // the sizes of the label buckets add up to the number of unmasked pairs
        XC_LAUNCH(K_HEADS_WRITE, st, (heads_write_kernel<<<pl.n_buckets + 1, 256, 0, st>>>(kin, pl.P, pl.chunk, Lk, pl.n_buckets, head_cnt,
                                                                                     totals, touched, seg_start, seg_idx0, n_touched, totals, bases,
                                                                                     fuse ? single_slot : nullptr, multi_cnt, multi_list, stats)));
        XC_HIP_CHECK(hipGetLastError());
    } else {
        for (int pass = 0; pass < pl.passes; ++pass) {
            const int shift = pass * pl.rb;
            const int radix = 1 << pl.rb;
            if (pass == 0) XC_LAUNCH(K_RADIX_COUNT, st, (radix_count_kernel<true><<<pl.nb, 256, 0, st>>>(nullptr, pl.P, pl.chunk, shift, pl.rb, pl.nb, counts, 0xffffffffu, 0, ks, kin, stats)));
            else XC_LAUNCH(K_RADIX_COUNT, st, (radix_count_kernel<false><<<pl.nb, 256, 0, st>>>(kin, pl.P, pl.chunk, shift, pl.rb, pl.nb, counts, 0xffffffffu, 0, ks, nullptr, stats)));
            XC_LAUNCH(K_RADIX_SCAN, st, (radix_prefix_kernel<<<radix, kWave, 0, st>>>(counts, pl.nb, totals)));
            XC_LAUNCH(K_RADIX_SCATTER, st, (radix_scatter_kernel<<<pl.nb, kSortTile, sort_lds_bytes(pl.rb), st>>>(kin, kout, pl.P, pl.chunk, shift, pl.rb, pl.nb, counts, totals, 0xffffffffu, 0, nullptr)));
            XC_HIP_CHECK(hipGetLastError());
            uint2* tk = kin; kin = kout; kout = tk;
        }
        XC_LAUNCH(K_HEADS_COUNT, st, (heads_count_kernel<<<pl.nb, 256, 0, st>>>(kin, pl.P, pl.chunk, static_cast<uint32_t>(L), head_cnt, valid_cnt, multi_cnt)));
        XC_LAUNCH(K_HEADS_WRITE, st, (heads_write_kernel<<<pl.nb + 1, 256, 0, st>>>(kin, pl.P, pl.chunk, static_cast<uint32_t>(L), pl.nb, head_cnt,
                                                                                valid_cnt, touched, seg_start, seg_idx0, n_touched, nullptr, nullptr,
                                                                                fuse ? single_slot : nullptr, multi_cnt, multi_list, stats)));
        XC_HIP_CHECK(hipGetLastError());
    }

    // S3 + S4 (+ the row update of every label with a single pair)
    const int SQ = kind == XC_LOSS_BCE ? pl.sq : 1;      // the soft-max normaliser needs the whole query
    float* dz_target = SQ > 1 ? reinterpret_cast<float*>(w8 + pl.off_dzpart) : dZ;
    if (t == XC_BF16) {
        if (kind == XC_LOSS_BCE)
            launch_gather<bf16_t, XC_LOSS_BCE>(pl, st, Z, W, B, L, d, pos, k_p, neg, logq, n_neg, fuse ? single_slot : nullptr, lr, W_rows_out, gco, loss_q, dz_target, SQ);
        else
            launch_gather<bf16_t, XC_LOSS_SOFTMAX>(pl, st, Z, W, B, L, d, pos, k_p, neg, logq, n_neg, fuse ? single_slot : nullptr, lr, W_rows_out, gco, loss_q, dz_target, SQ);
    } else {
        if (kind == XC_LOSS_BCE)
            launch_gather<float, XC_LOSS_BCE>(pl, st, Z, W, B, L, d, pos, k_p, neg, logq, n_neg, fuse ? single_slot : nullptr, lr, W_rows_out, gco, loss_q, dz_target, SQ);
        else
            launch_gather<float, XC_LOSS_SOFTMAX>(pl, st, Z, W, B, L, d, pos, k_p, neg, logq, n_neg, fuse ? single_slot : nullptr, lr, W_rows_out, gco, loss_q, dz_target, SQ);
    }
    XC_HIP_CHECK(hipGetLastError());

    // S5, second half: the rows of the labels with several pairs
    const int64_t n_loss = B * SQ;
    const float inv_B = 1.0f / static_cast<float>(B);
    if (t == XC_BF16) launch_update<bf16_t>(pl, st, Z, W, d, kin, gco, touched, seg_start, seg_idx0, n_touched, lr, W_rows_out, dz_target, SQ, B * static_cast<int64_t>(d), dZ, fuse ? multi_list : nullptr, stats + 1, loss_q, n_loss, inv_B, loss);
    else launch_update<float>(pl, st, Z, W, d, kin, gco, touched, seg_start, seg_idx0, n_touched, lr, W_rows_out, dz_target, SQ, B * static_cast<int64_t>(d), dZ, fuse ? multi_list : nullptr, stats + 1, loss_q, n_loss, inv_B, loss);
    XC_HIP_CHECK(hipGetLastError());
    return XC_OK;
}

// ---------------------------------------------------------------------------
// Scratch memory of the entry point that allocates nothing: one array per GPU, part of the
// library's device image, held until the process ends.  In host code the array's name is only a
// handle; its device address is asked for once per device and kept.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[XC_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex scratch_mu;
static void* scratch_ptr[kMaxDevices];      // device address of `scratch` on each GPU, null = not asked yet

static int static_scratch(void** out) {
    int dev = 0;
    XC_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return XC_ESHAPE;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        XC_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) return XC_EHIP;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return XC_OK;
}
}  // namespace xc

extern "C" int xc_step(const void* Z, void* W, int64_t B, int64_t L, int d, const int32_t* pos, int k_p,
                       const int32_t* neg, const float* logq, int n_neg, float lr, xc_loss kind,
                       xc_dtype t, float* loss, float* dZ, int32_t* touched, int32_t* n_touched,
                       void* W_rows_out, void* ws, size_t ws_bytes, void* stream) {
    return xc::step_impl(Z, W, B, L, d, pos, k_p, neg, logq, n_neg, lr, kind, t, loss, dZ, touched, n_touched,
                         W_rows_out, ws, ws_bytes, stream);
}

extern "C" int xc_step_static(const void* Z, void* W, int64_t B, int64_t L, int d, const int32_t* pos, int k_p,
                              const int32_t* neg, const float* logq, int n_neg, float lr, xc_loss kind,
                              xc_dtype t, float* loss, float* dZ, int32_t* touched, int32_t* n_touched,
                              void* W_rows_out, void* stream) {
    // host-side checks first, the device is not touched before they pass: sizes (a shape whose temporaries do
    // not fit the array is refused), then pointers
    size_t need = 0;
    const int rc = xc_step_workspace(B, d, k_p, n_neg, t, &need);
    if (rc != XC_OK) return rc;
    if (need > static_cast<size_t>(XC_STATIC_SCRATCH_BYTES)) return XC_ESCRATCH;
    {
        xc::StepPlan pl;
        const int rp = xc::check_step_args(Z, W, B, L, d, pos, k_p, neg, logq, n_neg, kind, t, loss, dZ, touched,
                                           n_touched, W_rows_out, &pl);
        if (rp != XC_OK) return rp;
    }
    void* ws = nullptr;
    const int rs = xc::static_scratch(&ws);
    if (rs != XC_OK) return rs;
    // every temporary of the step is written before it is read, so what an earlier call left in the
    // array does not matter and nothing has to be cleared
    return xc::step_impl(Z, W, B, L, d, pos, k_p, neg, logq, n_neg, lr, kind, t, loss, dZ, touched, n_touched,
                         W_rows_out, ws, static_cast<size_t>(XC_STATIC_SCRATCH_BYTES), stream);
}
