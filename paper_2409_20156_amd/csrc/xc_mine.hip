// Hard-negative mining: exact top-k inner product of every query against all
// classifier rows (Alg. 1, "ANNS refresh" step, with exact search in place of
// the index; score of Sec. 2.1).
//
// The labels are swept in phases of geometrically growing size (256 labels,
// then 8x more each time).  Within a phase every query has a FIXED threshold
// tau: the exact k-th best score over all labels of the earlier phases, so the
// k best labels overall are never below it and only about 8k scores per query
// pass it.
//   mine_tile_kernel    persistent tiled MFMA product W_tile x Z_tile^T (256
//       labels x 256 queries per workgroup, 8 waves of 128 x 64), K staged 64
//       elements at a time through two LDS buffers that are filled by direct
//       global->LDS loads one stage ahead.  Labels run along the MFMA M axis
//       and queries along N, so one lane owns one query column and compares its
//       accumulators with that query's tau; the score matrix never leaves
//       registers.  Passing scores are parked in a per-wave pool in LDS (slot
//       from a ballot, no atomic on the path) that lives as long as the label
//       slice; the pool is emptied into a 1024-key list per query when it
//       fills, and the lists are appended to the queries' global candidate
//       lists when the workgroup finishes its slice.  The filter of a tile
//       needs no barrier: the workgroup meets only after a tile in which a
//       pool was emptied, to cut any list that could overflow to its best k
//       (radix select by one wave; tau rises locally).
//   mine_select_kernel  after each phase, one wave per query cuts the global
//       candidate list to its best k and publishes the new tau; after the last
//       phase it sorts the winners by (score descending, id ascending).
#include <cstdlib>
#include <mutex>
#include <type_traits>

#include "xc_common.h"

namespace xc {

constexpr int kBM = 256;            // labels per tile   (MFMA M)
constexpr int kBN = 256;            // queries per tile  (MFMA N)
constexpr int kStageBytes = 128;    // bytes of a row staged in LDS per K step (= LDS row pitch; the
                                    // 16-byte chunks of a row are stored swizzled, see lds_chunk_swizzle)
constexpr int kCandCap = 1024;      // keys per query candidate list
constexpr int kPool = 320;          // passing scores a wave parks in LDS before it empties them into the lists
constexpr int kPoolCheck = 4;       // accumulators between two looks at the pool's fill (each adds <= 64 entries)
constexpr int kPoolKeep = kPool - kPoolCheck * 64;      // entries a wave may carry from one tile to the next
constexpr int kMineThreads = 512;   // 8 waves: 2 along labels x 4 along queries
constexpr int kMineWaves = kMineThreads / kWave;
static_assert(kPoolKeep >= 0, "the pool holds what can arrive between two looks at its fill");
constexpr int kMineGrid = 256;      // persistent workgroups, one per compute unit
constexpr int kXcds = 8;            // workgroup w runs on XCD w % 8
constexpr int kCusPerXcd = kMineGrid / kXcds;
constexpr int kPhaseGrowth = 8;     // labels of a phase / labels before it
constexpr int kMaxSlices = 64;      // label slices of a phase at most (one lane per slice in the select)
constexpr int kSelectRegs = 16;     // keys per lane held in registers by the phase select
constexpr uint32_t kTauInit = 0x007fffffu;   // ordered image of -inf

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------
// Reduce a candidate list of n > k keys to its k smallest keys (best scores).
// One wave; n <= 64*R keys, fetched by load(index) and held in registers.  Radix select, most significant byte first, with a
// 256-bin histogram in LDS; stops as soon as every key sharing the prefix is
// needed.  Writes the survivors to buf[0..k), returns the score of the k-th.
// ---------------------------------------------------------------------------
template <int R, typename Load>
__device__ __noinline__ float wave_select_k(uint64_t* __restrict__ buf, Load load, int n, int k, int* hist) {
    const int lane = lane_id();
    uint64_t key[R];
    bool valid[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int idx = r * kWave + lane;
        valid[r] = idx < n;
        key[r] = valid[r] ? load(idx) : kKeySentinel;
    }
    // leading bytes shared by every key (scores of one query lie close together) need no pass:
    // all keys would fall into one histogram bin, one atomic after the other
    uint64_t diff = 0;
    const uint64_t ref = __shfl(key[0], 0, kWave);          // index 0 is valid (n > k >= 1)
#pragma unroll
    for (int r = 0; r < R; ++r) diff |= valid[r] ? (key[r] ^ ref) : 0ull;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) diff |= __shfl_xor(diff, off, kWave);
    const int first_pass = diff == 0ull ? 8 : (__clzll(static_cast<long long>(diff)) >> 3);
    uint64_t pmask = first_pass == 0 ? 0ull : (~0ull << (64 - 8 * first_pass));
    uint64_t prefix = ref & pmask;
    int need = k;
    for (int pass = first_pass; pass < 8; ++pass) {
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

struct MineArgs {
    const unsigned char* Z;
    const unsigned char* W;
    int64_t Zq, L, row_bytes;
    int k, kcap;
    int nkb;                 // K stages per tile
    int64_t nQT;             // query tiles
    int64_t tile_lo, tile_hi;   // label tiles of this phase
    int64_t tiles_per_slice;
    int S;                   // label slices of the phase
    int Qx;                  // > 0: query tiles in flight per XCD (slices bound to XCDs);
                             // 0: plain order, item = qtile * S + slice
    int append_max;          // keys one slice may append per query (>= kcap)
    int glist_cap;           // keys per query in the global candidate lists
    uint64_t* lists;         // [kMineGrid][kBN][kCandCap] per-workgroup lists
    uint64_t* glist;         // [nQT*kBN][glist_cap] per-query candidates across slices and phases
    int32_t* gcnt;           // [nQT*kBN] fill of glist
    const uint32_t* tau_g;   // [nQT*kBN] ordered image of the phase threshold
    const unsigned char* zeros;   // 256 zero bytes (source of the chunks past the end of a row)
    const int32_t* cond;     // not null: repeat of a warm search; cond[0] != 0 if any query tile needs it,
                             // cond[1 + qt] != 0 if query tile qt does
};

// ---------------------------------------------------------------------------
// LDS staging.  One K stage is 512 rows (256 of W, then 256 of Z) x 128 bytes, row pitch 128.
// Chunk c (16 bytes) of row r is stored at chunk position c ^ ((r >> 1) & 7): the 16 lanes
// that read the same chunk of 16 consecutive rows for an MFMA operand then hit 16 different
// 16-byte bank groups.  The stage is filled by direct global->LDS loads: lane i of a wave
// instruction writes bytes [16 i, 16 i + 16) of a 1 KiB block (8 rows), so the swizzle is
// applied to the SOURCE address of each lane.  The loads are written as inline assembly so
// that the compiler does not serialise later LDS reads behind them; they are awaited with an
// explicit vmcnt wait followed by a workgroup barrier.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void lds_dma16(const void* gptr, uint32_t lds_addr /* wave-uniform */) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gptr), "s"(lds_addr) : "memory");
}
// The same with a wave-uniform 64-bit base and a 32-bit lane offset: no vector arithmetic is needed
// to form the address, so issuing the load never competes with another wave's MFMAs for the VALU.
template <int V> using IC = std::integral_constant<int, V>;

template <int kLdsOffset>
__device__ __forceinline__ void lds_dma16_sbase(const void* sbase /* wave-uniform */, uint32_t voff,
                                                uint32_t lds_addr /* wave-uniform; kLdsOffset is added */) {
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr), "n"(kLdsOffset) : "memory", "scc");
}
__device__ __forceinline__ void wait_all_vmem() {
    __builtin_amdgcn_s_waitcnt(0x0070 | 0x0f00);      // vmcnt(0); expcnt and lgkmcnt untouched
}

// Stage fill of a ragged tile (rows past the end repeat the last row) or of rows whose length is
// not a multiple of the stage (chunks past the end come from the zero block): lane addresses are
// formed one by one.  Kept out of line so that its registers do not burden the main loop.
template <bool KTAIL>
__device__ __noinline__ void issue_stage_slow(const unsigned char* base, int64_t last_row, int64_t row_bytes,
                                              uint32_t kb, int drow, uint32_t dcol0, uint32_t dcol1,
                                              uint32_t dst, const unsigned char* zeros) {
#pragma unroll 1
    for (int t = 0; t < 16; ++t) {
        const int64_t r = drow + 8 * t;
        const uint32_t dc = (t & 1) ? dcol1 : dcol0;
        const unsigned char* g = base + ((r < last_row ? r : last_row) * row_bytes + dc + kb);
        if (KTAIL && kb + dc >= static_cast<uint32_t>(row_bytes)) g = zeros;
        lds_dma16(g, __builtin_amdgcn_readfirstlane(dst + t * 1024));
    }
}

template <typename T, bool KTAIL>
__global__ __launch_bounds__(kMineThreads, 1)
void mine_tile_kernel(const MineArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    if (a.cond != nullptr && a.cond[0] == 0) return;          // uniform: a repeat that is not needed
    // two stage buffers, each: W rows then Z rows
    constexpr int kStageBuf = (kBM + kBN) * kStageBytes;
    float* tau = reinterpret_cast<float*>(smem + 2 * kStageBuf);
    int* cnt = reinterpret_cast<int*>(tau + kBN);
    int* hist = cnt + kBN;                                   // [kMineWaves][256]
    uint2* pools = reinterpret_cast<uint2*>(hist + kMineWaves * 256);       // [kMineWaves][kPool]
    int* dirty = reinterpret_cast<int*>(pools + kMineWaves * kPool);        // [2], by tile parity
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) unsigned char*)smem));

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1;          // which 128-label half
    const int wn = wave >> 1;         // which 64-query quarter
    uint64_t* my_lists = a.lists + static_cast<size_t>(blockIdx.x) * kBN * kCandCap;

    // ---- which (query tile, label slice) items this workgroup processes
    int item, item_step, item_end;     // (nQT * S fits: at most 2^23 query tiles, 64 slices)
    int slice_fixed = -1;
    if (a.Qx > 0) {                   // slices bound to XCDs: workgroup w runs on XCD w % 8
        const int xcd = blockIdx.x % kXcds;
        const int cu = blockIdx.x / kXcds;
        slice_fixed = xcd + kXcds * (cu / a.Qx);
        item = cu % a.Qx; item_step = a.Qx; item_end = static_cast<int>(a.nQT);        // items are query tiles
        if (slice_fixed >= a.S) item_end = 0;
    } else {
        item = blockIdx.x; item_step = kMineGrid; item_end = static_cast<int>(a.nQT * a.S);
    }

    // ---- fragment reads: lane reads row (lane & 31) of a 32-row block, chunk 2 kk + (lane >> 5);
    // the swizzle term of those rows is (lane >> 1) & 7, and the k-step enters as an xor of 32 kk
    const int swz = (lane >> 1) & 7;
    const int frag_a = (wm * 128 + (lane & 31)) * kStageBytes + (((lane >> 5) ^ swz) * 16);
    const int frag_b = (kBM + wn * 64 + (lane & 31)) * kStageBytes + (((lane >> 5) ^ swz) * 16);

    // ---- stage fill.  A stage is brought in by four waves, one per SIMD, while their SIMD-mates
    // (waves w and w + 4 share a SIMD) start on the MFMAs at once; the two halves of the workgroup
    // take turns from stage to stage.  The issuing waves wait in the texture unit's queue, not in
    // front of the matrix pipe.  Wave w (and w + 4) owns 128 rows: W rows 0..127 / 128..255 for
    // w & 3 = 0 / 1, Z rows likewise for 2 / 3; instruction t covers rows 8 t .. 8 t + 7 of them,
    // lane i -> row i / 8, position i % 8.  The chunk a lane fetches is position ^ swizzle(row),
    // which depends on t only through t & 1.
    const bool dma_z = (wave & 3) >= 2;
    const int drow = (wave & 1) * 128 + (lane >> 3);
    const uint32_t dcol[2] = {static_cast<uint32_t>(((lane & 7) ^ (lane >> 4)) * 16),
                              static_cast<uint32_t>(((lane & 7) ^ ((lane >> 4) + 4)) * 16)};
    const uint32_t dma_dst = lds_base + (dma_z ? kBM * kStageBytes : 0) + (wave & 1) * 128 * kStageBytes;
    const uint32_t voff[2] = {static_cast<uint32_t>(drow * a.row_bytes) + dcol[0],
                              static_cast<uint32_t>((drow + 8) * a.row_bytes) + dcol[1]};

    for (; item < item_end; item += item_step) {
        const int64_t qtile = a.Qx > 0 ? item : item / a.S;
        if (a.cond != nullptr && a.cond[1 + qtile] == 0) continue;     // uniform: this query tile came out complete
        const int slice = a.Qx > 0 ? slice_fixed : static_cast<int>(item % a.S);
        const int64_t t_begin = a.tile_lo + static_cast<int64_t>(slice) * a.tiles_per_slice;
        // tiles of the slice are counted from t_begin in 32 bits (a slice has at most 2^31 / 256 / 8 tiles)
        int n_tiles;
        {
            int64_t t_end = t_begin + a.tiles_per_slice;
            t_end = t_end < a.tile_hi ? t_end : a.tile_hi;
            if (t_end <= t_begin) continue;                  // uniform: an empty slice
            n_tiles = static_cast<int>(t_end - t_begin);
        }
        // tiles [0, full_tiles) of the slice have all kBM rows
        int full_tiles;
        {
            const int64_t f = a.L / kBM - t_begin;
            full_tiles = f < 0 ? 0 : (f < n_tiles ? static_cast<int>(f) : n_tiles);
        }
        const int64_t q0 = qtile * kBN;
        if (tid < kBN) { tau[tid] = ordered_to_float(a.tau_g[q0 + tid]); cnt[tid] = 0; }
        if (tid < 2) dirty[tid] = 0;

        // ---- the load stream runs one stage ahead of the compute stream and stops at the last stage
        const unsigned char* zbase = a.Z + q0 * a.row_bytes;
        const unsigned char* wld = a.W + t_begin * kBM * a.row_bytes;       // W rows of the tile being loaded
        const bool z_full = a.Zq - q0 >= kBN;
        int ld_tile = 0;
        int ld_kb = 0, ld_slot = 0;
        int to_issue = n_tiles * a.nkb;
        auto issue_stage = [&]() {
            const bool full = dma_z ? z_full : ld_tile < full_tiles;
            const unsigned char* base = dma_z ? zbase : wld;
            const uint32_t kb = static_cast<uint32_t>(ld_kb) * kStageBytes;
            const uint32_t dst = dma_dst + static_cast<uint32_t>(ld_slot) * kStageBuf;
            if ((wave < 4) == (ld_slot == 0)) {              // this half's turn
                if (!KTAIL && full) {
                    // the usual case: every row of the tile exists.  Lane offsets voff[t & 1] are the
                    // same for all stages; everything else is added to the scalar base.
                    const uint64_t b64 = reinterpret_cast<uint64_t>(base + kb);     // wave-uniform
                    // (readfirstlane returns a signed int: widen each half as unsigned)
                    const uint64_t sb =
                        (static_cast<uint64_t>(static_cast<uint32_t>(
                             __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64 >> 32)))) << 32) |
                        static_cast<uint64_t>(static_cast<uint32_t>(
                            __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64))));
                    const uint64_t pair_step = 16u * static_cast<uint64_t>(a.row_bytes);     // 16 rows per two instructions
                    auto pair = [&](auto tc) {
                        constexpr int t = decltype(tc)::value;
                        const unsigned char* sp = reinterpret_cast<const unsigned char*>(sb + (t >> 1) * pair_step);
                        lds_dma16_sbase<t * 1024>(sp, voff[0], dst);
                        lds_dma16_sbase<(t + 1) * 1024>(sp, voff[1], dst);
                    };
                    pair(std::integral_constant<int, 0>{});  pair(std::integral_constant<int, 2>{});
                    pair(std::integral_constant<int, 4>{});  pair(std::integral_constant<int, 6>{});
                    pair(std::integral_constant<int, 8>{});  pair(std::integral_constant<int, 10>{});
                    pair(std::integral_constant<int, 12>{}); pair(std::integral_constant<int, 14>{});
                } else {
                    const int64_t last_row = dma_z ? a.Zq - 1 - q0 : a.L - 1 - (t_begin + ld_tile) * kBM;
                    issue_stage_slow<KTAIL>(base, last_row, a.row_bytes, kb, drow, dcol[0], dcol[1], dst, a.zeros);
                }
            }
            ld_slot ^= 1;
            --to_issue;
            if (++ld_kb == a.nkb) { ld_kb = 0; ++ld_tile; wld += kBM * a.row_bytes; }
        };

        f32x16 acc[4][2];            // (never cleared: the first k-step of a tile multiplies into zeros, see below)

        // ---- main loop.  At the top of a stage its data is visible in LDS, the next stage's loads
        // have been issued into the other buffer, and the fragments of its first k-step are already
        // in registers.  The barrier that publishes the next stage sits before the last k-step's
        // MFMAs, so the first fragment reads of the next stage (and the loads of the stage after it)
        // are under way while those MFMAs run.
        uint4 fa[2][4], fb[2][2];
        auto read_frags = [&](const unsigned char* buf, int kk, int sel) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                fa[sel][mt] = *reinterpret_cast<const uint4*>(buf + ((frag_a ^ (kk * 32)) + mt * 32 * kStageBytes));
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                fb[sel][nt] = *reinterpret_cast<const uint4*>(buf + ((frag_b ^ (kk * 32)) + nt * 32 * kStageBytes));
        };
        auto products = [&](int sel) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    MineTraits<T>::mma(fa[sel][mt], fb[sel][nt], acc[mt][nt]);
        };
        // the first k-step of a tile: the accumulators start from a zero operand instead of being cleared
        // one register at a time after the filter (128 vector moves per tile and wave)
        auto products_first = [&](int sel) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
                    f32x16 c = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    MineTraits<T>::mma(fa[sel][mt], fb[sel][nt], c);
                    acc[mt][nt] = c;
                }
        };
        int buf_sel = 0;
        auto publish_next = [&](const unsigned char* next_buf) {
            wait_all_vmem();                                 // this wave's part of the next stage has landed
            __syncthreads();                                 // everyone's has; the current buffer is free
            if (to_issue > 0) issue_stage();                 // the stage after it, into the current buffer
            read_frags(next_buf, 0, 0);
        };

        __syncthreads();                                     // tau/cnt visible; both stage buffers free
        issue_stage();
        publish_next(smem);                                  // stage 0 visible, stage 1 under way

        // ---- a passing score is first parked, with its query and label offset, in this wave's pool:
        // the slot comes from a ballot and a wave-uniform fill count, so nothing waits on an atomic.
        // The pool is emptied into the per-query lists (slots from LDS counters) when it fills up, at
        // the end of a tile if it holds more than kPoolKeep entries, and at the end of the slice.
        // No barrier is needed for any of that; what does need the whole workgroup - cutting a list
        // that could overflow, closing the slice - is done at the start of the next tile's filter,
        // when a flag says that lists have grown.
        uint2* pool = pools + wave * kPool;
        int fill = 0;
        int pool_tile = 0;                                   // labels in the pool count from this tile
        auto flush = [&]() {
            const int64_t l0 = (t_begin + pool_tile) * kBM;
#pragma unroll 1
            for (int e0 = 0; e0 < fill; e0 += 2 * kWave) {   // two batches of 64 at a time: the slot atomics overlap
                uint2 en[2];
                int slot[2];
                bool ok[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int e = e0 + u * kWave + lane;
                    ok[u] = e < fill;
                    en[u] = ok[u] ? pool[e] : make_uint2(0u, 0u);
                    ok[u] = ok[u] && (l0 + (en[u].y & 0xffffffu) < a.L);   // rows past the end repeat the last row
                }
#pragma unroll
                for (int u = 0; u < 2; ++u) slot[u] = ok[u] ? atomicAdd(&cnt[en[u].y >> 24], 1) : 0;
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (ok[u])
                        my_lists[static_cast<size_t>(en[u].y >> 24) * kCandCap + slot[u]] =
                            make_key(__uint_as_float(en[u].x) + 0.0f /* -0 -> +0 */,
                                     static_cast<int32_t>(l0 + (en[u].y & 0xffffffu)));
                }
            }
            fill = 0;
        };

        for (int tile = 0; tile < n_tiles; ++tile) {          // counted from t_begin
            const int par = tile & 1;
            for (int kb = 0; kb < a.nkb; ++kb) {
                const unsigned char* cur = smem + buf_sel * kStageBuf;
                const unsigned char* nxt = smem + (buf_sel ^ 1) * kStageBuf;
                buf_sel ^= 1;
                read_frags(cur, 1, 1);
                __builtin_amdgcn_sched_barrier(0);
                if (kb == 0) products_first(0); else products(0);
                __builtin_amdgcn_sched_barrier(0);
                read_frags(cur, 2, 0);
                __builtin_amdgcn_sched_barrier(0);
                products(1);
                __builtin_amdgcn_sched_barrier(0);
                read_frags(cur, 3, 1);
                __builtin_amdgcn_sched_barrier(0);
                products(0);
                __builtin_amdgcn_sched_barrier(0);
                // the next stage - of this tile or of the next one - is published before the last products
                if (kb + 1 < a.nkb || tile + 1 < n_tiles) publish_next(nxt);
                __builtin_amdgcn_sched_barrier(0);
                products(1);
                __builtin_amdgcn_sched_barrier(0);
            }


            // ---- threshold filter: lane owns query column (lane & 31) of each N tile
            const bool last = tile + 1 == n_tiles;
            // The flag this tile may set shares its slot with the flag of two tiles back, which the waves
            // read after the previous tile's filter: a barrier has to lie between that read and this
            // tile's filter.  Every tile has one in its main loop except a one-stage last tile.
            if (last && a.nkb == 1) __syncthreads();
            bool grew = false;                               // this wave emptied its pool during the tile
            auto filter = [&](auto ntc) {
                constexpr int nt = decltype(ntc)::value;
                const int qloc = wn * 64 + nt * 32 + (lane & 31);
                const float t = (q0 + qloc) < a.Zq ? tau[qloc] : INFINITY;
                float mx = acc[0][nt][0];
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc[mt][nt][i]);
                if (__ballot(mx >= t) != 0ull) {
                    // entry: score bits, query << 24 | label offset from the pool's first tile
                    auto row_word = [&]() {
                        uint32_t w = (static_cast<uint32_t>(qloc) << 24) |
                                     (static_cast<uint32_t>(tile - pool_tile) * kBM + static_cast<uint32_t>(4 * (lane >> 5)));
                        asm volatile("" : "+v"(w));          // keep the 64 row words out of registers
                        return w;
                    };
                    uint32_t qrow = row_word();
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
                        for (int i0 = 0; i0 < 16; i0 += kPoolCheck) {
#pragma unroll
                            for (int ii = 0; ii < kPoolCheck; ++ii) {
                                const int i = i0 + ii;
                                const float v = acc[mt][nt][i];
                                const bool hit = v >= t;
                                const uint64_t m = __ballot(hit);
                                if (__builtin_expect(m != 0ull, 0)) {    // out of line: a taken branch costs more
                                    if (hit) {
                                        const int pos = fill + static_cast<int>(__builtin_amdgcn_mbcnt_hi(
                                            static_cast<uint32_t>(m >> 32),
                                            __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(m), 0u)));
                                        pool[pos] = make_uint2(
                                            __float_as_uint(v),
                                            qrow + static_cast<uint32_t>(wm * 128 + mt * 32 + 8 * (i >> 2) + (i & 3)));
                                    }
                                    fill += __popcll(m);
                                }
                            }
                            // kPoolCheck accumulators add at most kPool - kPoolKeep entries
                            if (__builtin_expect(fill > kPoolKeep, 0)) {
                                flush();
                                pool_tile = tile;
                                qrow = row_word();
                                grew = true;
                            }
                        }
                    }
                }
            };
            filter(IC<0>{});
            filter(IC<1>{});
            // the label offset of an entry has 24 bits
            if (fill > 0 && (tile + 1 == n_tiles || tile - pool_tile >= 60000)) {
                flush();
                pool_tile = tile;
                grew = true;
            }
            if (grew && lane == 0) dirty[par] = 1;

            // ---- lists grown during the previous tile (the flag was set before barriers that every
            // wave has passed since), or the end of the slice: wave w looks after queries 32w..32w+31.
            // A list that could overflow before the next look (two tiles add at most 2 kBM entries, the
            // two pools that feed it at most kPoolKeep each), or, at the end of the slice, exceeds what
            // a slice may append, is cut to its best k and tau rises for the rest of the slice.
            if (last || dirty[par ^ 1] != 0) {               // uniform
                __syncthreads();                             // the pools' stores to the lists are complete
                const int qloc = wave * 32 + (lane & 31);
                const bool qok = (q0 + qloc) < a.Zq;
                int n = cnt[qloc];
                const bool want = lane < 32 && qok &&
                                  (last ? n > a.append_max : n > kCandCap - 2 * kBM - 2 * kPoolKeep);
                uint64_t todo = __ballot(want);
                if (todo != 0ull || last) {
                    float t_new = -INFINITY;
                    while (todo) {
                        const int src = __ffsll(static_cast<long long>(todo)) - 1;
                        todo &= todo - 1;
                        const int qsel = wave * 32 + src;
                        const int nsel = __shfl(n, src, kWave);
                        uint64_t* lsel = my_lists + static_cast<size_t>(qsel) * kCandCap;
                        const float t = wave_select_k<kCandCap / kWave>(
                            lsel, [lsel](int idx) { return lsel[idx]; }, nsel, a.k, hist + wave * 256);
                        if (lane == src) { t_new = t; n = a.k; }
                    }
                    if (want) { tau[qloc] = fmaxf(tau[qloc], t_new); cnt[qloc] = n; }
                    if (last) {
                        // ---- close the slice: append the survivors to the global list of each query
                        int base = 0;
                        const bool have = lane < 32 && qok && n > 0;
                        if (have) base = atomicAdd(&a.gcnt[q0 + qloc], n);
                        if (__ballot(have && n > 16) == 0ull) {
                            // short lists (the usual case): lanes l and l + 32 copy the list of query l,
                            // even and odd entries, all loads issued before the stores
                            const int nq = __shfl(have ? n : 0, lane & 31, kWave);
                            const int bq = __shfl(base, lane & 31, kWave);
                            const int ql = wave * 32 + (lane & 31);
                            const uint64_t* list = my_lists + static_cast<size_t>(ql) * kCandCap;
                            uint64_t* out = a.glist + static_cast<size_t>(q0 + ql) * a.glist_cap + bq;
                            uint64_t v[8];
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                const int e = (lane >> 5) + 2 * j;
                                v[j] = e < nq ? list[e] : 0ull;
                            }
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                const int e = (lane >> 5) + 2 * j;
                                if (e < nq && bq + e < a.glist_cap) out[e] = v[j];
                            }
                        } else {
                            // long lists (dense early phases): 64 entries of 8 queries per round,
                            // loads before stores
                            const int nv = have ? n : 0;
                            for (int c0 = 0; __ballot(nv > c0) != 0ull; c0 += kWave) {
                                const int e = c0 + lane;
                                for (int qb = 0; qb < 32; qb += 8) {
                                    uint64_t v[8];
                                    int dst[8];
#pragma unroll
                                    for (int u = 0; u < 8; ++u) {
                                        const int nsel = __shfl(nv, qb + u, kWave);
                                        const int bsel = __shfl(base, qb + u, kWave);
                                        dst[u] = (e < nsel && bsel + e < a.glist_cap) ? bsel + e : -1;
                                        v[u] = dst[u] >= 0
                                                   ? my_lists[static_cast<size_t>(wave * 32 + qb + u) * kCandCap + e]
                                                   : 0ull;
                                    }
#pragma unroll
                                    for (int u = 0; u < 8; ++u)
                                        if (dst[u] >= 0)
                                            a.glist[static_cast<size_t>(q0 + wave * 32 + qb + u) * a.glist_cap + dst[u]] = v[u];
                                }
                            }
                        }
                    }
                }
                if (tid == 0) { dirty[par ^ 1] = 0; if (last) dirty[par] = 0; }
                __syncthreads();
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The same work item (256 queries x one label slice) for bf16 rows of at most 512 bytes
// (NK = row bytes / 128 = 1..4), where a wave's share of the query tile fits its registers.
//   * The query tile never passes through LDS: wave (wm, wn) keeps the MFMA B operands of its 64
//     queries for the whole row in registers (NK * 32 of them), loaded once per work item.
//   * Only W is streamed: a label tile is 64 WM labels, staged 128 bytes of each row at a time
//     through a ring of kRing stages in LDS, filled kRing - 1 stages ahead by direct
//     global->LDS loads, issued by one wave per SIMD in turn.  2 operand reads from LDS per 4
//     MFMAs instead of 6 per 8.
//   * A wave computes 64 labels x 64 queries (2 x 2 MFMA blocks); the 8 waves are laid out WM
//     along the labels x 8 / WM along the queries.  WM = 2: 128 labels x 256 queries per tile,
//     half the bytes staged per flop of the general kernel.  WM = 1: 64 labels x 512 queries
//     (two adjacent 256-query tiles form one work item), a quarter; for pools that fill it.
//   * A lane owns two query columns and the thresholds of exactly those, which it keeps in
//     registers.  A passing score goes straight to a candidate list that belongs to the lane
//     alone (2 WM owners per query: WM waves x 2 lane halves, 256 keys each, in the workgroup's
//     part of the workspace), at a position the lane counts itself: no atomics, no LDS, no
//     barrier on the path.
//   * A lane's list that could overflow in the next tile is cut to its best k by the lane's wave
//     (every label of the overall best k that is in this list is among the list's own best k),
//     and the lane's threshold rises to the k-th of them.  Nothing of that involves other waves.
//   * At the end of the slice the lists of a query are appended to its global list, cut to
//     the best k of them all first if they hold more than a slice may append.
// ---------------------------------------------------------------------------
constexpr int kRing = 8;            // stages in LDS (8 or 16 KiB each)
static_assert(kRing >= 4 && (kRing & (kRing - 1)) == 0, "stage slots are indexed modulo a power of two, and the two halves of the workgroup fill them in turn");
constexpr int kSubCap = kCandCap / 4;            // keys of a lane's own list
constexpr int kSubFull = kSubCap - 32;           // above this a tile could overflow it (a lane adds <= 32 per column)
constexpr size_t rows_lds_bytes(int wm) {     // ring, list fills at the end of a slice, select histograms
    return static_cast<size_t>(kRing) * wm * 64 * kStageBytes + kBN * 4 * sizeof(int) + kMineWaves * 256 * sizeof(int);
}

// XC_MINE_GENERAL=1 in the environment (read at every call) sends every shape through the general tile
// kernel, for A/B timing and for tests
static bool force_general_kernel() {
    const char* e = getenv("XC_MINE_GENERAL");
    return e != nullptr && e[0] == '1';
}

// The lane number, computed where it is asked for (the compiler can neither hoist nor keep it).
__device__ __forceinline__ uint32_t lane_now() {
    uint32_t l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

template <int N>
__device__ __forceinline__ void wait_vmem_at_most() {   // until at most N vector memory operations are outstanding
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | 0x0070 | 0x0f00);
}

// Stage fill of the last, ragged label tile: per-lane addresses, rows past the end repeat the last row.
__device__ __noinline__ void issue_stage_ragged(const unsigned char* W, int64_t L, int64_t row, int row_bytes, int kbyte,
                                                uint32_t dcol0, uint32_t dcol1, uint32_t dst, int n_instr) {
#pragma unroll 1
    for (int t = 0; t < n_instr; ++t) {
        int64_t r = row + 8 * t;
        r = r < L ? r : L - 1;
        lds_dma16(W + r * row_bytes + kbyte + ((t & 1) ? dcol1 : dcol0), __builtin_amdgcn_readfirstlane(dst + t * 1024));
    }
}

template <int NK, int WM>
__global__ __launch_bounds__(kMineThreads, 1)
void mine_rows_kernel(const MineArgs a) {
    static_assert(WM == 1 || WM == 2, "wave layouts");
    constexpr int kRowTile = 64 * WM;                   // labels per tile
    constexpr int kRowStage = kRowTile * kStageBytes;   // bytes of a stage
    constexpr int kQN = (kMineWaves / WM) * 64;         // queries per work item
    constexpr int kOwn = 2 * WM;                        // lists per query (kOwn * kQN = 4 kBN)
    constexpr int kQCap = kOwn * kSubCap;               // keys of a query's lists together
    constexpr int kLd = 2 * WM;                         // load instructions of a wave per stage it brings in
    extern __shared__ __align__(16) unsigned char smem[];
    if (a.cond != nullptr && a.cond[0] == 0) return;          // uniform: a repeat that is not needed
    int* cnt4 = reinterpret_cast<int*>(smem + kRing * kRowStage);            // [kQN][kOwn] list fills at the end of a slice
    int* hist = cnt4 + kBN * 4;                                             // [kMineWaves][256]
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) unsigned char*)smem));

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM;         // which 64 labels of the tile
    const int wn = wave / WM;         // which 64 queries of the work item
    const int half = lane >> 5;
    uint64_t* my_lists = a.lists + static_cast<size_t>(blockIdx.x) * kBN * kCandCap;
    constexpr int row_bytes = NK * kStageBytes;
    // a query takes part if it exists and, in the repeat of a warm search, if its 256-query tile needs it
    auto live = [&](int64_t q) { return q < a.Zq && (a.cond == nullptr || a.cond[1 + q / kBN] != 0); };

    int item, item_step, item_end;
    int slice_fixed = -1;
    if (a.Qx > 0) {                   // slices bound to XCDs: workgroup w runs on XCD w % 8
        const int xcd = blockIdx.x % kXcds;
        const int cu = blockIdx.x / kXcds;
        slice_fixed = xcd + kXcds * (cu / a.Qx);
        item = cu % a.Qx; item_step = a.Qx; item_end = static_cast<int>(a.nQT);
        if (slice_fixed >= a.S) item_end = 0;
    } else {
        item = blockIdx.x; item_step = kMineGrid; item_end = static_cast<int>(a.nQT * a.S);
    }

    // fragment reads of the A operand (as in the general kernel: row pitch 128, chunks swizzled by (row >> 1) & 7)
    const int swz = (lane >> 1) & 7;
    const int frag_a = (wm * 64 + (lane & 31)) * kStageBytes + ((half ^ swz) * 16);
    // stage fill.  Waves w and w + 4 share a SIMD.  A stage is brought in by four waves, one per SIMD, while
    // their SIMD-mates start on the MFMAs at once (a wave that issues loads queues at the texture unit behind
    // the other waves' loads; if all eight issued, every SIMD's matrix pipe would idle meanwhile); waves 0..3
    // take the even stages, waves 4..7 the odd ones.  Wave w brings in rows 8 kLd (w & 3) .. + 8 kLd - 1 of the stage
    // with kLd instructions of 8 rows; lane i -> row i / 8, position i % 8, source chunk = position ^ swizzle(row)
    const int drow = lane >> 3;
    const int wq = wave & 3;
    const int my_parity = wave >> 2;
    const uint32_t dcol[2] = {static_cast<uint32_t>(((lane & 7) ^ (lane >> 4)) * 16),
                              static_cast<uint32_t>(((lane & 7) ^ ((lane >> 4) + 4)) * 16)};
    const uint32_t voff[2] = {static_cast<uint32_t>(drow * row_bytes) + dcol[0],
                              static_cast<uint32_t>((drow + 8) * row_bytes) + dcol[1]};
    const uint32_t dma_dst = lds_base + wq * kLd * 1024;

    for (; item < item_end; item += item_step) {
        const int64_t qtile = a.Qx > 0 ? item : item / a.S;
        const int64_t q0 = qtile * kQN;
        if (a.cond != nullptr) {                             // uniform: every 256-query tile of the item came out complete
            bool any = false;
            for (int64_t qt = q0 / kBN; qt < (q0 + kQN) / kBN && qt * kBN < a.Zq; ++qt) any = any || a.cond[1 + qt] != 0;
            if (!any) continue;
        }
        const int slice = a.Qx > 0 ? slice_fixed : static_cast<int>(item % a.S);
        const int64_t t_begin = a.tile_lo + static_cast<int64_t>(slice) * a.tiles_per_slice;
        int64_t lab_begin, lab_end;
        {
            int64_t t_end = t_begin + a.tiles_per_slice;
            t_end = t_end < a.tile_hi ? t_end : a.tile_hi;
            if (t_end <= t_begin) continue;                  // uniform: an empty slice
            lab_begin = t_begin * kBM;
            lab_end = t_end * kBM;
            lab_end = lab_end < a.L ? lab_end : a.L;
        }
        const int n_tiles = static_cast<int>((lab_end - lab_begin + kRowTile - 1) / kRowTile);
        const int n_stages = n_tiles * NK;

        // ---- this wave's queries: B operands for the whole row, thresholds of the lane's two columns
        uint4 zf[NK * 4][2];
        float tau[2];
        int cnt[2] = {0, 0};
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int64_t q = q0 + wn * 64 + nt * 32 + (lane & 31);
            const int64_t qc = q < a.Zq ? q : a.Zq - 1;
            tau[nt] = live(q) ? ordered_to_float(a.tau_g[q]) : INFINITY;
            const unsigned char* zr = a.Z + qc * row_bytes + half * 16;
#pragma unroll
            for (int ks = 0; ks < NK * 4; ++ks) zf[ks][nt] = *reinterpret_cast<const uint4*>(zr + ks * 32);
        }

        // every load so far has landed before the first stage load is issued: from here on the only vector memory
        // operations in flight are the stage loads (and the filter's rare stores), counted by the waits below
        wait_all_vmem();

        // ---- the load stream: stage g = (tile g / NK, bytes 128 (g % NK) .. of the rows) goes to slot g % kRing
        int ld_stage = 0, ld_kb = 0, ld_tile = 0;
        uint32_t ld_dst = dma_dst;
        const unsigned char* ld_w = a.W + (lab_begin + wq * 8 * kLd) * row_bytes;   // this wave's rows of the tile being loaded
        const int full_tiles = static_cast<int>((a.L - lab_begin) / kRowTile < n_tiles ? (a.L - lab_begin) / kRowTile : n_tiles);
        auto issue_stage = [&]() {
            if ((ld_stage & 1) != my_parity) {
                // the other half's turn
            } else if (ld_tile < full_tiles) {
                const uint64_t b64 = reinterpret_cast<uint64_t>(ld_w + ld_kb * kStageBytes);
                const uint64_t sb =
                    (static_cast<uint64_t>(static_cast<uint32_t>(
                         __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64 >> 32)))) << 32) |
                    static_cast<uint64_t>(static_cast<uint32_t>(
                        __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64))));
                const unsigned char* sp = reinterpret_cast<const unsigned char*>(sb);
                lds_dma16_sbase<0>(sp, voff[0], ld_dst);
                lds_dma16_sbase<1024>(sp, voff[1], ld_dst);
                if (WM == 2) {
                    const unsigned char* sp2 = sp + 16 * row_bytes;
                    lds_dma16_sbase<2048>(sp2, voff[0], ld_dst);
                    lds_dma16_sbase<3072>(sp2, voff[1], ld_dst);
                }
            } else {
                // the last tile of the label range: rows past the end repeat the last row (dropped by the filter)
                issue_stage_ragged(a.W, a.L, lab_begin + static_cast<int64_t>(ld_tile) * kRowTile + wq * 8 * kLd + drow,
                                   row_bytes, ld_kb * kStageBytes, dcol[0], dcol[1], ld_dst, kLd);
            }
            ++ld_stage;
            ld_dst += kRowStage;
            if ((ld_stage & (kRing - 1)) == 0) ld_dst = dma_dst;
            if (++ld_kb == NK) { ld_kb = 0; ++ld_tile; ld_w += kRowTile * row_bytes; }
        };
        // This wave's part of stage g (if it has one) is complete once at most kLd * (its stages issued after g)
        // loads are outstanding: of the kRing - 2 stages issued after g in the steady state half are this
        // wave's, whichever half g belongs to.  Stores of the filter only make the wait stricter (loads complete
        // in order among themselves).  Near the end of the work item everything is awaited.
        auto wait_stage = [&](int g) {
            if (ld_stage - 1 - g >= kRing - 2) wait_vmem_at_most<kLd * ((kRing - 2) / 2)>();
            else wait_all_vmem();
        };

        f32x16 acc[2][2];
        uint4 fa[2][2];
        auto read_frags = [&](int slot, int kk, int sel) {
            const unsigned char* buf = smem + slot * kRowStage;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                fa[sel][mt] = *reinterpret_cast<const uint4*>(buf + ((frag_a ^ (kk * 32)) + mt * 32 * kStageBytes));
        };
        // stage g + 1 visible to everyone, stage g's slot free: refill it, and fetch the first operands of stage g + 1
        auto publish = [&](int g_next) {
            wait_stage(g_next);
            lds_barrier();
            if (ld_stage < n_stages) issue_stage();
            read_frags(g_next % kRing, 0, 0);
        };

        __syncthreads();                                     // the ring and cnt4 are free (previous item closed)
        for (int s = 0; s < kRing - 1 && s < n_stages; ++s) issue_stage();
        publish(0);

        // ---- threshold filter of one N block (the lane owns query column (lane & 31) of it) of the tile that
        // starts at label l0: the block's largest score per lane, and, where some lane's reaches its threshold,
        // the scores one by one
        auto block_max = [&](auto ntc) {
            constexpr int nt = decltype(ntc)::value;
            float mx = acc[0][nt][0];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc[mt][nt][i]);
            return mx;
        };
        auto push_block = [&](auto ntc, int64_t l0, float mx) {
            constexpr int nt = decltype(ntc)::value;
            const float t = tau[nt];
            if (__ballot(mx >= t) != 0ull) {
                // Everything a push needs is formed here from the lane number, read afresh, and from wave-uniform
                // values: a per-lane pointer or row number kept in a register over the main loop would be
                // spilled there, and its reload would wait for every stage load in flight.
                const int32_t lmax = static_cast<int32_t>(a.L);
                const int32_t lbase = static_cast<int32_t>(l0) + wm * 64;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float v = acc[mt][nt][i];
                        if (__builtin_expect(__ballot(v >= t) != 0ull, 0)) {
                            const uint32_t l = lane_now();
                            const int32_t lab = lbase + 4 * static_cast<int32_t>(l >> 5) + mt * 32 + 8 * (i >> 2) + (i & 3);
                            if (v >= t && lab < lmax) {             // rows past the end repeat the last row
                                const uint32_t sub = static_cast<uint32_t>(((wn * 64 + nt * 32) * kOwn + wm * 2)) + (l & 31u) * kOwn + (l >> 5);
                                my_lists[sub * kSubCap + static_cast<uint32_t>(cnt[nt])] = make_key(v + 0.0f /* -0 -> +0 */, lab);
                                ++cnt[nt];
                            }
                        }
                    }
            }
        };
        // ---- a list that the next tile could overflow: cut to its best k, by this wave alone
        auto cut_lists = [&]() {
            if (__builtin_expect(__ballot(cnt[0] > kSubFull || cnt[1] > kSubFull) != 0ull, 0)) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");       // this wave's list stores are complete ...
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");       // ... and are what the loads below see
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
                    uint64_t todo = __ballot(cnt[nt] > kSubFull);
                    while (todo) {
                        const int src = __ffsll(static_cast<long long>(todo)) - 1;
                        todo &= todo - 1;
                        const int qsel = wn * 64 + nt * 32 + (src & 31);
                        const int nsel = __shfl(cnt[nt], src, kWave);
                        uint64_t* lsel = my_lists + static_cast<size_t>(qsel * kOwn + wm * 2 + (src >> 5)) * kSubCap;
                        const float tk = wave_select_k<kSubCap / kWave>(
                            lsel, [lsel](int idx) { return lsel[idx]; }, nsel, a.k, hist + wave * 256);
                        if (lane == src) { cnt[nt] = a.k; tau[nt] = fmaxf(tau[nt], tk); }
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            }
        };

        // ---- main loop.  (Deferring a block's filter into the next tile's first products, so that the vector
        // ALU works while the matrix pipe does, was measured and gained nothing: the kernel runs at the chip's
        // power limit, where the clock falls as the matrix pipe fills.)
        int g = 0;                                           // stage being computed
        for (int tile = 0; tile < n_tiles; ++tile) {
            const int64_t l0 = lab_begin + static_cast<int64_t>(tile) * kRowTile;
#pragma unroll
            for (int kb = 0; kb < NK; ++kb) {
                const int slot = g % kRing;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const int sel = kk & 1;
                    if (kk < 3) {
                        read_frags(slot, kk + 1, sel ^ 1);
                    } else {
                        // (reads into fa[0], which the products of kk = 2 have left.  Also after the last stage,
                        // where the operands read are never used: one way through the loop body, so that no wait
                        // meant for another way in holds up the products below)
                        publish(g + 1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                        for (int nt = 0; nt < 2; ++nt) {
                            bf16x8 av, bv;
                            __builtin_memcpy(&av, &fa[sel][mt], 16);
                            __builtin_memcpy(&bv, &zf[kb * 4 + kk][nt], 16);
                            if (kb == 0 && kk == 0) {
                                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                                acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, zero, 0, 0, 0);
                            } else {
                                acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[mt][nt], 0, 0, 0);
                            }
                        }
                    __builtin_amdgcn_sched_barrier(0);
                }
                ++g;
            }
            // one test per tile on the usual way: does any lane see a score at its threshold, or a list to cut?
            const float mx0 = block_max(IC<0>{}), mx1 = block_max(IC<1>{});
            const bool look = mx0 >= tau[0] || mx1 >= tau[1] || cnt[0] > kSubFull || cnt[1] > kSubFull;
            if (__builtin_expect(__ballot(look) != 0ull, 0)) {
                push_block(IC<0>{}, l0, mx0);
                push_block(IC<1>{}, l0, mx1);
                cut_lists();
            }
        }

        // ---- close the slice: the lists of a query go to its global list
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) cnt4[(wn * 64 + nt * 32 + (lane & 31)) * kOwn + wm * 2 + half] = cnt[nt];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
#pragma unroll 1
        for (int qr = 0; qr < kQN; qr += kMineWaves * 32) {
            const int qw = qr + wave * 32;                   // lanes l and l + 32 look after query qw + l
            const int ql = qw + (lane & 31);
            const bool qok = live(q0 + ql);
            int c[kOwn];
            int n = 0;
#pragma unroll
            for (int s = 0; s < kOwn; ++s) { c[s] = qok ? cnt4[ql * kOwn + s] : 0; n += c[s]; }
            uint64_t* qlist = my_lists + static_cast<size_t>(ql) * kQCap;
            uint64_t todo = __ballot(lane < 32 && n > a.append_max);
            while (todo) {                                   // more than a slice may append: the best k of them all
                const int src = __ffsll(static_cast<long long>(todo)) - 1;
                todo &= todo - 1;
                int cs[kOwn];
                int ntot = 0;
#pragma unroll
                for (int s = 0; s < kOwn; ++s) { cs[s] = __shfl(c[s], src, kWave); ntot += cs[s]; }
                uint64_t* lsel = my_lists + static_cast<size_t>(qw + src) * kQCap;
                auto at = [lsel, &cs](int idx) {
                    int s = 0;
#pragma unroll
                    for (int u = 0; u + 1 < kOwn; ++u)
                        if (s == u && idx >= cs[u]) { idx -= cs[u]; s = u + 1; }
                    return lsel[s * kSubCap + idx];
                };
                wave_select_k<kQCap / kWave>(lsel, at, ntot, a.k, hist + wave * 256);
                if ((lane & 31) == src) {
                    c[0] = a.k;
#pragma unroll
                    for (int s = 1; s < kOwn; ++s) c[s] = 0;
                    n = a.k;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            int base = 0;
            if (lane < 32 && n > 0) base = atomicAdd(&a.gcnt[q0 + ql], n);
            base = __shfl(base, lane & 31, kWave);
            uint64_t* out = a.glist + static_cast<size_t>(q0 + ql) * a.glist_cap;
            int off = base;
#pragma unroll
            for (int s = 0; s < kOwn; ++s) {
                for (int e = half; e < c[s]; e += 2)
                    if (off + e < a.glist_cap) out[off + e] = qlist[s * kSubCap + e];
                off += c[s];
            }
        }
    }
}

// The instances of the row kernel: rows of 128..512 bytes in either wave layout.  (With four waves, one per
// SIMD and 512 registers each, the queries of rows up to 1 KiB fit as well; measured at 1 KiB rows that
// ran 15 % slower than the general kernel - no second wave covers a wave's barrier and filter time.)
typedef void (*RowsKernelFn)(const MineArgs);
struct RowsKernel { RowsKernelFn fn; int nk, wm; };
static const RowsKernel kRowsKernels[] = {
    {&mine_rows_kernel<1, 2>, 1, 2}, {&mine_rows_kernel<2, 2>, 2, 2},
    {&mine_rows_kernel<3, 2>, 3, 2}, {&mine_rows_kernel<4, 2>, 4, 2},
    {&mine_rows_kernel<1, 1>, 1, 1}, {&mine_rows_kernel<2, 1>, 2, 1},
    {&mine_rows_kernel<3, 1>, 3, 1}, {&mine_rows_kernel<4, 1>, 4, 1},
};
static const RowsKernel* find_rows_kernel(int nk, int wm) {
    for (const RowsKernel& k : kRowsKernels)
        if (k.nk == nk && k.wm == wm) return &k;
    return nullptr;
}

__global__ void mine_init_kernel(uint32_t* tau_g, int32_t* gcnt, int64_t n, uint32_t* zeros /* [64] */,
                                 const int32_t* cond) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < 64) zeros[i] = 0u;
    if (i < n && (cond == nullptr || cond[1 + i / kBN] != 0)) { tau_g[i] = kTauInit; gcnt[i] = 0; }
}

// Start of a warm search: the thresholds the previous search left behind, lowered by rel * |tau|,
// are the thresholds of one sweep over all labels.  Whatever they are, the outcome is exact: a query
// that ends the sweep with fewer than k candidates raises the flag of its query tile, and the full
// search is repeated for the flagged tiles.
__global__ void mine_warm_init_kernel(uint32_t* tau_g, int32_t* gcnt, int64_t n, uint32_t* zeros /* [64] */,
                                      int32_t* flag /* [1 + n / kBN] */, float rel) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) {
        const float t = ordered_to_float(tau_g[i]);
        tau_g[i] = float_to_ordered(t - rel * fabsf(t));
        gcnt[i] = 0;
    }
    if (i < 64) zeros[i] = 0u;
    if (i <= n / kBN) flag[i] = 0;
}

// ---------------------------------------------------------------------------
// Radix select for lists too long for registers (n > 64*kSelectRegs): the keys
// are streamed from memory in every pass.  Same result as wave_select_k.
// ---------------------------------------------------------------------------
__device__ __noinline__ float wave_select_stream(uint64_t* __restrict__ buf, int n, int k, int* hist) {
    const int lane = lane_id();
    uint64_t prefix = 0, pmask = 0;
    int need = k;
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
#pragma unroll
        for (int j = 0; j < 4; ++j) hist[lane * 4 + j] = 0;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        for (int idx = lane; idx < n; idx += kWave) {
            const uint64_t key = buf[idx];
            if ((key & pmask) == prefix) atomicAdd(&hist[static_cast<int>((key >> shift) & 255u)], 1);
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
        const int src = __ffsll(static_cast<long long>(bal)) - 1;
        dsel = __shfl(dsel, src, kWave);
        needn = __shfl(needn, src, kWave);
        have = __shfl(have, src, kWave);
        prefix |= static_cast<uint64_t>(dsel) << shift;
        pmask |= 0xffull << shift;
        need = needn;
        if (have == need) break;
    }
    const uint64_t bound = prefix | ~pmask;
    // compaction in place: a chunk is read into registers before anything of it is
    // overwritten, and the write position never passes the read position
    uint64_t kmax = 0;
    int base = 0;
    for (int c0 = 0; c0 < n; c0 += kWave) {
        const int idx = c0 + lane;
        const uint64_t key = idx < n ? buf[idx] : kKeySentinel;
        const bool sel = idx < n && key <= bound;
        const uint64_t m = __ballot(sel);
        const int p = base + __popcll(m & lanemask_lt());
        if (sel && p < k) {
            buf[p] = key;
            kmax = key > kmax ? key : kmax;
        }
        base += __popcll(m);
    }
    kmax = wave_max_u64(kmax);
    return key_score(kmax);
}

// ---------------------------------------------------------------------------
// After a phase: one wave per query cuts the global candidate list to its best
// k and publishes the k-th score as the threshold of the next phase.  After the
// last phase the winners are sorted and written out.
// ---------------------------------------------------------------------------
constexpr int kSelectWaves = 4;

__global__ __launch_bounds__(kSelectWaves * kWave)
void mine_select_kernel(uint64_t* __restrict__ glist, int32_t* __restrict__ gcnt,
                        uint32_t* __restrict__ tau_g, int64_t Zq, int glist_cap, int k, int final_phase,
                        int32_t* __restrict__ shortlist, float* __restrict__ scores,
                        const int32_t* __restrict__ cond /* not null: only query tiles qt with cond[1 + qt] != 0 */,
                        int32_t* __restrict__ short_flag /* not null: [0] and [1 + qt] are set when a query of tile qt
                                                            has fewer than k candidates */) {
    __shared__ int hist[kSelectWaves][256];
    __shared__ uint64_t sorted[kSelectWaves][XC_MAX_K_MINE];
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int64_t q = static_cast<int64_t>(blockIdx.x) * kSelectWaves + wave;
    if (q >= Zq) return;                               // wave-uniform; no workgroup barrier below
    if (cond != nullptr && cond[1 + q / kBN] == 0) return;
    uint64_t* list = glist + static_cast<size_t>(q) * glist_cap;
    int n = gcnt[q];
    n = n < glist_cap ? n : glist_cap;
    if (short_flag != nullptr && n < k && lane == 0) { short_flag[0] = 1; short_flag[1 + q / kBN] = 1; }
    if (n > k) {
        auto at = [list](int idx) { return list[idx]; };
        const float t = (n <= kSelectRegs / 2 * kWave) ? wave_select_k<kSelectRegs / 2>(list, at, n, k, hist[wave])
                        : (n <= kSelectRegs * kWave)   ? wave_select_k<kSelectRegs>(list, at, n, k, hist[wave])
                                                       : wave_select_stream(list, n, k, hist[wave]);
        n = k;
        if (lane == 0) { gcnt[q] = k; tau_g[q] = float_to_ordered(t); }
    }
    if (!final_phase) return;
    // bitonic sort of the (at most 128) winners inside the wave
    uint64_t* srt = sorted[wave];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // the select's stores to `list` are visible
    for (int e = lane; e < XC_MAX_K_MINE; e += kWave) srt[e] = e < n ? list[e] : kKeySentinel;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    for (int size = 2; size <= XC_MAX_K_MINE; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const int t = lane;                       // 64 compare-exchanges cover 128 keys
            const int lo = 2 * t - (t & (stride - 1));
            const int hi = lo + stride;
            const bool up = (lo & size) == 0;
            const uint64_t x = srt[lo], y = srt[hi];
            if ((x > y) == up) { srt[lo] = y; srt[hi] = x; }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        }
    }
    for (int r = lane; r < k; r += kWave) {
        const uint64_t v = srt[r];
        shortlist[q * k + r] = key_id(v);
        if (scores) scores[q * k + r] = (v == kKeySentinel) ? -INFINITY : key_score(v);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct MinePlan {
    int64_t nQT, nLT;
    int kcap, nkb, glist_cap;
    size_t off_flag, off_lists, off_glist, off_gcnt, off_tau, off_zero, ws_bytes;
    size_t lds_tile;
};

static int slices_cap(int kcap) { return kcap <= 64 ? kMaxSlices : kMaxSlices / 2; }    // slices per phase at most

// Number of label tiles of the phase that starts at tile `lo`.  Phases end at powers of the growth
// factor (1, 8, 64, ... tiles seen).  A phase of fewer than 8 tiles deals its items (query tile,
// label tile) to the workgroups in plain order, so it is shortened by up to a third if the number
// of items then comes out just under a multiple of the grid.
static int64_t phase_tiles(int64_t lo, int64_t nQT) {
    if (lo == 0) return 1;
    int64_t end = kPhaseGrowth;
    while (end < 2 * lo) end *= kPhaseGrowth;           // a shortened phase still ends in this decade
    const int64_t want = end - lo;
    if (want >= kXcds) return want;
    int64_t best = want;
    double best_fill = 0.0;
    for (int64_t n = (2 * want + 2) / 3; n <= want; ++n) {
        if (n < 1) continue;
        const int64_t items = nQT * n;
        const int64_t rounds = (items + kMineGrid - 1) / kMineGrid;
        const double fill = static_cast<double>(items) / static_cast<double>(rounds * kMineGrid);
        if (fill >= best_fill) { best_fill = fill; best = n; }
    }
    return best;
}

// Slices per XCD for the kernel that keeps the query tile in registers.  The compute units of an XCD
// that work on one slice read the same stream of W tiles, a few tiles apart, so all but the first find
// them in that XCD's L2: the fewer slices per XCD, the fewer times W comes from memory (with 8 slices
// per XCD the search of 16 384 queries over 120 M rows of 512 bytes ran at the rate the memory system
// delivered W, with one slice 19 % faster).  The other side: 32 / slices query tiles are in flight per
// XCD, and compute units without a query tile idle.  Among the counts the phase allows (<= sx_max) take
// the one that keeps the most compute units busy, and of those the smallest.
static int rows_slices_per_xcd(int64_t nQT, int sx_max) {
    int best = sx_max;
    double best_eff = -1.0;
    for (int sx = 1; sx <= sx_max; sx <<= 1) {
        const int qx = kCusPerXcd / sx;
        const int64_t rounds = (nQT + qx - 1) / qx;
        const double eff = static_cast<double>(nQT) / static_cast<double>(rounds * qx);
        if (eff > best_eff + 1e-9) { best_eff = eff; best = sx; }
    }
    return best;
}

// Work items of 512 queries (the row kernel with all eight waves along the queries) stage half the
// bytes of W per flop; they are taken where padding the pool to a multiple of 512 costs no more than
// padding it to a multiple of 256, or less than a sixteenth of the pool.  XC_MINE_ROWS=narrow or wide
// in the environment (read at every call) overrides the rule, for A/B timing and for tests.
static bool rows_wide_items(int64_t Zq) {
    const char* e = getenv("XC_MINE_ROWS");
    if (e != nullptr && e[0] == 'n') return false;
    if (e != nullptr && e[0] == 'w') return true;
    const int64_t pad_w = (Zq + 2 * kBN - 1) / (2 * kBN) * (2 * kBN) - Zq;
    const int64_t pad_n = (Zq + kBN - 1) / kBN * kBN - Zq;
    return pad_w <= pad_n || pad_w * 16 <= Zq;
}

static int plan_mine(int64_t Zq, int64_t L, int d, int k_h, xc_dtype t, MinePlan* p) {
    if (t != XC_F32 && t != XC_BF16) return XC_EDTYPE;
    if (Zq < 1 || L < 1 || d < 1 || k_h < 1 || k_h > XC_MAX_K_MINE || k_h > L) return XC_ESHAPE;
    const int64_t row_bytes = static_cast<int64_t>(d) * (t == XC_F32 ? 4 : 2);
    if (row_bytes % 16 != 0 || row_bytes > (1 << 20)) return XC_ESHAPE;
    if (L > 0x7fffffffLL || Zq > 0x7fffffffLL) return XC_ESHAPE;
    int kcap = 8;
    while (kcap < k_h) kcap <<= 1;
    p->kcap = kcap;
    p->nkb = static_cast<int>((row_bytes + kStageBytes - 1) / kStageBytes);
    p->nQT = (Zq + kBN - 1) / kBN;
    p->nLT = (L + kBM - 1) / kBM;
    // a phase appends at most kcap keys per slice to a list that holds at most k keys
    p->glist_cap = kcap * (slices_cap(kcap) + 1);
    size_t off = 0;
    auto take = [&off](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
    const size_t nq = static_cast<size_t>(p->nQT) * kBN;
    // first word: 1 if the last warm search had to repeat the full search for some query tile; then one word per tile
    p->off_flag = take(4 * (static_cast<size_t>(p->nQT) + 1));
    p->off_lists = take(static_cast<size_t>(kMineGrid) * kBN * kCandCap * sizeof(uint64_t));
    p->off_glist = take(nq * p->glist_cap * sizeof(uint64_t));
    p->off_gcnt = take(nq * sizeof(int32_t));
    p->off_tau = take(nq * sizeof(uint32_t));
    p->off_zero = take(256);
    p->ws_bytes = off;
    p->lds_tile = 2 * static_cast<size_t>(kBM + kBN) * kStageBytes + kBN * 8 + kMineWaves * 256 * 4 +
                  static_cast<size_t>(kMineWaves) * kPool * 8 + 16;
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

namespace xc {
// The search proper.  warm: one sweep with the thresholds found in the workspace (lowered by
// rel_margin * |tau|), then the full search if some query came out short; the kernels of the full
// search are enqueued in any case and return at once when the flag says they are not needed.
static int run_mine(const void* Z, const void* W, int64_t Zq, int64_t L, int d, int k_h, xc_dtype t,
                    bool warm, float rel_margin, int32_t* shortlist, float* scores, void* ws,
                    size_t ws_bytes, void* stream) {
    MinePlan p;
    const int rc = plan_mine(Zq, L, d, k_h, t, &p);
    if (rc != XC_OK) return rc;
    if (!Z || !W || !shortlist || !ws) return XC_EINVAL;
    if (warm && !(rel_margin >= 0.0f)) return XC_EINVAL;
    if (!aligned16(Z) || !aligned16(W) || !aligned16(ws)) return XC_EINVAL;
    if (ws_bytes < p.ws_bytes) return XC_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* w8 = static_cast<unsigned char*>(ws);
    MineArgs a;
    a.Z = static_cast<const unsigned char*>(Z);
    a.W = static_cast<const unsigned char*>(W);
    a.Zq = Zq; a.L = L;
    a.row_bytes = static_cast<int64_t>(d) * (t == XC_F32 ? 4 : 2);
    a.k = k_h; a.kcap = p.kcap; a.nkb = p.nkb;
    a.nQT = p.nQT;
    a.glist_cap = p.glist_cap;
    a.lists = reinterpret_cast<uint64_t*>(w8 + p.off_lists);
    a.glist = reinterpret_cast<uint64_t*>(w8 + p.off_glist);
    a.gcnt = reinterpret_cast<int32_t*>(w8 + p.off_gcnt);
    uint32_t* tau_g = reinterpret_cast<uint32_t*>(w8 + p.off_tau);
    a.tau_g = tau_g;
    a.zeros = w8 + p.off_zero;
    a.cond = nullptr;
    int32_t* flag = reinterpret_cast<int32_t*>(w8 + p.off_flag);

    // raise the dynamic LDS limit of the tile kernels: once per device and process (the attribute
    // belongs to the device's copy of the kernel)
    static std::mutex attr_mu;
    static uint64_t attr_done_mask = 0;          // bit = device ordinal (< 64)
    {
        int dev = 0;
        XC_HIP_CHECK(hipGetDevice(&dev));
        std::lock_guard<std::mutex> lock(attr_mu);
        if (dev < 0 || dev >= 64 || !(attr_done_mask & (1ull << dev))) {
            const void* fns[4] = {reinterpret_cast<const void*>(&mine_tile_kernel<bf16_t, false>),
                                  reinterpret_cast<const void*>(&mine_tile_kernel<bf16_t, true>),
                                  reinterpret_cast<const void*>(&mine_tile_kernel<float, false>),
                                  reinterpret_cast<const void*>(&mine_tile_kernel<float, true>)};
            for (const void* fn : fns)
                XC_HIP_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 static_cast<int>(p.lds_tile)));
            for (const RowsKernel& k : kRowsKernels)
                XC_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(k.fn),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 static_cast<int>(rows_lds_bytes(k.wm))));
            if (dev >= 0 && dev < 64) attr_done_mask |= 1ull << dev;
        }
    }
    const int64_t nq = p.nQT * kBN;
    const dim3 init_grid(static_cast<unsigned>((nq + 255) / 256));
    const dim3 select_grid(static_cast<unsigned>((Zq + kSelectWaves - 1) / kSelectWaves));
    uint32_t* zeros32 = reinterpret_cast<uint32_t*>(w8 + p.off_zero);

    // one phase: the tile kernel over label tiles [lo, hi), then the select
    auto phase = [&](int64_t lo, int64_t hi, const int32_t* cond, int32_t* short_flag) -> int {
        const int64_t nT = hi - lo;
        // bf16 rows of whole stages whose queries fit a wave's registers take the row kernel: work items of
        // 512 queries where the pool fills them about as well as items of 256
        const RowsKernel* rk = nullptr;
        if (t == XC_BF16 && a.row_bytes % kStageBytes == 0 && !force_general_kernel()) {
            const int nk = static_cast<int>(a.row_bytes / kStageBytes);
            rk = find_rows_kernel(nk, rows_wide_items(Zq) ? 1 : 2);
        }
        const bool rows_kernel = rk != nullptr;
        a.nQT = rows_kernel ? (Zq + 2 * kBN / rk->wm - 1) / (2 * kBN / rk->wm) : p.nQT;
        if (nT >= kXcds) {
            // slices per XCD: as many as the phase supports, so that few query tiles are in
            // flight per XCD and their Z rows stay in that XCD's L2
            int Sx = 8;
            while (Sx > 1 && (nT < static_cast<int64_t>(kXcds) * Sx || kXcds * Sx > slices_cap(p.kcap))) Sx >>= 1;
            if (rows_kernel) Sx = rows_slices_per_xcd(a.nQT, Sx);
            a.S = kXcds * Sx;
            a.Qx = kCusPerXcd / Sx;
        } else {                                           // a few tiles: one slice per tile, plain order
            a.S = static_cast<int>(nT);
            a.Qx = 0;
        }
        a.tile_lo = lo; a.tile_hi = hi;
        a.tiles_per_slice = (nT + a.S - 1) / a.S;
        a.append_max = (p.glist_cap - p.kcap) / a.S;
        if (a.append_max > kCandCap) a.append_max = kCandCap;
        a.cond = cond;
        const bool ktail = (a.row_bytes % kStageBytes) != 0;
        if (rows_kernel) {
            // the query tile stays in registers, only W is streamed
            XC_LAUNCH(K_MINE_TILE, st, (rk->fn<<<kMineGrid, kMineThreads, rows_lds_bytes(rk->wm), st>>>(a)));
        } else if (t == XC_BF16) {
            if (ktail) XC_LAUNCH(K_MINE_TILE, st, (mine_tile_kernel<bf16_t, true><<<kMineGrid, kMineThreads, p.lds_tile, st>>>(a)));
            else XC_LAUNCH(K_MINE_TILE, st, (mine_tile_kernel<bf16_t, false><<<kMineGrid, kMineThreads, p.lds_tile, st>>>(a)));
        } else {
            if (ktail) XC_LAUNCH(K_MINE_TILE, st, (mine_tile_kernel<float, true><<<kMineGrid, kMineThreads, p.lds_tile, st>>>(a)));
            else XC_LAUNCH(K_MINE_TILE, st, (mine_tile_kernel<float, false><<<kMineGrid, kMineThreads, p.lds_tile, st>>>(a)));
        }
        XC_HIP_CHECK(hipGetLastError());
        const int final_phase = hi == p.nLT ? 1 : 0;
        XC_LAUNCH(K_MINE_SELECT, st, (mine_select_kernel<<<select_grid, kSelectWaves * kWave, 0, st>>>(
            a.glist, a.gcnt, tau_g, Zq, p.glist_cap, k_h, final_phase, shortlist, scores, cond, short_flag)));
        XC_HIP_CHECK(hipGetLastError());
        return XC_OK;
    };

    const int32_t* cond = nullptr;
    if (warm) {
        mine_warm_init_kernel<<<init_grid, 256, 0, st>>>(tau_g, a.gcnt, nq, zeros32, flag, rel_margin);
        XC_HIP_CHECK(hipGetLastError());
        const int rcw = phase(0, p.nLT, nullptr, flag);
        if (rcw != XC_OK) return rcw;
        cond = flag;
    }
    mine_init_kernel<<<init_grid, 256, 0, st>>>(tau_g, a.gcnt, nq, zeros32, cond);
    XC_HIP_CHECK(hipGetLastError());
    int64_t lo = 0;
    while (lo < p.nLT) {
        // phases end at about 1, 8, 64, ... tiles: each sees about 8x the labels seen before it
        int64_t hi = lo + phase_tiles(lo, p.nQT);
        if (hi > p.nLT || p.nLT - hi < hi / 4) hi = p.nLT;      // fold a short remainder into this phase
        const int rcp = phase(lo, hi, cond, nullptr);
        if (rcp != XC_OK) return rcp;
        lo = hi;
    }
    return XC_OK;
}
}  // namespace xc

extern "C" int xc_mine_negatives(const void* Z, const void* W, int64_t Zq, int64_t L, int d, int k_h,
                                 xc_dtype t, int32_t* shortlist, float* scores, void* ws,
                                 size_t ws_bytes, void* stream) {
    return xc::run_mine(Z, W, Zq, L, d, k_h, t, false, 0.0f, shortlist, scores, ws, ws_bytes, stream);
}

extern "C" int xc_mine_negatives_warm(const void* Z, const void* W, int64_t Zq, int64_t L, int d, int k_h,
                                      xc_dtype t, float rel_margin, int32_t* shortlist, float* scores,
                                      void* ws, size_t ws_bytes, void* stream) {
    return xc::run_mine(Z, W, Zq, L, d, k_h, t, true, rel_margin, shortlist, scores, ws, ws_bytes, stream);
}
