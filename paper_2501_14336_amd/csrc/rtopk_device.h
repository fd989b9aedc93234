// Device-side building blocks of the radix top-k kernels (gfx950, wave64).
//
// Notation follows the paper: X input row, n its length, k, digit width d, radix r = 2^d,
// candidates, bin, histogram, pivot (Section 2.3.1, Algorithm 1).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "rtopk.h"

namespace rtopk {

typedef uint32_t u32;
typedef uint64_t u64;

constexpr int kMaxBins = 4096;            // r for d = 12, the widest digit (Section 5.2 uses d = 12)
constexpr int kSwgStride = kMaxBins + 8;  // per-workgroup suffix-sum record: r + 1 entries, padded
constexpr int kMaxPasses = RTOPK_TRACE_MAX_PASSES;

enum { SRC_SCALED = 0, SRC_KEY = 1, SRC_IDX = 2, SRC_RUNTIME = -1 };

// One digit pass: bits [shift, shift + bits) of the 32-bit ordered key of `src`.
struct PassInfo {
    u32 src, shift, bits;
};

// Kernel arguments (passed by value).
struct Params {
    const void* keys;        // X, [batch][n]
    void* out_values;        // Y values, [batch][k]
    long long* out_indices;  // Y indices, [batch][k]
    rtopk_row_trace* state;  // per-row loop state + trace, stride RTOPK_TRACE_STRIDE bytes
    u32* ghist;              // [2][batch][kMaxBins]  global histogram, one buffer per pass parity
    u32* bases;              // [batch][G][2]       per-workgroup output / candidate write offsets
    u32* swg;                // [batch][G][kSwgStride]  per-workgroup suffix sums of its local histogram
    uint2* cand[2];          // [batch][n]          (raw bits, index) candidates, ping-pong
    long long n, k;
    int batch, G;
    u32 dirmask;             // 0 for "largest"; all key bits set for "smallest" (complements the key)
    u32 idx_max;             // 2^ceil(log2 n) - 1: the index digit source is idx_max - index
    u32 small;               // candidate count at or below which one workgroup finishes the row
    int npass;
    u32 flags;
    u64 seed;
    PassInfo pass[kMaxPasses];
};

__device__ __forceinline__ rtopk_row_trace* row_state(const Params& P, int row) {
    return (rtopk_row_trace*)((char*)P.state + (size_t)row * RTOPK_TRACE_STRIDE);
}

// ------------------------------------------------------------------------------------------------
// wave64 helpers
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ u32 lane_id() {
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}
// number of set bits of m below this lane
__device__ __forceinline__ u32 mbcnt64(u64 m) {
    return __builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u));
}
__device__ __forceinline__ u64 ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// ------------------------------------------------------------------------------------------------
// order-preserving keys (the paper treats elements as bit strings, Section 5.2, and notes the sign bit
// is the most significant one, Section 4.2; raw IEEE bits do not order negatives, so: flip all bits of
// negatives, set the sign bit of non-negatives, send every NaN to the all-ones key).
// 16-bit keys are returned in the UPPER half of the word so digit windows are the same for all types.
// ------------------------------------------------------------------------------------------------
template <int DT>
struct KeyOf;
template <>
struct KeyOf<RTOPK_F32> {
    static constexpr int kBytes = 4;
    __device__ static __forceinline__ u32 key(u32 b) {
        u32 m = (u32)((int32_t)b >> 31) | 0x80000000u;
        u32 u = b ^ m;
        return ((b & 0x7fffffffu) > 0x7f800000u) ? 0xffffffffu : u;
    }
};
template <>
struct KeyOf<RTOPK_F16> {
    static constexpr int kBytes = 2;
    __device__ static __forceinline__ u32 key(u32 h) {
        u32 m = (h & 0x8000u) ? 0xffffu : 0x8000u;
        u32 u = (h ^ m) & 0xffffu;
        u = ((h & 0x7fffu) > 0x7c00u) ? 0xffffu : u;
        return u << 16;
    }
};
template <>
struct KeyOf<RTOPK_BF16> {
    static constexpr int kBytes = 2;
    __device__ static __forceinline__ u32 key(u32 h) {
        u32 m = (h & 0x8000u) ? 0xffffu : 0x8000u;
        u32 u = (h ^ m) & 0xffffu;
        u = ((h & 0x7fffu) > 0x7f80u) ? 0xffffu : u;
        return u << 16;
    }
};

// Digit of one (raw bits, index) element for a pass.
//   SRC_KEY     ordered key of the element
//   SRC_SCALED  ordered key of fl(x - a_s), fp32 only (adaptive scaling, Section 4.3)
//   SRC_IDX     idx_max - index, so that among equal keys the lowest index ranks best
template <int DT, int SRC>
__device__ __forceinline__ u32 digit_of(const PassInfo pi, u32 raw, u32 idx, u32 dirmask, u32 idx_max, float a_s) {
    const int src = (SRC == SRC_RUNTIME) ? (int)pi.src : SRC;
    u32 u;
    if (src == SRC_IDX) {
        u = idx_max - idx;
    } else if (src == SRC_KEY) {
        u = KeyOf<DT>::key(raw) ^ dirmask;
    } else {
        float y = __uint_as_float(raw) - a_s;
        u = KeyOf<RTOPK_F32>::key(__float_as_uint(y)) ^ dirmask;
    }
    return (u >> pi.shift) & ((1u << pi.bits) - 1u);
}

// ------------------------------------------------------------------------------------------------
// tile sources.  A tile is B*V 16-byte vectors; lane t of the workgroup owns vectors t, t+B, ...
// so that every load instruction of a wave covers 1 KiB of consecutive addresses.
// ------------------------------------------------------------------------------------------------

// Registers of one lane's share of a tile.
template <int V>
struct TileRegs {
    uint4 r[V];
    u32 e0[V];  // index of element 0 of each vector (row index for X, position for candidates)
    bool full;  // every element of the tile is valid
};

// The input row X.  Loads start at the 16-byte aligned address at or before the row's first element
// and elements outside [0, n) are masked (on-demand offset padding, Section 3.2.2).
template <int DT, int B, int V>
struct KeySource {
    static constexpr int kElemBytes = KeyOf<DT>::kBytes;
    static constexpr int E = 16 / kElemBytes;  // elements per vector
    static constexpr int kSlots = V * E;       // elements per lane per tile
    static constexpr int kTileVecs = B * V;
    typedef TileRegs<V> Tile;

    const uint4* abase;
    u32 lead;  // elements between abase and the row's first element
    u32 n;
    u64 nvec;  // vectors covering [abase, row end)

    __device__ __forceinline__ void init(const void* keys, long long n_, int row) {
        const char* p = (const char*)keys + (size_t)row * (size_t)n_ * kElemBytes;
        uintptr_t a = (uintptr_t)p;
        abase = (const uint4*)(a & ~(uintptr_t)15);
        lead = (u32)((a & 15) / kElemBytes);
        n = (u32)n_;
        nvec = ((u64)lead + (u64)n + E - 1) / E;
    }
    __device__ __forceinline__ u32 ntiles() const { return (u32)((nvec + kTileVecs - 1) / kTileVecs); }
    __device__ __forceinline__ void load(u32 tile, u32 tid, Tile& t) const {
        u64 v0 = (u64)tile * kTileVecs;
        t.full = (tile != 0 || lead == 0) && ((v0 + kTileVecs) * E <= (u64)lead + (u64)n);
#pragma unroll
        for (int u = 0; u < V; ++u) {
            u64 v = v0 + (u64)u * B + tid;
            t.e0[u] = (u32)(v * E) - lead;
            if (t.full || v < nvec)
                t.r[u] = abase[v];
            else
                t.r[u] = make_uint4(0, 0, 0, 0);
        }
    }
    __device__ __forceinline__ void get(const Tile& t, int s, u32& raw, u32& idx, bool& valid) const {
        const int u = s / E, j = s % E;
        idx = t.e0[u] + j;
        valid = t.full || idx < n;  // the lead-in wraps to huge values, vectors past the end start at >= n
        const uint4 q = t.r[u];
        if (E == 4) {
            raw = j == 0 ? q.x : j == 1 ? q.y : j == 2 ? q.z : q.w;
        } else {
            const int w = j >> 1;
            u32 word = w == 0 ? q.x : w == 1 ? q.y : w == 2 ? q.z : q.w;
            raw = (j & 1) ? (word >> 16) : (word & 0xffffu);
        }
    }
};

// A candidate array of (raw bits, index) pairs, two per vector.
template <int B, int V>
struct CandSource {
    static constexpr int E = 2;
    static constexpr int kSlots = V * E;
    static constexpr int kTileVecs = B * V;
    typedef TileRegs<V> Tile;

    const uint4* base;
    u32 count;
    u64 nvec;

    __device__ __forceinline__ void init(const uint2* c, u32 count_) {
        base = (const uint4*)c;
        count = count_;
        nvec = ((u64)count_ + 1) / 2;
    }
    __device__ __forceinline__ u32 ntiles() const { return (u32)((nvec + kTileVecs - 1) / kTileVecs); }
    __device__ __forceinline__ void load(u32 tile, u32 tid, Tile& t) const {
        u64 v0 = (u64)tile * kTileVecs;
        t.full = (v0 + kTileVecs) * E <= (u64)count;
#pragma unroll
        for (int u = 0; u < V; ++u) {
            u64 v = v0 + (u64)u * B + tid;
            t.e0[u] = (u32)(v * E);
            if (t.full || v < nvec)
                t.r[u] = base[v];
            else
                t.r[u] = make_uint4(0, 0, 0, 0);
        }
    }
    __device__ __forceinline__ void get(const Tile& t, int s, u32& raw, u32& idx, bool& valid) const {
        const int u = s / E, j = s % E;
        valid = t.full || (t.e0[u] + j) < count;
        raw = j ? t.r[u].z : t.r[u].x;
        idx = j ? t.r[u].w : t.r[u].y;
    }
};

// ------------------------------------------------------------------------------------------------
// workgroup-wide scans
// ------------------------------------------------------------------------------------------------

// Inclusive prefix sum of v over the workgroup's threads.  wsum: LDS, B/64 words.  Contains barriers.
template <int B>
__device__ __forceinline__ u32 block_inclusive_scan(u32 v, u32* wsum) {
    const u32 lane = lane_id();
    const u32 wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        u32 t = __shfl_up(v, o, 64);
        if (lane >= (u32)o) v += t;
    }
    if (lane == 63) wsum[wave] = v;
    __syncthreads();
    u32 add = 0;
    for (u32 w = 0; w < wave; ++w) add += wsum[w];
    __syncthreads();
    return v + add;
}

// Sums of a and b over the workgroup, returned to every thread.  red: LDS, 2 * B/64 words.  Contains barriers.
template <int B>
__device__ __forceinline__ void block_sum2(u32& a, u32& b, u32* red) {
    const u32 lane = lane_id();
    const u32 wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        a += __shfl_down(a, o, 64);
        b += __shfl_down(b, o, 64);
    }
    if (lane == 0) { red[2 * wave] = a; red[2 * wave + 1] = b; }
    __syncthreads();
    u32 sa = 0, sb = 0;
#pragma unroll
    for (int w = 0; w < B / 64; ++w) { sa += red[2 * w]; sb += red[2 * w + 1]; }
    __syncthreads();
    a = sa;
    b = sb;
}

// In place: h[j] <- sum of h[i] for i >= j  (number of candidates whose digit is at least j).
template <int B>
__device__ __forceinline__ void suffix_sums_in_place(u32* h, int nb, u32* wsum) {
    const int ipt = (nb + B - 1) / B;
    const int r0 = threadIdx.x * ipt;  // position counted from the TOP bin
    u32 s = 0;
    for (int i = 0; i < ipt; ++i) {
        int r = r0 + i;
        if (r < nb) s += h[nb - 1 - r];
    }
    u32 run = block_inclusive_scan<B>(s, wsum) - s;
    for (int i = 0; i < ipt; ++i) {
        int r = r0 + i;
        if (r < nb) {
            run += h[nb - 1 - r];
            h[nb - 1 - r] = run;
        }
    }
    __syncthreads();
}

// selectBin (Section 2.3.1): given suffix sums S in LDS, the bin b with S[b+1] < k <= S[b].
// *sel is an LDS word.  Returns b to every thread; contains barriers.
template <int B>
__device__ __forceinline__ u32 select_bin(const u32* S, int nb, u32 k, u32* sel) {
    if (threadIdx.x == 0) *sel = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < nb; j += B) {
        u32 sj = S[j];
        u32 sn = (j + 1 < nb) ? S[j + 1] : 0u;
        if (sj >= k && sn < k) *sel = (u32)j;
    }
    __syncthreads();
    return *sel;
}

// countBin's inner step (Section 3.1.1): add one element to the workgroup-local histogram.
// Lanes holding the same digit as the wave's first active lane are merged into one LDS atomic
// (register-level aggregation, the "warp" level of the paper's Table 1); everything else goes
// straight to the LDS atomic (the "block" level).  Called by the lanes that hold a valid element.
__device__ __forceinline__ void hist_add(u32* h, u32 dg) {
    const u32 d0 = __builtin_amdgcn_readfirstlane(dg);
    const bool same = dg == d0;
    const u64 m = ballot64(same);
    const u32 cnt = (u32)__popcll(m);
    const bool leader = mbcnt64(m) == 0;  // lowest lane of the merged group
    if (!same || leader) atomicAdd(&h[dg], same ? cnt : 1u);
}

}  // namespace rtopk
