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
constexpr u32 kInternalStream = 1u << 31;  // Params::flags: the input is much larger than the last-level cache
constexpr int kStageCap = 256;             // entries per wave in each LDS write buffer (Section 3.1.2)

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
    u32* ghist;              // [6][batch][kMaxBins]  global histograms: a ring of four for the passes, the sample's, the prefilter's second
    u32* seg;                // [2][batch][G][2]    (start, count) of the candidates each workgroup wrote, per candidate array
    u32* swg;                // [4][batch][G][kSwgStride]  per-workgroup suffix sums of its local histogram: a ring of three, the prefilter's second
    uint2* cand[2];          // [batch][n]          (raw bits, index) candidates, ping-pong
    unsigned long long* dbg; // [batch][G][16]      optional per-workgroup timestamps (diagnostic builds only)
    u32* sort_hist;          // [batch][256][Gs]    sorted output of long rows: per-chunk digit counts, then offsets
    void* sort_state;        // [batch] records of 128 bytes: which array holds the keys, which passes are skipped
    long long n, k;          // row length and k; with row_offsets: the LARGEST row length and k (outputs are [batch][k] either way)
    const long long* row_offsets;  // ragged batch (device, batch + 1 entries, in elements): row r is keys[row_offsets[r] .. row_offsets[r+1]); else null
    const long long* row_k;        // ragged batch (device, batch entries): k of every row
    int batch, G, Gs;
    u32 dirmask;             // 0 for "largest"; all key bits set for "smallest" (complements the key)
    u32 idx_max;             // 2^ceil(log2 n) - 1: the index digit source is idx_max - index
    u32 small;               // candidate count at or below which one workgroup finishes the row
    int npass;
    u32 flags;               // RTOPK_FLAG_* | kInternalStream
    u32 keep_from_tile;      // streamed inputs: the first sweep reads tiles from this one on with ordinary loads
    u32 pre_stride;          // 0, or: a prefilter sweep stands before pass 0; a row's sample is every pre_stride-th full tile
    size_t cand_stride;      // entries per row of the candidate arrays
    u64 seed;
    PassInfo pass[kMaxPasses];
};

__device__ __forceinline__ rtopk_row_trace* row_state(const Params& P, int row) {
    return (rtopk_row_trace*)((char*)P.state + (size_t)row * RTOPK_TRACE_STRIDE);
}

// One row of the batch: where its elements start, how many there are, how many are wanted.  A batch is either
// [batch][n] with one k, or ragged (Section 3.2.2): rows of any length one after the other in one array, each with
// its own k.  In a ragged batch a row with k = 0 (or no elements) is skipped by every kernel; a k beyond the row's
// length or beyond the output row is cut down to it and reported in the row's record (error bit 8).
struct RowShape {
    const char* x;
    u32 n, k;
    bool bad;
};
template <int ELEM_BYTES>
__device__ __forceinline__ RowShape row_shape(const Params& P, int row) {
    RowShape r;
    r.bad = false;
    if (P.row_offsets) {
        const long long o0 = P.row_offsets[row], o1 = P.row_offsets[row + 1];
        long long n = o1 - o0, k = P.row_k[row];
        if (n < 0 || n > P.n) { r.bad = true; n = n < 0 ? 0 : P.n; }
        if (k < 0 || k > n || k > P.k) { r.bad = true; k = k < 0 ? 0 : (n < P.k ? n : P.k); }
        r.x = (const char*)P.keys + (size_t)o0 * ELEM_BYTES;
        r.n = (u32)n;
        r.k = (u32)k;
    } else {
        r.x = (const char*)P.keys + (size_t)row * (size_t)P.n * ELEM_BYTES;
        r.n = (u32)P.n;
        r.k = (u32)P.k;
    }
    return r;
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
    return (u >> pi.shift) & (pi.bits >= 32u ? 0xffffffffu : (1u << pi.bits) - 1u);
}

// Everything a kernel needs to turn elements into digits of one pass, as wave-uniform scalars.
// The last four fields drive the branch-free key of the first pass over X:
//   key = b ^ (((b >>arith 31) ^ xd) & am | om), NaN -> nanv
// which is the ordered key for "largest" (xd 0, am ~0, om sign bit) and its complement for
// "smallest" (xd ~0, am ~sign bit, om 0), without a separate direction step.
struct DigitCtx {
    PassInfo pi;
    u32 dirmask, idx_max;
    float a_s;
    u32 xd, am, om, nanv;
};

__device__ __forceinline__ DigitCtx make_digit_ctx(const Params& P, int p, float a_s) {
    DigitCtx c;
    c.pi = P.pass[p];
    c.dirmask = P.dirmask;
    c.idx_max = P.idx_max;
    c.a_s = a_s;
    const bool largest = P.dirmask == 0;
    c.xd = largest ? 0u : 0xffffffffu;
    c.am = largest ? 0xffffffffu : 0x7fffffffu;
    c.om = largest ? 0x80000000u : 0u;
    c.nanv = largest ? 0xffffffffu : 0u;
    return c;
}

// ------------------------------------------------------------------------------------------------
// tile sources.  A tile is B*V 16-byte vectors; lane t of the workgroup owns vectors t, t+B, ...
// so that every load instruction of a wave covers 1 KiB of consecutive addresses.
// ------------------------------------------------------------------------------------------------

typedef u32 u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* global_vec_ptr;
// 16-byte load from global memory (explicitly global, so that it counts on the vector-memory
// counter only and never waits for LDS traffic).  NT: the data is far larger than the last-level
// cache and is streamed with non-temporal loads so that it does not displace what is reused.
template <bool NT>
__device__ __forceinline__ uint4 load16(const uint4* p) {
    const global_vec_ptr g = (global_vec_ptr)p;
    const u32x4 v = NT ? __builtin_nontemporal_load(g) : *g;
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Registers of one lane's share of a tile.
template <int V>
struct TileRegs {
    uint4 r[V];
    u32 tile;   // tile number (wave-uniform)
    bool full;  // every element of the tile is valid (wave-uniform)
};

// The input row X.  Loads start at the 16-byte aligned address at or before the row's first element
// and elements outside [0, n) are masked (on-demand offset padding, Section 3.2.2).
template <int DT, int B, int V, bool NT>
struct KeySource {
    static constexpr int kElemBytes = KeyOf<DT>::kBytes;
    static constexpr int E = 16 / kElemBytes;  // elements per vector
    static constexpr int kSlots = V * E;       // elements per lane per tile
    static constexpr int kTileVecs = B * V;
    static constexpr bool kStreams = NT;
    typedef TileRegs<V> Tile;

    const uint4* abase;
    u32 lead;  // elements between abase and the row's first element
    u32 n;
    u64 nvec;  // vectors covering [abase, row end)

    __device__ __forceinline__ void init(const RowShape& rs) {
        uintptr_t a = (uintptr_t)rs.x;
        const u32 n_ = rs.n;
        abase = (const uint4*)(a & ~(uintptr_t)15);
        lead = (u32)((a & 15) / kElemBytes);
        n = (u32)n_;
        nvec = ((u64)lead + (u64)n + E - 1) / E;
    }
    __device__ __forceinline__ u32 ntiles() const { return (u32)((nvec + kTileVecs - 1) / kTileVecs); }
    // tiles [f0, f1) contain only elements of the row
    __device__ __forceinline__ void full_range(u32& f0, u32& f1) const {
        f0 = lead != 0 ? 1u : 0u;
        f1 = (u32)(((u64)lead + (u64)n) / ((u64)kTileVecs * E));
        if (f1 < f0) f1 = f0;
    }
    __device__ __forceinline__ void load_full(u32 tile, u32 tid, Tile& t) const {
        const u64 v0 = (u64)tile * kTileVecs;
        t.tile = tile;
        t.full = true;
#pragma unroll
        for (int u = 0; u < V; ++u) t.r[u] = load16<NT>(abase + (v0 + (u64)u * B + tid));
    }
    // The same row read with ordinary (cache-allocating) loads.
    __device__ __forceinline__ KeySource<DT, B, V, false> plain() const {
        KeySource<DT, B, V, false> p;
        p.abase = abase;
        p.lead = lead;
        p.n = n;
        p.nvec = nvec;
        return p;
    }
    __device__ __forceinline__ void load(u32 tile, u32 tid, Tile& t) const {
        u64 v0 = (u64)tile * kTileVecs;
        t.tile = tile;
        t.full = (tile != 0 || lead == 0) && ((v0 + kTileVecs) * E <= (u64)lead + (u64)n);
#pragma unroll
        for (int u = 0; u < V; ++u) {
            u64 v = v0 + (u64)u * B + tid;
            if (t.full || v < nvec)
                t.r[u] = load16<NT>(abase + v);
            else
                t.r[u] = make_uint4(0, 0, 0, 0);
        }
    }
    // Digits of the E elements of vector u for the FIRST pass, whose digit is the key's top bits
    // (pi.shift + pi.bits == 32).  SRC is SRC_KEY or, fp32 only, SRC_SCALED.
    template <int SRC>
    __device__ __forceinline__ void digits(const Tile& t, int u, const DigitCtx& c, u32 (&dg)[E]) const {
        const uint4 q = t.r[u];
        const u32 w[4] = {q.x, q.y, q.z, q.w};
        if (E == 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u32 b = w[j];
                if (SRC == SRC_SCALED) b = __float_as_uint(__uint_as_float(b) - c.a_s);
                const u32 sgn = (u32)((int32_t)b >> 31);
                u32 key = b ^ (((sgn ^ c.xd) & c.am) | c.om);
                const float f = __uint_as_float(b);
                key = (f != f) ? c.nanv : key;
                dg[j] = key >> c.pi.shift;
            }
        } else {
            // two 16-bit keys per word, transformed together
            const u32 thr = (DT == RTOPK_F16) ? 0x03ff03ffu : 0x007f007fu;  // 0x7fff - (largest non-NaN magnitude)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32 x = w[j];
                const u32 sb = x & 0x80008000u;
                u32 key = x ^ ((sb - (sb >> 15)) | 0x80008000u);          // negatives: all bits, others: sign bit
                const u32 nb = ((x & 0x7fff7fffu) + thr) & 0x80008000u;  // bit 15 of a half set iff it is NaN
                key |= (nb - (nb >> 15)) | nb;                            // NaN halves -> 0xffff
                key ^= c.xd;                                               // "smallest": complement
                dg[2 * j] = (key & 0xffffu) >> (c.pi.shift - 16);
                dg[2 * j + 1] = key >> c.pi.shift;
            }
        }
    }
    // Digits of the E elements of vector u for ANY pass (source and window chosen at run time): the sweeps over X
    // that come after an in-place pass.
    template <int DT2>
    __device__ __forceinline__ void digits_of_pass(const Tile& t, int u, const DigitCtx& c, u32 (&dg)[E]) const {
#pragma unroll
        for (int j = 0; j < E; ++j) {
            u32 raw, idx;
            bool valid;
            get(t, u * E + j, raw, idx, valid);
            dg[j] = digit_of<DT2, SRC_RUNTIME>(c.pi, raw, idx, c.dirmask, c.idx_max, c.a_s);
        }
    }
    // Element s of the tile as an fp32 number that orders like the element (exact widening for
    // 16-bit types; x - a_s under scaling).  NaN stays NaN.
    template <int SRC>
    __device__ __forceinline__ float value(const Tile& t, int s, float a_s) const {
        const int u = s / E, j = s % E;
        const uint4 q = t.r[u];
        if (E == 4) {
            const float f = __uint_as_float(j == 0 ? q.x : j == 1 ? q.y : j == 2 ? q.z : q.w);
            return SRC == SRC_SCALED ? f - a_s : f;
        } else {
            const int w = j >> 1;
            const u32 word = w == 0 ? q.x : w == 1 ? q.y : w == 2 ? q.z : q.w;
            if (DT == RTOPK_BF16) {
                return __uint_as_float((j & 1) ? (word & 0xffff0000u) : (word << 16));
            } else {
                const uint16_t h = (uint16_t)((j & 1) ? (word >> 16) : word);
                return (float)__builtin_bit_cast(_Float16, h);
            }
        }
    }
    __device__ __forceinline__ void get(const Tile& t, int s, u32& raw, u32& idx, bool& valid) const {
        const int u = s / E, j = s % E;
        // row index of the element; the lead-in wraps to huge values, vectors past the end start at >= n
        idx = (t.tile * (u32)kTileVecs + (u32)(u * B) + threadIdx.x) * (u32)E + (u32)j - lead;
        valid = t.full || idx < n;
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

// A segment [start, start + count) of a candidate array of (raw bits, index) pairs, two per 16-byte vector.
// Loads start at the even entry at or before `start`; the lead-in entry is masked.
template <int B, int V>
struct CandSource {
    static constexpr int E = 2;
    static constexpr int kSlots = V * E;
    static constexpr int kTileVecs = B * V;
    typedef TileRegs<V> Tile;

    const uint4* base;  // vector holding entry `start`
    u32 lead;           // 1 if `start` is odd
    u32 count;
    u64 nvec;

    // cap: entries in the array.  The segment is clipped to it, so that counts from an inconsistent run (which
    // sets the row's error flag elsewhere) can never send a load outside the workspace.
    __device__ __forceinline__ void init(const uint2* c, u32 start, u32 count_, u32 cap) {
        if (start > cap) start = cap;
        if (count_ > cap - start) count_ = cap - start;
        lead = start & 1u;
        base = (const uint4*)(c + (start - lead));
        count = count_;
        nvec = ((u64)lead + (u64)count_ + 1) / 2;
    }
    __device__ __forceinline__ u32 ntiles() const { return (u32)((nvec + kTileVecs - 1) / kTileVecs); }
    __device__ __forceinline__ void full_range(u32& f0, u32& f1) const {
        f0 = lead;
        f1 = (u32)(((u64)lead + (u64)count) / ((u64)kTileVecs * E));
        if (f1 < f0) f1 = f0;
    }
    __device__ __forceinline__ void load_full(u32 tile, u32 tid, Tile& t) const {
        const u64 v0 = (u64)tile * kTileVecs;
        t.tile = tile;
        t.full = true;
#pragma unroll
        for (int u = 0; u < V; ++u) t.r[u] = load16<false>(base + (v0 + (u64)u * B + tid));
    }
    __device__ __forceinline__ void load(u32 tile, u32 tid, Tile& t) const {
        u64 v0 = (u64)tile * kTileVecs;
        t.tile = tile;
        t.full = (tile != 0 || lead == 0) && ((v0 + kTileVecs) * E <= (u64)lead + (u64)count);
#pragma unroll
        for (int u = 0; u < V; ++u) {
            u64 v = v0 + (u64)u * B + tid;
            if (t.full || v < nvec)
                t.r[u] = load16<false>(base + v);
            else
                t.r[u] = make_uint4(0, 0, 0, 0);
        }
    }
    // Digits of the two elements of vector u for any pass (source chosen at run time).
    template <int DT>
    __device__ __forceinline__ void digits_of_pass(const Tile& t, int u, const DigitCtx& c, u32 (&dg)[E]) const {
        dg[0] = digit_of<DT, SRC_RUNTIME>(c.pi, t.r[u].x, t.r[u].y, c.dirmask, c.idx_max, c.a_s);
        dg[1] = digit_of<DT, SRC_RUNTIME>(c.pi, t.r[u].z, t.r[u].w, c.dirmask, c.idx_max, c.a_s);
    }
    __device__ __forceinline__ void get(const Tile& t, int s, u32& raw, u32& idx, bool& valid) const {
        const int u = s / E, j = s % E;
        // position inside the segment; the lead-in wraps to a huge value
        const u32 pos = (t.tile * (u32)kTileVecs + (u32)(u * B) + threadIdx.x) * (u32)E + (u32)j - lead;
        valid = t.full || pos < count;
        raw = j ? t.r[u].z : t.r[u].x;
        idx = j ? t.r[u].w : t.r[u].y;
    }
};

// Visit the tiles wg, wg + G, wg + 2G, ... of a source.
//
// Tiles that lie entirely inside the data (all but possibly the first and the last of a row) go through a
// software pipeline of DEPTH tiles: DEPTH + 1 register sets take turns, the loads of the next DEPTH tiles
// are in flight while one is processed, every load in the steady state is unconditional and no register
// set is ever copied, so the compiler can wait for exactly the oldest set instead of draining the queue.
// The at most two partial tiles are handled afterwards, unpipelined, by fedge(tile).
// Only tiles in [lo, hi) are visited (for callers that split a row into ranges).
// before_load() runs ahead of every prefetch of the steady state: work that issues stores belongs there.  (The
// memory counter a wave waits on counts loads and stores alike, in issue order, with a bound fixed at compile
// time: stores issued after the prefetches would make every wait for a tile also wait for all younger prefetches.)
struct NoHook {
    __device__ __forceinline__ void operator()() const {}
};
template <int DEPTH, class Source, class FFull, class FEdge, class Hook = NoHook>
__device__ __forceinline__ void for_each_tile(const Source& src, u32 wg, u32 G, u32 ntiles, FFull&& f, FEdge&& fedge,
                                              u32 lo = 0u, u32 hi = 0xffffffffu, Hook&& before_load = Hook()) {
    const u32 tid = threadIdx.x;
    u32 f0, f1;  // tiles [f0, f1) are full
    src.full_range(f0, f1);
    const u32 e0 = f0, e1 = f1;  // the partial tiles are those outside [e0, e1)
    if (f0 < lo) f0 = lo;
    if (f1 > hi) f1 = hi;
    if (f1 < f0) f1 = f0;
    // my first full tile and how many I own
    u32 first = wg;
    if (first < f0) first += ((f0 - first + G - 1) / G) * G;
    const u32 m = first < f1 ? (f1 - first + G - 1) / G : 0u;
    auto tile_at = [&](u32 i) __attribute__((always_inline)) { return first + i * G; };
    if (m != 0) {
        if constexpr (DEPTH == 2) {
            typename Source::Tile a, b, c;
            u32 i = 0;
            if (m > 4) {
                // Both loads that the steady state finds in flight are issued unconditionally right before it, and
                // nothing that uses a tile may be scheduled ahead of the prefetch that precedes it in program order:
                // then the compiler's bound on outstanding loads at each use is the steady state's own (two tiles
                // stay in flight while one is processed).
                src.load_full(tile_at(0), tid, a);
                src.load_full(tile_at(1), tid, b);
                for (; i + 4 < m; i += 3) {
                    before_load();
                    src.load_full(tile_at(i + 2), tid, c);
                    __builtin_amdgcn_sched_barrier(0);
                    f(a);
                    before_load();
                    src.load_full(tile_at(i + 3), tid, a);
                    __builtin_amdgcn_sched_barrier(0);
                    f(b);
                    before_load();
                    src.load_full(tile_at(i + 4), tid, b);
                    __builtin_amdgcn_sched_barrier(0);
                    f(c);
                }
                // tiles i and i + 1 are loaded; at most two more follow
                f(a);
                f(b);
                i += 2;
            }
            for (; i < m; ++i) {
                src.load_full(tile_at(i), tid, a);
                f(a);
            }
        } else if constexpr (DEPTH == 1) {
            typename Source::Tile a, b;
            src.load_full(tile_at(0), tid, a);
            u32 i = 0;
            for (; i + 2 < m; i += 2) {
                before_load();
                src.load_full(tile_at(i + 1), tid, b);
                f(a);
                before_load();
                src.load_full(tile_at(i + 2), tid, a);
                f(b);
            }
            f(a);
            if (i + 1 < m) {
                src.load_full(tile_at(i + 1), tid, b);
                f(b);
            }
        } else {
            for (u32 i = 0; i < m; ++i) {
                typename Source::Tile a;
                src.load_full(tile_at(i), tid, a);
                f(a);
            }
        }
    }
    // partial tiles: those of mine outside [e0, e1)
    for (u32 t = wg; t < ntiles; t += G) {
        if (t >= e0 && t < e1) {
            // skip the full range in one step
            const u32 skip = (e1 - t + G - 1) / G;
            t += (skip - 1) * G;
            continue;
        }
        if (t < lo || t >= hi) continue;
        typename Source::Tile e;
        src.load(t, tid, e);
        fedge(e);
    }
}

// ------------------------------------------------------------------------------------------------
// workgroup-wide scans
// ------------------------------------------------------------------------------------------------

// Inclusive prefix sum of v over the 64 lanes of a wave, on the data-parallel-primitive lane network (no
// LDS round trips): shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of rows 0 and 2 is
// added to rows 1 and 3, then lane 31 to the upper half.  Lanes without a source read 0.
__device__ __forceinline__ u32 wave_inclusive_scan(u32 v) {
    v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);  // row_shr:1
    v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);  // row_shr:2
    v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);  // row_shr:4
    v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);  // row_shr:8
    v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // row_bcast:15 -> rows 1, 3
    v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // row_bcast:31 -> rows 2, 3
    return v;
}

// Inclusive prefix sum of v over the workgroup's threads.  wsum: LDS, B/64 words.  Contains one barrier;
// wsum must not be written again before the workgroup's next barrier.
template <int B>
__device__ __forceinline__ u32 block_inclusive_scan(u32 v, u32* wsum) {
    const u32 lane = lane_id();
    const u32 wave = threadIdx.x >> 6;
    v = wave_inclusive_scan(v);
    if (lane == 63) wsum[wave] = v;
    __syncthreads();
    u32 add = 0;
#pragma unroll
    for (u32 w = 0; w < (u32)(B / 64); ++w) add += w < wave ? wsum[w] : 0u;
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

// countBin's inner step (Section 3.1.1): add one element to the workgroup-local histogram.
// Lanes holding the same digit as the wave's first active lane are merged into one LDS atomic
// (register-level aggregation, the "warp" level of the paper's Table 1); everything else goes
// straight to the LDS atomic (the "block" level).  Called by the lanes that hold a valid element.
// A histogram may be kept as several copies, each lane adding to copy (lane mod copies): lanes of one wave
// that hold the same digit then fall on different LDS addresses, which matters when the digits pile into a
// few bins (a wave's adds to one word are served one after the other).  The copies lie one after the other,
// a word more than the bin count apart, so that the same bin of different copies is in different LDS banks.
// HistSlot is one lane's view: the start of its copy (or of the only one).
struct HistSlot {
    u32* h;
    __device__ __forceinline__ u32* at(u32 dg) const { return h + dg; }
};

__device__ __forceinline__ void hist_add_plain(const HistSlot& hs, u32 dg) { atomicAdd(hs.at(dg), 1u); }

__device__ __forceinline__ void hist_add(const HistSlot& hs, u32 dg, u32 lane) {
    const u32 d0 = __builtin_amdgcn_readfirstlane(dg);
    const bool same = dg == d0;
    const u64 m = ballot64(same);
    const u32 cnt = (u32)__popcll(m);
    const bool leader = lane == (u32)__builtin_ctzll(m);  // lowest lane of the merged group
    if (!same || leader) atomicAdd(hs.at(dg), same ? cnt : 1u);
}

}  // namespace rtopk
