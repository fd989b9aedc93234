// Radix top-k kernels for gfx950 (templates; instantiated once per key type by rtopk_f32/f16/bf16.hip).
//
// The first digit pass (paper Section 2.3.1) is two sweeps over the input; every later pass is one sweep
// over the candidates, because CLASSIFY also counts the NEXT digit of what it keeps:
//
//   HIST      countBin.  Every workgroup builds a local histogram of the pass's digit in LDS (hierarchical
//             atomics, Section 3.1.1), adds it to the row's global histogram, and stores the suffix sums of
//             its local histogram.
//   CLASSIFY  selectBin, then selectCandidate fused with the filter.  Every workgroup picks the bin b that
//             holds the k-th key from the row's histogram and turns the stored suffix sums of the workgroups
//             before it into its exact write offsets, so the sweep needs no global atomics.  digit > b: the
//             element is certainly in the top k and goes straight to the output (value bits + int64 index).
//             digit == b: it stays a candidate and is appended, with its index, to the next candidate array.
//             digit < b: dropped.
//
//   While it writes candidates out, CLASSIFY adds their next digit to a fresh LDS histogram; at its end it
//   publishes the histogram (global atomics) and its suffix sums exactly as HIST does.  The next pass's
//   workgroup w then reads the segment of the candidate array that workgroup w wrote, so its per-workgroup
//   counts are already known and no separate histogram sweep over the candidates is needed.
//
//   A row that one workgroup handles alone keeps all of this in LDS and registers (k_row, k_row_resident,
//   k_finish); once at most 512 candidates are left they are ranked against each other directly.
//
//   Where it pays, the two sweeps over the input become one: a bin to filter by is taken from a part of the
//   row first (k_row_stream: the row's first part, a guaranteed bound; k_prefilter_keys: a sample, checked
//   against the exact counts afterwards, with the second sweep as the fallback).
//
// Passes walk the digits of the key from the most significant one down and then the digits of
// (idx_max - index), which makes every element's extended key unique: the loop ends when the chosen
// bin holds exactly as many candidates as are still wanted (all of them win), at the latest on the last
// index digit.  Ties at the k-th key therefore go to the lowest indices, deterministically.
//
// Differences from the paper's CUDA kernels are deliberate (its design targets a different GPU): the
// original input is swept twice, not three times (winners leave in the sweep that discovers them, the final
// filter over X disappears); candidates carry their index; write positions come from per-workgroup
// counts instead of a global counter bumped per flush.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "rtopk.h"
#include "rtopk_device.h"
#include "rtopk_host.h"
#include <type_traits>

namespace rtopk {

// Diagnostic builds (-DRTOPK_TIMING) leave wall-clock stamps of a workgroup's phases in the workspace.
#ifdef RTOPK_TIMING
#define RTOPK_STAMP(i) do { if (SINGLE && threadIdx.x == 0) P.dbg[(size_t)row * P.G * 16 + (i)] = wall_clock64(); } while (0)
#else
#define RTOPK_STAMP(i) do { } while (0)
#endif

#ifndef RTOPK_GRID_BLOCK
#define RTOPK_GRID_BLOCK 512
#endif
#ifndef RTOPK_VECS
#define RTOPK_VECS 4
#endif
constexpr int kGridBlock = RTOPK_GRID_BLOCK;  // threads per workgroup, many-workgroups-per-row kernels
static_assert(kGridBlock == kHostGridBlock && RTOPK_VECS * 4 == kHostElemsPerLane, "host and device tile geometry differ");
constexpr int kRowBlock = 1024;               // threads per workgroup, one-workgroup-per-row kernels
constexpr int kVecs = RTOPK_VECS;             // 16-byte loads per lane per tile (candidate arrays, fp32 rows)
template <int DT> constexpr int key_vecs() { return DT == RTOPK_F32 ? RTOPK_VECS : RTOPK_VECS / 2; }  // 16 elements per lane

constexpr int kStage = 2 * kStageCap;      // entries per wave in the staging area
constexpr int kStageGroup = 4;             // slots of a tile between two looks at the fill level (at most 64 entries each)

// ST: entries per wave in the staging area.  kStage by default; the sweep that filters a streamed row stages more
// when one workgroup has a compute unit's LDS to itself (see k_prefilter_keys).
template <int B, int ST = kStage>
struct Shared {
    static constexpr int kStageEntries = ST;
    u32 hist[kMaxBins];
    u32 hist2[kMaxBins];               // the prefilter sweep's second histogram: next digit of what it keeps in its bound's bin
    u32 wsum[B / 64];
    u32 red[2 * (B / 64)];
    u32 selv[5];                      // selectBin's result: bin, count above it, count inside it; distrust flag; total
    float a_s;                        // the row's scaling constant, broadcast by the thread that drew it
    u32 runW, runC;                   // next free output / candidate position of this workgroup's range
    union {
        // per-wave staging area of (raw bits, index) entries: winners are stacked from the bottom up,
        // candidates from the top down, so either kind may use what the other leaves free
        uint2 stage[B / 64][ST];
        // the same bytes while nothing is staged: interleaved copies of the histogram a single workgroup
        // builds of its whole row
        u32 wide[2 * (B / 64) * ST + 32];
    };
};

// Loop state on entry to pass p (Algorithm 1's candidates / k, plus the output fill level).
struct PassEntry {
    u32 cand;        // candidates entering the pass (n for the first pass)
    u32 k_rem;       // how many of them are still wanted
    u32 out_before;  // outputs already written
    bool finished;   // an earlier pass completed the row
    bool prev_multi; // the previous pass was run by the many-workgroup kernels
    bool in_lds;     // the candidates are in the workgroup's LDS list (few of them), not in the candidate array
    u32 src_array;   // which of the two candidate arrays holds them (meaningless for pass 0 over X)
    bool src_in_x;   // they were never copied: they are the elements of X that match the passes so far
    u32 chain;       // how many passes directly before this one left their candidates in place (see in-place passes)
};
// Which candidate array a pass wrote is part of its record (bit 24 of `window`): a pass that reads array a writes
// array 1 - a, a pass over X writes array 0, the prefilter sweep writes array 1.
constexpr u32 kWindowArrayBit = 24;
// In-place passes.  A pass whose chosen bin holds at least 7/8 of its candidates (keys crowded into a narrow range,
// many duplicates: Section 4.2) does not copy them: it only sends its few winners to the output and counts the next
// digit of the elements in the bin.  The next pass then reads the same source (X itself, or the candidate array of
// the last pass that did copy) and tells candidates from the rest by the digits of all the in-place passes before it,
// read as one wide digit together with its own; once the key's digits are used up that way, the index digits go on
// with "key equals the pivot's" as the condition.  Bits 25 and 26 of a record's `window`: the pass left its
// candidates in place; in place in X.
constexpr u32 kWindowInPlaceBit = 25, kWindowInXBit = 26;

// Few enough candidates are ranked directly against each other (one per lane) instead of walking the
// remaining digits; the list lives where the LDS histogram is, which no longer has a use then.
constexpr u32 kRankCap = 512;
constexpr int SRC_RANK = 3;  // `window` source code of the record the ranking step leaves

__device__ __forceinline__ PassEntry pass_entry(const Params& P, const rtopk_row_trace* st, int p, const RowShape& rs) {
    PassEntry e;
    if (p == 0) {
        e.cand = rs.n;
        e.k_rem = rs.k;
        e.out_before = 0;
        e.finished = false;
        e.prev_multi = true;
        e.in_lds = false;
        e.src_array = 1;  // (what a prefilter sweep kept)
        e.src_in_x = false;
        e.chain = 0;
    } else {
        e.cand = st->pass_rec[p - 1].cand_after;
        e.k_rem = st->pass_rec[p - 1].k_after;
        e.out_before = st->pass_rec[p - 1].out_before + st->pass_rec[p - 1].winners;
        e.finished = e.cand == 0;
        e.prev_multi = st->pass_rec[p - 1].where == 1u;
        e.in_lds = false;
        e.src_array = (st->pass_rec[p - 1].window >> kWindowArrayBit) & 1u;
        e.src_in_x = ((st->pass_rec[p - 1].window >> kWindowInXBit) & 1u) != 0;
        e.chain = 0;
        for (int q = p - 1; q >= 0 && ((st->pass_rec[q].window >> kWindowInPlaceBit) & 1u); --q) ++e.chain;
    }
    return e;
}

// What selectBin decides for one pass.
struct Selection {
    u32 bin;        // b: the bin holding the k-th key
    u32 above;      // g: candidates in better bins -- certain winners
    u32 inside;     // candidates in bin b
    u32 k_inside;   // rank of the k-th key inside bin b
    u32 total;      // candidates counted in all bins
    bool emit_all;  // inside == k_inside: the whole bin wins and the row is finished
};

// selectBin (Section 2.3.1): the bin b with S[b+1] < k <= S[b], S[j] = number of candidates whose digit is at
// least j, together with S[b+1] and the bin's own count.  count(j) reads bin j's count (LDS or global).
// The suffix sums are never stored: every thread sums a few consecutive bins (from the top bin down), one
// scan over the workgroup gives each thread the count above its bins, and the one thread whose range
// contains the k-th candidate walks its bins.  Two barriers; count() is not called after the first, and
// after_read() runs between them (the place to recycle the memory the counts were in).
// A count function may also report that its bins cannot be trusted (see hist_tile_raw): count(j, &bad).
template <int B, class Count, class AfterRead, class SM>
__device__ __forceinline__ Selection select_from_counts(Count&& count, int nb, u32 k_rem, SM& sm,
                                                        rtopk_row_trace* st, AfterRead&& after_read, bool* distrust) {
    constexpr int kMaxPer = kMaxBins / B;
    const int ipt = (nb + B - 1) / B;
    const int r0 = threadIdx.x * ipt;  // position counted from the TOP bin
    u32 c[kMaxPer];
    u32 s = 0;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < kMaxPer; ++i) {
        const int r = r0 + i;
        c[i] = (i < ipt && r < nb) ? count((u32)(nb - 1 - r), &bad) : 0u;
        s += c[i];
    }
    if (threadIdx.x == 0) sm.selv[0] = sm.selv[1] = sm.selv[2] = sm.selv[3] = 0;
    // (selv[4], the total, is written by the last thread below: no clearing needed)
    const u32 incl = block_inclusive_scan<B>(s, sm.wsum);
    after_read();
    const u32 before = incl - s;  // candidates in bins above this thread's
    if (before < k_rem && k_rem <= incl) {
        u32 run = before;
#pragma unroll
        for (int i = 0; i < kMaxPer; ++i) {
            if (run < k_rem && k_rem <= run + c[i]) {
                sm.selv[0] = (u32)(nb - 1 - (r0 + i));
                sm.selv[1] = run;
                sm.selv[2] = c[i];
            }
            run += c[i];
        }
    }
    if (bad) sm.selv[3] = 1u;
    if (threadIdx.x == B - 1) {
        sm.selv[4] = incl;
        if (!distrust && (k_rem == 0 || k_rem > incl)) st->error |= 1u;  // never expected
    }
    __syncthreads();
    Selection r;
    r.bin = sm.selv[0];
    r.above = sm.selv[1];
    r.inside = sm.selv[2];
    r.k_inside = k_rem - r.above;
    r.total = sm.selv[4];
    r.emit_all = r.inside == r.k_inside;
    if (distrust) *distrust = sm.selv[3] != 0u;
    return r;
}

// selectBin for pass entry e, plus the housekeeping that fits between its barriers: the LDS histogram is
// cleared for the next digit's counts and the workgroup's running write positions start at the row's
// (a workgroup that shares the row adds its own offsets afterwards).
template <int B, class Count, int ST>
__device__ __forceinline__ Selection select_pass(Count&& count, int nb, const PassEntry& e, Shared<B, ST>& sm,
                                                 rtopk_row_trace* st, bool* distrust = nullptr) {
    return select_from_counts<B>(
        count, nb, e.k_rem, sm, st,
        [&]() __attribute__((always_inline)) {
            for (int j = threadIdx.x; j < kMaxBins; j += B) sm.hist[j] = 0;
            if (threadIdx.x == 0) {
                sm.runW = e.out_before;
                sm.runC = 0;
            }
        },
        distrust);
}
// The usual count functions: a plain array of bin counts in LDS or in global memory.
struct PlainCounts {
    const u32* c;
    __device__ __forceinline__ u32 operator()(u32 j, bool*) const { return c[j]; }
};

// The row's global histogram for pass p.  Four buffers in rotation: pass p reads p % 4, fills (p + 1) % 4 with the
// next digit's counts and clears (p + 2) % 4, which the pass after it fills (a buffer is never cleared by the launch
// that reads it: the pass that stands for two digits reads two of them).  A fifth buffer holds the histogram of the
// row's sample before a prefilter sweep.
// And a sixth the prefilter sweep's second histogram (the digit after its own, of what it kept in its bound's bin),
// which is read only if pass 0 finds that bin to be the k-th key's.
constexpr int kHistRing = 4, kHistSample = 4, kHistSecond = 5, kSwgRing = 3, kSwgSecond = 3;
__device__ __forceinline__ u32* hist_buffer(const Params& P, int which, int row) {
    return P.ghist + ((size_t)which * P.batch + row) * kMaxBins;
}
__device__ __forceinline__ u32* global_hist(const Params& P, int p, int row) { return hist_buffer(P, p % kHistRing, row); }
// Per-workgroup suffix sums of pass p's digit (three buffers in rotation, for the same reason; a fourth for the
// prefilter sweep's second histogram).
__device__ __forceinline__ u32* swg_buffer(const Params& P, int which, int row) {
    return P.swg + ((size_t)which * P.batch + row) * P.G * kSwgStride;
}
__device__ __forceinline__ u32* swg_records(const Params& P, int p, int row) { return swg_buffer(P, p % kSwgRing, row); }
// (start, count) of the candidates each workgroup wrote into candidate array a.
__device__ __forceinline__ u32* seg_records(const Params& P, u32 a, int row) {
    return P.seg + ((size_t)a * P.batch + row) * P.G * 2;
}

__device__ __forceinline__ void write_pass_record(rtopk_row_trace* st, int p, const PassInfo pi, const PassEntry& e,
                                                  const Selection& sel, u32 where, u32 out_array, bool in_place = false,
                                                  bool in_x = false) {
    // one thread; every field is written exactly once per call
    st->pass_rec[p].bin = sel.bin;
    st->pass_rec[p].k_after = sel.emit_all ? 0u : sel.k_inside;
    st->pass_rec[p].cand_after = sel.emit_all ? 0u : sel.inside;
    st->pass_rec[p].winners = sel.above + (sel.emit_all ? sel.inside : 0u);
    st->pass_rec[p].out_before = e.out_before;
    st->pass_rec[p].cand_before = e.cand;
    st->pass_rec[p].window = pi.src | (pi.shift << 8) | (pi.bits << 16) | (out_array << kWindowArrayBit) |
                             ((in_place ? 1u : 0u) << kWindowInPlaceBit) | ((in_x ? 1u : 0u) << kWindowInXBit);
    st->pass_rec[p].where = where;
}

// ------------------------------------------------------------------------------------------------
// HIST phase: countBin (Section 3.1.1).  Leaves the suffix sums of the workgroup's histogram in LDS.
// With many workgroups per row it also adds the histogram to the row's global one and stores the
// suffix sums for the CLASSIFY sweep.
// ------------------------------------------------------------------------------------------------

// Digits of vector u of a tile: first-pass fast path for X, generic path for candidate arrays.
template <int DT, int SRC, class Source>
__device__ __forceinline__ void vector_digits(const Source& src, const typename Source::Tile& t, int u,
                                              const DigitCtx& c, u32 (&dg)[Source::E]) {
    if constexpr (SRC == SRC_RUNTIME)
        src.template digits_of_pass<DT>(t, u, c, dg);
    else
        src.template digits<SRC>(t, u, c, dg);
}

// MERGE: aggregate lanes that share the first lane's digit before the LDS atomic (pays when one bin
// is hot); otherwise every lane issues its own atomic (cheapest when digits are spread).
template <bool FULL, bool MERGE, class Source, int DT, int SRC>
__device__ __forceinline__ void hist_tile(const Source& src, const typename Source::Tile& t, const DigitCtx& c,
                                          const HistSlot& hist, u32 lane) {
    constexpr int E = Source::E;
#pragma unroll
    for (int u = 0; u < Source::kSlots / E; ++u) {
        u32 dg[E];
        vector_digits<DT, SRC>(src, t, u, c, dg);
#pragma unroll
        for (int j = 0; j < E; ++j) {
            if (FULL) {
                if (MERGE) hist_add(hist, dg[j], lane); else hist_add_plain(hist, dg[j]);
            } else {
                u32 raw, idx;
                bool valid;
                src.get(t, u * E + j, raw, idx, valid);
                if (valid) {
                    if (MERGE) hist_add(hist, dg[j], lane); else hist_add_plain(hist, dg[j]);
                }
            }
        }
    }
}

// How many lanes of this wave share the first lane's digit for the tile's first element: a cheap
// probe of how skewed the digits are (Section 4.2: clustered inputs pile into one bin).
template <class Source, int DT, int SRC>
__device__ __forceinline__ u32 hot_lanes(const Source& src, const typename Source::Tile& t, const DigitCtx& c) {
    u32 dg[Source::E];
    vector_digits<DT, SRC>(src, t, 0, c, dg);
    const u32 d0 = __builtin_amdgcn_readfirstlane(dg[0]);
    return (u32)__popcll(ballot64(dg[0] == d0));
}

// The first digit of a key is a one-to-one function of the top bits of the element's own bit pattern -- set
// the sign bit of non-negatives, complement negatives (then everything, for "smallest") -- for every element
// that is not a NaN: all NaNs share one key whatever their bits.  So a row can be counted by its raw top bits
// (one or two instructions per element instead of the key transform) and the bins renamed afterwards, as long
// as the raw bins that could hold a NaN (exponent field all ones, which also covers the infinities) turn out
// empty; if they do not, the caller counts again with the exact transform.
template <bool FULL, class Source>
__device__ __forceinline__ void hist_tile_raw(const Source& src, const typename Source::Tile& t, const DigitCtx& c,
                                              const HistSlot& hs) {
    constexpr int E = Source::E;
    auto add = [&](int s, u32 draw) __attribute__((always_inline)) {
        if (FULL) {
            atomicAdd(hs.at(draw), 1u);
        } else {
            u32 raw, idx;
            bool valid;
            src.get(t, s, raw, idx, valid);
            if (valid) atomicAdd(hs.at(draw), 1u);
        }
    };
#pragma unroll
    for (int u = 0; u < Source::kSlots / E; ++u) {
        const uint4 q = t.r[u];
        const u32 w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (E == 4) {
                add(u * 4 + j, w[j] >> c.pi.shift);
            } else {  // two 16-bit elements per word; their digit windows sit in bits 16..31 of the aligned key
                add(u * 8 + 2 * j, (w[j] & 0xffffu) >> (c.pi.shift - 16u));
                add(u * 8 + 2 * j + 1, w[j] >> c.pi.shift);
            }
        }
    }
}

// Key digit of a raw top-bits digit (see hist_tile_raw).
__device__ __forceinline__ u32 key_digit_of_raw(u32 draw, u32 bits, bool largest) {
    const u32 top = 1u << (bits - 1u), mask = (top << 1) - 1u;
    const u32 dk = (draw & top) ? (~draw & mask) : (draw | top);
    return largest ? dk : mask - dk;
}

// The sample of a row that is counted before a prefilter sweep: full tiles first, first + stride, ... (spread
// over the row, so that a trend along the row does not mislead), and the rank in the sample whose bin the sweep
// takes as its bound.  The k-th key of the row is expected near rank k * elems / n of the sample; the margin
// (an eighth, eight standard deviations of a binomial count, and 16) makes a bound above the k-th key's bin
// rare, and such a miss costs a second sweep, never the result.
struct RowSample {
    u32 first, stride, tiles, elems;
    u64 rank;
    __device__ __forceinline__ u32 tile(u32 j) const { return first + j * stride; }
};
template <class Source>
__device__ __forceinline__ RowSample row_sample(const Source& src, const Params& P, u32 src_k) {
    RowSample r;
    u32 f0, f1;
    src.full_range(f0, f1);
    r.first = f0;
    r.stride = P.pre_stride;
    r.tiles = (f1 - f0 + r.stride - 1u) / r.stride;
    r.elems = r.tiles * (u32)(Source::kTileVecs * Source::E);
    const u64 ks = ((u64)src_k * r.elems + (u64)src.n - 1u) / (u64)src.n;
    r.rank = ks + ks / 8u + 8u * ((u64)sqrtf((float)ks) + 2u) + 16u;
    return r;
}

// `Resident`: NoResident, or a callable r(f) that calls f(tile) for every tile of a row the workgroup
// holds (or is receiving) in registers.
struct NoResident {};

// Many workgroups per row (SINGLE false): the returned Selection is meaningless (selectBin happens in CLASSIFY,
// on the row's global histogram).  SINGLE: this workgroup owns the row, and selectBin for loop state e is done
// here, straight on the counts.
template <class Source, int DT, int SRC, int B, bool SINGLE, class Resident = NoResident>
__device__ __forceinline__ Selection hist_phase(const Source& src, const Params& P, int p, int row, u32 wg, u32 G,
                                                float a_s, const PassEntry& e, rtopk_row_trace* st, Shared<B>& sm,
                                                const Resident& resident = Resident()) {
    constexpr bool kResident = !std::is_same<Resident, NoResident>::value;
    const DigitCtx ctx = make_digit_ctx(P, p, a_s);
    const int nb = 1 << ctx.pi.bits;
    const u32 tid = threadIdx.x;
    const u32 lane = lane_id();
    const u32 ntiles = src.ntiles();
    Selection none{};
    if (!SINGLE && wg >= ntiles) return none;  // nothing to count; CLASSIFY ignores this workgroup's record

    // One workgroup counting a whole row spreads every bin over interleaved copies (as many as fit the idle
    // staging buffers, at most 8): real inputs put most keys in a few bins, and lanes of a wave that add to
    // one LDS word are served one after the other.
    HistSlot hs{sm.hist};
    u32 copies = 1;
    const u32 stride = (u32)nb + 1u;
    // (with many workgroups per row one copy: two copies changed nothing on 2^28 uniform fp32 keys, 365 against
    // 366 us, nor on 1024 rows of 2^17 bf16 logits with one workgroup per row, 222 against 219-224 us)
    constexpr bool kSpread = SINGLE;
    if (kSpread) {
        constexpr u32 kWideLog2 = B == 1024 ? 14 : 13;
        static_assert(sizeof(sm.wide) / 4 >= (1u << kWideLog2) + 8, "wide histogram size");
        const u32 room = kWideLog2 - ctx.pi.bits;
        copies = 1u << (room < 3u ? room : 3u);
        hs.h = sm.wide + (lane & (copies - 1u)) * stride;
    }
    auto clear = [&]() __attribute__((always_inline)) {
        if (kSpread) {
            for (u32 j = tid; j < copies * stride; j += B) sm.wide[j] = 0;
        } else {
            for (int j = tid; j < nb; j += B) sm.hist[j] = 0;
        }
        __syncthreads();
    };
    auto copies_of = [&](u32 j) __attribute__((always_inline)) {
        u32 c = 0;
        if (copies == 8u) {  // the usual case
#pragma unroll
            for (u32 q = 0; q < 8u; ++q) c += sm.wide[q * stride + j];
        } else {
            for (u32 q = 0; q < copies; ++q) c += sm.wide[q * stride + j];
        }
        return c;
    };

    // The single-workgroup kernels count an unscaled first digit by raw bits first (the digit window is the
    // top of the key: shift + bits == 32).
    constexpr bool kRawFirst = SINGLE && SRC == SRC_KEY;
    if constexpr (kRawFirst) {
        clear();
        RTOPK_STAMP(5);
        if constexpr (kResident) {
            resident([&](const typename Source::Tile& cur) __attribute__((always_inline)) {
                if (cur.full)
                    hist_tile_raw<true, Source>(src, cur, ctx, hs);
                else
                    hist_tile_raw<false, Source>(src, cur, ctx, hs);
            });
        } else {
            for_each_tile<1>(
                src, wg, G, ntiles,
                [&](const typename Source::Tile& cur) __attribute__((always_inline)) { hist_tile_raw<true, Source>(src, cur, ctx, hs); },
                [&](const typename Source::Tile& cur) __attribute__((always_inline)) { hist_tile_raw<false, Source>(src, cur, ctx, hs); });
        }
        __syncthreads();
        RTOPK_STAMP(6);
        // selectBin on the raw-bit bins, visited in key order; a non-empty bin that may hold NaNs spoils it
        const u32 top = (u32)nb >> 1, mask = (u32)nb - 1u;
        const u32 first_special = (DT == RTOPK_F16 ? 0x7c000000u : 0x7f800000u) >> ctx.pi.shift;
        const bool largest = P.dirmask == 0;
        bool distrust = false;
        const Selection sel = select_pass<B>(
            [&](u32 keybin, bool* bad) __attribute__((always_inline)) {
                const u32 dk = largest ? keybin : mask - keybin;
                const u32 draw = (dk & top) ? (dk & ~top) : (~dk & mask);  // inverse of key_digit_of_raw
                const u32 c = copies_of(draw);
                if (c != 0 && (draw & (top - 1u)) >= first_special) *bad = true;
                return c;
            },
            nb, e, sm, st, &distrust);
        RTOPK_STAMP(7);
        if (!distrust) return sel;
    }
    clear();
    if constexpr (kResident) {
        // (two variants only, to bound the code size: the merging one also serves partial tiles)
        resident([&](const typename Source::Tile& cur) __attribute__((always_inline)) {
            if (!cur.full || hot_lanes<Source, DT, SRC>(src, cur, ctx) >= 12u)
                hist_tile<false, true, Source, DT, SRC>(src, cur, ctx, hs, lane);
            else
                hist_tile<true, false, Source, DT, SRC>(src, cur, ctx, hs, lane);
        });
    } else {
        auto full = [&](const typename Source::Tile& cur) __attribute__((always_inline)) {
            if (hot_lanes<Source, DT, SRC>(src, cur, ctx) >= 12u)  // wave-uniform
                hist_tile<true, true, Source, DT, SRC>(src, cur, ctx, hs, lane);
            else
                hist_tile<true, false, Source, DT, SRC>(src, cur, ctx, hs, lane);
        };
        auto edge = [&](const typename Source::Tile& cur) __attribute__((always_inline)) {
            hist_tile<false, true, Source, DT, SRC>(src, cur, ctx, hs, lane);
        };
        if (!SINGLE && P.pre_stride != 0) {
            // before a prefilter sweep only a sample of the row is counted: every pre_stride-th full tile
            const RowSample sample = row_sample(src, P, e.k_rem);
            typename Source::Tile a, b;
            const auto plain = src.plain();
            u32 j = wg;
            if (j < sample.tiles) {
                plain.load_full(sample.tile(j), tid, a);
                for (;;) {
                    const bool more_b = j + G < sample.tiles;
                    if (more_b) plain.load_full(sample.tile(j + G), tid, b);
                    full(a);
                    if (!more_b) break;
                    const bool more_a = j + 2 * G < sample.tiles;
                    if (more_a) plain.load_full(sample.tile(j + 2 * G), tid, a);
                    full(b);
                    if (!more_a) break;
                    j += 2 * G;
                }
            }
            if (wg == 0 && tid == 0) st->pre_elems = sample.elems;
        } else if constexpr (!SINGLE && Source::kStreams) {
            // A streamed row: everything but its tail is read with non-temporal loads; the tail is read with
            // ordinary loads and so stays in the last-level cache, where the CLASSIFY sweep finds it (its own
            // loads are all non-temporal and displace nothing on the way there).
            for_each_tile<2>(src, wg, G, ntiles, full, edge, 0u, P.keep_from_tile);
            for_each_tile<2>(src.plain(), wg, G, ntiles, full, edge, P.keep_from_tile, 0xffffffffu);
        } else {
            for_each_tile<SINGLE ? 1 : 2>(src, wg, G, ntiles, full, edge);
        }
    }
    __syncthreads();
    if (SINGLE) {
        return select_pass<B>([&](u32 j, bool*) __attribute__((always_inline)) { return copies_of(j); }, nb, e, sm, st);
    } else {
        if (kSpread) {
            for (int j = tid; j < nb; j += B) sm.hist[j] = copies_of((u32)j);
            __syncthreads();
        }
        // (the sample's histogram has a buffer of its own; nobody needs its per-workgroup records)
        u32* ghist = P.pre_stride != 0 ? hist_buffer(P, kHistSample, row) : global_hist(P, p, row);
        for (int j = tid; j < nb; j += B) {
            u32 c = sm.hist[j];
            if (c) atomicAdd(&ghist[j], c);
        }
        if (P.pre_stride != 0) return none;
        suffix_sums_in_place<B>(sm.hist, nb, sm.wsum);
        u32* mine = swg_records(P, p, row) + (size_t)wg * kSwgStride;
        for (int j = tid; j < nb; j += B) mine[j] = sm.hist[j];
        if (tid == 0) mine[nb] = 0;
        return none;
    }
}

// ------------------------------------------------------------------------------------------------
// CLASSIFY phase: selectBin, then selectCandidate fused with the filter.
// ------------------------------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void store_value(void* out_row, u32 pos, u32 raw) {
    if (DT == RTOPK_F32)
        ((u32*)out_row)[pos] = raw;
    else
        ((uint16_t*)out_row)[pos] = (uint16_t)raw;
}

// Where one workgroup's share of a pass goes, and how elements are classified.
template <int DT>
struct ClassifyOut {
    void* out_v;         // row's output values
    long long* out_i;    // row's output indices
    uint2* cand_out;     // row's next candidate array
    uint2* cand_lds;     // or, when the candidates are few and one workgroup owns the row, the LDS list
    u32 kk, ncap;        // capacities (writes beyond them are dropped; they never happen in a consistent run)
    // integer mode: an element wins iff wmin <= digit <= wmax and stays a candidate iff digit == b and it does not
    // win.  An ordinary pass: wmin = b + 1 (b when the whole bin wins), wmax = the largest digit.  The digit may be
    // a window of several passes' digits (see classify_phase, MERGED).
    u32 wmin, wmax;
    u32 b;
    // after in-place passes over all of the key's digits: the index digits' candidates are the elements whose ordered
    // key (direction applied) is the pivot's
    bool need_key_eq;
    u32 key_eq;
    // float mode (first pass over X only): the same two tests as comparisons of the element itself with the
    // numbers whose keys are the bin's boundaries:  win = (x < t1) ^ flip,  at-least-candidate = (x < t2) ^ flip
    float t1, t2;
    u64 flip;            // all ones for "largest" (tests become "not less than", true for NaN), 0 for "smallest"
};

// The number whose ordered key is T, if comparing with it reproduces "key < T" for every element.
// That fails when T is 0 or 2^32 (no such number), when the bit pattern is a NaN, and at the boundary between
// the zeros (a float comparison cannot tell -0 from +0).  T is a multiple of 2^16 for 16-bit types.
template <int DT>
__device__ __forceinline__ bool threshold_number(u64 T, float* out) {
    if (T == 0 || T >= (1ull << 32) || T == 0x80000000ull) return false;
    const u32 t = (u32)T;
    if (DT == RTOPK_F16) {
        const u32 t16 = t >> 16;
        const u32 bits = (t16 & 0x8000u) ? (t16 ^ 0x8000u) : (~t16 & 0xffffu);
        if ((bits & 0x7fffu) > 0x7c00u) return false;
        *out = (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
        return true;
    }
    const u32 bits = (t & 0x80000000u) ? (t ^ 0x80000000u) : ~t;
    if ((bits & 0x7fffffffu) > 0x7f800000u) return false;
    *out = __uint_as_float(bits);
    return true;
}

// Winner / candidate lane masks of slot s of a tile.
// PRE (the prefilter sweep): nothing wins yet, and everything whose digit is at least o.b stays a candidate.
template <bool FULL, bool FLOATCMP, class Source, int DT, int SRC, bool PRE = false, bool MERGE = false>
__device__ __forceinline__ void slot_masks(const Source& src, const typename Source::Tile& t, int s, const DigitCtx& c,
                                           const ClassifyOut<DT>& o, u64& mw, u64& mc, const HistSlot& count = HistSlot{nullptr},
                                           u32 lane = 0) {
    static_assert(!(PRE && FLOATCMP), "the prefilter sweep counts digits, so it needs them");
    u64 vm = ~0ull;
    bool valid = true;
    if (!FULL) {
        u32 raw, idx;
        src.get(t, s, raw, idx, valid);
        vm = ballot64(valid);
    }
    if constexpr (FLOATCMP) {
        const float x = src.template value<SRC>(t, s, c.a_s);
        mw = (ballot64(x < o.t1) ^ o.flip) & vm;
        mc = (ballot64(x < o.t2) ^ o.flip) & vm & ~mw;
    } else {
        u32 dg[Source::E];
        vector_digits<DT, SRC>(src, t, s / Source::E, c, dg);  // shared by the slots of one vector
        const u32 d = dg[s % Source::E];
        if constexpr (PRE) {
            // countBin of pass 0 for every element of X, and the filter: keep what lies in bin o.b or a better one
            if (FULL || valid) {
                if (MERGE) hist_add(count, d, lane); else hist_add_plain(count, d);
            }
            mw = 0;
            mc = ballot64(d >= o.b) & vm;
        } else {
            mw = ballot64(d >= o.wmin && d <= o.wmax) & vm;
            mc = ballot64(d == o.b) & vm & ~mw;
            if (o.need_key_eq) {
                u32 raw, idx;
                bool v2;
                src.get(t, s, raw, idx, v2);
                const u64 ok = ballot64((KeyOf<DT>::key(raw) ^ c.dirmask) == o.key_eq);
                mw &= ok;
                mc &= ok;
            }
        }
    }
}

// Write-back of the LDS write buffers (Section 3.1.2).  Every wave stages its survivors in a private
// LDS buffer and, when the buffer cannot take another 64, reserves a range with one LDS atomic on
// the workgroup's running position (the workgroup's whole range is known exactly beforehand, so no
// global atomic is involved) and writes the buffer out as one burst of consecutive addresses.
// Which wave gets which part of the workgroup's range depends on timing: the ORDER of the outputs
// may differ between runs, the selected set does not.
// The two flush routines are the only out-of-line calls of the sweeps (inlined, every slot of every tile variant
// would carry a copy).  Everything they need comes in as scalar arguments, LDS addresses as LDS pointers: an
// argument passed by reference would sit in scratch memory, and each use of it in the loop would be a round
// trip to memory that also waits for the stores just issued (a 256-entry flush took 7 us that way).
template <class T>
using Lds = __attribute__((address_space(3))) T;
template <class T>
using Glb = __attribute__((address_space(1))) T;

__device__ __forceinline__ Lds<u64>* lds_words(const uint2* p) { return (Lds<u64>*)p; }
__device__ __forceinline__ Lds<u32>* lds_word(u32* p) { return (Lds<u32>*)p; }

template <int DT>
__device__ __forceinline__ void flush_winners_body(void* out_v, long long* out_i, u32 kk, Lds<u64>* buf, Lds<u32>* run,
                                                   u32 fill, u32 lane) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    u32 base = 0;
    if (lane == 0) base = __hip_atomic_fetch_add(run, fill, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    base = __builtin_amdgcn_readfirstlane(base);
    for (u32 i = lane; i < fill; i += 64) {
        const u64 e = buf[i];
        const u32 pos = base + i;
        if (pos < kk) {
            if (DT == RTOPK_F32)
                ((Glb<u32>*)out_v)[pos] = (u32)e;
            else
                ((Glb<uint16_t>*)out_v)[pos] = (uint16_t)e;
            ((Glb<long long>*)out_i)[pos] = (long long)(e >> 32);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
}
template <int DT>
__device__ __noinline__ void flush_wave_winners(void* out_v, long long* out_i, u32 kk, Lds<u64>* buf, Lds<u32>* run,
                                                u32 fill, u32 lane) {
    flush_winners_body<DT>(out_v, out_i, kk, buf, run, fill, lane);
}
// What the candidate flush needs to count the next pass's digit (countBin of pass p + 1 happens here, on
// full waves, rather than element by element in the sweep).
struct NextCount {
    HistSlot hist;    // LDS histogram of the next digit (hist.h == nullptr when there is no next pass)
    PassInfo pi;
    u32 dirmask, idx_max;
    float a_s;
    // The prefilter sweep (nothing of the following applies to any other pass):
    // it counts its own digit for every element in the sweep, not here; what it does leave to the write-back is
    bool nan_fix = false;   // (raw-bit counting, prefilter_tile_raw) move the count of every staged NaN from the raw
                            // bin of its bits (digit shift nan_shift) to the NaNs' own bin nan_bin of `hist`
    bool discard = false;   // ... and write nothing (the prefilter declined: what is staged is staged for this only)
    bool count_if = false;  // count digit `pi` (the digit AFTER the sweep's own) into hist2, for the entries whose
                            // key above that digit equals only_bin, i.e. that lie in the sweep's bound bin
    HistSlot hist2{nullptr};
    u32 only_bin = 0, nan_shift = 0, nan_bin = 0;
    // ... or, when the prefilter declined because the sample shows the keys crowded into one bin: the sweep itself counts
    // digit `pi`, by raw bits, of every element whose raw first digit is crowd_raw, into hist2 (prefilter_tile_raw)
    u32 crowd_raw = 0;
};
enum : u32 { kFlushToList = 1u, kFlushCount = 2u, kFlushNanFix = 4u, kFlushDiscard = 8u, kFlushCountIf = 16u };

// what (kFlush* bits): to-list -- the candidates go to the LDS list cand_lds instead of cand_out; count -- the next
// pass's digit, described by (src, shift, bits, dirmask, idx_max, a_s), is counted into the LDS histogram hist;
// the other three are the prefilter sweep's (see NextCount).
// (Flags, not null tests: an LDS pointer to the start of the workgroup's LDS is the number 0, and a null generic
// pointer casts to -1.)
template <int DT>
__device__ __forceinline__ void flush_candidates_body(uint2* cand_out, Lds<u64>* cand_lds, u32 ncap, Lds<u64>* buf,
                                                      Lds<u32>* run, u32 fill, u32 lane, Lds<u32>* hist, Lds<u32>* hist2,
                                                      u32 src, u32 shift, u32 bits, u32 dirmask, u32 idx_max, float a_s,
                                                      u32 what, u32 only_bin, u32 nan_shift, u32 nan_bin) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    u32 base = 0;
    if (!(what & kFlushDiscard)) {
        if (lane == 0) base = __hip_atomic_fetch_add(run, fill, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        base = __builtin_amdgcn_readfirstlane(base);
    }
    const PassInfo pi{src, shift, bits};
    for (u32 i = lane; i < fill; i += 64) {
        const u64 e = buf[i];
        const u32 pos = base + i;
        if (what & kFlushDiscard) {
        } else if (what & kFlushToList) {
            if (pos < kRankCap) cand_lds[pos] = e;
        } else if (pos < ncap) {
            ((Glb<u64>*)cand_out)[pos] = e;
        }
        if (what & (kFlushCount | kFlushCountIf)) {
            u32 dg;
            Lds<u32>* h = hist;
            bool mine = true;
            if (what & kFlushCountIf) {
                const u32 key = KeyOf<DT>::key((u32)e) ^ dirmask;
                mine = (key >> (shift + bits)) == only_bin;
                dg = (key >> shift) & ((1u << bits) - 1u);
                h = hist2;
            } else {
                dg = digit_of<DT, SRC_RUNTIME>(pi, (u32)e, (u32)(e >> 32), dirmask, idx_max, a_s);
            }
            if (mine) {
                // as hist_add: the lanes that hold the first active lane's digit share one LDS atomic
                const u32 d0 = __builtin_amdgcn_readfirstlane(dg);
                const bool same = dg == d0;
                const u64 m = ballot64(same);
                const bool leader = lane == (u32)__builtin_ctzll(m);
                if (!same || leader)
                    __hip_atomic_fetch_add(h + dg, same ? (u32)__popcll(m) : 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
        if (DT == RTOPK_F32 && (what & kFlushNanFix)) {
            const u32 raw = (u32)e;
            if ((raw & 0x7fffffffu) > 0x7f800000u) {
                __hip_atomic_fetch_add(hist + (raw >> nan_shift), ~0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __hip_atomic_fetch_add(hist + nan_bin, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
}
template <int DT>
__device__ __noinline__ void flush_wave_candidates(uint2* cand_out, Lds<u64>* cand_lds, u32 ncap, Lds<u64>* buf,
                                                   Lds<u32>* run, u32 fill, u32 lane, Lds<u32>* hist, Lds<u32>* hist2,
                                                   u32 src, u32 shift, u32 bits, u32 dirmask, u32 idx_max, float a_s,
                                                   u32 what, u32 only_bin, u32 nan_shift, u32 nan_bin) {
    flush_candidates_body<DT>(cand_out, cand_lds, ncap, buf, run, fill, lane, hist, hist2, src, shift, bits, dirmask, idx_max,
                              a_s, what, only_bin, nan_shift, nan_bin);
}

// INLINE: the write-back is expanded in place.  A call costs more than its instructions: a function starts by
// waiting for every outstanding memory operation of the wave, so each call made in the middle of a sweep drains
// the tiles the wave has prefetched.  The sweeps that stream from memory therefore look at the fill level only
// every kStageGroup slots and expand the write-back at those few places; calls remain where nothing is in flight
// (the sweep over a row held in registers) and for what is left at the end of a sweep.
template <int DT, bool INLINE = false>
__device__ __forceinline__ void flush_winners(const ClassifyOut<DT>& o, const uint2* buf, u32* run, u32 fill, u32 lane) {
    if constexpr (INLINE)
        flush_winners_body<DT>(o.out_v, o.out_i, o.kk, lds_words(buf), lds_word(run), fill, lane);
    else
        flush_wave_winners<DT>(o.out_v, o.out_i, o.kk, lds_words(buf), lds_word(run), fill, lane);
}
template <int DT, bool INLINE = false>
__device__ __forceinline__ void flush_candidates(const ClassifyOut<DT>& o, const uint2* buf, u32* run, u32 fill, u32 lane,
                                                 const NextCount& nc) {
    const bool pre = nc.nan_fix || nc.count_if || nc.discard;
    const u32 what = (o.cand_lds != nullptr ? kFlushToList : 0u) | (nc.hist.h != nullptr && !pre ? kFlushCount : 0u) |
                     (nc.nan_fix ? kFlushNanFix : 0u) | (nc.discard ? kFlushDiscard : 0u) | (nc.count_if ? kFlushCountIf : 0u);
    if constexpr (INLINE)
        flush_candidates_body<DT>(o.cand_out, lds_words(o.cand_lds), o.ncap, lds_words(buf), lds_word(run), fill, lane,
                                  lds_word(nc.hist.h), lds_word(nc.hist2.h), nc.pi.src, nc.pi.shift, nc.pi.bits, nc.dirmask,
                                  nc.idx_max, nc.a_s, what, nc.only_bin, nc.nan_shift, nc.nan_bin);
    else
        flush_wave_candidates<DT>(o.cand_out, lds_words(o.cand_lds), o.ncap, lds_words(buf), lds_word(run), fill, lane,
                                  lds_word(nc.hist.h), lds_word(nc.hist2.h), nc.pi.src, nc.pi.shift, nc.pi.bits, nc.dirmask,
                                  nc.idx_max, nc.a_s, what, nc.only_bin, nc.nan_shift, nc.nan_bin);
}

// Entries waiting in this wave's staging area (wave-uniform): winners in [0, fillW), candidates in
// [ST - fillC, ST), ST being the area's size.
struct WriteState {
    u32 fillW, fillC;
};

// Write back whatever is staged.
template <int DT, bool INLINE, int B, int ST>
__device__ __forceinline__ void flush_staged(const ClassifyOut<DT>& o, Shared<B, ST>& sm, u32 lane, u32 wave, WriteState& ws,
                                             const NextCount& nc) {
    uint2* st = sm.stage[wave];
    if (ws.fillW) flush_winners<DT, INLINE>(o, st, &sm.runW, ws.fillW, lane);
    if (ws.fillC) flush_candidates<DT, INLINE>(o, st + (ST - ws.fillC), &sm.runC, ws.fillC, lane, nc);
    ws.fillW = ws.fillC = 0;
}
// Before a group of kStageGroup slots: make room for everything the group can add.
template <int DT, bool INLINE = true, int B, int ST>
__device__ __forceinline__ void make_room(const ClassifyOut<DT>& o, Shared<B, ST>& sm, u32 lane, u32 wave, WriteState& ws,
                                          const NextCount& nc) {
    if (ws.fillW + ws.fillC > (u32)(ST - 64 * kStageGroup)) flush_staged<DT, INLINE>(o, sm, lane, wave, ws, nc);
}
// Between two tiles of a streaming sweep, before the next prefetch is issued (see for_each_tile): the place where a
// write-back costs least, so what has piled up goes out here already at a slightly lower fill level.
constexpr u32 kStageEarlyRoom = 320;

// One tile, one sweep over its slots: classify, append survivors to the wave's staging area.
// RARE: survivors are expected to be few and nothing is being prefetched (the row held in registers, fully
// unrolled): the append code is kept off the straight path and the write-back is a call, made when fewer than 64
// entries are free.
template <bool FULL, bool FLOATCMP, class Source, int DT, int SRC, int B, bool RARE = false, bool PRE = false,
          bool MERGE = false, int ST = kStage>
__device__ __forceinline__ void classify_tile(const Source& src, const typename Source::Tile& t, const DigitCtx& c,
                                              const ClassifyOut<DT>& o, Shared<B, ST>& sm, u32 lane, u32 wave,
                                              WriteState& ws, const NextCount& nc) {
    constexpr int E = Source::E;
    constexpr int S = Source::kSlots;
    uint2* st = sm.stage[wave];
    const u64 me_bit = 1ull << lane;
    // (the prefilter sweep counts every element; MERGE: lanes that share the first lane's digit merge their adds)
#pragma unroll
    for (int s = 0; s < S; ++s) {
        if (!RARE && s % kStageGroup == 0) make_room<DT>(o, sm, lane, wave, ws, nc);
        u64 mw, mc;
        if constexpr (PRE)
            slot_masks<FULL, FLOATCMP, Source, DT, SRC, PRE, MERGE>(src, t, s, c, o, mw, mc, HistSlot{sm.hist}, lane);
        else
            slot_masks<FULL, FLOATCMP, Source, DT, SRC, PRE>(src, t, s, c, o, mw, mc);
        const bool any = (mw | mc) != 0;
        if (RARE ? __builtin_expect(any, false) : any) {
            u32 raw, idx;
            bool valid;
            src.get(t, s, raw, idx, valid);
            if (mw) {
                if (mw & me_bit) st[ws.fillW + mbcnt64(mw)] = make_uint2(raw, idx);
                ws.fillW += (u32)__popcll(mw);
            }
            if (mc) {
                if (mc & me_bit) st[(u32)(ST - 1) - (ws.fillC + mbcnt64(mc))] = make_uint2(raw, idx);
                ws.fillC += (u32)__popcll(mc);
            }
            if (RARE && ws.fillW + ws.fillC > (u32)(ST - 64)) flush_staged<DT, false>(o, sm, lane, wave, ws, nc);
        }
    }
}

// One tile of an in-place pass (see in-place passes): nearly every element read is a candidate and stays where it
// is; its next digit is counted (lanes that share the first lane's digit with one LDS add -- the crowd these passes
// exist for usually shares it), the few winners are staged as usual.  OWN / NEXT: what this pass's digit and the next
// one's are taken from, fixed at compile time so that the slot loop holds no decisions: both from the key, both from
// the scaled key, both from the index, or the key's last digit followed by the index's first.  KEY_EQ (index digits
// after in-place key digits): only elements with the pivot's key count at all.
// Full tiles first ask whether the crowd is total: if all 64 lanes' first elements are candidates with one and the same
// next digit, the tile is taken a vector at a time -- a vector whose every element in every lane is such a candidate is
// counted with one LDS add by one lane (no winners can be among them), any other vector goes the element-wise way.
// (All keys equal, 2^28 fp32: an in-place sweep 340 -> see the measurements at the in-place passes.)
template <bool FULL, int OWN, int NEXT, bool KEY_EQ, class Source, int DT, int B, int ST>
__device__ __forceinline__ void inplace_tile(const Source& src, const typename Source::Tile& t, const DigitCtx& c,
                                             const ClassifyOut<DT>& o, Shared<B, ST>& sm, u32 lane, u32 wave, WriteState& ws,
                                             const NextCount& nc) {
    constexpr int S = Source::kSlots;
    constexpr int E = Source::E;
    uint2* st = sm.stage[wave];
    const u64 me_bit = 1ull << lane;
    const u32 wmask = c.pi.bits >= 32u ? 0xffffffffu : (1u << c.pi.bits) - 1u;
    const u32 nmask = (1u << nc.pi.bits) - 1u;
    // one element: is it a candidate (cand), its window digit (wd) and its next digit (nd)
    auto look = [&](int s, u32& raw, u32& idx, u32& wd, u32& nd, bool& ok) __attribute__((always_inline)) {
        bool valid;
        src.get(t, s, raw, idx, valid);
        u32 u;  // the 32 bits this pass's digit is a window of
        if (OWN == SRC_IDX)
            u = c.idx_max - idx;
        else if (OWN == SRC_KEY)
            u = KeyOf<DT>::key(raw) ^ c.dirmask;
        else
            u = KeyOf<RTOPK_F32>::key(__float_as_uint(__uint_as_float(raw) - c.a_s)) ^ c.dirmask;
        wd = (u >> c.pi.shift) & wmask;
        ok = FULL || valid;
        if (KEY_EQ) ok = ok && (KeyOf<DT>::key(raw) ^ c.dirmask) == o.key_eq;
        const u32 v = NEXT == OWN ? u : c.idx_max - idx;
        nd = (v >> nc.pi.shift) & nmask;
    };
    auto slot = [&](int s) __attribute__((always_inline)) {
        if (s % kStageGroup == 0) make_room<DT, false>(o, sm, lane, wave, ws, nc);  // (winners are few: a call will do)
        u32 raw, idx, wd, nd;
        bool ok;
        look(s, raw, idx, wd, nd, ok);
        const u64 mw = ballot64(ok && wd >= o.wmin && wd <= o.wmax);
        const u64 mc = ballot64(ok && wd == o.b);
        if (mc & me_bit) hist_add(nc.hist, nd, lane);
        if (mw) {
            if (mw & me_bit) st[ws.fillW + mbcnt64(mw)] = make_uint2(raw, idx);
            ws.fillW += (u32)__popcll(mw);
        }
    };
    bool total = false;
    if constexpr (FULL) {
        u32 raw, idx, wd, nd;
        bool ok;
        look(0, raw, idx, wd, nd, ok);
        total = ballot64(ok && wd == o.b && nd == (u32)__builtin_amdgcn_readfirstlane(nd)) == ~0ull;
    }
    if (FULL && total) {
#pragma unroll
        for (int v = 0; v < S / E; ++v) {
            bool all = true;
            u32 d0 = 0;
#pragma unroll
            for (int j = 0; j < E; ++j) {
                u32 raw, idx, wd, nd;
                bool ok;
                look(v * E + j, raw, idx, wd, nd, ok);
                if (j == 0) d0 = (u32)__builtin_amdgcn_readfirstlane(nd);
                all = all && ok && wd == o.b && nd == d0;
            }
            if (ballot64(all) == ~0ull) {
                if (lane == 0) atomicAdd(nc.hist.at(d0), 64u * (u32)E);
            } else {
#pragma unroll
                for (int j = 0; j < E; ++j) slot(v * E + j);
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < S; ++s) slot(s);
    }
}
// ... with OWN / NEXT / KEY_EQ taken from the pass at run time, once per tile.
template <bool FULL, class Source, int DT, int B, int ST>
__device__ __forceinline__ void inplace_tile_any(const Source& src, const typename Source::Tile& t, const DigitCtx& c,
                                                 const ClassifyOut<DT>& o, Shared<B, ST>& sm, u32 lane, u32 wave,
                                                 WriteState& ws, const NextCount& nc) {
    if (c.pi.src == SRC_KEY && nc.pi.src == SRC_KEY)
        inplace_tile<FULL, SRC_KEY, SRC_KEY, false>(src, t, c, o, sm, lane, wave, ws, nc);
    else if (c.pi.src == SRC_KEY)
        inplace_tile<FULL, SRC_KEY, SRC_IDX, false>(src, t, c, o, sm, lane, wave, ws, nc);
    else if (c.pi.src == SRC_IDX && o.need_key_eq)
        inplace_tile<FULL, SRC_IDX, SRC_IDX, true>(src, t, c, o, sm, lane, wave, ws, nc);
    else if (c.pi.src == SRC_IDX)
        inplace_tile<FULL, SRC_IDX, SRC_IDX, false>(src, t, c, o, sm, lane, wave, ws, nc);
    else if constexpr (DT == RTOPK_F32)
        inplace_tile<FULL, SRC_SCALED, SRC_SCALED, false>(src, t, c, o, sm, lane, wave, ws, nc);
}

// One tile of the prefilter sweep over fp32 keys, the cheap way.  countBin needs only the element's raw top bits
// (hist_tile_raw: the bins are renamed afterwards), and "digit >= bound" is one float comparison with the number at
// the bound's edge (o.t2), so the straight path is a shift, an LDS add and a compare per element.  The comparison
// is written so that a NaN passes it in either direction: whatever passes is staged and nothing else is done here
// (each further instruction on this path is paid in 4 of 10 slots at 1 % kept) -- the write-back moves every NaN's
// count from the raw bin its bits fell in to the one bin all NaNs share, raw bin 2^bits/2 - 1 (the top of the
// positive half: its key digit is the best for "largest", the worst for "smallest").  For "smallest" the NaNs are
// kept although they rank below the bound; pass 0 drops them like anything else below the k-th key's bin.  When
// the prefilter declined, the edge is an infinity: only NaNs (and infinities of one sign) are staged, to have
// their counts moved, and nothing is written.
// CROWD: the sweep keeps nothing, and counts the next digit of the elements of one raw bin (see NextCount::crowd_raw).
template <bool FULL, bool MERGE, bool LARGEST, bool CROWD = false, class Source, int B, int ST>
__device__ __forceinline__ void prefilter_tile_raw(const Source& src, const typename Source::Tile& t, const DigitCtx& c,
                                                   const ClassifyOut<RTOPK_F32>& o, Shared<B, ST>& sm, u32 lane, u32 wave,
                                                   WriteState& ws, const NextCount& nc) {
    static_assert(Source::E == 4, "fp32 keys");
    constexpr int S = Source::kSlots;
    uint2* st = sm.stage[wave];
    const u64 me_bit = 1ull << lane;
    const HistSlot hs{sm.hist};
    auto slot = [&](int s) __attribute__((always_inline)) {
        // (sparse by design: the room made between tiles nearly always suffices, so this one may be a call)
        if (s % kStageGroup == 0) make_room<RTOPK_F32, false>(o, sm, lane, wave, ws, nc);
        u32 raw, idx;
        bool valid;
        src.get(t, s, raw, idx, valid);  // (full tiles: raw is a register, idx and valid are not computed unless used)
        const u32 draw = raw >> c.pi.shift;
        if (FULL || valid) {
            if (MERGE) hist_add(hs, draw, lane); else hist_add_plain(hs, draw);
        }
        if (CROWD) {
            if ((FULL || valid) && draw == nc.crowd_raw) hist_add(nc.hist2, (raw >> nc.pi.shift) & ((1u << nc.pi.bits) - 1u), lane);
        }
        const float x = __uint_as_float(raw);
        u64 m = ballot64(LARGEST ? !(x < o.t2) : !(x >= o.t2));
        if (!FULL) m &= ballot64(valid);
        if (m) {
            if (m & me_bit) st[(u32)(ST - 1) - (ws.fillC + mbcnt64(m))] = make_uint2(raw, idx);
            ws.fillC += (u32)__popcll(m);
        }
    };
    // CROWD, full tiles: a vector whose every element, in every lane, lies in the crowded bin with one and the same
    // next digit is counted by one lane with two LDS adds (the bin can hold neither NaN nor infinity: nothing to
    // stage).  Tried for the tiles whose first vector is of that kind (a narrow range of many values never is, and
    // pays nothing for the question beyond that one look).
    if constexpr (CROWD && FULL) {
        const u32 nmask = (1u << nc.pi.bits) - 1u;
        const u32 sh = nc.pi.shift;
        auto total = [&](int v, u32& d0) __attribute__((always_inline)) {
            const uint4 q = t.r[v];
            d0 = (u32)__builtin_amdgcn_readfirstlane((q.x >> sh) & nmask);
            const u32 hi = (nc.crowd_raw << (c.pi.shift - sh)) | d0;  // both digits, as the top bits of the element
            return ballot64((q.x >> sh) == hi && (q.y >> sh) == hi && (q.z >> sh) == hi && (q.w >> sh) == hi) == ~0ull;
        };
        u32 d0;
        if (total(0, d0)) {
#pragma unroll
            for (int v = 0; v < S / 4; ++v) {
                if (total(v, d0)) {
                    if (lane == 0) {
                        atomicAdd(hs.at(nc.crowd_raw), 256u);
                        atomicAdd(nc.hist2.at(d0), 256u);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) slot(v * 4 + j);
                }
            }
            return;
        }
    }
#pragma unroll
    for (int s = 0; s < S; ++s) slot(s);
}

// Where the histogram of a pass is.
enum { HIST_IN_LDS = 0, HIST_IN_GLOBAL = 1 };

// Are the digits of passes p and p + 1 adjacent windows of the ordered key itself, so that both can be read as one digit?
__device__ __forceinline__ bool pass_pair_is_one_window(const Params& P, int p) {
    return p + 1 < P.npass && P.pass[p].src == SRC_KEY && P.pass[p + 1].src == SRC_KEY &&
           P.pass[p + 1].shift + P.pass[p + 1].bits == P.pass[p].shift;
}

// `sel` is selectBin's decision for this pass, made by select_pass (which also prepared the LDS histogram and
// the running write positions).  SINGLE: the row is handled by this workgroup alone (wg = 0, G = 1);
// otherwise G workgroups share the row.
// Returns the loop state for pass p + 1 (what the pass record written here says, without the trip through memory).
// PRE: the prefilter sweep over X (many workgroups, first digit): `sel` comes from the histogram of a sample of
// the row, so its bin is only probably at or below the true one; nothing is written to the output, every element
// of a bin >= sel.bin goes to the candidate array (into a segment of fixed position: there are no counts yet to
// derive exact offsets from), and this same first digit is counted for EVERY element of X, kept or not (the
// exact histogram pass 0 selects on, and the per-workgroup records either kind of pass 0 takes its offsets from).
// sel0 (many workgroups, pass 1 on what a prefilter sweep kept, only): pass 0 had no sweep of its own.  The prefilter
// sweep counted pass 1's digit for what it kept in its bound's bin; when the exact counts make that bin the k-th
// key's bin (sel0->bin), `sel` is pass 1's selectBin on those counts, and this one sweep stands for both passes: it
// classifies by the two digits taken as one (better than bin 0's digit, or in it and better than bin 1's: a winner).
template <class Source, int DT, int SRC, int B, bool SINGLE, class Resident = NoResident, bool PRE = false, int ST = kStage>
__device__ __forceinline__ PassEntry classify_phase(const Source& src, const Params& P, int p, int row, u32 row_k, u32 wg, u32 G,
                                                    const PassEntry& e, rtopk_row_trace* st, float a_s, Shared<B, ST>& sm,
                                                    u32 where, const Selection& sel, u32 records, bool own_segment,
                                                    const Resident& resident = Resident(), const Selection* sel0 = nullptr,
                                                    u32 crowd_bin = 0xffffffffu) {
    constexpr bool kResident = !std::is_same<Resident, NoResident>::value;
    static_assert(!PRE || (!SINGLE && !kResident && SRC != SRC_RUNTIME), "the prefilter is a grid sweep over X");
    DigitCtx ctx = make_digit_ctx(P, p, a_s);
    const PassInfo own_pi = ctx.pi;
    if (sel0) ctx.pi.bits += P.pass[p - 1].bits;  // the digit window of both passes
    // In-place passes before this one: their digits, read as one wide digit with this pass's own, tell this pass's
    // candidates from the rest of what it reads.  (Index digits after in-place key digits: the key must be the pivot's.)
    u32 prefix = sel0 ? sel0->bin : 0u;
    bool need_key_eq = false;
    u32 key_eq = 0;
    if (!PRE && !sel0 && e.chain != 0) {
        int q = p - 1;
        u32 sh = 0;
        for (; q >= p - (int)e.chain && P.pass[q].src == own_pi.src; --q) {
            prefix |= st->pass_rec[q].bin << sh;
            sh += P.pass[q].bits;
        }
        ctx.pi.bits += sh;
        if (q >= p - (int)e.chain) {
            // the chain goes on into the key's digits: every one of them belongs to the pivot's key
            need_key_eq = true;
            for (int z = 0; z < p; ++z)
                if (P.pass[z].src == SRC_KEY) key_eq |= st->pass_rec[z].bin << P.pass[z].shift;
        }
    }
    const int nb = 1 << own_pi.bits;
    const u32 tid = threadIdx.x;
    const u32 lane = lane_id();
    const u32 wave = tid >> 6;
    const u32 ntiles = src.ntiles();
    // Leave the candidates where they are?  (Many workgroups per row only; see in-place passes.)
    // (sel0: only when the two digits are read from X itself, the crowded case, where the rest of the key is likely
    // to be just as crowded)
    constexpr bool from_x = !std::is_same<Source, CandSource<B, kVecs>>::value;
    bool inplace = false;
    if (!SINGLE && !PRE && (!sel0 || from_x) && !sel.emit_all && p + 1 < P.npass && sel.inside > P.small &&
        (u64)sel.inside * 8u > (u64)e.cand * 7u) {
        const PassInfo nx = P.pass[p + 1];
        const bool same = nx.src == own_pi.src && ctx.pi.bits + nx.bits <= 32u;    // the next digit extends this window
        const bool into_index = own_pi.src == SRC_KEY && nx.src == SRC_IDX;        // the key's last digit
        inplace = same || into_index;
    }

#ifdef RTOPK_TIMING
    unsigned long long t_begin = wall_clock64(), t_pro = 0, t_sweep = 0;
#endif
    u32 runW = e.out_before, runC = 0, myC = 0;
    // which candidate array this pass writes: the other one than it reads; array 0 from X; a prefilter sweep array 1
    const u32 out_array = PRE ? 1u : from_x ? 0u : 1u - e.src_array;
    const u32 rec_array = inplace ? e.src_array : out_array;
    const bool rec_inplace = inplace, rec_in_x = inplace && (from_x || e.src_in_x);
    if constexpr (PRE) {
        // this workgroup's segment starts where the tiles of the workgroups before it would end if every element
        // of theirs were kept (tiles are dealt round-robin: workgroup v has ntiles / G of them, one more if
        // v < ntiles % G)
        const u32 q = ntiles / G, r = ntiles % G;
        runC = (wg * q + (wg < r ? wg : r)) * (u32)(B * Source::kSlots);
    } else if (!SINGLE) {
        // exact write offsets: sum, at the chosen bin, the stored suffix sums of the workgroups before this one
        // (`records` workgroups have a record for this pass)
        const u32 upto = wg < records ? wg : records;
        const u32* swg_row = sel0 ? swg_buffer(P, kSwgSecond, row) : swg_records(P, p, row);
        const u32* swg_row0 = sel0 ? swg_records(P, p - 1, row) : swg_row;
        u32 W = 0, C = 0;
        for (u32 w = tid; w < upto; w += B) {
            const u32* rec = swg_row + (size_t)w * kSwgStride;
            const u32 sb = rec[sel.bin], sb1 = rec[sel.bin + 1];
            W += sel.emit_all ? sb : sb1;
            C += sel.emit_all ? 0u : sb - sb1;
            if (sel0) W += swg_row0[(size_t)w * kSwgStride + sel0->bin + 1];
        }
        block_sum2<B>(W, C, sm.red);
        runW = (sel0 ? 0u : e.out_before) + W;
        runC = C;
        if (wg < records && !sel.emit_all) {
            const u32* rec = swg_row + (size_t)wg * kSwgStride;
            myC = rec[sel.bin] - rec[sel.bin + 1];
        }
        if (wg == 0) {
            // the histogram buffer two ahead in the ring is filled by the next pass: clear it (its last reader was
            // an earlier launch)
            u32* other = global_hist(P, p + 2, row);
            for (int j = tid; j < kMaxBins; j += B) other[j] = 0;
        }
    }
    if (!PRE && wg == 0 && tid == 0) {
        if (sel0) {
            // pass 0's record: what its selectBin decided; its winners leave in this sweep
            // (from X: the prefilter sweep kept nothing, the candidates of both passes are the row's own elements)
            PassEntry e0 = e;  // (only what a record takes from it matters)
            u32 cand0 = st->pre_kept;
            if constexpr (from_x) cand0 = (u32)src.n;
            e0.cand = cand0;
            e0.out_before = 0;
            write_pass_record(st, 0, P.pass[0], e0, *sel0, where, e.src_array, from_x, from_x);
            st->pre_merged = 1u;
        }
        write_pass_record(st, p, own_pi, e, sel, where, rec_array, rec_inplace, rec_in_x);
        // after a prefilter the first digit pass looks at what the prefilter kept, not at all of X
        if (!SINGLE && SRC == SRC_RUNTIME && p == 0) st->pass_rec[0].cand_before = st->pre_kept;  // after a prefilter
    }

    // few candidates left and the row is this workgroup's alone: keep them in LDS for the ranking step
    // (which orders by key and index, so every scaled-key digit must have been used by then)
    const bool to_rank = SINGLE && !sel.emit_all && sel.inside <= kRankCap && p + 1 < P.npass &&
                         P.pass[p + 1].src != SRC_SCALED;
    // the next pass: does it exist, and will the many-workgroup kernels run it?
    const bool count_next = PRE || (!sel.emit_all && p + 1 < P.npass && !to_rank);
    const bool next_multi = PRE || (!SINGLE && count_next && sel.inside > P.small);
    const PassInfo next_pi = PRE ? P.pass[p] : P.pass[p + 1 < P.npass ? p + 1 : p];
    const int nb_next = 1 << next_pi.bits;
    // buffers of the "next" pass: p + 1, or p itself after a prefilter (which stands before pass p as pass p - 1)
    const int pn = PRE ? p : p + 1;

    ClassifyOut<DT> o;
    o.out_v = (char*)P.out_values + (size_t)row * (size_t)P.k * KeyOf<DT>::kBytes;
    o.out_i = P.out_indices + (size_t)row * (size_t)P.k;
    o.cand_out = P.cand[out_array] + (size_t)row * P.cand_stride;
    o.cand_lds = to_rank ? (uint2*)sm.hist : nullptr;
    o.kk = row_k;
    o.ncap = (u32)P.cand_stride;
    // The window holds the digits of earlier passes above pass p's own: of the in-place passes before it (whatever
    // differs from them there is no candidate of this pass: neither winner nor kept), or, with sel0, pass p - 1's
    // (whatever is better there is a winner of that pass, emitted here).
    o.b = (prefix << own_pi.bits) | sel.bin;
    o.wmax = sel0 ? (ctx.pi.bits >= 32u ? 0xffffffffu : (1u << ctx.pi.bits) - 1u) : (prefix << own_pi.bits) | ((1u << own_pi.bits) - 1u);
    o.wmin = sel.emit_all ? o.b : o.b + 1u;
    if (!sel.emit_all && o.b == o.wmax) { o.wmin = 1u; o.wmax = 0u; }  // the top bin: nothing lies above it
    o.need_key_eq = need_key_eq;
    o.key_eq = key_eq;
    // First pass over X: the digit is the key's top bits, so "digit > b" and "digit >= b" are comparisons of
    // the element with two numbers -- two instructions per element instead of the whole key transform.
    bool floatcmp = false;
    o.t1 = o.t2 = 0.0f;
    o.flip = 0;
    if constexpr (SRC != SRC_RUNTIME && !PRE) {
        const bool largest = P.dirmask == 0;
        const u32 maxd = (1u << ctx.pi.bits) - 1u;
        const u64 Bo = largest ? sel.bin : maxd - sel.bin;  // the chosen bin in the uncomplemented key domain
        // (only the very first pass over X gets here: no digits of earlier passes above this one's)
        const u64 Ta = Bo << ctx.pi.shift, Tb = (Bo + 1) << ctx.pi.shift;
        float ta, tb;
        if (threshold_number<DT>(Ta, &ta) && threshold_number<DT>(Tb, &tb)) {
            floatcmp = true;
            if (largest) {  // win: key >= Tb (Ta if the whole bin wins); at least candidate: key >= Ta
                o.t1 = sel.emit_all ? ta : tb;
                o.t2 = ta;
                o.flip = ~0ull;
            } else {        // win: key < Ta (Tb if the whole bin wins); at least candidate: key < Tb
                o.t1 = sel.emit_all ? tb : ta;
                o.t2 = tb;
            }
        }
    }

    // The prefilter sweep over fp32 keys: raw-bit counting and one float comparison with the bound's edge, whenever
    // that edge is a number (not at the boundary between the zeros, not among the NaNs).  A bound above every bin
    // (the prefilter declined) keeps nothing: the edge is then an infinity no kept-test passes but NaNs'.
    bool raw_pre = false, keep_none = false;
    if constexpr (PRE && DT == RTOPK_F32 && SRC == SRC_KEY) {
        const bool largest = P.dirmask == 0;
        const u32 maxd = (1u << ctx.pi.bits) - 1u;
        if (ctx.pi.shift + ctx.pi.bits == 32u) {
            if (sel.bin > maxd) {
                raw_pre = keep_none = true;
                o.t2 = largest ? __builtin_inff() : -__builtin_inff();
            } else {
                const u64 Bo = largest ? sel.bin : maxd - sel.bin;
                raw_pre = threshold_number<DT>((largest ? Bo : Bo + 1u) << ctx.pi.shift, &o.t2);
            }
        }
    }

    // The prefilter declined (keys crowded into few bins): if the sample's own bin for the k-th key is one that no
    // NaN can fall into, the sweep also counts the next digit of that bin's elements, by raw bits.  Should the exact
    // counts confirm the bin and it holds nearly the whole row, pass 0 then needs no sweep of its own: the launch after
    // this one classifies X by both digits at once (k_pass0_after_prefilter).
    bool crowd = false;
    u32 crowd_raw = 0, crowd_flip = 0;
    if constexpr (PRE && DT == RTOPK_F32 && SRC == SRC_KEY) {
        const u32 maxd = (1u << ctx.pi.bits) - 1u, top = 1u << (ctx.pi.bits - 1u);
        if (keep_none && crowd_bin <= maxd && pass_pair_is_one_window(P, p)) {
            const bool largest = P.dirmask == 0;
            const u32 dk = largest ? crowd_bin : maxd - crowd_bin;
            crowd_raw = (dk & top) ? (dk & ~top) : (~dk & maxd);  // inverse of key_digit_of_raw
            if ((crowd_raw & (top - 1u)) < (0x7f800000u >> ctx.pi.shift)) {
                crowd = true;
                // below the first digit the ordered key is the raw bits, complemented for negative elements, and once
                // more for "smallest": one rule for the whole bin, whose elements share their sign
                const bool negative = (crowd_raw & top) != 0;
                crowd_flip = negative != !largest ? (1u << P.pass[p + 1].bits) - 1u : 0u;
            }
        }
        if (wg == 0 && tid == 0) st->pre_crowd = crowd ? crowd_bin : 0xffffffffu;
    }
    bool count_second = false;
    if constexpr (PRE) {
        count_second = crowd || (pass_pair_is_one_window(P, p) && sel.bin < (1u << ctx.pi.bits));
        if (count_second)
            for (int j = tid; j < kMaxBins; j += B) sm.hist2[j] = 0;
    }

    if (!SINGLE) {
        if (tid == 0) {
            sm.runW = runW;
            sm.runC = runC;
        }
        __syncthreads();
    }
#ifdef RTOPK_TIMING
    t_pro = wall_clock64();
    if (p == 0) RTOPK_STAMP(8);
#endif
    // An index digit read from X itself (every pass before it left its candidates in place): the digit window reaches
    // up to the top of the inverted index, so what this pass can still want -- its winners and its bin -- are the
    // elements of one stretch of positions, and only the tiles that cover it are read (ties at the k-th key go to the
    // lowest positions: all keys equal, 2^28 of them, k = 2^20: the first 2^20 elements of the row instead of all).
    u32 tile_lo = 0u, tile_hi = 0xffffffffu;
    if constexpr (from_x && !PRE && !SINGLE && SRC == SRC_RUNTIME) {
        if (own_pi.src == SRC_IDX && ctx.pi.shift + ctx.pi.bits >= 32u - (u32)__builtin_clz(ctx.idx_max | 1u)) {
            const bool none_above = o.wmin > o.wmax;
            const u64 w_lo = none_above || o.b < o.wmin ? o.b : o.wmin, w_hi = none_above || o.b > o.wmax ? o.b : o.wmax;
            const u64 u_lo = w_lo << ctx.pi.shift, u_top = ((w_hi + 1u) << ctx.pi.shift) - 1u;
            const u64 u_hi = u_top < (u64)ctx.idx_max ? u_top : (u64)ctx.idx_max;
            if (u_lo <= u_hi) {
                const u64 tile_elems = (u64)B * Source::kSlots;
                const u64 pos_lo = (u64)ctx.idx_max - u_hi + src.lead, pos_hi = (u64)ctx.idx_max - u_lo + src.lead;
                tile_lo = (u32)(pos_lo / tile_elems);
                const u64 th = pos_hi / tile_elems + 1u;
                tile_hi = th < 0xffffffffull ? (u32)th : 0xffffffffu;
            }
        }
    }
    WriteState ws;
    ws.fillW = ws.fillC = 0;
    NextCount nc;
    nc.hist = HistSlot{count_next && !PRE ? sm.hist : nullptr};  // (the prefilter counts in the sweep, every element)
    nc.pi = next_pi;
    nc.dirmask = ctx.dirmask;
    nc.idx_max = ctx.idx_max;
    nc.a_s = ctx.a_s;
    // The prefilter sweep counts pass p + 1's digit of what it keeps in its bound's bin, so that pass p needs no
    // sweep of its own when that bin turns out to be the k-th key's (see sel0).
    if (count_second) {
        nc.count_if = !crowd;
        nc.hist2 = HistSlot{sm.hist2};
        nc.pi = P.pass[p + 1];
        nc.only_bin = sel.bin;
        nc.crowd_raw = crowd_raw;
    }
    if (raw_pre) {
        nc.hist = HistSlot{sm.hist};
        nc.nan_fix = true;
        nc.discard = keep_none;
        nc.nan_shift = ctx.pi.shift;
        nc.nan_bin = (1u << (ctx.pi.bits - 1u)) - 1u;
    }
    if constexpr (kResident && SRC != SRC_RUNTIME) {
        resident([&](const typename Source::Tile& cur) __attribute__((always_inline)) {
            if (cur.full && floatcmp)
                classify_tile<true, true, Source, DT, SRC, B, true>(src, cur, ctx, o, sm, lane, wave, ws, nc);
            else
                classify_tile<false, false, Source, DT, SRC, B, true>(src, cur, ctx, o, sm, lane, wave, ws, nc);
        });
    } else
    // tiles of X are dealt round-robin to the row's workgroups; a candidate segment belongs to one workgroup
    // (one tile prefetched while one is processed; the sweeps that write into the stream of reads measured faster
    // that way than with two)
    // (the tile code is expanded at each of its few places in the pipeline: called, it would find everything it needs
    // in memory, and a call first waits for all the wave's outstanding loads)
    for_each_tile<1>(
        src, own_segment ? 0u : wg, own_segment ? 1u : G, ntiles,
        [&](const typename Source::Tile& cur) __attribute__((always_inline)) {
            if constexpr (PRE && DT == RTOPK_F32 && SRC == SRC_KEY) {
                if (raw_pre && crowd) {
                    if (P.dirmask == 0) prefilter_tile_raw<true, true, true, true, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                    else prefilter_tile_raw<true, true, false, true, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                    return;
                }
                if (raw_pre) {
                    const bool hot = hot_lanes<Source, DT, SRC>(src, cur, ctx) >= 12u;
                    if (P.dirmask == 0) {
                        if (hot) prefilter_tile_raw<true, true, true, false, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                        else prefilter_tile_raw<true, false, true, false, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                    } else {
                        if (hot) prefilter_tile_raw<true, true, false, false, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                        else prefilter_tile_raw<true, false, false, false, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                    }
                    return;
                }
            }
            if constexpr (PRE) {
                // merged adds when the tile's digits are seen to pile up, as in the HIST sweep
                if (hot_lanes<Source, DT, SRC>(src, cur, ctx) >= 12u)
                    classify_tile<true, false, Source, DT, SRC, B, false, true, true>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                else
                    classify_tile<true, false, Source, DT, SRC, B, false, true, false>(src, cur, ctx, o, sm, lane, wave, ws, nc);
            } else if constexpr (SRC != SRC_RUNTIME) {
                if constexpr (!SINGLE) {
                    if (inplace) {
                        inplace_tile_any<true>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                        return;
                    }
                }
                if (floatcmp)
                    classify_tile<true, true, Source, DT, SRC, B, false, false>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                else
                    classify_tile<true, false, Source, DT, SRC, B, false, false>(src, cur, ctx, o, sm, lane, wave, ws, nc);
            } else {
                if constexpr (!SINGLE) {
                    if (inplace) {
                        inplace_tile_any<true>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                        return;
                    }
                }
                classify_tile<true, false, Source, DT, SRC, B>(src, cur, ctx, o, sm, lane, wave, ws, nc);
            }
        },
        [&](const typename Source::Tile& cur) __attribute__((always_inline)) {
            if constexpr (PRE && DT == RTOPK_F32 && SRC == SRC_KEY) {
                if (raw_pre && crowd) {
                    if (P.dirmask == 0) prefilter_tile_raw<false, true, true, true, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                    else prefilter_tile_raw<false, true, false, true, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                    return;
                }
                if (raw_pre) {
                    if (P.dirmask == 0) prefilter_tile_raw<false, true, true, false, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                    else prefilter_tile_raw<false, true, false, false, Source>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                    return;
                }
            }
            if constexpr (!SINGLE && !PRE) {
                if (inplace) {
                    inplace_tile_any<false>(src, cur, ctx, o, sm, lane, wave, ws, nc);
                    return;
                }
            }
            classify_tile<false, false, Source, DT, SRC, B, false, PRE, true>(src, cur, ctx, o, sm, lane, wave, ws, nc);
        },
        tile_lo, tile_hi,
        [&]() __attribute__((always_inline)) {
            if (ws.fillW + ws.fillC > (u32)ST - kStageEarlyRoom) flush_staged<DT, true>(o, sm, lane, wave, ws, nc);
        });
    flush_staged<DT, false>(o, sm, lane, wave, ws, nc);

#ifdef RTOPK_TIMING
    t_sweep = wall_clock64();
    if (p == 0) RTOPK_STAMP(9);
#endif
    if (count_next) {
        // publish the next pass's histogram: LDS -> global (agent-scope atomics), then the suffix sums the
        // next CLASSIFY needs for its offsets, and the segment of the candidate array this workgroup wrote
        __syncthreads();
        if (raw_pre) {
            // the sweep counted by raw top bits: move every count to the bin of its key digit
            constexpr int kPer = kMaxBins / B;
            u32 v[kPer];
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int j = (int)tid + i * B;
                v[i] = j < nb_next ? sm.hist[j] : 0u;
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int j = (int)tid + i * B;
                if (j < nb_next) sm.hist[key_digit_of_raw((u32)j, next_pi.bits, P.dirmask == 0)] = v[i];
            }
            __syncthreads();
        }
        if (!SINGLE) {
            u32* gnext = global_hist(P, pn, row);
            for (int j = tid; j < nb_next; j += B) {
                const u32 c = sm.hist[j];
                if (c) atomicAdd(&gnext[j], c);
            }
        }
        if (next_multi) suffix_sums_in_place<B>(sm.hist, nb_next, sm.wsum);
        if (next_multi) {
            u32* mine = swg_records(P, pn, row) + (size_t)wg * kSwgStride;
            for (int j = tid; j < nb_next; j += B) mine[j] = sm.hist[j];
            if (tid == 0) {
                mine[nb_next] = 0;
                if (!inplace) {  // (in place: the segments are those of the pass that wrote the array, or there are none: X)
                    u32* seg = seg_records(P, out_array, row) + (size_t)wg * 2;
                    seg[0] = runC;
                    seg[1] = PRE ? sm.runC - runC : myC;  // (the prefilter learns its count by writing)
                }
                if (PRE) atomicAdd(&st->pre_kept, sm.runC - runC);
            }
        }
        if (count_second) {
            // the second histogram of a prefilter sweep, published like the first, in buffers of its own
            const int nb2 = 1 << P.pass[pn + 1].bits;
            if (crowd && crowd_flip != 0u) {
                // counted by raw bits: move every count to the bin of its key digit
                constexpr int kPer = kMaxBins / B;
                u32 v[kPer];
#pragma unroll
                for (int i = 0; i < kPer; ++i) {
                    const int j = (int)tid + i * B;
                    v[i] = j < nb2 ? sm.hist2[j] : 0u;
                }
                __syncthreads();
#pragma unroll
                for (int i = 0; i < kPer; ++i) {
                    const int j = (int)tid + i * B;
                    if (j < nb2) sm.hist2[(u32)j ^ crowd_flip] = v[i];
                }
                __syncthreads();
            }
            u32* g2 = hist_buffer(P, kHistSecond, row);
            for (int j = tid; j < nb2; j += B) {
                const u32 c = sm.hist2[j];
                if (c) atomicAdd(&g2[j], c);
            }
            suffix_sums_in_place<B>(sm.hist2, nb2, sm.wsum);
            u32* mine2 = swg_buffer(P, kSwgSecond, row) + (size_t)wg * kSwgStride;
            for (int j = tid; j < nb2; j += B) mine2[j] = sm.hist2[j];
            if (tid == 0) mine2[nb2] = 0;
        }
    }
#ifdef RTOPK_TIMING
    if (!SINGLE && p == 0 && tid == 0) {
        unsigned long long* d = P.dbg + ((size_t)row * P.G + wg) * 16;
        u32 hwid;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hwid));
        d[0] = t_begin; d[1] = t_pro; d[2] = t_sweep; d[3] = wall_clock64(); d[4] = hwid;
    }
#endif
    PassEntry next;
    next.cand = sel.emit_all ? 0u : sel.inside;
    next.k_rem = sel.emit_all ? 0u : sel.k_inside;
    next.out_before = e.out_before + sel.above + (sel.emit_all ? sel.inside : 0u);
    next.finished = sel.emit_all;
    next.prev_multi = !SINGLE;
    next.in_lds = to_rank;
    next.src_array = inplace ? e.src_array : out_array;
    next.src_in_x = inplace && (from_x || e.src_in_x);
    next.chain = inplace ? e.chain + 1u : 0u;
    return next;
}

// ------------------------------------------------------------------------------------------------
// per-row initialisation (Algorithm 1: all inputs are candidates; Section 4.3: draw a_s)
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ u64 mix64(u64 z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

// Called by every thread of a workgroup of at least 128 threads; returns a_s to thread 0 only.
// keep_why: the row was handed over by the one-sweep kernel; what it noted as the reason stays in the record.
template <int DT>
__device__ __forceinline__ float init_row(const Params& P, int row, rtopk_row_trace* st, const RowShape& rs,
                                          bool keep_why = false) {
    static_assert(sizeof(rtopk_row_trace) / 4 <= 128 && offsetof(rtopk_row_trace, a_s) == 0, "trace layout");
    static_assert(offsetof(rtopk_row_trace, redo_why) == 12, "trace layout");
    u32* w = (u32*)st;
    if (threadIdx.x >= 2 && threadIdx.x < sizeof(rtopk_row_trace) / 4 && !(keep_why && threadIdx.x == 3)) w[threadIdx.x] = 0;
    float a_s = 0.0f;
    if (threadIdx.x == 0) {
        if (DT == RTOPK_F32 && (P.flags & RTOPK_FLAG_SCALING) && rs.n != 0) {
            const u64 j = mix64(P.seed + 0x9E3779B97F4A7C15ull * (u64)(row + 1)) % (u64)rs.n;
            const u32 bits = ((const u32*)rs.x)[j];
            if ((bits & 0x7f800000u) != 0x7f800000u) a_s = __uint_as_float(bits);  // finite only
        }
        st->a_s = a_s;
        st->error = rs.bad ? 8u : 0u;
    }
    return a_s;
}

template <int DT>
__global__ void __launch_bounds__(256) k_init(Params P) {
    const int row = blockIdx.x;
    // (the sample's histogram and the second digit's exist only with the prefilter sweep)
    const int buffers = P.pre_stride != 0 ? kHostHistBuffers : kHistRing;
    int bins = 1;  // (as many bins as the widest digit has: with many rows this clearing is the launch's whole time)
    for (int p = 0; p < P.npass; ++p) bins = bins > (1 << P.pass[p].bits) ? bins : 1 << P.pass[p].bits;
    for (int h = 0; h < buffers; ++h) {
        u32* ghist = P.ghist + ((size_t)h * P.batch + row) * kMaxBins;
        for (int j = threadIdx.x; j < bins; j += 256) ghist[j] = 0;
    }
    init_row<DT>(P, row, row_state(P, row), row_shape<KeyOf<DT>::kBytes>(P, row));
}

// ------------------------------------------------------------------------------------------------
// many workgroups per row: one launch per phase per pass, covering every row (task rescheduling,
// Section 3.2.1: pass i of all tasks runs together; grid = workgroups-per-row x rows).
// A pass runs here if the previous one did and left more than `small` candidates; every workgroup
// evaluates that on records no kernel of the same pass writes, so all of them agree.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ bool multi_runs_pass(const Params& P, const PassEntry& e, int p) {
    if (p == 0) return true;
    return e.prev_multi && !e.finished && e.cand > P.small;
}

template <int DT, int SRC, bool NT>
__global__ void __launch_bounds__(kGridBlock) k_hist_keys(Params P) {
    __shared__ Shared<kGridBlock> sm;
    const int row = blockIdx.y;
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    if (rs.k == 0) return;  // (ragged batches: an empty row, or nothing wanted from it)
    rtopk_row_trace* st = row_state(P, row);
    KeySource<DT, kGridBlock, key_vecs<DT>(), NT> src;
    src.init(rs);
    hist_phase<decltype(src), DT, SRC, kGridBlock, false>(src, P, 0, row, blockIdx.x, gridDim.x, st->a_s,
                                                          pass_entry(P, st, 0, rs), st, sm);
}

template <int DT, int SRC, bool NT>
__global__ void __launch_bounds__(kGridBlock) k_classify_keys(Params P) {
    __shared__ Shared<kGridBlock> sm;
    const int row = blockIdx.y;
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    if (rs.k == 0) return;  // (ragged batches: an empty row, or nothing wanted from it)
    rtopk_row_trace* st = row_state(P, row);
    const PassEntry e = pass_entry(P, st, 0, rs);
    KeySource<DT, kGridBlock, key_vecs<DT>(), NT> src;
    src.init(rs);
    const u32 ntiles = src.ntiles();
    // every workgroup repeats selectBin on the row's global histogram (cheap, and it spares a grid-wide hand-off)
    const Selection sel = select_pass<kGridBlock>(PlainCounts{global_hist(P, 0, row)}, 1 << P.pass[0].bits, e, sm, st);
    classify_phase<decltype(src), DT, SRC, kGridBlock, false>(src, P, 0, row, rs.k, blockIdx.x, gridDim.x, e, st, st->a_s, sm, 1u,
                                                              sel, ntiles < gridDim.x ? ntiles : gridDim.x, false);
}

// The prefilter sweep.  selectBin on the sample's histogram, for the sample rank that stands for the row's k-th
// key (with a margin), gives a bin that very probably is the k-th key's or lies below it.  ONE sweep over X then
// does pass 0's countBin for every element (so selectBin of pass 0 is exact, as after a HIST sweep) and moves
// everything from that bin upwards into the candidate array.  Pass 0 runs on those candidates like any later
// pass: X is read once instead of twice.  When the exact counts put the k-th key's bin below the bound, pass 0
// is the ordinary CLASSIFY sweep over X instead (k_pass0_after_prefilter decides); the result never depends on
// the sample.
// BIG: the launch puts at most one workgroup on a compute unit, so each wave can stage three times as much
// before it has to write.  That matters more than its size suggests: a wave's stores and its prefetches share one
// in-order completion counter, so every write-back in mid-sweep holds the wave until the stores are acknowledged
// (config 4, 0.85 % of the row kept: about six write-backs per wave cost 25 us of a 190 us sweep; with room for
// 1536 entries nearly everything a wave keeps leaves in one piece when its sweep has ended).
constexpr int kStageBig = 1536;
template <int DT, int SRC, bool NT, bool BIG>
__global__ void __launch_bounds__(kGridBlock) k_prefilter_keys(Params P) {
    __shared__ Shared<kGridBlock, BIG ? kStageBig : kStage> sm;
    const int row = blockIdx.y;
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    if (rs.k == 0) return;  // (ragged batches: an empty row, or nothing wanted from it)
    rtopk_row_trace* st = row_state(P, row);
    PassEntry e = pass_entry(P, st, 0, rs);
    KeySource<DT, kGridBlock, key_vecs<DT>(), NT> src;
    src.init(rs);
    const RowSample sample = row_sample(src, P, rs.k);
    // a rank beyond the sample (or an empty sample) selects nothing: bin 0, everything is kept
    e.k_rem = sample.rank < (u64)sample.elems ? (u32)sample.rank : sample.elems + 1u;
    bool ignored;
    Selection sel = select_pass<kGridBlock>(PlainCounts{hist_buffer(P, kHistSample, row)}, 1 << P.pass[0].bits, e, sm, st, &ignored);
    // If the sample says that more than an eighth of the row (a sixteenth for 16-bit keys, whose candidates are
    // four times their size) lies in the bins that would be kept -- keys crowded into one bin: a narrow range,
    // many duplicates --, writing that much out and reading it back costs more than the second sweep over X:
    // keep nothing (a bound above every bin), only count, and let pass 0 sweep X.
    constexpr u32 kCrowded = DT == RTOPK_F32 ? 8u : 16u;
    u32 crowd_bin = 0xffffffffu;  // ... and say which bin the sample puts the k-th key in (see classify_phase: crowd)
    if ((u64)(sel.above + sel.inside) * kCrowded > (u64)sample.elems) {
        crowd_bin = sel.bin;
        sel.bin = 1u << P.pass[0].bits;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) st->pre_bound = sel.bin;
    e.k_rem = rs.k;
    classify_phase<decltype(src), DT, SRC, kGridBlock, false, NoResident, true>(src, P, 0, row, rs.k, blockIdx.x, gridDim.x, e, st,
                                                                                st->a_s, sm, 1u, sel, gridDim.x, false,
                                                                                NoResident(), nullptr, crowd_bin);
}

// Pass 0 after a prefilter sweep.  Every workgroup repeats selectBin on the exact counts that sweep left.  If the
// k-th key's bin is among those the sweep kept (nearly always), workgroup w classifies the candidates workgroup w
// kept, as in any later pass; otherwise the sample misled the prefilter and this is the ordinary CLASSIFY sweep
// over X (same tiles per workgroup as in the prefilter sweep, whose per-workgroup records give the offsets).
template <int DT, bool NT>
__global__ void __launch_bounds__(kGridBlock) k_pass0_after_prefilter(Params P) {
    __shared__ Shared<kGridBlock> sm;
    const int row = blockIdx.y;
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    if (rs.k == 0) return;  // (ragged batches: an empty row, or nothing wanted from it)
    rtopk_row_trace* st = row_state(P, row);
    const PassEntry e = pass_entry(P, st, 0, rs);
    const Selection sel = select_pass<kGridBlock>(PlainCounts{global_hist(P, 0, row)}, 1 << P.pass[0].bits, e, sm, st);
    const u32 bound = st->pre_bound;
    if (sel.bin >= bound) {
        const u32* seg = seg_records(P, 1u, row) + (size_t)blockIdx.x * 2;
        CandSource<kGridBlock, kVecs> src;
        src.init(P.cand[1] + (size_t)row * P.cand_stride, seg[0], seg[1], (u32)P.cand_stride);
        if (sel.bin == bound && !sel.emit_all && pass_pair_is_one_window(P, 0)) {
            // The bound's bin is the k-th key's: the sweep has counted pass 1's digit for exactly this bin, so pass 0
            // is its selectBin and nothing else, and pass 1's sweep over what was kept classifies by both digits.
            PassEntry e1;
            e1.cand = sel.inside;
            e1.k_rem = sel.k_inside;
            e1.out_before = sel.above;
            e1.finished = false;
            e1.prev_multi = true;
            e1.in_lds = false;
            e1.src_array = 1u;
            e1.src_in_x = false;
            e1.chain = 0;
            __syncthreads();  // everybody has read the first selectBin's result: its LDS words may be reused
            const Selection sel1 = select_pass<kGridBlock>(PlainCounts{hist_buffer(P, kHistSecond, row)}, 1 << P.pass[1].bits,
                                                           e1, sm, st);
            classify_phase<decltype(src), DT, SRC_RUNTIME, kGridBlock, false>(src, P, 1, row, rs.k, blockIdx.x, gridDim.x, e1, st,
                                                                              st->a_s, sm, 1u, sel1, gridDim.x, true,
                                                                              NoResident(), &sel);
        } else {
            classify_phase<decltype(src), DT, SRC_RUNTIME, kGridBlock, false>(src, P, 0, row, rs.k, blockIdx.x, gridDim.x, e, st,
                                                                              st->a_s, sm, 1u, sel, gridDim.x, true);
        }
    } else {
        const bool declined = bound == (1u << P.pass[0].bits);
        if (blockIdx.x == 0 && threadIdx.x == 0) st->pre_missed = declined ? 2u : 1u;
        KeySource<DT, kGridBlock, key_vecs<DT>(), NT> src;
        src.init(rs);
        const u32 ntiles = src.ntiles();
        const u32 records = ntiles < gridDim.x ? ntiles : gridDim.x;
        if (declined && st->pre_crowd == sel.bin && !sel.emit_all && pass_pair_is_one_window(P, 0) && sel.inside > P.small &&
            (u64)sel.inside * 8u > (u64)e.cand * 7u) {
            // The sweep declined to keep anything, named the bin the sample crowds into, and counted pass 1's digit for
            // that bin; the exact counts confirm the bin and it holds nearly the whole row.  Pass 0 is then an in-place
            // pass with no sweep, and pass 1 classifies X by both digits at once.
            PassEntry e1;
            e1.cand = sel.inside;
            e1.k_rem = sel.k_inside;
            e1.out_before = sel.above;
            e1.finished = false;
            e1.prev_multi = true;
            e1.in_lds = false;
            e1.src_array = 0u;
            e1.src_in_x = true;
            e1.chain = 1u;
            __syncthreads();  // everybody has read the first selectBin's result: its LDS words may be reused
            const Selection sel1 = select_pass<kGridBlock>(PlainCounts{hist_buffer(P, kHistSecond, row)}, 1 << P.pass[1].bits,
                                                           e1, sm, st);
            classify_phase<decltype(src), DT, SRC_RUNTIME, kGridBlock, false>(src, P, 1, row, rs.k, blockIdx.x, gridDim.x, e1, st,
                                                                              st->a_s, sm, 1u, sel1, records, false, NoResident(),
                                                                              &sel);
        } else {
            classify_phase<decltype(src), DT, SRC_KEY, kGridBlock, false>(src, P, 0, row, rs.k, blockIdx.x, gridDim.x, e, st,
                                                                          st->a_s, sm, 1u, sel, records, false);
        }
    }
}

// Pass p >= 1 on the grid: workgroup w classifies the candidates workgroup w kept in the sweep before -- or, after
// in-place passes that began with the first, its tiles of X once more.
template <int DT, bool NT>
__global__ void __launch_bounds__(kGridBlock) k_classify_cand(Params P, int p) {
    __shared__ Shared<kGridBlock> sm;
    const int row = blockIdx.y;
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    if (rs.k == 0) return;  // (ragged batches: an empty row, or nothing wanted from it)
    rtopk_row_trace* st = row_state(P, row);
    // (pass 1 may have been done together with pass 0, by the launch before this one: st->pre_merged, which that
    // launch wrote and this one only reads)
    if (p == 1 && st->pre_merged != 0u) return;
    const PassEntry e = pass_entry(P, st, p, rs);
    if (!multi_runs_pass(P, e, p)) return;
    const Selection sel = select_pass<kGridBlock>(PlainCounts{global_hist(P, p, row)}, 1 << P.pass[p].bits, e, sm, st);
    if (e.src_in_x) {
        KeySource<DT, kGridBlock, key_vecs<DT>(), NT> src;
        src.init(rs);
        const u32 ntiles = src.ntiles();
        classify_phase<decltype(src), DT, SRC_RUNTIME, kGridBlock, false>(src, P, p, row, rs.k, blockIdx.x, gridDim.x, e, st,
                                                                          st->a_s, sm, 1u, sel,
                                                                          ntiles < gridDim.x ? ntiles : gridDim.x, false);
    } else {
        const u32* seg = seg_records(P, e.src_array, row) + (size_t)blockIdx.x * 2;
        CandSource<kGridBlock, kVecs> src;
        src.init(P.cand[e.src_array] + (size_t)row * P.cand_stride, seg[0], seg[1], (u32)P.cand_stride);
        // its own tiles only: the segment is this workgroup's alone
        classify_phase<decltype(src), DT, SRC_RUNTIME, kGridBlock, false>(src, P, p, row, rs.k, blockIdx.x, gridDim.x, e, st,
                                                                          st->a_s, sm, 1u, sel, gridDim.x, true);
    }
}

// ------------------------------------------------------------------------------------------------
// one workgroup per row
// ------------------------------------------------------------------------------------------------

// The ranking step: C <= kRankCap candidates, one per lane, are ordered directly by their extended key
// (ordered key, then idx_max - index: all distinct).  A candidate's rank is the number of candidates that
// beat it; the k_rem best go to the output at the position their rank gives, so this part of the output is
// written in rank order.  It stands for every digit pass still to come (same winners as Algorithm 1's
// remaining iterations would find, since those order by exactly these bits), and leaves one record.
template <int DT>
__device__ __forceinline__ void rank_finish(const Params& P, int row, u32 row_k, rtopk_row_trace* st, Shared<kRowBlock>& sm,
                                            int p, const PassEntry& e, u32 where) {
    static_assert(kRankCap + 8 <= (u32)kRowBlock && kRankCap * 16 + 64 <= sizeof(sm.hist), "one lane per candidate");
    const u32 tid = threadIdx.x;
    const u32 C = e.cand;
    uint2* list = (uint2*)sm.hist;                    // (raw bits, index)
    u64* ext = (u64*)(sm.hist + 2 * kRankCap);        // extended keys
    if (!e.in_lds) {
        const uint2* cand = P.cand[e.src_array] + (size_t)row * P.cand_stride;
        if (tid < C) list[tid] = cand[tid];
    }
    __syncthreads();
    uint2 mine = make_uint2(0u, 0u);
    u64 my = 0;
    if (tid < C) {
        mine = list[tid];
        my = ((u64)(KeyOf<DT>::key(mine.x) ^ P.dirmask) << 32) | (u64)(P.idx_max - mine.y);
        ext[tid] = my;
    } else if (tid < C + 8u) {
        ext[tid] = 0;
    }
    __syncthreads();
    if (tid < ((C + 63u) & ~63u)) {  // whole waves: the loop's LDS reads are wave-uniform broadcasts
        u32 rank = 0;
        for (u32 j = 0; j < C; j += 8) {  // (the list is padded with keys that beat nobody)
            u64 q[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) q[i] = ext[j + i];
#pragma unroll
            for (int i = 0; i < 8; ++i) rank += q[i] > my ? 1u : 0u;
        }
        if (tid < C && rank < e.k_rem) {
            const u32 pos = e.out_before + rank;
            if (pos < row_k) {
                store_value<DT>((char*)P.out_values + (size_t)row * (size_t)P.k * KeyOf<DT>::kBytes, pos, mine.x);
                P.out_indices[(size_t)row * (size_t)P.k + pos] = (long long)mine.y;
            }
        }
    }
    if (tid == 0) {
        if (e.k_rem == 0 || e.k_rem > C) st->error |= 1u;  // inconsistent state: never expected
        st->pass_rec[p].bin = 0;
        st->pass_rec[p].k_after = 0;
        st->pass_rec[p].cand_after = 0;
        st->pass_rec[p].winners = e.k_rem;
        st->pass_rec[p].out_before = e.out_before;
        st->pass_rec[p].cand_before = C;
        st->pass_rec[p].window = SRC_RANK;
        st->pass_rec[p].where = where;
    }
}

// Remaining passes of one row on its candidate arrays, by a single workgroup, starting at pass p with loop
// state e.  `hist_from` says where pass p's histogram is; every later pass finds its counts in LDS, left there
// by the pass before it.
template <int DT>
__device__ __forceinline__ void finish_row(const Params& P, int row, const RowShape& rs, rtopk_row_trace* st, float a_s,
                                           Shared<kRowBlock>& sm, int p, PassEntry e, int hist_from, u32 where) {
    for (; p < P.npass; ++p) {
        if (e.finished) return;
        __syncthreads();  // the previous pass's candidates are visible to the whole workgroup
        if (e.cand <= kRankCap && P.pass[p].src != SRC_SCALED) {
            rank_finish<DT>(P, row, rs.k, st, sm, p, e, where);
            return;
        }
        CandSource<kRowBlock, kVecs> src;
        src.init(P.cand[e.src_array] + (size_t)row * P.cand_stride, 0u, e.cand, (u32)P.cand_stride);
        const int nb = 1 << P.pass[p].bits;
        const Selection sel = hist_from == HIST_IN_GLOBAL
            ? select_pass<kRowBlock>(PlainCounts{global_hist(P, p, row)}, nb, e, sm, st)
            : select_pass<kRowBlock>(PlainCounts{sm.hist}, nb, e, sm, st);
        e = classify_phase<decltype(src), DT, SRC_RUNTIME, kRowBlock, true>(src, P, p, row, rs.k, 0u, 1u, e, st, a_s, sm, where,
                                                                            sel, 1u, true);
        hist_from = HIST_IN_LDS;
    }
    // digits exhausted: extended keys are unique, so the last pass must have taken its whole bin
    if (threadIdx.x == 0 && !e.finished) st->error |= 2u;
}

template <int DT>
__global__ void __launch_bounds__(kRowBlock) k_finish(Params P) {
    __shared__ Shared<kRowBlock> sm;
    const int row = blockIdx.x;
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    if (rs.k == 0) return;  // (ragged batches: an empty row, or nothing wanted from it)
    rtopk_row_trace* st = row_state(P, row);
    int p = 0;
    while (p < P.npass && st->pass_rec[p].where != 0u) ++p;  // first pass the grid kernels left undone
    if (p == P.npass) return;
    const PassEntry e = pass_entry(P, st, p, rs);
    if (e.src_in_x) {  // never expected: a pass that leaves its candidates in X leaves more than this kernel takes
        if (threadIdx.x == 0) st->error |= 16u;
        return;
    }
    finish_row<DT>(P, row, rs, st, st->a_s, sm, p, e, HIST_IN_GLOBAL, 2u);  // its histogram was published by the pass before it
}

// Whole selection of one row in one kernel (many short rows: no global atomics, no extra launches).
// only_redo: handle just the rows the one-sweep kernel marked.
template <int DT, int SRC>
__global__ void __launch_bounds__(kRowBlock) k_row(Params P, bool only_redo) {
    __shared__ Shared<kRowBlock> sm;
    const int row = blockIdx.x;
    rtopk_row_trace* st = row_state(P, row);
    if (only_redo && st->redo != 1u) return;
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    const float drawn = init_row<DT>(P, row, st, rs, only_redo);
    if (rs.k == 0) return;  // (ragged batches: an empty row, or nothing wanted from it)
    if (threadIdx.x == 0) sm.a_s = drawn;
    __syncthreads();
    const float a_s = sm.a_s;
    const PassEntry e = pass_entry(P, st, 0, rs);
    KeySource<DT, kRowBlock, key_vecs<DT>(), false> src;
    src.init(rs);
    const Selection sel = hist_phase<decltype(src), DT, SRC, kRowBlock, true>(src, P, 0, row, 0u, 1u, a_s, e, st, sm);
    const PassEntry e1 = classify_phase<decltype(src), DT, SRC, kRowBlock, true>(src, P, 0, row, rs.k, 0u, 1u, e, st, a_s, sm, 3u,
                                                                                 sel, 1u, true);
    finish_row<DT>(P, row, rs, st, a_s, sm, 1, e1, HIST_IN_LDS, 3u);
}

// The same for a row that fits one workgroup's registers (1024 lanes x 16 vectors x 16 bytes = 256 KiB):
// X is read from HBM exactly once -- the histogram sweep consumes the tiles as they arrive and keeps them, the
// classify sweep runs on the registers.
constexpr int kResidentVecs = 16;
// f(tile) for each of the first `ntiles` tiles, unrolled by recursion: every tile must stay a named set of
// registers (a loop over the array, even one asked to unroll, may be kept as a loop and spill the row).
template <int C, int N, class Tile, class F>
__device__ __forceinline__ void each_resident_tile(const Tile (&t)[N], u32 ntiles, F&& f) {
    if constexpr (C < N) {
        if ((u32)C < ntiles) f(t[C]);
        each_resident_tile<C + 1>(t, ntiles, f);
    }
}
// The same while the row is still arriving: tile C + AHEAD is requested before tile C is used, so the lanes
// that wait for memory and the lanes that count overlap.
template <int C, int AHEAD, int N, class Source, class F>
__device__ __forceinline__ void each_arriving_tile(const Source& src, typename Source::Tile (&t)[N], u32 ntiles, F&& f) {
    if constexpr (C < N) {
        if constexpr (C + AHEAD < N)
            if ((u32)(C + AHEAD) < ntiles) src.load(C + AHEAD, threadIdx.x, t[C + AHEAD]);
        if ((u32)C < ntiles) f(t[C]);
        each_arriving_tile<C + 1, AHEAD>(src, t, ntiles, f);
    }
}

template <int DT, int SRC>
__global__ void __launch_bounds__(kRowBlock) k_row_resident(Params P, bool only_redo) {
    __shared__ Shared<kRowBlock> sm;
    typedef KeySource<DT, kRowBlock, key_vecs<DT>(), false> Source;
    constexpr int kTiles = kResidentVecs / key_vecs<DT>();
    if (only_redo && row_state(P, blockIdx.x)->redo != 1u) return;
#ifdef RTOPK_X_AHEAD
    constexpr int kAhead = RTOPK_X_AHEAD;
#else
    constexpr int kAhead = kTiles / 2;
#endif
    typename Source::Tile t[kTiles];
    const int row = blockIdx.x;
    rtopk_row_trace* st = row_state(P, row);
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    Source src;
    src.init(rs);
    const u32 ntiles = src.ntiles();
#ifdef RTOPK_TIMING
    unsigned long long tt[6];
    tt[4] = wall_clock64();
#endif
    const float drawn = init_row<DT>(P, row, st, rs, only_redo);
    if (rs.k == 0) return;  // (ragged batches: an empty row, or nothing wanted from it)
    if (threadIdx.x == 0) sm.a_s = drawn;
    __syncthreads();
    const float a_s = sm.a_s;
    const PassEntry e = pass_entry(P, st, 0, rs);
    auto arriving = [&](auto&& f) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < kAhead; ++c)
            if ((u32)c < ntiles) src.load(c, threadIdx.x, t[c]);
        each_arriving_tile<0, kAhead>(src, t, ntiles, f);
    };
    auto resident = [&](auto&& f) __attribute__((always_inline)) { each_resident_tile<0>(t, ntiles, f); };
#ifdef RTOPK_TIMING
    tt[0] = wall_clock64();
#endif
    const Selection sel = hist_phase<Source, DT, SRC, kRowBlock, true>(src, P, 0, row, 0u, 1u, a_s, e, st, sm, arriving);
#ifdef RTOPK_TIMING
    tt[1] = wall_clock64();
#endif
    const PassEntry e1 = classify_phase<Source, DT, SRC, kRowBlock, true>(src, P, 0, row, rs.k, 0u, 1u, e, st, a_s, sm, 3u, sel,
                                                                          1u, true, resident);
#ifdef RTOPK_TIMING
    tt[2] = wall_clock64();
#endif
    finish_row<DT>(P, row, rs, st, a_s, sm, 1, e1, HIST_IN_LDS, 3u);
#ifdef RTOPK_TIMING
    tt[3] = wall_clock64();
    if (threadIdx.x == 0) {
        unsigned long long* d = P.dbg + (size_t)row * P.G * 16;
        for (int i = 0; i < 5; ++i) d[i] = tt[i];
    }
#endif
}

// ------------------------------------------------------------------------------------------------
// one workgroup per row, ONE sweep (small k)
//
// selectBin on any part of a row bounds the whole row's answer from below: the k-th best key of a subset
// is never better than the k-th best of the row, so the bin b0 it falls in satisfies b0 <= b.  And selectBin
// only ever needs the counts of the bins from b upwards.  So the kernel counts the first part of the row
// (countBin as usual), takes b0 from it, and then sweeps the whole row once doing nothing but comparing each
// element with the lower edge of bin b0: the few that are not below it are noted and then set aside in LDS,
// with their index.  Those are all the elements of bins >= b0, so their histogram is the top of the row's histogram,
// exactly: selectBin, selectCandidate and the filter run on the list.  There is no second sweep, the bulk of
// the row is never counted, and the row is not kept anywhere, so the kernel needs few registers and little
// LDS and three workgroups share a compute unit: one row's trip from HBM overlaps the others' work.
//
// Whatever does not fit the short way -- inf/NaN in the first part (see hist_tile_raw), more set aside than the
// list holds, more than kStreamRank candidates in the chosen bin, a bin edge that is not
// a number -- is left to the two-sweep kernel: the row is marked (`redo`) and the launch that follows handles exactly the marked
// rows.
// ------------------------------------------------------------------------------------------------
constexpr int kStreamBlock = 512;
constexpr u32 kStreamList = 2048;                    // elements set aside per row, at most (k <= kStreamSmallK)
constexpr u32 kStreamListMid = 2816;                 // ... for larger k: what still lets four workgroups share 160 KB of LDS
constexpr u32 kStreamSmallK = 256;                   // up to here the bound comes from the row's first part, beyond from a sample
constexpr u32 kStreamSampleStride = 4;               // the sample: every 4th tile of the row
constexpr u32 kStreamRank = 2 * kStreamBlock - 64;   // candidates ranked directly, at most (two per lane)
constexpr u32 kStreamWide = kMaxBins + 8;            // words for the copies of the histogram (1 x 4097, 2 x 2049)
constexpr u32 kStreamChunk = 16;                     // tiles swept between two rounds of fetching the hits
constexpr unsigned long long kStreamStagger = 1000;  // ticks of the 100 MHz wall clock between the starts of two groups

template <u32 LIST>
struct SharedStream {
    union {
        u32 wide[kStreamWide];              // copies of the first part's histogram (see HistSlot); then the lanes'
                                            // hit masks of one chunk (16 bits x kStreamBlock x kStreamChunk); then
                                            // the list's histogram
        struct {                            // after the last selectBin: the ranking step's arrays
            uint2 rank_list[2 * kStreamBlock];
            u64 rank_ext[2 * kStreamBlock];
        };
    };
    uint2 list[LIST];                       // (raw bits, index) of the elements set aside
    u32 wsum[kStreamBlock / 64];
    u32 selv[5];
    u32 nlist, runW, runC;
};

// Raw-bit bins visited in key order, with the distrust rule of hist_tile_raw.
struct RawCounts {
    const u32* wide;
    u32 copies, stride, top, mask, first_special;
    bool largest;
    __device__ __forceinline__ u32 operator()(u32 keybin, bool* bad) const {
        const u32 dk = largest ? keybin : mask - keybin;
        const u32 draw = (dk & top) ? (dk & ~top) : (~dk & mask);  // inverse of key_digit_of_raw
        u32 c = 0;
        for (u32 q = 0; q < copies; ++q) c += wide[q * stride + draw];
        if (c != 0 && (draw & (top - 1u)) >= first_special) *bad = true;
        return c;
    }
};

// One tile of the single sweep: an element is a hit iff it is not below thr (LARGEST; true for a NaN) or below
// thr (otherwise).  Neither a branch per 64 elements nor much arithmetic per element is affordable here
// (measured: with either the sweep takes 2-3 times what the row's trip from HBM takes), and hits are too
// frequent -- one slot in five has some -- to be tested for in bulk.  So the sweep only notes them: every lane
// shifts one bit per slot into a private mask (compare + add-with-carry) and leaves the mask of the tile's
// kSlots slots in LDS; the elements are fetched again afterwards, by the same lane, from the caches.
// Returns the lane's mask: slot s is bit kSlots - 1 - s.
template <bool FULL, bool LARGEST, class Source, int DT>
__device__ __forceinline__ u32 stream_tile(const Source& src, const typename Source::Tile& t, float thr) {
    u32 bits = 0;
#pragma unroll
    for (int s = 0; s < Source::kSlots; ++s) {
        const float x = src.template value<SRC_KEY>(t, s, 0.0f);
        if (FULL) {
            // bits = 2 * bits + hit, as compare-into-carry + add-with-carry: two instructions per element (the
            // compiler's own choice -- select 0/1, shift, or -- is three, and this loop is bound by them)
            if (LARGEST)
                asm("v_cmp_ngt_f32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(bits) : "v"(thr), "v"(x) : "vcc");
            else
                asm("v_cmp_gt_f32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(bits) : "v"(thr), "v"(x) : "vcc");
        } else {
            u32 raw, idx;
            bool valid;
            src.get(t, s, raw, idx, valid);
            const bool hit = (LARGEST ? !(x < thr) : (x < thr)) && valid;
            bits = bits + bits + (hit ? 1u : 0u);
        }
    }
    return bits;
}

template <int DT, u32 LIST>
__global__ void __launch_bounds__(kStreamBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) k_row_stream(Params P) {
    static_assert(4 * sizeof(SharedStream<LIST>) <= 160 * 1024, "four workgroups per compute unit");
    __shared__ SharedStream<LIST> sm;
    constexpr int B = kStreamBlock;
    constexpr bool SINGLE = true;  // (for the diagnostic stamps)
    typedef KeySource<DT, B, key_vecs<DT>(), false> Source;
    const int row = blockIdx.x;
    rtopk_row_trace* st = row_state(P, row);
    const u32 tid = threadIdx.x, lane = lane_id();
    // Four of these workgroups share a compute unit, and workgroups launched together march through their phases
    // together: all count (LDS), then all sweep (memory), then all fetch (latency).  The groups of 256 workgroups --
    // one per compute unit each -- therefore start 10 us apart, for as many groups as are resident at once, so that
    // on a compute unit one row's trip to memory overlaps the others' counting (1024 rows of 2^17 bf16 keys:
    // 82 -> 75 us; 3 or 6 us apart: 80; 15 us: 84).  The wait is bounded by the clock it reads.
    {
        const unsigned long long t0 = wall_clock64(), wait = (unsigned long long)((blockIdx.x >> 8) & 3u) * kStreamStagger;
        while (wall_clock64() - t0 < wait) __builtin_amdgcn_s_sleep(16);
    }
    RTOPK_STAMP(0);
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    init_row<DT>(P, row, st, rs);
    if (rs.k == 0) return;  // (ragged batches: an empty row, or nothing wanted from it)
    Source src;
    src.init(rs);
    const u32 ntiles = src.ntiles();
    const DigitCtx ctx = make_digit_ctx(P, 0, 0.0f);
    const int nb = 1 << ctx.pi.bits;
    const bool largest = P.dirmask == 0;
    // copies of the histogram: as many as fit (a power of two, at most 8)
    const u32 stride = (u32)nb + 1u;
    u32 copies = 1;
    while (copies < 8u && 2u * copies * stride <= kStreamWide) copies *= 2u;
    HistSlot hs{sm.wide + (lane & (copies - 1u)) * stride};
    RawCounts counts{sm.wide, copies, stride, (u32)nb >> 1, (u32)nb - 1u,
                     (DT == RTOPK_F16 ? 0x7c000000u : 0x7f800000u) >> ctx.pi.shift, largest};
    for (u32 j = tid; j < copies * stride; j += B) sm.wide[j] = 0;
    if (tid == 0) sm.nlist = 0;
    __syncthreads();

    // ---- countBin on the first part of the row: an eighth of it, more for larger k (about k * row / part
    // elements will be set aside: keep that near 512), and enough to hold k elements
    // For larger k a first part long enough would be most of the row.  There the bound comes from a SAMPLE -- every
    // 4th tile, so a trend along the row cannot mislead it -- for a rank with a margin (as the grid prefilter's), and
    // is checked afterwards: if the list ends up with at least k elements, the k-th key is in it and the list is the
    // top of the row, exactly as with a guaranteed bound; if not, the sample misled and the row is handed over.
    constexpr u32 kTileElems = (u32)B * Source::kSlots;
    const bool sampled = rs.k > kStreamSmallK;
    u32 t0 = (ntiles + 7u) / 8u;
    const u32 by_k = (u32)(((u64)rs.k * ntiles + 511u) / 512u);
    const u32 need = (rs.k + src.lead + kTileElems - 1u) / kTileElems;
    if (t0 < by_k) t0 = by_k;
    if (t0 < need) t0 = need;
    if (t0 > ntiles || sampled) t0 = ntiles;
    auto nothing = []() __attribute__((always_inline)) {};
    for_each_tile<2>(
        src, 0u, sampled ? kStreamSampleStride : 1u, ntiles,
        [&](const typename Source::Tile& cur) __attribute__((always_inline)) { hist_tile_raw<true, Source>(src, cur, ctx, hs); },
        [&](const typename Source::Tile& cur) __attribute__((always_inline)) { hist_tile_raw<false, Source>(src, cur, ctx, hs); }, 0u, t0);
    __syncthreads();
    RTOPK_STAMP(1);
    u32 why = 0;  // diagnostic: what sent the row to the two-sweep kernel
    float thr = 0.0f;
    u32 b0 = 0;
    {
        // how many elements have been counted?  (tiles [0, t0) hold elements [0, t0 * tile - lead) of the row; of the
        // sampled tiles 0, 4, 8, ... only the row's last one can be short)
        u32 seen, want = rs.k;
        if (sampled) {
            const u32 ns = (ntiles + kStreamSampleStride - 1u) / kStreamSampleStride;
            u64 s64 = (u64)ns * kTileElems - src.lead;
            if ((ntiles - 1u) % kStreamSampleStride == 0u) s64 -= (u64)ntiles * kTileElems - src.lead - rs.n;
            seen = (u32)s64;
            // the sample rank that stands for the row's k-th key: its share, an eighth more, eight standard deviations
            // of a binomial count, and 16
            const u32 ks = (u32)(((u64)rs.k * seen + rs.n - 1u) / rs.n);
            want = ks + ks / 8u + 8u * (u32)__builtin_sqrtf((float)ks) + 16u;
        } else {
            const u64 seen64 = (u64)t0 * kTileElems - src.lead;
            seen = seen64 < (u64)rs.n ? (u32)seen64 : rs.n;
        }
        bool distrust = false;
        Selection s0{};
        if (seen >= want) s0 = select_from_counts<B>(counts, nb, want, sm, st, nothing, &distrust);
        b0 = s0.bin;
        // the bound as a number: set aside what is not below the lower edge of bin b0 ("largest"), or what
        // is below its upper edge ("smallest": keys are complemented, bin b0 is raw bin maxd - b0)
        const u32 maxd = (u32)nb - 1u;
        const u64 Bo = largest ? b0 : maxd - b0;
        const u64 T = (largest ? Bo : Bo + 1u) << ctx.pi.shift;
        if (seen < want) why = 2u;
        else if (distrust) why = 1u;
        else if (!threshold_number<DT>(T, &thr)) why = 3u;
        // the part's own share of bins >= b0, scaled to the row, is what the sweep will set aside: give up now
        // if that will not fit (a wide bin at the edge, say uniform data just below a power of two)
        else if (!sampled && (u64)(s0.above + s0.inside) * ntiles > (u64)(LIST * 3u / 4u) * t0) why = 7u;
        else if (sampled && (u64)(s0.above + s0.inside) * rs.n > (u64)(LIST * 9u / 10u) * seen) why = 7u;
    }
    RTOPK_STAMP(2);
    if (why == 0) {
        // ---- the sweep, in chunks of kStreamChunk tiles: the sweep notes the hits, then every lane fetches its own
        static_assert(Source::kSlots == 16, "one 16-bit mask per lane and tile");
        unsigned short* masks = (unsigned short*)sm.wide;  // [tile in chunk][lane]; the first part's histogram is done with
        const char* row_bytes = rs.x;
        for (u32 c0 = 0; c0 < ntiles; c0 += kStreamChunk) {
            const u32 c1 = c0 + kStreamChunk < ntiles ? c0 + kStreamChunk : ntiles;
            auto note = [&](const typename Source::Tile& cur, u32 bits) __attribute__((always_inline)) {
                masks[(cur.tile - c0) * (u32)B + tid] = (unsigned short)bits;
            };
            if (largest)
                for_each_tile<2>(
                    src, 0u, 1u, ntiles,
                    [&](const typename Source::Tile& cur) __attribute__((always_inline)) { note(cur, stream_tile<true, true, Source, DT>(src, cur, thr)); },
                    [&](const typename Source::Tile& cur) __attribute__((always_inline)) { note(cur, stream_tile<false, true, Source, DT>(src, cur, thr)); },
                    c0, c1);
            else
                for_each_tile<2>(
                    src, 0u, 1u, ntiles,
                    [&](const typename Source::Tile& cur) __attribute__((always_inline)) { note(cur, stream_tile<true, false, Source, DT>(src, cur, thr)); },
                    [&](const typename Source::Tile& cur) __attribute__((always_inline)) { note(cur, stream_tile<false, false, Source, DT>(src, cur, thr)); },
                    c0, c1);
            if (c0 == 0) RTOPK_STAMP(6);
            // (each lane reads back only what it wrote itself: no barrier.)  A lane collects up to four hits and
            // then fetches them together, so that a wave waits for the caches once or twice, not once per hit.
            u32 h0 = 0, h1 = 0, h2 = 0, h3 = 0, nh = 0;
            auto fetch = [&]() __attribute__((always_inline)) {
                auto element = [&](u32 idx) __attribute__((always_inline)) {
                    return KeyOf<DT>::kBytes == 4 ? ((const Glb<u32>*)row_bytes)[idx]
                                                  : (u32)((const Glb<unsigned short>*)row_bytes)[idx];
                };
                const u32 r0 = nh > 0 ? element(h0) : 0u, r1 = nh > 1 ? element(h1) : 0u;
                const u32 r2 = nh > 2 ? element(h2) : 0u, r3 = nh > 3 ? element(h3) : 0u;
                const u32 base = nh ? atomicAdd(&sm.nlist, nh) : 0u;
                if (nh > 0 && base + 0 < LIST) sm.list[base + 0] = make_uint2(r0, h0);
                if (nh > 1 && base + 1 < LIST) sm.list[base + 1] = make_uint2(r1, h1);
                if (nh > 2 && base + 2 < LIST) sm.list[base + 2] = make_uint2(r2, h2);
                if (nh > 3 && base + 3 < LIST) sm.list[base + 3] = make_uint2(r3, h3);
                nh = 0;
            };
            for (u32 tl = 0; tl < c1 - c0; ++tl) {
                u32 m = masks[tl * (u32)B + tid];
                while (m != 0) {
                    const u32 bit = 31u - (u32)__builtin_clz(m);
                    m &= ~(1u << bit);
                    const u32 slot = 15u - bit;
                    // element of slot s of tile t for this lane: vector u = s / E of the tile, element j = s % E
                    constexpr u32 E = Source::E;
                    const u32 idx = ((c0 + tl) * (u32)Source::kTileVecs + (slot / E) * (u32)B + tid) * E + slot % E - src.lead;
                    if (nh == 4) fetch();
                    h3 = h2;
                    h2 = h1;
                    h1 = h0;
                    h0 = idx;
                    ++nh;
                }
            }
            fetch();
        }
        __syncthreads();
        if (sm.nlist > LIST) why = 5u;
        else if (sampled && sm.nlist < rs.k) why = 8u;  // the sample misled: the k-th key lies below the bound
    }
    RTOPK_STAMP(3);
    Selection sel{};
    const u32 nlist = sm.nlist;
    if (why == 0) {
        // ---- countBin on the list (exact key digits; all of them are >= b0), then selectBin
        for (u32 j = tid; j < (u32)nb; j += B) sm.wide[j] = 0;
        __syncthreads();
        for (u32 i = tid; i < nlist; i += B) {
            const uint2 e = sm.list[i];
            atomicAdd(&sm.wide[digit_of<DT, SRC_KEY>(ctx.pi, e.x, e.y, ctx.dirmask, ctx.idx_max, 0.0f)], 1u);
        }
        __syncthreads();
        sel = select_from_counts<B>(PlainCounts{sm.wide}, nb, rs.k, sm, st,
                                    [&]() __attribute__((always_inline)) {
                                        if (tid == 0) {
                                            sm.runW = 0;
                                            sm.runC = 0;
                                        }
                                    },
                                    nullptr);
        if (!sel.emit_all && sel.inside > kStreamRank) why = 6u;
    }
    if (why != 0) {
        if (tid == 0) {
            st->redo = 1u;
            st->redo_why = why;
        }
        return;
    }
    RTOPK_STAMP(4);
    // ---- selectCandidate + filter on the list (the histogram's memory now holds the ranking arrays)
    const int bw = sel.emit_all ? (int)sel.bin - 1 : (int)sel.bin;
    char* out_v = (char*)P.out_values + (size_t)row * (size_t)P.k * KeyOf<DT>::kBytes;
    long long* out_i = P.out_indices + (size_t)row * (size_t)P.k;
    for (u32 i = tid; i < nlist; i += B) {
        const uint2 e = sm.list[i];
        const u32 d = digit_of<DT, SRC_KEY>(ctx.pi, e.x, e.y, ctx.dirmask, ctx.idx_max, 0.0f);
        if ((int)d > bw) {
            const u32 pos = atomicAdd(&sm.runW, 1u);
            if (pos < rs.k) {
                store_value<DT>(out_v, pos, e.x);
                out_i[pos] = (long long)e.y;
            }
        } else if (d == sel.bin) {
            const u32 pos = atomicAdd(&sm.runC, 1u);
            if (pos < kStreamRank) sm.rank_list[pos] = e;
        }
    }
    const PassEntry e0 = pass_entry(P, st, 0, rs);
    if (tid == 0) write_pass_record(st, 0, ctx.pi, e0, sel, 4u, 0u);
    if (sel.emit_all) return;
    __syncthreads();
    // ---- the ranking step (see rank_finish): C candidates, up to two per lane
    const u32 C = sel.inside;
    uint2 mine[2];
    u64 my[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const u32 i = tid + (u32)r * B;
        mine[r] = make_uint2(0u, 0u);
        my[r] = 0;
        if (i < C) {
            mine[r] = sm.rank_list[i];
            my[r] = ((u64)(KeyOf<DT>::key(mine[r].x) ^ P.dirmask) << 32) | (u64)(P.idx_max - mine[r].y);
            sm.rank_ext[i] = my[r];
        } else if (i < C + 8u) {
            sm.rank_ext[i] = 0;  // padding: keys that beat nobody
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const u32 i = tid + (u32)r * B;
        if ((i & ~63u) < C) {  // whole waves: the loop's LDS reads are wave-uniform broadcasts
            u32 rank = 0;
            for (u32 j = 0; j < C; j += 8) {
                u64 q[8];
#pragma unroll
                for (int z = 0; z < 8; ++z) q[z] = sm.rank_ext[j + z];
#pragma unroll
                for (int z = 0; z < 8; ++z) rank += q[z] > my[r] ? 1u : 0u;
            }
            if (i < C && rank < sel.k_inside) {
                const u32 pos = sel.above + rank;
                if (pos < rs.k) {
                    store_value<DT>(out_v, pos, mine[r].x);
                    out_i[pos] = (long long)mine[r].y;
                }
            }
        }
    }
    if (tid == 0) {
        if (sm.runW != sel.above || sm.runC != C) st->error |= 4u;  // the list missed something: never expected
        st->pass_rec[1].bin = 0;
        st->pass_rec[1].k_after = 0;
        st->pass_rec[1].cand_after = 0;
        st->pass_rec[1].winners = sel.k_inside;
        st->pass_rec[1].out_before = sel.above;
        st->pass_rec[1].cand_before = C;
        st->pass_rec[1].window = SRC_RANK;
        st->pass_rec[1].where = 4u;
    }
    RTOPK_STAMP(5);
}

#include "rtopk_sort.inl"

static void mark(void* const* events, int i, hipStream_t st) {
    if (events && events[i]) (void)hipEventRecord((hipEvent_t)events[i], st);
}

template <int DT>
static rtopk_status launch_all(const Params& P, const Config& c, bool scaled, hipStream_t st, void* const* events) {
    const int batch = P.batch;
    mark(events, 0, st);
    constexpr int kScaledSrc = DT == RTOPK_F32 ? SRC_SCALED : SRC_KEY;  // 16-bit keys are never scaled
    if (DT != RTOPK_F32) scaled = false;
    if (c.path == 1) {
        mark(events, 1, st);
        mark(events, 2, st);
        mark(events, 3, st);
        // does every row, lead-in included, fit the registers of one workgroup?
        const long long cap = (long long)kRowBlock * kResidentVecs * (16 / KeyOf<DT>::kBytes);
        // (a row that does not start on a 16-byte boundary has up to E - 1 lead-in elements in its first vector)
        constexpr int kE = 16 / KeyOf<DT>::kBytes;
        const bool aligned = (uintptr_t)P.keys % 16 == 0 && (batch == 1 || P.n % kE == 0) && !P.row_offsets;
        const bool resident = P.n + (aligned ? 0 : kE - 1) <= cap;
        // small k, unscaled: the one-sweep kernel first; the two-sweep kernel then takes the rows it marked
        const bool one_sweep = c.one_sweep && !scaled;
        if (one_sweep && (u32)P.k <= kStreamSmallK)
            hipLaunchKernelGGL((k_row_stream<DT, kStreamList>), dim3(batch), dim3(kStreamBlock), 0, st, P);
        else if (one_sweep)
            hipLaunchKernelGGL((k_row_stream<DT, kStreamListMid>), dim3(batch), dim3(kStreamBlock), 0, st, P);
        if (resident && scaled)
            hipLaunchKernelGGL((k_row_resident<DT, kScaledSrc>), dim3(batch), dim3(kRowBlock), 0, st, P, false);
        else if (resident)
            hipLaunchKernelGGL((k_row_resident<DT, SRC_KEY>), dim3(batch), dim3(kRowBlock), 0, st, P, one_sweep);
        else if (scaled)
            hipLaunchKernelGGL((k_row<DT, kScaledSrc>), dim3(batch), dim3(kRowBlock), 0, st, P, false);
        else
            hipLaunchKernelGGL((k_row<DT, SRC_KEY>), dim3(batch), dim3(kRowBlock), 0, st, P, one_sweep);
        if (P.flags & RTOPK_FLAG_SORTED) launch_sort<DT>(P, st);
        mark(events, 4, st);
        return hipGetLastError() == hipSuccess ? RTOPK_OK : RTOPK_ERR_HIP;
    }
    const dim3 grid(c.G, batch), block(kGridBlock);
    hipLaunchKernelGGL((k_init<DT>), dim3(batch), dim3(256), 0, st, P);
    mark(events, 1, st);
    const bool nt = (P.flags & kInternalStream) != 0;
    if (c.prefilter) {
        // the sample's histogram, then the prefilter sweep (never scaled: make_config)
        // (fp32 rows swept by at most one workgroup per compute unit: the variant that stages more per wave)
        const bool big = DT == RTOPK_F32 && (long long)c.G * batch <= 256;
        if (nt) {
            hipLaunchKernelGGL((k_hist_keys<DT, SRC_KEY, true>), grid, block, 0, st, P);
            mark(events, 2, st);
            if constexpr (DT == RTOPK_F32) {
                if (big) hipLaunchKernelGGL((k_prefilter_keys<DT, SRC_KEY, true, true>), grid, block, 0, st, P);
            }
            if (!big) hipLaunchKernelGGL((k_prefilter_keys<DT, SRC_KEY, true, false>), grid, block, 0, st, P);
        } else {
            hipLaunchKernelGGL((k_hist_keys<DT, SRC_KEY, false>), grid, block, 0, st, P);
            mark(events, 2, st);
            if constexpr (DT == RTOPK_F32) {
                if (big) hipLaunchKernelGGL((k_prefilter_keys<DT, SRC_KEY, false, true>), grid, block, 0, st, P);
            }
            if (!big) hipLaunchKernelGGL((k_prefilter_keys<DT, SRC_KEY, false, false>), grid, block, 0, st, P);
        }
    } else if (scaled && nt) {
        hipLaunchKernelGGL((k_hist_keys<DT, kScaledSrc, true>), grid, block, 0, st, P);
        mark(events, 2, st);
        hipLaunchKernelGGL((k_classify_keys<DT, kScaledSrc, true>), grid, block, 0, st, P);
    } else if (scaled) {
        hipLaunchKernelGGL((k_hist_keys<DT, kScaledSrc, false>), grid, block, 0, st, P);
        mark(events, 2, st);
        hipLaunchKernelGGL((k_classify_keys<DT, kScaledSrc, false>), grid, block, 0, st, P);
    } else if (nt) {
        hipLaunchKernelGGL((k_hist_keys<DT, SRC_KEY, true>), grid, block, 0, st, P);
        mark(events, 2, st);
        hipLaunchKernelGGL((k_classify_keys<DT, SRC_KEY, true>), grid, block, 0, st, P);
    } else {
        hipLaunchKernelGGL((k_hist_keys<DT, SRC_KEY, false>), grid, block, 0, st, P);
        mark(events, 2, st);
        hipLaunchKernelGGL((k_classify_keys<DT, SRC_KEY, false>), grid, block, 0, st, P);
    }
    mark(events, 3, st);
    if (c.prefilter) {
        // pass 0: on what the prefilter kept, or over X again for rows whose sample misled it
        if (nt)
            hipLaunchKernelGGL((k_pass0_after_prefilter<DT, true>), grid, block, 0, st, P);
        else
            hipLaunchKernelGGL((k_pass0_after_prefilter<DT, false>), grid, block, 0, st, P);
    }
    for (int p = 1; p <= c.multi_last && p < c.npass; ++p) {
        if (nt)
            hipLaunchKernelGGL((k_classify_cand<DT, true>), grid, block, 0, st, P, p);
        else
            hipLaunchKernelGGL((k_classify_cand<DT, false>), grid, block, 0, st, P, p);
    }
    hipLaunchKernelGGL((k_finish<DT>), dim3(batch), dim3(kRowBlock), 0, st, P);
    if (P.flags & RTOPK_FLAG_SORTED) launch_sort<DT>(P, st);
    mark(events, 4, st);
    return hipGetLastError() == hipSuccess ? RTOPK_OK : RTOPK_ERR_HIP;
}

}  // namespace rtopk
