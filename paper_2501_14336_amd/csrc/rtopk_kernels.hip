// Radix top-k kernels for gfx950 and the C-ABI entry points declared in include/rtopk.h.
//
// One digit pass (paper Section 2.3.1) is two sweeps over the current candidates:
//
//   HIST      countBin + selectBin.  Every workgroup builds a local histogram of the pass's digit in LDS
//             (hierarchical atomics, Section 3.1.1), adds it to the row's global histogram, and stores the
//             suffix sums of its local histogram.  The last workgroup of the row to finish picks the bin b
//             that holds the k-th key and turns the stored suffix sums into exact write offsets for every
//             workgroup, so the second sweep needs no global atomics and its output order is fixed.
//   CLASSIFY  selectCandidate fused with the filter.  digit > b: the element is certainly in the top k and
//             goes straight to the output (value bits + int64 index).  digit == b: it stays a candidate and
//             is appended, with its index, to the next candidate array.  digit < b: dropped.
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

namespace rtopk {

constexpr int kGridBlock = 512;   // threads per workgroup, many-workgroups-per-row kernels
constexpr int kRowBlock = 1024;   // threads per workgroup, one-workgroup-per-row kernels
constexpr int kVecs = 4;          // 16-byte loads in flight per lane

template <int B>
struct Shared {
    u32 hist[kMaxBins];
    u32 wsum[B / 64];
    u32 wcnt[2][B / 64][2];
    u32 sel;
    u32 flag;
    u32 carry[2];
};

// ------------------------------------------------------------------------------------------------
// HIST phase
// ------------------------------------------------------------------------------------------------
template <class Source, int DT, int SRC, int B, bool SINGLE>
__device__ __forceinline__ void hist_phase(Source& src, const Params& P, int p, int row, u32 wg, u32 G,
                                           rtopk_row_trace* st, Shared<B>& sm, u32 where) {
    const PassInfo pi = P.pass[p];
    const int nb = 1 << pi.bits;
    const u32 tid = threadIdx.x;
    const float a_s = st->a_s;
    const u32 ntiles = src.ntiles();
    u32* ghist = P.ghist + (size_t)row * kMaxBins;
    u32* swg_row = P.swg + (size_t)row * P.G * kSwgStride;

    if (SINGLE || wg < ntiles) {
        for (int j = tid; j < nb; j += B) sm.hist[j] = 0;
        __syncthreads();
        for (u32 tile = wg; tile < ntiles; tile += G) {
            src.load(tile, tid);
#pragma unroll
            for (int s = 0; s < Source::kSlots; ++s) {
                u32 raw, idx;
                bool valid;
                src.get(s, raw, idx, valid);
                if (valid) hist_add(sm.hist, digit_of<DT, SRC>(pi, raw, idx, P.dirmask, P.idx_max, a_s));
            }
        }
        __syncthreads();
        if (!SINGLE) {
            for (int j = tid; j < nb; j += B) {
                u32 c = sm.hist[j];
                if (c) atomicAdd(&ghist[j], c);
            }
        }
        suffix_sums_in_place<B>(sm.hist, nb, sm.wsum);
        if (!SINGLE) {
            u32* mine = swg_row + (size_t)wg * kSwgStride;
            for (int j = tid; j < nb; j += B) mine[j] = sm.hist[j];
            if (tid == 0) mine[nb] = 0;
        }
    }
    if (!SINGLE) {
        // publish, then find out whether this workgroup is the row's last one
        __threadfence();
        __syncthreads();
        if (tid == 0) sm.flag = (atomicAdd(&st->ticket, 1u) == G - 1) ? 1u : 0u;
        __syncthreads();
        if (!sm.flag) return;
        __threadfence();
        for (int j = tid; j < nb; j += B) {
            sm.hist[j] = ghist[j];
            ghist[j] = 0;  // ready for the next pass
        }
        __syncthreads();
        suffix_sums_in_place<B>(sm.hist, nb, sm.wsum);
    }

    // selectBin on the row's suffix sums
    const u32 k_rem = st->k_rem;
    const u32 out_count = st->out_count;
    const u32 b = select_bin<B>(sm.hist, nb, k_rem, &sm.sel);
    const u32 g = (b + 1 < (u32)nb) ? sm.hist[b + 1] : 0u;  // candidates in better bins: certain winners
    const u32 cp = sm.hist[b] - g;                          // candidates inside the chosen bin
    const u32 kp = k_rem - g;                               // rank of the k-th key inside the bin
    const bool emit_all = (cp == kp);                       // the whole bin wins: selection is complete
    const bool bad = (k_rem == 0) || (k_rem > sm.hist[0]);  // inconsistent state: never expected

    if (!SINGLE) {
        // exact write offsets for every workgroup of the CLASSIFY sweep
        const u32 active = ntiles < G ? ntiles : G;
        u32* bases = P.bases + (size_t)row * P.G * 2;
        if (tid == 0) { sm.carry[0] = 0; sm.carry[1] = 0; }
        __syncthreads();
        for (u32 w0 = 0; w0 < active; w0 += B) {
            const u32 w = w0 + tid;
            u32 W = 0, C = 0;
            if (w < active) {
                const u32* rec = swg_row + (size_t)w * kSwgStride;
                const u32 sb = rec[b], sb1 = rec[b + 1];
                C = sb - sb1;
                W = sb1;
                if (emit_all) { W += C; C = 0; }
            }
            const u32 cw = sm.carry[0], cc = sm.carry[1];
            const u32 iw = block_inclusive_scan<B>(W, sm.wsum);
            const u32 ic = block_inclusive_scan<B>(C, sm.wsum);
            if (w < active) {
                bases[2 * w] = out_count + cw + iw - W;
                bases[2 * w + 1] = cc + ic - C;
            }
            __syncthreads();
            if (tid == B - 1) { sm.carry[0] = cw + iw; sm.carry[1] = cc + ic; }
            __syncthreads();
        }
    }
    if (tid == 0) {
        st->bin = b;
        st->emit_all = emit_all ? 1u : 0u;
        st->win_total = g + (emit_all ? cp : 0u);
        st->next_count = emit_all ? 0u : cp;
        st->k_rem = kp;
        st->ticket = 0;
        if (bad) st->error |= 1u;
        if (p < kMaxPasses) {
            st->pass_rec[p].bin = b;
            st->pass_rec[p].k_after = emit_all ? 0u : kp;
            st->pass_rec[p].cand_after = emit_all ? 0u : cp;
            st->pass_rec[p].winners = g + (emit_all ? cp : 0u);
            st->pass_rec[p].source = pi.src;
            st->pass_rec[p].shift = pi.shift;
            st->pass_rec[p].bits = pi.bits;
            st->pass_rec[p].where = where;
        }
        st->passes_run = (u32)p + 1u;
    }
}

// ------------------------------------------------------------------------------------------------
// CLASSIFY phase
// ------------------------------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void store_value(void* out_row, u32 pos, u32 raw) {
    if (DT == RTOPK_F32)
        ((u32*)out_row)[pos] = raw;
    else
        ((uint16_t*)out_row)[pos] = (uint16_t)raw;
}

template <class Source, int DT, int SRC, int B, bool SINGLE>
__device__ __forceinline__ void classify_phase(Source& src, const Params& P, int p, int row, u32 wg, u32 G,
                                               rtopk_row_trace* st, Shared<B>& sm) {
    const PassInfo pi = P.pass[p];
    const u32 tid = threadIdx.x;
    const u32 lane = lane_id();
    const u32 wave = tid >> 6;
    constexpr int NW = B / 64;
    const float a_s = st->a_s;
    const u32 b = st->bin;
    const bool emit_all = st->emit_all != 0;
    const u32 ntiles = src.ntiles();
    const u32 kk = (u32)P.k;
    const u32 ncap = (u32)P.n;

    void* out_v = (char*)P.out_values + (size_t)row * (size_t)P.k * KeyOf<DT>::kBytes;
    long long* out_i = P.out_indices + (size_t)row * (size_t)P.k;
    uint2* cand_out = P.cand[p & 1] + (size_t)row * (size_t)P.n;

    u32 runW, runC;
    if (SINGLE) {
        runW = st->out_count;
        runC = 0;
    } else {
        const u32* bases = P.bases + (size_t)row * P.G * 2;
        runW = (wg < ntiles) ? bases[2 * wg] : 0u;
        runC = (wg < ntiles) ? bases[2 * wg + 1] : 0u;
    }
    u32 parity = 0;
    for (u32 tile = wg; tile < ntiles; tile += G) {
        src.load(tile, tid);
        u32 winbits = 0, candbits = 0, totW = 0, totC = 0;
#pragma unroll
        for (int s = 0; s < Source::kSlots; ++s) {
            u32 raw, idx;
            bool valid;
            src.get(s, raw, idx, valid);
            const u32 dg = digit_of<DT, SRC>(pi, raw, idx, P.dirmask, P.idx_max, a_s);
            const bool eq = valid && dg == b;
            const bool w = valid && (dg > b || (emit_all && eq));
            const bool c = eq && !emit_all;
            winbits |= (w ? 1u : 0u) << s;
            candbits |= (c ? 1u : 0u) << s;
            totW += (u32)__popcll(ballot64(w));
            totC += (u32)__popcll(ballot64(c));
        }
        if (lane == 0) {
            sm.wcnt[parity][wave][0] = totW;
            sm.wcnt[parity][wave][1] = totC;
        }
        __syncthreads();
        u32 preW = 0, preC = 0, allW = 0, allC = 0;
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) {
            const u32 cw = sm.wcnt[parity][w2][0], cc = sm.wcnt[parity][w2][1];
            if ((u32)w2 < wave) { preW += cw; preC += cc; }
            allW += cw;
            allC += cc;
        }
        u32 posW = runW + preW, posC = runC + preC;
        if (allW | allC) {
#pragma unroll
            for (int s = 0; s < Source::kSlots; ++s) {
                const bool w = (winbits >> s) & 1u;
                const bool c = (candbits >> s) & 1u;
                const u64 mw = ballot64(w);
                const u64 mc = ballot64(c);
                if (mw | mc) {
                    u32 raw, idx;
                    bool valid;
                    src.get(s, raw, idx, valid);
                    if (w) {
                        const u32 pos = posW + mbcnt64(mw);
                        if (pos < kk) {
                            store_value<DT>(out_v, pos, raw);
                            out_i[pos] = (long long)idx;
                        }
                    }
                    if (c) {
                        const u32 pos = posC + mbcnt64(mc);
                        if (pos < ncap) cand_out[pos] = make_uint2(raw, idx);
                    }
                    posW += (u32)__popcll(mw);
                    posC += (u32)__popcll(mc);
                }
            }
        }
        runW += allW;
        runC += allC;
        parity ^= 1u;
    }

    // the row's last workgroup moves the loop state on (Algorithm 1: next digit)
    bool last = true;
    if (!SINGLE) {
        __threadfence();
        __syncthreads();
        if (tid == 0) sm.flag = (atomicAdd(&st->ticket, 1u) == G - 1) ? 1u : 0u;
        __syncthreads();
        last = sm.flag != 0;
    } else {
        __syncthreads();
    }
    if (last && tid == 0) {
        const u32 next = st->next_count;
        st->out_count += st->win_total;
        st->cand_count = next;
        st->pass = (u32)p + 1u;
        st->ticket = 0;
        if (emit_all || next == 0) {
            st->done = 1;
        } else if (p + 1 >= P.npass) {
            st->done = 1;
            st->error |= 2u;  // digits exhausted with candidates left: impossible for unique extended keys
        }
    }
    if (SINGLE) __syncthreads();
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

template <int DT>
__device__ __forceinline__ void init_row(const Params& P, int row, rtopk_row_trace* st) {
    // called by one thread
    u32* w = (u32*)st;
    for (int i = 0; i < (int)(sizeof(rtopk_row_trace) / 4); ++i) w[i] = 0;
    st->k_rem = (u32)P.k;
    st->cand_count = (u32)P.n;
    float a_s = 0.0f;
    if (DT == RTOPK_F32 && (P.flags & RTOPK_FLAG_SCALING)) {
        const u64 j = mix64(P.seed + 0x9E3779B97F4A7C15ull * (u64)(row + 1)) % (u64)P.n;
        const u32 bits = ((const u32*)P.keys)[(size_t)row * (size_t)P.n + j];
        if ((bits & 0x7f800000u) != 0x7f800000u) a_s = __uint_as_float(bits);  // finite only
    }
    st->a_s = a_s;
}

template <int DT>
__global__ void __launch_bounds__(256) k_init(Params P) {
    const int row = blockIdx.x;
    u32* ghist = P.ghist + (size_t)row * kMaxBins;
    for (int j = threadIdx.x; j < kMaxBins; j += 256) ghist[j] = 0;
    if (threadIdx.x == 0) init_row<DT>(P, row, row_state(P, row));
}

// ------------------------------------------------------------------------------------------------
// many workgroups per row: one launch per phase per pass, covering every row (task rescheduling,
// Section 3.2.1: pass i of all tasks runs together; grid = workgroups-per-row x rows)
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ bool row_skips_pass(const Params& P, const rtopk_row_trace* st, int p) {
    if (st->done || st->pass != (u32)p) return true;
    return p > 0 && st->cand_count <= P.small;  // few candidates left: the finish kernel takes over
}

template <int DT, int SRC>
__global__ void __launch_bounds__(kGridBlock) k_hist_keys(Params P) {
    __shared__ Shared<kGridBlock> sm;
    const int row = blockIdx.y;
    rtopk_row_trace* st = row_state(P, row);
    if (row_skips_pass(P, st, 0)) return;
    KeySource<DT, kGridBlock, kVecs> src;
    src.init(P.keys, P.n, row);
    hist_phase<decltype(src), DT, SRC, kGridBlock, false>(src, P, 0, row, blockIdx.x, gridDim.x, st, sm, 1u);
}

template <int DT, int SRC>
__global__ void __launch_bounds__(kGridBlock) k_classify_keys(Params P) {
    __shared__ Shared<kGridBlock> sm;
    const int row = blockIdx.y;
    rtopk_row_trace* st = row_state(P, row);
    if (row_skips_pass(P, st, 0)) return;
    KeySource<DT, kGridBlock, kVecs> src;
    src.init(P.keys, P.n, row);
    classify_phase<decltype(src), DT, SRC, kGridBlock, false>(src, P, 0, row, blockIdx.x, gridDim.x, st, sm);
}

template <int DT>
__global__ void __launch_bounds__(kGridBlock) k_hist_cand(Params P, int p) {
    __shared__ Shared<kGridBlock> sm;
    const int row = blockIdx.y;
    rtopk_row_trace* st = row_state(P, row);
    if (row_skips_pass(P, st, p)) return;
    CandSource<kGridBlock, kVecs> src;
    src.init(P.cand[(p - 1) & 1] + (size_t)row * (size_t)P.n, st->cand_count);
    hist_phase<decltype(src), DT, SRC_RUNTIME, kGridBlock, false>(src, P, p, row, blockIdx.x, gridDim.x, st, sm, 1u);
}

template <int DT>
__global__ void __launch_bounds__(kGridBlock) k_classify_cand(Params P, int p) {
    __shared__ Shared<kGridBlock> sm;
    const int row = blockIdx.y;
    rtopk_row_trace* st = row_state(P, row);
    if (row_skips_pass(P, st, p)) return;
    CandSource<kGridBlock, kVecs> src;
    src.init(P.cand[(p - 1) & 1] + (size_t)row * (size_t)P.n, st->cand_count);
    classify_phase<decltype(src), DT, SRC_RUNTIME, kGridBlock, false>(src, P, p, row, blockIdx.x, gridDim.x, st, sm);
}

// ------------------------------------------------------------------------------------------------
// one workgroup per row
// ------------------------------------------------------------------------------------------------

// Remaining passes of one row on its candidate arrays, by a single workgroup.
template <int DT>
__device__ __forceinline__ void finish_row(const Params& P, int row, rtopk_row_trace* st, Shared<kRowBlock>& sm,
                                           u32 where) {
    for (;;) {
        // state is rewritten by thread 0 at the end of each phase, behind a barrier
        if (st->done) break;
        const int p = (int)st->pass;
        if (p >= P.npass) break;
        CandSource<kRowBlock, kVecs> src;
        src.init(P.cand[(p - 1) & 1] + (size_t)row * (size_t)P.n, st->cand_count);
        hist_phase<decltype(src), DT, SRC_RUNTIME, kRowBlock, true>(src, P, p, row, 0u, 1u, st, sm, where);
        __syncthreads();
        classify_phase<decltype(src), DT, SRC_RUNTIME, kRowBlock, true>(src, P, p, row, 0u, 1u, st, sm);
    }
}

template <int DT>
__global__ void __launch_bounds__(kRowBlock) k_finish(Params P) {
    __shared__ Shared<kRowBlock> sm;
    const int row = blockIdx.x;
    rtopk_row_trace* st = row_state(P, row);
    finish_row<DT>(P, row, st, sm, 2u);
}

// Whole selection of one row in one kernel (many short rows: no global atomics, no extra launches).
template <int DT, int SRC>
__global__ void __launch_bounds__(kRowBlock) k_row(Params P) {
    __shared__ Shared<kRowBlock> sm;
    const int row = blockIdx.x;
    rtopk_row_trace* st = row_state(P, row);
    if (threadIdx.x == 0) init_row<DT>(P, row, st);
    __syncthreads();
    {
        KeySource<DT, kRowBlock, kVecs> src;
        src.init(P.keys, P.n, row);
        hist_phase<decltype(src), DT, SRC, kRowBlock, true>(src, P, 0, row, 0u, 1u, st, sm, 3u);
        __syncthreads();
        classify_phase<decltype(src), DT, SRC, kRowBlock, true>(src, P, 0, row, 0u, 1u, st, sm);
    }
    finish_row<DT>(P, row, st, sm, 3u);
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct Layout {
    size_t state_off, ghist_off, bases_off, swg_off, cand0_off, cand1_off, total;
};

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Config {
    int d, path, G;
    u32 small;
    int npass;
    u32 idx_max, dirmask;
    PassInfo pass[kMaxPasses];
};

static int elem_bytes(rtopk_dtype dt) { return dt == RTOPK_F32 ? 4 : 2; }

static rtopk_status make_config(int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest, uint32_t flags,
                                const rtopk_tuning* tn, Config* c) {
    if (batch < 1 || batch > 0x7fffffff || n < 1 || n > RTOPK_MAX_N || k < 1 || k > n) return RTOPK_ERR_INVALID_ARG;
    if (dt != RTOPK_F32 && dt != RTOPK_F16 && dt != RTOPK_BF16) return RTOPK_ERR_INVALID_ARG;
    if (flags & ~(uint32_t)RTOPK_FLAG_SCALING) return RTOPK_ERR_INVALID_ARG;
    int d = dt == RTOPK_F32 ? 12 : 11;
    int path = 0, G = 0;
    u32 small = 32768;
    if (tn) {
        if (tn->digit_bits) {
            if (tn->digit_bits < 8 || tn->digit_bits > 12) return RTOPK_ERR_INVALID_ARG;
            d = tn->digit_bits;
        }
        if (tn->path < 0 || tn->path > 2 || tn->wgs_per_row < 0 || tn->small_threshold < 0) return RTOPK_ERR_INVALID_ARG;
        path = tn->path;
        G = tn->wgs_per_row;
        if (tn->small_threshold) small = (u32)tn->small_threshold;
    }
    if (path == 0) {
        // short rows, or enough rows to occupy every compute unit: one workgroup per row
        path = (n <= (1 << 18) || (batch >= 256 && n <= (1 << 20))) ? 1 : 2;
        if (batch > 65535) path = 1;
    }
    if (path == 2 && batch > 65535) return RTOPK_ERR_INVALID_ARG;  // rows are the grid's y dimension
    const int eb = elem_bytes(dt);
    const int64_t tile_elems = (int64_t)kGridBlock * kVecs * (16 / eb);
    const int64_t ntiles = (n + 16 / eb - 1 + tile_elems) / tile_elems;  // one spare for the lead-in
    if (path == 2) {
        if (G == 0) {
            int64_t want = 512 / batch;  // about two workgroups per compute unit in total
            if (want < 1) want = 1;
            G = (int)want;
        }
        if (G > ntiles) G = (int)ntiles;
        if (G > 4096) G = 4096;
        if (G < 1) G = 1;
    } else {
        G = 1;
    }
    c->d = d;
    c->path = path;
    c->G = G;
    c->small = small;
    c->dirmask = largest ? 0u : (dt == RTOPK_F32 ? 0xffffffffu : 0xffff0000u);

    int np = 0;
    const int kw = dt == RTOPK_F32 ? 32 : 16;
    if ((flags & RTOPK_FLAG_SCALING) && dt == RTOPK_F32) {
        for (int hi = 32; hi > 0;) {
            int bits = d < hi ? d : hi;
            c->pass[np++] = PassInfo{SRC_SCALED, (u32)(hi - bits), (u32)bits};
            hi -= bits;
        }
    }
    for (int hi = 32; hi > 32 - kw;) {
        int bits = d < hi - (32 - kw) ? d : hi - (32 - kw);
        c->pass[np++] = PassInfo{SRC_KEY, (u32)(hi - bits), (u32)bits};
        hi -= bits;
    }
    int ib = 0;
    while (((int64_t)1 << ib) < n) ++ib;
    c->idx_max = ib == 0 ? 0u : (u32)(((u64)1 << ib) - 1);
    for (int hi = ib; hi > 0;) {
        int bits = d < hi ? d : hi;
        c->pass[np++] = PassInfo{SRC_IDX, (u32)(hi - bits), (u32)bits};
        hi -= bits;
    }
    if (np > kMaxPasses) return RTOPK_ERR_INVALID_ARG;
    c->npass = np;
    return RTOPK_OK;
}

static Layout make_layout(int64_t batch, int64_t n, const Config& c) {
    Layout L;
    size_t off = 0;
    L.state_off = off;
    off = align_up(off + (size_t)batch * RTOPK_TRACE_STRIDE, 256);
    L.ghist_off = off;
    off = align_up(off + (size_t)batch * kMaxBins * 4, 256);
    L.bases_off = off;
    off = align_up(off + (size_t)batch * c.G * 2 * 4, 256);
    L.swg_off = off;
    off = align_up(off + (size_t)batch * c.G * kSwgStride * 4, 256);
    L.cand0_off = off;
    off = align_up(off + (size_t)batch * (size_t)n * 8, 256);
    L.cand1_off = off;
    off = align_up(off + (size_t)batch * (size_t)n * 8, 256);
    L.total = off + 256;  // the last 16-byte load of an odd-length candidate array may touch 8 bytes past it
    return L;
}

template <int DT>
static rtopk_status launch_all(const Params& P, const Config& c, bool scaled, hipStream_t st) {
    const int batch = P.batch;
    if (c.path == 1) {
        if (scaled)
            hipLaunchKernelGGL((k_row<DT, SRC_SCALED>), dim3(batch), dim3(kRowBlock), 0, st, P);
        else
            hipLaunchKernelGGL((k_row<DT, SRC_KEY>), dim3(batch), dim3(kRowBlock), 0, st, P);
        return hipGetLastError() == hipSuccess ? RTOPK_OK : RTOPK_ERR_HIP;
    }
    const dim3 grid(c.G, batch), block(kGridBlock);
    hipLaunchKernelGGL((k_init<DT>), dim3(batch), dim3(256), 0, st, P);
    if (scaled) {
        hipLaunchKernelGGL((k_hist_keys<DT, SRC_SCALED>), grid, block, 0, st, P);
        hipLaunchKernelGGL((k_classify_keys<DT, SRC_SCALED>), grid, block, 0, st, P);
    } else {
        hipLaunchKernelGGL((k_hist_keys<DT, SRC_KEY>), grid, block, 0, st, P);
        hipLaunchKernelGGL((k_classify_keys<DT, SRC_KEY>), grid, block, 0, st, P);
    }
    for (int p = 1; p < c.npass; ++p) {
        hipLaunchKernelGGL((k_hist_cand<DT>), grid, block, 0, st, P, p);
        hipLaunchKernelGGL((k_classify_cand<DT>), grid, block, 0, st, P, p);
    }
    hipLaunchKernelGGL((k_finish<DT>), dim3(batch), dim3(kRowBlock), 0, st, P);
    return hipGetLastError() == hipSuccess ? RTOPK_OK : RTOPK_ERR_HIP;
}

}  // namespace rtopk

using namespace rtopk;

extern "C" {

const char* rtopk_status_string(rtopk_status s) {
    switch (s) {
        case RTOPK_OK: return "ok";
        case RTOPK_ERR_INVALID_ARG: return "invalid argument";
        case RTOPK_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case RTOPK_ERR_UNSUPPORTED: return "unsupported (misaligned buffer)";
        case RTOPK_ERR_HIP: return "HIP runtime rejected a launch";
    }
    return "unknown status";
}

const char* rtopk_version(void) { return "0.1"; }

rtopk_status rtopk_workspace_bytes(int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, uint32_t flags,
                                   const rtopk_tuning* tuning, size_t* bytes_out) {
    if (!bytes_out) return RTOPK_ERR_INVALID_ARG;
    Config c;
    rtopk_status s = make_config(batch, n, k, dt, 1, flags, tuning, &c);
    if (s != RTOPK_OK) return s;
    *bytes_out = make_layout(batch, n, c).total;
    return RTOPK_OK;
}

rtopk_status rtopk_select_ex(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                             uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices, void* workspace,
                             size_t workspace_bytes, void* hip_stream, const rtopk_tuning* tuning) {
    if (!keys || !out_values || !out_indices || !workspace) return RTOPK_ERR_INVALID_ARG;
    Config c;
    rtopk_status s = make_config(batch, n, k, dt, largest, flags, tuning, &c);
    if (s != RTOPK_OK) return s;
    const int eb = elem_bytes(dt);
    if (((uintptr_t)keys % eb) || ((uintptr_t)out_values % eb) || ((uintptr_t)out_indices % 8) ||
        ((uintptr_t)workspace % 256))
        return RTOPK_ERR_UNSUPPORTED;
    const Layout L = make_layout(batch, n, c);
    if (workspace_bytes < L.total) return RTOPK_ERR_WORKSPACE_TOO_SMALL;

    Params P;
    memset(&P, 0, sizeof(P));
    char* ws = (char*)workspace;
    P.keys = keys;
    P.out_values = out_values;
    P.out_indices = (long long*)out_indices;
    P.state = (rtopk_row_trace*)(ws + L.state_off);
    P.ghist = (u32*)(ws + L.ghist_off);
    P.bases = (u32*)(ws + L.bases_off);
    P.swg = (u32*)(ws + L.swg_off);
    P.cand[0] = (uint2*)(ws + L.cand0_off);
    P.cand[1] = (uint2*)(ws + L.cand1_off);
    P.n = n;
    P.k = k;
    P.batch = (int)batch;
    P.G = c.G;
    P.dirmask = c.dirmask;
    P.idx_max = c.idx_max;
    P.small = c.small;
    P.npass = c.npass;
    P.flags = flags;
    P.seed = seed;
    for (int i = 0; i < c.npass; ++i) P.pass[i] = c.pass[i];

    hipStream_t st = (hipStream_t)hip_stream;
    const bool scaled = (flags & RTOPK_FLAG_SCALING) && dt == RTOPK_F32;
    switch (dt) {
        case RTOPK_F32: return launch_all<RTOPK_F32>(P, c, scaled, st);
        case RTOPK_F16: return launch_all<RTOPK_F16>(P, c, false, st);
        case RTOPK_BF16: return launch_all<RTOPK_BF16>(P, c, false, st);
    }
    return RTOPK_ERR_INVALID_ARG;
}

rtopk_status rtopk_select(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                          uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    return rtopk_select_ex(keys, batch, n, k, dt, largest, flags, seed, out_values, out_indices, workspace,
                           workspace_bytes, hip_stream, nullptr);
}

}  // extern "C"
