// C-ABI entry points declared in include/rtopk.h: argument validation, the digit plan, workspace layout,
// and the hand-off to the per-type kernel launchers.  Host code, plus the one device object the library owns:
// the built-in scratch buffer of rtopk_select_static.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "rtopk.h"
#include "rtopk_device.h"
#include "rtopk_host.h"

namespace rtopk {

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct Layout {
    size_t state_off, dbg_off, ghist_off, seg_off, swg_off, sort_hist_off, sort_state_off, cand0_off, cand1_off, cand_stride, total;
};

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int elem_bytes(rtopk_dtype dt) { return dt == RTOPK_F32 ? 4 : 2; }

static rtopk_status make_config(int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest, uint32_t flags,
                                const rtopk_tuning* tn, Config* c) {
    if (batch < 1 || batch > 0x7fffffff || n < 1 || n > RTOPK_MAX_N || k < 1 || k > n) return RTOPK_ERR_INVALID_ARG;
    if (dt != RTOPK_F32 && dt != RTOPK_F16 && dt != RTOPK_BF16) return RTOPK_ERR_INVALID_ARG;
    if (flags & ~(uint32_t)(RTOPK_FLAG_SCALING | RTOPK_FLAG_DEBUG_COUNTERS | RTOPK_FLAG_SORTED)) return RTOPK_ERR_INVALID_ARG;
    int d = dt == RTOPK_F32 ? 12 : 11;
    int path = 0, G = 0;
    u32 small = 65536;
    if (tn) {
        if (tn->digit_bits) {
            if (tn->digit_bits < 8 || tn->digit_bits > 12) return RTOPK_ERR_INVALID_ARG;
            d = tn->digit_bits;
        }
        if (tn->path < 0 || tn->path > 3 || tn->wgs_per_row < 0 || tn->small_threshold < 0) return RTOPK_ERR_INVALID_ARG;
        path = tn->path;
        G = tn->wgs_per_row;
        if (tn->small_threshold) small = (u32)tn->small_threshold;
    }
    if (path == 0) {
        // short rows, or enough rows to occupy the compute units: one workgroup per row.  (fp32, k = 16 or 1024, row
        // kernel / grid kernels in us.  Uniform [0,1) keys, whose best bins are full: 1 x 2^15 32 / 36, 1 x 2^16
        // 45 / 36, 16 x 2^16 47 / 39, 64 x 2^16 46 / 45, 128 x 2^16 49 / 55, 1 x 2^18 86 / 50, 16 x 2^18 87 / 60,
        // 64 x 2^18 88 / 83, 128 x 2^18 90 / 107, 256 x 2^18 118 / 152.  Normal keys: 64 x 2^16 25 / 35,
        // 128 x 2^17 40 / 67, 256 x 2^18 100 / 130.)
        path = (n <= (1 << 16) || (batch >= 96 && n <= (1 << 18)) || (batch >= 256 && n <= (1 << 20))) ? 1 : 2;
        // ... unless a large part of every row is wanted: a workgroup that owns a row goes through its phases one
        // after the other (1024 rows of 2^17 bf16 keys, k = 8192: 51 + 36 us per row, 360 us in all), while the
        // grid kernels, one workgroup per row here, keep several rows per compute unit in flight (277 us; k = 2048:
        // 281 against 230, k = 1024: 217 against 224)
        if (path == 1 && batch >= 256 && batch <= 65535 && n >= 65536 && k * 128 >= n) path = 2;
        if (batch > 65535) path = 1;
    }
    // The one-sweep kernel sets aside a few hundred elements of a row (its bound comes from the row's first
    // eighth, more for larger k) and holds 2048.  Rows it cannot finish go to the two-sweep kernel, so the choice
    // never changes the result.
    bool one_sweep = path == 3;
    if (path == 3) path = 1;
    // (k up to 512 on rows of 64K keys up: the bound then comes from a sample of the row and is checked afterwards --
    // 1024 rows of 2^17 bf16 keys, k = 1024: see the measurements beside the kernel)
    // (against the two-sweep row kernel, fp32, k = 16, in us: normal keys 128 x 2^17 32 / 40, 256 x 2^17 41 / 57,
    // 256 x 2^18 60 / 100, 512 x 2^17 63 / 102; uniform [0,1) keys, where the first part shows a full bin at the top and
    // most rows are handed over: 256 x 2^16 61 / 55, 256 x 2^18 123 / 118.  With fewer rows than a quarter of the
    // compute units there is nothing to overlap: 16 x 2^16 uniform keys 47 / 41, 64 x 2^16 normal keys 24 / 25.)
    else if (path == 1 && (!tn || tn->path == 0) && (k <= 256 || (k <= 512 && n >= 65536)) && n >= 16384 && batch >= 64)
        one_sweep = true;
    if (path == 2 && batch > 65535) return RTOPK_ERR_INVALID_ARG;  // rows are the grid's y dimension
    // 16-bit keys on long rows: a 12-bit first digit (4 bits left for the second) instead of 11 + 5 -- the first
    // sweep then keeps a bin of half the width (bf16 logits, 64 x 2^22, k = 50: 200 -> 167 us; 2^29 uniform bf16
    // keys: 1052 -> 788 us); the one-workgroup-per-row kernels stay at 11, where twice the histogram copies fit
    // (not where one workgroup has a whole row of such a batch and k is small: 1024 rows of 2^17 bf16 keys, 11 against
    // 12 bits: k = 1024 203 against 222 us, k = 2048 222 against 230, k = 4096 290 both, k = 8192 283 against 276)
    if (path == 2 && dt != RTOPK_F32 && !(tn && tn->digit_bits) && !(batch >= 256 && k * 32 <= n)) d = 12;
    const int eb = elem_bytes(dt);
    const int64_t tile_elems = (int64_t)kHostGridBlock * kHostElemsPerLane;  // 16 elements per lane for every type
    const int64_t ntiles = (n + 16 / eb - 1 + tile_elems) / tile_elems;  // one spare for the lead-in
    // Prefilter (many workgroups per row, unscaled): count a sample of the row (every 31st tile: a prime stride,
    // so that no power-of-two period in the data lines up with the sample), take from it a bin that very
    // probably lies at or below the k-th key's, and sweep X ONCE, counting every element's digit and keeping the
    // elements from that bin upwards; pass 0 then runs on what was kept.  If the full counts show the bin was
    // too high, pass 0 is the ordinary second sweep over X instead.
    // It pays while k is well below n (what is kept is written out and read again): 2^28 uniform fp32 keys,
    // k = 2^24 (a sixteenth: 9 % of the row kept) 395 us against 526 with two sweeps; from k = 2^25 on the sample
    // shows more than an eighth of the row in the bins to keep and the sweep would decline anyway.
    c->prefilter = false;
    c->pre_stride = 0;
    if (tn && (tn->prefilter < -1 || tn->prefilter > 1)) return RTOPK_ERR_INVALID_ARG;
    const int pre_knob = tn ? tn->prefilter : 0;
    const bool scaling_on = (flags & RTOPK_FLAG_SCALING) && dt == RTOPK_F32;
    // (inputs of 64 to 256 MB: two sweeps from the caches cost little more than one, and the call is bound by its
    // launches; for fp32 keys the prefilter still wins where pass 0 would otherwise write many candidates -- 2^24
    // normal keys, k = 2^16: 62 against 82 us, k = 2^12: 61 against 65, k = 16: 61 against 56 -- and for batches,
    // whatever k: 16 rows of 2^20, k = 16: 79 against 106; 64 rows of 2^20: 132 against 189; 2^26 fp16 keys that
    // all fall into one bin lost 100 us to the counting sweep that then stands before the two others)
    const int64_t in_bytes = batch * n * eb;
    // (up to a sixteenth of the row for fp32 inputs of 256 MB up; a 32nd otherwise: 2^24 fp32 keys, k = 2^20: 93 against
    // 83 us; 1024 rows of 2^17 bf16 keys, k = 2^13: the sample declines, 298 against 273 us)
    const bool big_f32 = dt == RTOPK_F32 && in_bytes >= ((int64_t)256 << 20);
    if (path == 2 && !scaling_on &&
        (pre_knob == 1 || (pre_knob == 0 && k <= n / (big_f32 ? 16 : 32) &&
                           (in_bytes >= ((int64_t)256 << 20) ||
                            (dt == RTOPK_F32 && in_bytes >= ((int64_t)64 << 20) && (batch > 1 || k * 4096 >= n)))))) {
        c->prefilter = true;
        c->pre_stride = 31;
    }
    if (path == 2) {
        if (G == 0) {
            // about two workgroups per compute unit in total; one for the fp32 sweep that counts and keeps, which
            // then stages three times as much per wave (measured on n = 2^28: k = 2^20 239 us with 256 workgroups,
            // 280 with 512, 298 with 384; k = 2^22 321 against 332; k = 2^24 389 against 395; two sweeps with
            // k = 2^24: 603 against 526)
            // (16-bit keys: whole bins of an 11-bit digit are kept, more of the row; 2^29 fp16 keys, k = 2^20:
            // 260 us with 512, 346 with 256; bf16 with k = 50 or 2^10: no difference)
            // (and one for inputs that the caches hold: 2^24 fp32 keys, two sweeps: 53-61 us against 58-65; not
            // 128 MB: 2^26 fp16 keys of few distinct values, 355-385 us against 270-303)
            const bool cached = in_bytes <= ((int64_t)64 << 20);
            int64_t want = ((c->prefilter && dt == RTOPK_F32) || cached ? 256 : 512) / batch;
            if (want < 1) want = 1;
            G = (int)want;
        }
        if (G > ntiles) G = (int)ntiles;
        if (G > 4096) G = 4096;
        if (G < 1) G = 1;
    } else {
        G = 1;
    }
    // sorted output of rows too long for one workgroup's LDS: a radix sort on the grid, chunks of at least 8192 keys
    c->Gs = 0;
    if ((flags & RTOPK_FLAG_SORTED) && k > kHostSortSmall) {
        int64_t want = 512 / batch, by_k = (k + 8191) / 8192;
        if (want < 1) want = 1;
        if (want > by_k) want = by_k;
        c->Gs = (int)want;
        if (batch > 65535) return RTOPK_ERR_INVALID_ARG;  // rows are the grid's y dimension there
    }
    c->d = d;
    c->path = path;
    c->one_sweep = one_sweep;
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
    // How far can a row keep more than `small` candidates?  Key digits may keep all n (equal keys); after an
    // index digit at most 2^shift candidates share the bin, the indices being distinct.  Later passes are
    // certain to fit the single-workgroup finish and get no grid launch.
    c->multi_last = np - 1;
    for (int p = 0; p < np; ++p) {
        const bool idx = c->pass[p].src == SRC_IDX;
        const uint64_t bound = idx && c->pass[p].shift < 63 && ((uint64_t)1 << c->pass[p].shift) < (uint64_t)n
                                   ? (uint64_t)1 << c->pass[p].shift : (uint64_t)n;
        if (bound <= small) {
            c->multi_last = p;
            break;
        }
    }
    return RTOPK_OK;
}

static Layout make_layout(int64_t batch, int64_t n, const Config& c) {
    Layout L;
    size_t off = 0;
    L.state_off = off;
    off = align_up(off + (size_t)batch * RTOPK_TRACE_STRIDE, 256);
    L.dbg_off = off;
    off = align_up(off + (size_t)batch * c.G * 128, 256);
    // global histograms, per-workgroup records and segments exist only when several workgroups share a row
    const size_t shared_rows = c.path == 2 ? (size_t)batch : 0;
    L.ghist_off = off;
    off = align_up(off + (size_t)kHostHistBuffers * shared_rows * kMaxBins * 4, 256);
    L.seg_off = off;
    off = align_up(off + (size_t)2 * shared_rows * c.G * 2 * 4, 256);
    L.swg_off = off;
    off = align_up(off + (size_t)kHostSwgBuffers * shared_rows * c.G * kSwgStride * 4, 256);
    L.sort_hist_off = off;
    off = align_up(off + (size_t)batch * 256 * c.Gs * 4, 256);
    L.sort_state_off = off;
    off = align_up(off + (c.Gs ? (size_t)batch * 128 : 0), 256);
    // (the prefilter's per-workgroup segments are laid out by whole tiles: up to two tiles beyond n)
    L.cand_stride = (size_t)n + (c.prefilter ? (size_t)2 * kHostGridBlock * kHostElemsPerLane : 0);
    L.cand0_off = off;
    off = align_up(off + (size_t)batch * L.cand_stride * 8, 256);
    L.cand1_off = off;
    off = align_up(off + (size_t)batch * L.cand_stride * 8, 256);
    L.total = off + 256;  // the last 16-byte load of an odd-length candidate array may touch 8 bytes past it
    return L;
}

}  // namespace rtopk

using namespace rtopk;

// The scratch memory of rtopk_select_static: part of the device code, one copy per GPU.  In host code this
// name is only a handle for hipGetSymbolAddress; kernels and copies get the address looked up below.
static __device__ __align__(256) unsigned char scratch[RTOPK_STATIC_SCRATCH_BYTES];

// Address of `scratch` on the current device, looked up once per device (each GPU has its own copy at its own
// address).  Returns nullptr if the runtime cannot tell.
static void* static_scratch_of_current_device() {
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> known[kMaxDevices];
    static std::mutex lookup;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = known[dev].load(std::memory_order_acquire);
    if (p) return p;
    std::lock_guard<std::mutex> hold(lookup);
    p = known[dev].load(std::memory_order_relaxed);
    if (!p) {
        void* found = nullptr;
        if (hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)) != hipSuccess || !found) return nullptr;
        p = found;
        known[dev].store(p, std::memory_order_release);
    }
    return p;
}

// How much of a streamed row (its tail) the first sweep reads with cache-allocating loads, for the second sweep
// to find in the caches (MI355X: 256 MB last-level cache + 32 MB of L2).  Measured on n = 2^28 fp32: the whole call takes
// 462 us with nothing kept, 449 with 256 MB, 444-445 with 288-320 MB, 451 with 352 MB and more (the first sweep
// slows down by more than the second gains).
static const size_t kKeepBytes = (size_t)288 << 20;

extern "C" {

const char* rtopk_status_string(rtopk_status s) {
    switch (s) {
        case RTOPK_OK: return "ok";
        case RTOPK_ERR_INVALID_ARG: return "invalid argument";
        case RTOPK_ERR_WORKSPACE_TOO_SMALL:
            return "workspace too small for these arguments and tuning (size it with rtopk_workspace_bytes_ex and the same tuning)";
        case RTOPK_ERR_UNSUPPORTED: return "unsupported (misaligned buffer)";
        case RTOPK_ERR_HIP: return "HIP runtime rejected a launch";
        case RTOPK_ERR_STATIC_SCRATCH:
            return "these arguments need more scratch memory than the built-in buffer of rtopk_select_static holds "
                   "(RTOPK_STATIC_SCRATCH_BYTES); use rtopk_select with a caller-owned workspace";
    }
    return "unknown status";
}

const char* rtopk_version(void) { return "0.1"; }

rtopk_status rtopk_workspace_bytes_ex(int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, uint32_t flags,
                                      const rtopk_tuning* tuning, size_t* bytes_out) {
    if (!bytes_out) return RTOPK_ERR_INVALID_ARG;
    Config c;
    rtopk_status s = make_config(batch, n, k, dt, 1, flags, tuning, &c);
    if (s != RTOPK_OK) return s;
    *bytes_out = make_layout(batch, n, c).total;
    return RTOPK_OK;
}

rtopk_status rtopk_workspace_bytes(int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, uint32_t flags,
                                   size_t* bytes_out) {
    return rtopk_workspace_bytes_ex(batch, n, k, dt, flags, nullptr, bytes_out);
}

// Every entry point ends here.  row_offsets / row_k: null, or the ragged batch's device arrays (n and k are then the
// largest row length and the largest k).
static rtopk_status select_impl(const void* keys, const int64_t* row_offsets, const int64_t* row_k, int64_t batch, int64_t n,
                                int64_t k, rtopk_dtype dt, int largest, uint32_t flags, uint64_t seed, void* out_values,
                                int64_t* out_indices, void* workspace, size_t workspace_bytes, void* hip_stream,
                                const rtopk_tuning* tuning, void* const* events) {
    if (!keys || !out_values || !out_indices || !workspace) return RTOPK_ERR_INVALID_ARG;
    if ((row_offsets == nullptr) != (row_k == nullptr)) return RTOPK_ERR_INVALID_ARG;
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
    P.row_offsets = (const long long*)row_offsets;
    P.row_k = (const long long*)row_k;
    P.out_values = out_values;
    P.out_indices = (long long*)out_indices;
    P.state = (rtopk_row_trace*)(ws + L.state_off);
    P.ghist = (u32*)(ws + L.ghist_off);
    P.seg = (u32*)(ws + L.seg_off);
    P.dbg = (unsigned long long*)(ws + L.dbg_off);
    P.swg = (u32*)(ws + L.swg_off);
    P.sort_hist = (u32*)(ws + L.sort_hist_off);
    P.sort_state = (void*)(ws + L.sort_state_off);
    P.Gs = c.Gs;
    P.cand[0] = (uint2*)(ws + L.cand0_off);
    P.cand[1] = (uint2*)(ws + L.cand1_off);
    P.cand_stride = L.cand_stride;
    P.pre_stride = c.prefilter ? c.pre_stride : 0u;
    P.n = n;
    P.k = k;
    P.batch = (int)batch;
    P.G = c.G;
    P.dirmask = c.dirmask;
    P.idx_max = c.idx_max;
    P.small = c.small;
    P.npass = c.npass;
    P.flags = flags;
    // two sweeps over more data than the 256 MB last-level cache holds: stream it past the caches
    P.keep_from_tile = 0xffffffffu;
    if ((size_t)batch * (size_t)n * (size_t)eb > ((size_t)384 << 20)) {
        P.flags |= kInternalStream;
        // a single long row: leave its last kKeepBytes in the last-level cache for the second sweep
        const size_t tile_bytes = (size_t)kHostGridBlock * kHostElemsPerLane * eb;
        const size_t row_tiles = ((size_t)n * eb + tile_bytes - 1) / tile_bytes;
        const size_t keep_tiles = kKeepBytes / tile_bytes;
        // (not when the second sweep writes a lot: with k = 2^24 and 2^27 of 2^28 the kept tail made the call
        // 3 % and 7 % slower instead of 4 % faster)
        const bool small_output = (size_t)k * (size_t)(eb + 8) <= ((size_t)32 << 20);
        if (batch == 1 && !row_offsets && small_output && row_tiles > keep_tiles) P.keep_from_tile = (u32)(row_tiles - keep_tiles);
    }
    P.seed = seed;
    for (int i = 0; i < c.npass; ++i) P.pass[i] = c.pass[i];

    hipStream_t st = (hipStream_t)hip_stream;
    (void)hipGetLastError();  // an error left by earlier HIP calls of the process is not this call's
    const bool scaled = (flags & RTOPK_FLAG_SCALING) && dt == RTOPK_F32;
    switch (dt) {
        case RTOPK_F32: return launch_f32(P, c, scaled, st, events);
        case RTOPK_F16: return launch_f16(P, c, false, st, events);
        case RTOPK_BF16: return launch_bf16(P, c, false, st, events);
    }
    return RTOPK_ERR_INVALID_ARG;
}

rtopk_status rtopk_select_events(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                                 uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices,
                                 void* workspace, size_t workspace_bytes, void* hip_stream,
                                 const rtopk_tuning* tuning, void* const* events) {
    return select_impl(keys, nullptr, nullptr, batch, n, k, dt, largest, flags, seed, out_values, out_indices, workspace,
                       workspace_bytes, hip_stream, tuning, events);
}

rtopk_status rtopk_select_ragged(const void* keys, const int64_t* row_offsets, const int64_t* row_k, int64_t batch,
                                 int64_t n_max, int64_t k_max, rtopk_dtype dt, int largest, uint32_t flags, uint64_t seed,
                                 void* out_values, int64_t* out_indices, void* workspace, size_t workspace_bytes,
                                 void* hip_stream, const rtopk_tuning* tuning) {
    if (!row_offsets || !row_k) return RTOPK_ERR_INVALID_ARG;
    if (((uintptr_t)row_offsets % 8) || ((uintptr_t)row_k % 8)) return RTOPK_ERR_UNSUPPORTED;
    return select_impl(keys, row_offsets, row_k, batch, n_max, k_max, dt, largest, flags, seed, out_values, out_indices,
                       workspace, workspace_bytes, hip_stream, tuning, nullptr);
}

rtopk_status rtopk_select_ex(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                             uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices, void* workspace,
                             size_t workspace_bytes, void* hip_stream, const rtopk_tuning* tuning) {
    return rtopk_select_events(keys, batch, n, k, dt, largest, flags, seed, out_values, out_indices, workspace,
                               workspace_bytes, hip_stream, tuning, nullptr);
}

rtopk_status rtopk_select(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                          uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    return rtopk_select_ex(keys, batch, n, k, dt, largest, flags, seed, out_values, out_indices, workspace,
                           workspace_bytes, hip_stream, nullptr);
}

rtopk_status rtopk_select_static(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                                 uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices,
                                 void* hip_stream) {
    size_t need = 0;
    const rtopk_status sized = rtopk_workspace_bytes(batch, n, k, dt, flags, &need);
    if (sized != RTOPK_OK) return sized;
    if (need > RTOPK_STATIC_SCRATCH_BYTES) return RTOPK_ERR_STATIC_SCRATCH;
    if (!keys || !out_values || !out_indices) return RTOPK_ERR_INVALID_ARG;
    void* ws = static_scratch_of_current_device();
    if (!ws) return RTOPK_ERR_HIP;
    // (every kernel chain starts by clearing the records, histograms and counters it relies on, so what the
    // previous call left in the buffer does not matter)
    return rtopk_select(keys, batch, n, k, dt, largest, flags, seed, out_values, out_indices, ws,
                        RTOPK_STATIC_SCRATCH_BYTES, hip_stream);
}

}  // extern "C"
