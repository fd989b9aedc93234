// Sorted output (RTOPK_FLAG_SORTED): after the selection, the k (value, index) pairs of every row are put into
// the order best element first, lowest index first among equal elements.  The paper's output is unsorted by
// nature (Section 2.3.1) and its evaluation sorts it afterwards (Section 5.2); this is that step, on the GPU.
//
// Every pair becomes one 64-bit sort key: the complement of the element's ordered key (so that ascending order is
// best first) above its index.  The keys of a row are distinct.
//   k <= kSortSmall: one workgroup per row sorts the keys in LDS (bitonic network).
//   larger k: least-significant-digit radix sort, 8 bits per pass, on the two candidate arrays of the workspace
//   (idle once the selection is done): per pass a histogram per workgroup chunk, one scan of the (bin, chunk)
//   table, and a stable scatter.  A pass whose digit is the same for all keys of the row (the zero low half of a
//   16-bit key, index bits above log2 n) is skipped.
// The sorted keys are unpacked into the outputs; values are gathered again from X by index, so they keep their
// original bits (NaN payloads, zero signs).
//
// Included by rtopk_kernels.inl (inside namespace rtopk).

constexpr int kSortSmall = kHostSortSmall;  // pairs one workgroup sorts in LDS
constexpr int kSortBlock = 512;         // threads per workgroup, radix sort kernels
constexpr int kSortBins = 256;
constexpr int kSortPasses = 8;
// per-row state of the radix sort, in the workspace: cur[j] = which candidate array holds the keys when pass j
// starts (cur[kSortPasses]: when all are done), skip[j] = pass j moves nothing
struct SortState {
    u32 cur[kSortPasses + 1];
    u32 skip[kSortPasses];
    u32 pad[32 - 2 * kSortPasses - 1];
};
static_assert(sizeof(SortState) == 128, "sort state record");

template <int DT>
__device__ __forceinline__ u64 sort_key_of(u32 raw, u32 idx, u32 dirmask) {
    const u32 okey = KeyOf<DT>::key(raw) ^ dirmask;
    return ((u64)(~okey) << 32) | (u64)idx;
}
template <int DT>
__device__ __forceinline__ u32 load_value(const void* v, size_t i) {
    return DT == RTOPK_F32 ? ((const u32*)v)[i] : (u32)((const uint16_t*)v)[i];
}

// Up to three consecutive levels of the bitonic network (strides S, S/2, ... down to h = S >> (L - 1)) in one go:
// the 2^L elements that these levels connect -- h apart, starting at a multiple of 2 S plus an offset below h -- are
// held by one thread, which exchanges among them in registers.  One barrier and one trip through LDS per group of
// levels instead of one per level.  (All of a group's elements lie in one block of `size` elements: one direction.)
template <int L>
__device__ __forceinline__ void bitonic_levels(u64* buf, u32 m, u32 size, u32 S, u32 tid) {
    constexpr u32 N = 1u << L;
    const u32 h = S >> (L - 1);
    for (u32 g = tid; g < (m >> L); g += kRowBlock) {
        const u32 base = (g / h) * (h << L) + (g & (h - 1u));
        const bool up = (base & size) == 0;
        u64 e[N];
#pragma unroll
        for (u32 j = 0; j < N; ++j) e[j] = buf[base + j * h];
#pragma unroll
        for (int l = L - 1; l >= 0; --l) {
#pragma unroll
            for (u32 j = 0; j < N; ++j) {
                if ((j >> l) & 1u) continue;
                const u64 a = e[j], b = e[j | (1u << l)];
                const bool swap = (a > b) == up;
                e[j] = swap ? b : a;
                e[j | (1u << l)] = swap ? a : b;
            }
        }
#pragma unroll
        for (u32 j = 0; j < N; ++j) buf[base + j * h] = e[j];
    }
}

// k <= kSortSmall: bitonic sort of one row's keys in LDS.
template <int DT>
__global__ void __launch_bounds__(kRowBlock) k_sort_small(Params P) {
    __shared__ u64 buf[kSortSmall];
    constexpr int B = kRowBlock;
    const int row = blockIdx.x;
    const u32 tid = threadIdx.x;
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    const u32 k = rs.k;
    if (k == 0) return;
    char* out_v = (char*)P.out_values + (size_t)row * (size_t)P.k * KeyOf<DT>::kBytes;
    long long* out_i = P.out_indices + (size_t)row * (size_t)P.k;
    const char* x = rs.x;
    u32 m = 64;
    while (m < k) m <<= 1;
    for (u32 i = tid; i < m; i += B)
        buf[i] = i < k ? sort_key_of<DT>(load_value<DT>(out_v, i), (u32)out_i[i], P.dirmask) : ~0ull;  // padding sorts last
    for (u32 size = 2, levels = 1; size <= m; size <<= 1, ++levels) {
        // the levels of this size, largest stride first: a first group of levels % 3 (if any), then groups of three,
        // so that the group with the smallest strides -- the one whose threads touch neighbouring words -- is a full one
        u32 stride = size >> 1, left = levels;
        while (left > 0) {
            const u32 L = left % 3u ? left % 3u : 3u;
            __syncthreads();
            if (L == 1) bitonic_levels<1>(buf, m, size, stride, tid);
            else if (L == 2) bitonic_levels<2>(buf, m, size, stride, tid);
            else bitonic_levels<3>(buf, m, size, stride, tid);
            stride >>= L;
            left -= L;
        }
    }
    __syncthreads();
    for (u32 i = tid; i < k; i += B) {
        const u32 idx = (u32)buf[i];
        out_i[i] = (long long)idx;
        store_value<DT>(out_v, i, load_value<DT>(x, idx));
    }
}

// ---- radix sort of long rows ----
__device__ __forceinline__ SortState* sort_state(const Params& P, int row) { return (SortState*)P.sort_state + row; }
__device__ __forceinline__ u64* sort_buffer(const Params& P, u32 which, int row) {
    return (u64*)(P.cand[which] + (size_t)row * P.cand_stride);
}
// the chunk of workgroup w: [begin, end), a whole number of kSortBlock-element tiles but for the row's end
__device__ __forceinline__ void sort_chunk(const Params& P, u32 k, u32 w, u32& begin, u32& end) {
    u32 per = (k + (u32)P.Gs - 1u) / (u32)P.Gs;
    per = (per + kSortBlock - 1u) / kSortBlock * kSortBlock;
    const u64 b = (u64)w * per, e = b + per;
    begin = b < k ? (u32)b : k;
    end = e < k ? (u32)e : k;
}

// outputs -> keys in candidate array 0
template <int DT>
__global__ void __launch_bounds__(kSortBlock) k_sort_pack(Params P) {
    const int row = blockIdx.y;
    const u32 row_k = row_shape<KeyOf<DT>::kBytes>(P, row).k;
    const char* out_v = (const char*)P.out_values + (size_t)row * (size_t)P.k * KeyOf<DT>::kBytes;
    const long long* out_i = P.out_indices + (size_t)row * (size_t)P.k;
    u64* dst = sort_buffer(P, 0u, row);
    u32 begin, end;
    sort_chunk(P, row_k, blockIdx.x, begin, end);
    for (u32 i = begin + threadIdx.x; i < end; i += kSortBlock)
        dst[i] = sort_key_of<DT>(load_value<DT>(out_v, i), (u32)out_i[i], P.dirmask);
    if (blockIdx.x == 0 && threadIdx.x < sizeof(SortState) / 4) ((u32*)sort_state(P, row))[threadIdx.x] = 0;
}

// histogram of pass j's digit over each workgroup's chunk: table[workgroup][bin]
template <int DT>
__global__ void __launch_bounds__(kSortBlock) k_sort_hist(Params P, int j) {
    __shared__ u32 h[kSortBins];
    const int row = blockIdx.y;
    const u32 row_k = row_shape<KeyOf<DT>::kBytes>(P, row).k;
    const u64* src = sort_buffer(P, sort_state(P, row)->cur[j], row);
    if (threadIdx.x < kSortBins) h[threadIdx.x] = 0;
    __syncthreads();
    u32 begin, end;
    sort_chunk(P, row_k, blockIdx.x, begin, end);
    for (u32 i = begin + threadIdx.x; i < end; i += kSortBlock) atomicAdd(&h[(u32)(src[i] >> (8 * j)) & 255u], 1u);
    __syncthreads();
    u32* table = P.sort_hist + (size_t)row * kSortBins * P.Gs;
    if (threadIdx.x < kSortBins) table[(size_t)blockIdx.x * kSortBins + threadIdx.x] = h[threadIdx.x];
}

// exclusive scan of the table in (bin, workgroup) order: where each workgroup's elements of each bin go.
// Four threads share a bin, each owning a quarter of the workgroups' counts of that bin; the 256 threads of a
// quarter read consecutive words (the table is laid out [workgroup][bin]).  One scan over the threads' sums,
// taken in (bin, quarter) order, gives every thread the offset its stretch starts at.
template <int DT>
__global__ void __launch_bounds__(kRowBlock) k_sort_scan(Params P, int j) {
    static_assert(kRowBlock == 4 * kSortBins, "four threads per bin");
    __shared__ u32 wsum[kRowBlock / 64];
    __shared__ u32 sums[kRowBlock], upto[kRowBlock];
    __shared__ u32 all_in_one;
    const int row = blockIdx.x;
    const u32 tid = threadIdx.x;
    const u32 row_k = row_shape<KeyOf<DT>::kBytes>(P, row).k;
    u32* table = P.sort_hist + (size_t)row * kSortBins * P.Gs;
    const u32 Gs = (u32)P.Gs, per = (Gs + 3u) / 4u;
    const u32 bin = tid & (u32)(kSortBins - 1), quarter = tid / (u32)kSortBins;
    const u32 w0 = quarter * per < Gs ? quarter * per : Gs, w1 = w0 + per < Gs ? w0 + per : Gs;
    if (tid == 0) all_in_one = 0;
    u32 sum = 0;
    for (u32 w = w0; w < w1; ++w) sum += table[(size_t)w * kSortBins + bin];
    sums[bin * 4u + quarter] = sum;
    __syncthreads();
    const u32 v = sums[tid];  // thread order is now (bin, quarter) order
    const u32 incl = block_inclusive_scan<kRowBlock>(v, wsum);
    upto[tid] = incl;
    __syncthreads();
    // is the digit the same for every key?  (then some bin holds all k; also a row with nothing to sort)
    if ((tid & 3u) == 3u && incl - (tid >= 4u ? upto[tid - 4u] : 0u) == row_k) all_in_one = 1;
    __syncthreads();
    const bool skip = all_in_one != 0;
    if (!skip) {
        u32 run = upto[bin * 4u + quarter] - sum;
        for (u32 w = w0; w < w1; ++w) {
            const u32 c = table[(size_t)w * kSortBins + bin];
            table[(size_t)w * kSortBins + bin] = run;
            run += c;
        }
    }
    if (tid == 0) {
        SortState* st = sort_state(P, row);
        st->skip[j] = skip ? 1u : 0u;
        st->cur[j + 1] = skip ? st->cur[j] : 1u - st->cur[j];
    }
}

// stable scatter of pass j: elements keep their order within a bin
template <int DT>
__global__ void __launch_bounds__(kSortBlock) k_sort_scatter(Params P, int j) {
    constexpr int W = kSortBlock / 64;
    __shared__ u32 base[kSortBins];          // next free position of every bin for this workgroup
    __shared__ u32 wcount[W][kSortBins];     // per wave: elements of each bin in the current tile; then their offset
    const int row = blockIdx.y;
    const u32 row_k = row_shape<KeyOf<DT>::kBytes>(P, row).k;
    const SortState* st = sort_state(P, row);
    if (st->skip[j]) return;
    const u32 tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const u64* src = sort_buffer(P, st->cur[j], row);
    u64* dst = sort_buffer(P, 1u - st->cur[j], row);
    const u32* table = P.sort_hist + (size_t)row * kSortBins * P.Gs;
    if (tid < kSortBins) base[tid] = table[(size_t)blockIdx.x * kSortBins + tid];
    u32 begin, end;
    sort_chunk(P, row_k, blockIdx.x, begin, end);
    for (u32 t0 = begin; t0 < end; t0 += kSortBlock) {
        for (u32 q = tid; q < (u32)(W * kSortBins); q += kSortBlock) (&wcount[0][0])[q] = 0;
        __syncthreads();
        const u32 i = t0 + tid;
        const bool have = i < end;
        const u64 key = have ? src[i] : 0ull;
        const u32 d = (u32)(key >> (8 * j)) & 255u;
        // lanes of this wave that hold the same digit
        u64 peers = ballot64(have);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = ((d >> b) & 1u) != 0;
            const u64 m = ballot64(bit);
            peers &= bit ? m : ~m;
        }
        const u32 rank_in_wave = mbcnt64(peers);
        if (have && rank_in_wave == 0) wcount[wave][d] = (u32)__popcll(peers);
        __syncthreads();
        // per bin (thread t owns bin t): offsets of the waves, in wave order, and the tile's total
        u32 tile_total = 0;
        if (tid < kSortBins) {
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const u32 c = wcount[w][tid];
                wcount[w][tid] = tile_total;
                tile_total += c;
            }
        }
        __syncthreads();
        if (have) dst[base[d] + wcount[wave][d] + rank_in_wave] = key;
        __syncthreads();
        if (tid < kSortBins) base[tid] += tile_total;
    }
}

// sorted keys -> outputs; values are gathered from X by index
template <int DT>
__global__ void __launch_bounds__(kSortBlock) k_sort_unpack(Params P) {
    const int row = blockIdx.y;
    const RowShape rs = row_shape<KeyOf<DT>::kBytes>(P, row);
    const u32 row_k = rs.k;
    const u64* src = sort_buffer(P, sort_state(P, row)->cur[kSortPasses], row);
    char* out_v = (char*)P.out_values + (size_t)row * (size_t)P.k * KeyOf<DT>::kBytes;
    long long* out_i = P.out_indices + (size_t)row * (size_t)P.k;
    const char* x = rs.x;
    u32 begin, end;
    sort_chunk(P, row_k, blockIdx.x, begin, end);
    for (u32 i = begin + threadIdx.x; i < end; i += kSortBlock) {
        const u32 idx = (u32)src[i];
        out_i[i] = (long long)idx;
        store_value<DT>(out_v, i, load_value<DT>(x, idx));
    }
}

// Enqueue the sort of every row's output.
template <int DT>
static void launch_sort(const Params& P, hipStream_t st) {
    if (P.k <= kSortSmall) {
        hipLaunchKernelGGL((k_sort_small<DT>), dim3(P.batch), dim3(kRowBlock), 0, st, P);
        return;
    }
    const dim3 grid(P.Gs, P.batch), block(kSortBlock);
    hipLaunchKernelGGL((k_sort_pack<DT>), grid, block, 0, st, P);
    for (int j = 0; j < kSortPasses; ++j) {
        hipLaunchKernelGGL((k_sort_hist<DT>), grid, block, 0, st, P, j);
        hipLaunchKernelGGL((k_sort_scan<DT>), dim3(P.batch), dim3(kRowBlock), 0, st, P, j);
        hipLaunchKernelGGL((k_sort_scatter<DT>), grid, block, 0, st, P, j);
    }
    hipLaunchKernelGGL((k_sort_unpack<DT>), grid, block, 0, st, P);
}
