/*
 * rtopk -- batched radix top-k selection on AMD Instinct MI355X (gfx950).
 *
 * C ABI.  Plain pointers and sizes only; no exceptions cross the boundary; no
 * global state apart from an immutable tuning default.  Every pointer named
 * "device" is GPU memory (hipMalloc or a PyTorch CUDA/HIP tensor's data_ptr()),
 * everything else is host memory.
 *
 * The operation (paper, Section 1: top-k of n elements, values and their
 * positions, largest or smallest, any k <= n; Section 2.3.1, Algorithm 1: radix
 * select of the k-th element followed by a filter; Section 2.3.2 / 3.2: a batch
 * of B independent tasks):
 *
 *   for every row r of keys[batch][n]:
 *     choose the k elements that rank best under the order
 *         NaN (any sign/payload) > +inf > ... > +0 > -0 > ... > -inf      (largest)
 *       or its reverse                                                    (smallest),
 *     ties at the k-th key resolved towards the LOWEST index,
 *     and write their original bit patterns and their positions in the row.
 *
 * The selected SET is unique and reproducible.  The order of the k outputs
 * inside a row is unspecified (the paper's output is unsorted, Section 2.3.1);
 * the order may differ between runs with the same arguments (the set never does).
 * With RTOPK_FLAG_SORTED the order is fixed too: best first, lowest index first among equals.
 */
#ifndef RTOPK_H
#define RTOPK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { RTOPK_F32 = 0, RTOPK_F16 = 1, RTOPK_BF16 = 2 } rtopk_dtype;

typedef enum {
    RTOPK_OK = 0,
    RTOPK_ERR_INVALID_ARG = 1,          /* null pointer, k < 1, k > n, batch < 1, n out of range, bad dtype/flags */
    RTOPK_ERR_WORKSPACE_TOO_SMALL = 2,  /* workspace_bytes below rtopk_workspace_bytes() for these arguments    */
    RTOPK_ERR_UNSUPPORTED = 3,          /* misaligned buffers (see rtopk_select)                                */
    RTOPK_ERR_HIP = 4,                  /* a kernel launch was rejected by the runtime                          */
    RTOPK_ERR_STATIC_SCRATCH = 5        /* rtopk_select_static: the arguments need more scratch memory than the
                                           library's built-in buffer holds (use rtopk_select with a workspace)  */
} rtopk_status;

enum {
    /* Adaptive scaling (paper Section 4.3): one element a_s of each row is drawn with `seed` and
     * subtracted (one fp32 rounding) from every element before digits are taken, which spreads
     * the exponents of keys clustered near a_s.  The rounded difference orders keys weakly, so
     * the library finishes the selection on the unscaled key; the result is identical with and
     * without the flag and for every seed.  Ignored for 16-bit keys. */
    RTOPK_FLAG_SCALING = 1u << 0,
    /* Accepted and without effect: the per-pass records (rtopk_row_trace below) are the library's own
     * loop state, so they are written on every call. */
    RTOPK_FLAG_DEBUG_COUNTERS = 1u << 1,
    /* Sorted output: every row's k outputs in the order best element first (descending for "largest",
     * ascending for "smallest"; NaN ranks above +inf, -0 below +0), lowest index first among equal elements.
     * The paper's output is unsorted by nature (Section 2.3.1); its evaluation sorts afterwards and counts
     * that time (Section 5.2).  Costs a sort of the k pairs after the selection: in LDS for k <= 8192, a
     * radix sort in the workspace beyond. */
    RTOPK_FLAG_SORTED = 1u << 2
};

/* Maximum row length: indices are kept in 32 bits inside the library. */
#define RTOPK_MAX_N ((int64_t)1 << 31)

/*
 * Optional tuning knobs.  The selected set never depends on them (the paper calls the digit
 * width and block/grid sizes hyper-parameters, Section 5.2); tests use them to exercise every
 * code path on the same input.  A field left 0 means "library default".
 */
typedef struct {
    int32_t digit_bits;      /* radix digit width d, 8..12 (default 12; 11 for 16-bit keys when one workgroup
                                handles a row)                                                                  */
    int32_t path;            /* 0 auto, 1 one workgroup per row (fused kernel), 2 many workgroups per row,
                                3 like 1, with the one-sweep kernel for small k first (auto picks it for
                                batches of 64 rows up with k <= 256, k <= 512 on rows of 64K keys up)           */
    int32_t wgs_per_row;     /* workgroups cooperating on one row in path 2 (default: fill 256 CUs)            */
    int32_t small_threshold; /* candidate count at or below which one workgroup finishes a row by itself       */
    int32_t prefilter;       /* path 2: 0 auto, 1 always, -1 never: histogram of a sample of the row, then ONE
                                sweep over X that counts every digit and keeps everything from a bin chosen
                                from the sample upwards (pass 0 then runs on what was kept), instead of two
                                sweeps over X; the second sweep still runs if the sample misled               */
} rtopk_tuning;

/*
 * Size in bytes of the device scratch buffer rtopk_select needs for these arguments
 * (two candidate arrays of n (value, index) pairs per row, per-workgroup histograms, per-row
 * state -- the "workspace in global memory" of paper Section 2.2.3).  Host-only, launches nothing.
 * Returns RTOPK_ERR_INVALID_ARG on bad arguments and leaves *bytes_out.
 *
 * The two sizing calls pair with the two selection calls: rtopk_workspace_bytes with rtopk_select
 * (library defaults), rtopk_workspace_bytes_ex with rtopk_select_ex / rtopk_select_events and the SAME
 * tuning (NULL = defaults, the same size as rtopk_workspace_bytes).  A tuning that forces many workgroups
 * per row on a shape whose default is one workgroup per row needs the larger buffer; a buffer sized
 * without it is rejected with RTOPK_ERR_WORKSPACE_TOO_SMALL before anything is launched.
 */
rtopk_status rtopk_workspace_bytes(int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, uint32_t flags,
                                   size_t* bytes_out);
rtopk_status rtopk_workspace_bytes_ex(int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, uint32_t flags,
                                      const rtopk_tuning* tuning, size_t* bytes_out);

/*
 * Enqueue the selection on `hip_stream` (a hipStream_t; NULL = the default stream) and return
 * without synchronising.  No memory is allocated or freed.  Nothing is read back to the host:
 * loop control lives in the workspace (Algorithm 1's loop state, Section 2.3.1).
 *
 *   keys         device, [batch][n] row-major, element type dt, read-only.  The first row must
 *                start on a multiple of the element size; rows need NOT be 16-byte aligned (loads
 *                start at the aligned address at or before the row and mask the lead-in, the
 *                paper's on-demand offset padding, Section 3.2.2).
 *   batch, n, k  1 <= batch, 1 <= n <= RTOPK_MAX_N, 1 <= k <= n.
 *   largest      non-zero: k largest; zero: k smallest.
 *   flags        OR of RTOPK_FLAG_*; unknown bits are rejected.
 *   seed         only drives the draw of a_s under RTOPK_FLAG_SCALING.
 *   out_values   device, [batch][k], element type dt, aligned to the element size; receives the
 *                selected elements' original bits (NaN payloads and zero signs preserved).
 *   out_indices  device, [batch][k] int64, 8-byte aligned; position of each selected element in its row.
 *   workspace    device, 256-byte aligned, at least rtopk_workspace_bytes(...) bytes computed with the
 *                same batch, n, k, dt and flags (rtopk_workspace_bytes_ex with the same tuning for the
 *                calls that take one).  Contents are undefined afterwards.  Two calls that may overlap in
 *                time must not share a workspace.
 *
 * The returned status covers the arguments and the launches only: argument errors are detected on the
 * host before anything is launched (no output is written then), and RTOPK_ERR_HIP reports a launch the
 * runtime rejected during THIS call (an error left behind by earlier HIP calls of the process is cleared
 * first, not reported).  The kernels run after the call returns; if one of them meets a state that cannot
 * occur in a consistent run (counts that do not add up), it sets a bit in rtopk_row_trace.error of that
 * row, drops the writes that would leave the buffers, and the row's output is then incomplete.  A caller
 * that wants this checked reads the row records after the stream has drained (see rtopk_row_trace).
 */
rtopk_status rtopk_select(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                          uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* Same as rtopk_select with explicit tuning knobs (NULL = defaults). */
rtopk_status rtopk_select_ex(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                             uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices,
                             void* workspace, size_t workspace_bytes, void* hip_stream,
                             const rtopk_tuning* tuning);

/*
 * Ragged batch (paper Section 3.2.2: tasks of different lengths stored one after the other, with the padding a
 * 16-byte load needs supplied on demand; the ablation of Section 5.3.3 uses such a batch): row r is
 * keys[row_offsets[r] .. row_offsets[r + 1]) of ONE array and has its own k, row_k[r].
 *
 *   keys         device, the rows one after the other, element type dt, aligned to the element size
 *   row_offsets  device, batch + 1 int64, in elements, non-decreasing; rows need no alignment
 *   row_k        device, batch int64, 0 <= row_k[r] <= length of row r
 *   n_max, k_max host: no row is longer than n_max, no row_k exceeds k_max; 1 <= k_max <= n_max <= RTOPK_MAX_N.
 *                They size the workspace -- rtopk_workspace_bytes_ex(batch, n_max, k_max, dt, flags, tuning) --
 *                and choose the kernels; the result does not depend on them.
 *   out_values   device, [batch][k_max]; out_indices device, [batch][k_max] int64: row r's row_k[r] results are
 *                the first entries of output row r (positions within the row, from 0); the rest is left alone.
 * Everything else as in rtopk_select_ex.  The two arrays live on the device, so they are checked there: a row
 * whose k is 0 (or that is empty) is skipped and has no pass records; a row_k beyond the row's length or k_max, a
 * negative one, or a row longer than n_max is cut down to what fits and reported as bit 8 of that row's
 * rtopk_row_trace.error.
 */
rtopk_status rtopk_select_ragged(const void* keys, const int64_t* row_offsets, const int64_t* row_k, int64_t batch,
                                 int64_t n_max, int64_t k_max, rtopk_dtype dt, int largest, uint32_t flags, uint64_t seed,
                                 void* out_values, int64_t* out_indices, void* workspace, size_t workspace_bytes,
                                 void* hip_stream, const rtopk_tuning* tuning);

/*
 * rtopk_select for callers that cannot allocate device memory and have no workspace to pass: code under
 * HIP graph capture, tight serving loops (top-k over a batch of logit rows at every decoding step),
 * harnesses that forbid hipMalloc.  Identical to rtopk_select in arguments, defaults, result and error
 * behaviour, except that the scratch memory is not the caller's: it is a buffer of
 * RTOPK_STATIC_SCRATCH_BYTES that is part of the library's device code (every GPU the library runs on
 * holds one copy from the first call on that GPU until the process ends).  The call allocates and frees
 * nothing and synchronises nothing; the first call on a device looks the buffer's address up once.
 *
 * Limits: rtopk_workspace_bytes(batch, n, k, dt, flags) must not exceed RTOPK_STATIC_SCRATCH_BYTES --
 * otherwise RTOPK_ERR_STATIC_SCRATCH is returned and nothing is launched.  The workspace holds two candidate
 * arrays of 8 bytes per key, so that admits inputs of up to about 4 million keys in total (batch * n), of any
 * shape: 32 rows of 2^17 logits, one row of 2^22 keys.
 * All calls on one GPU share that GPU's buffer: two calls that may overlap in time on the same GPU (different
 * streams, different host threads) race; the caller orders them.  The buffer keeps the previous call's
 * contents; every call clears what it needs cleared itself.
 */
#define RTOPK_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
rtopk_status rtopk_select_static(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                                 uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices,
                                 void* hip_stream);

/*
 * Profiling variant of rtopk_select_ex: additionally records caller-created HIP events (hipEvent_t handles,
 * host array `events` of RTOPK_NUM_EVENTS entries, NULL entries are skipped) on `hip_stream` at fixed points,
 * so that a harness can time the two sweeps over the input (the countBin and selectCandidate/filter sweeps of
 * paper Section 2.3.1, which dominate the run time, Section 3.2.1) without an external profiler:
 *   events[0] before anything is enqueued          events[1] before the first-pass HIST kernel
 *   events[2] between first-pass HIST and CLASSIFY  events[3] after the first-pass CLASSIFY kernel
 *   events[4] after the last kernel
 * With one workgroup per row (a single fused kernel) events[1..3] are recorded together with events[0].
 * Nothing is synchronised; the caller reads the events after the stream has drained.
 */
#define RTOPK_NUM_EVENTS 5
rtopk_status rtopk_select_events(const void* keys, int64_t batch, int64_t n, int64_t k, rtopk_dtype dt, int largest,
                                 uint32_t flags, uint64_t seed, void* out_values, int64_t* out_indices,
                                 void* workspace, size_t workspace_bytes, void* hip_stream,
                                 const rtopk_tuning* tuning, void* const* events);

/*
 * Per-pass record of the last rtopk_select that used `workspace`, for tests and profiling:
 * which bin each digit pass chose and how many candidates and winners it left (the quantities
 * selectBin and selectCandidate produce, paper Section 2.3.1).  The records live at the start of
 * the workspace: row r's record is RTOPK_TRACE_STRIDE bytes at byte offset r * RTOPK_TRACE_STRIDE,
 * laid out as rtopk_row_trace.  Read it with any device-to-host copy after the stream has drained.
 * The library keeps its loop state in these records (each is written once per call).
 */
#define RTOPK_TRACE_STRIDE 512
#define RTOPK_TRACE_MAX_PASSES 12
typedef struct {
    float a_s;                 /* the element subtracted under RTOPK_FLAG_SCALING (0 if unused)      */
    uint32_t error;            /* 0, or a bit set if the device saw an impossible state              */
    uint32_t redo;             /* 1: the one-sweep row kernel left this row to the two-sweep kernel
                                  (which clears the record, redo_why excepted, when it takes the row
                                  over)                                                              */
    uint32_t redo_why;         /* diagnostic; non-zero: the one-sweep kernel handed the row over.
                                  1 inf/NaN in the part counted first, 2 that part shorter than k,
                                  3 bin edge not a number, 5 list full, 6 too many candidates in the
                                  chosen bin, 7 list expected to overflow, 8 the sample misled (fewer
                                  than k elements at or above its bound)                              */
    uint32_t pre_elems;        /* elements in the row's sample, counted before a prefilter sweep
                                  (0: no prefilter, the whole row was counted)                       */
    uint32_t pre_bound;        /* with a prefilter: the bin taken from the sample; the sweep kept the
                                  elements of this bin and the better ones                           */
    uint32_t pre_kept;         /* how many elements that were                                        */
    uint32_t pre_missed;       /* 1: the k-th key's bin lies below pre_bound (the sample misled), so
                                  pass 0 swept the row again instead of reading what was kept;
                                  2: the same on purpose -- the sample showed the keys crowded into the
                                  bins to keep (over 1/8 of the row; 1/16 for 16-bit keys), so the sweep kept nothing
                                  (pre_bound is the bin count) and only counted                     */
    uint32_t pre_merged;       /* 1: the prefilter's bound bin was the k-th key's bin, and pass 0 had no
                                  sweep of its own -- pass 1's sweep over what was kept classified by both
                                  digits at once (pass 0's record: its selectBin; winners are what lay above
                                  its bin; neither read nor wrote anything).  Also after a sweep that
                                  declined (pre_missed 2), when the exact counts confirm pre_crowd and that
                                  bin holds at least 7/8 of the row: both digits are then read from X    */
    uint32_t pre_crowd;        /* with pre_bound = 2^bits (the sweep declined): the bin the sample puts the
                                  k-th key in, whose elements' second digit the sweep counted as well;
                                  0xffffffff if it counted none                                         */
    uint32_t reserved[6];
    struct {
        uint32_t where;        /* 0 pass not run; 1 many workgroups; 2 single-workgroup finish;
                                  3 fused one-workgroup-per-row kernel; 4 one-sweep row kernel       */
        uint32_t bin;          /* chosen bin of this digit                                           */
        uint32_t k_after;      /* rank of the k-th key inside the bin (0 if the whole bin was taken) */
        uint32_t cand_after;   /* candidates passed on to the next digit (0: the row is finished)    */
        uint32_t winners;      /* elements sent to the output by this pass                           */
        uint32_t out_before;   /* outputs already written when this pass started                     */
        uint32_t cand_before;  /* candidates this pass looked at                                     */
        uint32_t window;       /* source | shift << 8 | bits << 16 | array << 24; source 0 scaled key, 1 key,
                                  2 index (tie break); the digit is bits [shift, shift + bits); array: which
                                  of the two candidate arrays the pass wrote.
                                  Source 3: not a digit pass -- at most 512 candidates were left and
                                  were ranked against each other directly (by key, then index),
                                  which stands for all the digit passes that would have followed;
                                  bin and k_after are 0, winners is the number of them that won      */
    } pass_rec[RTOPK_TRACE_MAX_PASSES];
} rtopk_row_trace;

/* Static description of an error code. */
const char* rtopk_status_string(rtopk_status status);

/* Library version, "major.minor". */
const char* rtopk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RTOPK_H */
