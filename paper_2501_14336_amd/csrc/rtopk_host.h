// Host-side plan of one call: which kernels run, with what geometry.  Shared by the API translation
// unit and the per-type kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include "rtopk.h"
#include "rtopk_device.h"

namespace rtopk {

struct Config {
    int d, path, G;
    int Gs;          // sorted output of long rows: workgroups per row of the radix sort (0: not needed)
    u32 small;
    int npass;
    bool one_sweep;  // path 1: try the one-sweep kernel (small k) first
    bool prefilter;  // path 2: histogram of a sample + ONE sweep over X that counts and filters, instead of two sweeps
    unsigned pre_stride;
    int multi_last;  // last digit pass that may still hold more than `small` candidates (grid kernels run up to it)
    u32 idx_max, dirmask;
    PassInfo pass[kMaxPasses];
};

// Enqueue every kernel of one call for one key type (defined in rtopk_f32.hip / rtopk_f16.hip / rtopk_bf16.hip).
rtopk_status launch_f32(const Params& P, const Config& c, bool scaled, hipStream_t st, void* const* events);
rtopk_status launch_f16(const Params& P, const Config& c, bool scaled, hipStream_t st, void* const* events);
rtopk_status launch_bf16(const Params& P, const Config& c, bool scaled, hipStream_t st, void* const* events);

// Launch geometry the host needs for sizing.
constexpr int kHostHistBuffers = 6;  // global histograms per row: four in rotation, the sample's, the prefilter's second
constexpr int kHostSwgBuffers = 4;   // per-workgroup record sets per row: three in rotation, the prefilter's second
constexpr int kHostSortSmall = 8192;  // sorted output: rows of up to this many outputs are sorted by one workgroup in LDS
constexpr int kHostGridBlock = 512;
constexpr int kHostElemsPerLane = 16;

}  // namespace rtopk
