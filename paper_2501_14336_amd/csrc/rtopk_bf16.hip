// Kernel instantiations for RTOPK_BF16 keys.
#include "rtopk_kernels.inl"

namespace rtopk {
rtopk_status launch_bf16(const Params& P, const Config& c, bool scaled, hipStream_t st, void* const* events) {
    return launch_all<RTOPK_BF16>(P, c, scaled, st, events);
}
}  // namespace rtopk
