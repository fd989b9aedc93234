// Kernel instantiations for RTOPK_F16 keys.
#include "rtopk_kernels.inl"

namespace rtopk {
rtopk_status launch_f16(const Params& P, const Config& c, bool scaled, hipStream_t st, void* const* events) {
    return launch_all<RTOPK_F16>(P, c, scaled, st, events);
}
}  // namespace rtopk
