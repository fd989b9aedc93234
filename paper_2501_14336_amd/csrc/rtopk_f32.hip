// Kernel instantiations for RTOPK_F32 keys.
#include "rtopk_kernels.inl"

namespace rtopk {
rtopk_status launch_f32(const Params& P, const Config& c, bool scaled, hipStream_t st, void* const* events) {
    return launch_all<RTOPK_F32>(P, c, scaled, st, events);
}
}  // namespace rtopk
