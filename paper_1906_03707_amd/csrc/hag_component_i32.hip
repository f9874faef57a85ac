// component-local pass, i32 features
#include "hag_component.inc"

namespace hag {
template int launch_component_kernel<int32_t>(const CompArgs<int32_t> &, int, int64_t, unsigned, unsigned, size_t, hipStream_t);
}
