// component-local pass, f32 features
#include "hag_component.inc"

namespace hag {
template int launch_component_kernel<float>(const CompArgs<float> &, int, int64_t, unsigned, unsigned, size_t, hipStream_t);
}
