// gather-reduce, f32 features, max
#include "hag_gather.inc"

namespace hag {
template int launch_gather<float, R_MAX, 0>(const GatherArgs<float> &, hipStream_t);
template int launch_gather<float, R_MAX, 3>(const GatherArgs<float> &, hipStream_t);
template int launch_gather<float, R_MAX, 5>(const GatherArgs<float> &, hipStream_t);
template int launch_gather<float, R_MAX, 6>(const GatherArgs<float> &, hipStream_t);
template int launch_fused<float, R_MAX, G_HAG_FWD>(const FusedArgs<float> &, hipStream_t);
}
