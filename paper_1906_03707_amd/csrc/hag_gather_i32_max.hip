// gather-reduce, i32 features, max
#include "hag_gather.inc"

namespace hag {
template int launch_gather<int32_t, R_MAX, 0>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_MAX, 3>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_MAX, 5>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_MAX, 6>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_fused<int32_t, R_MAX, G_HAG_FWD>(const FusedArgs<int32_t> &, hipStream_t);
}
