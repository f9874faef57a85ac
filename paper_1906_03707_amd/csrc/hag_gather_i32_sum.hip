// gather-reduce, i32 features, sum
#include "hag_gather.inc"

namespace hag {
template int launch_gather<int32_t, R_SUM, 0>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_SUM, 1>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_SUM, 2>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_SUM, 3>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_SUM, 4>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_SUM, 5>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_SUM, 6>(const GatherArgs<int32_t> &, hipStream_t);
template int launch_fused<int32_t, R_SUM, G_HAG_FWD>(const FusedArgs<int32_t> &, hipStream_t);
template int launch_fused<int32_t, R_SUM, G_HAG_BWD_SRC>(const FusedArgs<int32_t> &, hipStream_t);
template int launch_gather<int32_t, R_SUMIF, G_NAIVE_BWD>(const GatherArgs<int32_t> &, hipStream_t);
}
