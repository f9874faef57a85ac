// gather-reduce, f32 features, sum
#include "hag_gather.inc"

namespace hag {
template int launch_gather<float, R_SUM, 0>(const GatherArgs<float> &, hipStream_t);
template int launch_gather<float, R_SUM, 1>(const GatherArgs<float> &, hipStream_t);
template int launch_gather<float, R_SUM, 2>(const GatherArgs<float> &, hipStream_t);
template int launch_gather<float, R_SUM, 3>(const GatherArgs<float> &, hipStream_t);
template int launch_gather<float, R_SUM, 4>(const GatherArgs<float> &, hipStream_t);
template int launch_gather<float, R_SUM, 5>(const GatherArgs<float> &, hipStream_t);
template int launch_gather<float, R_SUM, 6>(const GatherArgs<float> &, hipStream_t);
template int launch_fused<float, R_SUM, G_HAG_FWD>(const FusedArgs<float> &, hipStream_t);
template int launch_fused<float, R_SUM, G_HAG_BWD_SRC>(const FusedArgs<float> &, hipStream_t);
template int launch_gather<float, R_SUMIF, G_NAIVE_BWD>(const GatherArgs<float> &, hipStream_t);
}
