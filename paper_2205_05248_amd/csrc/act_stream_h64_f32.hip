// Streaming decision step: the instantiations for hidden 64, fp32 weights (two bf16 planes) (see act_stream_kernel.h).
#include "act_stream_kernel.h"

namespace marl {

hipError_t launch_act_stream_h64_f32(const ActStreamArgs &a, int groups, hipStream_t stream) { return stream_launch<64, 2>(a, groups, stream); }

}  // namespace marl
