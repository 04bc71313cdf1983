// Streaming decision step: the instantiations for hidden 64, bf16 weights (see act_stream_kernel.h).
#include "act_stream_kernel.h"

namespace marl {

hipError_t launch_act_stream_h64_bf16(const ActStreamArgs &a, int groups, hipStream_t stream) { return stream_launch<64, 1>(a, groups, stream); }

}  // namespace marl
