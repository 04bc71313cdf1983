// Streaming decision step: the instantiations for hidden 128, bf16 weights (see act_stream_kernel.h).
#include "act_stream_kernel.h"

namespace marl {

hipError_t launch_act_stream_h128(const ActStreamArgs &a, int groups, hipStream_t stream) { return stream_launch<128, 1>(a, groups, stream); }

}  // namespace marl
