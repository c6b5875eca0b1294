// Instantiates one group of the weight-streaming family; see config_list.h and moe_stream.h.
#include "config_list.h"
#include "moe_stream.h"

namespace ramp {
void register_stream_group2(KernelInfo *out, int *n)
{
#define X(BM, FBW, WF, WK, U) out[(*n)++] = make_stream_info<BM, FBW, WF, WK, U>();
    RAMP_STREAM_GROUP2(X)
#undef X
}
}  // namespace ramp
