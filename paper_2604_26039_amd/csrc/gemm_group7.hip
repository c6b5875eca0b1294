// Instantiates the ping-pong group of the tile family; see config_list.h and moe_pingpong.h.
#include "config_list.h"
#include "moe_pingpong.h"

namespace ramp {
void register_group7(KernelInfo *out, int *n)
{
#define X(BM, BN, BK, WM, WN, NS) out[(*n)++] = make_pingpong_info<BM, BN, BK, WM, WN, NS>();
    RAMP_CONFIG_GROUP7(X)
#undef X
}
}  // namespace ramp
