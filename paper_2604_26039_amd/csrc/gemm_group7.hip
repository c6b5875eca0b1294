// Instantiates the ping-pong group of the tile family; see config_list.h and moe_pingpong.h.
#include "config_list.h"
#include "moe_pingpong.h"

namespace ramp {
void register_group7(KernelInfo *out, int *n)
{
#define X(BM, BN, BK, WM, WN, NS) out[(*n)++] = make_pingpong_info<BM, BN, BK, WM, WN, NS>();
    RAMP_CONFIG_GROUP7(X)
#undef X
    // GROUP_M variants (Sec. 4.1, Eq. 4) of the 256x256 tile: every XCD takes blocks of 4 x 8 or 8 x 4 tiles
    // (M x N) instead of a few M-tiles x all N-tiles; same kernels, different workgroup -> tile map
    out[(*n)++] = make_pingpong_info<256, 256, 32, 2, 4, 4>(2);
    out[(*n)++] = make_pingpong_info<256, 256, 32, 2, 4, 4>(3);
}
}  // namespace ramp
