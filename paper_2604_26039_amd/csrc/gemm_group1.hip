// Instantiates one group of the tile family; see config_list.h and moe_gemm.h.
#include "config_list.h"
#include "moe_gemm.h"

namespace ramp {
void register_group1(KernelInfo *out, int *n)
{
#define X(BM, BN, BK, WM, WN, NS, LOOP) out[(*n)++] = make_info<BM, BN, BK, WM, WN, NS, LOOP>();
    RAMP_CONFIG_GROUP1(X)
#undef X
}
}  // namespace ramp
