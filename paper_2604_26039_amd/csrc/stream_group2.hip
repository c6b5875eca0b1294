// Instantiates one group of the weight-streaming family and its decode twins; see config_list.h, moe_stream.h, moe_decode.h.
#include "config_list.h"
#include "moe_decode.h"

namespace ramp {
template <int BM, int FBW, int WF, int WK, int U>
static KernelInfo make_decode_info()
{
    KernelInfo ki = make_stream_info<BM, FBW, WF, WK, U>();
    ki.cfg.mode |= kModeDecode;
    ki.launch_decode_up = &launch_decode_up<BM, FBW, WF, WK, U>;
    return ki;
}

void launch_decode_down_any(const DecodeDownArgs &d, hipStream_t stream) { launch_decode_down(d, stream); }

void register_stream_group2(KernelInfo *out, int *n)
{
#define X(BM, FBW, WF, WK, U) out[(*n)++] = make_stream_info<BM, FBW, WF, WK, U>();
    RAMP_STREAM_GROUP2(X)
#undef X
#define X(BM, FBW, WF, WK, U) out[(*n)++] = make_decode_info<BM, FBW, WF, WK, U>();
    RAMP_DECODE_GROUP(X)
#undef X
}
}  // namespace ramp
