// Instantiations of the convolution kernel that streams its operands straight into LDS.
#include "gemm_conv_direct.h"

namespace nt {

nt_status launch_conv_direct(const ConvArgs &a, int bn, bool bf16, int64_t nwg, hipStream_t s)
{
    if (bn == 256) return bf16 ? launch_conv_direct_inst<256, true>(a, nwg, s) : launch_conv_direct_inst<256, false>(a, nwg, s);
    if (bn == 128) return bf16 ? launch_conv_direct_inst<128, true>(a, nwg, s) : launch_conv_direct_inst<128, false>(a, nwg, s);
    if (bn == 64) return bf16 ? launch_conv_direct_inst<64, true>(a, nwg, s) : launch_conv_direct_inst<64, false>(a, nwg, s);
    return fail(NT_ERR_UNSUPPORTED, "no convolution kernel for this tile");
}

}  // namespace nt
