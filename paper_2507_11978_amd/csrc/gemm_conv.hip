// Instantiations of the implicit-GEMM convolution kernel.
#include "gemm_conv.h"

namespace nt {

nt_status launch_conv(const ConvArgs &a, int bn, bool bf16, bool edge_b, int64_t nwg, hipStream_t s)
{
#define NT_CONV(BN, BF, E) launch_conv_inst<BN, BF, E>(a, nwg, s)
    if (bn == 256) {
        if (bf16) return edge_b ? NT_CONV(256, true, true) : NT_CONV(256, true, false);
        return edge_b ? NT_CONV(256, false, true) : NT_CONV(256, false, false);
    }
    if (bn == 128) {
        if (bf16) return edge_b ? NT_CONV(128, true, true) : NT_CONV(128, true, false);
        return edge_b ? NT_CONV(128, false, true) : NT_CONV(128, false, false);
    }
#undef NT_CONV
    return fail(NT_ERR_UNSUPPORTED, "no convolution kernel for this tile");
}

}  // namespace nt
