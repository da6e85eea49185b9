// Instantiations of the loader traces (one workgroup of the real kernels, stopped after one slice has landed in LDS).
#include "gemm_conv_direct.h"
#include "gemm_direct16.h"

namespace nt {

template <int BM, int BN, bool EDGE>
static nt_status trace_layouts(const FastArgs &a, int alay, int blay, hipStream_t s)
{
    if (alay == KCONTIG && blay == MNCONTIG) return launch_direct16_trace_inst<BM, BN, KCONTIG, MNCONTIG, EDGE>(a, s);
    if (alay == KCONTIG && blay == KCONTIG) return launch_direct16_trace_inst<BM, BN, KCONTIG, KCONTIG, EDGE>(a, s);
    if (alay == MNCONTIG && blay == MNCONTIG) return launch_direct16_trace_inst<BM, BN, MNCONTIG, MNCONTIG, EDGE>(a, s);
    return launch_direct16_trace_inst<BM, BN, MNCONTIG, KCONTIG, EDGE>(a, s);
}

template <bool EDGE>
static nt_status trace_tiles(const FastArgs &a, int bm, int bn, int alay, int blay, hipStream_t s)
{
    if (bm == 128 && bn == 128) return trace_layouts<128, 128, EDGE>(a, alay, blay, s);
    if (bm == 256 && bn == 128) return trace_layouts<256, 128, EDGE>(a, alay, blay, s);
    if (bm == 128 && bn == 256) return trace_layouts<128, 256, EDGE>(a, alay, blay, s);
    if (bm == 256 && bn == 256) return trace_layouts<256, 256, EDGE>(a, alay, blay, s);
    return fail(NT_ERR_UNSUPPORTED, "no direct kernel for this tile");
}

nt_status launch_direct16_trace(const FastArgs &a, int bm, int bn, int alay, int blay, bool edge, hipStream_t s)
{
    return edge ? trace_tiles<true>(a, bm, bn, alay, blay, s) : trace_tiles<false>(a, bm, bn, alay, blay, s);
}

nt_status launch_conv_direct_trace(const ConvArgs &a, int bn, hipStream_t s)
{
    if (bn == 256) return launch_conv_direct_inst<256, false, true>(a, 1, s);
    if (bn == 128) return launch_conv_direct_inst<128, false, true>(a, 1, s);
    if (bn == 64) return launch_conv_direct_inst<64, false, true>(a, 1, s);
    return fail(NT_ERR_UNSUPPORTED, "no convolution kernel for this tile");
}

}  // namespace nt
