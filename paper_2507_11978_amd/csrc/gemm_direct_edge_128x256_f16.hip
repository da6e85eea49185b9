// Instantiations of the direct-to-LDS kernel for tiles that may overhang M or N, 128 x 256 x 64 tile, f16 inputs.
#include "gemm_direct.h"

namespace nt {
nt_status launch_direct_edge_128x256_f16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s)
{
    return launch_direct_t<128, 256, false, true>(a, alay, blay, nwg, s);
}
}  // namespace nt
