// Instantiations of the direct-to-LDS kernel for the 128 x 256 x 64 tile, f16 inputs.
#include "gemm_direct.h"

namespace nt {
nt_status launch_direct_128x256_f16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s)
{
    return launch_direct_t<128, 256, false>(a, alay, blay, nwg, s);
}
}  // namespace nt
