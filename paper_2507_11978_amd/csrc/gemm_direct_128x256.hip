// Instantiations of the direct kernel for the 128 x 256 x 64 tile.
#include "gemm_direct.h"

namespace nt {
nt_status launch_direct_128x256(const FastArgs &a, bool bf16, int alay, int blay, int64_t nwg, hipStream_t s)
{
    return launch_direct_t<128, 256>(a, bf16, alay, blay, nwg, s);
}
}  // namespace nt
