// Instantiations of the fast kernel for the 256 x 256 x 64 tile.
#include "gemm_fast.h"

namespace nt {
nt_status launch_fast_256x256(const FastArgs &a, bool bf16, bool edge, int alay, int blay, int64_t nwg, hipStream_t s)
{
    return launch_fast_t<256, 256>(a, bf16, edge, alay, blay, nwg, s);
}
}  // namespace nt
