// Instantiations of the fast kernel for the 128 x 128 x 64 tile.
#include "gemm_fast.h"

namespace nt {
nt_status launch_fast_128x128(const FastArgs &a, bool bf16, bool edge, int alay, int blay, int64_t nwg, hipStream_t s)
{
    return launch_fast_t<128, 128>(a, bf16, edge, alay, blay, nwg, s);
}
}  // namespace nt
