// Instantiations of the direct kernel for the 256 x 128 x 64 tile.
#include "gemm_direct.h"

namespace nt {
nt_status launch_direct_256x128(const FastArgs &a, bool bf16, int alay, int blay, int64_t nwg, hipStream_t s)
{
    return launch_direct_t<256, 128>(a, bf16, alay, blay, nwg, s);
}
}  // namespace nt
