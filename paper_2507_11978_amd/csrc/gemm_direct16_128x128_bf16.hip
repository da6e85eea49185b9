// Instantiations of the direct-to-LDS kernel on 16 x 16 x 32 matrix instructions for the 128 x 128 x 64 tile, bf16 inputs.
#include "gemm_direct16.h"

namespace nt {
nt_status launch_direct16_128x128_bf16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s)
{
    return launch_direct16_t<128, 128, true>(a, alay, blay, nwg, s);
}
}  // namespace nt
