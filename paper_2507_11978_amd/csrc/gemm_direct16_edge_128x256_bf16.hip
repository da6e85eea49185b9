// Instantiations of the range-checked flavour of the direct-to-LDS kernel on 16 x 16 x 32 matrix instructions, 128 x 256 x 64 tile, bf16 inputs.
#include "gemm_direct16.h"

namespace nt {
nt_status launch_direct16_edge_128x256_bf16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s)
{
    return launch_direct16_t<128, 256, true, true>(a, alay, blay, nwg, s);
}
}  // namespace nt
