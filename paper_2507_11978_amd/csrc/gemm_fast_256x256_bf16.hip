// Instantiations of the staged (register-staged, masked) kernel for the 256 x 256 x 64 tile, bf16 inputs.
#include "gemm_fast.h"

namespace nt {
nt_status launch_fast_256x256_bf16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s)
{
    return launch_fast_t<256, 256, true>(a, alay, blay, nwg, s);
}
}  // namespace nt
