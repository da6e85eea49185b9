// Instantiations of the convolution kernel that walks the reduction tap by tap, and the filter's copy in that order.
#include "gemm_conv_tap.h"

namespace nt {

// filter [F][C][R * S] (row pitch ldb) -> [F][R * S][C] (row pitch K = C R S)
__global__ __launch_bounds__(256) void conv_repack_filter_kernel(const uint16_t *w, int64_t ldb, uint16_t *out, int32_t F, int32_t C, int32_t RS)
{
    const int64_t K = (int64_t)C * RS, total = (int64_t)F * K;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t f = i / K;
        const int32_t kk = (int32_t)(i - f * K), tap = kk / C, c = kk - tap * C;
        out[i] = w[f * ldb + (int64_t)c * RS + tap];
    }
}

nt_status launch_conv_tap(const ConvArgs &a, int rows, bool bf16, int64_t nwg, hipStream_t s)
{
    if (rows == 256) return bf16 ? launch_conv_tap_inst<true, 8>(a, nwg, s) : launch_conv_tap_inst<false, 8>(a, nwg, s);
    if (rows == 224) return bf16 ? launch_conv_tap_inst<true, 7>(a, nwg, s) : launch_conv_tap_inst<false, 7>(a, nwg, s);
    return fail(NT_ERR_UNSUPPORTED, "no convolution kernel for this tile height");
}

nt_status launch_conv_tap_trace(const ConvArgs &a, int rows, hipStream_t s)
{
    if (rows == 256) return launch_conv_tap_inst<false, 8, true>(a, 1, s);
    if (rows == 224) return launch_conv_tap_inst<false, 7, true>(a, 1, s);
    return fail(NT_ERR_UNSUPPORTED, "no convolution kernel for this tile height");
}

nt_status launch_conv_repack_filter(const uint16_t *w, int64_t ldb, uint16_t *out, int32_t F, int32_t C, int32_t RS, hipStream_t s)
{
    const int64_t total = (int64_t)F * C * RS;
    const int64_t blocks = std::min<int64_t>((total + 255) / 256, 2048);
    hipLaunchKernelGGL(conv_repack_filter_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w, ldb, out, F, C, RS);
    return check_launch("conv_repack_filter_kernel");
}

}  // namespace nt
