// Instantiations of the convolution kernel that walks the reduction tap by tap, and the filter's copy in that order.
#include "gemm_conv_tap.h"

namespace nt {

// filter [F][C][R * S] (row pitch ldb) -> [F][R * S][C] (row pitch K = C R S): one workgroup per filter, the row read and
// written with consecutive lanes on consecutive elements, permuted on its way through LDS
__global__ __launch_bounds__(256) void conv_repack_filter_kernel(const uint16_t *w, int64_t ldb, uint16_t *out, int32_t C, int32_t RS)
{
    extern __shared__ uint16_t row[];
    const int32_t K = C * RS;
    const uint16_t *src = w + (int64_t)blockIdx.x * ldb;
    uint16_t *dst = out + (int64_t)blockIdx.x * K;
    for (int32_t i = threadIdx.x; i < K; i += 256) row[i] = src[i];
    __syncthreads();
    for (int32_t j = threadIdx.x; j < K; j += 256) {
        const int32_t tap = j / C, c = j - tap * C;
        dst[j] = row[c * RS + tap];
    }
}

nt_status launch_conv_tap(const ConvArgs &a, int rows, bool bf16, int64_t nwg, hipStream_t s)
{
    if (rows == 256) return bf16 ? launch_conv_tap_inst<true, 8, 7>(a, nwg, s) : launch_conv_tap_inst<false, 8, 7>(a, nwg, s);
    if (rows == 224) return bf16 ? launch_conv_tap_inst<true, 7, 6>(a, nwg, s) : launch_conv_tap_inst<false, 7, 6>(a, nwg, s);
    return fail(NT_ERR_UNSUPPORTED, "no convolution kernel for this tile height");
}

nt_status launch_conv_tap_trace(const ConvArgs &a, int rows, hipStream_t s)
{
    if (rows == 256) return launch_conv_tap_inst<false, 8, 7, true>(a, 1, s);
    if (rows == 224) return launch_conv_tap_inst<false, 7, 6, true>(a, 1, s);
    return fail(NT_ERR_UNSUPPORTED, "no convolution kernel for this tile height");
}

nt_status launch_conv_repack_filter(const uint16_t *w, int64_t ldb, uint16_t *out, int32_t F, int32_t C, int32_t RS, hipStream_t s)
{
    // (the reduction is below 2^16 elements: a row fits LDS)
    hipLaunchKernelGGL(conv_repack_filter_kernel, dim3((unsigned)F), dim3(256), (size_t)C * RS * sizeof(uint16_t), s, w, ldb, out, C, RS);
    return check_launch("conv_repack_filter_kernel");
}

}  // namespace nt
