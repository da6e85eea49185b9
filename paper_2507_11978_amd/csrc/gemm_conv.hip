// Instantiations of the implicit-GEMM convolution kernel.
#include "gemm_conv.h"

namespace nt {

// k split, second step: Y[n, f, x] = sum_i ws[i][n][f][x] in slice order (the same order on every run: the result is reproducible)
__global__ __launch_bounds__(256) void conv_ws_sum_kernel(const float *ws, int ksplit, int64_t slice, void *Y, int64_t fpq, int64_t pq,
                                                          int64_t syn, int64_t syf, int out_dtype)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < slice; i += (int64_t)gridDim.x * 256) {
        float sum = ws[i];
        for (int j = 1; j < ksplit; ++j) sum += ws[j * slice + i];
        const int64_t n = i / fpq, r = i - n * fpq, f = r / pq, x = r - f * pq;
        store_out(Y, n * syn + f * syf + x, sum, out_dtype);
    }
}

nt_status launch_conv_ws_sum(const float *ws, int ksplit, int64_t slice, void *Y, int64_t fpq, int64_t pq, int64_t syn, int64_t syf, int out_dtype, hipStream_t s)
{
    const int64_t blocks = std::min<int64_t>((slice + 255) / 256, 4096);
    hipLaunchKernelGGL(conv_ws_sum_kernel, dim3((unsigned)blocks), dim3(256), 0, s, ws, ksplit, slice, Y, fpq, pq, syn, syf, out_dtype);
    return check_launch("conv_ws_sum_kernel");
}

nt_status launch_conv(const ConvArgs &a, int bn, bool bf16, bool edge_b, int64_t nwg, hipStream_t s)
{
#define NT_CONV(BN, BF, E) launch_conv_inst<BN, BF, E>(a, nwg, s)
    if (bn == 256) {
        if (bf16) return edge_b ? NT_CONV(256, true, true) : NT_CONV(256, true, false);
        return edge_b ? NT_CONV(256, false, true) : NT_CONV(256, false, false);
    }
    if (bn == 128) {
        if (bf16) return edge_b ? NT_CONV(128, true, true) : NT_CONV(128, true, false);
        return edge_b ? NT_CONV(128, false, true) : NT_CONV(128, false, false);
    }
#undef NT_CONV
    return fail(NT_ERR_UNSUPPORTED, "no convolution kernel for this tile");
}

}  // namespace nt
