// Measurement aid: the matrix pipe alone.  Every wavefront (one per SIMD, as in the product kernels) keeps two sets of
// 4 + 8 operand fragments, read once from the caller's data, and issues v_mfma_f32_16x16x32 instructions on them back to
// back: no LDS, no memory traffic, no barrier.  On this power-managed part the rate such a loop sustains depends on the
// operand values (2.4 PFLOP/s on zeros, about 1.85 on the benchmark's N(0,1)/sqrt(K) fp16 data): it is the ceiling that
// a product kernel on the same instruction and data can approach, and the benchmark reports it beside the kernel's rate.
#include "gemm_direct16.h"

namespace nt {

template <bool BF16>
__global__ __launch_bounds__(kThreads, 1) void mfma_probe_kernel(const u32x4 *src, int64_t n_vec, int32_t iters, float *out)
{
    constexpr int TA = 4, TB = 8;
    u32x4 a[2][TA], b[2][TB];
    const int64_t at = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 37;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < TA; ++i) a[s][i] = src[(at + s * 16 + i) % n_vec];
#pragma unroll
        for (int i = 0; i < TB; ++i) b[s][i] = src[(at + s * 16 + 4 + i) % n_vec];
    }
    float4v acc[TA][TB];
#pragma unroll
    for (int i = 0; i < TA; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    for (int32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < TA; ++i)
#pragma unroll
                for (int j = 0; j < TB; ++j) mfma16<BF16>(acc[i][j], a[s][i], b[s][j]);
    }
    asm volatile("s_nop 15" ::: "memory");
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < TA; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j) {
            float4v blk = acc[i][j];
            asm volatile("" : "+a"(blk));
#pragma unroll
            for (int v = 0; v < 4; ++v) sum += blk[v];
        }
    out[(int64_t)blockIdx.x * kThreads + threadIdx.x] = sum;
}

nt_status launch_mfma_probe(const void *data, int64_t n_elems, int dtype, int32_t iters, int32_t blocks, float *out, void *stream)
{
    const int64_t n_vec = n_elems / 8;
    if (dtype == NT_BF16) hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, (const u32x4 *)data, n_vec, iters, out);
    else hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, (const u32x4 *)data, n_vec, iters, out);
    return check_launch("mfma_probe_kernel");
}

}  // namespace nt
