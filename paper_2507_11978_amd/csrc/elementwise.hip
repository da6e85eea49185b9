// Memory-bound kernels of the paper's task list (Section 5.1): add, silu, softmax, rms_norm.
//
// Arrangements: add and silu tile every vector into blocks of BLOCK_SIZE (Section 4.1,
// `tile((BLOCK_SIZE,))`); the application is element-wise, so which program owns which block
// does not show in the result and the kernels split the vectors their own way: 16-byte vectors
// (8 elements), four in flight per thread and operand, one contiguous 16 KB chunk per workgroup.  softmax and rms_norm tile a
// matrix into rows (`tile((1, -1))`): one program per row; a row of up to 8192 elements is read
// once into the registers of one wavefront, reduced with cross-lane exchanges, and written once.
// Everything is computed in fp32 and converted once (round to nearest even) to the 16-bit format.
//
// All four are bound by HBM traffic: add moves 3 x 2 bytes per element, the others 2 x 2.
#include "gemm_device.h"

namespace nt {

constexpr int kVecPerThread = 4;

__device__ __forceinline__ float to_f32(uint16_t h, int dtype)
{
    if (dtype == NT_F16) return (float)__builtin_bit_cast(_Float16, h);
    return __builtin_bit_cast(float, (uint32_t)h << 16);
}

__device__ __forceinline__ uint16_t from_f32(float v, int dtype) { return dtype == NT_F16 ? f32_to_f16_rne(v) : f32_to_bf16_rne(v); }

template <bool BF16>
__device__ __forceinline__ void unpack8(u32x4 v, float (&f)[8])
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t w = v[q];
        if constexpr (BF16) {
            f[2 * q] = __builtin_bit_cast(float, w << 16);
            f[2 * q + 1] = __builtin_bit_cast(float, w & 0xffff0000u);
        } else {
            f[2 * q] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
            f[2 * q + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
        }
    }
}

template <bool BF16>
__device__ __forceinline__ u32x4 pack8(const float (&f)[8])
{
    u32x4 v;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t w;
        if constexpr (BF16) {
            w = (uint32_t)f32_to_bf16_rne(f[2 * q]) | ((uint32_t)f32_to_bf16_rne(f[2 * q + 1]) << 16);
        } else {
            typedef _Float16 half2v __attribute__((ext_vector_type(2)));
            w = __builtin_bit_cast(uint32_t, half2v{(_Float16)f[2 * q], (_Float16)f[2 * q + 1]});
        }
        v[q] = w;
    }
    return v;
}

// (v_rcp_f32 is accurate to 1 ulp of fp32: far below the 16-bit output's rounding)
__device__ __forceinline__ float silu_f32(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

// OP 0: out = x + y;  OP 1: out = silu(x).  Unit strides; n8 whole 8-element vectors, then a tail.
template <int OP, bool BF16>
__global__ __launch_bounds__(256) void map_vec_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ y,
                                                      uint16_t *__restrict__ out, int64_t n)
{
    const int64_t n8 = n / 8;
    // a workgroup takes one contiguous chunk of 256 * kVecPerThread vectors at a time (16 KB per operand): measured
    // 4 - 6 % faster than a thread's four vectors lying a whole grid apart (add 14.7 against 15.6 us, silu 10.5 against
    // 11.0 us on 16.7 M elements), and than fewer workgroups walking several chunks each
    for (int64_t c = blockIdx.x; c * (256 * kVecPerThread) < n8; c += gridDim.x) {
        const int64_t v0 = c * (256 * kVecPerThread) + threadIdx.x;
        u32x4 a[kVecPerThread], b[kVecPerThread];
#pragma unroll
        for (int u = 0; u < kVecPerThread; ++u) {
            const int64_t v = v0 + u * 256;
            if (v < n8) {
                __builtin_memcpy(&a[u], x + v * 8, 16);
                if constexpr (OP == 0) __builtin_memcpy(&b[u], y + v * 8, 16);
            }
        }
#pragma unroll
        for (int u = 0; u < kVecPerThread; ++u) {
            const int64_t v = v0 + u * 256;
            if (v < n8) {
                float fa[8], fb[8];
                unpack8<BF16>(a[u], fa);
                if constexpr (OP == 0) unpack8<BF16>(b[u], fb);
#pragma unroll
                for (int e = 0; e < 8; ++e) fa[e] = OP == 0 ? fa[e] + fb[e] : silu_f32(fa[e]);
                const u32x4 r = pack8<BF16>(fa);
                // (the result is streamed past L2 where that pays -- one operand: 12.3 -> 7.9 us on 16.7 M elements; with two
                // operands it costs 2 %, and streaming the loads costs 15 - 20 % in either case)
                if constexpr (OP == 0) __builtin_memcpy(out + v * 8, &r, 16);
                else __builtin_nontemporal_store(r, reinterpret_cast<u32x4 *>(out + v * 8));
            }
        }
    }
    // tail: fewer than 8 elements
    const int64_t t = n8 * 8 + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t < n) {
        const int dt = BF16 ? NT_BF16 : NT_F16;
        const float a = to_f32(x[t], dt);
        out[t] = from_f32(OP == 0 ? a + to_f32(y[t], dt) : silu_f32(a), dt);
    }
}

// the same for any strides (elements)
template <int OP>
__global__ __launch_bounds__(256) void map_strided_kernel(const uint16_t *__restrict__ x, int64_t sx, const uint16_t *__restrict__ y, int64_t sy,
                                                          uint16_t *__restrict__ out, int64_t so, int64_t n, int dtype)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const float a = to_f32(x[i * sx], dtype);
        out[i * so] = from_f32(OP == 0 ? a + to_f32(y[i * sy], dtype) : silu_f32(a), dtype);
    }
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// OP 0: softmax;  OP 1: rms_norm.  One wavefront per row; the row (cols a multiple of 8, at most
// 512 * NV, unit column stride) sits in registers as NV 8-element vectors per lane.
template <int OP, int NV, bool BF16>
__global__ __launch_bounds__(256) void row_wave_kernel(const uint16_t *__restrict__ x, int64_t sxr, uint16_t *__restrict__ out, int64_t sor,
                                                       int64_t rows, int64_t cols, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;                                  // (no barrier follows)
    const int64_t nvec = cols / 8;
    const uint16_t *xr = x + row * sxr;
    float f[NV][8];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int64_t idx = (int64_t)v * 64 + lane;
        u32x4 raw{0, 0, 0, 0};
        if (idx < nvec) __builtin_memcpy(&raw, xr + idx * 8, 16);
        unpack8<BF16>(raw, f[v]);
        if (OP == 0 && idx >= nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[v][e] = -INFINITY;
        }
    }
    float scale;
    if constexpr (OP == 0) {
        float m = -INFINITY;
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int e = 0; e < 8; ++e) m = fmaxf(m, f[v][e]);
        m = wave_max(m);
        float s = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                f[v][e] = __expf(f[v][e] - m);
                s += f[v][e];
            }
        scale = 1.0f / wave_sum(s);
    } else {
        float s = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int e = 0; e < 8; ++e) s = __builtin_fmaf(f[v][e], f[v][e], s);
        scale = 1.0f / sqrtf(wave_sum(s) / (float)cols + eps);
    }
    uint16_t *orow = out + row * sor;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int64_t idx = (int64_t)v * 64 + lane;
        if (idx < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[v][e] *= scale;
            const u32x4 r = pack8<BF16>(f[v]);
            __builtin_nontemporal_store(r, reinterpret_cast<u32x4 *>(orow + idx * 8));       // (streamed: softmax 12.4 -> 10.3 us, rms_norm 11.3 -> 8.4 us at 4096 x 4096)
        }
    }
}

// Any row length and strides: one workgroup per row, the row is read once per pass.
template <int OP>
__global__ __launch_bounds__(256) void row_block_kernel(const uint16_t *__restrict__ x, int64_t sxr, int64_t sxc, uint16_t *__restrict__ out,
                                                        int64_t sor, int64_t soc, int64_t cols, float eps, int dtype)
{
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint16_t *xr = x + (int64_t)blockIdx.x * sxr;
    uint16_t *orow = out + (int64_t)blockIdx.x * sor;
    auto block_reduce = [&](float v, bool is_max) {
        v = is_max ? wave_max(v) : wave_sum(v);
        __syncthreads();                                      // red[] of the previous reduction has been read
        if (lane == 0) red[wave] = v;
        __syncthreads();
        return is_max ? fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) : (red[0] + red[1]) + (red[2] + red[3]);
    };
    float scale, m = 0.f;
    if constexpr (OP == 0) {
        float mx = -INFINITY;
        for (int64_t c = tid; c < cols; c += 256) mx = fmaxf(mx, to_f32(xr[c * sxc], dtype));
        m = block_reduce(mx, true);
        float s = 0.f;
        for (int64_t c = tid; c < cols; c += 256) s += __expf(to_f32(xr[c * sxc], dtype) - m);
        scale = 1.0f / block_reduce(s, false);
    } else {
        float s = 0.f;
        for (int64_t c = tid; c < cols; c += 256) {
            const float v = to_f32(xr[c * sxc], dtype);
            s = __builtin_fmaf(v, v, s);
        }
        scale = 1.0f / sqrtf(block_reduce(s, false) / (float)cols + eps);
    }
    for (int64_t c = tid; c < cols; c += 256) {
        const float v = to_f32(xr[c * sxc], dtype);
        orow[c * soc] = from_f32((OP == 0 ? __expf(v - m) : v) * scale, dtype);
    }
}

// ------------------------------------------------------------------ host launchers
nt_status launch_map(int op, const void *x, int64_t sx, const void *y, int64_t sy, void *out, int64_t so, int64_t n, int dtype, void *stream)
{
    if (n <= 0) return NT_OK;
    hipStream_t s = (hipStream_t)stream;
    const uint16_t *X = (const uint16_t *)x, *Y = (const uint16_t *)y;
    uint16_t *O = (uint16_t *)out;
    const bool bf16 = dtype == NT_BF16;
    if (sx == 1 && so == 1 && (op == 1 || sy == 1)) {
        const int64_t per_wg = 256 * kVecPerThread;
        const int64_t wgs = std::max<int64_t>(1, std::min<int64_t>((n / 8 + per_wg - 1) / per_wg, 1 << 20));   // one chunk per workgroup
        dim3 grid((unsigned)wgs), block(256);
        if (op == 0) {
            if (bf16) hipLaunchKernelGGL((map_vec_kernel<0, true>), grid, block, 0, s, X, Y, O, n);
            else hipLaunchKernelGGL((map_vec_kernel<0, false>), grid, block, 0, s, X, Y, O, n);
        } else {
            if (bf16) hipLaunchKernelGGL((map_vec_kernel<1, true>), grid, block, 0, s, X, Y, O, n);
            else hipLaunchKernelGGL((map_vec_kernel<1, false>), grid, block, 0, s, X, Y, O, n);
        }
        return check_launch("map_vec_kernel");
    }
    const int64_t wgs = std::max<int64_t>(1, std::min<int64_t>((n + 255) / 256, 256 * 16));
    if (op == 0) hipLaunchKernelGGL((map_strided_kernel<0>), dim3((unsigned)wgs), dim3(256), 0, s, X, sx, Y, sy, O, so, n, dtype);
    else hipLaunchKernelGGL((map_strided_kernel<1>), dim3((unsigned)wgs), dim3(256), 0, s, X, sx, Y, sy, O, so, n, dtype);
    return check_launch("map_strided_kernel");
}

template <int OP, int NV>
static void launch_row_wave(const uint16_t *x, int64_t sxr, uint16_t *out, int64_t sor, int64_t rows, int64_t cols, float eps, bool bf16, hipStream_t s)
{
    dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    if (bf16) hipLaunchKernelGGL((row_wave_kernel<OP, NV, true>), grid, block, 0, s, x, sxr, out, sor, rows, cols, eps);
    else hipLaunchKernelGGL((row_wave_kernel<OP, NV, false>), grid, block, 0, s, x, sxr, out, sor, rows, cols, eps);
}

template <int OP>
static nt_status launch_rows_t(const void *x, int64_t sxr, int64_t sxc, void *out, int64_t sor, int64_t soc, int64_t rows, int64_t cols,
                               float eps, int dtype, hipStream_t s)
{
    const uint16_t *X = (const uint16_t *)x;
    uint16_t *O = (uint16_t *)out;
    const bool bf16 = dtype == NT_BF16;
    if (sxc == 1 && soc == 1 && cols % 8 == 0 && cols <= 8192 && rows < (1LL << 33)) {
        if (cols <= 512) launch_row_wave<OP, 1>(X, sxr, O, sor, rows, cols, eps, bf16, s);
        else if (cols <= 1024) launch_row_wave<OP, 2>(X, sxr, O, sor, rows, cols, eps, bf16, s);
        else if (cols <= 2048) launch_row_wave<OP, 4>(X, sxr, O, sor, rows, cols, eps, bf16, s);
        else if (cols <= 4096) launch_row_wave<OP, 8>(X, sxr, O, sor, rows, cols, eps, bf16, s);
        else launch_row_wave<OP, 16>(X, sxr, O, sor, rows, cols, eps, bf16, s);
        return check_launch("row_wave_kernel");
    }
    if (rows > 0x7fffffffLL) return fail(NT_ERR_UNSUPPORTED, "too many rows");
    hipLaunchKernelGGL((row_block_kernel<OP>), dim3((unsigned)rows), dim3(256), 0, s, X, sxr, sxc, O, sor, soc, cols, eps, dtype);
    return check_launch("row_block_kernel");
}

nt_status launch_rows(int op, const void *x, int64_t sxr, int64_t sxc, void *out, int64_t sor, int64_t soc, int64_t rows, int64_t cols,
                      float eps, int dtype, void *stream)
{
    if (rows <= 0 || cols <= 0) return NT_OK;
    return op == 0 ? launch_rows_t<0>(x, sxr, sxc, out, sor, soc, rows, cols, eps, dtype, (hipStream_t)stream)
                   : launch_rows_t<1>(x, sxr, sxc, out, sor, soc, rows, cols, eps, dtype, (hipStream_t)stream);
}

}  // namespace nt
