// HIP kernels for gfx950 (CDNA4): the tiled contraction that the matmul arrangement
// describes (Section 4.2).  One workgroup = one program = one (BM x BN) output tile
// (tile-to-program mapping, Section 3.2.1); per k tile it stages the (BM x BK) block of A
// and the (BK x BN) block of B in LDS (source-to-target mapping, Section 3.2.2, masked
// elements read as zero), multiplies them on the matrix cores with an fp32 accumulator and
// finally stores the converted accumulator through C's map.
//
// LDS layout (both operands): [row][BK] 16-bit elements with k contiguous, where "row" is
// the m index for A and the n index for B, i.e. B is transposed on its way into LDS so that
// both MFMA operands are read as 8 consecutive k values (one ds_read_b128) per lane.  The
// 16-byte chunk index of a row is XOR-swizzled with the row number so that the reads of 16
// consecutive rows, and the writes of both loaders, fall in distinct banks.
//
// Two kernels share the LDS->MFMA core:
//   gemm_generic_kernel  any operand map (arbitrary strides, implicit-GEMM convolution),
//                        element-wise gathers through the lowered operand map;
//   gemm_fast_kernel     unit-stride operands (either orientation), 16-byte global loads,
//                        register-staged prefetch of the next k tile, double-buffered LDS.
#pragma once
#include <atomic>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <string>

#include "kernels.h"

namespace nt {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bhalf8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;       // 4 wavefronts, arranged 2 x 2 over the output tile

// ------------------------------------------------------------------ small helpers
template <bool BF16>
__device__ __forceinline__ float16v mfma32(u32x4 a, u32x4 b, float16v c)
{
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bhalf8, a), __builtin_bit_cast(bhalf8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    return __builtin_bit_cast(uint16_t, (__bf16)f);          // v_cvt_pk_bf16_f32: round to nearest even, NaN stays NaN
}

__device__ __forceinline__ uint16_t f32_to_f16_rne(float f)
{
    _Float16 h = (_Float16)f;                    // v_cvt_f16_f32: round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ void store_out(void *C, int64_t off, float v, int out_dtype)
{
    if (out_dtype == NT_F32)
        reinterpret_cast<float *>(C)[off] = v;
    else if (out_dtype == NT_F16)
        reinterpret_cast<uint16_t *>(C)[off] = f32_to_f16_rne(v);
    else
        reinterpret_cast<uint16_t *>(C)[off] = f32_to_bf16_rne(v);
}

// element `off` of a tensor of type `dtype`, as fp32
__device__ __forceinline__ float load_as_f32(const void *D, int64_t off, int dtype)
{
    if (dtype == NT_F32) return reinterpret_cast<const float *>(D)[off];
    const uint16_t h = reinterpret_cast<const uint16_t *>(D)[off];
    if (dtype == NT_F16) return (float)__builtin_bit_cast(_Float16, h);
    return __builtin_bit_cast(float, (uint32_t)h << 16);
}

// the addmm combination, in fp32: alpha * accumulator + beta * addend
__device__ __forceinline__ float combine(float acc, float d, float alpha, float beta) { return __builtin_fmaf(alpha, acc, beta * d); }

// Activation applied to the combined value before the single conversion to the output type (codes:
// nt_activation).  One branch-free formula serves all of them, so that the fully unrolled epilogues
// carry a single short instruction sequence per element:
//   t = max(x, lo);  y = t * (g1 + g0 / (1 + 2^(-t (c1 + c3 t^2))))
//   relu       lo = 0,     g1 = 1, g0 = 0                     -> max(x, 0) exactly
//   silu       lo = -inf,  g1 = 0, g0 = 1, c1 = log2(e)       -> x sigmoid(x)
//   gelu_tanh  lo = -inf,  g1 = 0, g0 = 1, c1 = 2 sqrt(2/pi) log2(e), c3 = 0.044715 c1
//              (0.5 (1 + tanh u) is the logistic function of 2u)
// The gate's argument is built from t clamped to +-1e15, where the gate has long saturated, so that
// t^2 cannot overflow into 0 * inf.
struct ActParams {
    float lo, c1, c3, g0, g1;
};

__device__ __forceinline__ ActParams act_params(int act)
{
    ActParams p;
    p.lo = act == 1 ? 0.f : -INFINITY;
    p.g1 = act == 1 ? 1.f : 0.f;
    p.g0 = act == 1 ? 0.f : 1.f;
    p.c1 = act == 2 ? 1.4426950408889634f : (act == 3 ? 2.302208198f : 0.f);      // 2 * 0.7978845608 * 1.4426950409
    p.c3 = act == 3 ? 0.102943240f : 0.f;                                         // 0.044715 * 2.302208198
    return p;
}

__device__ __forceinline__ float activate(float x, const ActParams &p)
{
    const float t = fmaxf(x, p.lo);
    const float tc = __builtin_amdgcn_fmed3f(t, -1e15f, 1e15f);
    const float z = tc * __builtin_fmaf(p.c3, tc * tc, p.c1);
    const float gate = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-z));
    return t * __builtin_fmaf(p.g0, gate, p.g1);
}

// Swizzled LDS position (in 16-bit elements) of 16-byte chunk `chunk` of row `row`.
template <int BK>
__device__ __forceinline__ int lds_chunk_pos(int row, int chunk)
{
    constexpr int CPR = BK / 8;                  // chunks per row
    constexpr int RPL = 8 / CPR > 0 ? 8 / CPR : 1;   // rows per 128-byte line
    const int s = ((row / RPL) ^ (row >> 3)) & (CPR - 1);
    return row * BK + ((chunk ^ s) << 3);
}

// hardware workgroup index -> (batch, tile row, tile col).  The divisions run on the vector
// unit; the results (below 2^31, checked at launch) are moved to scalar registers so that
// everything derived from them is wavefront-uniform for the compiler as well.
__device__ __forceinline__ void locate_program(int64_t mt, int64_t nt, int64_t *b, int64_t *i, int64_t *j)
{
    const uint32_t m32 = (uint32_t)mt, n32 = (uint32_t)nt;
    uint32_t bb, pid;
    program_of_workgroup_batched_t<uint32_t>(blockIdx.x, gridDim.x / (m32 * n32), m32, n32, &bb, &pid);
    const uint32_t ii = pid / n32;
    *b = __builtin_amdgcn_readfirstlane((int)bb);
    *i = __builtin_amdgcn_readfirstlane((int)ii);
    *j = __builtin_amdgcn_readfirstlane((int)(pid - ii * n32));
}

// The LDS -> MFMA core for one staged k tile: acc[tm][tn] += A_tile . B_tile.
template <int BM, int BN, int BK, bool BF16>
__device__ __forceinline__ void mma_tile(const uint16_t *__restrict__ as, const uint16_t *__restrict__ bs,
                                         float16v (&acc)[BM / 64][BN / 64], int wave_m, int wave_n, int lane)
{
    constexpr int TM = BM / 64, TN = BN / 64;
    const int l32 = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
        u32x4 af[TM], bf[TN];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int row = wave_m * (BM / 2) + tm * 32 + l32;
            af[tm] = *reinterpret_cast<const u32x4 *>(as + lds_chunk_pos<BK>(row, ks * 2 + hi));
        }
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int row = wave_n * (BN / 2) + tn * 32 + l32;
            bf[tn] = *reinterpret_cast<const u32x4 *>(bs + lds_chunk_pos<BK>(row, ks * 2 + hi));
        }
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                acc[tm][tn] = mfma32<BF16>(af[tm], bf[tn], acc[tm][tn]);
    }
}

// The parts of a tile's rows and columns under one operand map, kept in LDS (one entry per row / column).
template <int BM, int BN>
struct TileParts {
    int64_t row_off[BM], col_off[BN];
    int32_t row_chk[BM][kMaxChecks], col_chk[BN][kMaxChecks];

    __device__ __forceinline__ void fill(const OperandMap &m, int64_t row0, int64_t col0, int tid)
    {
        for (int r = tid; r < BM; r += kThreads) {
            const AxisPart p = row_part(m, row0 + r);
            row_off[r] = p.off;
            for (int q = 0; q < kMaxChecks; ++q) row_chk[r][q] = p.chk[q];
        }
        for (int n = tid; n < BN; n += kThreads) {
            const AxisPart p = col_part(m, col0 + n);
            col_off[n] = p.off;
            for (int q = 0; q < kMaxChecks; ++q) col_chk[n][q] = p.chk[q];
        }
    }
    __device__ __forceinline__ AxisPart row(int r) const
    {
        AxisPart p;
        p.off = row_off[r];
        for (int q = 0; q < kMaxChecks; ++q) p.chk[q] = row_chk[r][q];
        return p;
    }
    __device__ __forceinline__ AxisPart col(int n) const
    {
        AxisPart p;
        p.off = col_off[n];
        for (int q = 0; q < kMaxChecks; ++q) p.chk[q] = col_chk[n][q];
        return p;
    }
};

// Store act(alpha * accumulators + beta * D) (D read through its operand map, if given) through C's operand
// map (masked: out-of-range elements dropped).  pc / pd: the parts of the tile's rows and columns under
// C's and D's maps, filled beforehand, so that the unrolled element code does no index decomposition.
template <int BM, int BN>
__device__ __forceinline__ void store_tile_generic(void *C, const OperandMap &mc, int64_t c_batch_off,
                                                   float16v (&acc)[BM / 64][BN / 64], int64_t row0, int64_t col0,
                                                   int wave_m, int wave_n, int lane, int out_dtype,
                                                   const void *D, const OperandMap &md, int64_t d_batch_off, float alpha, float beta, int act,
                                                   const TileParts<BM, BN> &pc, const TileParts<BM, BN> &pd)
{
    constexpr int TM = BM / 64, TN = BN / 64;
    const int l32 = lane & 31, hi = lane >> 5;
    const ActParams ap = act_params(act);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int cl = wave_n * (BN / 2) + tn * 32 + l32;
        const int64_t col = col0 + cl;
        const AxisPart cp = pc.col(cl);
        AxisPart dcp = cp;
        if (D) dcp = pd.col(cl);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rl = wave_m * (BM / 2) + tm * 32 + 8 * (v / 4) + 4 * hi + (v % 4);
                const int64_t row = row0 + rl;
                int64_t off;
                if (element_at(mc, row, col, pc.row(rl), cp, &off)) {
                    float x = acc[tm][tn][v];
                    if (D) {
                        int64_t doff;
                        const bool in = element_at(md, row, col, pd.row(rl), dcp, &doff);
                        x = combine(x, in ? load_as_f32(D, d_batch_off + doff, out_dtype) : 0.f, alpha, beta);
                    } else {
                        x *= alpha;
                    }
                    store_out(C, c_batch_off + off, act ? activate(x, ap) : x, out_dtype);
                }
            }
        }
    }
}

// One (E x BK) operand block of the operand-map kernel into its k-contiguous LDS image `dst`.
// e_* : parts of the block's E rows (m for A, n for B), k_* : parts of its BK k indices, both in LDS.
// `e_is_row`: the operand's logical matrix is indexed (e, k) (A) or (k, e) (B).
// Lanes run along whichever axis has the smaller memory stride, so that a wavefront's element loads
// fall into few cache lines: along e (each thread keeps one row, gathers 8 consecutive k and writes
// them with one 16-byte LDS store) or along k (2-byte LDS stores to consecutive addresses).
template <int E, int BK>
__device__ __forceinline__ void stage_mapped(const uint16_t *__restrict__ src, const OperandMap &m, bool e_is_row, bool lanes_along_e,
                                             int64_t e0, int64_t k0, const int64_t *e_off, const int32_t (*e_chk)[kMaxChecks],
                                             const int64_t *k_off, const int32_t (*k_chk)[kMaxChecks], uint16_t *dst, int tid)
{
    auto element = [&](int e, int k, const AxisPart &ep, const AxisPart &kp) -> uint16_t {
        int64_t off;
        const bool ok = e_is_row ? element_at(m, e0 + e, k0 + k, ep, kp, &off) : element_at(m, k0 + k, e0 + e, kp, ep, &off);
        return ok ? src[off] : (uint16_t)0;
    };
    auto part_of = [&](const int64_t *off, const int32_t (*chk)[kMaxChecks], int i) {
        AxisPart p;
        p.off = off[i];
        for (int q = 0; q < kMaxChecks; ++q) p.chk[q] = chk[i][q];
        return p;
    };
    if (lanes_along_e) {
        constexpr int GROUPS = kThreads / E > 0 ? kThreads / E : 1;      // threads per row
        const int e = tid % E;
        const AxisPart ep = part_of(e_off, e_chk, e);
        for (int c8 = (tid / E) * 8; c8 < BK; c8 += GROUPS * 8) {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t lo = element(e, c8 + 2 * j, ep, part_of(k_off, k_chk, c8 + 2 * j));
                const uint32_t hi = element(e, c8 + 2 * j + 1, ep, part_of(k_off, k_chk, c8 + 2 * j + 1));
                w[j] = lo | (hi << 16);
            }
            *reinterpret_cast<u32x4 *>(dst + lds_chunk_pos<BK>(e, c8 >> 3)) = u32x4{w[0], w[1], w[2], w[3]};
        }
    } else {
        constexpr int STEP = kThreads / BK, TRIPS = E / STEP;                // rows per pass, passes
        constexpr int BATCH = TRIPS % 16 == 0 ? 16 : (TRIPS % 8 == 0 ? 8 : (TRIPS % 4 == 0 ? 4 : 1));   // loads in flight per thread
        const int c = tid % BK;
        const AxisPart kp = part_of(k_off, k_chk, c);
        for (int t = 0; t < TRIPS; t += BATCH) {
            uint16_t v[BATCH];
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int e = tid / BK + (t + u) * STEP;
                v[u] = element(e, c, part_of(e_off, e_chk, e), kp);
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int e = tid / BK + (t + u) * STEP;
                dst[lds_chunk_pos<BK>(e, c >> 3) + (c & 7)] = v[u];
            }
        }
    }
}

// =========================================================================== generic kernel
template <int BM, int BN, int BK, bool BF16>
__global__ __launch_bounds__(kThreads) void gemm_generic_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, void *__restrict__ C,
    const OperandMap ma, const OperandMap mb, const OperandMap mc,
    int64_t sa_batch, int64_t sb_batch, int64_t sc_batch, int64_t mt, int64_t nt, int64_t kt, int out_dtype,
    const void *__restrict__ D, const OperandMap md, int64_t sd_batch, float alpha, float beta, int act)
{
    __shared__ __attribute__((aligned(16))) uint16_t as[BM * BK];
    __shared__ __attribute__((aligned(16))) uint16_t bs[BN * BK];
    // The mixed-radix decompositions (64-bit divisions) are done once per index, not once per element: the parts of
    // the tile's rows of A and columns of B once per program, those of a k tile's 2 BK k indices once per k tile.
    __shared__ int64_t a_row_off[BM], b_col_off[BN], a_k_off[BK], b_k_off[BK];
    __shared__ int32_t a_row_chk[BM][kMaxChecks], b_col_chk[BN][kMaxChecks], a_k_chk[BK][kMaxChecks], b_k_chk[BK][kMaxChecks];
    __shared__ TileParts<BM, BN> parts_c, parts_d;             // for the epilogue
    int64_t bi, ti, tj;
    locate_program(mt, nt, &bi, &ti, &tj);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int64_t row0 = ti * BM, col0 = tj * BN;
    const uint16_t *Ab = A + bi * sa_batch;
    const uint16_t *Bb = B + bi * sb_batch;

    float16v acc[BM / 64][BN / 64];
#pragma unroll
    for (int a = 0; a < BM / 64; ++a)
#pragma unroll
        for (int b = 0; b < BN / 64; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // lanes run along the axis with the smaller memory stride (the innermost digit's)
    auto mag = [](int64_t v) { return v < 0 ? -v : v; };
    const bool a_lanes_rows = mag(ma.roff[ma.nrd - 1]) < mag(ma.coff[ma.ncd - 1]);
    const bool b_lanes_cols = mag(mb.coff[mb.ncd - 1]) <= mag(mb.roff[mb.nrd - 1]);
    for (int r = tid; r < BM; r += kThreads) {
        const AxisPart p = row_part(ma, row0 + r);
        a_row_off[r] = p.off;
        for (int q = 0; q < kMaxChecks; ++q) a_row_chk[r][q] = p.chk[q];
    }
    for (int n = tid; n < BN; n += kThreads) {
        const AxisPart p = col_part(mb, col0 + n);
        b_col_off[n] = p.off;
        for (int q = 0; q < kMaxChecks; ++q) b_col_chk[n][q] = p.chk[q];
    }

    for (int64_t k = 0; k < kt; ++k) {
        const int64_t k0 = k * BK;
        if (tid < BK) {
            const AxisPart p = col_part(ma, k0 + tid);
            a_k_off[tid] = p.off;
            for (int q = 0; q < kMaxChecks; ++q) a_k_chk[tid][q] = p.chk[q];
        } else if (tid < 2 * BK) {
            const AxisPart p = row_part(mb, k0 + tid - BK);
            b_k_off[tid - BK] = p.off;
            for (int q = 0; q < kMaxChecks; ++q) b_k_chk[tid - BK][q] = p.chk[q];
        }
        __syncthreads();
        // A tile: element (r, c) is A_view[row0 + r, k0 + c]; B tile: element (c, n) is B_view[k0 + c, col0 + n], stored transposed
        stage_mapped<BM, BK>(Ab, ma, true, a_lanes_rows, row0, k0, a_row_off, a_row_chk, a_k_off, a_k_chk, as, tid);
        stage_mapped<BN, BK>(Bb, mb, false, b_lanes_cols, col0, k0, b_col_off, b_col_chk, b_k_off, b_k_chk, bs, tid);
        __syncthreads();
        mma_tile<BM, BN, BK, BF16>(as, bs, acc, wave_m, wave_n, lane);
        __syncthreads();
    }
    parts_c.fill(mc, row0, col0, tid);
    if (D) parts_d.fill(md, row0, col0, tid);
    __syncthreads();
    store_tile_generic<BM, BN>(C, mc, bi * sc_batch, acc, row0, col0, wave_m, wave_n, lane, out_dtype, D, md, bi * sd_batch, alpha, beta, act,
                               parts_c, parts_d);
}

// ---- host-side helper shared by the translation units that instantiate the kernels
inline nt_status check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
    return NT_OK;
}

// "Done once on this device" flag for per-kernel set-up (hipFuncSetAttribute is a per-device setting); the work it
// guards is idempotent, so two threads that both find it unset merely do it twice.
struct DeviceOnce {
    std::atomic<bool> flag[64];
    DeviceOnce() { for (auto &f : flag) f.store(false); }
    static int device() { int d = 0; return hipGetDevice(&d) == hipSuccess && d >= 0 && d < 64 ? d : 0; }
    bool done() const { return flag[device()].load(std::memory_order_acquire); }
    void set() { flag[device()].store(true, std::memory_order_release); }
};

// Compute units of the current device (0 if the query fails), asked once per device.
inline int64_t compute_units()
{
    static std::atomic<int> count[64];
    const int d = DeviceOnce::device();
    int n = count[d].load(std::memory_order_acquire);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, d) != hipSuccess || n < 0) n = 0;
        count[d].store(n, std::memory_order_release);
    }
    return n;
}

nt_status launch_generic(const GemmLaunch &g);

}  // namespace nt
