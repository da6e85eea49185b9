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
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
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

// Swizzled LDS position (in 16-bit elements) of 16-byte chunk `chunk` of row `row`.
template <int BK>
__device__ __forceinline__ int lds_chunk_pos(int row, int chunk)
{
    constexpr int CPR = BK / 8;                  // chunks per row
    constexpr int RPL = 8 / CPR > 0 ? 8 / CPR : 1;   // rows per 128-byte line
    const int s = ((row / RPL) ^ (row >> 3)) & (CPR - 1);
    return row * BK + ((chunk ^ s) << 3);
}

// hardware workgroup index -> (batch, tile row, tile col)
__device__ __forceinline__ void locate_program(int64_t mt, int64_t nt, int64_t *b, int64_t *i, int64_t *j)
{
    const int64_t per = mt * nt;
    const int64_t w = blockIdx.x;
    *b = w / per;
    const int64_t pid = program_of_workgroup(w - *b * per, mt, nt);
    *i = pid / nt;
    *j = pid % nt;
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

// Store the accumulators through C's operand map (masked: out-of-range elements dropped).
template <int BM, int BN>
__device__ __forceinline__ void store_tile_generic(void *C, const OperandMap &mc, int64_t c_batch_off,
                                                   float16v (&acc)[BM / 64][BN / 64], int64_t row0, int64_t col0,
                                                   int wave_m, int wave_n, int lane, int out_dtype)
{
    constexpr int TM = BM / 64, TN = BN / 64;
    const int l32 = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int64_t col = col0 + wave_n * (BN / 2) + tn * 32 + l32;
        const AxisPart cp = col_part(mc, col);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = row0 + wave_m * (BM / 2) + tm * 32 + 8 * (v / 4) + 4 * hi + (v % 4);
                const AxisPart rp = row_part(mc, row);
                int64_t off;
                if (element_at(mc, row, col, rp, cp, &off)) store_out(C, c_batch_off + off, acc[tm][tn][v], out_dtype);
            }
        }
    }
}

// =========================================================================== generic kernel
template <int BM, int BN, int BK, bool BF16>
__global__ __launch_bounds__(kThreads) void gemm_generic_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, void *__restrict__ C,
    const OperandMap ma, const OperandMap mb, const OperandMap mc,
    int64_t sa_batch, int64_t sb_batch, int64_t sc_batch, int64_t mt, int64_t nt, int64_t kt, int out_dtype)
{
    __shared__ __attribute__((aligned(16))) uint16_t as[BM * BK];
    __shared__ __attribute__((aligned(16))) uint16_t bs[BN * BK];
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

    for (int64_t k = 0; k < kt; ++k) {
        const int64_t k0 = k * BK;
        // A tile: element (r, c) of the tile is A_view[row0 + r, k0 + c]
        {
            const int c = tid % BK;
            const AxisPart cp = col_part(ma, k0 + c);
            for (int r = tid / BK; r < BM; r += kThreads / BK) {
                const AxisPart rp = row_part(ma, row0 + r);
                int64_t off;
                uint16_t v = 0;
                if (element_at(ma, row0 + r, k0 + c, rp, cp, &off)) v = Ab[off];
                as[lds_chunk_pos<BK>(r, c >> 3) + (c & 7)] = v;
            }
        }
        // B tile: element (c, n) of the tile is B_view[k0 + c, col0 + n]; stored transposed
        {
            const int n = tid % BN;
            const AxisPart cp = col_part(mb, col0 + n);
            for (int c = tid / BN; c < BK; c += (kThreads / BN > 0 ? kThreads / BN : 1)) {
                const AxisPart rp = row_part(mb, k0 + c);
                int64_t off;
                uint16_t v = 0;
                if (element_at(mb, k0 + c, col0 + n, rp, cp, &off)) v = Bb[off];
                bs[lds_chunk_pos<BK>(n, c >> 3) + (c & 7)] = v;
            }
        }
        __syncthreads();
        mma_tile<BM, BN, BK, BF16>(as, bs, acc, wave_m, wave_n, lane);
        __syncthreads();
    }
    store_tile_generic<BM, BN>(C, mc, bi * sc_batch, acc, row0, col0, wave_m, wave_n, lane, out_dtype);
}

// ============================================================================== fast kernel
// Operand orientations handled by the fast loaders.
//   A: KCONTIG = rows of A contiguous along k (row-major [M,K]);  MNCONTIG = contiguous along m
//   B: MNCONTIG = rows of B contiguous along n (row-major [K,N]); KCONTIG = contiguous along k
constexpr int KCONTIG = 0, MNCONTIG = 1;

struct FastArgs {
    const uint16_t *A;
    const uint16_t *B;
    void *C;
    int64_t lda, ldb;              // stride of the non-contiguous axis (elements)
    int64_t scm, scn;              // C strides
    int64_t sa_batch, sb_batch, sc_batch;
    int64_t M, N, K;
    int64_t mt, nt, kt;
    int out_dtype;
};

__device__ __forceinline__ u32x4 load16(const uint16_t *p)
{
    // 16 bytes from a possibly only 2-byte aligned address (unaligned vector loads are legal
    // for global memory on this target)
    u32x4 v;
    __builtin_memcpy(&v, p, 16);
    return v;
}

__device__ __forceinline__ u32x2 load8(const uint16_t *p)
{
    u32x2 v;
    __builtin_memcpy(&v, p, 8);
    return v;
}

// Masked variant: elements [0, nvalid) of the 8 are read, the rest are zero.
__device__ __forceinline__ u32x4 load16_partial(const uint16_t *p, int nvalid)
{
    uint16_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = i < nvalid ? p[i] : (uint16_t)0;
    u32x4 v;
    v[0] = e[0] | ((uint32_t)e[1] << 16);
    v[1] = e[2] | ((uint32_t)e[3] << 16);
    v[2] = e[4] | ((uint32_t)e[5] << 16);
    v[3] = e[6] | ((uint32_t)e[7] << 16);
    return v;
}

// Loader for an operand tile whose LDS rows are contiguous in memory along k:
// (ROWS x BK) tile, element (r, c) at base[r * ld + c].  CH chunks of 16 bytes per thread.
template <int ROWS, int BK, bool EDGE>
struct KContigLoader {
    static constexpr int CPR = BK / 8;
    static constexpr int CH = ROWS * CPR / kThreads;
    static_assert(ROWS * CPR % kThreads == 0, "tile too small for the chunk loader");
    u32x4 r[CH];

    // row_lim / k_lim: number of valid rows / k elements counted from the tile origin
    __device__ __forceinline__ void load(const uint16_t *base, int64_t ld, int tid, int64_t row_lim, int64_t k_lim)
    {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int idx = i * kThreads + tid;
            const int row = idx / CPR, ch = idx % CPR;
            const uint16_t *p = base + (int64_t)row * ld + ch * 8;
            if constexpr (!EDGE) {
                r[i] = load16(p);
            } else {
                const int64_t left = k_lim - ch * 8;
                if (row < row_lim && left >= 8) r[i] = load16(p);
                else if (row < row_lim && left > 0) r[i] = load16_partial(p, (int)left);
                else r[i] = u32x4{0, 0, 0, 0};
            }
        }
    }
    __device__ __forceinline__ void store(uint16_t *lds, int tid) const
    {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int idx = i * kThreads + tid;
            const int row = idx / CPR, ch = idx % CPR;
            *reinterpret_cast<u32x4 *>(lds + lds_chunk_pos<BK>(row, ch)) = r[i];
        }
    }
};

// Loader for an operand tile whose memory is contiguous along the LDS *row* index (m for A,
// n for B): element (row, c) at base[c * ld + row].  Each thread owns 8(k) x NW(row) blocks,
// loads NW contiguous elements from each of 8 consecutive k lines and transposes them in
// registers into NW chunks of 8 consecutive k.
template <int ROWS, int BK, bool EDGE>
struct MnContigLoader {
    static constexpr int KB = BK / 8;                                   // k blocks
    static constexpr int NW = (KB * (ROWS / 8) >= kThreads) ? 8 : 4;    // rows per block
    static constexpr int NBLK = KB * (ROWS / NW);
    static constexpr int PER = NBLK / kThreads;
    static_assert(NBLK % kThreads == 0 && PER >= 1, "tile too small for the transposing loader");
    static constexpr int RB = ROWS / NW;                                // blocks along the row axis
    uint32_t r[PER][8][NW / 2];                                         // [block][k line][packed pairs]

    __device__ __forceinline__ void load(const uint16_t *base, int64_t ld, int tid, int64_t row_lim, int64_t k_lim)
    {
#pragma unroll
        for (int b = 0; b < PER; ++b) {
            const int idx = b * kThreads + tid;
            const int kb = idx / RB, rb = idx % RB;
            const int row = rb * NW;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int kk = kb * 8 + j;
                const uint16_t *p = base + (int64_t)kk * ld + row;
                if constexpr (!EDGE) {
                    if constexpr (NW == 8) {
                        u32x4 v = load16(p);
                        r[b][j][0] = v[0]; r[b][j][1] = v[1]; r[b][j][2] = v[2]; r[b][j][3] = v[3];
                    } else {
                        u32x2 v = load8(p);
                        r[b][j][0] = v[0]; r[b][j][1] = v[1];
                    }
                } else {
                    const int64_t left = row_lim - row;
                    if (kk < k_lim && left >= NW) {
                        if constexpr (NW == 8) {
                            u32x4 v = load16(p);
                            r[b][j][0] = v[0]; r[b][j][1] = v[1]; r[b][j][2] = v[2]; r[b][j][3] = v[3];
                        } else {
                            u32x2 v = load8(p);
                            r[b][j][0] = v[0]; r[b][j][1] = v[1];
                        }
                    } else {
#pragma unroll
                        for (int h = 0; h < NW / 2; ++h) {
                            uint32_t lo = (kk < k_lim && 2 * h < left) ? p[2 * h] : 0;
                            uint32_t hi2 = (kk < k_lim && 2 * h + 1 < left) ? p[2 * h + 1] : 0;
                            r[b][j][h] = lo | (hi2 << 16);
                        }
                    }
                }
            }
        }
    }
    __device__ __forceinline__ void store(uint16_t *lds, int tid) const
    {
#pragma unroll
        for (int b = 0; b < PER; ++b) {
            const int idx = b * kThreads + tid;
            const int kb = idx / RB, rb = idx % RB;
#pragma unroll
            for (int n = 0; n < NW; ++n) {
                // chunk for row rb*NW + n: element j (k = kb*8 + j) is half (n & 1) of r[b][j][n >> 1]
                u32x4 v;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t lo = r[b][2 * q][n >> 1], hi2 = r[b][2 * q + 1][n >> 1];
                    v[q] = (n & 1) ? __builtin_amdgcn_perm(hi2, lo, 0x07060302u) : __builtin_amdgcn_perm(hi2, lo, 0x05040100u);
                }
                *reinterpret_cast<u32x4 *>(lds + lds_chunk_pos<BK>(rb * NW + n, kb)) = v;
            }
        }
    }
};

template <int ROWS, int BK, int LAYOUT, bool EDGE>
struct LoaderSel { using type = KContigLoader<ROWS, BK, EDGE>; };
template <int ROWS, int BK, bool EDGE>
struct LoaderSel<ROWS, BK, MNCONTIG, EDGE> { using type = MnContigLoader<ROWS, BK, EDGE>; };

template <int BM, int BN, int BK, bool BF16, int ALAY, int BLAY, bool EDGE>
__global__ __launch_bounds__(kThreads) void gemm_fast_kernel(const FastArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *as0 = smem, *as1 = smem + BM * BK;
    uint16_t *bs0 = smem + 2 * BM * BK, *bs1 = bs0 + BN * BK;

    int64_t bi, ti, tj;
    locate_program(g.mt, g.nt, &bi, &ti, &tj);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int64_t row0 = ti * BM, col0 = tj * BN;

    // tile origins: A_tile(r, c) and B_tile(c, n) for k tile 0
    const uint16_t *Ab = g.A + bi * g.sa_batch + (ALAY == KCONTIG ? row0 * g.lda : row0);
    const uint16_t *Bb = g.B + bi * g.sb_batch + (BLAY == KCONTIG ? col0 * g.ldb : col0);
    const int64_t a_kstep = ALAY == KCONTIG ? (int64_t)BK : (int64_t)BK * g.lda;
    const int64_t b_kstep = BLAY == KCONTIG ? (int64_t)BK : (int64_t)BK * g.ldb;
    const int64_t m_lim = g.M - row0, n_lim = g.N - col0;

    typename LoaderSel<BM, BK, ALAY, EDGE>::type la;
    typename LoaderSel<BN, BK, BLAY, EDGE>::type lb;

    float16v acc[BM / 64][BN / 64];
#pragma unroll
    for (int a = 0; a < BM / 64; ++a)
#pragma unroll
        for (int b = 0; b < BN / 64; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    if (g.kt > 0) {
        la.load(Ab, g.lda, tid, m_lim, g.K);
        lb.load(Bb, g.ldb, tid, n_lim, g.K);
        la.store(as0, tid);
        lb.store(bs0, tid);
    }
    __syncthreads();
    for (int64_t k = 0; k < g.kt; ++k) {
        const bool more = k + 1 < g.kt;
        uint16_t *as_cur = (k & 1) ? as1 : as0, *bs_cur = (k & 1) ? bs1 : bs0;
        uint16_t *as_nxt = (k & 1) ? as0 : as1, *bs_nxt = (k & 1) ? bs0 : bs1;
        if (more) {
            const int64_t k_lim = g.K - (k + 1) * BK;
            la.load(Ab + (k + 1) * a_kstep, g.lda, tid, m_lim, k_lim);
            lb.load(Bb + (k + 1) * b_kstep, g.ldb, tid, n_lim, k_lim);
        }
        mma_tile<BM, BN, BK, BF16>(as_cur, bs_cur, acc, wave_m, wave_n, lane);
        if (more) {
            la.store(as_nxt, tid);
            lb.store(bs_nxt, tid);
        }
        __syncthreads();
    }

    // epilogue: masked, strided store of the converted accumulator
    constexpr int TM = BM / 64, TN = BN / 64;
    const int l32 = lane & 31, hi = lane >> 5;
    char *Cb = reinterpret_cast<char *>(g.C);
    const int64_t cb = bi * g.sc_batch;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int64_t col = col0 + wave_n * (BN / 2) + tn * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = row0 + wave_m * (BM / 2) + tm * 32 + 8 * (v / 4) + 4 * hi + (v % 4);
                if (!EDGE || (row < g.M && col < g.N))
                    store_out(Cb, cb + row * g.scm + col * g.scn, acc[tm][tn][v], g.out_dtype);
            }
        }
}


// ---- host-side helpers shared by the translation units that instantiate the kernels
inline nt_status check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
    return NT_OK;
}

template <int BM, int BN, int BK, bool BF16, int ALAY, int BLAY, bool EDGE>
static nt_status launch_fast_inst(const FastArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)2 * (BM + BN) * BK * sizeof(uint16_t);
    auto kern = gemm_fast_kernel<BM, BN, BK, BF16, ALAY, BLAY, EDGE>;
    static bool configured = false;              // raise the dynamic LDS limit once per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_fast_kernel");
}

template <int BM, int BN, int BK, bool BF16, bool EDGE>
static nt_status launch_fast_lay(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s)
{
    if (alay == KCONTIG && blay == MNCONTIG) return launch_fast_inst<BM, BN, BK, BF16, KCONTIG, MNCONTIG, EDGE>(a, nwg, s);
    if (alay == KCONTIG && blay == KCONTIG) return launch_fast_inst<BM, BN, BK, BF16, KCONTIG, KCONTIG, EDGE>(a, nwg, s);
    if (alay == MNCONTIG && blay == MNCONTIG) return launch_fast_inst<BM, BN, BK, BF16, MNCONTIG, MNCONTIG, EDGE>(a, nwg, s);
    return launch_fast_inst<BM, BN, BK, BF16, MNCONTIG, KCONTIG, EDGE>(a, nwg, s);
}

template <int BM, int BN, int BK>
static nt_status launch_fast_t(const FastArgs &a, bool bf16, bool edge, int alay, int blay, int64_t nwg, hipStream_t s)
{
    if (bf16) return edge ? launch_fast_lay<BM, BN, BK, true, true>(a, alay, blay, nwg, s)
                          : launch_fast_lay<BM, BN, BK, true, false>(a, alay, blay, nwg, s);
    return edge ? launch_fast_lay<BM, BN, BK, false, true>(a, alay, blay, nwg, s)
                : launch_fast_lay<BM, BN, BK, false, false>(a, alay, blay, nwg, s);
}

// one translation unit per tile shape defines these (parallel compilation)
nt_status launch_fast_128x128(const FastArgs &a, bool bf16, bool edge, int alay, int blay, int64_t nwg, hipStream_t s);
nt_status launch_fast_256x128(const FastArgs &a, bool bf16, bool edge, int alay, int blay, int64_t nwg, hipStream_t s);
nt_status launch_fast_128x256(const FastArgs &a, bool bf16, bool edge, int alay, int blay, int64_t nwg, hipStream_t s);
nt_status launch_fast_256x256(const FastArgs &a, bool bf16, bool edge, int alay, int blay, int64_t nwg, hipStream_t s);
nt_status launch_generic(const GemmLaunch &g);

}  // namespace nt
