// Direct kernel: full tiles of 16-byte aligned, unit-stride operands.
//
// One workgroup (4 wavefronts, 2 x 2) computes one BM x BN output tile (one program of
// the tile-to-program mapping, Section 3.2.1).  The (BM x 64) block of A and the
// (64 x BN) block of B of each k tile (source-to-target mapping, Section 3.2.2) travel
// from global memory straight into LDS (global_load_lds, 16 bytes per lane, no staging
// registers); two LDS copies of each block alternate so the next k tile streams in while
// the current one is multiplied.
//
// LDS layouts, chosen by how the operand lies in memory:
//   k-major  (operand contiguous along k)    [row = m or n][64 k], 128 bytes per row; a
//            lane's MFMA operand (8 consecutive k) is one ds_read_b128.
//   mn-major (operand contiguous along m/n)  [k][E = BM or BN]; the MFMA operand is
//            gathered with two transposing reads (ds_read_b64_tr_b16), each of which turns
//            a 4(k) x 16(m/n) patch into 4 consecutive k per lane.
// A direct-to-LDS load always writes lane l's 16 bytes to (instruction base + 16 l), so the
// bank swizzle is applied on the global side: lane l fetches the chunk that belongs in
// its slot.  k-major: chunk ^= (row ^ row/8) & 7; mn-major: chunk ^= (k & 3) * 4.
#pragma once
#include <type_traits>

#include "gemm_fast.h"

namespace nt {

typedef short short4v __attribute__((ext_vector_type(4)));

// vmcnt(0) only: expcnt and lgkmcnt fields at "no wait"
#define NT_WAIT_VMCNT0() __builtin_amdgcn_s_waitcnt(0x0F70)

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at
// lds_addr + 16 l.  gbase and lds_addr are wavefront-uniform, voff is the lane's byte offset.
// Issued through inline assembly so that the compiler does not serialise later LDS reads of
// the *other* LDS copy behind it; completion is awaited explicitly with NT_WAIT_VMCNT0.
__device__ __forceinline__ void dma16(const char *gbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(gbase)
                 : "memory");   // m0 is not otherwise used by these kernels
}

template <int E, int LAY>
struct DirectTile;

// ---- k-major block: E rows (m or n) x 64 k
template <int E>
struct DirectTile<E, KCONTIG> {
    static constexpr uint32_t BYTES = E * kBK * 2;
    static constexpr int PER = BYTES / 1024 / 4;           // load instructions per wavefront
    uint32_t voff[PER];                                    // global byte offset of this lane's chunk
    uint32_t rd;                                           // LDS read base of this lane

    __device__ __forceinline__ void init(int wave, int lane, int64_t ld, int wave_origin)
    {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int row = (wave * PER + j) * 8 + (lane >> 3);
            const int c = (lane & 7) ^ ((row ^ (row >> 3)) & 7);
            voff[j] = ((uint32_t)row * (uint32_t)ld + (uint32_t)(c * 8)) * 2u;
        }
        const int r = wave_origin + (lane & 31);
        rd = (uint32_t)(r * 128 + (((lane >> 5) ^ ((r ^ (r >> 3)) & 7)) << 4));
    }
    __device__ __forceinline__ void issue(const char *g, uint32_t lds_base, int wave) const
    {
#pragma unroll
        for (int j = 0; j < PER; ++j) dma16(g, voff[j], lds_base + (uint32_t)((wave * PER + j) * 1024));
    }
    __device__ __forceinline__ u32x4 frag(const char *smem, int t, int ks, uint32_t lds_base) const
    {
        return lds_read16(smem, (rd ^ (uint32_t)(((2 * ks) ^ ((t & 1) << 2)) << 4)) + t * 4096 + lds_base);
    }
};

// ---- mn-major block: 64 k rows x E (m or n)
template <int E>
struct DirectTile<E, MNCONTIG> {
    static constexpr uint32_t BYTES = E * kBK * 2;
    static constexpr int PER = BYTES / 1024 / 4;
    static constexpr int RB = 2 * E;                       // bytes per k row
    static constexpr int CPR = E / 8;                      // 16-byte chunks per k row
    static constexpr int RPI = 1024 / RB;                  // k rows per load instruction
    static constexpr int T = E / 64;                       // 32-wide operand blocks per wavefront
    uint32_t voff[PER];
    uint32_t rd[T];

    __device__ __forceinline__ void init(int wave, int lane, int64_t ld, int wave_origin)
    {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int krow = (wave * PER + j) * RPI + lane / CPR;
            const int c = (lane % CPR) ^ ((krow & 3) << 2);
            voff[j] = ((uint32_t)krow * (uint32_t)ld + (uint32_t)(c * 8)) * 2u;
        }
        // transposing read: 16-lane group g covers k rows 8*(g/2) .. +3 (+4 for the second
        // read) and columns 16*(g%2) .. +15; lane i of the group points at row i/4, 4 columns
        // starting at 4*(i%4), and receives 4 consecutive k of column i
        const int g = lane >> 4, i = lane & 15;
        const int kl = 8 * (g >> 1) + (i >> 2);
        const int mn = wave_origin + 16 * (g & 1) + 4 * (i & 3);
        const int sw = (i >> 2) << 2;                      // (k & 3) * 4 for every row this lane touches
#pragma unroll
        for (int t = 0; t < T; ++t)
            rd[t] = (uint32_t)(kl * RB + ((((mn >> 3) + 4 * t) ^ sw) << 4) + ((mn >> 2) & 1) * 8);
    }
    __device__ __forceinline__ void issue(const char *g, uint32_t lds_base, int wave) const
    {
#pragma unroll
        for (int j = 0; j < PER; ++j) dma16(g, voff[j], lds_base + (uint32_t)((wave * PER + j) * 1024));
    }
    __device__ __forceinline__ u32x4 frag(const char *smem, int t, int ks, uint32_t lds_base) const
    {
        typedef short4v __attribute__((address_space(3))) * lds_s4;
        const uint32_t a = rd[t] + (uint32_t)(ks * 16 * RB) + lds_base;
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(smem + a));
        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(smem + a + 4 * RB));
        const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
        return u32x4{l2[0], l2[1], h2[0], h2[1]};
    }
};

template <int BM, int BN, bool BF16, int ALAY, int BLAY>
__global__ __launch_bounds__(kThreads) void gemm_direct_kernel(const FastArgs g)
{
    constexpr int TM = BM / 64, TN = BN / 64;
    using TileA = DirectTile<BM, ALAY>;
    using TileB = DirectTile<BN, BLAY>;
    constexpr uint32_t A_BYTES = TileA::BYTES, B_BYTES = TileB::BYTES, B_BASE = 2 * A_BYTES;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int64_t bi, ti, tj;
    locate_program(g.mt, g.nt, &bi, &ti, &tj);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int l32 = lane & 31, hi = lane >> 5;
    const int64_t row0 = ti * BM, col0 = tj * BN;

    const char *gA = reinterpret_cast<const char *>(g.A + bi * g.sa_batch + (ALAY == KCONTIG ? row0 * g.lda : row0));
    const char *gB = reinterpret_cast<const char *>(g.B + bi * g.sb_batch + (BLAY == KCONTIG ? col0 * g.ldb : col0));
    const int64_t a_step = (ALAY == KCONTIG ? (int64_t)kBK : (int64_t)kBK * g.lda) * 2;
    const int64_t b_step = (BLAY == KCONTIG ? (int64_t)kBK : (int64_t)kBK * g.ldb) * 2;

    TileA ta;
    TileB tb;
    ta.init(wave, lane, g.lda, wave_m * (BM / 2));
    tb.init(wave, lane, g.ldb, wave_n * (BN / 2));

    float16v acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // LDS byte address of the dynamic segment (it starts the workgroup's allocation)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    u32x4 fa[2][TM], fb[2][TN];
    auto fetch = [&](int slot, int ks, uint32_t copy) {
#pragma unroll
        for (int t = 0; t < TM; ++t) fa[slot][t] = ta.frag(smem, t, ks, copy * A_BYTES);
#pragma unroll
        for (int t = 0; t < TN; ++t) fb[slot][t] = tb.frag(smem, t, ks, B_BASE + copy * B_BYTES);
    };
    auto mma = [&](int slot) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = mfma32<BF16>(fa[slot][tm], fb[slot][tn], acc[tm][tn]);
    };

    // k tile 0 -> copy 0, then its first fragments
    ta.issue(gA, lds0, wave);
    tb.issue(gB, lds0 + B_BASE, wave);
    NT_WAIT_VMCNT0();
    __syncthreads();
    fetch(0, 0, 0);

    // One k tile per trip, one basic block.  The next tile (clamped to the last one, whose
    // surplus copy is never read) streams into the idle LDS copy while the current copy is
    // multiplied; operand fragments are double buffered, each k step fetching the next
    // step's fragments before issuing its own MFMAs.  The barrier sits before the last k
    // step so that the first fragments of the next tile are fetched under its MFMAs.
    const int64_t last = g.kt - 1;
    uint32_t cur = 0;
    for (int64_t k = 0; k < g.kt; ++k) {
        const uint32_t nxt = cur ^ 1u;
        const int64_t kn = k < last ? k + 1 : last;
        ta.issue(gA + kn * a_step, lds0 + nxt * A_BYTES, wave);
        tb.issue(gB + kn * b_step, lds0 + B_BASE + nxt * B_BYTES, wave);
        __builtin_amdgcn_sched_barrier(0);
        fetch(1, 1, cur);
        __builtin_amdgcn_sched_barrier(0);
        mma(0);
        __builtin_amdgcn_sched_barrier(0);
        fetch(0, 2, cur);
        __builtin_amdgcn_sched_barrier(0);
        mma(1);
        __builtin_amdgcn_sched_barrier(0);
        fetch(1, 3, cur);
        __builtin_amdgcn_sched_barrier(0);
        mma(0);
        __builtin_amdgcn_sched_barrier(0);
        NT_WAIT_VMCNT0();                                  // this wave's share of the next tile has landed
        __syncthreads();                                   // ... and everyone's; all reads of `cur` are done
        fetch(0, 0, nxt);
        __builtin_amdgcn_sched_barrier(0);
        mma(1);
        __builtin_amdgcn_sched_barrier(0);
        cur = nxt;
    }

    const int64_t row_base = row0 + wave_m * (BM / 2) + 4 * hi;
    const int64_t col_base = col0 + wave_n * (BN / 2) + l32;
    const int64_t cb = bi * g.sc_batch;
    if (g.out_dtype == NT_F32)
        store_tile_fast<BM, BN, float>(reinterpret_cast<float *>(g.C) + cb, g.scm, g.scn, acc, row_base, col_base, g.M, g.N, false, g.out_dtype);
    else
        store_tile_fast<BM, BN, uint16_t>(reinterpret_cast<uint16_t *>(g.C) + cb, g.scm, g.scn, acc, row_base, col_base, g.M, g.N, false, g.out_dtype);
}

template <int BM, int BN, bool BF16, int ALAY, int BLAY>
static nt_status launch_direct_inst(const FastArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)2 * (BM + BN) * kBK * sizeof(uint16_t);
    auto kern = gemm_direct_kernel<BM, BN, BF16, ALAY, BLAY>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_direct_kernel");
}

template <int BM, int BN>
static nt_status launch_direct_t(const FastArgs &a, bool bf16, int alay, int blay, int64_t nwg, hipStream_t s)
{
#define NT_DIRECT(BF, AL, BL) launch_direct_inst<BM, BN, BF, AL, BL>(a, nwg, s)
    if (bf16) {
        if (alay == KCONTIG) return blay == MNCONTIG ? NT_DIRECT(true, KCONTIG, MNCONTIG) : NT_DIRECT(true, KCONTIG, KCONTIG);
        return blay == MNCONTIG ? NT_DIRECT(true, MNCONTIG, MNCONTIG) : NT_DIRECT(true, MNCONTIG, KCONTIG);
    }
    if (alay == KCONTIG) return blay == MNCONTIG ? NT_DIRECT(false, KCONTIG, MNCONTIG) : NT_DIRECT(false, KCONTIG, KCONTIG);
    return blay == MNCONTIG ? NT_DIRECT(false, MNCONTIG, MNCONTIG) : NT_DIRECT(false, MNCONTIG, KCONTIG);
#undef NT_DIRECT
}

nt_status launch_direct_128x128(const FastArgs &a, bool bf16, int alay, int blay, int64_t nwg, hipStream_t s);
nt_status launch_direct_256x128(const FastArgs &a, bool bf16, int alay, int blay, int64_t nwg, hipStream_t s);
nt_status launch_direct_128x256(const FastArgs &a, bool bf16, int alay, int blay, int64_t nwg, hipStream_t s);
nt_status launch_direct_256x256(const FastArgs &a, bool bf16, int alay, int blay, int64_t nwg, hipStream_t s);

}  // namespace nt
