// Fast kernel for plain operands that have unit stride along one of their axes.
//
// One workgroup (4 wavefronts, 2 x 2) computes one BM x BN output tile (one program of the
// tile-to-program mapping, Section 3.2.1).  Per k tile (BK = 64) every thread fetches its
// share of the A and B blocks with 16-byte global loads into staging registers, writes
// them to LDS in the swizzled k-contiguous layout (B, or a column-major A, is transposed
// in registers on the way) and the wavefronts read 8-element k runs as MFMA operands.
//
// This is the path for a ragged K and for operands that are not 16-byte aligned.  Every k tile but the
// last ones is fetched with range-checked buffer loads (what lies past an operand's end reads as zero,
// so tiles that overhang M or N need no predicates); the last k tiles are fetched with predicated
// loads, the one vector per row or k line that straddles a ragged end is fetched early and shifted into
// place with zero fill (masked elements read as zero); stores are masked.  Aligned operands with whole
// k tiles take the direct kernel instead.
#pragma once
#include <type_traits>

#include "gemm_device.h"

namespace nt {

// Operand orientations:
//   A: KCONTIG = A[m, k] contiguous along k (row-major [M,K]); MNCONTIG = contiguous along m
//   B: MNCONTIG = B[k, n] contiguous along n (row-major [K,N]); KCONTIG = contiguous along k
constexpr int KCONTIG = 0, MNCONTIG = 1;
constexpr int kBK = 64;

struct FastArgs {
    const uint16_t *A;
    const uint16_t *B;
    void *C;
    int64_t lda, ldb;              // stride (elements) of the axis that is not contiguous
    int64_t scm, scn;              // C strides (elements)
    int64_t sa_batch, sb_batch, sc_batch;
    int64_t M, N, K;
    int64_t mt, nt, kt;
    int out_dtype;
    // epilogue C = alpha * acc + beta * D (D: out_dtype elements, read only if beta != 0 and D != nullptr)
    const void *D;
    int64_t sdm, sdn, sd_batch;
    float alpha, beta;
    int32_t act;                   // activation of the combined value (0 = none)
    // bytes from the first to one past the last element of A / B (one batch entry): the bound of the range-checked loads
    int64_t a_extent, b_extent;
    // direct kernel, range-checked flavour: bit 0 / 1 = the word of a load that holds A's / B's very last element can end
    // past the operand (odd pitch or extent) and is dropped by the range check; the kernel then puts that element in place itself
    int32_t patch;
    // persistent kernel: the launch's number of programs (each workgroup walks programs w, w + grid, w + 2 grid, ...)
    int64_t nprog;
    // ... and the start-up stagger: workgroup w starts ((w / 8) % 4) * stagger hundredths of a microsecond late (0: none)
    int32_t stagger;
    // loader trace (nt_trace_loader_tile; nullptr otherwise): one workgroup runs program trace_program's loads of 32-k slice
    // trace_slice for real and writes what they left in LDS for operand trace_operand (0 = A, 1 = B), element by element
    uint16_t *trace_out;
    int64_t trace_program;
    int32_t trace_slice, trace_operand;
};

__device__ __forceinline__ u32x4 gload16(const char *base, uint32_t off)
{
    // 16 bytes from a possibly only 2-byte aligned address (unaligned vector loads are
    // legal for global memory on this target); uniform base + 32-bit lane offset
    u32x4 v;
    __builtin_memcpy(&v, base + off, 16);
    return v;
}

__device__ __forceinline__ u32x2 gload8(const char *base, uint32_t off)
{
    u32x2 v;
    __builtin_memcpy(&v, base + off, 8);
    return v;
}

__device__ __forceinline__ uint32_t gload2(const char *base, uint32_t off)
{
    return *reinterpret_cast<const uint16_t *>(base + off);
}

__device__ __forceinline__ void lds_write16(char *smem, uint32_t addr, u32x4 v)
{
    *reinterpret_cast<u32x4 *>(smem + addr) = v;
}

__device__ __forceinline__ u32x4 lds_read16(const char *smem, uint32_t addr)
{
    return *reinterpret_cast<const u32x4 *>(smem + addr);
}

// The 8 (4) 16-bit elements of v moved down by sh (0..7 / 0..3) element positions, zero filled
// from the top: what a vector load that started sh elements early has to undergo.
__device__ __forceinline__ u32x4 shift_down(u32x4 v, int sh)
{
    const uint32_t hb = (uint32_t)(sh & 1) * 16u;
    uint32_t w0 = __builtin_amdgcn_alignbit(v[1], v[0], hb), w1 = __builtin_amdgcn_alignbit(v[2], v[1], hb);
    uint32_t w2 = __builtin_amdgcn_alignbit(v[3], v[2], hb), w3 = v[3] >> hb;
    if (sh & 2) { w0 = w1; w1 = w2; w2 = w3; w3 = 0; }
    if (sh & 4) { w0 = w2; w1 = w3; w2 = 0; w3 = 0; }
    return u32x4{w0, w1, w2, w3};
}
__device__ __forceinline__ u32x2 shift_down(u32x2 v, int sh)
{
    const uint32_t hb = (uint32_t)(sh & 1) * 16u;
    uint32_t w0 = __builtin_amdgcn_alignbit(v[1], v[0], hb), w1 = v[1] >> hb;
    if (sh & 2) { w0 = w1; w1 = 0; }
    return u32x2{w0, w1};
}

// ---- staging of a (ROWS x 64) operand block whose LDS rows are contiguous in memory along k
template <int ROWS, bool EDGE>
struct StageK {
    static constexpr int CH = ROWS * 8 / kThreads;        // 16-byte chunks per thread
    u32x4 r[CH];
    uint32_t voff0;                                       // byte offset of the thread's first chunk from the tile origin
    int64_t step;                                         // bytes between its chunks (32 rows; wavefront-uniform)
    uint32_t wbase;                                       // swizzled LDS byte offset of chunk 0
    int row0, ch;
    int shift;                                            // >= 0: pending shift of the last masked load

    __device__ __forceinline__ void init(int tid, int64_t ld)
    {
        shift = -1;
        row0 = tid >> 3;
        ch = tid & 7;
        voff0 = ((uint32_t)row0 * (uint32_t)ld + (uint32_t)(ch * 8)) * 2u;
        step = 64 * ld;
        const int s0 = (row0 & 7) ^ (tid >> 6);
        wbase = (uint32_t)(row0 * 128 + ((ch ^ s0) << 4));
    }
    // rows_left / k_left: valid rows and k elements counted from the tile origin.  Chunks are
    // fetched with one predicated 16-byte load each.  The one chunk per row that straddles the
    // ragged end of K (left of its 8 elements valid) is fetched sh = 8 - left elements early,
    // so that the load ends on the last valid element, and moved down by sh elements with zero
    // fill in settle(); K must be at least 8 for that address to stay inside the operand.
    // Masked elements read as zero.
    // MASKED = false: the caller knows the whole block is inside the operand.
    // One of the PIECES loads of a block that lies inside the operand (rows and k).
    __device__ __forceinline__ void load_piece(const char *base, int i)
    {
        r[i] = gload16(base + i * step, voff0);
        shift = -1;
    }
    // The same load through a range-checked buffer access (rsrc covers the operand, soff = byte offset of the
    // block's origin in it): rows past the operand's end lie past the buffer's and read as zero, so a block on
    // the ragged m / n end needs neither predicate nor clamp.  Only for blocks whose 64 k lie inside the operand.
    __device__ __forceinline__ void load_piece_buf(__amdgpu_buffer_rsrc_t rsrc, uint32_t soff, int i)
    {
        r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff0, soff + (uint32_t)i * (uint32_t)step, 0);
        shift = -1;
    }
    template <bool MASKED = EDGE>
    __device__ __forceinline__ void load(const char *base, int64_t rows_left, int64_t k_left)
    {
        if constexpr (!MASKED) {
#pragma unroll
            for (int i = 0; i < CH; ++i) load_piece(base, i);
        } else {
            const int left = (int)(k_left < kBK ? k_left : kBK) - ch * 8;
            const int sh = (left > 0 && left < 8) ? 8 - left : 0;
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                u32x4 v{0, 0, 0, 0};
                if (i * 32 + row0 < rows_left && left > 0) __builtin_memcpy(&v, base + i * step + ((int64_t)voff0 - 2 * sh), 16);
                r[i] = v;
            }
            shift = k_left < kBK ? sh : -1;
        }
    }
    // second half of a masked load, run when the data is needed (after the multiplications
    // that hide the load latency)
    __device__ __forceinline__ void settle()
    {
        if (shift >= 0) {                                  // wavefront-uniform
#pragma unroll
            for (int i = 0; i < CH; ++i) r[i] = shift_down(r[i], shift);
        }
    }
    static constexpr int PIECES = CH;                     // LDS writes per thread and block
    __device__ __forceinline__ void store_piece(char *smem, uint32_t buf_off, int i) const
    {
        lds_write16(smem, buf_off + (wbase ^ ((i & 1) << 6)) + i * 4096, r[i]);
    }
    __device__ __forceinline__ void store(char *smem, uint32_t buf_off) const
    {
#pragma unroll
        for (int i = 0; i < CH; ++i) store_piece(smem, buf_off, i);
    }
};

// ---- staging of a (ROWS x 64) block whose memory is contiguous along the LDS row index
// (m for a column-major A, n for a row-major B).  Each thread owns one 8(k) x NW(rows)
// block: NW contiguous elements from each of 8 consecutive k lines, transposed in
// registers into NW chunks of 8 consecutive k.
template <int ROWS, bool EDGE>
struct StageMN {
    static constexpr int NW = ROWS / 32;                  // 8 for 256 rows, 4 for 128 rows
    static_assert(NW == 8 || NW == 4, "transposing loader supports 128 or 256 rows");
    uint32_t r[8][NW / 2];                                // [k line][packed pairs of rows]
    uint32_t voff0;                                       // byte offset of the thread's first k line from the tile origin
    int64_t step;                                         // bytes between k lines (wavefront-uniform)
    uint32_t wbase;
    int kb, rb;
    int shift;                                            // >= 0: pending shift of the last masked load (see settle)

    __device__ __forceinline__ void init(int tid, int64_t ld)
    {
        shift = -1;
        kb = tid >> 5;
        rb = tid & 31;
        voff0 = ((uint32_t)(kb * 8) * (uint32_t)ld + (uint32_t)(rb * NW)) * 2u;
        step = 2 * ld;
        const int s = NW == 8 ? (rb & 7) : ((((rb & 1) << 2) ^ (rb >> 1)) & 7);
        wbase = (uint32_t)(rb * NW * 128 + ((kb ^ s) << 4));
    }
    // Blocks are fetched with one predicated vector load per k line.  The one block per k line
    // that straddles the ragged m/n end (rl of its NW elements valid) is fetched sh = NW - rl
    // elements early, so that the load ends on the last valid element, and shifted down by sh
    // elements with zero fill; the operand must be at least NW long along its contiguous axis
    // for that address to stay inside it.  Masked elements read as zero.
    // MASKED = false: the caller knows the whole block is inside the operand.
    // plain load of k line j (and j + NW for the narrower block, so that there are PIECES loads)
    // of a block that lies inside the operand
    // Plain load of k line p (and p + NW for the narrower block, so that there are PIECES loads) of a block that
    // lies inside the operand.
    __device__ __forceinline__ void load_piece(const char *base, int p)
    {
#pragma unroll
        for (int j = p; j < 8; j += NW) {
            if constexpr (NW == 8) {
                const u32x4 v = gload16(base + j * step, voff0);
                r[j][0] = v[0]; r[j][1] = v[1]; r[j][2] = v[2]; r[j][3] = v[3];
            } else {
                const u32x2 v = gload8(base + j * step, voff0);
                r[j][0] = v[0]; r[j][1] = v[1];
            }
        }
        shift = -1;
    }
    // The same through a range-checked buffer access (see StageK::load_piece_buf).  A block on the ragged m / n
    // end reads on into the next k line (or, past the operand's end, zeros): what it fetches beyond the valid
    // rows only reaches outputs that are never stored.
    __device__ __forceinline__ void load_piece_buf(__amdgpu_buffer_rsrc_t rsrc, uint32_t soff, int p)
    {
#pragma unroll
        for (int j = p; j < 8; j += NW) {
            if constexpr (NW == 8) {
                const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff0, soff + (uint32_t)j * (uint32_t)step, 0);
                r[j][0] = v[0]; r[j][1] = v[1]; r[j][2] = v[2]; r[j][3] = v[3];
            } else {
                const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff0, soff + (uint32_t)j * (uint32_t)step, 0);
                r[j][0] = v[0]; r[j][1] = v[1];
            }
        }
        shift = -1;
    }
    template <bool MASKED = EDGE>
    __device__ __forceinline__ void load(const char *base, int64_t rows_left, int64_t k_left)
    {
        if constexpr (!MASKED) {
#pragma unroll
            for (int p = 0; p < NW; ++p) load_piece(base, p);
            return;
        }
        const int rl = (int)(rows_left < ROWS ? rows_left : ROWS) - rb * NW;     // valid rows of this block
        const int kl = (int)(k_left < kBK ? k_left : kBK) - kb * 8;              // valid k lines of this block
        const int sh = (rl > 0 && rl < NW) ? NW - rl : 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if constexpr (!MASKED) {
                if constexpr (NW == 8) {
                    const u32x4 v = gload16(base + j * step, voff0);
                    r[j][0] = v[0]; r[j][1] = v[1]; r[j][2] = v[2]; r[j][3] = v[3];
                } else {
                    const u32x2 v = gload8(base + j * step, voff0);
                    r[j][0] = v[0]; r[j][1] = v[1];
                }
            } else {
                const bool any = j < kl && rl > 0;
                const char *p = base + j * step + ((int64_t)voff0 - 2 * sh);
                if constexpr (NW == 8) {
                    u32x4 v{0, 0, 0, 0};
                    if (any) __builtin_memcpy(&v, p, 16);
                    r[j][0] = v[0]; r[j][1] = v[1]; r[j][2] = v[2]; r[j][3] = v[3];
                } else {
                    u32x2 v{0, 0};
                    if (any) __builtin_memcpy(&v, p, 8);
                    r[j][0] = v[0]; r[j][1] = v[1];
                }
            }
        }
        shift = MASKED && rows_left < ROWS ? sh : -1;
    }
    // second half of a masked load, run when the data is needed (after the multiplications
    // that hide the load latency): moves early-fetched straddling blocks into place
    __device__ __forceinline__ void settle()
    {
        if (shift >= 0) {                                  // wavefront-uniform
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if constexpr (NW == 8) {
                    const u32x4 v = shift_down(u32x4{r[j][0], r[j][1], r[j][2], r[j][3]}, shift);
                    r[j][0] = v[0]; r[j][1] = v[1]; r[j][2] = v[2]; r[j][3] = v[3];
                } else {
                    const u32x2 v = shift_down(u32x2{r[j][0], r[j][1]}, shift);
                    r[j][0] = v[0]; r[j][1] = v[1];
                }
            }
        }
    }
    static constexpr int PIECES = NW;                     // LDS writes per thread and block
    __device__ __forceinline__ void store_piece(char *smem, uint32_t buf_off, int n) const
    {
        u32x4 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t lo = r[2 * q][n >> 1], hi = r[2 * q + 1][n >> 1];
            v[q] = (n & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
        lds_write16(smem, buf_off + (wbase ^ (n << 4)) + n * 128, v);
    }
    __device__ __forceinline__ void store(char *smem, uint32_t buf_off) const
    {
#pragma unroll
        for (int n = 0; n < NW; ++n) store_piece(smem, buf_off, n);
    }
};

template <int ROWS, int LAY, bool EDGE> struct StageSel { using type = StageK<ROWS, EDGE>; };
template <int ROWS, bool EDGE> struct StageSel<ROWS, MNCONTIG, EDGE> { using type = StageMN<ROWS, EDGE>; };

// ---- epilogue (output = accumulator, Section 4.2).
// The kernels in this file issue every MFMA with the B fragment as its first operand, so the
// 32 x 32 accumulator block comes out transposed: a lane holds one row m = lane % 32 and 16 of
// its columns, register v <-> n = 8 (v / 4) + 4 (lane / 32) + v % 4.

// The 16 consecutive columns 16 (lane / 32) .. + 15 of the lane's row: the two half-wavefronts
// trade register groups (v_permlane32_swap: the upper half's first operand <-> the lower half's
// second), after which columns ascend through registers 0-3, 8-11, 4-7, 12-15.  All lanes
// must be active.
__device__ __forceinline__ void gather_row16(const float16v &acc, uint32_t (&o)[16])
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        // (elements are copied out first: a bit cast applied to a vector element directly reads element 0)
        const float g0 = acc[q], g1 = acc[4 + q], g2 = acc[8 + q], g3 = acc[12 + q];
        const auto lo = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, g0), __builtin_bit_cast(uint32_t, g2), false, false);
        const auto up = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, g1), __builtin_bit_cast(uint32_t, g3), false, false);
        o[q] = lo[0];
        o[4 + q] = lo[1];
        o[8 + q] = up[0];
        o[12 + q] = up[1];
    }
}

template <int OUT>
__device__ __forceinline__ uint32_t pack_pair(uint32_t lo, uint32_t hi)
{
    const float a = __builtin_bit_cast(float, lo), b = __builtin_bit_cast(float, hi);
    if constexpr (OUT == NT_F16) {
        typedef _Float16 half2v __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, half2v{(_Float16)a, (_Float16)b});          // round to nearest even
    } else {
        typedef float float2v __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(float2v{a, b}, bf16x2v));   // one v_cvt_pk_bf16_f32
    }
}

// 16 consecutive elements of type OUT at p, as fp32
template <int OUT>
__device__ __forceinline__ void load_row16(const char *p, float (&d)[16])
{
    if constexpr (OUT == NT_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u32x4 v;
            __builtin_memcpy(&v, p + 16 * i, 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t w = v[q];               // (copied out: a bit cast of a vector element reads element 0)
                d[4 * i + q] = __builtin_bit_cast(float, w);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            u32x4 v;
            __builtin_memcpy(&v, p + 16 * i, 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t w = v[q];
                if constexpr (OUT == NT_F16) {
                    d[8 * i + 2 * q] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
                    d[8 * i + 2 * q + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
                } else {
                    d[8 * i + 2 * q] = __builtin_bit_cast(float, w << 16);
                    d[8 * i + 2 * q + 1] = __builtin_bit_cast(float, w & 0xffff0000u);
                }
            }
        }
    }
}

// C with unit stride along n.  The wavefront's (BM/2) x (BN/2) part of the tile goes through LDS
// (free by now; each wavefront uses a region of its own) so that global stores are whole lines:
//   write phase  every lane gathers 16 consecutive columns of its row per 32 x 32 block, applies
//                alpha / beta * D in fp32 if asked (D: elements of the output type with unit stride
//                along n and row stride sdm), converts once, and writes 16-byte chunks to
//                [row][RB bytes], chunk index XOR-swizzled with the row so that the 16-byte writes
//                of 16 lanes (16 rows, same chunk) fall on different banks;
//   read phase   RB / 16 consecutive lanes read one row, so a store instruction covers 64 / (RB/16)
//                rows of RB contiguous bytes each.
// An fp32 tile takes two passes (one per half of the columns) through the same region.
// (Storing 16-bit outputs straight from registers, two 16-byte stores per lane and block, completes a
// line of C with several instructions and moved 1.3 times the output's bytes to memory.)
// row_w / col_w: first row / column of the wavefront's part.  CHECK masks rows >= M and columns
// >= N (a partly valid 16-byte chunk is stored element-wise).
template <int BM, int BN, int OUT, bool CHECK>
__device__ __forceinline__ void store_tile_rows(char *smem, int wave, char *C, int64_t scm, const float16v (&acc)[BM / 64][BN / 64],
                                                int64_t row_w, int64_t col_w, int lane, int64_t M, int64_t N,
                                                bool affine, const char *D, int64_t sdm, float alpha, float beta, int act)
{
    constexpr int TM = BM / 64, TN = BN / 64, WM = BM / 2, WN = BN / 2;
    constexpr int ES = OUT == NT_F32 ? 4 : 2;
    constexpr int PASSES = OUT == NT_F32 ? 2 : 1;
    constexpr int TNP = TN / PASSES;                      // 32-column blocks per pass
    constexpr int RB = WN * 2;                            // bytes per region row (16-bit: WN elements; fp32: WN / 2)
    constexpr int CPR = RB / 16;                          // 16-byte chunks per row: 16 or 8
    constexpr int RSH = RB == 256 ? 0 : 1;                // log2(rows per 256 bytes of LDS)
    constexpr int EPC = 16 / ES;                          // elements per chunk
    constexpr int RPI = 64 / CPR;                         // rows per store instruction
    const int l32 = lane & 31, hi = lane >> 5;
    const ActParams ap = act_params(act);
    char *reg = smem + wave * (WM * RB);
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
        // ---- write phase
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int r = tm * 32 + l32;
            const int64_t row = row_w + r;
            const bool row_ok = !CHECK || row < M;
#pragma unroll
            for (int tnp = 0; tnp < TNP; ++tnp) {
                const int tn = pass * TNP + tnp;
                uint32_t o[16];
                gather_row16(acc[tm][tn], o);
                if (affine) {                                         // wavefront-uniform
                    float d[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) d[i] = 0.f;
                    if (D) {
                        const int64_t col = col_w + tn * 32 + 16 * hi;
                        const char *dp = D + (row * sdm + col) * ES;
                        const int64_t nv = CHECK ? N - col : 16;      // valid columns from the lane's first
                        if (row_ok && nv >= 16) {
                            load_row16<OUT>(dp, d);
                        } else if (CHECK && row_ok && nv > 0) {
#pragma unroll
                            for (int i = 0; i < 16; ++i)
                                if (i < nv) d[i] = load_as_f32(dp, i, OUT);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[i] = __builtin_bit_cast(uint32_t, combine(__builtin_bit_cast(float, o[i]), d[i], alpha, beta));
                if (act) {                                            // wavefront-uniform
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[i] = __builtin_bit_cast(uint32_t, activate(__builtin_bit_cast(float, o[i]), ap));
                }
                }
                const int c0 = (tnp * 32 + 16 * hi) / EPC;
                const int sw = (r >> RSH) & (CPR - 1);
                char *prow = reg + r * RB;
                if constexpr (OUT == NT_F32) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        lds_write16(prow, (uint32_t)(((c0 + q) ^ sw) << 4), u32x4{o[4 * q], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]});
                } else {
#pragma unroll
                    for (int q = 0; q < 2; ++q)
                        lds_write16(prow, (uint32_t)(((c0 + q) ^ sw) << 4),
                                    u32x4{pack_pair<OUT>(o[8 * q], o[8 * q + 1]), pack_pair<OUT>(o[8 * q + 2], o[8 * q + 3]),
                                          pack_pair<OUT>(o[8 * q + 4], o[8 * q + 5]), pack_pair<OUT>(o[8 * q + 6], o[8 * q + 7])});
                }
            }
        }
        // ---- read phase (same wavefront: LDS operations complete in order)
#pragma unroll
        for (int it = 0; it < WM / RPI; ++it) {
            const int r = it * RPI + lane / CPR, c = lane % CPR;
            const u32x4 v = lds_read16(reg, (uint32_t)(r * RB + ((c ^ ((r >> RSH) & (CPR - 1))) << 4)));
            const int64_t row = row_w + r;
            const int64_t col = col_w + pass * (WN / PASSES) + c * EPC;
            char *p = C + (row * scm + col) * ES;
            if (!CHECK || (row < M && col + EPC <= N)) {
                __builtin_memcpy(p, &v, 16);
            } else if (row < M && col < N) {
                const int nv = (int)(N - col);
#pragma unroll
                for (int e = 0; e < EPC; ++e)
                    if (e < nv) {
                        const uint32_t w = v[ES == 4 ? e : e / 2];
                        if constexpr (OUT == NT_F32) *reinterpret_cast<uint32_t *>(p + 4 * e) = w;
                        else *reinterpret_cast<uint16_t *>(p + 2 * e) = (uint16_t)((e & 1) ? w >> 16 : w & 0xffffu);
                    }
            }
        }
    }
}

// C (and D) with any strides: one store per element, always masked.
template <int BM, int BN>
__device__ __forceinline__ void store_tile_strided(void *C, int64_t scm, int64_t scn, const float16v (&acc)[BM / 64][BN / 64],
                                                   int64_t row_w, int64_t col_w, int lane, int64_t M, int64_t N, int out_dtype,
                                                   const void *D, int64_t sdm, int64_t sdn, float alpha, float beta, int act)
{
    constexpr int TM = BM / 64, TN = BN / 64;
    const int l32 = lane & 31, hi = lane >> 5;
    const ActParams ap = act_params(act);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int64_t row = row_w + tm * 32 + l32;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t col = col_w + tn * 32 + 8 * (v / 4) + 4 * hi + (v % 4);
                if (row < M && col < N) {
                    const float d = D ? load_as_f32(D, row * sdm + col * sdn, out_dtype) : 0.f;
                    const float x = combine(acc[tm][tn][v], d, alpha, beta);
                    store_out(C, row * scm + col * scn, act ? activate(x, ap) : x, out_dtype);
                }
            }
    }
}

// Epilogue of the transposed-accumulator kernels: picks the store routine for C's layout and format.
// EDGE = false (the direct kernel): full tiles, C and D with unit stride along n.
// smem: the workgroup's LDS, no longer in use by any wavefront (the caller has passed a barrier).
template <int BM, int BN, bool EDGE>
__device__ __forceinline__ void store_tile(const FastArgs &g, char *smem, int wave, int64_t bi, const float16v (&acc)[BM / 64][BN / 64],
                                           int64_t row_w, int64_t col_w, int lane, bool ragged)
{
    const int64_t esz = g.out_dtype == NT_F32 ? 4 : 2;
    char *C = reinterpret_cast<char *>(g.C) + bi * g.sc_batch * esz;
    const char *D = g.D ? reinterpret_cast<const char *>(g.D) + bi * g.sd_batch * esz : nullptr;
    if constexpr (EDGE) {       // (launches with such a C or D always take the EDGE flavour)
        if (g.scn != 1 || (D && g.sdn != 1)) {
            store_tile_strided<BM, BN>(C, g.scm, g.scn, acc, row_w, col_w, lane, g.M, g.N, g.out_dtype, D, g.sdm, g.sdn, g.alpha, g.beta, g.act);
            return;
        }
    }
    const bool affine = D != nullptr || g.alpha != 1.f || g.act != 0;
#define NT_ROWS(OUT, CHECK) store_tile_rows<BM, BN, OUT, CHECK>(smem, wave, C, g.scm, acc, row_w, col_w, lane, g.M, g.N, affine, D, g.sdm, g.alpha, g.beta, g.act)
    if constexpr (EDGE) {
        if (ragged) {
            if (g.out_dtype == NT_F32) NT_ROWS(NT_F32, true);
            else if (g.out_dtype == NT_F16) NT_ROWS(NT_F16, true);
            else NT_ROWS(NT_BF16, true);
            return;
        }
    }
    if (g.out_dtype == NT_F32) NT_ROWS(NT_F32, false);
    else if (g.out_dtype == NT_F16) NT_ROWS(NT_F16, false);
    else NT_ROWS(NT_BF16, false);
#undef NT_ROWS
}

template <int BM, int BN, bool BF16, int ALAY, int BLAY>
__global__ __launch_bounds__(kThreads) void gemm_fast_kernel(const FastArgs g)
{
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr uint32_t A_BYTES = BM * kBK * 2, B_BYTES = BN * kBK * 2;
    constexpr uint32_t B_BASE = 2 * A_BYTES;                 // LDS map: [A0][A1][B0][B1]
    extern __shared__ __attribute__((aligned(16))) char smem[];

    int64_t bi, ti, tj;
    locate_program(g.mt, g.nt, &bi, &ti, &tj);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int l32 = lane & 31, hi = lane >> 5;
    const int64_t row0 = ti * BM, col0 = tj * BN;

    // uniform tile origins (bytes) and per-k-tile steps
    const char *gA = reinterpret_cast<const char *>(g.A + bi * g.sa_batch + (ALAY == KCONTIG ? row0 * g.lda : row0));
    const char *gB = reinterpret_cast<const char *>(g.B + bi * g.sb_batch + (BLAY == KCONTIG ? col0 * g.ldb : col0));
    const int64_t a_step = (ALAY == KCONTIG ? (int64_t)kBK : (int64_t)kBK * g.lda) * 2;
    const int64_t b_step = (BLAY == KCONTIG ? (int64_t)kBK : (int64_t)kBK * g.ldb) * 2;
    const int64_t m_left = g.M - row0, n_left = g.N - col0;
    // Range-checked views of the operands from this program's tile origin on: a buffer access past the operand's end
    // reads as zero instead of faulting.  (Offsets inside a tile's footprint stay below 2^32: the launcher bounds the
    // pitches; the record count saturates for operands that go on for more than 2 GB past the origin.)
    const int64_t a_org = (ALAY == KCONTIG ? row0 * g.lda : row0) * 2, b_org = (BLAY == KCONTIG ? col0 * g.ldb : col0) * 2;
    const int64_t a_rest = g.a_extent - a_org, b_rest = g.b_extent - b_org;
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(gA), 0, (int)(a_rest < 0x7fffffffLL ? a_rest : 0x7fffffffLL), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(gB), 0, (int)(b_rest < 0x7fffffffLL ? b_rest : 0x7fffffffLL), 0x00020000);

    // two sets of staging registers: a tile is requested two trips before it is multiplied
    typename StageSel<BM, ALAY, true>::type sa0, sa1;
    typename StageSel<BN, BLAY, true>::type sb0, sb1;
    sa0.init(tid, g.lda);
    sb0.init(tid, g.ldb);
    sa1.init(tid, g.lda);
    sb1.init(tid, g.ldb);

    // per-lane LDS read bases: row (wave origin + l32) of each operand, chunk hi, swizzled
    const int ra = wave_m * (BM / 2) + l32, rb = wave_n * (BN / 2) + l32;
    const uint32_t a_rd = (uint32_t)(ra * 128 + ((hi ^ ((ra ^ (ra >> 3)) & 7)) << 4));
    const uint32_t b_rd = (uint32_t)(rb * 128 + ((hi ^ ((rb ^ (rb >> 3)) & 7)) << 4)) + B_BASE;

    float16v acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // MFMA operand fragments, double buffered: [slot][32-row block]
    u32x4 fa[2][TM], fb[2][TN];
    constexpr int NM = TM * TN, NR = TM + TN;
    // LDS read r of k step ks of LDS copy `copy`, in the order the MFMAs need the data:
    // A block 0, every B block, then the remaining A blocks
    auto frag_read = [&](int r, int slot, int ks, uint32_t copy) {
        const int t = r == 0 ? 0 : (r <= TN ? r - 1 : r - TN);
        const uint32_t kx = (uint32_t)(((2 * ks) ^ ((t & 1) << 2)) << 4);
        if (r == 0 || r > TN) fa[slot][t] = lds_read16(smem, (a_rd ^ kx) + t * 4096 + copy * A_BYTES);
        else fb[slot][t] = lds_read16(smem, (b_rd ^ kx) + t * 4096 + copy * B_BYTES);
    };
    // One k step: the MFMAs on fragment slot `slot`.  Between them, one at a time: the LDS reads of
    // the next k step's fragments (k step ks_next of copy rcopy, into the other slot) and, if
    // `moving`, the pieces of the tile held in staging set (ha, hb) on their way to LDS copy wcopy.
    // `fetch` (callable or nullptr): called with the MFMA's number after every MFMA, to issue its
    // share of a block's global loads.
    auto kstep = [&](int slot, int ks_next, uint32_t rcopy, auto moving, auto &ha, auto &hb, uint32_t wcopy, auto fetch) {
        constexpr int PA = std::remove_reference_t<decltype(ha)>::PIECES, PB = std::remove_reference_t<decltype(hb)>::PIECES;
        constexpr int PER = (PA + PB + NM - 1) / NM;          // pieces after each MFMA
        constexpr int RQ = (NR + NM - 1) / NM;                // reads after each MFMA, if one per MFMA is not enough
        constexpr int GAP = NM / NR > 0 ? NM / NR : 1;        // otherwise one read after every GAP MFMAs
#pragma unroll
        for (int idx = 0; idx < NM; ++idx) {
            acc[idx / TN][idx % TN] = mfma32<BF16>(fb[slot][idx % TN], fa[slot][idx / TN], acc[idx / TN][idx % TN]);   // transposed block
            if (idx % GAP == 0)
#pragma unroll
                for (int q = 0; q < RQ; ++q)
                    if ((idx / GAP) * RQ + q < NR) frag_read((idx / GAP) * RQ + q, slot ^ 1, ks_next, rcopy);
            if constexpr (decltype(moving)::value) {
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int piece = idx * PER + q;
                    if (piece < PA) ha.store_piece(smem, wcopy * A_BYTES, piece);
                    else if (piece < PA + PB) hb.store_piece(smem, B_BASE + wcopy * B_BYTES, piece - PA);
                }
            }
            if constexpr (!std::is_same_v<decltype(fetch), std::nullptr_t>) fetch(idx);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- prologue: tile 0 -> LDS copy 0 (through set 0), tile 1 requested into set 1
    const int64_t last = g.kt - 1;
    sa0.load(gA, m_left, g.K);
    sb0.load(gB, n_left, g.K);
    if (last > 1) {                                  // tile 1 is not the last: its 64 k lie inside the operands
#pragma unroll
        for (int i = 0; i < decltype(sa1)::PIECES; ++i) sa1.load_piece_buf(rsrc_a, (uint32_t)a_step, i);
#pragma unroll
        for (int i = 0; i < decltype(sb1)::PIECES; ++i) sb1.load_piece_buf(rsrc_b, (uint32_t)b_step, i);
    } else {
        sa1.load(gA + last * a_step, m_left, g.K - last * kBK);
        sb1.load(gB + last * b_step, n_left, g.K - last * kBK);
    }
    sa0.settle();
    sb0.settle();
    sa0.store(smem, 0);
    sb0.store(smem, B_BASE);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) frag_read(r, 0, 0, 0);

    // One k tile (four k steps) per trip.  Trip k multiplies LDS copy k % 2 (tile k).  It requests
    // tile k + 2 (clamped to the last one; surplus copies are never read) into the staging set
    // that trip k - 1 emptied (fa_set / fb_set), before the multiplications: memory latency (about
    // 2 us under load) exceeds one trip.  Tile k + 1, requested a trip earlier into the other set
    // (ha / hb), moves to the idle LDS copy during k step 2; after the barrier that publishes it,
    // k step 3 already reads its first fragments.
    uint32_t cur = 0;
    // mode 1: the requested tile's 64 k lie inside the operands, its rows may not (range-checked buffer
    // loads, no predicates); 2: anything (predicated loads that zero what lies outside, and a fix-up of
    // the vectors that straddle a ragged end).
    auto trip = [&](auto mode_tag, auto &fa_set, auto &fb_set, auto &ha, auto &hb, int64_t k) {
        constexpr int mode = decltype(mode_tag)::value;
        const uint32_t nxt = cur ^ 1u;
        const int64_t kn = k + 2 < last ? k + 2 : last;
        const char *pa = gA + kn * a_step, *pb = gB + kn * b_step;
        if constexpr (mode == 2) {
            fa_set.template load<true>(pa, m_left, g.K - kn * kBK);
            fb_set.template load<true>(pb, n_left, g.K - kn * kBK);
            __builtin_amdgcn_sched_barrier(0);       // the loads stay ahead of the multiplications that hide their latency
            kstep(0, 1, cur, std::false_type{}, ha, hb, nxt, nullptr);
            kstep(1, 2, cur, std::false_type{}, ha, hb, nxt, nullptr);
        } else {
            // requests without predicates go out one at a time between the MFMAs of k steps 0 and 1
            constexpr int PA = std::remove_reference_t<decltype(fa_set)>::PIECES, PB = std::remove_reference_t<decltype(fb_set)>::PIECES;
            const uint32_t oa = (uint32_t)(kn * a_step), ob = (uint32_t)(kn * b_step);
            kstep(0, 1, cur, std::false_type{}, ha, hb, nxt, [&](int idx) {
#pragma unroll
                for (int i = idx * PA / NM; i < (idx + 1) * PA / NM; ++i) fa_set.load_piece_buf(rsrc_a, oa, i);
            });
            kstep(1, 2, cur, std::false_type{}, ha, hb, nxt, [&](int idx) {
#pragma unroll
                for (int i = idx * PB / NM; i < (idx + 1) * PB / NM; ++i) fb_set.load_piece_buf(rsrc_b, ob, i);
            });
        }
        if constexpr (mode == 2) {                   // (trips in modes 0 and 1 only ever hold tiles requested without predicates)
            ha.settle();
            hb.settle();
        }
        kstep(0, 3, cur, std::true_type{}, ha, hb, nxt, nullptr);
        __syncthreads();
        kstep(1, 0, nxt, std::false_type{}, ha, hb, nxt, nullptr);
        cur = nxt;
    };
    // Every k tile but the last ones is requested with range-checked loads (trip k requests tile
    // k + 2), by programs on the ragged m / n edge as well; the last k tiles mask.  Trips come in
    // pairs so that the roles of the two staging sets are fixed at compile time.
    int64_t k = 0;
    typedef std::integral_constant<int, 1> Ranged;
    typedef std::integral_constant<int, 2> Masked;
    for (; k + 1 <= g.kt - 4; k += 2) {
        trip(Ranged{}, sa0, sb0, sa1, sb1, k);
        trip(Ranged{}, sa1, sb1, sa0, sb0, k + 1);
    }
    for (; k + 1 < g.kt; k += 2) {
        trip(Masked{}, sa0, sb0, sa1, sb1, k);
        trip(Masked{}, sa1, sb1, sa0, sb0, k + 1);
    }
    if (k < g.kt) trip(Masked{}, sa0, sb0, sa1, sb1, k);
    __syncthreads();                                 // every wavefront is done with the LDS copies: the epilogue reuses them

    // ---- epilogue: convert and store (masked on ragged tiles)
    store_tile<BM, BN, true>(g, smem, wave, bi, acc, row0 + wave_m * (BM / 2), col0 + wave_n * (BN / 2), lane, m_left < BM || n_left < BN);
}

// ------------------------------------------------------------------ host launch helpers
template <int BM, int BN, bool BF16, int ALAY, int BLAY>
static nt_status launch_fast_inst(const FastArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)2 * (BM + BN) * kBK * sizeof(uint16_t);
    auto kern = gemm_fast_kernel<BM, BN, BF16, ALAY, BLAY>;
    static DeviceOnce configured;              // raise the dynamic LDS limit once per instantiation
    if (!configured.done()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured.set();
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_fast_kernel");
}

template <int BM, int BN, bool BF16>
static nt_status launch_fast_t(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s)
{
    if (alay == KCONTIG && blay == MNCONTIG) return launch_fast_inst<BM, BN, BF16, KCONTIG, MNCONTIG>(a, nwg, s);
    if (alay == KCONTIG && blay == KCONTIG) return launch_fast_inst<BM, BN, BF16, KCONTIG, KCONTIG>(a, nwg, s);
    if (alay == MNCONTIG && blay == MNCONTIG) return launch_fast_inst<BM, BN, BF16, MNCONTIG, MNCONTIG>(a, nwg, s);
    return launch_fast_inst<BM, BN, BF16, MNCONTIG, KCONTIG>(a, nwg, s);
}

// one translation unit per tile shape and input format defines these (parallel compilation)
#define NT_FAST_DECL(T) \
    nt_status launch_fast_##T##_f16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s); \
    nt_status launch_fast_##T##_bf16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s);
NT_FAST_DECL(128x128)
NT_FAST_DECL(256x128)
NT_FAST_DECL(128x256)
NT_FAST_DECL(256x256)
#undef NT_FAST_DECL

}  // namespace nt
