// Direct kernel on 16 x 16 x 32 matrix instructions: full tiles of 16-byte aligned, unit-stride operands.
//
// One workgroup (4 wavefronts, 2 x 2) computes one BM x BN output tile (one program of the tile-to-program mapping,
// Section 3.2.1).  The blocks of A and B that the program multiplies (source-to-target mapping, Section 3.2.2) travel
// from global memory straight into LDS (16 bytes per lane, no staging registers) in slices of 32 k (each 64-wide k tile
// of the arrangement is two such slices).  LDS holds a ring of three or four slices per operand (see ring_of), so a
// slice is requested two or three slice-times before it is multiplied: long enough to cover an L2 miss.
//
// The matrix instruction is v_mfma_f32_16x16x32: it multiplies a 16 x 32 block by a 32 x 16 block, so one instruction
// consumes a whole 32-k slice of its two 16-row fragments, and a wavefront's (BM/2) x (BN/2) part of the tile is
// (BM/32) x (BN/32) accumulator blocks of 4 registers each.  Measured on this part with operands of the benchmark's
// distribution and nothing else running, a wavefront-per-SIMD loop of these instructions sustains 1.85 PFLOP/s against
// 1.60 PFLOP/s for v_mfma_f32_32x32x16 (both reach 2.4 with all-zero operands): the chip is power managed, the narrower
// instruction moves fewer accumulator bits per flop, and the difference is clock.
//
// One trip of the loop = one slice.  A trip multiplies the fragments of slice s (all in registers, read during the
// trip before) while it reads the fragments of slice s+1 into the other register set and requests slice s+ring
// into the ring position that slice s has just left; one barrier per trip, at its top, says that slice s+1 has
// landed in LDS and that nobody reads slice s there any more.
//
// Fragment layouts.  Lane l of a wavefront supplies row (or column) l % 16 of its fragment and the 8 consecutive
// k 8 (l / 16) .. + 7.
//   k-major slice  [row][32 k], 64 bytes per row, 16-byte chunk c of row r stored at chunk c ^ ((-(r / 4)) & 3): one
//            ds_read_b128 per fragment, conflict free (see DirectTile16<E, KCONTIG>::swizzle).
//   mn-major slice [k][E], chunk c of k row k stored at chunk c ^ (4 (k & 3) + 2 ((k / 8) & 1)): two transposing
//            reads (ds_read_b64_tr_b16) per fragment, each of which turns a 4 (k) x 16 (m / n) patch per quarter
//            wavefront into 4 consecutive k per lane; the four 32-byte row segments of a quarter wavefront g (k rows
//            8 g .. 8 g + 3) fall into the four 64-byte quarters of the 256 bytes, those of quarter wavefront g + 1
//            into the other halves of the same quarters.  (With the four segments of a quarter wavefront in two
//            64-byte quarters the counters show one conflict cycle in three.)
// The matrix instructions are issued through inline assembly with the accumulator tied to the destination (the
// compiler's own choice for this instruction copies accumulators between registers inside the loop).
#pragma once
#include "gemm_direct.h"

namespace nt {

typedef float float4v __attribute__((ext_vector_type(4)));

template <bool BF16>
__device__ __forceinline__ void mfma16(float4v &acc, const u32x4 &a, const u32x4 &b)
{
    if constexpr (BF16) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

template <int E, int LAY>
struct DirectTile16;

// ---- k-major slice: E rows (m or n) x 32 k
template <int E>
struct DirectTile16<E, KCONTIG> {
    static constexpr uint32_t BYTES = E * kSliceK * 2;
    static constexpr int PER = BYTES / 1024 / 4;           // load instructions per wavefront and slice
    static constexpr int RPF = 1;                          // LDS reads per operand fragment
    static constexpr int T = E / 32;                       // 16-row fragments per wavefront
    uint32_t voff[PER];                                    // global byte offset of this lane's chunk
    uint32_t rd;                                           // LDS read base of this lane

    // Chunk c of row r is stored at chunk c ^ swizzle(r).  A ds_read_b128 is served in four cycles, 16 lanes each, and the
    // 16 lanes are not consecutive ones: within either half of the wavefront the eight groups of four lanes are split by
    // the parity of their group number's bits (groups 0, 3, 5, 6 and groups 1, 2, 4, 7; found with a one-wavefront probe
    // and the bank-conflict counter).  In a fragment read, lane group q holds rows 4 (q % 4) .. + 3 and k chunk q / 4: a
    // cycle sees row groups {0, 3} with one chunk and {1, 2} with the next, so the four must land in four different
    // 16-byte columns: swizzle = (-(r / 4)) % 4.
    static __device__ __forceinline__ int swizzle(int row) { return (4 - ((row >> 2) & 3)) & 3; }

    __device__ __forceinline__ void init(int wave, int lane, int64_t ld, int wave_origin, uint32_t region)
    {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int row = (wave * PER + j) * 16 + (lane >> 2);
            const int c = (lane & 3) ^ swizzle(row);
            voff[j] = ((uint32_t)row * (uint32_t)ld + (uint32_t)(c * 8)) * 2u;
        }
        const int r = wave_origin + (lane & 15);           // (wave_origin is a multiple of 16: fragment t is rows r + 16 t, same swizzle bits)
        rd = (uint32_t)(r * 64 + (((lane >> 4) ^ swizzle(r)) << 4)) + region;
    }
    __device__ __forceinline__ void issue_one(int j, const char *g, uint32_t lds_slice, int wave) const
    {
        dma16(g, voff[j], lds_slice + (uint32_t)((wave * PER + j) * 1024));
    }
    __device__ __forceinline__ void issue_one_buf(int j, u32x4 rsrc, uint32_t soff, uint32_t lds_slice, int wave) const
    {
        dma16_buf(rsrc, voff[j], soff, lds_slice + (uint32_t)((wave * PER + j) * 1024));
    }
    // where element (row r, k kk) of a slice lies in it (byte offset), and which wavefront's load brings it in
    static __device__ __forceinline__ uint32_t place(int r, int kk)
    {
        return (uint32_t)((r >> 4) * 1024 + (((r & 15) << 2) + ((kk >> 3) ^ swizzle(r))) * 16 + (kk & 7) * 2);
    }
    static __device__ __forceinline__ int owner(int r, int) { return (r >> 4) / PER; }
    // Ragged K: the slice that has just landed at byte offset slot_off holds only `keep` valid k (< 32); what this
    // lane fetched past them -- the beginning of the operand's next row -- is overwritten with zeros.
    __device__ __forceinline__ void zero_tail(char *smem, uint32_t slot_off, int wave, int lane, int keep) const
    {
        const int left = keep - 8 * ((lane & 3) ^ swizzle(lane >> 2));     // valid k in this lane's chunks (the same chunk column for all of them)
        if (left >= 8) return;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const uint32_t at = slot_off + (uint32_t)((wave * PER + j) * 1024 + lane * 16);
            u32x4 v = lds_read16(smem, at);
#pragma unroll
            for (int w = 0; w < 4; ++w) v[w] &= left > 2 * w + 1 ? 0xffffffffu : (left > 2 * w ? 0x0000ffffu : 0u);
            lds_write16(smem, at, v);
        }
    }
    // read q of the slice at byte offset slice_off: fragment q, whole
    __device__ __forceinline__ void read(u32x4 (&f)[T], const char *smem, int q, uint32_t slice_off) const
    {
        f[q] = lds_read16(smem, rd + slice_off + q * 1024);
    }
};

// ---- mn-major slice: 32 k rows x E (m or n)
template <int E>
struct DirectTile16<E, MNCONTIG> {
    static constexpr uint32_t BYTES = E * kSliceK * 2;
    static constexpr int PER = BYTES / 1024 / 4;
    static constexpr int RPF = 2;
    static constexpr int RB = 2 * E;                       // bytes per k row
    static constexpr int CPR = E / 8;                      // 16-byte chunks per k row
    static constexpr int RPI = 1024 / RB;                  // k rows per load instruction
    static constexpr int T = E / 32;
    uint32_t voff[PER];
    uint32_t rd[T];

    static __device__ __forceinline__ int swizzle(int krow) { return ((krow & 3) << 2) | (((krow >> 3) & 1) << 1); }

    __device__ __forceinline__ void init(int wave, int lane, int64_t ld, int wave_origin, uint32_t region)
    {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int krow = (wave * PER + j) * RPI + lane / CPR;
            const int c = (lane % CPR) ^ swizzle(krow);
            voff[j] = ((uint32_t)krow * (uint32_t)ld + (uint32_t)(c * 8)) * 2u;
        }
        // transposing read: quarter wavefront g covers k rows 8 g .. 8 g + 3 (+ 4 for the second read) and the
        // fragment's 16 columns; lane i of the quarter points at row i / 4, 4 columns starting at 4 (i % 4), and
        // receives 4 consecutive k of column i
        const int g = lane >> 4, i = lane & 15;
        const int kl = 8 * g + (i >> 2);
        const int mn = wave_origin + 4 * (i & 3);
        const int sw = swizzle(kl);                        // the same for kl + 4
#pragma unroll
        for (int t = 0; t < T; ++t)
            rd[t] = (uint32_t)(kl * RB + ((((mn >> 3) + 2 * t) ^ sw) << 4) + ((mn >> 2) & 1) * 8) + region;
    }
    __device__ __forceinline__ void issue_one(int j, const char *g, uint32_t lds_slice, int wave) const
    {
        dma16(g, voff[j], lds_slice + (uint32_t)((wave * PER + j) * 1024));
    }
    __device__ __forceinline__ void issue_one_buf(int j, u32x4 rsrc, uint32_t soff, uint32_t lds_slice, int wave) const
    {
        dma16_buf(rsrc, voff[j], soff, lds_slice + (uint32_t)((wave * PER + j) * 1024));
    }
    // where element (column r along m / n, k row kk) of a slice lies in it, and which wavefront's load brings it in
    static __device__ __forceinline__ uint32_t place(int r, int kk)
    {
        return (uint32_t)((kk / RPI) * 1024 + ((kk % RPI) * CPR + ((r >> 3) ^ swizzle(kk))) * 16 + (r & 7) * 2);
    }
    static __device__ __forceinline__ int owner(int, int kk) { return (kk / RPI) / PER; }
    // (ragged K: the k rows past K lie past the operand's end and arrive as zeros by themselves)
    __device__ __forceinline__ void zero_tail(char *, uint32_t, int, int, int) const {}
    // read q of the slice: half q % 2 (k 0..3 or 4..7 of the lane's run) of fragment q / 2
    __device__ __forceinline__ void read(u32x4 (&f)[T], const char *smem, int q, uint32_t slice_off) const
    {
        typedef short4v __attribute__((address_space(3))) * lds_s4;
        const int t = q >> 1, part = q & 1;
        const u32x2 v = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(smem + (rd[t] + slice_off + (uint32_t)(part * 4 * RB)))));
        f[t][2 * part] = v[0];
        f[t][2 * part + 1] = v[1];
    }
};

// ---- epilogue (output = accumulator, Section 4.2).  Every matrix instruction is issued with the B fragment first,
// so a 16 x 16 accumulator block comes out transposed: a lane holds row m = lane % 16 of the block and its 4
// consecutive columns 4 (lane / 16) .. + 3.  C (and D) have unit stride along n, the tile is full.  The wavefront's
// part goes through its own region of the (idle) LDS so that global stores are whole 256-byte row segments:
//   write phase  per block, alpha / beta * D / activation in fp32 if asked, one conversion, then the lane's 4 values
//                (8 bytes, or one 16-byte chunk of fp32) to [row][256 bytes] with the chunk index XOR-ed with the row
//                (16 rows, same chunk: 16 different chunks);
//   read phase   16 consecutive lanes read one row; a store instruction covers 4 rows of 256 contiguous bytes.
// An fp32 tile takes two passes (one per half of the columns) through the same region.
// CHECK masks rows >= M and columns >= N (a partly valid 16-byte chunk is stored element-wise; D is read element-wise there).
// RP: the wavefront's 128 rows go through the region in RP passes of 128 / RP rows (a region of 32 / RP KB per wavefront:
// the persistent kernel stages through the 32 KB of LDS that its ring leaves free).
// AFFINE: alpha, beta * D or an activation is asked for.  A variant of its own, because the plain product's epilogue must be
// straight-line code: a wavefront-uniform test per accumulator block costs an instruction fetch each, which nothing hides
// with one wavefront per SIMD (measured on the 256 x 256 tile: 5.6 us per program with the tests, 6 % of a 4096-cubed product).
// STREAM: full 16-byte stores carry the non-temporal hint (the output is not read again by the launch and should not push
// the operands out of L2: 18 % on a batch of 32 2048 x 2048 x 512 products); not for the range-checked kernels, whose rows
// need not be 16-byte aligned (there the hint costs more than it saves: partial lines).
template <int BM, int BN, int OUT, bool CHECK, int RP, bool AFFINE, bool STREAM>
__device__ __forceinline__ void store_tile16_rows(char *smem, int wave, char *C, int64_t scm, const float4v (&acc)[BM / 32][BN / 32],
                                                  int64_t row_w, int64_t col_w, int lane, int64_t M, int64_t N, const char *D,
                                                  int64_t sdm, float alpha, float beta, int act)
{
    constexpr int TM = BM / 32, WM = BM / 2, WN = BN / 2;
    constexpr int ES = OUT == NT_F32 ? 4 : 2;
    constexpr int PASSES = ES / 2;                        // an fp32 tile takes one pass per half of the columns
    constexpr int PW = WN / PASSES;                       // columns per pass
    constexpr int RB = WN * 2;                            // bytes per region row: 256 or 128
    constexpr int CPR = RB / 16;                          // 16-byte chunks per row
    constexpr int RSH = RB == 256 ? 0 : 1;                // log2(rows per 256 bytes of LDS)
    constexpr int EPC = 16 / ES;                          // elements per chunk
    constexpr int RPI = 64 / CPR;                         // rows per store instruction
    constexpr int TNP = PW / 16;                          // blocks per pass
    const int l16 = lane & 15, g = lane >> 4;
    const ActParams ap = act_params(act);
    constexpr int TMP = TM / RP, WMP = WM / RP;           // blocks and rows per row pass
    static_assert(TM % RP == 0 && WMP % RPI == 0, "row passes");
    constexpr int NBR = !AFFINE ? 1 : (TMP * TNP <= 8 ? TMP : (TNP >= 8 ? 1 : 8 / TNP));      // rows of blocks per batch of the write phase (8 blocks)
    static_assert(NBR >= 1 && TMP % NBR == 0, "batches of the write phase");
    char *reg = smem + wave * (WMP * RB);
#pragma unroll
    for (int rp = 0; rp < RP; ++rp)
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
        // ---- write phase, NBR rows of blocks (8 blocks) at a time: their accumulators; with AFFINE the loads of D for all of
        // them before the first is waited for, the combination, the activation; the conversions and LDS writes
#pragma unroll
        for (int tb = 0; tb < TMP; tb += NBR) {
            float o[NBR][TNP][4];
#pragma unroll
            for (int i = 0; i < NBR; ++i)
#pragma unroll
                for (int tnp = 0; tnp < TNP; ++tnp) {
                    // (the block is pinned in its accumulator registers up to this point: without this the compiler moves all
                    // 256 accumulators to ordinary registers ahead of the three output formats' code and spills them)
                    float4v blk = acc[rp * TMP + tb + i][pass * TNP + tnp];
                    asm volatile("" : "+a"(blk));
#pragma unroll
                    for (int v = 0; v < 4; ++v) o[i][tnp][v] = blk[v];
                }
            if constexpr (AFFINE) {
                if (D) {                                                  // wavefront-uniform
                    typedef uint32_t raw_t __attribute__((ext_vector_type(ES)));      // the lane's 4 elements of D as stored
                    raw_t w[NBR][TNP];
#pragma unroll
                    for (int i = 0; i < NBR; ++i) {
                        const int64_t row = row_w + rp * WMP + (tb + i) * 16 + l16;
#pragma unroll
                        for (int tnp = 0; tnp < TNP; ++tnp) {
                            const int64_t col = col_w + (pass * TNP + tnp) * 16 + 4 * g;
                            const int64_t nv = CHECK ? N - col : 4;                   // valid columns from the lane's first
                            if (CHECK && (row >= M || nv < 4)) {
                                uint32_t e[4] = {0u, 0u, 0u, 0u};                      // element by element, as 32- or 16-bit patterns
                                if (row < M)
#pragma unroll
                                    for (int v = 0; v < 4; ++v)
                                        if (v < nv) {
                                            if constexpr (ES == 4) e[v] = *reinterpret_cast<const uint32_t *>(D + (row * sdm + col + v) * 4);
                                            else e[v] = *reinterpret_cast<const uint16_t *>(D + (row * sdm + col + v) * 2);
                                        }
                                if constexpr (ES == 4) w[i][tnp] = raw_t{e[0], e[1], e[2], e[3]};
                                else w[i][tnp] = raw_t{e[0] | (e[1] << 16), e[2] | (e[3] << 16)};
                            } else {
                                __builtin_memcpy(&w[i][tnp], D + (row * sdm + col) * ES, 4 * ES);
                            }
                        }
                    }
#pragma unroll
                    for (int i = 0; i < NBR; ++i)
#pragma unroll
                        for (int tnp = 0; tnp < TNP; ++tnp) {
                            float d[4];
                            if constexpr (OUT == NT_F32) {
#pragma unroll
                                for (int v = 0; v < 4; ++v) { const uint32_t x = w[i][tnp][v]; d[v] = __builtin_bit_cast(float, x); }
                            } else {
#pragma unroll
                                for (int v = 0; v < 2; ++v) {
                                    const uint32_t x = w[i][tnp][v];
                                    if constexpr (OUT == NT_F16) {
                                        d[2 * v] = (float)__builtin_bit_cast(_Float16, (uint16_t)(x & 0xffffu));
                                        d[2 * v + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(x >> 16));
                                    } else {
                                        d[2 * v] = __builtin_bit_cast(float, x << 16);
                                        d[2 * v + 1] = __builtin_bit_cast(float, x & 0xffff0000u);
                                    }
                                }
                            }
#pragma unroll
                            for (int v = 0; v < 4; ++v) o[i][tnp][v] = combine(o[i][tnp][v], d[v], alpha, beta);
                        }
                } else {
#pragma unroll
                    for (int i = 0; i < NBR; ++i)
#pragma unroll
                        for (int tnp = 0; tnp < TNP; ++tnp)
#pragma unroll
                            for (int v = 0; v < 4; ++v) o[i][tnp][v] = combine(o[i][tnp][v], 0.f, alpha, beta);
                }
                if (act) {                                                // wavefront-uniform
#pragma unroll
                    for (int i = 0; i < NBR; ++i)
#pragma unroll
                        for (int tnp = 0; tnp < TNP; ++tnp)
#pragma unroll
                            for (int v = 0; v < 4; ++v) o[i][tnp][v] = activate(o[i][tnp][v], ap);
                }
            }
#pragma unroll
            for (int i = 0; i < NBR; ++i) {
                const int r = (tb + i) * 16 + l16;
                const int sw = (r >> RSH) & (CPR - 1);
                char *prow = reg + r * RB;
#pragma unroll
                for (int tnp = 0; tnp < TNP; ++tnp) {
                    const float *ov = o[i][tnp];
                    if constexpr (OUT == NT_F32) {
                        const int c = tnp * 4 + g;
                        lds_write16(prow, (uint32_t)((c ^ sw) << 4), u32x4{__builtin_bit_cast(uint32_t, ov[0]), __builtin_bit_cast(uint32_t, ov[1]),
                                                                            __builtin_bit_cast(uint32_t, ov[2]), __builtin_bit_cast(uint32_t, ov[3])});
                    } else {
                        const int c = tnp * 2 + (g >> 1);
                        *reinterpret_cast<u32x2 *>(prow + (((c ^ sw) << 4) + 8 * (g & 1))) =
                            u32x2{pack_pair<OUT>(__builtin_bit_cast(uint32_t, ov[0]), __builtin_bit_cast(uint32_t, ov[1])),
                                  pack_pair<OUT>(__builtin_bit_cast(uint32_t, ov[2]), __builtin_bit_cast(uint32_t, ov[3]))};
                    }
                }
            }
        }
        // ---- read phase (same wavefront: LDS operations complete in order)
#pragma unroll
        for (int it = 0; it < WMP / RPI; ++it) {
            const int r = it * RPI + lane / CPR, c = lane % CPR;
            const u32x4 v = lds_read16(reg, (uint32_t)(r * RB + ((c ^ ((r >> RSH) & (CPR - 1))) << 4)));
            const int64_t row = row_w + rp * WMP + r, col = col_w + pass * PW + c * EPC;
            char *p = C + (row * scm + col) * ES;
            if (!CHECK || (row < M && col + EPC <= N)) {
                // (streamed where rows are 16-byte aligned: the output is not read again by this launch and should not
                // push the operands out of L2)
                if constexpr (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
                else __builtin_memcpy(p, &v, 16);
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

template <int BM, int BN, bool EDGE = false, int RP = 1>
__device__ __forceinline__ void store_tile16(const FastArgs &g, char *smem, int wave, int64_t bi, const float4v (&acc)[BM / 32][BN / 32],
                                             int64_t row_w, int64_t col_w, int lane, bool ragged = false)
{
    const int64_t esz = g.out_dtype == NT_F32 ? 4 : 2;
    char *C = reinterpret_cast<char *>(g.C) + bi * g.sc_batch * esz;
    const char *D = g.D ? reinterpret_cast<const char *>(g.D) + bi * g.sd_batch * esz : nullptr;
    const bool affine = D != nullptr || g.alpha != 1.f || g.act != 0;
    // (the plain product's path is straight-line code: with one wavefront per SIMD nothing hides an instruction fetch that
    // a branch per accumulator block would cost)
#define NT_ROWS16(OUT, CHECK) do { \
        if (affine) store_tile16_rows<BM, BN, OUT, CHECK, RP, true, !EDGE>(smem, wave, C, g.scm, acc, row_w, col_w, lane, g.M, g.N, D, g.sdm, g.alpha, g.beta, g.act); \
        else store_tile16_rows<BM, BN, OUT, CHECK, RP, false, !EDGE>(smem, wave, C, g.scm, acc, row_w, col_w, lane, g.M, g.N, D, g.sdm, g.alpha, g.beta, g.act); \
    } while (0)
    if constexpr (EDGE) {
        if (ragged) {
            if (g.out_dtype == NT_F32) NT_ROWS16(NT_F32, true);
            else if (g.out_dtype == NT_F16) NT_ROWS16(NT_F16, true);
            else NT_ROWS16(NT_BF16, true);
            return;
        }
    }
    if (g.out_dtype == NT_F32) NT_ROWS16(NT_F32, false);
    else if (g.out_dtype == NT_F16) NT_ROWS16(NT_F16, false);
    else NT_ROWS16(NT_BF16, false);
#undef NT_ROWS16
}

// EDGE = false: every tile is full, every load 16-byte aligned, K a whole number of 64-k tiles.  EDGE = true: tiles may
// overhang M or N, K need not be a whole number of slices, rows need only the element's own 2-byte alignment: the operand
// loads are range checked (what lies past an operand's end reads as zero, what an overhanging tile reads inside it only
// reaches outputs that are never stored, except the k past K of a k-contiguous operand, which are zeroed in LDS) and the
// stores are masked.
// TRACE: not a product at all.  One workgroup sets itself up as program g.trace_program, requests that program's 32-k slice
// g.trace_slice with the very loads of the kernel (swizzle, range check), applies what the kernel applies to a slice once
// it has landed, and copies one operand's slice out of LDS in (row, k) order: the source-to-target mapping (Section 3.2.2)
// as this kernel's loader executes it, for a caller who has filled the operand with the elements' own indices.
template <int BM, int BN, bool BF16, int ALAY, int BLAY, bool EDGE, bool TRACE = false>
__global__ __launch_bounds__(kThreads, residency_of(BM, BN)) void gemm_direct16_kernel(const FastArgs g)
{
    constexpr int TM = BM / 32, TN = BN / 32;
    constexpr int kRing = ring_of(BM, BN);
    using TileA = DirectTile16<BM, ALAY>;
    using TileB = DirectTile16<BN, BLAY>;
    constexpr uint32_t A_BYTES = TileA::BYTES, B_BYTES = TileB::BYTES, B_BASE = kRing * A_BYTES;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int64_t bi, ti, tj;
    if constexpr (TRACE) {
        bi = g.trace_program / (g.mt * g.nt);
        ti = (g.trace_program - bi * g.mt * g.nt) / g.nt;
        tj = g.trace_program % g.nt;
    } else {
        locate_program(g.mt, g.nt, &bi, &ti, &tj);
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int64_t row0 = ti * BM, col0 = tj * BN;

    const char *gA = reinterpret_cast<const char *>(g.A + bi * g.sa_batch + (ALAY == KCONTIG ? row0 * g.lda : row0));
    const char *gB = reinterpret_cast<const char *>(g.B + bi * g.sb_batch + (BLAY == KCONTIG ? col0 * g.ldb : col0));
    const int64_t a_step = (ALAY == KCONTIG ? (int64_t)kSliceK : (int64_t)kSliceK * g.lda) * 2;
    const int64_t b_step = (BLAY == KCONTIG ? (int64_t)kSliceK : (int64_t)kSliceK * g.ldb) * 2;
    // (EDGE: K need not be a whole number of slices; the tail of the last one is zeroed in LDS, see zero_tail)
    const int64_t n_slices = EDGE ? (g.K + kSliceK - 1) / kSliceK : g.kt * (kBK / kSliceK);

    TileA ta;
    TileB tb;
    ta.init(wave, lane, g.lda, wave_m * (BM / 2), 0);
    tb.init(wave, lane, g.ldb, wave_n * (BN / 2), B_BASE);

    float4v acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.f;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    // operand fragments of one slice, two sets: [set][fragment]
    u32x4 fa[2][TM], fb[2][TN];
    constexpr int NRA = TM * TileA::RPF, NRB = TN * TileB::RPF, NR = NRA + NRB;   // LDS reads per slice
    // LDS read r of a slice, in the order the next trip's matrix instructions need the data:
    // A fragment 0, every B fragment, then the remaining A fragments
    auto lds_read = [&](int r, int set, uint32_t ring) {
        if (r < TileA::RPF) ta.read(fa[set], smem, r, ring * A_BYTES);
        else if (r < TileA::RPF + NRB) tb.read(fb[set], smem, r - TileA::RPF, ring * B_BYTES);
        else ta.read(fa[set], smem, r - NRB, ring * A_BYTES);
    };
    constexpr int NM = TM * TN, ND = TileA::PER + TileB::PER;
    u32x4 rsrc_a{0, 0, 0, 0}, rsrc_b{0, 0, 0, 0};
    if constexpr (EDGE) {
        rsrc_a = make_rsrc(gA, g.a_extent - (gA - reinterpret_cast<const char *>(g.A + bi * g.sa_batch)));
        rsrc_b = make_rsrc(gB, g.b_extent - (gB - reinterpret_cast<const char *>(g.B + bi * g.sb_batch)));
    }
    auto dma = [&](int d, const char *pa, const char *pb, uint32_t ring) {
        if constexpr (!EDGE) {
            if (d < TileA::PER) ta.issue_one(d, pa, lds0 + ring * A_BYTES, wave);
            else tb.issue_one(d - TileA::PER, pb, lds0 + B_BASE + ring * B_BYTES, wave);
        } else {
            if (d < TileA::PER) ta.issue_one_buf(d, rsrc_a, (uint32_t)(pa - gA), lds0 + ring * A_BYTES, wave);
            else tb.issue_one_buf(d - TileA::PER, rsrc_b, (uint32_t)(pb - gB), lds0 + B_BASE + ring * B_BYTES, wave);
        }
    };
    // One trip: the TM x TN matrix instructions on fragment set `set`; between them, spread evenly so that neither
    // the LDS queue nor the memory queue holds the in-order wavefront back while the matrix pipe runs dry, the LDS
    // reads of the next slice (ring position rring) into the other set and the ND global -> LDS loads of the slice
    // at (pa, pb) into ring position dring.
    auto trip = [&](int set, uint32_t rring, const char *pa, const char *pb, uint32_t dring) {
        constexpr int RS = NM * 3 / 4;                      // the reads go out during the first three quarters: all have returned by the next barrier
#pragma unroll
        for (int idx = 0; idx < NM; ++idx) {
            const int tm = idx / TN, tn = idx % TN;
            mfma16<BF16>(acc[tm][tn], fb[set][tn], fa[set][tm]);      // transposed block (see store_tile16_rows)
            if (idx < RS)
#pragma unroll
                for (int r = idx * NR / RS; r < (idx + 1) * NR / RS; ++r) lds_read(r, set ^ 1, rring);
#pragma unroll
            for (int d = idx * ND / NM; d < (idx + 1) * ND / NM; ++d) dma(d, pa, pb, dring);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    const int64_t last = n_slices - 1;
    // The range check of a buffer load works on the load's 4-byte words: with an odd pitch or extent the word that holds an
    // operand's very last element can end 2 bytes past the operand, and then arrives as zero.  The wavefront whose load
    // brings that word in fetches the element by itself (a 2-byte load inside the operand) and puts it in its place once
    // the last slice has landed (g.patch: bit 0 = A, bit 1 = B; set by the host for such operands only).
    int patch_a = -1, patch_b = -1;
    if constexpr (EDGE) {
        const int kk = (int)(g.K - 1 - last * kSliceK);
        const int64_t ra = g.M - 1 - row0, rb = g.N - 1 - col0;
        if ((g.patch & 1) && ra < BM && TileA::owner((int)ra, kk) == wave) patch_a = (int)TileA::place((int)ra, kk);
        if ((g.patch & 2) && rb < BN && TileB::owner((int)rb, kk) == wave) patch_b = (int)TileB::place((int)rb, kk);
    }
    // what has to happen to slice `s`, which has just landed at ring position `pos` (this wavefront's part), before the
    // barrier that publishes it: only the last slice of a ragged or odd-sized problem needs anything
    auto settle = [&](int64_t s, uint32_t pos) {
        if constexpr (EDGE) {
            if (s != last) return;
            if ((s + 1) * kSliceK > g.K) {
                const int keep = (int)(g.K - s * kSliceK);
                ta.zero_tail(smem, pos * A_BYTES, wave, lane, keep);
                tb.zero_tail(smem, B_BASE + pos * B_BYTES, wave, lane, keep);
            }
            if (g.patch && lane == 0) {
                if (patch_a >= 0)
                    *reinterpret_cast<uint16_t *>(smem + pos * A_BYTES + patch_a) =
                        *reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(g.A + bi * g.sa_batch) + g.a_extent - 2);
                if (patch_b >= 0)
                    *reinterpret_cast<uint16_t *>(smem + B_BASE + pos * B_BYTES + patch_b) =
                        *reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(g.B + bi * g.sb_batch) + g.b_extent - 2);
            }
        }
    };
    // Slices past the last one are requested all the same (the loop has one shape).  Full tiles: the last slice again, never
    // multiplied.  EDGE: an offset beyond any buffer (2^31; the lanes' own offsets stay below 2^31), so that zeros arrive:
    // an odd number of slices is rounded up to whole passes of the loop below by one trip that multiplies zeros.
    auto slice_a = [&](int64_t s) { return gA + (s <= last ? s * a_step : (EDGE ? (int64_t)0x80000000LL : last * a_step)); };
    auto slice_b = [&](int64_t s) { return gB + (s <= last ? s * b_step : (EDGE ? (int64_t)0x80000000LL : last * b_step)); };

    if constexpr (TRACE) {
        const int64_t s = g.trace_slice;
#pragma unroll
        for (int d = 0; d < ND; ++d) dma(d, slice_a(s), slice_b(s), 0);
        NT_WAIT_VMCNT(0);
        settle(s, 0);
        __syncthreads();
        const bool first = g.trace_operand == 0;
        for (int e = tid; e < (first ? BM : BN) * kSliceK; e += kThreads) {
            const uint32_t at = first ? TileA::place(e / kSliceK, e % kSliceK) : B_BASE + TileB::place(e / kSliceK, e % kSliceK);
            g.trace_out[e] = *reinterpret_cast<const uint16_t *>(smem + at);
        }
        return;
    }
    // prologue: slices 0 .. kRing-1 requested; wait for slice 0; its fragments into set 0
#pragma unroll
    for (int s = 0; s < kRing; ++s)
#pragma unroll
        for (int d = 0; d < ND; ++d) dma(d, slice_a(s), slice_b(s), s);
    NT_WAIT_VMCNT((kRing - 1) * ND);
    settle(0, 0);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) lds_read(r, 0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // Slice s sits at ring position s % kRing.  At the top of trip s this wavefront's part of slice s+1 must have
    // landed (the loads of the younger slices may still be in flight); the barrier then says that slice s+1 is
    // complete and that every wavefront holds its fragments of slice s in registers, so the position of slice s can
    // be overwritten by slice s+kRing.  Two trips per pass (the fragment sets alternate).
    uint32_t ring = 0;
    for (int64_t sl = 0; sl < n_slices; sl += 2) {
        uint32_t nxt = ring + 1 == kRing ? 0 : ring + 1;
        NT_WAIT_VMCNT((kRing - 2) * ND);
        settle(sl + 1, nxt);
        __syncthreads();
        trip(0, nxt, slice_a(sl + kRing), slice_b(sl + kRing), ring);
        ring = nxt;
        nxt = ring + 1 == kRing ? 0 : ring + 1;
        NT_WAIT_VMCNT((kRing - 2) * ND);
        settle(sl + 2, nxt);
        __syncthreads();
        trip(1, nxt, slice_a(sl + 1 + kRing), slice_b(sl + 1 + kRing), ring);
        ring = nxt;
    }
    NT_WAIT_VMCNT(0);                                      // drain the surplus prefetches ...
    __syncthreads();                                       // ... of every wavefront: the epilogue reuses the LDS
    // The accumulators are read by ordinary instructions from here on, and the compiler does not know that the inline
    // assembly above is a matrix instruction whose result needs wait states before it can be read: 16 wait states
    // here, and the epilogue takes every accumulator block through an assembly statement of its own before it reads
    // it (statements of this kind stay in program order, so every read follows the wait states).
    asm volatile("s_nop 15" ::: "memory");

    store_tile16<BM, BN, EDGE>(g, smem, wave, bi, acc, row0 + wave_m * (BM / 2), col0 + wave_n * (BN / 2), lane,
                               EDGE && (g.M - row0 < BM || g.N - col0 < BN));
}

// ---- the same kernel with the ring unrolled, for the 256 x 256 tile (ring of four).
// A wavefront is alone on its SIMD, so every instruction it issues costs the SIMD one issue turn (4 cycles) and only
// three fit behind a 16-cycle matrix instruction.  With the ring position a compile-time constant, every LDS read is a
// per-lane base plus an immediate offset and every LDS target of a global -> LDS load a precomputed scalar (no address
// arithmetic in the loop).  At most two other instructions follow any matrix instruction.
// EDGE = false (full tiles of aligned operands, a whole number of 128-k steps): plain loads; the global pointers advance by
// one scalar addition per slice and operand; no clamping per load: the last pass of the loop, which has nothing left to
// request, fetches the last slice again.
// EDGE = true (see gemm_direct16_kernel): range-checked loads at a scalar offset per slice and operand; slices past the last
// are requested at an offset beyond any buffer, arrive as zeros, and their trips add nothing (any number of slices is
// rounded up to whole passes); the last slice's ragged tail and the operand's last odd element are put right once it has
// landed, behind one uniform test per trip.
template <int BM, int BN, bool BF16, int ALAY, int BLAY, bool EDGE = false>
__global__ __launch_bounds__(kThreads, residency_of(BM, BN)) void gemm_direct16u_kernel(const FastArgs g)
{
    constexpr int TM = BM / 32, TN = BN / 32;
    constexpr int kRing = 4;
    static_assert(ring_of(BM, BN) == kRing, "ring of four");
    using TileA = DirectTile16<BM, ALAY>;
    using TileB = DirectTile16<BN, BLAY>;
    constexpr uint32_t A_BYTES = TileA::BYTES, B_BYTES = TileB::BYTES, B_BASE = kRing * A_BYTES;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int64_t bi, ti, tj;
    locate_program(g.mt, g.nt, &bi, &ti, &tj);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int64_t row0 = ti * BM, col0 = tj * BN;

    const char *pa = reinterpret_cast<const char *>(g.A + bi * g.sa_batch + (ALAY == KCONTIG ? row0 * g.lda : row0));
    const char *pb = reinterpret_cast<const char *>(g.B + bi * g.sb_batch + (BLAY == KCONTIG ? col0 * g.ldb : col0));
    const int64_t a_step = (ALAY == KCONTIG ? (int64_t)kSliceK : (int64_t)kSliceK * g.lda) * 2;
    const int64_t b_step = (BLAY == KCONTIG ? (int64_t)kSliceK : (int64_t)kSliceK * g.ldb) * 2;
    // (full tiles: a multiple of 4, at least 4, checked by the host)
    const int64_t n_slices = EDGE ? (g.K + kSliceK - 1) / kSliceK : g.kt * (kBK / kSliceK);
    const int32_t last = (int32_t)n_slices - 1;

    TileA ta;
    TileB tb;
    ta.init(wave, lane, g.lda, wave_m * (BM / 2), 0);
    tb.init(wave, lane, g.ldb, wave_n * (BN / 2), B_BASE);

    float4v acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.f;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    constexpr int NRA = TM * TileA::RPF, NRB = TN * TileB::RPF, NR = NRA + NRB;   // LDS reads per slice
    constexpr int NM = TM * TN, ND = TileA::PER + TileB::PER;
    static_assert(2 * NR <= NM * 3 / 2 && 8 * ND <= NM, "the trip's schedule: a read every other matrix instruction, a load every eighth");

    // LDS targets of this wavefront's loads, per ring position: scalars
    uint32_t tgt[kRing][ND];
#pragma unroll
    for (int r = 0; r < kRing; ++r)
#pragma unroll
        for (int d = 0; d < ND; ++d)
            tgt[r][d] = d < TileA::PER ? lds0 + r * A_BYTES + (uint32_t)((wave * TileA::PER + d) * 1024)
                                       : lds0 + B_BASE + r * B_BYTES + (uint32_t)((wave * TileB::PER + d - TileA::PER) * 1024);

    // EDGE: range-checked views of the operands from this program's tile origin on, the scalar offsets of the slice that is
    // requested next (slice `rq`), and the one element that the range check may have dropped (see gemm_direct16_kernel)
    u32x4 rsrc_a{0, 0, 0, 0}, rsrc_b{0, 0, 0, 0};
    uint32_t rq_aoff = 0, rq_boff = 0;
    int32_t rq = 0;
    int patch_a = -1, patch_b = -1;
    if constexpr (EDGE) {
        rsrc_a = make_rsrc(pa, g.a_extent - (pa - reinterpret_cast<const char *>(g.A + bi * g.sa_batch)));
        rsrc_b = make_rsrc(pb, g.b_extent - (pb - reinterpret_cast<const char *>(g.B + bi * g.sb_batch)));
        const int kk = (int)(g.K - 1 - (int64_t)last * kSliceK);
        const int64_t ra = g.M - 1 - row0, rb = g.N - 1 - col0;
        if ((g.patch & 1) && ra < BM && TileA::owner((int)ra, kk) == wave) patch_a = (int)TileA::place((int)ra, kk);
        if ((g.patch & 2) && rb < BN && TileB::owner((int)rb, kk) == wave) patch_b = (int)TileB::place((int)rb, kk);
    }
    auto aim_request = [&]() {                               // (after a change of rq)
        const bool live = rq <= last;                          // (uniform)
        rq_aoff = live ? (uint32_t)rq * (uint32_t)a_step : 0x80000000u;
        rq_boff = live ? (uint32_t)rq * (uint32_t)b_step : 0x80000000u;
    };
    // what the last slice needs once this wavefront's part of it has landed at ring position `pos`
    auto settle_last = [&](uint32_t pos) {
        if ((int64_t)(last + 1) * kSliceK > g.K) {
            const int keep = (int)(g.K - (int64_t)last * kSliceK);
            ta.zero_tail(smem, pos * A_BYTES, wave, lane, keep);
            tb.zero_tail(smem, B_BASE + pos * B_BYTES, wave, lane, keep);
        }
        if (g.patch && lane == 0) {
            if (patch_a >= 0)
                *reinterpret_cast<uint16_t *>(smem + pos * A_BYTES + patch_a) =
                    *reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(g.A + bi * g.sa_batch) + g.a_extent - 2);
            if (patch_b >= 0)
                *reinterpret_cast<uint16_t *>(smem + B_BASE + pos * B_BYTES + patch_b) =
                    *reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(g.B + bi * g.sb_batch) + g.b_extent - 2);
        }
    };

    u32x4 fa[2][TM], fb[2][TN];
    auto lds_read = [&](int r, int set, uint32_t ring) {
        if (r < TileA::RPF) ta.read(fa[set], smem, r, ring * A_BYTES);
        else if (r < TileA::RPF + NRB) tb.read(fb[set], smem, r - TileA::RPF, ring * B_BYTES);
        else ta.read(fa[set], smem, r - NRB, ring * A_BYTES);
    };
    // load d of the slice at (pa, pb) / at the request offsets into ring position `ring`, in two halves that go behind
    // different matrix instructions (the matrix instruction between them is the wait state the hardware wants after a
    // write to m0)
    auto dma_aim = [&](int d, int ring) { asm volatile("s_mov_b32 m0, %0" : : "s"(tgt[ring][d]) : "memory"); };
    auto dma_go = [&](int d) {
        if constexpr (EDGE) {
            if (d < TileA::PER) asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" : : "v"(ta.voff[d]), "s"(rsrc_a), "s"(rq_aoff) : "memory");
            else asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" : : "v"(tb.voff[d - TileA::PER]), "s"(rsrc_b), "s"(rq_boff) : "memory");
        } else {
            if (d < TileA::PER) asm volatile("global_load_lds_dwordx4 %0, %1" : : "v"(ta.voff[d]), "s"(pa) : "memory");
            else asm volatile("global_load_lds_dwordx4 %0, %1" : : "v"(tb.voff[d - TileA::PER]), "s"(pb) : "memory");
        }
    };

    // One trip = one slice: the matrix instructions on fragment set SET (slice s); behind them the LDS reads of slice
    // s+1 (ring position RING+1) into the other set and the loads of slice s+4 into ring position RING.
    auto trip = [&](auto ring_c, auto set_c, int64_t a_adv, int64_t b_adv) {
        constexpr int RING = decltype(ring_c)::value, SET = decltype(set_c)::value;
        constexpr int NXT = (RING + 1) % kRing;
#pragma unroll
        for (int idx = 0; idx < NM; ++idx) {
            const int tm = idx / TN, tn = idx % TN;
            mfma16<BF16>(acc[tm][tn], fb[SET][tn], fa[SET][tm]);      // transposed block (see store_tile16_rows)
            if (idx % 2 == 0 && idx / 2 < NR) lds_read(idx / 2, SET ^ 1, NXT);
            if (EDGE && idx == 0) { ++rq; aim_request(); }
            if (idx % 8 == 1 && idx / 8 < ND) dma_aim(idx / 8, RING);
            if (idx % 8 == 3 && idx / 8 < ND) {
                dma_go(idx / 8);
                if constexpr (!EDGE) {
                    // the operand's last load of this trip is out: its pointer moves on to the next slice
                    if (idx / 8 == TileA::PER - 1) { pa += a_adv; asm volatile("" : "+s"(pa)); }
                    if (idx / 8 == ND - 1) { pb += b_adv; asm volatile("" : "+s"(pb)); }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using std::integral_constant;

    // prologue: slices 0 .. 3 requested; wait for slice 0; its fragments into set 0
#pragma unroll
    for (int s = 0; s < kRing; ++s) {
        if constexpr (EDGE) { rq = s; aim_request(); }
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            dma_aim(d, s);
            asm volatile("s_nop 0");
            dma_go(d);
        }
        pa += a_step;
        pb += b_step;
    }
    asm volatile("" : "+s"(pa), "+s"(pb));
    NT_WAIT_VMCNT((kRing - 1) * ND);
    if constexpr (EDGE) {
        if (last == 0) settle_last(0);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) lds_read(r, 0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // Slice s sits at ring position s % 4.  At the top of trip s this wavefront's part of slice s+1 must have landed
    // (the loads of the two younger slices may still be in flight); the barrier then says that slice s+1 is complete
    // and that every wavefront holds its fragments of slice s in registers, so that slice s+4 can overwrite it.
    // One pass of the loop = four trips.  Full tiles: the last pass has nothing left to request; its loads fetch the last
    // slice again (the pointers are set back to it and stand still) into ring positions that nobody reads any more, so that
    // the loop has one shape, one wait count, and no second copy of its body.
    const char *pa_last = pa - a_step, *pb_last = pb - b_step;         // (after the prologue's four steps: slice 3)
    pa_last += (n_slices - kRing) * a_step;
    pb_last += (n_slices - kRing) * b_step;
    int64_t a_adv = a_step, b_adv = b_step;
    // (EDGE) the trip of slice s fixes up slice s + 1 when that is the last one
    auto top = [&](int64_t s, uint32_t nxt) {
        NT_WAIT_VMCNT(2 * ND);
        if constexpr (EDGE) {
            if (s + 1 == last) settle_last(nxt);                       // (uniform)
        }
        __syncthreads();
    };
    for (int64_t sl = 0; sl < n_slices; sl += kRing) {
        if constexpr (!EDGE) {
            if (sl + kRing >= n_slices) { pa = pa_last; pb = pb_last; a_adv = 0; b_adv = 0; }     // wavefront-uniform
            asm volatile("" : "+s"(pa), "+s"(pb), "+s"(a_adv), "+s"(b_adv));
        }
        top(sl + 0, 1); trip(integral_constant<int, 0>{}, integral_constant<int, 0>{}, a_adv, b_adv);
        top(sl + 1, 2); trip(integral_constant<int, 1>{}, integral_constant<int, 1>{}, a_adv, b_adv);
        top(sl + 2, 3); trip(integral_constant<int, 2>{}, integral_constant<int, 0>{}, a_adv, b_adv);
        top(sl + 3, 0); trip(integral_constant<int, 3>{}, integral_constant<int, 1>{}, a_adv, b_adv);
        // (wait states between the last matrix instruction and anything the compiler may do to an accumulator at the
        // loop's end: it does not know that the inline assembly is a matrix instruction)
        asm volatile("s_nop 7" ::: "memory");
    }
    NT_WAIT_VMCNT(0);                                      // drain the surplus loads ...
    __syncthreads();                                       // ... of every wavefront: the epilogue reuses the LDS
    // The accumulators are read by ordinary instructions from here on: 16 more wait states here, and the epilogue takes
    // every accumulator block through an assembly statement of its own before it reads it (statements of this kind stay
    // in program order, so every read follows the wait states).
    asm volatile("s_nop 15" ::: "memory");

    store_tile16<BM, BN, EDGE>(g, smem, wave, bi, acc, row0 + wave_m * (BM / 2), col0 + wave_n * (BN / 2), lane,
                               EDGE && (g.M - row0 < BM || g.N - col0 < BN));
}

// ---- the unrolled kernel as a persistent one: one workgroup per compute unit walks programs w, w + grid, w + 2 grid, ...
// (full tiles of aligned operands, a whole number of 128-k steps).  The slices of consecutive programs form one stream: the
// last pass of a program, which has nothing of its own left to request, requests the first four slices of the next program,
// so that program's prologue (and the latency of its first loads) is hidden behind this one's last trips and epilogue.  The
// epilogue therefore must leave the ring alone: it stages through the 32 KB of LDS behind the ring, a quarter of the
// wavefront's rows at a time.  Loads and stores share one counter of outstanding operations, and a count cannot tell which
// are which: everything requested is awaited before the epilogue's stores go out, and the first three trips of the next
// program (whose slices are then resident) wait for nothing, so the stores drain while the matrix pipe works.
template <int BM, int BN, bool BF16, int ALAY, int BLAY>
__global__ __launch_bounds__(kThreads, 1) void gemm_direct16p_kernel(const FastArgs g)
{
    constexpr int TM = BM / 32, TN = BN / 32;
    constexpr int kRing = 4;
    static_assert(ring_of(BM, BN) == kRing, "ring of four");
    using TileA = DirectTile16<BM, ALAY>;
    using TileB = DirectTile16<BN, BLAY>;
    constexpr uint32_t A_BYTES = TileA::BYTES, B_BYTES = TileB::BYTES, B_BASE = kRing * A_BYTES;
    constexpr uint32_t STAGE = kRing * (A_BYTES + B_BYTES);         // the epilogue's staging region, behind the ring
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const uint32_t mt32 = (uint32_t)g.mt, nt32 = (uint32_t)g.nt, nb32 = (uint32_t)g.nprog / (mt32 * nt32);
    const int64_t a_step = (ALAY == KCONTIG ? (int64_t)kSliceK : (int64_t)kSliceK * g.lda) * 2;
    const int64_t b_step = (BLAY == KCONTIG ? (int64_t)kSliceK : (int64_t)kSliceK * g.ldb) * 2;
    const int64_t n_slices = g.kt * (kBK / kSliceK);       // a multiple of 4, at least 4 (checked by the host)

    // program v of the launch: batch entry, tile row and column, the operands' tile origins
    struct Where { int64_t bi, row0, col0; const char *pa, *pb; };
    auto locate = [&](int64_t v) {
        uint32_t bb, pid;
        program_of_workgroup_batched_t<uint32_t>((uint32_t)v, nb32, mt32, nt32, &bb, &pid);
        const uint32_t ti = pid / nt32;
        Where w;
        w.bi = __builtin_amdgcn_readfirstlane((int)bb);
        w.row0 = (int64_t)__builtin_amdgcn_readfirstlane((int)ti) * BM;
        w.col0 = (int64_t)__builtin_amdgcn_readfirstlane((int)(pid - ti * nt32)) * BN;
        w.pa = reinterpret_cast<const char *>(g.A + w.bi * g.sa_batch + (ALAY == KCONTIG ? w.row0 * g.lda : w.row0));
        w.pb = reinterpret_cast<const char *>(g.B + w.bi * g.sb_batch + (BLAY == KCONTIG ? w.col0 * g.ldb : w.col0));
        return w;
    };

    TileA ta;
    TileB tb;
    ta.init(wave, lane, g.lda, wave_m * (BM / 2), 0);
    tb.init(wave, lane, g.ldb, wave_n * (BN / 2), B_BASE);

    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    constexpr int NRA = TM * TileA::RPF, NRB = TN * TileB::RPF, NR = NRA + NRB;   // LDS reads per slice
    constexpr int NM = TM * TN, ND = TileA::PER + TileB::PER;
    static_assert(2 * NR <= NM * 3 / 2 && 8 * ND <= NM, "the trip's schedule: a read every other matrix instruction, a load every eighth");
    uint32_t tgt[kRing][ND];
#pragma unroll
    for (int r = 0; r < kRing; ++r)
#pragma unroll
        for (int d = 0; d < ND; ++d)
            tgt[r][d] = d < TileA::PER ? lds0 + r * A_BYTES + (uint32_t)((wave * TileA::PER + d) * 1024)
                                       : lds0 + B_BASE + r * B_BYTES + (uint32_t)((wave * TileB::PER + d - TileA::PER) * 1024);

    float4v acc[TM][TN];
    u32x4 fa[2][TM], fb[2][TN];
    auto lds_read = [&](int r, int set, uint32_t ring) {
        if (r < TileA::RPF) ta.read(fa[set], smem, r, ring * A_BYTES);
        else if (r < TileA::RPF + NRB) tb.read(fb[set], smem, r - TileA::RPF, ring * B_BYTES);
        else ta.read(fa[set], smem, r - NRB, ring * A_BYTES);
    };
    const char *pa, *pb;                                     // the slice that is requested next
    auto dma_aim = [&](int d, int ring) { asm volatile("s_mov_b32 m0, %0" : : "s"(tgt[ring][d]) : "memory"); };
    auto dma_go = [&](int d) {
        if (d < TileA::PER) asm volatile("global_load_lds_dwordx4 %0, %1" : : "v"(ta.voff[d]), "s"(pa) : "memory");
        else asm volatile("global_load_lds_dwordx4 %0, %1" : : "v"(tb.voff[d - TileA::PER]), "s"(pb) : "memory");
    };
    auto trip = [&](auto ring_c, auto set_c, int64_t a_adv, int64_t b_adv) {
        constexpr int RING = decltype(ring_c)::value, SET = decltype(set_c)::value;
        constexpr int NXT = (RING + 1) % kRing;
#pragma unroll
        for (int idx = 0; idx < NM; ++idx) {
            const int tm = idx / TN, tn = idx % TN;
            mfma16<BF16>(acc[tm][tn], fb[SET][tn], fa[SET][tm]);      // transposed block (see store_tile16_rows)
            if (idx % 2 == 0 && idx / 2 < NR) lds_read(idx / 2, SET ^ 1, NXT);
            if (idx % 8 == 1 && idx / 8 < ND) dma_aim(idx / 8, RING);
            if (idx % 8 == 3 && idx / 8 < ND) {
                dma_go(idx / 8);
                if (idx / 8 == TileA::PER - 1) { pa += a_adv; asm volatile("" : "+s"(pa)); }
                if (idx / 8 == ND - 1) { pb += b_adv; asm volatile("" : "+s"(pb)); }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using std::integral_constant;

    int64_t v = blockIdx.x;
    Where cur = locate(v);
    // Start-up stagger (short programs only, the host decides).  Units that start together stay in step: they all multiply,
    // then all store, and the output leaves in bursts at HBM's write rate while every matrix pipe idles.  Four groups of
    // units (every XCD has all four) that start 2 us apart keep that distance, and a group's burst overlaps the other
    // groups' multiplications.  The wait is on the constant 100 MHz counter: it ends whatever else happens.
    if (g.stagger > 0) {
        const uint64_t t0 = __builtin_amdgcn_s_memrealtime();
        const uint64_t late = (uint64_t)((blockIdx.x >> 3) & 3) * (uint64_t)g.stagger;
        while (__builtin_amdgcn_s_memrealtime() - t0 < late) __builtin_amdgcn_s_sleep(8);
    }
    // the first program's slices 0 .. 3
    pa = cur.pa;
    pb = cur.pb;
#pragma unroll
    for (int s = 0; s < kRing; ++s) {
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            dma_aim(d, s);
            asm volatile("s_nop 0");
            dma_go(d);
        }
        pa += a_step;
        pb += b_step;
    }
    asm volatile("" : "+s"(pa), "+s"(pb));
    bool resident = false;                                   // all four slices at the head of the ring have landed (every program but the first)

    for (;;) {
        const int64_t vn = v + gridDim.x;
        const bool more = vn < g.nprog;                      // (uniform)
        Where nxt = cur;
        if (more) nxt = locate(vn);
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int x = 0; x < 4; ++x) acc[a][b][x] = 0.f;
        if (!resident) NT_WAIT_VMCNT((kRing - 1) * ND);
        __syncthreads();
#pragma unroll
        for (int r = 0; r < NR; ++r) lds_read(r, 0, 0);
        __builtin_amdgcn_sched_barrier(0);

        // this program's slices 4 .. continue at pa / pb; its last pass requests the next program's slices 0 .. 3 (or, if
        // there is none, this program's last slice again, into ring positions that nobody reads any more)
        const char *pa_end = cur.pa + (n_slices - 1) * a_step, *pb_end = cur.pb + (n_slices - 1) * b_step;
        int64_t a_adv = a_step, b_adv = b_step;
        for (int64_t sl = 0; sl < n_slices; sl += kRing) {
            if (sl + kRing >= n_slices) {                    // (uniform)
                if (more) { pa = nxt.pa; pb = nxt.pb; }
                else { pa = pa_end; pb = pb_end; a_adv = 0; b_adv = 0; }
            }
            asm volatile("" : "+s"(pa), "+s"(pb), "+s"(a_adv), "+s"(b_adv));
            const bool wait = !(resident && sl == 0);        // (uniform) slices 1 .. 3 of a program whose head is resident need no wait
            if (wait) NT_WAIT_VMCNT(2 * ND);
            __syncthreads(); trip(integral_constant<int, 0>{}, integral_constant<int, 0>{}, a_adv, b_adv);
            if (wait) NT_WAIT_VMCNT(2 * ND);
            __syncthreads(); trip(integral_constant<int, 1>{}, integral_constant<int, 1>{}, a_adv, b_adv);
            if (wait) NT_WAIT_VMCNT(2 * ND);
            __syncthreads(); trip(integral_constant<int, 2>{}, integral_constant<int, 0>{}, a_adv, b_adv);
            NT_WAIT_VMCNT(2 * ND);
            __syncthreads(); trip(integral_constant<int, 3>{}, integral_constant<int, 1>{}, a_adv, b_adv);
            asm volatile("s_nop 7" ::: "memory");
        }
        // everything requested has to have landed before stores join the count of outstanding operations
        NT_WAIT_VMCNT(0);
        asm volatile("s_nop 15" ::: "memory");
        store_tile16<BM, BN, false, 4>(g, smem + STAGE, wave, cur.bi, acc, cur.row0 + wave_m * (BM / 2), cur.col0 + wave_n * (BN / 2), lane);
        if (!more) break;
        v = vn;
        cur = nxt;
        resident = true;
        // (the next program's slices 0 .. 3 were requested by the last pass: the request pointers stand at its slice 4)
    }
}

template <int BM, int BN, bool BF16, int ALAY, int BLAY, bool EDGE = false>
static nt_status launch_direct16_inst(const FastArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)ring_of(BM, BN) * (BM + BN) * kSliceK * sizeof(uint16_t);
    auto kern = gemm_direct16_kernel<BM, BN, BF16, ALAY, BLAY, EDGE>;
    static DeviceOnce configured;
    if (!configured.done()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if constexpr (BM == 256 && BN == 256)
            if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_direct16u_kernel<BM, BN, BF16, ALAY, BLAY, EDGE>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured.set();
    }
    // (the 256 x 256 tile -- one workgroup per compute unit, every issue turn counts -- with a reduction of whole 128-k steps:
    // the kernel with the unrolled ring)
    if constexpr (BM == 256 && BN == 256 && !EDGE) {
        // several programs per compute unit: the persistent kernel (one workgroup per unit, 160 KB of LDS)
        // (a grid that is a multiple of 8 keeps every program of a workgroup on the workgroup's own XCD)
        const int64_t units = compute_units() / 8 * 8;
        if (a.kt % 2 == 0 && a.kt >= 2 && units > 0 && nwg > units) {
            constexpr size_t smem_p = smem + 32768;
            auto kp = gemm_direct16p_kernel<BM, BN, BF16, ALAY, BLAY>;
            static DeviceOnce configured_p;
            if (!configured_p.done()) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kp), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_p);
                if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
                configured_p.set();
            }
            FastArgs ap = a;
            ap.nprog = nwg;
            // (measured on 2 .. 16 programs per unit: 6 - 14 % for K <= 512, 2 - 4 % at K = 1024, nothing or a small loss beyond)
            // (every unit has at least two programs: with fewer the late starters would only lengthen the launch)
            ap.stagger = a.kt <= 16 && nwg >= 2 * units ? 200 : 0;
            hipLaunchKernelGGL(kp, dim3((unsigned)units), dim3(kThreads), smem_p, s, ap);
            return check_launch("gemm_direct16p_kernel");
        }
    }
    if constexpr (BM == 256 && BN == 256) {
        // (range-checked flavour: any number of slices is rounded up to whole passes of four; worth it from three passes on)
        if (EDGE ? a.K > 8 * kSliceK : (a.kt % 2 == 0 && a.kt >= 2)) {
            hipLaunchKernelGGL((gemm_direct16u_kernel<BM, BN, BF16, ALAY, BLAY, EDGE>), dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
            return check_launch("gemm_direct16u_kernel");
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_direct16_kernel");
}

// the loader trace of the same kernel (see TRACE): one workgroup
template <int BM, int BN, int ALAY, int BLAY, bool EDGE>
static nt_status launch_direct16_trace_inst(const FastArgs &a, hipStream_t s)
{
    constexpr size_t smem = (size_t)ring_of(BM, BN) * (BM + BN) * kSliceK * sizeof(uint16_t);
    auto kern = gemm_direct16_kernel<BM, BN, false, ALAY, BLAY, EDGE, true>;
    static DeviceOnce configured;
    if (!configured.done()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured.set();
    }
    hipLaunchKernelGGL(kern, dim3(1), dim3(kThreads), smem, s, a);
    return check_launch("gemm_direct16_kernel (trace)");
}

template <int BM, int BN, bool BF16, bool EDGE = false>
static nt_status launch_direct16_t(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s)
{
    if (alay == KCONTIG && blay == MNCONTIG) return launch_direct16_inst<BM, BN, BF16, KCONTIG, MNCONTIG, EDGE>(a, nwg, s);
    if (alay == KCONTIG && blay == KCONTIG) return launch_direct16_inst<BM, BN, BF16, KCONTIG, KCONTIG, EDGE>(a, nwg, s);
    if (alay == MNCONTIG && blay == MNCONTIG) return launch_direct16_inst<BM, BN, BF16, MNCONTIG, MNCONTIG, EDGE>(a, nwg, s);
    return launch_direct16_inst<BM, BN, BF16, MNCONTIG, KCONTIG, EDGE>(a, nwg, s);
}

#define NT_DIRECT16_DECL(T) \
    nt_status launch_direct16_##T##_f16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s); \
    nt_status launch_direct16_##T##_bf16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s); \
    nt_status launch_direct16_edge_##T##_f16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s); \
    nt_status launch_direct16_edge_##T##_bf16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s);
NT_DIRECT16_DECL(128x128)
NT_DIRECT16_DECL(256x128)
NT_DIRECT16_DECL(128x256)
NT_DIRECT16_DECL(256x256)
#undef NT_DIRECT16_DECL
// loader trace: bm x bn in {128, 256}^2, either flavour
nt_status launch_direct16_trace(const FastArgs &a, int bm, int bn, int alay, int blay, bool edge, hipStream_t s);

}  // namespace nt
