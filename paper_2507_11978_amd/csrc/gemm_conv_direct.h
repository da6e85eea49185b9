// Implicit-GEMM convolution (Section 4.3) whose operand blocks travel straight into LDS.
//
// Same problem class as gemm_conv.h (contiguous NCHW input, unit conv stride, k-contiguous filter, output dense
// in (p, q)), same numbering of the output positions (row pitch rounded up to a multiple of 8), with the pipeline
// of the direct GEMM kernel on 16 x 16 x 32 matrix instructions (gemm_direct16.h): 32-k slices in a ring of three or four
// LDS slots, no staging registers, one trip of the loop per slice.
//
// The unfolded input A[m, kk] = x[n, c, p + r - pad_h, q + s - pad_w] is contiguous along m, so its slice is the
// mn-major LDS layout [32 kk][256 m] read with transposing LDS reads.  One 16-byte chunk is a run of 8 consecutive
// q of one (c, r, s) line; the lane that owns the chunk's LDS slot computes where the run starts inside x and fetches
// it with a range-checked buffer load (2-byte aligned).  What cannot be fetched as it is:
//   * a run whose input row lies in the top / bottom padding, whose kk is past the program's k range or whose
//     position is past M: the lane passes an offset outside the buffer and zeros arrive;
//   * the one element of a run that falls into the left / right padding: fetched (it is the neighbouring row's end /
//     start, inside x) and overwritten with zero in LDS by the same lane once the run has landed, before the
//     barrier that publishes the slice;
//   * the tensor's very first run with a tap left of it, and its last runs with taps right of them, would start
//     outside x: fetched one element late / up to 7 early and shifted into place in LDS by the same lane.
// The filter is the direct kernel's k-major B operand (range checked: rows past the last filter read as zero).
// Requirements checked by the host: K % 32 == 0 (no ragged slice), filter pitch and base 16-byte aligned,
// R, S <= 8, byte offsets inside x below 2^31.
#pragma once
#include "gemm_conv.h"
#include "gemm_direct16.h"

namespace nt {

// mn-major slice of the unfolded input: 32 kk rows x 256 positions
struct ConvTileA {
    static constexpr int E = 256;
    static constexpr uint32_t BYTES = E * kSliceK * 2;
    static constexpr int PER = BYTES / 1024 / 4;           // load instructions per wavefront and slice (4)
    static constexpr int RPF = 2;
    static constexpr int RB = 2 * E;                       // bytes per kk row
    static constexpr int T = E / 32;                       // 16-position fragments per wavefront
    static constexpr uint32_t kOutside = 0x80000000u;      // byte offset past every buffer this kernel accepts
    enum { CLEAR_FIRST = 1, CLEAR_LAST = 2, MOVE_UP = 4, DOWN_SHIFT = 3 /* bits 3..6: elements to move down by (0..8) */ };

    uint32_t rd[T];
    // Load j of a slice covers kk row 8 * wave + 2 * j + lane / 32 and, because of the bank swizzle (that of
    // DirectTile16<E, MNCONTIG>: chunk ^= 4 (kk & 3) + 2 ((kk / 8) & 1), the second term being the wavefront's parity),
    // one of two runs of 8 positions: run j % 2.
    int32_t base[2];               // element offset of x[n, 0, p - ph, q0 - pw] of the run
    uint32_t masks[2];             // bits 0..7: input row p + r - ph inside the image (and m < M); bit 8 + 2 s: with tap s the
                                   // run's first element is padding; bit 9 + 2 s: with tap s its element last_e is padding
    // the kk row of load j in the slice that is requested next: 4 * (r * S + s), c * HW, and the tap's table entry
    // (looked up one slice ahead, so that nobody waits for it)
    uint32_t rs4[PER];
    int32_t coff[PER];
    uint32_t tap[PER];

    // Table of the R * S filter taps in LDS (at byte offset `table`): r * W + s | (1 << r) << 16 | (8 + 2 s) << 24
    static constexpr uint32_t kTableBytes = 64 * 4 + 64 * 4;      // the table, and a spare word per lane (see settle)
    static __device__ __forceinline__ void fill_table(char *smem, uint32_t table, const ConvArgs &g, int tid)
    {
        if (tid < g.RS) {
            const uint32_t r = udiv_small((uint32_t)tid, g.inv_s), sx = (uint32_t)tid - r * (uint32_t)g.S;
            *reinterpret_cast<uint32_t *>(smem + table + 4 * tid) = (r * (uint32_t)g.W + sx) | (0x10000u << r) | ((8 + 2 * sx) << 24);
        }
    }

    // k_first: first kk of the program; the table must be complete
    __device__ __forceinline__ void init(int wave, int lane, const ConvArgs &g, int64_t row0, int32_t k_first, int wave_origin, uint32_t region,
                                         const char *smem, uint32_t table)
    {
        const int hi = lane >> 5;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int chunk = (lane & 31) ^ (((2 * e + hi) << 2) | ((wave & 1) << 1));
            const int64_t m = row0 + chunk * 8;
            const bool m_ok = m < g.M;
            const uint32_t mm = m_ok ? (uint32_t)m : 0u;
            const uint32_t nn = mm / (uint32_t)g.PQ8;
            const uint32_t pq = mm - nn * (uint32_t)g.PQ8;
            const uint32_t p = pq / (uint32_t)g.Q8;
            const int32_t q0 = (int32_t)(pq - p * (uint32_t)g.Q8);
            base[e] = (int32_t)(nn * (uint32_t)g.CHW) + ((int32_t)p - g.ph) * g.W + q0 - g.pw;
            uint32_t mk = 0;
            for (int rr = 0; rr < g.R; ++rr) {
                const int h = (int)p + rr - g.ph;
                if (m_ok && h >= 0 && h < g.H) mk |= 1u << rr;
            }
            for (int sx = 0; sx < g.S; ++sx) {
                if (q0 + sx - g.pw < 0) mk |= 0x100u << (2 * sx);
                if (q0 + 8 >= g.Q && g.Q - 1 + sx - g.pw >= g.W) mk |= 0x200u << (2 * sx);
            }
            masks[e] = mk;
        }
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const uint32_t k = (uint32_t)(k_first + 8 * wave + 2 * j + hi);
            const uint32_t c = udiv_small(k, g.inv_rs);
            rs4[j] = 4u * (k - c * (uint32_t)g.RS);
            coff[j] = (int32_t)c * g.HW;
            tap[j] = *reinterpret_cast<const uint32_t *>(smem + table + rs4[j]);
        }
        // transposing read (see DirectTile16<E, MNCONTIG>)
        const int gq = lane >> 4, i = lane & 15;
        const int kl = 8 * gq + (i >> 2);
        const int mn = wave_origin + 4 * (i & 3);
        const int sw = DirectTile16<E, MNCONTIG>::swizzle(kl);
#pragma unroll
        for (int t = 0; t < T; ++t)
            rd[t] = (uint32_t)(kl * RB + ((((mn >> 3) + 2 * t) ^ sw) << 4) + ((mn >> 2) & 1) * 8) + region;
    }

    // Requests load j of the next slice into the LDS slot at lds_slice and moves the state on by one slice
    // (step4 = 4 * (32 % RS), stepc = 32 / RS * HW); returns what has to be done to the run once it has landed
    // (0: nothing).  beyond: the slice lies past the program's k range; it is requested like any other (the loop has
    // one shape) but from outside the buffer, so that zeros arrive (a surplus trip multiplies it).
    __device__ __forceinline__ uint32_t issue_one(int j, const ConvArgs &g, u32x4 rsrc, uint32_t step4, int32_t stepc,
                                                  const char *smem, uint32_t table, uint32_t lds_slice, int wave, bool beyond)
    {
        const int e = j & 1;
        const uint32_t t = tap[j], mk = masks[e];
        const int32_t l_off = base[e] + coff[j] + (int32_t)(t & 0xffffu);
        const int32_t hi_lim = (int32_t)g.x_numel - 8;
        // a run that would start before x (by one element: only pw <= 1 is accepted) or end after it is fetched from
        // the nearest place inside and moved by settle(); 8 or more elements late: nothing of the run lies inside x
        const int32_t late = std::min(std::max(l_off - hi_lim, 0), 8);
        const int32_t offc = std::min(std::max(l_off, 0), hi_lim);
        uint32_t code = (mk >> (t >> 24)) & 3u;
        code |= ((uint32_t)l_off >> 29) & (uint32_t)MOVE_UP;
        code |= (uint32_t)late << DOWN_SHIFT;
        const bool ok = (mk & (t >> 16) & 0xffu) != 0 && !beyond;
        dma16_buf(rsrc, ok ? (uint32_t)offc * 2u : kOutside, 0u, lds_slice + (uint32_t)((wave * PER + j) * 1024));
        // the same row of the slice after it
        uint32_t nrs = rs4[j] + step4;
        int32_t nco = coff[j] + stepc;
        if (nrs >= 4u * (uint32_t)g.RS) { nrs -= 4u * (uint32_t)g.RS; nco += g.HW; }
        rs4[j] = nrs;
        coff[j] = nco;
        tap[j] = *reinterpret_cast<const uint32_t *>(smem + table + nrs);
        return ok ? code : 0u;
    }

    // What issue_one() noted for the four runs of a slice (8 bits each in `codes`), applied in LDS.  The common work -- the one
    // element of a run that lies in the left / right padding is overwritten with zero -- has no branch: a run without such an
    // element writes its zero to a spare place of its own (at byte offset `spare`).  (With a branch per run and case, this
    // function was 300 instructions between the wait for the slice and the barrier that publishes it, every trip, with the
    // matrix pipe idle.)  The rare work -- a run that had to be fetched from another place, the tensor's first and last
    // runs -- sits behind one wavefront-uniform test.
    __device__ __forceinline__ void settle(uint32_t codes, char *smem, const ConvArgs &g, uint32_t slot_off, int wave, int lane, uint32_t spare) const
    {
        constexpr uint32_t kClears = 0x01010101u * (uint32_t)(CLEAR_FIRST | CLEAR_LAST);
        if (__builtin_amdgcn_ballot_w64(codes != 0) == 0) return;                       // (uniform)
        if (__builtin_amdgcn_ballot_w64((codes & ~kClears) != 0) != 0) {                // (uniform, rare)
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                const uint32_t code = (codes >> (8 * j)) & 0xffu;
                if ((code & ~(uint32_t)(CLEAR_FIRST | CLEAR_LAST)) == 0) continue;
                const uint32_t at = slot_off + (uint32_t)((wave * PER + j) * 1024 + lane * 16);
                u32x4 v = lds_read16(smem, at);
                if (code & MOVE_UP) {                              // element i <- element i - 1 (element 0 is cleared below)
                    v = u32x4{v[0] << 16, __builtin_amdgcn_alignbit(v[1], v[0], 16), __builtin_amdgcn_alignbit(v[2], v[1], 16),
                              __builtin_amdgcn_alignbit(v[3], v[2], 16)};
                } else {
                    const uint32_t d = code >> DOWN_SHIFT;                 // element i <- element i + d, zeros from the top
                    v = d < 8 ? shift_down(v, (int)d) : u32x4{0, 0, 0, 0};
                }
                lds_write16(smem, at, v);
            }
        }
        const uint32_t own = spare + (uint32_t)lane * 4u;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const uint32_t at = slot_off + (uint32_t)((wave * PER + j) * 1024 + lane * 16);
            const uint32_t a_first = (codes >> (8 * j)) & (uint32_t)CLEAR_FIRST ? at : own;
            const uint32_t a_last = (codes >> (8 * j)) & (uint32_t)CLEAR_LAST ? at + 2u * (uint32_t)g.last_e : own;
            *reinterpret_cast<uint16_t *>(smem + a_first) = 0;
            *reinterpret_cast<uint16_t *>(smem + a_last) = 0;
        }
    }

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

// Epilogue of the kernels that stream their operands into LDS.  Their matrix instructions are issued with the input's fragment first, so a lane holds one FILTER
// f = lane % 16 of each 16 x 16 block and four consecutive POSITIONS 4 (lane / 16) .. + 3 of it: eight (four) contiguous
// bytes of the output, whose unit-stride axis is the position.  As in store_tile16_rows the wavefront's part (BN / 2 filters x
// 16 TM positions) goes through its own region (BN / 2 x 256 bytes) of the idle ring so that the global stores are 16-byte chunks and a
// store instruction covers 4 filters x 256 contiguous bytes (an epilogue that stored from the registers, one position and four
// filters per lane, wrote 2 bytes per lane: eight times the store instructions, in 32-byte pieces):
//   write phase  per block one conversion, the lane's 4 values to [filter][256 bytes] with the 16-byte chunk index XOR-ed
//                with the filter (16 filters, same chunk: 16 different chunks);
//   read phase   16 consecutive lanes read one filter's 256 bytes; a lane's chunk is 16 / ES consecutive positions of one
//                output row (the kernel numbers positions with the row pitch rounded up to a multiple of 8, so a chunk never
//                crosses a row), decomposed into (image, row, column) once per lane and pass.
// An fp32 tile takes two passes (64 positions each).  A chunk that lies wholly inside its row and starts at a 4-byte
// boundary is stored whole, any other element by element (the last chunk of rows whose length is no multiple of the chunk,
// 16-bit rows of odd length).  Positions past M
// and a row's surplus positions are not stored.  part: which part of the k range the program multiplied.
template <int BM, int BN, int OUT>
__device__ __forceinline__ void conv_store_rows16(const ConvArgs &g, char *smem, int wave, const float4v (&acc)[BM / 32][BN / 32], int64_t part,
                                                  int64_t row0w, int64_t col0w, int lane)
{
    constexpr int TM = BM / 32;                            // blocks of 16 positions per wavefront
    constexpr int TNW = BN / 32, FW = BN / 2;              // blocks of 16 filters, and filters, per wavefront
    constexpr int ES = OUT == NT_F32 ? 4 : 2;
    constexpr int PASSES = ES / 2;
    constexpr int BPP = 8 / PASSES;                        // position blocks per pass
    constexpr int EPC = 16 / ES;                           // positions per chunk
    constexpr int RB = 256;                                // bytes per region row (one filter)
    const int l16 = lane & 15, gq = lane >> 4;
    char *reg = smem + wave * (FW * RB);
    const int64_t f_pitch = g.syf * ES;
    char *const y0 = reinterpret_cast<char *>(g.Y) + part * g.slice * ES + col0w * f_pitch;
    const int64_t filters = g.N - col0w;                   // filters from this wavefront's first on
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
        // ---- write phase
#pragma unroll
        for (int tmp = 0; tmp < BPP; ++tmp) {
            const int tm = pass * BPP + tmp;
            if (tm >= TM) break;
#pragma unroll
            for (int tn = 0; tn < TNW; ++tn) {
                // (the block is pinned in its accumulator registers up to this point, see store_tile16_rows)
                float4v blk = acc[tm][tn];
                asm volatile("" : "+a"(blk));
                float o[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) o[v] = blk[v];
                const int r = tn * 16 + l16;
                char *prow = reg + r * RB;
                if constexpr (OUT == NT_F32) {
                    const int c = tmp * 4 + gq;
                    lds_write16(prow, (uint32_t)((c ^ l16) << 4), u32x4{__builtin_bit_cast(uint32_t, o[0]), __builtin_bit_cast(uint32_t, o[1]),
                                                                         __builtin_bit_cast(uint32_t, o[2]), __builtin_bit_cast(uint32_t, o[3])});
                } else {
                    const int c = tmp * 2 + (gq >> 1);
                    *reinterpret_cast<u32x2 *>(prow + (((c ^ l16) << 4) + 8 * (gq & 1))) =
                        u32x2{pack_pair<OUT>(__builtin_bit_cast(uint32_t, o[0]), __builtin_bit_cast(uint32_t, o[1])),
                              pack_pair<OUT>(__builtin_bit_cast(uint32_t, o[2]), __builtin_bit_cast(uint32_t, o[3]))};
                }
            }
        }
        // ---- read phase (same wavefront: LDS operations complete in order).  The lane's chunk: positions m .. m + EPC - 1
        const int c = lane & 15;
        const int pos = pass * (128 / PASSES) + c * EPC;                         // first position, within the wavefront's part
        const int64_t m = row0w + pos;
        const bool live = pos < 16 * TM && m < g.M;
        const uint32_t mm = live ? (uint32_t)m : 0u;
        const uint32_t n = mm / (uint32_t)g.PQ8;
        const uint32_t pq = mm - n * (uint32_t)g.PQ8;
        const uint32_t p = pq / (uint32_t)g.Q8;
        const int q = (int)(pq - p * (uint32_t)g.Q8);
        const int nv = !live ? 0 : (g.Q - q >= EPC ? EPC : (g.Q - q > 0 ? g.Q - q : 0));   // positions of the chunk that exist
        const int64_t lane_off = ((int64_t)n * g.syn + (int64_t)p * g.Q + q) * ES;
        // a whole chunk is stored with one instruction if it starts at a 4-byte boundary; streamed if all of the wavefront's
        // chunks are whole and start at 16-byte boundaries (see store_tile16_rows)
        const uintptr_t at0 = reinterpret_cast<uintptr_t>(y0) + (uintptr_t)lane_off;
        const bool whole = nv == EPC && (at0 & 3) == 0 && (f_pitch & 3) == 0;
        const bool stream = __builtin_amdgcn_ballot_w64((whole && (at0 & 15) == 0 && (f_pitch & 15) == 0) || nv == 0) == ~0ull;      // (uniform)
        if (stream) {
#pragma unroll
            for (int it = 0; it < FW / 4; ++it) {
                const int r = it * 4 + gq;
                const u32x4 v = lds_read16(reg, (uint32_t)(r * RB + ((c ^ (r & 15)) << 4)));
                if (nv != 0 && r < filters) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(y0 + r * f_pitch + lane_off));
            }
        } else {
#pragma unroll
            for (int it = 0; it < FW / 4; ++it) {
                const int r = it * 4 + gq;
                const u32x4 v = lds_read16(reg, (uint32_t)(r * RB + ((c ^ (r & 15)) << 4)));
                char *at = y0 + r * f_pitch + lane_off;
                if (r < filters) {
                    if (whole) {
                        __builtin_memcpy(at, &v, 16);
                    } else if (ES == 2 && (at0 & 3) == 0 && (f_pitch & 3) == 0) {
                        // (the part of a 16-bit chunk that exists, pairs of positions at a time)
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            if (2 * d + 1 < nv) *reinterpret_cast<uint32_t *>(at + 4 * d) = v[d];
                            else if (2 * d < nv) *reinterpret_cast<uint16_t *>(at + 4 * d) = (uint16_t)(v[d] & 0xffffu);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < EPC; ++e)
                            if (e < nv) {
                                const uint32_t w = v[ES == 4 ? e : e / 2];
                                if constexpr (OUT == NT_F32) *reinterpret_cast<uint32_t *>(at + 4 * e) = w;
                                else *reinterpret_cast<uint16_t *>(at + 2 * e) = (uint16_t)((e & 1) ? w >> 16 : w & 0xffffu);
                            }
                    }
                }
            }
        }
    }
}

// Epilogue of a k split's programs (few, short programs whose fp32 partial tiles go to the workspace): straight from the
// registers, a lane's 4 consecutive positions of one filter as one 16-byte store where they lie in one output row at a
// 4-byte boundary (they do: the workspace slices are dense and fp32), else element by element.  No LDS round trip: with
// at most one such program per compute unit its latency would not be hidden by anything.
template <int BM, int BN>
__device__ __forceinline__ void conv_store_partial16(const ConvArgs &g, const float4v (&acc)[BM / 32][BN / 32], int64_t part, int64_t row0w, int64_t col0w, int lane)
{
    constexpr int TM = BM / 32, TN = BN / 32;
    const int l16 = lane & 15, gq = lane >> 4;
    const int64_t f_pitch = g.syf * 4;
    char *const y0 = reinterpret_cast<char *>(g.Y) + part * g.slice * 4 + (col0w + l16) * f_pitch;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int64_t m = row0w + tm * 16 + 4 * gq;                  // the lane's first position (a multiple of 4: one output row)
        const uint32_t mm = m < g.M ? (uint32_t)m : 0u;
        const uint32_t n = mm / (uint32_t)g.PQ8;
        const uint32_t pq = mm - n * (uint32_t)g.PQ8;
        const uint32_t p = pq / (uint32_t)g.Q8;
        const int q = (int)(pq - p * (uint32_t)g.Q8);
        const int nv = m < g.M ? (g.Q - q >= 4 ? 4 : (g.Q - q > 0 ? g.Q - q : 0)) : 0;
        char *const at0 = y0 + ((int64_t)n * g.syn + (int64_t)p * g.Q + q) * 4;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            // (the block is pinned in its accumulator registers up to this point, see store_tile16_rows)
            float4v blk = acc[tm][tn];
            asm volatile("" : "+a"(blk));
            float o[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] = blk[v];
            if (col0w + tn * 16 + l16 >= g.N) continue;               // a filter past the last
            char *at = at0 + (tn * 16) * f_pitch;
            if (nv == 4) {
                const u32x4 w{__builtin_bit_cast(uint32_t, o[0]), __builtin_bit_cast(uint32_t, o[1]), __builtin_bit_cast(uint32_t, o[2]), __builtin_bit_cast(uint32_t, o[3])};
                __builtin_memcpy(at, &w, 16);
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (v < nv) *reinterpret_cast<float *>(at + 4 * v) = o[v];
            }
        }
    }
}

// TRACE: one workgroup as program g.trace_program; the loader is stepped slice by slice up to g.trace_slice (its state moves
// on with every request), that slice is fixed up as in the loop, and one operand's slice is copied out of LDS in
// (position or filter, k) order (see gemm_direct16_kernel).
template <int BN, bool BF16, bool TRACE = false>
__global__ __launch_bounds__(kThreads, residency_of(256, BN)) void gemm_conv_direct_kernel(const ConvArgs g)
{
    constexpr int BM = 256;
    constexpr int TM = BM / 32, TN = BN / 32;
    constexpr int kRing = ring_of(BM, BN);
    using TileA = ConvTileA;
    using TileB = DirectTile16<BN, KCONTIG>;
    constexpr uint32_t A_BYTES = TileA::BYTES, B_BYTES = TileB::BYTES, B_BASE = kRing * A_BYTES;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int64_t bi, ti, tj;                                  // bi: which part of the k range (k split)
    if constexpr (TRACE) { bi = 0; ti = g.trace_program / g.nt; tj = g.trace_program % g.nt; }
    else locate_program(g.mt, g.nt, &bi, &ti, &tj);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int64_t row0 = ti * BM, col0 = tj * BN;
    const int64_t kt0 = bi * g.kt_per;                                                   // first k tile of this program
    const int64_t kt_n = g.kt - kt0 < g.kt_per ? g.kt - kt0 : g.kt_per;                  // and how many
    const int32_t k_first = (int32_t)(kt0 * kBK);
    const int32_t k_end = (int32_t)((kt0 + kt_n) * kBK < g.K ? (kt0 + kt_n) * kBK : g.K);
    const int64_t n_slices = (k_end - k_first) / kSliceK;                                // (K is a multiple of 32)

    const char *gB0 = reinterpret_cast<const char *>(g.Wt);
    const char *gB = reinterpret_cast<const char *>(g.Wt + col0 * g.ldb + k_first);
    constexpr int64_t b_step = (int64_t)kSliceK * 2;

    constexpr uint32_t TABLE = kRing * (A_BYTES + B_BYTES);
    TileA::fill_table(smem, TABLE, g, tid);
    __syncthreads();
    TileA ta;
    TileB tb;
    ta.init(wave, lane, g, row0, k_first, wave_m * (BM / 2), 0, smem, TABLE);
    tb.init(wave, lane, g.ldb, wave_n * (BN / 2), B_BASE);
    const uint32_t step4 = 4u * (uint32_t)(kSliceK % g.RS);
    const int32_t stepc = (kSliceK / g.RS) * g.HW;
    const u32x4 rsrc_a = make_rsrc(g.X, g.x_numel * 2);
    const u32x4 rsrc_b = make_rsrc(gB, ((int64_t)(g.N - 1) * g.ldb + g.K) * 2 - (gB - gB0));

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
    constexpr int NRA = TM * TileA::RPF, NRB = TN * TileB::RPF, NR = NRA + NRB;
    auto lds_read = [&](int r, int set, uint32_t ring) {
        if (r < TileA::RPF) ta.read(fa[set], smem, r, ring * A_BYTES);
        else if (r < TileA::RPF + NRB) tb.read(fb[set], smem, r - TileA::RPF, ring * B_BYTES);
        else ta.read(fa[set], smem, r - NRB, ring * A_BYTES);
    };
    constexpr int NM = TM * TN, ND = TileA::PER + TileB::PER;
    const int64_t last = n_slices - 1;
    // load d of slice s (counted from the program's first) into ring position `ring`; the codes of the input's runs
    // are collected in `codes`.  A slice past the program's range is requested all the same (the loop has one shape),
    // from outside both buffers: zeros arrive, and the surplus trip of an odd number of slices multiplies zeros.
    auto dma = [&](int d, int64_t s, uint32_t ring, uint32_t &codes) {
        if (d < TileA::PER) {
            codes |= ta.issue_one(d, g, rsrc_a, step4, stepc, smem, TABLE, lds0 + ring * A_BYTES, wave, s > last) << (8 * d);
        } else {
            tb.issue_one_buf(d - TileA::PER, rsrc_b, s <= last ? (uint32_t)(s * b_step) : 0x80000000u, lds0 + B_BASE + ring * B_BYTES, wave);
        }
    };
    // One trip: the matrix instructions on fragment set `set`; behind them the LDS reads of the next slice (ring position
    // rring) into the other set and the loads of slice s into ring position dring (see gemm_direct16_kernel).
    auto trip = [&](int set, uint32_t rring, int64_t s, uint32_t dring, uint32_t &codes) {
        constexpr int RS = NM * 3 / 4;
#pragma unroll
        for (int idx = 0; idx < NM; ++idx) {
            const int tm = idx / TN, tn = idx % TN;
            mfma16<BF16>(acc[tm][tn], fa[set][tm], fb[set][tn]);      // a lane holds filter lane % 16 and 4 positions (see conv_store_rows16)
            if (idx < RS)
#pragma unroll
                for (int r = idx * NR / RS; r < (idx + 1) * NR / RS; ++r) lds_read(r, set ^ 1, rring);
#pragma unroll
            for (int d = idx * ND / NM; d < (idx + 1) * ND / NM; ++d) dma(d, s, dring, codes);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if constexpr (TRACE) {
        uint32_t codes = 0;
        for (int64_t s = 0; s <= g.trace_slice; ++s) {
            codes = 0;
#pragma unroll
            for (int d = 0; d < ND; ++d) dma(d, s, 0, codes);
            NT_WAIT_VMCNT(0);
        }
        ta.settle(codes, smem, g, 0, wave, lane, TABLE + 256);
        __syncthreads();
        const bool first = g.trace_operand == 0;
        for (int e = tid; e < (first ? BM : BN) * kSliceK; e += kThreads) {
            const uint32_t at = first ? DirectTile16<BM, MNCONTIG>::place(e / kSliceK, e % kSliceK) : B_BASE + TileB::place(e / kSliceK, e % kSliceK);
            g.trace_out[e] = *reinterpret_cast<const uint16_t *>(smem + at);
        }
        return;
    }
    // codes of the slices in flight, oldest first: pending[i] belongs to slice (current + 1 + i)
    uint32_t pending[kRing - 1];
    {
        uint32_t c0 = 0;
#pragma unroll
        for (int d = 0; d < ND; ++d) dma(d, 0, 0, c0);
#pragma unroll
        for (int s = 1; s < kRing; ++s) {
            pending[s - 1] = 0;
#pragma unroll
            for (int d = 0; d < ND; ++d) dma(d, s, s, pending[s - 1]);
        }
        NT_WAIT_VMCNT((kRing - 1) * ND);
        ta.settle(c0, smem, g, 0, wave, lane, TABLE + 256);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) lds_read(r, 0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // one slice per trip, two trips per pass (the fragment sets alternate), as in gemm_direct16_kernel; the runs of slice
    // s + 1 are put right between the wait for this wavefront's loads and the barrier that publishes the slice
    uint32_t ring = 0;
    for (int64_t sl = 0; sl < n_slices; sl += 2) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const uint32_t nxt = ring + 1 == kRing ? 0 : ring + 1;
            uint32_t fresh = 0;
            NT_WAIT_VMCNT((kRing - 2) * ND);
            ta.settle(pending[0], smem, g, nxt * A_BYTES, wave, lane, TABLE + 256);
            __syncthreads();
            trip(half, nxt, sl + half + kRing, ring, fresh);
#pragma unroll
            for (int i = 0; i + 1 < kRing - 1; ++i) pending[i] = pending[i + 1];
            pending[kRing - 2] = fresh;
            ring = nxt;
        }
    }
    NT_WAIT_VMCNT(0);
    __syncthreads();
    // (wait states before ordinary instructions read the accumulators, see gemm_direct16_kernel)
    asm volatile("s_nop 15" ::: "memory");

    const int64_t row_w = row0 + wave_m * (BM / 2), col_w = col0 + wave_n * (BN / 2);
    if (g.ksplit > 1) conv_store_partial16<BM, BN>(g, acc, bi, row_w, col_w, lane);       // (fp32 partial tiles)
    else if (g.out_dtype == NT_F32) conv_store_rows16<BM, BN, NT_F32>(g, smem, wave, acc, bi, row_w, col_w, lane);
    else if (g.out_dtype == NT_F16) conv_store_rows16<BM, BN, NT_F16>(g, smem, wave, acc, bi, row_w, col_w, lane);
    else conv_store_rows16<BM, BN, NT_BF16>(g, smem, wave, acc, bi, row_w, col_w, lane);
}

template <int BN, bool BF16, bool TRACE = false>
static nt_status launch_conv_direct_inst(const ConvArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)ring_of(256, BN) * (256 + BN) * kSliceK * sizeof(uint16_t) + ConvTileA::kTableBytes;
    auto kern = gemm_conv_direct_kernel<BN, BF16, TRACE>;
    static DeviceOnce configured;
    if (!configured.done()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured.set();
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_conv_direct_kernel");
}

// bn: 64, 128 or 256 filters per program; nwg = ksplit * mt * nt
nt_status launch_conv_direct(const ConvArgs &a, int bn, bool bf16, int64_t nwg, hipStream_t s);
// the loader trace of the same kernel: one workgroup
nt_status launch_conv_direct_trace(const ConvArgs &a, int bn, hipStream_t s);

}  // namespace nt
