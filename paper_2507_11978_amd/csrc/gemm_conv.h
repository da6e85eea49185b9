// Implicit-GEMM convolution kernel (Section 4.3) for the common dense case: contiguous
// NCHW input, unit conv stride, contiguous KCRS filter, output dense in (p, q).
//
// The arrangement of Section 4.3 lowers the input to the matrix A[m, kk] with
// m = (n, p, q), kk = (c, r, s) and A[m, kk] = x[n, c, p + r - pad_h, q + s - pad_w]
// (zero outside the image).  A is contiguous along m, so its (256 x 64) block is staged
// like a column-major operand: every thread owns 8 consecutive m (one run of q inside an
// image row: the kernel numbers the output positions with the row pitch Q rounded up to a
// multiple of 8, positions q >= Q are computed and never stored) for 8 consecutive kk, loads each run with one 16-byte
// load from the unfolded position inside x -- the unfolded matrix itself never exists --
// clears the one element that can fall into the left / right padding, zeroes runs whose
// input row lies in the top / bottom padding, and transposes the 8 x 8 patch in registers
// into the k-contiguous LDS layout.  The filter is a k-contiguous B operand; the MFMA core
// and the LDS layout are those of the staged GEMM kernel.  The output tile is written
// along m (contiguous in NKPQ), 32 consecutive m per half-wavefront and store (conv_store_points).
#pragma once
#include "gemm_fast.h"

namespace nt {

struct ConvArgs {
    const uint16_t *X;             // input, contiguous [N, C, H, W]
    const uint16_t *Wt;            // filter as B[kk, f] = Wt[f * ldb + kk]
    void *Y;                       // output: element (m = n*PQ + pq, f) at n*syn + f*syf + pq
    int64_t ldb, syn, syf;
    int64_t x_numel;               // N*C*H*W
    int32_t M, N, K;               // GEMM sizes: N*P*Q8 (positions as the kernel numbers them), filters, C*R*S
    int32_t Q8, PQ8;               // output row pitch rounded up to a multiple of 8, and P times that
    int32_t last_e;                // (Q - 1) % 8: place of a row's last output position in its run
    int32_t PQ, Q, H, W, HW, CHW, RS, S, R, ph, pw;
    uint32_t inv_rs, inv_s;        // reciprocals of R*S and S (see udiv_small)
    int64_t mt, nt, kt;
    // the kernel that walks the reduction tap by tap: the first mt_a of the mt tiles of positions are of its first height, the
    // others of its second (32 positions lower)
    int32_t mt_a;
    int out_dtype;
    // k split: the grid holds `ksplit` copies of the mt x nt programs; copy i multiplies k tiles [i * kt_per, (i + 1) * kt_per)
    // and writes its partial tile at Y + i * slice elements (Y then being an fp32 workspace of ksplit dense [n][f][p][q] slices
    // that conv_ws_sum_kernel adds up in a fixed order).  Without a split: ksplit = 1, kt_per = kt, slice = 0.
    int32_t ksplit, kt_per;
    int64_t slice;
    // the filter is stored tap-major already, [filter][r][s][c] (a channels-last filter): Wt[f * ldb + (r * S + s) * C + c];
    // only the kernel that walks the reduction tap by tap takes it
    int32_t filter_tap_major;
    // loader trace of the direct kernel (nullptr otherwise), see FastArgs
    uint16_t *trace_out;
    int64_t trace_program;
    int32_t trace_slice, trace_operand;
};

// floor(t / d) for 0 <= t < 2^16 with inv = floor(2^32 / d) + 1 (d >= 2), inv = 0 standing for d = 1
// (no branch: the loaders that call this sit between MFMAs)
__device__ __forceinline__ uint32_t udiv_small(uint32_t t, uint32_t inv) { return __umulhi(t, inv) + (t & (inv ? 0u : 0xffffffffu)); }

// staging of the (256 x 64) block of the unfolded input
struct StageConv {
    uint32_t r[8][4];              // [k line][packed pairs of m]
    uint32_t wbase;
    int kb, rb;
    int32_t base;                  // element offset of x[n, 0, p - ph, q0 - pw]
    int32_t q0;
    uint32_t hmask;                // bit r: input row p + r - ph lies inside the image (and m < M)
    uint32_t todo[2];              // what settle() has to do to each fetched line
    uint32_t first_mask, last_mask;   // bit s: with filter column s this run's first / last element lies in the padding
    int32_t l_rr, l_ss, l_off;     // filter row, column and input offset of the next line to fetch
    int32_t c, rs;                 // channel and r*S+s of this thread's first k line in the current k tile

    // first_tile: the k tile this set fetches first
    __device__ __forceinline__ void init(int tid, const ConvArgs &g, int64_t row0, int first_tile)
    {
        kb = tid >> 5;
        rb = tid & 31;
        todo[0] = todo[1] = 0;
        wbase = (uint32_t)(rb * 8 * 128 + ((kb ^ (rb & 7)) << 4));
        const int64_t m = row0 + rb * 8;
        const bool m_ok = m < g.M;
        const uint32_t mm = m_ok ? (uint32_t)m : 0u;
        const uint32_t nn = mm / (uint32_t)g.PQ8;
        const uint32_t pq = mm - nn * (uint32_t)g.PQ8;
        const uint32_t p = pq / (uint32_t)g.Q8;
        q0 = (int32_t)(pq - p * (uint32_t)g.Q8);
        base = (int32_t)(nn * (uint32_t)g.CHW) + ((int32_t)p - g.ph) * g.W + q0 - g.pw;
        first_mask = last_mask = 0;
        for (int sx = 0; sx < g.S; ++sx) {
            if (q0 + sx - g.pw < 0) first_mask |= 1u << sx;                          // the run's first position reads column -1
            if (q0 + 8 >= g.Q && g.Q - 1 + sx - g.pw >= g.W) last_mask |= 1u << sx;  // the row's last position (in this run) reads column W
        }
        l_rr = l_ss = l_off = 0;
        hmask = 0;
        for (int rr = 0; rr < g.R; ++rr) {
            const int h = (int)p + rr - g.ph;
            if (m_ok && h >= 0 && h < g.H) hmask |= 1u << rr;
        }
        const uint32_t kk0 = (uint32_t)(first_tile * kBK + kb * 8);
        c = (int32_t)(kk0 / (uint32_t)g.RS);
        rs = (int32_t)(kk0 - (uint32_t)c * (uint32_t)g.RS);
    }

    // Line j (one (c, r, s) combination, 8 consecutive output positions) of the block of the k
    // tile the state points at; k_left: valid k from the tile origin.  The load itself is
    // unconditional, from the run's position clamped into the tensor, and nothing here looks at
    // the data, so that it can stay in flight; what has to happen to it -- zeroing a line that lies
    // in the top / bottom padding or past K, clearing the one element in the left / right padding,
    // moving a run that was clamped by one element back into place -- is noted in `todo` (8 bits per
    // line) and done by settle().
    enum { ZERO = 1, CLEAR_FIRST = 2, CLEAR_LAST = 4, MOVE_UP = 8, DOWN_SHIFT = 4 /* bits 4..6: elements to move down by */ };
    // Lines are fetched in order j = 0 .. 7; (l_rr, l_ss, l_off) walk through the (r, s) taps and
    // channels like an odometer, so only line 0 of a tile costs a division.
    __device__ __forceinline__ void load_line(const ConvArgs &g, int j, int64_t k_left)
    {
        if (j == 0) {
            l_rr = (int32_t)udiv_small((uint32_t)rs, g.inv_s);
            l_ss = rs - l_rr * g.S;
            l_off = base + c * g.HW + l_rr * g.W + l_ss;       // (all below 2^31: checked at launch)
        }
        const bool ok = kb * 8 + j < k_left && ((hmask >> l_rr) & 1u);
        const int32_t hi_lim = (int32_t)g.x_numel - 8;
        int32_t offc = l_off < 0 ? 0 : l_off;
        offc = offc > hi_lim ? hi_lim : offc;
        if (!ok) offc = 0;
        uint32_t code = ok ? 0u : (uint32_t)ZERO;
        code |= ((first_mask >> l_ss) & 1u) * CLEAR_FIRST;     // q0 + s - pad = -1: left padding
        code |= ((last_mask >> l_ss) & 1u) * CLEAR_LAST;       // the row's last position reads column W: right padding
        if (ok && l_off < 0) code |= MOVE_UP;                  // fetched one element late (very first run of the tensor)
        if (ok && l_off > hi_lim) {                            // fetched early (last runs of the tensor): move down, or, if the
            const int32_t d = l_off - hi_lim;                  // run starts at the tensor's end (its one valid position reads
            code |= d < 8 ? (uint32_t)d << DOWN_SHIFT : (uint32_t)ZERO;   // the right padding), nothing is left of it
        }
        if ((j & 3) == 0) todo[j >> 2] = code;
        else todo[j >> 2] |= code << (8 * (j & 3));
        u32x4 v;
        __builtin_memcpy(&v, g.X + offc, 16);
        r[j][0] = v[0]; r[j][1] = v[1]; r[j][2] = v[2]; r[j][3] = v[3];
        // next tap: s + 1, carrying into r and then into the channel
        const bool row_done = l_ss + 1 == g.S;
        l_ss = row_done ? 0 : l_ss + 1;
        l_off += row_done ? g.W - g.S + 1 : 1;
        l_rr += row_done ? 1 : 0;
        const bool chan_done = l_rr == g.R;
        l_rr = chan_done ? 0 : l_rr;
        l_off += chan_done ? g.HW - g.R * g.W : 0;
    }
    __device__ __forceinline__ void settle(const ConvArgs &g)
    {
        // CLEAR_LAST: the element at place last_e of the run (wavefront-uniform masks)
        const uint32_t half = (g.last_e & 1) ? 0x0000ffffu : 0xffff0000u;
        const uint32_t c0 = (g.last_e >> 1) == 0 ? half : ~0u, c1 = (g.last_e >> 1) == 1 ? half : ~0u;
        const uint32_t c2 = (g.last_e >> 1) == 2 ? half : ~0u, c3 = (g.last_e >> 1) == 3 ? half : ~0u;
        // lines that were fetched early (only the last runs of the tensor): one test for all eight
        if ((todo[0] | todo[1]) & (0x07070707u << DOWN_SHIFT)) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int d = (int)((todo[j >> 2] >> (8 * (j & 3) + DOWN_SHIFT)) & 7u);
                const u32x4 v = shift_down(u32x4{r[j][0], r[j][1], r[j][2], r[j][3]}, d);   // element i <- element i + d, zeros from the top
                r[j][0] = v[0]; r[j][1] = v[1]; r[j][2] = v[2]; r[j][3] = v[3];
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t code = (todo[j >> 2] >> (8 * (j & 3))) & 0xffu;
            uint32_t v0 = r[j][0], v1 = r[j][1], v2 = r[j][2], v3 = r[j][3];
            if (code & MOVE_UP) {                              // element i <- element i - 1 (element 0 is cleared below)
                v3 = __builtin_amdgcn_alignbit(v3, v2, 16); v2 = __builtin_amdgcn_alignbit(v2, v1, 16);
                v1 = __builtin_amdgcn_alignbit(v1, v0, 16); v0 = v0 << 16;
            }
            if (code & CLEAR_FIRST) v0 &= 0xffff0000u;
            if (code & CLEAR_LAST) { v0 &= c0; v1 &= c1; v2 &= c2; v3 &= c3; }
            if (code & ZERO) { v0 = 0; v1 = 0; v2 = 0; v3 = 0; }
            r[j][0] = v0; r[j][1] = v1; r[j][2] = v2; r[j][3] = v3;
        }
    }
    // moves the state on by `tiles` k tiles (kk += 64 * tiles; tiles <= 2)
    __device__ __forceinline__ void advance(const ConvArgs &g, int tiles)
    {
        const uint32_t t = (uint32_t)rs + 64u * (uint32_t)tiles;
        const uint32_t dq = udiv_small(t, g.inv_rs);
        c += (int32_t)dq;
        rs = (int32_t)(t - dq * (uint32_t)g.RS);
    }
    static constexpr int PIECES = 8;
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
        for (int n = 0; n < 8; ++n) store_piece(smem, buf_off, n);
    }
};

// Epilogue of the convolution kernels.  The MFMAs are issued with their operands swapped, so a lane holds one output
// position m = lane % 32 of each 32 x 32 block and, register by register, 16 of its filters
// (8 * (v / 4) + 4 * (lane / 32) + v % 4).  Every store instruction then writes, per half-wavefront, 32 consecutive
// positions of one filter: whole 64- or 128-byte segments of the output's contiguous (p, q) axis.  (With a lane holding
// one filter and runs of positions, a store touched 64 different cache lines with 16 bytes each and the epilogue of a
// 256 x 256 program took 16 us instead of 5.6.)  Positions past M and a row's surplus positions (the kernels number
// positions with the row pitch rounded up to a multiple of 8) are not stored.
// An element's address is a wavefront-uniform base (the filter) plus a lane offset (the position, and the lane half's
// 4 filters) of type OFF: uint32_t where the host has checked that the output's byte offsets fit 31 bits, else int64_t.
// row0w / col0w: first position / filter of this wavefront; part: which part of the k range the program multiplied
// (k split; 0 without).
template <int BM, int BN, int OUT, typename OFF>
__device__ __forceinline__ void conv_store_points(const ConvArgs &g, float16v (&acc)[BM / 64][BN / 64], int64_t part, int64_t row0w, int64_t col0w, int lane)
{
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int ES = OUT == NT_F32 ? 4 : 2;
    const int l32 = lane & 31, hi = lane >> 5;
    const int64_t f_pitch = g.syf * ES;
    char *const y0 = reinterpret_cast<char *>(g.Y) + part * g.slice * ES + col0w * f_pitch;
    const OFF half_off = (OFF)(4 * hi) * (OFF)f_pitch;
    auto put = [&](char *at, float x) {
        if constexpr (OUT == NT_F32) *reinterpret_cast<float *>(at) = x;
        else *reinterpret_cast<uint16_t *>(at) = (uint16_t)pack_pair<OUT>(__builtin_bit_cast(uint32_t, x), 0u);
    };
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int64_t m = row0w + tm * 32 + l32;
        const uint32_t mm = m < g.M ? (uint32_t)m : 0u;
        const uint32_t n = mm / (uint32_t)g.PQ8;
        const uint32_t pq = mm - n * (uint32_t)g.PQ8;
        const uint32_t p = pq / (uint32_t)g.Q8;
        const int q = (int)(pq - p * (uint32_t)g.Q8);
        if (m >= g.M || q >= g.Q) continue;                         // past the last position, or one of a row's surplus positions
        const OFF lane_off = (OFF)((int64_t)n * g.syn + (int64_t)p * g.Q + q) * (OFF)ES + half_off;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            char *const yb = y0 + (tn * 32) * f_pitch;              // (uniform)
            if (col0w + tn * 32 + 32 <= g.N) {                      // (the same for the whole wavefront)
#pragma unroll
                for (int v = 0; v < 16; ++v) put(yb + (8 * (v / 4) + v % 4) * f_pitch + lane_off, acc[tm][tn][v]);
            } else {
                const int64_t room = g.N - (col0w + tn * 32 + 4 * hi);   // filters from this lane's first on
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (8 * (v / 4) + v % 4 < room) put(yb + (8 * (v / 4) + v % 4) * f_pitch + lane_off, acc[tm][tn][v]);
            }
        }
    }
}

template <int BM, int BN, typename OFF>
__device__ __forceinline__ void conv_store_transposed(const ConvArgs &g, float16v (&acc)[BM / 64][BN / 64], int64_t part, int64_t row0w, int64_t col0w, int lane)
{
    if (g.out_dtype == NT_F32) conv_store_points<BM, BN, NT_F32, OFF>(g, acc, part, row0w, col0w, lane);
    else if (g.out_dtype == NT_F16) conv_store_points<BM, BN, NT_F16, OFF>(g, acc, part, row0w, col0w, lane);
    else conv_store_points<BM, BN, NT_BF16, OFF>(g, acc, part, row0w, col0w, lane);
}

template <int BN, bool BF16, bool EDGE_B>
__global__ __launch_bounds__(kThreads) void gemm_conv_kernel(const ConvArgs g)
{
    constexpr int BM = 256;
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr uint32_t A_BYTES = BM * kBK * 2, B_BYTES = BN * kBK * 2;
    constexpr uint32_t B_BASE = 2 * A_BYTES;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    int64_t bi, ti, tj;                                  // bi: which part of the k range (k split)
    locate_program(g.mt, g.nt, &bi, &ti, &tj);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int l32 = lane & 31, hi = lane >> 5;
    const int64_t row0 = ti * BM, col0 = tj * BN;
    const int64_t kt0 = bi * g.kt_per;                                                   // first k tile of this program
    const int64_t kt_n = g.kt - kt0 < g.kt_per ? g.kt - kt0 : g.kt_per;                  // and how many
    const int64_t k_end = (kt0 + kt_n) * kBK < g.K ? (kt0 + kt_n) * kBK : g.K;           // k past its range reads as zero

    const char *gB = reinterpret_cast<const char *>(g.Wt + col0 * g.ldb + kt0 * kBK);
    const int64_t n_left = g.N - col0;

    // two sets of staging registers: a tile is requested two trips before it is multiplied
    StageConv sa0, sa1;
    StageK<BN, true> sb0, sb1;
    sa0.init(tid, g, row0, (int)kt0);
    sa1.init(tid, g, row0, (int)kt0 + 1);
    sb0.init(tid, g.ldb);
    sb1.init(tid, g.ldb);

    const int ra = wave_m * (BM / 2) + l32, rbn = wave_n * (BN / 2) + l32;
    const uint32_t a_rd = (uint32_t)(ra * 128 + ((hi ^ ((ra ^ (ra >> 3)) & 7)) << 4));
    const uint32_t b_rd = (uint32_t)(rbn * 128 + ((hi ^ ((rbn ^ (rbn >> 3)) & 7)) << 4)) + B_BASE;

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
    // LDS read r of k step ks of LDS copy `copy`, in the order the MFMAs need the data
    auto frag_read = [&](int r, int slot, int ks, uint32_t copy) {
        const int t = r == 0 ? 0 : (r <= TN ? r - 1 : r - TN);
        const uint32_t kx = (uint32_t)(((2 * ks) ^ ((t & 1) << 2)) << 4);
        if (r == 0 || r > TN) fa[slot][t] = lds_read16(smem, (a_rd ^ kx) + t * 4096 + copy * A_BYTES);
        else fb[slot][t] = lds_read16(smem, (b_rd ^ kx) + t * 4096 + copy * B_BYTES);
    };
    // One k step: the MFMAs on fragment slot `slot`; between them, one at a time, the LDS reads of
    // the next k step's fragments (k step ks_next of copy rcopy, into the other slot), the pieces
    // of the held tile (ha, hb) on their way to LDS copy wcopy if `moving`, and whatever `fetch`
    // issues (called with the MFMA's number).
    auto kstep = [&](int slot, int ks_next, uint32_t rcopy, auto moving, auto &ha, auto &hb, uint32_t wcopy, auto fetch) {
        constexpr int PA = std::remove_reference_t<decltype(ha)>::PIECES, PB = std::remove_reference_t<decltype(hb)>::PIECES;
        constexpr int PER = (PA + PB + NM - 1) / NM;
        constexpr int RQ = (NR + NM - 1) / NM;
        constexpr int GAP = NM / NR > 0 ? NM / NR : 1;
#pragma unroll
        for (int idx = 0; idx < NM; ++idx) {
            acc[idx / TN][idx % TN] = mfma32<BF16>(fb[slot][idx % TN], fa[slot][idx / TN], acc[idx / TN][idx % TN]);   // transposed block (see conv_store_points)
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

    // ---- prologue: k tile 0 -> LDS copy 0 (through set 0), k tile 1 requested into set 1.
    // A block past the last k tile is fully masked (k_left <= 0): nothing is loaded, the surplus
    // LDS copy holds zeros that are never read.
    const int64_t k_span = k_end - kt0 * kBK;                      // valid k counted from this program's first k tile
#pragma unroll
    for (int j = 0; j < 8; ++j) sa0.load_line(g, j, k_span);
    sa0.advance(g, 2);
    sb0.template load<true>(gB, n_left, k_span);
#pragma unroll
    for (int j = 0; j < 8; ++j) sa1.load_line(g, j, k_span - kBK);
    sa1.advance(g, 2);
    sb1.template load<true>(gB + kBK * 2, n_left, k_span - kBK);
    sa0.settle(g);
    sb0.settle();
    sa0.store(smem, 0);
    sb0.store(smem, B_BASE);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) frag_read(r, 0, 0, 0);

    // One k tile (four k steps) per trip.  Trip k multiplies LDS copy k % 2 (tile k); requests tile
    // k + 2 into the staging set that trip k - 1 emptied, the 8 lines of the unfolded input one
    // after every second MFMA of k step 0 and the filter chunks during k step 1; moves tile k + 1
    // (held in the other set) to the idle LDS copy during k step 2; and after the barrier that
    // publishes it reads its first fragments during k step 3.
    uint32_t cur = 0;
    auto trip = [&](auto &fa_set, auto &fb_set, auto &ha, auto &hb, int64_t k) {
        const uint32_t nxt = cur ^ 1u;
        const int64_t k_left = k_span - (k + 2) * kBK;
        const char *pb = gB + (k + 2) * (kBK * 2);
        kstep(0, 1, cur, std::false_type{}, ha, hb, nxt, [&](int idx) {
#pragma unroll
            for (int j = idx * 8 / NM; j < (idx + 1) * 8 / NM; ++j) fa_set.load_line(g, j, k_left);
        });
        fa_set.advance(g, 2);
        if constexpr (EDGE_B) {
            fb_set.template load<true>(pb, n_left, k_left);
            kstep(1, 2, cur, std::false_type{}, ha, hb, nxt, nullptr);
            hb.settle();
        } else {
            constexpr int PB = std::remove_reference_t<decltype(fb_set)>::PIECES;
            // (K is a multiple of 64 here: the tile exists or it does not; a request past the end is
            // redirected to the first tile -- no branch -- and lands in a copy that is never read)
            const char *pbc = k_left >= kBK ? pb : gB;
            kstep(1, 2, cur, std::false_type{}, ha, hb, nxt, [&](int idx) {
#pragma unroll
                for (int i = idx * PB / NM; i < (idx + 1) * PB / NM; ++i) fb_set.load_piece(pbc, i);
            });
        }
        ha.settle(g);
        kstep(0, 3, cur, std::true_type{}, ha, hb, nxt, nullptr);
        __syncthreads();
        kstep(1, 0, nxt, std::false_type{}, ha, hb, nxt, nullptr);
        cur = nxt;
    };
    int64_t k = 0;
    for (; k + 1 < kt_n; k += 2) {
        trip(sa0, sb0, sa1, sb1, k);
        trip(sa1, sb1, sa0, sb0, k + 1);
    }
    if (k < kt_n) trip(sa0, sb0, sa1, sb1, k);

    conv_store_transposed<BM, BN, int64_t>(g, acc, bi, row0 + wave_m * (BM / 2), col0 + wave_n * (BN / 2), lane);
}

template <int BN, bool BF16, bool EDGE_B>
static nt_status launch_conv_inst(const ConvArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)2 * (256 + BN) * kBK * sizeof(uint16_t);
    auto kern = gemm_conv_kernel<BN, BF16, EDGE_B>;
    static DeviceOnce configured;
    if (!configured.done()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured.set();
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_conv_kernel");
}

// bn: 128 or 256; nwg = ksplit * mt * nt
nt_status launch_conv(const ConvArgs &a, int bn, bool bf16, bool edge_b, int64_t nwg, hipStream_t s);
// Y[n, f, p, q] (strides syn, syf, Q, 1; out_dtype) = sum over the ksplit slices of ws, added in slice order
nt_status launch_conv_ws_sum(const float *ws, int ksplit, int64_t slice, void *Y, int64_t fpq, int64_t pq, int64_t syn, int64_t syf, int out_dtype, hipStream_t s);

}  // namespace nt
