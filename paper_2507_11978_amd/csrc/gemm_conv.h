// Implicit-GEMM convolution kernel (Section 4.3) for the common dense case: contiguous
// NCHW input, unit conv stride, contiguous KCRS filter, output dense in (p, q).
//
// The arrangement of Section 4.3 lowers the input to the matrix A[m, kk] with
// m = (n, p, q), kk = (c, r, s) and A[m, kk] = x[n, c, p + r - pad_h, q + s - pad_w]
// (zero outside the image).  A is contiguous along m, so its (256 x 64) block is staged
// like a column-major operand: every thread owns 8 consecutive m (one run of q inside an
// image row; Q is a multiple of 8) for 8 consecutive kk, loads each run with one 16-byte
// load from the unfolded position inside x -- the unfolded matrix itself never exists --
// clears the one element that can fall into the left / right padding, zeroes runs whose
// input row lies in the top / bottom padding, and transposes the 8 x 8 patch in registers
// into the k-contiguous LDS layout.  The filter is a k-contiguous B operand; the MFMA core
// and the LDS layout are those of the staged GEMM kernel.  The output tile is written
// along m (contiguous in NKPQ), 4 consecutive m per store.
#pragma once
#include "gemm_fast.h"

namespace nt {

struct ConvArgs {
    const uint16_t *X;             // input, contiguous [N, C, H, W]
    const uint16_t *Wt;            // filter as B[kk, f] = Wt[f * ldb + kk]
    void *Y;                       // output: element (m = n*PQ + pq, f) at n*syn + f*syf + pq
    int64_t ldb, syn, syf;
    int64_t x_numel;               // N*C*H*W
    int32_t M, N, K;               // GEMM sizes: N*P*Q, filters, C*R*S
    int32_t PQ, Q, H, W, HW, CHW, RS, S, R, ph, pw;
    uint32_t inv_rs, inv_s;        // reciprocals of R*S and S (see udiv_small)
    int64_t mt, nt, kt;
    int out_dtype;
};

// floor(t / d) for 0 <= t < 2^16 with inv = floor(2^32 / d) + 1 (d >= 2), inv = 0 standing for d = 1
__device__ __forceinline__ uint32_t udiv_small(uint32_t t, uint32_t inv) { return inv ? __umulhi(t, inv) : t; }

// staging of the (256 x 64) block of the unfolded input
struct StageConv {
    uint32_t r[8][4];              // [k line][packed pairs of m]
    uint32_t wbase;
    int kb, rb;
    int32_t base;                  // element offset of x[n, 0, p - ph, q0 - pw]
    int32_t q0;
    uint32_t hmask;                // bit r: input row p + r - ph lies inside the image (and m < M)
    int32_t c, rs;                 // channel and r*S+s of this thread's first k line in the current k tile

    // first_tile: the k tile this set fetches first
    __device__ __forceinline__ void init(int tid, const ConvArgs &g, int64_t row0, int first_tile)
    {
        kb = tid >> 5;
        rb = tid & 31;
        wbase = (uint32_t)(rb * 8 * 128 + ((kb ^ (rb & 7)) << 4));
        const int64_t m = row0 + rb * 8;
        const bool m_ok = m < g.M;
        const uint32_t mm = m_ok ? (uint32_t)m : 0u;
        const uint32_t nn = mm / (uint32_t)g.PQ;
        const uint32_t pq = mm - nn * (uint32_t)g.PQ;
        const uint32_t p = pq / (uint32_t)g.Q;
        q0 = (int32_t)(pq - p * (uint32_t)g.Q);
        base = (int32_t)(nn * (uint32_t)g.CHW) + ((int32_t)p - g.ph) * g.W + q0 - g.pw;
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
    // tile the state points at; k_left: valid k from the tile origin.
    __device__ __forceinline__ void load_line(const ConvArgs &g, int j, int64_t k_left)
    {
        const uint16_t *X = g.X;
        const uint32_t t = (uint32_t)(rs + j);
        const uint32_t dq = udiv_small(t, g.inv_rs);          // t / RS
        const int32_t cj = c + (int32_t)dq;
        const uint32_t rsj = t - dq * (uint32_t)g.RS;
        const uint32_t rr = udiv_small(rsj, g.inv_s);          // rsj / S
        const int32_t ss = (int32_t)(rsj - rr * (uint32_t)g.S);
        const bool ok = kb * 8 + j < k_left && ((hmask >> rr) & 1u);
        const int64_t off = (int64_t)base + (int64_t)cj * g.HW + (int32_t)rr * g.W + ss;
        const int32_t w0 = q0 + ss - g.pw;
        u32x4 v{0, 0, 0, 0};
        if (ok) {
            if (off >= 0 && off + 8 <= g.x_numel) {
                __builtin_memcpy(&v, X + off, 16);
            } else {                                           // first / last run of the whole tensor
                uint32_t e[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) e[q] = (off + q >= 0 && off + q < g.x_numel) ? (uint32_t)X[off + q] : 0u;
                v = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
            }
            if (w0 < 0) v[0] &= 0xffff0000u;                   // q0 + s - pad = -1: left padding
            if (w0 + 7 >= g.W) v[3] &= 0x0000ffffu;            // ... = W: right padding
        }
        r[j][0] = v[0]; r[j][1] = v[1]; r[j][2] = v[2]; r[j][3] = v[3];
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

template <int BN, bool BF16, bool EDGE_B>
__global__ __launch_bounds__(kThreads) void gemm_conv_kernel(const ConvArgs g)
{
    constexpr int BM = 256;
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr uint32_t A_BYTES = BM * kBK * 2, B_BYTES = BN * kBK * 2;
    constexpr uint32_t B_BASE = 2 * A_BYTES;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    int64_t bi, ti, tj;
    locate_program(g.mt, g.nt, &bi, &ti, &tj);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int l32 = lane & 31, hi = lane >> 5;
    const int64_t row0 = ti * BM, col0 = tj * BN;

    const char *gB = reinterpret_cast<const char *>(g.Wt + col0 * g.ldb);
    const int64_t n_left = g.N - col0;

    // two sets of staging registers: a tile is requested two trips before it is multiplied
    StageConv sa0, sa1;
    StageK<BN, true> sb0, sb1;
    sa0.init(tid, g, row0, 0);
    sa1.init(tid, g, row0, 1);
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
            acc[idx / TN][idx % TN] = mfma32<BF16>(fa[slot][idx / TN], fb[slot][idx % TN], acc[idx / TN][idx % TN]);
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
#pragma unroll
    for (int j = 0; j < 8; ++j) sa0.load_line(g, j, g.K);
    sa0.advance(g, 2);
    sb0.template load<true>(gB, n_left, g.K);
#pragma unroll
    for (int j = 0; j < 8; ++j) sa1.load_line(g, j, (int64_t)g.K - kBK);
    sa1.advance(g, 2);
    sb1.template load<true>(gB + kBK * 2, n_left, (int64_t)g.K - kBK);
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
        const int64_t k_left = (int64_t)g.K - (k + 2) * kBK;
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
            const bool inside = k_left >= kBK;                  // (K is a multiple of 64 here)
            kstep(1, 2, cur, std::false_type{}, ha, hb, nxt, [&](int idx) {
                if (inside)
#pragma unroll
                    for (int i = idx * PB / NM; i < (idx + 1) * PB / NM; ++i) fb_set.template load_piece<false>(pb, i);
            });
        }
        kstep(0, 3, cur, std::true_type{}, ha, hb, nxt, nullptr);
        __syncthreads();
        kstep(1, 0, nxt, std::false_type{}, ha, hb, nxt, nullptr);
        cur = nxt;
    };
    int64_t k = 0;
    for (; k + 1 < g.kt; k += 2) {
        trip(sa0, sb0, sa1, sb1, k);
        trip(sa1, sb1, sa0, sb0, k + 1);
    }
    if (k < g.kt) trip(sa0, sb0, sa1, sb1, k);

    // epilogue: lane holds, per 32 x 32 block, 4 groups of 4 consecutive m for one filter f.
    // 4 consecutive m (aligned to 4) lie in one image because P*Q is a multiple of 8.
    const bool f16 = g.out_dtype == NT_F16;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int64_t m = row0 + wave_m * (BM / 2) + tm * 32 + 8 * gq + 4 * hi;
            if (m >= g.M) continue;
            const uint32_t n = (uint32_t)m / (uint32_t)g.PQ;
            const uint32_t pq = (uint32_t)m - n * (uint32_t)g.PQ;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int64_t f = col0 + wave_n * (BN / 2) + tn * 32 + l32;
                if (f >= g.N) continue;
                const int64_t o = (int64_t)n * g.syn + f * g.syf + pq;
                if (g.out_dtype == NT_F32) {
                    float *y = reinterpret_cast<float *>(g.Y) + o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) y[i] = acc[tm][tn][4 * gq + i];
                } else {
                    uint16_t h[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) h[i] = f16 ? f32_to_f16_rne(acc[tm][tn][4 * gq + i]) : f32_to_bf16_rne(acc[tm][tn][4 * gq + i]);
                    const u32x2 v{h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16)};
                    __builtin_memcpy(reinterpret_cast<uint16_t *>(g.Y) + o, &v, 8);
                }
            }
        }
}

template <int BN, bool BF16, bool EDGE_B>
static nt_status launch_conv_inst(const ConvArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)2 * (256 + BN) * kBK * sizeof(uint16_t);
    auto kern = gemm_conv_kernel<BN, BF16, EDGE_B>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_conv_kernel");
}

// bn: 128 or 256
nt_status launch_conv(const ConvArgs &a, int bn, bool bf16, bool edge_b, int64_t nwg, hipStream_t s);

}  // namespace nt
