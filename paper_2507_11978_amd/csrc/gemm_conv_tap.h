// Implicit-GEMM convolution (Section 4.3), 256 positions x 256 filters per program, reduction walked filter tap by filter tap.
//
// gemm_conv_direct.h walks the reduction index kk = (c, r, s) in the arrangement's order, so that the 32 kk of a slice mix
// several channels and taps and every load needs its own address arithmetic: about 190 vector and 50 scalar instructions
// per slice and wavefront, next to 64 matrix instructions.  A wavefront is alone on its SIMD in this tile, every
// instruction costs it an issue turn, and that arithmetic, not memory, bounded the kernel.  A sum may be taken in any
// order.  This kernel takes it tap-major: kk' = (r * S + s) * C + c, for C a multiple of 32.  A slice is then 32 consecutive
// channels of ONE tap, and everything that depends on the tap -- whether a run's input row lies in the top / bottom
// padding, whether its first or last element lies in the left / right padding -- is the same for the C / 32 slices of
// that tap and is recomputed only when the tap changes.  Per slice a load costs one addition: the lane's run offset
// (fixed) plus the slice's scalar offset c0 * H W + r * W + s.  The ring of four slices is unrolled as in
// gemm_direct16u_kernel (LDS addresses are immediates, load targets precomputed scalars).
// The filter is read from a copy in tap-major order, [filter][r * S + s][c], made by launch_conv_repack_filter.
//
// Runs that cannot be fetched as they are (see gemm_conv_direct.h for the layout and the numbering of positions):
//   * input row in the top / bottom padding, position past M: offset outside the buffer, zeros arrive;
//   * one element in the left / right padding: fetched, then overwritten with zero in LDS before the slice is published;
//   * the tensor's first run with a tap left of it starts before x, its last runs with taps right of them end after x:
//     the range check drops the 4-byte words that are not wholly inside x (counted from the run's start, so with a run
//     that starts at an odd element also the word that holds the tensor's last element).  Only wavefronts that hold such
//     runs (in the first and the last programs) look for them, only in a tap's first / last channel block, and then write
//     the run's elements that lie inside x into LDS one by one.
#pragma once
#include "gemm_conv_direct.h"

namespace nt {

template <bool BF16, bool TRACE = false>
__global__ __launch_bounds__(kThreads, 1) void gemm_conv_tap_kernel(const ConvArgs g)
{
    constexpr int BM = 256, BN = 256;
    constexpr int TM = BM / 32, TN = BN / 32;
    constexpr int kRing = 4;
    using TileB = DirectTile16<BN, KCONTIG>;
    constexpr int PER = 4;                                  // loads of the input per wavefront and slice
    constexpr int RB = 2 * BM;                              // bytes per kk row of the input's slice
    constexpr uint32_t A_BYTES = BM * kSliceK * 2, B_BYTES = TileB::BYTES, B_BASE = kRing * A_BYTES;
    constexpr uint32_t kOutside = 0x80000000u;
    static_assert(TileB::PER == 4 && TileB::RPF == 1, "schedule of the trip");
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int64_t bi, ti, tj;                                  // bi: which part of the k range (k split)
    if constexpr (TRACE) { bi = 0; ti = g.trace_program / g.nt; tj = g.trace_program % g.nt; }
    else locate_program(g.mt, g.nt, &bi, &ti, &tj);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int hi = lane >> 5;
    const int64_t row0 = ti * BM, col0 = tj * BN;
    const int64_t kt0 = bi * g.kt_per;
    const int64_t kt_n = g.kt - kt0 < g.kt_per ? g.kt - kt0 : g.kt_per;
    const int32_t k_first = (int32_t)(kt0 * kBK);
    const int32_t k_end = (int32_t)((kt0 + kt_n) * kBK < g.K ? (kt0 + kt_n) * kBK : g.K);
    const int32_t n_slices = (k_end - k_first) / kSliceK;
    const int32_t cb = g.CHW / g.HW / kSliceK;              // channel blocks (slices) per tap

    // ---- the filter: the direct kernel's k-major B operand, range checked
    const char *gB0 = reinterpret_cast<const char *>(g.Wt);
    const char *gB = reinterpret_cast<const char *>(g.Wt + col0 * g.ldb + k_first);
    TileB tb;
    tb.init(wave, lane, g.ldb, wave_n * (BN / 2), B_BASE);
    const u32x4 rsrc_a = make_rsrc(g.X, g.x_numel * 2);
    const u32x4 rsrc_b = make_rsrc(gB, ((int64_t)(g.N - 1) * g.ldb + g.K) * 2 - (gB - gB0));
    const u32x4 rsrc_z = u32x4{rsrc_a[0], rsrc_a[1], 0u, rsrc_a[3]};      // nothing is inside: every load reads zeros

    // ---- the input: per-lane state
    int32_t base[2];               // element offset of x[n, 0, p - ph, q0 - pw] of the lane's two runs (see ConvTileA)
    uint32_t masks[2];             // bits 0..7: input row p + r - ph inside the image (and m < M); bit 8 + 2 s / 9 + 2 s: with tap
                                   // column s the run's first element / its element last_e is padding
    bool risk_lo = false, risk_hi = false;
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
        // (conservative: a run of this lane may start before x in channel 0, or end after x in the last channel)
        risk_lo |= m_ok && base[e] < 0;
        risk_hi |= m_ok && (int64_t)base[e] + (int64_t)(g.CHW - g.HW) + (g.R - 1) * g.W + (g.S - 1) + 8 > g.x_numel;
    }
    const bool any_lo = __builtin_amdgcn_ballot_w64(risk_lo) != 0, any_hi = __builtin_amdgcn_ballot_w64(risk_hi) != 0;   // (uniform)
    // load j of a slice covers kk row 8 wave + 2 j + lane / 32 (one channel of the block) and run j % 2
    uint32_t rowoff[PER], voff[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) rowoff[j] = 2u * (uint32_t)(base[j & 1] + (8 * wave + 2 * j + hi) * g.HW);   // (wraps for the few negative ones)
    const uint32_t clr = (uint32_t)(wave * PER * 1024 + lane * 16);      // this lane's chunk inside a slice, load 0
    // transposing reads of the input's fragments (see DirectTile16<E, MNCONTIG>)
    uint32_t rd[TM];
    {
        const int gq = lane >> 4, i = lane & 15;
        const int kl = 8 * gq + (i >> 2);
        const int mn = wave_m * (BM / 2) + 4 * (i & 3);
        const int sw = DirectTile16<BM, MNCONTIG>::swizzle(kl);
#pragma unroll
        for (int t = 0; t < TM; ++t) rd[t] = (uint32_t)(kl * RB + ((((mn >> 3) + 2 * t) ^ sw) << 4) + ((mn >> 2) & 1) * 8);
    }

    // ---- the two walks over the program's slices (all scalar): the slice requested next, and the slice fixed up next
    const int32_t sl0 = k_first / kSliceK;
    int32_t rq_cblk = sl0 % cb, rq_r = (sl0 / cb) / g.S, rq_s = (sl0 / cb) % g.S, rq_left = n_slices;
    uint32_t rq_aoff = 2u * (uint32_t)(rq_cblk * kSliceK * g.HW + rq_r * g.W + rq_s), rq_boff = 0;
    int32_t st_cblk = rq_cblk, st_r = rq_r, st_s = rq_s, st_left = n_slices;
    auto retap_request = [&]() {                             // (after a change of rq_r: which runs are padding rows)
#pragma unroll
        for (int j = 0; j < PER; ++j) voff[j] = (masks[j & 1] >> rq_r) & 1u ? rowoff[j] : kOutside;
    };
    bool cf[2], cl[2], any_clear;
    auto retap_settle = [&]() {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            cf[e] = (masks[e] >> (8 + 2 * st_s)) & 1u & (masks[e] >> st_r);
            cl[e] = (masks[e] >> (9 + 2 * st_s)) & 1u & (masks[e] >> st_r);
        }
        any_clear = __builtin_amdgcn_ballot_w64(cf[0] || cf[1] || cl[0] || cl[1]) != 0;
    };
    retap_request();
    retap_settle();
    auto advance_request = [&]() {
        --rq_left;
        rq_boff += kSliceK * 2;
        rq_aoff += 2u * (uint32_t)(kSliceK * g.HW);
        if (++rq_cblk == cb) {                               // (uniform)
            rq_cblk = 0;
            if (++rq_s == g.S) { rq_s = 0; ++rq_r; }
            rq_aoff = 2u * (uint32_t)(rq_r * g.W + rq_s);
            retap_request();
        }
    };
    auto advance_settle = [&]() {
        --st_left;
        if (++st_cblk == cb) {                               // (uniform)
            st_cblk = 0;
            if (++st_s == g.S) { st_s = 0; ++st_r; }
            retap_settle();
        }
    };

    float4v acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.f;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    constexpr int NRA = 2 * TM, NRB = TN, NR = NRA + NRB;      // LDS reads per slice
    constexpr int NM = TM * TN, ND = PER + TileB::PER;
    static_assert(2 * NR <= NM * 3 / 2 && 8 * ND <= NM, "the trip's schedule: a read every other matrix instruction, a load every eighth");
    uint32_t tgt[kRing][ND];                                   // LDS targets of this wavefront's loads, per ring position: scalars
#pragma unroll
    for (int r = 0; r < kRing; ++r)
#pragma unroll
        for (int d = 0; d < ND; ++d)
            tgt[r][d] = d < PER ? lds0 + r * A_BYTES + (uint32_t)((wave * PER + d) * 1024)
                                : lds0 + B_BASE + r * B_BYTES + (uint32_t)((wave * TileB::PER + d - PER) * 1024);

    u32x4 fa[2][TM], fb[2][TN];
    typedef short4v __attribute__((address_space(3))) * lds_s4;
    auto read_a = [&](int q, int set, uint32_t ring) {         // half q % 2 (k 0..3 or 4..7 of the lane's run) of fragment q / 2
        const int t = q >> 1, part = q & 1;
        const u32x2 v = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(smem + (rd[t] + ring * A_BYTES + (uint32_t)(part * 4 * RB)))));
        fa[set][t][2 * part] = v[0];
        fa[set][t][2 * part + 1] = v[1];
    };
    auto lds_read = [&](int r, int set, uint32_t ring) {
        if (r < 2) read_a(r, set, ring);
        else if (r < 2 + NRB) tb.read(fb[set], smem, r - 2, ring * B_BYTES);
        else read_a(r - NRB, set, ring);
    };
    // load d of the slice the request walk stands at, into ring position `ring`; in two halves that go behind different
    // matrix instructions (see gemm_direct16u_kernel).  ra / rb: the operands' resources, or rsrc_z past the program's last slice.
    auto dma_aim = [&](int d, int ring) { asm volatile("s_mov_b32 m0, %0" : : "s"(tgt[ring][d]) : "memory"); };
    auto dma_go = [&](int d, const u32x4 &ra, const u32x4 &rb) {
        if (d < PER) {
            const uint32_t at = voff[d] + rq_aoff;
            asm volatile("buffer_load_dwordx4 %0, %1, 0 offen lds" : : "v"(at), "s"(ra) : "memory");
        } else {
            asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" : : "v"(tb.voff[d - PER]), "s"(rb), "s"(rq_boff) : "memory");
        }
    };

    // What a slice needs once it has landed at ring position `ring` (the settle walk stands at it).
    auto zero16 = [&](uint32_t at) { *reinterpret_cast<uint16_t *>(smem + at) = 0; };
    auto settle = [&](uint32_t ring) {
        if (st_left <= 0) return;                                                        // (uniform: a slice past the last is zeros and stays so)
        if ((any_lo && st_cblk == 0) || (any_hi && st_cblk == cb - 1)) {                 // (uniform, first / last programs only)
            const int32_t lim = (int32_t)g.x_numel;
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                const int32_t l_off = base[j & 1] + ((st_cblk * kSliceK + 8 * wave + 2 * j + hi) * g.HW + st_r * g.W + st_s);
                const bool row_in = (masks[j & 1] >> st_r) & 1u;
                if (row_in && (l_off < 0 || l_off + 8 > lim)) {
                    const uint32_t at = ring * A_BYTES + clr + (uint32_t)(j * 1024);
                    for (int i = 0; i < 8; ++i) {
                        const int32_t idx = l_off + i;
                        *reinterpret_cast<uint16_t *>(smem + at + 2 * i) = idx >= 0 && idx < lim ? g.X[idx] : (uint16_t)0;
                    }
                }
            }
        }
        if (any_clear) {                                                                 // (uniform)
            const uint32_t at = ring * A_BYTES + clr, last = at + 2u * (uint32_t)g.last_e;
            if (cf[0]) { zero16(at); zero16(at + 2048); }
            if (cf[1]) { zero16(at + 1024); zero16(at + 3072); }
            if (cl[0]) { zero16(last); zero16(last + 2048); }
            if (cl[1]) { zero16(last + 1024); zero16(last + 3072); }
        }
        advance_settle();
    };

    if constexpr (TRACE) {
        for (int32_t s = 0; s <= g.trace_slice; ++s) {
#pragma unroll
            for (int d = 0; d < ND; ++d) {
                dma_aim(d, 0);
                asm volatile("s_nop 0");
                dma_go(d, rsrc_a, rsrc_b);
            }
            advance_request();
            NT_WAIT_VMCNT(0);
            if (s < g.trace_slice) advance_settle();
        }
        settle(0);
        __syncthreads();
        const bool first = g.trace_operand == 0;
        for (int e = tid; e < (first ? BM : BN) * kSliceK; e += kThreads) {
            const uint32_t at = first ? DirectTile16<BM, MNCONTIG>::place(e / kSliceK, e % kSliceK) : B_BASE + TileB::place(e / kSliceK, e % kSliceK);
            g.trace_out[e] = *reinterpret_cast<const uint16_t *>(smem + at);
        }
        return;
    }

    // One trip = one slice: the matrix instructions on fragment set SET; behind them the LDS reads of the next slice (ring
    // position RING + 1) into the other set and the loads of the slice three further on into ring position RING.
    auto trip = [&](auto ring_c, auto set_c) {
        constexpr int RING = decltype(ring_c)::value, SET = decltype(set_c)::value;
        constexpr int NXT = (RING + 1) % kRing;
        const bool live = rq_left > 0;                             // (uniform)
        const u32x4 ra = live ? rsrc_a : rsrc_z, rb = live ? rsrc_b : rsrc_z;
#pragma unroll
        for (int idx = 0; idx < NM; ++idx) {
            const int tm = idx / TN, tn = idx % TN;
            mfma16<BF16>(acc[tm][tn], fb[SET][tn], fa[SET][tm]);      // transposed block: a lane holds position lane % 16 (see conv_store_points16)
            if (idx % 2 == 0 && idx / 2 < NR) lds_read(idx / 2, SET ^ 1, NXT);
            if (idx % 8 == 1 && idx / 8 < ND) dma_aim(idx / 8, RING);
            if (idx % 8 == 3 && idx / 8 < ND) dma_go(idx / 8, ra, rb);
            __builtin_amdgcn_sched_barrier(0);
        }
        advance_request();
    };
    using std::integral_constant;

    // prologue: slices 0 .. 3 requested; slice 0 fixed up and published; its fragments into set 0
#pragma unroll
    for (int s = 0; s < kRing; ++s) {
        const bool live = rq_left > 0;
        const u32x4 ra = live ? rsrc_a : rsrc_z, rb = live ? rsrc_b : rsrc_z;
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            dma_aim(d, s);
            asm volatile("s_nop 0");
            dma_go(d, ra, rb);
        }
        advance_request();
    }
    NT_WAIT_VMCNT((kRing - 1) * ND);
    settle(0);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) lds_read(r, 0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // Slice s sits at ring position s % 4.  At the top of trip s this wavefront's part of slice s + 1 must have landed; it
    // is fixed up, and the barrier then says that slice s + 1 is complete and that every wavefront holds its fragments of
    // slice s in registers, so that slice s + 4 can overwrite it.  One pass = four trips.  A number of slices that is no
    // multiple of four is rounded up: the slices past the last are requested from rsrc_z, arrive as zeros, and their trips
    // add nothing.
    for (int32_t sl = 0; sl < n_slices; sl += kRing) {
        NT_WAIT_VMCNT(2 * ND); settle(1); __syncthreads(); trip(integral_constant<int, 0>{}, integral_constant<int, 0>{});
        NT_WAIT_VMCNT(2 * ND); settle(2); __syncthreads(); trip(integral_constant<int, 1>{}, integral_constant<int, 1>{});
        NT_WAIT_VMCNT(2 * ND); settle(3); __syncthreads(); trip(integral_constant<int, 2>{}, integral_constant<int, 0>{});
        NT_WAIT_VMCNT(2 * ND); settle(0); __syncthreads(); trip(integral_constant<int, 3>{}, integral_constant<int, 1>{});
        // (wait states between the last matrix instruction and anything the compiler may do to an accumulator at the
        // loop's end: it does not know that the inline assembly is a matrix instruction)
        asm volatile("s_nop 7" ::: "memory");
    }
    NT_WAIT_VMCNT(0);
    __syncthreads();
    asm volatile("s_nop 15" ::: "memory");

    const int64_t row_w = row0 + wave_m * (BM / 2), col_w = col0 + wave_n * (BN / 2);
    if (g.out_dtype == NT_F32) conv_store_points16<BM, BN, NT_F32>(g, acc, bi, row_w, col_w, lane);
    else if (g.out_dtype == NT_F16) conv_store_points16<BM, BN, NT_F16>(g, acc, bi, row_w, col_w, lane);
    else conv_store_points16<BM, BN, NT_BF16>(g, acc, bi, row_w, col_w, lane);
}

template <bool BF16, bool TRACE = false>
static nt_status launch_conv_tap_inst(const ConvArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)4 * (256 + 256) * kSliceK * sizeof(uint16_t);
    auto kern = gemm_conv_tap_kernel<BF16, TRACE>;
    static DeviceOnce configured;
    if (!configured.done()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured.set();
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_conv_tap_kernel");
}

// a.Wt: the filter in tap-major order (see launch_conv_repack_filter), a.ldb its row pitch; nwg = ksplit * mt * nt
nt_status launch_conv_tap(const ConvArgs &a, bool bf16, int64_t nwg, hipStream_t s);
nt_status launch_conv_tap_trace(const ConvArgs &a, hipStream_t s);
// filter [F][C][R * S] (row pitch ldb) -> out [F][R * S][C] (row pitch C R S)
nt_status launch_conv_repack_filter(const uint16_t *w, int64_t ldb, uint16_t *out, int32_t F, int32_t C, int32_t RS, hipStream_t s);

}  // namespace nt
