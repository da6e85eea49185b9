// Implicit-GEMM convolution (Section 4.3), 256 positions x 256 filters per program, reduction walked filter tap by filter tap.
//
// gemm_conv_direct.h walks the reduction index kk = (c, r, s) in the arrangement's order, so that the 32 kk of a slice mix
// several channels and taps and every load needs its own address arithmetic: about 190 vector and 50 scalar instructions
// per slice and wavefront, next to 64 matrix instructions.  A wavefront is alone on its SIMD in this tile, every
// instruction costs it an issue turn, and that arithmetic, not memory, bounded the kernel.  A sum may be taken in any
// order.  This kernel takes it tap-major: kk' = (r * S + s) * C + c, for C a multiple of 32.  A slice is then 32 consecutive
// channels of ONE tap, and everything that depends on the tap -- whether a run's input row lies in the top / bottom
// padding, whether its first or last element lies in the left / right padding -- is the same for the C / 32 slices of
// that tap: one bit per tap and lane, tested per slice.  Per slice a load costs one addition: the lane's run offset
// (fixed) plus the slice's scalar offset c0 * H W + r * W + s.  The ring of four slices is unrolled as in
// gemm_direct16u_kernel (LDS addresses are immediates, load targets precomputed scalars), and all of a slice's
// bookkeeping -- the two walks over the slices, the tests -- is branch-free and sits between the matrix instructions
// (whatever precedes a trip's first matrix instruction is time in which the matrix pipe idles: with that bookkeeping in
// front of every trip, under branches, a trip took 1.6 times the time of its matrix instructions).
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

// One program: TM: its tile is 32 TM positions high (192, 224 or 256; the LDS slots are laid out for 256 either way), starts
// at position row_base + ti * 32 TM and at filter 256 tj; bi: which part of the k range (k split).
template <bool BF16, int TM, bool TRACE>
__device__ __forceinline__ void conv_tap_program(const ConvArgs &g, char *smem, int64_t bi, int64_t ti, int64_t tj, int64_t row_base)
{
    constexpr int BM = 32 * TM, BN = 256;
    constexpr int TN = BN / 32;
    constexpr int SLOT_M = 256;                             // positions per LDS slot
    constexpr int kRing = 4;
    using TileB = DirectTile16<BN, KCONTIG>;
    constexpr int PER = 4;                                  // loads of the input per wavefront and slice
    constexpr int RB = 2 * SLOT_M;                          // bytes per kk row of the input's slice
    constexpr uint32_t A_BYTES = SLOT_M * kSliceK * 2, B_BYTES = TileB::BYTES, B_BASE = kRing * A_BYTES;
    constexpr uint32_t kOutside = 0x80000000u;
    static_assert(TileB::PER == 4 && TileB::RPF == 1, "schedule of the trip");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int hi = lane >> 5;
    const int64_t row0 = row_base + ti * BM, col0 = tj * BN;
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

    // ---- the input: per-lane state.  A lane owns two runs of 8 positions (see ConvTileA); per run, one bit per filter tap
    // t = r * S + s (the host admits R * S <= 32):
    //   rows_in: the tap's input row p + r - ph lies inside the image (and the run's positions exist);
    //   pad_first / pad_last: rows_in, and with the tap's column s the run's first element / its element last_e is padding.
    int32_t base[2];               // element offset of x[n, 0, p - ph, q0 - pw]
    uint32_t rows_in[2], pad_first[2], pad_last[2];
    bool risk_lo = false, risk_hi = false;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int chunk = (lane & 31) ^ (((2 * e + hi) << 2) | ((wave & 1) << 1));
        const int64_t m = row0 + chunk * 8;
        const bool m_ok = m < g.M && chunk * 8 < BM;
        const uint32_t mm = m_ok ? (uint32_t)m : 0u;
        const uint32_t nn = mm / (uint32_t)g.PQ8;
        const uint32_t pq = mm - nn * (uint32_t)g.PQ8;
        const uint32_t p = pq / (uint32_t)g.Q8;
        const int32_t q0 = (int32_t)(pq - p * (uint32_t)g.Q8);
        base[e] = (int32_t)(nn * (uint32_t)g.CHW) + ((int32_t)p - g.ph) * g.W + q0 - g.pw;
        // (closed forms, no loop over the taps: `rep` has bit r * S set for every filter row r whose input row is inside the
        // image; a set of columns, as a mask of S bits, times rep is that set in every such row.  R * S <= 32.)
        auto low_bits = [](int n) { return n >= 32 ? 0xffffffffu : (1u << n) - 1u; };
        uint32_t rep = 0;
        for (int rr = 0; rr < g.R; ++rr) {
            const int h = (int)p + rr - g.ph;
            rep |= m_ok && (uint32_t)h < (uint32_t)g.H ? 1u << (rr * g.S) : 0u;
        }
        const uint32_t cols = low_bits(g.S);
        const int nf = g.pw - q0;                                   // columns s < nf: the run's first element is padding
        const int nl = g.W + g.pw - g.Q + 1;                        // columns s >= nl: the row's last output position reads padding
        const uint32_t in = rep * cols;
        const uint32_t pf = rep * low_bits(nf < 0 ? 0 : nf > g.S ? g.S : nf);
        const uint32_t pl = q0 + 8 >= g.Q ? rep * (cols & ~low_bits(nl < 0 ? 0 : nl > g.S ? g.S : nl)) : 0u;
        rows_in[e] = in; pad_first[e] = pf; pad_last[e] = pl;
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
    const uint32_t clr_last = clr + 2u * (uint32_t)g.last_e;
    // transposing reads of the input's fragments (see DirectTile16<E, MNCONTIG>)
    uint32_t rd[TM];
    {
        const int gq = lane >> 4, i = lane & 15;
        const int kl = 8 * gq + (i >> 2);
        const int mn = wave_m * (BM / 2) + 4 * (i & 3);
        const int sw = DirectTile16<SLOT_M, MNCONTIG>::swizzle(kl);
#pragma unroll
        for (int t = 0; t < TM; ++t) rd[t] = (uint32_t)(kl * RB + ((((mn >> 3) + 2 * t) ^ sw) << 4) + ((mn >> 2) & 1) * 8);
    }

    // ---- two walks over the program's slices, all scalar and branch-free: the slice requested next, the slice fixed up next
    // (each walk's step is cut into pieces of a few instructions, which the trip places behind different matrix instructions)
    struct Walk { int32_t idx, cblk, r, s, tap; bool wrap; };
    const int32_t sl0 = k_first / kSliceK;
    const Walk first{0, sl0 % cb, (sl0 / cb) / g.S, (sl0 / cb) % g.S, sl0 / cb, false};
    auto step_a = [&](Walk &w) {
        w.wrap = w.cblk + 1 == cb;
        ++w.idx;
        w.cblk = w.wrap ? 0 : w.cblk + 1;
        w.tap += w.wrap ? 1 : 0;
    };
    auto step_b = [&](Walk &w) {
        const int32_t s1 = w.s + (w.wrap ? 1 : 0);
        const bool wrap_s = s1 == g.S;
        w.s = wrap_s ? 0 : s1;
        w.r += wrap_s ? 1 : 0;
    };
    Walk rq = first, st = first;
    // request side: the slice's offsets, which loads fetch a padding row, and the resources (past the program's last slice:
    // records of length zero, so that zeros arrive)
    uint32_t rq_aoff, rq_boff;
    u32x4 ra = rsrc_a, rb = rsrc_b;
    auto aim_request_a = [&]() {
        rq_aoff = 2u * (uint32_t)(rq.cblk * kSliceK * g.HW + rq.r * g.W + rq.s);
        rq_boff = (uint32_t)rq.idx * (kSliceK * 2);
    };
    auto aim_request_b = [&](int e) {
        const bool in = (rows_in[e] & (1u << (rq.tap & 31))) != 0;
        voff[e] = in ? rowoff[e] : kOutside;
        voff[e + 2] = in ? rowoff[e + 2] : kOutside;
    };
    auto aim_request_c = [&]() {
        const bool live = rq.idx < n_slices;                                       // (uniform)
        ra[2] = live ? rsrc_a[2] : 0u;
        rb[2] = live ? rsrc_b[2] : 0u;
    };
    auto step_request = [&]() { step_a(rq); step_b(rq); };
    auto aim_request = [&]() { aim_request_a(); aim_request_b(0); aim_request_b(1); aim_request_c(); };
    // fix-up side: which of this lane's runs have a padding element to clear (as wavefront masks), and whether this wavefront
    // has to look for runs that cross an end of x
    uint64_t mf0, mf1, ml0, ml1;
    uint32_t st_bit;
    bool hazard;
    auto aim_settle_a = [&]() {
        const bool live = st.idx < n_slices;                                       // (a slice past the last is zeros and stays so)
        st_bit = live ? 1u << (st.tap & 31) : 0u;
        hazard = live & ((any_lo & (st.cblk == 0)) | (any_hi & (st.cblk == cb - 1)));
    };
    auto aim_settle_b = [&](int e) {
        if (e == 0) {
            mf0 = __builtin_amdgcn_ballot_w64((pad_first[0] & st_bit) != 0);
            ml0 = __builtin_amdgcn_ballot_w64((pad_last[0] & st_bit) != 0);
        } else {
            mf1 = __builtin_amdgcn_ballot_w64((pad_first[1] & st_bit) != 0);
            ml1 = __builtin_amdgcn_ballot_w64((pad_last[1] & st_bit) != 0);
        }
    };
    auto step_settle = [&]() { step_a(st); step_b(st); };
    auto aim_settle = [&]() { aim_settle_a(); aim_settle_b(0); aim_settle_b(1); };

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
    // The trip's schedule: PRE matrix instructions before the barrier; after it an LDS read behind every other one; the
    // pieces of the request walk's step behind the odd ones of the first HOLD; the halves of load d behind the 2nd and 4th
    // of the d-th group of STEP from then on; the pieces of the settle walk's step behind the 1st of the first groups.
    // (the lowest tile has 48 matrix instructions per trip: two fewer before the barrier and one fewer ahead of the loads leave
    // the 8 loads their 4 each)
    constexpr int PRE = TM >= 7 ? 8 : 6, HOLD = TM >= 7 ? 11 : 10, STEP = (NM - PRE - HOLD) / ND;
    static_assert(2 * NR <= NM - PRE && STEP >= 4 && HOLD >= 10, "the trip's schedule");
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
    // matrix instructions (see gemm_direct16u_kernel).  ra / rb: the operands' resources (of length zero past the program's last slice).
    // (loads of the input, two thirds of which start at an odd element and keep the texture addresser busy four times as long,
    // alternate with loads of the filter: i-th load = input load i / 2 or filter load i / 2)
    auto nth = [](int i) { return i % 2 == 0 ? i / 2 : PER + i / 2; };
    uint32_t a_at = 0;                                         // (the input load's address: computed a matrix instruction ahead of the load)
    auto dma_aim = [&](int d, int ring) {
        asm volatile("s_mov_b32 m0, %0" : : "s"(tgt[ring][d]) : "memory");
        if (d < PER) { a_at = voff[d] + rq_aoff; asm volatile("" : "+v"(a_at)); }
    };
    auto dma_go = [&](int d, const u32x4 &ra, const u32x4 &rb) {
        if (d < PER) {
            asm volatile("buffer_load_dwordx4 %0, %1, 0 offen lds" : : "v"(a_at), "s"(ra) : "memory");
        } else {
            asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" : : "v"(tb.voff[d - PER]), "s"(rb), "s"(rq_boff) : "memory");
        }
    };

    // What the slice the settle walk stands at needs once this wavefront's part of it has landed at ring position RING.
    // Common: the padding elements of runs are overwritten with zero, under the four wavefront masks (every lane is active
    // here; the execution mask is put back before the statement ends).  Rare: runs that cross an end of x.
    auto settle_hazard = [&](auto ring_c) {
        constexpr uint32_t o = decltype(ring_c)::value * A_BYTES;
        if (hazard) {                                                                    // (uniform, first / last programs only)
            const int32_t lim = (int32_t)g.x_numel;
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                const int32_t l_off = base[j & 1] + ((st.cblk * kSliceK + 8 * wave + 2 * j + hi) * g.HW + st.r * g.W + st.s);
                const bool row_in = (rows_in[j & 1] >> (st.tap & 31)) & 1u;
                if (row_in && (l_off < 0 || l_off + 8 > lim)) {
                    const uint32_t at = o + clr + (uint32_t)(j * 1024);
                    for (int i = 0; i < 8; ++i) {
                        const int32_t idx = l_off + i;
                        *reinterpret_cast<uint16_t *>(smem + at + 2 * i) = idx >= 0 && idx < lim ? g.X[idx] : (uint16_t)0;
                    }
                }
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);                                           // (those LDS writes before the ones below: lgkmcnt(0))
        }
    };
    // piece q = 0 .. 3 of the clears: the first elements of run 0, of run 1, the last elements of run 0, of run 1
    auto settle_piece = [&](auto ring_c, int q) {
        constexpr uint32_t o = decltype(ring_c)::value * A_BYTES;
        const uint64_t m = q == 0 ? mf0 : q == 1 ? mf1 : q == 2 ? ml0 : ml1;
        const uint32_t at = q < 2 ? clr : clr_last;
        if (q % 2 == 0)
            asm volatile("s_mov_b64 exec, %[m]\n\tds_write_b16 %[a], %[z] offset:%[o0]\n\tds_write_b16 %[a], %[z] offset:%[o2]\n\ts_mov_b64 exec, -1"
                         : : [m] "s"(m), [a] "v"(at), [z] "v"(0u), [o0] "n"(o), [o2] "n"(o + 2048) : "memory");
        else
            asm volatile("s_mov_b64 exec, %[m]\n\tds_write_b16 %[a], %[z] offset:%[o1]\n\tds_write_b16 %[a], %[z] offset:%[o3]\n\ts_mov_b64 exec, -1"
                         : : [m] "s"(m), [a] "v"(at), [z] "v"(0u), [o1] "n"(o + 1024), [o3] "n"(o + 3072) : "memory");
    };
    auto settle = [&](auto ring_c) {
        settle_hazard(ring_c);
#pragma unroll
        for (int q = 0; q < 4; ++q) settle_piece(ring_c, q);
    };
    using std::integral_constant;

    if constexpr (TRACE) {
        for (int32_t s = 0; s <= g.trace_slice; ++s) {
            if (s > 0) { step_request(); step_settle(); }
            aim_request();
#pragma unroll
            for (int d = 0; d < ND; ++d) {
                dma_aim(d, 0);
                asm volatile("s_nop 0");
                dma_go(d, ra, rb);
            }
            NT_WAIT_VMCNT(0);
        }
        aim_settle();
        settle(integral_constant<int, 0>{});
        __syncthreads();
        const bool first = g.trace_operand == 0;
        for (int e = tid; e < (first ? BM : BN) * kSliceK; e += kThreads) {
            const uint32_t at = first ? DirectTile16<SLOT_M, MNCONTIG>::place(e / kSliceK, e % kSliceK) : B_BASE + TileB::place(e / kSliceK, e % kSliceK);
            g.trace_out[e] = *reinterpret_cast<const uint16_t *>(smem + at);
        }
        return;
    }

    // One trip = one slice: the matrix instructions on fragment set SET (slice s, in registers since the trip before).  This
    // wavefront's part of slice s + 1 has landed (the caller has waited for it): it is fixed up behind the first four matrix
    // instructions (a piece of the clears each), and while those LDS writes are on their way the rest of the first PRE go out;
    // then the barrier, which says that slice s + 1 is complete
    // and that every wavefront holds its fragments of slice s, so that slice s + 4 may overwrite it.  Behind the remaining
    // matrix instructions: the LDS reads of slice s + 1 (ring position RING + 1) into the other set, the request walk's step
    // to slice s + 4 and that slice's loads into ring position RING, and the settle walk's step to slice s + 2.
    auto trip = [&](auto ring_c, auto set_c) {
        constexpr int RING = decltype(ring_c)::value, SET = decltype(set_c)::value;
        constexpr int NXT = (RING + 1) % kRing;
        settle_hazard(integral_constant<int, NXT>{});
#pragma unroll
        for (int idx = 0; idx < NM; ++idx) {
            const int tm = idx / TN, tn = idx % TN;
            if (idx == PRE) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");        // (the clears below have reached LDS)
                __syncthreads();
            }
            mfma16<BF16>(acc[tm][tn], fa[SET][tm], fb[SET][tn]);      // a lane holds filter lane % 16 and 4 positions (see conv_store_rows16)
            if (idx < 4) settle_piece(integral_constant<int, NXT>{}, idx);     // the clears of slice s + 1, one piece behind each of the first four
            if (idx >= PRE) {
                const int i = idx - PRE;
                if (i % 2 == 0 && i / 2 < NR) lds_read(i / 2, SET ^ 1, NXT);
                if (i == 1) step_a(rq);
                if (i == 3) step_b(rq);
                if (i == 5) aim_request_a();
                if (i == 7) aim_request_b(0);
                if (i == 9) { aim_request_b(1); aim_request_c(); }
                if (i >= HOLD) {
                    const int k = i - HOLD;
                    if (k % STEP == 1 && k / STEP < ND) dma_aim(nth(k / STEP), RING);
                    if (k % STEP == 3 && k / STEP < ND) dma_go(nth(k / STEP), ra, rb);
                    if (k == 0) step_a(st);
                    if (k == STEP) step_b(st);
                    if (k == 2 * STEP) aim_settle_a();
                    if (k == 3 * STEP) aim_settle_b(0);
                    if (k == 4 * STEP) aim_settle_b(1);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // prologue: slices 0 .. 3 requested; slice 0 fixed up and published; its fragments into set 0
#pragma unroll
    for (int s = 0; s < kRing; ++s) {
        if (s > 0) step_request();
        aim_request();
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            dma_aim(d, s);
            asm volatile("s_nop 0");
            dma_go(d, ra, rb);
        }
    }
    NT_WAIT_VMCNT((kRing - 1) * ND);
    aim_settle();
    settle(integral_constant<int, 0>{});
    step_settle();
    aim_settle();
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) lds_read(r, 0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // Slice s sits at ring position s % 4.  At the top of trip s this wavefront's part of slice s + 1 must have landed.
    // One pass = four trips.  A number of slices that is no multiple of four is rounded up: the slices past the last are
    // requested from records of length zero, arrive as zeros, and their trips add nothing.
    for (int32_t sl = 0; sl < n_slices; sl += kRing) {
        NT_WAIT_VMCNT(2 * ND); trip(integral_constant<int, 0>{}, integral_constant<int, 0>{});
        NT_WAIT_VMCNT(2 * ND); trip(integral_constant<int, 1>{}, integral_constant<int, 1>{});
        NT_WAIT_VMCNT(2 * ND); trip(integral_constant<int, 2>{}, integral_constant<int, 0>{});
        NT_WAIT_VMCNT(2 * ND); trip(integral_constant<int, 3>{}, integral_constant<int, 1>{});
        // (wait states between the last matrix instruction and anything the compiler may do to an accumulator at the
        // loop's end: it does not know that the inline assembly is a matrix instruction)
        asm volatile("s_nop 7" ::: "memory");
    }
    NT_WAIT_VMCNT(0);
    __syncthreads();
    asm volatile("s_nop 15" ::: "memory");

    const int64_t row_w = row0 + wave_m * (BM / 2), col_w = col0 + wave_n * (BN / 2);
    if (g.out_dtype == NT_F32) conv_store_rows16<BM, BN, NT_F32>(g, smem, wave, acc, bi, row_w, col_w, lane);
    else if (g.out_dtype == NT_F16) conv_store_rows16<BM, BN, NT_F16>(g, smem, wave, acc, bi, row_w, col_w, lane);
    else conv_store_rows16<BM, BN, NT_BF16>(g, smem, wave, acc, bi, row_w, col_w, lane);
}

// The grid: g.mt_a tiles of 32 TMA positions, then g.mt - g.mt_a tiles of 32 TMB positions, each kind times g.nt filter tiles
// times g.ksplit parts of the k range.  Two heights because whole rounds of programs (one per compute unit) cost their
// length: 100352 positions are 12.25 blocks of 32 per unit, which 448 tiles of 224 positions serve in two rounds of 7 blocks,
// and 256 tiles of 224 followed by 224 tiles of 192 in a round of 7 and a round of 6.  The host picks the heights and
// the counts (either count may be zero).
template <bool BF16, int TMA, int TMB, bool TRACE = false>
__global__ __launch_bounds__(kThreads, 1) void gemm_conv_tap_kernel(const ConvArgs g)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const uint32_t nt32 = (uint32_t)g.nt, mta = (uint32_t)g.mt_a, mtb = (uint32_t)g.mt - mta;
    const uint32_t ks = (uint32_t)(g.ksplit > 1 ? g.ksplit : 1);
    const uint32_t n_a = ks * mta * nt32;
    const int64_t base_b = (int64_t)mta * (32 * TMA);
    uint32_t w = TRACE ? (uint32_t)g.trace_program : blockIdx.x;
    // (the trace numbers programs tile row by tile row over both kinds, one k part)
    const bool first = TRACE ? w < mta * nt32 : w < n_a;                       // (uniform)
    uint32_t bb = 0, pid;
    if (first) {
        if constexpr (TRACE) pid = w;
        else program_of_workgroup_batched_t<uint32_t>(w, ks, mta, nt32, &bb, &pid);
    } else {
        if constexpr (TRACE) pid = w - mta * nt32;
        else program_of_workgroup_batched_t<uint32_t>(w - n_a, ks, mtb, nt32, &bb, &pid);
    }
    const uint32_t ti32 = pid / nt32;
    const int64_t bi = __builtin_amdgcn_readfirstlane((int)bb);
    const int64_t ti = __builtin_amdgcn_readfirstlane((int)ti32);
    const int64_t tj = __builtin_amdgcn_readfirstlane((int)(pid - ti32 * nt32));
    if (first) conv_tap_program<BF16, TMA, TRACE>(g, smem, bi, ti, tj, 0);
    else conv_tap_program<BF16, TMB, TRACE>(g, smem, bi, ti, tj, base_b);
}

template <bool BF16, int TMA, int TMB, bool TRACE = false>
static nt_status launch_conv_tap_inst(const ConvArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)4 * (256 + 256) * kSliceK * sizeof(uint16_t);
    auto kern = gemm_conv_tap_kernel<BF16, TMA, TMB, TRACE>;
    static DeviceOnce configured;
    if (!configured.done()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured.set();
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_conv_tap_kernel");
}

// a.Wt: the filter in tap-major order (see launch_conv_repack_filter), a.ldb its row pitch; rows: positions per program of
// the first a.mt_a tiles (256 or 224), the other a.mt - a.mt_a tiles being 32 positions lower; nwg = ksplit * mt * nt
nt_status launch_conv_tap(const ConvArgs &a, int rows, bool bf16, int64_t nwg, hipStream_t s);
nt_status launch_conv_tap_trace(const ConvArgs &a, int rows, hipStream_t s);
// filter [F][C][R * S] (row pitch ldb) -> out [F][R * S][C] (row pitch C R S)
nt_status launch_conv_repack_filter(const uint16_t *w, int64_t ldb, uint16_t *out, int32_t F, int32_t C, int32_t RS, hipStream_t s);

}  // namespace nt
