// Direct kernel: full tiles of 16-byte aligned, unit-stride operands.
//
// One workgroup (4 wavefronts, 2 x 2) computes one BM x BN output tile (one program of
// the tile-to-program mapping, Section 3.2.1).  The blocks of A and B that the program
// multiplies (source-to-target mapping, Section 3.2.2) travel from global memory straight
// into LDS (global_load_lds, 16 bytes per lane, no staging registers) in slices of 32 k
// (each 64-wide k tile of the arrangement is consumed as two such slices).  LDS holds a
// ring of three or four slices per operand (see ring_of), so a slice is requested two or three
// slice-times (2000 - 3000 cycles) before it is multiplied: long enough to cover an L2 miss.
//
// LDS layouts, chosen by how the operand lies in memory:
//   k-major  (operand contiguous along k)    [row = m or n][32 k], 64 bytes per row; a
//            lane's MFMA operand (8 consecutive k) is one ds_read_b128.
//   mn-major (operand contiguous along m/n)  [k][E = BM or BN]; the MFMA operand is
//            gathered with two transposing reads (ds_read_b64_tr_b16), each of which turns
//            a 4(k) x 16(m/n) patch into 4 consecutive k per lane.
// A direct-to-LDS load always writes lane l's 16 bytes to (instruction base + 16 l), so the
// bank swizzle is applied on the global side: lane l fetches the chunk that belongs in
// its slot.  k-major: chunk ^= (row / 4) & 3; mn-major: chunk ^= (k & 3) * 4.
#pragma once
#include <type_traits>

#include "gemm_fast.h"

namespace nt {

typedef short short4v __attribute__((ext_vector_type(4)));

constexpr int kSliceK = 32;      // k extent of one LDS slice
// Slices per operand resident in LDS, and workgroups the kernel is built to co-reside on a
// compute unit.  The 256 x 256 tile needs every accumulator register of its wavefronts (one
// workgroup per unit, ring of four = 128 KB).  Smaller tiles leave room for two workgroups
// per unit (at most 72 KB and 256 registers each), whose epilogues, launches and prologues
// then overlap the other's multiplications; their ring is three slices (256 x 128: 72 KB) or
// four (128 x 128: 64 KB).
constexpr int ring_of(int bm, int bn) { return bm + bn == 384 || bm + bn == 320 ? 3 : 4; }   // (320: the convolution kernel's 256 x 64, 60 KB)
constexpr int residency_of(int bm, int bn) { return bm + bn == 512 ? 1 : 2; }

// s_waitcnt that waits until at most n vector-memory operations are outstanding and leaves
// the other counters alone (vmcnt is split over bits [3:0] and [15:14] of the immediate)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }
#define NT_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(vmcnt_imm(n))

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at
// lds_addr + 16 l.  gbase and lds_addr are wavefront-uniform, voff is the lane's byte offset.
// Issued through inline assembly so that the compiler does not serialise later LDS reads of
// other slices behind it; completion is awaited explicitly with NT_WAIT_VMCNT.
__device__ __forceinline__ void dma16(const char *gbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(gbase)
                 : "memory");   // m0 is not otherwise used by these kernels
}

// The same through a range-checked buffer access: rsrc describes the memory from the program's tile origin to the
// operand's end, soff (wavefront-uniform) and voff are byte offsets into it; 4-byte words that do not lie wholly
// inside it arrive in LDS as zeros instead of being fetched.  Lets tiles on the ragged m / n edge use the same loads.
__device__ __forceinline__ void dma16_buf(u32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory");
}

// buffer resource (raw, no swizzle) over `bytes` bytes at p; all words wavefront-uniform
__device__ __forceinline__ u32x4 make_rsrc(const void *p, int64_t bytes)
{
    const uint64_t b = reinterpret_cast<uint64_t>(p);
    const uint32_t n = bytes < 0x7fffffffLL ? (uint32_t)bytes : 0x7fffffffu;
    return u32x4{(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b), (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((b >> 32) & 0xffffu)),
                 (uint32_t)__builtin_amdgcn_readfirstlane((int)n), 0x00020000u};
}

template <int E, int LAY>
struct DirectTile;

// ---- k-major slice: E rows (m or n) x 32 k
template <int E>
struct DirectTile<E, KCONTIG> {
    static constexpr uint32_t BYTES = E * kSliceK * 2;
    static constexpr int PER = BYTES / 1024 / 4;           // load instructions per wavefront and slice
    static constexpr int RPF = 1;                          // LDS reads per operand fragment
    uint32_t voff[PER];                                    // global byte offset of this lane's chunk
    uint32_t rd;                                           // LDS read base of this lane

    // region: LDS byte offset of this operand's ring (folded into the read base)
    __device__ __forceinline__ void init(int wave, int lane, int64_t ld, int wave_origin, uint32_t region)
    {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int row = (wave * PER + j) * 16 + (lane >> 2);
            const int c = (lane & 3) ^ ((row >> 2) & 3);
            voff[j] = ((uint32_t)row * (uint32_t)ld + (uint32_t)(c * 8)) * 2u;
        }
        const int r = wave_origin + (lane & 31);
        rd = (uint32_t)(r * 64 + (((lane >> 5) ^ ((r >> 2) & 3)) << 4)) + region;
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
        return (uint32_t)((r >> 4) * 1024 + (((r & 15) << 2) + ((kk >> 3) ^ ((r >> 2) & 3))) * 16 + (kk & 7) * 2);
    }
    static __device__ __forceinline__ int owner(int r, int) { return (r >> 4) / PER; }
    // Ragged K: the slice that has just landed at byte offset slot_off holds only `keep` valid k (< 32); what this
    // lane fetched past them -- the beginning of the operand's next row -- is overwritten with zeros.
    __device__ __forceinline__ void zero_tail(char *smem, uint32_t slot_off, int wave, int lane, int keep) const
    {
        const int left = keep - 8 * ((lane & 3) ^ ((lane >> 4) & 3));      // valid k in this lane's chunks (the same chunk column for all of them)
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
    // fragment t (32 rows) of k step ks (0 or 1) of the slice at byte offset slice_off: one 16-byte read
    __device__ __forceinline__ void read(u32x2 (&f)[2], const char *smem, int t, int ks, int part, uint32_t slice_off) const
    {
        const u32x4 v = lds_read16(smem, (rd ^ (uint32_t)(ks << 5)) + slice_off + t * 2048);
        f[0] = u32x2{v[0], v[1]};
        f[1] = u32x2{v[2], v[3]};
    }
};

// ---- mn-major slice: 32 k rows x E (m or n)
template <int E>
struct DirectTile<E, MNCONTIG> {
    static constexpr uint32_t BYTES = E * kSliceK * 2;
    static constexpr int PER = BYTES / 1024 / 4;
    static constexpr int RPF = 2;
    static constexpr int RB = 2 * E;                       // bytes per k row
    static constexpr int CPR = E / 8;                      // 16-byte chunks per k row
    static constexpr int RPI = 1024 / RB;                  // k rows per load instruction
    static constexpr int T = E / 64;                       // 32-wide operand blocks per wavefront
    uint32_t voff[PER];
    uint32_t rd[T];

    __device__ __forceinline__ void init(int wave, int lane, int64_t ld, int wave_origin, uint32_t region)
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
            rd[t] = (uint32_t)(kl * RB + ((((mn >> 3) + 4 * t) ^ sw) << 4) + ((mn >> 2) & 1) * 8) + region;
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
        return (uint32_t)((kk / RPI) * 1024 + ((kk % RPI) * CPR + ((r >> 3) ^ ((kk & 3) << 2))) * 16 + (r & 7) * 2);
    }
    static __device__ __forceinline__ int owner(int, int kk) { return (kk / RPI) / PER; }
    // (ragged K: the k rows past K lie past the operand's end and arrive as zeros by themselves)
    __device__ __forceinline__ void zero_tail(char *, uint32_t, int, int, int) const {}
    // half `part` (k 0..3 or 4..7 of the lane's run) of fragment t: one transposing 8-byte read
    __device__ __forceinline__ void read(u32x2 (&f)[2], const char *smem, int t, int ks, int part, uint32_t slice_off) const
    {
        typedef short4v __attribute__((address_space(3))) * lds_s4;
        const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(smem + (rd[t] + slice_off + (uint32_t)((ks * 16 + part * 4) * RB))));
        f[part] = __builtin_bit_cast(u32x2, v);
    }
};

// EDGE = false: every tile is full, every load 16-byte aligned.  EDGE = true: tiles may overhang M or N, K need not be
// a whole number of slices, rows need only the element's own 2-byte alignment: the operand loads are range checked
// (what lies past an operand's end reads as zero, what an overhanging tile reads inside it only reaches outputs that
// are never stored, except the k past K of a k-contiguous operand, which are zeroed in LDS) and the stores are masked.
template <int BM, int BN, bool BF16, int ALAY, int BLAY, bool EDGE>
__global__ __launch_bounds__(kThreads, residency_of(BM, BN)) void gemm_direct_kernel(const FastArgs g)
{
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int kRing = ring_of(BM, BN);
    using TileA = DirectTile<BM, ALAY>;
    using TileB = DirectTile<BN, BLAY>;
    constexpr uint32_t A_BYTES = TileA::BYTES, B_BYTES = TileB::BYTES, B_BASE = kRing * A_BYTES;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int64_t bi, ti, tj;
    locate_program(g.mt, g.nt, &bi, &ti, &tj);
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

    float16v acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // LDS byte address of the dynamic segment (it starts the workgroup's allocation)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    // operand fragments, double buffered: [slot][32-row block][low / high 4 k of the lane's run]
    u32x2 fa[2][TM][2], fb[2][TN][2];
    constexpr int NRB = TN * TileB::RPF, NR = TM * TileA::RPF + NRB;   // LDS reads per k step
    // LDS read r of a k step, in the order the next step's MFMAs need the data:
    // A block 0, every B block, then the remaining A blocks
    auto lds_read = [&](int r, int slot, int ks, uint32_t ring) {
        if (r < TileA::RPF) {
            ta.read(fa[slot][0], smem, 0, ks, r, ring * A_BYTES);
        } else if (r < TileA::RPF + NRB) {
            const int q = r - TileA::RPF;
            tb.read(fb[slot][q / TileB::RPF], smem, q / TileB::RPF, ks, q % TileB::RPF, ring * B_BYTES);
        } else {
            const int q = r - NRB;
            ta.read(fa[slot][q / TileA::RPF], smem, q / TileA::RPF, ks, q % TileA::RPF, ring * A_BYTES);
        }
    };
    // The global->LDS loads of one slice, numbered 0 .. ND-1 (A's first): load d of the slice
    // at (pa, pb) into ring position `ring`.
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
    // One k step: the TM x TN MFMAs on fragment slot `slot`.  Between them, one at a time so
    // that neither the LDS queue nor the memory queue ever holds the in-order wavefront back
    // while the matrix pipe runs dry: the LDS reads of the next step's fragments (k step
    // `ks_next` of ring position `rring`, into the other slot) and, if nd > 0, the nd
    // global->LDS loads of the slice at (pa, pb) into ring position `dring`.
    auto step = [&](int slot, int ks_next, uint32_t rring, int nd, const char *pa, const char *pb, uint32_t dring) {
        constexpr int RQ = (NR + NM - 1) / NM;              // LDS reads after each MFMA
#pragma unroll
        for (int idx = 0; idx < NM; ++idx) {
            const int tm = idx / TN, tn = idx % TN;
            const u32x4 xa{fa[slot][tm][0][0], fa[slot][tm][0][1], fa[slot][tm][1][0], fa[slot][tm][1][1]};
            const u32x4 xb{fb[slot][tn][0][0], fb[slot][tn][0][1], fb[slot][tn][1][0], fb[slot][tn][1][1]};
            acc[tm][tn] = mfma32<BF16>(xb, xa, acc[tm][tn]);   // transposed block (see store_tile)
#pragma unroll
            for (int q = 0; q < RQ; ++q)
                if (idx * RQ + q < NR) lds_read(idx * RQ + q, slot ^ 1, ks_next, rring);
            if (nd > 0) {
                const int per = (nd + NM - 1) / NM;         // loads after each MFMA (when there are more loads than MFMAs)
                const int gap = nd >= NM ? 1 : NM / nd;     // otherwise one load after every `gap` MFMAs
                if (idx % gap == gap - 1)
#pragma unroll
                    for (int q = 0; q < per; ++q)
                        if ((idx / gap) * per + q < nd) dma((idx / gap) * per + q, pa, pb, dring);
            }
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
    auto patch_last = [&](uint32_t slot_a, uint32_t slot_b) {
        if (lane == 0) {
            if (patch_a >= 0)
                *reinterpret_cast<uint16_t *>(smem + slot_a + patch_a) = *reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(g.A + bi * g.sa_batch) + g.a_extent - 2);
            if (patch_b >= 0)
                *reinterpret_cast<uint16_t *>(smem + slot_b + patch_b) = *reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(g.B + bi * g.sb_batch) + g.b_extent - 2);
        }
    };
    auto slice_a = [&](int64_t s) { return gA + (s < last ? s : last) * a_step; };   // clamped: surplus slices are never read
    auto slice_b = [&](int64_t s) { return gB + (s < last ? s : last) * b_step; };

    // prologue: slices 0 .. 3 requested into the ring; wait for slice 0; its first fragments
#pragma unroll
    for (int s = 0; s < kRing; ++s)
#pragma unroll
        for (int d = 0; d < ND; ++d) dma(d, slice_a(s), slice_b(s), s);
    NT_WAIT_VMCNT((kRing - 1) * ND);
    if constexpr (EDGE) {
        if (g.K < kSliceK) {
            ta.zero_tail(smem, 0, wave, lane, (int)g.K);
            tb.zero_tail(smem, B_BASE, wave, lane, (int)g.K);
        }
        if (last == 0 && g.patch) patch_last(0, B_BASE);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) lds_read(r, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // One slice per trip, one basic block.  Slice s sits at ring position s % kRing.
    //   step A  multiplies k step 0 of slice s while reading its k step 1 fragments;
    //   then waits until this wavefront's part of slice s+1 has landed (the loads of the
    //   younger slices may still be in flight) and meets the other wavefronts: slice s+1 is
    //   complete, and nobody reads the ring position of slice s any more;
    //   step B  multiplies k step 1 while reading the first fragments of slice s+1 and
    //   requesting slice s+kRing into the position just released.
    uint32_t ring = 0;
    for (int64_t sl = 0; sl < n_slices; ++sl) {
        const uint32_t nxt = ring + 1 == kRing ? 0 : ring + 1;
        step(0, 1, ring, 0, nullptr, nullptr, 0);
        NT_WAIT_VMCNT((kRing - 2) * ND);
        if constexpr (EDGE) {
            if (sl + 1 == last && (sl + 2) * kSliceK > g.K) {          // the last slice has landed, and K ends inside it
                const int keep = (int)(g.K - (sl + 1) * kSliceK);
                ta.zero_tail(smem, nxt * A_BYTES, wave, lane, keep);
                tb.zero_tail(smem, B_BASE + nxt * B_BYTES, wave, lane, keep);
            }
            if (sl + 1 == last && g.patch) patch_last(nxt * A_BYTES, B_BASE + nxt * B_BYTES);
        }
        __syncthreads();
        step(1, 0, nxt, ND, slice_a(sl + kRing), slice_b(sl + kRing), ring);
        ring = nxt;
    }
    NT_WAIT_VMCNT(0);                                      // drain the surplus prefetches ...
    __syncthreads();                                       // ... of every wavefront: the epilogue reuses the LDS

    store_tile<BM, BN, EDGE>(g, smem, wave, bi, acc, row0 + wave_m * (BM / 2), col0 + wave_n * (BN / 2), lane,
                             EDGE && (g.M - row0 < BM || g.N - col0 < BN));
}

template <int BM, int BN, bool BF16, int ALAY, int BLAY, bool EDGE = false>
static nt_status launch_direct_inst(const FastArgs &a, int64_t nwg, hipStream_t s)
{
    constexpr size_t smem = (size_t)ring_of(BM, BN) * (BM + BN) * kSliceK * sizeof(uint16_t);
    auto kern = gemm_direct_kernel<BM, BN, BF16, ALAY, BLAY, EDGE>;
    static DeviceOnce configured;
    if (!configured.done()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
        configured.set();
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kThreads), smem, s, a);
    return check_launch("gemm_direct_kernel");
}

template <int BM, int BN, bool BF16, bool EDGE = false>
static nt_status launch_direct_t(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s)
{
    if (alay == KCONTIG && blay == MNCONTIG) return launch_direct_inst<BM, BN, BF16, KCONTIG, MNCONTIG, EDGE>(a, nwg, s);
    if (alay == KCONTIG && blay == KCONTIG) return launch_direct_inst<BM, BN, BF16, KCONTIG, KCONTIG, EDGE>(a, nwg, s);
    if (alay == MNCONTIG && blay == MNCONTIG) return launch_direct_inst<BM, BN, BF16, MNCONTIG, MNCONTIG, EDGE>(a, nwg, s);
    return launch_direct_inst<BM, BN, BF16, MNCONTIG, KCONTIG, EDGE>(a, nwg, s);
}

// one translation unit per tile shape and input format defines these (parallel compilation)
#define NT_DIRECT_DECL(T) \
    nt_status launch_direct_##T##_f16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s); \
    nt_status launch_direct_##T##_bf16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s); \
    nt_status launch_direct_edge_##T##_f16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s); \
    nt_status launch_direct_edge_##T##_bf16(const FastArgs &a, int alay, int blay, int64_t nwg, hipStream_t s);
NT_DIRECT_DECL(128x128)
NT_DIRECT_DECL(256x128)
NT_DIRECT_DECL(128x256)
NT_DIRECT_DECL(256x256)
#undef NT_DIRECT_DECL

}  // namespace nt
