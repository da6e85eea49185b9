// Scaled dot-product attention, forward (Section 5.1: the paper's sdpa kernels implement the
// FlashAttention-2 algorithm): O = softmax(scale * Q K^T) V per (batch, head), head size 64.
//
// Arrangement: Q and O are tiled into blocks of 128 query rows, one program per (batch, head,
// block); K and V are tiled into blocks of 64 keys, all of which every program visits in turn.
// Application (per program): a row reference M (close to the running row maximum), row sum l,
// accumulator O; per key block
//   S = Q K_j^T;  P = 2^(c S - M)  (c = scale * log2 e);  l += rowsum P;  O += P V_j;   finally O / l.
// M only has to stay within a band of the running maximum for this to be exact up to rounding:
// every term carries the same factor 2^-M, which cancels in O / l.  M is raised (and O, l scaled
// by 2^(M - M')) when a block holds a score more than 15 above it, which the row sum of that block
// reveals (2^15 is half the largest fp16 number), and it is set to the block's maximum at the first
// block.  FlashAttention-2 raises M to the exact maximum at every block; keeping a lagging one
// removes the maximum search from all but a few blocks.
//
// Mapping onto the matrix cores: everything is computed transposed.  A wavefront owns 32 query
// rows.  S^T = K_j Q^T puts the query on the lane axis of the 32 x 32 MFMA result (lane % 32) and
// the keys on the register axis, so the row maximum and sum run over a lane's own registers plus
// one exchange with the other half-wavefront.  The fp32 P^T values a lane holds (keys in groups of
// four, interleaved between the half-wavefronts) are, packed to 16 bits, already a valid B
// operand of the second product O^T = V_j^T P^T if the matching A operand lists the keys in the
// same order: V_j sits in LDS as [key][d] and the transposing LDS read (ds_read_b64_tr_b16)
// delivers, for a lane's d, four consecutive keys at any position.  O^T again has the query on
// the lane axis, so rescaling by 2^(M - M') is a per-lane scalar.  Q fragments stay in registers.
// K_j and V_j go global -> registers -> LDS (double buffered), the next block's loads in flight
// during the current block's arithmetic; 32 KB of LDS and ~160 registers per workgroup let
// several workgroups share a compute unit, which hides the exponentials of one behind the MFMAs
// of another.
#include "gemm_fast.h"
#include <type_traits>

namespace nt {

struct SdpaArgs {
    const uint16_t *Q, *K, *V;
    uint16_t *O;
    int64_t q_sb, q_sh, q_ss;        // strides (elements) of batch, head, sequence; the head dimension has stride 1
    int64_t k_sb, k_sh, k_ss;
    int64_t v_sb, v_sh, v_ss;
    int64_t o_sb, o_sh, o_ss;
    int32_t H, Sq, Sk;
    int32_t BH, nqb;                 // batch * heads, query blocks per head (the grid is their product)
    float scale_log2e;               // scale * log2(e): exponentials are taken in base 2
};

constexpr int kHeadDim = 64, kQBlock = 128, kKeyBlock = 64;

typedef short short4v_a __attribute__((ext_vector_type(4)));

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));

// two fp32 values -> one register of two 16-bit values, round to nearest even (v_cvt_pk_{f16,bf16}_f32)
template <bool BF16>
__device__ __forceinline__ uint32_t pack2(float a, float b)
{
    if constexpr (BF16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(float2v{a, b}, bf16x2v));
    else return __builtin_bit_cast(uint32_t, half2v{(_Float16)a, (_Float16)b});
}

// acc + the two 16-bit values of w (v_dot2c_f32_{f16,bf16} against a pair of ones)
template <bool BF16>
__device__ __forceinline__ float add_pair(uint32_t w, float acc)
{
    if constexpr (BF16) return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2v, w), __builtin_bit_cast(bf16x2v, 0x3f803f80u), acc, false);
    else return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, w), __builtin_bit_cast(half2v, 0x3c003c00u), acc, false);
}

template <bool BF16>
__global__ __launch_bounds__(256, 2) void sdpa_kernel(const SdpaArgs g)
{
    constexpr uint32_t BLK = kKeyBlock * kHeadDim * 2;                 // bytes of one K or V block in LDS (8 KB)
    __shared__ __attribute__((aligned(16))) char smem[4 * BLK];        // [K0][K1][V0][V1]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    // Workgroup -> (batch * head, query block).  Consecutive workgroup indices go to different XCDs (index mod 8),
    // each with an L2 of its own; the query blocks of one head all read that head's K and V, so every group of
    // eight heads is dealt out one head per XCD instead of one head across all eight.
    const int w = blockIdx.x, nqb = g.nqb;
    int bh = w / nqb, qblk = w % nqb;
    if (w < (g.BH & ~7) * nqb) {
        const int j = w >> 3;
        bh = (j / nqb) * 8 + (w & 7);
        qblk = j % nqb;
    }
    const int b = bh / g.H, h = bh % g.H;
    const uint16_t *Qp = g.Q + b * g.q_sb + h * g.q_sh;
    const uint16_t *Kp = g.K + b * g.k_sb + h * g.k_sh;
    const uint16_t *Vp = g.V + b * g.v_sb + h * g.v_sh;
    uint16_t *Op = g.O + b * g.o_sb + h * g.o_sh;

    // ---- Q fragments (B operand of S^T = K Q^T: column = query l32, 8 consecutive d per k step)
    const int qrow = qblk * kQBlock + wave * 32 + l32;
    const int qrow_c = qrow < g.Sq ? qrow : g.Sq - 1;
    u32x4 qf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) __builtin_memcpy(&qf[ks], Qp + (int64_t)qrow_c * g.q_ss + 16 * ks + 8 * hi, 16);

    // ---- staging of a K / V block: 512 16-byte chunks each, two per thread; rows past Sk read as zero
    u32x4 kst[2], vst[2];
    auto fetch = [&](int key0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int c = tid + 256 * u, row = c >> 3, ch = c & 7;
            const int key = key0 + row;
            u32x4 kk{0, 0, 0, 0}, vv{0, 0, 0, 0};
            if (key < g.Sk) {
                __builtin_memcpy(&kk, Kp + (int64_t)key * g.k_ss + ch * 8, 16);
                __builtin_memcpy(&vv, Vp + (int64_t)key * g.v_ss + ch * 8, 16);
            }
            kst[u] = kk;
            vst[u] = vv;
        }
    };
    auto stash = [&](uint32_t buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int c = tid + 256 * u, row = c >> 3, ch = c & 7;
            lds_write16(smem, buf * BLK + (uint32_t)(row * 128 + ((ch ^ ((row ^ (row >> 3)) & 7)) << 4)), kst[u]);
            lds_write16(smem, (2 + buf) * BLK + (uint32_t)(row * 128 + ((ch ^ (((row >> 1) & 1) << 2)) << 4)), vst[u]);
        }
    };

    // ---- per-lane LDS read addresses
    // K fragment (A operand, row = key l32 of a 32-key half, chunk 2 ks + hi, swizzled like the write)
    // Key row 32 + l32 has the swizzle of row l32 with bit 2 flipped, so its chunk for k step ks sits where row
    // l32's chunk for k step ks ^ 2 does: four addresses serve both halves, everything else is an immediate offset.
    uint32_t k_rd[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) k_rd[ks] = (uint32_t)(l32 * 128 + (((hi + 2 * ks) ^ ((l32 ^ (l32 >> 3)) & 7)) << 4));
    // V^T fragment through the transposing read: 16-lane group gq covers d = 16 (gq & 1) .. + 15 and
    // keys 4 (gq >> 1) .. + 3 of an 8-key part; lane i of the group points at key i / 4, columns 4 (i % 4) .. + 3
    const int gq = lane >> 4, li = lane & 15;
    const int v_key = 4 * (gq >> 1) + (li >> 2);                       // + jb * 32 + 16 * s2 + 8 * part
    const int v_c8 = 4 * (gq & 1) + (li & 3);                          // 8-byte chunk within the 32-d block; + 8 * db
    // the swizzle flips bit 3 of the 8-byte chunk index on keys with bit 1 set (key offsets added later are multiples of 8)
    uint32_t v_rd[2];
#pragma unroll
    for (int db = 0; db < 2; ++db)
        v_rd[db] = (uint32_t)(v_key * 128) + ((((uint32_t)(v_c8 + 8 * db)) ^ (uint32_t)(((v_key >> 1) & 1) << 3)) << 3);

    float16v ot[2];
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) ot[db][v] = 0.f;
    float m_ref = 0.f, l_run = 0.f;                                    // row reference M (base-2 units of the scaled scores), row sum
    bool first = true;

    const int nblk = (g.Sk + kKeyBlock - 1) / kKeyBlock;
    fetch(0);
    stash(0);
    __syncthreads();
    // one key block; the LDS buffer index is a compile-time constant so that every LDS address is base + immediate
    auto block = [&](auto cur_c, const int kb) {
        constexpr uint32_t cur = (uint32_t)decltype(cur_c)::value;
        if (kb + 1 < nblk) fetch((kb + 1) * kKeyBlock);                // in flight during this block's arithmetic

        // ---- S^T = K Q^T: st[jb][v] <-> key jb * 32 + 8 (v / 4) + 4 hi + v % 4, query l32
        float16v st[2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) st[jb][v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const u32x4 kf = lds_read16(smem, k_rd[jb ? (ks ^ 2) : ks] + (cur * BLK + (uint32_t)(jb * 4096)));
                st[jb] = mfma32<BF16>(kf, qf[ks], st[jb]);
            }
        }
        // ---- keys past Sk (last block only) get weight 0: their scaled score becomes -inf
        const int key_base = kb * kKeyBlock;
        if (key_base + kKeyBlock > g.Sk) {                                // wavefront-uniform
            const float out = g.scale_log2e >= 0.f ? -INFINITY : INFINITY;
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (key_base + jb * 32 + 8 * (v / 4) + 4 * hi + (v % 4) >= g.Sk) st[jb][v] = out;
        }
        // ---- P^T = 2^(c S^T - M), packed to 16 bits, and its row sum (this lane's keys only; the halves are added at the end)
        float rs;
        u32x4 pk[2][2];
        auto exponentials = [&](const float m) {
            rs = 0.f;
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[jb][8 * s2 + 2 * j], g.scale_log2e, -m));
                        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[jb][8 * s2 + 2 * j + 1], g.scale_log2e, -m));
                        const uint32_t w = pack2<BF16>(p0, p1);
                        pk[jb][s2][j] = w;
                        rs = add_pair<BF16>(w, rs);
                    }
        };
        bool accept = false;
        if (!first) {
            exponentials(m_ref);
            accept = __all(rs < 32768.f);                                // no weight beyond 2^15: the reference is close enough
        }
        if (!accept) {                                                   // wavefront-uniform: first block, or a score far above M
            float mx = st[0][0] * g.scale_log2e;
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, st[jb][v] * g.scale_log2e);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));                      // block maximum of the scaled scores
            const float m_new = first ? mx : fmaxf(m_ref, mx);           // M only rises after the first block
            const float alpha = first ? 0.f : __builtin_amdgcn_exp2f(m_ref - m_new);
            exponentials(m_new);
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) ot[db][v] *= alpha;
            m_ref = m_new;
            first = false;
        }
        l_run += rs;
        // ---- O^T += V^T P^T: k step (jb, s2) lists its 16 keys as jb*32 + 16 s2 + 8 part + 4 hi + 0..3
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int db = 0; db < 2; ++db) {
                    u32x2 part[2];
#pragma unroll
                    for (int pt = 0; pt < 2; ++pt) {
                        const uint32_t addr = v_rd[db] + ((2 + cur) * BLK + (uint32_t)((jb * 32 + 16 * s2 + 8 * pt) * 128));
                        typedef short4v_a __attribute__((address_space(3))) * lds_s4;
                        const short4v_a t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(smem + addr));
                        part[pt] = __builtin_bit_cast(u32x2, t);
                    }
                    const u32x2 p0 = part[0], p1 = part[1];
                    ot[db] = mfma32<BF16>(u32x4{p0[0], p0[1], p1[0], p1[1]}, pk[jb][s2], ot[db]);
                }
        // ---- next block into the other LDS buffer
        if (kb + 1 < nblk) stash(cur ^ 1u);
        __syncthreads();
    };
    for (int kb = 0; kb < nblk; kb += 2) {
        block(std::integral_constant<int, 0>{}, kb);
        if (kb + 1 < nblk) block(std::integral_constant<int, 1>{}, kb + 1);
    }

    // ---- O = O^T / l, stored along d: after the half-wavefronts trade register groups a lane owns
    // d = 32 db + 16 hi .. + 15 of its query row
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
#pragma unroll
    for (int db = 0; db < 2; ++db) {
#pragma unroll
        for (int v = 0; v < 16; ++v) ot[db][v] *= inv;
        uint32_t o[16];
        gather_row16(ot[db], o);                                       // (all lanes take part)
        if (qrow < g.Sq) {
            uint16_t *dst = Op + (int64_t)qrow * g.o_ss + 32 * db + 16 * hi;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const u32x4 w{pack2<BF16>(__builtin_bit_cast(float, o[8 * i]), __builtin_bit_cast(float, o[8 * i + 1])),
                              pack2<BF16>(__builtin_bit_cast(float, o[8 * i + 2]), __builtin_bit_cast(float, o[8 * i + 3])),
                              pack2<BF16>(__builtin_bit_cast(float, o[8 * i + 4]), __builtin_bit_cast(float, o[8 * i + 5])),
                              pack2<BF16>(__builtin_bit_cast(float, o[8 * i + 6]), __builtin_bit_cast(float, o[8 * i + 7]))};
                __builtin_memcpy(dst + 8 * i, &w, 16);
            }
        }
    }
}

nt_status launch_sdpa(const SdpaArgs &a, int64_t batch, bool bf16, void *stream)
{
    if (batch <= 0 || a.H <= 0 || a.Sq <= 0) return NT_OK;
    const int64_t bh = batch * a.H, nqb = (a.Sq + kQBlock - 1) / kQBlock;
    if (bh * nqb > 0x7fffffffLL) return fail(NT_ERR_UNSUPPORTED, "batch * heads * query blocks exceeds 2^31 - 1");
    SdpaArgs k = a;
    k.BH = (int32_t)bh;
    k.nqb = (int32_t)nqb;
    dim3 grid((unsigned)(bh * nqb)), block(256);
    if (bf16) hipLaunchKernelGGL((sdpa_kernel<true>), grid, block, 0, (hipStream_t)stream, k);
    else hipLaunchKernelGGL((sdpa_kernel<false>), grid, block, 0, (hipStream_t)stream, k);
    return check_launch("sdpa_kernel");
}

nt_status launch_sdpa_desc(const void *q, const nt_tensor_desc *dq, const void *k, const nt_tensor_desc *dk,
                           const void *v, const nt_tensor_desc *dv, void *o, const nt_tensor_desc *dout,
                           float scale, int dtype, void *stream)
{
    const nt_tensor_desc *d[4] = {dq, dk, dv, dout};
    for (const nt_tensor_desc *t : d) {
        if (!t) return fail(NT_ERR_INVALID_ARG, "null tensor descriptor");
        if (t->ndim != 4) return fail(NT_ERR_SHAPE_MISMATCH, "sdpa tensors must be 4-D [batch, heads, seq, head_dim]");
        for (int i = 0; i < 4; ++i)
            if (t->size[i] < 0) return fail(NT_ERR_INVALID_ARG, "negative size");
        if (t->size[0] != dq->size[0] || t->size[1] != dq->size[1]) return fail(NT_ERR_SHAPE_MISMATCH, "batch / head counts differ");
        if (t->size[3] != kHeadDim) return fail(NT_ERR_UNSUPPORTED, "sdpa is built for head_dim 64");
        if (t->size[3] > 1 && t->stride[3] != 1) return fail(NT_ERR_UNSUPPORTED, "sdpa needs unit stride along the head dimension");
    }
    if (dk->size[2] != dv->size[2]) return fail(NT_ERR_SHAPE_MISMATCH, "K and V sequence lengths differ");
    if (dout->size[2] != dq->size[2]) return fail(NT_ERR_SHAPE_MISMATCH, "Q and O sequence lengths differ");
    if (dq->size[0] == 0 || dq->size[1] == 0 || dq->size[2] == 0) return NT_OK;
    if (dk->size[2] == 0) return fail(NT_ERR_INVALID_ARG, "sdpa over an empty key sequence is undefined");
    if (!q || !k || !v || !o) return fail(NT_ERR_INVALID_ARG, "null device pointer");
    if (dq->size[2] > 0x7fffffffLL - kQBlock || dk->size[2] > 0x7fffffffLL - kKeyBlock || dq->size[1] > 65535) return fail(NT_ERR_UNSUPPORTED, "sequence too long");
    if (!(scale == scale)) return fail(NT_ERR_INVALID_ARG, "scale is NaN");
    SdpaArgs a{};
    a.Q = (const uint16_t *)q; a.K = (const uint16_t *)k; a.V = (const uint16_t *)v; a.O = (uint16_t *)o;
    a.q_sb = dq->stride[0]; a.q_sh = dq->stride[1]; a.q_ss = dq->stride[2];
    a.k_sb = dk->stride[0]; a.k_sh = dk->stride[1]; a.k_ss = dk->stride[2];
    a.v_sb = dv->stride[0]; a.v_sh = dv->stride[1]; a.v_ss = dv->stride[2];
    a.o_sb = dout->stride[0]; a.o_sh = dout->stride[1]; a.o_ss = dout->stride[2];
    a.H = (int32_t)dq->size[1]; a.Sq = (int32_t)dq->size[2]; a.Sk = (int32_t)dk->size[2];
    const float sc = scale == 0.f ? 0.125f : scale;                  // default 1 / sqrt(64)
    a.scale_log2e = sc * 1.4426950408889634f;
    return launch_sdpa(a, dq->size[0], dtype == NT_BF16, stream);
}

}  // namespace nt
