// Dispatch between the kernels, plus the small auxiliary kernels (zero fill, address trace).
#include "gemm_direct.h"

namespace nt {

// ------------------------------------------------------------- auxiliary kernels
__global__ void fill_zero_kernel(void *C, const OperandMap mc, int64_t sc_batch, int out_dtype)
{
    const int64_t total = mc.rows * mc.cols;
    const int64_t b = blockIdx.y;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / mc.cols, col = e % mc.cols;
        int64_t off;
        if (element_at(mc, row, col, row_part(mc, row), col_part(mc, col), &off))
            store_out(C, b * sc_batch + off, 0.f, out_dtype);
    }
}

__global__ void trace_tile_kernel(const OperandMap m, int64_t batch_off, int64_t row0, int64_t col0,
                                  int32_t rows, int32_t cols, int64_t *offsets_out, uint8_t *mask_out)
{
    const int64_t total = (int64_t)rows * cols;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = row0 + e / cols, col = col0 + e % cols;
        int64_t off;
        const bool ok = element_at(m, row, col, row_part(m, row), col_part(m, col), &off);
        offsets_out[e] = ok ? batch_off + off : -1;
        mask_out[e] = ok ? 1 : 0;
    }
}

struct TileEntry { int bm, bn, bk; };
static const TileEntry kTiles[] = {{64, 64, 32}, {128, 128, 64}, {256, 128, 64}, {128, 256, 64}, {256, 256, 64}};

bool tile_is_built(nt_tile_cfg cfg)
{
    for (const TileEntry &t : kTiles)
        if (t.bm == cfg.bm && t.bn == cfg.bn && t.bk == cfg.bk) return true;
    return false;
}

// A map is "plain" when it is a strided matrix without bounds checks beyond rows / cols.
static bool plain(const OperandMap &m) { return m.nrd == 1 && m.ncd == 1 && m.nchk == 0; }

nt_status launch_gemm(const GemmLaunch &g, int *path_out)
{
    if (g.batch * g.mt * g.nt > 0x7fffffffLL) return fail(NT_ERR_UNSUPPORTED, "grid too large");
    const nt_tile_cfg t = g.tile;
    // fast path: plain operands, each with unit stride along one of its axes
    bool fast = plain(g.ma) && plain(g.mb) && plain(g.mc) && t.bk == 64 && t.bm >= 128 && t.bn >= 128;
    int alay = KCONTIG, blay = MNCONTIG;
    FastArgs a{};
    if (fast) {
        if (g.ma.coff[0] == 1) { alay = KCONTIG; a.lda = g.ma.roff[0]; }
        else if (g.ma.roff[0] == 1) { alay = MNCONTIG; a.lda = g.ma.coff[0]; }
        else fast = false;
        if (g.mb.coff[0] == 1) { blay = MNCONTIG; a.ldb = g.mb.roff[0]; }
        else if (g.mb.roff[0] == 1) { blay = KCONTIG; a.ldb = g.mb.coff[0]; }
        else fast = false;
        if (a.lda < 0 || a.ldb < 0 || a.lda >= (1 << 22) || a.ldb >= (1 << 22)) fast = false;   // 32-bit lane offsets
    }
    if (path_out) *path_out = fast ? PATH_FAST : PATH_GENERIC;
    if (fast) {
        a.A = (const uint16_t *)g.A + g.ma.base;
        a.B = (const uint16_t *)g.B + g.mb.base;
        a.C = g.C;
        a.scm = g.mc.roff[0];
        a.scn = g.mc.coff[0];
        const int64_t esz = g.out_dtype == NT_F32 ? 4 : 2;
        a.C = (char *)g.C + g.mc.base * esz;
        a.sa_batch = g.sa_batch; a.sb_batch = g.sb_batch; a.sc_batch = g.sc_batch;
        a.M = g.M; a.N = g.N; a.K = g.K;
        a.mt = g.mt; a.nt = g.nt; a.kt = g.kt;
        a.out_dtype = g.out_dtype;
        const bool edge = (g.M % t.bm) || (g.N % t.bn) || (g.K % t.bk);
        const bool bf16 = g.in_dtype == NT_BF16;
        const int64_t nwg = g.batch * g.mt * g.nt;
        hipStream_t s = (hipStream_t)g.stream;
        // full tiles of 16-byte aligned operands stream straight into LDS
        auto al16 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
        const bool direct = !edge && al16(a.A) && al16(a.B) && a.lda % 8 == 0 && a.ldb % 8 == 0 &&
                            a.sa_batch % 8 == 0 && a.sb_batch % 8 == 0;
        if (path_out) *path_out = direct ? PATH_DIRECT : PATH_FAST;
        if (direct) {
            if (t.bm == 128 && t.bn == 128) return launch_direct_128x128(a, bf16, alay, blay, nwg, s);
            if (t.bm == 256 && t.bn == 128) return launch_direct_256x128(a, bf16, alay, blay, nwg, s);
            if (t.bm == 128 && t.bn == 256) return launch_direct_128x256(a, bf16, alay, blay, nwg, s);
            if (t.bm == 256 && t.bn == 256) return launch_direct_256x256(a, bf16, alay, blay, nwg, s);
        }
        if (t.bm == 128 && t.bn == 128) return launch_fast_128x128(a, bf16, edge, alay, blay, nwg, s);
        if (t.bm == 256 && t.bn == 128) return launch_fast_256x128(a, bf16, edge, alay, blay, nwg, s);
        if (t.bm == 128 && t.bn == 256) return launch_fast_128x256(a, bf16, edge, alay, blay, nwg, s);
        if (t.bm == 256 && t.bn == 256) return launch_fast_256x256(a, bf16, edge, alay, blay, nwg, s);
        return fail(NT_ERR_UNSUPPORTED, "no fast kernel for this tile");
    }
    return launch_generic(g);
}

nt_status launch_fill_zero(void *C, const OperandMap &mc, int64_t batch, int64_t sc_batch, int out_dtype, void *stream)
{
    const int64_t total = mc.rows * mc.cols;
    if (total <= 0 || batch <= 0) return NT_OK;
    const int64_t blocks = std::min<int64_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks, (unsigned)batch), dim3(256), 0, (hipStream_t)stream,
                       C, mc, sc_batch, out_dtype);
    return check_launch("fill_zero_kernel");
}

nt_status launch_trace(const OperandMap &m, int64_t batch_off, int64_t row0, int64_t col0, int32_t rows, int32_t cols,
                       int64_t *offsets_out, uint8_t *mask_out, void *stream)
{
    const int64_t total = (int64_t)rows * cols;
    if (total <= 0) return NT_OK;
    const int64_t blocks = std::min<int64_t>((total + 255) / 256, 1024);
    hipLaunchKernelGGL(trace_tile_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       m, batch_off, row0, col0, rows, cols, offsets_out, mask_out);
    return check_launch("trace_tile_kernel");
}

}  // namespace nt
