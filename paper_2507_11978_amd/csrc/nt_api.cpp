// C ABI entry points (declared in include/nt.h): argument checking, the library's own
// arrangements, lowering to device operand maps and kernel launches.
#include <cstring>
#include <string>

#include "arrange.h"
#include "kernels.h"

namespace nt {
const std::string &last_error();
}

using nt::Arrangement;
using nt::fail;
using nt::MatmulArrangement;
using nt::OperandMap;

namespace {

#define NT_TRY(x) do { nt_status st__ = (x); if (st__ != NT_OK) return st__; } while (0)

bool dtype_in_ok(int d) { return d == NT_F16 || d == NT_BF16; }
bool dtype_out_ok(int d) { return d == NT_F16 || d == NT_BF16 || d == NT_F32; }

enum Kind { KIND_GEMM = 0, KIND_BMM = 1, KIND_CONV = 2, KIND_VIEWS = 3 };

// meta-operation programs of the three operands of nt_matmul_views
struct ViewPrograms { const nt_meta_op *ops[3]; int32_t n[3]; };

// Default meta-parameters (the tile sizes are the arrangement's meta-parameters, Section 3.1.2).
// GEMM / BMM: the built tile with the lowest estimated time.  A compute unit works through
// p = ceil(programs / 256) programs; a program costs kt steps of `step` microseconds (time of
// one 64-wide k tile with the whole unit's matrix rate) plus a fixed `fixed` microseconds of
// launch, prologue and epilogue, which `resident` co-resident workgroups overlap with each
// other's multiplications.  The constants are fits to measurements on 8192 x 8192 x K and
// batched 2048 x 2048 x K problems.
// unit_stride: a convolution with stride 1 (the class the dedicated convolution kernels take)
nt_tile_cfg pick_tile(int kind, int64_t batch, int64_t M, int64_t N, int64_t K, nt_tile_cfg cfg, bool unit_stride = false)
{
    if (cfg.bm || cfg.bn || cfg.bk) return cfg;
    // The 64 x 64 tile of the operand-map kernel is for small strided convolutions and small caller-arranged views.
    // Plain products, however small or skinny, run better as overhanging 128-wide tiles of the MFMA kernels (measured:
    // 64 x 64 x 64 in 10.7 us against 18.3, 16 x 4096 x 256 in 11 us against 34, 64 x 64 x 4096 in 13.5 us against 552),
    // and unit-stride convolutions on the convolution kernels' 256-position tile although most of it may stay empty
    // ((32,64,56,56) * (64,64,3,3): 35 us against 242; (1,64,8,8) * (64,64,3,3): 19 us against 104).
    const bool tiny = (M <= 64 || N <= 64) && ((kind == KIND_CONV && !unit_stride) || kind == KIND_VIEWS);
    if (tiny) return nt_tile_cfg{64, 64, 32};
    if (kind == KIND_CONV) return nt::pick_conv_tile(M, N, K);     // 256 output positions per program, 256 or 128 filters
    return nt::pick_gemm_tile(batch, M, N, K);
}


// Views of a caller (nt_matmul_views) recognised as the implicit-GEMM views of a convolution (Section 4.3), possibly one per
// group of a grouped convolution along the batch axis: the convolution of one group, and the element steps between groups.
struct ViewConv {
    bool found = false;
    int64_t groups = 1;
    nt::ConvHint hint{};
    int64_t step_a = 0, step_b = 0, step_c = 0;
};

struct Problem {
    Arrangement va, vb, vc;          // single-level matrix views of the three operands
    MatmulArrangement mm;            // the matmul arrangement applied to them
    nt_tile_cfg tile;
    int64_t batch = 1, M = 0, N = 0, K = 0;
    ViewConv vconv;
};

bool same_map(const OperandMap &a, const OperandMap &b)
{
    if (a.rows != b.rows || a.cols != b.cols || a.base != b.base || a.nrd != b.nrd || a.ncd != b.ncd || a.nchk != b.nchk) return false;
    for (int i = 0; i < a.nrd; ++i)
        if ((i > 0 && a.rrad[i] != b.rrad[i]) || a.roff[i] != b.roff[i]) return false;
    for (int i = 0; i < a.ncd; ++i)
        if ((i > 0 && a.crad[i] != b.crad[i]) || a.coff[i] != b.coff[i]) return false;
    for (int q = 0; q < a.nchk; ++q) {
        if (a.chk0[q] != b.chk0[q] || a.chk_size[q] != b.chk_size[q]) return false;
        for (int i = 0; i < a.nrd; ++i)
            if (a.rchk[q][i] != b.rchk[q][i]) return false;
        for (int i = 0; i < a.ncd; ++i)
            if (a.cchk[q][i] != b.cchk[q][i]) return false;
    }
    return true;
}

// Do the caller's three views address their tensors exactly like the library's own Section 4.3 arrangement of some
// convolution (input (N, G Cg, H, W), filter (G Kg, Cg, R, S), output (N, G Kg, P, Q), G = the views' batch size)?  The
// candidate's stride, dilation and padding are read off the input view's offsets; the answer is yes only if the
// library's arrangement of that candidate lowers to the same three operand maps, field by field.  Then the views can run
// on the convolution routes (the dedicated kernels, the padded copy, the unfolded input) instead of the operand-map kernel.
void recognise_conv(const nt_tensor_desc *dx, const nt_tensor_desc *dw, const nt_tensor_desc *dy, const Arrangement &va,
                    const Arrangement &vb, const Arrangement &vc, ViewConv *out)
{
    out->found = false;
    if (dx->ndim != 4 || dw->ndim != 4 || dy->ndim != 4) return;
    OperandMap ma, mb, mc;
    int64_t ga = 1, gb = 1, gc = 1, sa = 0, sb = 0, sc = 0;
    if (va.lower_matrix_view(&ma, &ga, &sa) != NT_OK || vb.lower_matrix_view(&mb, &gb, &sb) != NT_OK ||
        vc.lower_matrix_view(&mc, &gc, &sc) != NT_OK)
        return;
    const int64_t G = va.level_shape(0).size() == 3 ? ga : 1;
    const int64_t N = dx->size[0], H = dx->size[2], W = dx->size[3];
    const int64_t F = dw->size[0], Cg = dw->size[1], R = dw->size[2], S = dw->size[3];
    const int64_t P = dy->size[2], Q = dy->size[3];
    if (G < 1 || N < 1 || Cg < 1 || R < 1 || S < 1 || P < 1 || Q < 1 || H < 1 || W < 1 || F < 1 || F % G) return;
    const int64_t Kg = F / G;
    if (dx->size[1] != G * Cg || dy->size[0] != N || dy->size[1] != F) return;
    if (ma.rows != N * P * Q || ma.cols != Cg * R * S || mb.rows != ma.cols || mb.cols != Kg || mc.rows != ma.rows || mc.cols != Kg) return;
    const int64_t xs2 = dx->stride[2], xs3 = dx->stride[3];
    if (xs2 <= 0 || xs3 <= 0 || ma.rows >= (1LL << 40)) return;
    auto at = [&](int64_t n, int64_t pp, int64_t q, int64_t c, int64_t r, int64_t s_) {
        const int64_t row = (n * P + pp) * Q + q, col = (c * R + r) * S + s_;
        int64_t off = 0;
        (void)nt::element_at(ma, row, col, nt::row_part(ma, row), nt::col_part(ma, col), &off);
        return off;
    };
    const int64_t f0 = at(0, 0, 0, 0, 0, 0);
    auto step = [&](int64_t d, int64_t unit, int64_t *v) {      // a step of d elements along an axis of pitch `unit`: how many coordinates
        if (d <= 0 || d % unit) return false;
        *v = d / unit;
        return *v < (1 << 20);
    };
    int64_t sh = 1, sw = 1, dh = 1, dw_ = 1;
    if (P > 1 && !step(at(0, 1, 0, 0, 0, 0) - f0, xs2, &sh)) return;
    if (Q > 1 && !step(at(0, 0, 1, 0, 0, 0) - f0, xs3, &sw)) return;
    if (R > 1 && !step(at(0, 0, 0, 0, 1, 0) - f0, xs2, &dh)) return;
    if (S > 1 && !step(at(0, 0, 0, 0, 0, 1) - f0, xs3, &dw_)) return;
    // one group's tensors
    nt_tensor_desc gx = *dx, gw = *dw, gy = *dy;
    gx.size[1] = Cg; gw.size[0] = Kg; gy.size[1] = Kg;
    for (int64_t ph = 0; ph <= (R - 1) * dh; ++ph)
        for (int64_t pw = 0; pw <= (S - 1) * dw_; ++pw) {
            if (-ph * xs2 - pw * xs3 != f0) continue;
            Arrangement ex, ew, ey;
            if (nt::conv2d_views(&gx, &gw, &gy, (int32_t)sh, (int32_t)sw, (int32_t)ph, (int32_t)pw, &ex, &ew, &ey, (int32_t)dh, (int32_t)dw_) != NT_OK) continue;
            OperandMap ea, eb, ec;
            int64_t b1, s1;
            if (ex.lower_matrix_view(&ea, &b1, &s1) != NT_OK || ew.lower_matrix_view(&eb, &b1, &s1) != NT_OK ||
                ey.lower_matrix_view(&ec, &b1, &s1) != NT_OK)
                continue;
            if (!same_map(ea, ma) || !same_map(eb, mb) || !same_map(ec, mc)) continue;
            if (G > 1 && (sa != Cg * dx->stride[1] || sb != Kg * dw->stride[0] || sc != Kg * dy->stride[1])) continue;
            nt::ConvHint &h = out->hint;
            h.valid = true;
            h.N = N; h.C = Cg; h.H = H; h.W = W; h.K = Kg; h.R = R; h.S = S; h.P = P; h.Q = Q;
            h.sh = sh; h.sw = sw; h.ph = ph; h.pw = pw; h.dh = 1; h.dw = 1; h.dh = dh; h.dw = dw_;
            for (int d = 0; d < 4; ++d) { h.xs[d] = dx->stride[d]; h.ws[d] = dw->stride[d]; h.ys[d] = dy->stride[d]; }
            out->groups = G;
            out->step_a = sa; out->step_b = sb; out->step_c = sc;
            out->found = true;
            return;
        }
}

nt_status build_problem(int kind, const nt_tensor_desc *d0, const nt_tensor_desc *d1, const nt_tensor_desc *d2,
                        int32_t sh, int32_t sw, int32_t ph, int32_t pw, nt_tile_cfg cfg, Problem *p,
                        const ViewPrograms *views = nullptr)
{
    if (!d0 || !d1 || !d2) return fail(NT_ERR_INVALID_ARG, "null tensor descriptor");
    if (cfg.bm < 0 || cfg.bn < 0 || cfg.bk < 0) return fail(NT_ERR_INVALID_ARG, "negative tile size");
    if ((cfg.bm || cfg.bn || cfg.bk) && !(cfg.bm && cfg.bn && cfg.bk))
        return fail(NT_ERR_INVALID_ARG, "tile sizes must be all zero (default) or all positive");
    if (kind == KIND_CONV) {
        NT_TRY(nt::conv2d_views(d0, d1, d2, sh, sw, ph, pw, &p->va, &p->vb, &p->vc));
    } else if (kind == KIND_VIEWS) {
        if (!views) return fail(NT_ERR_INVALID_ARG, "null meta-operation programs");
        Arrangement *v[3] = {&p->va, &p->vb, &p->vc};
        const nt_tensor_desc *d[3] = {d0, d1, d2};
        for (int t = 0; t < 3; ++t) {
            if (views->n[t] < 0 || (views->n[t] > 0 && !views->ops[t])) return fail(NT_ERR_INVALID_ARG, "null meta-operation program");
            NT_TRY(v[t]->init(d[t]));
            NT_TRY(v[t]->apply_all(views->ops[t], views->n[t]));
            if (v[t]->n_levels() != 1) return fail(NT_ERR_SHAPE_MISMATCH, "an operand's program must end in a single level (a matrix view)");
        }
        const size_t ra = p->va.level_shape(0).size(), rb = p->vb.level_shape(0).size(), rc = p->vc.level_shape(0).size();
        if (ra != rb || ra != rc || (ra != 2 && ra != 3))
            return fail(NT_ERR_SHAPE_MISMATCH, "the three views must all be [rows, cols] or all [batch, rows, cols]");
        recognise_conv(d0, d1, d2, p->va, p->vb, p->vc, &p->vconv);
        (void)fail(NT_OK, "");                       // (attempts that did not fit leave no error text behind)
    } else {
        const int want = kind == KIND_BMM ? 3 : 2;
        if (d0->ndim != want || d1->ndim != want || d2->ndim != want)
            return fail(NT_ERR_SHAPE_MISMATCH, kind == KIND_BMM ? "bmm tensors must be 3-D" : "gemm tensors must be 2-D");
        NT_TRY(p->va.init(d0));
        NT_TRY(p->vb.init(d1));
        NT_TRY(p->vc.init(d2));
    }
    const std::vector<int64_t> sa = p->va.level_shape(0), sb = p->vb.level_shape(0), sc = p->vc.level_shape(0);
    const size_t o = sa.size() == 3 ? 1 : 0;
    if (o == 1) {
        if (sa[0] != sb[0] || sa[0] != sc[0]) return fail(NT_ERR_SHAPE_MISMATCH, "batch sizes differ");
        p->batch = sa[0];
    }
    p->M = sa[o];
    p->K = sa[o + 1];
    p->N = sb[o + 1];
    if (sb[o] != p->K) return fail(NT_ERR_SHAPE_MISMATCH, "inner dimensions of A and B differ");
    if (sc[o] != p->M || sc[o + 1] != p->N) return fail(NT_ERR_SHAPE_MISMATCH, "output shape differs from [M, N]");
    if (p->vconv.found) {
        const nt::ConvHint &h = p->vconv.hint;
        p->tile = pick_tile(KIND_CONV, 1, p->M, p->N, p->K, cfg, h.sh == 1 && h.sw == 1 && h.dh == 1 && h.dw == 1);
    } else {
        p->tile = pick_tile(kind, p->batch, p->M, p->N, p->K, cfg, sh == 1 && sw == 1);
    }
    NT_TRY(nt::arrange_matmul(p->va, p->vb, p->vc, p->tile, &p->mm));
    return NT_OK;
}

nt_status arrange_query(int kind, const nt_tensor_desc *d0, const nt_tensor_desc *d1, const nt_tensor_desc *d2,
                        int32_t sh, int32_t sw, int32_t ph, int32_t pw, nt_tile_cfg cfg,
                        int64_t *grid_out, int64_t *kt_out, int32_t operand, int64_t program_id, int64_t k,
                        int64_t *offsets_out, uint8_t *mask_out, size_t capacity, int64_t *tile_shape_out)
{
    Problem p;
    NT_TRY(build_problem(kind, d0, d1, d2, sh, sw, ph, pw, cfg, &p));
    if (grid_out) { grid_out[0] = p.mm.batch; grid_out[1] = p.mm.mt; grid_out[2] = p.mm.nt; }
    if (kt_out) *kt_out = p.mm.kt;
    if (!offsets_out && !mask_out && !tile_shape_out) return NT_OK;
    if (operand < NT_OPERAND_A || operand > NT_OPERAND_C) return fail(NT_ERR_INVALID_ARG, "operand must be 0 (A), 1 (B) or 2 (C)");
    const Arrangement &arr = operand == NT_OPERAND_A ? p.mm.a : operand == NT_OPERAND_B ? p.mm.b : p.mm.c;
    int64_t shape[NT_MAX_DIMS] = {0}, gshape[NT_MAX_DIMS];
    int32_t nd = 0, gnd = 0;
    const int64_t mid[1] = {k};
    const int n_mid = operand == NT_OPERAND_C ? 0 : 1;
    nt_status st = arr.tile_index_set(program_id, mid, n_mid, offsets_out, mask_out, capacity, shape, &nd, gshape, &gnd);
    if (tile_shape_out) { tile_shape_out[0] = shape[0]; tile_shape_out[1] = shape[1]; }
    return st;
}

// D / dD / alpha / beta: the addmm epilogue C = beta * D + alpha * (A . B); dD == nullptr: plain product
thread_local int t_last_path = -1;

nt_status run(int kind, const void *A, const nt_tensor_desc *dA, const void *B, const nt_tensor_desc *dB,
              void *C, const nt_tensor_desc *dC, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
              nt_dtype in_dtype, nt_dtype out_dtype, nt_tile_cfg cfg, void *stream,
              const void *D = nullptr, const nt_tensor_desc *dD = nullptr, float alpha = 1.f, float beta = 0.f,
              const ViewPrograms *views = nullptr, int act = 0, bool static_ws = false, const nt::LoaderTrace *trace = nullptr)
{
    t_last_path = -1;
    if (!dtype_in_ok(in_dtype)) return fail(NT_ERR_UNSUPPORTED, "input dtype must be NT_F16 or NT_BF16");
    if (!dtype_out_ok(out_dtype)) return fail(NT_ERR_UNSUPPORTED, "output dtype must be NT_F16, NT_BF16 or NT_F32");
    if ((cfg.bm || cfg.bn || cfg.bk) && cfg.bm > 0 && cfg.bn > 0 && cfg.bk > 0 && !nt::tile_is_built(cfg))
        return fail(NT_ERR_UNSUPPORTED, "no kernel built for this tile shape (see nt_tile_supported)");
    Problem p;
    NT_TRY(build_problem(kind, dA, dB, dC, sh, sw, ph, pw, cfg, &p, views));
    if (p.batch == 0 || p.M == 0 || p.N == 0) return NT_OK;
    if (!C || (p.K > 0 && (!A || !B))) return fail(NT_ERR_INVALID_ARG, "null device pointer");
    nt::GemmLaunch g{};
    int64_t nb;
    NT_TRY(p.va.lower_matrix_view(&g.ma, &nb, &g.sa_batch));
    NT_TRY(p.vb.lower_matrix_view(&g.mb, &nb, &g.sb_batch));
    NT_TRY(p.vc.lower_matrix_view(&g.mc, &nb, &g.sc_batch));
    g.alpha = alpha;
    g.beta = beta;
    g.act = act;
    g.has_d = dD != nullptr && beta != 0.f;
    if (g.has_d) {
        if (!D) return fail(NT_ERR_INVALID_ARG, "null input pointer with beta != 0");
        nt::Arrangement vd;
        NT_TRY(vd.init(dD));
        const std::vector<int64_t> sd = vd.level_shape(0);
        if (sd.size() != 2 || sd[0] != p.M || sd[1] != p.N) return fail(NT_ERR_SHAPE_MISMATCH, "input shape differs from [M, N]");
        NT_TRY(vd.lower_matrix_view(&g.md, &nb, &g.sd_batch));
        g.D = D;
    }
    if (p.K == 0) {
        if (!g.has_d) return nt::launch_fill_zero(C, g.mc, p.batch, g.sc_batch, out_dtype, stream);
        // C = beta * input: the operand-map kernel with no k tiles (its grid is that of the 64 x 64 tile)
        if (p.tile.bm != 64) return run(kind, A, dA, B, dB, C, dC, sh, sw, ph, pw, in_dtype, out_dtype, nt_tile_cfg{64, 64, 32}, stream, D, dD, alpha, beta, views, act, static_ws);
    }
    if (kind == KIND_CONV) {
        nt::ConvHint &h = g.conv;
        h.valid = true;
        h.N = dA->size[0]; h.C = dA->size[1]; h.H = dA->size[2]; h.W = dA->size[3];
        h.K = dB->size[0]; h.R = dB->size[2]; h.S = dB->size[3];
        h.P = dC->size[2]; h.Q = dC->size[3];
        h.sh = sh; h.sw = sw; h.ph = ph; h.pw = pw; h.dh = 1; h.dw = 1;
        for (int d = 0; d < 4; ++d) { h.xs[d] = dA->stride[d]; h.ws[d] = dB->stride[d]; h.ys[d] = dC->stride[d]; }
    }
    g.A = A; g.B = B; g.C = C;
    g.batch = p.batch;
    g.M = p.M; g.N = p.N; g.K = p.K;
    g.mt = p.mm.mt; g.nt = p.mm.nt; g.kt = p.mm.kt;
    g.tile = p.tile;
    g.user_tile = cfg.bm || cfg.bn || cfg.bk;
    g.in_dtype = in_dtype;
    g.out_dtype = out_dtype;
    g.stream = stream;
    if (trace) g.trace = *trace;
    if (kind == KIND_VIEWS && p.vconv.found && !g.has_d) {
        // the views are a convolution's: one launch per group on the convolution routes
        const ViewConv &v = p.vconv;
        const int64_t esz = out_dtype == NT_F32 ? 4 : 2;
        g.conv = v.hint;
        g.batch = 1;
        for (int64_t gi = 0; gi < v.groups; ++gi) {
            g.A = (const char *)A + gi * v.step_a * 2;
            g.B = (const char *)B + gi * v.step_b * 2;
            g.C = (char *)C + gi * v.step_c * esz;
            NT_TRY(nt::launch_gemm(g, &t_last_path));
        }
        return NT_OK;
    }
    if (static_ws) {
        // the library's workspace is out of bounds (it is allocated on first use); a k split goes through the fixed array
        void *p = nullptr;
        size_t bytes = 0;
        NT_TRY(nt::static_scratch(&p, &bytes));
        g.no_workspace = true;
        g.ws_given = (float *)p;
        g.ws_given_bytes = bytes;
        g.ws_strict = true;
    }
    return nt::launch_gemm(g, &t_last_path);
}

}  // namespace

extern "C" {

nt_status nt_arrange_levels(const nt_tensor_desc *src, const nt_meta_op *ops, int32_t n_ops,
                            int32_t *n_levels_out, int32_t *level_ndim_out, int64_t *level_shape_out)
{
    if (!n_levels_out || !level_ndim_out || !level_shape_out) return fail(NT_ERR_INVALID_ARG, "null output pointer");
    Arrangement a;
    NT_TRY(a.init(src));
    NT_TRY(a.apply_all(ops, n_ops));
    *n_levels_out = a.n_levels();
    for (int l = 0; l < a.n_levels(); ++l) {
        const std::vector<int64_t> s = a.level_shape(l);
        level_ndim_out[l] = (int32_t)s.size();
        for (size_t d = 0; d < s.size(); ++d) level_shape_out[l * NT_MAX_DIMS + d] = s[d];
    }
    return NT_OK;
}

nt_status nt_arrange_tile(const nt_tensor_desc *src, const nt_meta_op *ops, int32_t n_ops,
                          int64_t program_id, const int64_t *mid_idx, int32_t n_mid,
                          int64_t *offsets_out, uint8_t *mask_out, size_t capacity,
                          int64_t *tile_shape_out, int32_t *tile_ndim_out,
                          int64_t *grid_shape_out, int32_t *grid_ndim_out)
{
    Arrangement a;
    NT_TRY(a.init(src));
    NT_TRY(a.apply_all(ops, n_ops));
    return a.tile_index_set(program_id, mid_idx, n_mid, offsets_out, mask_out, capacity,
                            tile_shape_out, tile_ndim_out, grid_shape_out, grid_ndim_out);
}

nt_status nt_arrange_gemm(const nt_tensor_desc *dA, const nt_tensor_desc *dB, const nt_tensor_desc *dC,
                          nt_tile_cfg cfg, int64_t *grid_out, int64_t *kt_out,
                          int32_t operand, int64_t program_id, int64_t k,
                          int64_t *offsets_out, uint8_t *mask_out, size_t capacity, int64_t *tile_shape_out)
{
    return arrange_query(KIND_GEMM, dA, dB, dC, 1, 1, 0, 0, cfg, grid_out, kt_out, operand, program_id, k,
                         offsets_out, mask_out, capacity, tile_shape_out);
}

nt_status nt_arrange_bmm(const nt_tensor_desc *dA, const nt_tensor_desc *dB, const nt_tensor_desc *dC,
                         nt_tile_cfg cfg, int64_t *grid_out, int64_t *kt_out,
                         int32_t operand, int64_t program_id, int64_t k,
                         int64_t *offsets_out, uint8_t *mask_out, size_t capacity, int64_t *tile_shape_out)
{
    return arrange_query(KIND_BMM, dA, dB, dC, 1, 1, 0, 0, cfg, grid_out, kt_out, operand, program_id, k,
                         offsets_out, mask_out, capacity, tile_shape_out);
}

nt_status nt_arrange_conv2d(const nt_tensor_desc *dx, const nt_tensor_desc *dw, const nt_tensor_desc *dy,
                            int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                            nt_tile_cfg cfg, int64_t *grid_out, int64_t *kt_out,
                            int32_t operand, int64_t program_id, int64_t k,
                            int64_t *offsets_out, uint8_t *mask_out, size_t capacity, int64_t *tile_shape_out)
{
    return arrange_query(KIND_CONV, dx, dw, dy, stride_h, stride_w, pad_h, pad_w, cfg, grid_out, kt_out,
                         operand, program_id, k, offsets_out, mask_out, capacity, tile_shape_out);
}

nt_status nt_program_order(int64_t batch, int64_t mt, int64_t nt_, int64_t *pid_out)
{
    if (!pid_out) return fail(NT_ERR_INVALID_ARG, "null output pointer");
    if (batch < 0 || mt < 0 || nt_ < 0) return fail(NT_ERR_INVALID_ARG, "negative grid size");
    const int64_t per = mt * nt_;
    for (int64_t w = 0; w < batch * per; ++w) {
        int64_t b, pid;
        nt::program_of_workgroup_batched(w, batch, mt, nt_, &b, &pid);
        pid_out[w] = b * per + pid;
    }
    return NT_OK;
}

int32_t nt_tile_supported(nt_tile_cfg cfg)
{
    if (cfg.bm == 0 && cfg.bn == 0 && cfg.bk == 0) return 1;
    return nt::tile_is_built(cfg) ? 1 : 0;
}

int32_t nt_last_kernel_path(void) { return t_last_path; }
int32_t nt_last_k_split(void) { return t_last_path < 0 ? 1 : nt::last_k_split(); }

nt_status nt_matmul_views(const void *A, const nt_tensor_desc *dA, const nt_meta_op *opsA, int32_t nA,
                          const void *B, const nt_tensor_desc *dB, const nt_meta_op *opsB, int32_t nB,
                          void *C, const nt_tensor_desc *dC, const nt_meta_op *opsC, int32_t nC,
                          nt_dtype in_dtype, nt_dtype out_dtype, nt_tile_cfg cfg, void *hip_stream)
{
    const ViewPrograms views{{opsA, opsB, opsC}, {nA, nB, nC}};
    return run(KIND_VIEWS, A, dA, B, dB, C, dC, 1, 1, 0, 0, in_dtype, out_dtype, cfg, hip_stream, nullptr, nullptr, 1.f, 0.f, &views);
}

nt_status nt_gemm(const void *A, const nt_tensor_desc *dA, const void *B, const nt_tensor_desc *dB,
                  void *C, const nt_tensor_desc *dC, nt_dtype in_dtype, nt_dtype out_dtype,
                  nt_tile_cfg cfg, void *hip_stream)
{
    return run(KIND_GEMM, A, dA, B, dB, C, dC, 1, 1, 0, 0, in_dtype, out_dtype, cfg, hip_stream);
}

nt_status nt_gemm_noalloc(const void *A, const nt_tensor_desc *dA, const void *B, const nt_tensor_desc *dB,
                          void *C, const nt_tensor_desc *dC, nt_dtype in_dtype, nt_dtype out_dtype,
                          nt_tile_cfg cfg, void *hip_stream)
{
    return run(KIND_GEMM, A, dA, B, dB, C, dC, 1, 1, 0, 0, in_dtype, out_dtype, cfg, hip_stream, nullptr, nullptr, 1.f, 0.f, nullptr, 0, true);
}

nt_status nt_addmm(const void *input, const nt_tensor_desc *dI, const void *A, const nt_tensor_desc *dA,
                   const void *B, const nt_tensor_desc *dB, void *C, const nt_tensor_desc *dC,
                   float alpha, float beta, nt_dtype in_dtype, nt_dtype out_dtype, nt_tile_cfg cfg, void *hip_stream)
{
    if (!dI) return fail(NT_ERR_INVALID_ARG, "null tensor descriptor");
    if (!(alpha == alpha) || !(beta == beta)) return fail(NT_ERR_INVALID_ARG, "alpha / beta is NaN");
    return run(KIND_GEMM, A, dA, B, dB, C, dC, 1, 1, 0, 0, in_dtype, out_dtype, cfg, hip_stream, input, dI, alpha, beta);
}

nt_status nt_addmm_act(const void *input, const nt_tensor_desc *dI, const void *A, const nt_tensor_desc *dA,
                       const void *B, const nt_tensor_desc *dB, void *C, const nt_tensor_desc *dC,
                       float alpha, float beta, nt_activation act, nt_dtype in_dtype, nt_dtype out_dtype,
                       nt_tile_cfg cfg, void *hip_stream)
{
    if (!(alpha == alpha) || !(beta == beta)) return fail(NT_ERR_INVALID_ARG, "alpha / beta is NaN");
    if (act != NT_ACT_NONE && act != NT_ACT_RELU && act != NT_ACT_SILU && act != NT_ACT_GELU_TANH)
        return fail(NT_ERR_INVALID_ARG, "unknown activation");
    if (!dI && beta != 0.f) return fail(NT_ERR_INVALID_ARG, "null input descriptor with beta != 0");
    return run(KIND_GEMM, A, dA, B, dB, C, dC, 1, 1, 0, 0, in_dtype, out_dtype, cfg, hip_stream, input, dI, alpha, beta, nullptr, (int)act);
}

static nt_status check_1d(const nt_tensor_desc *d, const void *p, int64_t *n, int64_t *stride)
{
    if (!d) return fail(NT_ERR_INVALID_ARG, "null tensor descriptor");
    if (d->ndim != 1) return fail(NT_ERR_SHAPE_MISMATCH, "tensor must be 1-D");
    if (d->size[0] < 0) return fail(NT_ERR_INVALID_ARG, "negative size");
    if (d->size[0] > 0 && !p) return fail(NT_ERR_INVALID_ARG, "null device pointer");
    *n = d->size[0];
    *stride = d->stride[0];
    return NT_OK;
}

static nt_status map_op(int op, const void *x, const nt_tensor_desc *dx, const void *y, const nt_tensor_desc *dy,
                        void *out, const nt_tensor_desc *dout, nt_dtype dtype, int64_t block_size, void *stream)
{
    if (!dtype_in_ok(dtype)) return fail(NT_ERR_UNSUPPORTED, "dtype must be NT_F16 or NT_BF16");
    if (block_size < 0) return fail(NT_ERR_INVALID_ARG, "block_size must be positive (0 = default)");
    int64_t n, sx, ny = 0, sy = 0, no, so;
    NT_TRY(check_1d(dx, x, &n, &sx));
    if (op == 0) NT_TRY(check_1d(dy, y, &ny, &sy));
    NT_TRY(check_1d(dout, out, &no, &so));
    if (no != n || (op == 0 && ny != n)) return fail(NT_ERR_SHAPE_MISMATCH, "tensor sizes differ");
    return nt::launch_map(op, x, sx, y, sy, out, so, n, dtype, stream);
}

static nt_status rows_op(int op, const void *x, const nt_tensor_desc *dx, void *out, const nt_tensor_desc *dout,
                         float eps, nt_dtype dtype, void *stream)
{
    if (!dtype_in_ok(dtype)) return fail(NT_ERR_UNSUPPORTED, "dtype must be NT_F16 or NT_BF16");
    if (!dx || !dout) return fail(NT_ERR_INVALID_ARG, "null tensor descriptor");
    if (dx->ndim != 2 || dout->ndim != 2) return fail(NT_ERR_SHAPE_MISMATCH, "tensors must be 2-D");
    if (dx->size[0] < 0 || dx->size[1] < 0) return fail(NT_ERR_INVALID_ARG, "negative size");
    if (dx->size[0] != dout->size[0] || dx->size[1] != dout->size[1]) return fail(NT_ERR_SHAPE_MISMATCH, "input and output shapes differ");
    if (!(eps >= 0.f)) return fail(NT_ERR_INVALID_ARG, "eps must be >= 0");
    if (dx->size[0] > 0 && dx->size[1] > 0 && (!x || !out)) return fail(NT_ERR_INVALID_ARG, "null device pointer");
    return nt::launch_rows(op, x, dx->stride[0], dx->stride[1], out, dout->stride[0], dout->stride[1], dx->size[0], dx->size[1], eps, dtype, stream);
}

nt_status nt_add(const void *x, const nt_tensor_desc *dx, const void *y, const nt_tensor_desc *dy,
                 void *out, const nt_tensor_desc *dout, nt_dtype dtype, int64_t block_size, void *hip_stream)
{
    return map_op(0, x, dx, y, dy, out, dout, dtype, block_size, hip_stream);
}

nt_status nt_silu(const void *x, const nt_tensor_desc *dx, void *out, const nt_tensor_desc *dout,
                  nt_dtype dtype, int64_t block_size, void *hip_stream)
{
    return map_op(1, x, dx, nullptr, nullptr, out, dout, dtype, block_size, hip_stream);
}

nt_status nt_softmax(const void *x, const nt_tensor_desc *dx, void *out, const nt_tensor_desc *dout, nt_dtype dtype, void *hip_stream)
{
    return rows_op(0, x, dx, out, dout, 0.f, dtype, hip_stream);
}

nt_status nt_rms_norm(const void *x, const nt_tensor_desc *dx, void *out, const nt_tensor_desc *dout,
                      float eps, nt_dtype dtype, void *hip_stream)
{
    return rows_op(1, x, dx, out, dout, eps, dtype, hip_stream);
}

nt_status nt_sdpa(const void *q, const nt_tensor_desc *dq, const void *k, const nt_tensor_desc *dk,
                  const void *v, const nt_tensor_desc *dv, void *o, const nt_tensor_desc *dout,
                  float scale, nt_dtype dtype, void *hip_stream)
{
    if (!dtype_in_ok(dtype)) return fail(NT_ERR_UNSUPPORTED, "dtype must be NT_F16 or NT_BF16");
    return nt::launch_sdpa_desc(q, dq, k, dk, v, dv, o, dout, scale, dtype, hip_stream);
}

nt_status nt_bmm(const void *A, const nt_tensor_desc *dA, const void *B, const nt_tensor_desc *dB,
                 void *C, const nt_tensor_desc *dC, nt_dtype in_dtype, nt_dtype out_dtype,
                 nt_tile_cfg cfg, void *hip_stream)
{
    return run(KIND_BMM, A, dA, B, dB, C, dC, 1, 1, 0, 0, in_dtype, out_dtype, cfg, hip_stream);
}

nt_status nt_conv2d_implicit(const void *x, const nt_tensor_desc *dx, const void *w, const nt_tensor_desc *dw,
                             void *y, const nt_tensor_desc *dy,
                             int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                             nt_dtype in_dtype, nt_dtype out_dtype, nt_tile_cfg cfg, void *hip_stream)
{
    return run(KIND_CONV, x, dx, w, dw, y, dy, stride_h, stride_w, pad_h, pad_w, in_dtype, out_dtype, cfg, hip_stream);
}

nt_status nt_trace_tile(int32_t kind, const nt_tensor_desc *d0, const nt_tensor_desc *d1, const nt_tensor_desc *d2,
                        int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                        nt_tile_cfg cfg, int32_t operand, int64_t program_id, int64_t k,
                        int64_t *offsets_out, uint8_t *mask_out, size_t capacity, void *hip_stream)
{
    if (kind < KIND_GEMM || kind > KIND_CONV) return fail(NT_ERR_INVALID_ARG, "kind must be 0 (gemm), 1 (bmm) or 2 (conv2d)");
    if (operand < NT_OPERAND_A || operand > NT_OPERAND_C) return fail(NT_ERR_INVALID_ARG, "operand must be 0, 1 or 2");
    if (!offsets_out || !mask_out) return fail(NT_ERR_INVALID_ARG, "null output pointer");
    Problem p;
    NT_TRY(build_problem(kind, d0, d1, d2, stride_h, stride_w, pad_h, pad_w, cfg, &p));
    const int64_t per = p.mm.mt * p.mm.nt;
    if (program_id < 0 || program_id >= p.mm.batch * per) return fail(NT_ERR_INVALID_ARG, "program_id outside the grid");
    if (operand != NT_OPERAND_C && (k < 0 || k >= p.mm.kt)) return fail(NT_ERR_INVALID_ARG, "k outside the k tiles");
    const int64_t b = program_id / per, i = (program_id % per) / p.mm.nt, j = program_id % p.mm.nt;
    OperandMap m;
    int64_t nb, bstride;
    const Arrangement &view = operand == NT_OPERAND_A ? p.va : operand == NT_OPERAND_B ? p.vb : p.vc;
    NT_TRY(view.lower_matrix_view(&m, &nb, &bstride));
    int64_t row0, col0;
    int32_t rows, cols;
    if (operand == NT_OPERAND_A) { row0 = i * p.tile.bm; col0 = k * p.tile.bk; rows = p.tile.bm; cols = p.tile.bk; }
    else if (operand == NT_OPERAND_B) { row0 = k * p.tile.bk; col0 = j * p.tile.bn; rows = p.tile.bk; cols = p.tile.bn; }
    else { row0 = i * p.tile.bm; col0 = j * p.tile.bn; rows = p.tile.bm; cols = p.tile.bn; }
    if ((size_t)rows * (size_t)cols > capacity) return fail(NT_ERR_BUFFER_TOO_SMALL, "trace buffers smaller than the tile");
    return nt::launch_trace(m, b * bstride, row0, col0, rows, cols, offsets_out, mask_out, hip_stream);
}

nt_status nt_trace_loader_slice(int32_t kind, const void *A, const nt_tensor_desc *dA, const void *B, const nt_tensor_desc *dB,
                                const nt_tensor_desc *dC, int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                                nt_dtype in_dtype, nt_dtype out_dtype, nt_tile_cfg cfg, int32_t operand, int64_t program_id, int64_t slice,
                                uint16_t *values_out, size_t capacity, void *hip_stream)
{
    if (kind < KIND_GEMM || kind > KIND_CONV) return fail(NT_ERR_INVALID_ARG, "kind must be 0 (gemm), 1 (bmm) or 2 (conv2d)");
    if (operand != NT_OPERAND_A && operand != NT_OPERAND_B) return fail(NT_ERR_INVALID_ARG, "operand must be 0 (A) or 1 (B)");
    if (!values_out) return fail(NT_ERR_INVALID_ARG, "null output pointer");
    const nt::LoaderTrace tr{values_out, capacity, program_id, (int32_t)slice, operand};
    if (slice < 0 || slice > 0x7fffffff) return fail(NT_ERR_INVALID_ARG, "slice outside the reduction");
    // (the output pointer only has to be non-null: a trace stores nothing through it)
    return run(kind, A, dA, B, dB, values_out, dC, stride_h, stride_w, pad_h, pad_w, in_dtype, out_dtype, cfg, hip_stream,
               nullptr, nullptr, 1.f, 0.f, nullptr, 0, false, &tr);
}

nt_status nt_mfma_probe(const void *data, int64_t n_elems, nt_dtype dtype, int32_t iters, int32_t blocks, float *out, void *hip_stream)
{
    if (!dtype_in_ok(dtype)) return fail(NT_ERR_UNSUPPORTED, "dtype must be NT_F16 or NT_BF16");
    if (!data || !out) return fail(NT_ERR_INVALID_ARG, "null device pointer");
    if (n_elems < 8 || iters < 0 || blocks <= 0) return fail(NT_ERR_INVALID_ARG, "n_elems >= 8, iters >= 0 and blocks > 0 wanted");
    if ((reinterpret_cast<uintptr_t>(data) & 15) != 0) return fail(NT_ERR_INVALID_ARG, "data must be 16-byte aligned");
    return nt::launch_mfma_probe(data, n_elems, dtype, iters, blocks, out, hip_stream);
}

const char *nt_last_error(void) { return nt::last_error().c_str(); }

const char *nt_version(void) { return "nt-mi355x 0.4 (gfx950)"; }

}  // extern "C"
