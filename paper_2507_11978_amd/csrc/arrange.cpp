// Host-side arrangement engine (see arrange.h).  Pure integer code, no device calls.
#include "arrange.h"

#include <algorithm>
#include <map>
#include <sstream>

namespace nt {

static thread_local std::string g_last_error;

void set_error(const std::string &msg) { g_last_error = msg; }
const std::string &last_error() { return g_last_error; }

nt_status fail(nt_status st, const std::string &msg)
{
    g_last_error = msg;
    return st;
}

static int64_t ceil_div(int64_t a, int64_t b)   // b > 0, a of either sign
{
    return a >= 0 ? (a + b - 1) / b : -((-a) / b);
}

// ------------------------------------------------------------------ construction
nt_status Arrangement::init(const nt_tensor_desc *src)
{
    if (!src) return fail(NT_ERR_INVALID_ARG, "null tensor descriptor");
    if (src->ndim < 1 || src->ndim > NT_MAX_DIMS) return fail(NT_ERR_INVALID_ARG, "ndim must be 1..6");
    for (int i = 0; i < src->ndim; ++i)
        if (src->size[i] < 0) return fail(NT_ERR_INVALID_ARG, "negative size");
    src_ = *src;
    size_.assign(src->size, src->size + src->ndim);
    nodes_.clear();
    levels_.assign(1, std::vector<int>());
    for (int i = 0; i < src->ndim; ++i) levels_[0].push_back(i);
    cursor_ = 0;
    return NT_OK;
}

std::vector<int64_t> Arrangement::level_shape(int l) const
{
    std::vector<int64_t> s;
    for (int id : levels_[l]) s.push_back(size_[id]);
    return s;
}

int64_t Arrangement::num_programs() const
{
    int64_t g = 1;
    for (int id : levels_[0]) g *= size_[id];
    return g;
}

nt_status Arrangement::tile(std::vector<int64_t> shape, std::vector<int64_t> strides,
                            std::vector<int64_t> pad_lo, std::vector<int64_t> pad_hi, std::vector<int64_t> dilation)
{
    std::vector<int> &lv = levels_[cursor_];
    const size_t r = lv.size();
    if (shape.size() != r) return fail(NT_ERR_SHAPE_MISMATCH, "tile: rank of tile_shape differs from the level's rank");
    if ((!strides.empty() && strides.size() != r) || (!pad_lo.empty() && pad_lo.size() != r) ||
        (!pad_hi.empty() && pad_hi.size() != r) || (!dilation.empty() && dilation.size() != r))
        return fail(NT_ERR_INVALID_ARG, "tile: strides/padding/dilation rank differs from the level's rank");
    if ((int)levels_.size() + 1 > NT_MAX_LEVELS) return fail(NT_ERR_UNSUPPORTED, "tile: too many levels");
    std::vector<int> outer(r), inner(r);
    std::vector<Node> fresh;
    std::vector<int64_t> new_sizes;
    for (size_t i = 0; i < r; ++i) {
        const int p = lv[i];
        const int64_t S = size_[p];
        const bool whole = shape[i] == -1;
        const int64_t T = whole ? S : shape[i];
        if (T < 0 || (T == 0 && S != 0)) return fail(NT_ERR_INVALID_ARG, "tile: tile sizes must be positive (or -1)");
        int64_t st = (strides.empty() || strides[i] <= 0) ? T : strides[i];
        if (st <= 0) st = 1;
        const int64_t lo = pad_lo.empty() ? 0 : pad_lo[i];
        const int64_t hi = pad_hi.empty() ? 0 : pad_hi[i];
        const int64_t dil = (dilation.empty() || dilation[i] == -1 || dilation[i] == 0) ? 1 : dilation[i];
        if (dil < 1) return fail(NT_ERR_INVALID_ARG, "tile: dilation must be positive");
        const int64_t ext = S + lo + hi;
        const int64_t span = T > 0 ? (T - 1) * dil + 1 : 0;     // source coordinates from a tile's first to its last element
        int64_t O;
        if (ext > 0)
            O = std::max<int64_t>(ceil_div(ext - span, st) + 1, 0);
        else
            O = whole ? 1 : 0;
        Node nd;
        nd.kind = Node::TILE;
        nd.in0 = (int)(size_.size() + new_sizes.size());
        new_sizes.push_back(O);
        nd.in1 = (int)(size_.size() + new_sizes.size());
        new_sizes.push_back(T);
        nd.out[0] = p;
        nd.nout = 1;
        nd.st = st;
        nd.lo = lo;
        nd.dil = dil;
        nd.bound = S;
        outer[i] = nd.in0;
        inner[i] = nd.in1;
        fresh.push_back(nd);
    }
    size_.insert(size_.end(), new_sizes.begin(), new_sizes.end());
    nodes_.insert(nodes_.end(), fresh.begin(), fresh.end());
    levels_[cursor_] = outer;
    levels_.insert(levels_.begin() + cursor_ + 1, inner);
    return NT_OK;
}

nt_status Arrangement::expand(std::vector<int64_t> shape)
{
    std::vector<int> &lv = levels_[cursor_];
    if (shape.size() != lv.size()) return fail(NT_ERR_SHAPE_MISMATCH, "expand: rank differs from the level's rank");
    for (size_t i = 0; i < lv.size(); ++i) {
        const int64_t S = size_[lv[i]];
        if (shape[i] == -1 || shape[i] == S) continue;
        if (shape[i] < 0) return fail(NT_ERR_INVALID_ARG, "expand: negative size");
        if (S != 1) return fail(NT_ERR_SHAPE_MISMATCH, "expand: only singleton dimensions can be expanded");
    }
    for (size_t i = 0; i < lv.size(); ++i) {
        const int64_t S = size_[lv[i]];
        if (shape[i] == -1 || shape[i] == S) continue;
        Node nd;
        nd.kind = Node::ZERO;
        nd.out[0] = lv[i];
        nd.nout = 1;
        nodes_.push_back(nd);
        size_.push_back(shape[i]);
        lv[i] = (int)size_.size() - 1;
    }
    return NT_OK;
}

nt_status Arrangement::squeeze(int64_t dim)
{
    std::vector<int> &lv = levels_[cursor_];
    if (dim < 0 || dim >= (int64_t)lv.size()) return fail(NT_ERR_INVALID_ARG, "squeeze: dimension out of range");
    if (size_[lv[dim]] != 1) return fail(NT_ERR_SHAPE_MISMATCH, "squeeze: dimension is not a singleton");
    Node nd;
    nd.kind = Node::ZERO;
    nd.out[0] = lv[dim];
    nd.nout = 1;
    nodes_.push_back(nd);
    lv.erase(lv.begin() + dim);
    return NT_OK;
}

nt_status Arrangement::permute(std::vector<int64_t> order)
{
    std::vector<int> &lv = levels_[cursor_];
    if (order.size() != lv.size()) return fail(NT_ERR_SHAPE_MISMATCH, "permute: rank differs from the level's rank");
    std::vector<int64_t> sorted = order;
    std::sort(sorted.begin(), sorted.end());
    for (size_t i = 0; i < sorted.size(); ++i)
        if (sorted[i] != (int64_t)i) return fail(NT_ERR_INVALID_ARG, "permute: not a permutation");
    std::vector<int> nl(lv.size());
    for (size_t i = 0; i < lv.size(); ++i) nl[i] = lv[order[i]];
    lv = nl;
    return NT_OK;
}

nt_status Arrangement::flatten(int64_t start, int64_t end)
{
    std::vector<int> &lv = levels_[cursor_];
    if (start < 0 || end < start || end > (int64_t)lv.size())
        return fail(NT_ERR_INVALID_ARG, "flatten: range outside the level");
    Node nd;
    nd.kind = Node::SPLIT;
    int64_t total = 1;
    for (int64_t i = start; i < end; ++i) {
        nd.out[nd.nout] = lv[i];
        nd.radix[nd.nout] = size_[lv[i]];
        ++nd.nout;
        total *= size_[lv[i]];
    }
    size_.push_back(total);
    nd.in0 = (int)size_.size() - 1;
    nodes_.push_back(nd);
    lv.erase(lv.begin() + start, lv.begin() + end);
    lv.insert(lv.begin() + start, nd.in0);
    return NT_OK;
}

nt_status Arrangement::ravel()
{
    std::vector<int> flat;
    for (size_t l = cursor_; l < levels_.size(); ++l) flat.insert(flat.end(), levels_[l].begin(), levels_[l].end());
    if (flat.size() > NT_MAX_DIMS) return fail(NT_ERR_UNSUPPORTED, "ravel: more than NT_MAX_DIMS dimensions in one level");
    levels_.resize(cursor_ + 1);
    levels_[cursor_] = flat;
    return NT_OK;
}

nt_status Arrangement::descend()
{
    if (cursor_ + 1 >= (int)levels_.size()) return fail(NT_ERR_SHAPE_MISMATCH, "descend: no inner level");
    ++cursor_;
    return NT_OK;
}

nt_status Arrangement::ascend()
{
    if (cursor_ == 0) return fail(NT_ERR_INVALID_ARG, "ascend: already at the outermost level");
    --cursor_;
    return NT_OK;
}

nt_status Arrangement::apply(const nt_meta_op &op)
{
    if (op.n < 0 || op.n > NT_MAX_DIMS) return fail(NT_ERR_INVALID_ARG, "meta-op: n out of range");
    auto vec = [&](const int64_t *p) { return std::vector<int64_t>(p, p + op.n); };
    switch (op.kind) {
    case NT_OP_TILE: return tile(vec(op.a), vec(op.b), vec(op.c), vec(op.d), vec(op.e));
    case NT_OP_EXPAND: return expand(vec(op.a));
    case NT_OP_SQUEEZE: return squeeze(op.a[0]);
    case NT_OP_PERMUTE: return permute(vec(op.a));
    case NT_OP_FLATTEN: return flatten(op.a[0], op.a[1]);
    case NT_OP_RAVEL: return ravel();
    case NT_OP_DESCEND: return descend();
    case NT_OP_ASCEND: return ascend();
    default: return fail(NT_ERR_INVALID_ARG, "meta-op: unknown kind");
    }
}

nt_status Arrangement::apply_all(const nt_meta_op *ops, int32_t n_ops)
{
    if (n_ops < 0 || (n_ops > 0 && !ops)) return fail(NT_ERR_INVALID_ARG, "null meta-op array");
    for (int32_t i = 0; i < n_ops; ++i) {
        nt_status st = apply(ops[i]);
        if (st != NT_OK) return st;
    }
    cursor_ = 0;
    return NT_OK;
}

// -------------------------------------------------------------------- evaluation
bool Arrangement::eval(std::vector<int64_t> &vals, int64_t *offset) const
{
    bool valid = true;
    for (size_t n = nodes_.size(); n-- > 0;) {
        const Node &nd = nodes_[n];
        if (nd.kind == Node::TILE) {
            const int64_t v = vals[nd.in0] * nd.st + vals[nd.in1] * nd.dil - nd.lo;
            valid = valid && v >= 0 && v < nd.bound;
            vals[nd.out[0]] = v;
        } else if (nd.kind == Node::ZERO) {
            vals[nd.out[0]] = 0;
        } else {
            int64_t rem = vals[nd.in0];
            for (int i = nd.nout - 1; i >= 0; --i) {
                const int64_t r = nd.radix[i];
                vals[nd.out[i]] = r ? rem % r : 0;
                rem = r ? rem / r : 0;
            }
        }
    }
    int64_t off = 0;
    for (int s = 0; s < src_.ndim; ++s) {
        valid = valid && vals[s] >= 0 && vals[s] < src_.size[s];
        off += vals[s] * src_.stride[s];
    }
    *offset = valid ? off : -1;
    return valid;
}

nt_status Arrangement::tile_index_set(int64_t program_id, const int64_t *mid_idx, int32_t n_mid,
                                      int64_t *offsets_out, uint8_t *mask_out, size_t capacity,
                                      int64_t *tile_shape_out, int32_t *tile_ndim_out,
                                      int64_t *grid_shape_out, int32_t *grid_ndim_out) const
{
    const int nl = (int)levels_.size();
    const std::vector<int> &grid = levels_[0];
    static const std::vector<int> none;
    const std::vector<int> &inner = nl > 1 ? levels_[nl - 1] : none;
    if (grid_shape_out)
        for (size_t i = 0; i < grid.size(); ++i) grid_shape_out[i] = size_[grid[i]];
    if (grid_ndim_out) *grid_ndim_out = (int32_t)grid.size();
    if (tile_shape_out)
        for (size_t i = 0; i < inner.size(); ++i) tile_shape_out[i] = size_[inner[i]];
    if (tile_ndim_out) *tile_ndim_out = (int32_t)inner.size();
    if (!offsets_out && !mask_out) return NT_OK;

    int64_t count = 1;
    for (int id : inner) count *= size_[id];
    if ((size_t)count > capacity) {
        std::ostringstream os;
        os << "tile has " << count << " elements, capacity is " << capacity;
        return fail(NT_ERR_BUFFER_TOO_SMALL, os.str());
    }
    const int64_t G = num_programs();
    if (program_id < 0 || program_id >= G) return fail(NT_ERR_INVALID_ARG, "program_id outside the grid");
    int want_mid = 0;
    for (int l = 1; l < nl - 1; ++l) want_mid += (int)levels_[l].size();
    if (n_mid != want_mid || (want_mid > 0 && !mid_idx))
        return fail(NT_ERR_INVALID_ARG, "wrong number of middle-level indices");

    std::vector<int64_t> vals(size_.size(), 0);
    int64_t rem = program_id;
    for (size_t i = grid.size(); i-- > 0;) {           // row-major: last dimension fastest
        const int64_t s = size_[grid[i]];
        vals[grid[i]] = rem % s;
        rem /= s;
    }
    int pos = 0;
    for (int l = 1; l < nl - 1; ++l)
        for (int id : levels_[l]) {
            if (mid_idx[pos] < 0 || mid_idx[pos] >= size_[id])
                return fail(NT_ERR_INVALID_ARG, "middle-level index out of range");
            vals[id] = mid_idx[pos++];
        }
    std::vector<int64_t> ctr(inner.size(), 0);
    for (int64_t e = 0; e < count; ++e) {
        for (size_t i = 0; i < inner.size(); ++i) vals[inner[i]] = ctr[i];
        int64_t off;
        const bool ok = eval(vals, &off);
        if (offsets_out) offsets_out[e] = off;
        if (mask_out) mask_out[e] = ok ? 1 : 0;
        for (size_t i = inner.size(); i-- > 0;) {       // odometer, last dimension fastest
            if (++ctr[i] < size_[inner[i]]) break;
            ctr[i] = 0;
        }
    }
    return NT_OK;
}

// ---------------------------------------------------------------------- lowering
namespace {
struct Lin {                       // c + sum coef[v] * var v
    int64_t c = 0;
    std::map<int, int64_t> coef;
};
struct Var {
    int axis;                      // 0 row, 1 col, 2 batch
    int64_t hi;                    // range [0, hi]
    int64_t radix;                 // size of the digit
    bool split = false;
};
}  // namespace

nt_status Arrangement::lower_matrix_view(OperandMap *map, int64_t *batch_out, int64_t *batch_stride_out) const
{
    if (levels_.size() != 1) return fail(NT_ERR_UNSUPPORTED, "lowering needs a single-level matrix view");
    const std::vector<int> &lv = levels_[0];
    const int rank = (int)lv.size();
    if (rank != 2 && rank != 3) return fail(NT_ERR_SHAPE_MISMATCH, "matrix view must have rank 2 (or 3 with batch)");
    std::vector<Var> vars;
    std::vector<std::vector<int>> digits(3);      // per axis: variable ids, slowest first
    std::map<int, Lin> lin;                       // dimension id -> linear form
    for (int i = 0; i < rank; ++i) {
        const int axis = rank == 3 ? (i == 0 ? 2 : i - 1) : i;
        Var v{axis, std::max<int64_t>(size_[lv[i]] - 1, 0), size_[lv[i]]};
        vars.push_back(v);
        digits[axis].push_back((int)vars.size() - 1);
        Lin l;
        l.coef[(int)vars.size() - 1] = 1;
        lin[lv[i]] = l;
    }
    auto range = [&](const Lin &l, int64_t *mn, int64_t *mx) {
        *mn = *mx = l.c;
        for (auto &kv : l.coef) {
            if (kv.second >= 0) *mx += kv.second * vars[kv.first].hi;
            else *mn += kv.second * vars[kv.first].hi;
        }
    };
    std::vector<char> checked(src_.ndim, 0);
    for (size_t n = nodes_.size(); n-- > 0;) {
        const Node &nd = nodes_[n];
        if (nd.kind == Node::ZERO) {
            lin[nd.out[0]] = Lin();
        } else if (nd.kind == Node::TILE) {
            if (!lin.count(nd.in0) || !lin.count(nd.in1))
                return fail(NT_ERR_UNSUPPORTED, "lowering: tile fed by a dimension outside the view");
            Lin r;
            r.c = lin[nd.in0].c * nd.st + lin[nd.in1].c * nd.dil - nd.lo;
            for (auto &kv : lin[nd.in0].coef) r.coef[kv.first] += kv.second * nd.st;
            for (auto &kv : lin[nd.in1].coef) r.coef[kv.first] += kv.second * nd.dil;
            int64_t mn, mx;
            range(r, &mn, &mx);
            if (mn < 0 || mx >= nd.bound) {
                if (nd.out[0] >= src_.ndim)
                    return fail(NT_ERR_UNSUPPORTED, "lowering: ragged tile of a non-source dimension");
                checked[nd.out[0]] = 1;
            }
            lin[nd.out[0]] = r;
        } else {
            if (!lin.count(nd.in0)) return fail(NT_ERR_UNSUPPORTED, "lowering: flatten outside the view");
            const Lin &m = lin[nd.in0];
            if (m.c != 0 || m.coef.size() != 1 || m.coef.begin()->second != 1)
                return fail(NT_ERR_UNSUPPORTED, "lowering: flatten of a non-trivial index");
            const int parent = m.coef.begin()->first;
            if (vars[parent].split) return fail(NT_ERR_UNSUPPORTED, "lowering: dimension flattened twice");
            vars[parent].split = true;
            const int axis = vars[parent].axis;
            std::vector<int> fresh;
            for (int i = 0; i < nd.nout; ++i) {
                Var v{axis, std::max<int64_t>(nd.radix[i] - 1, 0), nd.radix[i]};
                vars.push_back(v);
                fresh.push_back((int)vars.size() - 1);
                Lin l;
                l.coef[(int)vars.size() - 1] = 1;
                lin[nd.out[i]] = l;
            }
            auto &dl = digits[axis];
            auto it = std::find(dl.begin(), dl.end(), parent);
            it = dl.erase(it);
            dl.insert(it, fresh.begin(), fresh.end());
        }
    }
    for (int s = 0; s < src_.ndim; ++s) {
        if (!lin.count(s)) return fail(NT_ERR_UNSUPPORTED, "lowering: a source dimension is not addressed");
        int64_t mn, mx;
        range(lin[s], &mn, &mx);
        if (mn < 0 || mx >= src_.size[s]) checked[s] = 1;
    }
    if (digits[2].size() > 1) return fail(NT_ERR_UNSUPPORTED, "lowering: batch dimension must stay whole");

    // per-variable offset step and check coefficients
    std::vector<int> chk_dims;
    for (int s = 0; s < src_.ndim; ++s)
        if (checked[s]) chk_dims.push_back(s);
    if ((int)chk_dims.size() > kMaxChecks) return fail(NT_ERR_UNSUPPORTED, "lowering: too many checked coordinates");
    struct Digit { int64_t radix, off; int64_t chk[kMaxChecks]; };
    auto collect = [&](int axis, std::vector<Digit> *out) {
        for (int v : digits[axis]) {
            if (vars[v].split) continue;
            Digit d{};
            d.radix = vars[v].radix;
            for (int s = 0; s < src_.ndim; ++s) {
                auto it = lin[s].coef.find(v);
                if (it != lin[s].coef.end()) d.off += it->second * src_.stride[s];
            }
            for (size_t q = 0; q < chk_dims.size(); ++q) {
                auto it = lin[chk_dims[q]].coef.find(v);
                d.chk[q] = it != lin[chk_dims[q]].coef.end() ? it->second : 0;
            }
            out->push_back(d);
        }
        // merge neighbours that step uniformly: digit i counts radix(i+1) units of digit i+1
        for (size_t i = 0; i + 1 < out->size();) {
            Digit &a = (*out)[i], &b = (*out)[i + 1];
            bool same = a.off == b.off * b.radix;
            for (size_t q = 0; q < chk_dims.size(); ++q) same = same && a.chk[q] == b.chk[q] * b.radix;
            if (same) {
                b.radix *= a.radix;
                out->erase(out->begin() + i);
            } else {
                ++i;
            }
        }
    };
    std::vector<Digit> rd, cd, bd;
    collect(0, &rd);
    collect(1, &cd);
    collect(2, &bd);
    if (rd.empty() || cd.empty() || rd.size() > (size_t)kMaxDigits || cd.size() > (size_t)kMaxDigits)
        return fail(NT_ERR_UNSUPPORTED, "lowering: too many index digits on one axis");
    for (auto &d : bd)
        for (size_t q = 0; q < chk_dims.size(); ++q)
            if (d.chk[q]) return fail(NT_ERR_UNSUPPORTED, "lowering: batch index enters a bounds check");

    OperandMap m{};
    const int ri = rank == 3 ? 1 : 0;
    m.rows = size_[lv[ri]];
    m.cols = size_[lv[ri + 1]];
    m.nrd = (int32_t)rd.size();
    m.ncd = (int32_t)cd.size();
    m.nchk = (int32_t)chk_dims.size();
    for (int s = 0; s < src_.ndim; ++s) m.base += lin[s].c * src_.stride[s];
    auto fits = [](int64_t v) { return v >= INT32_MIN && v <= INT32_MAX; };
    for (size_t i = 0; i < rd.size(); ++i) {
        m.rrad[i] = rd[i].radix;
        m.roff[i] = rd[i].off;
        for (size_t q = 0; q < chk_dims.size(); ++q) {
            if (!fits(rd[i].chk[q])) return fail(NT_ERR_UNSUPPORTED, "lowering: coefficient overflow");
            m.rchk[q][i] = (int32_t)rd[i].chk[q];
        }
    }
    for (size_t i = 0; i < cd.size(); ++i) {
        m.crad[i] = cd[i].radix;
        m.coff[i] = cd[i].off;
        for (size_t q = 0; q < chk_dims.size(); ++q) {
            if (!fits(cd[i].chk[q])) return fail(NT_ERR_UNSUPPORTED, "lowering: coefficient overflow");
            m.cchk[q][i] = (int32_t)cd[i].chk[q];
        }
    }
    for (size_t q = 0; q < chk_dims.size(); ++q) {
        if (!fits(lin[chk_dims[q]].c) || !fits(src_.size[chk_dims[q]]))
            return fail(NT_ERR_UNSUPPORTED, "lowering: coordinate overflow");
        m.chk0[q] = (int32_t)lin[chk_dims[q]].c;
        m.chk_size[q] = (int32_t)src_.size[chk_dims[q]];
    }
    *map = m;
    if (batch_out) *batch_out = rank == 3 ? size_[lv[0]] : 1;
    if (batch_stride_out) *batch_stride_out = bd.empty() ? 0 : bd[0].off;
    return NT_OK;
}

// ------------------------------------------------- the library's own arrangements
// Section 4.2: C tiled (BM, BN); A tiled (BM, BK), its block grid re-tiled into row sets,
// repeated across C's block columns, the leftover singleton of the middle level removed;
// B mirrored.  With a leading batch dimension every tile has extent 1 along it.
nt_status arrange_matmul(const Arrangement &va, const Arrangement &vb, const Arrangement &vc,
                         nt_tile_cfg cfg, MatmulArrangement *out)
{
    if (cfg.bm <= 0 || cfg.bn <= 0 || cfg.bk <= 0) return fail(NT_ERR_INVALID_ARG, "tile sizes must be positive");
    if (va.n_levels() != 1 || vb.n_levels() != 1 || vc.n_levels() != 1)
        return fail(NT_ERR_SHAPE_MISMATCH, "matmul operands must be single-level views");
    const size_t rank = vc.level(0).size();
    if ((rank != 2 && rank != 3) || va.level(0).size() != rank || vb.level(0).size() != rank)
        return fail(NT_ERR_SHAPE_MISMATCH, "matmul operands must all be 2-D, or all 3-D with a batch dimension");
    const bool bt = rank == 3;
    const std::vector<int64_t> sa = va.level_shape(0), sb = vb.level_shape(0), sc = vc.level_shape(0);
    const size_t o = bt ? 1 : 0;
    if (sa[o + 1] != sb[o]) return fail(NT_ERR_SHAPE_MISMATCH, "inner dimensions of A and B differ");
    out->a = va;
    out->b = vb;
    out->c = vc;
    out->batched = bt;
    nt_status st;
    auto pre = [&](std::vector<int64_t> v) {
        if (bt) v.insert(v.begin(), 1);
        return v;
    };
#define NT_TRY(x) do { st = (x); if (st != NT_OK) return st; } while (0)
    // output
    NT_TRY(out->c.tile(pre({cfg.bm, cfg.bn})));
    if (bt) { NT_TRY(out->c.descend()); NT_TRY(out->c.squeeze(0)); NT_TRY(out->c.ascend()); }
    const std::vector<int64_t> grid = out->c.level_shape(0);
    const int64_t Mt = grid[o], Nt = grid[o + 1];
    // input
    NT_TRY(out->a.tile(pre({cfg.bm, cfg.bk})));
    NT_TRY(out->a.tile(pre({1, -1})));
    NT_TRY(out->a.expand(bt ? std::vector<int64_t>{-1, -1, Nt} : std::vector<int64_t>{-1, Nt}));
    NT_TRY(out->a.descend());
    if (bt) NT_TRY(out->a.squeeze(0));
    NT_TRY(out->a.squeeze(0));
    if (bt) { NT_TRY(out->a.descend()); NT_TRY(out->a.squeeze(0)); NT_TRY(out->a.ascend()); }
    NT_TRY(out->a.ascend());
    // other
    NT_TRY(out->b.tile(pre({cfg.bk, cfg.bn})));
    NT_TRY(out->b.tile(pre({-1, 1})));
    NT_TRY(out->b.expand(bt ? std::vector<int64_t>{-1, Mt, -1} : std::vector<int64_t>{Mt, -1}));
    NT_TRY(out->b.descend());
    if (bt) NT_TRY(out->b.squeeze(0));
    NT_TRY(out->b.squeeze(1));
    if (bt) { NT_TRY(out->b.descend()); NT_TRY(out->b.squeeze(0)); NT_TRY(out->b.ascend()); }
    NT_TRY(out->b.ascend());
#undef NT_TRY
    // tile-to-program mapping: the three outermost shapes must agree (Section 3.2.1)
    if (out->a.level_shape(0) != grid || out->b.level_shape(0) != grid) {
        std::ostringstream os;
        os << "outermost shapes of the arranged operands differ (A/B/C grids)";
        return fail(NT_ERR_SHAPE_MISMATCH, os.str());
    }
    if (out->a.level_shape(1) != out->b.level_shape(1))
        return fail(NT_ERR_SHAPE_MISMATCH, "A and B disagree on the number of k tiles");
    out->batch = bt ? grid[0] : 1;
    out->mt = Mt;
    out->nt = Nt;
    out->kt = out->a.level_shape(1)[0];
    return NT_OK;
}

// Section 4.3: input tiled by (1, C, R, S) with unit strides along H and W (the conv
// stride in general), singleton dimensions squeezed, levels ravelled to (N,P,Q,C,R,S) and
// flattened to (N*P*Q, C*R*S); filter flattened and transposed to (C*R*S, K); output
// permuted and flattened to (N*P*Q, K).
nt_status conv2d_views(const nt_tensor_desc *dx, const nt_tensor_desc *dw, const nt_tensor_desc *dy,
                       int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                       Arrangement *vx, Arrangement *vw, Arrangement *vy, int32_t dh, int32_t dw_)
{
    if (!dx || !dw || !dy) return fail(NT_ERR_INVALID_ARG, "null tensor descriptor");
    if (dx->ndim != 4 || dw->ndim != 4 || dy->ndim != 4)
        return fail(NT_ERR_SHAPE_MISMATCH, "conv2d tensors must be 4-D (NCHW, KCRS, NKPQ)");
    if (sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw_ < 1) return fail(NT_ERR_INVALID_ARG, "conv2d stride and dilation must be >= 1, padding >= 0");
    const int64_t N = dx->size[0], C = dx->size[1], H = dx->size[2], W = dx->size[3];
    const int64_t K = dw->size[0], R = dw->size[2], S = dw->size[3];
    if (dw->size[1] != C) return fail(NT_ERR_SHAPE_MISMATCH, "conv2d: channel counts of input and filter differ");
    if (R < 1 || S < 1 || C < 1) return fail(NT_ERR_INVALID_ARG, "conv2d: empty filter");
    const int64_t span_h = (R - 1) * dh + 1, span_w = (S - 1) * dw_ + 1;      // input rows / columns under one filter
    const int64_t P = H + 2 * ph >= span_h ? (H + 2 * ph - span_h) / sh + 1 : 0;
    const int64_t Q = W + 2 * pw >= span_w ? (W + 2 * pw - span_w) / sw + 1 : 0;
    if (dy->size[0] != N || dy->size[1] != K || dy->size[2] != P || dy->size[3] != Q) {
        std::ostringstream os;
        os << "conv2d: output must be [" << N << "," << K << "," << P << "," << Q << "]";
        return fail(NT_ERR_SHAPE_MISMATCH, os.str());
    }
    nt_status st;
#define NT_TRY(x) do { st = (x); if (st != NT_OK) return st; } while (0)
    NT_TRY(vx->init(dx));
    NT_TRY(vw->init(dw));
    NT_TRY(vy->init(dy));
    const int64_t hi_h = (P - 1) * sh + span_h - H - ph, hi_w = (Q - 1) * sw + span_w - W - pw;
    NT_TRY(vx->tile({1, C, R, S}, {-1, -1, sh, sw}, {0, 0, ph, pw}, {0, 0, hi_h, hi_w}, {1, 1, dh, dw_}));
    NT_TRY(vx->squeeze(1));
    NT_TRY(vx->descend());
    NT_TRY(vx->squeeze(0));
    NT_TRY(vx->ascend());
    NT_TRY(vx->ravel());
    NT_TRY(vx->flatten(0, 3));
    NT_TRY(vx->flatten(1, 4));
    NT_TRY(vw->flatten(1, 4));
    NT_TRY(vw->permute({1, 0}));
    NT_TRY(vy->permute({0, 2, 3, 1}));
    NT_TRY(vy->flatten(0, 3));
#undef NT_TRY
    return NT_OK;
}

}  // namespace nt
