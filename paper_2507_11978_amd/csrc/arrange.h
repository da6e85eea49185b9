// Host-side arrangement engine: hierarchical tensors as a dataflow graph of index nodes.
//
// A hierarchical tensor (Section 3.1.2) is a list of levels, each a list of dimension
// ids.  Every meta-operation (Table 1) adds nodes that say how the index of an older
// dimension is obtained from the indices of newer ones:
//   TILE   parent = outer * stride + inner - pad_lo, valid iff 0 <= parent < parent size
//   ZERO   parent = 0               (a squeezed or expanded singleton)
//   SPLIT  parents = mixed-radix digits of the merged index (flatten), first slowest
// Evaluating the nodes newest-to-oldest turns one index per current dimension into source
// coordinates and a mask (the source-to-target mapping, Section 3.2.2).  The same graph is
// evaluated symbolically to lower a 2-D (or batched 3-D) matrix view into the digit/affine
// form the device address generator consumes.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/nt.h"
#include "opmap.h"

namespace nt {

void set_error(const std::string &msg);
nt_status fail(nt_status st, const std::string &msg);

struct Node {
    enum Kind { TILE, ZERO, SPLIT } kind;
    int in0 = -1, in1 = -1;          // TILE: outer, inner.  SPLIT: merged.  ZERO: unused
    int out[NT_MAX_DIMS];            // TILE/ZERO: one parent.  SPLIT: nout parents
    int nout = 0;
    int64_t st = 1, lo = 0, bound = 0, dil = 1;     // TILE: parent = outer * st + inner * dil - lo, valid in [0, bound)
    int64_t radix[NT_MAX_DIMS];
};

class Arrangement {
public:
    nt_status init(const nt_tensor_desc *src);
    nt_status apply(const nt_meta_op &op);
    nt_status apply_all(const nt_meta_op *ops, int32_t n_ops);

    // convenience builders used by the library's own arrangements
    nt_status tile(std::vector<int64_t> shape, std::vector<int64_t> strides = {},
                   std::vector<int64_t> pad_lo = {}, std::vector<int64_t> pad_hi = {}, std::vector<int64_t> dilation = {});
    nt_status expand(std::vector<int64_t> shape);
    nt_status squeeze(int64_t dim);
    nt_status permute(std::vector<int64_t> order);
    nt_status flatten(int64_t start, int64_t end);
    nt_status ravel();
    nt_status descend();
    nt_status ascend();

    int n_levels() const { return (int)levels_.size(); }
    const std::vector<int> &level(int l) const { return levels_[l]; }
    int64_t dim_size(int id) const { return size_[id]; }
    std::vector<int64_t> level_shape(int l) const;
    int64_t num_programs() const;

    // One tile: offsets (-1 where masked) and masks, row-major over the innermost level.
    nt_status tile_index_set(int64_t program_id, const int64_t *mid_idx, int32_t n_mid,
                             int64_t *offsets_out, uint8_t *mask_out, size_t capacity,
                             int64_t *tile_shape_out, int32_t *tile_ndim_out,
                             int64_t *grid_shape_out, int32_t *grid_ndim_out) const;

    // Lower a single-level view of rank 2 ([rows, cols]) or 3 ([batch, rows, cols]) to the
    // device operand map.  batch_stride_out receives the batch dimension's offset step.
    nt_status lower_matrix_view(OperandMap *map, int64_t *batch_out, int64_t *batch_stride_out) const;

private:
    bool eval(std::vector<int64_t> &vals, int64_t *offset) const;
    nt_tensor_desc src_;
    std::vector<int64_t> size_;             // size of every dimension ever created
    std::vector<Node> nodes_;
    std::vector<std::vector<int>> levels_;
    int cursor_ = 0;
};

// The library's own arrangements (the ones the kernels execute).
struct MatmulArrangement {
    Arrangement a, b, c;
    int64_t batch = 1, mt = 0, nt = 0, kt = 0;
    bool batched = false;
};
nt_status arrange_matmul(const Arrangement &va, const Arrangement &vb, const Arrangement &vc,
                         nt_tile_cfg cfg, MatmulArrangement *out);
nt_status conv2d_views(const nt_tensor_desc *dx, const nt_tensor_desc *dw, const nt_tensor_desc *dy,
                       int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                       Arrangement *vx, Arrangement *vw, Arrangement *vy, int32_t dh = 1, int32_t dw_ = 1);

}  // namespace nt
