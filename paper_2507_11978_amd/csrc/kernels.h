// Launch interface between the C ABI layer and the HIP kernels (host side).
#pragma once
#include <cstdint>
#include <string>

#include "../../include/nt.h"
#include "opmap.h"

namespace nt {

nt_status fail(nt_status st, const std::string &msg);   // records the thread-local error text

// What nt_conv2d_implicit was called with (strides in elements), so that the dense case can be
// given to the convolution kernel; the lowered operand maps describe the same operands.
struct ConvHint {
    bool valid;
    int64_t N, C, H, W, K, R, S, P, Q, sh, sw, ph, pw;
    int64_t dh, dw;                 // dilation (1 unless the views say otherwise)
    int64_t xs[4], ws[4], ys[4];
};

// Request for a loader trace instead of a product (nt_trace_loader_slice); out == nullptr: none.
struct LoaderTrace {
    uint16_t *out;
    size_t capacity;
    int64_t program;
    int32_t slice, operand;
};

struct GemmLaunch {
    const void *A;
    const void *B;
    void *C;
    OperandMap ma, mb, mc;            // lowered operand maps (rows x cols views)
    int64_t batch;                    // number of batch entries (1 for gemm / conv)
    int64_t sa_batch, sb_batch, sc_batch;
    int64_t M, N, K;
    int64_t mt, nt, kt;               // grid of programs and k tiles (from the arrangement)
    nt_tile_cfg tile;
    int in_dtype, out_dtype;
    void *stream;
    // epilogue: C = alpha * (A . B) + beta * D; D (elements of out_dtype, map md) is read only if has_d
    const void *D;
    OperandMap md;
    int64_t sd_batch;
    float alpha, beta;
    int act;                                // activation of the combined value (nt_activation)
    bool has_d;
    ConvHint conv;
    bool user_tile;                         // the caller named the tile (then the kernels the library would prefer are not substituted)
    bool no_workspace;                      // the library's workspace is in use by the caller of this launch, or must not be touched: a k split only
    float *ws_given;                        // inside the region the caller has set aside for it (ws_given_bytes; may be none)
    size_t ws_given_bytes;
    bool ws_strict;                         // a k split that would need more than ws_given_bytes is an error (else: run unsplit)
    LoaderTrace trace;
};

// Which code path a launch would take (reported for tests and the benchmark).
enum KernelPath { PATH_GENERIC = 0, PATH_FAST = 1, PATH_DIRECT = 2, PATH_CONV = 3, PATH_CONV_DIRECT = 4, PATH_CONV_UNFOLD = 5, PATH_CONV_TAP = 6 };

bool tile_is_built(nt_tile_cfg cfg);
// into how many parts the calling thread's last launch_gemm split its reduction (1: no split)
int last_k_split();
// the tile the MFMA kernels run a plain (batched) product of this size fastest with, by a cost model fitted to measurements
nt_tile_cfg pick_gemm_tile(int64_t batch, int64_t M, int64_t N, int64_t K);
// the tile of a dense unit-stride convolution (M positions, N filters, reduction K), by an estimate that includes the k split
nt_tile_cfg pick_conv_tile(int64_t M, int64_t N, int64_t K);
nt_status launch_gemm(const GemmLaunch &g, int *path_out);
// device address and size of the fixed scratch array of the entry point that allocates nothing (this device's copy)
nt_status static_scratch(void **ptr_out, size_t *bytes_out);
nt_status launch_fill_zero(void *C, const OperandMap &mc, int64_t batch, int64_t sc_batch, int out_dtype, void *stream);
nt_status launch_trace(const OperandMap &m, int64_t batch_off, int64_t row0, int64_t col0, int32_t rows, int32_t cols,
                       int64_t *offsets_out, uint8_t *mask_out, void *stream);

// matrix-instruction-only loop on the caller's operand data (a measurement aid, see nt_mfma_probe)
nt_status launch_mfma_probe(const void *data, int64_t n_elems, int dtype, int32_t iters, int32_t blocks, float *out, void *stream);

// memory-bound kernels: op 0 = add (x + y), 1 = silu (y unused); strides in elements
nt_status launch_map(int op, const void *x, int64_t sx, const void *y, int64_t sy, void *out, int64_t so, int64_t n, int dtype, void *stream);
// row-wise kernels: op 0 = softmax, 1 = rms_norm (eps used)
nt_status launch_rows(int op, const void *x, int64_t sxr, int64_t sxc, void *out, int64_t sor, int64_t soc, int64_t rows, int64_t cols,
                      float eps, int dtype, void *stream);

// scaled dot-product attention over [batch, heads, seq, 64] tensors (strides in elements, unit stride along the head dimension)
nt_status launch_sdpa_desc(const void *q, const nt_tensor_desc *dq, const void *k, const nt_tensor_desc *dk,
                           const void *v, const nt_tensor_desc *dv, void *o, const nt_tensor_desc *dout,
                           float scale, int dtype, void *stream);

// workgroup index -> logical program id (shared by host query and device code)
// Position seq of the tile sequence -> program id: the grid is walked in bands of up to 8 tile
// rows, column by column inside a band, so that programs that run at the same time share operand
// rows / columns.
// (I: int64_t on the host; uint32_t in the kernels, whose launchers have checked that every count is below 2^31 -- a
// 64-bit division costs a wavefront some hundred instructions, and a program's start has eight of them)
template <typename I>
NT_HD I program_of_sequence_t(I seq, I mt, I nt)
{
    const I band = 8;
    const I per_band = band * nt;
    const I b = seq / per_band;
    const I first = b * band;
    const I rows = mt - first < band ? mt - first : band;
    const I in = seq - b * per_band;
    const I j = in / rows;
    const I i = first + (in - j * rows);
    return i * nt + j;
}
NT_HD int64_t program_of_sequence(int64_t seq, int64_t mt, int64_t nt) { return program_of_sequence_t<int64_t>(seq, mt, nt); }

template <typename I>
NT_HD I program_of_workgroup_t(I w, I mt, I nt)
{
    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD one contiguous share of
    // the tile sequence so that tiles resident on one L2 share operand rows / columns.
    const I G = mt * nt;
    const I nx = 8;
    const I q = G / nx, r = G % nx;          // first r XCDs get q+1 tiles
    const I x = w % nx, l = w / nx;
    const I seq = x < r ? x * (q + 1) + l : r * (q + 1) + (x - r) * q + l;
    return program_of_sequence_t<I>(seq, mt, nt);
}
NT_HD int64_t program_of_workgroup(int64_t w, int64_t mt, int64_t nt) { return program_of_workgroup_t<int64_t>(w, mt, nt); }

// Batched grids (nb problems of mt x nt programs): every complete group of 8 problems is dealt out
// one whole problem per XCD (its operands then pass through one L2 only); the problems left over are
// split across the XCDs like a single problem.
template <typename I>
NT_HD void program_of_workgroup_batched_t(I w, I nb, I mt, I nt, I *b, I *pid)
{
    const I per = mt * nt;
    if (w < (nb / 8) * 8 * per) {
        const I l = w / 8;
        const I grp = l / per;
        *b = grp * 8 + w % 8;
        *pid = program_of_sequence_t<I>(l - grp * per, mt, nt);
    } else {
        const I bb = w / per;
        *b = bb;
        *pid = program_of_workgroup_t<I>(w - bb * per, mt, nt);
    }
}
NT_HD void program_of_workgroup_batched(int64_t w, int64_t nb, int64_t mt, int64_t nt, int64_t *b, int64_t *pid)
{
    program_of_workgroup_batched_t<int64_t>(w, nb, mt, nt, b, pid);
}

}  // namespace nt
