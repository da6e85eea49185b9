/*
 * nt.h -- C ABI of the MI355X (gfx950) arrange-and-apply tiled-contraction library.
 *
 * The library implements the tiled computation that the paper's code generator emits
 * for its canonical arrangement: a matrix multiply whose output tiles are programs
 * (tile-to-program mapping, Section 3.2.1) and whose operand tiles are located through
 * per-program index sets (source-to-target mapping, Section 3.2.2), plus batched matmul
 * and 2D convolution lowered to the same product (Section 4.3).
 *
 * Conventions for every entry point
 *   - Plain C types only.  "device" pointers are HIP device addresses (for example
 *     torch.Tensor.data_ptr()); "host" pointers are ordinary process memory.
 *   - Strides are in ELEMENTS, not bytes, and may describe any non-overlapping view.
 *   - The caller owns every buffer it passes.  The library keeps one thing between calls: a workspace of 256 MB
 *     per GPU, allocated by the first call on that GPU that needs one (see "Memory" at nt_gemm and
 *     nt_conv2d_implicit) and kept, never moved, until the process ends.  Calls that need it while another call's
 *     work on it is still queued -- from other host threads or on other streams of the same GPU -- wait their turn:
 *     the later call's stream waits (on the device, through an event) for the earlier call's last kernel that
 *     touches the workspace.  Results never depend on what other calls do.
 *   - Kernel-launching calls enqueue on `hip_stream` (a hipStream_t, NULL = default
 *     stream) and return without waiting.  nt_arrange_* calls are synchronous host code.
 *   - Errors are returned as nt_status; nothing throws or aborts across the ABI.
 *     nt_last_error() gives a thread-local message for the last failing call.
 */
#ifndef NT_H
#define NT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NT_MAX_DIMS 8
#define NT_MAX_LEVELS 8

typedef enum {
    NT_OK = 0,
    NT_ERR_INVALID_ARG = 1,      /* null pointer, ndim out of range, negative size, bad enum */
    NT_ERR_SHAPE_MISMATCH = 2,   /* improper arrangement (Section 3.2.1), K mismatch, expand/squeeze of non-singleton */
    NT_ERR_UNSUPPORTED = 3,      /* dtype / tile combination that is not built */
    NT_ERR_BUFFER_TOO_SMALL = 4, /* `capacity` smaller than the tile; required size is still reported */
    NT_ERR_DEVICE = 5            /* HIP runtime error (launch failure, no device) */
} nt_status;

typedef enum { NT_F16 = 0, NT_BF16 = 1, NT_F32 = 2 } nt_dtype;

/* A source tensor: sizes and element strides, as a framework front end reports them
 * (Section 3.2.1, last paragraph). */
typedef struct {
    int32_t ndim;
    int64_t size[NT_MAX_DIMS];
    int64_t stride[NT_MAX_DIMS];
} nt_tensor_desc;

/* One meta-operation (Table 1).  An arrangement is an array of these, applied in order
 * to the level the cursor points at (initially the outermost).
 *   TILE     a = tile shape (-1 = whole dimension), b = strides between tiles (-1 or 0 =
 *            default = tile shape; Section 3.1.3), c = low padding, d = high padding,
 *            e = dilation (-1, 0 or 1 = none): element j of tile o is source coordinate
 *            o * b + j * e - c.  (c, d, e: 0 / none in the paper; needed for padded and
 *            dilated convolutions.)  n = rank.
 *   EXPAND   a = new shape (-1 keeps a dimension); only singleton dimensions grow.
 *   SQUEEZE  a[0] = dimension to drop; it must have size 1.
 *   PERMUTE  a = order (new dimension i is old dimension a[i]).
 *   FLATTEN  a[0] = start_dim, a[1] = end_dim, EXCLUSIVE (the shapes printed in Section
 *            4.3 require it), first merged dimension slowest.
 *   RAVEL    concatenates all levels from the cursor inwards into one level.
 *   DESCEND  move the cursor one level inwards (the paper's `.dtype`).
 *   ASCEND   move it back out (assigning the edited `.dtype` back).
 */
typedef enum {
    NT_OP_TILE = 0, NT_OP_EXPAND = 1, NT_OP_SQUEEZE = 2, NT_OP_PERMUTE = 3,
    NT_OP_FLATTEN = 4, NT_OP_RAVEL = 5, NT_OP_DESCEND = 6, NT_OP_ASCEND = 7
} nt_op_kind;

typedef struct {
    int32_t kind;               /* nt_op_kind */
    int32_t n;                  /* number of valid entries in a/b/c/d */
    int64_t a[NT_MAX_DIMS];
    int64_t b[NT_MAX_DIMS];
    int64_t c[NT_MAX_DIMS];
    int64_t d[NT_MAX_DIMS];
    int64_t e[NT_MAX_DIMS];
} nt_meta_op;

/* Meta-parameters of the matmul arrangement (BLOCK_SIZE_M/N/K of Section 4.2).
 * 0 in all three = library default for the problem.  Built tiles: see nt_tile_supported. */
typedef struct { int32_t bm, bn, bk; } nt_tile_cfg;

/* Operand selector for the *_arrange_tile calls. */
typedef enum { NT_OPERAND_A = 0, NT_OPERAND_B = 1, NT_OPERAND_C = 2 } nt_operand;

/* ---------------------------------------------------------------- arrangement (host, integer)
 *
 * nt_arrange_levels: run `ops` on `src` and report the resulting hierarchy
 * (Section 3.1.2): n_levels_out, and for level l its rank level_ndim_out[l] and shape
 * level_shape_out[l*NT_MAX_DIMS + d].  Arrays must hold NT_MAX_LEVELS (x NT_MAX_DIMS).
 */
nt_status nt_arrange_levels(const nt_tensor_desc *src, const nt_meta_op *ops, int32_t n_ops,
                            int32_t *n_levels_out, int32_t *level_ndim_out, int64_t *level_shape_out);

/*
 * nt_arrange_tile: the source-to-target map of one tile (Section 3.2.2).  `program_id`
 * selects the outermost index (row-major, last dimension fastest -- the paper fixes only
 * the number of programs, Section 3.2.1); `mid_idx[n_mid]` indexes every dimension of the
 * levels strictly between outermost and innermost (e.g. {k} for a matmul operand).  Writes,
 * in row-major order over the innermost level, the element offset into the source
 * (-1 where masked) and the mask (1 valid, 0 masked; masked loads read as zero, masked
 * stores are dropped).  offsets_out / mask_out are host arrays of `capacity` entries;
 * if the tile is larger, nothing is written to them, NT_ERR_BUFFER_TOO_SMALL is returned
 * and the shapes are still reported.  tile_shape_out / grid_shape_out hold NT_MAX_DIMS
 * entries.  Any of the *_out pointers except the shape outputs may be NULL to query shapes.
 */
nt_status nt_arrange_tile(const nt_tensor_desc *src, const nt_meta_op *ops, int32_t n_ops,
                          int64_t program_id, const int64_t *mid_idx, int32_t n_mid,
                          int64_t *offsets_out, uint8_t *mask_out, size_t capacity,
                          int64_t *tile_shape_out, int32_t *tile_ndim_out,
                          int64_t *grid_shape_out, int32_t *grid_ndim_out);

/*
 * The matmul arrangement of Section 4.2 applied to A [M,K], B [K,N], C [M,N]
 * (nt_arrange_gemm), to [batch,M,K] x [batch,K,N] -> [batch,M,N] (nt_arrange_bmm; the
 * paper does not print this arrangement: the matmul one with a leading batch dimension
 * tiled by 1 is used) and to the implicit-GEMM view of a convolution (nt_arrange_conv2d,
 * Section 4.3: input NCHW, filter KCRS, output NKPQ).  Each checks that the three
 * outermost shapes agree (else NT_ERR_SHAPE_MISMATCH, Section 3.2.1) and reports the grid
 * (grid_out[3] = {batch or 1, Mt, Nt}) and the number of k tiles.  With operand/program_id/k
 * and non-NULL offsets_out they also evaluate that operand's tile exactly like
 * nt_arrange_tile (tile_shape_out[2]).  These are the arrangements the kernels execute.
 */
nt_status nt_arrange_gemm(const nt_tensor_desc *dA, const nt_tensor_desc *dB, const nt_tensor_desc *dC,
                          nt_tile_cfg cfg, int64_t *grid_out, int64_t *kt_out,
                          int32_t operand, int64_t program_id, int64_t k,
                          int64_t *offsets_out, uint8_t *mask_out, size_t capacity, int64_t *tile_shape_out);
nt_status nt_arrange_bmm(const nt_tensor_desc *dA, const nt_tensor_desc *dB, const nt_tensor_desc *dC,
                         nt_tile_cfg cfg, int64_t *grid_out, int64_t *kt_out,
                         int32_t operand, int64_t program_id, int64_t k,
                         int64_t *offsets_out, uint8_t *mask_out, size_t capacity, int64_t *tile_shape_out);
nt_status nt_arrange_conv2d(const nt_tensor_desc *dx, const nt_tensor_desc *dw, const nt_tensor_desc *dy,
                            int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                            nt_tile_cfg cfg, int64_t *grid_out, int64_t *kt_out,
                            int32_t operand, int64_t program_id, int64_t k,
                            int64_t *offsets_out, uint8_t *mask_out, size_t capacity, int64_t *tile_shape_out);

/*
 * nt_program_order: the permutation the kernels apply between the hardware workgroup
 * index and the logical program id (cache-locality swizzle; any bijection yields the same
 * result because programs are independent, Section 3.2.1).  Writes pid_out[w] for
 * w in [0, batch*mt*nt).  Host arrays.
 */
nt_status nt_program_order(int64_t batch, int64_t mt, int64_t nt, int64_t *pid_out);

/* Which kernel the calling thread's last nt_gemm / nt_addmm / nt_addmm_act / nt_bmm / nt_conv2d_implicit call launched:
 * 0 operand-map (generic) kernel, 1 staged kernel, 2 direct-to-LDS kernel, 3 convolution kernel (operands staged
 * through registers), 4 convolution kernel (operands streamed straight into LDS), 5 unfolded input written to the
 * workspace + the matrix kernels, 6 convolution kernel that streams into LDS and walks the reduction filter tap by filter
 * tap (256 filters per program, channels in whole blocks of 32; reads a tap-major copy of the filter that it puts in the
 * workspace),
 * -1 none (nothing launched yet, an error, or an empty problem).  For tests and diagnostics. */
int32_t nt_last_kernel_path(void);

/* Into how many parts the reduction of that call was split (see "Memory" at nt_gemm and nt_conv2d_implicit); 1: not split.
 * For tests and diagnostics. */
int32_t nt_last_k_split(void);

/* 1 if kernels for this (bm, bn, bk) are built, else 0.  (0,0,0) is always supported. */
int32_t nt_tile_supported(nt_tile_cfg cfg);

/* ------------------------------------------------------------------------- kernels (device)
 *
 * nt_gemm: C[M,N] = A[M,K] . B[K,N]  -- the matmul application of Section 4.2 run over the
 * arrangement above: fp32 accumulator, one dot per k tile, store converted to out_dtype
 * (round to nearest even).  A, B, C are device pointers; descriptors are host structs
 * with ndim 2.  in_dtype is NT_F16 or NT_BF16; out_dtype NT_F16, NT_BF16 or NT_F32.
 * Any strides are accepted; unit-stride operands with 16-byte aligned rows take the
 * fastest path.  M or N of 0: nothing is launched.  K of 0: C is zero-filled.
 * C must not alias A or B.
 * Memory (nt_gemm, nt_addmm, nt_addmm_act): a product with few output tiles and a long reduction (a skinny
 * product such as 16 x 4096 x 4096) has K dealt to several programs per tile; their fp32 partial tiles go
 * through the library's workspace, the same one, under the same rules, as described at nt_conv2d_implicit
 * (one allocation of 256 MB per GPU, made by the first call that needs it, handed from call to call in stream
 * order; partial tiles added in a fixed order).
 */
nt_status nt_gemm(const void *A, const nt_tensor_desc *dA, const void *B, const nt_tensor_desc *dB,
                  void *C, const nt_tensor_desc *dC, nt_dtype in_dtype, nt_dtype out_dtype,
                  nt_tile_cfg cfg, void *hip_stream);

/* nt_gemm_noalloc: nt_gemm for callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results bit for bit; it calls
 * no hipMalloc / hipFree and never touches the library's workspace.  The k split of a skinny product puts its fp32
 * partial tiles into a fixed array of NT_NOALLOC_SCRATCH_BYTES inside the library's device image instead (every GPU
 * the library is loaded on holds its own copy from load time until the process ends).  A product whose split needs
 * more (parts x M x N x 4 bytes) is refused with NT_ERR_UNSUPPORTED and a message that names both sizes; nothing is
 * launched then.  Every call on a GPU shares that GPU's array and nothing orders them: calls that overlap on one
 * GPU (different streams or host threads, both splitting) race on it -- keep them on one stream.  The array needs no
 * clearing between calls: every part writes its whole slice before the sum reads it. */
#define NT_NOALLOC_SCRATCH_BYTES (32u << 20)
nt_status nt_gemm_noalloc(const void *A, const nt_tensor_desc *dA, const void *B, const nt_tensor_desc *dB,
                          void *C, const nt_tensor_desc *dC, nt_dtype in_dtype, nt_dtype out_dtype,
                          nt_tile_cfg cfg, void *hip_stream);

/* nt_addmm: C[M,N] = beta * input[M,N] + alpha * (A[M,K] . B[K,N])  -- the addmm kernel of the paper's
 * task list (Section 5.1): the matmul arrangement and application of Section 4.2 with `input` arranged
 * like the output (tile(BM, BN)) and combined with the accumulator in fp32 before the one conversion to
 * out_dtype.  `input` is a device pointer to elements of out_dtype, described by a host struct with
 * ndim 2 and the sizes of C; a stride of 0 broadcasts (a bias row is {0, 1}).  beta == 0 leaves `input`
 * unread (it may then be NULL).  K of 0: C = beta * input.  Everything else as nt_gemm.  C may alias
 * `input` only if both have identical descriptors (each element is read before it is written).
 */
nt_status nt_addmm(const void *input, const nt_tensor_desc *dI, const void *A, const nt_tensor_desc *dA,
                   const void *B, const nt_tensor_desc *dB, void *C, const nt_tensor_desc *dC,
                   float alpha, float beta, nt_dtype in_dtype, nt_dtype out_dtype,
                   nt_tile_cfg cfg, void *hip_stream);

/* nt_addmm_act: C = act(beta * input + alpha * (A . B))  -- nt_addmm with an activation fused into the
 * epilogue (bias + activation in one pass over the accumulators; the paper's generated kernels fuse
 * their whole application into one kernel in the same way, Section 3.2).  The activation acts on the fp32
 * combined value, before the one conversion to out_dtype:
 *   NT_ACT_NONE       x
 *   NT_ACT_RELU       max(x, 0)
 *   NT_ACT_SILU       x / (1 + exp(-x))
 *   NT_ACT_GELU_TANH  0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))
 * `input` / dI may be NULL when beta == 0 (then C = act(alpha * A . B)).  Everything else as nt_addmm.
 * NT_ACT_RELU maps a NaN to 0 (the hardware maximum returns its number operand); the others propagate it.
 */
typedef enum { NT_ACT_NONE = 0, NT_ACT_RELU = 1, NT_ACT_SILU = 2, NT_ACT_GELU_TANH = 3 } nt_activation;
nt_status nt_addmm_act(const void *input, const nt_tensor_desc *dI, const void *A, const nt_tensor_desc *dA,
                       const void *B, const nt_tensor_desc *dB, void *C, const nt_tensor_desc *dC,
                       float alpha, float beta, nt_activation act, nt_dtype in_dtype, nt_dtype out_dtype,
                       nt_tile_cfg cfg, void *hip_stream);

/* ------------------------------------------------------------------ memory-bound kernels (device)
 *
 * The element-wise and row-wise kernels of the paper's task list (Section 5.1).  x, y, out are device
 * pointers to 16-bit elements of `dtype` (NT_F16 or NT_BF16, the same for inputs and output);
 * descriptors are host structs, strides in elements, any strides accepted (unit strides take the
 * vector path).  Arithmetic is fp32 with one round-to-nearest-even conversion of the result.
 * `out` may alias an input only with an identical descriptor.  Empty tensors: nothing is launched.
 *
 * nt_add: out[i] = x[i] + y[i] over 1-D tensors of equal size -- vector addition as arranged in
 * Section 4.1: each vector tiled into blocks (`tile((BLOCK_SIZE,))`), application
 * `output = input + other`.  block_size is that meta-parameter (0 = 1024, the paper's value; it
 * must be positive otherwise); the result does not depend on it (nt_arrange_tile with one TILE
 * operation gives the blocks' index sets).  Sizes that differ: NT_ERR_SHAPE_MISMATCH.
 */
nt_status nt_add(const void *x, const nt_tensor_desc *dx, const void *y, const nt_tensor_desc *dy,
                 void *out, const nt_tensor_desc *dout, nt_dtype dtype, int64_t block_size, void *hip_stream);

/* nt_silu: out[i] = x[i] / (1 + exp(-x[i])), arranged like nt_add. */
nt_status nt_silu(const void *x, const nt_tensor_desc *dx, void *out, const nt_tensor_desc *dout,
                  nt_dtype dtype, int64_t block_size, void *hip_stream);

/* nt_softmax: softmax along the last axis of a 2-D tensor [rows, cols]; each row is one program
 * (`tile((1, -1))`): out[r, c] = exp(x[r, c] - max_c x[r, :]) / sum_c exp(x[r, c] - max_c x[r, :]). */
nt_status nt_softmax(const void *x, const nt_tensor_desc *dx, void *out, const nt_tensor_desc *dout,
                     nt_dtype dtype, void *hip_stream);

/* nt_rms_norm: out[r, c] = x[r, c] / sqrt(mean_c x[r, :]^2 + eps) along the last axis of a 2-D tensor,
 * without a weight (the task takes one tensor), rows arranged as in nt_softmax.  eps >= 0. */
nt_status nt_rms_norm(const void *x, const nt_tensor_desc *dx, void *out, const nt_tensor_desc *dout,
                      float eps, nt_dtype dtype, void *hip_stream);

/* nt_matmul_views: the matmul arrangement and application of Section 4.2 over operands that are
 * themselves arranged tensors -- the way Section 4.3 builds a convolution: each operand is a tensor
 * plus a meta-operation program (Table 1; same encoding as nt_arrange_tile) that must end in a single
 * level of rank 2 ([rows, cols]) or, for all three, rank 3 ([batch, rows, cols]).  C_view = A_view . B_view,
 * where elements of A_view / B_view that fall outside their tensor (padding, ragged tiles) read as zero
 * and elements of C_view outside C are dropped.  C_view must not address an element of C twice.  The
 * operands may use any composition of tile (with strides and padding), expand, squeeze, permute,
 * flatten, ravel and level navigation; the lowered views drive the operand-map kernel, and views that
 * reduce to plain strided matrices take the kernels of nt_gemm / nt_bmm.  Errors as nt_arrange_tile and
 * nt_gemm.  (n_ops = 0: the tensor itself is the view.)
 */
nt_status nt_matmul_views(const void *A, const nt_tensor_desc *dA, const nt_meta_op *opsA, int32_t nA,
                          const void *B, const nt_tensor_desc *dB, const nt_meta_op *opsB, int32_t nB,
                          void *C, const nt_tensor_desc *dC, const nt_meta_op *opsC, int32_t nC,
                          nt_dtype in_dtype, nt_dtype out_dtype, nt_tile_cfg cfg, void *hip_stream);

/* nt_sdpa: scaled dot-product attention, O[b,h,i,:] = sum_j softmax_j(scale * <Q[b,h,i,:], K[b,h,j,:]>) V[b,h,j,:]
 * (no mask, no dropout), computed with the FlashAttention-2 scheme the paper's sdpa kernels use (Section 5.1):
 * Q and O tiled into blocks of query rows (one program per batch, head and block), K and V into blocks of keys
 * that every program visits in turn with a running maximum and sum; scores and sums in fp32, the probabilities
 * rounded to the 16-bit format before they multiply V.  All four tensors are device pointers to 16-bit elements
 * of `dtype` (NT_F16 or NT_BF16) with descriptors [batch, heads, seq, 64]: any strides along the first three axes,
 * unit stride along the last; other head sizes: NT_ERR_UNSUPPORTED.  K and V share their sequence length (>= 1),
 * Q and O theirs.  scale = 0 stands for 1 / sqrt(64).  O must not alias an input.
 */
nt_status nt_sdpa(const void *q, const nt_tensor_desc *dq, const void *k, const nt_tensor_desc *dk,
                  const void *v, const nt_tensor_desc *dv, void *o, const nt_tensor_desc *dout,
                  float scale, nt_dtype dtype, void *hip_stream);

/* nt_bmm: the same per batch index; descriptors have ndim 3: [batch,M,K], [batch,K,N], [batch,M,N]
 * (listed among the paper's kernels in Section 5.1). */
nt_status nt_bmm(const void *A, const nt_tensor_desc *dA, const void *B, const nt_tensor_desc *dB,
                 void *C, const nt_tensor_desc *dC, nt_dtype in_dtype, nt_dtype out_dtype,
                 nt_tile_cfg cfg, void *hip_stream);

/*
 * nt_conv2d_implicit: y[N,K,P,Q] = cross-correlation of x[N,C,H,W] with w[K,C,R,S]
 * (Section 4.3), computed as the matmul (N*P*Q, C*R*S) x (C*R*S, K) without materialising
 * the unfolded input: the input tile is gathered through the arrangement's index map,
 * out-of-image positions (padding) read as zero.  dy must have P = (H + 2*pad_h - R) /
 * stride_h + 1 (integer division), likewise Q; otherwise NT_ERR_SHAPE_MISMATCH.
 * Descriptors have ndim 4 with arbitrary strides.
 * Dense unit-stride calls (contiguous NCHW input, at most one column of padding) never materialise the unfolded input; with
 * more than 128 filters and channels in whole blocks of 32 they copy the filter (only) into the workspace in tap-major order,
 * unless it is stored that way already (a channels-last filter: strides (R S C, 1, S C, C)), which is then read as it is.  The
 * other convolutions on the library's own tile go through the library's workspace when what they need fits it:
 * unit-stride ones (wide padding, channels-last views) make a dense zero-padded copy of the input and run on that;
 * strided ones write the unfolded input once and run the product on the matrix kernels.  Else, or with a tile
 * named by the caller, every tile is gathered through the index map.
 * Memory: a dense unit-stride call with few output tiles and a long reduction has its reduction dealt to
 * several programs per tile, whose fp32 partial tiles go through a workspace that the library owns: one device
 * allocation of 256 MB per GPU, made by the first call on that GPU that needs it (that one call allocates, and
 * cannot be captured in a HIP graph), never moved or freed until the process ends.  All calls on a GPU share it,
 * one after the other: a call that finds it last used on another stream makes its own stream wait for that use
 * to finish (an event), so overlapping calls queue up for the workspace instead of racing.  What does not fit
 * the workspace, or a failed allocation, runs without it (no split, or through the index map).  The partial tiles
 * are added in a fixed order: a call repeated on the same data gives the same bits.
 */
nt_status nt_conv2d_implicit(const void *x, const nt_tensor_desc *dx, const void *w, const nt_tensor_desc *dw,
                             void *y, const nt_tensor_desc *dy,
                             int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                             nt_dtype in_dtype, nt_dtype out_dtype, nt_tile_cfg cfg, void *hip_stream);

/*
 * nt_trace_tile: device twin of the *_arrange_tile calls.  Launches a small kernel that
 * runs the operand-map address generator (the one the operand-map kernel gathers through; the
 * matrix and convolution kernels derive their own per-lane addresses), for one operand tile of
 * program `program_id` at k tile `k`, and writes offsets (int64, -1 where masked) and masks
 * (uint8) to the DEVICE arrays offsets_out / mask_out of `capacity` entries (row-major over
 * the tile).  kind: 0 = gemm, 1 = bmm, 2 = conv2d (conv arguments ignored otherwise).
 */
nt_status nt_trace_tile(int32_t kind, const nt_tensor_desc *d0, const nt_tensor_desc *d1, const nt_tensor_desc *d2,
                        int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                        nt_tile_cfg cfg, int32_t operand, int64_t program_id, int64_t k,
                        int64_t *offsets_out, uint8_t *mask_out, size_t capacity, void *hip_stream);

/*
 * nt_trace_loader_slice: the source-to-target mapping (Section 3.2.2) as the matrix-instruction kernels execute it.  Those
 * kernels do not go through the operand map that nt_trace_tile runs: each lane derives its own addresses (swizzled LDS slots,
 * range-checked loads, for the convolution the unfolded input generated on the fly with its padding fix-ups).  This call
 * launches ONE workgroup of the very kernel that nt_gemm / nt_bmm / nt_conv2d_implicit would launch for the same arguments
 * (kind: 0 / 1 / 2 as in nt_trace_tile; no k split), as program `program_id` (b * mt * nt + i * nt + j).  The workgroup
 * requests that program's 32-k slice `slice` (slice s covers k 32 s .. 32 s + 31; a k tile of 64 is two slices) with the
 * kernel's own loads, waits, applies what the kernel applies to a slice once it has landed (zeroing the k past K, the
 * padding elements of the convolution's runs), and copies the slice out of LDS:
 *   values_out[r * 32 + kk] = the 16-bit pattern the matrix instructions would read for row r of the operand's tile
 *   (A: output row, or output position of a convolution; B: output column / filter) and k index kk of the slice.
 * A caller who fills the operand with its elements' own indices (16 bits at a time) reads back, element by element, which
 * source element the loader put there, and zero where it fed a zero: compare with nt_arrange_* / the arrangement.
 * A, B: device pointers, read.  dC: the output's descriptor (shape only; nothing is stored).  values_out: DEVICE array of
 * `capacity` entries, at least 32 * (tile rows of the operand).  Only launches that stream their operands straight into LDS
 * (nt_last_kernel_path() 2, 4 or 6 for the same arguments) can be traced: otherwise NT_ERR_UNSUPPORTED.  The ring-unrolled
 * variant of the 256 x 256 kernel and its persistent form (one workgroup walking several programs) have the same per-lane
 * offsets and slice stepping as the kernel traced here.
 * Path 6 may run tile rows of two heights (the first ones 256 or 224 positions, the rest 32 fewer; tile row i starts where
 * the tile rows before it end): the rows of values_out past the traced program's height are left untouched.
 * Path 6 sums over the reduction index in another order than the arrangement lists it: its slice s, index kk is channel
 * c = 32 (s % (C / 32)) + kk of filter tap t = s / (C / 32), i.e. the arrangement's k = c * R * S + t.
 */
nt_status nt_trace_loader_slice(int32_t kind, const void *A, const nt_tensor_desc *dA, const void *B, const nt_tensor_desc *dB,
                                const nt_tensor_desc *dC, int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                                nt_dtype in_dtype, nt_dtype out_dtype, nt_tile_cfg cfg, int32_t operand, int64_t program_id, int64_t slice,
                                uint16_t *values_out, size_t capacity, void *hip_stream);

/*
 * nt_mfma_probe: a measurement aid for the roofline of the matrix kernels (the application of Section 4.2 is one `dot` per k
 * tile; this runs that instruction and nothing else).  `blocks` workgroups of 4 wavefronts each read a few operand fragments
 * from `data` (device pointer, 16-byte aligned, n_elems >= 8 elements of `dtype`, NT_F16 or NT_BF16) and issue
 * iters x 64 v_mfma_f32_16x16x32 instructions per wavefront on them, back to back: 2 * 16 * 16 * 32 * 64 * iters * 4 * blocks
 * flop per call, no memory traffic inside the loop.  The part is power managed and the rate depends on the operand values, so
 * the rate this call sustains on a workload's own data is the ceiling for a kernel on that instruction and data.
 * out: device array of blocks * 256 floats (checksums; written so that the loop cannot be optimised away).
 */
nt_status nt_mfma_probe(const void *data, int64_t n_elems, nt_dtype dtype, int32_t iters, int32_t blocks, float *out, void *hip_stream);

/* Thread-local, statically stored description of the last error on this thread ("" if none). */
const char *nt_last_error(void);

/* Library version string (static storage). */
const char *nt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NT_H */
