// Dispatch between the kernels, plus the small auxiliary kernels (zero fill, address trace).
#include <mutex>

#include "gemm_conv_direct.h"
#include "gemm_conv_tap.h"
#include "gemm_direct.h"
#include "gemm_direct16.h"

namespace nt {

// ------------------------------------------------------------- auxiliary kernels
__global__ void fill_zero_kernel(void *C, const OperandMap mc, int64_t batch, int64_t sc_batch, int out_dtype)
{
    const int64_t total = mc.rows * mc.cols;
    for (int64_t b = blockIdx.y; b < batch; b += gridDim.y)
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

// A compute unit works through p = ceil(programs / 256) programs; a program costs kt steps of `step` microseconds
// (time of one 64-wide k tile with the whole unit's matrix rate) plus a fixed `fixed` microseconds of launch, prologue and
// epilogue, which `resident` co-resident workgroups overlap with each other's multiplications.  The constants are fits to
// measurements on 8192 x 8192 x K and batched 2048 x 2048 x K problems.
nt_tile_cfg pick_gemm_tile(int64_t batch, int64_t M, int64_t N, int64_t K)
{
    struct Cand { int bm, bn; double fixed, step; int resident; };
    // (fits to 8192 x 8192 x K, 4096 x 4096 x K and 32 x 2048 x 2048 x K for K = 256 .. 8192 on a chip with every unit busy;
    // the 256 x 256 figures are those of the persistent kernel)
    const Cand cands[] = {{256, 256, 8.5, 1.42, 1}, {128, 256, 7.0, 0.82, 2}, {256, 128, 6.5, 0.915, 2}, {128, 128, 4.5, 0.51, 2}};
    const double kt = (double)((K + 63) / 64);
    nt_tile_cfg best{128, 128, 64};
    double best_cost = 0;
    for (const Cand &c : cands) {
        const int64_t programs = batch * ((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
        const int64_t p = (programs + 255) / 256;
        // (problems that are not whole aligned tiles run with one workgroup per unit for every tile but the smallest)
        const bool full = M % c.bm == 0 && N % c.bn == 0 && K % 64 == 0;
        const int resident = full || (c.bm == 128 && c.bn == 128) ? c.resident : 1;
        // (the persistent kernel staggers short programs: a program's fixed part then overlaps other units' multiplications)
        const bool staggered = c.bm == 256 && c.bn == 256 && full && programs >= 512 && kt <= 16;
        const double cost = staggered ? 4.0 + (double)p * (6.0 + kt * c.step)
                                      : (double)((p + resident - 1) / resident) * c.fixed + (double)p * kt * c.step;
        if (best_cost == 0 || cost < best_cost) { best_cost = cost; best = nt_tile_cfg{c.bm, c.bn, 64}; }
    }
    return best;
}

// Dense zero-padded copy of a convolution's input: P[n][c][h'][w'] = x[n, c, h' - ph, w' - pw] (zero outside the image),
// rows Wp = W + 2 pw long (the caller rounds nothing: the copy is as dense as a tensor).  For unit-stride convolutions
// that the implicit kernels do not take as they are (more than one column of padding, channels-last or otherwise strided
// input): on the copy they are convolutions without padding.  One thread: 8 consecutive elements of the copy, offsets
// first, the eight loads back to back (see conv_unfold_kernel).  The workspace holds total rounded up to 8 elements.
struct PadArgs {
    const uint16_t *x;
    uint16_t *P;
    int64_t xs[4];
    int64_t total;                 // N * C * Hp * Wp
    int32_t C, H, W, Hp, Wp, ph, pw;
};

__global__ __launch_bounds__(256) void conv_pad_kernel(const PadArgs g)
{
    const int64_t groups = (g.total + 7) / 8;
    const int32_t xs2 = (int32_t)g.xs[2], xs3 = (int32_t)g.xs[3];
    for (int64_t grp = (int64_t)blockIdx.x * 256 + threadIdx.x; grp < groups; grp += (int64_t)gridDim.x * 256) {
        const int64_t e0 = grp * 8;
        const int64_t plane = e0 / ((int64_t)g.Hp * g.Wp);                  // (n, c)
        const int32_t rem = (int32_t)(e0 - plane * ((int64_t)g.Hp * g.Wp));
        const int64_t n = plane / g.C, c = plane - n * g.C;
        const int64_t n2 = c + 1 == g.C ? n + 1 : n, c2 = c + 1 == g.C ? 0 : c + 1;     // the plane after it (a group may run into it)
        const int64_t base = n * g.xs[0] + c * g.xs[1], base2 = n2 * g.xs[0] + c2 * g.xs[1];
        int32_t h = rem / g.Wp, w = rem - h * g.Wp;
        int64_t off[8];
        uint32_t keep = 0;
        bool next = false;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool in = e0 + e < g.total && (uint32_t)(h - g.ph) < (uint32_t)g.H && (uint32_t)(w - g.pw) < (uint32_t)g.W;
            off[e] = in ? (next ? base2 : base) + (h - g.ph) * xs2 + (w - g.pw) * xs3 : 0;
            keep |= (in ? 1u : 0u) << e;
            const bool row_end = ++w == g.Wp;
            w = row_end ? 0 : w;
            h += row_end ? 1 : 0;
            const bool plane_end = h == g.Hp;
            h = plane_end ? 0 : h;
            next = next || plane_end;
        }
        uint32_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = g.x[off[e]];
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2)
            o[e >> 1] = ((keep >> e) & 1u ? v[e] : 0u) | (((keep >> (e + 1)) & 1u ? v[e + 1] : 0u) << 16);
        const u32x4 ov{o[0], o[1], o[2], o[3]};
        __builtin_memcpy(g.P + e0, &ov, 16);
    }
}

// The same copy for a dense channels-last input (x[n][h][w][c]): a transposition.  One workgroup: 64 channels x 32
// positions of one padded row, read along c (128 contiguous bytes per wavefront), turned in LDS, written along w.
// (conv_pad_kernel reads such an input with its lanes C elements apart: 70 us for 51 MB.)
__global__ __launch_bounds__(256) void conv_pad_nhwc_kernel(const PadArgs g)
{
    __shared__ uint16_t tile[32][66];
    const int32_t ctiles = (g.C + 63) / 64;
    const int32_t n = blockIdx.z / ctiles, c0 = (blockIdx.z - n * ctiles) * 64;
    const int32_t hp = blockIdx.y, w0 = blockIdx.x * 32, h = hp - g.ph;
    const int tid = threadIdx.x;
    {
        const int c = tid & 63, wl = tid >> 6;
        const uint16_t *row = g.x + (((int64_t)n * g.H + h) * g.W) * g.C + c0 + c;
        const bool hc_ok = (uint32_t)h < (uint32_t)g.H && c0 + c < g.C;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int32_t w = w0 + wl + 4 * i - g.pw;
            const bool in = hc_ok && (uint32_t)w < (uint32_t)g.W;
            tile[wl + 4 * i][c] = in ? row[(int64_t)w * g.C] : (uint16_t)0;
        }
    }
    __syncthreads();
    {
        const int w = tid & 31, cl = tid >> 5;
        if (w0 + w < g.Wp) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int c = cl + 8 * i;
                if (c0 + c < g.C) g.P[(((int64_t)n * g.C + c0 + c) * g.Hp + hp) * g.Wp + w0 + w] = tile[w][c];
            }
        }
    }
}

// Unfolded input of a convolution (Section 4.3: A[m, kk] = x[n, c, p sh + r - ph, q sw + s - pw], zero outside the
// image), written out for the convolutions the implicit kernels do not take (strided, widely padded, channels-last):
// U[kk][m] with m = (n, p, q) contiguous and the row pitch Mp (a multiple of 8; the surplus columns are zeros);
// x has any strides.
struct UnfoldArgs {
    const uint16_t *x;
    uint16_t *U;
    int64_t xs[4];
    int64_t M, Mp, K;
    int32_t C, H, W, R, S, P, Q, sh, sw, ph, pw, dh, dw;
};

__global__ __launch_bounds__(256) void conv_unfold_kernel(const UnfoldArgs g)
{
    // blockIdx.y: the line kk = (c, r, s), taken apart once per workgroup in scalar registers; x: groups of 8 positions.
    // Element offsets are 32-bit (the host admits inputs whose offsets stay below 2^31).
    const uint32_t kk = blockIdx.y;
    const uint32_t c = kk / (uint32_t)(g.R * g.S), rs = kk - c * (uint32_t)(g.R * g.S);
    const uint32_t r = rs / (uint32_t)g.S, sx = rs - r * (uint32_t)g.S;
    const uint16_t *xc = g.x + (int64_t)c * g.xs[1];
    const int32_t xs0 = (int32_t)g.xs[0], xs2 = (int32_t)g.xs[2], xs3 = (int32_t)g.xs[3];
    const uint32_t groups = (uint32_t)(g.Mp / 8), pq = (uint32_t)(g.P * g.Q);
    for (uint32_t grp = blockIdx.x * 256 + threadIdx.x; grp < groups; grp += gridDim.x * 256) {
        const uint32_t m0 = grp * 8;
        uint32_t n = m0 / pq;
        const uint32_t rem = m0 - n * pq;
        int32_t p = (int32_t)(rem / (uint32_t)g.Q), q = (int32_t)(rem - (uint32_t)p * (uint32_t)g.Q);
        // A group that lies in one output row and reads 8 (conv stride 1) or 16 (stride 2) consecutive elements of one
        // input row, all inside the image: one or two 16-byte loads (2-byte aligned), every second element picked for
        // stride 2.  (Input contiguous along w only.)
        if (xs3 == 1 && g.sw <= 2 && q + 8 <= g.Q && m0 + 8 <= (uint32_t)g.M) {
            const int32_t h = p * g.sh + (int32_t)r * g.dh - g.ph, col = q * g.sw + (int32_t)sx * g.dw - g.pw;
            if ((uint32_t)h < (uint32_t)g.H && col >= 0 && col + 8 * g.sw <= g.W) {
                const uint16_t *src = xc + ((int32_t)n * xs0 + h * xs2 + col);
                u32x4 a;
                __builtin_memcpy(&a, src, 16);
                if (g.sw == 2) {
                    u32x4 b;
                    __builtin_memcpy(&b, src + 8, 16);
                    a = u32x4{__builtin_amdgcn_perm(a[1], a[0], 0x05040100u), __builtin_amdgcn_perm(a[3], a[2], 0x05040100u),
                              __builtin_amdgcn_perm(b[1], b[0], 0x05040100u), __builtin_amdgcn_perm(b[3], b[2], 0x05040100u)};
                }
                __builtin_memcpy(g.U + (int64_t)kk * g.Mp + m0, &a, 16);
                continue;
            }
        }
        // Otherwise all eight offsets first (an element outside the image or past M points at element 0 and is dropped),
        // then the eight loads back to back, with no branch between them: this part is bound by the latency of its loads
        int32_t off[8];
        uint32_t keep = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int32_t h = p * g.sh + (int32_t)r * g.dh - g.ph, col = q * g.sw + (int32_t)sx * g.dw - g.pw;
            const bool in = m0 + e < (uint32_t)g.M && (uint32_t)h < (uint32_t)g.H && (uint32_t)col < (uint32_t)g.W;
            off[e] = in ? (int32_t)n * xs0 + h * xs2 + col * xs3 : 0;
            keep |= (in ? 1u : 0u) << e;
            const bool row_end = ++q == g.Q;
            q = row_end ? 0 : q;
            p += row_end ? 1 : 0;
            const bool image_end = p == g.P;
            p = image_end ? 0 : p;
            n += image_end ? 1 : 0;
        }
        uint32_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = xc[off[e]];
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2)
            w[e >> 1] = ((keep >> e) & 1u ? v[e] : 0u) | (((keep >> (e + 1)) & 1u ? v[e + 1] : 0u) << 16);
        const u32x4 o{w[0], w[1], w[2], w[3]};
        __builtin_memcpy(g.U + (int64_t)kk * g.Mp + m0, &o, 16);
    }
}

// k split of a GEMM, second step: C[m, n] = act(alpha * sum_i ws[i][m][n] + beta * D[m, n]) with the slices added in slice
// order (reproducible), converted once.  C and D are plain strided matrices.
__global__ __launch_bounds__(256) void splitk_sum_kernel(const float *ws, int ksplit, int64_t M, int64_t N, void *C, int64_t scm, int64_t scn, int out_dtype,
                                                         const void *D, int64_t sdm, int64_t sdn, float alpha, float beta, int act)
{
    const ActParams ap = act_params(act);
    const int64_t total = M * N;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        float sum = ws[i];
        for (int j = 1; j < ksplit; ++j) sum += ws[j * total + i];
        const int64_t m = i / N, n = i - m * N;
        const float x = combine(sum, D ? load_as_f32(D, m * sdm + n * sdn, out_dtype) : 0.f, alpha, beta);
        store_out(C, m * scm + n * scn, act ? activate(x, ap) : x, out_dtype);
    }
}

bool tile_is_built(nt_tile_cfg cfg)
{
    for (const TileEntry &t : kTiles)
        if (t.bm == cfg.bm && t.bn == cfg.bn && t.bk == cfg.bk) return true;
    return false;
}

// The dense convolution that the convolution kernels handle: contiguous NCHW input, conv stride 1, at
// most one element of left / right padding, a filter whose (c, r, s) are contiguous, an output with
// contiguous (p, q).  Everything else runs on the operand-map kernel.
static bool conv_tap_ok(const GemmLaunch &g, const ConvArgs &c, size_t *repack_bytes);

static bool match_conv(const GemmLaunch &g, ConvArgs *a)
{
    const ConvHint &h = g.conv;
    if (!h.valid || g.batch != 1 || g.tile.bm != 256 || g.tile.bk != 64 || (g.tile.bn != 128 && g.tile.bn != 256)) return false;
    if (h.sh != 1 || h.sw != 1 || h.dh != 1 || h.dw != 1 || h.ph < 0 || h.pw < 0 || h.pw > 1 || h.R > 31 || h.S > 31 || h.P <= 0 || h.Q <= 0) return false;
    if (h.xs[3] != 1 || h.xs[2] != h.W || h.xs[1] != h.H * h.W || h.xs[0] != h.C * h.H * h.W) return false;
    // filter rows contiguous in (c, r, s), or in (r, s, c) (a channels-last filter, which is the tap-major kernel's own order)
    const bool krsc = h.ws[1] == 1 && h.ws[3] == h.C && h.ws[2] == h.S * h.C && (h.C > 1 || h.R * h.S == 1);
    if (!krsc && (h.ws[3] != 1 || h.ws[2] != h.S || h.ws[1] != h.R * h.S)) return false;
    if (h.ws[0] <= 0 || h.ws[0] >= (1 << 22)) return false;
    if (h.ys[3] != 1 || h.ys[2] != h.Q) return false;
    // the kernel numbers the output positions with the row pitch rounded up to a multiple of 8
    const int64_t Q8 = (h.Q + 7) / 8 * 8;
    const int64_t CRS = h.C * h.R * h.S, NPQ = h.N * h.P * Q8, numel = h.N * h.C * h.H * h.W;
    if (numel >= (1LL << 31) || numel < 8 || NPQ >= (1LL << 31) - 256 || CRS >= (1 << 16) - 128 || CRS < 8) return false;   // (the filter loader needs K >= 8)
    a->X = (const uint16_t *)g.A;
    a->Wt = (const uint16_t *)g.B;
    a->Y = g.C;
    a->ldb = h.ws[0];
    a->syn = h.ys[0];
    a->syf = h.ys[1];
    a->x_numel = numel;
    a->M = (int32_t)NPQ; a->N = (int32_t)g.N; a->K = (int32_t)CRS;
    a->PQ = (int32_t)(h.P * h.Q); a->Q = (int32_t)h.Q; a->H = (int32_t)h.H; a->W = (int32_t)h.W;
    a->Q8 = (int32_t)Q8; a->PQ8 = (int32_t)(h.P * Q8); a->last_e = (int32_t)((h.Q - 1) % 8);
    a->HW = (int32_t)(h.H * h.W); a->CHW = (int32_t)(h.C * h.H * h.W);
    a->RS = (int32_t)(h.R * h.S); a->S = (int32_t)h.S; a->R = (int32_t)h.R; a->ph = (int32_t)h.ph; a->pw = (int32_t)h.pw;
    a->inv_rs = h.R * h.S > 1 ? (uint32_t)((1ULL << 32) / (uint64_t)(h.R * h.S)) + 1u : 0u;
    a->inv_s = h.S > 1 ? (uint32_t)((1ULL << 32) / (uint64_t)h.S) + 1u : 0u;
    a->mt = (NPQ + 255) / 256; a->nt = g.nt; a->kt = g.kt;
    a->out_dtype = g.out_dtype;
    a->ksplit = 1; a->kt_per = (int32_t)g.kt; a->slice = 0;
    a->filter_tap_major = krsc && !(h.ws[3] == 1 && h.ws[2] == h.S && h.ws[1] == h.R * h.S) ? 1 : 0;
    if (a->filter_tap_major) {                               // (no other kernel reads that layout)
        size_t unused = 0;
        if (!conv_tap_ok(g, *a, &unused)) return false;
    }
    return true;
}

// Workspace of the k splits (convolution, skinny GEMM), of the zero-padded copy and of the unfolded input of a convolution:
// one allocation of kSplitWsMax bytes per device, made by the first call on that device that needs it and kept until the
// process ends (never freed or moved, so work in flight never loses it).  Every call on a device shares it.  A call holds it
// through a WorkspaceLease from before its first launch that touches it until after its last: the lease serialises host
// threads (a mutex) and streams (an event recorded behind the last consumer, which a call on any other stream makes its
// stream wait for before its own first launch), so calls that overlap on one device queue up instead of racing.
static constexpr size_t kSplitWsMax = 256u << 20;

class WorkspaceLease {
public:
    WorkspaceLease() = default;
    WorkspaceLease(const WorkspaceLease &) = delete;
    WorkspaceLease &operator=(const WorkspaceLease &) = delete;
    // nullptr: more than the workspace holds, no memory, or no device -- the caller then runs without it
    void *acquire(size_t bytes, hipStream_t stream)
    {
        int dev = 0;
        if (slot_ || bytes > kSplitWsMax || hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
        Slot &w = table()[dev];
        w.mu.lock();
        bool ok = true;
        if (!w.p) {
            void *p = nullptr;
            hipEvent_t ev = nullptr;
            if (hipMalloc(&p, kSplitWsMax) != hipSuccess) { (void)hipGetLastError(); ok = false; }
            else if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); (void)hipFree(p); ok = false; }
            else { w.p = p; w.done = ev; }
        }
        if (ok && w.used && w.last != stream && hipStreamWaitEvent(stream, w.done, 0) != hipSuccess) { (void)hipGetLastError(); ok = false; }
        if (!ok) { w.mu.unlock(); return nullptr; }
        slot_ = &w;
        stream_ = stream;
        return w.p;
    }
    ~WorkspaceLease()
    {
        if (!slot_) return;
        if (hipEventRecord(slot_->done, stream_) == hipSuccess) { slot_->last = stream_; slot_->used = true; }
        else {
            // without the marker a later call on another stream could not wait for this one's work: wait for it here
            (void)hipGetLastError();
            (void)hipStreamSynchronize(stream_);
            slot_->used = false;
        }
        slot_->mu.unlock();
    }

private:
    struct Slot { void *p = nullptr; hipEvent_t done = nullptr; hipStream_t last = nullptr; bool used = false; std::mutex mu; };
    static Slot *table() { static Slot t[64]; return t; }
    Slot *slot_ = nullptr;
    hipStream_t stream_ = nullptr;
};

// Scratch memory for callers that cannot allocate (nt_gemm_noalloc): a fixed array in the library's device image, one copy
// per GPU, held from the moment the library is loaded on that GPU until the process ends.  Host code never uses the array's
// name as an address: the device address is looked up once per device, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[NT_NOALLOC_SCRATCH_BYTES];

nt_status static_scratch(void **ptr_out, size_t *bytes_out)
{
    static void *table[64] = {};
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(NT_ERR_DEVICE, std::string("hipGetDevice: ") + hipGetErrorString(e));
    if (dev < 0 || dev >= 64) return fail(NT_ERR_UNSUPPORTED, "device index beyond 63");
    std::lock_guard<std::mutex> lock(mu);
    if (!table[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { (void)hipGetLastError(); return fail(NT_ERR_DEVICE, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e)); }
        table[dev] = p;
    }
    *ptr_out = table[dev];
    *bytes_out = sizeof(scratch);
    return NT_OK;
}

// Estimated time (us) of a dense unit-stride convolution -- an implicit GEMM of M positions x N filters x kt k tiles -- on
// tiles of 256 positions x bn filters with `per` k tiles per program (ks = ceil(kt / per) programs per output tile).  A
// program costs a fixed part plus its 32-k slices (0.8 us each on the 256-filter tile, 1.15 on the narrower ones, which do
// half the work or less per slice: their loader, not the matrix pipe, sets the pace; the 256-filter tile's fixed part
// includes the copy of the filter); programs run in rounds of one per compute unit (two for the narrower tiles, which are
// co-resident); a split adds a second launch and the partial tiles' trip through memory.  Fits (us, measured):
// (256,512,7,7)*(512,512,3,3) 172 on 128-filter tiles, 111-119 on 256-filter tiles split in two; (32,512,14,14)*(512,512,3,3)
// 99 / 73; (8,256,56,56)*(256,256,3,3) 73 / 60; (16,256,28,28)*(256,256,3,3) 58.5 / 57.8; (32,256,14,14)*(1024,256,1,1) 18 / 31.
static double conv_cost(int64_t M, int64_t N, int64_t kt, int bn, int64_t per)
{
    const int64_t ks = (kt + per - 1) / per;
    const int64_t programs = ((M + 255) / 256) * ((N + bn - 1) / bn) * ks;
    const int64_t slots = bn == 256 ? 256 : 512;
    const double fixed = bn == 256 ? 14.0 : 7.0, slice = bn == 256 ? 0.8 : 1.15;
    double c = (double)((programs + slots - 1) / slots) * (fixed + 2.0 * (double)per * slice);
    if (ks > 1) c += 6.0 + (double)ks * (double)M * (double)N * 8.0 / 5.0e6;
    return c;
}

// The split of the reduction for that tile: `*kt_per` k tiles per program (none with fewer than 4), the number of parts
// returned.  Small grids (fewer than 48 tiles of 256 x 256): enough parts for about one program per compute unit
// (measured on 13 shapes from 1 to 112 programs and 8 to 72 k tiles: the split run is faster in every one, e.g.
// (8,64,14,14) * (64,64,3,3) 26 -> 21 us, (4,256,14,14) * (256,256,3,3) 78 -> 23 us).  Larger ones: the cheapest by the
// estimate above, which knows about whole rounds (5 parts of 56 tiles are 280 programs and cost two rounds, 4 parts one).
static bool conv_small(int64_t M, int64_t N) { return ((M + 255) / 256) * ((N + 255) / 256) < 48; }
static int conv_ksplit(int64_t M, int64_t N, int64_t kt, int bn, int32_t *kt_per, double *cost_out = nullptr)
{
    *kt_per = (int32_t)kt;
    if (conv_small(M, N)) {
        const int64_t programs = ((M + 255) / 256) * ((N + bn - 1) / bn);
        if (programs >= 128 || kt < 8) return 1;
        const int64_t want = std::min<int64_t>((256 + programs / 2) / programs, kt / 4);
        if (want < 2) return 1;
        const int64_t per = (kt + want - 1) / want;
        *kt_per = (int32_t)per;
        return (int)((kt + per - 1) / per);
    }
    int64_t best_per = kt;
    double best = conv_cost(M, N, kt, bn, kt);
    for (int64_t ks = 2; ks <= 64; ++ks) {
        const int64_t per = (kt + ks - 1) / ks;
        if (per < 4 || (double)ks * (double)M * (double)N * 4.0 > (double)kSplitWsMax) break;
        if ((kt + per - 1) / per != ks) continue;                              // (that many parts come out one fewer)
        const double c = conv_cost(M, N, kt, bn, per);
        if (c < best) { best = c; best_per = per; }
    }
    *kt_per = (int32_t)best_per;
    if (cost_out) *cost_out = best;
    return (int)((kt + best_per - 1) / best_per);
}

// The tile of filters for such a convolution.  Small grids: 256 filters per program when 256 would not leave half the
// compute units without a program, else 128; larger ones: by the estimate, each tile with its best split.
nt_tile_cfg pick_conv_tile(int64_t M, int64_t N, int64_t K)
{
    if (N <= 128) return nt_tile_cfg{256, 128, 64};
    if (conv_small(M, N)) return nt_tile_cfg{256, 128, 64};
    const int64_t kt = (K + 63) / 64;
    int32_t per = 0;
    double c256 = 0, c128 = 0;
    conv_ksplit(M, N, kt, 256, &per, &c256);
    conv_ksplit(M, N, kt, 128, &per, &c128);
    return c256 <= c128 ? nt_tile_cfg{256, 256, 64} : nt_tile_cfg{256, 128, 64};
}

// A map is "plain" when it is a strided matrix without bounds checks beyond rows / cols.
static bool plain(const OperandMap &m) { return m.nrd == 1 && m.ncd == 1 && m.nchk == 0; }

// The same for a GEMM with few output tiles and a long reduction (a skinny product): the split is run as a batched
// product over equal parts of K, so only a number of parts that divides the k tiles evenly is taken (at least 8 k tiles
// each).  Two dependent launches and the trip of the partial tiles through memory have their price: the split is taken
// when an estimate of it (12 us for the launches, 0.37 us per k tile of a program that has its compute unit to
// itself, the slices written and read at 3 TB/s) beats the estimate of the single launch (7 us + 0.37 us per k tile).
// Measured: 1024 x 1024 x 1024 11 us unsplit against 19 split, 1024 x 1024 x 4096 31 against 24, 256 x 256 x 8192 55
// against 15, 512 x 512 x 2048 17 against 13.
static int gemm_ksplit(int64_t programs, int64_t kt, int64_t M, int64_t N)
{
    if (programs >= 128 || kt < 32) return 1;
    const int64_t want = std::min<int64_t>((256 + programs / 2) / programs, kt / 8);
    for (int64_t d = want; d >= 2; --d) {
        if (kt % d) continue;
        const double single = 7.0 + 0.37 * (double)kt;
        const double split = 12.0 + 0.37 * (double)kt / (double)d + (double)d * (double)M * (double)N * 8.0 / 3.0e6;
        return split < single ? (int)d : 1;
    }
    return 1;
}

static thread_local int t_k_split = 1;
int last_k_split() { return t_k_split; }

// Where a k split's fp32 partial tiles go: the region the caller of this launch has set aside (a route that already holds
// the workspace, or an entry point that brings its own scratch memory), else the library's workspace through `lease`.
// nullptr: none (then the launch runs unsplit); *status is set when the caller's region is too small and must be.
static float *split_region(const GemmLaunch &g, size_t bytes, WorkspaceLease &lease, nt_status *status)
{
    *status = NT_OK;
    if (g.ws_given) {
        if (bytes <= g.ws_given_bytes) return g.ws_given;
        if (g.ws_strict)
            *status = fail(NT_ERR_UNSUPPORTED, "this product's k split needs " + std::to_string(bytes) + " bytes of scratch memory, more than the " +
                                                   std::to_string(g.ws_given_bytes) + " this entry point has");
        return nullptr;
    }
    if (g.no_workspace) return nullptr;
    return (float *)lease.acquire(bytes, (hipStream_t)g.stream);
}

// operands that can stream straight into LDS: whole 32-k slices, 16-byte aligned filter rows, 32-bit byte offsets
static bool conv_direct_ok(const GemmLaunch &g, const ConvArgs &c)
{
    return c.K % 32 == 0 && c.ldb % 8 == 0 && (reinterpret_cast<uintptr_t>(c.Wt) & 15) == 0 && c.R <= 8 && c.S <= 8 &&
           c.x_numel < (1LL << 30) && ((int64_t)(c.N - 1) * c.ldb + c.K) < (1LL << 30) &&
           ((g.conv.N - 1) * c.syn + (int64_t)(c.N - 1) * c.syf + c.PQ) < (1LL << 29);   // (output offsets: 31 bits of bytes)
}

// ... and that the kernel which walks the reduction tap by tap takes (gemm_conv_tap.h): 256 filters per program, channels in
// whole blocks of 32, padding smaller than the image; it reads the filter from a tap-major copy of `*repack_bytes` bytes
static bool conv_tap_ok(const GemmLaunch &g, const ConvArgs &c, size_t *repack_bytes)
{
    *repack_bytes = c.filter_tap_major ? 0 : ((size_t)c.N * c.K * 2 + 255) / 256 * 256;
    // (a filter row fits the LDS of the kernel that copies it: K <= 32768; one bit per tap: R S <= 32)
    return conv_direct_ok(g, c) && g.tile.bn == 256 && c.N > 128 && g.conv.C % 32 == 0 && c.ph < c.H && c.pw < c.W && c.K <= 32768 && c.RS <= 32;
}

// workspace that route 1 asks for: the filter's tap-major copy, then the fp32 slices of the k split
static size_t conv_scratch_need(const GemmLaunch &g, const ConvArgs &c)
{
    size_t repack = 0;
    const bool tap = conv_tap_ok(g, c, &repack);
    int32_t kt_per = 0;
    const int ks = conv_ksplit(c.M, c.N, c.kt, g.tile.bn, &kt_per);
    return (tap ? repack : 0) + (ks > 1 ? (size_t)ks * g.conv.N * c.N * c.PQ * 4 : 0);
}

// ---- route 1: the dense unit-stride convolution on the implicit-GEMM kernels (with the k split for small grids)
static nt_status route_conv_implicit(const GemmLaunch &g, const ConvArgs &c, int *path_out)
{
    const nt_tile_cfg t = g.tile;
    if (path_out) *path_out = PATH_CONV;
    const bool edge_b = (g.N % t.bn) || (g.K % t.bk);
    hipStream_t s = (hipStream_t)g.stream;
    int32_t kt_per = 0;
    const int ksplit = g.trace.out ? 1 : conv_ksplit(c.M, c.N, c.kt, t.bn, &kt_per);
    const int64_t slice = g.conv.N * (int64_t)c.N * c.PQ;
    const bool direct = conv_direct_ok(g, c);
    size_t repack_bytes = 0;
    bool tap = conv_tap_ok(g, c, &repack_bytes);
    const size_t split_bytes = ksplit > 1 ? (size_t)ksplit * slice * 4 : 0;
    // one piece of workspace: the filter's copy, then the split's slices.  None to be had (too large, no memory, a caller
    // who holds the workspace and has set aside less): the copy is given up first (the kernel in the arrangement's k
    // order needs none), then the split.
    WorkspaceLease lease;
    char *region = nullptr;
    if ((tap && repack_bytes) || ksplit > 1) {
        nt_status st;
        region = (char *)split_region(g, (tap ? repack_bytes : 0) + split_bytes, lease, &st);
        if (!region && tap && !c.filter_tap_major) {
            tap = false;
            if (ksplit > 1) region = (char *)split_region(g, split_bytes, lease, &st);
        }
        if (st != NT_OK) return st;
    }
    uint16_t *wt_tap = tap && repack_bytes ? (uint16_t *)region : nullptr;
    float *ws = region && ksplit > 1 ? (float *)(region + (tap ? repack_bytes : 0)) : nullptr;
    if (direct && path_out) *path_out = tap ? PATH_CONV_TAP : PATH_CONV_DIRECT;
    const bool bf16 = g.in_dtype == NT_BF16;
    ConvArgs base = c;
    int tap_rows = 256;
    if (tap) {
        if (wt_tap) {
            const nt_status st = launch_conv_repack_filter(c.Wt, c.ldb, wt_tap, c.N, (int32_t)g.conv.C, c.RS, s);
            if (st != NT_OK) return st;
            base.Wt = wt_tap;
            base.ldb = c.K;
        }
        // Tile heights: the kernel is built for a first height of h = 8 or 7 blocks of 32 positions and a second of h - 1.
        // Whole rounds of programs (one per compute unit) cost their length, h blocks plus a fixed part; ra rounds of the
        // first height, then as many of the second as the remaining positions need: the cheapest (h, ra).  With a k split
        // (small grids) one height only.
        const int64_t units = 256, blocks = ((int64_t)c.M + 31) / 32;
        const int64_t per_round = units / (c.nt * ksplit) > 0 ? units / (c.nt * ksplit) : 1;      // tiles of positions per round
        const double fixed = 1.5;
        double best = 0;
        int64_t best_a = 0, best_mt = 0;
        auto consider = [&](int h, int64_t mt_a) {
            const int64_t left = blocks - mt_a * h > 0 ? blocks - mt_a * h : 0;
            const int64_t mt_b = (left + h - 2) / (h - 1);
            const int64_t ra = (mt_a * c.nt * ksplit + units - 1) / units, rb = (mt_b * c.nt * ksplit + units - 1) / units;
            const double cost = (double)ra * (h + fixed) + (double)rb * (h - 1 + fixed);
            if (best == 0 || cost < best) { best = cost; tap_rows = 32 * h; best_a = mt_a; best_mt = mt_a + mt_b; }
        };
        for (int h = 8; h >= 7; --h) {
            const int64_t all_a = (blocks + h - 1) / h;                        // tiles if every tile had the first height
            consider(h, 0);
            if (ksplit == 1)
                for (int64_t mt_a = per_round; mt_a < all_a; mt_a += per_round) consider(h, mt_a);
            consider(h, all_a);
        }
        base.mt_a = (int32_t)best_a;
        base.mt = best_mt;
    }
    if (g.trace.out) {
        if (!direct) return fail(NT_ERR_UNSUPPORTED, "this convolution does not run on the kernels that stream their operands into LDS");
        const int bn = c.N <= 64 ? 64 : (c.N <= 128 ? 128 : t.bn);
        // (positions per program: the traced program's own height)
        const int64_t rows = g.trace.operand == 0 ? (tap ? (g.trace.program < base.mt_a * c.nt ? tap_rows : tap_rows - 32) : 256) : bn;
        if ((size_t)rows * 32 > g.trace.capacity) return fail(NT_ERR_BUFFER_TOO_SMALL, "trace buffer smaller than the slice");
        if (g.trace.program < 0 || g.trace.program >= base.mt * c.nt) return fail(NT_ERR_INVALID_ARG, "program_id outside the grid");
        if (g.trace.slice < 0 || g.trace.slice >= c.K / 32) return fail(NT_ERR_INVALID_ARG, "slice outside the reduction");
        base.trace_out = g.trace.out; base.trace_program = g.trace.program; base.trace_slice = g.trace.slice; base.trace_operand = g.trace.operand;
        return tap ? launch_conv_tap_trace(base, tap_rows, s) : launch_conv_direct_trace(base, bn, s);
    }
    auto launch = [&](const ConvArgs &ca, int64_t nwg) {
        if (tap) return launch_conv_tap(ca, tap_rows, bf16, nwg, s);
        // (one column of tiles with few filters: the same grid is run by the kernel built for 64 or 128 filters per
        // program, which spends a quarter or half of the MFMAs)
        const int bn = ca.N <= 64 && direct ? 64 : (ca.N <= 128 ? 128 : t.bn);
        return direct ? launch_conv_direct(ca, bn, bf16, nwg, s) : launch_conv(ca, bn, bf16, edge_b || (ca.N % bn) != 0, nwg, s);
    };
    if (!ws) return launch(base, base.mt * c.nt);
    t_k_split = ksplit;
    ConvArgs part = base;
    part.Y = ws; part.syn = (int64_t)c.N * c.PQ; part.syf = c.PQ; part.out_dtype = NT_F32;
    part.ksplit = ksplit; part.kt_per = kt_per; part.slice = slice;
    const nt_status st = launch(part, base.mt * c.nt * ksplit);
    if (st != NT_OK) return st;
    return launch_conv_ws_sum(ws, ksplit, slice, c.Y, (int64_t)c.N * c.PQ, c.PQ, c.syn, c.syf, c.out_dtype, s);
}

static bool conv_is_bare(const GemmLaunch &g)        // a convolution and nothing else: library tile, no epilogue terms, free to use the workspace
{
    return g.conv.valid && !g.user_tile && !g.no_workspace && !g.ws_given && g.batch == 1 && !g.has_d && g.alpha == 1.f && g.act == 0;
}

// ---- route 2: a unit-stride convolution that the implicit kernels do not take as it is (more than one column of padding, a
// channels-last or otherwise strided input): on a dense zero-padded copy of its input, made once in the workspace (the
// input's size, not C R S times it), it is a dense convolution without padding.  *taken = false: not this route.
static nt_status route_conv_padded_copy(const GemmLaunch &g, int *path_out, bool *taken)
{
    *taken = false;
    const ConvHint &h = g.conv;
    if (!(conv_is_bare(g) && h.sh == 1 && h.sw == 1 && h.dh == 1 && h.dw == 1 && h.ph >= 0 && h.pw >= 0 && h.xs[0] >= 0 && h.xs[1] >= 0 && h.xs[2] >= 0 && h.xs[3] >= 0 &&
          (h.H - 1) * h.xs[2] + (h.W - 1) * h.xs[3] < (1LL << 31)))
        return NT_OK;
    const int64_t Hp = h.H + 2 * h.ph, Wp = h.W + 2 * h.pw, total = h.N * h.C * Hp * Wp;
    GemmLaunch g2 = g;
    g2.conv.H = Hp; g2.conv.W = Wp; g2.conv.ph = 0; g2.conv.pw = 0;
    g2.conv.xs[3] = 1; g2.conv.xs[2] = Wp; g2.conv.xs[1] = Hp * Wp; g2.conv.xs[0] = h.C * Hp * Wp;
    g2.no_workspace = true;                              // (this route holds the workspace)
    ConvArgs probe{};
    const size_t bytes = ((size_t)((total + 7) / 8 * 8) * 2 + 255) / 256 * 256;
    if (!(Hp * Wp >= 8 && total < (1LL << 31) && match_conv(g2, &probe))) return NT_OK;
    // the copy and, behind it, what the convolution on it will ask for (the filter's tap-major copy, the k split's slices)
    size_t split_bytes = conv_scratch_need(g2, probe);
    if (bytes + split_bytes > kSplitWsMax) split_bytes = 0;
    WorkspaceLease lease;
    uint16_t *P = (uint16_t *)lease.acquire(bytes + split_bytes, (hipStream_t)g.stream);
    if (!P) return NT_OK;
    *taken = true;
    if (split_bytes) { g2.ws_given = (float *)((char *)P + bytes); g2.ws_given_bytes = split_bytes; }
    PadArgs pa{};
    pa.x = (const uint16_t *)g.A; pa.P = P;
    for (int d = 0; d < 4; ++d) pa.xs[d] = h.xs[d];
    pa.total = total;
    pa.C = (int32_t)h.C; pa.H = (int32_t)h.H; pa.W = (int32_t)h.W; pa.Hp = (int32_t)Hp; pa.Wp = (int32_t)Wp;
    pa.ph = (int32_t)h.ph; pa.pw = (int32_t)h.pw;
    const bool nhwc = h.xs[1] == 1 && h.xs[3] == h.C && h.xs[2] == h.W * h.C && h.xs[0] == h.H * h.W * h.C &&
                      Hp <= 65535 && h.N * ((h.C + 63) / 64) <= 65535;
    if (nhwc) {
        hipLaunchKernelGGL(conv_pad_nhwc_kernel, dim3((unsigned)((Wp + 31) / 32), (unsigned)Hp, (unsigned)(h.N * ((h.C + 63) / 64))), dim3(256), 0,
                           (hipStream_t)g.stream, pa);
    } else {
        const int64_t blocks = std::min<int64_t>(((total + 7) / 8 + 255) / 256, 1 << 20);
        hipLaunchKernelGGL(conv_pad_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)g.stream, pa);
    }
    { const nt_status lst = check_launch("conv_pad_kernel"); if (lst != NT_OK) return lst; }
    g2.A = P;
    return launch_gemm(g2, path_out);
}

// ---- route 3: any other convolution on the library's own tile: the unfolded input is written out once (if it fits the
// workspace) and the product runs per image on the MFMA kernels, Y[n] (filters x positions) = W (filters x CRS) .
// U[:, n] (CRS x positions) -- far faster than gathering every element of every tile through the operand map.
static nt_status route_conv_unfold(const GemmLaunch &g, int *path_out, bool *taken)
{
    *taken = false;
    const ConvHint &h = g.conv;
    if (!(conv_is_bare(g) && h.ys[3] == 1 && h.ys[2] == h.Q && h.ws[3] == 1 && h.ws[2] == h.S && h.ws[1] == h.R * h.S && h.ws[0] >= h.C * h.R * h.S &&
          h.ws[0] < (1 << 22) && h.N * h.C * h.H * h.W > 0 && (h.N - 1) * h.xs[0] + (h.H - 1) * h.xs[2] + (h.W - 1) * h.xs[3] < (1LL << 31) &&
          h.xs[0] >= 0 && h.xs[2] >= 0 && h.xs[3] >= 0 && h.P * h.Q >= 8 && h.C * h.R * h.S >= 8 && h.C * h.R * h.S <= 65535))
        return NT_OK;
    const int64_t K = h.C * h.R * h.S, PQ = h.P * h.Q, M = h.N * PQ, Mp = (M + 7) / 8 * 8;
    if (Mp >= (1 << 22)) return NT_OK;
    WorkspaceLease lease;
    uint16_t *U = (uint16_t *)lease.acquire((size_t)K * Mp * 2, (hipStream_t)g.stream);
    if (!U) return NT_OK;
    *taken = true;
    hipStream_t s = (hipStream_t)g.stream;
    UnfoldArgs ua{};
    ua.x = (const uint16_t *)g.A; ua.U = U;
    for (int d = 0; d < 4; ++d) ua.xs[d] = h.xs[d];
    ua.M = M; ua.Mp = Mp; ua.K = K;
    ua.C = (int32_t)h.C; ua.H = (int32_t)h.H; ua.W = (int32_t)h.W; ua.R = (int32_t)h.R; ua.S = (int32_t)h.S;
    ua.P = (int32_t)h.P; ua.Q = (int32_t)h.Q; ua.sh = (int32_t)h.sh; ua.sw = (int32_t)h.sw; ua.ph = (int32_t)h.ph; ua.pw = (int32_t)h.pw;
    ua.dh = (int32_t)h.dh; ua.dw = (int32_t)h.dw;
    const int64_t blocks = std::min<int64_t>((Mp / 8 + 255) / 256, 1 << 16);
    hipLaunchKernelGGL(conv_unfold_kernel, dim3((unsigned)blocks, (unsigned)K), dim3(256), 0, s, ua);
    { const nt_status lst = check_launch("conv_unfold_kernel"); if (lst != NT_OK) return lst; }
    auto matrix = [](int64_t rows, int64_t cols, int64_t row_pitch) {
        OperandMap m{};
        m.rows = rows; m.cols = cols; m.base = 0; m.nrd = 1; m.ncd = 1; m.nchk = 0;
        m.rrad[0] = rows; m.crad[0] = cols; m.roff[0] = row_pitch; m.coff[0] = 1;
        return m;
    };
    GemmLaunch u{};
    u.A = g.B; u.B = U; u.C = g.C;
    u.ma = matrix(h.K, K, h.ws[0]);                      // filters x CRS
    u.mb = matrix(K, PQ, Mp);                            // CRS x the image's positions
    u.mc = matrix(h.K, PQ, h.ys[1]);                     // filters x positions
    u.batch = h.N; u.sa_batch = 0; u.sb_batch = PQ; u.sc_batch = h.ys[0];
    u.M = h.K; u.N = PQ; u.K = K;
    u.tile = pick_gemm_tile(u.batch, u.M, u.N, u.K);
    u.mt = (u.M + u.tile.bm - 1) / u.tile.bm; u.nt = (u.N + u.tile.bn - 1) / u.tile.bn; u.kt = (u.K + u.tile.bk - 1) / u.tile.bk;
    u.in_dtype = g.in_dtype; u.out_dtype = g.out_dtype; u.stream = g.stream;
    u.alpha = 1.f; u.beta = 0.f; u.act = 0; u.has_d = false;
    u.no_workspace = true;                               // (this route holds the workspace)
    const nt_status st = launch_gemm(u, nullptr);
    if (path_out) *path_out = PATH_CONV_UNFOLD;
    return st;
}

// Plain operands, each with unit stride along one of its axes, on a tile the MFMA kernels are built for: the arguments
// of those kernels.  false: the operand-map kernel takes the launch.
static bool lower_plain(const GemmLaunch &g, FastArgs *out, int *alay_out, int *blay_out)
{
    const nt_tile_cfg t = g.tile;
    if (!(plain(g.ma) && plain(g.mb) && plain(g.mc) && (!g.has_d || plain(g.md)) && t.bk == 64 && t.bm >= 128 && t.bn >= 128 && g.kt > 0)) return false;
    FastArgs a{};
    int alay, blay;
    if (g.ma.coff[0] == 1) { alay = KCONTIG; a.lda = g.ma.roff[0]; }
    else if (g.ma.roff[0] == 1) { alay = MNCONTIG; a.lda = g.ma.coff[0]; }
    else return false;
    if (g.mb.coff[0] == 1) { blay = MNCONTIG; a.ldb = g.mb.roff[0]; }
    else if (g.mb.roff[0] == 1) { blay = KCONTIG; a.ldb = g.mb.coff[0]; }
    else return false;
    if (a.lda < 0 || a.ldb < 0 || a.lda >= (1 << 22) || a.ldb >= (1 << 22)) return false;   // 32-bit lane offsets
    // the staged loader fetches a block that straddles the ragged end of the contiguous
    // axis up to 7 elements early: that axis must be at least one block (8 elements) long
    if ((alay == MNCONTIG ? g.M : g.K) < 8 || (blay == MNCONTIG ? g.N : g.K) < 8) return false;
    const int64_t esz = g.out_dtype == NT_F32 ? 4 : 2;
    a.A = (const uint16_t *)g.A + g.ma.base;
    a.B = (const uint16_t *)g.B + g.mb.base;
    a.C = (char *)g.C + g.mc.base * esz;
    a.scm = g.mc.roff[0];
    a.scn = g.mc.coff[0];
    a.sa_batch = g.sa_batch; a.sb_batch = g.sb_batch; a.sc_batch = g.sc_batch;
    a.M = g.M; a.N = g.N; a.K = g.K;
    a.mt = g.mt; a.nt = g.nt; a.kt = g.kt;
    a.out_dtype = g.out_dtype;
    a.alpha = g.alpha;
    a.beta = g.has_d ? g.beta : 0.f;
    a.act = g.act;
    // bounds of the range-checked loads (the pitches are below 2^22, so every offset inside a tile's footprint fits 32 bits)
    a.a_extent = (alay == KCONTIG ? (g.M - 1) * a.lda + g.K : (g.K - 1) * a.lda + g.M) * 2;
    a.b_extent = (blay == KCONTIG ? (g.N - 1) * a.ldb + g.K : (g.K - 1) * a.ldb + g.N) * 2;
    if (g.has_d) {
        a.D = (const char *)g.D + g.md.base * esz;
        a.sdm = g.md.roff[0];
        a.sdn = g.md.coff[0];
        a.sd_batch = g.sd_batch;
    }
    *out = a;
    *alay_out = alay;
    *blay_out = blay;
    return true;
}

// ---- route 4: plain matrices on the MFMA kernels (with the k split for skinny products)
static nt_status route_matrix(const GemmLaunch &g, FastArgs a, int alay, int blay, int *path_out)
{
    const nt_tile_cfg t = g.tile;
    const bool bf16 = g.in_dtype == NT_BF16;
    const int64_t nwg = g.batch * g.mt * g.nt;
    hipStream_t s = (hipStream_t)g.stream;
    // Operands stored to a C (and added to a D) with unit stride along n stream straight into LDS.  Full tiles of
    // 16-byte aligned operands: plain loads.  Everything else -- tiles that overhang M or N, a ragged K, rows with
    // only the element's 2-byte alignment -- takes the same loads as range-checked buffer accesses (EDGE kernels),
    // which needs every offset inside a tile's footprint to fit 32 bits.  The range check works on the 4-byte words
    // of a load, counted from the load's own start: with an odd pitch, or an extent that is no multiple of 4 bytes,
    // the word that holds the operand's last element can end 2 bytes past it and is then dropped; the kernel is told
    // (patch) and fetches that one element by itself.  The range never extends past the operand.
    const bool ragged_mn = (g.M % t.bm) || (g.N % t.bn), ragged_k = (g.K % t.bk) != 0;
    auto al16 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
    const bool out_ok = a.scn == 1 && (!a.D || a.sdn == 1);
    const bool aligned = al16(a.A) && al16(a.B) && a.lda % 8 == 0 && a.ldb % 8 == 0 && a.sa_batch % 8 == 0 && a.sb_batch % 8 == 0;
    const bool plain_direct = out_ok && aligned && !ragged_k && !ragged_mn;
    auto words_aligned = [&](int64_t ld, int64_t s_batch, int64_t extent) {      // every word of every load lies at a multiple of 4 bytes from the operand's start
        return extent % 4 == 0 && ld % 2 == 0 && s_batch % 2 == 0;
    };
    const bool direct = plain_direct || (out_ok && (alay == KCONTIG || g.K * a.lda < (1LL << 30)) && (blay == KCONTIG || g.K * a.ldb < (1LL << 30)));
    if (direct && !plain_direct)
        a.patch = (words_aligned(a.lda, a.sa_batch, a.a_extent) ? 0 : 1) | (words_aligned(a.ldb, a.sb_batch, a.b_extent) ? 0 : 2);
    if (path_out) *path_out = direct ? PATH_DIRECT : PATH_FAST;
    if (g.trace.out) {
        if (!direct) return fail(NT_ERR_UNSUPPORTED, "this product does not run on the kernels that stream their operands into LDS");
        const int64_t rows = g.trace.operand == 0 ? t.bm : t.bn;
        if ((size_t)rows * 32 > g.trace.capacity) return fail(NT_ERR_BUFFER_TOO_SMALL, "trace buffer smaller than the slice");
        if (g.trace.program < 0 || g.trace.program >= nwg) return fail(NT_ERR_INVALID_ARG, "program_id outside the grid");
        if (g.trace.slice < 0 || g.trace.slice >= (g.K + 31) / 32) return fail(NT_ERR_INVALID_ARG, "slice outside the reduction");
        a.trace_out = g.trace.out; a.trace_program = g.trace.program; a.trace_slice = g.trace.slice; a.trace_operand = g.trace.operand;
        return launch_direct16_trace(a, t.bm, t.bn, alay, blay, !plain_direct, s);
    }
    typedef nt_status (*Launcher)(const FastArgs &, int, int, int64_t, hipStream_t);
    // [f16, bf16]; direct: full aligned tiles (the kernel on 16 x 16 x 32 matrix instructions: fewer accumulator bits moved per
    // flop, which on this power-managed part is clock), edge: the range-checked flavour, staged: through registers
    struct Entry { int bm, bn; Launcher direct[2], edge[2], staged[2]; };
#define NT_ENTRY(BM, BN, T) {BM, BN, {launch_direct16_##T##_f16, launch_direct16_##T##_bf16}, {launch_direct16_edge_##T##_f16, launch_direct16_edge_##T##_bf16}, \
                             {launch_fast_##T##_f16, launch_fast_##T##_bf16}}
    static const Entry table[] = {NT_ENTRY(128, 128, 128x128), NT_ENTRY(256, 128, 256x128), NT_ENTRY(128, 256, 128x256), NT_ENTRY(256, 256, 256x256)};
#undef NT_ENTRY
    for (const Entry &e : table) {
        if (e.bm != t.bm || e.bn != t.bn) continue;
        const Launcher launch = (direct ? (plain_direct ? e.direct : e.edge) : e.staged)[bf16 ? 1 : 0];
        // k split: `ksplit` equal parts of K as the entries of a batched product into fp32 slices of the workspace
        const int ksplit = g.batch == 1 && !ragged_k ? gemm_ksplit(g.mt * g.nt, g.kt, g.M, g.N) : 1;
        WorkspaceLease lease;
        float *ws = nullptr;                                 // (none: too large, or no memory; then no split)
        if (ksplit > 1) {
            nt_status st;
            ws = split_region(g, (size_t)ksplit * g.M * g.N * 4, lease, &st);
            if (st != NT_OK) return st;
        }
        if (!ws) return launch(a, alay, blay, nwg, s);
        t_k_split = ksplit;
        FastArgs part = a;
        const int64_t Kp = g.K / ksplit;
        part.K = Kp; part.kt = g.kt / ksplit;
        part.sa_batch = alay == KCONTIG ? Kp : Kp * a.lda;
        part.sb_batch = blay == KCONTIG ? Kp : Kp * a.ldb;
        // (K and Kp are multiples of 64: a part's words are as aligned as the whole's, and a part is as streamable)
        part.a_extent = (alay == KCONTIG ? (g.M - 1) * a.lda + Kp : (Kp - 1) * a.lda + g.M) * 2;
        part.b_extent = (blay == KCONTIG ? (g.N - 1) * a.ldb + Kp : (Kp - 1) * a.ldb + g.N) * 2;
        part.C = ws; part.scm = g.N; part.scn = 1; part.sc_batch = g.M * g.N; part.out_dtype = NT_F32;
        part.D = nullptr; part.alpha = 1.f; part.beta = 0.f; part.act = 0;
        const nt_status st = launch(part, alay, blay, nwg * ksplit, s);
        if (st != NT_OK) return st;
        const int64_t blocks = std::min<int64_t>((g.M * g.N + 255) / 256, 4096);
        hipLaunchKernelGGL(splitk_sum_kernel, dim3((unsigned)blocks), dim3(256), 0, s, ws, ksplit, g.M, g.N, a.C, a.scm, a.scn, a.out_dtype,
                           (const void *)a.D, a.sdm, a.sdn, a.alpha, a.beta, a.act);
        return check_launch("splitk_sum_kernel");
    }
    return fail(NT_ERR_UNSUPPORTED, "no fast kernel for this tile");
}

nt_status launch_gemm(const GemmLaunch &g, int *path_out)
{
    if (!g.no_workspace || g.ws_strict) t_k_split = 1;
    if (g.batch * g.mt * g.nt > 0x7fffffffLL) return fail(NT_ERR_UNSUPPORTED, "grid too large");
    FastArgs a{};
    int alay = KCONTIG, blay = MNCONTIG;
    if (lower_plain(g, &a, &alay, &blay)) return route_matrix(g, a, alay, blay, path_out);
    if (path_out) *path_out = PATH_GENERIC;
    ConvArgs c{};
    if (!g.has_d && g.alpha == 1.f && g.act == 0 && match_conv(g, &c)) return route_conv_implicit(g, c, path_out);
    if (g.trace.out) return fail(NT_ERR_UNSUPPORTED, "this launch does not run on the kernels that stream their operands into LDS");
    bool taken = false;
    nt_status st = route_conv_padded_copy(g, path_out, &taken);
    if (taken || st != NT_OK) return st;
    st = route_conv_unfold(g, path_out, &taken);
    if (taken || st != NT_OK) return st;
    return launch_generic(g);
}

nt_status launch_fill_zero(void *C, const OperandMap &mc, int64_t batch, int64_t sc_batch, int out_dtype, void *stream)
{
    const int64_t total = mc.rows * mc.cols;
    if (total <= 0 || batch <= 0) return NT_OK;
    const int64_t blocks = std::min<int64_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks, (unsigned)std::min<int64_t>(batch, 1024)), dim3(256), 0, (hipStream_t)stream,
                       C, mc, batch, sc_batch, out_dtype);
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
