// Instantiations of the generic (operand-map driven) kernel for every built tile.
#include "gemm_device.h"

namespace nt {

template <int BM, int BN, int BK>
static nt_status launch_generic_t(const GemmLaunch &g)
{
    const dim3 grid((unsigned)(g.batch * g.mt * g.nt));
    hipStream_t s = (hipStream_t)g.stream;
    if (g.in_dtype == NT_BF16)
        hipLaunchKernelGGL((gemm_generic_kernel<BM, BN, BK, true>), grid, dim3(kThreads), 0, s,
                           (const uint16_t *)g.A, (const uint16_t *)g.B, g.C, g.ma, g.mb, g.mc,
                           g.sa_batch, g.sb_batch, g.sc_batch, g.mt, g.nt, g.kt, g.out_dtype,
                           g.has_d ? g.D : nullptr, g.md, g.sd_batch, g.alpha, g.beta, g.act);
    else
        hipLaunchKernelGGL((gemm_generic_kernel<BM, BN, BK, false>), grid, dim3(kThreads), 0, s,
                           (const uint16_t *)g.A, (const uint16_t *)g.B, g.C, g.ma, g.mb, g.mc,
                           g.sa_batch, g.sb_batch, g.sc_batch, g.mt, g.nt, g.kt, g.out_dtype,
                           g.has_d ? g.D : nullptr, g.md, g.sd_batch, g.alpha, g.beta, g.act);
    return check_launch("gemm_generic_kernel");
}

nt_status launch_generic(const GemmLaunch &g)
{
    const nt_tile_cfg t = g.tile;
    if (t.bm == 64 && t.bn == 64 && t.bk == 32) return launch_generic_t<64, 64, 32>(g);
    if (t.bm == 128 && t.bn == 128 && t.bk == 64) return launch_generic_t<128, 128, 64>(g);
    if (t.bm == 256 && t.bn == 128 && t.bk == 64) return launch_generic_t<256, 128, 64>(g);
    if (t.bm == 128 && t.bn == 256 && t.bk == 64) return launch_generic_t<128, 256, 64>(g);
    if (t.bm == 256 && t.bn == 256 && t.bk == 64) return launch_generic_t<256, 256, 64>(g);
    return fail(NT_ERR_UNSUPPORTED, "tile shape not built");
}

}  // namespace nt
