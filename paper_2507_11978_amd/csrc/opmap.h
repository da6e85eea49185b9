// Device-visible form of one arranged matrix operand (source-to-target mapping,
// Section 3.2.2, after lowering): element (row, col) of the logical matrix view lives at
//   offset = base + sum_i roff[i] * rdigit[i] + sum_j coff[j] * cdigit[j]
// where the digits are the mixed-radix decomposition of row / col (digit 0 slowest, the
// others bounded by rrad / crad).  The element is valid (unmasked) iff row < rows,
// col < cols and every checked source coordinate
//   x_q = chk0[q] + sum_i rchk[q][i] * rdigit[i] + sum_j cchk[q][j] * cdigit[j]
// lies in [0, chk_size[q]).  A plain strided matrix has one digit per axis and no checked
// coordinate; the implicit-GEMM input of a convolution (Section 4.3) has digits (n,p,q) and
// (c,r,s) and checks h and w.
#pragma once
#include <cstdint>

#ifndef NT_HD
#ifdef __HIPCC__
#include <hip/hip_runtime.h>
#define NT_HD __host__ __device__ __forceinline__
#else
#define NT_HD inline
#endif
#endif

namespace nt {

constexpr int kMaxDigits = 3;
constexpr int kMaxChecks = 4;

struct OperandMap {
    int64_t rows, cols;
    int64_t base;
    int32_t nrd, ncd;
    int32_t nchk;
    int32_t reserved;
    int64_t rrad[kMaxDigits], crad[kMaxDigits];
    int64_t roff[kMaxDigits], coff[kMaxDigits];
    int32_t rchk[kMaxChecks][kMaxDigits], cchk[kMaxChecks][kMaxDigits];
    int32_t chk0[kMaxChecks], chk_size[kMaxChecks];
};

// Contribution of one axis index to the offset and to the checked coordinates.
struct AxisPart {
    int64_t off;
    int32_t chk[kMaxChecks];
};

// (Loops run over the fixed capacities with the live counts as predicates: every array index is then a
// compile-time constant and the map stays in scalar registers on the device.)
NT_HD AxisPart axis_part(int64_t idx, int nd, const int64_t *rad, const int64_t *off,
                         const int32_t (*chk)[kMaxDigits], int nchk)
{
    AxisPart p;
    p.off = 0;
    for (int q = 0; q < kMaxChecks; ++q) p.chk[q] = 0;
    int64_t rem = idx;
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
#endif
    for (int i = kMaxDigits - 1; i >= 0; --i) {
        if (i < nd) {
            int64_t d = rem;
            if (i > 0) {
                d = rem % rad[i];
                rem = rem / rad[i];
            }
            p.off += d * off[i];
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
#endif
            for (int q = 0; q < kMaxChecks; ++q)
                if (q < nchk) p.chk[q] += (int32_t)d * chk[q][i];
        }
    }
    return p;
}

NT_HD AxisPart row_part(const OperandMap &m, int64_t row)
{
    return axis_part(row, m.nrd, m.rrad, m.roff, m.rchk, m.nchk);
}

NT_HD AxisPart col_part(const OperandMap &m, int64_t col)
{
    return axis_part(col, m.ncd, m.crad, m.coff, m.cchk, m.nchk);
}

// Combine the two axis contributions: returns validity, writes the element offset.
NT_HD bool element_at(const OperandMap &m, int64_t row, int64_t col, const AxisPart &r, const AxisPart &c,
                      int64_t *offset)
{
    bool ok = row < m.rows && col < m.cols;
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
#endif
    for (int q = 0; q < kMaxChecks; ++q) {
        const int32_t x = m.chk0[q] + r.chk[q] + c.chk[q];
        ok = ok && (q >= m.nchk || (x >= 0 && x < m.chk_size[q]));
    }
    *offset = m.base + r.off + c.off;
    return ok;
}

}  // namespace nt
