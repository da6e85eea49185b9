// Pieces shared by the kernels whose operand blocks travel from global memory straight into LDS (gemm_direct16.h,
// gemm_conv_direct.h): the size of a slice and of the ring of slices, the wait for outstanding loads, and the global -> LDS
// load itself, plain or range checked.
//
// A direct-to-LDS load always writes lane l's 16 bytes to (instruction base + 16 l), so a bank swizzle of the LDS layout is
// applied on the global side: lane l fetches the chunk that belongs in its slot.
#pragma once
#include <type_traits>

#include "gemm_fast.h"

namespace nt {

typedef short short4v __attribute__((ext_vector_type(4)));

constexpr int kSliceK = 32;      // k extent of one LDS slice
// Slices per operand resident in LDS, and workgroups the kernel is built to co-reside on a
// compute unit.  The 256 x 256 tile needs every accumulator register of its wavefronts (one
// workgroup per unit, ring of four = 128 KB).  Smaller tiles leave room for two workgroups
// per unit (at most 72 KB and 256 registers each), whose epilogues, launches and prologues
// then overlap the other's multiplications; their ring is three slices (256 x 128: 72 KB) or
// four (128 x 128: 64 KB).
constexpr int ring_of(int bm, int bn) { return bm + bn == 384 || bm + bn == 320 ? 3 : 4; }   // (320: the convolution kernel's 256 x 64, 60 KB)
constexpr int residency_of(int bm, int bn) { return bm + bn == 512 ? 1 : 2; }

// s_waitcnt that waits until at most n vector-memory operations are outstanding and leaves
// the other counters alone (vmcnt is split over bits [3:0] and [15:14] of the immediate)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }
#define NT_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(vmcnt_imm(n))

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at
// lds_addr + 16 l.  gbase and lds_addr are wavefront-uniform, voff is the lane's byte offset.
// Issued through inline assembly so that the compiler does not serialise later LDS reads of
// other slices behind it; completion is awaited explicitly with NT_WAIT_VMCNT.
__device__ __forceinline__ void dma16(const char *gbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(gbase)
                 : "memory");   // m0 is not otherwise used by these kernels
}

// The same through a range-checked buffer access: rsrc describes the memory from the program's tile origin to the
// operand's end, soff (wavefront-uniform) and voff are byte offsets into it; 4-byte words that do not lie wholly
// inside it arrive in LDS as zeros instead of being fetched.  Lets tiles on the ragged m / n edge use the same loads.
__device__ __forceinline__ void dma16_buf(u32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory");
}

// buffer resource (raw, no swizzle) over `bytes` bytes at p; all words wavefront-uniform
__device__ __forceinline__ u32x4 make_rsrc(const void *p, int64_t bytes)
{
    const uint64_t b = reinterpret_cast<uint64_t>(p);
    const uint32_t n = bytes < 0x7fffffffLL ? (uint32_t)bytes : 0x7fffffffu;
    return u32x4{(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b), (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((b >> 32) & 0xffffu)),
                 (uint32_t)__builtin_amdgcn_readfirstlane((int)n), 0x00020000u};
}

}  // namespace nt
