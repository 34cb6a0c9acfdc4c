// Loads that go from global memory straight into LDS (buffer loads with the LDS bit) and the pieces
// around them, shared by the kernels that stage their operands this way (igemm_i8_wide.hip,
// igemm_f32_p3.hip).
#pragma once
#include <hip/hip_runtime.h>

namespace glowmi {

typedef int v4i __attribute__((ext_vector_type(4)));

#define GLOWMI_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))

// 16 bytes per lane from a range-checked buffer straight into LDS at lds_addr + 16 * lane (lanes whose
// offset is out of range write zeros).  Issued as inline assembly on purpose: for the intrinsic form
// the compiler cannot tell which later LDS reads depend on which load and waits for all outstanding
// loads before every LDS read, which would serialise the ring of slab buffers; here the kernel
// places the vmcnt waits itself.  lds_addr is wave-uniform.
__device__ __forceinline__ void load16_to_lds(v4i rsrc, unsigned lds_addr, unsigned voffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :
               : "s"(lds_addr), "v"(voffset), "s"(rsrc)
               : "memory");   // m0 is written here and nowhere else in the kernels that use this header
                              // (it is a reserved register: the compiler warns about it on a clobber list
                              // and keeps nothing live in it in a kernel without LDS-direct intrinsics)
}

__device__ __forceinline__ v4i make_rsrc(const void* base, unsigned bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(base);
  v4i r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
  r[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((a >> 32) & 0xffffu));   // stride 0: raw buffer
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);                              // num_records in bytes
  r[3] = 0x00020000;
  return r;
}

__device__ __forceinline__ unsigned lds_offset_of(const void* p) {
  return (unsigned)(unsigned long long)GLOWMI_LDS_PTR(p);
}

// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding and
// leaves the other counters alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8).
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

}  // namespace glowmi
