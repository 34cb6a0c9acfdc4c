// Cutting an fp32 value into three bf16 pieces, shared by the kernels that multiply fp32 operands on the
// bf16 matrix cores (igemm_f32_p3.hip, conv_pw_f32.hip).
//
//   x = hi + mid + lo exactly: mask off the upper 16 bits of the word (a bf16 with eight significant bits,
//   truncated, so it never overflows), subtract (exact), repeat; what is left after two steps has at most
//   eight significant bits and is a bf16 as it stands.  A product x*y is then taken as the six piece
//   products down to weight 2^-16 -- hi*hi, hi*mid, mid*hi, mid*mid, hi*lo, lo*hi -- which
//   v_mfma_f32_32x32x16_bf16 multiplies exactly and accumulates in fp32.  Dropped: mid*lo, lo*mid, lo*lo,
//   together below 2^-22 of |x*y|, the size of the rounding an fp32 multiply-add makes anyway.
#pragma once
#include <hip/hip_runtime.h>

namespace glowmi {

typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

struct Pieces { unsigned h, m, l; };     // each piece's bf16 is the upper half of the word
__device__ __forceinline__ Pieces split3(float x) {
  Pieces r;
  r.h = __builtin_bit_cast(unsigned, x) & 0xffff0000u;
  const float r1 = x - __builtin_bit_cast(float, r.h);
  r.m = __builtin_bit_cast(unsigned, r1) & 0xffff0000u;
  r.l = __builtin_bit_cast(unsigned, r1 - __builtin_bit_cast(float, r.m));   // eight significant bits: already a bf16
  return r;
}
// the upper halves of two words side by side: a in the low half (earlier index), b in the high half
__device__ __forceinline__ unsigned pack_upper(unsigned a, unsigned b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// eight consecutive values -> eight bf16 (16 bytes) per piece
__device__ __forceinline__ void split8(const float (&v)[8], v4u& h, v4u& m, v4u& l) {
  Pieces e[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) e[i] = split3(v[i]);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    h[i] = pack_upper(e[2 * i].h, e[2 * i + 1].h);
    m[i] = pack_upper(e[2 * i].m, e[2 * i + 1].m);
    l[i] = pack_upper(e[2 * i].l, e[2 * i + 1].l);
  }
}

// (input piece, filter piece) of the six products, smallest first
constexpr int kPieceTermA[6] = {2, 0, 1, 1, 0, 0};
constexpr int kPieceTermB[6] = {0, 2, 1, 0, 1, 0};

}  // namespace glowmi
