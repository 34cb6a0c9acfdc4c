// Device-side pieces of the quantized epilogue shared by the int8 kernels: the integer rescale of
// an int32 accumulator to the output's scale/offset (the rescale the paper folds into the producing
// operation, Section 4.3) with Relu as the lower clamp bound, and packing of codes into dwords.
#pragma once
#include <hip/hip_runtime.h>

namespace glowmi {

// round_half_up(acc * mant / 2^shift) + y_off, clamped to [lo, 127].
// With P = acc * mant = hi * 2^32 + lo32 and shift >= 33 the rounding constant 2^(shift-1) is a
// multiple of 2^32, so (P + 2^(shift-1)) >> shift == (hi + 2^(shift-33)) >> (shift-32) exactly:
// one 32-bit multiply-high instead of 64-bit arithmetic.  That covers every multiplier below 1/4
// (the usual case); larger multipliers take the 64-bit form.  FAST is uniform over a launch.
template <bool FAST>
__device__ __forceinline__ int requantize_as(int acc, int mant, int shift, int y_off, int lo) {
  int q;
  if (FAST) {
    q = (__mulhi(acc, mant) + (1 << (shift - 33))) >> (shift - 32);
  } else {
    long long t = (long long)acc * (long long)mant + (1LL << (shift - 1));
    t >>= shift;                            // arithmetic shift: floor, so ties round up
    t = t < -4096 ? -4096 : t;              // far outside the int8 range either way
    t = t > 4096 ? 4096 : t;
    q = (int)t;
  }
  q += y_off;
  q = q < lo ? lo : q;
  q = q > 127 ? 127 : q;
  return q;
}

// round_half_up(d * mant / 2^shift): a quantized addend's code difference d = r - r_offset brought
// to the accumulator's scale (the rescale node of Section 4.3 in front of the add), shift in [1, 62].
__device__ __forceinline__ int rescale_term(int d, int mant, int shift) {
  const long long t = (long long)d * (long long)mant + (1LL << (shift - 1));
  return (int)(t >> shift);                 // arithmetic shift: floor, so ties round up
}

// the low bytes of four ints as one dword, a in the lowest byte
__device__ __forceinline__ unsigned pack_codes(int a, int b, int c, int d) {
  const unsigned ab = __builtin_amdgcn_perm((unsigned)b, (unsigned)a, 0x0c0c0400u);
  const unsigned cd = __builtin_amdgcn_perm((unsigned)d, (unsigned)c, 0x0c0c0400u);
  return __builtin_amdgcn_perm(cd, ab, 0x05040100u);
}

}  // namespace glowmi
