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

// The same for shift in [33, 54] with the rounding constant and the output offset folded into one
// addend  K = 2^(shift-33) + y_off * 2^(shift-32):
//   ((hi + 2^(shift-33)) >> (shift-32)) + y_off == (hi + K) >> (shift-32)
// exactly (a multiple of 2^(shift-32) added before an arithmetic shift adds that multiple of one
// after it), and |hi| < 2^30, |K| < 2^30, so the sum cannot overflow.  The clamp to [lo, 127] is one
// median-of-three; the compiler does not form it from a variable lower bound, hence the asm (VOP3
// reads at most one scalar register here, so `lo` comes in a vector register).
struct FoldedRequant {
  int s, K;           // shift - 32, folded addend
  bool ok;            // shift in [33, 54]
};
__device__ __forceinline__ FoldedRequant make_folded_requant(int shift, int y_off) {
  FoldedRequant f;
  f.ok = shift >= 33 && shift <= 54;
  f.s = f.ok ? shift - 32 : 1;
  f.K = (1 << (f.s - 1)) + y_off * (1 << f.s);
  return f;
}
__device__ __forceinline__ int requantize_folded(int acc, int mant, const FoldedRequant& f, int lo_vgpr) {
  const int q = (__mulhi(acc, mant) + f.K) >> f.s;
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(q), "v"(lo_vgpr), "s"(127));
  return r;
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
