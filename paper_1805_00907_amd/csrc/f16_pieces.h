// Cutting an fp32 tensor into two fp16 planes, shared by the kernels that multiply fp32 operands on the
// fp16 matrix cores with three piece products per fp32 product (igemm_f32_p3.hip, conv_k3_f32.hip,
// conv_k3v_f32.hip, conv_k3c64_f32.hip).
//
//   A tensor gets one power-of-two scale 2^se chosen from its largest magnitude so that the scaled values
//   stay below 2^15 (se = 141 - biased exponent of the largest magnitude; scaling by a power of two is
//   exact).  A scaled value v is cut into
//       h1 = fp16(v)                      (round to nearest: 11 significant bits)
//       H2 = fp16((v - h1) * 2^11)        (the remainder, exact in fp32, scaled up so that it keeps fp16's
//                                          normal range wherever h1 does; 11 more bits)
//   so v = h1 + 2^-11 H2 up to 2^-22 |v| (each piece rounds at half a unit of its 11th bit; typically a quarter
//   of that).  A product of two such values is taken as
//       h1 h1'  +  2^-11 (h1 H2' + H2 h1')
//   with v_mfma_f32_32x32x16_f16, which multiplies fp16 exactly and accumulates in fp32: the first term into
//   one accumulator set, the two cross terms into a second one that is scaled by 2^-11 and added at the end,
//   and the sum is scaled back by 2^-(se + se').  Dropped: 2^-22 H2 H2', at most 2^-22 of |v v'|; with the cuts'
//   own rounding a product is within 3 * 2^-22 of |v v'| in the worst case, a few times the rounding an fp32
//   multiply-add makes anyway and far below what accumulating a long reduction in fp32 adds.
//   Values more than 2^28 below the tensor's largest magnitude fall under fp16's normal range after scaling;
//   they are carried by H2 alone (h1 = 0) with 11 significant bits, an absolute error below 2^-39 of the
//   largest magnitude, and the product of two such values (one from each operand, below 2^-56 of the largest
//   product) is dropped.
#pragma once
#include <hip/hip_runtime.h>

namespace glowmi {

typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

constexpr float kLowPieceWeight = 0x1p-11f;            // weight of the second accumulator set

// Scale exponent of a tensor from the bits of its largest magnitude (sign cleared).
__device__ __forceinline__ int scale_exponent(unsigned max_bits) {
  int eb = (int)(max_bits >> 23) & 0xff;
  if (eb < 1) eb = 1;                                  // all zero (or subnormal): any scale will do
  return 141 - eb;
}

// Largest of n words at src, by one wavefront on its own (no LDS, no barrier); every lane returns it.
__device__ __forceinline__ unsigned wave_max_words(const unsigned* __restrict__ src, int n) {
  unsigned m = 0;
  for (int i = (int)(threadIdx.x & 63); i < n; i += 64) {
    const unsigned v = src[i];
    m = v > m ? v : m;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const unsigned o = (unsigned)__shfl_xor((int)m, d, 64);
    m = o > m ? o : m;
  }
  return (unsigned)__builtin_amdgcn_readfirstlane((int)m);
}

// Largest magnitude (bits) among 8 * N prefetched values held as N pairs of float4, over the whole wavefront.
template <int N, typename V4>
__device__ __forceinline__ unsigned wave_max_of(const V4 (&pre)[N][2]) {
  unsigned m = 0;
#pragma unroll
  for (int q = 0; q < N; ++q)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const unsigned b = __builtin_bit_cast(unsigned, pre[q][h][e]) & 0x7fffffffu;
        m = b > m ? b : m;
      }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const unsigned o = (unsigned)__shfl_xor((int)m, d, 64);
    m = o > m ? o : m;
  }
  return (unsigned)__builtin_amdgcn_readfirstlane((int)m);
}

// The largest of the eight words the wavefronts of a workgroup left at `words` (LDS).
__device__ __forceinline__ unsigned max_of_eight(const unsigned* words) {
  const v4u a = *reinterpret_cast<const v4u*>(words), b = *reinterpret_cast<const v4u*>(words + 4);
  unsigned m = a[0];
#pragma unroll
  for (int e = 1; e < 4; ++e) m = a[e] > m ? a[e] : m;
#pragma unroll
  for (int e = 0; e < 4; ++e) m = b[e] > m ? b[e] : m;
  return (unsigned)__builtin_amdgcn_readfirstlane((int)m);
}

struct Cut2 { _Float16 h1, h2; };
__device__ __forceinline__ Cut2 cut2(float x, int se) {
  const float v = __builtin_ldexpf(x, se);
  _Float16 h1 = (_Float16)v;
  if (__builtin_fabsf(v) < 0x1p-14f) h1 = (_Float16)0.f;   // below fp16's normal range: the second piece carries it
  const float r = v - (float)h1;
  Cut2 c;
  c.h1 = h1;
  c.h2 = (_Float16)(r * 2048.f);
  return c;
}

// eight consecutive values -> eight fp16 (16 bytes) per piece
__device__ __forceinline__ void cut8(const float (&v)[8], int se, v4u& p1, v4u& p2) {
  Cut2 e[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) e[i] = cut2(v[i], se);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    p1[i] = __builtin_bit_cast(unsigned, v2h{e[2 * i].h1, e[2 * i + 1].h1});
    p2[i] = __builtin_bit_cast(unsigned, v2h{e[2 * i].h2, e[2 * i + 1].h2});
  }
}

// The two operands' largest magnitudes (bits) -> what the accumulators are scaled back by, and what is added to
// every result: 0, or NaN when an operand holds an infinity or a NaN (its largest "magnitude" is then not finite and
// no scale fits: the whole call's results are NaN rather than finite numbers that are wrong).
struct ScaleBack { int neg_se; float poison; };
__device__ __forceinline__ ScaleBack scale_back(unsigned x_max_bits, unsigned w_max_bits) {
  ScaleBack s;
  s.neg_se = -(scale_exponent(x_max_bits) + scale_exponent(w_max_bits));
  const bool finite = x_max_bits < 0x7f800000u && w_max_bits < 0x7f800000u;
  s.poison = finite ? 0.f : __builtin_nanf("");
  return s;
}
// The same from the scale exponents in use and whether every magnitude seen was finite.
__device__ __forceinline__ ScaleBack scale_back_of(int se_x, int se_w, bool finite) {
  ScaleBack s;
  s.neg_se = -(se_x + se_w);
  s.poison = finite ? 0.f : __builtin_nanf("");
  return s;
}

// A finished sum from the two accumulator sets of scaled operands.
__device__ __forceinline__ float join_sets(float hi, float lo, ScaleBack sb) {
  return __builtin_ldexpf(__builtin_fmaf(lo, kLowPieceWeight, hi), sb.neg_se) + sb.poison;
}

}  // namespace glowmi
