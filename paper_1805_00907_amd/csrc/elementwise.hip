// Conversions at the borders of the integer "islands" of Section 4.2 of the paper, as device kernels
// so that quantized layers can be chained without a trip through the host:
//   quantize    float  -> int8   q = sat(round_to_nearest_even(v / scale) + offset)   (inverse of the
//                                Section 4.1 formula value = (q - offset) * scale)
//   dequantize  int8   -> float  v = (q - offset) * scale                             (Section 4.1)
//   rescale     int8   -> int8   the same real values on another scale/offset         (rescale node,
//                                Section 4.3), integer arithmetic like the fused requantize
// All three stream their tensor once: 16 elements per thread and step, 16-byte accesses on the int8
// side; they are bound by HBM bandwidth.
#include <hip/hip_runtime.h>

#include "igemm.h"
#include "quant_epilogue.h"

namespace glowmi {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int EW_THREADS = 256;
constexpr int EW_PER_THREAD = 16;

// The quotient is formed in double (the float operands are exact there and the division is correctly
// rounded), so the rounding decision is the same wherever it is evaluated.
__device__ __forceinline__ int quantize_one(float v, double scale, int offset) {
  double t = __builtin_rint((double)v / scale) + (double)offset;   // ties to even
  t = t != t ? (double)offset : t;                                 // NaN has no code: it takes the code of real zero
  t = t < -128.0 ? -128.0 : t;
  t = t > 127.0 ? 127.0 : t;
  return (int)t;
}

__global__ __launch_bounds__(EW_THREADS) void quantize_kernel(const float* __restrict__ x,
                                                             signed char* __restrict__ q, long long count,
                                                             float scale, int offset) {
  const double s = (double)scale;
  const long long groups = count / EW_PER_THREAD;
  for (long long g = (long long)blockIdx.x * EW_THREADS + threadIdx.x; g < groups;
       g += (long long)gridDim.x * EW_THREADS) {
    const v4f* src = reinterpret_cast<const v4f*>(x + g * EW_PER_THREAD);
    v4i out;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const v4f v = src[j];
      out[j] = (int)pack_codes(quantize_one(v[0], s, offset), quantize_one(v[1], s, offset),
                               quantize_one(v[2], s, offset), quantize_one(v[3], s, offset));
    }
    *reinterpret_cast<v4i*>(q + g * EW_PER_THREAD) = out;
  }
  // ragged tail, one element per thread of the first workgroup
  if (blockIdx.x == 0)
    for (long long i = groups * EW_PER_THREAD + threadIdx.x; i < count; i += EW_THREADS)
      q[i] = (signed char)quantize_one(x[i], s, offset);
}

__global__ __launch_bounds__(EW_THREADS) void dequantize_kernel(const signed char* __restrict__ q,
                                                               float* __restrict__ x, long long count,
                                                               float scale, int offset) {
  const long long groups = count / EW_PER_THREAD;
  for (long long g = (long long)blockIdx.x * EW_THREADS + threadIdx.x; g < groups;
       g += (long long)gridDim.x * EW_THREADS) {
    const v4i in = *reinterpret_cast<const v4i*>(q + g * EW_PER_THREAD);
    v4f* dst = reinterpret_cast<v4f*>(x + g * EW_PER_THREAD);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v4f v;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int code = (int)(signed char)((unsigned)in[j] >> (8 * t));
        v[t] = (float)(code - offset) * scale;        // small integer times float: one rounding
      }
      dst[j] = v;
    }
  }
  if (blockIdx.x == 0)
    for (long long i = groups * EW_PER_THREAD + threadIdx.x; i < count; i += EW_THREADS)
      x[i] = (float)((int)q[i] - offset) * scale;
}

__global__ __launch_bounds__(EW_THREADS) void rescale_kernel(const signed char* __restrict__ in,
                                                            signed char* __restrict__ out, long long count,
                                                            int in_offset, int mant, int shift,
                                                            int out_offset) {
  const long long groups = count / EW_PER_THREAD;
  auto one = [&](int code) {
    return shift >= 33 ? requantize_as<true>(code - in_offset, mant, shift, out_offset, -128)
                       : requantize_as<false>(code - in_offset, mant, shift, out_offset, -128);   // uniform
  };
  for (long long g = (long long)blockIdx.x * EW_THREADS + threadIdx.x; g < groups;
       g += (long long)gridDim.x * EW_THREADS) {
    const v4i v = *reinterpret_cast<const v4i*>(in + g * EW_PER_THREAD);
    v4i o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) c[t] = one((int)(signed char)((unsigned)v[j] >> (8 * t)));
      o[j] = (int)pack_codes(c[0], c[1], c[2], c[3]);
    }
    *reinterpret_cast<v4i*>(out + g * EW_PER_THREAD) = o;
  }
  if (blockIdx.x == 0)
    for (long long i = groups * EW_PER_THREAD + threadIdx.x; i < count; i += EW_THREADS)
      out[i] = (signed char)one((int)in[i]);
}

unsigned grid_for(long long count) {
  long long blocks = (count / EW_PER_THREAD + EW_THREADS - 1) / EW_THREADS;
  if (blocks < 1) blocks = 1;
  if (blocks > 256 * 16) blocks = 256 * 16;       // grid-stride beyond 16 workgroups per CU
  return (unsigned)blocks;
}

}  // namespace

hipError_t launch_quantize(const float* x, signed char* q, long long count, float scale, int offset,
                           hipStream_t stream) {
  hipLaunchKernelGGL(quantize_kernel, dim3(grid_for(count)), dim3(EW_THREADS), 0, stream, x, q, count, scale, offset);
  return hipGetLastError();
}

hipError_t launch_dequantize(const signed char* q, float* x, long long count, float scale, int offset,
                             hipStream_t stream) {
  hipLaunchKernelGGL(dequantize_kernel, dim3(grid_for(count)), dim3(EW_THREADS), 0, stream, q, x, count, scale,
                     offset);
  return hipGetLastError();
}

hipError_t launch_rescale(const signed char* in, signed char* out, long long count, int in_offset, int mant,
                          int shift, int out_offset, hipStream_t stream) {
  hipLaunchKernelGGL(rescale_kernel, dim3(grid_for(count)), dim3(EW_THREADS), 0, stream, in, out, count, in_offset,
                     mant, shift, out_offset);
  return hipGetLastError();
}

}  // namespace glowmi
