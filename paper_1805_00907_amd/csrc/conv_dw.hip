// Depthwise 3x3 Convolution (groups == input channels == output channels, one filter per channel), fp32 and the
// scale/offset int8 form: the loop nest of Section 3.1 of the paper with groups, where the reduction of an
// output is nine products.  With nine multiply-adds per output the layer is a stream of the input and the
// output through the chip: nothing here is a matrix product, so no matrix cores and no LDS; what matters is that
// every byte is fetched in whole cache lines and as few times as possible.
//   - a thread owns four consecutive channels (fp32: one 16-byte piece of a pixel; int8: one dword) and a run of
//     DW_RUN consecutive output pixels of one row; consecutive threads own consecutive channel quads, so a
//     wavefront's load covers whole pixels (C = 128: two pixels of 512 bytes per fp32 load instruction);
//   - the 3 x (DW_RUN - 1) * stride + 3 input columns the run needs are loaded once into registers and serve all
//     of its outputs (stride 1: 18 loads for 4 outputs instead of 36); rows and columns outside the image come
//     back as zeros from range-checked buffer loads (int8: and are then replaced by the code of real zero);
//   - a thread's channel quad never changes (the grid is a multiple of the channel quads), so its 36 filter values
//     and its bias are fetched once and stay in registers while it walks over runs;
//   - bias, Relu (int8: the requantize of Section 4.3 with Relu as the lower clamp bound) and one 16-byte (int8:
//     4-byte) store per output pixel.
// Other filter sizes, strides above 2, channel counts that are not a multiple of four and layers with a tensor
// operand behind them stay on the generic kernels.
#include <hip/hip_runtime.h>

#include <cstdio>

#include "igemm.h"
#include "quant_epilogue.h"

namespace glowmi {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v4i_ __attribute__((ext_vector_type(4)));

constexpr int DW_RUN = 4;                      // output pixels per run
constexpr int DW_THREADS = 256;
constexpr unsigned DW_OOB = 0xFFFFFF00u;       // beyond any tensor these kernels accept: loads give zeros

struct DwGrid {
  int cq;                                      // channel quads
  int runs_w;                                  // runs per output row
  long long runs;                              // n * oh * runs_w
  int slots;                                   // threads per channel quad
};

template <int STRIDE>
__global__ __launch_bounds__(DW_THREADS) void conv_dw_f32_kernel(const Problem p, const DwGrid g) {
  constexpr int COLS = (DW_RUN - 1) * STRIDE + 3;
  const long long gid = (long long)blockIdx.x * DW_THREADS + threadIdx.x;
  if (gid >= (long long)g.cq * g.slots) return;
  const int cq = (int)(gid % g.cq);
  const int slot = (int)(gid / g.cq);
  const int c0 = cq * 4;

  const float* __restrict__ W = static_cast<const float*>(p.w);
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  float* __restrict__ Y = static_cast<float*>(p.y);

  // filter [k][3][3][1]: channel c's nine values are contiguous
  v4f w[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) w[t] = v4f{W[(c0 + 0) * 9 + t], W[(c0 + 1) * 9 + t], W[(c0 + 2) * 9 + t], W[(c0 + 3) * 9 + t]};
  v4f bv = {0.f, 0.f, 0.f, 0.f};
  if (bias) bv = v4f{bias[c0], bias[c0 + 1], bias[c0 + 2], bias[c0 + 3]};
  const bool relu = p.act == 1;

  for (long long run = slot; run < g.runs; run += g.slots) {
    const int rw = (int)(run % g.runs_w);
    const long long t2 = run / g.runs_w;
    const int oh = (int)(t2 % p.oh);
    const int img = (int)(t2 / p.oh);
    const int ow0 = rw * DW_RUN;
    const int ih0 = oh * STRIDE - p.pad_t, iw0 = ow0 * STRIDE - p.pad_l;

    v4f x[3][COLS];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
      const int ih = ih0 + r;
      const bool row_ok = (unsigned)ih < (unsigned)p.h;
#pragma unroll
      for (int c = 0; c < COLS; ++c) {
        const int iw = iw0 + c;
        const bool ok = row_ok && (unsigned)iw < (unsigned)p.w_;
        const unsigned off = ok ? ((unsigned)((img * p.h + ih) * p.w_ + iw) * (unsigned)p.c + (unsigned)c0) * 4u : DW_OOB;
        x[r][c] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0));
      }
    }
#pragma unroll
    for (int o = 0; o < DW_RUN; ++o) {
      const int ow = ow0 + o;
      if (ow >= p.ow) break;
      v4f acc = bv;
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) acc += x[r][o * STRIDE + s] * w[r * 3 + s];
      if (relu) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = fmaxf(acc[e], 0.f);
      }
      *reinterpret_cast<v4f*>(Y + ((size_t)(img * p.oh + oh) * p.ow + ow) * p.k + c0) = acc;
    }
  }
}

// The int8 form: codes minus offsets multiplied in int32 (a tap on padding is the code of real zero, i.e. adds
// nothing), int32 bias, requantize with the integer multiplier, Relu as the lower clamp bound, four codes per store.
template <int STRIDE>
__global__ __launch_bounds__(DW_THREADS) void conv_dw_i8_kernel(const Problem p, const DwGrid g) {
  constexpr int COLS = (DW_RUN - 1) * STRIDE + 3;
  const long long gid = (long long)blockIdx.x * DW_THREADS + threadIdx.x;
  if (gid >= (long long)g.cq * g.slots) return;
  const int cq = (int)(gid % g.cq);
  const int slot = (int)(gid / g.cq);
  const int c0 = cq * 4;

  const signed char* __restrict__ W = static_cast<const signed char*>(p.w);
  const int* __restrict__ bias = static_cast<const int*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  signed char* __restrict__ Y = static_cast<signed char*>(p.y);

  int w[9][4];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int e = 0; e < 4; ++e) w[t][e] = (int)W[(c0 + e) * 9 + t] - p.w_off;
  int bv[4] = {0, 0, 0, 0};
  if (bias) {
#pragma unroll
    for (int e = 0; e < 4; ++e) bv[e] = bias[c0 + e];
  }
  const int xo_fill = (p.x_off & 0xff) * 0x01010101;     // padding = the code of real zero
  const bool fast = p.shift >= 33;                        // uniform

  for (long long run = slot; run < g.runs; run += g.slots) {
    const int rw = (int)(run % g.runs_w);
    const long long t2 = run / g.runs_w;
    const int oh = (int)(t2 % p.oh);
    const int img = (int)(t2 / p.oh);
    const int ow0 = rw * DW_RUN;
    const int ih0 = oh * STRIDE - p.pad_t, iw0 = ow0 * STRIDE - p.pad_l;

    int x[3][COLS];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
      const int ih = ih0 + r;
      const bool row_ok = (unsigned)ih < (unsigned)p.h;
#pragma unroll
      for (int c = 0; c < COLS; ++c) {
        const int iw = iw0 + c;
        const bool ok = row_ok && (unsigned)iw < (unsigned)p.w_;
        const unsigned off = ok ? (unsigned)((img * p.h + ih) * p.w_ + iw) * (unsigned)p.c + (unsigned)c0 : DW_OOB;
        const int v = __builtin_amdgcn_raw_buffer_load_b32(rsrc_x, off, 0, 0);   // issued whatever `ok` is: zeros when out of range
        x[r][c] = ok ? v : xo_fill;
      }
    }
#pragma unroll
    for (int o = 0; o < DW_RUN; ++o) {
      const int ow = ow0 + o;
      if (ow >= p.ow) break;
      int q[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int acc = bv[e];
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
          for (int s = 0; s < 3; ++s) {
            const int code = (int)(signed char)(x[r][o * STRIDE + s] >> (8 * e));
            acc += (code - p.x_off) * w[r * 3 + s][e];
          }
        q[e] = fast ? requantize_as<true>(acc, p.mant, p.shift, p.y_off, p.lo)
                    : requantize_as<false>(acc, p.mant, p.shift, p.y_off, p.lo);
      }
      *reinterpret_cast<unsigned*>(Y + ((size_t)(img * p.oh + oh) * p.ow + ow) * p.k + c0) = pack_codes(q[0], q[1], q[2], q[3]);
    }
  }
}

bool dw_shape(const Problem& p) {
  if (knob_or(KNOB_DW, 1) == 0) return false;
  if (p.b_is_kn || p.chain_n > 0 || p.addend) return false;
  if (p.groups != p.c || p.k != p.c || p.cg != 1 || p.kg != 1) return false;
  if (p.r != 3 || p.s != 3 || p.stride_h != p.stride_w || (p.stride_h != 1 && p.stride_h != 2)) return false;
  if (p.c % 4 != 0) return false;
  return p.x_bytes < 0xF0000000u;
}

DwGrid dw_grid(const Problem& p) {
  DwGrid g;
  g.cq = p.c / 4;
  g.runs_w = (p.ow + DW_RUN - 1) / DW_RUN;
  g.runs = (long long)p.n * p.oh * g.runs_w;
  // enough threads to fill the chip (256 CUs x 2048) without leaving a thread less than one run
  long long slots = (256LL * 2048 + g.cq - 1) / g.cq;
  if (slots > g.runs) slots = g.runs;
  if (slots < 1) slots = 1;
  g.slots = (int)slots;
  return g;
}

template <typename Kern>
hipError_t launch_dw(Kern kern, const Problem& p, hipStream_t stream) {
  const DwGrid g = dw_grid(p);
  const long long threads = (long long)g.cq * g.slots;
  const long long blocks = (threads + DW_THREADS - 1) / DW_THREADS;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(DW_THREADS), 0, stream, p, g);
  return hipGetLastError();
}

}  // namespace

bool dw_f32_applicable(const Problem& p) { return dw_shape(p); }
bool dw_i8_applicable(const Problem& p) { return dw_shape(p); }

hipError_t launch_dw_f32(const Problem& p, hipStream_t stream, const char** variant) {
  *variant = p.stride_h == 1 ? "conv_dw_f32_3x3s1" : "conv_dw_f32_3x3s2";
  return p.stride_h == 1 ? launch_dw(conv_dw_f32_kernel<1>, p, stream) : launch_dw(conv_dw_f32_kernel<2>, p, stream);
}

hipError_t launch_dw_i8(const Problem& p, hipStream_t stream, const char** variant) {
  *variant = p.stride_h == 1 ? "conv_dw_i8_3x3s1" : "conv_dw_i8_3x3s2";
  return p.stride_h == 1 ? launch_dw(conv_dw_i8_kernel<1>, p, stream) : launch_dw(conv_dw_i8_kernel<2>, p, stream);
}

}  // namespace glowmi
