// Depthwise 3x3 Convolution (groups == input channels == output channels, one filter per channel), fp32 and the
// scale/offset int8 form: the loop nest of Section 3.1 of the paper with groups, where the reduction of an
// output is nine products.  With nine multiply-adds per output the layer is a stream of the input and the
// output through the chip: nothing here is a matrix product, so no matrix cores and no LDS; what matters is that
// every byte is fetched in whole cache lines and as few times as possible.
//   - a thread owns four consecutive channels (fp32: one 16-byte piece of a pixel; int8: one dword) and a run of
//     DW_RUN consecutive output pixels on one or two output rows; consecutive threads own consecutive channel
//     quads, so a wavefront's load covers whole pixels (C = 128: two pixels of 512 bytes per fp32 load instruction);
//   - the input window of the run (two rows at stride 1: 4 x 6 pixels for 8 outputs) is loaded once into registers
//     and serves all of its outputs; rows and columns outside the image come back as zeros from range-checked
//     buffer loads (int8: and are then replaced by the code of real zero);
//   - a thread's channel quad never changes (the grid is a multiple of the channel quads), so its 36 filter values
//     and its bias are fetched once and stay in registers while it walks over runs;
//   - neighbouring runs share input rows, so every XCD works on one contiguous eighth of the runs and finds the
//     shared rows in its own L2 (12.8 M outputs of 128 channels at 56 x 56: 32 -> 24 us);
//   - bias, Relu (int8: the requantize of Section 4.3 with Relu as the lower clamp bound) and one 16-byte (int8:
//     4-byte) store per output pixel, predicated on the pixel being inside the output.
// Other filter sizes, strides above 2, channel counts that are not a multiple of four and layers with a tensor
// operand behind them stay on the generic kernels.
#include <hip/hip_runtime.h>

#include <cstdio>

#include "igemm.h"
#include "quant_epilogue.h"

namespace glowmi {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int DW_RUN = 4;                      // output pixels of one row per run
constexpr int DW_THREADS = 256;
constexpr unsigned DW_OOB = 0xFFFFFF00u;       // beyond any tensor these kernels accept: loads give zeros

struct DwGrid {
  int cq;                                      // channel quads
  int runs_w;                                  // runs per output row
  int strips;                                  // strips of ROWS output rows per image
  long long runs;                              // n * strips * runs_w
  int slots;                                   // threads per channel quad
  int blocks;                                  // workgroups that hold threads
  int per_xcd;                                 // workgroups per XCD (the launch has 8 * per_xcd)
};

// Workgroups are dealt to the eight XCDs in turn; a filter window's rows are shared by neighbouring runs, so
// each XCD takes one contiguous eighth of the runs and finds its neighbours' rows in its own L2.
__device__ __forceinline__ long long dw_thread(const DwGrid& g) {
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
  const int logical = xcd * g.per_xcd + idx;
  if (idx >= g.per_xcd || logical >= g.blocks) return -1;
  return (long long)logical * DW_THREADS + threadIdx.x;
}

struct DwRun {
  int img, oh0, ow0;
};

__device__ __forceinline__ DwRun dw_run(const DwGrid& g, unsigned run, int rows) {
  DwRun r;
  const unsigned rw = run % (unsigned)g.runs_w;
  const unsigned t2 = run / (unsigned)g.runs_w;
  r.oh0 = (int)(t2 % (unsigned)g.strips) * rows;
  r.img = (int)(t2 / (unsigned)g.strips);
  r.ow0 = (int)rw * DW_RUN;
  return r;
}

// Byte offsets of the XROWS x COLS input pixels of a run, for the thread's channels: the window's first pixel plus
// whole rows and columns, or the out-of-range mark where the row or column lies outside the image.
template <int XROWS, int COLS>
struct DwWindow {
  unsigned base;            // of pixel (ih0, iw0), channel c0; wraps when that pixel is outside: never used then
  bool row_ok[XROWS], col_ok[COLS];
  __device__ __forceinline__ DwWindow(const Problem& p, const DwRun& rn, int stride, unsigned c0_bytes, unsigned elem) {
    const int ih0 = rn.oh0 * stride - p.pad_t, iw0 = rn.ow0 * stride - p.pad_l;
    base = (unsigned)((rn.img * p.h + ih0) * p.w_ + iw0) * ((unsigned)p.c * elem) + c0_bytes;
#pragma unroll
    for (int r = 0; r < XROWS; ++r) row_ok[r] = (unsigned)(ih0 + r) < (unsigned)p.h;
#pragma unroll
    for (int c = 0; c < COLS; ++c) col_ok[c] = (unsigned)(iw0 + c) < (unsigned)p.w_;
  }
};

template <int STRIDE, int ROWS>
__global__ __launch_bounds__(DW_THREADS) void conv_dw_f32_kernel(const Problem p, const DwGrid g) {
  constexpr int COLS = (DW_RUN - 1) * STRIDE + 3, XROWS = (ROWS - 1) * STRIDE + 3;
  const long long gid = dw_thread(g);
  if (gid < 0 || gid >= (long long)g.cq * g.slots) return;
  const int cq = (int)((unsigned)gid % (unsigned)g.cq);
  const int slot = (int)((unsigned)gid / (unsigned)g.cq);
  const int c0 = cq * 4;

  const float* __restrict__ W = static_cast<const float*>(p.w);
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  float* __restrict__ Y = static_cast<float*>(p.y);

  // filter [k][3][3][1]: channel c's nine values are contiguous, the quad's 36 values one 144-byte piece:
  // nine 16-byte loads, then sorted by tap
  v4f wq[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) wq[i] = reinterpret_cast<const v4f*>(W + (size_t)c0 * 9)[i];
  v4f w[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int e = 0; e < 4; ++e) w[t][e] = wq[(e * 9 + t) / 4][(e * 9 + t) % 4];
  v4f bv = {0.f, 0.f, 0.f, 0.f};
  if (bias) bv = v4f{bias[c0], bias[c0 + 1], bias[c0 + 2], bias[c0 + 3]};     // bias is only 4-byte aligned
  const bool relu = p.act == 1;
  const unsigned col_bytes = (unsigned)p.c * 4u, row_bytes = (unsigned)p.w_ * col_bytes;

  for (unsigned run = (unsigned)slot; run < (unsigned)g.runs; run += (unsigned)g.slots) {
    const DwRun rn = dw_run(g, run, ROWS);
    const DwWindow<XROWS, COLS> win(p, rn, STRIDE, (unsigned)c0 * 4u, 4u);

    v4f x[XROWS][COLS];
#pragma unroll
    for (int r = 0; r < XROWS; ++r)
#pragma unroll
      for (int c = 0; c < COLS; ++c)
        x[r][c] = __builtin_bit_cast(
            v4f, __builtin_amdgcn_raw_buffer_load_b128(
                     rsrc_x, win.row_ok[r] && win.col_ok[c] ? win.base + r * row_bytes + c * col_bytes : DW_OOB, 0, 0));
    float* yrow = Y + ((size_t)(rn.img * p.oh + rn.oh0) * p.ow + rn.ow0) * p.k + c0;
#pragma unroll
    for (int ro = 0; ro < ROWS; ++ro) {
#pragma unroll
      for (int o = 0; o < DW_RUN; ++o) {
        v4f acc = bv;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
          for (int s = 0; s < 3; ++s) acc += x[ro * STRIDE + r][o * STRIDE + s] * w[r * 3 + s];
        if (relu) {
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[e] = fmaxf(acc[e], 0.f);
        }
        if (rn.oh0 + ro < p.oh && rn.ow0 + o < p.ow)
          *reinterpret_cast<v4f*>(yrow + ((size_t)ro * p.ow + o) * p.k) = acc;
      }
    }
  }
}

// The int8 form.  A thread's dword of the input holds the codes of its four channels at one pixel; the three
// codes of a channel along a filter row are gathered into one dword with two byte permutes and multiplied with
// the row's three filter codes by one four-way dot product.  Offsets are taken out of the sum,
//   sum (x - xo)(w - wo) = sum x w - wo sum x - xo sum (w - wo),
// where a tap on padding holds the code xo (it then adds nothing, as real zero must): the last term is a constant
// of the channel and joins the bias, the middle one costs a second dot product and is left out (PLAIN) when the
// filter has no offset.  All of it is arithmetic modulo 2^32, so the order does not matter.  Then the requantize
// of Section 4.3 with the integer multiplier (PLAIN: the form with the rounding constant and the output offset
// folded into one addend), Relu as the lower clamp bound, four codes per store.
template <int STRIDE, int ROWS, bool PLAIN>
__global__ __launch_bounds__(DW_THREADS) void conv_dw_i8_kernel(const Problem p, const DwGrid g) {
  constexpr int COLS = (DW_RUN - 1) * STRIDE + 3, XROWS = (ROWS - 1) * STRIDE + 3;
  const long long gid = dw_thread(g);
  if (gid < 0 || gid >= (long long)g.cq * g.slots) return;
  const int cq = (int)((unsigned)gid % (unsigned)g.cq);
  const int slot = (int)((unsigned)gid / (unsigned)g.cq);
  const int c0 = cq * 4;

  const signed char* __restrict__ W = static_cast<const signed char*>(p.w);
  const int* __restrict__ bias = static_cast<const int*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  signed char* __restrict__ Y = static_cast<signed char*>(p.y);

  // the quad's 36 filter codes are nine dwords; per channel and filter row one dword (w0, w1, w2, 0)
  unsigned wq[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) wq[i] = reinterpret_cast<const unsigned*>(W + (size_t)c0 * 9)[i];
  int wr[3][4];
  int kb[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    int wsum = 0;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
      // codes i .. i + 2 of the 36 start in byte i % 4 of dword i / 4: an alignbyte of two dwords, top byte cleared
      const int i = e * 9 + r * 3;
      const unsigned lo = wq[i / 4], hi = wq[(i / 4 + 1) % 9];
      const unsigned d = (i % 4 == 0 ? lo : __builtin_amdgcn_alignbyte(hi, lo, i % 4)) & 0x00ffffffu;
      wr[r][e] = (int)d;
      wsum = __builtin_amdgcn_sdot4((int)d, 0x00010101, wsum, false);
    }
    kb[e] = (bias ? bias[c0 + e] : 0) - p.x_off * (wsum - 9 * p.w_off);
  }
  const unsigned xo_fill = (unsigned)(p.x_off & 0xff) * 0x01010101u;     // padding = the code of real zero
  const FoldedRequant fold = make_folded_requant(p.shift, p.y_off);
  const bool fast = p.shift >= 33;                                        // uniform
  const int lo_v = p.lo;
  const unsigned col_bytes = (unsigned)p.c, row_bytes = (unsigned)p.w_ * col_bytes;

  for (unsigned run = (unsigned)slot; run < (unsigned)g.runs; run += (unsigned)g.slots) {
    const DwRun rn = dw_run(g, run, ROWS);
    const DwWindow<XROWS, COLS> win(p, rn, STRIDE, (unsigned)c0, 1u);

    unsigned x[XROWS][COLS];
#pragma unroll
    for (int r = 0; r < XROWS; ++r)
#pragma unroll
      for (int c = 0; c < COLS; ++c) {
        const bool ok = win.row_ok[r] && win.col_ok[c];
        const unsigned v = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(
            rsrc_x, ok ? win.base + r * row_bytes + c * col_bytes : DW_OOB, 0, 0);
        x[r][c] = ok ? v : xo_fill;
      }
    signed char* yrow = Y + ((size_t)(rn.img * p.oh + rn.oh0) * p.ow + rn.ow0) * p.k + c0;
#pragma unroll
    for (int ro = 0; ro < ROWS; ++ro) {
#pragma unroll
      for (int o = 0; o < DW_RUN; ++o) {
        int q[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          int acc = kb[e], xsum = 0;
#pragma unroll
          for (int r = 0; r < 3; ++r) {
            const unsigned* row = x[ro * STRIDE + r] + o * STRIDE;
            // bytes (row[0].e, row[1].e, 0, 0), then (.., .., row[2].e, 0): selectors 0..3 name the second
            // operand's bytes, 4..7 the first operand's, 12 a zero byte
            const unsigned two = __builtin_amdgcn_perm(row[1], row[0], 0x0c0c0000u | (unsigned)e | ((4u + e) << 8));
            const unsigned three = __builtin_amdgcn_perm(row[2], two, 0x0c000100u | ((4u + e) << 16));
            acc = __builtin_amdgcn_sdot4((int)three, wr[r][e], acc, false);
            if (!PLAIN) xsum = __builtin_amdgcn_sdot4((int)three, 0x00010101, xsum, false);
          }
          if (PLAIN) {
            q[e] = requantize_folded(acc, p.mant, fold, lo_v);
          } else {
            acc -= p.w_off * xsum;
            q[e] = fast ? requantize_as<true>(acc, p.mant, p.shift, p.y_off, p.lo)
                        : requantize_as<false>(acc, p.mant, p.shift, p.y_off, p.lo);
          }
        }
        if (rn.oh0 + ro < p.oh && rn.ow0 + o < p.ow)
          *reinterpret_cast<unsigned*>(yrow + ((size_t)ro * p.ow + o) * p.k) = pack_codes(q[0], q[1], q[2], q[3]);
      }
    }
  }
}

bool dw_shape(const Problem& p) {
  if (knob_or(KNOB_DW, 1) == 0) return false;
  if (p.b_is_kn || p.chain_n > 0 || p.addend) return false;
  if (p.groups != p.c || p.k != p.c || p.cg != 1 || p.kg != 1) return false;
  if (p.r != 3 || p.s != 3 || p.stride_h != p.stride_w || (p.stride_h != 1 && p.stride_h != 2)) return false;
  if (p.c % 4 != 0) return false;
  if ((long long)p.n * p.oh * p.ow * p.k >= (1LL << 31)) return false;      // 32-bit run and thread indices
  return p.x_bytes < 0xF0000000u;
}

// Output rows per run.  Two rows share two of their three (stride 2: one of their three) input rows in registers;
// at stride 2 the five-row window costs more registers than the sharing saves.  Knob DW: 0 off, 1 this choice,
// 2 one row, 3 two rows.
int dw_rows(const Problem& p) {
  const int v = knob_or(KNOB_DW, 1);
  if (v == 2 || v == 3) return v - 1;
  return p.stride_h == 1 ? 2 : 1;
}

DwGrid dw_grid(const Problem& p, int rows) {
  DwGrid g;
  g.cq = p.c / 4;
  g.runs_w = (p.ow + DW_RUN - 1) / DW_RUN;
  g.strips = (p.oh + rows - 1) / rows;
  g.runs = (long long)p.n * g.strips * g.runs_w;
  // a thread for every run up to 2048 threads per CU; above that every thread walks the same number of runs
  long long cap = (256LL * 2048 + g.cq - 1) / g.cq;
  if (cap < 1) cap = 1;
  const long long passes = (g.runs + cap - 1) / cap;
  long long slots = passes > 0 ? (g.runs + passes - 1) / passes : 1;
  if (slots < 1) slots = 1;
  g.slots = (int)slots;
  const long long threads = (long long)g.cq * g.slots;
  g.blocks = (int)((threads + DW_THREADS - 1) / DW_THREADS);
  g.per_xcd = (g.blocks + 7) / 8;
  return g;
}

template <typename Kern>
hipError_t launch_dw(Kern kern, const Problem& p, int rows, hipStream_t stream) {
  const DwGrid g = dw_grid(p, rows);
  hipLaunchKernelGGL(kern, dim3((unsigned)(8 * g.per_xcd)), dim3(DW_THREADS), 0, stream, p, g);
  return hipGetLastError();
}

}  // namespace

bool dw_f32_applicable(const Problem& p) { return dw_shape(p); }
bool dw_i8_applicable(const Problem& p) { return dw_shape(p); }

hipError_t launch_dw_f32(const Problem& p, hipStream_t stream, const char** variant) {
  const int rows = dw_rows(p);
  if (p.stride_h == 1) {
    *variant = "conv_dw_f32_3x3s1";
    return rows == 1 ? launch_dw(conv_dw_f32_kernel<1, 1>, p, 1, stream) : launch_dw(conv_dw_f32_kernel<1, 2>, p, 2, stream);
  }
  *variant = "conv_dw_f32_3x3s2";
  return rows == 1 ? launch_dw(conv_dw_f32_kernel<2, 1>, p, 1, stream) : launch_dw(conv_dw_f32_kernel<2, 2>, p, 2, stream);
}

hipError_t launch_dw_i8(const Problem& p, hipStream_t stream, const char** variant) {
  const int rows = dw_rows(p);
  // the plain form: no filter offset, and a requantize shift the folded addend covers
  const bool plain = p.w_off == 0 && p.shift >= 33 && p.shift <= 54;
  if (p.stride_h == 1) {
    *variant = "conv_dw_i8_3x3s1";
    if (plain) return rows == 1 ? launch_dw(conv_dw_i8_kernel<1, 1, true>, p, 1, stream) : launch_dw(conv_dw_i8_kernel<1, 2, true>, p, 2, stream);
    return rows == 1 ? launch_dw(conv_dw_i8_kernel<1, 1, false>, p, 1, stream) : launch_dw(conv_dw_i8_kernel<1, 2, false>, p, 2, stream);
  }
  *variant = "conv_dw_i8_3x3s2";
  if (plain) return rows == 1 ? launch_dw(conv_dw_i8_kernel<2, 1, true>, p, 1, stream) : launch_dw(conv_dw_i8_kernel<2, 2, true>, p, 2, stream);
  return rows == 1 ? launch_dw(conv_dw_i8_kernel<2, 1, false>, p, 1, stream) : launch_dw(conv_dw_i8_kernel<2, 2, false>, p, 2, stream);
}

}  // namespace glowmi
