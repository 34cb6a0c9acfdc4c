// int8 3x3 Convolution over 64 input channels on many pixels (the first 3x3 layers of a residual
// network at batch): the quantized form (Section 4 of the paper: int8 codes with per-tensor
// scale/offset, int32 accumulation, rescale folded into the producer, Relu as an integer lower
// bound) of one more kind of convolution that gets a strategy of its own (Section 5.3).
//
// With 64 channels the whole filter of 64 output channels (64 x 576 bytes) fits LDS, and the three
// taps of one filter row are 192 contiguous bytes of the NHWC input.  So the layer is run like the
// pointwise kernel (conv_pw_i8.hip), with the reduction cut into one chunk per filter row:
//   - a persistent workgroup stages its filter slice (64 output channels) into LDS once, in the row
//     order the MFMA needs, and derives the per-channel term  bias - x_offset * sum w  from it
//     (filter offset 0 only; other filters take the generic kernels);
//   - a wavefront owns blocks of 32 output pixels.  Per block and filter row it gathers 32 x 192
//     bytes (two lanes per pixel, six 16-byte loads each; taps outside the image are replaced by the
//     input's offset code, which represents 0.0) into a private LDS region while the previous chunk
//     is multiplied: no workgroup barrier after the prologue;
//   - per chunk 6 MFMA steps (v_mfma_i32_32x32x32_i8) x 2 halves of the 64 channels, the filter as
//     the row operand and the channels permuted so that a lane ends with 32 consecutive channels of
//     one pixel (the accumulators start at the channel term): requantize, clamp, pack, two 16-byte
//     stores.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "igemm.h"
#include "pw_common.h"
#include "quant_epilogue.h"

namespace glowmi {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int K3_C = 64;                       // input channels
constexpr int K3_ROW = 3 * K3_C;               // bytes of one filter row of one pixel: a chunk
constexpr int K3_K = 3 * K3_ROW;               // whole reduction
constexpr int K3_BN = 64;                      // output channels per workgroup
constexpr int K3_WPITCH = K3_K + 16;           // LDS pitch of a filter row
constexpr int K3_APITCH = K3_ROW + 16;         // LDS pitch of a pixel's chunk
constexpr int K3_AREGION = 32 * K3_APITCH;     // bytes per wavefront
constexpr int K3_LOADS = K3_ROW / 2 / 16;      // 16-byte loads per lane and chunk (two lanes per pixel)

template <int WAVES>
constexpr int k3_lds_bytes() { return K3_BN * K3_WPITCH + WAVES * K3_AREGION + K3_BN * 4 + 256 * 4; }   // + addend table

// Row of the staged filter slice that holds output channel `c` (0..63).  MFMA nb (0/1) multiplies
// rows nb*32 .. nb*32+31; result register e of a lane with half h is MFMA row (e/4)*8 + 4h + e%4,
// and this order makes that row channel 32h + 16nb + e: a lane's 16 registers are 16 consecutive
// channels.
__host__ __device__ constexpr int k3_staged_row(int c) {
  return ((c >> 4) & 1) * 32 + ((c >> 2) & 3) * 8 + (c >> 5) * 4 + (c & 3);
}

// ADD: the element-wise chain has a tensor-add link (p.addend, int8 of the output's shape, rescaled
// to the accumulator's scale before it is added).
template <int WAVES, bool ADD>
__global__ __launch_bounds__(WAVES * 64, 1) void conv_k3c64_i8_kernel(const Problem p, int blocks_div,
                                                                      int blocks_rem) {
  extern __shared__ __align__(16) unsigned char smem[];   // filter slice, chunk regions, channel terms
  unsigned char* wlds = smem;
  int* cterm = reinterpret_cast<int*>(smem + K3_BN * K3_WPITCH + WAVES * K3_AREGION);
  int* addlut = cterm + K3_BN;   // [256] the addend's code (as an unsigned byte) -> its term at the accumulator's scale

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int slice = blockIdx.y;
  unsigned char* alds = smem + K3_BN * K3_WPITCH + wave * K3_AREGION;

  const int* __restrict__ bias = static_cast<const int*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_y =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)((unsigned)p.M * (unsigned)p.k), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_add = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(ADD ? p.addend : p.y), 0, (int)((unsigned)p.M * (unsigned)p.k), 0x00020000);

  // ---- this wavefront's contiguous range of pixel blocks
  const int wv = blockIdx.x * WAVES + wave;
  int rb, rb_end_;
  deal_range(wv, (int)gridDim.x * WAVES, blocks_div, blocks_rem, rb, rb_end_);
  const int rb_end = rb_end_;
  const int ohow = p.oh * p.ow;

  // ---- gathering a chunk: lane l fetches the half `l & 1` (96 bytes) of filter row r of pixel l / 2.
  // Byte b of a chunk belongs to tap b / 64, so the six loads of a lane cover taps
  // {0,0,0,0,1,1} (first half) or {1,1,2,2,2,2} (second half).
  const int spix = lane >> 1, shalf = lane & 1;
  const unsigned fill = (unsigned)(p.x_off & 0xff) * 0x01010101u;
  unsigned fbase = 0;     // byte offset of the lane's half of row 0 of the block being fetched
  int row_ok = 0;         // bit r: filter row r of the lane's pixel lies inside the image
  int tap_ok = 0;         // bit i: the tap of load i lies inside the image (columns only)
  int okmask = 0;         // bit i: load i of the chunk in flight was inside the image
  v4i st[K3_LOADS];
  auto decode = [&](int block) {
    int m = block * 32 + spix;
    if (m >= p.M) m = p.M - 1;                             // results of such rows are never stored
    const int img = p.div_ohow.div(m);
    const int rem = m - img * ohow;
    const int oh = p.div_ow.div(rem);
    const int ow = rem - oh * p.ow;
    const int ih0 = oh * p.stride_h - p.pad_t, iw0 = ow * p.stride_w - p.pad_l;
    fbase = ((unsigned)(img * p.h + ih0) * (unsigned)p.w_ + (unsigned)iw0) * (unsigned)K3_C + 96u * shalf;
    row_ok = 0;
    int col_ok = 0;
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      row_ok |= ((unsigned)(ih0 + t) < (unsigned)p.h) << t;
      col_ok |= ((unsigned)(iw0 + t) < (unsigned)p.w_) << t;
    }
    tap_ok = 0;
#pragma unroll
    for (int i = 0; i < K3_LOADS; ++i) {
      const int tap_first = i >= 4 ? 1 : 0, tap_second = i >= 2 ? 2 : 1;
      const int tap = shalf ? tap_second : tap_first;
      tap_ok |= ((col_ok >> tap) & 1) << i;
    }
  };
  auto fetch = [&](int r) {
    okmask = ((row_ok >> r) & 1) ? tap_ok : 0;
    const unsigned rbase = fbase + (unsigned)r * (unsigned)p.w_ * (unsigned)K3_C;
#pragma unroll
    for (int i = 0; i < K3_LOADS; ++i) {
      // an offset past the end of the tensor makes the range-checked load return zeros
      const unsigned off = ((okmask >> i) & 1) ? rbase + 16u * i : 0x80000000u;
      st[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0);
    }
  };
  auto commit = [&]() {
#pragma unroll
    for (int i = 0; i < K3_LOADS; ++i) {
      v4i v = st[i];
      if (!((okmask >> i) & 1)) { v[0] = (int)fill; v[1] = (int)fill; v[2] = (int)fill; v[3] = (int)fill; }
      *reinterpret_cast<v4i*>(alds + spix * K3_APITCH + 96 * shalf + 16 * i) = v;
    }
  };

  // the first chunk's loads go out before the filter slice's, so both latencies overlap
  const bool has_work = rb < rb_end;
  if (has_work) { decode(rb); fetch(0); }

  // ---- filter slice -> LDS in MFMA row order.  The slice is one contiguous run of the [k][3][3][64]
  // filter; rows past the last output channel lie past the end of the tensor and the range-checked
  // loads return zeros.
  {
    constexpr int V4_PER_ROW = K3_K / 16;
    constexpr int TOTAL = K3_BN * V4_PER_ROW;
    constexpr int THREADS = WAVES * 64;
    constexpr int PASSES = (TOTAL + THREADS - 1) / THREADS;
    const unsigned base = (unsigned)slice * (unsigned)(K3_BN * K3_K);
    v4i stage[PASSES];
#pragma unroll
    for (int q = 0; q < PASSES; ++q) {
      const int i = tid + q * THREADS;
      stage[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, i < TOTAL ? base + (unsigned)i * 16u : 0x80000000u, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < PASSES; ++q) {
      const int i = tid + q * THREADS;
      const int ch = i / V4_PER_ROW, kq = i % V4_PER_ROW;
      if (i < TOTAL) *reinterpret_cast<v4i*>(wlds + k3_staged_row(ch) * K3_WPITCH + kq * 16) = stage[q];
    }
  }
  __syncthreads();
  // every value a quantized addend can contribute: 256 codes, so the 64-bit rescale is done once per
  // code here instead of once per output in the epilogue
  if (ADD && tid < 256) addlut[tid] = rescale_term((int)(signed char)tid - p.r_off, p.r_mant, p.r_shift);
  // per-channel additive term, combined modulo 2^32 (the true accumulator fits int32 by contract)
  if (tid < K3_BN) {
    const int ch = slice * K3_BN + tid;
    const unsigned char* wrow = wlds + k3_staged_row(tid) * K3_WPITCH;
    int wsum = 0;
#pragma unroll 4
    for (int j = 0; j < K3_K / 16; ++j) {
      const v4i v = *reinterpret_cast<const v4i*>(wrow + 16 * j);
#pragma unroll
      for (int t = 0; t < 4; ++t) wsum = __builtin_amdgcn_sdot4(v[t], 0x01010101, wsum, false);
    }
    unsigned ct = 0u - (unsigned)p.x_off * (unsigned)wsum;
    if (bias && ch < p.k) ct += (unsigned)bias[ch];
    cterm[tid] = (int)ct;
  }
  __syncthreads();
  if (!has_work) return;

  const unsigned char* a_lane = alds + l32 * K3_APITCH + 16 * lh;
  const unsigned char* w_lane = wlds + l32 * K3_WPITCH + 16 * lh;
  const bool fast = p.shift >= 33;                         // uniform
  const FoldedRequant fold = make_folded_requant(p.shift, p.y_off);   // uniform
  const int lo_v = p.lo;
  const int ch0 = slice * K3_BN + 32 * lh;                 // first of the lane's 32 channels

  commit();
  for (; rb < rb_end; ++rb) {
    const unsigned off = (unsigned)(rb * 32 + l32) * (unsigned)p.k + (unsigned)ch0;
    // the lane's 32 addend codes, fetched ahead of the MFMAs
    v4i addq[2];
    if (ADD) {
      addq[0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_add, off, 0, 0);
      addq[1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_add, off + 16u, 0, 0);
    }
    // the accumulators start at the channel terms: register e of acc<nb> = channel 32*lh + 16*nb + e
    v16i acc0, acc1;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const v4i c0 = *reinterpret_cast<const v4i*>(cterm + 32 * lh + 4 * q4);
      const v4i c1 = *reinterpret_cast<const v4i*>(cterm + 32 * lh + 16 + 4 * q4);
#pragma unroll
      for (int t = 0; t < 4; ++t) { acc0[4 * q4 + t] = c0[t]; acc1[4 * q4 + t] = c1[t]; }
    }
    const bool more = rb + 1 < rb_end;                     // uniform: this wavefront owns block rb + 1 too
#pragma unroll
    for (int r = 0; r < 3; ++r) {
      // the next chunk is in flight while this one is multiplied
      const bool has_next = r < 2 || more;
      if (r == 2 && more) decode(rb + 1);
      if (has_next) fetch(r == 2 ? 0 : r + 1);
      const unsigned char* wl = w_lane + r * K3_ROW;
#pragma unroll
      for (int s = 0; s < K3_ROW / 32; ++s) {
        // each lane feeds 16 consecutive codes of its row; lanes 32..63 take the upper 16 of the 32
        const v4i a = *reinterpret_cast<const v4i*>(a_lane + 32 * s);
        const v4i b0 = *reinterpret_cast<const v4i*>(wl + 32 * s);
        const v4i b1 = *reinterpret_cast<const v4i*>(wl + 32 * K3_WPITCH + 32 * s);
        acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b0, a, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b1, a, acc1, 0, 0, 0);
      }
      if (has_next) commit();                              // after this chunk's fragment reads, in order
    }

    // ---- epilogue: lane (l32, lh) holds pixel l32, channels 32*lh + 16*nb + e of the slice
    auto finish = [&](auto mode_tag) {
      constexpr int MODE = decltype(mode_tag)::value;      // 2 folded, 1 multiply-high, 0 64-bit
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const v16i& acc = nb == 0 ? acc0 : acc1;
        v4i out;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          int q[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            unsigned v = (unsigned)acc[4 * q4 + t];
            if (ADD) {
              v += (unsigned)addlut[((unsigned)addq[nb][q4] >> (8 * t)) & 0xffu];
            }
            q[t] = MODE == 2 ? requantize_folded((int)v, p.mant, fold, lo_v)
                             : requantize_as<MODE == 1>((int)v, p.mant, p.shift, p.y_off, p.lo);
          }
          out[q4] = (int)pack_codes(q[0], q[1], q[2], q[3]);
        }
        // channels are stored in runs of 16 (k % 16 == 0): a run is wholly inside or outside;
        // rows past M fall outside the output buffer's range and the checked store drops them
        if (ch0 + 16 * nb < p.k) __builtin_amdgcn_raw_buffer_store_b128(out, rsrc_y, off + 16u * nb, 0, 0);
      }
    };
    if (fold.ok) finish(std::integral_constant<int, 2>{});
    else if (fast) finish(std::integral_constant<int, 1>{});
    else finish(std::integral_constant<int, 0>{});
  }
}

// ---------------------------------------------------------------------------------------------------
// The same layer at stride 1, with the input staged once instead of once per filter row: a wavefront
// owns blocks of 4 x 8 output pixels and keeps the 6 x 10-pixel input patch of its block (64 codes per
// pixel) in its LDS region; the MFMA operand of tap (r, s) is then one 16-byte read at the lane's pixel
// shifted by (r, s), so nothing is fetched or stored twice (3.8 KB per block instead of 18 KB through
// the L2 -> LDS path, 4 loads and 4 LDS writes per lane and block instead of 18).  Pixel pitch 80 bytes
// and row pitch 896 bytes (= 128 mod 256) keep the fragment reads of 16 lanes (two rows of eight
// pixels) on distinct banks.  The next block's patch is in flight (registers) while the current block
// is multiplied and is written to the region after the block's last fragment read (a wavefront's LDS
// operations execute in order), as in the kernel above.  Patch pixels outside the image hold the
// input's offset code; which ones is a 60-bit mask built with scalar instructions from the block's
// position (the scalar unit is shared by the CU: positions are stepped, not divided out).
constexpr int T2_BH = 4, T2_BW = 8;            // block of output pixels
constexpr int T2_PH = T2_BH + 2, T2_PW = T2_BW + 2;
constexpr int T2_PP = 80;                      // bytes per patch pixel
constexpr int T2_RP = 896;                     // bytes per patch row
constexpr int T2_REGION = T2_PH * T2_RP;       // bytes per wavefront
constexpr int T2_LOADS = 4;                    // 16-byte loads per lane and block: 60 pixels x 4 quarters <= 256
static_assert(T2_PW * T2_PP <= T2_RP && T2_PH * T2_PW * 4 <= 64 * T2_LOADS, "patch geometry");

template <int WAVES>
constexpr int t2_lds_bytes() { return K3_BN * K3_WPITCH + WAVES * T2_REGION + K3_BN * 4 + 256 * 4; }

template <int WAVES, bool ADD>
__global__ __launch_bounds__(WAVES * 64, 1) void conv_k3c64_i8_tile_kernel(const Problem p, int blocks_y, int blocks_x,
                                                                           int items_div, int items_rem) {
  extern __shared__ __align__(16) unsigned char smem[];   // filter slice, patch regions, channel terms
  unsigned char* wlds = smem;
  int* cterm = reinterpret_cast<int*>(smem + K3_BN * K3_WPITCH + WAVES * T2_REGION);
  int* addlut = cterm + K3_BN;   // [256] the addend's code (as an unsigned byte) -> its term at the accumulator's scale

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int slice = blockIdx.y;
  unsigned char* alds = smem + K3_BN * K3_WPITCH + wave * T2_REGION;

  const int* __restrict__ bias = static_cast<const int*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_y =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)((unsigned)p.M * (unsigned)p.k), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_add = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(ADD ? p.addend : p.y), 0, (int)((unsigned)p.M * (unsigned)p.k), 0x00020000);
  constexpr unsigned OOB = 0x80000000u;          // past the end of any tensor this kernel accepts

  // ---- this wavefront's contiguous range of blocks (image major, then block row, then block column)
  const int wv = blockIdx.x * WAVES + wave;
  int it, it_end_;
  deal_range(wv, (int)gridDim.x * WAVES, items_div, items_rem, it, it_end_);
  const int it_end = it_end_;
  struct Pos {
    int bx, by, img;
  };
  auto advance = [&](Pos& q) {
    q.bx += 1;
    const bool wx = q.bx == blocks_x;
    q.bx = wx ? 0 : q.bx;
    q.by += wx ? 1 : 0;
    const bool wy = q.by == blocks_y;
    q.by = wy ? 0 : q.by;
    q.img += wy ? 1 : 0;
  };

  // ---- patch staging: load i of lane l covers quarter (l % 4) of patch pixel 16 i + l / 4
  unsigned g_rel[T2_LOADS], l_off[T2_LOADS];     // the pixel's offset from the patch origin in the input / in the region
#pragma unroll
  for (int i = 0; i < T2_LOADS; ++i) {
    const int pix = 16 * i + (lane >> 2), quarter = lane & 3;
    const int pr = pix / T2_PW, pc = pix - pr * T2_PW;                 // (pixels 60..63 do not exist: never inside)
    g_rel[i] = (unsigned)((pr * p.w_ + pc) * K3_C + 16 * quarter);
    l_off[i] = (unsigned)(pr * T2_RP + pc * T2_PP + 16 * quarter);
  }
  const unsigned fill = (unsigned)(p.x_off & 0xff) * 0x01010101u;
  v4i st[T2_LOADS];
  unsigned okbits = 0;                           // bit i: load i of the patch in flight was inside the image
  auto fetch = [&](const Pos& q) {
    const int ih0 = q.by * T2_BH - p.pad_t, iw0 = q.bx * T2_BW - p.pad_l;
    // rows / columns of the patch inside the image, as bit ranges (scalar)
    const int rlo = ih0 < 0 ? -ih0 : 0, rhi = p.h - ih0 < T2_PH ? p.h - ih0 : T2_PH;
    const int clo = iw0 < 0 ? -iw0 : 0, chi = p.w_ - iw0 < T2_PW ? p.w_ - iw0 : T2_PW;
    const unsigned rm = rhi > rlo ? (1u << rhi) - (1u << rlo) : 0u;
    const unsigned long long cm = chi > clo ? (unsigned long long)((1u << chi) - (1u << clo)) : 0ull;
    unsigned long long inside = 0;               // bit 10 pr + pc
#pragma unroll
    for (int pr = 0; pr < T2_PH; ++pr) inside |= ((rm >> pr) & 1u) ? cm << (T2_PW * pr) : 0ull;
    const unsigned base = (unsigned)((q.img * p.h + ih0) * p.w_ + iw0) * (unsigned)K3_C;   // may wrap: used with inside pixels only
    okbits = 0;
#pragma unroll
    for (int i = 0; i < T2_LOADS; ++i) {
      const unsigned m16 = (unsigned)(inside >> (16 * i)) & 0xffffu;   // scalar
      const unsigned ok = (m16 >> (lane >> 2)) & 1u;
      okbits |= ok << i;
      st[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, ok ? base + g_rel[i] : OOB, 0, 0);   // OOB: zeros, no access
    }
  };
  auto commit = [&]() {
#pragma unroll
    for (int i = 0; i < T2_LOADS; ++i) {
      v4i v = st[i];
      if (!((okbits >> i) & 1u)) { v[0] = (int)fill; v[1] = (int)fill; v[2] = (int)fill; v[3] = (int)fill; }
      if (16 * i + (lane >> 2) < T2_PH * T2_PW) *reinterpret_cast<v4i*>(alds + l_off[i]) = v;
    }
  };

  // the first patch's loads go out before the filter slice's, so both latencies overlap
  const bool has_work = it < it_end;
  Pos cur, nxt;
  {
    const int first = has_work ? it : 0;
    cur.bx = first % blocks_x;
    const int t2 = first / blocks_x;
    cur.by = t2 % blocks_y;
    cur.img = t2 / blocks_y;
    nxt = cur;
  }
  if (has_work) fetch(cur);

  // ---- filter slice -> LDS in MFMA row order (as in the kernel above)
  {
    constexpr int V4_PER_ROW = K3_K / 16;
    constexpr int TOTAL = K3_BN * V4_PER_ROW;
    constexpr int THREADS = WAVES * 64;
    constexpr int PASSES = (TOTAL + THREADS - 1) / THREADS;
    const unsigned base = (unsigned)slice * (unsigned)(K3_BN * K3_K);
    v4i stage[PASSES];
#pragma unroll
    for (int q = 0; q < PASSES; ++q) {
      const int i = tid + q * THREADS;
      stage[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, i < TOTAL ? base + (unsigned)i * 16u : OOB, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < PASSES; ++q) {
      const int i = tid + q * THREADS;
      const int ch = i / V4_PER_ROW, kq = i % V4_PER_ROW;
      if (i < TOTAL) *reinterpret_cast<v4i*>(wlds + k3_staged_row(ch) * K3_WPITCH + kq * 16) = stage[q];
    }
  }
  __syncthreads();
  if (ADD && tid < 256) addlut[tid] = rescale_term((int)(signed char)tid - p.r_off, p.r_mant, p.r_shift);
  if (tid < K3_BN) {
    const int ch = slice * K3_BN + tid;
    const unsigned char* wrow = wlds + k3_staged_row(tid) * K3_WPITCH;
    int wsum = 0;
#pragma unroll 4
    for (int j = 0; j < K3_K / 16; ++j) {
      const v4i v = *reinterpret_cast<const v4i*>(wrow + 16 * j);
#pragma unroll
      for (int t = 0; t < 4; ++t) wsum = __builtin_amdgcn_sdot4(v[t], 0x01010101, wsum, false);
    }
    unsigned ct = 0u - (unsigned)p.x_off * (unsigned)wsum;
    if (bias && ch < p.k) ct += (unsigned)bias[ch];
    cterm[tid] = (int)ct;
  }
  __syncthreads();
  if (!has_work) return;

  // lane = pixel (row l32 / 8, column l32 % 8 of the block) as the MFMA column operand
  const int py = l32 >> 3, px = l32 & 7;
  const unsigned char* a_lane = alds + py * T2_RP + px * T2_PP + 16 * lh;
  const unsigned char* w_lane = wlds + l32 * K3_WPITCH + 16 * lh;
  const bool fast = p.shift >= 33;                         // uniform
  const FoldedRequant fold = make_folded_requant(p.shift, p.y_off);   // uniform
  const int lo_v = p.lo;
  const int ch0 = slice * K3_BN + 32 * lh;                 // first of the lane's 32 channels
  const unsigned lane_off = (unsigned)((py * p.ow + px) * p.k + ch0);

  commit();
  for (; it < it_end; ++it) {
    const bool more = it + 1 < it_end;                     // uniform: this wavefront owns the next block too
    if (more) {
      advance(nxt);
      fetch(nxt);
    }
    const int oh0 = cur.by * T2_BH, ow0 = cur.bx * T2_BW;  // uniform
    const bool pix_ok = py < p.oh - oh0 && px < p.ow - ow0;
    // pixels outside the output get an offset past its end: the range-checked accesses drop them
    const unsigned off = pix_ok ? (unsigned)(((cur.img * p.oh + oh0) * p.ow + ow0) * p.k) + lane_off : OOB;
    cur = nxt;
    // the lane's 32 addend codes, fetched ahead of the MFMAs
    v4i addq[2];
    if (ADD) {
      addq[0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_add, off, 0, 0);
      addq[1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_add, off + 16u, 0, 0);
    }
    // the accumulators start at the channel terms: register e of acc<nb> = channel 32*lh + 16*nb + e
    v16i acc0, acc1;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const v4i c0 = *reinterpret_cast<const v4i*>(cterm + 32 * lh + 4 * q4);
      const v4i c1 = *reinterpret_cast<const v4i*>(cterm + 32 * lh + 16 + 4 * q4);
#pragma unroll
      for (int t = 0; t < 4; ++t) { acc0[4 * q4 + t] = c0[t]; acc1[4 * q4 + t] = c1[t]; }
    }
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int s = 0; s < 3; ++s)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          // 32 codes of tap (r, s): each lane feeds 16 consecutive ones of its shifted pixel
          const v4i a = *reinterpret_cast<const v4i*>(a_lane + r * T2_RP + s * T2_PP + 32 * q);
          const unsigned char* wl = w_lane + (r * 3 + s) * K3_C + 32 * q;
          const v4i b0 = *reinterpret_cast<const v4i*>(wl);
          const v4i b1 = *reinterpret_cast<const v4i*>(wl + 32 * K3_WPITCH);
          acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b0, a, acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b1, a, acc1, 0, 0, 0);
        }
    if (more) commit();                                    // after this block's fragment reads, in order

    // ---- epilogue: lane (l32, lh) holds its pixel's channels 32*lh + 16*nb + e of the slice
    auto finish = [&](auto mode_tag) {
      constexpr int MODE = decltype(mode_tag)::value;      // 2 folded, 1 multiply-high, 0 64-bit
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const v16i& acc = nb == 0 ? acc0 : acc1;
        v4i out;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          int q[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            unsigned v = (unsigned)acc[4 * q4 + t];
            if (ADD) v += (unsigned)addlut[((unsigned)addq[nb][q4] >> (8 * t)) & 0xffu];
            q[t] = MODE == 2 ? requantize_folded((int)v, p.mant, fold, lo_v)
                             : requantize_as<MODE == 1>((int)v, p.mant, p.shift, p.y_off, p.lo);
          }
          out[q4] = (int)pack_codes(q[0], q[1], q[2], q[3]);
        }
        // channels are stored in runs of 16 (k % 16 == 0): a run is wholly inside or outside
        if (ch0 + 16 * nb < p.k) __builtin_amdgcn_raw_buffer_store_b128(out, rsrc_y, off + 16u * nb, 0, 0);
      }
    };
    if (fold.ok) finish(std::integral_constant<int, 2>{});
    else if (fast) finish(std::integral_constant<int, 1>{});
    else finish(std::integral_constant<int, 0>{});
  }
}

int k3_min_blocks() {
  return knob_or(KNOB_I8_K3_MIN_BLOCKS, 768);   // measured on 56 x 56 maps: batch 8 (784 blocks) 8.0 -> 7.5 us, batch 4 and below no faster than the tiled kernel
}

template <int WAVES, bool ADD>
hipError_t launch_k3(const Problem& p, hipStream_t stream) {
  auto kern = conv_k3c64_i8_kernel<WAVES, ADD>;
  constexpr int lds = k3_lds_bytes<WAVES>();
  // once per instantiation; initialisation of a function-local static is thread-safe
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (attr_status != hipSuccess) return attr_status;
  const int num_cu = num_compute_units();
  if (num_cu < 1) return hipErrorInvalidDevice;
  const int slices = (p.k + K3_BN - 1) / K3_BN;
  const int row_blocks = (p.M + 31) / 32;
  long long wgs = num_cu / slices;                                    // persistent workgroups per slice
  if (wgs < 1) wgs = 1;
  if (wgs > (row_blocks + WAVES - 1) / WAVES) wgs = (row_blocks + WAVES - 1) / WAVES;
  const long long waves = wgs * WAVES;
  dim3 grid((unsigned)wgs, (unsigned)slices, 1), block(WAVES * 64, 1, 1);
  hipLaunchKernelGGL(kern, grid, block, lds, stream, p, (int)(row_blocks / waves), (int)(row_blocks % waves));
  return hipGetLastError();
}

template <int WAVES, bool ADD>
hipError_t launch_t2(const Problem& p, hipStream_t stream) {
  auto kern = conv_k3c64_i8_tile_kernel<WAVES, ADD>;
  constexpr int lds = t2_lds_bytes<WAVES>();
  // once per instantiation; initialisation of a function-local static is thread-safe
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (attr_status != hipSuccess) return attr_status;
  const int num_cu = num_compute_units();
  if (num_cu < 1) return hipErrorInvalidDevice;
  const int slices = (p.k + K3_BN - 1) / K3_BN;
  const int blocks_y = (p.oh + T2_BH - 1) / T2_BH, blocks_x = (p.ow + T2_BW - 1) / T2_BW;
  const long long items = (long long)p.n * blocks_y * blocks_x;
  long long wgs = num_cu / slices;                                    // persistent workgroups per slice
  if (wgs < 1) wgs = 1;
  if (wgs > (items + WAVES - 1) / WAVES) wgs = (items + WAVES - 1) / WAVES;
  const long long waves = wgs * WAVES;
  dim3 grid((unsigned)wgs, (unsigned)slices, 1), block(WAVES * 64, 1, 1);
  hipLaunchKernelGGL(kern, grid, block, lds, stream, p, blocks_y, blocks_x, (int)(items / waves), (int)(items % waves));
  return hipGetLastError();
}

}  // namespace

bool k3c64_i8_applicable(const Problem& p) {
  if (p.b_is_kn || p.groups != 1 || p.r != 3 || p.s != 3 || p.c != K3_C) return false;
  if (p.w_off != 0 || p.k % 16 != 0 || p.k > 65536) return false;
  if (p.x_bytes > 0x7FFFFFFFu || p.w_bytes > 0x7FFFFFFFu) return false;
  if ((unsigned long long)p.M * (unsigned long long)p.k > 0x7FFFFFFFull) return false;
  const int blocks = (p.M + 31) / 32;
  return blocks >= k3_min_blocks();
}

hipError_t launch_k3c64_i8(const Problem& p, hipStream_t stream, const char** variant) {
  int waves = 16;     // four wavefronts per SIMD hide the chunk hand-over better than two (measured)
  waves = knob_or(KNOB_I8_K3_WAVES, waves);                                // experiments and tests
  // stride 1: the form that stages each block's input patch once; other strides gather per filter row
  const long long t2_items = (long long)p.n * ((p.oh + T2_BH - 1) / T2_BH) * ((p.ow + T2_BW - 1) / T2_BW);
  bool tiled = p.stride_h == 1 && p.stride_w == 1 && t2_items < (1LL << 30);
  if (knob_or(KNOB_I8_K3_GATHER, 0) != 0) tiled = false;                   // experiments and tests
  static thread_local char name[48];
  snprintf(name, sizeof(name), "conv_k3c64_i8_w%d%s%s", waves == 8 ? 8 : 16, tiled ? "_2d" : "", p.addend ? "_add" : "");
  *variant = name;
  if (tiled) {
    if (waves != 8) return p.addend ? launch_t2<16, true>(p, stream) : launch_t2<16, false>(p, stream);
    return p.addend ? launch_t2<8, true>(p, stream) : launch_t2<8, false>(p, stream);
  }
  if (waves != 8) return p.addend ? launch_k3<16, true>(p, stream) : launch_k3<16, false>(p, stream);
  return p.addend ? launch_k3<8, true>(p, stream) : launch_k3<8, false>(p, stream);
}

}  // namespace glowmi
