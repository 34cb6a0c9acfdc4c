// int8 Convolution for the few-input-channel first layer (7x7 stride 2 on 3 channels), quantized form
// of Section 4 of the paper; the same "small number of channels" kind of convolution that the
// paper's CPU backend gives its own strategy (Section 5.3).
//
// The generic int8 kernel would gather this layer byte by byte.  Here a wavefront keeps the input
// patch of a 2 x 16 pixel block of outputs in a private LDS region with every pixel widened from 3 to
// 4 codes (one dword), so that for one filter row r the codes a pixel needs -- 8 pixels x 4 codes =
// 32 bytes, the 8th pixel and the 4th code being padding that meets a zero filter code -- are
// contiguous and 8-byte aligned: one v_mfma_i32_32x32x32_i8 per filter row and half of the 64
// channels, its pixel operand two ds_read_b64.  Out-of-image pixels are staged as the code x_off
// (real zero).  The next block's patch is fetched into registers while the current one is
// multiplied and written to the region afterwards (a wavefront's LDS operations execute in order),
// so after the prologue there is no workgroup barrier and blocks are dealt to wavefronts, not to
// workgroups.  The filter fragments (2 x 7 rows x 16 bytes per lane, the same for every wavefront)
// are built once per persistent workgroup, straight from global memory, and kept in LDS, with the channels dealt to MFMA rows so
// that a lane ends with 32 consecutive channels of its pixel.  Offsets are removed after the MFMAs:
//   sum (x - xo) * w = sum x*w - xo * sum w          (this kernel requires a filter offset of 0)
// then bias, requantize, clamp (Relu = lower bound), pack, two 16-byte stores per lane.  The layer
// is bound by that per-output arithmetic and by the 64 bytes written per pixel, not by the MFMAs.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <type_traits>

#include "igemm.h"
#include "pw_common.h"
#include "quant_epilogue.h"

namespace glowmi {
namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BH = 2, BW = 16;            // block of output pixels of one wavefront
constexpr int QS_THREADS = 256;
constexpr int QS_WAVES = QS_THREADS / 64;
constexpr int R = 7, S = 7, C = 3, STRIDE = 2;
constexpr int FB = R * S * C;                             // filter bytes per channel
constexpr int PH = (BH - 1) * STRIDE + R;                 // 9 patch rows
constexpr int PW = (BW - 1) * STRIDE + S + 1;             // 38 pixels: one more than needed, read by the padding tap
constexpr int PITCH = 40;                                 // dwords per patch row
constexpr int PATCH = PH * PITCH;                         // dwords per wavefront
constexpr int LDS_DWORDS = QS_WAVES * PATCH + 2 * R * 64 * 4 + 64;   // patches, filter fragments, per-channel term
static_assert(PATCH % 4 == 0 && PW <= 64, "16-byte alignment of the LDS areas; one lane per patch column");

// Channel (0..63) whose filter is MFMA row j (0..31) of channel block nb (0/1).  Result register e of
// a lane with half h is MFMA row (e/4)*8 + 4h + e%4; this assignment makes that row channel
// 32h + 16nb + e, so a lane's 16 registers of a block are 16 consecutive channels.
__device__ __forceinline__ int channel_of_row(int nb, int j) {
  return 32 * ((j >> 2) & 1) + 16 * nb + (j >> 3) * 4 + (j & 3);
}

// The 4 bytes at byte offset `off` of a buffer of `bytes` bytes (>= 4), any alignment, with bytes past
// the end reading as zero, in two steps so that a lane's loads are all in flight before the first
// result is touched: load4_issue fetches the dword (from the last whole dword of the buffer when the
// wanted one would straddle or pass the end: a range-checked load would drop a straddling dword as a
// whole) and load4_over says by how many bytes (at most 4) the result must be shifted down.
__device__ __forceinline__ unsigned load4_over(unsigned off, unsigned bytes) {
  const unsigned last = bytes - 4u;
  const unsigned over = off < last ? 0u : off - last;
  return over < 4u ? over : 4u;
}
__device__ __forceinline__ unsigned load4_issue(__amdgpu_buffer_rsrc_t rsrc, unsigned off, unsigned bytes) {
  const unsigned last = bytes - 4u;
  return (unsigned)__builtin_amdgcn_raw_buffer_load_b32(rsrc, off < last ? off : last, 0, 0);
}
__device__ __forceinline__ unsigned load4_shift(unsigned d, unsigned over) {
  return (unsigned)((unsigned long long)d >> (8u * over));
}

__global__ __launch_bounds__(QS_THREADS, 4) void conv_smallc_i8_kernel(const Problem p, int blocks_y, int blocks_x,
                                                                      int items_div, int items_rem) {
  __shared__ __align__(16) int lds[LDS_DWORDS];
  v4i* wfrag = reinterpret_cast<v4i*>(lds + QS_WAVES * PATCH);            // [2][R][64 lanes]
  int* cterm = lds + QS_WAVES * PATCH + 2 * R * 64 * 4;                   // [64]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lrow = lane & 31, lhalf = lane >> 5;
  const int n_tile = blockIdx.y;
  int* patch = lds + wave * PATCH;                         // [PH][PITCH] dwords, one pixel each

  const int* __restrict__ bias = static_cast<const int*>(p.bias);
  signed char* __restrict__ Y = static_cast<signed char*>(p.y);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);

  const unsigned xo_byte = (unsigned)p.x_off & 0xffu;
  const unsigned xo_pix = xo_byte * 0x01010101u;

  // ---- this wavefront's contiguous range of pixel blocks (image major, then block row, then column)
  const int wv = blockIdx.x * QS_WAVES + wave;
  int it, it_end_;
  deal_range(wv, (int)gridDim.x * QS_WAVES, items_div, items_rem, it, it_end_);
  const int it_end = it_end_;

  // ---- input patch: lane l < PW fetches column l of each of the PH patch rows, one pixel (3 codes)
  // per load as the 4 bytes that start at the pixel; the 4th byte (the next pixel's first code) is
  // replaced by x_off when the pixel is written to LDS, a block later.  Every load is issued
  // unconditionally at an address inside the tensor: a branch around a load, which is what the
  // compiler makes of a conditional on a loaded value, would put a wait behind each of them.  Rows
  // are uniform over the wavefront, so their part of the address and their validity are scalar.
  // The dword of the very last pixel of the tensor would end one byte outside: that one load starts
  // a byte earlier and is shifted before use (tail_row >= 0 only in the block that holds the pixel).
  unsigned stage[PH];
  bool col_ok = false;        // the lane's patch column lies inside the image
  unsigned row_mask = 0;      // bit i: patch row i lies inside the image (uniform)
  int tail_row = -1, tail_lane = -1;
  // Position of an item as (block column, block row, image), stepped instead of divided out per item:
  // the scalar unit is shared by the whole CU and a block is only a few hundred vector instructions.
  struct Pos {
    int bx, by, img;
  };
  auto pos_of = [&](int item) {
    Pos q;
    q.bx = item % blocks_x;
    const int t2 = item / blocks_x;
    q.by = t2 % blocks_y;
    q.img = t2 / blocks_y;
    return q;
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
  auto load_patch = [&](const Pos& q) {
    const int ih0 = q.by * BH * STRIDE - p.pad_t;
    const int iw0 = q.bx * BW * STRIDE - p.pad_l;
    const int iw = iw0 + lane;
    col_ok = lane < PW && (unsigned)iw < (unsigned)p.w_;
    tail_lane = p.w_ - 1 - iw0;
    tail_row = q.img == p.n - 1 && tail_lane < PW ? p.h - 1 - ih0 : -1;
    if (tail_row >= PH) tail_row = -1;
    const unsigned voff = col_ok ? (unsigned)iw * (unsigned)C : 0u;
    const unsigned row_bytes = (unsigned)p.w_ * (unsigned)C;
    if (ih0 >= 0 && ih0 + PH <= p.h && tail_row < 0) {
      // all patch rows inside the image, and not the block with the tensor's last pixel (almost every
      // block): one scalar add per row
      row_mask = (1u << PH) - 1u;
      unsigned soff = (unsigned)(q.img * p.h + ih0) * row_bytes;
#pragma unroll
      for (int i = 0; i < PH; ++i) {
        stage[i] = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(rsrc_x, voff, soff, 0);
        soff += row_bytes;
      }
      return;
    }
    row_mask = 0;
#pragma unroll
    for (int i = 0; i < PH; ++i) {
      const int ih = ih0 + i;
      const bool rok = (unsigned)ih < (unsigned)p.h;
      row_mask |= (rok ? 1u : 0u) << i;
      const unsigned soff = rok ? (unsigned)(q.img * p.h + ih) * row_bytes : 0u;
      unsigned vo = voff;
      if (i == tail_row && lane == tail_lane) vo -= 1u;     // (uniform test first: false almost always)
      stage[i] = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(rsrc_x, vo, soff, 0);
    }
  };
  auto store_patch = [&]() {
    if (tail_row >= 0) {
#pragma unroll
      for (int i = 0; i < PH; ++i)
        if (i == tail_row && lane == tail_lane) stage[i] >>= 8;
    }
#pragma unroll
    for (int i = 0; i < PH; ++i) {
      const bool ok = col_ok && ((row_mask >> i) & 1u);
      const unsigned v = ok ? (stage[i] & 0x00ffffffu) | (xo_byte << 24) : xo_pix;
      if (lane < PW) patch[i * PITCH + lane] = (int)v;
    }
  };

  const bool has_work = it < it_end;
  Pos cur = pos_of(has_work ? it : 0), nxt = cur;
  if (has_work) load_patch(cur);           // in flight while the filter is fetched

  // ---- filter fragments: for channel block nb and filter row r, lane (MFMA row j, half) feeds the 16
  // codes W[channel_of_row(nb, j)][r][s = 4*half + 0..3][c = 0..3]; s = 7 and c = 3 do not exist and
  // are zero codes.  The 12 bytes a lane needs for one fragment are contiguous in the [k][7][7][3]
  // filter: three dword loads at any alignment, all 21 of a lane in flight together, repacked 3 -> 4
  // bytes per tap.  Wavefront nb (0/1) builds the seven fragments of its channel block, which are the
  // same for every wavefront and stay in LDS in lane order (one conflict-free 16-byte read per
  // MFMA), and from them the per-channel term  bias - x_off * sum(w)  (modulo 2^32, exact because the
  // true value fits).  Channels past the last one read as zeros.
  if (wave < 2) {
    const int nb = wave;
    const int lc = channel_of_row(nb, lrow);
    const int ch = n_tile * 64 + lc;
    const unsigned base = (unsigned)ch * (unsigned)FB + 12u * lhalf;
    unsigned wd[R][3];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < 3; ++j) wd[r][j] = load4_issue(rsrc_w, base + (unsigned)(r * S * C + 4 * j), p.w_bytes);
    int wsum = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      unsigned w[3];
#pragma unroll
      for (int j = 0; j < 3; ++j)
        w[j] = load4_shift(wd[r][j], load4_over(base + (unsigned)(r * S * C + 4 * j), p.w_bytes));
      v4i frag;
      frag[0] = (int)(w[0] & 0x00ffffffu);
      frag[1] = (int)(((w[0] >> 24) | (w[1] << 8)) & 0x00ffffffu);
      frag[2] = (int)(((w[1] >> 16) | (w[2] << 16)) & 0x00ffffffu);
      frag[3] = lhalf ? 0 : (int)(w[2] >> 8);               // tap 7 does not exist
#pragma unroll
      for (int si = 0; si < 4; ++si) wsum = __builtin_amdgcn_sdot4(frag[si], 0x01010101, wsum, false);
      wfrag[(nb * R + r) * 64 + lane] = frag;
    }
    wsum += __shfl_xor(wsum, 32);            // both halves of the channel's filter
    if (lhalf == 0) {
      unsigned ct = 0u - (unsigned)p.x_off * (unsigned)wsum;
      if (ch < p.k && bias) ct += (unsigned)bias[ch];
      cterm[lc] = (int)ct;
    }
  }
  __syncthreads();                           // fragments and channel terms; the only barrier of the kernel
  if (!has_work) return;

  // lane = pixel (row lrow / 16 of the block's two, column lrow % 16) as the MFMA column operand
  const int* src = patch + ((lrow >> 4) * STRIDE) * PITCH + (lrow & 15) * STRIDE + 4 * lhalf;
  const FoldedRequant fold = make_folded_requant(p.shift, p.y_off);   // uniform
  const bool fast = p.shift >= 33;           // uniform
  const bool wide = p.k % 16 == 0;           // uniform: runs of 16 channels are wholly inside or outside
  const int col0 = n_tile * 64 + 32 * lhalf; // first of the lane's 32 channels
  const int lo_v = p.lo;
  // the lane's part of the output address, the same for every block
  const int prow = lrow >> 4, pcol = lrow & 15;
  const size_t lane_off = ((size_t)prow * p.ow + pcol) * p.k + col0;

  store_patch();
  for (; it < it_end; ++it) {
    const bool has_next = it + 1 < it_end;
    if (has_next) {
      advance(nxt);
      load_patch(nxt);
    }

    // the accumulators start at the channel terms: register e of block nb = channel 32*half + 16*nb + e
    v16i acc[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const v4i ct = *reinterpret_cast<const v4i*>(cterm + 32 * lhalf + 16 * nb + 4 * q4);
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[nb][4 * q4 + t] = ct[t];
      }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int* a = src + r * PITCH;
      const v2i lo2 = *reinterpret_cast<const v2i*>(a);
      const v2i hi2 = *reinterpret_cast<const v2i*>(a + 2);
      const v4i av = {lo2[0], lo2[1], hi2[0], hi2[1]};
      // filter fragment as the row operand: result rows = channels, columns = pixels
      acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wfrag[r * 64 + lane], av, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wfrag[(R + r) * 64 + lane], av, acc[1], 0, 0, 0);
    }

    if (has_next) store_patch();             // after this block's reads, in order

    // ---- epilogue: requantize, clamp, pack, store the lane's 32 channels of pixel lane % 32
    const int oh0 = cur.by * BH, ow0 = cur.bx * BW;         // uniform
    const bool pix_ok = prow < p.oh - oh0 && pcol < p.ow - ow0;
    signed char* dst = Y + (((size_t)cur.img * p.oh + oh0) * p.ow + ow0) * p.k + lane_off;
    cur = nxt;
    auto finish = [&](auto mode_tag) {
      constexpr int MODE = decltype(mode_tag)::value;      // 2 folded, 1 multiply-high, 0 64-bit
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        v4i out;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          int q[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int v = acc[nb][4 * q4 + t];
            q[t] = MODE == 2 ? requantize_folded(v, p.mant, fold, lo_v)
                             : requantize_as<MODE == 1>(v, p.mant, p.shift, p.y_off, p.lo);
          }
          out[q4] = (int)pack_codes(q[0], q[1], q[2], q[3]);
        }
        const int col = col0 + 16 * nb;
        if (!pix_ok || col >= p.k) continue;
        if (wide) {
          *reinterpret_cast<v4i*>(dst + 16 * nb) = out;
        } else {
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (col + e < p.k) dst[16 * nb + e] = (signed char)((unsigned)out[e >> 2] >> (8 * (e & 3)));
        }
      }
    };
    if (fold.ok) finish(std::integral_constant<int, 2>{});
    else if (fast) finish(std::integral_constant<int, 1>{});
    else finish(std::integral_constant<int, 0>{});
  }
}

}  // namespace

bool smallc_i8_applicable(const Problem& p) {
  return !p.b_is_kn && p.groups == 1 && p.r == R && p.s == S && p.c == C && p.stride_h == STRIDE &&
         p.stride_w == STRIDE && p.w_off == 0 && p.x_bytes >= 4u && p.x_bytes <= 0x7FFFFFFFu &&
         p.w_bytes <= 0x7FFFFFFFu &&
         (long long)p.n * ((p.oh + BH - 1) / BH) * ((p.ow + BW - 1) / BW) < (1LL << 30);
}

hipError_t launch_smallc_i8(const Problem& p, hipStream_t stream, const char** variant) {
  *variant = "conv_smallc_i8_7x7s2c3";
  auto kern = conv_smallc_i8_kernel;
  const int num_cu = num_compute_units();
  if (num_cu < 1) return hipErrorInvalidDevice;
  const int blocks_y = (p.oh + BH - 1) / BH, blocks_x = (p.ow + BW - 1) / BW;
  const long long items = (long long)p.n * blocks_y * blocks_x;
  const int n_tiles = (p.k + 63) / 64;
  int per_cu = 4;            // persistent workgroups per CU (measured: 3, 4 and 5 are within 1 % at batch 32; 4 is best at batch 1)
  per_cu = knob_or(KNOB_SMALLC_I8_WGS, per_cu);                               // experiments
  if (per_cu < 1) per_cu = 1;
  if (per_cu > 8) per_cu = 8;
  long long gx = (long long)num_cu * per_cu / n_tiles;
  if (gx < 1) gx = 1;
  if (gx > (items + QS_WAVES - 1) / QS_WAVES) gx = (items + QS_WAVES - 1) / QS_WAVES;
  const long long waves = gx * QS_WAVES;
  dim3 grid((unsigned)gx, n_tiles, 1), block(QS_THREADS, 1, 1);
  hipLaunchKernelGGL(kern, grid, block, 0, stream, p, blocks_y, blocks_x, (int)(items / waves), (int)(items % waves));
  return hipGetLastError();
}

}  // namespace glowmi
