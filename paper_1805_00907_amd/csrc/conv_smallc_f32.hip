// fp32 Convolution for layers with very few input channels (a network's first layer: 7x7 stride 2 on
// 3 channels).  The paper's CPU backend singles out "convolutions with a small number of channels"
// as one of three kinds that get their own strategy (Section 5.3); this is that kind on gfx950.
//
// With 3 channels the generic implicit-GEMM gather degenerates into scalar loads with per-element
// index arithmetic and the vector ALUs, not the matrix cores, set the pace.  Here instead:
//   - a workgroup owns a tile of 8 x 16 output pixels and 64 output channels and keeps the raw
//     input patch it needs ((8-1)*stride + R rows of (16-1)*stride + S pixels, all channels) in LDS,
//     fetched with fully coalesced row loads and zero-filled outside the image (double buffered:
//     the next tile's patch is in flight during the MFMAs);
//   - the reduction index v = (r, s, c) is walked two at a time (v_mfma_f32_32x32x2_f32).  Within a
//     filter row r the (s, c) run is contiguous both in the patch and in the filter, so the A
//     operand of a lane is one ds_read_b32 at a compile-time offset from a per-lane base;
//   - the filter fragment of the wavefront's 32 output channels (ceil(R*S*C/2) registers per lane)
//     is loaded once and stays in registers while the persistent workgroup walks over its tiles.
// Epilogue as everywhere: bias + Relu on the accumulators, one store.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <type_traits>

#include "f16_pieces.h"
#include "igemm.h"

namespace glowmi {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int TW = 16;                  // output tile width (pixels); 4 wavefronts = 2 pixel halves x 2 channel halves
// Tile height TH = 8 (each wavefront two 32-pixel MFMA blocks) or 4 (one block): the persistent grid
// walks total_tiles / workgroups tiles each, and with few tiles per workgroup the taller tile loses a
// fifth of the chip to the uneven last round (3136 tiles on 768 workgroups: 5 rounds for 4.08).
constexpr int SC_THREADS = 256;

template <int R, int S, int C, int STRIDE, int TH>
struct SmallC {
  static constexpr int K = R * S * C;                    // reduction length
  static constexpr int STEPS = (K + 1) / 2;              // MFMA steps (two k each)
  static constexpr int RUN = S * C;                      // contiguous (s, c) run per filter row
  static constexpr int PH = (TH - 1) * STRIDE + R;       // patch rows
  static constexpr int PWC = ((TW - 1) * STRIDE + S) * C;   // patch row length in floats
  static constexpr int PITCH = ((PWC + 15) / 16) * 16;   // multiple of 16 floats: see bank note below
  static constexpr int PATCH = (PH + 1) * PITCH;         // +1 row: the k = K padding step reads it
  static constexpr int LOADS = (PH * PWC + SC_THREADS - 1) / SC_THREADS;
  // two patch buffers; the same space first holds half a filter slice (32 channels) while the
  // filter fragments are picked
  static constexpr int lds_bytes = (2 * PATCH > 32 * K ? 2 * PATCH : 32 * K) * (int)sizeof(float);
  // patch offset of reduction index v relative to a pixel's patch origin
  static constexpr int off(int v) { return (v / RUN) * PITCH + (v % RUN); }
};

template <int R, int S, int C, int STRIDE, int TH>
__global__ __launch_bounds__(SC_THREADS) void conv_smallc_f32_kernel(const Problem p, int tiles_y, int tiles_x,
                                                                    int total_tiles) {
  using G = SmallC<R, S, C, STRIDE, TH>;
  static_assert(TH == 4 || TH == 8, "tile height");
  constexpr int NB = TH / 4;             // 32-pixel blocks (2 rows x 16) per wavefront
  extern __shared__ __align__(16) float patch[];          // [2][PH + 1][PITCH]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lrow = lane & 31, lhalf = lane >> 5;
  const int wpix = wave >> 1;            // which half of the tile's pixels (rows 2*NB*wpix .. + 2*NB - 1)
  const int wch = wave & 1;              // which 32 of the 64 output channels
  const int n_tile = blockIdx.y;

  const float* __restrict__ X = static_cast<const float*>(p.x);
  const float* __restrict__ Wt = static_cast<const float*>(p.w);
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_y = __builtin_amdgcn_make_buffer_rsrc(
      p.y, 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);

  const int ch = n_tile * 64 + wch * 32 + lrow;
  const bool ch_ok = ch < p.k;
  const float bv = (ch_ok && bias) ? bias[ch] : 0.f;

  // ---- per-lane patch bases.  Lane = pixel (prow, pcol) of a 32-pixel MFMA block (2 rows x 16)
  // and half h; step t reads patch[origin + off(2t + h)].  off(2t+1) - off(2t) is 1 except where the
  // pair straddles two filter rows; a second base register covers those steps, so every read uses a
  // compile-time immediate.  Bank note: pixels of a row are 6 floats apart and PITCH is a multiple
  // of 16, so the 64 lanes of one read hit 64 different banks.
  const int pix_origin = ((wpix * 2 * NB + (lrow >> 4)) * STRIDE) * G::PITCH + (lrow & 15) * STRIDE * C;
  const int base_norm = pix_origin + lhalf;                          // off(2t+1) = off(2t) + 1
  const int base_cross = pix_origin + lhalf * (G::PITCH - (G::RUN - 1));   // 2t is the last index of a run


  float stage[G::LOADS];
  auto load_patch = [&](int tile) {
    const int tx = tile % tiles_x;
    const int t2 = tile / tiles_x;
    const int ty = t2 % tiles_y;
    const int img = t2 / tiles_y;
    const int ih0 = ty * TH * STRIDE - p.pad_t;
    const int fx0 = (tx * TW * STRIDE - p.pad_l) * C;                // float offset inside an image row
    const int row_floats = p.w_ * C;
#pragma unroll
    for (int i = 0; i < G::LOADS; ++i) {
      const int idx = tid + i * SC_THREADS;
      const int pr = idx / G::PWC, pc = idx % G::PWC;               // compile-time divisor
      const int ih = ih0 + pr, fx = fx0 + pc;
      const bool ok = idx < G::PH * G::PWC && (unsigned)ih < (unsigned)p.h && (unsigned)fx < (unsigned)row_floats;
      stage[i] = ok ? X[((size_t)img * p.h + ih) * row_floats + fx] : 0.f;
    }
  };
  auto store_patch = [&](int buf) {
    float* dst = patch + buf * G::PATCH;
#pragma unroll
    for (int i = 0; i < G::LOADS; ++i) {
      const int idx = tid + i * SC_THREADS;
      if (idx < G::PH * G::PWC) dst[(idx / G::PWC) * G::PITCH + idx % G::PWC] = stage[i];
    }
  };

  // persistent walk over tiles: blockIdx.x, + gridDim.x, ...
  int tile = blockIdx.x;
  if (tile >= total_tiles) return;
  load_patch(tile);                        // in flight while the filter is fetched

  // ---- filter fragment: lane (channel, half) keeps W[channel][2t + half] for every step t.  Picked
  // straight from global memory every lane of a load sits on its own cache line (channels are K
  // floats apart) and the 74 loads of a wavefront keep the CU's address unit busy for ~5000 cycles,
  // times the wavefronts resident on the CU: a quarter of the whole layer at batch 32.  Instead the
  // 32 channels of each channel half (32 x K floats, contiguous in memory) are copied into LDS
  // with coalesced loads, in the space of the patch buffers, and the lanes pick from there; rows past
  // the last output channel lie past the end of the tensor and the range-checked loads return zeros.
  float wfrag[G::STEPS];
  {
    const __amdgpu_buffer_rsrc_t rsrc_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Wt), 0, (int)p.w_bytes, 0x00020000);
    constexpr int HALF_FLOATS = 32 * G::K;
    constexpr int W_LOADS = (HALF_FLOATS + SC_THREADS - 1) / SC_THREADS;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const unsigned base = (unsigned)((n_tile * 64 + half * 32) * G::K) * 4u;
      float wst[W_LOADS];
#pragma unroll
      for (int i = 0; i < W_LOADS; ++i) {
        const int e = tid + i * SC_THREADS;
        wst[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                               rsrc_w, e < HALF_FLOATS ? base + 4u * e : 0xFFFFFFFCu, 0, 0));
      }
#pragma unroll
      for (int i = 0; i < W_LOADS; ++i) {
        const int e = tid + i * SC_THREADS;
        if (e < HALF_FLOATS) patch[e] = wst[i];
      }
      __syncthreads();
      if (wch == half) {
#pragma unroll
        for (int t = 0; t < G::STEPS; ++t) {
          const int v = 2 * t + lhalf;
          wfrag[t] = v < G::K ? patch[lrow * G::K + v] : 0.f;
        }
      }
      __syncthreads();
    }
  }
  // zero the padding row of both buffers once (never overwritten by patch loads)
  for (int i = tid; i < G::PITCH; i += SC_THREADS) {
    patch[G::PH * G::PITCH + i] = 0.f;
    patch[G::PATCH + G::PH * G::PITCH + i] = 0.f;
  }
  store_patch(0);
  __syncthreads();
  int buf = 0;
  for (;;) {
    const int next = tile + gridDim.x;
    const bool has_next = next < total_tiles;
    if (has_next) load_patch(next);

    v16f acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    const float* src = patch + buf * G::PATCH;
    const float* pn = src + base_norm;
    const float* pc_ = src + base_cross;
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t) {
      constexpr int blk = 2 * STRIDE * G::PITCH;                     // second 32-pixel block: two rows down
      const bool cross = (2 * t) % G::RUN == G::RUN - 1;             // compile-time after unrolling
      const float* b = cross ? pc_ : pn;
      const int o = G::off(2 * t);
#pragma unroll
      for (int i = 0; i < NB; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[o + i * blk], wfrag[t], acc[i], 0, 0, 0);
    }

    if (has_next) store_patch(buf ^ 1);

    // ---- epilogue of this tile.  32x32 result: register e of a lane is pixel (e/4)*8 + 4*half + e%4
    // of the block (2 rows x 16 columns), channel = lane % 32: relative to the lane's first pixel
    // (row 0, column 4*half) register e lies drow = e/8 rows down and dcol = e%4 + 8*((e/4)%2) columns
    // right.  The stores go through a range-checked buffer with the (uniform) pixel step in the scalar
    // offset, so a store costs a compare against the lane's remaining rows / columns instead of a
    // 64-bit address computation; a pixel outside the image gets an offset past the buffer (outputs are
    // below 2 GiB here, so 2^31 plus any pixel step is past the end without wrapping) and is dropped by
    // the hardware.
    {
      const int tx = tile % tiles_x;
      const int t2 = tile / tiles_x;
      const int ty = t2 % tiles_y;
      const int img = t2 / tiles_y;
      const int ow0 = tx * TW + 4 * lhalf;
      const int cols_left = ch_ok ? p.ow - ow0 : 0;                  // dcol is stored iff dcol < cols_left
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int oh0 = ty * TH + wpix * 2 * NB + i * 2;
        const int rows_left = p.oh - oh0;                            // uniform
        const unsigned base = (unsigned)(((img * p.oh + oh0) * p.ow + ow0) * p.k + ch) * 4u;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int drow = e >> 3, dcol = (e & 3) + 8 * ((e >> 2) & 1);
          float v = acc[i][e] + bv;
          if (p.act == 1) v = fmaxf(v, 0.f);
          const bool ok = dcol < cols_left && drow < rows_left;
          const unsigned soff = (unsigned)((drow * p.ow + dcol) * p.k) * 4u;   // uniform
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), rsrc_y, ok ? base : 0x80000000u, soff, 0);
        }
      }
    }
    if (!has_next) break;
    __syncthreads();
    buf ^= 1;
    tile = next;
  }
}

// ---------------------------------------------------------------------------------------------------
// The same design on the fp16 matrix cores: every operand scaled by a power of two and cut into two fp16
// pieces, three piece products per fp32 product, the cross terms in an accumulator set of their own
// (f16_pieces.h).  v_mfma_f32_32x32x16_f16 wants eight consecutive reduction
// indices per lane, so the reduction is ordered filter row by filter row with each row's S*C run padded to
// a multiple of 8 (7 x 3 = 21 -> 24): a lane's eight values are then eight consecutive patch elements, and
// where the run is over they overlap the neighbouring pixels' data, which the zero pieces of the filter
// cancel (the patch holds finite values or zeros everywhere, including one spare row).  The patch is cut
// once per tile while it is written to LDS (two fp16 planes), scaled by its own largest magnitude (the
// workgroup takes it from the registers the patch was fetched into: one more barrier per tile); the filter
// fragments (11 steps x 2 pieces x 8 values per lane) are cut once per workgroup, scaled by the largest
// magnitude of the workgroup's 64 filters, and stay in registers.  11 x 3 fp16 MFMAs of 32 cycles
// replace 74 fp32 MFMAs of 64 per 32 x 32 block (the first form of this kernel took 11 x 6 bf16 MFMAs over
// three bf16 pieces per operand: batch 32 62 -> 52 us).
// ---------------------------------------------------------------------------------------------------
template <int R, int S, int C, int STRIDE, int TH>
struct SmallCB {
  static constexpr int K = R * S * C;
  static constexpr int RUN = S * C;                      // contiguous (s, c) run per filter row
  static constexpr int RUN8 = (RUN + 7) / 8;             // groups of 8 per filter row
  static constexpr int GROUPS = R * RUN8;                // groups of 8 reduction indices (padded)
  static constexpr int STEPS = (GROUPS + 1) / 2;         // MFMA steps (two groups each)
  static constexpr int PH = (TH - 1) * STRIDE + R;       // patch rows
  static constexpr int PWC = ((TW - 1) * STRIDE + S) * C;   // patch row length in elements
  static constexpr int PITCH = ((PWC + 8 + 15) / 16) * 16;  // elements; the last pixel's padded run stays inside the row
  static constexpr int PLANE = (PH + 2) * PITCH;         // elements; two spare rows: the padded steps read them
  static constexpr int PATCH = 2 * PLANE;                // elements of one buffer
  static constexpr int LOADS = (PH * PWC + SC_THREADS - 1) / SC_THREADS;
  static constexpr int stage_bytes = (2 * PATCH * 2 > 32 * K * 4 ? 2 * PATCH * 2 : 32 * K * 4);
  static constexpr int lds_bytes = stage_bytes + 32;     // + the eight wavefronts' largest magnitudes
  // patch offset (elements) of group g relative to a pixel's patch origin
  static constexpr int off(int g) { return (g / RUN8) * PITCH + (g % RUN8) * 8; }
};

template <int R, int S, int C, int STRIDE, int TH>
__global__ __launch_bounds__(SC_THREADS, 2) void conv_smallc_f32_f16_kernel(const Problem p, int tiles_y, int tiles_x,
                                                                            int total_tiles) {
  using G = SmallCB<R, S, C, STRIDE, TH>;
  static_assert(TH == 4, "tile height: one 32-pixel block per wavefront");
  static_assert((STRIDE * C) % 2 == 0 && G::PITCH % 2 == 0, "a pixel's run starts on a 4-byte boundary");
  constexpr int NB = TH / 4;
  extern __shared__ __align__(16) unsigned short patchb[];   // [2][2][PH + 2][PITCH]; first the filter halves as fp32
  float* wstage = reinterpret_cast<float*>(patchb);
  unsigned* maxw = reinterpret_cast<unsigned*>(reinterpret_cast<unsigned char*>(patchb) + G::stage_bytes);
  static_assert(SC_THREADS == 256, "four wavefronts leave their largest magnitudes in words 0-3; words 4-7 stay zero");

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lrow = lane & 31, lhalf = lane >> 5;
  const int wpix = wave >> 1;
  const int wch = wave & 1;
  const int n_tile = blockIdx.y;

  const float* __restrict__ X = static_cast<const float*>(p.x);
  const float* __restrict__ Wt = static_cast<const float*>(p.w);
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_y = __builtin_amdgcn_make_buffer_rsrc(
      p.y, 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);

  const int ch = n_tile * 64 + wch * 32 + lrow;
  const bool ch_ok = ch < p.k;
  const float bv = (ch_ok && bias) ? bias[ch] : 0.f;

  // ---- per-lane patch bases (elements).  Step t multiplies groups 2t (lanes 0..31) and 2t + 1 (lanes 32..63);
  // off(2t + 1) - off(2t) is 8 except where 2t is the last group of a filter row; a second base covers those
  // steps, so every read uses a compile-time offset.
  const int pix_origin = ((wpix * 2 * NB + (lrow >> 4)) * STRIDE) * G::PITCH + (lrow & 15) * STRIDE * C;
  const int base_norm = pix_origin + lhalf * 8;
  const int base_cross = pix_origin + lhalf * (G::PITCH - (G::RUN8 - 1) * 8);

  float stage[G::LOADS];
  auto load_patch = [&](int tile) {
    const int tx = tile % tiles_x;
    const int t2 = tile / tiles_x;
    const int ty = t2 % tiles_y;
    const int img = t2 / tiles_y;
    const int ih0 = ty * TH * STRIDE - p.pad_t;
    const int fx0 = (tx * TW * STRIDE - p.pad_l) * C;
    const int row_floats = p.w_ * C;
#pragma unroll
    for (int i = 0; i < G::LOADS; ++i) {
      const int idx = tid + i * SC_THREADS;
      const int pr = idx / G::PWC, pc = idx % G::PWC;
      const int ih = ih0 + pr, fx = fx0 + pc;
      const bool ok = idx < G::PH * G::PWC && (unsigned)ih < (unsigned)p.h && (unsigned)fx < (unsigned)row_floats;
      stage[i] = ok ? X[((size_t)img * p.h + ih) * row_floats + fx] : 0.f;
    }
  };
  auto store_patch = [&](int buf, int se) {
    unsigned short* dst = patchb + buf * G::PATCH;
#pragma unroll
    for (int i = 0; i < G::LOADS; ++i) {
      const int idx = tid + i * SC_THREADS;
      if (idx < G::PH * G::PWC) {
        const Cut2 pc = cut2(stage[i], se);
        unsigned short* d = dst + (idx / G::PWC) * G::PITCH + idx % G::PWC;
        d[0] = __builtin_bit_cast(unsigned short, pc.h1);
        d[G::PLANE] = __builtin_bit_cast(unsigned short, pc.h2);
      }
    }
  };
  // Largest magnitude (bits) of the patch held in `stage`, over the wavefront; the workgroup's follows from the
  // eight words the wavefronts leave in maxw.
  auto stage_max = [&]() {
    unsigned m = 0;
#pragma unroll
    for (int i = 0; i < G::LOADS; ++i) {
      const unsigned b = __builtin_bit_cast(unsigned, stage[i]) & 0x7fffffffu;
      m = b > m ? b : m;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const unsigned o = (unsigned)__shfl_xor((int)m, d, 64);
      m = o > m ? o : m;
    }
    return m;
  };

  int tile = blockIdx.x;
  if (tile >= total_tiles) return;
  if (tid >= 4 && tid < 8) maxw[tid] = 0u;  // never written again; visible after the first barrier
  load_patch(tile);                        // in flight while the filter is fetched

  // ---- filter fragments: lane (channel, half) keeps, for every step t and piece, the eight values of group
  // 2t + half.  The 32 channels of each channel half are copied into LDS with coalesced loads (in the space of
  // the patch buffers) and the lanes pick from there; rows past the last output channel lie past the end of
  // the tensor and the range-checked loads return zeros.  Both halves are fetched first: their largest magnitude
  // is the scale the fragments are cut at.
  v8h wfrag[G::STEPS][2];
  int se_w;
  bool finite;
  {
    const __amdgpu_buffer_rsrc_t rsrc_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Wt), 0, (int)p.w_bytes, 0x00020000);
    constexpr int HALF_FLOATS = 32 * G::K;
    constexpr int W_LOADS = (HALF_FLOATS + SC_THREADS - 1) / SC_THREADS;
    float wst[2][W_LOADS];
    unsigned wm = 0;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const unsigned base = (unsigned)((n_tile * 64 + half * 32) * G::K) * 4u;
#pragma unroll
      for (int i = 0; i < W_LOADS; ++i) {
        const int e = tid + i * SC_THREADS;
        wst[half][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                     rsrc_w, e < HALF_FLOATS ? base + 4u * e : 0xFFFFFFFCu, 0, 0));
      }
    }
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int i = 0; i < W_LOADS; ++i) {
        const unsigned b = __builtin_bit_cast(unsigned, wst[half][i]) & 0x7fffffffu;
        wm = b > wm ? b : wm;
      }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const unsigned o = (unsigned)__shfl_xor((int)wm, d, 64);
      wm = o > wm ? o : wm;
    }
    if (lane == 0) maxw[wave] = wm;
    __syncthreads();
    const unsigned w_max_bits = max_of_eight(maxw);
    se_w = scale_exponent(w_max_bits);
    finite = w_max_bits < 0x7f800000u;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
      for (int i = 0; i < W_LOADS; ++i) {
        const int e = tid + i * SC_THREADS;
        if (e < HALF_FLOATS) wstage[e] = wst[half][i];
      }
      __syncthreads();
      if (wch == half) {
#pragma unroll
        for (int t = 0; t < G::STEPS; ++t) {
          float v[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            // group 2t + lhalf: filter row gr, positions 8 * part + e of its run
            const int g0 = 2 * t, g1 = 2 * t + 1;
            const int r0 = g0 / G::RUN8, q0 = (g0 % G::RUN8) * 8 + e;
            const int r1 = g1 / G::RUN8, q1 = (g1 % G::RUN8) * 8 + e;
            const bool ok0 = r0 < R && q0 < G::RUN, ok1 = r1 < R && q1 < G::RUN;    // compile-time
            const float v0 = ok0 ? wstage[lrow * G::K + r0 * G::RUN + q0] : 0.f;
            const float v1 = ok1 ? wstage[lrow * G::K + r1 * G::RUN + q1] : 0.f;
            v[e] = lhalf ? v1 : v0;
          }
          v4u p1, p2;
          cut8(v, se_w, p1, p2);
          wfrag[t][0] = __builtin_bit_cast(v8h, p1);
          wfrag[t][1] = __builtin_bit_cast(v8h, p2);
        }
      }
      __syncthreads();
    }
  }
  // zero both buffers once: the spare rows and the row tails are never overwritten by patch stores and must
  // hold finite values (they meet zero filter pieces)
  for (int i = tid; i < 2 * G::PATCH / 2; i += SC_THREADS) reinterpret_cast<unsigned*>(patchb)[i] = 0u;
  {
    const unsigned share = stage_max();
    if (lane == 0) maxw[wave] = share;                   // (the filter's words were read before the last barrier)
  }
  __syncthreads();
  int se_x;                                              // scale exponent of the patch in `buf`
  {
    const unsigned m = max_of_eight(maxw);
    finite = finite && m < 0x7f800000u;
    se_x = scale_exponent(m);
  }
  store_patch(0, se_x);
  __syncthreads();
  int buf = 0;
  for (;;) {
    const int next = tile + gridDim.x;
    const bool has_next = next < total_tiles;
    if (has_next) load_patch(next);

    v16f acc[NB], acc_lo[NB];                            // the h1 h1' products; the cross terms (weight 2^-11)
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        acc[i][e] = 0.f;
        acc_lo[i][e] = 0.f;
      }
    const unsigned short* src = patchb + buf * G::PATCH;
    const unsigned short* pn = src + base_norm;
    const unsigned short* pcx = src + base_cross;
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t) {
      constexpr int blk = 2 * STRIDE * G::PITCH;                     // second 32-pixel block: two output rows down
      const bool cross = (2 * t) % G::RUN8 == G::RUN8 - 1;           // compile-time after unrolling
      const unsigned short* b = (cross ? pcx : pn) + G::off(2 * t);
      v8h a[2][NB];
#pragma unroll
      for (int pc = 0; pc < 2; ++pc)
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          const unsigned* q = reinterpret_cast<const unsigned*>(b + pc * G::PLANE + i * blk);   // 4-byte aligned
          a[pc][i] = __builtin_bit_cast(v8h, v4u{q[0], q[1], q[2], q[3]});
        }
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        acc_lo[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], wfrag[t][1], acc_lo[i], 0, 0, 0);
        acc_lo[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[1][i], wfrag[t][0], acc_lo[i], 0, 0, 0);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], wfrag[t][0], acc[i], 0, 0, 0);
      }
    }

    // ---- the next tile's patch: its largest magnitude, then (everyone is done with the other buffer since the
    // barrier that ended the last tile) scaled, cut and written while this tile's results are stored
    const ScaleBack sb = scale_back_of(se_x, se_w, finite);
    if (has_next) {
      const unsigned share = stage_max();
      if (lane == 0) maxw[wave] = share;
      __syncthreads();
      const unsigned m = max_of_eight(maxw);
      finite = finite && m < 0x7f800000u;
      se_x = scale_exponent(m);
      store_patch(buf ^ 1, se_x);
    }

    // ---- epilogue of this tile: as in the kernel above
    {
      const int tx = tile % tiles_x;
      const int t2 = tile / tiles_x;
      const int ty = t2 % tiles_y;
      const int img = t2 / tiles_y;
      const int ow0 = tx * TW + 4 * lhalf;
      const int cols_left = ch_ok ? p.ow - ow0 : 0;
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int oh0 = ty * TH + wpix * 2 * NB + i * 2;
        const int rows_left = p.oh - oh0;
        const unsigned base = (unsigned)(((img * p.oh + oh0) * p.ow + ow0) * p.k + ch) * 4u;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int drow = e >> 3, dcol = (e & 3) + 8 * ((e >> 2) & 1);
          float v = join_sets(acc[i][e], acc_lo[i][e], sb) + bv;
          if (p.act == 1) v = fmaxf(v, 0.f);
          const bool ok = dcol < cols_left && drow < rows_left;
          const unsigned soff = (unsigned)((drow * p.ow + dcol) * p.k) * 4u;
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), rsrc_y, ok ? base : 0x80000000u, soff, 0);
        }
      }
    }
    if (!has_next) break;
    __syncthreads();
    buf ^= 1;
    tile = next;
  }
}

template <int R, int S, int C, int STRIDE, int TH, bool BF16>
hipError_t launch_smallc(const Problem& p, hipStream_t stream) {
  using G = std::conditional_t<BF16, SmallCB<R, S, C, STRIDE, TH>, SmallC<R, S, C, STRIDE, TH>>;
  auto kern = [] {
    if constexpr (BF16) return conv_smallc_f32_f16_kernel<R, S, C, STRIDE, TH>;
    else return conv_smallc_f32_kernel<R, S, C, STRIDE, TH>;
  }();
  // once per instantiation; initialisation of a function-local static is thread-safe
  struct Setup { hipError_t status; int wg_per_cu; };
  static const Setup setup = [&]() {
    Setup s{hipSuccess, 1};
    s.status = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   G::lds_bytes);
    int occ = 0;
    if (s.status == hipSuccess)
      s.status = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, reinterpret_cast<const void*>(kern), SC_THREADS,
                                                              G::lds_bytes);
    s.wg_per_cu = occ < 1 ? 1 : occ;
    return s;
  }();
  if (setup.status != hipSuccess) return setup.status;
  const int wg_per_cu = setup.wg_per_cu;
  const int num_cu = num_compute_units();
  if (num_cu < 1) return hipErrorInvalidDevice;
  const int tiles_y = (p.oh + TH - 1) / TH, tiles_x = (p.ow + TW - 1) / TW;
  const long long total = (long long)p.n * tiles_y * tiles_x;
  const int n_tiles = (p.k + 63) / 64;
  long long gx = (long long)num_cu * wg_per_cu / n_tiles;
  if (gx < 1) gx = 1;
  if (gx > total) gx = total;
  dim3 grid((unsigned)gx, n_tiles, 1), block(SC_THREADS, 1, 1);
  hipLaunchKernelGGL(kern, grid, block, G::lds_bytes, stream, p, tiles_y, tiles_x, (int)total);
  return hipGetLastError();
}

}  // namespace

bool smallc_f32_applicable(const Problem& p) {
  return !p.b_is_kn && p.groups == 1 && p.r == 7 && p.s == 7 && p.c == 3 && p.stride_h == 2 && p.stride_w == 2 &&
         (long long)p.M * p.k * 4 < (1LL << 31) && p.w_bytes <= 0x7FFFFFFFu &&
         (long long)p.n * ((p.oh + 3) / 4) * ((p.ow + TW - 1) / TW) < (1LL << 31);
}

hipError_t launch_smallc_f32(const Problem& p, hipStream_t stream, const char** variant) {
  // The fp16-piece form pays a longer prologue (the filter fragments are cut per workgroup): batch 32 90 -> 52 us,
  // batch 8 27 -> 22 us, but batch 1 (196 tiles, launch-bound) 8.2 -> 11.7 us, which therefore keeps the fp32 form.
  // The knob forces one.
  const long long tiles4 = (long long)p.n * ((p.oh + 3) / 4) * ((p.ow + TW - 1) / TW);
  const bool bf16 = knob_or(KNOB_F32_SMALLC_BF16, tiles4 >= 1536 ? 1 : 0) != 0;
  *variant = bf16 ? "conv_smallc_f32_7x7s2c3_f16x3" : "conv_smallc_f32_7x7s2c3";
  // the taller tile is the faster one per tile (two independent MFMA chains per wavefront); the
  // shorter one doubles the number of tiles, which pays while there are fewer than about two per
  // resident workgroup (batch 1: 13.8 -> 11.1 us; batch 32: 97.8 vs 100.5 us)
  const long long tiles8 = (long long)p.n * ((p.oh + 7) / 8) * ((p.ow + TW - 1) / TW);
  int th = tiles8 < 1536 ? 4 : 8;
  if (knob_is_set(KNOB_SMALLC_TH)) th = knob(KNOB_SMALLC_TH) == 8 ? 8 : 4;   // experiments
  // (the fp16-piece form keeps 88 registers of filter fragments per lane and two accumulator sets: with two pixel
  // blocks per wavefront it would spill, so it always takes the four-row tile)
  if (bf16) return launch_smallc<7, 7, 3, 2, 4, true>(p, stream);
  return th == 8 ? launch_smallc<7, 7, 3, 2, 8, false>(p, stream) : launch_smallc<7, 7, 3, 2, 4, false>(p, stream);
}

}  // namespace glowmi
