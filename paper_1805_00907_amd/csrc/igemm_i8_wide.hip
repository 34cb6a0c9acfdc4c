// int8 implicit-GEMM Convolution / FullyConnected for large contractions on gfx950 (MI355X): the
// quantized form of Section 4 of the paper (int8 codes with per-tensor scale/offset, int32
// accumulation, the rescale folded into the producer, Relu as an integer lower bound) for layers
// whose cost is the contraction itself rather than moving bytes.
//
// For v_mfma_i32_32x32x32_i8 a wavefront gets about seven vector-ALU issue slots per MFMA and must
// reuse every operand fragment it reads from LDS at least twice, so the kernel spends as little as
// possible per reduction slab besides the MFMAs:
//   - one workgroup = 128 pixels x BN channels, eight wavefronts: 2 x 2 wavefronts tile the output
//     (64 x BN/2 each, 2 x BN/64 MFMA tiles) and two such sets split every 128-code slab between them
//     (codes 0..63 and 64..127); the two partial tiles are exchanged through LDS at the end and each
//     wavefront finishes half of them;
//   - both operands go from global memory straight into LDS (buffer loads with the LDS bit, 16 bytes
//     per lane, no staging registers, no LDS store instructions) into a ring of NBUF slab buffers,
//     NBUF-1 slabs in flight; out-of-range lanes (rows past the tensor, reduction tail, taps on
//     padding) make the hardware write zeros, and a padding chunk is then overwritten with the code
//     of real zero by the lane that issued it;
//   - a lane's LDS destination is fixed (base + 16 * lane), its global source is not: lane l of a
//     load fetches chunk (l % 8) ^ (l / 8) of row l / 8, which XOR-swizzles the 16-byte chunks of the
//     128-byte rows so that fragment reads are spread over the banks;
//   - the FullyConnected weight ([K][N], N contiguous) is staged as it lies in memory and the MFMA
//     fragments (16 consecutive reduction codes per lane) are read with the transposing LDS load
//     (ds_read_b64_tr_b8: within 16 lanes, result byte e of lane i comes from byte i % 8 of the 8
//     bytes addressed by lane 2e + i / 8);
//   - whether a filter tap falls on padding is one bit test against a per-pixel mask computed once;
//   - the code sums needed to remove the offsets are taken with dot-product instructions from the
//     fragments the wavefronts read anyway.
// Offsets are removed after the contraction exactly as in the generic kernel:
//   sum (x - xo)(w - wo) = sum x*w - xo * sum_k w - wo * sum_k x + Kcount * xo * wo,
// padded taps staged as the code xo.  Everything after the accumulator is integer arithmetic.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#include "igemm.h"
#include "lds_direct.h"
#include "quant_epilogue.h"

namespace glowmi {
namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WBM = 128;                 // pixels per workgroup tile
constexpr int WBK = 128;                 // codes per reduction slab
constexpr int WTHREADS = 512;

__device__ __forceinline__ int sum4(int packed, int acc) {   // acc + the four signed bytes
  return __builtin_amdgcn_sdot4(packed, 0x01010101, acc, false);
}

__device__ __forceinline__ int requantize(int acc, int mant, int shift, int y_off, int lo) {
  return shift >= 33 ? requantize_as<true>(acc, mant, shift, y_off, lo)
                     : requantize_as<false>(acc, mant, shift, y_off, lo);   // uniform branch
}

// PADDED: some filter tap of some pixel may fall on padding (otherwise the per-tap tests are dropped).
// XSUM: the filter offset is not zero, so the input code sums per pixel are needed as well.
// NBUF: slab buffers in the LDS ring (2: two workgroups per CU, 4: one workgroup with three slabs in flight).
template <int BN, bool B_KN, bool PADDED, bool XSUM, int NBUF>
// (second launch bound = wavefronts per SIMD: two workgroups of eight per CU need four, i.e. at most 128
// registers -- with a bound of two the padded 128-channel form took 130 and ran one workgroup per CU;
// the forms that also take input code sums do not fit 128 without spilling and stay at one per CU)
__global__ __launch_bounds__(WTHREADS, (NBUF <= 2 && !XSUM) ? 4 : 2) void igemm_i8_wide_kernel(const Problem p, int tiles_m,
                                                                                   int tiles_n, int band_n,
                                                                                   int total_work) {
  static_assert(BN == 64 || BN == 128, "channel tile");
  static_assert(!B_KN || BN == 128, "the [K][N] weight path stages 128 columns");
  constexpr int TN = BN / 64;                           // MFMA tiles along the channels per wavefront
  constexpr int BT = BN / 64;                           // filter loads per wavefront and slab ([k][r][s][c] layout)
  constexpr int LPI = 2 + (B_KN ? 2 : BT);              // loads one wavefront issues per slab
  constexpr int A_BYTES = WBM * WBK, B_BYTES = BN * WBK, BUF = A_BYTES + B_BYTES;
  constexpr int OUT_PITCH = BN + 16;
  static_assert(NBUF * BUF >= WBM * OUT_PITCH, "output staging fits the slab buffers");
  static_assert(NBUF * BUF >= 8 * TN * 16 * 64 * 4, "exchange of the partial tiles fits the slab buffers");

  extern __shared__ __align__(16) unsigned char lds[];
  int* xsum = reinterpret_cast<int*>(lds + NBUF * BUF); // [128] input code sums per pixel row
  int* wsum = xsum + WBM;                               // [BN]  filter code sums per channel
  int* cterm = wsum + BN;                               // [BN]  per-channel additive term

  // ---- which tile: consecutive workgroup ids go round-robin to the 8 XCDs, so id % 8 picks the XCD
  // and each XCD gets a contiguous run of tiles; within a (group, split) plane the tiles are walked
  // in bands of band_n tile columns so that the run of one XCD covers a compact block of the output
  // (its L2 then holds few distinct input rows and filter columns).
  const int per_xcd = gridDim.x >> 3;
  const int wk = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (wk >= total_work) return;
  const int plane = tiles_m * tiles_n;
  const int pl = wk / plane, wi = wk - pl * plane;
  const int g = pl % p.groups;
  const int split = pl / p.groups;
  const int band = wi / (tiles_m * band_n);
  const int in_band = wi - band * tiles_m * band_n;
  const int band_w = tiles_n - band * band_n < band_n ? tiles_n - band * band_n : band_n;
  const int tm = in_band / band_w;
  const int tn = band * band_n + (in_band - tm * band_w);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kgrp = wave >> 2;                           // which half of every slab this wavefront multiplies
  const int wm = (wave >> 1) & 1, wn = wave & 1;
  const int lrow = lane & 31, lhalf = lane >> 5;

  const v4i rsrc_x = make_rsrc(p.x, p.x_bytes);
  const v4i rsrc_w = make_rsrc(p.w, p.w_bytes);
  constexpr unsigned OOB = 0x80000000u;                 // beyond any tensor this kernel accepts: loads give 0

  for (int i = tid; i < WBM + BN; i += WTHREADS) xsum[i] = 0;   // xsum and wsum (visible after the first barrier)

  const int slab_begin = split * p.slabs_per_split;
  const int total_slabs = (p.Kgemm + WBK - 1) / WBK;
  int slab_end = slab_begin + p.slabs_per_split;
  if (slab_end > total_slabs) slab_end = total_slabs;
  int k_hi = slab_end * WBK;
  if (k_hi > p.Kgemm) k_hi = p.Kgemm;
  const int k_count = k_hi - slab_begin * WBK;          // codes this split really reduces over

  // ---- staging state.  Load t (0, 1) of wavefront w covers tile rows 8w + 64t .. + 7, lane l the row
  // 8w + 64t + l/8 and, of that row's eight 16-byte chunks, chunk cch = (l%8) ^ swz(row) with swz(row) =
  // (row % 8) ^ ((row / 8) % 4) = (l/8) ^ (w % 4); it lands at
  // chunk position l%8 of the row.
  const int srow = 8 * wave + (lane >> 3);              // tile row of load 0 (load 1: + 64)
  const int cch = (lane & 7) ^ (lane >> 3) ^ (wave & 3);
  unsigned a_base[2];                                   // byte offset of the pixel's window origin, OOB past M
  unsigned a_mask[2];                                   // bits 0..15: filter rows inside, 16..31: filter columns inside
  unsigned b_off[2];                                    // filter rows ([k][r][s][c]) or the lane's column offset ([K][N])
  int tap_r, tap_s, tap_c;                              // filter tap and channel of this lane's chunk in the next slab to issue
  const int xo_fill = (p.x_off & 0xff) * 0x01010101;    // padding = the code of real zero
  {
    const int ohow = p.oh * p.ow;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int m = tm * WBM + srow + 64 * t;
      a_base[t] = OOB;
      a_mask[t] = 0;
      if (m < p.M) {
        const int img = p.div_ohow.div(m);
        const int rem = m - img * ohow;
        const int oh = p.div_ow.div(rem);
        const int ow = rem - oh * p.ow;
        const int ih0 = oh * p.stride_h - p.pad_t, iw0 = ow * p.stride_w - p.pad_l;
        a_base[t] = (unsigned)(((img * p.h + ih0) * p.w_ + iw0) * p.c + g * p.cg);   // may wrap below 0: only used with an inside tap
        const int rlo = ih0 < 0 ? -ih0 : 0, rhi = p.h - ih0 < p.r ? p.h - ih0 : p.r;
        const int slo = iw0 < 0 ? -iw0 : 0, shi = p.w_ - iw0 < p.s ? p.w_ - iw0 : p.s;
        const unsigned rm = rhi > rlo ? (1u << rhi) - (1u << rlo) : 0u;
        const unsigned sm = shi > slo ? (1u << shi) - (1u << slo) : 0u;
        a_mask[t] = rm | (sm << 16);
      }
    }
    const int kg0 = slab_begin * WBK + cch * 16;
    const int tp = p.div_cg.div(kg0);
    tap_c = kg0 - tp * p.cg;
    tap_r = p.div_s.div(tp);
    tap_s = tp - tap_r * p.s;
    if (!B_KN) {
#pragma unroll
      for (int t = 0; t < BT; ++t) {
        const int n = tn * BN + srow + 64 * t;
        b_off[t] = n < p.kg ? (unsigned)((g * p.kg + n) * p.Kgemm + cch * 16) : OOB;
      }
    } else {
      const int col = tn * BN + cch * 16;               // k % 16 == 0 on this path: a chunk is whole or absent
      b_off[0] = col < p.k ? (unsigned)col : OOB;
    }
  }
  unsigned padq = 0;                                    // 2 bits per slab in flight: which of the lane's input chunks are padding

  // Issue the loads of slab `slab` into ring buffer `buf`; `slot` = how many slabs are already in flight.
  auto issue = [&](int slab, int buf, int slot) {
    const unsigned As = __builtin_amdgcn_readfirstlane(lds_offset_of(lds) + buf * BUF + (8 * wave) * WBK);
    const unsigned Bs = As + A_BYTES;
    {
      const unsigned tap_off = (unsigned)((tap_r * p.w_ + tap_s) * p.c + tap_c);
      if constexpr (PADDED || XSUM) {
        const bool kok = slab * WBK + cch * 16 < p.Kgemm;   // reduction tail: zeros
        unsigned bits = 0;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const bool inside = (a_mask[t] >> tap_r) & (a_mask[t] >> (16 + tap_s)) & 1u;
          load16_to_lds(rsrc_x, As + t * 64 * WBK, (inside && kok) ? a_base[t] + tap_off : OOB);
          if (!inside && kok && a_base[t] != OOB) bits |= 1u << t;
        }
        padq |= bits << (2 * slot);
      } else {
        // no tap can fall on padding and no code sums are taken: in the reduction tail the filter
        // side is zero, so whatever an in-range address holds there does not matter
#pragma unroll
        for (int t = 0; t < 2; ++t)
          load16_to_lds(rsrc_x, As + t * 64 * WBK, a_base[t] + tap_off);
      }
      tap_c += WBK;                                     // this lane's chunk one slab further
      while (tap_c >= p.cg) {
        tap_c -= p.cg;
        if (++tap_s == p.s) { tap_s = 0; ++tap_r; }
      }
    }
    if constexpr (!B_KN) {
      const bool kok = slab * WBK + cch * 16 < p.Kgemm;
      const unsigned koff = (unsigned)(slab * WBK);
#pragma unroll
      for (int t = 0; t < BT; ++t)
        load16_to_lds(rsrc_w, Bs + t * 64 * WBK, kok ? b_off[t] + koff : OOB);
    } else {
      // weight rows slab*128 + 8w + 64t + l/8 as they lie in memory; rows at or beyond Kgemm lie past
      // the end of the tensor: zeros
      const unsigned base = b_off[0] + (unsigned)(slab * WBK + srow) * (unsigned)p.k;
#pragma unroll
      for (int t = 0; t < 2; ++t)
        load16_to_lds(rsrc_w, Bs + t * 64 * WBK, base + (unsigned)(64 * t) * (unsigned)p.k);
    }
  };

  // After the loads of the oldest slab in flight have landed: chunks that are padding get the code of
  // real zero (the hardware wrote zeros there), by the lane that issued them.
  auto fix_padding = [&](int buf) {
    if constexpr (PADDED || XSUM) {
      if (padq & 3u) {
        unsigned char* As = lds + buf * BUF + (8 * wave) * WBK + lane * 16;
        const v4i fill = v4i{xo_fill, xo_fill, xo_fill, xo_fill};
        if (padq & 1u) *reinterpret_cast<v4i*>(As) = fill;
        if (padq & 2u) *reinterpret_cast<v4i*>(As + 64 * WBK) = fill;
      }
      padq >>= 2;
    }
  };

  // acc[i][j]: 32 output channels (rows of the MFMA result) x 32 pixels (columns)
  v16i acc[2][TN];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;
  int wacc = 0, xacc = 0;                               // this lane's share of a filter-row / pixel-row code sum

  // Fragment addresses inside a slab buffer.  K-contiguous rows: lane (lrow, lhalf) reads chunk
  // 2*k32 + lhalf of its row, stored at position chunk ^ swz(row).  [K][N] weight: lane i of a
  // 16-lane block addresses 8 bytes of reduction row 32*k32 + 16*lhalf + 8u + i/2 (u = 0, 1) at
  // columns (block's 16 columns) + 8*(i%2); that row's chunks are stored at position chunk ^ swz(row).
  int frag_a[2], frag_b[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const int k32 = kgrp * 2 + kk;
    const int c = (k32 * 2 + lhalf) ^ (lrow & 7) ^ ((lrow >> 3) & 3);
    frag_a[kk] = (wm * 64 + lrow) * WBK + (c << 4);
    if (!B_KN) {
      frag_b[kk] = A_BYTES + (wn * (BN / 2) + lrow) * WBK + (c << 4);
    } else {
      const int i16 = lane & 15, blk = (lane >> 4) & 1;
      const int krow = k32 * 32 + lhalf * 16 + (i16 >> 1);           // + 8u
      const int nchunk = wn * 4 + blk;                                // + 2j
      frag_b[kk] = A_BYTES + krow * WBK + ((nchunk ^ (i16 >> 1)) << 4) + 8 * (i16 & 1);
    }
  }

  auto compute = [&](int buf) {
    const unsigned char* base = lds + buf * BUF;
    v4i a[2][2], b[2][TN];                              // all fragment reads first: the MFMAs start as they arrive
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
      for (int i = 0; i < 2; ++i) a[kk][i] = *reinterpret_cast<const v4i*>(base + frag_a[kk] + i * 32 * WBK);
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if constexpr (!B_KN) {
          b[kk][j] = *reinterpret_cast<const v4i*>(base + frag_b[kk] + j * 32 * WBK);
        } else {
          // chunk index + 2j: XOR with a value below 8 commutes with adding 2j only when done on the
          // chunk number, so the position is recomputed from the parts
          const int i16 = lane & 15;
          const int chunk = (wn * 4 + ((lane >> 4) & 1) + 2 * j) ^ (i16 >> 1);   // ^ (row / 8) % 4 per read
          const int rowpart = frag_b[kk] & ~0x70;                     // row base + 8*(i%2), chunk bits cleared
          const unsigned char* q = base + rowpart;
          const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
              (v2i __attribute__((address_space(3)))*)(q + ((chunk ^ (lhalf * 2)) << 4)));
          const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
              (v2i __attribute__((address_space(3)))*)(q + 8 * WBK + ((chunk ^ (lhalf * 2 + 1)) << 4)));
          b[kk][j] = v4i{lo[0], lo[1], hi[0], hi[1]};
        }
      }
    }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)   // filter fragment as the row operand: result rows = channels
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[kk][j], a[kk][i], acc[i][j], 0, 0, 0);
    // code sums from the fragments: of the two wavefronts that read the same filter fragments
    // (wm = 0, 1) each sums half of them, likewise for the input fragments (wn = 0, 1)
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      if (TN == 2) {
        const v4i v = wm ? b[kk][TN - 1] : b[kk][0];
        wacc = sum4(v[0], sum4(v[1], sum4(v[2], sum4(v[3], wacc))));
      } else if (kk == 0) {
        const v4i v = wm ? b[1][0] : b[0][0];
        wacc = sum4(v[0], sum4(v[1], sum4(v[2], sum4(v[3], wacc))));
      }
      if constexpr (XSUM) {
        const v4i v = wn ? a[kk][1] : a[kk][0];
        xacc = sum4(v[0], sum4(v[1], sum4(v[2], sum4(v[3], xacc))));
      }
    }
  };

  // ---- main loop.  Iteration s: wait for slab s (the younger slabs stay in flight), patch padding,
  // barrier, refill the buffer that was multiplied last iteration with slab s + NBUF - 1, multiply
  // slab s.  Unrolled NBUF times so that buffer indices are compile-time constants; the steady-state
  // trips issue and wait unconditionally.
  {
#pragma unroll
    for (int d = 0; d < NBUF - 1; ++d)
      if (slab_begin + d < slab_end) issue(slab_begin + d, d, d);
    int s0 = slab_begin;
    for (; s0 + 2 * NBUF - 1 <= slab_end; s0 += NBUF) {
#pragma unroll
      for (int u = 0; u < NBUF; ++u) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NBUF - 2) * LPI));
        fix_padding(u);
        __syncthreads();
        issue(s0 + u + NBUF - 1, (u + NBUF - 1) % NBUF, NBUF - 2);
        compute(u);
      }
    }
    for (; s0 < slab_end; s0 += NBUF) {
#pragma unroll
      for (int u = 0; u < NBUF; ++u) {
        const int s = s0 + u;
        if (s < slab_end) {
          __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
          fix_padding(u);
          __syncthreads();
          if (s + NBUF - 1 < slab_end) issue(s + NBUF - 1, (u + NBUF - 1) % NBUF, NBUF - 2);
          compute(u);
        }
      }
    }
    __syncthreads();                                    // every wavefront is done with the slab buffers
  }

  // ---- code sums (LDS atomics; integer, so order is free)
  if (TN == 2) atomicAdd(&wsum[wn * (BN / 2) + wm * 32 + lrow], wacc);
  else atomicAdd(&wsum[wn * (BN / 2) + lrow], wacc);
  if constexpr (XSUM) atomicAdd(&xsum[wm * 64 + wn * 32 + lrow], xacc);

  // ---- exchange: the two wavefronts that hold partial sums of the same 64 x BN/2 sub-tile swap
  // halves; the kgrp-0 wavefront finishes pixel rows 0..31 of the sub-tile, the other rows 32..63.
  v16i keep[TN];
  {
    v4i* xch = reinterpret_cast<v4i*>(lds);
    const int mine = ((wave & 3) * 2 + kgrp) * TN * 4, theirs = ((wave & 3) * 2 + (kgrp ^ 1)) * TN * 4;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        v4i send;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int e = e4 * 4 + t;
          send[t] = kgrp ? acc[0][j][e] : acc[1][j][e];
          keep[j][e] = kgrp ? acc[1][j][e] : acc[0][j][e];
        }
        xch[(mine + j * 4 + e4) * 64 + lane] = send;
      }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const v4i got = xch[(theirs + j * 4 + e4) * 64 + lane];
#pragma unroll
        for (int t = 0; t < 4; ++t) keep[j][e4 * 4 + t] += got[t];
      }
    }
  }

  // The correction terms are combined modulo 2^32 (unsigned): each may exceed the final value, the
  // true accumulator fits int32 by contract, so the wrapped sum is exact.
  const int* __restrict__ bias = static_cast<const int*>(p.bias);
  for (int i = tid; i < BN; i += WTHREADS) {
    const int col = tn * BN + i;
    unsigned ct = (unsigned)k_count * (unsigned)(p.x_off * p.w_off) - (unsigned)p.x_off * (unsigned)wsum[i];
    if (p.split_k == 1 && bias && col < p.kg) ct += (unsigned)bias[g * p.kg + col];
    cterm[i] = (int)ct;
  }
  __syncthreads();                                      // exchange area read by everyone, cterm complete

  const int lr = wm * 64 + kgrp * 32 + lrow;            // pixel row inside the tile
  const int row = tm * WBM + lr;
  const unsigned rowterm = XSUM ? (unsigned)p.w_off * (unsigned)xsum[lr] : 0u;

  if (p.split_k == 1) {
    unsigned char* out = lds;                           // [128][OUT_PITCH] requantized tile, pixel-major
    const signed char* addend = static_cast<const signed char*>(p.addend);   // may be the output itself
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int lc = wn * (BN / 2) + j * 32 + q4 * 8 + lhalf * 4;   // first of 4 consecutive channels
        const v4i ct = *reinterpret_cast<const v4i*>(cterm + lc);
        int rcodes = 0;
        const int col = tn * BN + lc;
        const bool live = row < p.M && col < p.kg;
        if (addend && live)                                           // uniform test, then per-lane guard
          rcodes = *reinterpret_cast<const int*>(addend + (size_t)row * p.k + g * p.kg + col);
        int q[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          int v = (int)((unsigned)keep[j][q4 * 4 + t] + (unsigned)ct[t] - rowterm);
          if (addend) {
            const int code = live ? (int)(signed char)(rcodes >> (8 * t)) : p.r_off;
            v += rescale_term(code - p.r_off, p.r_mant, p.r_shift);
          }
          q[t] = requantize(v, p.mant, p.shift, p.y_off, p.lo);
        }
        *reinterpret_cast<unsigned*>(out + lr * OUT_PITCH + lc) = pack_codes(q[0], q[1], q[2], q[3]);
      }
    }
    __syncthreads();
    // copy out: 16 bytes of one pixel row per thread and pass
    signed char* __restrict__ Y = static_cast<signed char*>(p.y);
    constexpr int CHUNKS = BN / 16;
    const bool wide = (p.kg % 16 == 0) && (p.k % 16 == 0);
    for (int u = tid; u < WBM * CHUNKS; u += WTHREADS) {
      const int r_ = u / CHUNKS, ch = u % CHUNKS;
      const int orow = tm * WBM + r_, col = tn * BN + ch * 16;
      if (orow >= p.M || col >= p.kg) continue;
      signed char* dst = Y + (size_t)orow * p.k + g * p.kg + col;
      const unsigned char* src = out + r_ * OUT_PITCH + ch * 16;
      if (wide) {
        *reinterpret_cast<v4i*>(dst) = *reinterpret_cast<const v4i*>(src);
      } else {   // kg % 4 == 0 on this kernel: dword steps
        for (int e = 0; e < 16 && col + e < p.kg; e += 4)
          *reinterpret_cast<int*>(dst + e) = *reinterpret_cast<const int*>(src + e);
      }
    }
  } else {
    int* __restrict__ part = static_cast<int*>(p.partial);
    if (row < p.M) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int lc = wn * (BN / 2) + j * 32 + q4 * 8 + lhalf * 4;
          const int col = tn * BN + lc;
          if (col >= p.kg) continue;                                  // kg % 4 == 0: all four or none
          const v4i ct = *reinterpret_cast<const v4i*>(cterm + lc);
          v4i v;
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] = (int)((unsigned)keep[j][q4 * 4 + t] + (unsigned)ct[t] - rowterm);
          *reinterpret_cast<v4i*>(part + ((size_t)split * p.M + row) * p.k + g * p.kg + col) = v;
        }
      }
    }
  }
}

template <int BN, bool B_KN, bool PADDED, bool XSUM, int NBUF>
hipError_t launch_wide_variant(const Problem& p, const Plan& plan, hipStream_t stream) {
  auto kern = igemm_i8_wide_kernel<BN, B_KN, PADDED, XSUM, NBUF>;
  constexpr int lds_bytes = NBUF * (WBM + BN) * WBK + (WBM + 2 * BN) * 4;
  // once per instantiation; initialisation of a function-local static is thread-safe
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  if (attr_status != hipSuccess) return attr_status;
  const long long total_work = (long long)plan.tiles_m * plan.tiles_n * p.groups * plan.split_k;
  const long long grid_x = ((total_work + 7) / 8) * 8;
  // band width: the run of tiles one XCD gets should be roughly square in (pixel tiles, channel tiles)
  const long long per_xcd = grid_x / 8;
  int band_n = 1;
  while ((long long)band_n * band_n * 2 < per_xcd && band_n < plan.tiles_n) ++band_n;
  dim3 grid((unsigned)grid_x, 1, 1), block(WTHREADS, 1, 1);
  hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, p, plan.tiles_m, plan.tiles_n, band_n, (int)total_work);
  return hipGetLastError();
}

template <int BN, bool B_KN, int NBUF>
hipError_t launch_wide_flags(const Problem& p, const Plan& plan, hipStream_t stream) {
  // the general instantiation (tap tests and input code sums) serves every case; the common ones
  // (filter offset 0, with or without padding) have leaner copies
  const bool xsum = p.w_off != 0;
  const bool padded = p.pad_t != 0 || p.pad_l != 0 || (p.oh - 1) * p.stride_h - p.pad_t + p.r > p.h ||
                      (p.ow - 1) * p.stride_w - p.pad_l + p.s > p.w_;
  if (xsum) return launch_wide_variant<BN, B_KN, true, true, NBUF>(p, plan, stream);
  if (padded) return launch_wide_variant<BN, B_KN, true, false, NBUF>(p, plan, stream);
  return launch_wide_variant<BN, B_KN, false, false, NBUF>(p, plan, stream);
}

}  // namespace

bool wide_i8_applicable(const Problem& p) {
  if (p.r > 16 || p.s > 16) return false;                       // tap masks are 16 bits per axis
  if (p.x_bytes >= 0x80000000u || p.w_bytes >= 0x80000000u) return false;
  if (p.k % 4 != 0 || p.kg % 4 != 0) return false;              // dword-granular channel handling
  if (p.b_is_kn) return p.Kgemm % 16 == 0 && p.k % 16 == 0 && p.groups == 1;   // 16-byte chunks of weight rows
  return p.cg % 16 == 0 && p.c % 16 == 0;
}

// Tiles of 128 pixels x bn channels; the reduction is split over workgroups when the tiles alone
// leave most of the 256 CUs idle.  Cost model in units of one slab: rounds of 256 workgroups, each
// its slabs plus a fixed overhead, plus the traffic of the int32 partial sums.
Plan plan_wide_i8(const Problem& p, int bn, bool allow_split) {
  Plan pl;
  pl.kernel = KERNEL_WIDE;
  pl.tile = bn == 128 ? 4 : 5;
  pl.bm = WBM;
  pl.bn = bn;
  pl.bk = WBK;
  pl.tiles_m = (p.M + WBM - 1) / WBM;
  pl.tiles_n = (p.kg + bn - 1) / bn;
  pl.slabs = (p.Kgemm + WBK - 1) / WBK;
  pl.split_k = 1;
  pl.slabs_per_split = pl.slabs;
  const long long tiles = (long long)pl.tiles_m * pl.tiles_n * p.groups;
  if (allow_split && tiles < 192 && pl.slabs >= 8) {
    double best_cost = 1e30;
    int best = 1;
    for (int sk = 1; sk <= 32 && sk * 4 <= pl.slabs; ++sk) {
      const int sps = (pl.slabs + sk - 1) / sk;
      if ((pl.slabs + sps - 1) / sps != sk) continue;
      const double rounds = (double)((tiles * sk + 255) / 256);
      double cost = rounds * (sps + 8.0);
      if (sk > 1) cost += (double)(sk + 1) * p.M * p.k * 4.0 / 4e12 / 0.25e-6;
      if (cost < best_cost - 1e-9) { best_cost = cost; best = sk; }
    }
    if (knob_is_set(KNOB_I8_WIDE_SPLIT)) {                 // experiments: clamped to what the slabs allow
      best = knob(KNOB_I8_WIDE_SPLIT);
      if (best < 1) best = 1;
      if (best > pl.slabs) best = pl.slabs;
      if (best > 32) best = 32;
    }
    if (best > 1) {
      pl.slabs_per_split = (pl.slabs + best - 1) / best;
      pl.split_k = (pl.slabs + pl.slabs_per_split - 1) / pl.slabs_per_split;
    }
  }
  return pl;
}

hipError_t launch_wide_i8(const Problem& p, const Plan& plan, hipStream_t stream, const char** variant) {
  // ring depth: a grid of at most one workgroup per CU runs one round, so each workgroup gets the
  // whole LDS (four buffers, three slabs in flight); larger grids run two workgroups per CU with two
  // buffers each, which hides one workgroup's prologue and epilogue behind the other's main loop
  const long long work = (long long)plan.tiles_m * plan.tiles_n * p.groups * plan.split_k;
  int nbuf = work <= 256 ? 4 : 2;
  if (knob_is_set(KNOB_I8_WIDE_NBUF)) nbuf = knob(KNOB_I8_WIDE_NBUF) == 2 ? 2 : 4;   // experiments
  static thread_local char name[64];
  snprintf(name, sizeof(name), "igemm_i8_wide_128x%dk2w8r%d_%s", plan.bn, nbuf, p.b_is_kn ? "fc" : "conv");
  *variant = name;
  if (p.b_is_kn) return nbuf == 2 ? launch_wide_flags<128, true, 2>(p, plan, stream)
                                  : launch_wide_flags<128, true, 4>(p, plan, stream);
  if (plan.bn == 128) return nbuf == 2 ? launch_wide_flags<128, false, 2>(p, plan, stream)
                                       : launch_wide_flags<128, false, 4>(p, plan, stream);
  return nbuf == 2 ? launch_wide_flags<64, false, 2>(p, plan, stream)
                   : launch_wide_flags<64, false, 4>(p, plan, stream);
}

}  // namespace glowmi
