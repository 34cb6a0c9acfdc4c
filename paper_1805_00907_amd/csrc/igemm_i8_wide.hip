// int8 implicit-GEMM Convolution / FullyConnected for large contractions on gfx950 (MI355X): the
// quantized form of Section 4 of the paper (int8 codes with per-tensor scale/offset, int32
// accumulation, the rescale folded into the producer, Relu as an integer lower bound) for layers
// whose cost is the contraction itself rather than moving bytes.
//
// For v_mfma_i32_32x32x32_i8 a wavefront must reuse every operand fragment it reads from LDS at
// least twice, and the vector ALU gets about seven issue slots per MFMA, so this kernel is built
// around what is spent per reduction slab besides the MFMAs:
//   - one workgroup = 128 pixels x BN channels, eight wavefronts: 2 x 2 wavefronts tile the output
//     (64 x BN/2 each, 2 x BN/64 MFMA tiles) and two such sets split every 128-code slab between them
//     (codes 0..63 and 64..127), so each SIMD always has two wavefronts to interleave, however small
//     the grid is; the two partial tiles are exchanged through LDS at the end and each wavefront
//     finishes half of them;
//   - staging is specialised by wavefront: four stage the filter slab, four the input slab; the
//     gathers are 16-byte loads held in registers for three slabs (three slabs in flight) before
//     they are written to double-buffered LDS;
//   - whether a filter tap falls on padding is one bit test against a per-pixel mask computed once;
//   - the FullyConnected weight ([K][N], N contiguous) is turned K-contiguous with byte permutes
//     (16 x 4 bytes per thread, eight permutes per 16 bytes) on its way to LDS;
//   - LDS rows are 128 bytes, 16-byte chunks XOR-swizzled by the row so that fragment reads, the
//     row-wise writes of the gathers and the column-wise writes of the transposed weight are all
//     spread over the banks.
// Offsets are removed after the contraction exactly as in the generic kernel:
//   sum (x - xo)(w - wo) = sum x*w - xo * sum_k w - wo * sum_k x + Kcount * xo * wo,
// padded taps staged as the code xo.  Everything after the accumulator is integer arithmetic.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "igemm.h"
#include "quant_epilogue.h"

namespace glowmi {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WBM = 128;                 // pixels per workgroup tile
constexpr int WBK = 128;                 // codes per reduction slab
constexpr int WTHREADS = 512;
constexpr int WSTAGES = 3;               // slabs held in registers between the gather and LDS

// Byte offset of 16-byte chunk c (0..7) of row `row` inside a staged operand.
__device__ __forceinline__ int chunk_at(int row, int c) {
  return row * WBK + ((c ^ (row & 7) ^ ((row >> 3) & 3)) << 4);
}

__device__ __forceinline__ int sum4(int packed, int acc) {   // acc + the four signed bytes
  return __builtin_amdgcn_sdot4(packed, 0x01010101, acc, false);
}

__device__ __forceinline__ int requantize(int acc, int mant, int shift, int y_off, int lo) {
  return shift >= 33 ? requantize_as<true>(acc, mant, shift, y_off, lo)
                     : requantize_as<false>(acc, mant, shift, y_off, lo);   // uniform branch
}

// PADDED: some filter tap of some pixel may fall on padding (otherwise the per-tap tests are dropped).
// XSUM: the filter offset is not zero, so the input code sums per pixel are needed as well.
template <int BN, bool B_KN, bool PADDED, bool XSUM>
__global__ __launch_bounds__(WTHREADS) void igemm_i8_wide_kernel(const Problem p, int tiles_m, int tiles_n,
                                                                int band_n, int total_work) {
  static_assert(BN == 64 || BN == 128, "channel tile");
  static_assert(!B_KN || BN == 128, "the transposing weight path stages 128 columns");
  constexpr int TN = BN / 64;                           // MFMA tiles along the channels per wavefront
  constexpr int A_BYTES = WBM * WBK, B_BYTES = BN * WBK, BUF = A_BYTES + B_BYTES;
  constexpr int BQ = BN / 32;                           // 16-byte chunks a filter-staging thread moves per slab
  constexpr int OUT_PITCH = BN + 16;
  static_assert(2 * BUF >= WBM * OUT_PITCH, "output staging fits the slab buffers");
  static_assert(2 * BUF >= 8 * TN * 16 * 64 * 4, "exchange of the partial tiles fits the slab buffers");

  extern __shared__ __align__(16) unsigned char lds[];
  int* xsum = reinterpret_cast<int*>(lds + 2 * BUF);    // [128] input code sums per pixel row
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
  const bool stage_a = wave >= 4;                       // wavefronts 4..7 gather the input, 0..3 the filter
  const int st = tid & 255;                             // index among the 256 threads of one staging role
  const int lrow = lane & 31, lhalf = lane >> 5;

  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);
  constexpr unsigned OOB = 0x80000000u;                 // beyond any tensor this kernel accepts: loads give 0

  for (int i = tid; i < WBM + BN; i += WTHREADS) xsum[i] = 0;   // xsum and wsum (visible after the first barrier)

  const int slab_begin = split * p.slabs_per_split;
  const int total_slabs = (p.Kgemm + WBK - 1) / WBK;
  int slab_end = slab_begin + p.slabs_per_split;
  if (slab_end > total_slabs) slab_end = total_slabs;
  int k_hi = slab_end * WBK;
  if (k_hi > p.Kgemm) k_hi = p.Kgemm;
  const int k_count = k_hi - slab_begin * WBK;          // codes this split really reduces over

  // ---- staging state
  // input role: thread = (chunk kvec of the slab, pixel rows st/8 + 32q)
  // filter role, [k][r][s][c] layout: thread = (chunk kvec, channel rows st/8 + 32q)
  // filter role, [K][N] layout: thread = (4 columns ng, 16 reduction rows kblk)
  const int kvec = st & 7, row0 = st >> 3;
  unsigned a_base[4];                                   // byte offset of the pixel's window origin
  unsigned a_mask[4];                                   // bits 0..15: filter rows inside, 16..31: filter columns inside
  unsigned b_off[4];                                    // filter role: byte offset of each channel row / of the thread's column
  int tap_r = 0, tap_s = 0, tap_c = 0;                  // filter tap and channel of this thread's chunk in the next slab
  const int xo_fill = (p.x_off & 0xff) * 0x01010101;    // padding = the code of real zero
  constexpr bool need_xsum = XSUM;
  if (stage_a) {
    const int ohow = p.oh * p.ow;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int m = tm * WBM + row0 + q * 32;
      a_base[q] = OOB;                                  // rows past M: every load out of range
      a_mask[q] = 0;
      if (m < p.M) {
        const int img = p.div_ohow.div(m);
        const int rem = m - img * ohow;
        const int oh = p.div_ow.div(rem);
        const int ow = rem - oh * p.ow;
        const int ih0 = oh * p.stride_h - p.pad_t, iw0 = ow * p.stride_w - p.pad_l;
        a_base[q] = (unsigned)(((img * p.h + ih0) * p.w_ + iw0) * p.c + g * p.cg);   // may wrap below 0: only used with an inside tap
        const int rlo = ih0 < 0 ? -ih0 : 0, rhi = p.h - ih0 < p.r ? p.h - ih0 : p.r;
        const int slo = iw0 < 0 ? -iw0 : 0, shi = p.w_ - iw0 < p.s ? p.w_ - iw0 : p.s;
        const unsigned rm = rhi > rlo ? (1u << rhi) - (1u << rlo) : 0u;
        const unsigned sm = shi > slo ? (1u << shi) - (1u << slo) : 0u;
        a_mask[q] = rm | (sm << 16);
      }
    }
    const int kg0 = slab_begin * WBK + kvec * 16;
    const int t = p.div_cg.div(kg0);
    tap_c = kg0 - t * p.cg;
    tap_r = p.div_s.div(t);
    tap_s = t - tap_r * p.s;
  } else if (!B_KN) {
#pragma unroll
    for (int q = 0; q < BQ; ++q) {
      const int n = tn * BN + row0 + q * 32;
      b_off[q] = n < p.kg ? (unsigned)((g * p.kg + n) * p.Kgemm + kvec * 16) : OOB;
    }
  } else {
    const int col = tn * BN + (st & 31) * 4;
    b_off[0] = col < p.k ? (unsigned)((st >> 5) * 16 * p.k + col) : OOB;
  }

  v4i stage[WSTAGES][4];
  unsigned fill[WSTAGES] = {0, 0, 0};                   // input role: which of a stage's 4 chunks are padding
  int asum[4] = {0, 0, 0, 0};                           // input role: running code sums of its 4 pixel rows
  int bsum[4] = {0, 0, 0, 0};                           // filter role: running code sums of its rows / columns

  // Issue the gathers of slab `slab` into one register stage.
  // The staging role is a compile-time argument: the main loop exists once per role, so each copy
  // has a fixed number of loads per slab and waits exactly for the slab it is about to write to LDS
  // while the younger gathers stay in flight.
  using RoleInput = std::integral_constant<int, 0>;
  using RoleFilter = std::integral_constant<int, 1>;
  auto gather = [&](auto role, int slab, v4i (&r)[4], unsigned& pad) {
    constexpr bool INPUT = decltype(role)::value == 0;
    if constexpr (INPUT) {
      const int kg0 = slab * WBK + kvec * 16;
      const bool kok = kg0 < p.Kgemm;                   // reduction tail: zeros (the filter side is zero there too)
      const unsigned tap_off = (unsigned)((tap_r * p.w_ + tap_s) * p.c + tap_c);
      pad = 0;
      if constexpr (PADDED || XSUM) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const bool inside = (a_mask[q] >> tap_r) & (a_mask[q] >> (16 + tap_s)) & 1u;
          r[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, (inside && kok) ? a_base[q] + tap_off : OOB, 0, 0);
          if (!inside && kok) pad |= 1u << q;
        }
      } else {
        // no tap can fall on padding and no code sums are taken: in the reduction tail the filter
        // side is zero, so whatever an in-range address holds there does not matter
#pragma unroll
        for (int q = 0; q < 4; ++q) r[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, a_base[q] + tap_off, 0, 0);
      }
      tap_c += WBK;                                     // this thread's chunk one slab further
      while (tap_c >= p.cg) {
        tap_c -= p.cg;
        if (++tap_s == p.s) { tap_s = 0; ++tap_r; }
      }
    } else if constexpr (!B_KN) {
      const unsigned koff = (unsigned)(slab * WBK);
      const bool kok = slab * WBK + kvec * 16 < p.Kgemm;
#pragma unroll
      for (int q = 0; q < BQ; ++q)
        r[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, kok ? b_off[q] + koff : OOB, 0, 0);
    } else {
      // 16 reduction rows x 4 columns; rows at or beyond Kgemm lie past the end of the tensor: zeros
      const unsigned base = b_off[0] + (unsigned)(slab * WBK) * (unsigned)p.k;
#pragma unroll
      for (int j = 0; j < 16; ++j)
        r[j >> 2][j & 3] = __builtin_amdgcn_raw_buffer_load_b32(rsrc_w, base + (unsigned)j * (unsigned)p.k, 0, 0);
    }
  };

  // Write one register stage to LDS buffer `buf` (padding filled in, weight transposed, sums taken).
  auto commit = [&](auto role, int buf, v4i (&r)[4], unsigned pad) {
    constexpr bool INPUT = decltype(role)::value == 0;
    unsigned char* As = lds + buf * BUF;
    unsigned char* Bs = As + A_BYTES;
    if constexpr (INPUT) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        v4i v = r[q];
        if constexpr (PADDED || XSUM) {
          if ((pad >> q) & 1u) v = v4i{xo_fill, xo_fill, xo_fill, xo_fill};
        }
        *reinterpret_cast<v4i*>(As + chunk_at(row0 + q * 32, kvec)) = v;
        if (need_xsum) asum[q] = sum4(v[0], sum4(v[1], sum4(v[2], sum4(v[3], asum[q]))));
      }
    } else if constexpr (!B_KN) {
#pragma unroll
      for (int q = 0; q < BQ; ++q) {
        *reinterpret_cast<v4i*>(Bs + chunk_at(row0 + q * 32, kvec)) = r[q];
        bsum[q] = sum4(r[q][0], sum4(r[q][1], sum4(r[q][2], sum4(r[q][3], bsum[q]))));
      }
    } else {
      // r[t][i] holds row 4t+i of 16 reduction rows, 4 columns per dword: transpose 4x4 byte blocks
      // so that column nn becomes 16 consecutive reduction codes
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const unsigned d0 = r[t][0], d1 = r[t][1], d2 = r[t][2], d3 = r[t][3];
        const unsigned p01l = __builtin_amdgcn_perm(d1, d0, 0x05010400u), p01h = __builtin_amdgcn_perm(d1, d0, 0x07030602u);
        const unsigned p23l = __builtin_amdgcn_perm(d3, d2, 0x05010400u), p23h = __builtin_amdgcn_perm(d3, d2, 0x07030602u);
        r[t][0] = (int)__builtin_amdgcn_perm(p23l, p01l, 0x05040100u);   // column 0, reduction rows 4t..4t+3
        r[t][1] = (int)__builtin_amdgcn_perm(p23l, p01l, 0x07060302u);   // column 1
        r[t][2] = (int)__builtin_amdgcn_perm(p23h, p01h, 0x05040100u);   // column 2
        r[t][3] = (int)__builtin_amdgcn_perm(p23h, p01h, 0x07060302u);   // column 3
      }
      const int ng = st & 31, kblk = st >> 5;
#pragma unroll
      for (int nn = 0; nn < 4; ++nn) {
        const v4i v = v4i{r[0][nn], r[1][nn], r[2][nn], r[3][nn]};
        *reinterpret_cast<v4i*>(Bs + chunk_at(ng * 4 + nn, kblk)) = v;
        bsum[nn] = sum4(v[0], sum4(v[1], sum4(v[2], sum4(v[3], bsum[nn]))));
      }
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

  // Fragment addresses: lane (lrow, lhalf) reads chunk 2*k32 + lhalf of its row; the row's swizzle
  // only depends on lrow because fragment row blocks start at multiples of 32.
  const int swz = (lrow & 7) ^ ((lrow >> 3) & 3);
  int frag_a[2], frag_b[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const int c = ((kgrp * 2 + kk) * 2 + lhalf) ^ swz;
    frag_a[kk] = (wm * 64 + lrow) * WBK + (c << 4);
    frag_b[kk] = A_BYTES + (wn * (BN / 2) + lrow) * WBK + (c << 4);
  }

  auto compute = [&](int buf) {
    const unsigned char* base = lds + buf * BUF;
    v4i a[2][2], b[2][TN];                              // all fragment reads first: the MFMAs start as they arrive
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
      for (int i = 0; i < 2; ++i) a[kk][i] = *reinterpret_cast<const v4i*>(base + frag_a[kk] + i * 32 * WBK);
#pragma unroll
      for (int j = 0; j < TN; ++j) b[kk][j] = *reinterpret_cast<const v4i*>(base + frag_b[kk] + j * 32 * WBK);
    }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)   // filter fragment as the row operand: result rows = channels
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[kk][j], a[kk][i], acc[i][j], 0, 0, 0);
  };

  // ---- main loop: slab s is multiplied out of LDS buffer s%2 while slab s+1 waits in registers and
  // slab s+2 is being fetched.  Unrolled six times so that buffer and register-stage indices are
  // compile-time constants; the steady-state trips issue every gather unconditionally.  Both roles
  // execute the same number of barriers.
  auto run = [&](auto role) {
    gather(role, slab_begin, stage[0], fill[0]);
    if (slab_begin + 1 < slab_end) gather(role, slab_begin + 1, stage[1], fill[1]);
    commit(role, 0, stage[0], fill[0]);
    __syncthreads();
    int s0 = slab_begin;
    for (; s0 + 8 <= slab_end; s0 += 6) {
#pragma unroll
      for (int u = 0; u < 6; ++u) {
        gather(role, s0 + u + 2, stage[(u + 2) % 3], fill[(u + 2) % 3]);
        compute(u & 1);
        commit(role, (u & 1) ^ 1, stage[(u + 1) % 3], fill[(u + 1) % 3]);
        __syncthreads();
      }
    }
    for (; s0 < slab_end; s0 += 6) {
#pragma unroll
      for (int u = 0; u < 6; ++u) {
        const int s = s0 + u;
        if (s < slab_end) {
          if (s + 2 < slab_end) gather(role, s + 2, stage[(u + 2) % 3], fill[(u + 2) % 3]);
          compute(u & 1);
          if (s + 1 < slab_end) commit(role, (u & 1) ^ 1, stage[(u + 1) % 3], fill[(u + 1) % 3]);
          __syncthreads();
        }
      }
    }
  };
  if (stage_a) run(RoleInput{});
  else run(RoleFilter{});

  // ---- code sums: every staging thread adds what it saw (LDS atomics; integer, so order is free)
  if (stage_a) {
    if (need_xsum) {
#pragma unroll
      for (int q = 0; q < 4; ++q) atomicAdd(&xsum[row0 + q * 32], asum[q]);
    }
  } else if (!B_KN) {
#pragma unroll
    for (int q = 0; q < BQ; ++q) atomicAdd(&wsum[row0 + q * 32], bsum[q]);
  } else {
#pragma unroll
    for (int nn = 0; nn < 4; ++nn) atomicAdd(&wsum[(st & 31) * 4 + nn], bsum[nn]);
  }

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
  const unsigned rowterm = need_xsum ? (unsigned)p.w_off * (unsigned)xsum[lr] : 0u;

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

template <int BN, bool B_KN, bool PADDED, bool XSUM>
hipError_t launch_wide_variant(const Problem& p, const Plan& plan, hipStream_t stream) {
  auto kern = igemm_i8_wide_kernel<BN, B_KN, PADDED, XSUM>;
  constexpr int lds_bytes = 2 * (WBM + BN) * WBK + (WBM + 2 * BN) * 4;
  static bool attr_set = false;   // per instantiation; benign if two threads race to set it
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
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

}  // namespace

bool wide_i8_applicable(const Problem& p) {
  if (p.r > 16 || p.s > 16) return false;                       // tap masks are 16 bits per axis
  if (p.x_bytes >= 0x80000000u || p.w_bytes >= 0x80000000u) return false;
  if (p.k % 4 != 0 || p.kg % 4 != 0) return false;              // dword-granular channel handling
  if (p.b_is_kn) return p.Kgemm % 16 == 0 && p.groups == 1;
  return p.cg % 16 == 0 && p.c % 16 == 0;
}

// Tiles of 128 pixels x bn channels; the reduction is split over workgroups when the tiles alone
// leave most of the 256 CUs idle.  Cost model in units of one slab: rounds of 256 workgroups, each
// its slabs plus a fixed overhead, plus the traffic of the int32 partial sums.
Plan plan_wide_i8(const Problem& p, int bn, bool allow_split) {
  Plan pl;
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
    if (best > 1) {
      pl.slabs_per_split = (pl.slabs + best - 1) / best;
      pl.split_k = (pl.slabs + pl.slabs_per_split - 1) / pl.slabs_per_split;
    }
  }
  return pl;
}

hipError_t launch_wide_i8(const Problem& p, const Plan& plan, hipStream_t stream, const char** variant) {
  static thread_local char name[64];
  snprintf(name, sizeof(name), "igemm_i8_wide_128x%dk2w8_%s", plan.bn, p.b_is_kn ? "fc" : "conv");
  *variant = name;
  // the general instantiation (tap tests and input code sums) serves every case; the common ones
  // (filter offset 0, with or without padding) have leaner copies
  const bool xsum = p.w_off != 0;
  const bool padded = p.pad_t != 0 || p.pad_l != 0 || (p.oh - 1) * p.stride_h - p.pad_t + p.r > p.h ||
                      (p.ow - 1) * p.stride_w - p.pad_l + p.s > p.w_;
  if (p.b_is_kn) return xsum ? launch_wide_variant<128, true, true, true>(p, plan, stream)
                             : launch_wide_variant<128, true, false, false>(p, plan, stream);
  if (plan.bn == 128) {
    if (xsum) return launch_wide_variant<128, false, true, true>(p, plan, stream);
    return padded ? launch_wide_variant<128, false, true, false>(p, plan, stream)
                  : launch_wide_variant<128, false, false, false>(p, plan, stream);
  }
  if (xsum) return launch_wide_variant<64, false, true, true>(p, plan, stream);
  return padded ? launch_wide_variant<64, false, true, false>(p, plan, stream)
                : launch_wide_variant<64, false, false, false>(p, plan, stream);
}

}  // namespace glowmi
