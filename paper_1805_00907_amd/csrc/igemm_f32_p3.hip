// fp32 Convolution / FullyConnected on the fp16 matrix cores, accurate to fp32 level: the contraction of
// Section 3.4 / 3.1 of the paper (MatMul + broadcast add, the convolution loop nest) with every fp32
// operand cut into two fp16 pieces first (f16_pieces.h).
//
//   A tensor is scaled by a power of two taken from its largest magnitude (found by a pass over the tensor,
//   range_kernel) and every scaled value v is cut into h1 = fp16(v) and H2 = fp16((v - h1) * 2^11); a product
//   is taken as h1 h1' + 2^-11 (h1 H2' + H2 h1'): three v_mfma_f32_32x32x16_f16, which multiply fp16 exactly
//   and accumulate in fp32, the cross terms in an accumulator set of their own.  What is lost against an fp32
//   multiply-add chain is 2^-22 H2 H2' and the cuts' own rounding, each at most 2^-22 of |v v'|.  Three MFMAs
//   cover 16 reduction steps of a 32 x 32 block in 96 matrix-pipe cycles; v_mfma_f32_32x32x2_f32 needs 512 for
//   the same (and the earlier form of this kernel, three bf16 pieces and six products, 192).
//
// Cutting the operands inside the contraction kernel costs about six vector instructions per staged
// element, again for every tile that stages it (a 3 x 3 layer stages each input element 9 x N/128
// times), and measured that eats most of the gain.  So the pieces are made ONCE per call by a packing
// pass into two fp16 planes per operand (workspace), FullyConnected weights ([K][N]) transposed to
// K-contiguous on the way, and the contraction kernel has no vector ALU work in its loop at all:
//   - 128 pixels x 64*WN channels per workgroup; 2 x WN wavefronts tile the output (64 x 64 each) and two such
//     sets split every slab's 32 reduction indices between them (16 each); the two partial tiles are
//     exchanged through LDS at the end and each wavefront finishes half of them;
//   - slabs of 32 reduction indices = one 64-byte row piece per plane, always inside one filter tap
//     (channels per group are walked in steps of 32), so tap and channel offset are scalars;
//   - both operands' planes go from global memory straight into LDS (buffer loads with the LDS bit) into a
//     ring of NBUF slab buffers, NBUF - 1 slabs in flight; lanes that are out of range (rows past the
//     tensor, channel tail, taps on padding) get zeros from the hardware, which is what they must be;
//   - lane l of a load fetches chunk (l % 4) ^ ((l / 16) % 4) of row l / 4: the four 16-byte chunks of a
//     row are XOR-swizzled so that the 16 rows one phase of a fragment ds_read_b128 touches fall on 16
//     different bank groups, without padding;
//   - the epilogue is the fp32 one (the two accumulator sets joined and scaled back, bias, tensor add, Relu,
//     one store), or partial tiles for a split reduction that the common finishing kernel sums in split order.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <type_traits>

#include "f16_pieces.h"
#include "igemm.h"
#include "lds_direct.h"

namespace glowmi {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int PBM = 128;                 // pixels per workgroup tile
constexpr int PBK = 32;                  // reduction indices per slab
constexpr int PROW = 2 * PBK;            // bytes of one plane row in LDS
constexpr int P3_FLUSH = 32;             // accumulators are folded into a second set every 1024 reduction steps
constexpr size_t kPlaneAlign = 256;

// ------------------------------------------------------------------------------------------------
// Range pass and packing: fp32 -> two fp16 planes
// ------------------------------------------------------------------------------------------------
// Largest magnitude of a tensor as kRangeWords partial maxima (bits of |v|, which order like the values; a NaN
// orders above everything and so reaches the scale, where it turns the results into NaN as it should): workgroup
// b of a tensor's kRangeWords walks float4 number b, b + kRangeWords, .. and writes word b.  No atomics and
// nothing to clear beforehand; whoever needs the maximum takes the largest of the words (wave_max_words).
constexpr int kRangeThreads = 1024;     // sixteen wavefronts per workgroup: two workgroups keep a CU's memory pipeline full
// Non-temporal loads: the pass reads every element once, and measured on a 205 MB tensor that comes from HBM it
// runs at 6.3 TB/s with them against 3.0 TB/s with plain loads (which also allocate every line in the last-level
// cache on the way).
__device__ __forceinline__ v4u range_load(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
}
__device__ __forceinline__ void range_part(const float* __restrict__ src, long long count4, unsigned* __restrict__ out,
                                           int block, unsigned* red) {
  unsigned m = 0;
  const long long stride = (long long)kRangeWords * kRangeThreads;
  long long g = (long long)block * kRangeThreads + threadIdx.x;
  const long long lim = count4;
  for (; g + 3 * stride < lim; g += 4 * stride) {     // four loads in flight per thread
    const v4u a = range_load(src + 4 * g);
    const v4u b = range_load(src + 4 * (g + stride));
    const v4u c = range_load(src + 4 * (g + 2 * stride));
    const v4u d = range_load(src + 4 * (g + 3 * stride));
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const unsigned ma = a[e] & 0x7fffffffu, mb = b[e] & 0x7fffffffu, mc = c[e] & 0x7fffffffu, md = d[e] & 0x7fffffffu;
      const unsigned m1 = ma > mb ? ma : mb, m2 = mc > md ? mc : md;
      const unsigned m3 = m1 > m2 ? m1 : m2;
      m = m3 > m ? m3 : m;
    }
  }
  for (; g < lim; g += stride) {
    const v4u a = range_load(src + 4 * g);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const unsigned ma = a[e] & 0x7fffffffu;
      m = ma > m ? ma : m;
    }
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const unsigned o = (unsigned)__shfl_xor((int)m, d, 64);
    m = o > m ? o : m;
  }
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned r = red[0];
#pragma unroll
    for (int i = 1; i < kRangeThreads / 64; ++i) r = red[i] > r ? red[i] : r;
    out[block] = r;
  }
}

// One launch for both operands: workgroups 0 .. kRangeWords - 1 the input, the next kRangeWords the weights
// (launched without them when the weights' planes were made ahead of time).
__global__ __launch_bounds__(kRangeThreads) void range_kernel(const float* __restrict__ x, long long x_count4, unsigned* __restrict__ x_out,
                                                              const float* __restrict__ w, long long w_count4, unsigned* __restrict__ w_out) {
  __shared__ unsigned red[kRangeThreads / 64];
  const int b = (int)blockIdx.x;
  if (b < kRangeWords) range_part(x, x_count4, x_out, b, red);
  else range_part(w, w_count4, w_out, b - kRangeWords, red);
}

// The trailer behind a tensor's two planes: word 0 holds the bits of the tensor's largest magnitude (what the
// planes were scaled by follows from it), words kRangeWords .. 2 kRangeWords - 1 the partial maxima the range pass
// left there.
__device__ __forceinline__ int take_scale(const unsigned* __restrict__ trailer, bool publish) {
  __shared__ int se_shared;
  if (threadIdx.x < 64) {                                // the first wavefront reduces, the others wait for it
    const unsigned mx = wave_max_words(trailer + kRangeWords, kRangeWords);
    if (threadIdx.x == 0) {
      se_shared = scale_exponent(mx);
      if (publish) const_cast<unsigned*>(trailer)[0] = mx;
    }
  }
  __syncthreads();
  return se_shared;
}

// src: count8 groups of 8 consecutive floats; dst: two planes of plane_elems fp16 each, same order.
__device__ __forceinline__ void pack2_rows(const float* __restrict__ src, unsigned short* __restrict__ dst,
                                           long long count8, long long plane_elems, int block, int blocks,
                                           unsigned* __restrict__ trailer) {
  const int se = take_scale(trailer, block == 0);
  const long long stride = (long long)blocks * 256;
  for (long long g = (long long)block * 256 + threadIdx.x; g < count8; g += stride) {
    const v4f a = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(src + 8 * g));      // read once here
    const v4f b = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(src + 8 * g + 4));
    const float v[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    v4u p1, p2;
    cut8(v, se, p1, p2);
    *reinterpret_cast<v4u*>(dst + 8 * g) = p1;
    *reinterpret_cast<v4u*>(dst + plane_elems + 8 * g) = p2;
  }
}

// FullyConnected weight [K][N] (N contiguous) -> two planes [N][K] (K contiguous).  K % 8 == 0.
// One workgroup per 64 (k) x 64 (n) tile, transposed through LDS: rows of 256 bytes are read with one float4 per lane
// where N allows it (every load instruction covers whole 256-byte runs), a thread then gathers eight consecutive k of
// one n from the tile and writes 16 bytes per plane.  The tile's row pitch of 65 floats keeps both the row-wise
// stores and the column-wise gathers free of bank conflicts.
constexpr int kPackTile = 64;
__device__ __forceinline__ void pack2_transposed(const float* __restrict__ w, unsigned short* __restrict__ dst, int K, int N,
                                                 int tiles_n, int block, float (&tile)[kPackTile][kPackTile + 1],
                                                 unsigned* __restrict__ trailer) {
  const int se = take_scale(trailer, block == 0);
  const int tk = block / tiles_n, tn = block - tk * tiles_n;
  const int k0 = tk * kPackTile, n0 = tn * kPackTile;
  const int tid = threadIdx.x;
  if ((N & 3) == 0) {                                     // uniform: rows start on 16-byte boundaries
    const int n4 = tid & 15, kr = tid >> 4;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int k = kr + 16 * q;
      v4f v = {0.f, 0.f, 0.f, 0.f};
      if (k0 + k < K && n0 + 4 * n4 < N)
        v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(w + (size_t)(k0 + k) * N + n0 + 4 * n4));   // read once
#pragma unroll
      for (int e = 0; e < 4; ++e) tile[k][4 * n4 + e] = v[e];
    }
  } else {
    const int n = tid & 63, kr = tid >> 6;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int k = kr + 4 * q;
      tile[k][n] = (k0 + k < K && n0 + n < N) ? __builtin_nontemporal_load(w + (size_t)(k0 + k) * N + n0 + n) : 0.f;
    }
  }
  __syncthreads();
  const size_t plane = (size_t)K * N;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int item = tid + 256 * pass;
    const int n = item >> 3, kc = item & 7;
    if (n0 + n >= N || k0 + kc * 8 >= K) continue;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = tile[kc * 8 + e][n];
    v4u p1, p2;
    cut8(v, se, p1, p2);
    unsigned short* o = dst + (size_t)(n0 + n) * K + k0 + kc * 8;
    *reinterpret_cast<v4u*>(o) = p1;
    *reinterpret_cast<v4u*>(o + plane) = p2;
  }
}

__global__ __launch_bounds__(256) void pack2_rows_kernel(const float* __restrict__ src, unsigned short* __restrict__ dst,
                                                         long long count8, long long plane_elems,
                                                         unsigned* __restrict__ trailer) {
  pack2_rows(src, dst, count8, plane_elems, (int)blockIdx.x, (int)gridDim.x, trailer);
}

__global__ __launch_bounds__(256) void pack2_transposed_kernel(const float* __restrict__ w, unsigned short* __restrict__ dst,
                                                               int K, int N, int tiles_n, unsigned* __restrict__ trailer) {
  __shared__ float tile[kPackTile][kPackTile + 1];
  pack2_transposed(w, dst, K, N, tiles_n, (int)blockIdx.x, tile, trailer);
}

// Both operands of one contraction in one launch: the first blocks_x workgroups cut the input, the rest the
// weights, either in their own order or (FullyConnected, transposed != 0) one 64 x 64 tile per workgroup.
__global__ __launch_bounds__(256) void pack2_pair_kernel(const float* __restrict__ x, unsigned short* __restrict__ xp,
                                                         long long x_count8, long long x_elems, int blocks_x,
                                                         unsigned* __restrict__ x_trailer,
                                                         const float* __restrict__ w, unsigned short* __restrict__ wp,
                                                         long long w_count8, long long w_elems, int transposed, int K,
                                                         int N, int tiles_n, unsigned* __restrict__ w_trailer) {
  __shared__ float tile[kPackTile][kPackTile + 1];
  const int b = (int)blockIdx.x;
  if (b < blocks_x) pack2_rows(x, xp, x_count8, x_elems, b, blocks_x, x_trailer);
  else if (transposed) pack2_transposed(w, wp, K, N, tiles_n, b - blocks_x, tile, w_trailer);
  else pack2_rows(w, wp, w_count8, w_elems, b - blocks_x, (int)gridDim.x - blocks_x, w_trailer);
}

// ------------------------------------------------------------------------------------------------
// Contraction over the planes
// ------------------------------------------------------------------------------------------------
// WN: 64-channel columns of wavefronts (2: 128 channels, 512 threads; 1: 64 channels, 256 threads).
// PADDED: some filter tap of some pixel may fall on padding.  LONGK: reductions longer than P3_FLUSH slabs
// keep a second accumulator set.  NBUF: slab buffers in the LDS ring.
template <int WN, bool PADDED, bool LONGK, int NBUF>
__global__ __launch_bounds__(256 * WN, 2) void igemm_f32_p3_kernel(const Problem p, int tiles_m, int tiles_n,
                                                                   int band_n, int total_work) {
  constexpr int BN = 64 * WN;
  constexpr int WAVES = 4 * WN;
  constexpr int A_GROUPS = (PBM / 16) / WAVES;          // 16-row groups of the pixel tile one wavefront loads per plane
  static_assert(A_GROUPS * WAVES * 16 == PBM && WAVES * 16 == BN, "rows divide over the wavefronts");
  constexpr int LPI = 2 * (A_GROUPS + 1);               // loads one wavefront issues per slab
  constexpr int A_PLANE = PBM * PROW, B_PLANE = BN * PROW;
  constexpr int BUF = 2 * (A_PLANE + B_PLANE);
  static_assert(NBUF * BUF >= WAVES * 32 * 64 * 4, "exchange of the partial tiles fits the slab buffers");

  extern __shared__ __align__(16) unsigned char lds[];

  // ---- which tile: consecutive workgroup ids go round-robin to the 8 XCDs, so id % 8 picks the XCD and
  // each XCD gets a contiguous run of tiles, walked in bands of band_n tile columns so that the run of
  // one XCD covers a compact block of the output.
  const int per_xcd = gridDim.x >> 3;
  const int wk = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (wk >= total_work) return;
  const int plane = tiles_m * tiles_n;
  const int pl_i = wk / plane, wi = wk - pl_i * plane;
  const int g = pl_i % p.groups;
  const int split = pl_i / p.groups;
  const int band = wi / (tiles_m * band_n);
  const int in_band = wi - band * tiles_m * band_n;
  const int band_w = tiles_n - band * band_n < band_n ? tiles_n - band * band_n : band_n;
  const int tm = in_band / band_w;
  const int tn = band * band_n + (in_band - tm * band_w);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kgrp = wave / (2 * WN);                      // which 16 of every slab's 32 reduction indices
  const int wm = (wave / WN) & 1, wn = wave % WN;
  const int lrow = lane & 31, lhalf = lane >> 5;

  const unsigned xpb = p.x_bytes >> 1, wpb = p.w_bytes >> 1;          // bytes of one fp16 plane
  const v4i rsrc_x = make_rsrc(p.planes, 2u * xpb);
  const v4i rsrc_w = make_rsrc(p.w_planes, 2u * wpb);
  constexpr unsigned OOB = 0x80000000u;   // planes are at most 512 MiB each: OOB + a plane neither wraps nor lands inside
  // what the two accumulator sets are scaled back by: the operands' scale exponents, from their largest magnitudes
  const ScaleBack sb = scale_back(wave_max_words(p.x_range, p.x_range_n), wave_max_words(p.w_range, 1));

  // The bias values now, not in the epilogue: a load there would make the compiler wait for all memory operations
  // in front of every store (each store is a branch of its own, and each would wait for the store before it).
  float bias_v[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = tn * BN + wn * 64 + j * 32 + lrow;
    const float* __restrict__ bias_p = static_cast<const float*>(p.bias);
    bias_v[j] = (col < p.kg && p.split_k == 1 && bias_p) ? bias_p[g * p.kg + col] : 0.f;
  }

  const int spt = (p.cg + PBK - 1) / PBK;               // slabs per filter tap
  const int total_slabs = p.r * p.s * spt;
  const int slab_begin = split * p.slabs_per_split;
  int slab_end = slab_begin + p.slabs_per_split;
  if (slab_end > total_slabs) slab_end = total_slabs;

  // ---- staging state.  A load covers 16 tile rows: lane l the row (l / 4) of the group and chunk position l % 4,
  // where chunk (l % 4) ^ swz(row) of that row is stored, swz(row) = (row / 4) % 4 = (l / 16) % 4.
  const int cch = (lane & 3) ^ ((lane >> 4) & 3);
  unsigned a_base[A_GROUPS], a_mask[A_GROUPS];
  {
    const int ohow = p.oh * p.ow;
#pragma unroll
    for (int t = 0; t < A_GROUPS; ++t) {
      const int m = tm * PBM + 16 * (wave + WAVES * t) + (lane >> 2);
      a_base[t] = OOB;
      a_mask[t] = 0;
      if (m < p.M) {
        const int img = p.div_ohow.div(m);
        const int rem = m - img * ohow;
        const int oh = p.div_ow.div(rem);
        const int ow = rem - oh * p.ow;
        const int ih0 = oh * p.stride_h - p.pad_t, iw0 = ow * p.stride_w - p.pad_l;
        // byte offset of the window origin's channel run in plane 0 (may wrap below 0: only used with an inside tap)
        a_base[t] = 2u * (unsigned)(((img * p.h + ih0) * p.w_ + iw0) * p.c + g * p.cg + cch * 8);
        const int rlo = ih0 < 0 ? -ih0 : 0, rhi = p.h - ih0 < p.r ? p.h - ih0 : p.r;
        const int slo = iw0 < 0 ? -iw0 : 0, shi = p.w_ - iw0 < p.s ? p.w_ - iw0 : p.s;
        const unsigned rm = rhi > rlo ? (1u << rhi) - (1u << rlo) : 0u;
        const unsigned sm = shi > slo ? (1u << shi) - (1u << slo) : 0u;
        a_mask[t] = rm | (sm << 16);
      }
    }
  }
  unsigned b_base;                                      // byte offset of the filter row's chunk in plane 0
  {
    const int n = tn * BN + 16 * wave + (lane >> 2);
    b_base = n < p.kg ? 2u * ((unsigned)(g * p.kg + n) * (unsigned)p.Kgemm + (unsigned)(cch * 8)) : OOB;
  }
  // scalar walk over (tap, channel block): the next slab to issue
  int tap_r, tap_s, tap_c0, next_slab = slab_begin;
  {
    const int t = slab_begin / spt;
    tap_c0 = (slab_begin - t * spt) * PBK;
    tap_r = t / p.s;
    tap_s = t - tap_r * p.s;
  }

  // The loads of the next slab to issue, in LPI pieces so that they can be dealt out between the MFMAs of a trip
  // (a wavefront whose load waits for a slot in the address unit's queue issues nothing else meanwhile).
  unsigned is_a[A_GROUPS], is_b, is_lds;
  auto issue_prepare = [&](int buf) {
    is_lds = __builtin_amdgcn_readfirstlane(lds_offset_of(lds) + buf * BUF + wave * 16 * PROW);
    const bool live = next_slab < slab_end;             // ring positions past the end: zeros, no memory traffic
    const bool cok = live && tap_c0 + cch * 8 < p.cg;   // channel tail of a tap
    const unsigned tap_off = 2u * (unsigned)((tap_r * p.w_ + tap_s) * p.c + tap_c0);
    const unsigned k_off = 2u * (unsigned)((tap_r * p.s + tap_s) * p.cg + tap_c0);
#pragma unroll
    for (int t = 0; t < A_GROUPS; ++t) {
      bool ok = cok && a_base[t] != OOB;
      if constexpr (PADDED) ok = ok && ((a_mask[t] >> tap_r) & (a_mask[t] >> (16 + tap_s)) & 1u);
      is_a[t] = ok ? a_base[t] + tap_off : OOB;
    }
    is_b = (cok && b_base != OOB) ? b_base + k_off : OOB;
    ++next_slab;
    tap_c0 += PBK;
    if (tap_c0 >= p.cg) {
      tap_c0 = 0;
      if (++tap_s == p.s) { tap_s = 0; ++tap_r; }
    }
  };
  auto issue_piece = [&](int j) {                        // j = 0 .. LPI - 1, compile-time
    const int pc = j % 2, t = j / 2;
    if (t < A_GROUPS) load16_to_lds(rsrc_x, is_lds + pc * A_PLANE + t * WAVES * 16 * PROW, is_a[t] + pc * xpb);
    else load16_to_lds(rsrc_w, is_lds + 2 * A_PLANE + pc * B_PLANE, is_b + pc * wpb);
  };
  auto issue = [&](int buf) {
    issue_prepare(buf);
#pragma unroll
    for (int j = 0; j < LPI; ++j) issue_piece(j);
  };

  // acc[i][j]: 32 pixels (rows of the MFMA result) x 32 channels (columns, one per lane); acc the h1 h1' products,
  // acc_lo the cross terms (weight 2^-11)
  v16f acc[2][2], acc_lo[2][2], total[LONGK ? 2 : 1][LONGK ? 2 : 1];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        acc[i][j][e] = 0.f;
        acc_lo[i][j][e] = 0.f;
        if (LONGK) total[i][j][e] = 0.f;
      }

  // a lane holds 8 consecutive reduction indices of its row: chunk 2 * kgrp + lhalf, stored at chunk ^ swz(row)
  const int pos = ((kgrp * 2 + lhalf) ^ ((lrow >> 2) & 3)) << 4;
  const int frag_a = (wm * 64 + lrow) * PROW + pos;
  const int frag_b = 2 * A_PLANE + (wn * 64 + lrow) * PROW + pos;
  // All fragments of a slab are read up front (8 ds_read_b128) in the order the MFMAs use them, and the
  // refill loads are dealt out between the MFMAs.
  auto trip = [&](int buf, int refill_buf) {
    const unsigned char* base = lds + buf * BUF;
    v8h a[2][2], b[2][2];
#pragma unroll
    for (int o = 0; o < 2; ++o) {
      const int pa = o, pb = 1 - o;                       // the cross terms come first: a1 with b2, then a2 with b1
#pragma unroll
      for (int i = 0; i < 2; ++i)
        a[pa][i] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(base + pa * A_PLANE + frag_a + i * 32 * PROW));
#pragma unroll
      for (int j = 0; j < 2; ++j)
        b[pb][j] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(base + pb * B_PLANE + frag_b + j * 32 * PROW));
    }
    issue_prepare(refill_buf);
    __builtin_amdgcn_sched_barrier(0);
    constexpr int MFMAS = 3 * 4, EVERY = MFMAS / LPI;   // 12 MFMAs, a load after every EVERY of them
    static_assert(EVERY >= 1, "more loads than MFMAs");
#pragma unroll
    for (int q = 0; q < MFMAS; ++q) {
      const int t = q / 4, i = (q / 2) % 2, j = q % 2;
      if (t == 0) acc_lo[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], b[1][j], acc_lo[i][j], 0, 0, 0);
      else if (t == 1) acc_lo[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[1][i], b[0][j], acc_lo[i][j], 0, 0, 0);
      else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], b[0][j], acc[i][j], 0, 0, 0);
      if (q % EVERY == EVERY - 1 && q / EVERY < LPI) {
        __builtin_amdgcn_sched_barrier(0);
        issue_piece(q / EVERY);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  // ---- main loop.  Trip s: wait for slab s (the younger slabs stay in flight), barrier (everyone's part of
  // slab s has landed and everyone is done with the buffer multiplied last trip), read slab s's fragments,
  // refill that older buffer with slab s + NBUF - 1, multiply slab s.  Loads are issued on every trip, past the end as zero fills, so the waits are
  // compile-time constants.  Unrolled NBUF times so that buffer indices are constants.
  {
#pragma unroll
    for (int d = 0; d < NBUF - 1; ++d) issue(d);
    int since_flush = 0;
    for (int s0 = slab_begin; s0 < slab_end; s0 += NBUF) {
#pragma unroll
      for (int u = 0; u < NBUF; ++u) {
        if (s0 + u < slab_end) {                          // uniform
          __builtin_amdgcn_s_waitcnt(vmcnt_imm((NBUF - 2) * LPI));
          __syncthreads();
          trip(u, (u + NBUF - 1) % NBUF);
          if (LONGK && ++since_flush == P3_FLUSH) {
            since_flush = 0;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
              for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                  total[i][j][e] += __builtin_fmaf(acc_lo[i][j][e], kLowPieceWeight, acc[i][j][e]);
                  acc[i][j][e] = 0.f;
                  acc_lo[i][j][e] = 0.f;
                }
              }
          }
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));             // the zero fills past the end have landed too
    __syncthreads();                                      // every wavefront is done with the slab buffers
  }

  // ---- exchange: the two wavefronts that hold partial sums of the same 64 x 64 sub-tile (one per half of the
  // slabs) swap halves through LDS; the kgrp-0 wavefront finishes pixel rows 0..31 of the sub-tile, the other
  // rows 32..63.  Both add the same two numbers, so which of them finishes a row does not change its value.
  v16f keep[2];
  {
    v4f* xch = reinterpret_cast<v4f*>(lds);
    const int pair = wm * WN + wn;
    const int mine = (pair * 2 + kgrp) * 8, theirs = (pair * 2 + (kgrp ^ 1)) * 8;
    auto exchange_as = [&](auto kg_tag) {
      constexpr int KG = decltype(kg_tag)::value;         // sends block row 1 - KG, keeps block row KG
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        v16f snd, kp;
#pragma unroll
        for (int e = 0; e < 16; ++e) {                   // the two accumulator sets joined
          snd[e] = __builtin_fmaf(acc_lo[1 - KG][j][e], kLowPieceWeight, acc[1 - KG][j][e]);
          kp[e] = __builtin_fmaf(acc_lo[KG][j][e], kLowPieceWeight, acc[KG][j][e]);
        }
        keep[j] = kp;
        if (LONGK) {
          snd += total[1 - KG][j];
          keep[j] += total[KG][j];
        }
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4)
          xch[(mine + j * 4 + e4) * 64 + lane] = v4f{snd[e4 * 4], snd[e4 * 4 + 1], snd[e4 * 4 + 2], snd[e4 * 4 + 3]};
      }
    };
    if (kgrp) exchange_as(std::integral_constant<int, 1>{});
    else exchange_as(std::integral_constant<int, 0>{});
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const v4f got = xch[(theirs + j * 4 + e4) * 64 + lane];
#pragma unroll
        for (int t = 0; t < 4; ++t) keep[j][e4 * 4 + t] = __builtin_ldexpf(keep[j][e4 * 4 + t] + got[t], sb.neg_se) + sb.poison;   // scaled back
      }
  }

  // ---- epilogue: bias (+ tensor add) + activation on the finished sums, one store; or the partial tile.
  // 32x32 MFMA block: register e of a lane is row (e/4)*8 + (lane/32)*4 + e%4, column lane%32.
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));             // nothing is in flight any more; the compiler cannot see it
  float* __restrict__ Y = static_cast<float*>(p.y);
  const float* addend = static_cast<const float*>(p.addend);   // may be the output itself
  const bool finish = p.split_k == 1;
  const bool relu = finish && p.act == 1;
  const bool add = finish && addend != nullptr;
  float* dst_base = finish ? Y : static_cast<float*>(p.partial) + (size_t)split * p.M * p.k;
  const int row_base = tm * PBM + wm * 64 + kgrp * 32 + lhalf * 4;
  const bool full = (tm + 1) * PBM <= p.M && (tn + 1) * BN <= p.kg;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = tn * BN + wn * 64 + j * 32 + lrow;
    const bool cok = col < p.kg;
    const int ch = g * p.kg + col;
    const float bv = bias_v[j];
    float* dst = dst_base + (size_t)row_base * p.k + ch;
    const float* addp = add ? addend + (size_t)row_base * p.k + ch : nullptr;
    // the column's sixteen addend values first, all in flight together: loaded one by one in front of their stores,
    // each load would be waited for together with every store before it
    float addv[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int r = (e >> 2) * 8 + (e & 3);
      addv[e] = (add && (full || (cok && row_base + r < p.M))) ? addp[(size_t)r * p.k] : 0.f;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));            // once, here: not in front of each of the sixteen stores
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int r = (e >> 2) * 8 + (e & 3);               // compile-time row inside the 32-row block
      float v = keep[j][e] + bv + addv[e];
      const bool inside = full || (cok && row_base + r < p.M);
      if (relu) v = fmaxf(v, 0.f);
      if (inside) dst[(size_t)r * p.k] = v;
    }
  }
}

template <int WN, bool PADDED, bool LONGK, int NBUF>
hipError_t launch_p3_variant(const Problem& p, const Plan& plan, hipStream_t stream) {
  auto kern = igemm_f32_p3_kernel<WN, PADDED, LONGK, NBUF>;
  constexpr int lds_bytes = NBUF * 2 * (PBM + 64 * WN) * PROW;
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  if (attr_status != hipSuccess) return attr_status;
  const long long total_work = (long long)plan.tiles_m * plan.tiles_n * p.groups * plan.split_k;
  const long long grid_x = ((total_work + 7) / 8) * 8;
  const long long per_xcd = grid_x / 8;
  int band_n = 1;
  while ((long long)band_n * band_n * 2 < per_xcd && band_n < plan.tiles_n) ++band_n;
  dim3 grid((unsigned)grid_x, 1, 1), block(256 * WN, 1, 1);
  hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, p, plan.tiles_m, plan.tiles_n, band_n, (int)total_work);
  return hipGetLastError();
}

template <int WN, int NBUF>
hipError_t launch_p3_flags(const Problem& p, const Plan& plan, hipStream_t stream, bool padded, bool longk) {
  if (padded) return longk ? launch_p3_variant<WN, true, true, NBUF>(p, plan, stream)
                           : launch_p3_variant<WN, true, false, NBUF>(p, plan, stream);
  return longk ? launch_p3_variant<WN, false, true, NBUF>(p, plan, stream)
               : launch_p3_variant<WN, false, false, NBUF>(p, plan, stream);
}

size_t align_up(size_t v) { return (v + kPlaneAlign - 1) / kPlaneAlign * kPlaneAlign; }

}  // namespace

// A tensor's planes in memory: two fp16 planes of `elems` each, padded to 256 bytes, then the trailer.
size_t tensor_planes_bytes(size_t elems) { return align_up(4 * elems) + kPlaneTrailerBytes; }
size_t filter_planes_bytes(size_t w_elems) { return tensor_planes_bytes(w_elems); }
unsigned* planes_trailer(const void* planes, size_t elems) {
  return reinterpret_cast<unsigned*>(static_cast<unsigned char*>(const_cast<void*>(planes)) + align_up(4 * elems));
}

hipError_t launch_ranges(const float* x, long long x_elems, unsigned* x_out, const float* w, long long w_elems,
                         unsigned* w_out, hipStream_t stream) {
  const unsigned blocks = (unsigned)kRangeWords * (w ? 2u : 1u);
  hipLaunchKernelGGL(range_kernel, dim3(blocks), dim3(kRangeThreads), 0, stream, x, x_elems / 4, x_out, w, w_elems / 4, w_out);
  return hipGetLastError();
}

namespace {
// Cuts the weights whose partial maxima already lie in the trailer of dst.
hipError_t launch_cut_filter(const float* w, void* dst, int b_is_kn, int K, int N, long long w_elems, hipStream_t stream) {
  unsigned* trailer = planes_trailer(dst, (size_t)w_elems);
  if (!b_is_kn) {
    const long long c8 = w_elems / 8;
    long long blocks = (c8 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(pack2_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, w, static_cast<unsigned short*>(dst), c8,
                       w_elems, trailer);
    return hipGetLastError();
  }
  const int tn = (N + kPackTile - 1) / kPackTile;
  const long long blocks = (long long)((K + 63) / 64) * tn;
  hipLaunchKernelGGL(pack2_transposed_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, w, static_cast<unsigned short*>(dst), K,
                     N, tn, trailer);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_pack_filter(const float* w, void* dst, int b_is_kn, int K, int N, long long w_elems, hipStream_t stream) {
  const hipError_t e = launch_ranges(w, w_elems, planes_trailer(dst, (size_t)w_elems) + kRangeWords, nullptr, 0, nullptr, stream);
  if (e != hipSuccess) return e;
  return launch_cut_filter(w, dst, b_is_kn, K, N, w_elems, stream);
}

// For the kernels that cut the input themselves (conv_k3*_f32): the planes the caller made ahead of time, or the
// filter measured and cut into `dst` now.
hipError_t stage_filter_planes(Problem& p, const void* dst, hipStream_t stream) {
  const size_t w_elems = p.w_bytes >> 2;
  if (p.w_packed) {
    p.w_planes = p.w_packed;
    p.w_range = planes_trailer(p.w_packed, w_elems);
    return hipSuccess;
  }
  if (!dst) return hipErrorInvalidValue;                // the ABI layer never plans these kernels without a workspace
  p.w_planes = dst;
  p.w_range = planes_trailer(dst, w_elems);
  return launch_pack_filter(static_cast<const float*>(p.w), const_cast<void*>(dst), p.b_is_kn, p.Kgemm, p.k, (long long)w_elems,
                            stream);
}

size_t p3_pack_bytes(const Problem& p) {
  return tensor_planes_bytes(p.x_bytes >> 2) + (p.w_packed ? 0 : filter_planes_bytes(p.w_bytes >> 2));
}

// Worth it when the contraction is large against the one-off cost of measuring and cutting both operands (twelve
// bytes of memory traffic per element), the operands' shapes allow 16-byte plane chunks, and there are enough
// pixels and channels for the 128-pixel tiles.  Measured break-even: about 400 flops per operand element that the
// call has to cut (FullyConnected 256 x 4096 x 4096, 483 flops per element: 91 us here against 117 us on the fp32
// matrix cores inside a step of other layers, 84 against 103 launched back to back; 256 x 9216 x 4096 169 against
// 230 us).
bool p3_f32_applicable(const Problem& p) {
  if (knob_or(KNOB_F32_P3, 1) == 0) return false;
  if (p.chain_n > 0 || p.cg % 8 != 0 || p.c % 8 != 0) return false;
  if (p.b_is_kn && p.groups != 1) return false;
  if (p.r > 15 || p.s > 15) return false;               // the padding masks hold 16 taps per direction
  if (p.x_bytes > (1u << 30) || p.w_bytes > (1u << 30)) return false;
  const long long min_m = knob_or(KNOB_F32_P3_MIN_M, 256);
  if (p.M < min_m || p.kg < 64) return false;
  // a tile's fixed part (first slabs' latency, exchange, 64 KB of stores) is worth about eight slabs: with a
  // reduction of 256 the fp32 kernels are faster (measured: 1x1 256->1024 on 14x14 at batch 32, 72 against 44 us)
  if (min_m > 1 && p.Kgemm < 512) return false;
  const double flops = 2.0 * p.M * (double)p.kg * p.groups * p.Kgemm;
  // three launches (two packing kernels and the contraction) are worth ~15 us before any work is done
  if (min_m > 1 && flops < 2e9) return false;
  const double elems = (double)(p.x_bytes >> 2) + (p.w_packed ? 0.0 : (double)(p.w_bytes >> 2));   // what this call cuts
  return flops >= (double)knob_or(KNOB_F32_P3_RATIO, 400) * elems;
}

Plan plan_p3_f32(const Problem& p) {
  Plan pl;
  pl.kernel = KERNEL_P3;
  pl.bm = PBM;
  pl.bn = p.kg > 64 ? 128 : 64;
  if (knob_is_set(KNOB_F32_P3_BN)) pl.bn = knob(KNOB_F32_P3_BN) == 64 ? 64 : 128;
  pl.tile = pl.bn == 128 ? 0 : 1;
  pl.bk = PBK;
  pl.tiles_m = (p.M + PBM - 1) / PBM;
  pl.tiles_n = (p.kg + pl.bn - 1) / pl.bn;
  pl.slabs = p.r * p.s * ((p.cg + PBK - 1) / PBK);
  pl.split_k = 1;
  pl.slabs_per_split = pl.slabs;
  pl.pack_bytes = p3_pack_bytes(p);
  // Split the reduction when the tiles alone leave CUs idle: one workgroup per CU for the 128-channel tile, two
  // for the 64-channel one; among the factors that keep at least eight slabs per workgroup take the smallest that
  // fills 90 % of its last round, else the one that fills it best.
  const long long t = (long long)pl.tiles_m * pl.tiles_n * p.groups;
  const long long slots = pl.bn == 128 ? 256 : 512;
  if (t < slots && pl.slabs >= 16) {
    const int max_split = pl.slabs / 8 < 32 ? pl.slabs / 8 : 32;
    int best = 1;
    double best_u = 0.0;
    for (int sk = 1; sk <= max_split; ++sk) {
      const int sps = (pl.slabs + sk - 1) / sk;
      if ((pl.slabs + sps - 1) / sps != sk) continue;
      const long long blocks = t * sk;
      const double u = (double)blocks / (double)(((blocks + slots - 1) / slots) * slots);
      if (u > best_u + 1e-9) { best_u = u; best = sk; }
      if (u >= 0.9) { best = sk; break; }
    }
    if (knob_is_set(KNOB_F32_SPLIT)) {
      best = knob(KNOB_F32_SPLIT);
      if (best < 1) best = 1;
      if (best > pl.slabs) best = pl.slabs;
      if (best > 64) best = 64;
    }
    if (best > 1) {
      pl.slabs_per_split = (pl.slabs + best - 1) / best;
      pl.split_k = (pl.slabs + pl.slabs_per_split - 1) / pl.slabs_per_split;
    }
  }
  return pl;
}

hipError_t launch_p3_f32(const Problem& p_in, const Plan& plan, hipStream_t stream, const char** variant) {
  if (!p_in.planes) return hipErrorInvalidValue;        // the ABI layer never plans this kernel without a workspace (the input's planes)
  if (plan.split_k > 1 && !p_in.partial) return hipErrorInvalidValue;
  Problem p = p_in;
  p.split_k = plan.split_k;
  p.slabs_per_split = plan.slabs_per_split;
  const size_t x_elems = p.x_bytes >> 2, w_elems = p.w_bytes >> 2;
  unsigned short* xp = static_cast<unsigned short*>(const_cast<void*>(p.planes));
  unsigned short* wp = reinterpret_cast<unsigned short*>(reinterpret_cast<unsigned char*>(xp) + tensor_planes_bytes(x_elems));
  unsigned* x_trailer = planes_trailer(xp, x_elems);
  p.x_range = x_trailer;                                // word 0, written by the packing kernel
  p.x_range_n = 1;
  const long long xc8 = (long long)(x_elems / 8), wc8 = (long long)(w_elems / 8);
  long long bx = (xc8 + 255) / 256;
  if (bx > 8192) bx = 8192;
  if (bx < 1) bx = 1;
  hipError_t e;
  if (p.w_packed) {
    // ---- the weights' planes were made ahead of time: only the input is measured and cut
    p.w_planes = p.w_packed;
    p.w_range = planes_trailer(p.w_packed, w_elems);
    e = launch_ranges(static_cast<const float*>(p.x), (long long)x_elems, x_trailer + kRangeWords, nullptr, 0, nullptr, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(pack2_rows_kernel, dim3((unsigned)bx), dim3(256), 0, stream, static_cast<const float*>(p.x), xp, xc8,
                       (long long)x_elems, x_trailer);
  } else {
    // ---- both operands: one launch for their largest magnitudes, one that cuts them into planes
    p.w_planes = wp;
    unsigned* w_trailer = planes_trailer(wp, w_elems);
    p.w_range = w_trailer;
    e = launch_ranges(static_cast<const float*>(p.x), (long long)x_elems, x_trailer + kRangeWords,
                      static_cast<const float*>(p.w), (long long)w_elems, w_trailer + kRangeWords, stream);
    if (e != hipSuccess) return e;
    long long bw;
    int tn = 0;
    if (p.b_is_kn) {
      tn = (p.k + kPackTile - 1) / kPackTile;
      bw = (long long)((p.Kgemm + 63) / 64) * tn;
    } else {
      bw = (wc8 + 255) / 256;
      if (bw > 4096) bw = 4096;
      if (bw < 1) bw = 1;
    }
    hipLaunchKernelGGL(pack2_pair_kernel, dim3((unsigned)(bx + bw)), dim3(256), 0, stream, static_cast<const float*>(p.x), xp,
                       xc8, (long long)x_elems, (int)bx, x_trailer, static_cast<const float*>(p.w), wp, wc8,
                       (long long)w_elems, p.b_is_kn, p.Kgemm, p.k, tn, w_trailer);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  // ---- the contraction
  const bool padded = p.pad_t != 0 || p.pad_l != 0 || (p.oh - 1) * p.stride_h - p.pad_t + p.r > p.h ||
                      (p.ow - 1) * p.stride_w - p.pad_l + p.s > p.w_;
  const bool longk = plan.slabs_per_split > P3_FLUSH;
  static thread_local char name[64];
  snprintf(name, sizeof(name), "igemm_f32_p3_128x%d%s%s", plan.bn, padded ? "_pad" : "", longk ? "_longk" : "");
  *variant = name;
  if (plan.bn == 128) e = launch_p3_flags<2, 3>(p, plan, stream, padded, longk);
  else e = launch_p3_flags<1, 2>(p, plan, stream, padded, longk);
  if (e != hipSuccess) return e;
  if (plan.split_k > 1) e = launch_splitk_finish_f32(p, plan, stream);
  return e;
}

}  // namespace glowmi
