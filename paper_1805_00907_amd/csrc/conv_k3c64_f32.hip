// fp32 3x3 Convolution (stride 1) over 64 input channels on many pixels -- the first layer pair of a VGG
// stack, the 3x3 layers of a residual network's first stage -- on the fp16 matrix cores with every operand
// cut into two fp16 pieces and three piece products per fp32 product (f16_pieces.h).  One more kind
// of convolution with a strategy of its own (Section 5.3 of the paper); the arithmetic is the loop nest of
// Section 3.1 with the bias add and Relu stacked onto it (Section 5.2).
//
// With 64 channels in and 64 out the generic 128-pixel x 64-channel tile fetches every input element nine
// times (once per tap) for only 64 output channels each and is bound by the path from L2 into the CUs.  Here
//   - a workgroup owns a 16 x 16 block of output pixels x 64 output channels.  Its 18 x 18 x 64 input patch is
//     read from global memory ONCE (fp32, coalesced 32-byte pieces, zeros outside the image from the
//     range-checked loads), cut into pieces in registers and kept in LDS as two fp16 planes (83 KB); all
//     nine taps read their MFMA fragments from it at shifted addresses.  Per tile 83 KB of input are fetched
//     instead of nine times its planes, and no packing pass over the input is needed (only the pass that finds
//     its largest magnitude);
//   - the filter (64 x 576) is cut once per call by the packing kernel into two planes in the workspace
//     (147 KB, L2-resident) and streamed slab by slab (one tap x 32 channels, 8 KB) straight into a ring of
//     two LDS buffers;
//   - eight wavefronts: four pixel quarters (4 rows x 16 columns = two 32-pixel MFMA blocks) x two sets that
//     split every slab's 32 reduction indices, 64 x 64 outputs per wavefront; partial tiles exchanged through
//     LDS at the end;
//   - workgroups are persistent: the next tile's patch is fetched into registers while the current tile is
//     multiplied, so only cutting and writing it (about a tenth of a tile's MFMA time) is exposed; the next tile's
//     first two slabs are issued ahead of a tile's output stores, so that no slab load has to be waited for behind
//     them (loads and stores complete in order under one counter);
//   - a pixel's eight 16-byte chunks are stored at chunk ^ ((key / 2) % 8), key = 16 * patch row + patch column,
//     which spreads the two tile rows a fragment read touches over all bank groups whatever the tap.
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

constexpr int KT = 16;                         // tile side in output pixels
constexpr int KP = KT + 2;                     // patch side
constexpr int K_PATCH_PX = KP * KP;            // 324 pixels
constexpr int K_PIXB = 128;                    // bytes of a pixel's 64 channels in one plane
constexpr int K_APLANE = K_PATCH_PX * K_PIXB;  // 41472
constexpr int K_BROW = 64;                     // bytes of a filter row piece (32 reduction indices) in one plane
constexpr int K_BPLANE = 64 * K_BROW;          // 4096: 64 output channels
constexpr int K_BBUF = 2 * K_BPLANE;           // one slab
constexpr int K_NBUF = 2;
constexpr int K_STAGE = 2 * K_APLANE + K_NBUF * K_BBUF;
constexpr int K_LDS = K_STAGE + 32;            // + the eight wavefronts' largest magnitudes of the patch being written
constexpr int K_THREADS = 512;
constexpr int K_ITEMS = K_PATCH_PX * 8;        // (pixel, 8-channel chunk) pieces of a patch
constexpr int K_PASSES = (K_ITEMS + K_THREADS - 1) / K_THREADS;   // 6
constexpr int K_SLABS = 18;                    // 9 taps x 2 channel halves
static_assert(K_LDS <= 160 * 1024, "LDS of one CU");
static_assert(2 * K_APLANE >= 8 * 32 * 64 * 4, "exchange of the partial tiles fits the patch area");

template <bool ADD>
__global__ __launch_bounds__(K_THREADS, 2) void conv_k3c64_f32_kernel(const Problem p, int tiles_y, int tiles_x,
                                                                     int tiles_c, int total) {
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* bring = lds + 2 * K_APLANE;
  unsigned* maxw = reinterpret_cast<unsigned*>(lds + K_STAGE);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kgrp = wave >> 2;                           // which 16 of every slab's 32 reduction indices
  const int wm = wave & 3;                              // pixel quarter: tile rows 4wm .. 4wm + 3
  const int lrow = lane & 31, lhalf = lane >> 5;

  const float* __restrict__ X = static_cast<const float*>(p.x);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(X), 0, (int)p.x_bytes, 0x00020000);
  const unsigned wpb = p.w_bytes >> 1;                  // bytes of one filter plane
  const v4i rsrc_w = make_rsrc(p.w_planes, 2u * wpb);
  constexpr unsigned OOB = 0x80000000u;
  // The filter's scale exponent follows from its largest magnitude (the trailer of its planes).  The input is scaled
  // patch by patch: the workgroup takes the largest magnitude of the patch it is about to write (from the prefetch
  // registers), which costs no pass over the input.
  const unsigned w_max_bits = wave_max_words(p.w_range, 1);
  constexpr unsigned OOBX = 0xFFFFFF00u;                // beyond any fp32 tensor this library accepts

  // ---- tile decode: channel tile fastest (workgroups that share a patch run side by side), then x, y, image
  auto decode = [&](int t, int& img, int& ty, int& tx, int& ct) {
    ct = t % tiles_c;
    t /= tiles_c;
    tx = t % tiles_x;
    t /= tiles_x;
    ty = t % tiles_y;
    img = t / tiles_y;
  };

  // ---- patch: piece q = tid + 512 * pass is (pixel q / 8 of the patch, channels 8 * (q % 8) ..)
  v4f pre[K_PASSES][2];
  auto fetch_patch = [&](int t) {
    int img, ty, tx, ct;
    decode(t, img, ty, tx, ct);
#pragma unroll
    for (int q = 0; q < K_PASSES; ++q) {
      const int item = tid + q * K_THREADS;
      const int pp = item >> 3, c8 = item & 7;
      const int py = pp / KP, px = pp - py * KP;
      const int iy = ty * KT - p.pad_t + py, ix = tx * KT - p.pad_l + px;
      const bool ok = item < K_ITEMS && (unsigned)iy < (unsigned)p.h && (unsigned)ix < (unsigned)p.w_;
      const unsigned off = ok ? ((unsigned)((img * p.h + iy) * p.w_ + ix) * 64u + (unsigned)c8 * 8u) * 4u : OOBX;
      pre[q][0] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0));
      pre[q][1] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off == OOBX ? OOBX : off + 16u, 0, 0));
    }
  };
  auto commit_patch = [&](int se_x) {
#pragma unroll
    for (int q = 0; q < K_PASSES; ++q) {
      const int item = tid + q * K_THREADS;
      if (item < K_ITEMS) {
        const int pp = item >> 3, c8 = item & 7;
        const float v[8] = {pre[q][0][0], pre[q][0][1], pre[q][0][2], pre[q][0][3],
                            pre[q][1][0], pre[q][1][1], pre[q][1][2], pre[q][1][3]};
        v4u p1, p2;
        cut8(v, se_x, p1, p2);
        const int py = pp / KP;
        const int key = pp - 2 * py;                     // py * 16 + px: the pixel's index at the tile's own pitch
        unsigned char* dst = lds + pp * K_PIXB + ((c8 ^ ((key >> 1) & 7)) << 4);
        *reinterpret_cast<v4u*>(dst) = p1;
        *reinterpret_cast<v4u*>(dst + K_APLANE) = p2;
      }
    }
  };

  // ---- filter slab loads: 8 wavefront loads per slab (2 planes x 4 groups of 16 rows), one per wavefront.
  // Lane l: row l / 4 of the group, chunk position l % 4 holding chunk (l % 4) ^ ((row / 4) % 4) of the row
  // (the swizzle of igemm_f32_p3.hip).
  const int bch = (lane & 3) ^ ((lane >> 4) & 3);
  auto issue_b = [&](int ct, int slab, int buf) {
    const int tap = slab >> 1, half = slab & 1;
    const unsigned lbase = __builtin_amdgcn_readfirstlane(lds_offset_of(bring) + buf * K_BBUF);
    {
      const int plane = wave >> 2, rg = wave & 3;
      const int n = ct * 64 + rg * 16 + (lane >> 2);
      const bool ok = slab < K_SLABS && n < p.k;         // past the last slab: a zero fill, no memory traffic
      const unsigned off = ok ? 2u * ((unsigned)n * 576u + (unsigned)(tap * 64 + half * 32 + bch * 8)) + (unsigned)plane * wpb : OOB;
      load16_to_lds(rsrc_w, lbase + plane * K_BPLANE + rg * 16 * K_BROW, off);
    }
  };

  // ---- fragment addresses.  Input: MFMA block i of this wavefront is tile rows 4wm + 2i, + 1 (16 pixels each);
  // lane lrow is pixel (lrow / 16, lrow % 16) of the block.  Filter: row = output channel j * 32 + lrow.
  // The swizzle key is the pixel's index at the tile's own pitch (16), not at the patch's (18): the 32 lanes of a
  // fragment read are two tile rows of 16, i.e. 32 consecutive keys whatever the tap, and their addresses then
  // differ modulo 256 bytes within every 16 of them (keyed by the patch index, the second row's pixels fall on
  // the first row's banks: measured half the LDS read rate).
  int pp0[2], key0[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    pp0[i] = (4 * wm + 2 * i + (lrow >> 4)) * KP + (lrow & 15);
    key0[i] = (4 * wm + 2 * i) * KT + lrow;
  }
  const int b_pos = ((kgrp * 2 + lhalf) ^ ((lrow >> 2) & 3)) << 4;
  const int frag_b = lrow * K_BROW + b_pos;

  float* __restrict__ Y = static_cast<float*>(p.y);
  const __amdgpu_buffer_rsrc_t rsrc_y =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const float* addend = static_cast<const float*>(p.addend);   // may be the output itself
  const bool relu = p.act == 1;

  // Consecutive workgroup ids go round-robin to the 8 XCDs: give each XCD a contiguous run of tiles, so that the
  // channel tiles that share a patch (consecutive tile numbers) fetch it through the same L2.
  int t = (gridDim.x & 7) == 0 ? (int)((blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) : (int)blockIdx.x;
  if (t >= total) return;
  fetch_patch(t);
  // Vector-memory operations complete in order, stores included, and one counter covers them all: a slab load issued
  // behind a tile's 32 output stores cannot be waited for without waiting for the stores (measured: a fifth of the
  // kernel's time).  Without the add link the first two slabs of the NEXT tile are therefore issued before a tile's
  // stores (both slab buffers are free by then), every lane issues exactly 32 stores per tile (lanes outside the output
  // store out of the buffer's range), and the first two trips wait for "all but the operations issued after the slab":
  // the other slab, the 32 stores, the 12 loads of the next patch.  From the third trip on the wait is for everything,
  // and the stores have had the patch's conversion and two trips to drain.
  // (The first patch is waited for here, once: left to the compiler, its wait sits at the head of the tile loop and
  // there makes every later tile wait until all but eleven of the previous tile's stores have drained.)
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  constexpr bool EARLY = !ADD;
  constexpr int N_STORES = 32, N_PATCH = 2 * K_PASSES;
  static_assert(1 + N_STORES + N_PATCH <= 63, "vmcnt is six bits");
  bool first = true;
  for (; t < total; t += gridDim.x) {
    int img, ty, tx, ct;
    decode(t, img, ty, tx, ct);
    const unsigned share_max = wave_max_of(pre);        // every wavefront leaves the largest magnitude of its share
    if (lane == 0) maxw[wave] = share_max;
    __syncthreads();                                    // the previous tile's exchange has been read: the patch area is free
    const unsigned x_max_bits = max_of_eight(maxw);
    const int se_x = scale_exponent(x_max_bits);
    const ScaleBack sb = scale_back(x_max_bits, w_max_bits);
    commit_patch(se_x);
    const int t_next = t + gridDim.x;
    const bool prefetching = t_next < total;            // uniform
    if (!EARLY) {
      if (prefetching) fetch_patch(t_next);             // in flight during this tile's MFMAs
      issue_b(ct, 0, 0);
    } else {
      if (first) {
        issue_b(ct, 0, 0);
        issue_b(ct, 1, 1);
      }
      if (prefetching) fetch_patch(t_next);
    }
    // the tile's bias values now: a load in the epilogue would make the compiler wait there for everything issued
    // before it, the next tile's slabs included
    float bias_v[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int ch = ct * 64 + j * 32 + lrow;
      bias_v[j] = (ch < p.k && bias) ? bias[ch] : 0.f;
    }

    v16f acc[2][2], acc_lo[2][2];                       // the h1 h1' products; the cross terms (weight 2^-11)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          acc[i][j][e] = 0.f;
          acc_lo[i][j][e] = 0.f;
        }

    // ---- 18 slabs.  Trip s: slab s has landed (one slab in flight), barrier (also: the patch is written, everyone
    // is done with the other buffer), refill the other buffer with slab s + 1, multiply slab s.
#pragma unroll 2
    for (int s = 0; s < K_SLABS; ++s) {
      if (EARLY && s < 2) {
        // issued after slab s: (slab 1,) the previous tile's stores unless this is the first tile, the next patch
        if (s == 0) {
          if (first && prefetching) __builtin_amdgcn_s_waitcnt(vmcnt_imm(1 + N_PATCH));
          else if (first) __builtin_amdgcn_s_waitcnt(vmcnt_imm(1));
          else if (prefetching) __builtin_amdgcn_s_waitcnt(vmcnt_imm(1 + N_STORES + N_PATCH));
          else __builtin_amdgcn_s_waitcnt(vmcnt_imm(1 + N_STORES));
        } else {
          if (first && prefetching) __builtin_amdgcn_s_waitcnt(vmcnt_imm(N_PATCH));
          else if (first) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
          else if (prefetching) __builtin_amdgcn_s_waitcnt(vmcnt_imm(N_STORES + N_PATCH));
          else __builtin_amdgcn_s_waitcnt(vmcnt_imm(N_STORES));
        }
      } else {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      }
      __syncthreads();
      if (!EARLY || s > 0) issue_b(ct, s + 1, (s + 1) & 1);   // past the last slab: zero fills, no memory traffic
      const int tap = s >> 1, half = s & 1;
      const int tr = tap / 3, ts = tap - tr * 3;
      const int c8 = half * 4 + kgrp * 2 + lhalf;       // this lane's 16-byte chunk of the pixel
      const unsigned char* bb = bring + (s & 1) * K_BBUF + frag_b;
      v8h a[2][2], b[2][2];
      int a_off[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int pp = pp0[i] + tr * KP + ts;
        const int key = key0[i] + tr * KT + ts;
        a_off[i] = pp * K_PIXB + ((c8 ^ ((key >> 1) & 7)) << 4);
      }
#pragma unroll
      for (int o = 0; o < 2; ++o) {
        const int pa = o, pb = 1 - o;                    // the order the MFMAs use them in: cross terms first
#pragma unroll
        for (int i = 0; i < 2; ++i)
          a[pa][i] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(lds + pa * K_APLANE + a_off[i]));
#pragma unroll
        for (int j = 0; j < 2; ++j)
          b[pb][j] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(bb + pb * K_BPLANE + j * 32 * K_BROW));
      }
#pragma unroll
      for (int q = 0; q < 12; ++q) {
        const int tt = q / 4, i = (q / 2) % 2, j = q % 2;
        if (tt == 0) acc_lo[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], b[1][j], acc_lo[i][j], 0, 0, 0);
        else if (tt == 1) acc_lo[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[1][i], b[0][j], acc_lo[i][j], 0, 0, 0);
        else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], b[0][j], acc[i][j], 0, 0, 0);
      }
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));           // the zero fill past the last slab (and, conservatively, the prefetch)
    __syncthreads();                                    // everyone is done with the patch and the slab buffers
    if (EARLY && prefetching) {                         // the next tile's first two slabs, ahead of this tile's stores
      int n_img, n_ty, n_tx, n_ct;
      decode(t_next, n_img, n_ty, n_tx, n_ct);
      issue_b(n_ct, 0, 0);
      issue_b(n_ct, 1, 1);
    }
    first = false;

    // ---- exchange: the two wavefronts with partial sums of the same 64 pixels x 64 channels swap halves; the
    // kgrp-0 wavefront finishes block 0 (tile rows 4wm, 4wm + 1), the other block 1.
    v16f keep[2];
    {
      v4f* xch = reinterpret_cast<v4f*>(lds);
      const int mine = (wm * 2 + kgrp) * 8, theirs = (wm * 2 + (kgrp ^ 1)) * 8;
      auto exchange_as = [&](auto kg_tag) {
        constexpr int KG = decltype(kg_tag)::value;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          v16f snd;
#pragma unroll
          for (int e = 0; e < 16; ++e) {                 // the two accumulator sets joined
            keep[j][e] = __builtin_fmaf(acc_lo[KG][j][e], kLowPieceWeight, acc[KG][j][e]);
            snd[e] = __builtin_fmaf(acc_lo[1 - KG][j][e], kLowPieceWeight, acc[1 - KG][j][e]);
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
          for (int tq = 0; tq < 4; ++tq) keep[j][e4 * 4 + tq] = __builtin_ldexpf(keep[j][e4 * 4 + tq] + got[tq], sb.neg_se) + sb.poison;   // scaled back
        }
    }

    // ---- epilogue.  Register e of a lane is pixel (e/4)*8 + 4*lhalf + e%4 of the 32-pixel block, i.e. tile row
    // 4wm + 2kgrp + pixel / 16, column pixel % 16; channel j * 32 + lrow.
    const int oy0 = ty * KT + 4 * wm + 2 * kgrp, ox0 = tx * KT;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int ch = ct * 64 + j * 32 + lrow;
      const bool cok = ch < p.k;
      const float bv = bias_v[j];
      // the add link: a column's sixteen addend values first, all in flight together, then one wait the compiler can
      // see -- loaded one by one in front of their stores, each would be waited for together with the store before it
      float addv[16];
      if (ADD) {
        const __amdgpu_buffer_rsrc_t rsrc_add =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(addend), 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int px = (e >> 2) * 8 + lhalf * 4 + (e & 3);
          const int oy = oy0 + (px >> 4), ox = ox0 + (px & 15);
          const bool ok = cok && oy < p.oh && ox < p.ow;
          const unsigned off = ok ? ((unsigned)((img * p.oh + oy) * p.ow + ox) * (unsigned)p.k + (unsigned)ch) * 4u : OOBX;
          addv[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_add, off, 0, 0));
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int px = (e >> 2) * 8 + lhalf * 4 + (e & 3);
        const int oy = oy0 + (px >> 4), ox = ox0 + (px & 15);
        const bool ok = cok && oy < p.oh && ox < p.ow;
        if (ADD) {                                       // the same offsets as the addend's loads
          float v = keep[j][e] + bv + addv[e];
          if (relu) v = fmaxf(v, 0.f);
          const unsigned off = ok ? ((unsigned)((img * p.oh + oy) * p.ow + ox) * (unsigned)p.k + (unsigned)ch) * 4u : OOBX;
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), rsrc_y, off, 0, 0);
        } else if (EARLY) {                                     // always issued: the waits above count on it
          float v = keep[j][e] + bv;
          if (relu) v = fmaxf(v, 0.f);
          const unsigned off = ok ? ((unsigned)((img * p.oh + oy) * p.ow + ox) * (unsigned)p.k + (unsigned)ch) * 4u : OOBX;
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), rsrc_y, off, 0, 0);
        } else if (ok) {
          const size_t o = ((size_t)(img * p.oh + oy) * p.ow + ox) * p.k + ch;
          float v = keep[j][e] + bv;
          if (ADD) v += addend[o];
          if (relu) v = fmaxf(v, 0.f);
          Y[o] = v;
        }
      }
    }
  }
}

template <bool ADD>
hipError_t launch_k3_variant(const Problem& p, hipStream_t stream) {
  auto kern = conv_k3c64_f32_kernel<ADD>;
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, K_LDS);
  if (attr_status != hipSuccess) return attr_status;
  const int num_cu = num_compute_units();
  if (num_cu < 1) return hipErrorInvalidDevice;
  const int tiles_y = (p.oh + KT - 1) / KT, tiles_x = (p.ow + KT - 1) / KT, tiles_c = (p.k + 63) / 64;
  const long long total = (long long)p.n * tiles_y * tiles_x * tiles_c;
  const long long grid = total < num_cu ? total : num_cu;   // one persistent workgroup per CU
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(K_THREADS), K_LDS, stream, p, tiles_y, tiles_x, tiles_c, (int)total);
  return hipGetLastError();
}

}  // namespace

bool k3c64_f32_applicable(const Problem& p) {
  if (knob_or(KNOB_F32_K3C64, 1) == 0) return false;
  if (p.b_is_kn || p.chain_n > 0 || p.groups != 1 || p.c != 64 || p.r != 3 || p.s != 3) return false;
  if (p.stride_h != 1 || p.stride_w != 1) return false;
  if (p.x_bytes > 0xF0000000u || (long long)p.M * p.k * 4 > 0xF0000000LL) return false;     // 32-bit byte offsets
  const long long tiles = (long long)p.n * ((p.oh + KT - 1) / KT) * ((p.ow + KT - 1) / KT) * ((p.k + 63) / 64);
  if (tiles >= (1LL << 30)) return false;
  // enough tiles to give every CU a few (a tile's patch is fetched while the previous one is multiplied)
  return tiles >= knob_or(KNOB_F32_K3C64_MIN_TILES, 512);
}

size_t k3c64_f32_pack_bytes(const Problem& p) { return p.w_packed ? 0 : filter_planes_bytes(p.w_bytes >> 2); }

hipError_t launch_k3c64_f32(const Problem& p_in, hipStream_t stream, const char** variant) {
  Problem p = p_in;
  hipError_t e = stage_filter_planes(p, p.planes, stream);
  if (e != hipSuccess) return e;
  *variant = p.addend ? "conv_k3c64_f32_f16x3_add" : "conv_k3c64_f32_f16x3";
  return p.addend ? launch_k3_variant<true>(p, stream) : launch_k3_variant<false>(p, stream);
}

}  // namespace glowmi
