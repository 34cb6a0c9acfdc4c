// fp32 3x3 Convolution (stride 1) with 64 or more input channels and more than 64 output channels on maps that
// tile well into 16 x 16 pixel blocks -- the body of a VGG stack -- on the fp16 matrix cores with every operand
// cut into two fp16 pieces and three piece products per fp32 product (f16_pieces.h).  The arithmetic is
// the loop nest of Section 3.1 of the paper with the bias add and Relu stacked onto it (Section 5.2); this is one
// more kind of convolution with a strategy of its own (Section 5.3).
//
// The generic kernel over planes (igemm_f32_p3.hip) fetches every input element nine times (once per tap) as
// planes that a packing pass had to write first, and measured a third of its time is the fill path.  Here
//   - a workgroup owns a 16 x 16 block of output pixels x 128 output channels and walks the input channels in
//     chunks of 32.  The chunk's 18 x 18 x 32 input patch is read from the fp32 input ONCE (coalesced 32-byte
//     pieces, zeros outside the image from the range-checked loads), cut into pieces in registers and kept in
//     LDS as two fp16 planes (45 KB); all nine taps read their MFMA fragments from it at shifted addresses.
//     No packing pass over the input (only the pass that finds its largest magnitude), and a ninth of the
//     input traffic;
//   - the filter is cut once per call by the packing kernel into two planes in the workspace and streamed
//     slab by slab (one tap x 32 channels x 128 output channels, 16 KB) straight into a ring of two LDS
//     buffers;
//   - eight wavefronts = four pixel quarters (4 rows x 16 columns: two 32-pixel MFMA blocks) x two channel halves,
//     64 x 64 outputs each over the whole slab: 24 MFMAs per wavefront between two barriers, no exchange of
//     partial tiles;
//   - workgroups are persistent; the next chunk's (or the next tile's first) patch is fetched into registers
//     while the current chunk is multiplied, so only cutting and writing it is exposed;
//   - patch rows are kept TW + 4 pixels apart and a pixel's four 16-byte chunks are stored at
//     chunk ^ ((key / 4) % 4), key = TW * patch row + patch column, which spreads the tile rows a fragment read
//     touches over all bank groups whatever the tap.
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

constexpr int GT = 16;                         // tile height in output pixels
constexpr int G_CH = 32;                       // input channels per chunk = reduction indices per slab
constexpr int G_PIXB = 2 * G_CH;               // bytes of a pixel's chunk in one plane
constexpr int G_BROW = 2 * G_CH;               // bytes of a filter row piece in one plane
constexpr int G_NBUF = 2;
constexpr int G_THREADS = 512;
constexpr int G_DUMMY = 1024;                  // landing area of the loads issued only to keep the counts equal

// Tile shapes: TW output columns x 16 rows, BN output channels.  512 threads = eight wavefronts of 64 pixels x 64
// channels each: (16 x 16) x 128 is four pixel quarters x two channel halves, (16 x 32) x 64 eight pixel eighths.
template <int TW, int BN>
struct K3 {
  static_assert((TW == 16 && BN == 128) || (TW == 32 && BN == 64), "tile shapes");
  static constexpr int PW = TW + 4;                          // patch row pitch in pixels: TW + 2 used (see the swizzle below)
  static constexpr int PATCH_PX = (GT + 2) * PW;
  static constexpr int APLANE = PATCH_PX * G_PIXB;
  static constexpr int BPLANE = BN * G_BROW;
  static constexpr int BBUF = 2 * BPLANE;                    // one slab
  static constexpr int STAGE = 2 * APLANE + G_NBUF * BBUF + G_DUMMY;
  static constexpr int LDS = STAGE + 32;                     // + the eight wavefronts' largest magnitudes of the patch being written
  static constexpr int ITEMS = PATCH_PX * (G_CH / 8);        // (pixel, 8-channel piece) items of a patch chunk
  static constexpr int PASSES = (ITEMS + G_THREADS - 1) / G_THREADS;
  static constexpr int PREF = 2 * PASSES;                    // prefetch loads per thread
  static constexpr int WLOADS = 2 * BN / 16;                 // wavefront loads per filter slab (16 rows each)
  static constexpr int LPW = (WLOADS + 7) / 8;               // per wavefront (the last ones may be zero fills into the dummy area)
  static constexpr int WAVES_N = BN / 64;
  static_assert(LDS <= 160 * 1024, "LDS of one CU");
};

template <bool ADD, int TW, int BN>
__global__ __launch_bounds__(G_THREADS, 2) void conv_k3_f32_kernel(const Problem p, int tiles_y, int tiles_x,
                                                                  int tiles_c, int total) {
  using T = K3<TW, BN>;
  constexpr int GP = T::PW, G_APLANE = T::APLANE, G_BPLANE = T::BPLANE, G_BBUF = T::BBUF, G_BN = BN;
  constexpr int G_ITEMS = T::ITEMS, G_PASSES = T::PASSES, G_PREF = T::PREF;
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* bring = lds + 2 * G_APLANE;
  unsigned* maxw = reinterpret_cast<unsigned*>(lds + T::STAGE);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave % T::WAVES_N;                     // which 64 of the tile's output channels
  const int wm = wave / T::WAVES_N;                     // which 64 of the tile's pixels (row-major inside the tile)
  const int lrow = lane & 31, lhalf = lane >> 5;

  const float* __restrict__ X = static_cast<const float*>(p.x);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(X), 0, (int)p.x_bytes, 0x00020000);
  const unsigned wpb = p.w_bytes >> 1;                  // bytes of one filter plane
  const v4i rsrc_w = make_rsrc(p.w_planes, 2u * wpb);
  constexpr unsigned OOB = 0x80000000u;
  // The filter's scale exponent follows from its largest magnitude (the trailer of its planes).  The input is scaled
  // patch by patch: the workgroup takes the largest magnitude of the patch chunk it is about to write (from the
  // prefetch registers), which costs no pass over the input; within a tile the exponent only ever goes down, and
  // when it does the accumulators are scaled along (exact: a power of two).
  const unsigned w_max_bits = wave_max_words(p.w_range, 1);
  const int se_w = scale_exponent(w_max_bits);
  constexpr unsigned OOBX = 0xFFFFFF00u;                // beyond any fp32 tensor this library accepts

  const int chunks = p.c / G_CH;                        // p.c % 32 == 0 on this kernel
  const int slabs = 9 * chunks;

  // ---- tile decode: channel tile fastest (workgroups that share a patch run side by side), then x, y, image
  auto decode = [&](int t, int& img, int& ty, int& tx, int& ct) {
    ct = t % tiles_c;
    t /= tiles_c;
    tx = t % tiles_x;
    t /= tiles_x;
    ty = t % tiles_y;
    img = t / tiles_y;
  };

  // ---- patch chunk: item q = tid + 512 * pass is (pixel q / 4 of the patch, channels 8 * (q % 4) .. of the chunk)
  v4f pre[G_PASSES][2];
  auto fetch_patch = [&](int t, int chunk) {
    int img, ty, tx, ct;
    decode(t, img, ty, tx, ct);
#pragma unroll
    for (int q = 0; q < G_PASSES; ++q) {
      const int item = tid + q * G_THREADS;
      const int pp = item >> 2, c8 = item & 3;
      const int py = pp / GP, px = pp - py * GP;
      const int iy = ty * GT - p.pad_t + py, ix = tx * TW - p.pad_l + px;
      const bool ok = item < G_ITEMS && px < TW + 2 && (unsigned)iy < (unsigned)p.h && (unsigned)ix < (unsigned)p.w_;
      const unsigned off =
          ok ? ((unsigned)((img * p.h + iy) * p.w_ + ix) * (unsigned)p.c + (unsigned)(chunk * G_CH + c8 * 8)) * 4u : OOBX;
      pre[q][0] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0));
      pre[q][1] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off == OOBX ? OOBX : off + 16u, 0, 0));
    }
  };
  auto commit_patch = [&](int se_x) {
#pragma unroll
    for (int q = 0; q < G_PASSES; ++q) {
      const int item = tid + q * G_THREADS;
      if (item < G_ITEMS) {
        const int pp = item >> 2, c8 = item & 3;
        const float v[8] = {pre[q][0][0], pre[q][0][1], pre[q][0][2], pre[q][0][3],
                            pre[q][1][0], pre[q][1][1], pre[q][1][2], pre[q][1][3]};
        v4u p1, p2;
        cut8(v, se_x, p1, p2);
        const int key = pp - 4 * (pp / GP);               // TW * patch row + patch column
        unsigned char* dst = lds + pp * G_PIXB + ((c8 ^ ((key >> 2) & 3)) << 4);
        *reinterpret_cast<v4u*>(dst) = p1;
        *reinterpret_cast<v4u*>(dst + G_APLANE) = p2;
      }
    }
  };

  // ---- filter slab loads: 2 planes x BN / 16 groups of 16 rows per slab; wavefront w issues numbers w, w + 8, ..
  // (LPW of them; a number past the last is a zero fill into the dummy area, so that every wavefront has the same
  // number of loads outstanding).  Lane l: row l / 4 of the group, chunk position l % 4 holding chunk
  // (l % 4) ^ ((row / 4) % 4) of the row.
  const int bch = (lane & 3) ^ ((lane >> 4) & 3);
  auto issue_b = [&](int ct, int slab, int buf) {
    const int chunk = slab / 9, tap = slab - chunk * 9;
    const unsigned lbase = __builtin_amdgcn_readfirstlane(lds_offset_of(bring) + buf * G_BBUF);
    const unsigned k_off = (unsigned)(tap * p.c + chunk * G_CH + bch * 8);
#pragma unroll
    for (int u = 0; u < T::LPW; ++u) {
      const int j = wave + 8 * u;                        // load number: plane j / (BN / 16), row group j % (BN / 16)
      const int plane = j / (BN / 16), rg = j % (BN / 16);
      const int n = ct * G_BN + rg * 16 + (lane >> 2);
      const bool real = j < T::WLOADS;
      const bool ok = real && slab < slabs && n < p.k;   // past the last slab: zero fills, no memory traffic
      const unsigned off = ok ? 2u * ((unsigned)n * (unsigned)p.Kgemm + k_off) + (unsigned)plane * wpb : OOB;
      const unsigned dst = real ? lbase + plane * G_BPLANE + rg * 16 * G_BROW
                                : __builtin_amdgcn_readfirstlane(lds_offset_of(bring) + G_NBUF * G_BBUF);
      load16_to_lds(rsrc_w, dst, off);
    }
  };

  // ---- fragment addresses.  Input: MFMA block i of this wavefront holds tile pixels 64wm + 32i .. + 31 in row-major
  // order (TW = 16: two rows of 16; TW = 32: one row); lane lrow is the lrow-th of them.  Filter: row = output
  // channel wn * 64 + j * 32 + lrow.
  // Swizzle: a pixel's four 16-byte chunks sit at chunk ^ ((key / 4) % 4) with key = TW * patch row + patch column,
  // the pixel's index at the TILE's pitch, and patch rows are TW + 4 pixels apart.  The 32 lanes of a fragment read
  // are 32 consecutive tile pixels shifted by the tap, i.e. 32 consecutive keys, and address / 16 modulo 16 is then
  // key modulo 16 (the pitch's extra 4 pixels = 16 chunks drop out): no two of 16 consecutive lanes share a bank
  // group.  (At the natural pitch TW + 2 with the patch index as key the second tile row of a read falls on the
  // first row's banks: measured half the LDS read rate.)
  int pp0[2], key0[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int tp = 64 * wm + 32 * i + lrow;
    pp0[i] = (tp / TW) * GP + tp % TW;
    key0[i] = tp;
  }
  const int b_row = (wn * 64 + lrow) * G_BROW;
  const int b_sw = (lrow >> 2) & 3;

  float* __restrict__ Y = static_cast<float*>(p.y);
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const float* addend = static_cast<const float*>(p.addend);   // may be the output itself
  const bool relu = p.act == 1;

  // Consecutive workgroup ids go round-robin to the 8 XCDs: give each XCD a contiguous run of tiles, so that the
  // channel tiles that share a patch (consecutive tile numbers) fetch it through the same L2.
  int t = (gridDim.x & 7) == 0 ? (int)((blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) : (int)blockIdx.x;
  if (t >= total) return;
  fetch_patch(t, 0);
  for (; t < total; t += gridDim.x) {
    int img, ty, tx, ct;
    decode(t, img, ty, tx, ct);
    const int t_next = t + gridDim.x;
    __syncthreads();                                    // everyone is done with the previous tile's last slab buffer
    issue_b(ct, 0, 0);
    // The tile's bias values now, not in the epilogue: there every store sits in a branch of its own, and the compiler
    // would wait for all memory operations in front of each store's bias add, i.e. for the store before it.
    float bias_v[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int ch = ct * G_BN + wn * 64 + j * 32 + lrow;
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

    int s = 0;
    int se_x = 0;
    bool finite = w_max_bits < 0x7f800000u;
    for (int chunk = 0; chunk < chunks; ++chunk) {
      // ---- the chunk's patch: its largest magnitude (every wavefront leaves that of its share), everyone is done
      // with the previous patch, scale, write it, publish it (the barrier of the first trip below), and start
      // fetching the next: the next chunk of this tile or chunk 0 of the next tile
      const unsigned share_max = wave_max_of(pre);
      if (lane == 0) maxw[wave] = share_max;
      __syncthreads();
      {
        const unsigned m = max_of_eight(maxw);
        finite = finite && m < 0x7f800000u;
        const int need = scale_exponent(m);
        if (chunk == 0) {
          se_x = need;
        } else if (need < se_x) {                         // uniform, rare: larger values than any chunk before
          const int d = need - se_x;
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int e = 0; e < 16; ++e) {
                acc[i][j][e] = __builtin_ldexpf(acc[i][j][e], d);
                acc_lo[i][j][e] = __builtin_ldexpf(acc_lo[i][j][e], d);
              }
          se_x = need;
        }
      }
      commit_patch(se_x);
      const bool fetching = chunk + 1 < chunks || t_next < total;     // uniform
      if (chunk + 1 < chunks) fetch_patch(t, chunk + 1);
      else if (t_next < total) fetch_patch(t_next, 0);
      // ---- nine taps.  Trip: slab s has landed (the prefetch issued after it may still be in flight on the first
      // trip of a chunk; later trips wait for everything, by then about a slab's time has passed), barrier,
      // refill the other buffer with slab s + 1, multiply slab s.
#pragma unroll
      for (int tap = 0; tap < 9; ++tap, ++s) {
        if (tap == 0 && fetching) __builtin_amdgcn_s_waitcnt(vmcnt_imm(G_PREF));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __syncthreads();
        issue_b(ct, s + 1, (s + 1) & 1);
        const int tr = tap / 3, ts = tap - tr * 3;                     // compile-time
        const unsigned char* bb = bring + (s & 1) * G_BBUF + b_row;
        int a_base[2], a_key[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          a_base[i] = pp0[i] + tr * GP + ts;
          a_key[i] = key0[i] + tr * TW + ts;
        }
#pragma unroll
        for (int k16 = 0; k16 < 2; ++k16) {
          const int c8 = k16 * 2 + lhalf;                              // this lane's 16-byte chunk of the pixel / filter row
          v8h a[2][2], b[2][2];
          int a_off[2];
#pragma unroll
          for (int i = 0; i < 2; ++i) a_off[i] = a_base[i] * G_PIXB + ((c8 ^ ((a_key[i] >> 2) & 3)) << 4);
          const int b_off = (c8 ^ b_sw) << 4;
#pragma unroll
          for (int o = 0; o < 2; ++o) {
            const int pa = o, pb = 1 - o;                                // the order the MFMAs use them in: cross terms first
#pragma unroll
            for (int i = 0; i < 2; ++i)
              a[pa][i] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(lds + pa * G_APLANE + a_off[i]));
#pragma unroll
            for (int j = 0; j < 2; ++j)
              b[pb][j] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(bb + pb * G_BPLANE + j * 32 * G_BROW + b_off));
          }
#pragma unroll
          for (int q = 0; q < 12; ++q) {
            const int tt = q / 4, i = (q / 2) % 2, j = q % 2;
            if (tt == 0) acc_lo[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], b[1][j], acc_lo[i][j], 0, 0, 0);
            else if (tt == 1) acc_lo[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[1][i], b[0][j], acc_lo[i][j], 0, 0, 0);
            else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], b[0][j], acc[i][j], 0, 0, 0);
          }
        }
      }
    }

    // ---- epilogue.  Register e of a lane is pixel (e/4)*8 + 4*lhalf + e%4 of the 32-pixel block, i.e. tile pixel
    // 64wm + 32i + that; channel wn * 64 + j * 32 + lrow.
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));           // nothing is in flight any more; the compiler cannot see it
    const ScaleBack sb = scale_back_of(se_x, se_w, finite);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int ch = ct * G_BN + wn * 64 + j * 32 + lrow;
      const bool cok = ch < p.k;
      const float bv = bias_v[j];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int tp = 64 * wm + 32 * i + (e >> 2) * 8 + lhalf * 4 + (e & 3);
          const int oy = ty * GT + tp / TW, ox = tx * TW + tp % TW;
          if (cok && oy < p.oh && ox < p.ow) {
            const size_t o = ((size_t)(img * p.oh + oy) * p.ow + ox) * p.k + ch;
            float v = join_sets(acc[i][j][e], acc_lo[i][j][e], sb) + bv;
            if (ADD) v += addend[o];
            if (relu) v = fmaxf(v, 0.f);
            Y[o] = v;
          }
        }
      }
    }
  }
}

template <bool ADD, int TW, int BN>
hipError_t launch_k3g_variant(const Problem& p, hipStream_t stream) {
  using T = K3<TW, BN>;
  auto kern = conv_k3_f32_kernel<ADD, TW, BN>;
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS);
  if (attr_status != hipSuccess) return attr_status;
  const int num_cu = num_compute_units();
  if (num_cu < 1) return hipErrorInvalidDevice;
  const int tiles_y = (p.oh + GT - 1) / GT, tiles_x = (p.ow + TW - 1) / TW, tiles_c = (p.k + BN - 1) / BN;
  const long long total = (long long)p.n * tiles_y * tiles_x * tiles_c;
  const long long grid = total < num_cu ? total : num_cu;   // one persistent workgroup per CU
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(G_THREADS), T::LDS, stream, p, tiles_y, tiles_x, tiles_c, (int)total);
  return hipGetLastError();
}

// Few output channels take the wide pixel tile with 64 channels, the rest 16 x 16 pixels x 128 channels.
bool k3_wide_tile(const Problem& p) { return p.k <= 64; }

}  // namespace

bool k3_f32_applicable(const Problem& p) {
  if (knob_or(KNOB_F32_K3, 1) == 0) return false;
  if (p.b_is_kn || p.chain_n > 0 || p.groups != 1 || p.r != 3 || p.s != 3) return false;
  if (p.stride_h != 1 || p.stride_w != 1) return false;
  if (p.c < 64 || p.c % G_CH != 0) return false;
  if (p.x_bytes > 0xF0000000u || p.w_bytes > (1u << 30) || (long long)p.M * p.k * 4 > 0xF0000000LL) return false;   // 32-bit byte offsets
  const int tw = k3_wide_tile(p) ? 32 : 16, bn = k3_wide_tile(p) ? 64 : 128;
  const long long ty = (p.oh + GT - 1) / GT, tx = (p.ow + tw - 1) / tw, tc = (p.k + bn - 1) / bn;
  const long long tiles = (long long)p.n * ty * tx * tc;
  if (tiles >= (1LL << 30)) return false;
  if (knob_or(KNOB_F32_K3_ANY, 0) != 0) return true;    // tests: any size
  // more than 64 output channels: the kernel whose tile shape follows the map; worth it when most of what the
  // machine multiplies is real output (a 14 x 14 map at batch 16 gives 64 tiles for 256 CUs and stays on the
  // generic kernel over planes)
  if (!k3_wide_tile(p) && knob_or(KNOB_F32_K3V, 1) != 0) return k3v_f32_efficiency(p) >= 0.6;
  // the tiles must be mostly full (a 28 x 28 or 56 x 56 map fills 77 % of its 16 x 16 blocks, which still beats the
  // generic kernel: 512 -> 512 on 28 x 28 at batch 16 is 256 tiles = one round here, 361 -> 329 us; a 14 x 14 map at
  // batch 16 has only 64 tiles, 105 -> 252 us, and stays there), and there must be a tile for every CU
  const double fill = (double)p.oh * p.ow / (double)(ty * tx * GT * tw) * ((double)p.k / (double)(tc * bn));
  return fill >= 0.75 && tiles >= 256;
}

size_t k3_f32_pack_bytes(const Problem& p) { return p.w_packed ? 0 : filter_planes_bytes(p.w_bytes >> 2); }

hipError_t launch_k3_f32(const Problem& p_in, hipStream_t stream, const char** variant) {
  Problem p = p_in;
  hipError_t e = stage_filter_planes(p, p.planes, stream);
  if (e != hipSuccess) return e;
  if (!k3_wide_tile(p) && knob_or(KNOB_F32_K3V, 1) != 0 && !k3v_f32_prefers_fixed_tile(p)) return launch_k3v_f32(p, stream, variant);
  if (k3_wide_tile(p)) {
    *variant = p.addend ? "conv_k3_f32_f16x3_16x32x64_add" : "conv_k3_f32_f16x3_16x32x64";
    return p.addend ? launch_k3g_variant<true, 32, 64>(p, stream) : launch_k3g_variant<false, 32, 64>(p, stream);
  }
  *variant = p.addend ? "conv_k3_f32_f16x3_add" : "conv_k3_f32_f16x3";
  return p.addend ? launch_k3g_variant<true, 16, 128>(p, stream) : launch_k3g_variant<false, 16, 128>(p, stream);
}

}  // namespace glowmi
