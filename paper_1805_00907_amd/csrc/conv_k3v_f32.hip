// fp32 3x3 Convolution (stride 1) with 64 or more input channels and more than 64 output channels -- the body of a
// VGG stack -- on the fp16 matrix cores with every operand cut into two fp16 pieces and three piece products per
// fp32 product (f16_pieces.h), with a pixel tile whose SHAPE IS CHOSEN PER LAYER.  The arithmetic is
// the loop nest of Section 3.1 of the paper with the bias add and Relu stacked onto it (Section 5.2); Section 5.3
// gives every kind of convolution a tile size of its own, chosen from what the hardware holds.
//
// Why the shape matters.  A workgroup multiplies a block of output pixels x 128 output channels and runs alone on
// its CU, so a layer costs (tiles per CU, rounded up) x (time of a tile).  A fixed 16 x 16 block wastes a quarter
// of the machine on the maps of such a stack: 28 x 28 and 56 x 56 fill 77 % of their 16 x 16 blocks, and the
// 784 blocks of 16 images of 112 x 112 are 3.06 rounds on 256 CUs, i.e. four.  Here a tile is th x tw pixels with
// th * tw <= 32 * NB, NB = 5..8 MFMA row blocks of 32 pixels, and the time of a tile is proportional to NB: 7 x 28
// pixels (NB = 7) cover a 28 x 28 map exactly in 256 tiles of 7/8 the work, 8 x 28 a 56 x 56 map and a
// 112 x 112 map (the latter in 3.5 rounds of 7/8 tiles).  The host picks the shape that minimises rounds x NB.
//
// What makes NB free to choose: the tile's NB pixel blocks x 4 channel columns of 32 are dealt to the eight
// wavefronts as four squares of 2 x 2 blocks over pixel blocks 0-3 (wavefronts 0-3) and four strips of
// (NB - 4) x 1 blocks over the rest (wavefronts 4-7, one channel column each).  Wavefronts w and w + 4 share a SIMD,
// so every SIMD carries NB block products per 16 reduction indices whatever NB is, although its two wavefronts
// carry unequal parts.  No partial tiles to exchange; per 16 reduction indices the squares read 4 x 2 fragments
// for 12 MFMAs and the strips (NB - 3) x 2 for (NB - 4) x 3.
//
// Otherwise as the fixed-tile kernel (conv_k3_f32.hip): the input is walked in chunks of 32 channels whose
// (th + 2) x (tw + 2) patch is read ONCE from the fp32 input, cut in registers and kept in LDS as two fp16
// planes, all nine taps reading their fragments from it at shifted addresses; the filter's planes (cut once per
// call, or ahead of time by the caller) are streamed slab by slab into a ring of two LDS buffers; workgroups are
// persistent and fetch the next patch into registers while the current chunk is multiplied.
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

constexpr int V_CH = 32;                       // input channels per chunk = reduction indices per slab
constexpr int V_PIXB = 2 * V_CH;               // bytes of a pixel's chunk in one plane
constexpr int V_BROW = 2 * V_CH;               // bytes of a filter row piece in one plane
constexpr int V_BN = 128;                      // output channels per tile
constexpr int V_THREADS = 512;
constexpr int V_MAXPX = 360;                   // largest patch (th + 2) * (tw + 4): rows are kept two pixels apart, see below
constexpr int V_MAXTW = 64;
constexpr int V_APLANE = V_MAXPX * V_PIXB;
constexpr int V_BPLANE = V_BN * V_BROW;
constexpr int V_BBUF = 2 * V_BPLANE;           // one slab: a tap x 32 channels x 128 output channels x 2 planes
constexpr int V_STAGE = 2 * V_APLANE + 2 * V_BBUF;
constexpr int V_PASSES = (V_MAXPX * (V_CH / 8) + V_THREADS - 1) / V_THREADS;
constexpr int V_PREF = 2 * V_PASSES;           // prefetch loads per thread
constexpr int V_LPW = 2 * V_BN / 16 / 8;       // filter loads per wavefront and slab (16 rows each)
static_assert(V_LPW * 8 * 16 == 2 * V_BN, "filter loads divide over the wavefronts");

constexpr int V_LDS = V_STAGE + 32;            // + the eight wavefronts' largest magnitudes of the patch being written
static_assert(V_LDS <= 160 * 1024, "LDS of one CU");

template <bool ADD, int NB>
__global__ __launch_bounds__(V_THREADS, 2) void conv_k3v_f32_kernel(const Problem p, int th, int tw, int tiles_y,
                                                                   int tiles_x, int tiles_c, int total) {
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* bring = lds + 2 * V_APLANE;
  unsigned* maxw = reinterpret_cast<unsigned*>(lds + V_STAGE);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

  // Patch rows have a pitch of tw + 4 pixels (tw + 2 used), and a pixel's four 16-byte chunks are stored at
  // chunk ^ ((y * tw + x) / 4 % 4) for patch row y, column x.  A fragment read takes 16 lanes at a time: 16
  // consecutive pixels of the th x tw tile in row-major order, shifted by the tap, i.e. runs of consecutive
  // pixels from consecutive patch rows.  LDS serves 16 such 16-byte reads per cycle when their addresses
  // differ modulo 256 bytes; with this pitch and swizzle address / 16 modulo 16 is (y * tw + x) mod 16 (the
  // pitch - tw = 4 pixels = 16 chunks drop out), which runs on without a break from one tile row to the next
  // whatever tw is.  (With the natural pitch tw + 2 and a swizzle by the linear pixel index a 14-pixel row
  // measured half the LDS read rate.)
  const int pw = tw + 4;
  const int patch_px = (th + 2) * pw;
  const int tile_px = th * tw;
  const float inv_tw = 1.0f / (float)tw, inv_pw = 1.0f / (float)pw;
  // n / d for the small non-negative n of this kernel (below 512, d <= 66): (n + 0.5) / d is at least 0.5 / d away
  // from every integer, far more than the rounding of the reciprocal and the product
  auto div_small = [](int n, float inv) { return (int)(((float)n + 0.5f) * inv); };

  const int chunks = p.c / V_CH;                        // p.c % 32 == 0 on this kernel
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

  // ---- patch chunk: item q = tid + 512 * pass is (pixel q / 4 of the patch, channels 8 * (q % 4) .. of the chunk);
  // the pixel's place in the patch is the same for every tile, so it is taken apart once
  int pyx[V_PASSES];
#pragma unroll
  for (int q = 0; q < V_PASSES; ++q) {
    const int pp = (tid + q * V_THREADS) >> 2;
    const int py = div_small(pp, inv_pw);
    pyx[q] = (pp < patch_px && pp - py * pw < tw + 2) ? (py << 16) | (pp - py * pw) : -1;   // the pitch's last two columns stay empty
  }
  v4f pre[V_PASSES][2];
  auto fetch_patch = [&](int t, int chunk) {
    int img, ty, tx, ct;
    decode(t, img, ty, tx, ct);
#pragma unroll
    for (int q = 0; q < V_PASSES; ++q) {
      const int c8 = (tid + q * V_THREADS) & 3;
      const int iy = ty * th - p.pad_t + (pyx[q] >> 16), ix = tx * tw - p.pad_l + (pyx[q] & 0xffff);
      const bool ok = pyx[q] >= 0 && (unsigned)iy < (unsigned)p.h && (unsigned)ix < (unsigned)p.w_;
      const unsigned off =
          ok ? ((unsigned)((img * p.h + iy) * p.w_ + ix) * (unsigned)p.c + (unsigned)(chunk * V_CH + c8 * 8)) * 4u : OOBX;
      pre[q][0] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0));
      pre[q][1] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off == OOBX ? OOBX : off + 16u, 0, 0));
    }
  };
  auto commit_patch = [&](int se_x) {
#pragma unroll
    for (int q = 0; q < V_PASSES; ++q) {
      if (pyx[q] >= 0) {
        const int item = tid + q * V_THREADS;
        const int pp = item >> 2, c8 = item & 3;
        const float v[8] = {pre[q][0][0], pre[q][0][1], pre[q][0][2], pre[q][0][3],
                            pre[q][1][0], pre[q][1][1], pre[q][1][2], pre[q][1][3]};
        v4u p1, p2;
        cut8(v, se_x, p1, p2);
        const int key = (pyx[q] >> 16) * tw + (pyx[q] & 0xffff);
        unsigned char* dst = lds + pp * V_PIXB + ((c8 ^ ((key >> 2) & 3)) << 4);
        *reinterpret_cast<v4u*>(dst) = p1;
        *reinterpret_cast<v4u*>(dst + V_APLANE) = p2;
      }
    }
  };

  // ---- filter slab loads: 2 planes x 8 groups of 16 rows per slab; wavefront w loads row group w of every plane.
  // Lane l: row l / 4 of the group, chunk position l % 4 holding chunk (l % 4) ^ ((row / 4) % 4) of the row.
  const int bch = (lane & 3) ^ ((lane >> 4) & 3);
  auto issue_b = [&](int ct, int slab, int buf) {
    const int chunk = slab / 9, tap = slab - chunk * 9;
    const unsigned lbase = __builtin_amdgcn_readfirstlane(lds_offset_of(bring) + buf * V_BBUF + wave * 16 * V_BROW);
    const unsigned k_off = (unsigned)(tap * p.c + chunk * V_CH + bch * 8);
    const int n = ct * V_BN + wave * 16 + (lane >> 2);
    const unsigned row_off = n < p.k ? 2u * ((unsigned)n * (unsigned)p.Kgemm + k_off) : OOB;
#pragma unroll
    for (int plane = 0; plane < V_LPW; ++plane)
      load16_to_lds(rsrc_w, lbase + plane * V_BPLANE, row_off == OOB ? OOB : row_off + (unsigned)plane * wpb);
  };

  const int b_sw = (lrow >> 2) & 3;

  float* __restrict__ Y = static_cast<float*>(p.y);
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const float* addend = static_cast<const float*>(p.addend);   // may be the output itself
  const bool relu = p.act == 1;

  // Consecutive workgroup ids go round-robin to the 8 XCDs: give each XCD a contiguous run of tiles, so that the
  // channel tiles that share a patch (consecutive tile numbers) fetch it through the same L2.
  const int t_first = (gridDim.x & 7) == 0 ? (int)((blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) : (int)blockIdx.x;
  if (t_first >= total) return;

  // ---- the persistent loop over tiles for a wavefront that owns PX pixel blocks from block px_first on and CH
  // 32-channel columns from column ch_first on.  Both kinds of wavefront run the same sequence of barriers and
  // loads; only the fragments read and multiplied differ.
  auto run = [&](auto px_c, auto ch_c, int px_first, int ch_first) {
    constexpr int PX = decltype(px_c)::value, CH = decltype(ch_c)::value;
    // MFMA block i holds tile pixels 32 i .. 32 i + 31 in row-major order of the th x tw tile; lane lrow is the
    // lrow-th of them (pixels past the tile read patch pixel 0 and are never stored)
    int pp0[PX], key0[PX];
#pragma unroll
    for (int i = 0; i < PX; ++i) {
      const int tp = 32 * (px_first + i) + lrow;
      const int r = div_small(tp, inv_tw);
      pp0[i] = tp < tile_px ? r * pw + (tp - r * tw) : 0;
      key0[i] = tp < tile_px ? tp : 0;                     // r * tw + column
    }
    const int b_row = (ch_first * 32 + lrow) * V_BROW;
    int t = t_first;
    fetch_patch(t, 0);
    for (; t < total; t += gridDim.x) {
      int img, ty, tx, ct;
      decode(t, img, ty, tx, ct);
      const int t_next = t + gridDim.x;
      __syncthreads();                                  // everyone is done with the previous tile's last slab buffer
      issue_b(ct, 0, 0);
      // The tile's bias values now, not in the epilogue: there every store sits in a branch of its own, the compiler
      // cannot carry "already waited for" across them and waits for ALL memory operations in front of each store's
      // bias add, i.e. for the store before it.
      float bias_v[CH];
#pragma unroll
      for (int j = 0; j < CH; ++j) {
        const int ch = ct * V_BN + (ch_first + j) * 32 + lrow;
        bias_v[j] = (ch < p.k && bias) ? bias[ch] : 0.f;
      }

      v16f acc[PX][CH], acc_lo[PX][CH];                 // the h1 h1' products; the cross terms (weight 2^-11)
#pragma unroll
      for (int i = 0; i < PX; ++i)
#pragma unroll
        for (int j = 0; j < CH; ++j)
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
          } else if (need < se_x) {                       // uniform, rare: larger values than any chunk before
            const int d = need - se_x;
#pragma unroll
            for (int i = 0; i < PX; ++i)
#pragma unroll
              for (int j = 0; j < CH; ++j)
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
        // trip of a chunk), barrier, refill the other buffer with slab s + 1, multiply slab s.
        int tap_off = 0, tap_key = 0, ts = 0;
#pragma unroll 1
        for (int tap = 0; tap < 9; ++tap, ++s) {
          if (tap == 0 && fetching) __builtin_amdgcn_s_waitcnt(vmcnt_imm(V_PREF));
          else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
          __syncthreads();
          if (s + 1 < slabs) issue_b(ct, s + 1, (s + 1) & 1);
          const unsigned char* bb = bring + (s & 1) * V_BBUF + b_row;
          int ab[PX], sw[PX];
#pragma unroll
          for (int i = 0; i < PX; ++i) {
            ab[i] = (pp0[i] + tap_off) * V_PIXB;
            sw[i] = ((key0[i] + tap_key) >> 2) & 3;
          }
#pragma unroll
          for (int k16 = 0; k16 < 2; ++k16) {
            const int c8 = k16 * 2 + lhalf;                            // this lane's 16-byte chunk of the pixel / filter row
            v8h a[2][PX], b[2][CH];
#pragma unroll
            for (int o = 0; o < 2; ++o) {
              const int pa = o, pb = 1 - o;                              // the order the MFMAs use them in: cross terms first
#pragma unroll
              for (int i = 0; i < PX; ++i)
                a[pa][i] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(
                                                       lds + pa * V_APLANE + ab[i] + ((c8 ^ sw[i]) << 4)));
#pragma unroll
              for (int j = 0; j < CH; ++j)
                b[pb][j] = __builtin_bit_cast(v8h, *reinterpret_cast<const v4i*>(bb + pb * V_BPLANE + j * 32 * V_BROW + ((c8 ^ b_sw) << 4)));
            }
#pragma unroll
            for (int tt = 0; tt < 3; ++tt)
#pragma unroll
              for (int i = 0; i < PX; ++i)
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                  if (tt == 0) acc_lo[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], b[1][j], acc_lo[i][j], 0, 0, 0);
                  else if (tt == 1) acc_lo[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[1][i], b[0][j], acc_lo[i][j], 0, 0, 0);
                  else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0][i], b[0][j], acc[i][j], 0, 0, 0);
                }
          }
          if (++ts == 3) {                                 // next tap: down a patch row, or one column on
            ts = 0;
            tap_off += pw - 2;
            tap_key += tw - 2;
          } else {
            ++tap_off;
            ++tap_key;
          }
        }
      }

      // ---- epilogue.  Register e of a lane is pixel (e/4)*8 + 4*lhalf + e%4 of the 32-pixel block; channel = lrow
      // of the 32-channel column.
      // Nothing is in flight here (the last trip waited for everything and issued nothing), but the compiler cannot
      // see that through the loops: told so, it stops putting a wait for all memory operations in front of every
      // store's bias add, which made each store wait for the one before it.
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      const ScaleBack sb = scale_back_of(se_x, se_w, finite);
      int lh4 = lhalf * 4;
      asm volatile("" : "+v"(lh4));      // keeps the pixel arithmetic below inside the tile loop (hoisted, it is spilled)
#pragma unroll
      for (int j = 0; j < CH; ++j) {
        const int ch = ct * V_BN + (ch_first + j) * 32 + lrow;
        const bool cok = ch < p.k;
        const float bv = bias_v[j];
        if (ADD) {
          // The add link: eight addend values at a time, all in flight together, then one wait the compiler can see
          // and eight range-checked stores at the same offsets.  Loaded one by one in front of their stores, each
          // value would be waited for together with the store before it.
          const __amdgpu_buffer_rsrc_t rsrc_y = __builtin_amdgcn_make_buffer_rsrc(
              p.y, 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);
          const __amdgpu_buffer_rsrc_t rsrc_add = __builtin_amdgcn_make_buffer_rsrc(
              const_cast<float*>(addend), 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);
          auto offset_of = [&](int i, int e) -> unsigned {      // register e of pixel block i
            const int tp = 32 * (px_first + i) + (e >> 2) * 8 + lh4 + (e & 3);
            const int r = div_small(tp, inv_tw);
            const int c = tp - r * tw;
            const int oy = ty * th + r, ox = tx * tw + c;
            const bool ok = cok && tp < tile_px && oy < p.oh && ox < p.ow;
            return ok ? ((unsigned)((img * p.oh + oy) * p.ow + ox) * (unsigned)p.k + (unsigned)ch) * 4u : OOBX;
          };
#pragma unroll
          for (int i = 0; i < PX; ++i) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              float addv[8];
#pragma unroll
              for (int t = 0; t < 8; ++t)
                addv[t] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_add, offset_of(i, 8 * h + t), 0, 0));
              __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
#pragma unroll
              for (int t = 0; t < 8; ++t) {
                float v = join_sets(acc[i][j][8 * h + t], acc_lo[i][j][8 * h + t], sb) + bv + addv[t];
                if (relu) v = fmaxf(v, 0.f);
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), rsrc_y, offset_of(i, 8 * h + t), 0, 0);
              }
            }
          }
          continue;
        }
#pragma unroll
        for (int i = 0; i < PX; ++i) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            int tp = 32 * (px_first + i) + q * 8 + lh4;
            int r = div_small(tp, inv_tw);
            int c = tp - r * tw;
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
              const int oy = ty * th + r, ox = tx * tw + c;
              if (cok && tp < tile_px && oy < p.oh && ox < p.ow) {
                const size_t o = ((size_t)(img * p.oh + oy) * p.ow + ox) * p.k + ch;
                float v = join_sets(acc[i][j][4 * q + e4], acc_lo[i][j][4 * q + e4], sb) + bv;
                if (ADD) v += addend[o];
                if (relu) v = fmaxf(v, 0.f);
                Y[o] = v;
              }
              ++tp;
              if (++c == tw) { c = 0; ++r; }
            }
          }
        }
      }
    }
  };
  // Wavefronts 0-3: 2 x 2 blocks each over pixel blocks 0-3 (pixel pair w / 2, channel pair w % 2).
  // Wavefronts 4-7: the remaining NB - 4 pixel blocks of channel column w - 4.
  if (wave < 4) run(std::integral_constant<int, 2>{}, std::integral_constant<int, 2>{}, 2 * (wave >> 1), 2 * (wave & 1));
  else run(std::integral_constant<int, NB - 4>{}, std::integral_constant<int, 1>{}, 4, wave - 4);
}

struct TileShape {
  int th, tw, nb;
};

bool shape_ok(int th, int tw) {
  return th >= 1 && tw >= 1 && tw <= V_MAXTW && th * tw <= 256 && (th + 2) * (tw + 4) <= V_MAXPX;
}

long long tiles_of(const Problem& p, const TileShape& s) {
  return (long long)p.n * ((p.oh + s.th - 1) / s.th) * ((p.ow + s.tw - 1) / s.tw) * ((p.k + V_BN - 1) / V_BN);
}

// The tile shape of a layer: among all th x tw with 5 to 8 pixel blocks, the one with the least
// (rounds of tiles over the CUs) x (blocks per tile + the fixed part of a tile, about a third of a block);
// ties go to the shape that wastes fewer pixels, then the smaller patch, then the wider tile.
TileShape pick_tile(const Problem& p, int num_cu) {
  const int force_th = knob_or(KNOB_F32_K3_TH, 0), force_tw = knob_or(KNOB_F32_K3_TW, 0);
  if (force_th > 0 && force_tw > 0 && shape_ok(force_th, force_tw)) {       // tests and experiments
    const int nb = (force_th * force_tw + 31) / 32;
    return TileShape{force_th, force_tw, nb < 5 ? 5 : nb};
  }
  // the search below looks at a few hundred shapes: a layer asks three times per call (planner, kernel choice,
  // launch) and a caller issues the same layers again and again, so the last answer is kept per thread
  struct Memo {
    int n, oh, ow, k, num_cu;
    TileShape shape;
  };
  static thread_local Memo memo = {0, 0, 0, 0, 0, {16, 16, 8}};
  if (memo.n == p.n && memo.oh == p.oh && memo.ow == p.ow && memo.k == p.k && memo.num_cu == num_cu) return memo.shape;
  TileShape best{16, 16, 8};
  double best_cost = 1e300, best_fill = 0.0;
  int best_patch = 0;
  for (int tw = 4; tw <= V_MAXTW; ++tw) {
    for (int th = 1; th * tw <= 256; ++th) {
      if (!shape_ok(th, tw) || th * tw <= 128) continue;
      const TileShape s{th, tw, (th * tw + 31) / 32};
      const long long tiles = tiles_of(p, s);
      const long long rounds = (tiles + num_cu - 1) / num_cu;
      const double cost = (double)rounds * (s.nb + 0.3);
      const double fill = (double)p.oh * p.ow /
                          ((double)((p.oh + th - 1) / th) * th * (double)((p.ow + tw - 1) / tw) * tw) * (th * tw) / (32.0 * s.nb);
      const int patch = (th + 2) * (tw + 4);
      const bool better = cost < best_cost - 1e-9 ||
                          (cost < best_cost + 1e-9 &&
                           (fill > best_fill + 1e-9 ||
                            (fill > best_fill - 1e-9 && (patch < best_patch || (patch == best_patch && tw > best.tw)))));
      if (better) {
        best = s;
        best_cost = cost;
        best_fill = fill;
        best_patch = patch;
      }
    }
  }
  memo = Memo{p.n, p.oh, p.ow, p.k, num_cu, best};
  return best;
}

template <bool ADD, int NB>
hipError_t launch_k3v_variant(const Problem& p, const TileShape& s, int num_cu, hipStream_t stream) {
  auto kern = conv_k3v_f32_kernel<ADD, NB>;
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, V_LDS);
  if (attr_status != hipSuccess) return attr_status;
  const int tiles_y = (p.oh + s.th - 1) / s.th, tiles_x = (p.ow + s.tw - 1) / s.tw, tiles_c = (p.k + V_BN - 1) / V_BN;
  const long long total = (long long)p.n * tiles_y * tiles_x * tiles_c;
  const long long grid = total < num_cu ? total : num_cu;   // one persistent workgroup per CU
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(V_THREADS), V_LDS, stream, p, s.th, s.tw, tiles_y, tiles_x, tiles_c,
                     (int)total);
  return hipGetLastError();
}

template <bool ADD>
hipError_t launch_k3v_blocks(const Problem& p, const TileShape& s, int num_cu, hipStream_t stream) {
  switch (s.nb) {
    case 5: return launch_k3v_variant<ADD, 5>(p, s, num_cu, stream);
    case 6: return launch_k3v_variant<ADD, 6>(p, s, num_cu, stream);
    case 7: return launch_k3v_variant<ADD, 7>(p, s, num_cu, stream);
    case 8: return launch_k3v_variant<ADD, 8>(p, s, num_cu, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace

// Share of the machine's block products that are real outputs when this layer runs on the kernel:
// outputs / (rounds x CUs x pixels and channels of a tile).
double k3v_f32_efficiency(const Problem& p) {
  const int num_cu = num_compute_units() > 0 ? num_compute_units() : 256;
  const TileShape s = pick_tile(p, num_cu);
  const long long tiles = tiles_of(p, s);
  if (tiles >= (1LL << 30)) return 0.0;
  const long long rounds = (tiles + num_cu - 1) / num_cu;
  return (double)p.M * p.k / ((double)rounds * num_cu * 32.0 * s.nb * V_BN);
}

// The planner's own pick is the 16 x 16 tile: the fixed-tile kernel does that one with 2 x 2 blocks in every wavefront.
bool k3v_f32_prefers_fixed_tile(const Problem& p) {
  if (knob_or(KNOB_F32_K3_TH, 0) > 0 && knob_or(KNOB_F32_K3_TW, 0) > 0) return false;
  const int num_cu = num_compute_units() > 0 ? num_compute_units() : 256;
  const TileShape s = pick_tile(p, num_cu);
  return s.th == 16 && s.tw == 16;
}

hipError_t launch_k3v_f32(const Problem& p, hipStream_t stream, const char** variant) {
  const int num_cu = num_compute_units();
  if (num_cu < 1) return hipErrorInvalidDevice;
  const TileShape s = pick_tile(p, num_cu);
  static thread_local char name[64];
  snprintf(name, sizeof(name), "conv_k3_f32_f16x3_%dx%d%s", s.th, s.tw, p.addend ? "_add" : "");
  *variant = name;
  return p.addend ? launch_k3v_blocks<true>(p, s, num_cu, stream) : launch_k3v_blocks<false>(p, s, num_cu, stream);
}

}  // namespace glowmi
