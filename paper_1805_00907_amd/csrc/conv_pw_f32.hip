// fp32 pointwise (1x1, unpadded) Convolution with a short reduction: the "1x1 on many pixels" kind of
// layer that makes up two thirds of a residual network's convolutions.  The paper's CPU backend
// gives each kind of convolution its own strategy (Section 5.3); this is the one for this kind on
// gfx950.
//
// With C = 64 or 128 input channels the reduction is only a few MFMA steps long, so a tile-per-workgroup
// GEMM spends most of its time in set-up, barriers and the epilogue.  Here instead
//   - the filter slice of a workgroup (BN output channels x C, 64 KB) is staged into LDS once and
//     stays there: one persistent workgroup of eight wavefronts per CU, all reading their B
//     fragments from it;
//   - a wavefront owns blocks of 32 output pixels and walks their reduction in chunks of 64
//     channels.  A chunk (32 pixels x 256 bytes) is fetched with fully coalesced 16-byte loads - every
//     load instruction covers whole cache lines exactly once - and goes through a private 8.5 KB LDS
//     region of the wavefront, from which the A fragments are read in MFMA layout.  The region is
//     private, so no barrier is involved: a wavefront's LDS operations execute in order;
//   - after the one barrier that publishes the filter slice the wavefronts run independently, two
//     per SIMD overlapping each other's loads and MFMAs; the next chunk's global loads are in flight
//     during the MFMAs of the current one;
//   - work items are (pixel block, 64-channel group), or their 32-channel halves when there are few
//     per wavefront; a wavefront takes a contiguous range of them and computes the two halves of a
//     group together where it holds both
//     (with C = 64 consecutive items of one pixel block reuse the staged chunk), so the last round of
//     the grid is short.
// Epilogue as everywhere (operator stacking, Section 5.2): bias + Relu on the accumulators, one store.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "bf16_pieces.h"
#include "igemm.h"
#include "pw_common.h"

namespace glowmi {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int PW_THREADS = 512;
constexpr int PW_WAVES = PW_THREADS / 64;
constexpr int PW_CHUNK = 64;                  // channels per staged A chunk
constexpr int PW_APITCH = PW_CHUNK + 4;       // floats; conflict-free ds_read_b128 / ds_write_b128
constexpr int PW_AREGION = 32 * PW_APITCH;    // floats per wavefront

template <int K>
struct Pw {
  static constexpr int BN = 16384 / K;        // output channels per workgroup: BN * K * 4 = 64 KB
  static constexpr int NG = BN / 64;          // 64-channel groups per slice (power of two)
  static constexpr int PITCH = K + 4;         // LDS row pitch of the filter slice in floats
  static constexpr int KC = K / PW_CHUNK;     // chunks per reduction
  static constexpr int lds_bytes = (BN * PITCH + PW_WAVES * PW_AREGION + BN) * (int)sizeof(float);
  static_assert(BN >= 64 && (NG & (NG - 1)) == 0 && K % PW_CHUNK == 0, "slice shape");
};

// CONTIGUOUS: the input pixel of output pixel m is m itself (unit strides); otherwise it is derived
// from (image, row, column).
// ADD: the element-wise chain has a tensor-add link (p.addend, of the output's shape).
template <int K, bool CONTIGUOUS, bool ADD>
__global__ __launch_bounds__(PW_THREADS, 1) void conv_pw_f32_kernel(const Problem p, const PwRange full,
                                                                   const PwRange last, int halves) {
  using G = Pw<K>;
  extern __shared__ __align__(16) float smem[];            // filter slice [BN][PITCH], A regions, bias [BN]
  float* wlds = smem;
  float* blds = smem + G::BN * G::PITCH + PW_WAVES * PW_AREGION;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int slice = blockIdx.y;
  float* alds = smem + G::BN * G::PITCH + wave * PW_AREGION;

  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_y =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_add = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(ADD ? p.addend : p.y), 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);

  // ---- this wavefront's contiguous range of items (pixel block major, channel group minor)
  const PwRange& range = slice == (int)gridDim.y - 1 ? last : full;    // the last slice may be narrower
  const int wv = blockIdx.x * PW_WAVES + wave;
  int it, it_end_;
  deal_range(wv, (int)gridDim.x * PW_WAVES, range.items_div, range.items_rem, it, it_end_);
  const int it_end = it_end_;
  auto block_of = [&](int item) { return range.div_ngc.div(item); };

  const int ohow = p.oh * p.ow;
  const unsigned row_bytes = (unsigned)p.k * 4u;           // output pixel pitch
  const float floor_value = p.act == 1 ? 0.f : -__builtin_inff();   // Relu as a lower bound

  // (Measured and not kept: a second register set so that loads run two chunks ahead of the MFMAs --
  // 256 -> 64 on 56 x 56 at batch 32 49 -> 52 us, 128 -> 512 with the add link 47 -> 53 us: the loads
  // already have a whole chunk of MFMAs to arrive, and more of them in flight only lengthen the queue.)
  // Staging of one chunk: load i of a lane covers pixel 4i + lane/16 of the block, 16 bytes at
  // channel chunk*64 + 4*(lane%16): four whole 256-byte runs per instruction.
  const int srow = lane >> 4, sq = lane & 15;
  v4f st[8];
  auto fetch_chunk = [&](int rb, int chunk) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int m = rb * 32 + 4 * i + srow;
      if (m >= p.M) m = p.M - 1;                           // results of such rows are never stored
      int pix = m;
      if (!CONTIGUOUS) {
        const int img = p.div_ohow.div(m);
        const int rem = m - img * ohow;
        const int oh = p.div_ow.div(rem);
        const int ow = rem - oh * p.ow;
        pix = (img * p.h + oh * p.stride_h) * p.w_ + ow * p.stride_w;
      }
      const unsigned off = ((unsigned)pix * (unsigned)K + (unsigned)(chunk * PW_CHUNK + 4 * sq)) * 4u;
      st[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0));
    }
  };
  auto commit_chunk = [&]() {
#pragma unroll
    for (int i = 0; i < 8; ++i) *reinterpret_cast<v4f*>(alds + (4 * i + srow) * PW_APITCH + 4 * sq) = st[i];
  };

  // the first chunk's loads go out before the filter slice's, so both latencies overlap
  const bool has_work = it < it_end;
  if (has_work) fetch_chunk(block_of(it), 0);

  // ---- filter slice -> LDS.  The slice is one contiguous run of the [k][C] filter; rows past the
  // last output channel lie past the end of the tensor and the range-checked loads return zeros.
  {
    constexpr int V4_PER_ROW = K / 4;
    constexpr int PASSES = G::BN * V4_PER_ROW / PW_THREADS;
    const unsigned base = (unsigned)slice * (unsigned)(G::BN * K * 4);
    v4f stage[PASSES];
#pragma unroll
    for (int q = 0; q < PASSES; ++q) {
      const int i = tid + q * PW_THREADS;
      stage[q] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, base + (unsigned)i * 16u, 0, 0));
    }
#pragma unroll
    for (int q = 0; q < PASSES; ++q) {
      const int i = tid + q * PW_THREADS;
      const int ch = i / V4_PER_ROW, kq = i % V4_PER_ROW;
      *reinterpret_cast<v4f*>(wlds + ch * G::PITCH + kq * 4) = stage[q];
    }
    // the slice's bias values too: read in the epilogue from LDS, so that no global load (whose
    // wait would also wait for the stores before it) sits between one item's stores and the next
    if (tid < G::BN) {
      const int ch = slice * G::BN + tid;
      blds[tid] = (bias && ch < p.k) ? bias[ch] : 0.f;
    }
  }
  __syncthreads();

  const float* a_lane = alds + l32 * PW_APITCH + 4 * lh;
  const float* w_lane = wlds + l32 * G::PITCH + 4 * lh;

  if (!has_work) return;
  commit_chunk();
  // One item: NB = 2 (both 32-channel halves of a 64-channel group, sharing the pixel fragments) or
  // NB = 1 (the half `hsel` alone, where a wavefront's range begins or ends inside a group).
  auto process = [&](auto nb_tag, int rb, int ng, int hsel, bool more, int rb_next) {
    constexpr int NB = decltype(nb_tag)::value;
    // The addend values of this item are fetched before the MFMAs: a load issued in the epilogue
    // would wait for its own latency and, the memory counter being in order, for the stores before it.
    const unsigned item_off = (unsigned)(rb * 32 + 4 * lh) * row_bytes +
                              (unsigned)(slice * G::BN + ng * 64 + hsel * 32 + l32) * 4u;
    float addv[NB][16];
    if (ADD) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          addv[nb][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
              rsrc_add, item_off + 128u * nb + (unsigned)((e >> 2) * 8 + (e & 3)) * row_bytes, 0, 0));
    }

    v16f acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[nb][e] = 0.f;
    const float* wl = w_lane + (ng * 64 + hsel * 32) * G::PITCH;
#pragma unroll
    for (int c = 0; c < G::KC; ++c) {
      // the chunk after this one: the next of this item, or the first of the next item (with a
      // single chunk per reduction the staged one is reused while the pixel block stays the same)
      const bool stage_next = c + 1 < G::KC || (more && (G::KC > 1 || rb_next != rb));
      if (stage_next) fetch_chunk(c + 1 < G::KC ? rb : rb_next, c + 1 < G::KC ? c + 1 : 0);
#pragma unroll
      for (int j = 0; j < PW_CHUNK / 8; ++j) {
        // all operands hold channels {8j+t, 8j+4+t} in component t of the two half-waves
        const v4f a4 = *reinterpret_cast<const v4f*>(a_lane + 8 * j);
        v4f b[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          b[nb] = *reinterpret_cast<const v4f*>(wl + nb * 32 * G::PITCH + c * PW_CHUNK + 8 * j);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[t], b[nb][t], acc[nb], 0, 0, 0);
      }
      // in program order after this chunk's fragment reads: the wavefront's LDS operations execute
      // in order, so the region is overwritten only once it has been read
      if (stage_next) commit_chunk();
    }

    // ---- epilogue: register e of a lane is pixel (e/4)*8 + 4*lh + e%4 of the block, channel l32.
    // Rows past M fall outside the output buffer's range and the checked stores drop them.
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int ch = slice * G::BN + ng * 64 + (hsel + nb) * 32 + l32;
      {
        // no branch around the stores of a channel past the last one (they go out of the buffer's range): under a
        // branch the compiler cannot count on them, and its wait for the chunk fetched before them drains them all
        const float bv = blds[ng * 64 + (hsel + nb) * 32 + l32];
        unsigned lane_off = ch < p.k ? (unsigned)(rb * 32 + 4 * lh) * row_bytes + (unsigned)ch * 4u : 0xF0000000u;
        asm volatile("" : "+v"(lane_off));                 // keep the per-register row offsets scalar
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float v = fmaxf(acc[nb][e] + bv + (ADD ? addv[nb][e] : 0.f), floor_value);
          const unsigned off = lane_off + (unsigned)((e >> 2) * 8 + (e & 3)) * row_bytes;
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), rsrc_y, off, 0, 0);
        }
      }
    }
  };

  if (!halves) {
    // items are whole 64-channel groups
    for (; it < it_end; ++it) {
      const int rb = block_of(it);
      process(std::integral_constant<int, 2>{}, rb, it - rb * range.ngc, 0, it + 1 < it_end, block_of(it + 1));
    }
    return;
  }
  // Items are 32-channel halves (range.ngc of them per pixel block, an even number); a wavefront takes
  // the two halves of a group together wherever its range holds both.
  while (it < it_end) {
    const int rb = block_of(it), hh = it - rb * range.ngc;
    const bool pair = (hh & 1) == 0 && it + 1 < it_end;    // uniform
    const int step = pair ? 2 : 1;
    const bool more = it + step < it_end;
    const int rb_next = block_of(it + step);
    if (pair) process(std::integral_constant<int, 2>{}, rb, hh >> 1, 0, more, rb_next);
    else process(std::integral_constant<int, 1>{}, rb, hh >> 1, hh & 1, more, rb_next);
    it += step;
  }
}

// ---------------------------------------------------------------------------------------------------
// The same design on the bf16 matrix cores: every fp32 operand cut exactly into three bf16 pieces and a
// product taken as six piece products (bf16_pieces.h), 192 matrix-pipe cycles per 16 reduction steps of a
// 32 x 32 block instead of 512.  The filter slice is cut once per workgroup while it is staged (three
// bf16 planes in LDS).  The input is cut where it is used: a pointwise layer stages each input element
// once per filter slice, so cutting it costs the same ~6 vector instructions per element as a separate
// packing pass would, without that pass's memory traffic.  A wavefront's chunk is 32 pixels x 32 channels
// (128-byte runs, whole cache lines per load instruction), kept as fp32 in its private LDS region; the
// lane that feeds MFMA row l, reduction indices 8h .. 8h+7, reads those eight values and cuts them in
// registers.  Everything else (persistent workgroups, items, epilogue) as in the kernel above.
// ---------------------------------------------------------------------------------------------------
constexpr int PB_CHUNK = 32;                  // channels per staged chunk
constexpr int PB_APITCH = PB_CHUNK + 4;       // floats
constexpr int PB_AREGION = 32 * PB_APITCH;    // floats per wavefront

template <int K>
struct PwB {
  static constexpr int BN = 16384 / K;        // output channels per workgroup
  static constexpr int NG = BN / 64;
  static constexpr int PITCHB = 2 * K + 16;   // bytes per filter row of one plane: an odd number of 16-byte units
  static constexpr int PLANE = BN * PITCHB;   // bytes per plane
  static constexpr int KC = K / PB_CHUNK;
  static constexpr int lds_bytes = 3 * PLANE + (PW_WAVES * PB_AREGION + BN) * (int)sizeof(float);
  static_assert(BN >= 64 && (NG & (NG - 1)) == 0 && K % PB_CHUNK == 0 && KC >= 2, "slice shape");
  static_assert(lds_bytes <= 160 * 1024, "LDS of one CU");
};

template <int K, bool CONTIGUOUS, bool ADD>
__global__ __launch_bounds__(PW_THREADS, 1) void conv_pw_f32_bf16_kernel(const Problem p, const PwRange full,
                                                                        const PwRange last, int halves) {
  using G = PwB<K>;
  extern __shared__ __align__(16) unsigned char smem_b[];   // filter planes [3][BN][PITCHB], A regions, bias [BN]
  unsigned char* wlds = smem_b;
  float* fl = reinterpret_cast<float*>(smem_b + 3 * G::PLANE);
  float* blds = fl + PW_WAVES * PB_AREGION;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int slice = blockIdx.y;
  float* alds = fl + wave * PB_AREGION;

  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_y =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_add = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(ADD ? p.addend : p.y), 0, (int)((unsigned)p.M * (unsigned)p.k * 4u), 0x00020000);

  const PwRange& range = slice == (int)gridDim.y - 1 ? last : full;
  const int wv = blockIdx.x * PW_WAVES + wave;
  int it, it_end_;
  deal_range(wv, (int)gridDim.x * PW_WAVES, range.items_div, range.items_rem, it, it_end_);
  const int it_end = it_end_;
  auto block_of = [&](int item) { return range.div_ngc.div(item); };

  const int ohow = p.oh * p.ow;
  const unsigned row_bytes = (unsigned)p.k * 4u;
  const float floor_value = p.act == 1 ? 0.f : -__builtin_inff();

  // Staging of one chunk: load i of a lane covers pixel 8i + lane/8 of the block, 16 bytes at channel
  // chunk*32 + 4*(lane%8): eight whole 128-byte runs per instruction.
  // Up to two chunks are kept in flight per wavefront (a chunk is multiplied in a fraction of the memory latency, and
  // what a CU streams is the bytes it has in flight over that latency): chunk c + 2 is fetched into the registers
  // chunk c was committed from.  A reduction is an even number of chunks long, so a chunk's slot is its index's parity.
  const int srow = lane >> 3, sq = lane & 7;
  v4f st2[2][4];
  static_assert(G::KC % 2 == 0, "slot of a chunk = parity of its index, also across items");
  // (64 channels with the add link: two chunks ahead spill; 256 channels: measured no gain, 39.6 -> 40.5 us on
  // 32 x 56 x 56 x 256 -> 64; 64 -> 256: 35.3 -> 32.4 us, 128 -> 512 with the add link: 37.7 -> 36.4 us)
  constexpr int AHEAD = (K == 64 && ADD) || K == 256 ? 1 : 2;
  auto fetch_chunk = [&](int slot, int rb, int chunk) {      // slot: a constant once the chunk loop is unrolled
    v4f (&st)[4] = st2[slot];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int m = rb * 32 + 8 * i + srow;
      if (m >= p.M) m = p.M - 1;                           // results of such rows are never stored
      int pix = m;
      if (!CONTIGUOUS) {
        const int img = p.div_ohow.div(m);
        const int rem = m - img * ohow;
        const int oh = p.div_ow.div(rem);
        const int ow = rem - oh * p.ow;
        pix = (img * p.h + oh * p.stride_h) * p.w_ + ow * p.stride_w;
      }
      const unsigned off = ((unsigned)pix * (unsigned)K + (unsigned)(chunk * PB_CHUNK + 4 * sq)) * 4u;
      st[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0));
    }
  };
  auto commit_chunk = [&](int slot) {
    const v4f (&st)[4] = st2[slot];
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<v4f*>(alds + (8 * i + srow) * PB_APITCH + 4 * sq) = st[i];
  };

  const bool has_work = it < it_end;
  if (has_work) {
    fetch_chunk(0, block_of(it), 0);
    if (AHEAD == 2) fetch_chunk(1, block_of(it), 1);
  }

  // ---- filter slice -> three bf16 planes in LDS.  The slice is one contiguous run of the [k][C] filter; rows
  // past the last output channel lie past the end of the tensor and the range-checked loads return zeros.
  {
    constexpr int V8_PER_ROW = K / 8;
    constexpr int PASSES = G::BN * V8_PER_ROW / PW_THREADS;
    const unsigned base = (unsigned)slice * (unsigned)(G::BN * K * 4);
#pragma unroll
    for (int q = 0; q < PASSES; ++q) {
      const int i = tid + q * PW_THREADS;
      const v4f lo4 = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, base + (unsigned)i * 32u, 0, 0));
      const v4f hi4 = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, base + (unsigned)i * 32u + 16u, 0, 0));
      const float v[8] = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
      v4u h, m, l;
      split8(v, h, m, l);
      const int ch = i / V8_PER_ROW, kq = i % V8_PER_ROW;
      unsigned char* dst = wlds + ch * G::PITCHB + kq * 16;
      *reinterpret_cast<v4u*>(dst) = h;
      *reinterpret_cast<v4u*>(dst + G::PLANE) = m;
      *reinterpret_cast<v4u*>(dst + 2 * G::PLANE) = l;
    }
    if (tid < G::BN) {
      const int ch = slice * G::BN + tid;
      blds[tid] = (bias && ch < p.k) ? bias[ch] : 0.f;
    }
  }
  __syncthreads();

  const float* a_lane = alds + l32 * PB_APITCH + 8 * lh;
  const unsigned char* w_lane = wlds + l32 * G::PITCHB + 16 * lh;

  if (!has_work) return;
  commit_chunk(0);
  // With C = 64 the cut pixel fragments of a block stay in registers (48 per lane) and serve every channel group
  // the wavefront computes for that block: only the first item of a block stages and cuts, the others neither
  // touch the input nor the vector ALU for it.  (With C = 128 the 96 registers spill.)
  constexpr bool CACHE = K == 64;
  v8bf a_cache[CACHE ? G::KC : 1][2][3];
  int cached_rb = -1;
  const int rb_last = block_of(it_end - 1);
  auto process = [&](auto nb_tag, int rb, int ng, int hsel, bool more, int rb_next) {
    constexpr int NB = decltype(nb_tag)::value;
    const bool fresh = !CACHE || rb != cached_rb;          // uniform
    if (CACHE) {                                           // the next block whose first chunk must be staged
      more = rb < rb_last;
      rb_next = rb + 1;
      cached_rb = rb;
    }
    const unsigned item_off = (unsigned)(rb * 32 + 4 * lh) * row_bytes +
                              (unsigned)(slice * G::BN + ng * 64 + hsel * 32 + l32) * 4u;
    float addv[NB][16];
    if (ADD) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          addv[nb][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
              rsrc_add, item_off + 128u * nb + (unsigned)((e >> 2) * 8 + (e & 3)) * row_bytes, 0, 0));
    }

    v16f acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[nb][e] = 0.f;
    const unsigned char* wl = w_lane + (ng * 64 + hsel * 32) * G::PITCHB;
#pragma unroll
    for (int c = 0; c < G::KC; ++c) {
      // the chunk after this one: the next of this item, or the first of the next item (a reduction is at
      // least two chunks long, so the region never still holds chunk 0 when an item ends)
      const bool stage_next = fresh && (c + 1 < G::KC || more);
      // two ahead: chunk c's registers are free (committed), the chunk two on goes there
      if (fresh && (c + AHEAD < G::KC || more))
        fetch_chunk((c + AHEAD) % 2, c + AHEAD < G::KC ? rb : rb_next, (c + AHEAD) % G::KC);
#pragma unroll
      for (int j = 0; j < PB_CHUNK / 16; ++j) {
        v8bf b[3][NB];
#pragma unroll
        for (int pc = 0; pc < 3; ++pc)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            b[pc][nb] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4i*>(
                wl + pc * G::PLANE + nb * 32 * G::PITCHB + (c * PB_CHUNK + 16 * j) * 2));
        v8bf a[3];
        if (fresh) {
          // a lane holds reduction indices 16j + 8*lh .. + 7 of its pixel (input) / channel (filter)
          const v4f a0 = *reinterpret_cast<const v4f*>(a_lane + 16 * j);
          const v4f a1 = *reinterpret_cast<const v4f*>(a_lane + 16 * j + 4);
          const float v[8] = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
          v4u ah, am, al;
          split8(v, ah, am, al);
          a[0] = __builtin_bit_cast(v8bf, ah);
          a[1] = __builtin_bit_cast(v8bf, am);
          a[2] = __builtin_bit_cast(v8bf, al);
          if (CACHE) {
#pragma unroll
            for (int pc = 0; pc < 3; ++pc) a_cache[c][j][pc] = a[pc];
          }
        } else {
#pragma unroll
          for (int pc = 0; pc < 3; ++pc) a[pc] = a_cache[CACHE ? c : 0][j][pc];
        }
#pragma unroll
        for (int t = 0; t < 6; ++t)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kPieceTermA[t]], b[kPieceTermB[t]][nb], acc[nb], 0, 0, 0);
      }
      // in program order after this chunk's fragment reads: the wavefront's LDS operations execute
      // in order, so the region is overwritten only once it has been read
      if (stage_next) commit_chunk((c + 1) % 2);
    }

#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int ch = slice * G::BN + ng * 64 + (hsel + nb) * 32 + l32;
      {
        // No branch around the stores of a channel past the last one: they go out of the buffer's range instead.
        // With the stores under a branch the compiler cannot count on them having been issued, and its wait for
        // the input chunk fetched before them (four loads) becomes a wait for all of the item's stores to drain.
        const float bv = blds[ng * 64 + (hsel + nb) * 32 + l32];
        unsigned lane_off = ch < p.k ? (unsigned)(rb * 32 + 4 * lh) * row_bytes + (unsigned)ch * 4u : 0xF0000000u;
        asm volatile("" : "+v"(lane_off));                 // keep the per-register row offsets scalar
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float v = fmaxf(acc[nb][e] + bv + (ADD ? addv[nb][e] : 0.f), floor_value);
          const unsigned off = lane_off + (unsigned)((e >> 2) * 8 + (e & 3)) * row_bytes;
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), rsrc_y, off, 0, 0);
        }
      }
    }
  };

  if (!halves) {
    for (; it < it_end; ++it) {
      const int rb = block_of(it);
      process(std::integral_constant<int, 2>{}, rb, it - rb * range.ngc, 0, it + 1 < it_end, block_of(it + 1));
    }
    return;
  }
  while (it < it_end) {
    const int rb = block_of(it), hh = it - rb * range.ngc;
    const bool pair = (hh & 1) == 0 && it + 1 < it_end;    // uniform
    const int step = pair ? 2 : 1;
    const bool more = it + step < it_end;
    const int rb_next = block_of(it + step);
    if (pair) process(std::integral_constant<int, 2>{}, rb, hh >> 1, 0, more, rb_next);
    else process(std::integral_constant<int, 1>{}, rb, hh >> 1, hh & 1, more, rb_next);
    it += step;
  }
}

template <int K, bool CONTIGUOUS, bool ADD, bool BF16>
hipError_t launch_pw(const Problem& p, hipStream_t stream) {
  using G = std::conditional_t<BF16, PwB<K>, Pw<K>>;
  auto kern = BF16 ? conv_pw_f32_bf16_kernel<K, CONTIGUOUS, ADD> : conv_pw_f32_kernel<K, CONTIGUOUS, ADD>;
  // once per instantiation; initialisation of a function-local static is thread-safe
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, G::lds_bytes);
  if (attr_status != hipSuccess) return attr_status;
  const int num_cu = num_compute_units();
  if (num_cu < 1) return hipErrorInvalidDevice;
  const int slices = (p.k + G::BN - 1) / G::BN;
  const int row_blocks = (p.M + 31) / 32;
  const int groups_last = (p.k - (slices - 1) * G::BN + 63) / 64;      // 64-channel groups of the last slice
  const int groups_full = slices > 1 ? G::NG : groups_last;
  long long wgs = (long long)num_cu / slices;             // one persistent workgroup per CU
  if (wgs < 1) wgs = 1;
  const long long items_max = (long long)row_blocks * groups_full;
  if (wgs > (items_max + PW_WAVES - 1) / PW_WAVES) wgs = (items_max + PW_WAVES - 1) / PW_WAVES;
  const long long waves = wgs * PW_WAVES;
  dim3 grid((unsigned)wgs, (unsigned)slices, 1), block(PW_THREADS, 1, 1);
  // With few groups per wavefront (1.5 each on 256->64 at batch 32) whole groups leave a third of the
  // SIMDs a quarter longer than the rest: the work is then dealt in 32-channel halves (measured 44.4 ->
  // 41.3 us).  With many groups per wavefront halves only cost shared fragment reads (64->256: 6 groups
  // each, 44 -> 47 us inside the step), so whole groups stay.
  const int halves = items_max < 4 * waves ? 1 : 0;
  const int unit = halves ? 2 : 1;
  hipLaunchKernelGGL(kern, grid, block, G::lds_bytes, stream, p, make_pw_range(row_blocks, unit * groups_full, waves),
                     make_pw_range(row_blocks, unit * groups_last, waves), halves);
  return hipGetLastError();
}

int pw_min_items() {
  return knob_or(KNOB_F32_PW_MIN_ITEMS, 1024);   // the knob: experiments and tests
}

}  // namespace

bool pw_f32_applicable(const Problem& p) {
  if (p.b_is_kn || p.groups != 1 || p.r != 1 || p.s != 1 || p.pad_t != 0 || p.pad_l != 0) return false;
  if (p.c != 64 && p.c != 128 && p.c != 256) return false;   // longer reductions amortise the generic kernel's set-up
  // bottom/right padding would make output pixels read outside the image
  if ((long long)(p.oh - 1) * p.stride_h >= p.h || (long long)(p.ow - 1) * p.stride_w >= p.w_) return false;
  if ((unsigned long long)p.M * (unsigned long long)p.k * 4ull > 0xF0000000ull || p.k > 65536) return false;
  if (p.w_bytes > 0x7FFFFFFFu) return false;
  // enough (pixel block, 64-channel group) items over all filter slices to keep every CU's persistent
  // workgroup busy (measured: 1x1 256->1024 on 14x14 at batch 32, 196 blocks x 16 slices of one group,
  // 45.6 us tiled -> 38.4 us here)
  const long long items = (long long)((p.M + 31) / 32) * ((p.k + 63) / 64);
  return items >= pw_min_items() && items < (1LL << 30);
}

template <int K, bool BF16>
hipError_t launch_pw_k(const Problem& p, hipStream_t stream) {
  const bool contiguous = p.stride_h == 1 && p.stride_w == 1;
  if (p.addend) return contiguous ? launch_pw<K, true, true, BF16>(p, stream) : launch_pw<K, false, true, BF16>(p, stream);
  return contiguous ? launch_pw<K, true, false, BF16>(p, stream) : launch_pw<K, false, false, BF16>(p, stream);
}

hipError_t launch_pw_f32(const Problem& p, hipStream_t stream, const char** variant) {
  const bool contiguous = p.stride_h == 1 && p.stride_w == 1;
  // Measured at batch 32 (fp32 matrix cores -> here): 64 -> 256 on 56 x 56 44 -> 33 us, 256 -> 64 50 -> 44 us,
  // 64 -> 256 + add 52 -> 50 us (that one moves 232 MB for 3.3 GFLOP and is bound by memory on either matrix
  // core), 128 -> 512 + add on 28 x 28 47 -> 39 us, 256 -> 1024 + add on 14 x 14 44 -> 37 us.  The knob selects
  // the fp32 matrix-core form (tests, comparisons).
  const bool bf16 = knob_or(KNOB_F32_PW_BF16, 1) != 0;
  static thread_local char name[48];
  snprintf(name, sizeof(name), "conv_pw_f32_c%d%s%s%s", p.c, bf16 ? "_bf16x6" : "", contiguous ? "" : "_strided",
           p.addend ? "_add" : "");
  *variant = name;
  switch (p.c) {
    case 64: return bf16 ? launch_pw_k<64, true>(p, stream) : launch_pw_k<64, false>(p, stream);
    case 128: return bf16 ? launch_pw_k<128, true>(p, stream) : launch_pw_k<128, false>(p, stream);
    case 256: return bf16 ? launch_pw_k<256, true>(p, stream) : launch_pw_k<256, false>(p, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace glowmi
