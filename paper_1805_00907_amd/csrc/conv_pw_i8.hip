// int8 pointwise (1x1, unpadded) Convolution: the quantized form (Section 4 of the paper: int8 codes
// with per-tensor scale/offset, int32 accumulation, rescale folded into the producer, Relu as an
// integer lower bound) of the "1x1 on many pixels" kind of layer, one of the kinds of convolution
// that get a strategy of their own (Section 5.3).
//
// In int8 these layers are nowhere near MFMA-bound: the work is moving bytes and requantizing, so
// the kernel is built to spend as little as possible per output besides that:
//   - one persistent workgroup (eight wavefronts) stages its filter slice (BN channels x C bytes)
//     into LDS once, already in the row order the MFMA needs, and derives the per-channel additive
//     term  bias - x_offset * sum_c w  from it (filter offset 0 only; other filters take the generic
//     kernel);
//   - a wavefront owns blocks of 32 pixels.  A block's input (32 x C bytes, contiguous rows) is
//     fetched with coalesced 16-byte loads into a private LDS region (no barrier: a wavefront's LDS
//     operations execute in order) while the previous block is being worked on;
//   - per (block, 64-channel group) item: C/32 MFMA steps (v_mfma_i32_32x32x32_i8) with the filter
//     as the row operand and the channels permuted so that a lane ends up with 32 consecutive
//     channels of one pixel (the accumulators start at the channel term): requantize, clamp, pack,
//     two 16-byte stores.
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

constexpr int PWQ_THREADS = 512;
constexpr int PWQ_WAVES = PWQ_THREADS / 64;

template <int K>
struct PwQ {
  static constexpr int BN = K <= 128 ? 256 : 128;   // output channels per workgroup
  static constexpr int NG = BN / 64;                // 64-channel groups per slice
  static constexpr int PITCH = K + 16;              // LDS row pitch in bytes, filter rows and pixel rows
  static constexpr int STEPS = K / 32;              // MFMA steps per reduction
  static constexpr int LPR = K / 16;                // lanes per pixel row when staging
  static constexpr int RPI = 64 / LPR;              // pixel rows per staging instruction
  static constexpr int NI = 32 / RPI;               // staging instructions per block
  static constexpr int AREGION = 32 * PITCH;        // bytes per wavefront
  static constexpr int WG_PER_CU = K <= 128 ? 2 : 1;
  static constexpr int lds_bytes = BN * PITCH + PWQ_WAVES * AREGION + BN * 4 + 256 * 4;   // + addend table
  static_assert(K % 64 == 0 && K <= 256, "reduction length");
};

// Row of the staged filter slice that holds channel `c` (0..63) of a 64-channel group.  MFMA nb
// (0/1) of an item multiplies rows nb*32 .. nb*32+31; result register e of a lane with half h is MFMA
// row (e/4)*8 + 4h + e%4, and this order makes that row channel 32h + 16nb + e: a lane's 16 registers
// are 16 consecutive channels.
__host__ __device__ constexpr int staged_row(int c) {
  return ((c >> 4) & 1) * 32 + ((c >> 2) & 3) * 8 + (c >> 5) * 4 + (c & 3);
}

// ADD: the element-wise chain has a tensor-add link (p.addend, int8 of the output's shape, rescaled
// to the accumulator's scale before it is added).
template <int K, bool CONTIGUOUS, bool ADD>
__global__ __launch_bounds__(PWQ_THREADS, PwQ<K>::WG_PER_CU) void conv_pw_i8_kernel(const Problem p,
                                                                                  const PwRange full,
                                                                                  const PwRange last) {
  using G = PwQ<K>;
  extern __shared__ __align__(16) unsigned char smem[];   // filter slice, A regions, channel terms
  unsigned char* wlds = smem;
  int* cterm = reinterpret_cast<int*>(smem + G::BN * G::PITCH + PWQ_WAVES * G::AREGION);
  int* addlut = cterm + G::BN;   // [256] the addend's code (as an unsigned byte) -> its term at the accumulator's scale

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int slice = blockIdx.y;
  unsigned char* alds = smem + G::BN * G::PITCH + wave * G::AREGION;

  const int* __restrict__ bias = static_cast<const int*>(p.bias);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_y =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)((unsigned)p.M * (unsigned)p.k), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_add = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(ADD ? p.addend : p.y), 0, (int)((unsigned)p.M * (unsigned)p.k), 0x00020000);

  // ---- this wavefront's contiguous range of items (pixel block major, channel group minor)
  const PwRange& range = slice == (int)gridDim.y - 1 ? last : full;    // the last slice may be narrower
  const int wv = blockIdx.x * PWQ_WAVES + wave;
  int it, it_end_;
  deal_range(wv, (int)gridDim.x * PWQ_WAVES, range.items_div, range.items_rem, it, it_end_);
  const int it_end = it_end_;
  const int ohow = p.oh * p.ow;

  // Staging of a pixel block: load i of a lane covers pixel i*RPI + lane/LPR, 16 bytes at channel
  // 16*(lane%LPR): whole pixel rows, so every instruction reads complete runs of C bytes.
  const int srow = lane / G::LPR, sq = lane % G::LPR;
  v4i st[G::NI];
  auto fetch_block = [&](int rb) {
#pragma unroll
    for (int i = 0; i < G::NI; ++i) {
      int m = rb * 32 + i * G::RPI + srow;
      if (m >= p.M) m = p.M - 1;                           // results of such rows are never stored
      int pix = m;
      if (!CONTIGUOUS) {
        const int img = p.div_ohow.div(m);
        const int rem = m - img * ohow;
        const int oh = p.div_ow.div(rem);
        const int ow = rem - oh * p.ow;
        pix = (img * p.h + oh * p.stride_h) * p.w_ + ow * p.stride_w;
      }
      st[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, (unsigned)pix * (unsigned)K + 16u * sq, 0, 0);
    }
  };
  auto commit_block = [&]() {
#pragma unroll
    for (int i = 0; i < G::NI; ++i)
      *reinterpret_cast<v4i*>(alds + (i * G::RPI + srow) * G::PITCH + 16 * sq) = st[i];
  };

  // The lane's 32 addend codes of an item are fetched one item ahead: a load issued in the item that
  // uses it would expose its whole latency (the MFMAs of a short reduction hide none of it), and a
  // load in the epilogue would, the memory counter being in order, also wait for the stores before it.
  v4i addn[2];
  auto fetch_addend = [&](int item) {
    const int rbx = range.div_ngc.div(item);
    const int ngx = item - rbx * range.ngc;
    const unsigned offx = (unsigned)(rbx * 32 + l32) * (unsigned)p.k + (unsigned)(slice * G::BN + ngx * 64 + 32 * lh);
    addn[0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_add, offx, 0, 0);
    addn[1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_add, offx + 16u, 0, 0);
  };

  // the first block's loads go out before the filter slice's, so both latencies overlap
  const bool has_work = it < it_end;
  if (has_work) fetch_block(range.div_ngc.div(it));
  if (ADD && has_work) fetch_addend(it);

  // ---- filter slice -> LDS in MFMA row order.  The slice is one contiguous run of the [k][C]
  // filter; rows past the last output channel lie past the end of the tensor and the range-checked
  // loads return zeros.
  {
    constexpr int V4_PER_ROW = K / 16;
    constexpr int PASSES = G::BN * V4_PER_ROW / PWQ_THREADS;
    const unsigned base = (unsigned)slice * (unsigned)(G::BN * K);
    v4i stage[PASSES];
#pragma unroll
    for (int q = 0; q < PASSES; ++q)
      stage[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, base + (unsigned)(tid + q * PWQ_THREADS) * 16u, 0, 0);
#pragma unroll
    for (int q = 0; q < PASSES; ++q) {
      const int i = tid + q * PWQ_THREADS;
      const int ch = i / V4_PER_ROW, kq = i % V4_PER_ROW;
      const int row = (ch & ~63) + staged_row(ch & 63);
      *reinterpret_cast<v4i*>(wlds + row * G::PITCH + kq * 16) = stage[q];
    }
  }
  __syncthreads();
  // every value a quantized addend can contribute: 256 codes, so the 64-bit rescale is done once per
  // code here instead of once per output in the epilogue
  if (ADD && tid < 256) addlut[tid] = rescale_term((int)(signed char)tid - p.r_off, p.r_mant, p.r_shift);
  // per-channel additive term, combined modulo 2^32 (the true accumulator fits int32 by contract)
  if (tid < G::BN) {
    const int ch = slice * G::BN + tid;
    const unsigned char* wrow = wlds + ((tid & ~63) + staged_row(tid & 63)) * G::PITCH;
    int wsum = 0;
#pragma unroll
    for (int j = 0; j < K / 16; ++j) {
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

  const unsigned char* a_lane = alds + l32 * G::PITCH + 16 * lh;
  const unsigned char* w_lane = wlds + l32 * G::PITCH + 16 * lh;
  const bool fast = p.shift >= 33;                         // uniform
  const FoldedRequant fold = make_folded_requant(p.shift, p.y_off);   // uniform
  const int lo_v = p.lo;

  commit_block();
  while (it < it_end) {
    const int rb = range.div_ngc.div(it);
    int rb_items_end = (rb + 1) * range.ngc;
    const bool has_next = rb_items_end < it_end;           // this wavefront also owns (part of) block rb+1
    if (!has_next) rb_items_end = it_end;
    if (has_next) fetch_block(rb + 1);                     // in flight during all items of this block

    for (; it < rb_items_end; ++it) {
      const int ng = it - rb * range.ngc;
      const int ch0 = slice * G::BN + ng * 64 + 32 * lh;   // first of the lane's 32 channels
      const unsigned off = (unsigned)(rb * 32 + l32) * (unsigned)p.k + (unsigned)ch0;
      v4i addq[2];
      if (ADD) {
        addq[0] = addn[0];
        addq[1] = addn[1];
        if (it + 1 < it_end) fetch_addend(it + 1);
      }
      // the accumulators start at the channel terms: register e of acc<nb> = channel 32*lh + 16*nb + e
      v16i acc0, acc1;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const v4i c0 = *reinterpret_cast<const v4i*>(cterm + ng * 64 + 32 * lh + 4 * q4);
        const v4i c1 = *reinterpret_cast<const v4i*>(cterm + ng * 64 + 32 * lh + 16 + 4 * q4);
#pragma unroll
        for (int t = 0; t < 4; ++t) { acc0[4 * q4 + t] = c0[t]; acc1[4 * q4 + t] = c1[t]; }
      }
      const unsigned char* wl = w_lane + ng * 64 * G::PITCH;
#pragma unroll
      for (int s = 0; s < G::STEPS; ++s) {
        // each lane feeds 16 consecutive codes of its row; lanes 32..63 take the upper 16 of the 32
        const v4i a = *reinterpret_cast<const v4i*>(a_lane + 32 * s);
        const v4i b0 = *reinterpret_cast<const v4i*>(wl + 32 * s);
        const v4i b1 = *reinterpret_cast<const v4i*>(wl + 32 * G::PITCH + 32 * s);
        acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b0, a, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b1, a, acc1, 0, 0, 0);
      }

      // ---- epilogue: lane (l32, lh) holds pixel l32, channels 32*lh + 16*nb + e of the group
      auto finish = [&](auto mode_tag) {
        constexpr int MODE = decltype(mode_tag)::value;    // 2 folded, 1 multiply-high, 0 64-bit
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
    if (has_next) commit_block();                          // after this block's fragment reads, in order
  }
}

template <int K, bool CONTIGUOUS, bool ADD>
hipError_t launch_pwq(const Problem& p, hipStream_t stream) {
  using G = PwQ<K>;
  auto kern = conv_pw_i8_kernel<K, CONTIGUOUS, ADD>;
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
  long long wgs = (long long)num_cu * G::WG_PER_CU / slices;          // persistent workgroups per slice
  if (wgs < 1) wgs = 1;
  const long long items_max = (long long)row_blocks * groups_full;
  if (wgs > (items_max + PWQ_WAVES - 1) / PWQ_WAVES) wgs = (items_max + PWQ_WAVES - 1) / PWQ_WAVES;
  const long long waves = wgs * PWQ_WAVES;
  dim3 grid((unsigned)wgs, (unsigned)slices, 1), block(PWQ_THREADS, 1, 1);
  hipLaunchKernelGGL(kern, grid, block, G::lds_bytes, stream, p, make_pw_range(row_blocks, groups_full, waves),
                     make_pw_range(row_blocks, groups_last, waves));
  return hipGetLastError();
}

int pwq_min_items() {
  return knob_or(KNOB_I8_PW_MIN_ITEMS, 1024);   // the knob: experiments and tests
}

}  // namespace

bool pw_i8_applicable(const Problem& p) {
  if (p.b_is_kn || p.groups != 1 || p.r != 1 || p.s != 1 || p.pad_t != 0 || p.pad_l != 0) return false;
  if (p.c != 64 && p.c != 128 && p.c != 256) return false;
  if (p.w_off != 0 || p.k % 16 != 0) return false;
  // bottom/right padding would make output pixels read outside the image
  if ((long long)(p.oh - 1) * p.stride_h >= p.h || (long long)(p.ow - 1) * p.stride_w >= p.w_) return false;
  if ((unsigned long long)p.M * (unsigned long long)p.k > 0xF0000000ull || p.k > 65536) return false;
  if (p.w_bytes > 0x7FFFFFFFu) return false;
  // enough (pixel block, 64-channel group) items over all filter slices to keep the persistent workgroups
  // busy (measured: 1x1 256->1024 on 14x14 at batch 32, 196 blocks x 8 slices of two groups, 11.3 us with
  // the wide kernel -> 8.0 us here)
  const long long items = (long long)((p.M + 31) / 32) * ((p.k + 63) / 64);
  return items >= pwq_min_items() && items < (1LL << 30);
}

template <int K>
hipError_t launch_pwq_k(const Problem& p, hipStream_t stream) {
  const bool contiguous = p.stride_h == 1 && p.stride_w == 1;
  if (p.addend) return contiguous ? launch_pwq<K, true, true>(p, stream) : launch_pwq<K, false, true>(p, stream);
  return contiguous ? launch_pwq<K, true, false>(p, stream) : launch_pwq<K, false, false>(p, stream);
}

hipError_t launch_pw_i8(const Problem& p, hipStream_t stream, const char** variant) {
  const bool contiguous = p.stride_h == 1 && p.stride_w == 1;
  static thread_local char name[48];
  snprintf(name, sizeof(name), "conv_pw_i8_c%d%s%s", p.c, contiguous ? "" : "_strided", p.addend ? "_add" : "");
  *variant = name;
  switch (p.c) {
    case 64: return launch_pwq_k<64>(p, stream);
    case 128: return launch_pwq_k<128>(p, stream);
    case 256: return launch_pwq_k<256>(p, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace glowmi
