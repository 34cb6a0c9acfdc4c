// fp32 Convolution on few output pixels with a short reduction (the batch-1 layers of a network's
// early stages: a few thousand pixels, reduction r*s*c of a few hundred): the contraction the
// paper's lowering reduces the layer to (Section 3.4) with bias and Relu applied to the
// accumulators (operator stacking, Section 5.2).
//
// Such a layer is a few megaflops: what it costs is latency.  As an output-tiled GEMM it is either too
// few workgroups walking the reduction slab by slab (a chain of dependent memory round trips), or a
// split reduction with a second kernel that sums the partial tiles.  Here it is ONE launch with one
// memory round trip:
//   - a workgroup owns 32 output pixels x 32 output channels; its eight wavefronts split the
//     reduction in groups of 8 consecutive reduction indices (a group lies inside one filter tap:
//     c % 8 == 0) and every wavefront issues all loads of its groups at once, before touching any;
//   - no LDS staging: a lane loads float4 pieces of its pixel's input run and of its channel's filter
//     row straight into MFMA operand layout (v_mfma_f32_32x32x2_f32: lanes 0..31 and 32..63 hold the
//     two reduction indices of a step; with float4 loads at k and k + 4 the four steps of a group pair
//     index k + t with k + 4 + t, the same pairing for both operands);
//   - taps outside the image and rows past M / channels past k load from an offset past the tensor:
//     the range-checked loads return zeros;
//   - the filter is the row operand, so a lane ends with groups of four consecutive channels of one
//     pixel; the eight partial results are summed through LDS in wavefront order, then bias, Relu,
//     one 16-byte store per group.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "igemm.h"

namespace glowmi {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int CS_WAVES = 8;
constexpr int CS_THREADS = 64 * CS_WAVES;
constexpr int CS_MAXG = 10;                     // groups of 8 reduction indices per wavefront

template <int G>
__global__ __launch_bounds__(CS_THREADS, 1) void conv_small_f32_kernel(const Problem p, int groups_total,
                                                                       int groups_per_split) {
  __shared__ float part[CS_WAVES * 16 * 64];    // partial accumulators [wave][register][lane]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int m = blockIdx.x * 32 + l32;          // this lane's output pixel (as the column operand)
  const int n0 = blockIdx.y * 32;
  const int ch = n0 + l32;                      // this lane's output channel (as the row operand)

  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);
  constexpr unsigned OOB = 0x80000000u;         // tensors are below 2 GiB: past the end, the load returns zeros

  // pixel -> window origin
  int ih0 = 0, iw0 = 0;
  unsigned pix_base = 0;
  const bool m_ok = m < p.M;
  if (m_ok) {
    const int img = p.div_ohow.div(m);
    const int rem = m - img * (p.oh * p.ow);
    const int oh = p.div_ow.div(rem);
    const int ow = rem - oh * p.ow;
    ih0 = oh * p.stride_h - p.pad_t;
    iw0 = ow * p.stride_w - p.pad_l;
    pix_base = (unsigned)(((img * p.h + ih0) * p.w_ + iw0) * p.c) * 4u;   // may wrap below 0: only used with an inside tap
  }
  const unsigned w_base = ch < p.k ? (unsigned)ch * (unsigned)p.Kgemm * 4u : OOB;

  // ---- all loads of this wavefront's groups
  // blockIdx.z: which slice of the reduction this workgroup takes when it is split over the grid
  const int g_split_end = (blockIdx.z + 1) * groups_per_split < groups_total ? (blockIdx.z + 1) * groups_per_split : groups_total;
  const int g_begin = blockIdx.z * groups_per_split + wave * G;
  v4f a[G], b[G];
#pragma unroll
  for (int i = 0; i < G; ++i) {
    const int g = g_begin + i;
    const int kk = g * 8;                        // first reduction index of the group
    const int tap = p.div_cg.div(kk);            // groups == 1: cg == c
    const int c0 = kk - tap * p.c;
    const int r = p.div_s.div(tap);
    const int s = tap - r * p.s;
    const bool inside = g < g_split_end && m_ok && (unsigned)(ih0 + r) < (unsigned)p.h &&
                        (unsigned)(iw0 + s) < (unsigned)p.w_;
    const unsigned xoff = pix_base + (unsigned)(((r * p.w_ + s) * p.c + c0 + 4 * lh) * 4);
    a[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, inside ? xoff : OOB, 0, 0));
    const unsigned woff = w_base + (unsigned)((kk + 4 * lh) * 4);
    b[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(
                                       rsrc_w, (g < g_split_end && w_base != OOB) ? woff : OOB, 0, 0));
  }

  v16f acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
  for (int i = 0; i < G; ++i)
#pragma unroll
    for (int t = 0; t < 4; ++t)   // filter fragment as the row operand: result rows = channels, columns = pixels
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(b[i][t], a[i][t], acc, 0, 0, 0);

  // ---- partial results -> LDS, summed by wavefront 0 in wavefront order
#pragma unroll
  for (int e = 0; e < 16; ++e) part[(wave * 16 + e) * 64 + lane] = acc[e];
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int w = 1; w < CS_WAVES; ++w)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] += part[(w * 16 + e) * 64 + lane];

  // register e of lane (l32, lh) is channel n0 + (e/4)*8 + 4*lh + e%4 of pixel m
  if (m >= p.M) return;
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  float* __restrict__ Y = static_cast<float*>(p.y);
  const bool split = gridDim.z > 1;              // partial sums go to the workspace, the finishing kernel does the rest
  float* __restrict__ P = static_cast<float*>(p.partial) + (size_t)blockIdx.z * p.M * p.k;
#pragma unroll
  for (int g4 = 0; g4 < 4; ++g4) {
    const int c0 = n0 + 8 * g4 + 4 * lh;
    if (c0 >= p.k) continue;                     // k % 4 == 0: a group of four channels is whole or absent
    v4f v = {acc[4 * g4], acc[4 * g4 + 1], acc[4 * g4 + 2], acc[4 * g4 + 3]};
    if (split) {
      *reinterpret_cast<v4f*>(P + (size_t)m * p.k + c0) = v;
      continue;
    }
    if (bias) v += v4f{bias[c0], bias[c0 + 1], bias[c0 + 2], bias[c0 + 3]};   // bias is only 4-byte aligned
    if (p.act == 1) {
#pragma unroll
      for (int t = 0; t < 4; ++t) v[t] = fmaxf(v[t], 0.f);
    }
    *reinterpret_cast<v4f*>(Y + (size_t)m * p.k + c0) = v;
  }
}

int cs_max_tiles() {
  // the knob: experiments and tests
  return knob_or(KNOB_F32_SMALL_MAX_TILES, 512);
  // measured: 196 tiles 11.0 -> 5.5 us and 12.9 -> 8.3 us, 392 tiles 12.4 -> 8.2 us, 784 tiles 27.0 -> 26.2 us
}

template <int G>
hipError_t launch_cs(const Problem& p, hipStream_t stream, int groups_total, int groups_per_split, int splits) {
  dim3 grid((unsigned)((p.M + 31) / 32), (unsigned)((p.k + 31) / 32), (unsigned)splits), block(CS_THREADS, 1, 1);
  hipLaunchKernelGGL(conv_small_f32_kernel<G>, grid, block, 0, stream, p, groups_total, groups_per_split);
  return hipGetLastError();
}

bool shape_ok(const Problem& p) {
  if (p.b_is_kn || p.groups != 1) return false;
  if (p.c % 8 != 0 || p.k % 4 != 0) return false;
  return p.x_bytes <= 0x7FFFFFFFu && p.w_bytes <= 0x7FFFFFFFu;
}

}  // namespace

bool conv_small_f32_applicable(const Problem& p) {
  if (!shape_ok(p) || p.addend) return false;
  // eight wavefronts x up to CS_MAXG groups of 8; with fewer than two groups per wavefront the generic
  // kernel is as fast (measured: 1x1 64->256 on 56x56, one group each, 7.8 vs 7.2 us)
  if (p.Kgemm > 8 * CS_WAVES * CS_MAXG || p.Kgemm < 8 * CS_WAVES * 2) return false;
  const long long tiles = (long long)((p.M + 31) / 32) * ((p.k + 31) / 32);
  return tiles <= cs_max_tiles();
}

// The same kernel with the reduction also split over the grid, for the deep reductions on very few
// pixels (3x3 512->512 on a 7x7 map at batch 1): slices of at most 8 x CS_WAVES x 9 reduction indices,
// partial sums to the workspace, the generic finishing kernel sums them in split order.  Returns the
// number of slices, 0 if the layer is not of that kind.
int conv_small_f32_splits(const Problem& p) {
  if (!shape_ok(p) || p.Kgemm <= 8 * CS_WAVES * CS_MAXG) return 0;
  if (knob_or(KNOB_F32_SMALL_NO_SPLIT, 0) != 0) return 0;     // experiments
  const long long tiles = (long long)((p.M + 31) / 32) * ((p.k + 31) / 32);
  const int groups_total = p.Kgemm / 8;
  const int per_split = CS_WAVES * 9;
  const int splits = (groups_total + per_split - 1) / per_split;
  // enough workgroups to pull the filter through many CUs at once, few enough that the partial sums
  // (splits x M x k floats, written and read once) stay small next to the filter itself
  int min_wgs = 64, max_tiles = 128;
  max_tiles = knob_or(KNOB_F32_SMALL_SPLIT_MAX_TILES, max_tiles);   // experiments
  min_wgs = knob_or(KNOB_F32_SMALL_MIN_WGS, min_wgs);               // experiments and tests
  // (measured: 3x3 512->512 on 7x7 at batch 1, 256 workgroups: 16.2 -> 10.6 us; 3x3 128->128 on 28x28, 200:
  // 13.6 -> 10.4 us; 1x1 1024->256 on 14x14, 112: 11.1 -> 10.1 us; 3x3 512->512 on 7x7 at batch 4, 896: 27.7 -> 29.3 us)
  if (tiles > max_tiles || tiles * splits < min_wgs || tiles * splits > 512 || splits > 64) return 0;
  return splits;
}

hipError_t launch_conv_small_f32(const Problem& p, hipStream_t stream, const char** variant) {
  const int groups_total = p.Kgemm / 8;
  if (p.split_k > 1) {
    *variant = "conv_small_f32_splitk";
    return launch_cs<9>(p, stream, groups_total, CS_WAVES * 9, p.split_k);
  }
  *variant = "conv_small_f32";
  const int per_wave = (groups_total + CS_WAVES - 1) / CS_WAVES;
  switch (per_wave) {
    case 1: return launch_cs<1>(p, stream, groups_total, groups_total, 1);
    case 2: return launch_cs<2>(p, stream, groups_total, groups_total, 1);
    case 3: case 4: return launch_cs<4>(p, stream, groups_total, groups_total, 1);
    case 5: case 6: return launch_cs<6>(p, stream, groups_total, groups_total, 1);
    case 7: case 8: return launch_cs<8>(p, stream, groups_total, groups_total, 1);
    default: return launch_cs<CS_MAXG>(p, stream, groups_total, groups_total, 1);
  }
}

}  // namespace glowmi
