// fp32 FullyConnected with few rows (batch 1..64) in ONE launch with one pass over the weights.
//
// Section 3.4 of the paper lowers FullyConnected to a matrix multiplication followed by a broadcasted
// add; with a handful of rows the layer is a stream of the weight matrix through the chip, and what it
// costs beyond that stream is latency: kernels that follow each other on a stream, and dependent
// memory round trips inside a kernel.  The tiled kernels split the reduction over workgroups and
// finish in a second kernel; here a column strip of the output is owned by one workgroup and the
// reduction is split over its sixteen wavefronts instead, summed through LDS in a fixed order:
//
//   - workgroup = (strip of 16 * VW output columns, block of 16 rows); strips narrow enough that a
//     matrix with N = 1000..4096 columns still gives every CU (or at least a quarter of them, which is
//     enough L2 -> CU bandwidth for a few megabytes) a workgroup.  Neighbouring strips read the two
//     halves of the same cache lines; consecutive strips go to the same XCD, so the second reader finds
//     the line in that XCD's L2;
//   - a wavefront owns a contiguous range of 16-row steps of the reduction.  Lane (c, q) loads
//     W[k0 + 4q + t][n0 + VW c ..] for t = 0..3 straight into MFMA operand layout (no LDS staging) and
//     the float4 A[row c][k0 + 4q ..]; v_mfma_f32_16x16x4_f32 (t, j) multiplies reduction index
//     k0 + 4q + t into column n0 + VW c + j.  Loads run a chunk of steps ahead of the MFMAs in a second
//     register set, so a wavefront pays one memory latency, not one per step;
//   - every load is a range-checked buffer load: rows past K, columns past N and rows past M read zeros,
//     so ragged shapes need no branches;
//   - the sixteen partial results are summed through LDS in wavefront order (deterministic), then
//     bias + activation, one store.
#include <hip/hip_runtime.h>

#include "igemm.h"

namespace glowmi {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

constexpr int FSF_WAVES = 16;
constexpr int FSF_THREADS = 64 * FSF_WAVES;
constexpr int FSF_STEP = 16;                 // reduction indices per step

template <int VW> struct VecOf;
template <> struct VecOf<1> { typedef float type; };
template <> struct VecOf<2> { typedef v2f type; };
template <> struct VecOf<4> { typedef v4f type; };

template <int VW>
__device__ __forceinline__ typename VecOf<VW>::type load_w(__amdgpu_buffer_rsrc_t rsrc, unsigned off) {
  if constexpr (VW == 1) return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, 0, 0));
  else if constexpr (VW == 2) return __builtin_bit_cast(v2f, __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, 0, 0));
  else return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0));
}

template <int VW>
__device__ __forceinline__ float elem(const typename VecOf<VW>::type& v, int j) {
  if constexpr (VW == 1) return v;
  else return v[j];
}

template <int VW>
__global__ __launch_bounds__(FSF_THREADS) void fc_small_f32_kernel(const Problem p, int strips, int steps_per_wave) {
  constexpr int U = 4 / VW < 1 ? 1 : 4 / VW;       // steps per chunk: 16 weight registers per set
  constexpr int COLS = 16 * VW;
  typedef typename VecOf<VW>::type wvec;
  __shared__ float red[FSF_WAVES * VW * 4 * 64];

  // consecutive strips on one XCD (workgroup ids go round-robin over the 8 XCDs)
  const int per_xcd = gridDim.x >> 3;
  const int strip = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (strip >= strips) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, q = lane >> 4;
  const int n0 = strip * COLS;
  const int m0 = blockIdx.y * 16;
  const int K = p.Kgemm, N = p.k, M = p.M;

  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_a =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  constexpr unsigned OOB = 0xFFFFFF00u;            // beyond any tensor this library accepts

  const int col = n0 + c * VW;
  const bool col_ok = col < N;                     // N % VW == 0: the whole vector is inside or outside
  const bool row_ok = m0 + c < M;                  // as the A operand lane c holds activation row m0 + c
  const unsigned a_row = (unsigned)(m0 + c) * (unsigned)K;

  const int s_begin = wave * steps_per_wave;
  int s_end = s_begin + steps_per_wave;
  const int total_steps = (K + FSF_STEP - 1) / FSF_STEP;
  if (s_end > total_steps) s_end = total_steps;

  v4f acc[VW];
#pragma unroll
  for (int j = 0; j < VW; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};

  v4f a0[U], a1[U];
  wvec b0[U][4], b1[U][4];
  auto load_chunk = [&](int s0, v4f (&a)[U], wvec (&b)[U][4]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k0 = (s0 + u) * FSF_STEP + 4 * q;            // K % 4 == 0: the lane's four indices are in or out together
      const bool kok = s0 + u < s_end && k0 < K;
      const unsigned aoff = (kok && row_ok) ? (a_row + (unsigned)k0) * 4u : OOB;
      a[u] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, aoff, 0, 0));
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const unsigned woff = (kok && col_ok) ? ((unsigned)(k0 + t) * (unsigned)N + (unsigned)col) * 4u : OOB;
        b[u][t] = load_w<VW>(rsrc_w, woff);
      }
    }
  };
  auto mma_chunk = [&](const v4f (&a)[U], const wvec (&b)[U][4]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int j = 0; j < VW; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][t], elem<VW>(b[u][t], j), acc[j], 0, 0, 0);
  };

  // Two register sets: the loads of the next chunk are in flight while this one is multiplied.  The
  // loads are issued unconditionally (steps past the wavefront's range get the out-of-range offset and
  // cost no memory traffic): a load inside a branch would make the compiler wait for every outstanding
  // load at the join, which serialises the two sets.
  load_chunk(s_begin, a0, b0);
  for (int s = s_begin; s < s_end; s += 2 * U) {
    load_chunk(s + U, a1, b1);
    mma_chunk(a0, b0);
    load_chunk(s + 2 * U, a0, b0);
    mma_chunk(a1, b1);
  }

  // ---- partial results -> LDS; summed in wavefront order by the first VW * 256 threads
#pragma unroll
  for (int j = 0; j < VW; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) red[((wave * VW + j) * 4 + e) * 64 + lane] = acc[j][e];
  __syncthreads();
  const int tid = threadIdx.x;
  if (tid >= VW * 256) return;
  const int idx = tid >> 6;                        // j * 4 + e
  const int j = idx >> 2, e = idx & 3;
  float v = 0.f;
#pragma unroll
  for (int w = 0; w < FSF_WAVES; ++w) v += red[((w * VW + j) * 4 + e) * 64 + lane];
  // 16 x 16 result: register e of lane (c, q) is row 4q + e, column slot c = column n0 + VW c + j
  const int row = m0 + 4 * q + e, ocol = n0 + c * VW + j;
  if (row >= M || ocol >= N) return;
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  if (bias) v += bias[ocol];
  if (p.act == 1) v = fmaxf(v, 0.f);
  static_cast<float*>(p.y)[(size_t)row * N + ocol] = v;
}

template <int VW>
hipError_t launch_fsf(const Problem& p, hipStream_t stream) {
  constexpr int COLS = 16 * VW;
  const int strips = (p.k + COLS - 1) / COLS;
  const int total_steps = (p.Kgemm + FSF_STEP - 1) / FSF_STEP;
  const int steps_per_wave = (total_steps + FSF_WAVES - 1) / FSF_WAVES;
  dim3 grid((unsigned)(((strips + 7) / 8) * 8), (unsigned)((p.M + 15) / 16), 1), block(FSF_THREADS, 1, 1);
  hipLaunchKernelGGL(fc_small_f32_kernel<VW>, grid, block, 0, stream, p, strips, steps_per_wave);
  return hipGetLastError();
}

// Strip width in units of 16 columns: the widest loads that still give about three quarters of the CUs
// a workgroup (wider strips read whole cache lines per row; narrower ones reach more CUs).
int pick_vw(const Problem& p) {
  const int forced = knob_or(KNOB_F32_FC_SMALL_VW, 0);
  if ((forced == 4 && p.k % 4 == 0) || (forced == 2 && p.k % 2 == 0) || forced == 1) return forced;
  const int row_blocks = (p.M + 15) / 16;
  if (p.k % 4 == 0 && (long long)((p.k + 63) / 64) * row_blocks >= 192) return 4;
  if (p.k % 2 == 0 && (long long)((p.k + 31) / 32) * row_blocks >= 192) return 2;
  return 1;
}

}  // namespace

bool fc_small_f32_applicable(const Problem& p) {
  if (!p.b_is_kn || p.groups != 1 || p.addend || p.chain_n > 0) return false;
  if (knob_or(KNOB_F32_FC_SMALL_OFF, 0) != 0) return false;
  if (p.M > 64 || p.Kgemm % 4 != 0 || p.Kgemm < 64) return false;
  // One workgroup per column strip pulls its strip of the matrix at the rate ONE CU sustains from
  // memory: about 45 GB/s when the weights are resident in the last-level cache and a third of that
  // when they come from HBM.  Measured per launch, (rows x K x N): launched back to back on warm weights
  // 1 x 2048 x 1000 8.4 us here vs 11.3 us for the weight-streaming kernel + finishing kernel,
  // 64 x 2048 x 1000 9.5 vs 13.0 us (tiled), 16 x 4096 x 1000 14.5 vs 10.6 us; with the weights cold (other
  // layers in between) 1 x 2048 x 1000 13.1 vs 10.8 us, 64 x 2048 x 1000 15.5 vs 15.0 us.  So up to 16 rows
  // the streaming kernel, which spreads the matrix over every CU, stays the planner's choice (the knob
  // F32_FC_SMALL_MIN_M lowers the bound for tests and experiments); with 17 to 64 rows this kernel
  // replaces the tiled one for matrices of a few megabytes.
  if (p.M < knob_or(KNOB_F32_FC_SMALL_MIN_M, 17)) return false;
  const long long max_kb = knob_or(KNOB_F32_FC_SMALL_MAX_KB, 8704);      // the knob: experiments and tests
  if ((long long)p.w_bytes > (max_kb << 10) || p.w_bytes > 0x7FFFFFFFu || p.x_bytes > 0x7FFFFFFFu) return false;
  return true;
}

hipError_t launch_fc_small_f32(const Problem& p, hipStream_t stream, const char** variant) {
  switch (pick_vw(p)) {
    case 4: *variant = "fc_small_f32_w64"; return launch_fsf<4>(p, stream);
    case 2: *variant = "fc_small_f32_w32"; return launch_fsf<2>(p, stream);
    default: *variant = "fc_small_f32_w16"; return launch_fsf<1>(p, stream);
  }
}

}  // namespace glowmi
