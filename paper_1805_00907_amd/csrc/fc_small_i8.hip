// int8 FullyConnected with few rows (batch 1..64) and a reduction of a few thousand: the quantized
// form of Section 4 of the paper (int8 codes with scale/offset, int32 accumulation, rescale folded
// into the producer) for the layer that the lowering of Section 3.4 turns into MatMul + BatchedAdd.
//
// Such a layer is a few megabytes of weights and a few million multiply-accumulates: what it costs
// is latency.  Tiled over the output with the reduction split over workgroups it needs a second
// kernel to sum the partial tiles, and two dependent kernels plus their memory round trips are most
// of its time.  Here it is ONE launch with one memory round trip:
//   - a workgroup owns a strip of 32 output columns and a block of 32 rows; its eight wavefronts
//     split the reduction, 256 weight rows each per pass, and every wavefront issues all loads of
//     its slice at once (eight 16-byte loads per lane of weights, eight of activations) before
//     touching any;
//   - the weight slice [k][32 columns] goes into a private LDS region as it lies in memory, and the
//     K-contiguous MFMA fragments are read from it with the transposing load ds_read_b64_tr_b8 (within
//     16 lanes, result byte e of lane i is byte i%8 of the 8 bytes addressed by lane 2e + i/8);
//     the activation fragments (K-contiguous rows) come straight from global memory;
//   - v_mfma_i32_32x32x32_i8 with the weight fragment as the row operand: a lane ends with groups of
//     four consecutive output columns of one row; raw codes are multiplied and the offsets removed
//     afterwards with per-column / per-row code sums taken from the fragments (v_dot4);
//   - the eight partial results are summed through LDS in a fixed order, then bias, requantize,
//     clamp (Relu = lower bound), pack, one 4-byte store per group.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "igemm.h"
#include "quant_epilogue.h"

namespace glowmi {
namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int FS_WAVES = 8;
constexpr int FS_THREADS = 64 * FS_WAVES;
constexpr int FS_COLS = 32;                      // output columns per workgroup
constexpr int FS_KW = 256;                       // weight rows per wavefront and pass
constexpr int FS_STEPS = FS_KW / 32;             // MFMA steps per pass
constexpr int FS_WLOADS = FS_KW * FS_COLS / (64 * 16);   // 16-byte weight loads per lane and pass
constexpr int FS_PITCH = FS_COLS;                // bytes per staged weight row
constexpr int FS_REGION = FS_KW * FS_PITCH;      // bytes per wavefront: its weight slice, later its partial sums
static_assert(2 * 16 * 64 * 4 <= FS_REGION, "a wavefront's partial accumulators fit its region");

__device__ __forceinline__ int sum4(int packed, int acc) {
  return __builtin_amdgcn_sdot4(packed, 0x01010101, acc, false);
}

// MB: 32-row blocks of the activation matrix per workgroup (instantiated with 1).
template <int MB>
__global__ __launch_bounds__(FS_THREADS, 1) void fc_small_i8_kernel(const Problem p) {
  extern __shared__ __align__(16) unsigned char lds[];     // the wavefronts' regions, then the code sums
  int* wsum = reinterpret_cast<int*>(lds + FS_WAVES * FS_REGION);   // [32] sum over k of W[k][n0 + c]
  int* xsum = wsum + FS_COLS;                                        // [64] sum over k of A[m][k]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lrow = lane & 31, lhalf = lane >> 5;
  const int n0 = blockIdx.x * FS_COLS;
  const int m0 = blockIdx.y * (32 * MB);                  // first activation row of this workgroup
  const int K = p.Kgemm, N = p.k, M = p.M;
  unsigned char* region = lds + wave * FS_REGION;

  const __amdgpu_buffer_rsrc_t rsrc_a =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, (int)p.w_bytes, 0x00020000);

  if (tid < FS_COLS) wsum[tid] = 0;
  if (tid < 64) xsum[tid] = 0;

  v16i acc[MB];
#pragma unroll
  for (int b = 0; b < MB; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[b][e] = 0;
  int wacc = 0, xacc[MB];
#pragma unroll
  for (int b = 0; b < MB; ++b) xacc[b] = 0;

  // Weight staging: load i of a lane covers row 32i + lane/2 of the slice, 16 columns at 16*(lane%2).
  // Fragment reads (per 16-lane group: columns 16*cb .. +15 of the strip, reduction half lhalf): lane i16
  // addresses 8 bytes of row 16*lhalf + 8u + i16/2 (u = 0, 1) at columns 16*cb + 8*(i16%2) and receives
  // the 8 codes of column 16*cb + i16 for rows 16*lhalf + 8u .. +7.
  const int srow = lane >> 1, scol = 16 * (lane & 1);
  const int i16 = lane & 15, cb = (lane >> 4) & 1;
  const unsigned frag_off = (unsigned)((16 * lhalf + (i16 >> 1)) * FS_PITCH + 16 * cb + 8 * (i16 & 1));

  const int passes = (K + FS_WAVES * FS_KW - 1) / (FS_WAVES * FS_KW);
  for (int pass = 0; pass < passes; ++pass) {
    const int k0 = (pass * FS_WAVES + wave) * FS_KW;       // first weight row of this wavefront's slice
    // ---- all loads of the slice.  Rows at or past K lie past the end of the weight tensor (zeros).
    // A 16-byte run that would straddle the end of the tensor (last row of the last strip when N is
    // not a multiple of 16) is fetched from the last 16 bytes instead and shifted when it is stored.
    v4i wv[FS_WLOADS];
    unsigned wshift = 0;                                   // 2 bits per load: dwords to shift down
#pragma unroll
    for (int i = 0; i < FS_WLOADS; ++i) {
      const unsigned off = (unsigned)(k0 + 32 * i + srow) * (unsigned)N + (unsigned)(n0 + scol);
      const unsigned last = p.w_bytes - 16u;
      const bool straddle = off > last && off < p.w_bytes;
      wshift |= (straddle ? (off - last) >> 2 : 0u) << (2 * i);
      wv[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, straddle ? last : off, 0, 0);
    }
    v4i av[FS_STEPS][MB];
#pragma unroll
    for (int s = 0; s < FS_STEPS; ++s)
#pragma unroll
      for (int b = 0; b < MB; ++b) {
        const int m = m0 + 32 * b + lrow, k = k0 + 32 * s + 16 * lhalf;
        // rows past M and codes past K: an offset past the end, the range-checked load returns zeros
        const unsigned off = (m < M && k < K) ? (unsigned)m * (unsigned)K + (unsigned)k : 0x80000000u;
        av[s][b] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, off, 0, 0);
      }
    // ---- weights -> the wavefront's LDS region, as they lie in memory
#pragma unroll
    for (int i = 0; i < FS_WLOADS; ++i) {
      v4i v = wv[i];
      const unsigned sh = (wshift >> (2 * i)) & 3u;
      if (sh) {                                            // rare: shift down by sh dwords, zeros from above
        const int d[8] = {v[0], v[1], v[2], v[3], 0, 0, 0, 0};
        v = v4i{sh == 1 ? d[1] : sh == 2 ? d[2] : d[3], sh == 1 ? d[2] : sh == 2 ? d[3] : 0, sh == 1 ? d[3] : 0, 0};
      }
      *reinterpret_cast<v4i*>(region + (32 * i + srow) * FS_PITCH + scol) = v;
    }
    // (a wavefront's LDS operations execute in order: no barrier between its own writes and reads)
#pragma unroll
    for (int s = 0; s < FS_STEPS; ++s) {
      const unsigned char* q = region + 32 * s * FS_PITCH + frag_off;
      const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(q));
      const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(q + 8 * FS_PITCH));
      const v4i bw = {lo[0], lo[1], hi[0], hi[1]};         // column n0 + lrow, rows k0 + 32s + 16*lhalf .. +15
      wacc = sum4(bw[0], sum4(bw[1], sum4(bw[2], sum4(bw[3], wacc))));
#pragma unroll
      for (int b = 0; b < MB; ++b) {
        // weight fragment as the row operand: result rows = output columns, result columns = activation rows
        acc[b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bw, av[s][b], acc[b], 0, 0, 0);
        xacc[b] = sum4(av[s][b][0], sum4(av[s][b][1], sum4(av[s][b][2], sum4(av[s][b][3], xacc[b]))));
      }
    }
  }

  // ---- code sums and partial results of the eight wavefronts -> LDS
  __syncthreads();                                         // wsum / xsum zeroed; all fragment reads done
  atomicAdd(&wsum[lrow], wacc);
#pragma unroll
  for (int b = 0; b < MB; ++b) atomicAdd(&xsum[32 * b + lrow], xacc[b]);
  int* part = reinterpret_cast<int*>(region);              // [MB][16][64 lanes]
#pragma unroll
  for (int b = 0; b < MB; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) part[(b * 16 + e) * 64 + lane] = acc[b][e];
  __syncthreads();
  if (wave >= MB) return;

  // ---- wavefront b finishes row block b: sum the partials in wavefront order, remove the offsets
  //   sum (a - ao)(w - wo) = sum a*w - ao * sum_k w - wo * sum_k a + K * ao * wo       (modulo 2^32:
  // exact because the true value fits), add the bias, requantize, clamp, pack, store.
  // Register e of lane (lrow, lhalf) is output column n0 + (e/4)*8 + 4*lhalf + e%4 of row 32*b + lrow.
  const int b = wave;
  const int* bias = static_cast<const int*>(p.bias);
  const int m = m0 + 32 * b + lrow;
  const unsigned rowterm = (unsigned)K * (unsigned)(p.x_off * p.w_off) - (unsigned)p.w_off * (unsigned)xsum[32 * b + lrow];
  signed char* __restrict__ Y = static_cast<signed char*>(p.y);
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int c0 = 8 * g + 4 * lhalf;                      // first of four consecutive columns of the strip
    int q[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int e = 4 * g + t;
      unsigned v = 0;
#pragma unroll
      for (int w = 0; w < FS_WAVES; ++w)
        v += (unsigned)reinterpret_cast<const int*>(lds + w * FS_REGION)[(b * 16 + e) * 64 + lane];
      const int n = n0 + c0 + t;
      v += rowterm - (unsigned)p.x_off * (unsigned)wsum[c0 + t];
      if (bias && n < N) v += (unsigned)bias[n];
      q[t] = p.shift >= 33 ? requantize_as<true>((int)v, p.mant, p.shift, p.y_off, p.lo)
                           : requantize_as<false>((int)v, p.mant, p.shift, p.y_off, p.lo);   // uniform
    }
    // N % 4 == 0: a group of four columns is wholly inside or outside
    if (m < M && n0 + c0 < N)
      *reinterpret_cast<unsigned*>(Y + (size_t)m * N + n0 + c0) = pack_codes(q[0], q[1], q[2], q[3]);
  }
}

int fs_max_rows() {
  return knob_or(KNOB_I8_FC_SMALL_MAX_M, 64);   // the knob: experiments and tests
}

}  // namespace

bool fc_small_i8_applicable(const Problem& p) {
  if (!p.b_is_kn || p.groups != 1 || p.addend) return false;
  if (p.M > 64 || p.M > fs_max_rows()) return false;
  if (p.Kgemm % 16 != 0 || p.k % 4 != 0) return false;
  if (p.Kgemm > 8192) return false;                        // longer reductions: the split kernels amortise their second launch
  // larger weight matrices are a bandwidth problem again and the tiled kernels stream them faster
  // (measured: 16 x 4096 x 4096, 16 MB, 12.6 us tiled vs 18.2 us here; 16 x 4096 x 1000, 4 MB, 10.9 vs 9.5 us)
  if (p.w_bytes > (8u << 20)) return false;
  if (p.w_bytes < 16u || p.w_bytes > 0x7FFFFFFFu || p.x_bytes > 0x7FFFFFFFu) return false;
  // 32-bit byte offsets, also for the rows past K that the last pass addresses (and gets zeros for)
  if ((long long)(p.Kgemm + FS_WAVES * FS_KW) * p.k >= (1LL << 32)) return false;
  return true;
}

hipError_t launch_fc_small_i8(const Problem& p, hipStream_t stream, const char** variant) {
  *variant = "fc_small_i8";
  constexpr int lds_bytes = FS_WAVES * FS_REGION + (FS_COLS + 64) * (int)sizeof(int);
  // once; initialisation of a function-local static is thread-safe
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(fc_small_i8_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  if (attr_status != hipSuccess) return attr_status;
  // one workgroup per strip of 32 columns and block of 32 rows (measured with 64 rows: both row blocks
  // in one workgroup 10.5 us, in two workgroups 8.8 us: twice the workgroups in flight, half the loads
  // per lane)
  dim3 grid((unsigned)((p.k + FS_COLS - 1) / FS_COLS), (unsigned)((p.M + 31) / 32), 1), block(FS_THREADS, 1, 1);
  hipLaunchKernelGGL(fc_small_i8_kernel<1>, grid, block, lds_bytes, stream, p);
  return hipGetLastError();
}

}  // namespace glowmi
