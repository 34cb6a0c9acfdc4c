// int8 implicit-GEMM Convolution / FullyConnected for gfx950 (MI355X), the quantized form of
// Section 4 of the paper: int8 codes with per-tensor scale/offset (Section 4.1), int32 accumulation,
// and the rescale to the output range folded into the producing operation (Section 4.3), with Relu
// as a plain integer max against the output offset (same-scale max, Section 4.3).
//
// The matrix cores multiply raw codes (v_mfma_i32_32x32x32_i8).  Offsets are taken out afterwards:
//   sum (x - xo)(w - wo) = sum x*w - xo * sum_k w - wo * sum_k x + Kcount * xo * wo
// where padded taps are staged as the code xo (real value 0), so they cancel exactly.  The row sums
// are collected with dot-product instructions while the tiles are staged.  Everything after the
// accumulator is integer arithmetic, so results are reproducible bit for bit.
//
// Tiling mirrors the fp32 kernel: BM x BN output tile per workgroup of 4 or 8 wavefronts, reduction
// slabs of 128 codes staged in double-buffered LDS as K-contiguous rows of 128 + 16 pad bytes
// (conflict-free ds_read_b128), XCD-aware workgroup order.  The MFMA is issued with the filter
// fragment as its row operand, so a lane ends up with four consecutive output channels of one
// pixel: they are requantized, packed into one dword, transposed through LDS and leave the chip as
// 16-byte stores along the channel axis.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#include "igemm.h"
#include "quant_epilogue.h"

namespace glowmi {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BKQ = 128;                 // codes per reduction slab
constexpr int LDQ = BKQ + 16;            // LDS row pitch in bytes (36 dwords: conflict-free b128 reads)
constexpr int KV = BKQ / 16;             // 16-byte chunks per K-contiguous row
constexpr int INVALID_ROW = -(1 << 24);

struct Tap {
  int r, s, c;
  __device__ void init(int kg, int cg, int S, const FastDiv& dcg, const FastDiv& ds) {
    const int t = dcg.div(kg);
    c = kg - t * cg;
    r = ds.div(t);
    s = t - r * S;
  }
  __device__ void advance(int step, int cg, int S) {
    c += step;
    while (c >= cg) {
      c -= cg;
      if (++s == S) { s = 0; ++r; }
    }
  }
};

__device__ __forceinline__ int sum_bytes(int packed) {   // sum of the four signed bytes
  return __builtin_amdgcn_sdot4(packed, 0x01010101, 0, false);
}

__device__ __forceinline__ int requantize(int acc, int mant, int shift, int y_off, int lo) {
  return shift >= 33 ? requantize_as<true>(acc, mant, shift, y_off, lo)
                     : requantize_as<false>(acc, mant, shift, y_off, lo);   // uniform branch
}

// The ops of a general chain on one int32 accumulator value (quantized form: a scalar multiply only
// changed the scale on the host, bounds are integers on the accumulator's grid, an added tensor's code
// difference is rescaled to the accumulator's current scale).  `off` indexes [M][k] tensors.
__device__ __forceinline__ int apply_chain_i8(const Problem& p, int v, size_t off) {
  for (int o = 0; o < p.chain_n; ++o) {
    const ChainOpDev& op = p.chain[o];
    if (op.kind == CHAIN_ADD_TENSOR)
      v += rescale_term((int)static_cast<const signed char*>(op.tensor)[off] - op.t_off, op.t_mant, op.t_shift);
    else if (op.kind == CHAIN_MAX_SCALAR) v = v < op.ia ? op.ia : v;
    else if (op.kind == CHAIN_CLIP) { v = v < op.ia ? op.ia : v; v = v > op.ib ? op.ib : v; }
  }
  return v;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool VEC, bool B_KN, bool CHAINV = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void igemm_i8_kernel(const Problem p, int tiles_m,
                                                                         int tiles_n, int total_work) {
  constexpr int NTHREADS = 64 * WAVES_M * WAVES_N;
  constexpr int ROWS_PER_PASS = NTHREADS / KV;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "tile shape");
  static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile rows per pass");
  constexpr int A_PASSES = BM / ROWS_PER_PASS;
  constexpr int B_PASSES = BN / ROWS_PER_PASS;          // K-contiguous filter rows
  constexpr int B_UNITS = (BKQ / 4) * (BN / 4);         // FC weight: 4k x 4n byte blocks per slab
  constexpr int B_UPT = B_UNITS / NTHREADS;             // blocks per thread
  static_assert(B_UNITS % NTHREADS == 0, "FC weight tile does not divide over the threads");
  constexpr int A_BYTES = BM * LDQ, B_BYTES = BN * LDQ;
  constexpr int OUT_PITCH = BN + 16;                    // output tile staged in LDS, bytes per pixel row
  static_assert(2 * (A_BYTES + B_BYTES) >= BM * OUT_PITCH + (BM + 2 * BN) * 4, "epilogue reuses the staging LDS");

  extern __shared__ __align__(16) unsigned char ldsq[];

  const int per_xcd = gridDim.x >> 3;
  const int w = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (w >= total_work) return;
  const int tn = w % tiles_n;
  int t_ = w / tiles_n;
  const int tm = t_ % tiles_m;
  t_ /= tiles_m;
  const int g = t_ % p.groups;
  const int split = t_ / p.groups;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  const signed char* __restrict__ X = static_cast<const signed char*>(p.x);
  const signed char* __restrict__ Wt = static_cast<const signed char*>(p.w);

  const int kvec = tid % KV;
  const int row0 = tid / KV;
  int a_base[A_PASSES], a_ih0[A_PASSES], a_iw0[A_PASSES];
  {
    const int ohow = p.oh * p.ow;
#pragma unroll
    for (int q = 0; q < A_PASSES; ++q) {
      const int m = tm * BM + row0 + q * ROWS_PER_PASS;
      if (m < p.M) {
        const int img = p.div_ohow.div(m);
        const int rem = m - img * ohow;
        const int oh = p.div_ow.div(rem);
        const int ow = rem - oh * p.ow;
        a_ih0[q] = oh * p.stride_h - p.pad_t;
        a_iw0[q] = ow * p.stride_w - p.pad_l;
        a_base[q] = ((img * p.h + a_ih0[q]) * p.w_ + a_iw0[q]) * p.c + g * p.cg;
      } else {
        a_ih0[q] = INVALID_ROW;
        a_iw0[q] = INVALID_ROW;
        a_base[q] = 0;
      }
    }
  }

  const int slab_begin = split * p.slabs_per_split;
  const int total_slabs = (p.Kgemm + BKQ - 1) / BKQ;
  int slab_end = slab_begin + p.slabs_per_split;
  if (slab_end > total_slabs) slab_end = total_slabs;
  int k_hi = slab_end * BKQ;
  if (k_hi > p.Kgemm) k_hi = p.Kgemm;
  const int k_count = k_hi - slab_begin * BKQ;          // codes this split really reduces over

  Tap tap;
  tap.init(slab_begin * BKQ + kvec * 16, p.cg, p.s, p.div_cg, p.div_s);

  const int xo_byte = p.x_off & 0xff;
  const int xo_fill = xo_byte * 0x01010101;             // padding = the code of real zero
  const bool need_xsum = p.w_off != 0;

  v4i ra[A_PASSES];
  v4i rb[B_KN ? B_UPT : B_PASSES];
  int asum[A_PASSES];                                   // running sum of staged input codes per row
  int bsum[B_KN ? B_UPT * 4 : B_PASSES];                // running sum of staged filter codes
#pragma unroll
  for (int q = 0; q < A_PASSES; ++q) asum[q] = 0;
#pragma unroll
  for (int q = 0; q < (B_KN ? B_UPT * 4 : B_PASSES); ++q) bsum[q] = 0;

  auto load_global = [&](int slab) {
    const int kg0 = slab * BKQ + kvec * 16;
    if (VEC) {
      const bool kok = kg0 < p.Kgemm;                   // Kgemm % 16 == 0 on this path
      const int tap_off = (tap.r * p.w_ + tap.s) * p.c + tap.c;
#pragma unroll
      for (int q = 0; q < A_PASSES; ++q) {
        const int ih = a_ih0[q] + tap.r, iw = a_iw0[q] + tap.s;
        const bool inside = (unsigned)ih < (unsigned)p.h && (unsigned)iw < (unsigned)p.w_;
        if (!kok) ra[q] = v4i{0, 0, 0, 0};
        else if (inside) ra[q] = *reinterpret_cast<const v4i*>(X + a_base[q] + tap_off);
        else ra[q] = v4i{xo_fill, xo_fill, xo_fill, xo_fill};
      }
    } else {
      Tap t = tap;
#pragma unroll
      for (int q = 0; q < A_PASSES; ++q) ra[q] = v4i{0, 0, 0, 0};
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const bool kok = kg0 + e < p.Kgemm;
        const int tap_off = (t.r * p.w_ + t.s) * p.c + t.c;
#pragma unroll
        for (int q = 0; q < A_PASSES; ++q) {
          const int ih = a_ih0[q] + t.r, iw = a_iw0[q] + t.s;
          const bool inside = (unsigned)ih < (unsigned)p.h && (unsigned)iw < (unsigned)p.w_;
          int v = 0;
          if (kok) v = inside ? ((int)X[a_base[q] + tap_off] & 0xff) : xo_byte;
          ra[q][e >> 2] |= v << ((e & 3) * 8);
        }
        t.advance(1, p.cg, p.s);
      }
    }
    if (!B_KN) {
#pragma unroll
      for (int q = 0; q < B_PASSES; ++q) {
        const int n = tn * BN + row0 + q * ROWS_PER_PASS;
        const bool nok = n < p.kg;
        const signed char* src = Wt + (size_t)(g * p.kg + n) * p.Kgemm + kg0;
        if (VEC) {
          rb[q] = (nok && kg0 < p.Kgemm) ? *reinterpret_cast<const v4i*>(src) : v4i{0, 0, 0, 0};
        } else {
          rb[q] = v4i{0, 0, 0, 0};
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int v = (nok && kg0 + e < p.Kgemm) ? ((int)src[e] & 0xff) : 0;
            rb[q][e >> 2] |= v << ((e & 3) * 8);
          }
        }
      }
    } else {
      // FC weight [Kgemm][k], N contiguous: each thread takes 4 k-rows x 4 columns and transposes
      // the 4x4 byte block so that every column becomes one dword of 4 consecutive k.
#pragma unroll
      for (int q = 0; q < B_UPT; ++q) {
        const int u = tid + q * NTHREADS;
        const int ng = u % (BN / 4), kgp = u / (BN / 4);
        const int col = tn * BN + ng * 4;
        int d[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const int kgr = slab * BKQ + kgp * 4 + kk;
          const signed char* src = Wt + (size_t)kgr * p.k + col;
          if (kgr >= p.Kgemm) d[kk] = 0;
          else if (VEC) d[kk] = col < p.k ? *reinterpret_cast<const int*>(src) : 0;
          else {
            d[kk] = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (col + e < p.k) d[kk] |= ((int)src[e] & 0xff) << (e * 8);
          }
        }
#pragma unroll
        for (int nn = 0; nn < 4; ++nn) {
          int o = 0;
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) o |= ((d[kk] >> (nn * 8)) & 0xff) << (kk * 8);
          rb[q][nn] = o;
        }
      }
    }
  };

  auto store_lds = [&](int buf) {
    unsigned char* As = ldsq + buf * (A_BYTES + B_BYTES);
    unsigned char* Bs = As + A_BYTES;
#pragma unroll
    for (int q = 0; q < A_PASSES; ++q) {
      *reinterpret_cast<v4i*>(As + (row0 + q * ROWS_PER_PASS) * LDQ + kvec * 16) = ra[q];
      if (need_xsum)
        asum[q] += sum_bytes(ra[q][0]) + sum_bytes(ra[q][1]) + sum_bytes(ra[q][2]) + sum_bytes(ra[q][3]);
    }
    if (!B_KN) {
#pragma unroll
      for (int q = 0; q < B_PASSES; ++q) {
        *reinterpret_cast<v4i*>(Bs + (row0 + q * ROWS_PER_PASS) * LDQ + kvec * 16) = rb[q];
        bsum[q] += sum_bytes(rb[q][0]) + sum_bytes(rb[q][1]) + sum_bytes(rb[q][2]) + sum_bytes(rb[q][3]);
      }
    } else {
#pragma unroll
      for (int q = 0; q < B_UPT; ++q) {
        const int u = tid + q * NTHREADS;
        const int ng = u % (BN / 4), kgp = u / (BN / 4);
#pragma unroll
        for (int nn = 0; nn < 4; ++nn) {
          *reinterpret_cast<int*>(Bs + (ng * 4 + nn) * LDQ + kgp * 4) = rb[q][nn];
          bsum[q * 4 + nn] += sum_bytes(rb[q][nn]);
        }
      }
    }
  };

  // acc[i][j]: 32 output channels (rows of the MFMA result) x 32 pixels (columns)
  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

  const int lrow = lane & 31;
  const int lhalf = lane >> 5;

  auto compute = [&](int buf) {
    const unsigned char* As = ldsq + buf * (A_BYTES + B_BYTES);
    const unsigned char* Bs = As + A_BYTES;
#pragma unroll
    for (int k32 = 0; k32 < BKQ / 32; ++k32) {
      // each lane feeds 16 consecutive codes of its row; lanes 32..63 take the upper 16 of the 32
      v4i a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const v4i*>(As + (wm * WTM + i * 32 + lrow) * LDQ + k32 * 32 + lhalf * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = *reinterpret_cast<const v4i*>(Bs + (wn * WTN + j * 32 + lrow) * LDQ + k32 * 32 + lhalf * 16);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)   // filter fragment as the row operand: result rows = channels
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[j], a[i], acc[i][j], 0, 0, 0);
    }
  };

  if (slab_begin < slab_end) {
    load_global(slab_begin);
    store_lds(0);
    __syncthreads();
    int buf = 0;
    for (int slab = slab_begin; slab < slab_end; ++slab) {
      const bool more = slab + 1 < slab_end;
      if (more) {
        tap.advance(BKQ, p.cg, p.s);
        load_global(slab + 1);
      }
      compute(buf);
      if (more) store_lds(buf ^ 1);
      __syncthreads();
      buf ^= 1;
    }
  }

  // ---- epilogue.  LDS (staging buffers are free now):
  //   out   [BM][OUT_PITCH] bytes : requantized tile, pixel-major
  //   xsum  [BM] int, wsum [BN] int : code sums;  cterm [BN] int : per-channel additive term
  unsigned char* out = ldsq;
  int* xsum = reinterpret_cast<int*>(ldsq + BM * OUT_PITCH);
  int* wsum = xsum + BM;
  int* cterm = wsum + BN;
  for (int i = tid; i < BM + BN; i += NTHREADS) xsum[i] = 0;
  __syncthreads();
  if (need_xsum) {
#pragma unroll
    for (int q = 0; q < A_PASSES; ++q) atomicAdd(&xsum[row0 + q * ROWS_PER_PASS], asum[q]);
  }
  if (!B_KN) {
#pragma unroll
    for (int q = 0; q < B_PASSES; ++q) atomicAdd(&wsum[row0 + q * ROWS_PER_PASS], bsum[q]);
  } else {
#pragma unroll
    for (int q = 0; q < B_UPT; ++q) {
      const int u = tid + q * NTHREADS;
      const int ng = u % (BN / 4);
#pragma unroll
      for (int nn = 0; nn < 4; ++nn) atomicAdd(&wsum[ng * 4 + nn], bsum[q * 4 + nn]);
    }
  }
  __syncthreads();
  // The correction terms are combined modulo 2^32 (unsigned): each may exceed the final value, the
  // true accumulator fits int32 by contract, so the wrapped sum is exact.
  const int* __restrict__ bias = static_cast<const int*>(p.bias);
  for (int i = tid; i < BN; i += NTHREADS) {
    const int col = tn * BN + i;
    unsigned ct = (unsigned)k_count * (unsigned)(p.x_off * p.w_off) - (unsigned)p.x_off * (unsigned)wsum[i];
    if (p.split_k == 1 && bias && col < p.kg) ct += (unsigned)bias[g * p.kg + col];
    cterm[i] = (int)ct;
  }
  __syncthreads();

  const signed char* addend = static_cast<const signed char*>(p.addend);   // may be the output itself
  if (p.split_k == 1) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int lr = wm * WTM + i * 32 + lrow;                        // pixel row inside the tile
      const unsigned rowterm = need_xsum ? (unsigned)p.w_off * (unsigned)xsum[lr] : 0u;
      const int row = tm * BM + lr;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int lc = wn * WTN + j * 32 + q4 * 8 + lhalf * 4;      // first of 4 consecutive channels
          const v4i ct = *reinterpret_cast<const v4i*>(cterm + lc);
          unsigned packed = 0;
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            int v = (int)((unsigned)acc[i][j][q4 * 4 + t] + (unsigned)ct[t] - rowterm);
            if (CHAINV) {                                             // general op list
              const int col = tn * BN + lc + t;
              if (row < p.M && col < p.kg) v = apply_chain_i8(p, v, (size_t)row * p.k + g * p.kg + col);
            } else if (addend) {                                      // uniform: tensor-add link of the chain
              const int col = tn * BN + lc + t;
              const int code = (row < p.M && col < p.kg) ? (int)addend[(size_t)row * p.k + g * p.kg + col] : p.r_off;
              v += rescale_term(code - p.r_off, p.r_mant, p.r_shift);
            }
            packed |= ((unsigned)requantize(v, p.mant, p.shift, p.y_off, p.lo) & 0xffu) << (t * 8);
          }
          *reinterpret_cast<unsigned*>(out + lr * OUT_PITCH + lc) = packed;
        }
      }
    }
    __syncthreads();
    // copy out: 16 bytes of one pixel row per thread and pass
    signed char* __restrict__ Y = static_cast<signed char*>(p.y);
    constexpr int CHUNKS = BN / 16;
    const bool wide = (p.kg % 16 == 0) && (p.k % 16 == 0);
    for (int u = tid; u < BM * CHUNKS; u += NTHREADS) {
      const int lr = u / CHUNKS, ch = u % CHUNKS;
      const int row = tm * BM + lr, col = tn * BN + ch * 16;
      if (row >= p.M || col >= p.kg) continue;
      signed char* dst = Y + (size_t)row * p.k + g * p.kg + col;
      const unsigned char* src = out + lr * OUT_PITCH + ch * 16;
      if (wide) {
        *reinterpret_cast<v4i*>(dst) = *reinterpret_cast<const v4i*>(src);
      } else {
        for (int e = 0; e < 16 && col + e < p.kg; ++e) dst[e] = (signed char)src[e];
      }
    }
  } else {
    int* __restrict__ part = static_cast<int*>(p.partial);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int lr = wm * WTM + i * 32 + lrow;
      const int row = tm * BM + lr;
      const unsigned rowterm = need_xsum ? (unsigned)p.w_off * (unsigned)xsum[lr] : 0u;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int lc = wn * WTN + j * 32 + (e >> 2) * 8 + lhalf * 4 + (e & 3);
          const int col = tn * BN + lc;
          if (row >= p.M || col >= p.kg) continue;
          part[((size_t)split * p.M + row) * p.k + g * p.kg + col] =
              (int)((unsigned)acc[i][j][e] + (unsigned)cterm[lc] - rowterm);
        }
      }
    }
  }
}

// A thread owns W consecutive outputs (W = 4 when the row length allows: 16-byte loads of the int32
// partials, one dword of codes stored) and walks the splits eight at a time with the loads in flight
// together.  Integer sums: any order gives the same result.
template <int W>
__global__ __launch_bounds__(256) void splitk_finish_i8(const int* __restrict__ partial,
                                                        const int* __restrict__ bias,
                                                        const signed char* addend, int r_off, int r_mant,
                                                        int r_shift, signed char* y, int total, int k,
                                                        int split_k, int mant, int shift, int y_off,
                                                        int lo) {
  typedef unsigned vec __attribute__((ext_vector_type(W)));
  const int groups = total / W;                      // W divides total (the launcher checks)
  for (int gi = blockIdx.x * blockDim.x + threadIdx.x; gi < groups; gi += gridDim.x * blockDim.x) {
    const size_t i = (size_t)gi * W;
    vec v = {};
    for (int s = 0; s < split_k; s += 8) {
      vec t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int su = s + u < split_k ? s + u : s;
        t[u] = *reinterpret_cast<const vec*>(partial + (size_t)su * total + i);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (s + u < split_k) v += t[u];
    }
    if (bias) v += *reinterpret_cast<const vec*>(bias + i % k);      // W divides k: no wrap inside the vector
    int q[W];
#pragma unroll
    for (int e = 0; e < W; ++e) {
      unsigned a = v[e];
      if (addend) a += (unsigned)rescale_term((int)addend[i + e] - r_off, r_mant, r_shift);
      q[e] = requantize((int)a, mant, shift, y_off, lo);
    }
    if (W == 4) {
      *reinterpret_cast<unsigned*>(y + i) = pack_codes(q[0], q[1], q[2], q[3]);
    } else {
#pragma unroll
      for (int e = 0; e < W; ++e) y[i + e] = (signed char)q[e];
    }
  }
}

// Finish of a split reduction whose element-wise chain is a general op list.
__global__ __launch_bounds__(256) void splitk_finish_chain_i8(const Problem p, int total) {
  const int* __restrict__ partial = static_cast<const int*>(p.partial);
  const int* __restrict__ bias = static_cast<const int*>(p.bias);
  signed char* y = static_cast<signed char*>(p.y);
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    unsigned a = 0;
    for (int s = 0; s < p.split_k; ++s) a += (unsigned)partial[(size_t)s * total + i];
    if (bias) a += (unsigned)bias[i % p.k];
    const int v = apply_chain_i8(p, (int)a, (size_t)i);
    y[i] = (signed char)requantize(v, p.mant, p.shift, p.y_off, p.lo);
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool VEC, bool B_KN, bool CHAINV = false>
hipError_t launch_variant(const Problem& p, const Plan& plan, hipStream_t stream) {
  auto kern = igemm_i8_kernel<BM, BN, WAVES_M, WAVES_N, VEC, B_KN, CHAINV>;
  constexpr int lds_bytes = 2 * (BM + BN) * LDQ;
  constexpr int nthreads = 64 * WAVES_M * WAVES_N;
  // once per instantiation; initialisation of a function-local static is thread-safe
  static const hipError_t attr_status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  if (attr_status != hipSuccess) return attr_status;
  const long long total_work = (long long)plan.tiles_m * plan.tiles_n * p.groups * plan.split_k;
  const long long grid_x = ((total_work + 7) / 8) * 8;
  dim3 grid((unsigned)grid_x, 1, 1), block(nthreads, 1, 1);
  hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, p, plan.tiles_m, plan.tiles_n, (int)total_work);
  return hipGetLastError();
}

struct TileI8 { int bm, bn, wm, wn; const char* name; };
constexpr TileI8 kTilesI8[] = {
    {64, 64, 2, 2, "64x64w4"},       // 0: default
    {128, 64, 4, 2, "128x64w8"},     // 1
    {128, 128, 2, 4, "128x128w8"},   // 2
    {128, 128, 2, 2, "128x128w4"},   // 3
};
constexpr int kNumTilesI8 = sizeof(kTilesI8) / sizeof(kTilesI8[0]);

template <int BM, int BN, int WM, int WN>
hipError_t launch_tile(const Problem& p, const Plan& plan, hipStream_t stream, bool fc, bool vec) {
  if (fc) return vec ? launch_variant<BM, BN, WM, WN, true, true>(p, plan, stream)
                     : launch_variant<BM, BN, WM, WN, false, true>(p, plan, stream);
  return vec ? launch_variant<BM, BN, WM, WN, true, false>(p, plan, stream)
             : launch_variant<BM, BN, WM, WN, false, false>(p, plan, stream);
}

}  // namespace

Plan plan_i8(const Problem& p, bool allow_split) {
  Plan pl;
  pl.kernel = KERNEL_TILED;
  pl.tile = 0;
  pl.bm = pl.bn = pl.bk = 0;
  pl.tiles_m = pl.tiles_n = 1;
  pl.slabs = 1;
  pl.split_k = 1;
  pl.slabs_per_split = 1;
  int forced = knob_or(KNOB_I8_TILE, -1);         // experiments and tests: force a tile variant
  if (p.chain_n > 0) forced = 0;                  // a general chain: only the generic 64 x 64 kernel implements it
  if (forced < 0) {
    // kernels of their own, no workspace
    if (dw_i8_applicable(p)) { pl.kernel = KERNEL_DW; return pl; }
    if (smallc_i8_applicable(p) && !p.addend) { pl.kernel = KERNEL_SMALLC; return pl; }
    if (pw_i8_applicable(p)) { pl.kernel = KERNEL_PW; return pl; }
    if (k3c64_i8_applicable(p)) { pl.kernel = KERNEL_K3C64; return pl; }
    if (fc_small_i8_applicable(p)) { pl.kernel = KERNEL_FC_SMALL; return pl; }
  }
  pl.bk = BKQ;
  pl.slabs = (p.Kgemm + BKQ - 1) / BKQ;
  int tile = 0;
  if (forced >= 0 && forced < kNumTilesI8) tile = forced;
  // Large contractions (deep reduction, enough pixels and channels for 128-wide tiles) take the
  // kernel built for them.
  if (wide_i8_applicable(p)) {
    if (forced == 4 || forced == 5) return plan_wide_i8(p, (forced == 4 || p.b_is_kn) ? 128 : 64, allow_split);
    if (forced < 0 && p.Kgemm >= 256 && p.M >= 96 && p.kg >= 128 && !pw_i8_applicable(p)) {
      // convolutions with at most one 128 x 128 tile per CU take 128 x 64 tiles: twice the workgroups
      // for the same bytes per workgroup (measured: 3x3 512->512 on 7x7 at batch 32 21.8 -> 19.6 us,
      // 1x1 512->2048 on 7x7 9.1 -> 8.5 us; 1x1 256->1024 on 14x14 with 392 tiles stays at 128 x 128)
      const long long t128 = (long long)((p.M + 127) / 128) * ((p.kg + 127) / 128) * p.groups;
      return plan_wide_i8(p, (!p.b_is_kn && t128 <= 256) ? 64 : 128, allow_split);
    }
  }
  pl.tile = tile;
  pl.bm = kTilesI8[tile].bm;
  pl.bn = kTilesI8[tile].bn;
  pl.tiles_m = (p.M + pl.bm - 1) / pl.bm;
  pl.tiles_n = (p.kg + pl.bn - 1) / pl.bn;
  pl.split_k = 1;
  pl.slabs_per_split = pl.slabs;
  const long long t = (long long)pl.tiles_m * pl.tiles_n * p.groups;
  // Split the reduction when the tiles alone cannot fill the chip: among the split factors that keep
  // at least four slabs per workgroup, the smallest that fills >= 90 % of the resident-workgroup
  // slots of its last round, else the one that fills them best.
  constexpr long long slots = 1024;
  if (allow_split && t < slots && pl.slabs >= 8) {
    int max_split = pl.slabs / 4 < 64 ? pl.slabs / 4 : 64;
    if (t >= 256 && max_split > p.Kgemm / 3072) max_split = p.Kgemm / 3072;   // int32 partials are 4x the output
    int best = 1;
    double best_u = 0.0;
    for (int sk = 1; sk <= max_split; ++sk) {
      const int sps = (pl.slabs + sk - 1) / sk;
      const int real = (pl.slabs + sps - 1) / sps;
      if (real != sk) continue;
      const long long blocks = t * sk;
      const double u = (double)blocks / (double)(((blocks + slots - 1) / slots) * slots);
      if (u > best_u + 1e-9) { best_u = u; best = sk; }
      if (u >= 0.9) { best = sk; break; }
    }
    if (best > 1) {
      pl.slabs_per_split = (pl.slabs + best - 1) / best;
      pl.split_k = (pl.slabs + pl.slabs_per_split - 1) / pl.slabs_per_split;
    }
  }
  return pl;
}

hipError_t launch_i8(const Problem& p_in, const Plan& plan, hipStream_t stream, const char** variant) {
  switch (plan.kernel) {
    case KERNEL_DW: return launch_dw_i8(p_in, stream, variant);
    case KERNEL_SMALLC: return launch_smallc_i8(p_in, stream, variant);
    case KERNEL_PW: return launch_pw_i8(p_in, stream, variant);
    case KERNEL_K3C64: return launch_k3c64_i8(p_in, stream, variant);
    case KERNEL_FC_SMALL: return launch_fc_small_i8(p_in, stream, variant);
    default: break;
  }
  if (plan.split_k > 1 && !p_in.partial) return hipErrorInvalidValue;   // the ABI layer never plans a split without a workspace
  Problem p = p_in;
  p.split_k = plan.split_k;
  p.slabs_per_split = plan.slabs_per_split;
  const bool fc = p.b_is_kn != 0;
  const bool vec = fc ? (p.Kgemm % 16 == 0 && p.k % 4 == 0) : (p.cg % 16 == 0 && p.c % 16 == 0);
  hipError_t e;
  if (plan.kernel == KERNEL_WIDE) {
    e = launch_wide_i8(p, plan, stream, variant);
  } else if (p.chain_n > 0) {
    if (fc || plan.tile != 0) return hipErrorInvalidValue;
    *variant = vec ? "igemm_i8_64x64w4_conv_vec_chainv" : "igemm_i8_64x64w4_conv_scalar_chainv";
    e = vec ? launch_variant<64, 64, 2, 2, true, false, true>(p, plan, stream)
            : launch_variant<64, 64, 2, 2, false, false, true>(p, plan, stream);
  } else {
    static thread_local char name[64];
    snprintf(name, sizeof(name), "igemm_i8_%s_%s_%s", kTilesI8[plan.tile].name, fc ? "fc" : "conv",
             vec ? "vec" : "scalar");
    *variant = name;
    switch (plan.tile) {
      case 0: e = launch_tile<64, 64, 2, 2>(p, plan, stream, fc, vec); break;
      case 1: e = launch_tile<128, 64, 4, 2>(p, plan, stream, fc, vec); break;
      case 2: e = launch_tile<128, 128, 2, 4>(p, plan, stream, fc, vec); break;
      case 3: e = launch_tile<128, 128, 2, 2>(p, plan, stream, fc, vec); break;
      default: return hipErrorInvalidValue;
    }
  }
  if (e != hipSuccess) return e;
  if (plan.split_k > 1 && p.chain_n > 0) {
    const int total = p.M * p.k;
    int blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(splitk_finish_chain_i8, dim3(blocks), dim3(256), 0, stream, p, total);
    e = hipGetLastError();
  } else if (plan.split_k > 1) {
    const int total = p.M * p.k;
    const bool wide = p.k % 4 == 0 && (reinterpret_cast<uintptr_t>(p.bias) & 15) == 0;   // y, partial are 16-byte aligned
    int blocks = (total / (wide ? 4 : 1) + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    auto finish_kernel = wide ? splitk_finish_i8<4> : splitk_finish_i8<1>;
    hipLaunchKernelGGL(finish_kernel, dim3(blocks), dim3(256), 0, stream,
                       static_cast<const int*>(p.partial), static_cast<const int*>(p.bias),
                       static_cast<const signed char*>(p.addend), p.r_off, p.r_mant, p.r_shift,
                       static_cast<signed char*>(p.y), total, p.k, plan.split_k, p.mant, p.shift,
                       p.y_off, p.lo);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace glowmi
