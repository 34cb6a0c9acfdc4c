// fp32 implicit-GEMM Convolution / FullyConnected for gfx950 (MI355X).
//
// The contraction the paper's lowering phase reduces these layers to (Section 3.4: MatMul followed
// by a broadcasted add; Section 3.1: the convolution loop nest) runs on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32, fp32 accumulate).  The element-wise chain that follows -- bias add and
// Relu -- is applied to the accumulators in registers before the only store of the output, which
// is the paper's operator stacking (Section 5.2) in its GPU form.
//
// Work decomposition (one workgroup = 256 threads = 4 wavefronts of 64):
//   - the output matrix [M = n*oh*ow][k] is cut into BM x BN tiles, one per workgroup; workgroup
//     ids are remapped so that each of the 8 XCDs (own L2 each) walks a contiguous range of tiles
//     and re-reads of neighbouring input rows hit its L2;
//   - the reduction axis kg = (r, s, c) is walked in slabs of BK = 32; for each slab the input patch
//     tile (gathered on the fly from NHWC, 16-byte loads along c) and the filter tile are staged in
//     LDS, double buffered, with the next slab's global loads in flight during the MFMAs;
//   - each wavefront owns a (BM/WAVES_M) x (BN/WAVES_N) sub-tile made of 32x32 MFMA blocks and
//     feeds them with ds_read_b128 from K-contiguous, padded (bank-conflict-free) LDS rows.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "igemm.h"

namespace glowmi {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BK = 32;            // reduction slab
constexpr int LDK = BK + 4;       // K-contiguous LDS row, padded: 36 floats keeps ds_read_b128 conflict free
constexpr int KV = BK / 4;        // float4 chunks per K-contiguous row
constexpr int INVALID_ROW = -(1 << 24);
constexpr int FLUSH_SLABS = 32;   // MFMA accumulators are folded into a second set every 1024 k

template <int BN, int NT>
struct BkN {                      // FC weight tile [BK][BN] with N contiguous, staged by NT threads
  static constexpr int LD = BN + 8;             // +8 puts k and k+4 rows on disjoint bank halves
  static constexpr int NV = BN / 4;             // float4 chunks per row
  static constexpr int ROWS = NT / NV;          // k-rows per pass
  static constexpr int PASSES = BK / ROWS;
  static_assert(ROWS >= 1 && ROWS <= BK && BK % ROWS == 0, "FC weight tile does not divide over the threads");
};

template <int BM, int BN, bool B_KN>
constexpr int lds_floats() {
  return 2 * (BM * LDK + (B_KN ? BK * (BN + 8) : BN * LDK));
}

// Decomposition of a reduction index kg into filter row r, filter column s and channel c, with
// branch-free stepping (a data-dependent loop here would serialise the wavefront).
struct Tap {
  int r, s, c;
  __device__ void init(int kg, int cg, int S, const FastDiv& dcg, const FastDiv& ds) {
    const int t = dcg.div(kg);
    c = kg - t * cg;
    r = ds.div(t);
    s = t - r * S;
  }
  __device__ void advance1(int cg, int S) {
    c += 1;
    const bool wc = c == cg;
    c = wc ? 0 : c;
    s += wc ? 1 : 0;
    const bool ws = s == S;
    s = ws ? 0 : s;
    r += ws ? 1 : 0;
  }
};
// The same step for a whole slab of BK indices: BK = (dr * S + ds) * cg + dc, one carry per digit.
struct SlabStep {
  int dr, ds, dc;
  __device__ void init(int step, int cg, int S) {
    dc = step % cg;
    const int t = step / cg;
    ds = t % S;
    dr = t / S;
  }
  __device__ void apply(Tap& t, int cg, int S) const {
    t.c += dc;
    const bool wc = t.c >= cg;
    t.c -= wc ? cg : 0;
    t.s += ds + (wc ? 1 : 0);
    const bool ws = t.s >= S;
    t.s -= ws ? S : 0;
    t.r += dr + (ws ? 1 : 0);
  }
};

// One unit of work: an output tile of one group, for one slice of the reduction axis.
struct Item {
  int tm, tn, g, split;
  int slab_begin, slab_end;
};

template <int BM, int BN, int WAVES_M, int WAVES_N, bool VEC, bool B_KN, bool LONGK, bool CHAINV = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void igemm_f32_kernel(const Problem p, int tiles_m,
                                                                          int tiles_n, int total_work) {
  constexpr int NTHREADS = 64 * WAVES_M * WAVES_N;
  constexpr int ROWS_PER_PASS = NTHREADS / KV;            // tile rows staged per pass over the threads
  static_assert(NTHREADS == 256 || NTHREADS == 512, "four or eight wavefronts per workgroup");
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;   // wavefront tile
  constexpr int TM = WTM / 32, TN = WTN / 32;             // 32x32 MFMA blocks per wavefront
  static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "tile shape");
  static_assert(BM % ROWS_PER_PASS == 0 && (B_KN || BN % ROWS_PER_PASS == 0), "tile rows per pass");
  using BT = BkN<BN, NTHREADS>;
  constexpr int A_PASSES = BM / ROWS_PER_PASS;
  constexpr int B_PASSES = B_KN ? BT::PASSES : BN / ROWS_PER_PASS;
  constexpr int A_ELEMS = BM * LDK;
  constexpr int B_ELEMS = B_KN ? BK * BT::LD : BN * LDK;

  extern __shared__ __align__(16) float lds[];

  // ---- workgroup -> work item, XCD aware.  Hardware deals consecutive workgroup ids round-robin
  // over the 8 XCDs, so id % 8 names the XCD; each XCD gets a contiguous run of items, so tiles in
  // flight on one XCD are neighbours and the input rows / filter tiles they share hit its L2.
  const int per_xcd = gridDim.x >> 3;
  const int w = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (w >= total_work) return;
  const int total_slabs = (p.Kgemm + BK - 1) / BK;
  Item cur;
  {
    cur.tn = w % tiles_n;
    int t = w / tiles_n;
    cur.tm = t % tiles_m;
    t /= tiles_m;
    cur.g = t % p.groups;
    cur.split = t / p.groups;
    cur.slab_begin = cur.split * p.slabs_per_split;
    cur.slab_end = cur.slab_begin + p.slabs_per_split < total_slabs ? cur.slab_begin + p.slabs_per_split : total_slabs;
  }

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  const float* __restrict__ X = static_cast<const float*>(p.x);
  const float* __restrict__ Wt = static_cast<const float*>(p.w);

  // ---- per-thread description of the A (input patch) rows it stages for the item being loaded
  const int kvec = tid % KV;        // which float4 of the slab
  const int row0 = tid / KV;        // first tile row handled
  int a_base[A_PASSES], a_ih0[A_PASSES], a_iw0[A_PASSES];
  int ld_tn = 0, ld_g = 0;          // tile column and group of the item being loaded
  Tap tap;
  SlabStep slab_step;
  slab_step.init(BK, p.cg, p.s);
  // A pointwise layer (1x1 filter, stride 1, no padding; FullyConnected is one) maps output row m
  // straight to input pixel m: no (image, oh, ow) decomposition and no border test is needed.
  const bool pointwise = p.r == 1 && p.s == 1 && p.stride_h == 1 && p.stride_w == 1 && p.pad_t == 0 &&
                         p.pad_l == 0 && p.oh == p.h && p.ow == p.w_;
  auto setup_rows = [&](const Item& it) {
    const int ohow = p.oh * p.ow;
#pragma unroll
    for (int q = 0; q < A_PASSES; ++q) {
      const int m = it.tm * BM + row0 + q * ROWS_PER_PASS;
      if (pointwise) {
        const bool ok = m < p.M;
        a_ih0[q] = ok ? 0 : INVALID_ROW;
        a_iw0[q] = ok ? 0 : INVALID_ROW;
        a_base[q] = ok ? m * p.c + it.g * p.cg : 0;
      } else if (m < p.M) {
        const int img = p.div_ohow.div(m);
        const int rem = m - img * ohow;
        const int oh = p.div_ow.div(rem);
        const int ow = rem - oh * p.ow;
        a_ih0[q] = oh * p.stride_h - p.pad_t;
        a_iw0[q] = ow * p.stride_w - p.pad_l;
        a_base[q] = ((img * p.h + a_ih0[q]) * p.w_ + a_iw0[q]) * p.c + it.g * p.cg;
      } else {
        a_ih0[q] = INVALID_ROW;
        a_iw0[q] = INVALID_ROW;
        a_base[q] = 0;
      }
    }
    ld_tn = it.tn;
    ld_g = it.g;
    tap.init(it.slab_begin * BK + kvec * 4, p.cg, p.s, p.div_cg, p.div_s);
  };

  v4f ra[A_PASSES], rb[B_PASSES];
  // raw buffer descriptors (stride 0, range = tensor bytes); 0x00020000 = 32-bit data format word of gfx9
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(X), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Wt), 0, (int)p.w_bytes, 0x00020000);
  constexpr unsigned OOB = 0xFFFFFF00u;   // beyond any tensor this library accepts (< 4 GiB - 64)

  auto load_global = [&](int slab) {
    const int kg0 = slab * BK + kvec * 4;
    // Loads go through buffer resources: the hardware range check returns zeros for an offset beyond
    // the tensor, so an element that must read as zero (padding tap, reduction tail, row or column
    // outside the problem) simply gets the offset OOB -- no branch, no pre-zeroed registers.
    // ---------------- A: gather from NHWC
    if (VEC) {
      const bool kok = kg0 < p.Kgemm;                       // Kgemm % 4 == 0 on this path
      const int tap_off = (tap.r * p.w_ + tap.s) * p.c + tap.c;
#pragma unroll
      for (int q = 0; q < A_PASSES; ++q) {
        const int ih = a_ih0[q] + tap.r, iw = a_iw0[q] + tap.s;
        const bool ok = kok && (unsigned)ih < (unsigned)p.h && (unsigned)iw < (unsigned)p.w_;
        const unsigned off = ok ? (unsigned)(a_base[q] + tap_off) * 4u : OOB;
        ra[q] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0));
      }
    } else {
      Tap t = tap;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool kok = kg0 + e < p.Kgemm;
        const int tap_off = (t.r * p.w_ + t.s) * p.c + t.c;
#pragma unroll
        for (int q = 0; q < A_PASSES; ++q) {
          const int ih = a_ih0[q] + t.r, iw = a_iw0[q] + t.s;
          const bool ok = kok && (unsigned)ih < (unsigned)p.h && (unsigned)iw < (unsigned)p.w_;
          const unsigned off = ok ? (unsigned)(a_base[q] + tap_off) * 4u : OOB;
          ra[q][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_x, off, 0, 0));
        }
        t.advance1(p.cg, p.s);
      }
    }
    // ---------------- B: filter rows (K contiguous) or FC weight rows (N contiguous)
    if (!B_KN) {
#pragma unroll
      for (int q = 0; q < B_PASSES; ++q) {
        const int n = ld_tn * BN + row0 + q * ROWS_PER_PASS;
        const bool nok = n < p.kg;
        const unsigned row_off = ((unsigned)(ld_g * p.kg + n) * (unsigned)p.Kgemm + (unsigned)kg0) * 4u;
        if (VEC) {
          const unsigned off = (nok && kg0 < p.Kgemm) ? row_off : OOB;
          rb[q] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, off, 0, 0));
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const unsigned off = (nok && kg0 + e < p.Kgemm) ? row_off + 4u * e : OOB;
            rb[q][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_w, off, 0, 0));
          }
        }
      }
    } else {
      constexpr int NV = BT::NV, ROWS = BT::ROWS;
      const int nv = tid % NV, kr0 = tid / NV;
      const int col = ld_tn * BN + nv * 4;
#pragma unroll
      for (int q = 0; q < B_PASSES; ++q) {
        const int kgr = slab * BK + kr0 + q * ROWS;
        const bool kok = kgr < p.Kgemm;
        const unsigned row_off = ((unsigned)kgr * (unsigned)p.k + (unsigned)col) * 4u;
        if (VEC) {
          const unsigned off = (kok && col < p.k) ? row_off : OOB;
          rb[q] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, off, 0, 0));
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const unsigned off = (kok && col + e < p.k) ? row_off + 4u * e : OOB;
            rb[q][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_w, off, 0, 0));
          }
        }
      }
    }
  };

  auto store_lds = [&](int buf) {
    float* As = lds + buf * (A_ELEMS + B_ELEMS);
    float* Bs = As + A_ELEMS;
#pragma unroll
    for (int q = 0; q < A_PASSES; ++q)
      *reinterpret_cast<v4f*>(As + (row0 + q * ROWS_PER_PASS) * LDK + kvec * 4) = ra[q];
    if (!B_KN) {
#pragma unroll
      for (int q = 0; q < B_PASSES; ++q)
        *reinterpret_cast<v4f*>(Bs + (row0 + q * ROWS_PER_PASS) * LDK + kvec * 4) = rb[q];
    } else {
      constexpr int NV = BT::NV, ROWS = BT::ROWS, LD = BT::LD;
      const int nv = tid % NV, kr0 = tid / NV;
#pragma unroll
      for (int q = 0; q < B_PASSES; ++q)
        *reinterpret_cast<v4f*>(Bs + (kr0 + q * ROWS) * LD + nv * 4) = rb[q];
    }
  };

  // Two accumulator sets: the MFMAs add into `acc`; every FLUSH_SLABS slabs it is folded into
  // `total`.  Long reductions (FC with K in the tens of thousands) then round like a sum of short
  // chains, which keeps the fp32 result well inside 1e-5 of the exact sum.
  // Only instantiated (LONGK) for reductions longer than FLUSH_SLABS slabs; short ones keep a
  // single set and the registers that saves.
  v16f acc[TM][TN], total[LONGK ? TM : 1][LONGK ? TN : 1];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        acc[i][j][e] = 0.f;
        if (LONGK) total[i][j][e] = 0.f;
      }
  auto flush = [&]() {
    if (!LONGK) return;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        total[i][j] += acc[i][j];
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
      }
  };

  const int lrow = lane & 31;       // row (A) / column (B) inside a 32x32 MFMA block
  const int lhalf = lane >> 5;      // which half of the 8-deep K group this lane feeds

  auto compute = [&](int buf) {
    const float* As = lds + buf * (A_ELEMS + B_ELEMS);
    const float* Bs = As + A_ELEMS;
#pragma unroll
    for (int k8 = 0; k8 < BK / 8; ++k8) {
      // A lane holds 4 consecutive k of its row; MFMA step kk consumes element kk of both operands,
      // i.e. the pair k = {k8*8 + kk, k8*8 + 4 + kk}: any pairing works as long as A and B agree.
      v4f a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const v4f*>(As + (wm * WTM + i * 32 + lrow) * LDK + k8 * 8 + lhalf * 4);
      if (!B_KN) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
          b[j] = *reinterpret_cast<const v4f*>(Bs + (wn * WTN + j * 32 + lrow) * LDK + k8 * 8 + lhalf * 4);
      } else {
        constexpr int LD = BT::LD;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            b[j][kk] = Bs[(k8 * 8 + lhalf * 4 + kk) * LD + wn * WTN + j * 32 + lrow];
      }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][kk], b[j][kk], acc[i][j], 0, 0, 0);
    }
  };

  // ---- epilogue of one item: bias + activation on the accumulators, one store.
  // 32x32 MFMA block: register e of a lane is row (e/4)*8 + (lane/32)*4 + e%4, column lane%32.
  float* __restrict__ Y = static_cast<float*>(p.y);
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const float* addend = static_cast<const float*>(p.addend);   // may be the output itself
  auto epilogue_as = [&](const Item& it, auto add_tag) {
    constexpr bool ADD = decltype(add_tag)::value;   // the chain has a tensor-add link
    // One base pointer per lane; every element is then base + a wave-uniform row offset, so the
    // per-element cost is the arithmetic of the chain itself.  Tiles that lie completely inside the
    // output skip the bounds tests (uniform branch).
    float* dst_base = p.split_k == 1 ? Y : static_cast<float*>(p.partial) + (size_t)it.split * p.M * p.k;
    const int row_base = it.tm * BM + wm * WTM + lhalf * 4;
    const bool full = (it.tm + 1) * BM <= p.M && (it.tn + 1) * BN <= p.kg;
    const bool finish = p.split_k == 1;
    const bool relu = finish && p.act == 1;
    // Every store below sits in a branch of its own; a load whose result is pending when such a branch is entered
    // makes the compiler wait for ALL memory operations inside it, i.e. for the store before it.  So the loads come
    // first, in groups, each followed by one wait that the compiler can see: the bias values of the item, then per
    // 32 x 32 block the sixteen addend values.
    float bias_v[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = it.tn * BN + wn * WTN + j * 32 + lrow;
      bias_v[j] = (col < p.kg && finish && bias) ? bias[it.g * p.kg + col] : 0.f;
    }
    __builtin_amdgcn_s_waitcnt(0);                       // vmcnt(0), and the other counters: nothing else is in flight here
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = it.tn * BN + wn * WTN + j * 32 + lrow;
      const bool cok = col < p.kg;
      const int ch = it.g * p.kg + col;
      const float bv = bias_v[j];
      float* dst = dst_base + (size_t)row_base * p.k + ch;
      const float* add = ADD ? addend + (size_t)row_base * p.k + ch : nullptr;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        float addv[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int r = i * 32 + (e >> 2) * 8 + (e & 3);
          addv[e] = (ADD && (full || (cok && row_base + r < p.M))) ? add[(size_t)r * p.k] : 0.f;
        }
        if (ADD) __builtin_amdgcn_s_waitcnt(0);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int r = i * 32 + (e >> 2) * 8 + (e & 3);          // compile-time row inside the wave tile
          float v = (LONGK ? total[i][j][e] : acc[i][j][e]) + bv + addv[e];
          const bool inside = full || (cok && row_base + r < p.M);
          if (relu) v = fmaxf(v, 0.f);
          if (inside) dst[(size_t)r * p.k] = v;
        }
      }
    }
  };
  // General chain (CHAINV instantiations only): the op list of the problem applied in order to every
  // element, in registers, before the one store -- any stack of data-parallel operators, not just the
  // fixed bias -> add -> Relu shape.  The op kinds are uniform over the launch (scalar branches).
  auto epilogue_chainv = [&](const Item& it) {
    const int row_base = it.tm * BM + wm * WTM + lhalf * 4;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = it.tn * BN + wn * WTN + j * 32 + lrow;
      const bool cok = col < p.kg;
      const int ch = it.g * p.kg + col;
      const float bv = (cok && bias) ? bias[ch] : 0.f;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int r = i * 32 + (e >> 2) * 8 + (e & 3);
          if (!cok || row_base + r >= p.M) continue;
          const size_t off = (size_t)(row_base + r) * p.k + ch;
          float v = (LONGK ? total[i][j][e] : acc[i][j][e]) + bv;
          for (int o = 0; o < p.chain_n; ++o) {
            const ChainOpDev& op = p.chain[o];
            if (op.kind == CHAIN_ADD_TENSOR) v += static_cast<const float*>(op.tensor)[off];
            else if (op.kind == CHAIN_MUL_SCALAR) v *= op.a;
            else if (op.kind == CHAIN_MAX_SCALAR) v = fmaxf(v, op.a);
            else v = fminf(fmaxf(v, op.a), op.b);
          }
          Y[off] = v;
        }
      }
    }
  };
  auto epilogue = [&](const Item& it) {
    if (CHAINV && p.split_k == 1) epilogue_chainv(it);
    else if (!CHAINV && addend && p.split_k == 1) epilogue_as(it, std::true_type{});
    else epilogue_as(it, std::false_type{});
  };

  // ---- main loop: global loads of slab i+1 in flight while slab i is multiplied.  The loop is
  // nested so that the fold of `acc` into `total` sits outside the inner loop and the MFMA
  // accumulators never leave their registers inside it.
  setup_rows(cur);
  load_global(cur.slab_begin);
  store_lds(0);
  __syncthreads();
  int buf = 0;
  for (int chunk = cur.slab_begin; chunk < cur.slab_end; chunk += FLUSH_SLABS) {
    const int chunk_end = chunk + FLUSH_SLABS < cur.slab_end ? chunk + FLUSH_SLABS : cur.slab_end;
    for (int slab = chunk; slab < chunk_end; ++slab) {
      const bool more = slab + 1 < cur.slab_end;
      if (more) {
        slab_step.apply(tap, p.cg, p.s);
        load_global(slab + 1);
      }
      compute(buf);
      if (more) store_lds(buf ^ 1);
      __syncthreads();
      buf ^= 1;
    }
    flush();
  }
  epilogue(cur);
}

// Finish of a split reduction: sum the partial tiles in split order (deterministic), then the same
// fused bias (+ addend) + activation, one store.  A thread owns W consecutive outputs (W = 4 when the
// row length allows 16-byte accesses) and walks the splits eight at a time: the eight loads are
// independent and in flight together, the additions stay in split order.
template <int W>
__global__ __launch_bounds__(256) void splitk_finish_f32(const float* __restrict__ partial,
                                                         const float* __restrict__ bias,
                                                         const float* addend, float* y, int total, int k,
                                                         int split_k, int act) {
  typedef float vec __attribute__((ext_vector_type(W)));
  const int groups = total / W;                      // W divides total (the launcher checks)
  for (int gi = blockIdx.x * blockDim.x + threadIdx.x; gi < groups; gi += gridDim.x * blockDim.x) {
    const size_t i = (size_t)gi * W;
    vec v = {};
    for (int s = 0; s < split_k; s += 8) {
      vec t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int su = s + u < split_k ? s + u : s;  // a repeated row stands in past the end and is not added
        t[u] = *reinterpret_cast<const vec*>(partial + (size_t)su * total + i);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (s + u < split_k) v += t[u];
    }
    if (bias) v += *reinterpret_cast<const vec*>(bias + i % k);      // W divides k: no wrap inside the vector
    if (addend) v += *reinterpret_cast<const vec*>(addend + i);
    if (act == 1) {
#pragma unroll
      for (int e = 0; e < W; ++e) v[e] = fmaxf(v[e], 0.f);
    }
    *reinterpret_cast<vec*>(y + i) = v;
  }
}

// Finish of a split reduction whose element-wise chain is a general op list: partial sums in split
// order, bias, then the ops in order, one store.
__global__ __launch_bounds__(256) void splitk_finish_chain_f32(const Problem p, int total) {
  const float* __restrict__ partial = static_cast<const float*>(p.partial);
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  float* y = static_cast<float*>(p.y);
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    float v = 0.f;
    for (int s = 0; s < p.split_k; ++s) v += partial[(size_t)s * total + i];
    if (bias) v += bias[i % p.k];
    for (int o = 0; o < p.chain_n; ++o) {
      const ChainOpDev& op = p.chain[o];
      if (op.kind == CHAIN_ADD_TENSOR) v += static_cast<const float*>(op.tensor)[i];
      else if (op.kind == CHAIN_MUL_SCALAR) v *= op.a;
      else if (op.kind == CHAIN_MAX_SCALAR) v = fmaxf(v, op.a);
      else v = fminf(fmaxf(v, op.a), op.b);
    }
    y[i] = v;
  }
}

// ---------------------------------------------------------------------------------------------------
// FullyConnected with at most 16 rows (batch 1..16): the layer is a stream of the weight matrix
// through the chip, bound by HBM.  No LDS staging and no barriers in the main loop: every lane loads
// float4 pieces of weight rows straight into registers in the layout the MFMA wants, activations
// (a few rows, L2 resident) are read as float4 along K, the four wavefronts of a workgroup
// interleave K steps and are summed through LDS in a fixed order; if the grid also splits K the
// sums go to the workspace for the finishing kernel.
//
// v_mfma_f32_16x16x4_f32 is used because a 32-row MFMA would spend half of the matrix unit on
// padding rows, and at 64 cycles per 256 bytes of weights the matrix unit, not HBM, would set the
// pace.  Lane l = (c = l % 16, q = l / 16): loads float4 W[k0 + 4q + t][n0 + 4c..] for t = 0..3
// (16 lanes cover 256 contiguous bytes of one weight row) and float4 A[c][k0 + 4q..]; MFMA (t, j)
// multiplies k = k0 + 4q + t into the column group j, i.e. columns n0 + 4c + j, so the four
// accumulators of a lane hold four consecutive output columns (one float4 store).
// ---------------------------------------------------------------------------------------------------
constexpr int SK_WAVES = 4;
constexpr int SK16_COLS = 64;    // output columns per workgroup
constexpr int SK16_STEP = 16;    // weight rows per step

typedef float v4f_acc __attribute__((ext_vector_type(4)));

template <bool STREAM>
__global__ __launch_bounds__(64 * SK_WAVES) void fc_skinny16_f32_kernel(
    const float* __restrict__ A, const float* __restrict__ Wt, const float* __restrict__ bias,
    float* __restrict__ Y, float* __restrict__ partial, int M, int K, int N, int act, int split_k,
    int steps_per_split) {
  __shared__ float red[(SK_WAVES - 1) * 16 * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c16 = lane & 15, q = lane >> 4;
  const int n0 = blockIdx.x * SK16_COLS;
  const int split = blockIdx.y;
  const int total_steps = (K + SK16_STEP - 1) / SK16_STEP;
  const int step_begin = split * steps_per_split;
  const int step_end = step_begin + steps_per_split < total_steps ? step_begin + steps_per_split : total_steps;

  const int col = n0 + 4 * c16;
  const bool col_ok = col < N;                   // N % 4 == 0: all four or none
  const bool row_ok = c16 < M;                   // as the A operand, lane c16 holds activation row c16

  v4f_acc acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) acc[j] = v4f_acc{0.f, 0.f, 0.f, 0.f};

  // Full steps (16 weight rows inside K) are loaded without any predicate, so the compiler keeps
  // the loads in flight across the MFMAs.  Lanes whose row or column lies outside the problem load
  // from a clamped address: their products land in result rows / columns that are never stored.
  // The one partial step a K that is not a multiple of 16 leaves is done separately, masked.
  const float* a_base = A + (size_t)(row_ok ? c16 : 0) * K + q * 4;
  const float* w_base = Wt + (col_ok ? col : 0) + (size_t)(q * 4) * N;
  auto load_step = [&](int step, v4f& a, v4f (&b)[4]) {
    a = *reinterpret_cast<const v4f*>(a_base + (size_t)step * SK16_STEP);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      // a weight matrix larger than the last-level cache is a pure stream: non-temporal loads keep it
      // from displacing everything else on its way through (measured 78 -> 71 us on 25088 x 4096)
      const v4f* src = reinterpret_cast<const v4f*>(w_base + ((size_t)step * SK16_STEP + t) * N);
      b[t] = STREAM ? __builtin_nontemporal_load(src) : *src;
    }
  };
  auto mma_step = [&](const v4f& a, const v4f (&b)[4]) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t][j], acc[j], 0, 0, 0);
  };

  const int full_steps = K / SK16_STEP;
  const int fast_end = step_end < full_steps ? step_end : full_steps;
  const int stride = SK_WAVES;                   // the four wavefronts interleave steps
  // Plain loop, one step per trip: with 16 wavefronts resident per CU the hardware overlaps the
  // loads of some with the MFMAs of others (measured faster than explicit register double buffering:
  // 4096 x 4096 at 16 rows 16.2 us vs 19.1 us with the next step's loads issued ahead in a second register set).
  for (int step = step_begin + wave; step < fast_end; step += stride) {
    v4f a, b[4];
    load_step(step, a, b);
    mma_step(a, b);
  }
  if (step_end > full_steps && full_steps >= step_begin && (full_steps - step_begin) % stride == wave) {
    // wave-uniform branch: the partial last step.  K % 4 == 0, so a lane's group of four k is
    // entirely inside or outside; outside groups read group 0 and are cancelled by a zero operand.
    const int k0 = full_steps * SK16_STEP + q * 4;
    const bool kok = k0 < K;
    const int kc = kok ? k0 : 0;
    v4f a = *reinterpret_cast<const v4f*>(A + (size_t)(row_ok ? c16 : 0) * K + kc);
    if (!kok) a = v4f{0.f, 0.f, 0.f, 0.f};
    v4f b[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
      b[t] = *reinterpret_cast<const v4f*>(Wt + (col_ok ? col : 0) + (size_t)(kc + t) * N);
    mma_step(a, b);
  }

  if (wave > 0) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) red[((wave - 1) * 16 + j * 4 + e) * 64 + lane] = acc[j][e];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int wv = 0; wv < SK_WAVES - 1; ++wv)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[j][e] += red[(wv * 16 + j * 4 + e) * 64 + lane];

  if (!col_ok) return;
  v4f bv = {0.f, 0.f, 0.f, 0.f};
  if (split_k == 1 && bias) bv = v4f{bias[col], bias[col + 1], bias[col + 2], bias[col + 3]};   // bias is only 4-byte aligned
  // 16x16 result: register e of lane (c, q) is row 4q + e, column c
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int row = q * 4 + e;
    if (row >= M) continue;
    v4f v = {acc[0][e], acc[1][e], acc[2][e], acc[3][e]};
    if (split_k == 1) {
      v += bv;
      if (act == 1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = fmaxf(v[j], 0.f);
      }
      *reinterpret_cast<v4f*>(Y + (size_t)row * N + col) = v;
    } else {
      *reinterpret_cast<v4f*>(partial + ((size_t)split * M + row) * N + col) = v;
    }
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool VEC, bool B_KN, bool LONGK, bool CHAINV = false>
hipError_t launch_variant(const Problem& p, const Plan& plan, hipStream_t stream) {
  auto kern = igemm_f32_kernel<BM, BN, WAVES_M, WAVES_N, VEC, B_KN, LONGK, CHAINV>;
  constexpr int lds_bytes = lds_floats<BM, BN, B_KN>() * (int)sizeof(float);
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

}  // namespace

// Tile variants.  bm x bn output tile, waves_m x waves_n wavefronts.
struct TileF32 { int bm, bn, wm, wn; const char* name; };
constexpr TileF32 kTilesF32[] = {
    {64, 64, 2, 2, "64x64w4"},       // 0: default; 4 workgroups per CU keep the matrix cores fed
    {128, 64, 4, 2, "128x64w8"},     // 1
    {128, 128, 2, 4, "128x128w8"},   // 2
    {32, 128, 1, 4, "32x128w4"},     // 3: FC with a handful of rows
    {128, 64, 2, 2, "128x64w4"},     // 4
    {128, 128, 2, 2, "128x128w4"},   // 5
};
constexpr int kNumTilesF32 = sizeof(kTilesF32) / sizeof(kTilesF32[0]);

Plan plan_f32(const Problem& p, bool allow_split) {
  Plan pl;
  pl.kernel = KERNEL_TILED;
  pl.tile = 0;
  pl.bm = pl.bn = pl.bk = 0;
  pl.tiles_m = pl.tiles_n = 1;
  pl.slabs = 1;
  pl.split_k = 1;
  pl.slabs_per_split = 1;
  int forced_tile = knob(KNOB_F32_TILE);                 // experiments and tests: force a generic tile variant
  if (p.chain_n > 0) forced_tile = 0;                    // a general chain: only the generic 64 x 64 kernel implements it
  const bool forced = forced_tile != kKnobUnset;
  if (!forced) {
    // kernels of their own, no workspace
    if (dw_f32_applicable(p)) { pl.kernel = KERNEL_DW; return pl; }
    if (smallc_f32_applicable(p) && !p.addend) { pl.kernel = KERNEL_SMALLC; return pl; }
    // 3x3 over 64 channels on many pixels, with the filter's planes given or room in the workspace for them
    const bool filter_planes = p.w_packed != nullptr || (allow_split && p.allow_pack);   // given, or room to make them
    if (filter_planes && k3c64_f32_applicable(p)) {
      pl.kernel = KERNEL_K3C64;
      pl.pack_bytes = k3c64_f32_pack_bytes(p);
      return pl;
    }
    // 3x3 stride 1 with many channels on maps that tile into 16 x 16 blocks, again only the filter repacked
    if (filter_planes && k3_f32_applicable(p)) {
      pl.kernel = KERNEL_K3;
      pl.pack_bytes = k3_f32_pack_bytes(p);
      return pl;
    }
    // large contractions with a workspace to repack the operands into: the kernel over fp16 planes
    if (allow_split && p.allow_pack && p3_f32_applicable(p)) return plan_p3_f32(p);
    if (pw_f32_applicable(p)) { pl.kernel = KERNEL_PW; return pl; }
    if (conv_small_f32_applicable(p)) { pl.kernel = KERNEL_SMALL; return pl; }
    if (fc_small_f32_applicable(p)) { pl.kernel = KERNEL_FC_SMALL; return pl; }
  }
  if (p.b_is_kn && p.M <= 16 && p.groups == 1 && p.k % 4 == 0 && p.Kgemm % 4 == 0 && !p.addend && !forced) {
    // FC with a handful of rows: stream the weights (fc_skinny16_f32_kernel).  "slabs" are steps of
    // SK16_STEP weight rows; K is split over the grid until ~4 workgroups per CU exist, each
    // wavefront keeping at least two steps.
    const int cols = SK16_COLS, stepk = SK16_STEP;
    pl.kernel = KERNEL_SKINNY16;
    pl.bm = 16;
    pl.bn = cols;
    pl.bk = stepk;
    pl.tiles_m = 1;
    pl.tiles_n = (p.k + cols - 1) / cols;
    pl.slabs = (p.Kgemm + stepk - 1) / stepk;
    pl.split_k = 1;
    pl.slabs_per_split = pl.slabs;
    if (allow_split) {
      int want = (1024 + pl.tiles_n - 1) / pl.tiles_n;   // 1024 workgroups measured best (2048+ is slower)
      int max_split = pl.slabs / (2 * SK_WAVES);
      int sk = want < max_split ? want : max_split;
      if (sk > 128) sk = 128;
      if (sk > 1) {
        pl.slabs_per_split = (pl.slabs + sk - 1) / sk;
        pl.split_k = (pl.slabs + pl.slabs_per_split - 1) / pl.slabs_per_split;
      }
    }
    return pl;
  }
  if (allow_split && !forced) {
    // deep reduction on very few pixels: the single-round-trip kernel, reduction sliced over the grid
    const int slices = conv_small_f32_splits(p);
    if (slices > 1) {
      pl.kernel = KERNEL_SMALL_SPLIT;
      pl.bm = 32;
      pl.bn = 32;
      pl.bk = 576;
      pl.tiles_m = (p.M + 31) / 32;
      pl.tiles_n = (p.k + 31) / 32;
      pl.slabs = slices;
      pl.split_k = slices;
      pl.slabs_per_split = 1;
      return pl;
    }
  }
  pl.bk = BK;
  pl.slabs = (p.Kgemm + BK - 1) / BK;
  // Measured on VGG-19 / ResNet-50 shaped layers the 64x64 tile with four resident workgroups per
  // CU is within 2% of the best variant everywhere; FC with very few rows takes the 32-row tile.
  int tile = 0;
  if (p.M <= 32 && p.kg > 64) tile = 3;
  // Wide layers whose 128x128 tiling leaves between a quarter and one round of workgroups gain
  // from the larger tile once the reduction is split to fill the chip (measured: 3x3 512->512 on a
  // 28x28 map at batch 16 goes from 63 % to 70 % of the MFMA peak).
  {
    const long long t128 = (long long)((p.M + 127) / 128) * ((p.kg + 127) / 128) * p.groups;
    if (allow_split && p.kg >= 128 && t128 >= 256 && t128 < 1024 && p.Kgemm >= 4096) tile = 2;
  }
  if (forced && forced_tile >= 0 && forced_tile < kNumTilesF32) tile = forced_tile;
  pl.tile = tile;
  pl.bm = kTilesF32[tile].bm;
  pl.bn = kTilesF32[tile].bn;
  pl.tiles_m = (p.M + pl.bm - 1) / pl.bm;
  pl.tiles_n = (p.kg + pl.bn - 1) / pl.bn;
  pl.split_k = 1;
  pl.slabs_per_split = pl.slabs;
  const long long t = (long long)pl.tiles_m * pl.tiles_n * p.groups;
  // Split the reduction when the tiles alone cannot fill the chip.  `slots` = workgroups resident
  // at once (256 CUs x 4 for the default tile).  Among the split factors that keep at least four
  // slabs per workgroup, take the smallest one that fills >= 90 % of the slots of its last round,
  // else the one that fills them best.
  constexpr long long slots = 1024;
  if (allow_split && t < slots && pl.slabs >= 8) {
    int max_split = pl.slabs / 4 < 64 ? pl.slabs / 4 : 64;
    // With many tiles the partial sums are a real HBM cost (2 * split * M * N * 4 bytes against
    // 2 * M * N * K flops): keep it near a tenth of the MFMA time.
    if (t >= 256 && max_split > p.Kgemm / 768) max_split = p.Kgemm / 768;
    int best = 1;
    double best_u = 0.0;
    for (int sk = 1; sk <= max_split; ++sk) {
      const int sps = (pl.slabs + sk - 1) / sk;
      const int real = (pl.slabs + sps - 1) / sps;          // splits that actually get work
      if (real != sk) continue;
      const long long blocks = t * sk;
      const double u = (double)blocks / (double)(((blocks + slots - 1) / slots) * slots);
      if (u > best_u + 1e-9) { best_u = u; best = sk; }
      if (u >= 0.9) { best = sk; break; }
    }
    if (knob_is_set(KNOB_F32_SPLIT)) {                     // experiments: clamped to what the slabs allow
      best = knob(KNOB_F32_SPLIT);
      if (best < 1) best = 1;
      if (best > pl.slabs) best = pl.slabs;
      if (best > 256) best = 256;
    }
    if (best > 1) {
      pl.slabs_per_split = (pl.slabs + best - 1) / best;
      pl.split_k = (pl.slabs + pl.slabs_per_split - 1) / pl.slabs_per_split;
    }
  }
  return pl;
}

namespace {
template <int BM, int BN, int WM, int WN, bool LONGK>
hipError_t launch_tile2(const Problem& p, const Plan& plan, hipStream_t stream, bool fc, bool vec) {
  if (fc) return vec ? launch_variant<BM, BN, WM, WN, true, true, LONGK>(p, plan, stream)
                     : launch_variant<BM, BN, WM, WN, false, true, LONGK>(p, plan, stream);
  return vec ? launch_variant<BM, BN, WM, WN, true, false, LONGK>(p, plan, stream)
             : launch_variant<BM, BN, WM, WN, false, false, LONGK>(p, plan, stream);
}
template <int BM, int BN, int WM, int WN>
hipError_t launch_tile(const Problem& p, const Plan& plan, hipStream_t stream, bool fc, bool vec) {
  return plan.slabs_per_split > FLUSH_SLABS ? launch_tile2<BM, BN, WM, WN, true>(p, plan, stream, fc, vec)
                                            : launch_tile2<BM, BN, WM, WN, false>(p, plan, stream, fc, vec);
}
}  // namespace

hipError_t launch_splitk_finish_f32(const Problem& p, const Plan& plan, hipStream_t stream) {
  const int total = p.M * p.k;
  const bool wide = p.k % 4 == 0 && (reinterpret_cast<uintptr_t>(p.bias) & 15) == 0;   // y, partial, addend are 16-byte aligned
  int blocks = (total / (wide ? 4 : 1) + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  auto kern = wide ? splitk_finish_f32<4> : splitk_finish_f32<1>;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), 0, stream,
                     static_cast<const float*>(p.partial), static_cast<const float*>(p.bias),
                     static_cast<const float*>(p.addend),
                     static_cast<float*>(p.y), total, p.k, plan.split_k, p.act);
  return hipGetLastError();
}

hipError_t launch_f32(const Problem& p_in, const Plan& plan, hipStream_t stream, const char** variant) {
  switch (plan.kernel) {
    case KERNEL_DW: return launch_dw_f32(p_in, stream, variant);
    case KERNEL_SMALLC: return launch_smallc_f32(p_in, stream, variant);
    case KERNEL_PW: return launch_pw_f32(p_in, stream, variant);
    case KERNEL_SMALL: return launch_conv_small_f32(p_in, stream, variant);
    case KERNEL_FC_SMALL: return launch_fc_small_f32(p_in, stream, variant);
    case KERNEL_P3: return launch_p3_f32(p_in, plan, stream, variant);
    case KERNEL_K3C64: return launch_k3c64_f32(p_in, stream, variant);
    case KERNEL_K3: return launch_k3_f32(p_in, stream, variant);
    default: break;
  }
  if (plan.split_k > 1 && !p_in.partial) return hipErrorInvalidValue;   // the ABI layer never plans a split without a workspace
  Problem p = p_in;
  p.split_k = plan.split_k;
  p.slabs_per_split = plan.slabs_per_split;
  // 16-byte gathers need channel runs that are multiples of 4 floats
  const bool fc = p.b_is_kn != 0;
  const bool vec = fc ? (p.Kgemm % 4 == 0 && p.k % 4 == 0) : (p.cg % 4 == 0 && p.c % 4 == 0);
  static thread_local char name[64];
  hipError_t e;
  if (plan.kernel == KERNEL_SMALL_SPLIT) {
    e = launch_conv_small_f32(p, stream, variant);
  } else if (plan.kernel == KERNEL_SKINNY16) {
    *variant = "fc_skinny16_f32";
    dim3 grid(plan.tiles_n, plan.split_k, 1), block(64 * SK_WAVES, 1, 1);
    // Weights of 32 MB and more are loaded non-temporally: a layer's weights are read once per call and, in a
    // network whose tensors exceed the 256 MB last-level cache, come from HBM every time, where plain loads (which
    // allocate every line in that cache on the way) measured little more than half the rate: 4096 x 4096 at 16 rows
    // inside a step of other layers 25 -> 20 us (launched back to back on resident weights 16.9 -> 17.8 us), 25088 x
    // 4096 78 -> 71 us.  Smaller matrices stay resident between calls more often than not and keep plain loads.
    auto kern = p.w_bytes >= (32u << 20) ? fc_skinny16_f32_kernel<true> : fc_skinny16_f32_kernel<false>;
    hipLaunchKernelGGL(kern, grid, block, 0, stream, static_cast<const float*>(p.x),
                       static_cast<const float*>(p.w), static_cast<const float*>(p.bias),
                       static_cast<float*>(p.y), static_cast<float*>(p.partial), p.M, p.Kgemm, p.k, p.act,
                       plan.split_k, plan.slabs_per_split);
    e = hipGetLastError();
  } else if (p.chain_n > 0) {
    if (fc || plan.tile != 0) return hipErrorInvalidValue;
    const bool longk = plan.slabs_per_split > FLUSH_SLABS;
    snprintf(name, sizeof(name), "igemm_f32_64x64w4_conv_%s%s_chainv", vec ? "vec" : "scalar", longk ? "_longk" : "");
    *variant = name;
    if (vec) e = longk ? launch_variant<64, 64, 2, 2, true, false, true, true>(p, plan, stream)
                       : launch_variant<64, 64, 2, 2, true, false, false, true>(p, plan, stream);
    else e = longk ? launch_variant<64, 64, 2, 2, false, false, true, true>(p, plan, stream)
                   : launch_variant<64, 64, 2, 2, false, false, false, true>(p, plan, stream);
  } else {
    snprintf(name, sizeof(name), "igemm_f32_%s_%s_%s%s", kTilesF32[plan.tile].name, fc ? "fc" : "conv",
             vec ? "vec" : "scalar", plan.slabs_per_split > FLUSH_SLABS ? "_longk" : "");
    *variant = name;
    switch (plan.tile) {
      case 0: e = launch_tile<64, 64, 2, 2>(p, plan, stream, fc, vec); break;
      case 1: e = launch_tile<128, 64, 4, 2>(p, plan, stream, fc, vec); break;
      case 2: e = launch_tile<128, 128, 2, 4>(p, plan, stream, fc, vec); break;
      case 3: e = launch_tile<32, 128, 1, 4>(p, plan, stream, fc, vec); break;
      case 4: e = launch_tile<128, 64, 2, 2>(p, plan, stream, fc, vec); break;
      case 5: e = launch_tile<128, 128, 2, 2>(p, plan, stream, fc, vec); break;
      default: return hipErrorInvalidValue;
    }
  }
  if (e != hipSuccess) return e;
  if (plan.split_k > 1 && p.chain_n > 0) {
    const int total = p.M * p.k;
    int blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(splitk_finish_chain_f32, dim3(blocks), dim3(256), 0, stream, p, total);
    e = hipGetLastError();
  } else if (plan.split_k > 1) {
    e = launch_splitk_finish_f32(p, plan, stream);
  }
  return e;
}

}  // namespace glowmi
