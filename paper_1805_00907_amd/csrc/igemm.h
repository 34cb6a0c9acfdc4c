// Internal interface between the host-side C ABI (api.hip) and the kernel translation units.
// One problem description serves Convolution and FullyConnected: both are the contraction
//   Y[m][n] = sum_kg A[m][kg] * B[n][kg]
// with m = (image, oh, ow), n = output channel, kg = (r, s, c).  A is never materialised: the
// kernel gathers it from the NHWC input (no im2col buffer, the cost the paper's evaluation section
// attributes to im2col+GEMM).  FullyConnected is the same problem with h = w = r = s = 1 and the
// weight matrix stored [K][N] (b_is_kn).
#pragma once
#include <hip/hip_runtime_api.h>
#include <limits.h>
#include <stdint.h>

namespace glowmi {

// Tuning knobs for experiments and tests (force a tile variant, lower a kernel's size threshold so a
// small test shape reaches it).  Each is read ONCE from the environment variable GLOWMI_<name> when the
// library is first used and can be changed afterwards only through glowmi_tuning_set(): nothing on the
// dispatch path calls getenv.  kKnobUnset means "the planner's own choice".
enum Knob {
  KNOB_F32_TILE, KNOB_F32_SPLIT, KNOB_F32_P3, KNOB_F32_P3_MIN_M, KNOB_F32_P3_RATIO, KNOB_F32_P3_BN, KNOB_F32_K3C64, KNOB_F32_K3C64_MIN_TILES, KNOB_F32_K3, KNOB_F32_K3_ANY, KNOB_F32_K3V, KNOB_F32_K3_TH, KNOB_F32_K3_TW, KNOB_F32_PW_MIN_ITEMS, KNOB_F32_PW_BF16, KNOB_F32_SMALL_MAX_TILES, KNOB_F32_SMALL_NO_SPLIT,
  KNOB_F32_SMALL_SPLIT_MAX_TILES, KNOB_F32_SMALL_MIN_WGS, KNOB_F32_FC_SMALL_OFF, KNOB_F32_FC_SMALL_VW, KNOB_F32_FC_SMALL_MAX_KB, KNOB_F32_FC_SMALL_MIN_M, KNOB_SMALLC_TH, KNOB_F32_SMALLC_BF16,
  KNOB_I8_TILE, KNOB_I8_WIDE_SPLIT, KNOB_I8_WIDE_NBUF, KNOB_SMALLC_I8_WGS, KNOB_I8_PW_MIN_ITEMS,
  KNOB_I8_FC_SMALL_MAX_M, KNOB_I8_K3_MIN_BLOCKS, KNOB_I8_K3_WAVES, KNOB_I8_K3_GATHER, KNOB_DW,
  KNOB_COUNT
};
constexpr int kKnobUnset = INT_MIN;
int knob(Knob k);                                     // current value or kKnobUnset
inline bool knob_is_set(Knob k) { return knob(k) != kKnobUnset; }
inline int knob_or(Knob k, int dflt) { const int v = knob(k); return v == kKnobUnset ? dflt : v; }

// Compute units of the current device, queried once (0 if the query fails).
int num_compute_units();

// Division of an index below 2^31 by a fixed divisor d as one multiply-high and one shift:
// with s = ceil(log2 d) and mul = ceil(2^(31+s) / d), n / d == (n * mul) >> (31 + s) exactly.
// The host fills it once per call; the kernels use it wherever they take a tile or reduction index
// apart (output pixel -> image/row/column, reduction index -> filter tap/channel).
struct FastDiv {
  uint32_t mul, shift, d;
#if defined(__HIPCC__)
  __device__ __forceinline__ int div(int n) const {
    return d == 1 ? n : (int)(__umulhi((unsigned)n, mul) >> shift);
  }
#endif
};

inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  f.mul = 0;
  f.shift = 0;
  if (d <= 1) return f;                                // the device side short-cuts d == 1
  uint32_t s = 0;
  while ((1ull << s) < d) ++s;                         // ceil(log2 d)
  f.mul = (uint32_t)(((1ull << (31 + s)) + d - 1) / d);   // < 2^32 because d > 2^(s-1)
  f.shift = s - 1;
  return f;
}

// One link of a general element-wise chain behind the contraction (Section 5.2 of the paper: any run
// of data-parallel operators is stacked onto the producer).  fp32 uses a/b; the quantized form uses
// the integer bounds ia/ib on the int32 accumulator and, for an added tensor, its offset and the
// multiplier mant * 2^-shift that brings a code difference to the accumulator's current scale.
enum ChainKind { CHAIN_ADD_TENSOR = 1, CHAIN_MUL_SCALAR = 2, CHAIN_MAX_SCALAR = 3, CHAIN_CLIP = 4 };
constexpr int kMaxChainOps = 4;
struct ChainOpDev {
  int32_t kind;
  float a, b;
  int32_t ia, ib;
  int32_t t_off, t_mant, t_shift;
  const void* tensor;     // [M][k] like the output (float or int8); may be the output itself
};

struct Problem {
  const void* x;      // input  [n][h][w][c]            (float or int8)
  const void* w;      // filter [k][r][s][cg]  or FC weight [Kgemm][k] when b_is_kn
  const void* bias;   // [k] float or int32, may be null
  void* y;            // output [M][k]
  void* partial;      // split-K partial sums [split_k][M][k] (float or int32), null when split_k == 1
  const void* planes; // fp32 on the fp16 matrix cores: workspace for the input's planes (or only its partial maxima), then the weights' planes
  const void* w_packed; // the weights' planes as the caller made them ahead of time (glowmi_*_pack_filter), or null
  const void* w_planes; // where the kernel reads the weights' planes: w_packed, or inside `planes` (set by the launcher)
  const unsigned* x_range; // x_range_n words whose largest is the bits of the input's largest magnitude (set by the launcher)
  const unsigned* w_range; // one word: the same for the weights (the trailer of their planes)
  int32_t x_range_n;
  const void* addend; // tensor operand of the element-wise chain [M][k] (float or int8), may be null:
                      // added to the accumulator after the bias and before the activation
  int32_t n, h, w_, c;
  int32_t k, r, s;
  int32_t oh, ow;
  int32_t stride_h, stride_w, pad_t, pad_l;
  int32_t groups, cg, kg;   // channels per group: input (cg) and output (kg)
  int32_t M;                // n * oh * ow
  int32_t Kgemm;            // r * s * cg
  int32_t split_k;          // >= 1
  int32_t slabs_per_split;  // reduction slabs each split walks
  FastDiv div_ohow, div_ow, div_cg, div_s;   // divisors oh*ow, ow, cg, s
  uint32_t x_bytes, w_bytes; // sizes of the input and weight tensors (hardware-checked buffer loads)
  int32_t act;              // 0 none, 1 relu
  int32_t b_is_kn;          // FC weight layout
  int32_t allow_pack;       // the caller's workspace may hold repacked operands (fp32 three-piece form)
  // quantized form only
  int32_t x_off, w_off, y_off;
  int32_t mant, shift;      // requantize multiplier
  int32_t lo;               // lower clamp bound
  int32_t r_off, r_mant, r_shift;   // quantized addend: its offset and the multiplier that brings a
                                    // code difference to the accumulator's scale, mant * 2^-shift
  // general chain (chain_n > 0): replaces addend/act; only the generic 64 x 64 tiled kernels and the
  // finishing kernels of a split reduction implement it
  int32_t chain_n;
  ChainOpDev chain[kMaxChainOps];
};

// Which kernel family a call takes, and how the reduction is split over workgroups.  The ABI layer
// plans ONCE per call (with the workspace the caller gave in mind) and hands the plan to the launcher.
enum KernelKind {
  KERNEL_TILED = 0,     // generic implicit-GEMM tiles (igemm_f32.hip / igemm_i8.hip)
  KERNEL_SKINNY16,      // fp32 FullyConnected with at most 16 rows: weight stream
  KERNEL_SMALL,         // fp32 convolution on few pixels, one launch (conv_small_f32.hip)
  KERNEL_SMALL_SPLIT,   // the same with the reduction sliced over the grid
  KERNEL_SMALLC,        // 3-channel 7x7/2 first layer
  KERNEL_PW,            // pointwise convolution, persistent workgroups
  KERNEL_K3C64,         // 3x3 over 64 input channels (int8: conv_k3c64_i8.hip, fp32: conv_k3c64_f32.hip)
  KERNEL_FC_SMALL,      // FullyConnected with few rows in one launch (fp32: fc_small_f32.hip, int8: fc_small_i8.hip)
  KERNEL_WIDE,          // int8 large contractions (igemm_i8_wide.hip)
  KERNEL_K3,            // fp32 3x3 stride-1 convolution on well-tiling maps, fp16 matrix cores (conv_k3_f32.hip)
  KERNEL_P3,            // fp32 large contractions on the fp16 matrix cores, operands cut into two pieces (igemm_f32_p3.hip)
  KERNEL_DW             // depthwise 3x3 convolution, fp32 and int8 (conv_dw.hip)
};
struct Plan {
  int kernel;           // KernelKind
  int tile;             // index into the kernel file's tile table (KERNEL_TILED, KERNEL_WIDE)
  int bm, bn, bk;
  int tiles_m, tiles_n;
  int slabs;            // ceil(Kgemm / bk)
  int split_k;
  int slabs_per_split;
  size_t pack_bytes = 0;  // workspace bytes for repacked operands, ahead of the partial sums (KERNEL_P3)
};
Plan plan_f32(const Problem& p, bool allow_split);
Plan plan_i8(const Problem& p, bool allow_split);

// Each launcher validates nothing (the ABI layer did), launches what the plan says on `stream` and
// reports the variant name.  p.partial must be the workspace when plan.split_k > 1.  Returns the
// hipError_t of the launch.
hipError_t launch_f32(const Problem& p, const Plan& plan, hipStream_t stream, const char** variant);
hipError_t launch_i8(const Problem& p, const Plan& plan, hipStream_t stream, const char** variant);

// Few-input-channel first-layer convolution (conv_smallc_f32.hip); used by launch_f32 when applicable.
bool smallc_f32_applicable(const Problem& p);
hipError_t launch_smallc_f32(const Problem& p, hipStream_t stream, const char** variant);
// Pointwise convolution with a short reduction and many pixels (conv_pw_f32.hip).
bool pw_f32_applicable(const Problem& p);
hipError_t launch_pw_f32(const Problem& p, hipStream_t stream, const char** variant);
// fp32 convolution on few pixels with a short reduction, in one launch (conv_small_f32.hip).
bool conv_small_f32_applicable(const Problem& p);
hipError_t launch_conv_small_f32(const Problem& p, hipStream_t stream, const char** variant);
int conv_small_f32_splits(const Problem& p);   // > 1: the split form of that kernel applies, with this many reduction slices
// fp32 FullyConnected with few rows and a small weight matrix, in one launch (fc_small_f32.hip).
bool fc_small_f32_applicable(const Problem& p);
hipError_t launch_fc_small_f32(const Problem& p, hipStream_t stream, const char** variant);
// fp32 large contractions as three fp16 MFMAs per product over operands cut into two fp16 planes (igemm_f32_p3.hip).
bool p3_f32_applicable(const Problem& p);
Plan plan_p3_f32(const Problem& p);
hipError_t launch_p3_f32(const Problem& p, const Plan& plan, hipStream_t stream, const char** variant);
// A tensor's largest magnitude is found as kRangeWords partial maxima (a pass over the tensor), reduced by whoever
// needs it.  A tensor's planes: two fp16 planes of `elems` each, padded to 256 bytes, then a trailer of
// kPlaneTrailerBytes (word 0: the bits of the largest magnitude, the second half: the partial maxima).
constexpr int kRangeWords = 512;
constexpr size_t kRangeBytes = 4 * (size_t)kRangeWords;
constexpr size_t kPlaneTrailerBytes = 2 * kRangeBytes;
// The weights' planes, the form every fp16 three-product kernel reads them in: convolution filters in their own
// [k][r][s][cg] order, FullyConnected weights transposed to [N][K].
// filter_planes_bytes: bytes of that form (a multiple of 256).  launch_pack_filter: measures and writes it
// (b_is_kn: transposed).  stage_filter_planes, for the kernels that cut the input themselves: takes the planes the
// caller made ahead of time (p.w_packed) or measures and cuts the filter into `dst` now; sets p.w_planes / p.w_range.
size_t filter_planes_bytes(size_t w_elems);
hipError_t launch_pack_filter(const float* w, void* dst, int b_is_kn, int K, int N, long long w_elems, hipStream_t stream);
hipError_t stage_filter_planes(Problem& p, const void* dst, hipStream_t stream);
// fp32 3x3 stride-1 convolution over 64 input channels on many pixels, on the fp16 matrix cores (conv_k3c64_f32.hip).
bool k3c64_f32_applicable(const Problem& p);
size_t k3c64_f32_pack_bytes(const Problem& p);
hipError_t launch_k3c64_f32(const Problem& p, hipStream_t stream, const char** variant);
// fp32 3x3 stride-1 convolution with >= 64 input and > 64 output channels on maps that tile into 16 x 16 blocks (conv_k3_f32.hip).
bool k3_f32_applicable(const Problem& p);
size_t k3_f32_pack_bytes(const Problem& p);
hipError_t launch_k3_f32(const Problem& p, hipStream_t stream, const char** variant);
// The same layers with more than 64 output channels on a pixel tile whose shape is chosen per layer (conv_k3v_f32.hip);
// p.w_planes must be set.  k3v_f32_efficiency: share of the machine's block products that are real outputs there.
double k3v_f32_efficiency(const Problem& p);
bool k3v_f32_prefers_fixed_tile(const Problem& p);
hipError_t launch_k3v_f32(const Problem& p, hipStream_t stream, const char** variant);
// Depthwise 3x3 convolution, stride 1 or 2, channels a multiple of four, no tensor operand behind it (conv_dw.hip).
bool dw_f32_applicable(const Problem& p);
hipError_t launch_dw_f32(const Problem& p, hipStream_t stream, const char** variant);
bool dw_i8_applicable(const Problem& p);
hipError_t launch_dw_i8(const Problem& p, hipStream_t stream, const char** variant);
// Finishing kernel of a split fp32 reduction (igemm_f32.hip): sums p.partial in split order, bias, addend, activation.
hipError_t launch_splitk_finish_f32(const Problem& p, const Plan& plan, hipStream_t stream);
bool pw_i8_applicable(const Problem& p);
hipError_t launch_pw_i8(const Problem& p, hipStream_t stream, const char** variant);
// int8 3x3 convolution over 64 input channels on many pixels (conv_k3c64_i8.hip).
bool k3c64_i8_applicable(const Problem& p);
hipError_t launch_k3c64_i8(const Problem& p, hipStream_t stream, const char** variant);
bool smallc_i8_applicable(const Problem& p);
// int8 FullyConnected with at most 64 rows in one launch (fc_small_i8.hip).
bool fc_small_i8_applicable(const Problem& p);
hipError_t launch_fc_small_i8(const Problem& p, hipStream_t stream, const char** variant);
hipError_t launch_smallc_i8(const Problem& p, hipStream_t stream, const char** variant);

// Element-wise conversions between float and quantized tensors (elementwise.hip).
hipError_t launch_quantize(const float* x, signed char* q, long long count, float scale, int offset,
                           hipStream_t stream);
hipError_t launch_dequantize(const signed char* q, float* x, long long count, float scale, int offset,
                             hipStream_t stream);
hipError_t launch_rescale(const signed char* in, signed char* out, long long count, int in_offset, int mant,
                          int shift, int out_offset, hipStream_t stream);

// int8 kernel for large contractions (igemm_i8_wide.hip): 128 x 128 or 128 x 64 output tiles, tile
// indices 4 and 5 of the int8 plan.
bool wide_i8_applicable(const Problem& p);
Plan plan_wide_i8(const Problem& p, int bn, bool allow_split);
hipError_t launch_wide_i8(const Problem& p, const Plan& plan, hipStream_t stream, const char** variant);

}  // namespace glowmi
