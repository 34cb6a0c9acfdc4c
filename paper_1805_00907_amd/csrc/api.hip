// C ABI of glowmi: argument validation, problem set-up and dispatch.  No arithmetic of the
// operators lives here except the host-side derivation of the integer requantization multiplier.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "../../include/glowmi.h"
#include "api_internal.h"
#include "igemm.h"

namespace {

thread_local char g_error[256] = "";
thread_local const char* g_variant = "";

}  // namespace

namespace glowmi {

glowmi_status fail(glowmi_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return s;
}

// ---- tuning knobs: seeded once from the environment, changed only through glowmi_tuning_set ----
namespace {
const char* const kKnobNames[KNOB_COUNT] = {
    "F32_TILE", "F32_SPLIT", "F32_P3", "F32_P3_MIN_M", "F32_P3_RATIO", "F32_P3_BN", "F32_K3C64", "F32_K3C64_MIN_TILES", "F32_K3", "F32_K3_ANY", "F32_K3V", "F32_K3_TH", "F32_K3_TW", "F32_PW_MIN_ITEMS", "F32_PW_BF16", "F32_SMALL_MAX_TILES", "F32_SMALL_NO_SPLIT",
    "F32_SMALL_SPLIT_MAX_TILES", "F32_SMALL_MIN_WGS", "F32_FC_SMALL_OFF", "F32_FC_SMALL_VW", "F32_FC_SMALL_MAX_KB", "F32_FC_SMALL_MIN_M", "SMALLC_TH", "F32_SMALLC_BF16",
    "I8_TILE", "I8_WIDE_SPLIT", "I8_WIDE_NBUF", "SMALLC_I8_WGS", "I8_PW_MIN_ITEMS",
    "I8_FC_SMALL_MAX_M", "I8_K3_MIN_BLOCKS", "I8_K3_WAVES", "I8_K3_GATHER", "DW",
};
std::atomic<int> g_knobs[KNOB_COUNT];
std::once_flag g_knobs_once;

void seed_knobs_from_environment() {
  for (int i = 0; i < KNOB_COUNT; ++i) {
    char name[64];
    snprintf(name, sizeof(name), "GLOWMI_%s", kKnobNames[i]);
    const char* env = getenv(name);
    int v = kKnobUnset;
    if (env && *env) {
      char* end = nullptr;
      const long parsed = strtol(env, &end, 10);
      if (end != env && parsed > -(1L << 30) && parsed < (1L << 30)) v = (int)parsed;
    }
    g_knobs[i].store(v, std::memory_order_relaxed);
  }
}
}  // namespace

int knob(Knob k) {
  std::call_once(g_knobs_once, seed_knobs_from_environment);
  return g_knobs[k].load(std::memory_order_relaxed);
}

int num_compute_units() {
  static const int n = []() {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return cu;
  }();
  return n;
}

}  // namespace glowmi

namespace {
using glowmi::fail;

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

constexpr long long kMaxElems = (1LL << 31) - 1;
constexpr long long kMaxOperandBytes = (1LL << 32) - 64;   // inputs are read through 32-bit buffer offsets
constexpr int kMaxExtent = 1 << 20;       // spatial / filter extents; keeps row arithmetic in int32
constexpr int kMaxQuantDepth = 65535;     // deepest reduction the quantized kernels are built and tested for

struct Geometry {
  int oh, ow;
  long long x_elems, w_elems, y_elems;
};

glowmi_status check_desc(const glowmi_conv_desc* d, Geometry* geo) {
  if (!d) return fail(GLOWMI_ERR_NULL, "descriptor is NULL");
  if (d->n <= 0 || d->h <= 0 || d->w <= 0 || d->c <= 0 || d->k <= 0 || d->r <= 0 || d->s <= 0)
    return fail(GLOWMI_ERR_SHAPE, "extents must be positive (n=%d h=%d w=%d c=%d k=%d r=%d s=%d)", d->n,
                d->h, d->w, d->c, d->k, d->r, d->s);
  if (d->stride_h <= 0 || d->stride_w <= 0)
    return fail(GLOWMI_ERR_SHAPE, "strides must be positive (%d, %d)", d->stride_h, d->stride_w);
  if (d->pad_t < 0 || d->pad_l < 0 || d->pad_b < 0 || d->pad_r < 0)
    return fail(GLOWMI_ERR_SHAPE, "pads must be non-negative");
  if (d->groups <= 0 || d->c % d->groups != 0 || d->k % d->groups != 0)
    return fail(GLOWMI_ERR_SHAPE, "groups=%d must divide c=%d and k=%d", d->groups, d->c, d->k);
  const long long span_h = (long long)d->h + d->pad_t + d->pad_b - d->r;
  const long long span_w = (long long)d->w + d->pad_l + d->pad_r - d->s;
  if (span_h < 0 || span_w < 0)
    return fail(GLOWMI_ERR_SHAPE, "filter %dx%d larger than padded input %lldx%lld", d->r, d->s,
                (long long)d->h + d->pad_t + d->pad_b, (long long)d->w + d->pad_l + d->pad_r);
  if (d->h > kMaxExtent || d->w > kMaxExtent || d->r > kMaxExtent || d->s > kMaxExtent ||
      d->pad_t > kMaxExtent || d->pad_l > kMaxExtent || d->pad_b > kMaxExtent || d->pad_r > kMaxExtent ||
      d->stride_h > kMaxExtent || d->stride_w > kMaxExtent)
    return fail(GLOWMI_ERR_UNSUPPORTED, "spatial extents, pads and strides are limited to 2^20");
  const long long oh = span_h / d->stride_h + 1, ow = span_w / d->stride_w + 1;
  geo->oh = (int)oh;
  geo->ow = (int)ow;
  geo->x_elems = (long long)d->n * d->h * d->w * d->c;
  geo->w_elems = (long long)d->k * d->r * d->s * (d->c / d->groups);
  geo->y_elems = (long long)d->n * oh * ow * d->k;
  if (geo->x_elems > kMaxElems || geo->w_elems > kMaxElems || geo->y_elems > kMaxElems)
    return fail(GLOWMI_ERR_UNSUPPORTED, "a tensor has 2^31 or more elements");
  return GLOWMI_OK;
}

void fill_divs(glowmi::Problem& p) {
  p.addend = nullptr;
  p.r_off = 0; p.r_mant = 0; p.r_shift = 1;
  p.div_ohow = glowmi::make_fastdiv((uint32_t)p.oh * (uint32_t)p.ow);
  p.div_ow = glowmi::make_fastdiv((uint32_t)p.ow);
  p.div_cg = glowmi::make_fastdiv((uint32_t)p.cg);
  p.div_s = glowmi::make_fastdiv((uint32_t)p.s);
}

void fill_conv(glowmi::Problem& p, const glowmi_conv_desc* d, const Geometry& geo) {
  std::memset(&p, 0, sizeof(p));
  p.allow_pack = 1;
  p.n = d->n; p.h = d->h; p.w_ = d->w; p.c = d->c;
  p.k = d->k; p.r = d->r; p.s = d->s;
  p.oh = geo.oh; p.ow = geo.ow;
  p.stride_h = d->stride_h; p.stride_w = d->stride_w;
  p.pad_t = d->pad_t; p.pad_l = d->pad_l;
  p.groups = d->groups; p.cg = d->c / d->groups; p.kg = d->k / d->groups;
  p.M = d->n * geo.oh * geo.ow;
  p.Kgemm = d->r * d->s * p.cg;
  p.split_k = 1;
  p.slabs_per_split = 0;
  p.b_is_kn = 0;
  fill_divs(p);
}

glowmi_status check_fc(int32_t M, int32_t K, int32_t N) {
  if (M <= 0 || K <= 0 || N <= 0)
    return fail(GLOWMI_ERR_SHAPE, "extents must be positive (M=%d K=%d N=%d)", M, K, N);
  if ((long long)M * K > kMaxElems || (long long)K * N > kMaxElems || (long long)M * N > kMaxElems)
    return fail(GLOWMI_ERR_UNSUPPORTED, "a tensor has 2^31 or more elements");
  return GLOWMI_OK;
}

// FullyConnected as the same contraction: rows are "images" of a 1x1 map with K channels.
void fill_fc(glowmi::Problem& p, int32_t M, int32_t K, int32_t N) {
  std::memset(&p, 0, sizeof(p));
  p.allow_pack = 1;
  p.n = M; p.h = 1; p.w_ = 1; p.c = K;
  p.k = N; p.r = 1; p.s = 1;
  p.oh = 1; p.ow = 1;
  p.stride_h = 1; p.stride_w = 1;
  p.groups = 1; p.cg = K; p.kg = N;
  p.M = M;
  p.Kgemm = K;
  p.split_k = 1;
  p.b_is_kn = 1;
  fill_divs(p);
}

// Input and weight tensors are read with buffer loads whose range check covers 4 GiB.
glowmi_status set_operand_bytes(glowmi::Problem& p, long long x_elems, long long w_elems, int elem) {
  if (x_elems * elem > kMaxOperandBytes || w_elems * elem > kMaxOperandBytes)
    return fail(GLOWMI_ERR_UNSUPPORTED, "input or weight tensor larger than 4 GiB");
  p.x_bytes = (uint32_t)(x_elems * elem);
  p.w_bytes = (uint32_t)(w_elems * elem);
  return GLOWMI_OK;
}

glowmi_status check_act(glowmi_act act) {
  if (act != GLOWMI_ACT_NONE && act != GLOWMI_ACT_RELU)
    return fail(GLOWMI_ERR_UNSUPPORTED, "unknown activation %d", (int)act);
  return GLOWMI_OK;
}

glowmi_status check_ptrs(const void* x, const void* w, const void* bias, const void* y) {
  if (!x || !w || !y) return fail(GLOWMI_ERR_NULL, "input, weight and output pointers must not be NULL");
  if (!aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16))
    return fail(GLOWMI_ERR_ALIGN, "input, weight and output pointers must be 16-byte aligned");
  if (bias && !aligned(bias, 4)) return fail(GLOWMI_ERR_ALIGN, "bias must be 4-byte aligned");
  return GLOWMI_OK;
}

// The tensor operand of a chain: aligned, and either the output itself or disjoint from it.
glowmi_status check_addend(const void* addend, const void* y, size_t bytes) {
  if (!addend) return GLOWMI_OK;
  if (!aligned(addend, 16)) return fail(GLOWMI_ERR_ALIGN, "addend must be 16-byte aligned");
  const uintptr_t a = reinterpret_cast<uintptr_t>(addend), o = reinterpret_cast<uintptr_t>(y);
  if (a != o && a < o + bytes && o < a + bytes)
    return fail(GLOWMI_ERR_UNSUPPORTED, "addend overlaps the output without being the output itself");
  return GLOWMI_OK;
}

bool workspace_usable(const void* ws, size_t have, size_t need) {
  return ws != nullptr && need > 0 && have >= need && aligned(ws, 16);
}

// Largest magnitude the sum of products of a reduction of depth Kgemm can reach: a code minus its
// offset lies in [-128 - off, 127 - off], so |x - x_off| <= 128 + |x_off| and likewise for the filter
// (Section 4.1 tensor type: codes and offsets in [-128, 127]).  The call is accepted only when that
// bound leaves kAccHeadroom below 2^31 for the bias and the rescaled addend.
constexpr long long kAccHeadroom = 1LL << 27;
// Smallest shift accepted for the multiplier of a quantized addend: a code difference reaches 255 and
// mant < 2^31, so 255 * mant * 2^-shift < 2^27 needs shift >= 12.
constexpr int kMinAddendShift = 12;

glowmi_status quant_setup(glowmi::Problem& p, glowmi_qparam xq, glowmi_qparam wq, glowmi_qparam yq,
                          glowmi_act act) {
  if (xq.offset < -128 || xq.offset > 127 || wq.offset < -128 || wq.offset > 127 || yq.offset < -128 ||
      yq.offset > 127)
    return fail(GLOWMI_ERR_QUANT, "offsets must lie in [-128, 127] (x %d, w %d, y %d)", xq.offset, wq.offset,
                yq.offset);
  int32_t mant = 0, shift = 0;
  glowmi_status st = glowmi_requant_params(xq.scale, wq.scale, yq.scale, &mant, &shift);
  if (st != GLOWMI_OK) return st;
  if (p.Kgemm > kMaxQuantDepth)
    return fail(GLOWMI_ERR_UNSUPPORTED, "reduction depth %d exceeds %d", p.Kgemm, kMaxQuantDepth);
  const long long xmax = 128 + (xq.offset < 0 ? -xq.offset : xq.offset);
  const long long wmax = 128 + (wq.offset < 0 ? -wq.offset : wq.offset);
  const long long bound = (long long)p.Kgemm * xmax * wmax;
  if (bound > (1LL << 31) - kAccHeadroom)
    return fail(GLOWMI_ERR_UNSUPPORTED,
                "reduction depth %d with offsets x %d, w %d: the sum of products can reach %lld, too close to 2^31 "
                "for an int32 accumulator", p.Kgemm, xq.offset, wq.offset, bound);
  p.x_off = xq.offset; p.w_off = wq.offset; p.y_off = yq.offset;
  p.mant = mant; p.shift = shift;
  p.lo = (act == GLOWMI_ACT_RELU && yq.offset > -128) ? yq.offset : -128;
  return GLOWMI_OK;
}

glowmi_status finish(hipError_t e, const char* variant) {
  if (e != hipSuccess) return fail(GLOWMI_ERR_HIP, "launch failed: %s", hipGetErrorString(e));
  g_variant = variant;
  g_error[0] = 0;
  return GLOWMI_OK;
}

// Workspace a plan wants: repacked operands first (a multiple of 256 bytes), then the partial sums of a split reduction.
size_t split_bytes(const glowmi::Plan& pl, const glowmi::Problem& p) {
  return pl.pack_bytes + (pl.split_k > 1 ? (size_t)pl.split_k * (size_t)p.M * (size_t)p.k * 4u : 0u);
}

// Plan once per call: with what the planner wants from a workspace (repacked operands, a split reduction)
// when the caller's workspace can hold it, without either otherwise.  Sets p.planes and p.partial accordingly.
template <typename PlanFn>
glowmi::Plan plan_with_workspace(glowmi::Problem& p, PlanFn plan_fn, void* workspace, size_t workspace_bytes) {
  glowmi::Plan plan = plan_fn(p, true);
  const size_t need = split_bytes(plan, p);
  p.partial = nullptr;
  p.planes = nullptr;
  if (need > 0) {
    if (workspace_usable(workspace, workspace_bytes, need)) {
      if (plan.pack_bytes > 0) p.planes = workspace;
      if (plan.split_k > 1) p.partial = static_cast<unsigned char*>(workspace) + plan.pack_bytes;
    } else {
      plan = plan_fn(p, false);
    }
  }
  return plan;
}

// Bytes of the bf16 planes of a layer's weights, 0 when the shape has no plane form: the kernels that read
// planes fetch 8 consecutive reduction indices of one output channel at a time and address a plane with 29 bits.
constexpr long long kMaxPlaneElems = 1LL << 28;
size_t conv_planes_bytes(const glowmi_conv_desc* d, const Geometry& geo) {
  if ((d->c / d->groups) % 8 != 0 || geo.w_elems > kMaxPlaneElems) return 0;
  return glowmi::filter_planes_bytes((size_t)geo.w_elems);
}
size_t fc_planes_bytes(int32_t K, int32_t N) {
  if (K % 8 != 0 || (long long)K * N > kMaxPlaneElems) return 0;
  return glowmi::filter_planes_bytes((size_t)K * (size_t)N);
}

// The planes argument of the *_packed entry points: NULL, or aligned planes of a shape that has a plane form.
glowmi_status check_w_planes(const void* w_planes, size_t planes_bytes) {
  if (!w_planes) return GLOWMI_OK;
  if (planes_bytes == 0)
    return fail(GLOWMI_ERR_UNSUPPORTED, "this shape has no plane form of its weights: pass w_planes = NULL");
  if (!aligned(w_planes, 16)) return fail(GLOWMI_ERR_ALIGN, "w_planes must be 16-byte aligned");
  return GLOWMI_OK;
}

glowmi_status check_pack_args(const float* w, void* planes, size_t planes_bytes, size_t need) {
  if (!w || !planes) return fail(GLOWMI_ERR_NULL, "weight and plane pointers must not be NULL");
  if (!aligned(w, 16) || !aligned(planes, 16))
    return fail(GLOWMI_ERR_ALIGN, "weight and plane pointers must be 16-byte aligned");
  if (need == 0)
    return fail(GLOWMI_ERR_UNSUPPORTED, "this shape has no plane form of its weights (reduction extent per "
                "output channel not a multiple of 8, or more than 2^28 weights)");
  if (planes_bytes < need)
    return fail(GLOWMI_ERR_SHAPE, "planes_bytes %zu is less than the %zu the planes take", planes_bytes, need);
  return GLOWMI_OK;
}

glowmi_status setup_fc_f32(const float* a, const float* w, const float* bias, float* y, int32_t M, int32_t K,
                           int32_t N, glowmi_act act, glowmi::Problem& p) {
  glowmi_status st = check_fc(M, K, N);
  if (st != GLOWMI_OK) return st;
  if ((st = check_ptrs(a, w, bias, y)) != GLOWMI_OK) return st;
  if ((st = check_act(act)) != GLOWMI_OK) return st;
  fill_fc(p, M, K, N);
  if ((st = set_operand_bytes(p, (long long)M * K, (long long)K * N, 4)) != GLOWMI_OK) return st;
  p.x = a; p.w = w; p.bias = bias; p.y = y; p.act = (int)act;
  return GLOWMI_OK;
}

// ---- the scratch buffer of the entry point that allocates nothing (glowmi_fc_noalloc) --------------
// One copy per GPU, held until the process ends.  In host code the array's name is only a stand-in: the
// device address comes from hipGetSymbolAddress, once per device, and is what the kernels are given.
constexpr size_t kScratchBytes = 8u << 20;
constexpr int kMaxDevices = 64;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
struct ScratchSlot {
  std::once_flag once;
  hipError_t status = hipErrorNotInitialized;
  void* ptr = nullptr;
};
ScratchSlot g_scratch_slots[kMaxDevices];

// Device address of `scratch` on the current device (looked up on the first call there).
hipError_t scratch_pointer(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  ScratchSlot& slot = g_scratch_slots[dev];
  std::call_once(slot.once, [&slot]() {
    void* p = nullptr;
    slot.status = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    slot.ptr = slot.status == hipSuccess ? p : nullptr;
  });
  if (slot.status != hipSuccess) return slot.status;
  if (!slot.ptr) return hipErrorInvalidSymbol;
  *out = slot.ptr;
  return hipSuccess;
}
}  // namespace

namespace glowmi {

glowmi_status prepare_conv2d_chain(const float* x, const float* w, const float* bias, float* y,
                                   const glowmi_conv_desc* d, const glowmi_chain* chain, void* workspace,
                                   size_t workspace_bytes, PreparedCall* out, const void* w_planes) {
  if (!chain) return fail(GLOWMI_ERR_NULL, "chain must not be NULL");
  const glowmi_act act = chain->act;
  Geometry geo;
  glowmi_status st = check_desc(d, &geo);
  if (st != GLOWMI_OK) return st;
  if ((st = check_ptrs(x, w, bias, y)) != GLOWMI_OK) return st;
  if ((st = check_act(act)) != GLOWMI_OK) return st;
  if ((st = check_addend(chain->addend, y, (size_t)geo.y_elems * 4u)) != GLOWMI_OK) return st;
  if ((st = check_w_planes(w_planes, conv_planes_bytes(d, geo))) != GLOWMI_OK) return st;
  Problem& p = out->p;
  fill_conv(p, d, geo);
  if ((st = set_operand_bytes(p, geo.x_elems, geo.w_elems, 4)) != GLOWMI_OK) return st;
  p.x = x; p.w = w; p.bias = bias; p.y = y; p.act = (int)act;
  p.w_packed = w_planes;
  p.addend = chain->addend;
  out->plan = plan_with_workspace(p, plan_f32, workspace, workspace_bytes);
  out->quantized = false;
  return GLOWMI_OK;
}

glowmi_status prepare_qconv2d_chain(const int8_t* x, glowmi_qparam xq, const int8_t* w, glowmi_qparam wq,
                                    const int32_t* bias, int8_t* y, glowmi_qparam yq, const glowmi_conv_desc* d,
                                    const glowmi_chain* chain, void* workspace, size_t workspace_bytes,
                                    PreparedCall* out) {
  if (!chain) return fail(GLOWMI_ERR_NULL, "chain must not be NULL");
  const glowmi_act act = chain->act;
  Geometry geo;
  glowmi_status st = check_desc(d, &geo);
  if (st != GLOWMI_OK) return st;
  if ((st = check_ptrs(x, w, bias, y)) != GLOWMI_OK) return st;
  if ((st = check_act(act)) != GLOWMI_OK) return st;
  if ((st = check_addend(chain->addend, y, (size_t)geo.y_elems)) != GLOWMI_OK) return st;
  Problem& p = out->p;
  fill_conv(p, d, geo);
  if ((st = set_operand_bytes(p, geo.x_elems, geo.w_elems, 1)) != GLOWMI_OK) return st;
  if ((st = quant_setup(p, xq, wq, yq, act)) != GLOWMI_OK) return st;
  p.x = x; p.w = w; p.bias = bias; p.y = y; p.act = (int)act;
  if (chain->addend) {
    if (chain->addend_q.offset < -128 || chain->addend_q.offset > 127)
      return fail(GLOWMI_ERR_QUANT, "addend offset %d outside [-128, 127]", chain->addend_q.offset);
    int32_t r_mant = 0, r_shift = 0;
    if ((st = glowmi_rescale_params(chain->addend_q.scale, xq.scale, wq.scale, &r_mant, &r_shift)) != GLOWMI_OK)
      return st;
    // the rescaled term must fit the int32 accumulator with room to spare
    if (r_shift < kMinAddendShift)
      return fail(GLOWMI_ERR_QUANT,
                  "addend scale %g is more than 2^%d times the accumulator's scale %g: the rescaled addend "
                  "would not fit the int32 accumulator", (double)chain->addend_q.scale, 31 - kMinAddendShift,
                  (double)xq.scale * (double)wq.scale);
    p.addend = chain->addend;
    p.r_off = chain->addend_q.offset; p.r_mant = r_mant; p.r_shift = r_shift;
  }
  out->plan = plan_with_workspace(p, plan_i8, workspace, workspace_bytes);
  out->quantized = true;
  return GLOWMI_OK;
}

glowmi_status run_prepared(const PreparedCall& call, hipStream_t stream) {
  const char* variant = "";
  const hipError_t e = call.quantized ? launch_i8(call.p, call.plan, stream, &variant)
                                      : launch_f32(call.p, call.plan, stream, &variant);
  return finish(e, variant);
}

}  // namespace glowmi

extern "C" {

glowmi_status glowmi_conv_out_shape(const glowmi_conv_desc* d, int32_t* oh, int32_t* ow) {
  Geometry geo;
  glowmi_status st = check_desc(d, &geo);
  if (st != GLOWMI_OK) return st;
  if (oh) *oh = geo.oh;
  if (ow) *ow = geo.ow;
  return GLOWMI_OK;
}

size_t glowmi_conv2d_workspace_bytes(const glowmi_conv_desc* d) {
  Geometry geo;
  if (check_desc(d, &geo) != GLOWMI_OK) return 0;
  glowmi::Problem p;
  fill_conv(p, d, geo);
  if (set_operand_bytes(p, geo.x_elems, geo.w_elems, 4) != GLOWMI_OK) return 0;   // the planner sees what the call sees
  return split_bytes(glowmi::plan_f32(p, true), p);
}

glowmi_status glowmi_conv2d(const float* x, const float* w, const float* bias, float* y,
                            const glowmi_conv_desc* d, glowmi_act act, void* workspace,
                            size_t workspace_bytes, hipStream_t stream) {
  glowmi_chain chain;
  chain.addend = nullptr;
  chain.addend_q.scale = 1.0f;
  chain.addend_q.offset = 0;
  chain.act = act;
  return glowmi_conv2d_chain(x, w, bias, y, d, &chain, workspace, workspace_bytes, stream);
}

glowmi_status glowmi_conv2d_chain(const float* x, const float* w, const float* bias, float* y,
                                  const glowmi_conv_desc* d, const glowmi_chain* chain, void* workspace,
                                  size_t workspace_bytes, hipStream_t stream) {
  glowmi::PreparedCall call;
  glowmi_status st = glowmi::prepare_conv2d_chain(x, w, bias, y, d, chain, workspace, workspace_bytes, &call);
  if (st != GLOWMI_OK) return st;
  return glowmi::run_prepared(call, stream);
}

size_t glowmi_fc_workspace_bytes(int32_t M, int32_t K, int32_t N) {
  if (check_fc(M, K, N) != GLOWMI_OK) return 0;
  glowmi::Problem p;
  fill_fc(p, M, K, N);
  if (set_operand_bytes(p, (long long)M * K, (long long)K * N, 4) != GLOWMI_OK) return 0;
  return split_bytes(glowmi::plan_f32(p, true), p);
}

glowmi_status glowmi_fc(const float* a, const float* w, const float* bias, float* y, int32_t M,
                        int32_t K, int32_t N, glowmi_act act, void* workspace,
                        size_t workspace_bytes, hipStream_t stream) {
  return glowmi_fc_packed(a, w, nullptr, bias, y, M, K, N, act, workspace, workspace_bytes, stream);
}

// ---- filters transformed ahead of time ----------------------------------------------------------------
// The planner only asks whether planes were given, so the workspace queries plan with a stand-in address.
static const unsigned char kPlanesGiven = 0;

size_t glowmi_conv2d_filter_planes_bytes(const glowmi_conv_desc* d) {
  Geometry geo;
  if (check_desc(d, &geo) != GLOWMI_OK) return 0;
  return conv_planes_bytes(d, geo);
}

glowmi_status glowmi_conv2d_pack_filter(const float* w, const glowmi_conv_desc* d, void* planes,
                                        size_t planes_bytes, hipStream_t stream) {
  Geometry geo;
  glowmi_status st = check_desc(d, &geo);
  if (st != GLOWMI_OK) return st;
  if ((st = check_pack_args(w, planes, planes_bytes, conv_planes_bytes(d, geo))) != GLOWMI_OK) return st;
  return finish(glowmi::launch_pack_filter(w, planes, 0, 0, 0, geo.w_elems, stream), "pack_filter_rows");
}

size_t glowmi_conv2d_packed_workspace_bytes(const glowmi_conv_desc* d) {
  Geometry geo;
  if (check_desc(d, &geo) != GLOWMI_OK) return 0;
  glowmi::Problem p;
  fill_conv(p, d, geo);
  if (set_operand_bytes(p, geo.x_elems, geo.w_elems, 4) != GLOWMI_OK) return 0;
  if (conv_planes_bytes(d, geo) > 0) p.w_packed = &kPlanesGiven;
  return split_bytes(glowmi::plan_f32(p, true), p);
}

glowmi_status glowmi_conv2d_packed(const float* x, const float* w, const void* w_planes, const float* bias,
                                   float* y, const glowmi_conv_desc* d, const glowmi_chain* chain,
                                   void* workspace, size_t workspace_bytes, hipStream_t stream) {
  glowmi::PreparedCall call;
  glowmi_status st =
      glowmi::prepare_conv2d_chain(x, w, bias, y, d, chain, workspace, workspace_bytes, &call, w_planes);
  if (st != GLOWMI_OK) return st;
  return glowmi::run_prepared(call, stream);
}

size_t glowmi_fc_filter_planes_bytes(int32_t K, int32_t N) {
  if (check_fc(1, K, N) != GLOWMI_OK) return 0;
  return fc_planes_bytes(K, N);
}

glowmi_status glowmi_fc_pack_filter(const float* w, int32_t K, int32_t N, void* planes, size_t planes_bytes,
                                    hipStream_t stream) {
  glowmi_status st = check_fc(1, K, N);
  if (st != GLOWMI_OK) return st;
  if ((st = check_pack_args(w, planes, planes_bytes, fc_planes_bytes(K, N))) != GLOWMI_OK) return st;
  return finish(glowmi::launch_pack_filter(w, planes, 1, K, N, (long long)K * N, stream), "pack_filter_transposed");
}

size_t glowmi_fc_packed_workspace_bytes(int32_t M, int32_t K, int32_t N) {
  if (check_fc(M, K, N) != GLOWMI_OK) return 0;
  glowmi::Problem p;
  fill_fc(p, M, K, N);
  if (set_operand_bytes(p, (long long)M * K, (long long)K * N, 4) != GLOWMI_OK) return 0;
  if (fc_planes_bytes(K, N) > 0) p.w_packed = &kPlanesGiven;
  return split_bytes(glowmi::plan_f32(p, true), p);
}

glowmi_status glowmi_fc_packed(const float* a, const float* w, const void* w_planes, const float* bias,
                               float* y, int32_t M, int32_t K, int32_t N, glowmi_act act, void* workspace,
                               size_t workspace_bytes, hipStream_t stream) {
  glowmi::Problem p;
  glowmi_status st = setup_fc_f32(a, w, bias, y, M, K, N, act, p);
  if (st != GLOWMI_OK) return st;
  if ((st = check_w_planes(w_planes, fc_planes_bytes(K, N))) != GLOWMI_OK) return st;
  p.w_packed = w_planes;
  const glowmi::Plan plan = plan_with_workspace(p, glowmi::plan_f32, workspace, workspace_bytes);
  const char* variant = "";
  return finish(glowmi::launch_f32(p, plan, stream, &variant), variant);
}

size_t glowmi_fc_noalloc_max_scratch_bytes(void) { return kScratchBytes; }

glowmi_status glowmi_fc_noalloc(const float* a, const float* w, const float* bias, float* y, int32_t M,
                                int32_t K, int32_t N, glowmi_act act, hipStream_t stream) {
  glowmi::Problem p;
  glowmi_status st = setup_fc_f32(a, w, bias, y, M, K, N, act, p);
  if (st != GLOWMI_OK) return st;
  p.allow_pack = 0;     // the static buffer is for partial sums only: operands are never repacked into it
  const glowmi::Plan plan = glowmi::plan_f32(p, true);      // otherwise the plan glowmi_fc takes with a full workspace
  const size_t need = split_bytes(plan, p);
  if (need > kScratchBytes)
    return fail(GLOWMI_ERR_UNSUPPORTED,
                "FullyConnected %d x %d x %d needs %zu bytes of split-reduction scratch, more than the %zu the "
                "library's static buffer holds: use glowmi_fc with a workspace", M, K, N, need, kScratchBytes);
  if (need > 0) {
    void* ptr = nullptr;
    const hipError_t e = scratch_pointer(&ptr);
    if (e != hipSuccess) return fail(GLOWMI_ERR_HIP, "static scratch buffer unavailable: %s", hipGetErrorString(e));
    p.partial = ptr;     // every partial sum is written before it is read: nothing needs clearing
  }
  const char* variant = "";
  return finish(glowmi::launch_f32(p, plan, stream, &variant), variant);
}

size_t glowmi_qconv2d_workspace_bytes(const glowmi_conv_desc* d) {
  Geometry geo;
  if (check_desc(d, &geo) != GLOWMI_OK) return 0;
  glowmi::Problem p;
  fill_conv(p, d, geo);
  if (set_operand_bytes(p, geo.x_elems, geo.w_elems, 1) != GLOWMI_OK) return 0;
  return split_bytes(glowmi::plan_i8(p, true), p);
}

glowmi_status glowmi_qconv2d(const int8_t* x, glowmi_qparam xq, const int8_t* w, glowmi_qparam wq,
                             const int32_t* bias, int8_t* y, glowmi_qparam yq,
                             const glowmi_conv_desc* d, glowmi_act act, void* workspace,
                             size_t workspace_bytes, hipStream_t stream) {
  glowmi_chain chain;
  chain.addend = nullptr;
  chain.addend_q.scale = 1.0f;
  chain.addend_q.offset = 0;
  chain.act = act;
  return glowmi_qconv2d_chain(x, xq, w, wq, bias, y, yq, d, &chain, workspace, workspace_bytes, stream);
}

glowmi_status glowmi_qconv2d_chain(const int8_t* x, glowmi_qparam xq, const int8_t* w, glowmi_qparam wq,
                                   const int32_t* bias, int8_t* y, glowmi_qparam yq,
                                   const glowmi_conv_desc* d, const glowmi_chain* chain, void* workspace,
                                   size_t workspace_bytes, hipStream_t stream) {
  glowmi::PreparedCall call;
  glowmi_status st =
      glowmi::prepare_qconv2d_chain(x, xq, w, wq, bias, y, yq, d, chain, workspace, workspace_bytes, &call);
  if (st != GLOWMI_OK) return st;
  return glowmi::run_prepared(call, stream);
}

size_t glowmi_qfc_workspace_bytes(int32_t M, int32_t K, int32_t N) {
  if (check_fc(M, K, N) != GLOWMI_OK) return 0;
  glowmi::Problem p;
  fill_fc(p, M, K, N);
  if (set_operand_bytes(p, (long long)M * K, (long long)K * N, 1) != GLOWMI_OK) return 0;
  return split_bytes(glowmi::plan_i8(p, true), p);
}

glowmi_status glowmi_qfc(const int8_t* a, glowmi_qparam aq, const int8_t* w, glowmi_qparam wq,
                         const int32_t* bias, int8_t* y, glowmi_qparam yq, int32_t M, int32_t K,
                         int32_t N, glowmi_act act, void* workspace, size_t workspace_bytes,
                         hipStream_t stream) {
  glowmi_status st = check_fc(M, K, N);
  if (st != GLOWMI_OK) return st;
  if ((st = check_ptrs(a, w, bias, y)) != GLOWMI_OK) return st;
  if ((st = check_act(act)) != GLOWMI_OK) return st;
  glowmi::Problem p;
  fill_fc(p, M, K, N);
  if ((st = set_operand_bytes(p, (long long)M * K, (long long)K * N, 1)) != GLOWMI_OK) return st;
  if ((st = quant_setup(p, aq, wq, yq, act)) != GLOWMI_OK) return st;
  p.x = a; p.w = w; p.bias = bias; p.y = y; p.act = (int)act;
  const glowmi::Plan plan = plan_with_workspace(p, glowmi::plan_i8, workspace, workspace_bytes);
  const char* variant = "";
  return finish(glowmi::launch_i8(p, plan, stream, &variant), variant);
}

glowmi_status glowmi_tuning_set(const char* name, int32_t value) {
  if (!name) return fail(GLOWMI_ERR_NULL, "knob name is NULL");
  glowmi::knob(glowmi::KNOB_F32_TILE);                    // make sure the environment has been read first
  for (int i = 0; i < glowmi::KNOB_COUNT; ++i)
    if (std::strcmp(name, glowmi::kKnobNames[i]) == 0) {
      glowmi::g_knobs[i].store(value, std::memory_order_relaxed);
      return GLOWMI_OK;
    }
  return fail(GLOWMI_ERR_UNSUPPORTED, "unknown tuning knob \"%s\"", name);
}

void glowmi_tuning_reset(void) {
  glowmi::knob(glowmi::KNOB_F32_TILE);
  for (int i = 0; i < glowmi::KNOB_COUNT; ++i) glowmi::g_knobs[i].store(glowmi::kKnobUnset, std::memory_order_relaxed);
}

}  // extern "C"

// ---- general chains ---------------------------------------------------------------------------------
namespace {

// The op lists that are one of the fixed chain shapes take the entry points (and kernels) of those.
bool fixed_shape(const glowmi_chain_op* ops, int32_t n, glowmi_chain* chain) {
  chain->addend = nullptr;
  chain->addend_q.scale = 1.0f;
  chain->addend_q.offset = 0;
  chain->act = GLOWMI_ACT_NONE;
  int i = 0;
  if (i < n && ops[i].kind == GLOWMI_OP_ADD_TENSOR && ops[i].tensor) {
    chain->addend = ops[i].tensor;
    chain->addend_q = ops[i].tensor_q;
    ++i;
  }
  if (i < n && ops[i].kind == GLOWMI_OP_MAX_SCALAR && ops[i].a == 0.0f) {
    chain->act = GLOWMI_ACT_RELU;
    ++i;
  }
  return i == n;
}

glowmi_status check_op_list(const glowmi_chain_op* ops, int32_t n) {
  if (n < 0 || n > GLOWMI_MAX_CHAIN_OPS)
    return fail(GLOWMI_ERR_UNSUPPORTED, "a chain has 0 to %d ops (got %d)", GLOWMI_MAX_CHAIN_OPS, n);
  if (n > 0 && !ops) return fail(GLOWMI_ERR_NULL, "op list is NULL");
  for (int32_t i = 0; i < n; ++i)
    if (ops[i].kind < GLOWMI_OP_ADD_TENSOR || ops[i].kind > GLOWMI_OP_CLIP)
      return fail(GLOWMI_ERR_UNSUPPORTED, "op %d: unknown kind %d", i, (int)ops[i].kind);
  return GLOWMI_OK;
}

// Fill p.chain for the fp32 form; y_bytes for the overlap rule of added tensors.
glowmi_status fill_chain_f32(glowmi::Problem& p, const glowmi_chain_op* ops, int32_t n, const void* y, size_t y_bytes) {
  p.chain_n = n;
  p.addend = nullptr;
  p.act = 0;
  for (int32_t i = 0; i < n; ++i) {
    glowmi::ChainOpDev& o = p.chain[i];
    o.kind = (int32_t)ops[i].kind;
    o.a = ops[i].a; o.b = ops[i].b;
    o.tensor = nullptr;
    switch (ops[i].kind) {
      case GLOWMI_OP_ADD_TENSOR: {
        if (!ops[i].tensor) return fail(GLOWMI_ERR_NULL, "op %d: tensor is NULL", i);
        glowmi_status st = check_addend(ops[i].tensor, y, y_bytes);
        if (st != GLOWMI_OK) return st;
        o.tensor = ops[i].tensor;
        break;
      }
      case GLOWMI_OP_MUL_SCALAR:
      case GLOWMI_OP_MAX_SCALAR:
        if (std::isnan(ops[i].a)) return fail(GLOWMI_ERR_SHAPE, "op %d: scalar is NaN", i);
        break;
      case GLOWMI_OP_CLIP:
        if (!(ops[i].a <= ops[i].b)) return fail(GLOWMI_ERR_SHAPE, "op %d: clip bounds %g > %g or NaN", i, (double)ops[i].a, (double)ops[i].b);
        break;
    }
  }
  return GLOWMI_OK;
}

// A real bound on an accumulator grid of step s: floor(v / s + 0.5), saturated to int32.
int32_t grid_bound(float v, double s) {
  const double t = std::floor((double)v / s + 0.5);
  if (t != t) return 0;
  if (t <= -2147483648.0) return INT32_MIN;
  if (t >= 2147483647.0) return INT32_MAX;
  return (int32_t)t;
}

glowmi_status multiplier_params_fwd(double mr, int32_t* mant, int32_t* shift);

// Fill p.chain, p.mant, p.shift, p.lo for the quantized form.
glowmi_status fill_chain_i8(glowmi::Problem& p, const glowmi_chain_op* ops, int32_t n, glowmi_qparam xq, glowmi_qparam wq,
                            glowmi_qparam yq, const void* y, size_t y_bytes) {
  p.chain_n = n;
  p.addend = nullptr;
  p.act = 0;
  p.lo = -128;
  double s = (double)xq.scale * (double)wq.scale;     // the accumulator's scale
  for (int32_t i = 0; i < n; ++i) {
    glowmi::ChainOpDev& o = p.chain[i];
    o.kind = (int32_t)ops[i].kind;
    o.a = ops[i].a; o.b = ops[i].b;
    o.tensor = nullptr;
    o.ia = o.ib = 0; o.t_off = 0; o.t_mant = 0; o.t_shift = 1;
    switch (ops[i].kind) {
      case GLOWMI_OP_ADD_TENSOR: {
        if (!ops[i].tensor) return fail(GLOWMI_ERR_NULL, "op %d: tensor is NULL", i);
        glowmi_status st = check_addend(ops[i].tensor, y, y_bytes);
        if (st != GLOWMI_OK) return st;
        const glowmi_qparam tq = ops[i].tensor_q;
        if (!std::isfinite(tq.scale) || tq.scale <= 0.0f || tq.offset < -128 || tq.offset > 127)
          return fail(GLOWMI_ERR_QUANT, "op %d: tensor scale %g / offset %d unusable", i, (double)tq.scale, tq.offset);
        if ((st = multiplier_params_fwd((double)tq.scale / s, &o.t_mant, &o.t_shift)) != GLOWMI_OK) return st;
        if (o.t_shift < kMinAddendShift)
          return fail(GLOWMI_ERR_QUANT, "op %d: tensor scale %g is more than 2^%d times the accumulator's scale %g", i,
                      (double)tq.scale, 31 - kMinAddendShift, s);
        o.t_off = tq.offset;
        o.tensor = ops[i].tensor;
        break;
      }
      case GLOWMI_OP_MUL_SCALAR:
        if (!std::isfinite(ops[i].a) || ops[i].a <= 0.0f)
          return fail(GLOWMI_ERR_QUANT, "op %d: a quantized chain multiplies by positive finite factors only (got %g)", i, (double)ops[i].a);
        s = s * (double)ops[i].a;
        if (!std::isfinite(s) || s <= 0.0) return fail(GLOWMI_ERR_QUANT, "op %d: accumulator scale left the double range", i);
        break;
      case GLOWMI_OP_MAX_SCALAR:
        if (std::isnan(ops[i].a)) return fail(GLOWMI_ERR_QUANT, "op %d: scalar is NaN", i);
        o.ia = grid_bound(ops[i].a, s);
        break;
      case GLOWMI_OP_CLIP:
        if (!(ops[i].a <= ops[i].b)) return fail(GLOWMI_ERR_QUANT, "op %d: clip bounds %g > %g or NaN", i, (double)ops[i].a, (double)ops[i].b);
        o.ia = grid_bound(ops[i].a, s);
        o.ib = grid_bound(ops[i].b, s);
        break;
    }
  }
  if (!std::isfinite(yq.scale) || yq.scale <= 0.0f) return fail(GLOWMI_ERR_QUANT, "output scale %g unusable", (double)yq.scale);
  int32_t mant = 0, shift = 0;
  glowmi_status st = multiplier_params_fwd(s / (double)yq.scale, &mant, &shift);
  if (st != GLOWMI_OK) return st;
  p.mant = mant; p.shift = shift;
  return GLOWMI_OK;
}

}  // namespace

extern "C" {

size_t glowmi_conv2d_chainv_workspace_bytes(const glowmi_conv_desc* d, const glowmi_chain_op* ops, int32_t n_ops) {
  Geometry geo;
  if (check_desc(d, &geo) != GLOWMI_OK || check_op_list(ops, n_ops) != GLOWMI_OK) return 0;
  glowmi_chain chain;
  glowmi::Problem p;
  fill_conv(p, d, geo);
  if (set_operand_bytes(p, geo.x_elems, geo.w_elems, 4) != GLOWMI_OK) return 0;
  if (fixed_shape(ops, n_ops, &chain)) p.addend = chain.addend;
  else p.chain_n = n_ops;
  return split_bytes(glowmi::plan_f32(p, true), p);
}

glowmi_status glowmi_conv2d_chainv(const float* x, const float* w, const float* bias, float* y,
                                   const glowmi_conv_desc* d, const glowmi_chain_op* ops, int32_t n_ops,
                                   void* workspace, size_t workspace_bytes, hipStream_t stream) {
  glowmi_status st = check_op_list(ops, n_ops);
  if (st != GLOWMI_OK) return st;
  glowmi_chain chain;
  if (fixed_shape(ops, n_ops, &chain)) return glowmi_conv2d_chain(x, w, bias, y, d, &chain, workspace, workspace_bytes, stream);
  Geometry geo;
  if ((st = check_desc(d, &geo)) != GLOWMI_OK) return st;
  if ((st = check_ptrs(x, w, bias, y)) != GLOWMI_OK) return st;
  glowmi::Problem p;
  fill_conv(p, d, geo);
  if ((st = set_operand_bytes(p, geo.x_elems, geo.w_elems, 4)) != GLOWMI_OK) return st;
  p.x = x; p.w = w; p.bias = bias; p.y = y;
  if ((st = fill_chain_f32(p, ops, n_ops, y, (size_t)geo.y_elems * 4u)) != GLOWMI_OK) return st;
  const glowmi::Plan plan = plan_with_workspace(p, glowmi::plan_f32, workspace, workspace_bytes);
  const char* variant = "";
  return finish(glowmi::launch_f32(p, plan, stream, &variant), variant);
}

size_t glowmi_qconv2d_chainv_workspace_bytes(const glowmi_conv_desc* d, const glowmi_chain_op* ops, int32_t n_ops) {
  Geometry geo;
  if (check_desc(d, &geo) != GLOWMI_OK || check_op_list(ops, n_ops) != GLOWMI_OK) return 0;
  glowmi_chain chain;
  glowmi::Problem p;
  fill_conv(p, d, geo);
  if (set_operand_bytes(p, geo.x_elems, geo.w_elems, 1) != GLOWMI_OK) return 0;
  if (fixed_shape(ops, n_ops, &chain)) p.addend = chain.addend;
  else p.chain_n = n_ops;
  return split_bytes(glowmi::plan_i8(p, true), p);
}

glowmi_status glowmi_qconv2d_chainv(const int8_t* x, glowmi_qparam xq, const int8_t* w, glowmi_qparam wq,
                                    const int32_t* bias, int8_t* y, glowmi_qparam yq, const glowmi_conv_desc* d,
                                    const glowmi_chain_op* ops, int32_t n_ops, void* workspace,
                                    size_t workspace_bytes, hipStream_t stream) {
  glowmi_status st = check_op_list(ops, n_ops);
  if (st != GLOWMI_OK) return st;
  glowmi_chain chain;
  if (fixed_shape(ops, n_ops, &chain))
    return glowmi_qconv2d_chain(x, xq, w, wq, bias, y, yq, d, &chain, workspace, workspace_bytes, stream);
  Geometry geo;
  if ((st = check_desc(d, &geo)) != GLOWMI_OK) return st;
  if ((st = check_ptrs(x, w, bias, y)) != GLOWMI_OK) return st;
  glowmi::Problem p;
  fill_conv(p, d, geo);
  if ((st = set_operand_bytes(p, geo.x_elems, geo.w_elems, 1)) != GLOWMI_OK) return st;
  if ((st = quant_setup(p, xq, wq, yq, GLOWMI_ACT_NONE)) != GLOWMI_OK) return st;
  p.x = x; p.w = w; p.bias = bias; p.y = y;
  if ((st = fill_chain_i8(p, ops, n_ops, xq, wq, yq, y, (size_t)geo.y_elems)) != GLOWMI_OK) return st;
  const glowmi::Plan plan = plan_with_workspace(p, glowmi::plan_i8, workspace, workspace_bytes);
  const char* variant = "";
  return finish(glowmi::launch_i8(p, plan, stream, &variant), variant);
}

}  // extern "C"

extern "C" {

static glowmi_status check_elementwise(const void* in, const void* out, size_t count, size_t in_elem,
                                       size_t out_elem, bool in_place_ok) {
  if (!in || !out) return fail(GLOWMI_ERR_NULL, "input and output pointers must not be NULL");
  if (count == 0) return fail(GLOWMI_ERR_SHAPE, "count must be positive");
  if (count > (size_t)kMaxElems) return fail(GLOWMI_ERR_UNSUPPORTED, "a tensor has 2^31 or more elements");
  if (!aligned(in, 16) || !aligned(out, 16)) return fail(GLOWMI_ERR_ALIGN, "pointers must be 16-byte aligned");
  const uintptr_t a = reinterpret_cast<uintptr_t>(in), o = reinterpret_cast<uintptr_t>(out);
  if (!(in_place_ok && a == o) && a < o + count * out_elem && o < a + count * in_elem)
    return fail(GLOWMI_ERR_UNSUPPORTED, "output overlaps the input");
  return GLOWMI_OK;
}

static glowmi_status check_qparam(glowmi_qparam q, const char* what) {
  if (!std::isfinite(q.scale) || q.scale <= 0.0f)
    return fail(GLOWMI_ERR_QUANT, "%s scale %g is not finite and positive", what, (double)q.scale);
  if (q.offset < -128 || q.offset > 127) return fail(GLOWMI_ERR_QUANT, "%s offset %d outside [-128, 127]", what, q.offset);
  return GLOWMI_OK;
}

glowmi_status glowmi_quantize(const float* x, int8_t* q, size_t count, glowmi_qparam qp, hipStream_t stream) {
  glowmi_status st = check_elementwise(x, q, count, 4, 1, false);
  if (st != GLOWMI_OK) return st;
  if ((st = check_qparam(qp, "tensor")) != GLOWMI_OK) return st;
  return finish(glowmi::launch_quantize(x, reinterpret_cast<signed char*>(q), (long long)count, qp.scale, qp.offset, stream),
                "quantize");
}

glowmi_status glowmi_dequantize(const int8_t* q, float* x, size_t count, glowmi_qparam qp, hipStream_t stream) {
  glowmi_status st = check_elementwise(q, x, count, 1, 4, false);
  if (st != GLOWMI_OK) return st;
  if ((st = check_qparam(qp, "tensor")) != GLOWMI_OK) return st;
  return finish(glowmi::launch_dequantize(reinterpret_cast<const signed char*>(q), x, (long long)count, qp.scale,
                                          qp.offset, stream),
                "dequantize");
}

glowmi_status glowmi_rescale(const int8_t* in, glowmi_qparam from, int8_t* out, glowmi_qparam to, size_t count,
                             hipStream_t stream) {
  glowmi_status st = check_elementwise(in, out, count, 1, 1, true);
  if (st != GLOWMI_OK) return st;
  if ((st = check_qparam(from, "input")) != GLOWMI_OK) return st;
  if ((st = check_qparam(to, "output")) != GLOWMI_OK) return st;
  int32_t mant = 0, shift = 0;
  if ((st = glowmi_requant_params(from.scale, 1.0f, to.scale, &mant, &shift)) != GLOWMI_OK) return st;
  return finish(glowmi::launch_rescale(reinterpret_cast<const signed char*>(in), reinterpret_cast<signed char*>(out),
                                       (long long)count, from.offset, mant, shift, to.offset, stream),
                "rescale");
}

#pragma clang fp contract(off)   // every product and sum below is rounded on its own, as written
glowmi_status glowmi_fold_batchnorm(const float* w, const float* bias, const float* gamma, const float* beta,
                                    const float* mean, const float* var, float eps, int32_t k,
                                    int64_t elems_per_filter, float* w_out, float* bias_out) {
  if (!w || !gamma || !beta || !mean || !var || !w_out || !bias_out)
    return fail(GLOWMI_ERR_NULL, "filter, statistics and output pointers must not be NULL");
  if (k <= 0 || elems_per_filter <= 0) return fail(GLOWMI_ERR_SHAPE, "k and elems_per_filter must be positive");
  if (!std::isfinite(eps) || eps < 0.0f) return fail(GLOWMI_ERR_SHAPE, "eps must be finite and non-negative");
  for (int32_t i = 0; i < k; ++i) {
    const double denom = (double)var[i] + (double)eps;
    if (!(denom > 0.0) || !std::isfinite(denom))
      return fail(GLOWMI_ERR_SHAPE, "var[%d] + eps = %g is not positive and finite", i, denom);
  }
  for (int32_t i = 0; i < k; ++i) {
    const double root = std::sqrt((double)var[i] + (double)eps);
    const double scale = (double)gamma[i] / root;
    for (int64_t e = 0; e < elems_per_filter; ++e) {
      const double prod = (double)w[(int64_t)i * elems_per_filter + e] * scale;
      w_out[(int64_t)i * elems_per_filter + e] = (float)prod;
    }
    const double centred = (bias ? (double)bias[i] : 0.0) - (double)mean[i];
    const double scaled = centred * scale;
    const double shifted = scaled + (double)beta[i];
    bias_out[i] = (float)shifted;
  }
  g_error[0] = 0;
  return GLOWMI_OK;
}

// A positive multiplier as mant * 2^-shift, mant a 31-bit integer with its top bit set.
static glowmi_status multiplier_params(double mr, int32_t* mant, int32_t* shift);

// Mr = x_scale * w_scale / y_scale
glowmi_status glowmi_requant_params(float x_scale, float w_scale, float y_scale, int32_t* mant,
                                    int32_t* shift) {
  if (!mant || !shift) return fail(GLOWMI_ERR_NULL, "mant/shift output pointers are NULL");
  const float sc[3] = {x_scale, w_scale, y_scale};
  for (float v : sc)
    if (!std::isfinite(v) || v <= 0.0f) return fail(GLOWMI_ERR_QUANT, "scale %g is not finite and positive", (double)v);
  return multiplier_params((double)x_scale * (double)w_scale / (double)y_scale, mant, shift);
}

// Mres = r_scale / (x_scale * w_scale)
glowmi_status glowmi_rescale_params(float r_scale, float x_scale, float w_scale, int32_t* mant,
                                    int32_t* shift) {
  if (!mant || !shift) return fail(GLOWMI_ERR_NULL, "mant/shift output pointers are NULL");
  const float sc[3] = {r_scale, x_scale, w_scale};
  for (float v : sc)
    if (!std::isfinite(v) || v <= 0.0f) return fail(GLOWMI_ERR_QUANT, "scale %g is not finite and positive", (double)v);
  return multiplier_params((double)r_scale / ((double)x_scale * (double)w_scale), mant, shift);
}

namespace {
glowmi_status multiplier_params_fwd(double mr, int32_t* mant, int32_t* shift) { return multiplier_params(mr, mant, shift); }
}  // namespace

static glowmi_status multiplier_params(double mr, int32_t* mant, int32_t* shift) {
  if (!std::isfinite(mr) || mr <= 0.0) return fail(GLOWMI_ERR_QUANT, "combined multiplier %g is unusable", mr);
  int exponent = 0;
  const double frac = std::frexp(mr, &exponent);               // [0.5, 1)
  long long q31 = std::llround(std::ldexp(frac, 31));          // [2^30, 2^31]
  if (q31 == (1LL << 31)) {                                    // rounded up to the next binade
    q31 >>= 1;
    exponent += 1;
  }
  const int sh = 31 - exponent;
  if (sh < 1 || sh > 62)
    return fail(GLOWMI_ERR_QUANT, "combined multiplier %g needs shift %d outside [1, 62]", mr, sh);
  *mant = (int32_t)q31;
  *shift = sh;
  return GLOWMI_OK;
}

const char* glowmi_status_string(glowmi_status s) {
  switch (s) {
    case GLOWMI_OK: return "ok";
    case GLOWMI_ERR_NULL: return "null pointer";
    case GLOWMI_ERR_SHAPE: return "invalid shape";
    case GLOWMI_ERR_UNSUPPORTED: return "unsupported";
    case GLOWMI_ERR_ALIGN: return "misaligned pointer";
    case GLOWMI_ERR_QUANT: return "invalid quantization parameters";
    case GLOWMI_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* glowmi_last_error(void) { return g_error; }
const char* glowmi_last_variant(void) { return g_variant; }

}  // extern "C"
