// A sequence of convolution layers run back to back on one stream out of one arena: the step from
// a single operator towards the paper's compiled network.  The low-level IR of the paper marks the
// lifetime of every activation (alloc / dealloc, Section 3.5) and the compiler then allocates all of
// them statically in a single buffer (Section 5.3).  In a straight sequence an activation dies as
// soon as the next layer has consumed it, so two regions used alternately hold every intermediate;
// the plan below is that allocation plus a third region for the split-reduction workspace.
//
// Host code only: it validates, plans offsets and calls the layer entry points; it launches nothing
// of its own and never synchronises, so a caller can capture the whole sequence in a HIP graph.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <vector>

#include "../../include/glowmi.h"
#include "api_internal.h"

namespace {

using glowmi::fail;

constexpr size_t kAlign = 256;
constexpr int32_t kMaxLayers = 4096;
size_t round_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct SeqPlan {
  size_t region[2];     // bytes of the two alternating activation regions
  size_t workspace;     // bytes of the shared split-reduction workspace
  size_t total;
};

// Shapes must chain: layer i's input is layer i-1's output.  Returns GLOWMI_OK and the plan.
glowmi_status plan_sequence(const glowmi_seq_layer* layers, int32_t n, size_t elem, bool quantized, SeqPlan* plan) {
  if (!layers) return fail(GLOWMI_ERR_NULL, "layer array is NULL");
  if (n <= 0 || n > kMaxLayers) return fail(GLOWMI_ERR_SHAPE, "a sequence has 1 to %d layers (got %d)", kMaxLayers, n);
  plan->region[0] = plan->region[1] = plan->workspace = 0;
  for (int32_t i = 0; i < n; ++i) {
    const glowmi_conv_desc& d = layers[i].desc;
    int32_t oh = 0, ow = 0;
    glowmi_status st = glowmi_conv_out_shape(&d, &oh, &ow);
    if (st != GLOWMI_OK) return st;
    if (i + 1 < n) {
      const glowmi_conv_desc& nx = layers[i + 1].desc;
      if (nx.n != d.n || nx.h != oh || nx.w != ow || nx.c != d.k)
        return fail(GLOWMI_ERR_SHAPE, "layer %d reads %dx%dx%dx%d but layer %d writes %dx%dx%dx%d", i + 1, nx.n, nx.h,
                    nx.w, nx.c, i, d.n, oh, ow, d.k);
      const size_t bytes = round_up((size_t)d.n * oh * ow * d.k * elem);
      plan->region[i & 1] = std::max(plan->region[i & 1], bytes);
    }
    if (layers[i].add_input) {      // identity shortcut: the sequence input has the layer's output shape
      const glowmi_conv_desc& first = layers[0].desc;
      if (first.n != d.n || first.h != oh || first.w != ow || first.c != d.k)
        return fail(GLOWMI_ERR_SHAPE, "layer %d adds the sequence input, whose shape differs from the layer's output", i);
    }
    const size_t ws = quantized ? glowmi_qconv2d_workspace_bytes(&d) : glowmi_conv2d_workspace_bytes(&d);
    plan->workspace = std::max(plan->workspace, round_up(ws));
  }
  plan->total = plan->region[0] + plan->region[1] + plan->workspace;
  return GLOWMI_OK;
}

// Validate and plan EVERY layer before anything is launched, then launch them in order: a bad filter
// pointer or quantization parameter in layer 3 is reported with layers 0-2 still unlaunched.
glowmi_status run_sequence(const void* x, glowmi_qparam xq, const glowmi_seq_layer* layers, int32_t n, void* y,
                           void* arena, size_t arena_bytes, bool quantized, hipStream_t stream) {
  SeqPlan plan;
  glowmi_status st = plan_sequence(layers, n, quantized ? 1 : 4, quantized, &plan);
  if (st != GLOWMI_OK) return st;
  if (!x || !y) return fail(GLOWMI_ERR_NULL, "sequence input and output must not be NULL");
  if (plan.total && !arena) return fail(GLOWMI_ERR_NULL, "the sequence needs an arena of %zu bytes", plan.total);
  if (arena_bytes < plan.total) return fail(GLOWMI_ERR_ALIGN, "arena of %zu bytes, %zu needed", arena_bytes, plan.total);
  if (reinterpret_cast<uintptr_t>(arena) & 15) return fail(GLOWMI_ERR_ALIGN, "arena must be 16-byte aligned");
  char* base = static_cast<char*>(arena);
  char* region[2] = {base, base + plan.region[0]};
  void* ws = plan.workspace ? base + plan.region[0] + plan.region[1] : nullptr;
  std::vector<glowmi::PreparedCall> calls((size_t)n);
  const void* in = x;
  glowmi_qparam in_q = xq;
  for (int32_t i = 0; i < n; ++i) {
    void* out = i + 1 < n ? static_cast<void*>(region[i & 1]) : y;
    glowmi_chain chain;
    chain.addend = layers[i].add_input ? x : nullptr;
    chain.addend_q = xq;
    chain.act = layers[i].act;
    if (quantized)
      st = glowmi::prepare_qconv2d_chain(static_cast<const int8_t*>(in), in_q, static_cast<const int8_t*>(layers[i].w),
                                         layers[i].wq, static_cast<const int32_t*>(layers[i].bias),
                                         static_cast<int8_t*>(out), layers[i].yq, &layers[i].desc, &chain, ws,
                                         plan.workspace, &calls[(size_t)i]);
    else
      st = glowmi::prepare_conv2d_chain(static_cast<const float*>(in), static_cast<const float*>(layers[i].w),
                                        static_cast<const float*>(layers[i].bias), static_cast<float*>(out),
                                        &layers[i].desc, &chain, ws, plan.workspace, &calls[(size_t)i]);
    if (st != GLOWMI_OK) return st;          // nothing has been launched
    in = out;
    in_q = layers[i].yq;
  }
  for (int32_t i = 0; i < n; ++i)
    if ((st = glowmi::run_prepared(calls[(size_t)i], stream)) != GLOWMI_OK) return st;   // only a HIP launch failure
  return GLOWMI_OK;
}

}  // namespace

extern "C" {

size_t glowmi_seq_arena_bytes(const glowmi_seq_layer* layers, int32_t n, int32_t quantized) {
  SeqPlan plan;
  if (plan_sequence(layers, n, quantized ? 1 : 4, quantized != 0, &plan) != GLOWMI_OK) return 0;
  return plan.total ? plan.total : kAlign;
}

glowmi_status glowmi_seq_conv2d(const float* x, const glowmi_seq_layer* layers, int32_t n, float* y, void* arena,
                                size_t arena_bytes, hipStream_t stream) {
  glowmi_qparam none;
  none.scale = 1.0f;
  none.offset = 0;
  return run_sequence(x, none, layers, n, y, arena, arena_bytes, false, stream);
}

glowmi_status glowmi_seq_qconv2d(const int8_t* x, glowmi_qparam xq, const glowmi_seq_layer* layers, int32_t n,
                                 int8_t* y, void* arena, size_t arena_bytes, hipStream_t stream) {
  return run_sequence(x, xq, layers, n, y, arena, arena_bytes, true, stream);
}

}  // extern "C"
