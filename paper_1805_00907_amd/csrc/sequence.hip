// A sequence of convolution layers run back to back on one stream out of one arena: the step from
// a single operator towards the paper's compiled network.  The low-level IR of the paper marks the
// lifetime of every activation (alloc / dealloc, Section 3.5) and the compiler then allocates all of
// them statically in a single buffer (Section 5.3).  In a straight sequence an activation dies as
// soon as the next layer has consumed it, so two regions used alternately hold every intermediate;
// the plan below is that allocation plus a third region for the split-reduction workspace.
//
// Host code only: it validates, plans offsets and calls the layer entry points; it launches nothing
// of its own and never synchronises, so a caller can capture the whole sequence in a HIP graph.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdint>

#include "../../include/glowmi.h"

namespace {

constexpr size_t kAlign = 256;
size_t round_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct SeqPlan {
  size_t region[2];     // bytes of the two alternating activation regions
  size_t workspace;     // bytes of the shared split-reduction workspace
  size_t total;
};

// Shapes must chain: layer i's input is layer i-1's output.  Returns GLOWMI_OK and the plan.
glowmi_status plan_sequence(const glowmi_seq_layer* layers, int32_t n, size_t elem, bool quantized, SeqPlan* plan) {
  if (!layers || n <= 0) return GLOWMI_ERR_NULL;
  plan->region[0] = plan->region[1] = plan->workspace = 0;
  for (int32_t i = 0; i < n; ++i) {
    const glowmi_conv_desc& d = layers[i].desc;
    int32_t oh = 0, ow = 0;
    glowmi_status st = glowmi_conv_out_shape(&d, &oh, &ow);
    if (st != GLOWMI_OK) return st;
    if (i + 1 < n) {
      const glowmi_conv_desc& nx = layers[i + 1].desc;
      if (nx.n != d.n || nx.h != oh || nx.w != ow || nx.c != d.k) return GLOWMI_ERR_SHAPE;
      const size_t bytes = round_up((size_t)d.n * oh * ow * d.k * elem);
      plan->region[i & 1] = std::max(plan->region[i & 1], bytes);
    }
    if (layers[i].add_input) {      // identity shortcut: the sequence input has the layer's output shape
      const glowmi_conv_desc& first = layers[0].desc;
      if (first.n != d.n || first.h != oh || first.w != ow || first.c != d.k) return GLOWMI_ERR_SHAPE;
    }
    const size_t ws = quantized ? glowmi_qconv2d_workspace_bytes(&d) : glowmi_conv2d_workspace_bytes(&d);
    plan->workspace = std::max(plan->workspace, round_up(ws));
  }
  plan->total = plan->region[0] + plan->region[1] + plan->workspace;
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
  SeqPlan plan;
  glowmi_status st = plan_sequence(layers, n, 4, false, &plan);
  if (st != GLOWMI_OK) return st;
  if (!x || !y || (plan.total && !arena)) return GLOWMI_ERR_NULL;
  if (arena_bytes < plan.total || (reinterpret_cast<uintptr_t>(arena) & 15)) return GLOWMI_ERR_ALIGN;
  char* base = static_cast<char*>(arena);
  char* region[2] = {base, base + plan.region[0]};
  void* ws = plan.workspace ? base + plan.region[0] + plan.region[1] : nullptr;
  const float* in = x;
  for (int32_t i = 0; i < n; ++i) {
    float* out = i + 1 < n ? reinterpret_cast<float*>(region[i & 1]) : y;
    glowmi_chain chain;
    chain.addend = layers[i].add_input ? x : nullptr;
    chain.addend_q.scale = 1.0f;
    chain.addend_q.offset = 0;
    chain.act = layers[i].act;
    st = glowmi_conv2d_chain(in, static_cast<const float*>(layers[i].w), static_cast<const float*>(layers[i].bias),
                             out, &layers[i].desc, &chain, ws, plan.workspace, stream);
    if (st != GLOWMI_OK) return st;
    in = out;
  }
  return GLOWMI_OK;
}

glowmi_status glowmi_seq_qconv2d(const int8_t* x, glowmi_qparam xq, const glowmi_seq_layer* layers, int32_t n,
                                 int8_t* y, void* arena, size_t arena_bytes, hipStream_t stream) {
  SeqPlan plan;
  glowmi_status st = plan_sequence(layers, n, 1, true, &plan);
  if (st != GLOWMI_OK) return st;
  if (!x || !y || (plan.total && !arena)) return GLOWMI_ERR_NULL;
  if (arena_bytes < plan.total || (reinterpret_cast<uintptr_t>(arena) & 15)) return GLOWMI_ERR_ALIGN;
  char* base = static_cast<char*>(arena);
  char* region[2] = {base, base + plan.region[0]};
  void* ws = plan.workspace ? base + plan.region[0] + plan.region[1] : nullptr;
  const int8_t* in = x;
  glowmi_qparam in_q = xq;
  for (int32_t i = 0; i < n; ++i) {
    int8_t* out = i + 1 < n ? reinterpret_cast<int8_t*>(region[i & 1]) : y;
    glowmi_chain chain;
    chain.addend = layers[i].add_input ? x : nullptr;
    chain.addend_q = xq;
    chain.act = layers[i].act;
    st = glowmi_qconv2d_chain(in, in_q, static_cast<const int8_t*>(layers[i].w), layers[i].wq,
                              static_cast<const int32_t*>(layers[i].bias), out, layers[i].yq, &layers[i].desc,
                              &chain, ws, plan.workspace, stream);
    if (st != GLOWMI_OK) return st;
    in = out;
    in_q = layers[i].yq;
  }
  return GLOWMI_OK;
}

}  // extern "C"
