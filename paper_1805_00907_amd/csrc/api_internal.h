// Pieces of the ABI layer (api.hip) that the other host-side translation units use: the error
// record behind glowmi_last_error(), and "prepare" / "run" halves of the convolution entry points so
// that a caller issuing several layers (sequence.hip) can validate ALL of them before the first launch.
#pragma once
#include "../../include/glowmi.h"
#include "igemm.h"

namespace glowmi {

// Records the message glowmi_last_error() returns on this thread; returns `s`.
glowmi_status fail(glowmi_status s, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// One validated, planned layer call: everything needed to launch it later without further checks.
struct PreparedCall {
  Problem p;
  Plan plan;
  bool quantized;
};

// Validate the arguments of glowmi_conv2d_chain / glowmi_qconv2d_chain and plan the launch (tile,
// split of the reduction given the workspace).  Nothing is launched.  w_planes: the filter's bf16 planes made
// ahead of time (glowmi_conv2d_pack_filter), or null.
glowmi_status prepare_conv2d_chain(const float* x, const float* w, const float* bias, float* y,
                                   const glowmi_conv_desc* d, const glowmi_chain* chain, void* workspace,
                                   size_t workspace_bytes, PreparedCall* out, const void* w_planes = nullptr);
glowmi_status prepare_qconv2d_chain(const int8_t* x, glowmi_qparam xq, const int8_t* w, glowmi_qparam wq,
                                    const int32_t* bias, int8_t* y, glowmi_qparam yq, const glowmi_conv_desc* d,
                                    const glowmi_chain* chain, void* workspace, size_t workspace_bytes,
                                    PreparedCall* out);
// Launch a prepared call on `stream`.
glowmi_status run_prepared(const PreparedCall& call, hipStream_t stream);

}  // namespace glowmi
