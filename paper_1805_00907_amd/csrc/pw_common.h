// Shared by the pointwise-convolution kernels (conv_pw_f32.hip, conv_pw_i8.hip): how the work items
// of one filter slice are dealt to the wavefronts of the slice's persistent workgroups.
#pragma once
#include "igemm.h"

namespace glowmi {

// An item is (block of 32 output pixels, group of 64 output channels).  A slice has ngc channel
// groups that really exist, so items = pixel blocks * ngc; wavefront wv of the slice takes items_div
// (+1 for the first items_rem wavefronts) consecutive items, pixel block major.
struct PwRange {
  int ngc, items_div, items_rem;
  FastDiv div_ngc;
};

inline PwRange make_pw_range(int row_blocks, int ngc, long long waves) {
  PwRange r;
  const long long items = (long long)row_blocks * ngc;
  r.ngc = ngc;
  r.items_div = (int)(items / waves);
  r.items_rem = (int)(items % waves);
  r.div_ngc = make_fastdiv((uint32_t)ngc);
  return r;
}

}  // namespace glowmi
