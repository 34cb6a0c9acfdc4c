// Shared by the kernels with persistent workgroups (conv_pw_f32.hip, conv_pw_i8.hip, conv_k3c64_i8.hip,
// conv_smallc_i8.hip): how the work items of one filter slice are dealt to the wavefronts of the
// slice's workgroups.
#pragma once
#include "igemm.h"

namespace glowmi {

// An item is (block of 32 output pixels, group of 64 output channels).  A slice has ngc channel
// groups that really exist, so items = pixel blocks * ngc; wavefront wv of the slice takes items_div
// (+1 for items_rem of the wavefronts, see deal_range) consecutive items, pixel block major.
struct PwRange {
  int ngc, items_div, items_rem;
  FastDiv div_ngc;
};

// The contiguous range [begin, end) of wavefront wv out of `waves` over div * waves + rem items.  The
// rem ranges that are one item longer are spread evenly over the wavefronts: given to the first rem
// wavefronts they would all sit in the first workgroups, whose CUs then carry up to twice the work of
// the others (with 1.5 items per wavefront the first half of the CUs had two each, the rest one).
__device__ __forceinline__ void deal_range(int wv, int waves, int div, int rem, int& begin, int& end) {
  const unsigned e0 = ((unsigned)wv * (unsigned)rem) / (unsigned)waves;
  const unsigned e1 = ((unsigned)(wv + 1) * (unsigned)rem) / (unsigned)waves;
  begin = wv * div + (int)e0;
  end = (wv + 1) * div + (int)e1;
}

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
