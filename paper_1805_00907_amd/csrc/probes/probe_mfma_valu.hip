// Standalone probe (not part of the library): how much of one wavefront's vector-ALU work the fp32
// matrix pipe hides behind another wavefront's MFMAs.  Every wavefront alternates NM
// v_mfma_f32_32x32x2_f32 (two accumulator chains, register operands only) with NVREP x 96 vector
// instructions that depend on the results, as a convolution kernel alternates its reduction with its
// epilogue.  Build and run:
//   hipcc --offload-arch=gfx950 -O3 -Wno-unused-value -o probe_mfma_valu probe_mfma_valu.hip && ./probe_mfma_valu
#include <hip/hip_runtime.h>
#include <cstdio>
typedef float v16f __attribute__((ext_vector_type(16)));
template <int NM, int NVREP, int THREADS>
__global__ __launch_bounds__(THREADS) void k(float* out, int items, float a0, float b0) {
  float a[4], b[4];
  for (int i = 0; i < 4; ++i) { a[i] = a0 + i + threadIdx.x; b[i] = b0 - i; }
  float s = 0.f;
  for (int it = 0; it < items; ++it) {
    v16f acc0, acc1;
    for (int e = 0; e < 16; ++e) { acc0[e] = 0.f; acc1[e] = 0.f; }
#pragma unroll
    for (int u = 0; u < NM / 2; ++u) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u & 3], b[u & 3], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u & 3], b[(u + 1) & 3], acc1, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < NVREP; ++r)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        s += fmaxf(acc0[e] + b0 * r, 0.f);
        s += fmaxf(acc1[e] + a0 * r, 0.f);
      }
  }
  if (s == 12345.678f) out[threadIdx.x] = s;
}
template <int NM, int NVREP, int THREADS>
void run(int wgs_per_cu, int items) {
  float* out; hipMalloc(&out, 4096);
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  const int grid = 256 * wgs_per_cu;
  k<NM, NVREP, THREADS><<<grid, THREADS>>>(out, 4, 1.f, 2.f);
  hipDeviceSynchronize();
  hipEventRecord(e0);
  k<NM, NVREP, THREADS><<<grid, THREADS>>>(out, items, 1.f, 2.f);
  hipEventRecord(e1); hipEventSynchronize(e1);
  float ms; hipEventElapsedTime(&ms, e0, e1);
  const double flops = (double)grid * (THREADS / 64) * items * NM * 32 * 32 * 2 * 2;
  printf("MFMAs/item=%d valu-reps=%d threads=%d wgs/CU=%d: %.3f ms  %.1f TFLOP/s\n", NM, NVREP, THREADS, wgs_per_cu, ms, flops / ms / 1e9);
  hipFree(out);
}
int main() {
  run<64, 1, 256>(1, 400); run<64, 1, 256>(2, 400); run<64, 1, 512>(1, 400);
  run<64, 4, 256>(1, 400); run<64, 4, 256>(2, 400); run<64, 4, 512>(1, 400);
  run<64, 8, 512>(1, 400); run<256, 8, 512>(1, 100);
  return 0;
}
