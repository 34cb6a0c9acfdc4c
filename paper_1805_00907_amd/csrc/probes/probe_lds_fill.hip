// Standalone probe (not part of the library): at what rate a workgroup of 512 threads can pull
// 128-byte row pieces of two operand tiles (128 rows each, row pitch 9216 bytes, the staging pattern of
// the wide int8 kernel on a 1024 x 9216 x 4096 FullyConnected) out of the L2 / last-level cache
//   MODE 0: with buffer loads that write straight into LDS (ring of NBUF slab buffers, NBUF-1 in flight),
//   MODE 1: into registers, then ds_write_b128 into LDS (DEPTH slabs in flight in registers),
//   MODE 2: into registers only (no LDS traffic at all),
// with one workgroup on the whole chip and with 256 (8 x 32 tiles, one per CU).  Every access is inside
// the two buffers by construction.  Build and run:
//   hipcc --offload-arch=gfx950 -O3 -Wno-unused-value -o probe_lds_fill probe_lds_fill.hip && ./probe_lds_fill
#include <hip/hip_runtime.h>
#include <cstdio>

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int THREADS = 512;
constexpr int ROWS = 128;                 // rows per operand tile
constexpr int KB = 128;                   // bytes of a row per slab
constexpr int SLAB = 2 * ROWS * KB;       // 32 KB
constexpr int LOADS = SLAB / (THREADS * 16);   // 4 loads of 16 bytes per thread and slab
constexpr int PITCH = 9216;
constexpr int SLABS_PER_ROW = PITCH / KB; // 72

__device__ __forceinline__ v4i make_rsrc(const void* base, unsigned bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(base);
  v4i r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
  r[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((a >> 32) & 0xffffu));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;
  return r;
}

template <int MODE, int NBUF>
__global__ __launch_bounds__(THREADS) void fill(const char* a, unsigned a_bytes, const char* b, unsigned b_bytes,
                                                int tiles_n, int slabs, int* out) {
  extern __shared__ __align__(16) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
  // load i of a thread: i < 2 from the first operand's tile, else from the second's; row (tid/8) + 64*(i%2)
  unsigned voff[LOADS];
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int row = (i < 2 ? tm : tn) * ROWS + (tid >> 3) + 64 * (i & 1);
    voff[i] = (unsigned)row * PITCH + (unsigned)(tid & 7) * 16u;
  }
  const v4i ra = make_rsrc(a, a_bytes), rb = make_rsrc(b, b_bytes);
  int sink = 0;

  if (MODE == 0) {
    auto issue = [&](int slab) {
      const unsigned koff = (unsigned)(slab % SLABS_PER_ROW) * KB;
      const unsigned base = (unsigned)(slab % NBUF) * SLAB;
#pragma unroll
      for (int i = 0; i < LOADS; ++i) {
        const unsigned lds_addr = base + (unsigned)(i * 8 + wave) * 1024u;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     :
                     : "s"(lds_addr), "v"(voff[i] + koff), "s"(i < 2 ? ra : rb)
                     : "memory");
      }
    };
    for (int s = 0; s < NBUF - 1; ++s) issue(s);
    for (int s = 0; s < slabs; ++s) {
      issue(s + NBUF - 1);                       // (slab indices wrap inside the row: always in bounds)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NBUF - 1) * LOADS) : "memory");
      __syncthreads();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    sink = reinterpret_cast<int*>(lds)[tid];
  } else {
    constexpr int DEPTH = NBUF;                  // slabs in flight in registers
    v4i r[DEPTH][LOADS];
    const __amdgpu_buffer_rsrc_t qa = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(a), 0, (int)a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t qb = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(b), 0, (int)b_bytes, 0x00020000);
    auto issue = [&](int d, int slab) {
      const unsigned koff = (unsigned)(slab % SLABS_PER_ROW) * KB;
#pragma unroll
      for (int i = 0; i < LOADS; ++i)
        r[d][i] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(i < 2 ? qa : qb, voff[i] + koff, 0, 0));
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue(d, d);
    for (int s = 0; s < slabs; s += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        if (MODE == 1) {
          char* dst = lds + ((s + d) & 1) * SLAB;
#pragma unroll
          for (int i = 0; i < LOADS; ++i) *reinterpret_cast<v4i*>(dst + (i * 8 + wave) * 1024 + lane * 16) = r[d][i];
        } else {
#pragma unroll
          for (int i = 0; i < LOADS; ++i) sink ^= r[d][i][0] ^ r[d][i][1] ^ r[d][i][2] ^ r[d][i][3];
        }
        issue(d, s + d + DEPTH);
        __syncthreads();
      }
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
#pragma unroll
      for (int i = 0; i < LOADS; ++i) sink ^= r[d][i][0];
    if (MODE == 1) {
      __syncthreads();
      sink ^= reinterpret_cast<int*>(lds)[tid];
    }
  }
  if (sink == 0x12345678) out[tid] = sink;
}

template <int MODE, int NBUF>
void run(const char* a, unsigned a_bytes, const char* b, unsigned b_bytes, int* out, int tiles_m, int tiles_n) {
  const int slabs = 72 * 40;
  const int lds_bytes = MODE == 0 ? NBUF * SLAB : 2 * SLAB;
  auto kern = fill<MODE, NBUF>;
  hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  hipEvent_t e0, e1;
  hipEventCreate(&e0);
  hipEventCreate(&e1);
  const int grid = tiles_m * tiles_n;
  kern<<<grid, THREADS, lds_bytes>>>(a, a_bytes, b, b_bytes, tiles_n, 72, out);
  hipDeviceSynchronize();
  hipEventRecord(e0);
  kern<<<grid, THREADS, lds_bytes>>>(a, a_bytes, b, b_bytes, tiles_n, slabs, out);
  hipEventRecord(e1);
  hipEventSynchronize(e1);
  float ms = 0.f;
  hipEventElapsedTime(&ms, e0, e1);
  const double us_per_slab = ms * 1e3 / slabs;
  printf("mode %d depth %d workgroups %3d: %.3f us per 32 KB slab = %.1f B/clk per CU at 2.4 GHz, %.2f TB/s together (%s)\n",
         MODE, NBUF, grid, us_per_slab, SLAB / (us_per_slab * 2400.0), grid * (double)SLAB / us_per_slab * 1e-6,
         hipGetErrorString(hipGetLastError()));
  fflush(stdout);
}

int main() {
  const unsigned a_bytes = 1024u * PITCH, b_bytes = 4096u * PITCH;
  char *a, *b;
  int* out;
  hipMalloc(&a, a_bytes);
  hipMalloc(&b, b_bytes);
  hipMalloc(&out, 4096);
  hipMemset(a, 1, a_bytes);
  hipMemset(b, 2, b_bytes);
  for (int pass = 0; pass < 2; ++pass) {
    const int tm = pass == 0 ? 1 : 8, tn = pass == 0 ? 1 : 32;
    run<0, 2>(a, a_bytes, b, b_bytes, out, tm, tn);
    run<0, 4>(a, a_bytes, b, b_bytes, out, tm, tn);
    run<1, 2>(a, a_bytes, b, b_bytes, out, tm, tn);
    run<1, 3>(a, a_bytes, b, b_bytes, out, tm, tn);
    run<2, 2>(a, a_bytes, b, b_bytes, out, tm, tn);
    run<2, 3>(a, a_bytes, b, b_bytes, out, tm, tn);
  }
  return 0;
}
