// Measurement probe, not part of the library: the streaming-read ceiling of HBM on this chip, and how
// many 16-byte loads in flight per thread it takes to reach it (U) at different grid sizes.
// "read": grid-stride over one 3 GiB buffer; "slab": every workgroup walks its own contiguous slab;
// "copy": plain read+write.  Whole rounds only (the tail is skipped), so every access is in bounds.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

// Each wave reads contiguous 1 KB pieces; U independent loads in flight per thread.
template <int U>
__global__ void __launch_bounds__(256) read_kernel(const u32x4* __restrict__ p, size_t n16, unsigned* out) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  unsigned acc = 0;
  const size_t iters = n16 / (stride * U);     // whole rounds only; the tail is skipped (timing probe)
  for (size_t it = 0; it < iters; ++it) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(p + i + (size_t)u * stride);
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    i += stride * U;
  }
  if (acc == 0x12345678u) out[0] = acc;
}
// Same, but each block owns a contiguous slab (like a weight strip) and walks it sequentially.
template <int U>
__global__ void __launch_bounds__(256) slab_kernel(const u32x4* __restrict__ p, size_t n16, unsigned* out) {
  const size_t per_block = n16 / gridDim.x;
  const u32x4* q = p + (size_t)blockIdx.x * per_block;
  unsigned acc = 0;
  const size_t iters = per_block / (256 * U);
  size_t i = threadIdx.x;
  for (size_t it = 0; it < iters; ++it) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = q[i + (size_t)u * 256];
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    i += 256 * U;
  }
  if (acc == 0x12345678u) out[0] = acc;
}
__global__ void __launch_bounds__(256) copy_kernel(const u32x4* __restrict__ p, u32x4* __restrict__ o, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) o[i] = p[i];
}
template <class F> float timeit(F f, int reps) {
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  f(); CK(hipDeviceSynchronize());
  CK(hipEventRecord(a)); for (int i = 0; i < reps; ++i) f(); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms, a, b)); return ms / reps;
}
int main() {
  const size_t bytes = (size_t)3 << 30, n16 = bytes / 16;
  u32x4 *p, *o; unsigned* out;
  CK(hipMalloc(&p, bytes)); CK(hipMalloc(&o, bytes)); CK(hipMalloc(&out, 4));
  CK(hipMemset(p, 1, bytes)); CK(hipMemset(o, 0, bytes));
  const int grids[] = {256, 512, 1024, 2048, 4096};
  for (int g : grids) {
    float t;
    t = timeit([&] { read_kernel<4><<<g, 256>>>(p, n16, out); }, 5);   printf("read  U4  grid %5d: %.2f TB/s\n", g, bytes / t / 1e9); fflush(stdout);
    t = timeit([&] { read_kernel<16><<<g, 256>>>(p, n16, out); }, 5);  printf("read  U16 grid %5d: %.2f TB/s\n", g, bytes / t / 1e9); fflush(stdout);
    t = timeit([&] { slab_kernel<4><<<g, 256>>>(p, n16, out); }, 5);   printf("slab  U4  grid %5d: %.2f TB/s\n", g, bytes / t / 1e9); fflush(stdout);
    t = timeit([&] { slab_kernel<16><<<g, 256>>>(p, n16, out); }, 5);  printf("slab  U16 grid %5d: %.2f TB/s\n", g, bytes / t / 1e9); fflush(stdout);
  }
  for (int g : {2048, 8192, 65536}) {
    float t = timeit([&] { copy_kernel<<<g, 256>>>(p, o, n16); }, 5);  printf("copy      grid %5d: %.2f TB/s (read+write)\n", g, 2.0 * bytes / t / 1e9); fflush(stdout);
  }
  CK(hipDeviceSynchronize());
  CK(hipGetLastError());
  printf("done\n");
  return 0;
}
