// Small kernels of the step: the Gaussian inspection kernel, the stand-in MSE loss, the SPSA
// scalar (Definition 1) and the sparse ZO-SGD update (Section 3.4, fixed-parameter update rule).
#include <algorithm>
#include <cstring>
#include <vector>
#include "szo_internal.h"
#include "szo_rng.h"

namespace szo {

thread_local int g_last_hip_error = 0;

// ---- inspection: words and Gaussian of entries nnz_base + j ---------------------------------
__global__ void __launch_bounds__(256) debug_zbar_kernel(uint64_t nnz_base, int64_t nnz, uint64_t seed,
                                                         uint64_t step, uint32_t* words, float* z) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= nnz) return;
  const uint64_t J = nnz_base + (uint64_t)j;
  if (words) {
    const Words4 w = zbar_words(J >> 2, seed, step);
    words[4 * j + 0] = w.w0; words[4 * j + 1] = w.w1; words[4 * j + 2] = w.w2; words[4 * j + 3] = w.w3;
  }
  if (z) {
    float q[4];
    zbar_quad(J >> 2, seed, step, q);
    z[j] = q[J & 3];
  }
}

// ---- sparse update: one thread per counter = four consecutive entries ------------------------
// nnz_base is a multiple of 4, so thread t owns entries 4t..4t+3 and one 16-byte access.
__global__ void __launch_bounds__(256) sparse_update_kernel(float* __restrict__ sp_val, int64_t nnz,
                                                            uint64_t nnz_base, uint64_t seed, uint64_t step,
                                                            const double* __restrict__ g, float lr) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t j0 = 4 * t;
  if (j0 >= nnz) return;
  const float c = (float)((double)lr * *g);     // lr * g, rounded once
  float z[4];
  zbar_quad((nnz_base >> 2) + (uint64_t)t, seed, step, z);
  if (j0 + 4 <= nnz) {
    float4 v = *reinterpret_cast<float4*>(sp_val + j0);
    v.x = fmaf(-c, z[0], v.x);
    v.y = fmaf(-c, z[1], v.y);
    v.z = fmaf(-c, z[2], v.z);
    v.w = fmaf(-c, z[3], v.w);
    *reinterpret_cast<float4*>(sp_val + j0) = v;
  } else {
    for (int i = 0; j0 + i < nnz; ++i) sp_val[j0 + i] = fmaf(-c, z[i], sp_val[j0 + i]);
  }
}

// ---- MSE: sum (y - t)^2 in fp64, fixed order ---------------------------------------------------
constexpr int kMseBlocks = 2048;
constexpr int kMseThreads = 256;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__global__ void __launch_bounds__(kMseThreads) mse_kernel(const float* __restrict__ y,
                                                          const uint16_t* __restrict__ t, int64_t count,
                                                          LossSink sink, int vec_ok) {
  __shared__ double scratch[kMseThreads / 64];
  double acc = 0.0;
  const int64_t tid = (int64_t)blockIdx.x * kMseThreads + threadIdx.x;
  const int64_t nthreads = (int64_t)gridDim.x * kMseThreads;
  if (vec_ok) {
    const int64_t n4 = count >> 2;
    for (int64_t i = tid; i < n4; i += nthreads) {
      const float4 yv = reinterpret_cast<const float4*>(y)[i];
      const uint2 tv = reinterpret_cast<const uint2*>(t)[i];
      const double d0 = (double)yv.x - (double)bf16_bits_to_f32(tv.x & 0xFFFFu);
      const double d1 = (double)yv.y - (double)bf16_bits_to_f32(tv.x >> 16);
      const double d2 = (double)yv.z - (double)bf16_bits_to_f32(tv.y & 0xFFFFu);
      const double d3 = (double)yv.w - (double)bf16_bits_to_f32(tv.y >> 16);
      acc = fma(d0, d0, acc); acc = fma(d1, d1, acc); acc = fma(d2, d2, acc); acc = fma(d3, d3, acc);
    }
    for (int64_t i = (n4 << 2) + tid; i < count; i += nthreads) {
      const double d = (double)y[i] - (double)bf16_bits_to_f32(t[i]);
      acc = fma(d, d, acc);
    }
  } else {
    for (int64_t i = tid; i < count; i += nthreads) {
      const double d = (double)y[i] - (double)bf16_bits_to_f32(t[i]);
      acc = fma(d, d, acc);
    }
  }
  block_loss_commit(acc, scratch, sink, blockIdx.x, gridDim.x);
}

__global__ void spsa_g_kernel(const double* lp, const double* lm, float eps, double* g) {
  *g = (eps == 0.0f) ? 0.0 : (*lp - *lm) / (2.0 * (double)eps);
}

// Sum of v[0..count) by one workgroup of 1024 threads: thread t adds elements t, t+1024, ... in four
// interleaved chains (four loads in flight: the loop is bound by memory latency), then the chains and the
// 1024 thread sums are combined by a fixed tree.  Bit-reproducible.
__device__ __forceinline__ double block_sum_1024(const double* __restrict__ v, int count, double* scratch) {
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
  int i = threadIdx.x;
  for (; i + 3 * 1024 < count; i += 4 * 1024) {
    a0 += v[i]; a1 += v[i + 1024]; a2 += v[i + 2 * 1024]; a3 += v[i + 3 * 1024];
  }
  for (; i < count; i += 1024) a0 += v[i];
  double a = (a0 + a1) + (a2 + a3);
  a = wave_sum(a);
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = a;
  __syncthreads();
  double t = 0.0;
  for (int i = 0; i < 16; ++i) t += scratch[i];
  __syncthreads();
  return t;
}

__global__ void __launch_bounds__(1024) reduce_partials_kernel(const double* __restrict__ partials, int count,
                                                               double* loss_acc) {
  __shared__ double scratch[16];
  const double t = block_sum_1024(partials, count, scratch);
  if (threadIdx.x == 0) *loss_acc += t;
}

// The SPSA scalar of Definition 1 from the two passes' partial losses.
__global__ void __launch_bounds__(1024) reduce_step_kernel(const double* __restrict__ partials, int count, float eps,
                                                           double* scalars) {
  __shared__ double scratch[16];
  const double lp = block_sum_1024(partials, count, scratch);
  const double lm = block_sum_1024(partials + count, count, scratch);
  if (threadIdx.x == 0) {
    scalars[0] = lp;
    scalars[1] = lm;
    scalars[2] = (eps == 0.0f) ? 0.0 : (lp - lm) / (2.0 * (double)eps);
  }
}

// max |x| over bf16 values: the magnitude bits of non-negative floats order like unsigned integers, so
// an integer atomic max of (bits & 0x7FFF) << 16 is the float maximum (NaN patterns compare above infinity
// and come out as NaN).
__global__ void __launch_bounds__(256) absmax_bf16_kernel(const uint16_t* __restrict__ x, int64_t count, uint32_t* out_bits) {
  uint32_t m = 0u;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
    m = max(m, (uint32_t)(x[i] & 0x7FFFu));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, 64));
  if ((threadIdx.x & 63) == 0 && m) atomicMax(out_bits, m << 16);
}

__global__ void zero_words_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

int reduce_partials(const double* partials, int count, double* loss_acc, hipStream_t stream) {
  reduce_partials_kernel<<<1, 1024, 0, stream>>>(partials, count, loss_acc);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

int reduce_step(const double* partials, int count, float eps, double* scalars, hipStream_t stream) {
  reduce_step_kernel<<<1, 1024, 0, stream>>>(partials, count, eps, scalars);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

__global__ void __launch_bounds__(256) stage_copy_kernel(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst, int words) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < words) dst[i] = src[i];
}

// Pinned staging buffers of one host thread.  Eight slots: a tiled fused step stages two tables (its
// forwards and its update), so the host may run four steps ahead of the GPU; a slot is reused only
// after the copy kernel that read it has executed.  Released when the thread ends.
namespace {
struct StageSlot { void* host; const uint32_t* host_dev; size_t cap; hipEvent_t copied; bool used; };
struct StageRing {
  StageSlot slot[8] = {};
  unsigned turn = 0;
  ~StageRing() {
    for (StageSlot& s : slot) {               // errors are ignored: the runtime may already be shutting down
      if (s.used && s.copied) (void)hipEventSynchronize(s.copied);
      if (s.copied) (void)hipEventDestroy(s.copied);
      if (s.host) (void)hipHostFree(s.host);
    }
  }
};
}  // namespace

int stage_table(const void* src, size_t bytes, void* dst, hipStream_t stream) {
  if (bytes == 0) return SZO_OK;
  if (bytes & 3) return SZO_EINVAL;
  {
    // A captured launch would replay the copy from a slot that later calls overwrite.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    SZO_HIP(hipStreamIsCapturing(stream, &cap));
    if (cap != hipStreamCaptureStatusNone) return SZO_EUNSUPPORTED;
  }
  static thread_local StageRing ring;
  StageSlot& slot = ring.slot[ring.turn++ & 7];
  if (slot.used) SZO_HIP(hipEventSynchronize(slot.copied));
  if (!slot.copied) SZO_HIP(hipEventCreateWithFlags(&slot.copied, hipEventDisableTiming));
  if (bytes > slot.cap) {
    if (slot.host) (void)hipHostFree(slot.host);
    slot.host = nullptr; slot.cap = 0;
    const size_t cap = (bytes + 4095) & ~(size_t)4095;
    SZO_HIP(hipHostMalloc(&slot.host, cap, hipHostMallocMapped));
    SZO_HIP(hipHostGetDevicePointer((void**)&slot.host_dev, slot.host, 0));
    slot.cap = cap;
  }
  memcpy(slot.host, src, bytes);
  const int words = (int)(bytes / 4);
  stage_copy_kernel<<<(words + 255) / 256, 256, 0, stream>>>(slot.host_dev, (uint32_t*)dst, words);
  SZO_LAUNCH_CHECK();
  SZO_HIP(hipEventRecord(slot.copied, stream));
  slot.used = true;
  return SZO_OK;
}

bool stream_is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &cap) != hipSuccess) return false;
  return cap != hipStreamCaptureStatusNone;
}

int zero_words(void* p, int n, hipStream_t stream) {
  if (n <= 0) return SZO_OK;
  zero_words_kernel<<<(n + 255) / 256, 256, 0, stream>>>((uint32_t*)p, n);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

}  // namespace szo

using namespace szo;

// ---- optional timing of the forward kernels ---------------------------------------------------
// Process-wide, meant for one measuring thread: a growing pool of event pairs, one pair per
// forward-kernel launch since the last read.
namespace szo {
namespace {
struct TimingState {
  bool on = false;
  std::vector<hipEvent_t> start, stop;
  std::vector<int> kind;    // 0 = forward kernel, 1 = sparse update kernel
  size_t used = 0;          // pairs recorded since the last read
  bool open = false;        // a begin without its end
};
TimingState g_timing;
}  // namespace

int timing_begin(hipStream_t stream, int kind) {
  if (!g_timing.on) return SZO_OK;
  if (g_timing.used == g_timing.start.size()) {
    hipEvent_t a, b;
    SZO_HIP(hipEventCreate(&a));
    SZO_HIP(hipEventCreate(&b));
    g_timing.start.push_back(a);
    g_timing.stop.push_back(b);
    g_timing.kind.push_back(0);
  }
  g_timing.kind[g_timing.used] = kind;
  SZO_HIP(hipEventRecord(g_timing.start[g_timing.used], stream));
  g_timing.open = true;
  return SZO_OK;
}

int timing_end(hipStream_t stream) {
  if (!g_timing.on || !g_timing.open) return SZO_OK;
  SZO_HIP(hipEventRecord(g_timing.stop[g_timing.used], stream));
  g_timing.used += 1;
  g_timing.open = false;
  return SZO_OK;
}

}  // namespace szo

extern "C" {

int szo_kernel_timing(int enable) {
  szo::g_timing.on = enable != 0;
  szo::g_timing.used = 0;
  szo::g_timing.open = false;
  return SZO_OK;
}

int szo_kernel_timing_read2(double total_ms[2], int64_t launches[2]) {
  using szo::g_timing;
  if (!total_ms || !launches) return SZO_EINVAL;
  double sum[2] = {0.0, 0.0};
  int64_t cnt[2] = {0, 0};
  for (size_t i = 0; i < g_timing.used; ++i) {
    SZO_HIP(hipEventSynchronize(g_timing.stop[i]));
    float ms = 0.0f;
    SZO_HIP(hipEventElapsedTime(&ms, g_timing.start[i], g_timing.stop[i]));
    const int k = g_timing.kind[i] == 1 ? 1 : 0;
    sum[k] += (double)ms;
    cnt[k] += 1;
  }
  total_ms[0] = sum[0]; total_ms[1] = sum[1];
  launches[0] = cnt[0]; launches[1] = cnt[1];
  g_timing.used = 0;
  return SZO_OK;
}

int szo_kernel_timing_read(double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) return SZO_EINVAL;
  double ms[2];
  int64_t n[2];
  const int rc = szo_kernel_timing_read2(ms, n);
  if (rc != SZO_OK) return rc;
  *total_ms = ms[0];
  *launches = n[0];
  return SZO_OK;
}

int szo_last_hip_error(void) { return g_last_hip_error; }
int szo_version(void) { return 5; }
size_t szo_workspace_bytes(void) { return kWorkspaceBytes; }

int szo_workspace_init(void* workspace, void* stream) {
  if (!workspace || ((uintptr_t)workspace & 7)) return SZO_EINVAL;
  return zero_words(workspace, (int)(kWorkspaceHeader / 4), (hipStream_t)stream);
}

int szo_debug_zbar(uint64_t nnz_base, int64_t nnz, uint64_t seed, uint64_t step, uint32_t* words_out,
                   float* z_out, void* stream) {
  if (nnz < 0) return SZO_EINVAL;
  if (nnz == 0 || (!words_out && !z_out)) return SZO_OK;
  const int64_t blocks = (nnz + 255) / 256;
  if (blocks > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
  debug_zbar_kernel<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>(nnz_base, nnz, seed, step, words_out, z_out);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

int szo_sparse_update(float* sp_val, const uint32_t* sp_idx, int64_t nnz, uint64_t nnz_base, uint64_t seed,
                      uint64_t step, const double* g, float lr, void* stream) {
  (void)sp_idx;
  if (nnz < 0 || !g || (nnz_base & 3)) return SZO_EINVAL;
  if (nnz == 0) return SZO_OK;
  if (!sp_val || ((uintptr_t)sp_val & 15)) return SZO_EINVAL;
  const int64_t quads = (nnz + 3) / 4;
  const int64_t blocks = (quads + 255) / 256;
  if (blocks > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
  const int trc = timing_begin((hipStream_t)stream, 1);
  if (trc != SZO_OK) return trc;
  sparse_update_kernel<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>(sp_val, nnz, nnz_base, seed, step, g, lr);
  SZO_LAUNCH_CHECK();
  return timing_end((hipStream_t)stream);
}

int szo_mse_loss(const float* y, const void* target, int64_t count, double scale, double* loss_acc,
                 void* workspace, void* stream) {
  if (count < 0 || !loss_acc || !workspace || ((uintptr_t)workspace & 7)) return SZO_EINVAL;
  if (count == 0) return SZO_OK;
  if (!y || !target || ((uintptr_t)y & 3) || ((uintptr_t)target & 1)) return SZO_EINVAL;
  const int vec_ok = (((uintptr_t)y & 15) == 0) && (((uintptr_t)target & 7) == 0);
  int64_t blocks = (count / 4 + kMseThreads - 1) / kMseThreads;
  blocks = blocks < 1 ? 1 : (blocks > kMseBlocks ? kMseBlocks : blocks);
  mse_kernel<<<(unsigned)blocks, kMseThreads, 0, (hipStream_t)stream>>>(
      y, (const uint16_t*)target, count, make_sink(workspace, loss_acc, scale), vec_ok);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

int szo_activation_absmax(const void* x, int64_t count, float* absmax_out, void* stream) {
  if (count < 0 || !absmax_out || ((uintptr_t)absmax_out & 3)) return SZO_EINVAL;
  int rc = zero_words(absmax_out, 1, (hipStream_t)stream);
  if (rc != SZO_OK || count == 0) return rc;
  if (!x || ((uintptr_t)x & 1)) return SZO_EINVAL;
  const int64_t blocks = std::min<int64_t>((count + 255) / 256, 2048);
  absmax_bf16_kernel<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>((const uint16_t*)x, count, (uint32_t*)absmax_out);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

int szo_spsa_g(const double* loss_plus, const double* loss_minus, float eps, double* g, void* stream) {
  if (!loss_plus || !loss_minus || !g) return SZO_EINVAL;
  spsa_g_kernel<<<1, 1, 0, (hipStream_t)stream>>>(loss_plus, loss_minus, eps, g);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

}  // extern "C"
