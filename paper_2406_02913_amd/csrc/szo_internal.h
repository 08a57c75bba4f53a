// Shared by the translation units of libszo: error bookkeeping and the layout of the
// loss workspace.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "szo.h"

namespace szo {

extern thread_local int g_last_hip_error;

inline int hip_failed(hipError_t e) {
  if (e == hipSuccess) return 0;
  g_last_hip_error = (int)e;
  return 1;
}

#define SZO_HIP(expr) do { if (::szo::hip_failed((expr))) return SZO_ELAUNCH; } while (0)
#define SZO_LAUNCH_CHECK() SZO_HIP(hipGetLastError())

// Raises a kernel's dynamic LDS limit once per device (`done` holds one bit per device id); safe to
// call from several host threads.
inline int set_lds_limit_once(std::atomic<uint64_t>& done, const void* fn, size_t bytes) {
  int dev = 0;
  SZO_HIP(hipGetDevice(&dev));
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return SZO_OK;
  SZO_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  done.fetch_or(bit, std::memory_order_release);
  return SZO_OK;
}

// Loss workspace: a ticket counter (first 64 bytes) followed by one fp64 partial per
// workgroup.  The last workgroup to finish adds the partials in index order, which makes
// the sum independent of scheduling.
constexpr int kMaxLossPartials = 1 << 21;       // 16 MiB: a 32-block 7B stack at 4096 tokens has 2 x 340 000 dual-sign tiles
constexpr size_t kWorkspaceHeader = 64;
constexpr int kMaxStepMatrices = 4096;            // descriptor table of the few-token step
constexpr size_t kTableBytesPerMatrix = 144;
constexpr size_t kWorkspaceTableOffset = kWorkspaceHeader + sizeof(double) * (size_t)kMaxLossPartials;
constexpr size_t kWorkspaceBytes = kWorkspaceTableOffset + kTableBytesPerMatrix * (size_t)kMaxStepMatrices;

struct LossSink {
  unsigned int* ticket;   // device; zero between calls
  double* partials;       // device; [kMaxLossPartials]
  double* loss_acc;       // device; += scale * total
  double scale;
};

inline LossSink make_sink(void* workspace, double* loss_acc, double scale) {
  return LossSink{(unsigned int*)workspace, (double*)((char*)workspace + kWorkspaceHeader), loss_acc, scale};
}

// loss_acc[0] += sum of partials[0..count) in a fixed order (one workgroup).
int reduce_partials(const double* partials, int count, double* loss_acc, hipStream_t stream);
// scalars[0] = sum partials[0..count), scalars[1] = sum partials[count..2*count), scalars[2] = SPSA g.
int reduce_step(const double* partials, int count, float eps, double* scalars, hipStream_t stream);

// Few-token path (szo_smallm.hip): M <= 16, K % 128 == 0, fp16 tile.
bool small_m_eligible(const szo_linear_desc* d);
bool small_m_step_eligible(const szo_linear_desc* d);      // few enough tokens: sliced into passes of 16 or 32 token rows
int small_m_blocks(const szo_linear_desc* d);
int small_m_slices(const szo_linear_desc* d);              // passes over the weights: 16 or 32 token rows each
bool small_m_shape_eligible(const szo_linear_desc* d);     // the same without looking at the token count
void small_m_force_rblocks(int r);                         // testing hook: 0 = choose; 2, 3 = 32 / 48 token rows per pass wherever M > 16
void small_m_force_stream_once(bool on);                    // testing hook: non-temporal code stream in every one-slice launch
size_t small_m_table_bytes(int n);
int small_m_launch_one(const szo_linear_desc* d, uint64_t seed, uint64_t step, float eps, int sign, bool loss_mode,
                       double* partial_plus, double* partial_minus, hipStream_t stream);
int small_m_step(const szo_linear_desc* descs, int n, uint64_t seed, uint64_t step, float eps, float lr,
                 void* table_dev, double* partial_plus, double* scalars, bool do_forward, bool do_update,
                 hipStream_t stream);

// Optional kernel timing (szo_kernel_timing): when switched on, every launch of a forward kernel
// (kind 0) or of a sparse update kernel (kind 1) is bracketed by a pair of events on its own stream.
// Both calls are no-ops when timing is off.  Defined in szo_kernels.hip.
int timing_begin(hipStream_t stream, int kind = 0);
int timing_end(hipStream_t stream);

// Copies `bytes` (a multiple of 4) of host data into device memory `dst`, in stream order, without
// blocking the host: the data goes through a ring of eight pinned, device-mapped host buffers per host
// thread (grown on demand with hipHostMalloc, released when the thread ends) and a small copy kernel
// reads it from there.  SZO_EUNSUPPORTED while `stream` is being captured into a graph.  A kernel rather than a
// DMA copy because handing over from the copy engine to the compute queue costs more than reading a
// few tens of KB over the host link.  Defined in szo_kernels.hip.
int stage_table(const void* src, size_t bytes, void* dst, hipStream_t stream);

// True while `stream` is being captured into a HIP graph.
bool stream_is_capturing(hipStream_t stream);

// Sets n 32-bit words to zero with a small kernel (defined in szo_kernels.hip).
int zero_words(void* p, int n, hipStream_t stream);

// Wave-wide sum in a fixed order (64 lanes), result valid in every lane.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Called by every thread of every workgroup exactly once, with the thread's partial sum.
// `scratch` is LDS for one double per wave.  Grid is 1-D or flattened to `block_linear` of
// `nblocks`.
__device__ __forceinline__ void block_loss_commit(double local, double* scratch, const LossSink& sink,
                                                  unsigned int block_linear, unsigned int nblocks) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = (blockDim.x + 63) >> 6;
  const double w = wave_sum(local);
  if (lane == 0) scratch[wave] = w;
  __syncthreads();
  __shared__ unsigned int s_last;
  if (threadIdx.x == 0) {
    double b = 0.0;
    for (int i = 0; i < nwaves; ++i) b += scratch[i];
    __hip_atomic_store(&sink.partials[block_linear], b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __threadfence();
    const unsigned int t = __hip_atomic_fetch_add(sink.ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (t == nblocks - 1u);
  }
  __syncthreads();
  if (s_last && wave == 0) {
    __threadfence();
    double acc = 0.0;
    for (unsigned int i = lane; i < nblocks; i += 64)
      acc += __hip_atomic_load(&sink.partials[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    acc = wave_sum(acc);
    if (lane == 0) {
      *sink.loss_acc += sink.scale * acc;
      __hip_atomic_store(sink.ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

}  // namespace szo
