// Perturbed forward of one linear layer (Appendix C.5, "SparseAdd then DenseMM";
// perturbation of Definition 4) as one fused kernel for gfx950:
//
//   4-bit codes --dequantise--> 16-bit tile in LDS  <--scatter--  sp_val[j] + sign*eps*z_j
//   activations (bf16) -------> 16-bit tile in LDS
//   tiles --MFMA 32x32x16--> fp32 accumulators --> y (fp32) and/or sum (y - target)^2 (fp64)
//
// The dense fp weight never exists in memory and the perturbation costs no pass over HBM:
// it is regenerated from (seed, step, entry index) for exactly the entries of the tile being
// staged.  Each wave dequantises a band of weight rows AND scatters the sensitive entries of
// the same band, so the dense write and the sparse overwrite of one LDS word are ordered by
// program order inside one wave and no extra barrier is needed.
#include "szo_internal.h"
#include "szo_rng.cuh"

namespace szo {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int BK = 64;                 // K extent of one staged tile = SZO_TILE_COLS
constexpr int kThreads = 256;          // four waves, arranged 2 (M) x 2 (N)

struct FwdParams {
  const uint16_t* x;        // bf16 [M,K]
  const uint8_t* qweight;   // [N,K/2]
  const uint16_t* scales;   // fp16 [N,K/group]
  const uint32_t* tile_ptr;
  const uint32_t* sp_idx;
  const float* sp_val;
  float* y;                 // may be null when the loss is fused
  const uint16_t* target;   // bf16 [M,N] (fused loss only)
  int M, N, K;
  int group_shift;          // log2(group)
  int ktiles;               // K / 64
  int row_groups;           // ceil(N / 128)
  int grid_m, grid_n;
  uint32_t div_mul;         // exact division of a flat index by K: see fast_div
  int div_shift;
  uint64_t nnz_base, seed, step;
  float signed_eps;         // sign * eps; 0 = no perturbation
  LossSink sink;
};

// floor(v / d) for 32-bit v with a precomputed multiplier (Granlund-Montgomery, round-up form).
__device__ __forceinline__ uint32_t fast_div(uint32_t v, uint32_t mul, int shift) {
  const uint32_t t = __umulhi(mul, v);
  return (t + ((v - t) >> 1)) >> shift;
}

// Position of column kk (0..63) of tile row r inside the LDS tile, in 16-bit elements.
// Rows are 64 elements (128 bytes); the eight 16-byte chunks of a row are XOR-swizzled with
// the row number so that 32 lanes reading the same chunk of 32 consecutive rows spread over
// all banks.  In f16 mode the eight elements of a chunk are stored in the order
// 0,4,1,5,2,6,3,7 -- the order in which two nibbles per 16-bit lane fall out of a packed
// word -- and the activations are stored in the same order, which leaves the dot product
// unchanged.
template <int DT>
__device__ __forceinline__ int lds_pos(int r, int kk) {
  const int chunk = kk >> 3, w = kk & 7;
  const int p = (DT == SZO_TILE_F16) ? (((w & 3) << 1) | (w >> 2)) : w;
  return r * BK + (((chunk ^ (r & 7)) << 3) | p);
}

__device__ __forceinline__ int chunk_off(int r, int chunk) {   // in 16-bit elements
  return r * BK + ((chunk ^ (r & 7)) << 3);
}

// ---- activations: 8 bf16 (one 16-byte chunk) -> 8 tile elements ------------------------------
template <int DT>
__device__ __forceinline__ uint4 stage_x_chunk(uint4 u) {
  if (DT == SZO_TILE_BF16) return u;
  // bf16 -> fp32 is a shift; fp32 -> fp16 is exact for |x| in [2^-14, 65504] (8-bit significand)
  auto lo = [](uint32_t v) { return __uint_as_float(v << 16); };
  auto hi = [](uint32_t v) { return __uint_as_float(v & 0xFFFF0000u); };
  auto pk = [](float a, float b) {
    auto h = __builtin_amdgcn_cvt_pkrtz(a, b);
    return __builtin_bit_cast(uint32_t, h);
  };
  uint4 o;
  o.x = pk(lo(u.x), lo(u.z));   // elements 0,4
  o.y = pk(hi(u.x), hi(u.z));   // 1,5
  o.z = pk(lo(u.y), lo(u.w));   // 2,6
  o.w = pk(hi(u.y), hi(u.w));   // 3,7
  return o;
}

// ---- weights: 8 codes (one 32-bit word) -> 8 tile elements ------------------------------------
// dq = (code - 8) * scale, one rounding to the tile type.
template <int DT>
__device__ __forceinline__ uint4 dequant_word(uint32_t q, float scale_f32, half2_t scale_h2) {
  uint4 o;
  if (DT == SZO_TILE_F16) {
    // 0x6400 | c is the fp16 number 1024 + c; subtracting 1032 is exact; the product with the
    // fp16 scale is rounded once, which is the rounding of the exact (code-8)*scale.
    const half2_t bias = {(_Float16)1032.0f, (_Float16)1032.0f};
    auto cvt = [&](uint32_t bits) {
      half2_t h = __builtin_bit_cast(half2_t, bits);
      h = (h - bias) * scale_h2;
      return __builtin_bit_cast(uint32_t, h);
    };
    o.x = cvt((q & 0x000F000Fu) | 0x64006400u);          // codes 0,4
    o.y = cvt(((q >> 4) & 0x000F000Fu) | 0x64006400u);   // 1,5
    o.z = cvt(((q >> 8) & 0x000F000Fu) | 0x64006400u);   // 2,6
    o.w = cvt(((q >> 12) & 0x000F000Fu) | 0x64006400u);  // 3,7
  } else {
    const float m8s = -8.0f * scale_f32;
    auto one = [&](int i) { return fmaf((float)((q >> (4 * i)) & 15u), scale_f32, m8s); };   // exact in fp32
    auto pk = [&](int i) {
      float2_t f = {one(i), one(i + 1)};
      bf16x2_t b = __builtin_convertvector(f, bf16x2_t);     // round to nearest even
      return __builtin_bit_cast(uint32_t, b);
    };
    o.x = pk(0); o.y = pk(2); o.z = pk(4); o.w = pk(6);
  }
  return o;
}

template <int DT> struct Frag;
template <> struct Frag<SZO_TILE_F16> {
  typedef half8_t type;
  static __device__ __forceinline__ float16_t mfma(type a, type b, float16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ float load(const uint16_t* p) { return (float)*reinterpret_cast<const _Float16*>(p); }
  static __device__ __forceinline__ void store(uint16_t* p, float v) { *reinterpret_cast<_Float16*>(p) = (_Float16)v; }
};
template <> struct Frag<SZO_TILE_BF16> {
  typedef bf16x8_t type;
  static __device__ __forceinline__ float16_t mfma(type a, type b, float16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ float load(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
  static __device__ __forceinline__ void store(uint16_t* p, float v) { *reinterpret_cast<__bf16*>(p) = (__bf16)v; }
};

// WMB x WNB = number of 32x32 MFMA blocks per wave along M and N.
// Block tile: BM = 64*WMB rows of x, BN = 64*WNB rows of W.  WNB must be even: a wave then
// stages BN/4 = 16*WNB weight rows, i.e. whole 32-row bands of the sparse layout.
template <int WMB, int WNB, int DT, bool FUSE_LOSS>
__global__ void __launch_bounds__(kThreads) linear_fwd_kernel(FwdParams p) {
  static_assert(WNB % 2 == 0, "a wave must own whole 32-row bands");
  constexpr int BM = 64 * WMB, BN = 64 * WNB;
  constexpr int XP = BM / 32;            // 16-byte x chunks per thread per tile
  constexpr int WP = WNB / 2;            // 16-byte code chunks per lane per tile (= bands per wave)
  constexpr int RW = BN / 4;             // weight rows staged by one wave
  typedef typename Frag<DT>::type frag_t;

  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* const ldsA = lds;                       // [2][BM*BK]
  uint16_t* const ldsB = lds + 2 * BM * BK;         // [2][BN*BK]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int bm = blockIdx.x / p.grid_n, bn = blockIdx.x - bm * p.grid_n;
  const int m0 = bm * BM, n0 = bn * BN;

  // ---- per-thread global addresses ----
  const int xc = tid & 7, xr = tid >> 3;            // chunk, row (plus 32*i)
  const int wh = lane & 1, wr = wave * RW + (lane >> 1);   // half of the tile row, row (plus 32*i)

  uint4 xreg[XP];
  uint4 wreg[WP];
  uint16_t sreg[WP];

  auto load_tile = [&](int kt) {
    const int k0 = kt * BK;
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int m = m0 + xr + 32 * i;
      xreg[i] = (m < p.M) ? *reinterpret_cast<const uint4*>(p.x + (size_t)m * p.K + k0 + xc * 8)
                          : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int n = n0 + wr + 32 * i;
      const int kq = k0 + 32 * wh;
      if (n < p.N) {
        wreg[i] = *reinterpret_cast<const uint4*>(p.qweight + ((size_t)n * p.K + kq) / 2);
        sreg[i] = p.scales[(size_t)n * (p.K >> p.group_shift) + (kq >> p.group_shift)];
      } else {
        wreg[i] = make_uint4(0x88888888u, 0x88888888u, 0x88888888u, 0x88888888u);
        sreg[i] = 0;
      }
    }
  };

  auto store_tile = [&](int buf) {
    uint16_t* A = ldsA + buf * BM * BK;
    uint16_t* B = ldsB + buf * BN * BK;
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int r = xr + 32 * i;
      *reinterpret_cast<uint4*>(A + chunk_off(r, xc)) = stage_x_chunk<DT>(xreg[i]);
    }
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int r = wr + 32 * i;
      const _Float16 sh = __builtin_bit_cast(_Float16, sreg[i]);
      const half2_t sh2 = {sh, sh};
      const float sf = (float)sh;
      const uint32_t q[4] = {wreg[i].x, wreg[i].y, wreg[i].z, wreg[i].w};
#pragma unroll
      for (int c = 0; c < 4; ++c)
        *reinterpret_cast<uint4*>(B + chunk_off(r, 4 * wh + c)) = dequant_word<DT>(q[c], sf, sh2);
    }
  };

  // Sensitive entries of this wave's bands for column tile kt: add sp_val + sign*eps*z into
  // the staged tile (the dense code at a mask position is the zero code, so the add lands on 0).
  auto scatter_tile = [&](int kt, int buf) {
    uint16_t* B = ldsB + buf * BN * BK;
    const int nb0 = n0 + wave * RW;                 // first global row of the wave's bands (multiple of 32)
    const int grp = nb0 / SZO_GROUP_ROWS;
    if (grp >= p.row_groups) return;
    const int t0 = (grp * p.ktiles + kt) * 4 + (nb0 % SZO_GROUP_ROWS) / SZO_TILE_ROWS;
    const uint32_t j0 = p.tile_ptr[t0], j1 = p.tile_ptr[t0 + WP];
    for (uint32_t j = j0 + lane; j < j1; j += 64) {
      const uint32_t flat = p.sp_idx[j];
      float v = p.sp_val[j];
      if (p.signed_eps != 0.0f) {
        const uint64_t J = p.nnz_base + j;
        float z[4];
        zbar_quad(J >> 2, p.seed, p.step, z);
        const int sel = (int)(J & 3);
        const float zj = sel == 0 ? z[0] : sel == 1 ? z[1] : sel == 2 ? z[2] : z[3];
        v = fmaf(p.signed_eps, zj, v);
      }
      const uint32_t n = fast_div(flat, p.div_mul, p.div_shift);
      const int r = (int)n - n0, kk = (int)(flat - n * (uint32_t)p.K) - kt * BK;
      if ((unsigned)r < (unsigned)BN && (unsigned)kk < (unsigned)BK) {   // a malformed layout must not leave the tile
        uint16_t* w = B + lds_pos<DT>(r, kk);
        Frag<DT>::store(w, Frag<DT>::load(w) + v);
      }
    }
  };

  float16_t acc[WMB][WNB];
#pragma unroll
  for (int i = 0; i < WMB; ++i)
#pragma unroll
    for (int j = 0; j < WNB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  load_tile(0);
  store_tile(0);
  scatter_tile(0, 0);

  const int nk = p.ktiles;
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    const bool more = kt + 1 < nk;
    if (more) load_tile(kt + 1);
    __syncthreads();                         // tile kt complete; tile kt-1 no longer read
    const uint16_t* A = ldsA + buf * BM * BK;
    const uint16_t* B = ldsB + buf * BN * BK;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int chunk = 2 * ks + (lane >> 5);
      frag_t a[WMB], b[WNB];
#pragma unroll
      for (int i = 0; i < WMB; ++i)
        a[i] = *reinterpret_cast<const frag_t*>(A + chunk_off(wm * 32 * WMB + i * 32 + (lane & 31), chunk));
#pragma unroll
      for (int j = 0; j < WNB; ++j)
        b[j] = *reinterpret_cast<const frag_t*>(B + chunk_off(wn * 32 * WNB + j * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < WMB; ++i)
#pragma unroll
        for (int j = 0; j < WNB; ++j) acc[i][j] = Frag<DT>::mfma(a[i], b[j], acc[i][j]);
    }
    if (more) {
      store_tile(buf ^ 1);
      scatter_tile(kt + 1, buf ^ 1);
    }
  }

  // ---- epilogue: accumulator (i,j) register r holds
  //      row  32*i + 8*(r/4) + 4*(lane/32) + r%4 ,  column 32*j + lane%32  of the wave tile ----
  double loss = 0.0;
#pragma unroll
  for (int i = 0; i < WMB; ++i) {
#pragma unroll
    for (int j = 0; j < WNB; ++j) {
      const int n = n0 + wn * 32 * WNB + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 32 * WMB + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < p.M && n < p.N) {
          const float v = acc[i][j][r];
          if (p.y) p.y[(size_t)m * p.N + n] = v;
          if (FUSE_LOSS) {
            const double d = (double)v - (double)__uint_as_float((uint32_t)p.target[(size_t)m * p.N + n] << 16);
            loss = fma(d, d, loss);
          }
        }
      }
    }
  }
  if (FUSE_LOSS) {
    __shared__ double scratch[kThreads / 64];
    block_loss_commit(loss, scratch, p.sink, blockIdx.x, gridDim.x);
  }
}

// ---- host side -----------------------------------------------------------------------------

static int ilog2_exact(int v) {
  int s = 0;
  while ((1 << s) < v) ++s;
  return (1 << s) == v ? s : -1;
}

static int validate(const szo_linear_desc* d, int sign, bool need_y, bool need_target) {
  if (!d) return SZO_EINVAL;
  if (d->M < 0 || d->N < 0 || d->K <= 0 || d->nnz < 0) return SZO_EINVAL;
  if (sign < -1 || sign > 1) return SZO_EINVAL;
  if (d->tile_dtype != SZO_TILE_F16 && d->tile_dtype != SZO_TILE_BF16) return SZO_EINVAL;
  if (d->group <= 0 || d->K % d->group) return SZO_EINVAL;
  if (d->nnz_base & 3) return SZO_EINVAL;
  if (d->group != 32 && d->group != 64 && d->group != 128) return SZO_EUNSUPPORTED;
  if (d->K % BK) return SZO_EUNSUPPORTED;
  if ((uint64_t)d->N * (uint64_t)d->K > 0xFFFFFFFFull) return SZO_EUNSUPPORTED;
  if (d->M > 0x7FFFFFFF || d->N > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
  if (d->M == 0 || d->N == 0) return SZO_OK;
  if (!d->x || !d->qweight || !d->scales || !d->tile_ptr) return SZO_EINVAL;
  if (d->nnz > 0 && (!d->sp_idx || !d->sp_val)) return SZO_EINVAL;
  if (need_y && !d->y) return SZO_EINVAL;
  if (need_target && !d->target) return SZO_EINVAL;
  if (((uintptr_t)d->x & 15) || ((uintptr_t)d->qweight & 15) || ((uintptr_t)d->scales & 1) ||
      ((uintptr_t)d->tile_ptr & 3) || ((uintptr_t)d->sp_idx & 3) || ((uintptr_t)d->sp_val & 3) ||
      ((uintptr_t)d->y & 3) || ((uintptr_t)d->target & 1))
    return SZO_EINVAL;
  return SZO_OK;
}

template <int WMB, int WNB, int DT, bool FUSE>
static int launch(FwdParams& p, hipStream_t stream) {
  constexpr int BM = 64 * WMB, BN = 64 * WNB;
  p.grid_m = (p.M + BM - 1) / BM;
  p.grid_n = (p.N + BN - 1) / BN;
  const int64_t blocks = (int64_t)p.grid_m * p.grid_n;
  if (blocks > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
  if (FUSE && blocks > kMaxLossPartials) return SZO_EUNSUPPORTED;
  constexpr size_t lds_bytes = 2 * (size_t)(BM + BN) * BK * sizeof(uint16_t);
  auto kern = linear_fwd_kernel<WMB, WNB, DT, FUSE>;
  static bool attr_set = false;     // per instantiation
  if (!attr_set) {
    SZO_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
    attr_set = true;
  }
  kern<<<(unsigned)blocks, kThreads, lds_bytes, stream>>>(p);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

template <bool FUSE>
static int dispatch(FwdParams& p, int dt, hipStream_t stream) {
  if (dt == SZO_TILE_F16) return launch<2, 2, SZO_TILE_F16, FUSE>(p, stream);
  return launch<2, 2, SZO_TILE_BF16, FUSE>(p, stream);
}

static int run_forward(const szo_linear_desc* d, uint64_t seed, uint64_t step, int sign, float eps, bool fuse,
                       double scale, double* loss_acc, void* workspace, hipStream_t stream) {
  const int rc = validate(d, sign, !fuse, fuse);
  if (rc != SZO_OK) return rc;
  if (fuse && (!loss_acc || !workspace || ((uintptr_t)workspace & 7))) return SZO_EINVAL;
  if (d->M == 0 || d->N == 0) return SZO_OK;
  FwdParams p{};
  p.x = (const uint16_t*)d->x;
  p.qweight = d->qweight;
  p.scales = (const uint16_t*)d->scales;
  p.tile_ptr = d->tile_ptr;
  p.sp_idx = d->sp_idx;
  p.sp_val = d->sp_val;
  p.y = d->y;
  p.target = (const uint16_t*)d->target;
  p.M = (int)d->M; p.N = (int)d->N; p.K = (int)d->K;
  p.group_shift = ilog2_exact(d->group);
  p.ktiles = p.K / BK;
  p.row_groups = (p.N + SZO_GROUP_ROWS - 1) / SZO_GROUP_ROWS;
  {
    // multiplier for floor(v / K), v < 2^32: l = ceil(log2 K), mul = floor(2^32 (2^l - K) / K) + 1
    int l = 0;
    while ((1ull << l) < (uint64_t)p.K) ++l;
    p.div_mul = (uint32_t)((((1ull << l) - (uint64_t)p.K) << 32) / (uint64_t)p.K + 1ull);
    p.div_shift = l > 0 ? l - 1 : 0;
    if (l == 0) return SZO_EUNSUPPORTED;
  }
  p.nnz_base = d->nnz_base; p.seed = seed; p.step = step;
  p.signed_eps = (float)sign * eps;
  if (fuse) p.sink = make_sink(workspace, loss_acc, scale);
  return fuse ? dispatch<true>(p, d->tile_dtype, stream) : dispatch<false>(p, d->tile_dtype, stream);
}

}  // namespace szo

using namespace szo;

extern "C" {

int szo_linear_fwd(const szo_linear_desc* desc, uint64_t seed, uint64_t step, int sign, float eps, void* stream) {
  return run_forward(desc, seed, step, sign, eps, false, 0.0, nullptr, nullptr, (hipStream_t)stream);
}

int szo_linear_fwd_mse(const szo_linear_desc* desc, uint64_t seed, uint64_t step, int sign, float eps,
                       double scale, double* loss_acc, void* workspace, void* stream) {
  return run_forward(desc, seed, step, sign, eps, true, scale, loss_acc, workspace, (hipStream_t)stream);
}

int szo_zo_step(const szo_linear_desc* descs, int n, uint64_t seed, uint64_t step, float eps, float lr,
                double* scalars, void* workspace, int flags, void* stream) {
  if (n < 0 || (n > 0 && !descs) || !scalars || !workspace) return SZO_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const bool fuse = flags & SZO_STEP_FUSED_LOSS;
  for (int i = 0; i < n; ++i) {     // reject everything before anything is enqueued
    const int rc = validate(&descs[i], 1, !fuse, true);
    if (rc != SZO_OK) return rc;
    if (descs[i].nnz > 0 && ((uintptr_t)descs[i].sp_val & 15)) return SZO_EINVAL;
  }
  {
    const int rc0 = zero_words(scalars, 6, s);      // a fill kernel, not a memset node: safe under graph capture
    if (rc0 != SZO_OK) return rc0;
  }
  for (int pass = 0; pass < 2; ++pass) {
    const int sign = pass == 0 ? +1 : -1;
    for (int i = 0; i < n; ++i) {
      const szo_linear_desc* d = &descs[i];
      if (d->M == 0 || d->N == 0) continue;
      const double scale = 1.0 / ((double)d->M * (double)d->N);
      int rc;
      if (fuse) {
        rc = run_forward(d, seed, step, sign, eps, true, scale, scalars + pass, workspace, s);
      } else {
        rc = run_forward(d, seed, step, sign, eps, false, 0.0, nullptr, nullptr, s);
        if (rc == SZO_OK) rc = szo_mse_loss(d->y, d->target, d->M * d->N, scale, scalars + pass, workspace, s);
      }
      if (rc != SZO_OK) return rc;
    }
  }
  int rc = szo_spsa_g(scalars, scalars + 1, eps, scalars + 2, s);
  if (rc != SZO_OK) return rc;
  for (int i = 0; i < n; ++i) {
    rc = szo_sparse_update(descs[i].sp_val, descs[i].sp_idx, descs[i].nnz, descs[i].nnz_base, seed, step,
                           scalars + 2, lr, s);
    if (rc != SZO_OK) return rc;
  }
  return SZO_OK;
}

}  // extern "C"
