// Perturbed forward of one linear layer (Appendix C.5, "SparseAdd then DenseMM";
// perturbation of Definition 4) as one fused kernel for gfx950:
//
//   4-bit codes --dequantise--> 16-bit tile in LDS  <--scatter--  sp_val[j] + sign*eps*z_j
//   activations (bf16) -------> 16-bit tile in LDS
//   tiles --MFMA 32x32x16--> fp32 accumulators --> y (fp32) and/or sum (y - target)^2 (fp64)
//
// The dense fp weight never exists in memory and the perturbation costs no pass over HBM: it
// is regenerated from (seed, step, entry index) for exactly the entries of the band a wave
// stages.
//
// Work split inside a workgroup.  The first BN/64 waves ("weight waves") each own one 64-row
// band of the weight tile: they load its codes and scales, dequantise them into LDS, and
// scatter the band's sensitive entries on top.  Dense write and sparse overwrite of one LDS
// word are therefore ordered by program order inside one wave and need no barrier.  The other
// waves ("activation waves") convert and stage x.  All waves then run the MFMA loop on the
// staged tile while they stage the next one into the other LDS buffer.
//
// Sensitive entries.  The sparse layout orders entries by (64-row band, 64-column tile), so a
// weight wave consumes its band's entries as one stream while it walks along K.  It computes
// them 256 at a time (one Philox counter = four consecutive entries per lane) into a small
// LDS window holding (tile position, value), and each K step only copies the few entries of
// its tile from the window into the weight tile.
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
constexpr int kWindow = 256;           // sensitive entries computed per refill of a wave's window

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
  int bands;                // ceil(N / 64)
  int grid_m, grid_n;
  uint32_t nnz;
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

// Workgroup = WAVES_M x WAVES_N waves; each wave computes (32*WMB) x (32*WNB) outputs.
template <int WAVES_M, int WAVES_N, int WMB, int WNB, int DT, bool FUSE_LOSS>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) linear_fwd_kernel(FwdParams p) {
  constexpr int NWAVES = WAVES_M * WAVES_N;
  constexpr int BM = 32 * WMB * WAVES_M, BN = 32 * WNB * WAVES_N;
  constexpr int W_WAVES = BN / 64;                 // one per 64-row band of the weight tile
  constexpr int X_WAVES = NWAVES - W_WAVES;
  static_assert(BN % 64 == 0 && X_WAVES > 0, "need whole bands and at least one activation wave");
  constexpr int X_ROWS_PER_PASS = 8 * X_WAVES;     // 8 lanes cover one 128-byte row of x
  constexpr int XCH = BM / X_ROWS_PER_PASS;        // 16-byte chunks per activation lane per tile
  static_assert(BM % X_ROWS_PER_PASS == 0 && XCH % 4 == 0, "x staging must split over the four MFMA k-steps");
  typedef typename Frag<DT>::type frag_t;

  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* const ldsA = lds;                                   // [2][BM*BK]
  uint16_t* const ldsB = lds + 2 * BM * BK;                     // [2][BN*BK]
  float* const winVal = reinterpret_cast<float*>(lds + 2 * (BM + BN) * BK);        // [W_WAVES][kWindow]
  uint16_t* const winPos = reinterpret_cast<uint16_t*>(winVal + W_WAVES * kWindow);  // [W_WAVES][kWindow]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int bm = blockIdx.x / p.grid_n, bn = blockIdx.x - bm * p.grid_n;
  const int m0 = bm * BM, n0 = bn * BN;
  const int nk = p.ktiles;

  float16_t acc[WMB][WNB];
#pragma unroll
  for (int i = 0; i < WMB; ++i)
#pragma unroll
    for (int j = 0; j < WNB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // One MFMA k-step (16 of the tile's 64 columns) on LDS buffer `buf`.
  auto mfma_step = [&](int buf, int ks) {
    const uint16_t* A = ldsA + buf * BM * BK;
    const uint16_t* B = ldsB + buf * BN * BK;
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
  };

  if (wave < W_WAVES) {
    // =============================== weight wave ===============================================
    const int wr = wave * 64 + (lane >> 1), wh = lane & 1;       // tile row (plus 32*i), half of the row
    const int band = n0 / 64 + wave;                             // band of the sparse layout
    const bool band_ok = band < p.bands;
    const uint32_t tp_base = (uint32_t)band * (uint32_t)nk;
    uint32_t tile_lo = 0, band_end = 0;                          // entry range bookkeeping (uniform)
    if (band_ok) {
      tile_lo = __builtin_amdgcn_readfirstlane(p.tile_ptr[tp_base]);
      band_end = __builtin_amdgcn_readfirstlane(p.tile_ptr[tp_base + nk]);
    }
    uint32_t tp_reg = 0;                                         // lane l: tile_ptr[tp_base + 64*c + 1 + l]
    uint32_t win_lo = 0, win_hi = 0;                             // entries [win_lo, win_hi) are in the window
    float* const wv = winVal + wave * kWindow;
    uint16_t* const wp = winPos + wave * kWindow;

    uint4 qreg[2][2];
    uint16_t sreg[2][2];

    auto load_w = [&](int kt, int slot) {
      const int kq = kt * BK + 32 * wh;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int n = n0 + wr + 32 * i;
        if (n < p.N) {
          qreg[slot][i] = *reinterpret_cast<const uint4*>(p.qweight + ((size_t)n * p.K + kq) / 2);
          sreg[slot][i] = p.scales[(size_t)n * (p.K >> p.group_shift) + (kq >> p.group_shift)];
        } else {
          qreg[slot][i] = make_uint4(0x88888888u, 0x88888888u, 0x88888888u, 0x88888888u);
          sreg[slot][i] = 0;
        }
      }
    };

    // part in 0..3: a quarter of the lane's 8 code words
    auto store_w_part = [&](int buf, int slot, int part) {
      uint16_t* B = ldsB + buf * BN * BK;
      const int i = part >> 1;
      const int r = wr + 32 * i;
      const _Float16 sh = __builtin_bit_cast(_Float16, sreg[slot][i]);
      const half2_t sh2 = {sh, sh};
      const float sf = (float)sh;
      const uint32_t q0 = (part & 1) ? qreg[slot][i].z : qreg[slot][i].x;
      const uint32_t q1 = (part & 1) ? qreg[slot][i].w : qreg[slot][i].y;
      const int c = 2 * (part & 1);
      *reinterpret_cast<uint4*>(B + chunk_off(r, 4 * wh + c)) = dequant_word<DT>(q0, sf, sh2);
      *reinterpret_cast<uint4*>(B + chunk_off(r, 4 * wh + c + 1)) = dequant_word<DT>(q1, sf, sh2);
    };

    // Computes entries [s, s+256) of the band (s a multiple of 4) into the window.
    auto refill = [&](uint32_t s) {
      const uint32_t j = s + 4u * lane;
      if (j < band_end) {
        uint32_t idx[4];
        float val[4];
        if (j + 3 < p.nnz) {
          const uint4 iv = *reinterpret_cast<const uint4*>(p.sp_idx + j);
          const float4 vv = *reinterpret_cast<const float4*>(p.sp_val + j);
          idx[0] = iv.x; idx[1] = iv.y; idx[2] = iv.z; idx[3] = iv.w;
          val[0] = vv.x; val[1] = vv.y; val[2] = vv.z; val[3] = vv.w;
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const bool ok = j + c < p.nnz;
            idx[c] = ok ? p.sp_idx[j + c] : 0xFFFFFFFFu;
            val[c] = ok ? p.sp_val[j + c] : 0.0f;
          }
        }
        if (p.signed_eps != 0.0f) {
          float z[4];
          zbar_quad((p.nnz_base + j) >> 2, p.seed, p.step, z);
#pragma unroll
          for (int c = 0; c < 4; ++c) val[c] = fmaf(p.signed_eps, z[c], val[c]);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const uint32_t n = fast_div(idx[c], p.div_mul, p.div_shift);
          const uint32_t r = n - (uint32_t)(band * 64);                   // row inside the band
          const uint32_t kk = (idx[c] - n * (uint32_t)p.K) & 63u;
          wp[4 * lane + c] = (r < 64u) ? (uint16_t)lds_pos<DT>(wave * 64 + (int)r, (int)kk) : (uint16_t)0xFFFFu;
          wv[4 * lane + c] = val[c];
        }
      }
      win_lo = s;
      win_hi = min(s + (uint32_t)kWindow, band_end);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // window visible to the other lanes of the wave
    };

    // Adds the sensitive entries of (band, column tile kt) into LDS buffer `buf`.
    auto scatter = [&](int kt, int buf) {
      if (!band_ok) return;
      if ((kt & 63) == 0) {
        const uint32_t t = tp_base + (uint32_t)kt + 1u + lane;
        tp_reg = (t <= tp_base + (uint32_t)nk) ? p.tile_ptr[t] : band_end;
      }
      const uint32_t tile_hi = __builtin_amdgcn_readlane(tp_reg, kt & 63);
      uint16_t* B = ldsB + buf * BN * BK;
      uint32_t cur = tile_lo;
      tile_lo = tile_hi;
      while (cur < tile_hi) {
        if (cur >= win_hi || cur < win_lo) refill(cur & ~3u);
        const uint32_t hi = min(tile_hi, win_hi);
        for (uint32_t j = cur + lane; j < hi; j += 64) {
          const uint32_t e = j - win_lo;
          const uint32_t pos = wp[e];
          if (pos != 0xFFFFu) {
            uint16_t* w = B + pos;
            Frag<DT>::store(w, Frag<DT>::load(w) + wv[e]);
          }
        }
        cur = hi;
      }
    };

    auto body = [&](int kt, int buf, int slot_next) {
      // MFMA on tile kt (buffer buf) while tile kt+1 (registers slot_next) goes to buffer buf^1
      const bool more = kt + 1 < nk;
      __syncthreads();
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        mfma_step(buf, ks);
        if (more) store_w_part(buf ^ 1, slot_next, ks);
      }
      if (more) scatter(kt + 1, buf ^ 1);
      if (kt + 3 < nk) load_w(kt + 3, slot_next);
    };

    load_w(0, 0);
    if (nk > 1) load_w(1, 1);
#pragma unroll
    for (int part = 0; part < 4; ++part) store_w_part(0, 0, part);
    scatter(0, 0);
    if (nk > 2) load_w(2, 0);
    for (int kt = 0; kt < nk; kt += 2) {
      body(kt, 0, 1);
      if (kt + 1 < nk) body(kt + 1, 1, 0);
    }
  } else {
    // =============================== activation wave ===========================================
    const int xt = tid - 64 * W_WAVES;
    const int xc = xt & 7, xr = xt >> 3;                       // chunk, row (plus X_ROWS_PER_PASS*i)
    uint4 xreg[2][XCH];

    auto load_x = [&](int kt, int slot) {
      const int k0 = kt * BK;
#pragma unroll
      for (int i = 0; i < XCH; ++i) {
        const int m = m0 + xr + X_ROWS_PER_PASS * i;
        xreg[slot][i] = (m < p.M) ? *reinterpret_cast<const uint4*>(p.x + (size_t)m * p.K + k0 + xc * 8)
                                  : make_uint4(0, 0, 0, 0);
      }
    };
    auto store_x_part = [&](int buf, int slot, int part) {
      uint16_t* A = ldsA + buf * BM * BK;
#pragma unroll
      for (int i = part * (XCH / 4); i < (part + 1) * (XCH / 4); ++i) {
        const int r = xr + X_ROWS_PER_PASS * i;
        *reinterpret_cast<uint4*>(A + chunk_off(r, xc)) = stage_x_chunk<DT>(xreg[slot][i]);
      }
    };
    auto body = [&](int kt, int buf, int slot_next) {
      const bool more = kt + 1 < nk;
      __syncthreads();
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        mfma_step(buf, ks);
        if (more) store_x_part(buf ^ 1, slot_next, ks);
      }
      if (kt + 3 < nk) load_x(kt + 3, slot_next);
    };

    load_x(0, 0);
    if (nk > 1) load_x(1, 1);
#pragma unroll
    for (int part = 0; part < 4; ++part) store_x_part(0, 0, part);
    if (nk > 2) load_x(2, 0);
    for (int kt = 0; kt < nk; kt += 2) {
      body(kt, 0, 1);
      if (kt + 1 < nk) body(kt + 1, 1, 0);
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
    __shared__ double scratch[NWAVES];
    block_loss_commit(loss, scratch, p.sink, blockIdx.x, gridDim.x);
  }
}

// ---- host side -----------------------------------------------------------------------------

static int g_tile_config = 0;      // 0 = choose by shape, 1 = 128x128 (4 waves), 2 = 256x256 (8 waves)

static int ilog2_exact(int v) {
  int s = 0;
  while ((1 << s) < v) ++s;
  return (1 << s) == v ? s : -1;
}

static int validate_desc(const szo_linear_desc* d, int sign, bool need_y, bool need_target) {
  if (!d) return SZO_EINVAL;
  if (d->M < 0 || d->N < 0 || d->K <= 0 || d->nnz < 0) return SZO_EINVAL;
  if (sign < -1 || sign > 1) return SZO_EINVAL;
  if (d->tile_dtype != SZO_TILE_F16 && d->tile_dtype != SZO_TILE_BF16) return SZO_EINVAL;
  if (d->group <= 0 || d->K % d->group) return SZO_EINVAL;
  if (d->nnz_base & 3) return SZO_EINVAL;
  if (d->group != 32 && d->group != 64 && d->group != 128) return SZO_EUNSUPPORTED;
  if (d->K % BK) return SZO_EUNSUPPORTED;
  if ((uint64_t)d->N * (uint64_t)d->K > 0xFFFFFFFFull) return SZO_EUNSUPPORTED;
  if (d->M > 0x7FFFFFFF || d->N > 0x7FFFFFFF || d->nnz > 0xFFFFFFFFll) return SZO_EUNSUPPORTED;
  if (d->M == 0 || d->N == 0) return SZO_OK;
  if (!d->x || !d->qweight || !d->scales || !d->tile_ptr) return SZO_EINVAL;
  if (d->nnz > 0 && (!d->sp_idx || !d->sp_val)) return SZO_EINVAL;
  if (need_y && !d->y) return SZO_EINVAL;
  if (need_target && !d->target) return SZO_EINVAL;
  if (((uintptr_t)d->x & 15) || ((uintptr_t)d->qweight & 15) || ((uintptr_t)d->scales & 1) ||
      ((uintptr_t)d->tile_ptr & 3) || ((uintptr_t)d->sp_idx & 15) || ((uintptr_t)d->sp_val & 15) ||
      ((uintptr_t)d->y & 3) || ((uintptr_t)d->target & 1))
    return SZO_EINVAL;
  return SZO_OK;
}

template <int WAVES_M, int WAVES_N, int WMB, int WNB, int DT, bool FUSE>
static int launch(FwdParams& p, hipStream_t stream) {
  constexpr int BM = 32 * WMB * WAVES_M, BN = 32 * WNB * WAVES_N;
  p.grid_m = (p.M + BM - 1) / BM;
  p.grid_n = (p.N + BN - 1) / BN;
  const int64_t blocks = (int64_t)p.grid_m * p.grid_n;
  if (blocks > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
  if (FUSE && blocks > kMaxLossPartials) return SZO_EUNSUPPORTED;
  constexpr size_t lds_bytes = 2 * (size_t)(BM + BN) * BK * sizeof(uint16_t) + (size_t)(BN / 64) * kWindow * 6;
  auto kern = linear_fwd_kernel<WAVES_M, WAVES_N, WMB, WNB, DT, FUSE>;
  static bool attr_set = false;     // per instantiation
  if (!attr_set) {
    SZO_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
    attr_set = true;
  }
  kern<<<(unsigned)blocks, 64 * WAVES_M * WAVES_N, lds_bytes, stream>>>(p);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

template <int DT, bool FUSE>
static int dispatch_tile(FwdParams& p, hipStream_t stream) {
  int cfg = g_tile_config;
  if (cfg == 0) {
    const int64_t big_blocks = (int64_t)((p.M + 255) / 256) * ((p.N + 255) / 256);
    cfg = big_blocks >= 192 ? 2 : 1;
  }
  if (cfg == 2) return launch<2, 4, 4, 2, DT, FUSE>(p, stream);
  return launch<2, 2, 2, 2, DT, FUSE>(p, stream);
}

static int run_forward(const szo_linear_desc* d, uint64_t seed, uint64_t step, int sign, float eps, bool fuse,
                       double scale, double* loss_acc, void* workspace, hipStream_t stream) {
  const int rc = validate_desc(d, sign, !fuse, fuse);
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
  p.nnz = (uint32_t)d->nnz;
  p.group_shift = ilog2_exact(d->group);
  p.ktiles = p.K / BK;
  p.bands = (p.N + SZO_TILE_ROWS - 1) / SZO_TILE_ROWS;
  {
    // multiplier for floor(v / K), v < 2^32: l = ceil(log2 K), mul = floor(2^32 (2^l - K) / K) + 1
    int l = 0;
    while ((1ull << l) < (uint64_t)p.K) ++l;
    if (l == 0) return SZO_EUNSUPPORTED;
    p.div_mul = (uint32_t)((((1ull << l) - (uint64_t)p.K) << 32) / (uint64_t)p.K + 1ull);
    p.div_shift = l - 1;
  }
  p.nnz_base = d->nnz_base; p.seed = seed; p.step = step;
  p.signed_eps = (float)sign * eps;
  if (fuse) p.sink = make_sink(workspace, loss_acc, scale);
  if (d->tile_dtype == SZO_TILE_F16)
    return fuse ? dispatch_tile<SZO_TILE_F16, true>(p, stream) : dispatch_tile<SZO_TILE_F16, false>(p, stream);
  return fuse ? dispatch_tile<SZO_TILE_BF16, true>(p, stream) : dispatch_tile<SZO_TILE_BF16, false>(p, stream);
}

}  // namespace szo

using namespace szo;

extern "C" {

int szo_set_tile_config(int config) {
  if (config < 0 || config > 2) return SZO_EINVAL;
  g_tile_config = config;
  return SZO_OK;
}

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
    const int rc = validate_desc(&descs[i], 1, !fuse, true);
    if (rc != SZO_OK) return rc;
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
