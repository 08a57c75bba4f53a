// Few-token path (M <= 16): the forward is bound by streaming the 4-bit weights from HBM, not by
// the matrix cores, and the paper's own guideline for this regime (Appendix C.5) is the
// SparseAddMM association:   y = x Dequantize(Q(w_dense))^T  +  x w_sparse^T.
// Two consequences shape this kernel:
//   * the dense product does not depend on the perturbation, so ONE pass over the weights
//     serves both the +eps and the -eps forward of a ZO step (Definition 1 needs f at both);
//   * the sparse product is k << d rank-one column updates, accumulated per 64-row band.
//
// One workgroup = 256 output columns (4 bands, one wave each) x all of K, walked in chunks of
// 1024 columns of x that are staged in LDS as fp16 (16 token rows, zero padded).  Per chunk a wave
//   - streams its band's codes, 16 bytes per lane, eight loads in flight, dequantises them in
//     registers straight into the B operand of v_mfma_f32_16x16x32_f16 (no LDS round trip: every
//     weight is used once), and adds each 128-column partial product times the group scale;
//   - regenerates the Gaussians of the band's sensitive entries in the chunk (same routine and
//     same counters as the large-batch kernel and the update), splits the entries into four lists
//     by (row mod 4) so that four entries can be accumulated at once without two of them touching
//     the same row, and adds  (v +- eps z) x[:,k]  into a 64x16 (+,-) accumulator in LDS.
// The epilogue adds the two parts and either stores y for the requested sign or folds the
// squared error against the target into two fp64 partials per workgroup (one per sign).
// Everything is accumulated in a fixed order: results are bit-reproducible.
#include "szo_internal.h"
#include "szo_rng.cuh"

namespace szo {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int SM_ROWS = 16;             // token rows of the MFMA (M padded up to this)
constexpr int SM_BN = 256;              // output columns per workgroup = 4 bands of 64
constexpr int SM_KC = 512;              // columns of x staged per chunk (double buffered)
constexpr int SM_XSTRIDE = SM_KC + 8;   // LDS row stride of x in fp16 elements (+16 B against bank conflicts)
constexpr int SM_WIN = 256;             // sensitive entries computed per window refill

struct SmallMat {
  const uint16_t* x;        // bf16 [M,K]
  const uint8_t* qweight;   // [N,K/2]
  const uint16_t* scales;   // fp16 [N,K/group]
  const uint32_t* tile_ptr;
  const uint32_t* sp_idx;
  float* sp_val;
  const uint16_t* target;   // bf16 [M,N]   (loss mode)
  float* y;                 // fp32 [M,N]   (store mode)
  uint64_t nnz_base;
  double loss_scale;
  int N, K;
  uint32_t nnz;
  int group_shift;
  uint32_t div_mul;
  int div_shift;
  int first_block;          // workgroups of earlier matrices in this launch
  int partial_base;         // index of this matrix's first loss partial
  int64_t first_quad;       // Philox counters (groups of 4 entries) of earlier matrices: grouped update
};

struct SmallArgs {
  const SmallMat* table;    // device table of n_mats matrices, or null: use `one`
  SmallMat one;
  int n_mats;
  int M;
  int store_sign;           // store mode: which forward to write (-1, 0, +1); loss mode: unused
  int loss_mode;            // 1: write loss partials for both signs, 0: store y
  uint64_t seed, step;
  float eps;                // perturbation scale of the "+" forward (the "-" forward uses -eps)
  double* partial_plus;     // [total workgroups]
  double* partial_minus;
};

__device__ __forceinline__ uint32_t sm_fast_div(uint32_t v, uint32_t mul, int shift) {
  const uint32_t t = __umulhi(mul, v);
  return (t + ((v - t) >> 1)) >> shift;
}

// Position of column kk inside its 8-element chunk in LDS: chunks keep the order 0,4,1,5,2,6,3,7
// in which the dequantised nibbles come out, so that x and the weights pair up element by element.
__device__ __forceinline__ int sm_xpos(int kk) {
  const int w = kk & 7;
  return (kk & ~7) | ((w & 3) << 1) | (w >> 2);
}

__device__ __forceinline__ uint32_t sm_and_or(uint32_t a, uint32_t mask, uint32_t bits_vgpr) {
  uint32_t r;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(bits_vgpr));
  return r;
}

// 8 codes -> 8 fp16 values (code - 8), optionally times the group scale (PRESCALE), in the order
// (0,4)(1,5)(2,6)(3,7).  0x6400|c reads 1024+c and 0x5400|(c<<4) reads 64+c; both offsets are exact.
template <bool PRESCALE>
__device__ __forceinline__ half8_t sm_dequant_word(uint32_t q, uint32_t magic_lo, uint32_t magic_hi, half2_t s2) {
  const half2_t off_lo = {(_Float16)1032.0f, (_Float16)1032.0f}, off_hi = {(_Float16)72.0f, (_Float16)72.0f};
  const uint32_t q8 = q >> 8;
  half2_t h0 = __builtin_bit_cast(half2_t, sm_and_or(q, 0x000F000Fu, magic_lo)) - off_lo;
  half2_t h1 = __builtin_bit_cast(half2_t, sm_and_or(q, 0x00F000F0u, magic_hi)) - off_hi;
  half2_t h2 = __builtin_bit_cast(half2_t, sm_and_or(q8, 0x000F000Fu, magic_lo)) - off_lo;
  half2_t h3 = __builtin_bit_cast(half2_t, sm_and_or(q8, 0x00F000F0u, magic_hi)) - off_hi;
  if (PRESCALE) { h0 *= s2; h1 *= s2; h2 *= s2; h3 *= s2; }
  half8_t r;
  r[0] = h0[0]; r[1] = h0[1]; r[2] = h1[0]; r[3] = h1[1];
  r[4] = h2[0]; r[5] = h2[1]; r[6] = h3[0]; r[7] = h3[1];
  return r;
}

__device__ __forceinline__ uint32_t sm_stage_x_word(u32x4 u, int w) {
  const uint32_t first = (w < 2) ? u[0] : u[1], second = (w < 2) ? u[2] : u[3];
  float a, b;
  if ((w & 1) == 0) { a = __uint_as_float(first << 16); b = __uint_as_float(second << 16); }
  else              { a = __uint_as_float(first & 0xFFFF0000u); b = __uint_as_float(second & 0xFFFF0000u); }
  auto h = __builtin_amdgcn_cvt_pkrtz(a, b);
  return __builtin_bit_cast(uint32_t, h);
}

// G128 = quantisation group of 128: one scale per (row, 128-column block), prefetched four at a
// time and applied to the block's partial product.  Other group sizes take the scale from memory
// and apply it to every element before the product (a plain, slower path).
//
// Pipeline of one wave: the code stream (16-byte loads, 8 in flight per lane) runs ahead across
// chunk boundaries; x of the next chunk is loaded into registers before the current chunk's work and
// written to the other LDS buffer after it; the sparse arrays of the current chunk are requested
// before its dense loop and consumed after it.  One barrier per chunk.
template <bool G128>
__global__ void __launch_bounds__(256) small_m_kernel(SmallArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  _Float16* const xs = reinterpret_cast<_Float16*>(smem);                              // [2][16][SM_XSTRIDE]
  float2* const ysp = reinterpret_cast<float2*>(xs + 2 * SM_ROWS * SM_XSTRIDE);          // [4 waves][64 rows][16 m] (+,-)
  float2* const winv = ysp + 4 * 64 * SM_ROWS;                                           // [4 waves][SM_WIN] (value, eps*z)
  uint16_t* const winp = reinterpret_cast<uint16_t*>(winv + 4 * SM_WIN);                 // [4 waves][SM_WIN] row<<10 | column in chunk

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // ---- which matrix, which 256-column strip ----
  const SmallMat* mp = &a.one;
  if (a.table) {
    int lo = 0, hi = a.n_mats - 1;                          // last matrix whose first_block <= blockIdx.x
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (a.table[mid].first_block <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
    }
    mp = a.table + lo;
  }
  const SmallMat mt = *mp;
  const int strip = blockIdx.x - mt.first_block;
  const int n0 = strip * SM_BN;
  const int N = mt.N, K = mt.K, M = a.M;
  const int ktiles = K >> 6;
  const int band = (n0 >> 6) + wave;                        // band of the sparse layout owned by this wave
  const bool band_ok = band * 64 < N && mt.nnz > 0;
  const int nn = lane & 15, jj = lane >> 4;                 // B operand: column nn of a 16-column subtile, k-group jj
  const int nchunks = (K + SM_KC - 1) / SM_KC;
  const int nkb_total = K >> 7;

  uint32_t magic_lo = 0x64006400u, magic_hi = 0x54005400u;
  asm volatile("" : "+v"(magic_lo), "+v"(magic_hi));

  float2* const my_ysp = ysp + wave * 64 * SM_ROWS;
  float2* const my_winv = winv + wave * SM_WIN;
  uint16_t* const my_winp = winp + wave * SM_WIN;
  for (int i = lane; i < 64 * SM_ROWS; i += 64) my_ysp[i] = make_float2(0.0f, 0.0f);

  float4_t acc[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) acc[s] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

  // rows past N re-read row N-1: their outputs are never used
  const uint8_t* qrow[4];
  const uint16_t* srow[4];
  const int gshift = mt.group_shift;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int n = min(n0 + wave * 64 + 16 * s + nn, N - 1);
    qrow[s] = mt.qweight + (size_t)n * (K >> 1) + 16 * jj;
    srow[s] = mt.scales + (size_t)n * (K >> gshift);
  }

  // entry index at every chunk boundary of this band: lane c holds the boundary before chunk c
  uint32_t tp_chunk = 0;
  if (band_ok) tp_chunk = mt.tile_ptr[(uint32_t)band * (uint32_t)ktiles + (uint32_t)min(lane * (SM_KC / 64), ktiles)];

  // ---- x staging: thread = 16-byte chunk (tid & 63) of rows (tid >> 6) + 4 i ----
  u32x4 xr[4];
  auto load_x = [&](int c) {
    const int kc = c * SM_KC, kcl = min(SM_KC, K - kc);
    const int ch = tid & 63;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = (tid >> 6) + 4 * i;
      xr[i] = u32x4{0u, 0u, 0u, 0u};
      if (m < M && 8 * ch < kcl) xr[i] = *reinterpret_cast<const u32x4*>(mt.x + (size_t)m * K + kc + 8 * ch);
    }
  };
  auto store_x = [&](int buf) {
    const int ch = tid & 63;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = (tid >> 6) + 4 * i;
      u32x4 o;
#pragma unroll
      for (int w = 0; w < 4; ++w) o[w] = sm_stage_x_word(xr[i], w);
      *reinterpret_cast<u32x4*>(xs + (buf * SM_ROWS + m) * SM_XSTRIDE + 8 * ch) = o;
    }
  };

  // ---- code stream: slot h*4+s holds subtile s of an even (h=0) / odd (h=1) 128-column block ----
  u32x4 qbuf[8];
  auto load_q = [&](int slot, int gkb) {
    qbuf[slot] = *reinterpret_cast<const u32x4*>(qrow[slot & 3] + (size_t)min(gkb, nkb_total - 1) * 64);
  };
#pragma unroll
  for (int i = 0; i < 8; ++i) load_q(i, i >> 2);
  load_x(0);
  store_x(0);
  __syncthreads();

  for (int c = 0; c < nchunks; ++c) {
    const int kc = c * SM_KC, kcl = min(SM_KC, K - kc);
    const int nkb = kcl >> 7;                               // 128-column blocks in this chunk (1..4)
    const _Float16* const xc = xs + (c & 1) * SM_ROWS * SM_XSTRIDE;
    if (c + 1 < nchunks) load_x(c + 1);
    // scales of the chunk's four blocks for the lane's four rows (group 128)
    uint16_t sc4[4][4];
    if (G128) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) sc4[s][i] = srow[s][min(4 * c + i, nkb_total - 1)];
    }
    // sparse arrays of this chunk's first window
    const uint32_t j_lo = __builtin_amdgcn_readlane(tp_chunk, c), j_hi = __builtin_amdgcn_readlane(tp_chunk, c + 1);
    const uint32_t w_first = j_lo & ~3u;
    uint32_t pf_idx[4];
    float pf_val[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t je = w_first + 4u * lane + e;
      const bool ok = band_ok && je >= j_lo && je < j_hi;
      pf_idx[e] = ok ? mt.sp_idx[je] : 0u;
      pf_val[e] = ok ? mt.sp_val[je] : 0.0f;
    }

    // ---- dense: stream this band's codes ----
#pragma unroll
    for (int kbl = 0; kbl < 4; ++kbl) {
      if (kbl < nkb) {
        const int h = kbl & 1, gkb = 4 * c + kbl;
        half8_t af[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
          af[t] = *reinterpret_cast<const half8_t*>(xc + nn * SM_XSTRIDE + kbl * 128 + 32 * jj + 8 * t);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const u32x4 q = qbuf[h * 4 + s];
          load_q(h * 4 + s, gkb + 2);                       // reload this slot with the block two ahead
          _Float16 sh;
          if (G128) {
            sh = __builtin_bit_cast(_Float16, sc4[s][kbl]);
          } else {
            sh = __builtin_bit_cast(_Float16, srow[s][(kc + kbl * 128 + 32 * jj) >> gshift]);
          }
          const half2_t s2 = {sh, sh};
          float4_t tmp = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const half8_t b = sm_dequant_word<!G128>(q[t], magic_lo, magic_hi, s2);
            tmp = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[t], b, tmp, 0, 0, 0);
          }
          if (G128) {
            const float sf = (float)sh;                      // column nn of the subtile: the lane's own row of W
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[s][r] = fmaf(tmp[r], sf, acc[s][r]);
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[s][r] += tmp[r];
          }
        }
      }
    }

    // ---- sparse: sensitive entries of this band inside the chunk ----
    if (band_ok) {
      for (uint32_t w0 = w_first; w0 < j_hi; w0 += SM_WIN) {
        // window [w0, w0+256): one Philox counter (4 consecutive entries) per lane
        const uint32_t j = w0 + 4u * lane;
        uint32_t pos[4];
        float val[4], ez[4];
        bool ok[4];
        {
          float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
          if (j < j_hi && a.eps != 0.0f) zbar_quad((mt.nnz_base + j) >> 2, a.seed, a.step, z);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint32_t je = j + e;
            ok[e] = je >= j_lo && je < j_hi;
            uint32_t flat;
            if (w0 == w_first) { flat = pf_idx[e]; val[e] = pf_val[e]; }
            else { flat = ok[e] ? mt.sp_idx[je] : 0u; val[e] = ok[e] ? mt.sp_val[je] : 0.0f; }
            ez[e] = a.eps * z[e];
            const uint32_t n = sm_fast_div(flat, mt.div_mul, mt.div_shift);
            const uint32_t r = n - (uint32_t)(band * 64);
            const uint32_t kk = flat - n * (uint32_t)K - (uint32_t)kc;
            ok[e] = ok[e] && r < 64u && kk < (uint32_t)kcl;           // a malformed layout must not leave the band
            pos[e] = (r << 10) | (kk & 1023u);
          }
        }
        // split into four lists by (row mod 4): list q occupies window slots [start[q], start[q+1])
        uint32_t start[5];
        start[0] = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint32_t base = start[q];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bool mine = ok[e] && ((pos[e] >> 10) & 3u) == (uint32_t)q;
            const uint64_t mask = __ballot(mine);
            const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            if (mine) {
              my_winp[base + before] = (uint16_t)pos[e];
              my_winv[base + before] = make_float2(val[e], ez[e]);
            }
            base += (uint32_t)__popcll(mask);
          }
          start[q + 1] = base;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // lists visible to the whole wave
        // accumulate: lane group q (16 lanes = 16 token rows) walks list q; the four groups never share a row
        const int q = lane >> 4, m = lane & 15;
        const uint32_t my_lo = q == 0 ? start[0] : q == 1 ? start[1] : q == 2 ? start[2] : start[3];
        const uint32_t my_hi = q == 0 ? start[1] : q == 1 ? start[2] : q == 2 ? start[3] : start[4];
        uint32_t longest = 0;
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) longest = max(longest, start[qq + 1] - start[qq]);
        for (uint32_t it = 0; it < longest; ++it) {
          const uint32_t e = my_lo + it;
          if (e < my_hi) {
            const uint32_t p = my_winp[e];
            const float2 v = my_winv[e];
            const float xv = (float)xc[m * SM_XSTRIDE + sm_xpos((int)(p & 1023u))];
            float2* dst = my_ysp + (p >> 10) * SM_ROWS + m;
            float2 y = *dst;
            y.x = fmaf(v.x + v.y, xv, y.x);
            y.y = fmaf(v.x - v.y, xv, y.y);
            *dst = y;
          }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // done with the window before it is refilled
      }
    }

    if (c + 1 < nchunks) store_x((c + 1) & 1);
    __syncthreads();                                        // next chunk's x complete; this chunk's no longer read
  }

  // ---- epilogue: accumulator s, register r = token row 4*jj + r, column 16*s + nn of the band ----
  double lp = 0.0, lm = 0.0;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int nl = 16 * s + nn, n = n0 + wave * 64 + nl;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int m = 4 * jj + r;
      if (m < M && n < N) {
        const float2 sp = my_ysp[nl * SM_ROWS + m];
        const float yp = acc[s][r] + sp.x, ym = acc[s][r] + sp.y;
        if (a.loss_mode) {
          const float t = __uint_as_float((uint32_t)mt.target[(size_t)m * N + n] << 16);
          const float dp = yp - t, dm = ym - t;
          lp += (double)(dp * dp);
          lm += (double)(dm * dm);
        } else {
          mt.y[(size_t)m * N + n] = a.store_sign > 0 ? yp : a.store_sign < 0 ? ym : 0.5f * (yp + ym);
        }
      }
    }
  }
  if (a.loss_mode) {
    __shared__ double red[2][4];
    lp = wave_sum(lp);
    lm = wave_sum(lm);
    if (lane == 0) { red[0][wave] = lp; red[1][wave] = lm; }
    __syncthreads();
    if (tid == 0) {
      const int pi = mt.partial_base + strip;
      a.partial_plus[pi] = ((red[0][0] + red[0][1]) + (red[0][2] + red[0][3])) * mt.loss_scale;
      a.partial_minus[pi] = ((red[1][0] + red[1][1]) + (red[1][2] + red[1][3])) * mt.loss_scale;
    }
  }
}

// Sparse ZO-SGD update of every matrix of a table in one launch (Section 3.4, fixed-parameter
// update rule): thread = one Philox counter = four consecutive entries of one matrix.
__global__ void __launch_bounds__(256) sparse_update_table_kernel(const SmallMat* __restrict__ table, int n_mats,
                                                                  int64_t total_quads, uint64_t seed, uint64_t step,
                                                                  const double* __restrict__ g, float lr) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= total_quads) return;
  int lo = 0, hi = n_mats - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (table[mid].first_quad <= t) lo = mid; else hi = mid - 1;
  }
  const SmallMat& mt = table[lo];
  const int64_t tq = t - mt.first_quad, j0 = 4 * tq;
  if (j0 >= (int64_t)mt.nnz) return;
  const float c = (float)((double)lr * *g);
  float z[4];
  zbar_quad((mt.nnz_base >> 2) + (uint64_t)tq, seed, step, z);
  float* v = mt.sp_val + j0;
  if (j0 + 4 <= (int64_t)mt.nnz) {
    float4 w = *reinterpret_cast<float4*>(v);
    w.x = fmaf(-c, z[0], w.x); w.y = fmaf(-c, z[1], w.y); w.z = fmaf(-c, z[2], w.z); w.w = fmaf(-c, z[3], w.w);
    *reinterpret_cast<float4*>(v) = w;
  } else {
    for (int i = 0; j0 + i < (int64_t)mt.nnz; ++i) v[i] = fmaf(-c, z[i], v[i]);
  }
}

// ---- host side -----------------------------------------------------------------------------

static size_t small_lds_bytes() {
  return (size_t)2 * SM_ROWS * SM_XSTRIDE * 2 + (size_t)4 * 64 * SM_ROWS * 8 + (size_t)4 * SM_WIN * 8 +
         (size_t)4 * SM_WIN * 2;
}

bool small_m_eligible(const szo_linear_desc* d) {
  return d->M >= 1 && d->M <= SM_ROWS && d->N >= 1 && (d->K % 128) == 0 && d->K <= 63 * SM_KC &&
         d->tile_dtype == SZO_TILE_F16;
}

int small_m_blocks(const szo_linear_desc* d) { return (int)((d->N + SM_BN - 1) / SM_BN); }

size_t small_m_table_bytes(int n) { return sizeof(SmallMat) * (size_t)n; }

static void fill_mat(SmallMat& m, const szo_linear_desc* d) {
  m.x = (const uint16_t*)d->x; m.qweight = d->qweight; m.scales = (const uint16_t*)d->scales;
  m.tile_ptr = d->tile_ptr; m.sp_idx = d->sp_idx; m.sp_val = d->sp_val;
  m.target = (const uint16_t*)d->target; m.y = d->y;
  m.nnz_base = d->nnz_base;
  m.loss_scale = 1.0 / ((double)d->M * (double)d->N);
  m.N = (int)d->N; m.K = (int)d->K; m.nnz = (uint32_t)d->nnz;
  int gs = 0;
  while ((1 << gs) < d->group) ++gs;
  m.group_shift = gs;
  int l = 0;
  while ((1ull << l) < (uint64_t)m.K) ++l;
  m.div_mul = (uint32_t)((((1ull << l) - (uint64_t)m.K) << 32) / (uint64_t)m.K + 1ull);
  m.div_shift = l - 1;
  m.first_block = 0; m.partial_base = 0; m.first_quad = 0;
}

static int set_small_attrs() {
  static bool attr_set = false;
  if (!attr_set) {
    SZO_HIP(hipFuncSetAttribute((const void*)small_m_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)small_lds_bytes()));
    SZO_HIP(hipFuncSetAttribute((const void*)small_m_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)small_lds_bytes()));
    attr_set = true;
  }
  return SZO_OK;
}

// One matrix, descriptor passed in the kernel arguments (no device table needed).
int small_m_launch_one(const szo_linear_desc* d, uint64_t seed, uint64_t step, float eps, int sign, bool loss_mode,
                       double* partial_plus, double* partial_minus, hipStream_t stream) {
  const int rc = set_small_attrs();
  if (rc != SZO_OK) return rc;
  SmallArgs a{};
  fill_mat(a.one, d);
  a.table = nullptr; a.n_mats = 1; a.M = (int)d->M;
  a.store_sign = sign; a.loss_mode = loss_mode ? 1 : 0;
  a.seed = seed; a.step = step; a.eps = eps;
  a.partial_plus = partial_plus; a.partial_minus = partial_minus;
  const int blocks = small_m_blocks(d);
  if (d->group == 128) small_m_kernel<true><<<blocks, 256, small_lds_bytes(), stream>>>(a);
  else small_m_kernel<false><<<blocks, 256, small_lds_bytes(), stream>>>(a);
  SZO_LAUNCH_CHECK();
  return SZO_OK;
}

// A whole stack in one launch per group size.  The table is assembled on the host, longest K
// first (their workgroups run longest, so they should start first), copied into `table_dev`
// (device, small_m_table_bytes(n)) with an asynchronous copy on the stream, and also drives one
// grouped sparse update when `do_update` is set.  *total_partials receives the number of partials
// per sign.
int small_m_step(const szo_linear_desc* descs, int n, uint64_t seed, uint64_t step, float eps, float lr,
                 void* table_dev, double* partial_plus, double* scalars, bool do_update, hipStream_t stream) {
  int rc = set_small_attrs();
  if (rc != SZO_OK) return rc;
  // Pinned staging for the table: a ring of four, so that the host may run a few steps ahead of
  // the GPU; a slot is reused only after the copy that read it has executed.
  struct Slot { SmallMat* host; int cap; hipEvent_t copied; bool used; };
  static thread_local Slot ring[4] = {};
  static thread_local unsigned turn = 0;
  Slot& slot = ring[turn++ & 3];
  if (slot.used) SZO_HIP(hipEventSynchronize(slot.copied));
  if (!slot.copied) SZO_HIP(hipEventCreateWithFlags(&slot.copied, hipEventDisableTiming));
  if (n > slot.cap) {
    if (slot.host) (void)hipHostFree(slot.host);
    slot.host = nullptr; slot.cap = 0;
    SZO_HIP(hipHostMalloc((void**)&slot.host, sizeof(SmallMat) * (size_t)n, hipHostMallocDefault));
    slot.cap = n;
  }
  SmallMat* const host = slot.host;
  // order: group-128 matrices first (by K descending), then the others (by K descending)
  int order[4096];
  for (int i = 0; i < n; ++i) order[i] = i;
  for (int i = 1; i < n; ++i) {                       // insertion sort: n is a few hundred
    const int o = order[i];
    const int64_t key = (descs[o].group == 128 ? (int64_t)1 << 40 : 0) + descs[o].K;
    int j = i - 1;
    while (j >= 0) {
      const int64_t kj = (descs[order[j]].group == 128 ? (int64_t)1 << 40 : 0) + descs[order[j]].K;
      if (kj >= key) break;
      order[j + 1] = order[j];
      --j;
    }
    order[j + 1] = o;
  }
  int n128 = 0, blocks128 = 0, blocks_other = 0, partials = 0;
  int64_t quads = 0;
  for (int r = 0; r < n; ++r) {
    const szo_linear_desc* d = &descs[order[r]];
    SmallMat& m = host[r];
    fill_mat(m, d);
    const bool g128 = d->group == 128;
    m.first_block = g128 ? blocks128 : blocks_other;
    m.partial_base = partials;
    m.first_quad = quads;
    const int b = small_m_blocks(d);
    if (g128) { blocks128 += b; ++n128; } else blocks_other += b;
    partials += b;
    quads += ((int64_t)d->nnz + 3) / 4;
  }
  if (2 * (int64_t)partials > kMaxLossPartials) return SZO_EUNSUPPORTED;
  SZO_HIP(hipMemcpyAsync(table_dev, host, sizeof(SmallMat) * (size_t)n, hipMemcpyHostToDevice, stream));
  SZO_HIP(hipEventRecord(slot.copied, stream));
  slot.used = true;
  SmallArgs a{};
  a.M = (int)descs[0].M;
  a.store_sign = 1; a.loss_mode = 1;
  a.seed = seed; a.step = step; a.eps = eps;
  a.partial_plus = partial_plus; a.partial_minus = partial_plus + partials;
  const SmallMat* tdev = (const SmallMat*)table_dev;
  if (blocks128 > 0) {
    a.table = tdev; a.n_mats = n128;
    small_m_kernel<true><<<blocks128, 256, small_lds_bytes(), stream>>>(a);
    SZO_LAUNCH_CHECK();
  }
  if (blocks_other > 0) {
    a.table = tdev + n128; a.n_mats = n - n128;
    small_m_kernel<false><<<blocks_other, 256, small_lds_bytes(), stream>>>(a);
    SZO_LAUNCH_CHECK();
  }
  rc = reduce_step(partial_plus, partials, eps, scalars, stream);
  if (rc != SZO_OK) return rc;
  if (do_update && quads > 0) {
    const int64_t ub = (quads + 255) / 256;
    if (ub > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
    sparse_update_table_kernel<<<(unsigned)ub, 256, 0, stream>>>(tdev, n, quads, seed, step, scalars + 2, lr);
    SZO_LAUNCH_CHECK();
  }
  return SZO_OK;
}

}  // namespace szo
