// Host-side, one-time set-up of the static structures of a layer: synthetic mask
// positions, the tile-ordered sparse layout, and the sparse/dense split followed by
// 4-bit group quantisation of the dense part (Section 3.4, first equation; Section 3.5).
// No GPU is touched here.
#include "szo.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <numeric>
#include <thread>
#include <vector>

namespace {

inline void philox_round(uint32_t c[4], uint32_t k0, uint32_t k1) {
  const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
  const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
  const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
  const uint32_t n1 = (uint32_t)p1;
  const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
  const uint32_t n3 = (uint32_t)p0;
  c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

inline void philox10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c[4] = {ctr[0], ctr[1], ctr[2], ctr[3]};
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    philox_round(c, k0, k1);
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  std::memcpy(out, c, sizeof(c));
}

// Draw d of a stream: 64 bits from the first two words, reduced modulo `range`.
inline uint64_t draw(uint64_t mask_seed, uint32_t stream, uint64_t d, uint64_t range) {
  const uint32_t ctr[4] = {(uint32_t)d, (uint32_t)(d >> 32), stream, 0u};
  const uint32_t key[2] = {(uint32_t)mask_seed, (uint32_t)(mask_seed >> 32)};
  uint32_t r[4];
  philox10(ctr, key, r);
  return (((uint64_t)r[0] << 32) | r[1]) % range;
}

struct Bitmap {
  std::vector<uint64_t> w;
  explicit Bitmap(uint64_t n) : w((n + 63) / 64, 0) {}
  bool test_and_set(uint64_t i) {
    uint64_t& word = w[i >> 6];
    const uint64_t bit = 1ull << (i & 63);
    const bool was = word & bit;
    word |= bit;
    return was;
  }
};

// fp32 -> fp16 bit pattern, round to nearest even, subnormals kept, overflow -> inf.
inline uint16_t f32_to_f16_bits(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  const uint32_t absu = u & 0x7FFFFFFFu;
  if (absu >= 0x7F800000u) return (uint16_t)(sign | (absu > 0x7F800000u ? 0x7E00u : 0x7C00u));
  if (absu >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);         // rounds to >= 65520 -> inf
  if (absu < 0x33000001u) return sign;                                 // <= 2^-25 -> 0 (tie to even)
  const int e = (int)(absu >> 23) - 127;                               // unbiased exponent
  uint32_t mant = (absu & 0x7FFFFFu) | 0x800000u;                      // 24-bit significand
  int shift;                                                           // bits to drop
  uint32_t base;
  if (e >= -14) { shift = 13; base = (uint32_t)(e + 15) << 10; mant &= 0x7FFFFFu; }
  else          { shift = 13 + (-14 - e); base = 0; }
  const uint32_t kept = mant >> shift;
  const uint32_t rem = mant & ((1u << shift) - 1u);
  const uint32_t half = 1u << (shift - 1);
  uint32_t h = base + kept;                                            // carries propagate into the exponent
  if (rem > half || (rem == half && (kept & 1u))) ++h;
  return (uint16_t)(sign | h);
}

inline float f16_bits_to_f32(uint16_t h) {
  const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  const uint32_t e = (h >> 10) & 0x1Fu, m = h & 0x3FFu;
  float v;
  if (e == 0) v = std::ldexp((float)m, -24);
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = std::ldexp((float)(m | 0x400u), (int)e - 25);
  uint32_t u;
  std::memcpy(&u, &v, 4);
  u |= sign;
  std::memcpy(&v, &u, 4);
  return v;
}

inline int64_t tile_of(int64_t n, int64_t k, int64_t ktiles) {
  return (n / SZO_TILE_ROWS) * ktiles + k / SZO_TILE_COLS;
}

template <class F>
void parallel_rows(int64_t rows, int64_t work_per_row, F&& body) {
  unsigned hw = std::thread::hardware_concurrency();
  int64_t nt = std::min<int64_t>(hw ? hw : 1, 16);
  if (rows * work_per_row < (1 << 20)) nt = 1;
  nt = std::max<int64_t>(1, std::min(nt, rows));
  if (nt == 1) { body(0, rows); return; }
  std::vector<std::thread> th;
  const int64_t chunk = (rows + nt - 1) / nt;
  for (int64_t t = 0; t < nt; ++t) {
    const int64_t lo = t * chunk, hi = std::min(rows, lo + chunk);
    if (lo < hi) th.emplace_back([=, &body] { body(lo, hi); });
  }
  for (auto& t : th) t.join();
}

}  // namespace

extern "C" {

int szo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  if (!ctr || !key || !out) return SZO_EINVAL;
  philox10(ctr, key, out);
  return SZO_OK;
}

int64_t szo_num_tiles(int64_t N, int64_t K) {
  if (N < 0 || K < 0 || K % SZO_TILE_COLS) return 0;
  return ((N + SZO_TILE_ROWS - 1) / SZO_TILE_ROWS) * (K / SZO_TILE_COLS);
}

int szo_mask_generate(int64_t N, int64_t K, int64_t nnz, int kind, uint64_t mask_seed,
                      uint32_t* flat_out) {
  if (N <= 0 || K <= 0 || nnz < 0 || (nnz > 0 && !flat_out)) return SZO_EINVAL;
  if ((uint64_t)N * (uint64_t)K > 0xFFFFFFFFull) return SZO_EUNSUPPORTED;
  const uint64_t total = (uint64_t)N * (uint64_t)K;
  if ((uint64_t)nnz > total) return SZO_EINVAL;
  if (kind != 0 && kind != 1) return SZO_EINVAL;
  Bitmap taken(total);
  int64_t have = 0;
  if (kind == 1) {
    const int64_t H = (N + 99) / 100;
    const int64_t n_hot = nnz / 2;
    if ((uint64_t)n_hot > (uint64_t)H * (uint64_t)K) return SZO_EINVAL;
    std::vector<uint32_t> hot;
    {
      Bitmap rows((uint64_t)N);
      for (uint64_t d = 0; (int64_t)hot.size() < H; ++d) {
        const uint64_t r = draw(mask_seed, 1u, d, (uint64_t)N);
        if (!rows.test_and_set(r)) hot.push_back((uint32_t)r);
      }
      std::sort(hot.begin(), hot.end());
    }
    Bitmap inside((uint64_t)H * (uint64_t)K);
    for (uint64_t d = 0; have < n_hot; ++d) {
      const uint64_t v = draw(mask_seed, 2u, d, (uint64_t)H * (uint64_t)K);
      if (inside.test_and_set(v)) continue;
      const uint64_t flat = (uint64_t)hot[v / (uint64_t)K] * (uint64_t)K + v % (uint64_t)K;
      taken.test_and_set(flat);
      flat_out[have++] = (uint32_t)flat;
    }
  }
  const uint32_t stream = kind == 1 ? 3u : 0u;
  for (uint64_t d = 0; have < nnz; ++d) {
    const uint64_t v = draw(mask_seed, stream, d, total);
    if (!taken.test_and_set(v)) flat_out[have++] = (uint32_t)v;
  }
  std::sort(flat_out, flat_out + nnz);
  return SZO_OK;
}

int szo_tcsr_build(int64_t N, int64_t K, const uint32_t* flat_sorted, int64_t nnz,
                   uint32_t* tile_ptr_out, uint32_t* sp_idx_out, uint32_t* perm_out) {
  if (N <= 0 || K <= 0 || nnz < 0 || !tile_ptr_out) return SZO_EINVAL;
  if (nnz > 0 && (!flat_sorted || !sp_idx_out)) return SZO_EINVAL;
  if (K % SZO_TILE_COLS) return SZO_EUNSUPPORTED;
  if ((uint64_t)N * (uint64_t)K > 0xFFFFFFFFull) return SZO_EUNSUPPORTED;
  const uint64_t total = (uint64_t)N * (uint64_t)K;
  for (int64_t j = 0; j < nnz; ++j) {
    if (flat_sorted[j] >= total) return SZO_EINVAL;
    if (j && flat_sorted[j] <= flat_sorted[j - 1]) return SZO_EINVAL;
  }
  const int64_t ktiles = K / SZO_TILE_COLS;
  const int64_t ntiles = szo_num_tiles(N, K);
  std::vector<uint64_t> keyed((size_t)nnz);   // (tile, inner) packed above the source position
  std::vector<uint32_t> order((size_t)nnz);
  std::iota(order.begin(), order.end(), 0u);
  for (int64_t j = 0; j < nnz; ++j) {
    const int64_t n = flat_sorted[j] / K, k = flat_sorted[j] % K;
    const uint64_t inner = (uint64_t)((n % SZO_TILE_ROWS) * SZO_TILE_COLS + k % SZO_TILE_COLS);
    keyed[(size_t)j] = ((uint64_t)tile_of(n, k, ktiles) << 12) | inner;   // inner < 4096
  }
  std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return keyed[a] < keyed[b]; });
  std::fill(tile_ptr_out, tile_ptr_out + ntiles + 1, 0u);
  for (int64_t j = 0; j < nnz; ++j) {
    const uint32_t src = order[(size_t)j];
    sp_idx_out[j] = flat_sorted[src];
    if (perm_out) perm_out[j] = src;
    tile_ptr_out[(keyed[src] >> 12) + 1] += 1u;
  }
  for (int64_t t = 0; t < ntiles; ++t) tile_ptr_out[t + 1] += tile_ptr_out[t];
  return SZO_OK;
}

int szo_quantize_pack(const float* W, int64_t N, int64_t K, int group, const uint32_t* mask_flat,
                      int64_t nnz, uint8_t* q_out, uint16_t* scales_out, float* sp_val_out) {
  if (!W || !q_out || !scales_out || N <= 0 || K <= 0 || group <= 0 || nnz < 0) return SZO_EINVAL;
  if (nnz > 0 && (!mask_flat || !sp_val_out)) return SZO_EINVAL;
  if (K % group || (group & 1)) return SZO_EINVAL;
  if ((uint64_t)N * (uint64_t)K > 0xFFFFFFFFull) return SZO_EUNSUPPORTED;
  const uint64_t total = (uint64_t)N * (uint64_t)K;
  // bucket the mask by row so that every row can be handled independently
  std::vector<uint32_t> row_start((size_t)N + 1, 0u);
  for (int64_t j = 0; j < nnz; ++j) {
    if (mask_flat[j] >= total) return SZO_EINVAL;
    sp_val_out[j] = W[mask_flat[j]];
    row_start[mask_flat[j] / (uint64_t)K + 1] += 1u;
  }
  for (int64_t n = 0; n < N; ++n) row_start[(size_t)n + 1] += row_start[(size_t)n];
  std::vector<uint32_t> cols((size_t)nnz);
  {
    std::vector<uint32_t> fill(row_start.begin(), row_start.end() - 1);
    for (int64_t j = 0; j < nnz; ++j) cols[fill[mask_flat[j] / (uint64_t)K]++] = (uint32_t)(mask_flat[j] % (uint64_t)K);
  }
  const int64_t groups = K / group;
  std::atomic<int> bad{0};          // set by any worker thread
  parallel_rows(N, K, [&](int64_t lo, int64_t hi) {
    std::vector<float> row((size_t)K);
    for (int64_t n = lo; n < hi; ++n) {
      std::memcpy(row.data(), W + n * K, sizeof(float) * (size_t)K);
      for (uint32_t p = row_start[(size_t)n]; p < row_start[(size_t)n + 1]; ++p) row[cols[p]] = 0.0f;
      for (int64_t g = 0; g < groups; ++g) {
        const float* w = row.data() + g * group;
        float mx = 0.0f;
        for (int i = 0; i < group; ++i) mx = std::max(mx, std::fabs(w[i]));
        const uint16_t sb = f32_to_f16_bits(mx / 7.0f);
        if ((sb & 0x7C00u) == 0x7C00u) bad.store(1, std::memory_order_relaxed);              // inf / nan scale
        scales_out[n * groups + g] = sb;
        const float s = f16_bits_to_f32(sb);
        uint8_t* q = q_out + (n * K + g * group) / 2;
        for (int i = 0; i < group; i += 2) {
          int c[2];
          for (int h = 0; h < 2; ++h) {
            float r = (s == 0.0f) ? 0.0f : std::nearbyintf(w[i + h] / s);   // ties to even
            r = std::min(7.0f, std::max(-8.0f, r));
            c[h] = (int)r + 8;
          }
          q[i / 2] = (uint8_t)(c[0] | (c[1] << 4));
        }
      }
    }
  });
  return bad.load() ? SZO_EINVAL : SZO_OK;
}

int szo_quantize_pack_lut(const float* W, int64_t N, int64_t K, const uint32_t* mask_flat, int64_t nnz,
                          uint8_t* q_out, uint16_t* lut_out, float* sp_val_out) {
  if (!W || !q_out || !lut_out || N <= 0 || K <= 0 || nnz < 0) return SZO_EINVAL;
  if (nnz > 0 && (!mask_flat || !sp_val_out)) return SZO_EINVAL;
  if (K % 32) return SZO_EINVAL;
  if ((uint64_t)N * (uint64_t)K > 0xFFFFFFFFull) return SZO_EUNSUPPORTED;
  const uint64_t total = (uint64_t)N * (uint64_t)K;
  std::vector<uint32_t> row_start((size_t)N + 1, 0u);
  for (int64_t j = 0; j < nnz; ++j) {
    if (mask_flat[j] >= total) return SZO_EINVAL;
    sp_val_out[j] = W[mask_flat[j]];
    row_start[mask_flat[j] / (uint64_t)K + 1] += 1u;
  }
  for (int64_t n = 0; n < N; ++n) row_start[(size_t)n + 1] += row_start[(size_t)n];
  std::vector<uint32_t> cols((size_t)nnz);
  {
    std::vector<uint32_t> fill(row_start.begin(), row_start.end() - 1);
    for (int64_t j = 0; j < nnz; ++j) cols[fill[mask_flat[j] / (uint64_t)K]++] = (uint32_t)(mask_flat[j] % (uint64_t)K);
  }
  std::atomic<int> bad{0};          // set by any worker thread
  parallel_rows(N, 8 * K, [&](int64_t lo, int64_t hi) {
    std::vector<float> row((size_t)K), sorted((size_t)K);
    for (int64_t n = lo; n < hi; ++n) {
      std::memcpy(row.data(), W + n * K, sizeof(float) * (size_t)K);
      for (uint32_t p = row_start[(size_t)n]; p < row_start[(size_t)n + 1]; ++p) row[cols[p]] = 0.0f;
      sorted = row;
      std::sort(sorted.begin(), sorted.end());
      double centroid[16];
      for (int c = 0; c < 16; ++c) {
        const uint16_t b = f32_to_f16_bits(sorted[(size_t)((2 * c + 1) * (K / 32))]);
        if ((b & 0x7C00u) == 0x7C00u) bad.store(1, std::memory_order_relaxed);
        lut_out[n * 16 + c] = b;
        centroid[c] = (double)f16_bits_to_f32(b);
      }
      uint8_t* q = q_out + n * (K / 2);
      for (int64_t k = 0; k < K; k += 2) {
        int code[2];
        for (int h = 0; h < 2; ++h) {
          const double w = (double)row[(size_t)(k + h)];
          int best = 0;
          double bd = std::fabs(w - centroid[0]);
          for (int c = 1; c < 16; ++c) {
            const double d = std::fabs(w - centroid[c]);
            if (d < bd) { bd = d; best = c; }                 // strict: ties keep the lower index
          }
          code[h] = best;
        }
        q[k / 2] = (uint8_t)(code[0] | (code[1] << 4));
      }
    }
  });
  return bad.load() ? SZO_EINVAL : SZO_OK;
}

int szo_choose_tile_dtype(float x_absmax) {
  if (!(x_absmax >= 0.0f)) return SZO_EINVAL;                   // negative or NaN
  return x_absmax <= 65504.0f ? SZO_TILE_F16 : SZO_TILE_BF16;   // largest finite fp16
}

size_t szo_qweight_bytes(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0 || K % 64) return 0;
  return (size_t)((N + 63) / 64) * 64 * (size_t)(K / 2);
}

size_t szo_scales_count(int64_t N, int64_t K, int group) {
  if (N <= 0 || K <= 0 || group <= 0 || K % group) return 0;
  return (size_t)((N + 63) / 64) * 64 * (size_t)(K / group);
}

int szo_layout_weights(const uint8_t* q, const uint16_t* scales, int64_t N, int64_t K, int group,
                       uint8_t* q_banded, uint16_t* scales_banded) {
  if (!q || !q_banded || N <= 0 || K <= 0) return SZO_EINVAL;
  if ((scales == nullptr) != (scales_banded == nullptr)) return SZO_EINVAL;
  if (K % 64 || (scales && (group <= 0 || K % group))) return SZO_EINVAL;
  const int64_t bands = (N + 63) / 64, ktiles = K / 64, groups = scales ? K / group : 0;
  parallel_rows(bands, 64 * K, [&](int64_t lo, int64_t hi) {
    for (int64_t b = lo; b < hi; ++b) {
      for (int64_t t = 0; t < ktiles; ++t) {
        uint8_t* dst = q_banded + (b * ktiles + t) * 64 * 32;
        for (int64_t r = 0; r < 64; ++r) {
          const int64_t n = b * 64 + r;
          if (n < N) std::memcpy(dst + r * 32, q + n * (K / 2) + t * 32, 32);
          else std::memset(dst + r * 32, 0x88, 32);            // code 8 twice: weight zero
        }
      }
      for (int64_t g = 0; g < groups; ++g) {
        uint16_t* dst = scales_banded + (b * groups + g) * 64;
        for (int64_t r = 0; r < 64; ++r) {
          const int64_t n = b * 64 + r;
          dst[(r % 16) * 4 + r / 16] = n < N ? scales[n * groups + g] : (uint16_t)0;
        }
      }
    }
  });
  return SZO_OK;
}

}  // extern "C"
