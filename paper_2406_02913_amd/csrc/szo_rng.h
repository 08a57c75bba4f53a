// Device-side counter-based Gaussian shared by the forward, the update and the debug kernel:
// Philox-4x32-10 keyed on (seed, step, global entry index) followed by Box-Muller.  This is
// the random-seed trick of Section 3.5: the perturbation z_k of Section 3.4 is recomputed
// wherever it is needed and never stored.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace szo {

struct Words4 { uint32_t w0, w1, w2, w3; };

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Words4{c0, c1, c2, c3};
}

// Words of the counter shared by global entries 4*quad .. 4*quad+3.
__device__ __forceinline__ Words4 zbar_words(uint64_t quad, uint64_t seed, uint64_t step) {
  return philox4x32_10((uint32_t)quad, (uint32_t)(quad >> 32), (uint32_t)step, (uint32_t)(step >> 32),
                       (uint32_t)seed, (uint32_t)(seed >> 32));
}

// Two Gaussians from two words: u1 = ((ra>>8)+1) 2^-24 in (0,1], u2 = (rb>>8) 2^-24 in [0,1);
// (rho cos theta, rho sin theta) with rho = sqrt(-2 ln u1), theta = 2 pi u2.
__device__ __forceinline__ void box_muller(uint32_t ra, uint32_t rb, float& zc, float& zs) {
  const float u1 = (float)((ra >> 8) + 1u) * 0x1p-24f;
  const float two_u2 = (float)(rb >> 8) * 0x1p-23f;     // theta / pi, exact
  const float rho = sqrtf(-2.0f * logf(u1));
  float s, c;
  sincospif(two_u2, &s, &c);
  zc = rho * c;
  zs = rho * s;
}

// The four Gaussians of one counter: entries 4*quad + {0,1,2,3}.
__device__ __forceinline__ void zbar_quad(uint64_t quad, uint64_t seed, uint64_t step, float z[4]) {
  const Words4 w = zbar_words(quad, seed, step);
  box_muller(w.w0, w.w1, z[0], z[1]);
  box_muller(w.w2, w.w3, z[2], z[3]);
}

}  // namespace szo
