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
#include <algorithm>
#include <cstddef>
#include <vector>
#include "szo_internal.h"
#include "szo_rng.h"
#include <mutex>
#include <type_traits>

// Loss partials of szo_zo_step_noalloc: one fp64 value per workgroup and sign, written by the forward
// kernels and summed by reduce_step_kernel.  Lives in the code object, one copy per GPU, for callers
// that cannot allocate a workspace.  Host code never uses this name as an address: it asks the runtime
// for the array's device address once per device (noalloc_partials below).
constexpr int kNoAllocMaxPartials = 1 << 17;                 // 1 MiB per GPU
static __device__ __align__(256) double scratch[kNoAllocMaxPartials];

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
  double* partials;         // fused loss: one scaled partial per workgroup, [grid_m*grid_n]
  double loss_scale;
  int first_block;          // grouped launch: id of this entry's first workgroup (a multiple of 8)
  int pad_;
  const uint16_t* lut;      // fp16 [N,16], table format only
  // grouped launch: one entry runs BOTH forwards of its matrix; the fields above describe the +eps one
  const uint16_t* x_minus;  // activations of the -eps forward (= x unless the layer has a second set)
  double* partials_minus;   // loss partials of the -eps forward
};

// floor(v / d) for 32-bit v with a precomputed multiplier (Granlund-Montgomery, round-up form).
__device__ __forceinline__ uint32_t fast_div(uint32_t v, uint32_t mul, int shift) {
  const uint32_t t = __umulhi(mul, v);
  return (t + ((v - t) >> 1)) >> shift;
}

// Position of column kk (0..63) of tile row r inside the LDS tile, in 16-bit elements.
// Rows are 64 elements (128 bytes), so two rows span the 64 four-byte banks; the eight
// 16-byte chunks of a row are XOR-swizzled with row_swizzle(row), chosen for both ways the tile is
// accessed with 16 bytes per lane.  Reads are served 16 lanes (256 bytes) per cycle: 16 lanes reading the
// same chunk of 16 consecutive rows must touch every bank exactly once, which (row / 2) mod 8 gives.
// Writes are served 8 lanes (128 bytes) per cycle and conflict when two of them fall into the same 16 bytes
// modulo 128, whatever the row's parity (measured: a weight wave writing one chunk of 64 consecutive rows
// took 16 cycles instead of 8 with the (row / 2) swizzle alone, 15 % of all LDS cycles of the kernel);
// the extra (row & 1) * 4 makes 8 consecutive rows distinct as well, and keeps the read property.
// In f16 mode the eight elements of a chunk are stored in the order
// 0,4,1,5,2,6,3,7 -- the order in which two nibbles per 16-bit lane fall out of a packed
// word -- and the activations are stored in the same order, which leaves the dot product
// unchanged.
__device__ __forceinline__ int row_swizzle(int r) { return ((r >> 1) & 7) ^ ((r & 1) << 2); }

template <int DT>
__device__ __forceinline__ int lds_pos(int r, int kk) {
  const int chunk = kk >> 3, w = kk & 7;
  const int p = (DT == SZO_TILE_F16) ? (((w & 3) << 1) | (w >> 2)) : w;
  return r * BK + (((chunk ^ row_swizzle(r)) << 3) | p);
}

__device__ __forceinline__ int chunk_off(int r, int chunk) {   // in 16-bit elements
  return r * BK + ((chunk ^ row_swizzle(r)) << 3);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- activations: word w (0..3) of the staged form of one 16-byte chunk of 8 bf16 --------------
// f16 mode pairs elements (0,4) (1,5) (2,6) (3,7); bf16 -> fp32 is a shift and fp32 -> fp16 is
// exact for |x| in [2^-14, 65504] (8-bit significand).
template <int DT>
__device__ __forceinline__ uint32_t stage_x_word(u32x4 u, int w) {
  if (DT == SZO_TILE_BF16) return u[w];
  const uint32_t first = (w < 2) ? u[0] : u[1], second = (w < 2) ? u[2] : u[3];
  float a, b;
  if ((w & 1) == 0) { a = __uint_as_float(first << 16); b = __uint_as_float(second << 16); }
  else              { a = __uint_as_float(first & 0xFFFF0000u); b = __uint_as_float(second & 0xFFFF0000u); }
  auto h = __builtin_amdgcn_cvt_pkrtz(a, b);
  return __builtin_bit_cast(uint32_t, h);
}

// ---- weights: word w (0..3) of the 8 dequantised elements of one 32-bit word of codes ----------
// dq = (code - 8) * scale, one rounding to the tile type.  f16 mode: a nibble in mantissa bits
// 0..3 under exponent pattern 0x6400 reads 1024 + code, one in bits 4..7 under 0x5400 reads
// 64 + code; removing the offset is exact and the product with the fp16 scale is rounded once,
// which is the rounding of the exact (code-8)*scale.  Output pairs are codes (0,4) (1,5) (2,6) (3,7).
// (a & mask) | bits in one VALU instruction, `bits` in a VGPR.  Inline assembly keeps the instruction in
// the slot it is written in (as plain C the tiled step measured 1 % slower).  The compiler's hazard
// handling cannot see into it, which is safe here and only here: the result feeds packed-half arithmetic
// and an LDS store, never a matrix instruction, whose operands all come from LDS reads
// (tests/test_isa_hazards.py checks the generated code for exactly that).
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t bits_vgpr) {
  uint32_t r;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(bits_vgpr));
  return r;
}

struct DequantConsts { uint32_t magic_lo, magic_hi; };   // 0x64006400 and 0x54005400 held in VGPRs

template <int DT>
__device__ __forceinline__ uint32_t dequant_out(uint32_t q, int w, float scale_f32, half2_t scale_h2,
                                                const DequantConsts& k) {
  if (DT == SZO_TILE_F16) {
    const uint32_t src = (w < 2) ? q : (q >> 8);
    half2_t h;
    if ((w & 1) == 0) {
      h = __builtin_bit_cast(half2_t, and_or(src, 0x000F000Fu, k.magic_lo));
      const half2_t off = {(_Float16)1032.0f, (_Float16)1032.0f};
      h = (h - off) * scale_h2;
    } else {
      h = __builtin_bit_cast(half2_t, and_or(src, 0x00F000F0u, k.magic_hi));
      const half2_t off = {(_Float16)72.0f, (_Float16)72.0f};
      h = (h - off) * scale_h2;
    }
    return __builtin_bit_cast(uint32_t, h);
  } else {
    const float m8s = -8.0f * scale_f32;
    float2_t f = {fmaf((float)((q >> (8 * w)) & 15u), scale_f32, m8s),          // exact in fp32
                  fmaf((float)((q >> (8 * w + 4)) & 15u), scale_f32, m8s)};
    bf16x2_t b = __builtin_convertvector(f, bf16x2_t);                            // round to nearest even
    return __builtin_bit_cast(uint32_t, b);
  }
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
//
// Schedule of one K step of one wave.  The wave issues SLOTS = 4*WMB*WNB MFMAs.  Its staging
// work for the NEXT tile (8 units per lane: 16-byte chunks of x, or 32-bit words of codes) is
// cut into SLOTS slices of three to four VALU instructions, and one slice is issued behind
// each MFMA, where it executes in the shadow of the matrix pipeline.  The LDS reads of the
// next k-step's operands are issued the same way, one behind each of the first MFMAs of a
// k-step, into a second set of operand registers.  A scheduling fence after every slot keeps
// the compiler from regrouping the slots.  Global loads are in place: as soon as a unit's
// registers have been consumed they are reloaded with the same unit of the tile after next,
// which gives every load one full K step (about a microsecond) to arrive.
// Workgroup id -> output tile.  Workgroup ids go round-robin over the 8 XCDs, each with its own L2, so
// ids with equal (id % 8) are first made consecutive ("logical" id): the workgroups resident on one XCD
// at a time (32 with the 256x256 tile) are then a run of consecutive logical ids, and logical ids walk
// the tile grid in strips of `strip` row blocks, so that run covers strip x (32 / strip) tiles which
// share `strip` activation strips and 32 / strip weight strips through that L2.  `count` ids in all;
// `bid`'s residue mod 8 is its XCD both in a launch of its own and in a grouped launch (entries start
// at multiples of 8).
__device__ __forceinline__ int logical_block(int bid, int count) {
  const int q = count >> 3, r = count & 7;
  const int xcd = bid & 7, idx = bid >> 3;
  return xcd * q + min(xcd, r) + idx;
}
__device__ __forceinline__ void tile_of_logical(int L, int grid_m, int grid_n, int strip, int& bm, int& bn) {
  const int width = strip * grid_n, g = L / width, first_m = strip * g;
  const int gsize = min(grid_m - first_m, strip), rem = L - g * width;
  bm = first_m + rem % gsize;
  bn = rem / gsize;
}

// DUAL (grouped launch of a step, loss fused, both forwards read the same activations): the workgroup
// computes BOTH forwards of a tile of BM x BN/2 outputs.  Rows [0, BN/2) of the weight tile in LDS hold
// W + eps z, rows [BN/2, BN) the same rows of W with W - eps z: the codes are loaded and dequantised once
// and written twice, the two copies differ only at the sensitive entries.  Waves of the first half of a
// wave row compute the +eps forward, the others the -eps forward; every MFMA of both forwards is
// executed, only the staging of the weights is shared.  The MFMA loop is the same as without DUAL.
template <int WAVES_M, int WAVES_N, int WMB, int WNB, int DT, bool FUSE_LOSS, int FMT, bool DUAL = false>
__device__ __forceinline__ void linear_fwd_body(const FwdParams& p, const int bm, const int bn,
                                                const uint32_t __attribute__((address_space(4)))* entry = nullptr) {
  constexpr int NWAVES = WAVES_M * WAVES_N;
  constexpr int BM = 32 * WMB * WAVES_M, BN = 32 * WNB * WAVES_N;
  constexpr int TN = DUAL ? BN / 2 : BN;           // output columns of the tile
  static_assert(!DUAL || (FUSE_LOSS && FMT == SZO_FORMAT_UNIFORM && BN == 256), "dual-sign tiles: fused loss, uniform format, 256 rows");
  constexpr int W_WAVES = BN / 64;                 // one per 64-row band of the weight tile
  constexpr int X_WAVES = NWAVES - W_WAVES;
  static_assert(BN % 64 == 0 && X_WAVES > 0, "need whole bands and at least one activation wave");
  constexpr int X_ROWS_PER_PASS = 8 * X_WAVES;     // 8 lanes cover one 128-byte row of x
  static_assert(BM == 8 * X_ROWS_PER_PASS, "every activation lane stages 8 chunks per tile");
  constexpr int MPK = WMB * WNB;                   // MFMAs per k-step
  constexpr int SLOTS = 4 * MPK;                   // MFMAs per K step
  static_assert(SLOTS % 8 == 0 && SLOTS <= 32, "8 staging units must spread evenly over the slots");
  constexpr int SPU = SLOTS / 8;                   // slots per activation staging unit: 1, 2 or 4
  constexpr int WPS = 4 / SPU;                     // output words produced per slot
  // Weight waves of the 32-slot schedule finish their dense staging in the first 24 slots (3 per
  // unit) and spend the last 8 on the sensitive entries of the tile, so that the dependent LDS
  // round trips of the scatter also run in the shadow of MFMAs instead of after them.
  constexpr bool SCATTER_IN_SLOTS = (SLOTS == 32);
  constexpr int DSPU = SCATTER_IN_SLOTS ? 3 : SPU; // slots per weight staging unit
  static_assert(WMB + WNB <= MPK, "operand reads of the next k-step must fit behind this one's MFMAs");
  typedef typename Frag<DT>::type frag_t;

  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* const ldsA = lds;                                   // [2][BM*BK]
  uint16_t* const ldsB = lds + 2 * BM * BK;                     // [2][BN*BK]
  float* const winVal = reinterpret_cast<float*>(lds + 2 * (BM + BN) * BK);        // [W_WAVES][kWindow]
  uint16_t* const winPos = reinterpret_cast<uint16_t*>(winVal + W_WAVES * kWindow);  // [W_WAVES][kWindow]
  uint16_t* const sink16 = winPos + W_WAVES * kWindow;                              // [W_WAVES][64] write sink of idle lanes

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int m0 = bm * BM, n0 = bn * TN;
  const int nk = p.ktiles;
  // Fields that are only needed now and then (a window refill every ~64 K steps, the loss epilogue) are read
  // again from the table entry where they are used instead of occupying scalar registers for the whole
  // tile; the pointer is laundered so that the loads stay where they are written.  Only with dual-sign
  // tiles: otherwise the grouped launch has changed `p` for the -eps forward.
  auto cold = [&]() -> FwdParams {
    if (!DUAL || entry == nullptr) return p;
    constexpr int W = (int)(sizeof(FwdParams) / 4);
    const uint32_t __attribute__((address_space(4)))* e = entry;
    asm volatile("" : "+s"(e));
    struct Words { uint32_t w[W]; } raw;
#pragma unroll
    for (int i = 0; i < W; ++i) raw.w[i] = e[i];
    return __builtin_bit_cast(FwdParams, raw);
  };

  float16_t acc[WMB][WNB];
#pragma unroll
  for (int i = 0; i < WMB; ++i)
#pragma unroll
    for (int j = 0; j < WNB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // Operand t of k-step ks in buffer buf: t < WNB is the B (weight) operand of MFMA column
  // block t, otherwise the A (activation) operand of row block t - WNB.  B operands come first
  // because the first MFMAs of a k-step need all of them but only the first A operand.
  const int fragA_row = wm * 32 * WMB + (lane & 31), fragB_row = wn * 32 * WNB + (lane & 31);
  auto read_operand = [&](int buf, int ks, int t) -> frag_t {
    const int chunk = 2 * ks + (lane >> 5);
    if (t < WNB) return *reinterpret_cast<const frag_t*>(ldsB + buf * BN * BK + chunk_off(fragB_row + 32 * t, chunk));
    return *reinterpret_cast<const frag_t*>(ldsA + buf * BM * BK + chunk_off(fragA_row + 32 * (t - WNB), chunk));
  };

  // All MFMAs of one K step on buffer buf, with slice(s) issued behind MFMA s.
  auto run_tile = [&](int buf, auto&& slice) {
    frag_t op[2][WMB + WNB];
#pragma unroll
    for (int t = 0; t < WMB + WNB; ++t) op[0][t] = read_operand(buf, 0, t);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
      for (int t = 0; t < MPK; ++t) {
        const int i = t / WNB, j = t % WNB;
        acc[i][j] = Frag<DT>::mfma(op[ks & 1][WNB + i], op[ks & 1][j], acc[i][j]);
        if (ks < 3 && t < WMB + WNB) op[(ks + 1) & 1][t] = read_operand(buf, ks + 1, t);
        slice(ks * MPK + t);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  if (DUAL && wave >= W_WAVES / 2 && wave < W_WAVES) {
    // ============ DUAL: the bands of these waves are the -eps copies, written by waves 0 .. W_WAVES/2-1 ====
    auto nothing = [](int) {};
    for (int kt = 0; kt < nk; kt += 2) {
      __syncthreads();
      run_tile(0, nothing);
      if (kt + 1 < nk) {
        __syncthreads();
        run_tile(1, nothing);
      }
    }
  } else if (wave < W_WAVES) {
    // =============================== weight wave ===============================================
    // Lane l stages row l of the band: all 64 columns of a tile, as two halves i = 0, 1 of 32 columns
    // (16 bytes of codes, one scale each).  A wave-wide write of one chunk then touches 64 consecutive rows
    // at the same logical chunk -- the access pattern of the operand reads, which the swizzle makes
    // conflict-free (with two lanes per row the writes measured two-way bank conflicts).
    const int wr = wave * 64 + lane;                             // tile row
    const int band = n0 / 64 + wave;                             // band of the sparse layout
    const bool band_ok = band < p.bands;
    const uint32_t tp_base = (uint32_t)band * (uint32_t)nk;
    uint32_t tile_lo = 0, band_end = 0;                          // entry range bookkeeping (uniform)
    uint32_t tp_reg = 0;                                         // lane l: tile_ptr[tp_base + 64*c + 1 + l]
    uint32_t t_lo = 0, t_end = 0;
    if (band_ok) {
      // Three independent loads and (below, after the first codes have been requested too) one wait: the
      // tile's first K step cannot start before the band's first entries are known, so every memory
      // round trip here is dead time for the whole workgroup.
      t_lo = p.tile_ptr[tp_base];
      t_end = p.tile_ptr[tp_base + nk];
      tp_reg = p.tile_ptr[min(tp_base + 1u + (uint32_t)lane, tp_base + (uint32_t)nk)];
    }
    uint32_t win_lo = 0, win_hi = 0;                             // entries [win_lo, win_hi) are in the window
    float* const wv = winVal + wave * kWindow;
    float* const wv_minus = winVal + (wave + W_WAVES / 2) * kWindow;   // DUAL: value for the -eps copy (the idle waves' space)
    uint16_t* const wp = winPos + wave * kWindow;
    constexpr int kMinusCopy = (BN / 2) * BK;                    // DUAL: offset of the -eps copy of a tile position (128 rows:
                                                                 // the swizzle, a function of row mod 16, is the same there)

    // Banded layout: the 64 rows of this wave's band, one 64-column tile, are 2 KB in a row, so the two
    // load instructions of the wave (64 rows x 16 bytes each) cover it without gaps.  Bands past N re-read the
    // last band (their outputs are never stored) and column tiles past the end re-read the last
    // tile (never consumed): the loads stay unconditional and in order.
    const uint8_t* qrow[2];
    const uint16_t* srow[2];
    {
      const size_t bsafe = (size_t)min(band, p.bands - 1);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int r = lane;                                        // row inside the band
        qrow[i] = p.qweight + (bsafe * (size_t)nk * 64 + (size_t)r) * 32 + 16 * i;
        srow[i] = p.scales + bsafe * (size_t)(p.K >> p.group_shift) * 64 + (size_t)((r & 15) * 4 + (r >> 4));
      }
    }
    u32x4 qreg[2];
    uint16_t sreg[2];
    DequantConsts dqk;
    dqk.magic_lo = 0x64006400u; dqk.magic_hi = 0x54005400u;
    asm volatile("" : "+v"(dqk.magic_lo), "+v"(dqk.magic_hi));   // keep them in registers, not as literals
    auto load_q = [&](int kt, int i) {
      qreg[i] = *reinterpret_cast<const u32x4*>(qrow[i] + (size_t)min(kt, nk - 1) * (64 * BK / 2));
    };
    auto load_s = [&](int kt, int i) {
      sreg[i] = srow[i][(size_t)((min(kt, nk - 1) * BK + 32 * i) >> p.group_shift) * 64];
    };
    auto load_w = [&](int kt, int i) { load_q(kt, i); load_s(kt, i); };

    // Slice s of staging the registers into buffer dst while reloading them with tile load_kt.
    // Unit u = s / SPU is code word u%4 of row half u/4; each slot produces WPS of its 4 words.
    // ---- sensitive entries -------------------------------------------------------------------
    // Computes entries [s, s+256) of the band (s a multiple of 4) into the window.
    auto refill = [&](uint32_t s) {
      const FwdParams pr = cold();
      const uint32_t j = s + 4u * lane;
      if (j < band_end) {
        uint32_t idx[4];
        float val[4];
        if (j + 3 < pr.nnz) {
          const uint4 iv = *reinterpret_cast<const uint4*>(pr.sp_idx + j);
          const float4 vv = *reinterpret_cast<const float4*>(pr.sp_val + j);
          idx[0] = iv.x; idx[1] = iv.y; idx[2] = iv.z; idx[3] = iv.w;
          val[0] = vv.x; val[1] = vv.y; val[2] = vv.z; val[3] = vv.w;
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const bool ok = j + c < pr.nnz;
            idx[c] = ok ? pr.sp_idx[j + c] : 0xFFFFFFFFu;
            val[c] = ok ? pr.sp_val[j + c] : 0.0f;
          }
        }
        float val_minus[4] = {val[0], val[1], val[2], val[3]};
        if (pr.signed_eps != 0.0f) {
          float z[4];
          zbar_quad((pr.nnz_base + j) >> 2, pr.seed, pr.step, z);
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            if (DUAL) val_minus[c] = fmaf(-pr.signed_eps, z[c], val[c]);
            val[c] = fmaf(pr.signed_eps, z[c], val[c]);
          }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const uint32_t n = fast_div(idx[c], pr.div_mul, pr.div_shift);
          const uint32_t r = n - (uint32_t)(band * 64);                   // row inside the band
          const uint32_t kk = (idx[c] - n * (uint32_t)pr.K) & 63u;
          wp[4 * lane + c] = (r < 64u) ? (uint16_t)lds_pos<DT>(wave * 64 + (int)r, (int)kk) : (uint16_t)0xFFFFu;
          wv[4 * lane + c] = val[c];
          if (DUAL) wv_minus[4 * lane + c] = val_minus[c];
        }
      }
      win_lo = s;
      win_hi = min(s + (uint32_t)kWindow, band_end);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // window visible to the other lanes of the wave
    };

    // General path: adds entries [lo, hi) of the band into LDS buffer `buf`, any count.
    auto scatter_range = [&](uint32_t lo, uint32_t hi_end, int buf) {
      uint16_t* B = ldsB + buf * BN * BK;
      uint32_t cur = lo;
      while (cur < hi_end) {
        if (cur >= win_hi || cur < win_lo) refill(cur & ~3u);
        const uint32_t hi = min(hi_end, win_hi);
        for (uint32_t j = cur + lane; j < hi; j += 64) {
          const uint32_t e = j - win_lo;
          const uint32_t pos = wp[e];
          if (pos != 0xFFFFu) {
            uint16_t* w = B + pos;
            Frag<DT>::store(w, Frag<DT>::load(w) + wv[e]);
            if (DUAL) Frag<DT>::store(w + kMinusCopy, Frag<DT>::load(w + kMinusCopy) + wv_minus[e]);
          }
        }
        cur = hi;
      }
    };

    // Per-tile bookkeeping, done before the MFMA loop that stages the tile.  Tiles with at most 64
    // entries (the normal case) take the in-slot path: sc_cnt entries starting at window offset
    // sc_e0, one per lane.  Larger tiles are left to scatter_range after the loop.
    uint32_t sc_cnt = 0, sc_e0 = 0, big_lo = 0, big_hi = 0;
    auto prepare_scatter = [&](int kt) {
      sc_cnt = 0; big_lo = 0; big_hi = 0;
      if (!band_ok || kt >= nk) return;
      if ((kt & 63) == 0 && kt > 0) {                        // the first 64 boundaries were loaded with tile_lo
        const uint32_t t = tp_base + (uint32_t)kt + 1u + lane;
        tp_reg = (t <= tp_base + (uint32_t)nk) ? cold().tile_ptr[t] : band_end;
        asm volatile("" : "+v"(tp_reg));       // consume the load here, so that no wait on it is needed later
      }
      const uint32_t hi = __builtin_amdgcn_readlane(tp_reg, kt & 63), lo = tile_lo;
      tile_lo = hi;
      if (hi <= lo) return;
      if (SCATTER_IN_SLOTS && hi - lo <= 64u) {
        if (lo < win_lo || hi > win_hi) refill(lo & ~3u);
        sc_cnt = hi - lo;
        sc_e0 = lo - win_lo;
      } else {
        big_lo = lo; big_hi = hi;
      }
    };

    if constexpr (FMT == SZO_FORMAT_LUT) {
      // ---- table format: dq[n,k] = lut[n][code] (non-uniform 4-bit quantisers, Appendix C.5) -------
      // gfx950 has no register-indexed look-up, so the table of a row is held as four byte planes (low
      // and high bytes of entries 0-7 and of entries 8-15, two registers each) and looked up with the
      // byte-permute instruction, four codes at a time: low 3 bits of the codes select inside a plane,
      // bit 3 picks the plane.  That only pays if a lane keeps ONE row's table for the whole K loop:
      // lane l stages row l of the band, all 64 columns of a tile (32 bytes of codes, two 16-byte loads).
      static_assert(DT == SZO_TILE_F16 && SCATTER_IN_SLOTS, "table format: fp16 tile, 32-slot schedule");
      const int lrow = wave * 64 + lane;                           // row of the weight tile
      const uint8_t* const qr = p.qweight + ((size_t)min(band, p.bands - 1) * (size_t)nk * 64 + (size_t)lane) * 32;
      u32x4 qv[2];
      auto load_qv = [&](int kt, int h) {
        qv[h] = *reinterpret_cast<const u32x4*>(qr + (size_t)min(kt, nk - 1) * (64 * BK / 2) + 16 * h);
      };
      uint32_t lo_a0, lo_a1, lo_b0, lo_b1, hi_a0, hi_a1, hi_b0, hi_b1;
      {
        // rows past N re-read the last row's table: their outputs are never used
        const u32x4* const lp = reinterpret_cast<const u32x4*>(p.lut + (size_t)min(n0 + lrow, p.N - 1) * 16);
        const u32x4 a = lp[0], b = lp[1];                          // entries 0-7 and 8-15, two per word
        lo_a0 = __builtin_amdgcn_perm(a[1], a[0], 0x06040200u); lo_a1 = __builtin_amdgcn_perm(a[3], a[2], 0x06040200u);
        hi_a0 = __builtin_amdgcn_perm(a[1], a[0], 0x07050301u); hi_a1 = __builtin_amdgcn_perm(a[3], a[2], 0x07050301u);
        lo_b0 = __builtin_amdgcn_perm(b[1], b[0], 0x06040200u); lo_b1 = __builtin_amdgcn_perm(b[3], b[2], 0x06040200u);
        hi_b0 = __builtin_amdgcn_perm(b[1], b[0], 0x07050301u); hi_b1 = __builtin_amdgcn_perm(b[3], b[2], 0x07050301u);
      }
      // Slots 3d, 3d+1, 3d+2 turn code word d (columns 8d .. 8d+7) into chunk d of the row:
      //   selectors and plane masks  ->  eight look-ups and four selects  ->  interleave and store.
      // Even codes (0,2,4,6) sit in the low nibbles of the word's bytes, odd ones in the high nibbles;
      // the chunk keeps the element order (0,4)(1,5)(2,6)(3,7) that the activations are staged in.
      // Slots 24, 27 and 30 scatter the tile's sensitive entries as in the uniform format.
      uint32_t sel_e = 0, sel_o = 0, m_e = 0, m_o = 0, lo_e = 0, hi_e = 0, lo_o = 0, hi_o = 0;
      u32x4 outw;
      uint32_t sc_pos = 0xFFFFu;
      float sc_val = 0.0f, sc_old = 0.0f;
      uint16_t* sc_addr = nullptr;
      auto make_slice = [&](int dst, int load_kt) {
        return [&, dst, load_kt](int s) {
          if (s < 24) {
            const int d = s / 3, ph = s % 3;
            if (ph == 0) {
              const uint32_t q = qv[d >> 2][d & 3];
              sel_e = q & 0x07070707u;
              sel_o = (q >> 4) & 0x07070707u;
              // 0xFF in the bytes whose code has bit 3 set: byte 1 of the constant, else byte 0
              m_e = __builtin_amdgcn_perm(0u, 0x0000FF00u, (q >> 3) & 0x01010101u);
              m_o = __builtin_amdgcn_perm(0u, 0x0000FF00u, (q >> 7) & 0x01010101u);
              if ((d & 3) == 3) load_qv(load_kt, d >> 2);          // codes consumed: reload in place
            } else if (ph == 1) {
              auto pick = [](uint32_t m, uint32_t b, uint32_t a) { return (m & b) | (~m & a); };
              lo_e = pick(m_e, __builtin_amdgcn_perm(lo_b1, lo_b0, sel_e), __builtin_amdgcn_perm(lo_a1, lo_a0, sel_e));
              hi_e = pick(m_e, __builtin_amdgcn_perm(hi_b1, hi_b0, sel_e), __builtin_amdgcn_perm(hi_a1, hi_a0, sel_e));
              lo_o = pick(m_o, __builtin_amdgcn_perm(lo_b1, lo_b0, sel_o), __builtin_amdgcn_perm(lo_a1, lo_a0, sel_o));
              hi_o = pick(m_o, __builtin_amdgcn_perm(hi_b1, hi_b0, sel_o), __builtin_amdgcn_perm(hi_a1, hi_a0, sel_o));
            } else {
              outw[0] = __builtin_amdgcn_perm(hi_e, lo_e, 0x06020400u);      // codes 0, 4
              outw[1] = __builtin_amdgcn_perm(hi_o, lo_o, 0x06020400u);      // codes 1, 5
              outw[2] = __builtin_amdgcn_perm(hi_e, lo_e, 0x07030501u);      // codes 2, 6
              outw[3] = __builtin_amdgcn_perm(hi_o, lo_o, 0x07030501u);      // codes 3, 7
              *reinterpret_cast<u32x4*>(ldsB + dst * BN * BK + chunk_off(lrow, d)) = outw;
            }
          }
          const bool active = (uint32_t)lane < sc_cnt;
          if (s == 24) {
            const uint32_t e = active ? sc_e0 + lane : 0u;
            sc_pos = wp[e];
            sc_val = wv[e];
          } else if (s == 27) {                         // every dense word of the tile is written by slot 23
            const bool ok = active && sc_pos != 0xFFFFu;
            sc_addr = ok ? ldsB + dst * BN * BK + sc_pos : sink16 + wave * 64 + lane;
            sc_val = ok ? sc_val : 0.0f;
            sc_old = Frag<DT>::load(sc_addr);
          } else if (s == 30) {
            Frag<DT>::store(sc_addr, sc_old + sc_val);
          }
        };
      };

      __builtin_amdgcn_s_setprio(1);
      load_qv(0, 0);
      load_qv(0, 1);
      tile_lo = __builtin_amdgcn_readfirstlane(t_lo);
      band_end = __builtin_amdgcn_readfirstlane(t_end);
      prepare_scatter(0);
      {
        auto slice = make_slice(0, 1);
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) slice(s);
      }
      if (big_hi > big_lo) scatter_range(big_lo, big_hi, 0);
      for (int kt = 0; kt < nk; kt += 2) {
        __syncthreads();                       // tile kt complete in buffer 0; buffer 1 no longer read
        prepare_scatter(kt + 1);
        run_tile(0, make_slice(1, kt + 2));
        if (big_hi > big_lo) scatter_range(big_lo, big_hi, 1);
        if (kt + 1 < nk) {
          __syncthreads();
          prepare_scatter(kt + 2);
          run_tile(1, make_slice(0, kt + 3));
          if (big_hi > big_lo) scatter_range(big_lo, big_hi, 0);
        }
      }
    } else {
    // ---- slices ---------------------------------------------------------------------------------
    // Dense part: unit u = code word u%4 of row half u/4; DSPU slots per unit; the unit's four
    // output words are spread 4 | 2,2 | 2,1,1 | 1,1,1,1 over them.  In the 32-slot schedule the
    // three instructions of an output word (and_or, subtract offset, multiply by scale) run in
    // three consecutive slots, so no slot holds two dependent VALU instructions.
    // Scatter part (32-slot schedule only): window read, tile read, add + write, three slots
    // apart; lanes without an entry go through a per-lane sink in LDS, which keeps it branch-free.
    constexpr int PIPE = SCATTER_IN_SLOTS ? 1 : 0;      // slot distance between the stages of a word
    u32x4 outw;
    uint32_t st_a[3][2], st_b[3][2];
    uint32_t sc_pos = 0xFFFFu;
    float sc_val = 0.0f, sc_old = 0.0f, sc_val_minus = 0.0f, sc_old_minus = 0.0f;
    uint16_t* sc_addr = nullptr;
    uint16_t* sc_addr_minus = nullptr;
    auto make_slice = [&](int dst, int load_kt) {
      return [&, dst, load_kt](int s) {
        // the k-th (0 or 1) output word staged from slot `slot`: unit u, word w; false if none
        auto item = [](int slot, int k, int& u, int& w) -> bool {
          if (slot < 0 || slot >= 8 * DSPU) return false;
          u = slot / DSPU;
          const int ph = slot % DSPU;
          const int w0 = (DSPU == 3) ? (ph == 0 ? 0 : ph + 1) : ph * (4 / DSPU);
          const int nw = (DSPU == 3) ? (ph == 0 ? 2 : 1) : (4 / DSPU);
          w = w0 + k;
          return k < nw;
        };
        constexpr int KMAX = (DSPU == 1) ? 4 : 2;
        static_assert(KMAX <= 2 || PIPE == 0, "stage registers hold two words per slot");
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
          int u = 0, w = 0;
          if (PIPE == 0) {                              // all three stages at once
            if (item(s, k, u, w)) {
              const int i = u >> 2, c = u & 3;
              const _Float16 sh = __builtin_bit_cast(_Float16, sreg[i]);
              outw[w] = dequant_out<DT>(qreg[i][c], w, (float)sh, half2_t{sh, sh}, dqk);
              if (w == 3) {
                *reinterpret_cast<u32x4*>(ldsB + dst * BN * BK + chunk_off(wr, 4 * i + c)) = outw;
                if (DUAL) *reinterpret_cast<u32x4*>(ldsB + dst * BN * BK + kMinusCopy + chunk_off(wr, 4 * i + c)) = outw;
                if (c == 3) load_w(load_kt, i);
              }
            }
            continue;
          }
          if (item(s, k, u, w)) {                       // stage A: isolate the nibble pair under its exponent
            const int i = u >> 2, c = u & 3;
            const uint32_t q = qreg[i][c];
            if (DT == SZO_TILE_F16)
              st_a[s % 3][k] = and_or(w < 2 ? q : (q >> 8), (w & 1) ? 0x00F000F0u : 0x000F000Fu,
                                      (w & 1) ? dqk.magic_hi : dqk.magic_lo);
            if (w == 3 && c == 3 && DT == SZO_TILE_F16) load_q(load_kt, i);   // codes consumed: reload in place
          }
          if (item(s - 1, k, u, w) && DT == SZO_TILE_F16) {   // stage B: remove the exponent's offset (exact)
            const _Float16 o = (w & 1) ? (_Float16)72.0f : (_Float16)1032.0f;
            const half2_t h = __builtin_bit_cast(half2_t, st_a[(s - 1) % 3][k]) - half2_t{o, o};
            st_b[(s - 1) % 3][k] = __builtin_bit_cast(uint32_t, h);
          }
          if (item(s - 2, k, u, w)) {                   // stage C: scale, rounded once
            const int i = u >> 2, c = u & 3;
            const _Float16 sh = __builtin_bit_cast(_Float16, sreg[i]);
            if (DT == SZO_TILE_F16) {
              const half2_t h = __builtin_bit_cast(half2_t, st_b[(s - 2) % 3][k]) * half2_t{sh, sh};
              outw[w] = __builtin_bit_cast(uint32_t, h);
            } else {
              outw[w] = dequant_out<DT>(qreg[i][c], w, (float)sh, half2_t{sh, sh}, dqk);
            }
            if (w == 3) {
              *reinterpret_cast<u32x4*>(ldsB + dst * BN * BK + chunk_off(wr, 4 * i + c)) = outw;
              if (DUAL) *reinterpret_cast<u32x4*>(ldsB + dst * BN * BK + kMinusCopy + chunk_off(wr, 4 * i + c)) = outw;
              if (c == 3) {
                if (DT != SZO_TILE_F16) load_q(load_kt, i);
                load_s(load_kt, i);
              }
            }
          }
        }
        if (SCATTER_IN_SLOTS) {
          const bool active = (uint32_t)lane < sc_cnt;
          if (s == 24) {
            const uint32_t e = active ? sc_e0 + lane : 0u;
            sc_pos = wp[e];
            sc_val = wv[e];
            if (DUAL) sc_val_minus = wv_minus[e];
          } else if (s == 27) {                         // every dense word of the tile is written by slot 25
            const bool ok = active && sc_pos != 0xFFFFu;
            sc_addr = ok ? ldsB + dst * BN * BK + sc_pos : sink16 + wave * 64 + lane;
            sc_val = ok ? sc_val : 0.0f;
            sc_old = Frag<DT>::load(sc_addr);
            if (DUAL) {                                 // the same position in the -eps copy
              sc_addr_minus = ok ? ldsB + dst * BN * BK + kMinusCopy + sc_pos : sink16 + (wave + W_WAVES / 2) * 64 + lane;
              sc_val_minus = ok ? sc_val_minus : 0.0f;
              sc_old_minus = Frag<DT>::load(sc_addr_minus);
            }
          } else if (s == 30) {
            Frag<DT>::store(sc_addr, sc_old + sc_val);
            if (DUAL) Frag<DT>::store(sc_addr_minus, sc_old_minus + sc_val_minus);
          }
        }
      };
    };

    // Weight waves carry more staging instructions per MFMA slot than activation waves; a higher
    // issue priority lets the two waves of a SIMD finish their K step together.
    __builtin_amdgcn_s_setprio(1);
    load_w(0, 0);
    load_w(0, 1);
    tile_lo = __builtin_amdgcn_readfirstlane(t_lo);
    band_end = __builtin_amdgcn_readfirstlane(t_end);
    prepare_scatter(0);
    {
      auto slice = make_slice(0, 1);
#pragma unroll
      for (int s = 0; s < SLOTS; ++s) slice(s);
    }
    if (big_hi > big_lo) scatter_range(big_lo, big_hi, 0);
    for (int kt = 0; kt < nk; kt += 2) {
      __syncthreads();                       // tile kt complete in buffer 0; buffer 1 no longer read
      prepare_scatter(kt + 1);
      run_tile(0, make_slice(1, kt + 2));
      if (big_hi > big_lo) scatter_range(big_lo, big_hi, 1);
      if (kt + 1 < nk) {
        __syncthreads();
        prepare_scatter(kt + 2);
        run_tile(1, make_slice(0, kt + 3));
        if (big_hi > big_lo) scatter_range(big_lo, big_hi, 0);
      }
    }
    }  // uniform format
  } else {
    // =============================== activation wave ===========================================
    const int xt = tid - 64 * W_WAVES;
    const int xc = xt & 7, xr = xt >> 3;                       // chunk, row (plus X_ROWS_PER_PASS*u)
    const uint16_t* xrow[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      xrow[u] = p.x + (size_t)min(m0 + xr + X_ROWS_PER_PASS * u, p.M - 1) * p.K + xc * 8;
    u32x4 xreg[8];
    auto load_x = [&](int kt, int u) {
      xreg[u] = *reinterpret_cast<const u32x4*>(xrow[u] + min(kt, nk - 1) * BK);
    };
    u32x4 outw;
    auto make_slice = [&](int dst, int load_kt) {
      return [&, dst, load_kt](int s) {
        const int u = s / SPU;
#pragma unroll
        for (int o = 0; o < WPS; ++o) {
          const int w = (s % SPU) * WPS + o;
          outw[w] = stage_x_word<DT>(xreg[u], w);
        }
        if (s % SPU == SPU - 1) {
          *reinterpret_cast<u32x4*>(ldsA + dst * BM * BK + chunk_off(xr + X_ROWS_PER_PASS * u, xc)) = outw;
          load_x(load_kt, u);
        }
      };
    };

#pragma unroll
    for (int u = 0; u < 8; ++u) load_x(0, u);
    {
      auto slice = make_slice(0, 1);
#pragma unroll
      for (int s = 0; s < SLOTS; ++s) slice(s);
    }
    for (int kt = 0; kt < nk; kt += 2) {
      __syncthreads();
      run_tile(0, make_slice(1, kt + 2));
      if (kt + 1 < nk) {
        __syncthreads();
        run_tile(1, make_slice(0, kt + 3));
      }
    }
  }

  // ---- epilogue: accumulator (i,j) register r holds
  //      row  32*i + 8*(r/4) + 4*(lane/32) + r%4 ,  column 32*j + lane%32  of the wave tile ----
  // Fused loss: the bf16 target tile is first copied into the (now idle) LDS tile buffers with
  // coalesced 16-byte loads, then every lane picks its own elements from LDS.  Differences and
  // squares are formed in fp32, summed over the 16 registers of one MFMA block in fp32, and
  // every such partial is added in fp64 (the loss difference of the two passes is ~1e-6 of the
  // loss, far below fp32 resolution of a long sum).
  constexpr int TROW = TN * 2 + 32;               // LDS row stride of the target tile in bytes
  const FwdParams pe = cold();
  bool staged = false;
  if (FUSE_LOSS) {
    staged = ((pe.N & 7) == 0) && ((reinterpret_cast<uintptr_t>(pe.target) & 15) == 0);
    if (staged) {
      constexpr int CPR = TN / 8;                 // 16-byte chunks per tile row
      constexpr int ROWS_PER_PASS = 64 * NWAVES / CPR;
      uint8_t* const T = reinterpret_cast<uint8_t*>(lds);
      const int c = tid % CPR, r0 = tid / CPR;
      __syncthreads();                            // every wave is done with the tile buffers
      // The loads of a batch are issued before the first one is used: guarded loads in a loop would each
      // be waited for before the next is issued (16 memory round trips in a row).  Batches of four:
      // on the full stack larger bursts measured slower (8 at a time: +3 % step time), presumably because
      // they delay the operand loads of the neighbouring workgroups' main loops.  Rows and columns past
      // the matrix re-read its last row / last 8 columns; those LDS entries are never looked at.
      constexpr int PASSES = BM / ROWS_PER_PASS, BATCH = 4;
      static_assert(PASSES % BATCH == 0, "whole batches");
      const int ncl = min(n0 + 8 * c, pe.N - 8);
#pragma unroll
      for (int b = 0; b < PASSES; b += BATCH) {
        uint4 t[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
          const int m = min(m0 + r0 + ROWS_PER_PASS * (b + i), pe.M - 1);
          t[i] = *reinterpret_cast<const uint4*>(pe.target + (size_t)m * pe.N + ncl);
        }
#pragma unroll
        for (int i = 0; i < BATCH; ++i)
          *reinterpret_cast<uint4*>(T + (r0 + ROWS_PER_PASS * (b + i)) * TROW + 16 * c) = t[i];
      }
      __syncthreads();
    }
  }
  double loss = 0.0;
  // Element (i, j, r) of this lane: tile row ml0 + 32 i + 8 (r/4) + r%4, tile column nl0 + 32 j.
  // DUAL: the waves of the second half of a wave row hold the -eps forward of the same columns.
  const int wn_col = DUAL ? wn % (WAVES_N / 2) : wn;
  const int ml0 = wm * 32 * WMB + 4 * (lane >> 5), nl0 = wn_col * 32 * WNB + (lane & 31);
  const uint8_t* const trow = reinterpret_cast<const uint8_t*>(lds) + ml0 * TROW + nl0 * 2;
  // FULL: whole tile inside the matrix (no bounds checks).  STAGED: targets come from LDS.
  // STORE: y is written.  The three are compile-time so that the common cases are straight code.
  auto finish = [&](auto full_tag, auto staged_tag, auto store_tag) {
    constexpr bool FULL = decltype(full_tag)::value, STAGED = decltype(staged_tag)::value,
                   STORE = decltype(store_tag)::value;
    const uint32_t ybase = (uint32_t)(m0 + ml0) * (uint32_t)pe.N + (uint32_t)(n0 + nl0);   // M*N < 2^32 checked on the host
#pragma unroll
    for (int i = 0; i < WMB; ++i) {
#pragma unroll
      for (int j = 0; j < WNB; ++j) {
        float part = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int dm = 32 * i + 8 * (r >> 2) + (r & 3), dn = 32 * j;
          if (FULL || (m0 + ml0 + dm < pe.M && n0 + nl0 + dn < pe.N)) {
            const float v = acc[i][j][r];
            const uint32_t off = ybase + (uint32_t)dm * (uint32_t)pe.N + (uint32_t)dn;
            if (STORE) pe.y[off] = v;
            if (FUSE_LOSS) {
              uint32_t tb;
              if (STAGED) tb = *reinterpret_cast<const uint16_t*>(trow + dm * TROW + dn * 2);
              else tb = pe.target[off];
              const float d = v - __uint_as_float(tb << 16);
              part = fmaf(d, d, part);
            }
          }
        }
        loss += (double)part;
      }
    }
  };
  {
    using T = std::true_type;
    using F = std::false_type;
    const bool full = m0 + BM <= pe.M && n0 + TN <= pe.N;
    if (FUSE_LOSS) {
      if (full && staged && !pe.y) finish(T{}, T{}, F{});            // the step's path
      else if (staged) { if (pe.y) finish(F{}, T{}, T{}); else finish(F{}, T{}, F{}); }
      else { if (pe.y) finish(F{}, F{}, T{}); else finish(F{}, F{}, F{}); }
    } else {
      if (full) finish(T{}, F{}, T{});
      else finish(F{}, F{}, T{});
    }
  }
  if (FUSE_LOSS) {
    // One scaled partial per workgroup, plain store: a later kernel on the same stream adds them
    // up in index order, so the kernel boundary is the only synchronisation needed.
    __shared__ double wave_part[NWAVES];
    const double w = wave_sum(loss);
    if (lane == 0) wave_part[wave] = w;
    __syncthreads();
    if (tid == 0) {
      double b = 0.0, b_minus = 0.0;
#pragma unroll
      for (int i = 0; i < NWAVES; ++i) {
        if (DUAL && (i % WAVES_N) >= WAVES_N / 2) b_minus += wave_part[i];
        else b += wave_part[i];
      }
      pe.partials[bm * pe.grid_n + bn] = b * pe.loss_scale;       // indexed by tile: the sum does not depend on the launch order
      if (DUAL) pe.partials_minus[bm * pe.grid_n + bn] = b_minus * pe.loss_scale;
    }
  }
}

template <int WAVES_M, int WAVES_N, int WMB, int WNB, int DT, bool FUSE_LOSS, int FMT>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) linear_fwd_kernel(FwdParams p) {
  int bm, bn;
  tile_of_logical(logical_block((int)blockIdx.x, p.grid_m * p.grid_n), p.grid_m, p.grid_n, 4, bm, bn);
  linear_fwd_body<WAVES_M, WAVES_N, WMB, WNB, DT, FUSE_LOSS, FMT>(p, bm, bn);
}

// Grouped launch: every forward of a step (all matrices, both signs) in one grid, so that the only
// partly filled round of workgroups is the last one of the step, not the last one of every matrix.
// `table` holds one FwdParams per MATRIX, ordered by first_block; a workgroup finds its entry by
// binary search and reads it through the constant address space (scalar loads into scalar registers).
// An entry has 2 * grid_m * grid_n workgroups: neighbouring logical ids are the +eps and the -eps
// forward of the same tile, and pairs walk the grid in strips of 2 row blocks, so the 32 workgroups
// resident on an XCD are 2 x 8 tiles x 2 signs: both forwards of a tile read the same activations and
// the same codes while those are in that XCD's L2, instead of the second forward fetching everything
// again later.  Workgroups between an entry's last tile and the next multiple of 8 have nothing to do.
// With DUAL an entry has grid_m * grid_n workgroups, each computing both forwards of a tile of half the
// width (see linear_fwd_body); the 32 workgroups resident on an XCD are then 2 x 16 such tiles.
template <int WAVES_M, int WAVES_N, int WMB, int WNB, int DT, bool FUSE_LOSS, int FMT, bool DUAL = false>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) linear_fwd_table_kernel(const FwdParams* table, int n_entries) {
  constexpr int W = (int)(sizeof(FwdParams) / 4), FB = (int)(offsetof(FwdParams, first_block) / 4);
  static_assert(sizeof(FwdParams) % 4 == 0 && offsetof(FwdParams, first_block) % 4 == 0, "table entry is read as words");
  const auto* tab = (const uint32_t __attribute__((address_space(4)))*)table;
  int lo = 0, hi = n_entries - 1;                           // last entry whose first_block <= blockIdx.x
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if ((int)tab[mid * W + FB] <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
  }
  struct Words { uint32_t w[W]; } raw;
#pragma unroll
  for (int i = 0; i < W; ++i) raw.w[i] = tab[lo * W + i];
  FwdParams p = __builtin_bit_cast(FwdParams, raw);
  const int bid = (int)blockIdx.x - p.first_block, count = (DUAL ? 1 : 2) * p.grid_m * p.grid_n;
  if (bid >= count) return;
  const int L = logical_block(bid, count);
  int bm, bn;
  if (DUAL) {
    tile_of_logical(L, p.grid_m, p.grid_n, 2, bm, bn);
  } else {
    tile_of_logical(L >> 1, p.grid_m, p.grid_n, 2, bm, bn);
    if (L & 1) {                                            // the -eps forward of the tile
      p.x = p.x_minus;
      p.partials = p.partials_minus;
      p.signed_eps = -p.signed_eps;
    }
  }
  linear_fwd_body<WAVES_M, WAVES_N, WMB, WNB, DT, FUSE_LOSS, FMT, DUAL>(p, bm, bn, tab + lo * W);
}

// ---- host side -----------------------------------------------------------------------------

static int g_tile_config = 0;      // 0 = choose by shape, 1 = 128x128 (4 waves), 2 = 256x256 (8 waves), 3 = 2 + always group the step,
                                   // 4, 5 = as 0 with the few-token path's 32- / 48-row passes forced (see small_m_force_rblocks),
                                   // 6 = as 0 + always group the step, 7 = as 0 + non-temporal code stream in every one-slice launch
static bool few_token_enabled() { return g_tile_config == 0 || g_tile_config >= 4; }

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
  if (d->format != SZO_FORMAT_UNIFORM && d->format != SZO_FORMAT_LUT) return SZO_EINVAL;
  const bool table_format = d->format == SZO_FORMAT_LUT;
  if (!table_format && (d->group <= 0 || d->K % d->group)) return SZO_EINVAL;
  if (d->nnz_base & 3) return SZO_EINVAL;
  if (!table_format && d->group != 32 && d->group != 64 && d->group != 128) return SZO_EUNSUPPORTED;
  if (table_format && d->tile_dtype != SZO_TILE_F16) return SZO_EUNSUPPORTED;
  if (d->K % BK) return SZO_EUNSUPPORTED;
  if ((uint64_t)d->N * (uint64_t)d->K > 0xFFFFFFFFull) return SZO_EUNSUPPORTED;
  if (d->M > 0x7FFFFFFF || d->N > 0x7FFFFFFF || d->nnz > 0xFFFFFFFFll) return SZO_EUNSUPPORTED;
  if ((uint64_t)d->M * (uint64_t)d->N > 0xFFFFFFFFull) return SZO_EUNSUPPORTED;
  if (d->M == 0 || d->N == 0) return SZO_OK;
  if (!d->x || !d->qweight || !d->tile_ptr) return SZO_EINVAL;
  if (table_format ? (!d->lut || ((uintptr_t)d->lut & 15)) : !d->scales) return SZO_EINVAL;
  if (d->nnz > 0 && (!d->sp_idx || !d->sp_val)) return SZO_EINVAL;
  if (need_y && !d->y) return SZO_EINVAL;
  if (need_target && !d->target) return SZO_EINVAL;
  if (((uintptr_t)d->x & 15) || ((uintptr_t)d->x_minus & 15) || ((uintptr_t)d->qweight & 15) || ((uintptr_t)d->scales & 1) ||
      ((uintptr_t)d->tile_ptr & 3) || ((uintptr_t)d->sp_idx & 15) || ((uintptr_t)d->sp_val & 15) ||
      ((uintptr_t)d->y & 3) || ((uintptr_t)d->target & 1))
    return SZO_EINVAL;
  return SZO_OK;
}

template <int WAVES_M, int WAVES_N, int WMB, int WNB, int DT, bool FUSE, int FMT = SZO_FORMAT_UNIFORM>
static int launch(FwdParams& p, hipStream_t stream) {
  constexpr int BM = 32 * WMB * WAVES_M, BN = 32 * WNB * WAVES_N;
  p.grid_m = (p.M + BM - 1) / BM;
  p.grid_n = (p.N + BN - 1) / BN;
  const int64_t blocks = (int64_t)p.grid_m * p.grid_n;
  if (blocks > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
  constexpr size_t main_bytes = 2 * (size_t)(BM + BN) * BK * sizeof(uint16_t) + (size_t)(BN / 64) * (kWindow * 6 + 128);
  constexpr size_t target_bytes = FUSE ? (size_t)BM * (BN * 2 + 32) : 0;      // staged target tile of the fused loss
  constexpr size_t lds_bytes = main_bytes > target_bytes ? main_bytes : target_bytes;
  auto kern = linear_fwd_kernel<WAVES_M, WAVES_N, WMB, WNB, DT, FUSE, FMT>;
  static std::atomic<uint64_t> lds_limit_set{0};     // per instantiation
  int rc = set_lds_limit_once(lds_limit_set, (const void*)kern, lds_bytes);
  if (rc != SZO_OK) return rc;
  rc = timing_begin(stream);
  if (rc != SZO_OK) return rc;
  kern<<<(unsigned)blocks, 64 * WAVES_M * WAVES_N, lds_bytes, stream>>>(p);
  SZO_LAUNCH_CHECK();
  return timing_end(stream);
}

// Which workgroup tile a shape runs with, and how many workgroups (= loss partials) that makes.
static int plan_tiles(int M, int N, int format, int* blocks_out) {
  int cfg = g_tile_config >= 4 ? 0 : g_tile_config;
  if (format == SZO_FORMAT_LUT) cfg = 2;          // the table format exists for the 256x256 tile only
  if (cfg == 0) {
    const int64_t big_blocks = (int64_t)((M + 255) / 256) * ((N + 255) / 256);
    cfg = big_blocks >= 192 ? 2 : 1;
  }
  if (cfg == 3) cfg = 2;
  const int t = cfg == 2 ? 256 : 128;
  const int64_t blocks = (int64_t)((M + t - 1) / t) * ((N + t - 1) / t);
  *blocks_out = blocks > 0x7FFFFFFF ? -1 : (int)blocks;
  return cfg;
}

template <int DT, bool FUSE>
static int dispatch_tile(FwdParams& p, hipStream_t stream) {
  int blocks;
  if (plan_tiles(p.M, p.N, SZO_FORMAT_UNIFORM, &blocks) == 2) return launch<2, 4, 4, 2, DT, FUSE>(p, stream);
  return launch<2, 2, 2, 2, DT, FUSE>(p, stream);
}

// Enqueues one forward.  With `partials` set the loss is fused: workgroup b stores
// scale * sum (y - target)^2 of its tile to partials[b].
static int fill_params(FwdParams& p, const szo_linear_desc* d, uint64_t seed, uint64_t step, int sign, float eps,
                       double* partials, double scale) {
  p = FwdParams{};
  p.x = (const uint16_t*)d->x;
  p.qweight = d->qweight;
  p.scales = (const uint16_t*)d->scales;
  p.lut = (const uint16_t*)d->lut;
  p.tile_ptr = d->tile_ptr;
  p.sp_idx = d->sp_idx;
  p.sp_val = d->sp_val;
  p.y = d->y;
  p.target = (const uint16_t*)d->target;
  p.M = (int)d->M; p.N = (int)d->N; p.K = (int)d->K;
  p.nnz = (uint32_t)d->nnz;
  p.group_shift = d->format == SZO_FORMAT_LUT ? 0 : ilog2_exact(d->group);
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
  p.partials = partials;
  p.loss_scale = scale;
  return SZO_OK;
}

// `step_minus`: this is the -eps forward of a whole step, which reads desc->x_minus where that is set.
static int run_forward(const szo_linear_desc* d, uint64_t seed, uint64_t step, int sign, float eps,
                       double* partials, double scale, hipStream_t stream, bool step_minus = false) {
  const bool fuse = partials != nullptr;
  if (d->M == 0 || d->N == 0) return SZO_OK;
  FwdParams p;
  const int frc = fill_params(p, d, seed, step, sign, eps, partials, scale);
  if (frc != SZO_OK) return frc;
  if (step_minus && d->x_minus) p.x = (const uint16_t*)d->x_minus;
  if (d->format == SZO_FORMAT_LUT)
    return fuse ? launch<2, 4, 4, 2, SZO_TILE_F16, true, SZO_FORMAT_LUT>(p, stream)
                : launch<2, 4, 4, 2, SZO_TILE_F16, false, SZO_FORMAT_LUT>(p, stream);
  if (d->tile_dtype == SZO_TILE_F16)
    return fuse ? dispatch_tile<SZO_TILE_F16, true>(p, stream) : dispatch_tile<SZO_TILE_F16, false>(p, stream);
  return fuse ? dispatch_tile<SZO_TILE_BF16, true>(p, stream) : dispatch_tile<SZO_TILE_BF16, false>(p, stream);
}

static double* partial_area(void* workspace) { return (double*)((char*)workspace + kWorkspaceHeader); }

template <int DT, int FMT = SZO_FORMAT_UNIFORM, int TILE = 256, bool DUAL = false>
static int launch_table(const FwdParams* table_dev, int entries, int64_t blocks, hipStream_t stream) {
  static_assert(TILE == 256 || TILE == 128, "two workgroup tiles exist");
  constexpr int BM = TILE, BN = TILE;
  constexpr int WAVES_N = TILE == 256 ? 4 : 2, WMB = TILE == 256 ? 4 : 2;      // 2x4 waves of 128x64, or 2x2 of 64x64
  constexpr size_t main_bytes = 2 * (size_t)(BM + BN) * BK * sizeof(uint16_t) + (size_t)(BN / 64) * (kWindow * 6 + 128);
  constexpr size_t target_bytes = (size_t)BM * (BN * 2 + 32);
  constexpr size_t lds_bytes = main_bytes > target_bytes ? main_bytes : target_bytes;
  auto kern = linear_fwd_table_kernel<2, WAVES_N, WMB, 2, DT, true, FMT, DUAL>;
  static std::atomic<uint64_t> lds_limit_set{0};
  int rc = set_lds_limit_once(lds_limit_set, (const void*)kern, lds_bytes);
  if (rc != SZO_OK) return rc;
  rc = timing_begin(stream);
  if (rc != SZO_OK) return rc;
  kern<<<(unsigned)blocks, 128 * WAVES_N, lds_bytes, stream>>>(table_dev, entries);
  SZO_LAUNCH_CHECK();
  return timing_end(stream);
}

// Both forwards of every matrix of a step as ONE launch with the loss fused: 256x256 tiles, or 128x128
// when the library chooses the tiles and no matrix has more than 128 tokens (a 256-row tile would then
// be at least half padding).
// Returns SZO_EUNSUPPORTED when the stack does not qualify (the caller then launches per matrix):
// mixed tile types or formats, a table that does not fit the workspace, or too few tiles to fill the chip.
// On success *partials_per_sign is the number of loss partials of one sign: the "+" partials are
// partials[0 .. T), the "-" partials partials[T .. 2T).
static int grouped_forwards(const szo_linear_desc* descs, int n, uint64_t seed, uint64_t step, float eps,
                            void* table_dev, double* partials, int64_t* partials_per_sign, hipStream_t stream) {
  if (g_tile_config == 1) return SZO_EUNSUPPORTED;
  int64_t max_m = 0;
  for (int i = 0; i < n; ++i) max_m = std::max<int64_t>(max_m, descs[i].N > 0 ? descs[i].M : 0);
  const bool auto_tiles = g_tile_config == 0 || g_tile_config >= 4;
  const int tile = (auto_tiles && n > 0 && descs[0].format == SZO_FORMAT_UNIFORM && max_m <= 128) ? 128 : 256;
  // Dual-sign tiles (one workgroup computes both forwards of 256 x 128 outputs and dequantises the weights
  // once for both) when the library chooses the tiles and no layer has a second activation set.
  bool dual = auto_tiles && tile == 256 && n > 0 && descs[0].format == SZO_FORMAT_UNIFORM;
  for (int i = 0; dual && i < n; ++i) dual = descs[i].x_minus == nullptr;
  const int tile_n = dual ? tile / 2 : tile;
  int64_t T = 0, wgs = 0;          // loss partials per sign; workgroups of the launch
  int live = 0;
  for (int i = 0; i < n; ++i) {
    const szo_linear_desc* d = &descs[i];
    if (d->M == 0 || d->N == 0) continue;
    if (d->tile_dtype != descs[0].tile_dtype || d->format != descs[0].format) return SZO_EUNSUPPORTED;
    const int64_t t = (int64_t)((d->M + tile - 1) / tile) * ((d->N + tile_n - 1) / tile_n);
    T += t;
    wgs += dual ? t : 2 * t;
    ++live;
  }
  if ((wgs < 384 && g_tile_config != 3 && g_tile_config != 6) || T == 0 || 2 * T > kMaxLossPartials) return SZO_EUNSUPPORTED;
  if (sizeof(FwdParams) * (size_t)live > kTableBytesPerMatrix * (size_t)kMaxStepMatrices) return SZO_EUNSUPPORTED;
  static thread_local std::vector<FwdParams> table;
  table.clear();
  int64_t first_block = 0, offset = 0;
  for (int i = 0; i < n; ++i) {
    const szo_linear_desc* d = &descs[i];
    if (d->M == 0 || d->N == 0) continue;
    const double scale = 1.0 / ((double)d->M * (double)d->N);
    const int gm = (int)((d->M + tile - 1) / tile), gn = (int)((d->N + tile_n - 1) / tile_n);
    FwdParams p;
    const int rc = fill_params(p, d, seed, step, +1, eps, partials + offset, scale);
    if (rc != SZO_OK) return rc;
    p.x_minus = d->x_minus ? (const uint16_t*)d->x_minus : p.x;
    p.partials_minus = partials + T + offset;
    p.grid_m = gm; p.grid_n = gn;
    p.y = nullptr;                                          // the step's fused path never writes y
    p.first_block = (int)first_block;
    table.push_back(p);
    first_block += ((dual ? 1 : 2) * (int64_t)gm * gn + 7) & ~(int64_t)7;
    if (first_block > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
    offset += (int64_t)gm * gn;
  }
  int rc = stage_table(table.data(), sizeof(FwdParams) * table.size(), table_dev, stream);
  if (rc != SZO_OK) return rc;
  *partials_per_sign = T;
  if (descs[0].format == SZO_FORMAT_LUT)
    return launch_table<SZO_TILE_F16, SZO_FORMAT_LUT>((const FwdParams*)table_dev, (int)table.size(), first_block, stream);
  if (tile == 128) {
    if (descs[0].tile_dtype == SZO_TILE_F16)
      return launch_table<SZO_TILE_F16, SZO_FORMAT_UNIFORM, 128>((const FwdParams*)table_dev, (int)table.size(), first_block, stream);
    return launch_table<SZO_TILE_BF16, SZO_FORMAT_UNIFORM, 128>((const FwdParams*)table_dev, (int)table.size(), first_block, stream);
  }
  if (dual) {
    if (descs[0].tile_dtype == SZO_TILE_F16)
      return launch_table<SZO_TILE_F16, SZO_FORMAT_UNIFORM, 256, true>((const FwdParams*)table_dev, (int)table.size(), first_block, stream);
    return launch_table<SZO_TILE_BF16, SZO_FORMAT_UNIFORM, 256, true>((const FwdParams*)table_dev, (int)table.size(), first_block, stream);
  }
  if (descs[0].tile_dtype == SZO_TILE_F16)
    return launch_table<SZO_TILE_F16>((const FwdParams*)table_dev, (int)table.size(), first_block, stream);
  return launch_table<SZO_TILE_BF16>((const FwdParams*)table_dev, (int)table.size(), first_block, stream);
}

// Device address of `scratch` on the current device, looked up once per device.
static int noalloc_partials(double** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static double* ptr[kMaxDevices] = {};
  int dev = 0;
  SZO_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SZO_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    SZO_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SZO_ELAUNCH;
    ptr[dev] = (double*)p;
  }
  *out = ptr[dev];
  return SZO_OK;
}

}  // namespace szo

using namespace szo;

extern "C" {

int szo_zo_step_noalloc(const szo_linear_desc* descs, int n, uint64_t seed, uint64_t step, float eps, float lr,
                        double* scalars, void* stream) {
  if (n < 0 || (n > 0 && !descs) || !scalars) return SZO_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  // Kernel choice as in szo_zo_step: the few-token kernel (one launch per layer, both signs) when every
  // layer qualifies for it -- here also: no layer with a second activation set, which needs the grouped
  // launch's dual kernel -- else the tiled kernel, one launch per layer and sign.
  bool few_all = few_token_enabled() && n > 0;
  for (int i = 0; few_all && i < n; ++i) {
    if (descs[i].M <= 0 || descs[i].N <= 0) continue;
    few_all = !descs[i].x_minus && small_m_step_eligible(&descs[i]);
  }
  auto few_one = [few_all](const szo_linear_desc*) { return few_all; };
  int64_t T = 0;
  for (int i = 0; i < n; ++i) {     // reject everything before anything is enqueued
    const szo_linear_desc* d = &descs[i];
    const int rc = validate_desc(d, 1, false, true);
    if (rc != SZO_OK) return rc;
    if (d->nnz > 0 && (!d->sp_val || ((uintptr_t)d->sp_val & 15))) return SZO_EINVAL;
    if (d->M == 0 || d->N == 0) continue;
    int blocks;
    if (few_one(d)) blocks = small_m_blocks(d) * small_m_slices(d);
    else plan_tiles((int)d->M, (int)d->N, d->format, &blocks);
    if (blocks < 0) return SZO_EUNSUPPORTED;
    T += blocks;
  }
  if (2 * T > kNoAllocMaxPartials) return SZO_EUNSUPPORTED;
  double* part = nullptr;
  int rc = noalloc_partials(&part);
  if (rc != SZO_OK) return rc;
  int64_t off = 0;
  for (int i = 0; i < n; ++i) {
    const szo_linear_desc* d = &descs[i];
    if (d->M == 0 || d->N == 0) continue;
    if (few_one(d)) {
      rc = small_m_launch_one(d, seed, step, eps, 1, true, part + off, part + T + off, s);
      off += small_m_blocks(d) * small_m_slices(d);
    } else {
      const double scale = 1.0 / ((double)d->M * (double)d->N);
      int blocks;
      plan_tiles((int)d->M, (int)d->N, d->format, &blocks);
      rc = run_forward(d, seed, step, +1, eps, part + off, scale, s, false);
      if (rc == SZO_OK) rc = run_forward(d, seed, step, -1, eps, part + T + off, scale, s, true);
      off += blocks;
    }
    if (rc != SZO_OK) return rc;
  }
  rc = reduce_step(part, (int)T, eps, scalars, s);
  if (rc != SZO_OK) return rc;
  for (int i = 0; i < n; ++i) {
    rc = szo_sparse_update(descs[i].sp_val, descs[i].sp_idx, descs[i].nnz, descs[i].nnz_base, seed, step,
                           scalars + 2, lr, s);
    if (rc != SZO_OK) return rc;
  }
  return SZO_OK;
}

int szo_set_tile_config(int config) {
  if (config < 0 || config > 7) return SZO_EINVAL;
  g_tile_config = config;
  small_m_force_rblocks(config == 4 ? 2 : config == 5 ? 3 : 0);
  small_m_force_stream_once(config == 7);
  return SZO_OK;
}

int szo_linear_fwd(const szo_linear_desc* desc, uint64_t seed, uint64_t step, int sign, float eps, void* stream) {
  const int rc = validate_desc(desc, sign, true, false);
  if (rc != SZO_OK) return rc;
  if (desc->M == 0 || desc->N == 0) return SZO_OK;
  if (few_token_enabled() && small_m_step_eligible(desc))
    return small_m_launch_one(desc, seed, step, sign == 0 ? 0.0f : eps, sign == 0 ? 1 : sign, false, nullptr, nullptr,
                              (hipStream_t)stream);
  return run_forward(desc, seed, step, sign, eps, nullptr, 0.0, (hipStream_t)stream);
}

int szo_linear_fwd_mse(const szo_linear_desc* desc, uint64_t seed, uint64_t step, int sign, float eps,
                       double scale, double* loss_acc, void* workspace, void* stream) {
  int rc = validate_desc(desc, sign, false, true);
  if (rc != SZO_OK) return rc;
  if (!loss_acc || !workspace || ((uintptr_t)workspace & 7)) return SZO_EINVAL;
  if (desc->M == 0 || desc->N == 0) return SZO_OK;
  if (few_token_enabled() && small_m_step_eligible(desc) && scale == 1.0 / ((double)desc->M * (double)desc->N)) {
    // the few-token kernel computes both signs at once: make the requested one its "+" forward
    const int nb = small_m_blocks(desc) * small_m_slices(desc);           // partials of all slices
    if (2 * nb > kMaxLossPartials) return SZO_EUNSUPPORTED;
    rc = small_m_launch_one(desc, seed, step, (float)sign * eps, 1, true, partial_area(workspace),
                            partial_area(workspace) + nb, (hipStream_t)stream);
    if (rc != SZO_OK) return rc;
    return reduce_partials(partial_area(workspace), nb, loss_acc, (hipStream_t)stream);
  }
  int blocks;
  plan_tiles((int)desc->M, (int)desc->N, desc->format, &blocks);
  if (blocks < 0 || blocks > kMaxLossPartials) return SZO_EUNSUPPORTED;
  rc = run_forward(desc, seed, step, sign, eps, partial_area(workspace), scale, (hipStream_t)stream);
  if (rc != SZO_OK) return rc;
  return reduce_partials(partial_area(workspace), blocks, loss_acc, (hipStream_t)stream);
}

int szo_zo_step(const szo_linear_desc* descs, int n, uint64_t seed, uint64_t step, float eps, float lr,
                double* scalars, void* workspace, int flags, void* stream) {
  if (n < 0 || (n > 0 && !descs) || !scalars || !workspace || ((uintptr_t)workspace & 7)) return SZO_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  // The step's descriptor tables travel through pinned host buffers that later calls reuse: a captured
  // step would replay stale tables.
  if (stream_is_capturing(s)) return SZO_EUNSUPPORTED;
  const bool fuse = flags & SZO_STEP_FUSED_LOSS;
  int64_t total = 0;                // workgroups = loss partials of one pass
  for (int i = 0; i < n; ++i) {     // reject everything before anything is enqueued
    const int rc = validate_desc(&descs[i], 1, !fuse, true);
    if (rc != SZO_OK) return rc;
    // the update touches every layer's values, also those of a layer without tokens
    if (descs[i].nnz > 0 && (!descs[i].sp_val || ((uintptr_t)descs[i].sp_val & 15))) return SZO_EINVAL;
    if (descs[i].M == 0 || descs[i].N == 0) continue;
    int blocks;
    plan_tiles((int)descs[i].M, (int)descs[i].N, descs[i].format, &blocks);
    if (blocks < 0) return SZO_EUNSUPPORTED;
    total += blocks;
  }
  int rc;
  // Few-token stacks: one pass over the weights serves both forwards of the step.
  bool few = fuse && few_token_enabled() && n > 0 && n <= kMaxStepMatrices;
  const bool one_pass = flags & SZO_STEP_ONE_DENSE_PASS;     // the caller asks for the slicing path at any token count
  for (int i = 0; few && i < n; ++i) {
    if (descs[i].M == 0 || descs[i].N == 0) continue;        // an empty layer contributes nothing on either path
    few = one_pass ? small_m_shape_eligible(&descs[i]) : small_m_step_eligible(&descs[i]);
  }
  if (few) {
    rc = small_m_step(descs, n, seed, step, eps, lr, (char*)workspace + kWorkspaceTableOffset,
                      partial_area(workspace), scalars, true, true, s);
    if (rc != SZO_EUNSUPPORTED) return rc;      // too many slices for the table: nothing was enqueued, take the tiled path
  }
  bool grouped = false;
  if (fuse) {
    int64_t T = 0;
    rc = grouped_forwards(descs, n, seed, step, eps, (char*)workspace + kWorkspaceTableOffset, partial_area(workspace),
                          &T, s);
    if (rc == SZO_OK) {
      grouped = true;
      rc = reduce_step(partial_area(workspace), (int)T, eps, scalars, s);
      if (rc != SZO_OK) return rc;
    } else if (rc != SZO_EUNSUPPORTED) {
      return rc;
    }
  }
  if (!grouped) {
    if (fuse && 2 * total > kMaxLossPartials) return SZO_EUNSUPPORTED;
    if (!fuse) {
      rc = zero_words(scalars, 6, s);
      if (rc != SZO_OK) return rc;
    }
    for (int pass = 0; pass < 2; ++pass) {
      const int sign = pass == 0 ? +1 : -1;
      double* part = partial_area(workspace) + (size_t)pass * (size_t)total;
      for (int i = 0; i < n; ++i) {
        const szo_linear_desc* d = &descs[i];
        if (d->M == 0 || d->N == 0) continue;
        const double scale = 1.0 / ((double)d->M * (double)d->N);
        if (fuse) {
          int blocks;
          plan_tiles((int)d->M, (int)d->N, d->format, &blocks);
          rc = run_forward(d, seed, step, sign, eps, part, scale, s, pass == 1);
          part += blocks;
        } else {
          rc = run_forward(d, seed, step, sign, eps, nullptr, 0.0, s, pass == 1);
          if (rc == SZO_OK) rc = szo_mse_loss(d->y, d->target, d->M * d->N, scale, scalars + pass, workspace, s);
        }
        if (rc != SZO_OK) return rc;
      }
    }
    rc = fuse ? reduce_step(partial_area(workspace), (int)total, eps, scalars, s)
              : szo_spsa_g(scalars, scalars + 1, eps, scalars + 2, s);
    if (rc != SZO_OK) return rc;
  }
  // one grouped update launch for the whole stack (per-matrix launches when the table does not fit)
  if (n <= kMaxStepMatrices && small_m_table_bytes(n) <= kTableBytesPerMatrix * (size_t)kMaxStepMatrices)
    return small_m_step(descs, n, seed, step, eps, lr, (char*)workspace + kWorkspaceTableOffset, nullptr, scalars,
                        false, true, s);
  for (int i = 0; i < n; ++i) {
    rc = szo_sparse_update(descs[i].sp_val, descs[i].sp_idx, descs[i].nnz, descs[i].nnz_base, seed, step,
                           scalars + 2, lr, s);
    if (rc != SZO_OK) return rc;
  }
  return SZO_OK;
}

}  // extern "C"
