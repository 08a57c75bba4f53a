// Few-token path (16 or 32 token rows per pass; the host slices up to 128 tokens): the forward is bound by
// streaming the 4-bit weights from HBM, not by the matrix cores, and the paper's own guideline for this regime (Appendix C.5) is the
// SparseAddMM association:   y = x Dequantize(Q(w_dense))^T  +  x w_sparse^T.
// Two consequences shape this kernel:
//   * the dense product does not depend on the perturbation, so ONE pass over the weights
//     serves both the +eps and the -eps forward of a ZO step (Definition 1 needs f at both);
//   * the sparse weights are  v +- eps z  (Section 3.4), so the sparse product splits into
//     a = x v^T  (added to the dense part) and  b = x z^T:  y(+-) = dense + a +- eps b.
//
// One workgroup = 256 output columns (4 bands of 64 rows of W, one wave each) x all of K, walked in
// chunks of 256 columns of x that are staged in LDS as fp16 (16 or 32 token rows, zero padded).  The
// kernel is written for several small waves per SIMD (~150 registers, ~30 KB of LDS per workgroup):
// a streaming-read probe on this chip reaches its ceiling with a few 16-byte loads in flight per
// wave as long as enough waves are resident, and the resident waves hide each other's stalls.
// Per chunk a wave
//   - streams its band's codes, 16 bytes per lane, one 128-column block ahead, and turns them in registers into
//     the B operand of v_mfma_f32_16x16x32_f16 (no LDS round trip: every weight is used once).
//     With a quantisation group of 128 the codes are NOT re-centred: 0x6400|c reads 1024+c and
//     0x5400|(c<<4) reads 64+c, both exact in fp16, and the constant part
//     sum_k x[m,k] (1032 | 72) of each 128-column block comes out of one more MFMA chain per block
//     against a constant operand and seeds the chains of the block's four subtiles, negated.  The
//     block's partial product then takes the group scale in fp32.
//   - keeps a ring of its band's sensitive entries in LDS (position, fp16 v, fp16 z; z from the
//     same Philox/Box-Muller routine and counters as the large-batch kernel and the update, 256
//     entries per refill so that all lanes work), and multiplies them in groups of 16 entries as a
//     second, tiny MFMA: A = the entries' columns of x (gathered from LDS), B = a one-hot matrix
//     that routes entry e to its row (value v or z).  No atomics, no read-modify-write chains.
// The epilogue forms y(+-) and either stores y for the requested sign or folds the squared error
// against the target into two fp64 partials per workgroup (one per sign).
// Everything is accumulated in a fixed order: results are bit-reproducible.
#include <algorithm>
#include <cstddef>
#include <vector>
#include "szo_internal.h"
#include "szo_rng.h"

namespace szo {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

constexpr int SM_ROWS = 16;             // token rows of the MFMA (M padded up to this)
constexpr int SM_BN = 256;              // output columns per workgroup = 4 bands of 64
constexpr int SM_KC = 256;              // columns of x staged per chunk (double buffered) = 2 blocks of 128
constexpr int SM_XSTRIDE = SM_KC + 8;   // LDS row stride of x in fp16 elements (+16 B against bank conflicts)
constexpr int SM_WIN = 256;             // sensitive entries computed per refill (4 per lane)
constexpr int SM_CAP = 512;             // entries held per band (ring)
#ifndef SM_MIN_BLOCKS
#define SM_MIN_BLOCKS 4                 // workgroups per CU the register budget of a 16-row pass is set for (<= 128 registers, no spills;
                                        // the table format keeps its tables in 32 more registers: three workgroups)
#endif

struct SmallMat {
  const uint16_t* x;        // bf16 [M,K]
  const uint16_t* x2;       // bf16 [M,K] or null: the -eps forward's activations where they differ (DUAL kernels)
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
  int M;                    // token rows of this entry (<= 16 or <= 32, by instantiation): longer matrices are split into slices
  uint32_t nnz;
  int group_shift;
  uint32_t div_mul;
  int div_shift;
  int first_block;          // workgroups of earlier matrices in this launch
  int partial_base;         // index of this matrix's first loss partial
  int64_t first_quad;       // threads of earlier matrices in the grouped update (one per Philox counter = 4 entries,
                            // rounded up to whole waves of 64 per matrix)
};

static_assert(sizeof(SmallMat) <= kTableBytesPerMatrix, "table entries must fit the workspace's table area");

struct SmallArgs {
  const SmallMat* table;    // device table of n_mats matrices, or null: use `one`
  SmallMat one;
  int n_mats;
  int slices;               // slices of token rows per strip in this launch (the longest matrix's count)
  int stream_once;          // host's choice: load the codes as a non-temporal stream (see small_m_kernel, ONCE)
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

// (a & mask) | bits: one v_and_or_b32 when `bits` is in a register.  Plain C on purpose.  As inline assembly
// the instruction is opaque to the compiler's hazard handling, which keeps two wait states between a vector
// instruction that writes a register and a matrix instruction that reads it: here the result IS a matrix
// operand, and with the assembly form sequences with a single wait state were generated (harmless while
// other waves share the SIMD and issue in between, wrong products for a wave that has the SIMD to itself).
__device__ __forceinline__ uint32_t sm_and_or(uint32_t a, uint32_t mask, uint32_t bits_vgpr) {
  return (a & mask) | bits_vgpr;
}

// 8 codes -> 8 fp16 values in the order (0,4)(1,5)(2,6)(3,7).
// RAW: 1024+c for even positions and 64+c for odd ones (the caller removes the constants);
// otherwise (c - 8) times the group scale.
template <bool RAW>
__device__ __forceinline__ half8_t sm_dequant_word(uint32_t q, uint32_t magic_lo, uint32_t magic_hi, half2_t s2) {
  const uint32_t q8 = q >> 8;
  half2_t h0 = __builtin_bit_cast(half2_t, sm_and_or(q, 0x000F000Fu, magic_lo));
  half2_t h1 = __builtin_bit_cast(half2_t, sm_and_or(q, 0x00F000F0u, magic_hi));
  half2_t h2 = __builtin_bit_cast(half2_t, sm_and_or(q8, 0x000F000Fu, magic_lo));
  half2_t h3 = __builtin_bit_cast(half2_t, sm_and_or(q8, 0x00F000F0u, magic_hi));
  if (!RAW) {
    const half2_t off_lo = {(_Float16)1032.0f, (_Float16)1032.0f}, off_hi = {(_Float16)72.0f, (_Float16)72.0f};
    h0 = (h0 - off_lo) * s2; h1 = (h1 - off_hi) * s2; h2 = (h2 - off_lo) * s2; h3 = (h3 - off_hi) * s2;
  }
  half8_t r;
  r[0] = h0[0]; r[1] = h0[1]; r[2] = h1[0]; r[3] = h1[1];
  r[4] = h2[0]; r[5] = h2[1]; r[6] = h3[0]; r[7] = h3[1];
  return r;
}

// word w of the staged form of 8 bf16 values: (x[w], x[w+4]) as fp16
__device__ __forceinline__ uint32_t sm_stage_x_word(u32x4 u, int w) {
  const uint32_t first = (w < 2) ? u[0] : u[1], second = (w < 2) ? u[2] : u[3];
  float a, b;
  if ((w & 1) == 0) { a = __uint_as_float(first << 16); b = __uint_as_float(second << 16); }
  else              { a = __uint_as_float(first & 0xFFFF0000u); b = __uint_as_float(second & 0xFFFF0000u); }
  auto h = __builtin_amdgcn_cvt_pkrtz(a, b);
  return __builtin_bit_cast(uint32_t, h);
}

// Eight codes of one row -> eight fp16 table values in the order (0,4)(1,5)(2,6)(3,7).  The row's table of 16
// entries is held as four byte planes T = {low bytes of entries 0-7, high bytes of 0-7, low bytes of 8-15,
// high bytes of 8-15}, two registers each: the byte permute looks up four codes at a time by their low
// three bits, and bit 3 picks the plane through a byte mask.
__device__ __forceinline__ half8_t sm_lut_word(uint32_t q, const uint32_t (&T)[8]) {
  const uint32_t sel_e = q & 0x07070707u, sel_o = (q >> 4) & 0x07070707u;         // even codes 0,2,4,6 | odd codes 1,3,5,7
  const uint32_t m_e = __builtin_amdgcn_perm(0u, 0x0000FF00u, (q >> 3) & 0x01010101u);   // 0xFF where the code is >= 8
  const uint32_t m_o = __builtin_amdgcn_perm(0u, 0x0000FF00u, (q >> 7) & 0x01010101u);
  auto pick = [](uint32_t m, uint32_t b, uint32_t a) { return (m & b) | (~m & a); };
  const uint32_t lo_e = pick(m_e, __builtin_amdgcn_perm(T[5], T[4], sel_e), __builtin_amdgcn_perm(T[1], T[0], sel_e));
  const uint32_t hi_e = pick(m_e, __builtin_amdgcn_perm(T[7], T[6], sel_e), __builtin_amdgcn_perm(T[3], T[2], sel_e));
  const uint32_t lo_o = pick(m_o, __builtin_amdgcn_perm(T[5], T[4], sel_o), __builtin_amdgcn_perm(T[1], T[0], sel_o));
  const uint32_t hi_o = pick(m_o, __builtin_amdgcn_perm(T[7], T[6], sel_o), __builtin_amdgcn_perm(T[3], T[2], sel_o));
  const u32x4 w = {__builtin_amdgcn_perm(hi_e, lo_e, 0x06020400u),      // codes 0, 4
                   __builtin_amdgcn_perm(hi_o, lo_o, 0x06020400u),      // codes 1, 5
                   __builtin_amdgcn_perm(hi_e, lo_e, 0x07030501u),      // codes 2, 6
                   __builtin_amdgcn_perm(hi_o, lo_o, 0x07030501u)};     // codes 3, 7
  return __builtin_bit_cast(half8_t, w);
}

// MODE 1 (uniform format, quantisation group of 128): the scales of a block's four subtiles are
// prefetched with one 8-byte load and applied to each block's partial product, and the codes stay
// un-centred as described at the top.  MODE 0 (the other group sizes): the scale is read from memory
// where it is needed and applied to every element before the product (a plain, slower path).
// MODE 2 (table format): dq = lut[row][code]; a lane keeps the tables of its four rows in registers
// (32 of them; it needs neither scales nor the constants of the un-centred codes, so it still fits
// the register budget of three workgroups per CU).
// R = 16-row blocks of tokens per pass (1, 2 or 3).  With R > 1 every dequantised operand is multiplied
// with R blocks of token rows, so that matrices with more than 16 tokens stream their weights less
// often; each block costs 48 more registers (accumulators and activation operands): 196 and 253
// registers, i.e. two workgroups per CU instead of three.
constexpr int SM_PLAIN = 0, SM_FAST = 1, SM_LUT = 2;
// DUAL (R = 2 only): the two forwards read different activations (x for +eps, x2 for -eps).  Block 0 then
// holds 16 token rows of x and block 1 the same rows of x2: still one pass over the weights for both
// signs, but nothing else is shared, and y(+) = acc[0] + eps accz[0], y(-) = acc[1] - eps accz[1].
// ONCE: the codes are loaded as a non-temporal stream.  The host chooses it for launches that read every byte of
// their codes exactly once (one slice per strip) and stream more of them than the chip's last-level cache
// holds: they then do not displace what IS re-read -- the activations (by every strip of a matrix), the sparse
// values (by the update that follows).  Measured on a 32-block 7B-shaped stack at 16 tokens: 625 -> 592 us per
// launch, update 23.3 -> 21.3 us.  With several slices the slices of a strip share the codes through the L2
// and the hint costs 2 % (64 tokens) to 10 % (224 tokens); a stack that fits the last-level cache (one or two
// decoder blocks) is re-read from there step after step and loses 6 % with the hint: plain loads in both
// cases.  (A run-time choice between the two loads is folded into one plain load by the compiler, hence a
// template parameter.)
template <int MODE, int R, bool DUAL = false, bool ONCE = false>
__global__ void __launch_bounds__(256, R == 1 ? (MODE == SM_LUT ? 3 : SM_MIN_BLOCKS) : 2) small_m_kernel(SmallArgs a) {
  static_assert(R >= 1 && R <= 3, "one to three blocks of 16 token rows");
  static_assert(!DUAL || R == 2, "two activation sets: one block of rows each");
  constexpr bool FAST = MODE == SM_FAST, LUT = MODE == SM_LUT;
  constexpr int ROWS = SM_ROWS * R;                          // rows of activations staged per pass
  constexpr int TOK = DUAL ? SM_ROWS : ROWS;                 // token rows of one pass
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  _Float16* const xs = reinterpret_cast<_Float16*>(smem);                        // [2][ROWS][SM_XSTRIDE]
  uint16_t* const winp = reinterpret_cast<uint16_t*>(xs + 2 * ROWS * SM_XSTRIDE);      // [4 bands][SM_CAP] packed position (see refill)
  uint16_t* const winv = winp + 4 * SM_CAP;                                        // fp16 bits of v
  uint16_t* const winz = winv + 4 * SM_CAP;                                        // fp16 bits of z

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Workgroup ids go round-robin over the 8 XCDs, each with its own L2.  Remap them so that eight
  // consecutive strips (normally of one matrix, which all read the same x) run on one XCD and
  // consecutive groups of eight rotate over the XCDs; the ragged tail (< 64 ids) keeps its order.
  int bid = (int)blockIdx.x;
  if (bid < (int)(gridDim.x & ~63u)) {
    const int xcd = bid & 7, i = bid >> 3;
    bid = (((i >> 3) << 3) + xcd) * 8 + (i & 7);
  }
  // ---- which slice of token rows, which matrix, which 256-column strip ----
  // Consecutive (remapped) ids are the slices of one strip: they read the same weights, so they should
  // run at the same time on the same XCD and share them through its L2.
  const int slice = bid % a.slices;
  bid /= a.slices;
  // The table entry is read through the constant address space (scalar loads: the table is written
  // before the launch and never during it), so that its fields live in scalar registers like the
  // kernel arguments do; read through a generic pointer they would occupy ~30 vector registers.
  SmallMat mt = a.one;
  if (a.table) {
    constexpr int W = (int)(sizeof(SmallMat) / 4), FB = (int)(offsetof(SmallMat, first_block) / 4);
    static_assert(sizeof(SmallMat) % 4 == 0 && offsetof(SmallMat, first_block) % 4 == 0, "table entry is read as words");
    const auto* tab = (const uint32_t __attribute__((address_space(4)))*)a.table;
    int lo = 0, hi = a.n_mats - 1;                          // last matrix whose first_block <= bid
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if ((int)tab[mid * W + FB] <= bid) lo = mid; else hi = mid - 1;
    }
    struct Words { uint32_t w[W]; } raw;
#pragma unroll
    for (int i = 0; i < W; ++i) raw.w[i] = tab[lo * W + i];
    mt = __builtin_bit_cast(SmallMat, raw);
  }
  // a launch has as many slices of TOK token rows per strip as its longest matrix needs
  if (slice * TOK >= mt.M) return;
  mt.x += (size_t)slice * TOK * (size_t)mt.K;
  if (DUAL) mt.x2 += (size_t)slice * TOK * (size_t)mt.K;
  if (mt.target) mt.target += (size_t)slice * TOK * (size_t)mt.N;
  if (mt.y) mt.y += (size_t)slice * TOK * (size_t)mt.N;
  mt.M = min(TOK, mt.M - slice * TOK);
  mt.partial_base += slice * ((mt.N + SM_BN - 1) / SM_BN);      // slice i of a matrix: partials [i * strips ..)
  // Pointers read out of a table are generic to the compiler; say that they are global memory, or
  // every access becomes a flat load with conservative waits on both memory counters.
#define SZO_GLOBAL(T, p) ((const T __attribute__((address_space(1)))*)(p))
  const auto g_x = SZO_GLOBAL(uint16_t, mt.x);
  const auto g_x2 = SZO_GLOBAL(uint16_t, DUAL ? mt.x2 : mt.x);
  const auto g_q = SZO_GLOBAL(uint8_t, mt.qweight);
  const auto g_scales = SZO_GLOBAL(uint16_t, mt.scales);
  const auto g_tile_ptr = SZO_GLOBAL(uint32_t, mt.tile_ptr);
  const auto g_sp_idx = SZO_GLOBAL(uint32_t, mt.sp_idx);
  const auto g_sp_val = SZO_GLOBAL(float, mt.sp_val);
  const auto g_target = SZO_GLOBAL(uint16_t, mt.target);
  float __attribute__((address_space(1)))* const g_y = (float __attribute__((address_space(1)))*)mt.y;
  const int strip = bid - mt.first_block;
  const int n0 = strip * SM_BN;
  const int N = mt.N, K = mt.K, M = mt.M;
  const int ktiles = K >> 6;
  const int band = (n0 >> 6) + wave;                        // band of the sparse layout owned by this wave
  const bool band_ok = band * 64 < N && mt.nnz > 0;
  const int nn = lane & 15, jj = lane >> 4;                 // B operand: column nn of a 16-column subtile, k-group jj
  const int nchunks = (K + SM_KC - 1) / SM_KC;
  const int nkb_total = K >> 7;

  uint32_t magic_lo = 0x64006400u, magic_hi = 0x54005400u;
  asm volatile("" : "+v"(magic_lo), "+v"(magic_hi));
  // B operand of the constant-part chain: every column holds -(1032, 1032, 72, 72, 1032, 1032, 72, 72), the
  // offsets of the un-centred codes in the element order (0,4)(1,5)(2,6)(3,7)
  const half8_t minus_offsets = {(_Float16)-1032.0f, (_Float16)-1032.0f, (_Float16)-72.0f, (_Float16)-72.0f,
                                 (_Float16)-1032.0f, (_Float16)-1032.0f, (_Float16)-72.0f, (_Float16)-72.0f};

  uint16_t* const my_winp = winp + wave * SM_CAP;
  uint16_t* const my_winv = winv + wave * SM_CAP;
  uint16_t* const my_winz = winz + wave * SM_CAP;

  float4_t acc[R][4], accz[R][4];                           // per block of 16 token rows: dense + x v^T ;  x z^T
#pragma unroll
  for (int rb = 0; rb < R; ++rb)
#pragma unroll
    for (int s = 0; s < 4; ++s) { acc[rb][s] = float4_t{0.0f, 0.0f, 0.0f, 0.0f}; accz[rb][s] = float4_t{0.0f, 0.0f, 0.0f, 0.0f}; }

  // Banded layout (see the header): the band's 64 rows of one 64-column tile are 2 KB in a row, so
  // the 16 rows x 32 bytes that the lanes of one k-group pair read are contiguous, and a lane's four
  // scales of a group (rows nn, nn+16, nn+32, nn+48) are 8 bytes in a row.  Bands past N re-read the
  // last band: their outputs are never used.  32-bit byte offsets from the uniform base pointers
  // take half the registers of per-lane pointers.
  const uint32_t bsafe = (uint32_t)min(band, (N + 63) / 64 - 1);
  uint32_t qoff[4];
#pragma unroll
  for (int s = 0; s < 4; ++s)
    qoff[s] = (bsafe * (uint32_t)ktiles * 64u + (uint32_t)(16 * s + nn)) * 32u + (uint32_t)(jj >> 1) * 2048u + (uint32_t)(jj & 1) * 16u;
  const int gshift = mt.group_shift;
  const uint32_t soff = (bsafe * (uint32_t)(K >> gshift) * 64u + (uint32_t)nn * 4u) * 2u;
  // table format: the tables of rows nn, nn+16, nn+32, nn+48 of the band (mt.scales is the table array);
  // rows past N re-read the last row's table, their outputs are never used
  uint32_t tb[LUT ? 4 : 1][8];
  if (LUT) {
#pragma unroll
    for (int s = 0; s < (LUT ? 4 : 1); ++s) {
      const int n = min((int)bsafe * 64 + 16 * s + nn, N - 1);
      const auto* lp = reinterpret_cast<const u32x4 __attribute__((address_space(1)))*>(g_scales + (size_t)n * 16);
      const u32x4 lo = lp[0], hi = lp[1];                   // entries 0-7 and 8-15, two per word
      tb[s][0] = __builtin_amdgcn_perm(lo[1], lo[0], 0x06040200u); tb[s][1] = __builtin_amdgcn_perm(lo[3], lo[2], 0x06040200u);
      tb[s][2] = __builtin_amdgcn_perm(lo[1], lo[0], 0x07050301u); tb[s][3] = __builtin_amdgcn_perm(lo[3], lo[2], 0x07050301u);
      tb[s][4] = __builtin_amdgcn_perm(hi[1], hi[0], 0x06040200u); tb[s][5] = __builtin_amdgcn_perm(hi[3], hi[2], 0x06040200u);
      tb[s][6] = __builtin_amdgcn_perm(hi[1], hi[0], 0x07050301u); tb[s][7] = __builtin_amdgcn_perm(hi[3], hi[2], 0x07050301u);
    }
  }
  // ---- x staging: piece = 8 columns (16 bytes of bf16) of one row; thread handles pieces
  //      (row tid>>5, columns 8*(tid&31)..) and the same columns of rows 8 i + (tid>>5), i < 2 R ----
  // Loads are unconditional, from clamped addresses, and out-of-range parts are zeroed only when the
  // registers are stored to LDS: a branch or an early use here would make every later wait a full drain.
  u32x4 xr[2 * R];
  auto load_x = [&](int c) {
    const int col = min(c * SM_KC + 8 * (tid & 31), K - 8);
#pragma unroll
    for (int i = 0; i < 2 * R; ++i) {
      const int row = (tid >> 5) + 8 * i;                   // DUAL: staged rows 16.. are token rows 0.. of x2
      const int m = min(DUAL ? (row & 15) : row, M - 1);
      xr[i] = *reinterpret_cast<const u32x4 __attribute__((address_space(1)))*>(((DUAL && i >= 2) ? g_x2 : g_x) + (size_t)m * K + col);
    }
  };
  auto store_x = [&](int c) {
    const int ch = tid & 31, buf = c & 1;
    const bool col_ok = c * SM_KC + 8 * ch < K;
#pragma unroll
    for (int i = 0; i < 2 * R; ++i) {
      const int m = (tid >> 5) + 8 * i;
      const bool ok = col_ok && (DUAL ? (m & 15) : m) < M;
      u32x4 o;
#pragma unroll
      for (int w = 0; w < 4; ++w) o[w] = ok ? sm_stage_x_word(xr[i], w) : 0u;
      *reinterpret_cast<u32x4*>(xs + (buf * ROWS + m) * SM_XSTRIDE + 8 * ch) = o;
    }
  };

  // ---- code stream: slot kbl*4+s holds subtile s of the chunk's 128-column block kbl ----
#ifndef SM_RING
#define SM_RING 1                       // 128-column blocks of codes in flight per wave (1 or 2)
#endif
  // slot (b % SM_RING)*4 + s: subtile s of 128-column block b.  With two blocks in flight the stream
  // keeps running while the wave is busy with the sparse part and the barrier of a chunk.
  constexpr int RING = SM_RING;             // (two blocks in flight measured no faster with R = 2 either)
  u32x4 qbuf[4 * RING];
  auto load_q = [&](int slot, int gkb) {
    const auto* src = reinterpret_cast<const u32x4 __attribute__((address_space(1)))*>(g_q + (size_t)min(gkb, nkb_total - 1) * 4096 + qoff[slot & 3]);
    qbuf[slot] = ONCE ? __builtin_nontemporal_load(src) : *src;
  };
#pragma unroll
  for (int i = 0; i < 4 * RING; ++i) load_q(i, i >> 2);
  u32x2 sc[2] = {u32x2{0u, 0u}, u32x2{0u, 0u}};             // FAST: block kbl of the chunk: the lane's four scales (s = 0..3)
  auto load_scales = [&](int c) {
#pragma unroll
    for (int kbl = 0; kbl < 2; ++kbl)
      sc[kbl] = *reinterpret_cast<const u32x2 __attribute__((address_space(1)))*>(
          reinterpret_cast<const uint8_t __attribute__((address_space(1)))*>(g_scales) +
          (size_t)min(2 * c + kbl, nkb_total - 1) * 128 + soff);
  };
  if (FAST) load_scales(0);
  load_x(0);

  // ---- sensitive entries of this band: boundaries per chunk, ring of entries in LDS ----
  auto tp_at = [&](int c) -> uint32_t {                     // first entry of the band at or after chunk c
    return band_ok ? g_tile_ptr[(uint32_t)band * (uint32_t)ktiles + (uint32_t)min(c * (SM_KC / 64), ktiles)] : 0u;
  };
  uint32_t tp0 = tp_at(0), tp1 = tp_at(1);
  uint32_t w_hi = __builtin_amdgcn_readfirstlane(tp0) & ~3u;      // entries below w_hi have been generated
  // A refill is only reached with band_ok (some entry of the band is wanted), so nnz > 0 there.  Its
  // loads are issued where they are used: refills are rare (256 entries each) and the other resident
  // waves cover the wait, while holding the values across the dense loop would cost 8 registers.
  auto refill = [&]() {
    const uint32_t j = w_hi + 4u * lane;
    uint32_t pf_idx[4];
    float pf_val[4];
    {
      const uint32_t last = mt.nnz - 1u;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t je = min(j + e, last);               // clamped; entries past the end are never consumed
        pf_idx[e] = g_sp_idx[je];
        pf_val[e] = g_sp_val[je];
      }
    }
    float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (a.eps != 0.0f) zbar_quad((mt.nnz_base + j) >> 2, a.seed, a.step, z);
    uint32_t p[4];
    half4_t vh, zh;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t flat = pf_idx[e];
      const uint32_t n = sm_fast_div(flat, mt.div_mul, mt.div_shift);
      const uint32_t r = n - (uint32_t)(band * 64);
      const uint32_t k = flat - n * (uint32_t)K;
      // window word: bits 0-7 position of the column inside the staged chunk row, 8-11 row mod 16, 12-13 subtile
      p[e] = (uint32_t)sm_xpos((int)(k & (uint32_t)(SM_KC - 1))) | ((r & 15u) << 8) | (((r >> 4) & 3u) << 12);
      vh[e] = (_Float16)pf_val[e];
      zh[e] = (_Float16)z[e];
    }
    const uint32_t ring = j & (uint32_t)(SM_CAP - 1);
    *reinterpret_cast<u32x2*>(my_winp + ring) = u32x2{p[0] | (p[1] << 16), p[2] | (p[3] << 16)};
    *reinterpret_cast<u32x2*>(my_winv + ring) = __builtin_bit_cast(u32x2, vh);
    *reinterpret_cast<u32x2*>(my_winz + ring) = __builtin_bit_cast(u32x2, zh);
    w_hi += SM_WIN;
  };

  store_x(0);
  __syncthreads();

  for (int c = 0; c < nchunks; ++c) {
    const int kc = c * SM_KC;
    const _Float16* const xc = xs + (c & 1) * ROWS * SM_XSTRIDE;
    const uint32_t tp2 = tp_at(c + 2);
    // next chunk's x: requested before the dense part, so that it has landed when the (short) sparse part
    // is over and store_x wants it (two blocks of rows: 64 tokens 1.547 -> 1.535 ms; one block measured no gain,
    // and with three there are no registers to hold it that long)
    constexpr bool EARLY_X = R == 2;
    if (EARLY_X) load_x(min(c + 1, nchunks - 1));           // the last chunk re-reads itself; never stored

    // ---- dense: stream this band's codes ----
#pragma unroll
    for (int kbl = 0; kbl < 2; ++kbl) {
      // blocks past the end of K multiply clamped codes with the zeros staged for x: no branch needed
      // R = 1: the activation operands are read from LDS where they are used (16 registers less, which is
      // what lets four workgroups share a CU); with more blocks of rows they are read once per block.
      constexpr bool AF_LATE = R == 1;
      auto read_af = [&](int rb, int t) {
        return *reinterpret_cast<const half8_t*>(xc + (16 * rb + nn) * SM_XSTRIDE + kbl * 128 + 32 * jj + 8 * t);
      };
      half8_t af[AF_LATE ? 1 : R][AF_LATE ? 1 : 4];
      if (!AF_LATE) {
#pragma unroll
        for (int rb = 0; rb < R; ++rb)
#pragma unroll
          for (int t = 0; t < 4; ++t) af[rb][t] = read_af(rb, t);
      }
      auto af_of = [&](int rb, int t) { return AF_LATE ? read_af(rb, t) : af[AF_LATE ? 0 : rb][AF_LATE ? 0 : t]; };
      // FAST: minus the constant part of the un-centred codes, sum_k x[m,k] (1032 | 72) over the block, from
      // one more MFMA chain against a constant operand; it seeds the four subtiles' chains.
      float4_t init[R];
#pragma unroll
      for (int rb = 0; rb < R; ++rb) {
        init[rb] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
        if (FAST) {
#pragma unroll
          for (int t = 0; t < 4; ++t) init[rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af_of(rb, t), minus_offsets, init[rb], 0, 0, 0);
        }
      }
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        constexpr int kRingMask = RING - 1;
        const int slot = (kbl & kRingMask) * 4 + s;
        const u32x4 q = qbuf[slot];
        load_q(slot, 2 * c + kbl + RING);                   // the slot is free: fetch the block RING ahead
        _Float16 sh = (_Float16)0.0f;
        if (FAST) {
          sh = __builtin_bit_cast(half4_t, sc[kbl])[s];
        } else if (!LUT) {
          const uint32_t gi = (uint32_t)min((kc + kbl * 128 + 32 * jj) >> gshift, (K >> gshift) - 1);
          sh = __builtin_bit_cast(_Float16, *reinterpret_cast<const uint16_t __attribute__((address_space(1)))*>(
              reinterpret_cast<const uint8_t __attribute__((address_space(1)))*>(g_scales) + (size_t)gi * 128 + soff + 2 * s));
        }
        const half2_t s2 = {sh, sh};
        float4_t tmp[R];
#pragma unroll
        for (int rb = 0; rb < R; ++rb) tmp[rb] = init[rb];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const half8_t b = LUT ? sm_lut_word(q[t], tb[LUT ? s : 0]) : sm_dequant_word<FAST>(q[t], magic_lo, magic_hi, s2);
#pragma unroll
          for (int rb = 0; rb < R; ++rb) tmp[rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af_of(rb, t), b, tmp[rb], 0, 0, 0);
        }
#pragma unroll
        for (int rb = 0; rb < R; ++rb) {
          if (FAST) {
            const float sf = (float)sh;                      // column nn of the subtile: the lane's own row of W
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[rb][s][r] = fmaf(tmp[rb][r], sf, acc[rb][s][r]);
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[rb][s][r] += tmp[rb][r];
          }
        }
        // keep the subtiles in program order: hoisting the later ones' loads and unpacking costs registers,
        // and the latency they would hide is covered by the other resident waves
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // next chunk's x and scales: requested now that this chunk's are no longer needed, landing
    // while the sparse part runs
    if (!EARLY_X) load_x(min(c + 1, nchunks - 1));
    if (FAST) load_scales(c + 1);                           // clamped inside

    // ---- sparse: this band's entries inside the chunk, 16 at a time (4 per k-group of the MFMA) ----
    {
      const uint32_t j_lo = __builtin_amdgcn_readfirstlane(tp0), j_hi = __builtin_amdgcn_readfirstlane(tp1);
      const uint32_t span = j_hi - j_lo;
      const _Float16* const xrow = xc + nn * SM_XSTRIDE;
      for (uint32_t g0 = j_lo & ~3u; g0 < j_hi; g0 += 16u) {
        // refilling here never overwrites an entry at or above g0: w_hi < g0 + 16 and SM_WIN + 16 <= SM_CAP
        while (w_hi < min(g0 + 16u, j_hi)) refill();
        const uint32_t e0 = g0 + 4u * (uint32_t)jj;
        const uint32_t ring = e0 & (uint32_t)(SM_CAP - 1);
        const u32x2 pw = *reinterpret_cast<const u32x2*>(my_winp + ring);
        const u32x2 vw = *reinterpret_cast<const u32x2*>(my_winv + ring);
        const u32x2 zw = *reinterpret_cast<const u32x2*>(my_winz + ring);
        const uint32_t rel = e0 - j_lo;                      // wraps for entries before the chunk's first
        half4_t ax[R];
        uint32_t mlo[4], mhi[4];                            // entry i: 0xFFFF in halfword s of (mlo, mhi) iff this lane
#pragma unroll                                              // owns the entry's row in subtile s
        for (int i = 0; i < 4; ++i) {
          const uint32_t w = pw[i >> 1];
          const int sh = 16 * (i & 1);
          // Entries outside [j_lo, j_hi) are masked out below; their column field is < 256 whatever the
          // window holds, so the gather stays inside the staged row.
          const uint32_t col = __builtin_amdgcn_ubfe(w, sh, 8);
#pragma unroll
          for (int rb = 0; rb < R; ++rb) ax[rb][i] = xrow[16 * rb * SM_XSTRIDE + col];
          const bool mine = rel + (uint32_t)i < span && __builtin_amdgcn_ubfe(w, sh + 8, 4) == (uint32_t)nn;
          const uint32_t s16 = (w >> (sh + 8)) & 0x30u;     // 16 * subtile
          const uint64_t m = (uint64_t)0xFFFFu << s16;
          mlo[i] = mine ? (uint32_t)m : 0u;
          mhi[i] = mine ? (uint32_t)(m >> 32) : 0u;
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          u32x2 bv, bz;
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const uint32_t ma = (s < 2) ? mlo[2 * h] : mhi[2 * h], mb = (s < 2) ? mlo[2 * h + 1] : mhi[2 * h + 1];
            // halfword (s & 1) of ma -> low half, of mb -> high half
            const uint32_t mask = __builtin_amdgcn_perm(mb, ma, (s & 1) ? 0x07060302u : 0x05040100u);
            bv[h] = vw[h] & mask;
            bz[h] = zw[h] & mask;
          }
#pragma unroll
          for (int rb = 0; rb < R; ++rb) {
            acc[rb][s] = __builtin_amdgcn_mfma_f32_16x16x16f16(ax[rb], __builtin_bit_cast(half4_t, bv), acc[rb][s], 0, 0, 0);
            accz[rb][s] = __builtin_amdgcn_mfma_f32_16x16x16f16(ax[rb], __builtin_bit_cast(half4_t, bz), accz[rb][s], 0, 0, 0);
          }
        }
      }
    }
    tp0 = tp1; tp1 = tp2;

    if (c + 1 < nchunks) store_x(c + 1);
    __syncthreads();                                        // next chunk's x complete; this chunk's no longer read
  }

  // ---- epilogue: accumulator (rb, s), register r = token row 16*rb + 4*jj + r, column 16*s + nn of the band ----
  double lp = 0.0, lm = 0.0;
#pragma unroll
  for (int rb = 0; rb < R; ++rb)
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int nl = 16 * s + nn, n = n0 + wave * 64 + nl;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int m = (DUAL ? 0 : 16 * rb) + 4 * jj + r;     // token row
      if (m < M && n < N) {
        const float pz = a.eps * accz[rb][s][r];
        const float yp = acc[rb][s][r] + pz, ym = acc[rb][s][r] - pz;
        if (a.loss_mode) {
          const float t = __uint_as_float((uint32_t)g_target[(size_t)m * N + n] << 16);
          const float dp = yp - t, dm = ym - t;
          if (!DUAL || rb == 0) lp += (double)(dp * dp);    // DUAL: block 0 is the +eps forward, block 1 the -eps one
          if (!DUAL || rb == 1) lm += (double)(dm * dm);
        } else {
          g_y[(size_t)m * N + n] = a.store_sign > 0 ? yp : a.store_sign < 0 ? ym : acc[rb][s][r];
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
      ((double __attribute__((address_space(1)))*)a.partial_plus)[pi] = ((red[0][0] + red[0][1]) + (red[0][2] + red[0][3])) * mt.loss_scale;
      ((double __attribute__((address_space(1)))*)a.partial_minus)[pi] = ((red[1][0] + red[1][1]) + (red[1][2] + red[1][3])) * mt.loss_scale;
    }
  }
}

// Sparse ZO-SGD update of every matrix of a table in one launch (Section 3.4, fixed-parameter
// update rule): thread = one Philox counter = four consecutive entries of one matrix.  A matrix's
// counters start at a multiple of 64 threads, so a wave serves one matrix: it finds the table entry by
// a binary search on scalar loads (through the constant address space) and keeps the entry's fields in
// scalar registers.  (Searching per lane with vector loads made every wave wait for eight dependent
// memory round trips before it could touch its entries; the launch then took 27 us for 52 MB.)
__global__ void __launch_bounds__(256) sparse_update_table_kernel(const SmallMat* __restrict__ table, int n_mats,
                                                                  int64_t total_quads, uint64_t seed, uint64_t step,
                                                                  const double* __restrict__ g, float lr) {
  constexpr int W = (int)(sizeof(SmallMat) / 4), FQ = (int)(offsetof(SmallMat, first_quad) / 4);
  static_assert(offsetof(SmallMat, first_quad) % 8 == 0, "first_quad is read as two words");
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int64_t tw = (int64_t)blockIdx.x * 256 + 64 * wave;           // the wave's first thread
  if (tw >= total_quads) return;
  const auto* tab = (const uint32_t __attribute__((address_space(4)))*)table;
  int lo = 0, hi = n_mats - 1;                                        // last matrix whose first_quad <= tw
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    const int64_t fq = (int64_t)(((uint64_t)tab[mid * W + FQ + 1] << 32) | tab[mid * W + FQ]);
    if (fq <= tw) lo = mid; else hi = mid - 1;
  }
  struct Words { uint32_t w[W]; } raw;
#pragma unroll
  for (int i = 0; i < W; ++i) raw.w[i] = tab[lo * W + i];
  const SmallMat mt = __builtin_bit_cast(SmallMat, raw);
  const int64_t tq = tw + (int64_t)(threadIdx.x & 63) - mt.first_quad, j0 = 4 * tq;
  if (j0 >= (int64_t)mt.nnz) return;
  const float c = (float)((double)lr * *g);
  float z[4];
  zbar_quad((mt.nnz_base >> 2) + (uint64_t)tq, seed, step, z);
  float __attribute__((address_space(1)))* const v = (float __attribute__((address_space(1)))*)mt.sp_val + j0;
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  if (j0 + 4 <= (int64_t)mt.nnz) {
    f32x4 w = *reinterpret_cast<f32x4 __attribute__((address_space(1)))*>(v);
    w[0] = fmaf(-c, z[0], w[0]); w[1] = fmaf(-c, z[1], w[1]); w[2] = fmaf(-c, z[2], w[2]); w[3] = fmaf(-c, z[3], w[3]);
    *reinterpret_cast<f32x4 __attribute__((address_space(1)))*>(v) = w;
  } else {
    for (int i = 0; j0 + i < (int64_t)mt.nnz; ++i) v[i] = fmaf(-c, z[i], v[i]);
  }
}

// ---- host side -----------------------------------------------------------------------------

static size_t small_lds_bytes(int r) {
  return (size_t)2 * SM_ROWS * r * SM_XSTRIDE * 2 + (size_t)3 * 4 * SM_CAP * 2;
}
// Blocks of 16 token rows per pass for a matrix of a launch.  Two (half as many passes over the weights)
// only pay when the launch is large: two-block workgroups run two to a CU instead of three, and a launch
// that fits the chip in one go (measured: a single decoder block) is faster as more, smaller passes side
// by side.  `launch_wgs16` = workgroups the whole launch would have with 16 rows per pass.
constexpr int64_t kSmallWideWorkgroups = 1536;              // two rounds of the 768 workgroups the chip holds
static int g_force_rblocks = 0;                             // testing hook: 2 or 3 = that many wherever M > 16
void small_m_force_rblocks(int r) { g_force_rblocks = r; }
static int small_m_rblocks(const szo_linear_desc* d, int64_t launch_wgs16) {
  if (d->M <= SM_ROWS) return 1;
  if (g_force_rblocks) return g_force_rblocks;
  if (launch_wgs16 <= kSmallWideWorkgroups) return 1;
  // fewest passes weighted by what a pass costs (measured on a 32-block 7B stack: 0.62, 0.79, 1.0 ms)
  const int64_t cost[3] = {62 * ((d->M + 15) / 16), 79 * ((d->M + 31) / 32), 100 * ((d->M + 47) / 48)};
  int best = 0;
  for (int r = 1; r < 3; ++r) if (cost[r] < cost[best]) best = r;
  return best + 1;
}

bool small_m_eligible(const szo_linear_desc* d) {
  return d->M >= 1 && d->M <= SM_ROWS && d->N >= 1 && (d->K % 128) == 0 &&
         (d->format == SZO_FORMAT_LUT || d->group >= 32) && d->tile_dtype == SZO_TILE_F16 &&
         (uint64_t)((d->N + 63) / 64 * 64) * (uint64_t)d->K / 2 < (1ull << 32);   // 32-bit code offsets
}

// Which instantiation a matrix runs with: uniform format with a group of 128 (one scale per
// 128-column block) takes the fast one, the table format its own, everything else the plain one.
static int small_m_mode(const szo_linear_desc* d) {
  if (d->format == SZO_FORMAT_LUT) return SM_LUT;
  return d->group == 128 ? SM_FAST : SM_PLAIN;
}
// position of an instantiation (mode, row blocks) in a step's table and launch order
// (classes 9..11: two activation sets, always two blocks of rows)
constexpr int kSmallClasses = 12;
static int small_m_class(const szo_linear_desc* d, int rblocks, bool dual) {
  const int m = small_m_mode(d), mi = m == SM_FAST ? 0 : m == SM_LUT ? 1 : 2;
  return dual ? 9 + mi : 3 * mi + (rblocks - 1);
}
static bool class_dual(int cls) { return cls >= 9; }
static int class_mode(int cls) {
  const int mi = class_dual(cls) ? cls - 9 : cls / 3;
  return mi == 0 ? SM_FAST : mi == 1 ? SM_LUT : SM_PLAIN;
}
static int class_rblocks(int cls) { return class_dual(cls) ? 2 : cls % 3 + 1; }

template <int MODE, int R, bool DUAL>
static void launch_variant(dim3 blocks, const SmallArgs& a, hipStream_t stream) {
  const size_t lds = small_lds_bytes(R);
  if (a.stream_once) small_m_kernel<MODE, R, DUAL, true><<<blocks, 256, lds, stream>>>(a);
  else small_m_kernel<MODE, R, DUAL, false><<<blocks, 256, lds, stream>>>(a);
}
template <int R, bool DUAL>
static void launch_mode(int mode, dim3 blocks, const SmallArgs& a, hipStream_t stream) {
  if (mode == SM_FAST) launch_variant<SM_FAST, R, DUAL>(blocks, a, stream);
  else if (mode == SM_LUT) launch_variant<SM_LUT, R, DUAL>(blocks, a, stream);
  else launch_variant<SM_PLAIN, R, DUAL>(blocks, a, stream);
}
// Codes of a matrix in bytes, and the rule for the non-temporal stream: one slice per strip and more codes in
// the launch than the 256 MB last-level (memory-side) cache of the chip keeps from one step to the next.
constexpr int64_t kLastLevelCacheBytes = 256ll << 20;
static int64_t code_bytes(const szo_linear_desc* d) { return (int64_t)((d->N + 63) / 64 * 64) * (d->K / 2); }
static bool g_force_stream_once = false;                    // testing hook: the stream for every one-slice launch
void small_m_force_stream_once(bool on) { g_force_stream_once = on; }
static int stream_once_rule(int slices, int64_t launch_code_bytes) {
  return slices == 1 && (g_force_stream_once || launch_code_bytes > kLastLevelCacheBytes);
}

static void small_m_launch(int mode, int r, bool dual, dim3 blocks, const SmallArgs& a, hipStream_t stream) {
  if (dual) launch_mode<2, true>(mode, blocks, a, stream);
  else if (r == 1) launch_mode<1, false>(mode, blocks, a, stream);
  else if (r == 2) launch_mode<2, false>(mode, blocks, a, stream);
  else launch_mode<3, false>(mode, blocks, a, stream);
}

// The step also takes matrices with more tokens: they run as slices of 16 or 32 token rows, each a pass
// of its own over the weights.  On a 32-block 7B-shaped stack a 32-row pass takes 0.8-0.9 ms and a row of
// 256x256 tiles of the tiled kernel 6.4 ms, whatever part of its 256 rows is padding: slicing wins while
// ceil(M/32) stays below 7.5 ceil(M/256), e.g. up to 224 tokens and from 257 to 448; beyond 15 such
// slices the tiled kernel is the default (SZO_STEP_ONE_DENSE_PASS overrides that).
constexpr int kSmallMaxSlices = 15;
bool small_m_shape_eligible(const szo_linear_desc* d) {
  if (d->M < 1) return false;
  szo_linear_desc one = *d;
  one.M = 1;
  return small_m_eligible(&one);
}
bool small_m_step_eligible(const szo_linear_desc* d) {
  // two activation sets: a pass holds 16 token rows of each, so it is worth less
  const int64_t slices = (d->M + (d->x_minus ? 15 : 31)) / (d->x_minus ? 16 : 32), tile_rows = (d->M + 255) / 256;
  if (slices > kSmallMaxSlices || 2 * slices >= 15 * tile_rows) return false;
  return small_m_shape_eligible(d);
}

int small_m_blocks(const szo_linear_desc* d) { return (int)((d->N + SM_BN - 1) / SM_BN); }

static int64_t small_m_wgs16(const szo_linear_desc* d) {
  return (int64_t)small_m_blocks(d) * ((d->M + SM_ROWS - 1) / SM_ROWS);
}
static int slices_of(const szo_linear_desc* d, int rblocks, bool dual = false) {
  const int rows = dual ? SM_ROWS : SM_ROWS * rblocks;
  return (int)((d->M + rows - 1) / rows);
}
// passes of a single-matrix call
int small_m_slices(const szo_linear_desc* d) { return slices_of(d, small_m_rblocks(d, small_m_wgs16(d))); }

size_t small_m_table_bytes(int n) { return sizeof(SmallMat) * (size_t)n; }

static void fill_mat(SmallMat& m, const szo_linear_desc* d) {
  m.x = (const uint16_t*)d->x; m.x2 = (const uint16_t*)d->x_minus; m.qweight = d->qweight;
  m.scales = (const uint16_t*)(d->format == SZO_FORMAT_LUT ? d->lut : d->scales);
  m.tile_ptr = d->tile_ptr; m.sp_idx = d->sp_idx; m.sp_val = d->sp_val;
  m.target = (const uint16_t*)d->target; m.y = d->y;
  m.nnz_base = d->nnz_base;
  m.loss_scale = 1.0 / ((double)d->M * (double)d->N);
  m.N = (int)d->N; m.K = (int)d->K; m.M = (int)d->M; m.nnz = (uint32_t)d->nnz;
  int gs = 0;
  while (d->format == SZO_FORMAT_UNIFORM && (1 << gs) < d->group) ++gs;
  m.group_shift = gs;
  int l = 0;
  while ((1ull << l) < (uint64_t)m.K) ++l;
  m.div_mul = (uint32_t)((((1ull << l) - (uint64_t)m.K) << 32) / (uint64_t)m.K + 1ull);
  m.div_shift = l - 1;
  m.first_block = 0; m.partial_base = 0; m.first_quad = 0;
}

// Dynamic LDS limit of every instantiation, once per device.
template <int MODE, int R, bool DUAL>
static int set_attrs_of() {
  static std::atomic<uint64_t> done[2];
  int rc = set_lds_limit_once(done[0], (const void*)small_m_kernel<MODE, R, DUAL, false>, small_lds_bytes(R));
  if (rc != SZO_OK) return rc;
  return set_lds_limit_once(done[1], (const void*)small_m_kernel<MODE, R, DUAL, true>, small_lds_bytes(R));
}
template <int R, bool DUAL>
static int set_attrs_of_modes() {
  int rc = set_attrs_of<SM_FAST, R, DUAL>();
  if (rc == SZO_OK) rc = set_attrs_of<SM_PLAIN, R, DUAL>();
  if (rc == SZO_OK) rc = set_attrs_of<SM_LUT, R, DUAL>();
  return rc;
}
static int set_small_attrs() {
  int rc = set_attrs_of_modes<1, false>();
  if (rc == SZO_OK) rc = set_attrs_of_modes<2, false>();
  if (rc == SZO_OK) rc = set_attrs_of_modes<3, false>();
  if (rc == SZO_OK) rc = set_attrs_of_modes<2, true>();
  return rc;
}

// One matrix, descriptor passed in the kernel arguments (no device table needed).
// One launch of strips x slices workgroups.  In loss mode slice i writes its partials at
// partial_*[i * small_m_blocks(d) ..], scaled by 1 / (M N) of the whole matrix, so that their sum over
// all slices is the matrix's loss.
int small_m_launch_one(const szo_linear_desc* d, uint64_t seed, uint64_t step, float eps, int sign, bool loss_mode,
                       double* partial_plus, double* partial_minus, hipStream_t stream) {
  const int rc = set_small_attrs();
  if (rc != SZO_OK) return rc;
  const int blocks = small_m_blocks(d);
  const int rblocks = small_m_rblocks(d, small_m_wgs16(d));
  const int slices = slices_of(d, rblocks);
  SmallArgs a{};
  fill_mat(a.one, d);                                       // whole matrix: the kernel offsets rows by slice
  a.table = nullptr; a.n_mats = 1;
  a.store_sign = sign; a.loss_mode = loss_mode ? 1 : 0;
  a.seed = seed; a.step = step; a.eps = eps;
  a.partial_plus = partial_plus;
  a.partial_minus = partial_minus;
  const int trc = timing_begin(stream);
  if (trc != SZO_OK) return trc;
  a.slices = slices;
  a.stream_once = stream_once_rule(slices, code_bytes(d));
  small_m_launch(small_m_mode(d), rblocks, false, dim3((unsigned)(blocks * slices)), a, stream);
  SZO_LAUNCH_CHECK();
  const int erc = timing_end(stream);
  if (erc != SZO_OK) return erc;
  return SZO_OK;
}

// A whole stack in one launch per instantiation.  The table is assembled on the host, longest K
// first (their workgroups run longest, so they should start first), copied into `table_dev`
// (device, small_m_table_bytes(n)) with an asynchronous copy on the stream, and also drives one
// grouped sparse update when `do_update` is set.  With `do_forward` false only the table is staged
// and the update runs (used by the many-token step, whose forwards are launched per matrix).
int small_m_step(const szo_linear_desc* descs, int n, uint64_t seed, uint64_t step, float eps, float lr,
                 void* table_dev, double* partial_plus, double* scalars, bool do_forward, bool do_update,
                 hipStream_t stream) {
  int rc = set_small_attrs();
  if (rc != SZO_OK) return rc;
  if (n > kMaxStepMatrices) return SZO_EUNSUPPORTED;
  int64_t wgs16 = 0;
  for (int i = 0; i < n; ++i) wgs16 += small_m_wgs16(&descs[i]);
  // two activation sets (forward launches only): one block of rows for each, whatever the token count
  auto dual_of = [&](const szo_linear_desc* d) { return do_forward && d->x_minus != nullptr; };
  auto rblocks_of = [&](const szo_linear_desc* d) { return dual_of(d) ? 2 : small_m_rblocks(d, wgs16); };
  if (small_m_table_bytes(n) > kTableBytesPerMatrix * (size_t)kMaxStepMatrices) return SZO_EUNSUPPORTED;
  static thread_local std::vector<SmallMat> host_table;
  host_table.resize((size_t)std::max(n, 1));
  SmallMat* const host = host_table.data();
  // order: by instantiation (fast, table format, plain; fewer rows per pass first), inside each by K descending
  int order[kMaxStepMatrices];
  for (int i = 0; i < n; ++i) order[i] = i;
  auto sort_key = [&](int o) {
    return ((int64_t)(kSmallClasses - 1 - small_m_class(&descs[o], rblocks_of(&descs[o]), dual_of(&descs[o]))) << 40) + descs[o].K;
  };
  for (int i = 1; i < n; ++i) {                       // insertion sort: n is a few hundred
    const int o = order[i];
    const int64_t key = sort_key(o);
    int j = i - 1;
    while (j >= 0) {
      if (sort_key(order[j]) >= key) break;
      order[j + 1] = order[j];
      --j;
    }
    order[j + 1] = o;
  }
  // One table entry per matrix; a launch has (strips of its matrices) x (slices of its longest matrix)
  // workgroups (those past a matrix's last slice return at once), and slice i of a matrix writes its
  // loss partials behind those of slice i - 1.
  int class_entries[kSmallClasses] = {}, class_blocks[kSmallClasses] = {}, class_slices[kSmallClasses] = {}, entries = 0;
  int64_t class_code_bytes[kSmallClasses] = {};
  int64_t quads = 0, partials = 0;
  for (int r = 0; r < n; ++r) {
    const szo_linear_desc* d = &descs[order[r]];
    const int rblocks = rblocks_of(d);
    const int cls = small_m_class(d, rblocks, dual_of(d));
    // a layer without tokens or outputs has no workgroups; it keeps its table entry for the update
    const bool live = d->M > 0 && d->N > 0;
    const int slices = live ? slices_of(d, rblocks, dual_of(d)) : 0, b = live ? small_m_blocks(d) : 0;
    SmallMat& m = host[entries++];
    fill_mat(m, d);
    m.first_block = class_blocks[cls];
    m.partial_base = (int)partials;
    m.first_quad = quads;
    class_blocks[cls] += b;
    class_slices[cls] = std::max(class_slices[cls], slices);
    if (live) class_code_bytes[cls] += code_bytes(d);
    ++class_entries[cls];
    partials += (int64_t)b * slices;
    quads += (((int64_t)d->nnz + 3) / 4 + 63) & ~(int64_t)63;      // a wave of the update serves one matrix
    if (do_forward && 2 * partials > kMaxLossPartials) return SZO_EUNSUPPORTED;
    if ((int64_t)class_blocks[cls] * class_slices[cls] > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
  }
  rc = stage_table(host, sizeof(SmallMat) * (size_t)entries, table_dev, stream);
  if (rc != SZO_OK) return rc;
  SmallArgs a{};
  a.store_sign = 1; a.loss_mode = 1;
  a.seed = seed; a.step = step; a.eps = eps;
  a.partial_plus = partial_plus; a.partial_minus = do_forward ? partial_plus + partials : nullptr;
  const SmallMat* tdev = (const SmallMat*)table_dev;
  int first_entry = 0;
  for (int cls = 0; cls < kSmallClasses; ++cls) {
    if (do_forward && class_blocks[cls] > 0 && class_slices[cls] > 0) {
      a.table = tdev + first_entry; a.n_mats = class_entries[cls];
      a.slices = class_slices[cls];
      a.stream_once = stream_once_rule(a.slices, class_code_bytes[cls]);
      if ((rc = timing_begin(stream)) != SZO_OK) return rc;
      small_m_launch(class_mode(cls), class_rblocks(cls), class_dual(cls), dim3((unsigned)(class_blocks[cls] * class_slices[cls])), a, stream);
      SZO_LAUNCH_CHECK();
      if ((rc = timing_end(stream)) != SZO_OK) return rc;
    }
    first_entry += class_entries[cls];
  }
  if (do_forward) {
    rc = reduce_step(partial_plus, (int)partials, eps, scalars, stream);
    if (rc != SZO_OK) return rc;
  }
  if (do_update && quads > 0) {
    const int64_t ub = (quads + 255) / 256;
    if (ub > 0x7FFFFFFF) return SZO_EUNSUPPORTED;
    if ((rc = timing_begin(stream, 1)) != SZO_OK) return rc;
    sparse_update_table_kernel<<<(unsigned)ub, 256, 0, stream>>>(tdev, entries, quads, seed, step, scalars + 2, lr);
    SZO_LAUNCH_CHECK();
    if ((rc = timing_end(stream)) != SZO_OK) return rc;
  }
  return SZO_OK;
}

}  // namespace szo
