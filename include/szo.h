/*
 * szo.h -- C ABI of libszo: the hot path of sensitive-sparse zeroth-order
 * fine-tuning (arXiv 2406.02913) for AMD MI355X (gfx950).
 *
 * One ZO-SGD step over a stack of linear layers whose frozen dense weights are
 * 4-bit group-quantised and whose "sensitive" weights (a static mask of about
 * 0.1% of the coordinates) are kept as fp32 sparse values:
 *
 *   two forwards at  w_sparse + eps*z  and  w_sparse - eps*z   (Definition 1, Definition 4)
 *   g = (L+ - L-) / (2 eps)                                    (Definition 1)
 *   w_sparse <- w_sparse - lr * g * z                          (Section 3.4, fixed-parameter update rule)
 *
 * where each forward is  y = x (Dequantize(Q(w_dense)) + w_sparse)^T  evaluated
 * as ONE dense product after the sparse part has been added to the dequantised
 * tile (Appendix C.5, the SparseAdd-then-DenseMM form), and z is a Gaussian
 * regenerated from (seed, step, entry index) and never stored (Section 3.5,
 * random-seed trick).
 *
 * Conventions
 *   - Every function returns SZO_OK (0) or a negative error code.  Nothing
 *     throws, exits or prints.  SZO_ELAUNCH means a HIP call failed; the HIP
 *     error code is then available from szo_last_hip_error().
 *   - "device" pointers are HIP device memory owned by the caller (e.g. PyTorch
 *     tensors); the library never frees or keeps them.  "host" pointers are
 *     ordinary process memory, read or written before the call returns.
 *   - Calls that take a `stream` only enqueue work on that hipStream_t (passed
 *     as void*; NULL = the default stream).  They do not allocate and do not
 *     synchronise with the host.
 *   - Row-major everywhere.  x is [M,K], the weight is [N,K] (out x in),
 *     y = x W^T is [M,N].
 */
#ifndef SZO_H_
#define SZO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SZO_OK            0
#define SZO_EINVAL       (-1)   /* null pointer, bad shape, misalignment, bad enum */
#define SZO_EUNSUPPORTED (-2)   /* valid but outside what the kernels handle       */
#define SZO_ELAUNCH      (-3)   /* a HIP runtime call failed                        */

/* Sparse layout constants ("TCSR"): rows are cut into bands of 64, columns into
 * tiles of 64;  tile(n,k) = (n/64) * (K/64) + k/64, so the tiles of one band
 * follow each other along K.  Entries are ordered by (tile, (n%64)*64 + k%64);
 * tile_ptr[t]..tile_ptr[t+1] is the range of tile t.  The position j of an
 * entry in this order is its entry index: together with nnz_base it selects the
 * entry's Gaussian. */
#define SZO_TILE_ROWS   64
#define SZO_TILE_COLS   64

/* 16-bit type the dequantised weight tile and the activations are staged in
 * before the matrix-core product.
 *   SZO_TILE_F16 (default) keeps w_sparse +- eps*z within the estimator's error budget (11-bit
 *   significand), but NARROWS THE ACTIVATION DOMAIN: the bf16 activations are converted to fp16 with
 *   truncation, which is exact only for 2^-14 <= |x| <= 65504.  Larger magnitudes saturate at
 *   +-65504 (infinities stay infinite), smaller ones lose low bits and vanish below 2^-24; no error
 *   is raised.  A caller whose activations may leave that range (outlier channels of a real model)
 *   measures them with szo_activation_absmax() and takes what szo_choose_tile_dtype() returns.
 *   SZO_TILE_BF16 stages the activations unchanged (full bf16 range); the sensitive values are then
 *   rounded to 8 significant bits, which costs about 1-2 % of sigma_g on the SPSA scalar. */
#define SZO_TILE_F16   0
#define SZO_TILE_BF16  1

/* One linear layer.  Plain data; filled by the caller for every call. */
typedef struct szo_linear_desc {
  int64_t  M, N, K;        /* tokens, out features, in features; K % 64 == 0           */
  int32_t  group;          /* quantisation group along K: 32, 64 or 128; divides K      */
  int32_t  tile_dtype;     /* SZO_TILE_F16 or SZO_TILE_BF16                             */
  int64_t  nnz;            /* number of sensitive entries of this matrix (may be 0)     */
  uint64_t nnz_base;       /* global index of entry 0; multiple of 4                    */
  const void*     x;        /* device, bf16  [M,K]; with SZO_TILE_F16: |x| <= 65504 (see above) */
  const uint8_t*  qweight;  /* device, u4x2, banded layout (below), szo_qweight_bytes(N,K) */
  const void*     scales;   /* device, fp16, banded layout (below), szo_scales_count()     */
  const uint32_t* tile_ptr; /* device, u32   [szo_num_tiles(N,K) + 1]                   */
  const uint32_t* sp_idx;   /* device, u32   [nnz] flat n*K+k in TCSR order             */
  float*          sp_val;   /* device, fp32  [nnz] same order; read-only in forwards    */
  float*          y;        /* device, fp32  [M,N] output (may be NULL in szo_linear_fwd_mse) */
  const void*     target;   /* device, bf16  [M,N]; only read by the loss-fusing calls  */
  const void*     lut;      /* device, fp16  [N,16] row-major, 16-byte aligned; SZO_FORMAT_LUT only */
  int32_t  format;          /* SZO_FORMAT_UNIFORM (0) or SZO_FORMAT_LUT                  */
  int32_t  reserved;        /* 0                                                         */
  const void*     x_minus;  /* device, bf16 [M,K], 16-byte aligned, or NULL: what the -eps forward of
                             * szo_zo_step reads instead of x (the two forwards of a layer inside a
                             * model see different activations); ignored by the single-forward calls */
} szo_linear_desc;

/* Formats of the frozen 4-bit part (Section 3.5 allows any post-training quantiser; Appendix C.5,
 * "Integration with weight quantization method", distinguishes uniform and non-uniform ones and
 * has both dequantised before the SparseAdd form of the product):
 *   SZO_FORMAT_UNIFORM  dq[n,k] = (code - 8) * scales[n, k/group]
 *   SZO_FORMAT_LUT      dq[n,k] = lut[n][code]: 16 fp16 centroids per output row, no scales
 *                       (`scales` may be NULL and `group` is ignored).  fp16 tile only.
 * In both, the sensitive entries are ADDED to the dequantised tile. */
#define SZO_FORMAT_UNIFORM 0
#define SZO_FORMAT_LUT 1

/* Banded device layout of the frozen quantised part.  The weights are read exactly once per
 * forward, by waves that each own a band of 64 consecutive rows of W, so codes and scales are
 * stored band by band, 64-column tile by tile, such that what one wave needs next is contiguous
 * (whole 128-byte lines instead of one short piece per row).  Rows are padded up to a multiple
 * of 64 with code 8 (weight zero) and scale 0.  With B = n / 64, r = n % 64, T = k / 64:
 *   code of (n,k):   byte  ((B * (K/64) + T) * 64 + r) * 32 + (k % 64) / 2,
 *                    low nibble = even k, high nibble = odd k; code = q + 8
 *   scale of (n,g):  element  (B * (K/group) + g) * 64 + (r % 16) * 4 + r / 16
 * (the four rows r, r+16, r+32, r+48 that one lane of a 16-row matrix-core operand serves sit
 * side by side).  szo_layout_weights() produces both arrays from the row-major ones that
 * szo_quantize_pack() writes. */

/* ---- hot calls (device work, enqueued on `stream`) ------------------------------------- */

/* Perturbed forward of one layer (Appendix C.5, SparseAdd then DenseMM; perturbation of
 * Definition 4):  y = x (dq + S)^T with dq[n,k] = (code-8)*scale[n,k/group] and
 * S[n_j,k_j] = sp_val[j] + sign*eps*z_j.  sign in {-1,0,+1}; sign 0 or eps 0 = unperturbed.
 * z_j is the Gaussian of global entry nnz_base + j for (seed, step).
 * Errors: SZO_EINVAL on null/misaligned pointers (x, qweight 16-byte; others natural), bad
 * shape, bad sign/dtype; SZO_EUNSUPPORTED if K % 64 != 0, group not in {32,64,128} or N*K
 * does not fit 32 bits.  M == 0 or N == 0 is a no-op. */
int szo_linear_fwd(const szo_linear_desc* desc /* host */, uint64_t seed, uint64_t step,
                   int sign, float eps, void* stream);

/* Stand-in loss of the workloads: loss_acc += scale * sum_i (y[i] - target[i])^2, i < count
 * (Definition 1 only needs a scalar f).  Accumulates in fp64 in a fixed order: results are
 * bit-reproducible run to run.  y: device fp32; target: device bf16; loss_acc: device
 * double; workspace: device, at least szo_workspace_bytes() bytes, 8-byte aligned, not shared
 * with a call running concurrently on another stream.  count == 0 adds nothing. */
int szo_mse_loss(const float* y, const void* target, int64_t count, double scale,
                 double* loss_acc, void* workspace, void* stream);

/* Forward with the loss folded into the product's epilogue: same y as szo_linear_fwd (written
 * only if desc->y is not NULL) and loss_acc += scale * sum (y - desc->target)^2 without
 * re-reading y from memory.  Same determinism and workspace rules as szo_mse_loss. */
int szo_linear_fwd_mse(const szo_linear_desc* desc /* host */, uint64_t seed, uint64_t step,
                       int sign, float eps, double scale, double* loss_acc, void* workspace,
                       void* stream);

/* SPSA scalar (Definition 1): *g = (*loss_plus - *loss_minus) / (2 eps); eps == 0 gives 0.
 * All three pointers: device double. */
int szo_spsa_g(const double* loss_plus, const double* loss_minus, float eps, double* g,
               void* stream);

/* Sparse ZO-SGD update (Section 3.4, fixed-parameter update rule):
 * sp_val[j] -= lr * g * z_j, j < nnz, with exactly the z of the forwards for (seed, step).
 * g: device double.  sp_idx is accepted for symmetry with the forward and may be NULL (the
 * Gaussian is keyed by position j, not by matrix coordinates). */
int szo_sparse_update(float* sp_val, const uint32_t* sp_idx, int64_t nnz, uint64_t nnz_base,
                      uint64_t seed, uint64_t step, const double* g, float lr, void* stream);

/* One whole step over `n` layers: for every layer a +eps forward and a -eps forward, each
 * followed by its loss with scale 1/(M*N); then g; then the update of every layer.
 * scalars: device double[3], overwritten with (L+, L-, g).  flags: bit 0 set = use the
 * loss-fusing forward and never write y (desc->y may then be NULL); large steps then run all
 * forwards (every layer, both signs) as one launch driven by a descriptor table that is staged in
 * the workspace, and steps with few tokens per layer (up to 224, and 257 to 448: wherever slices of
 * 32 token rows beat rows of 256-row tiles) stream the weights once per 16 or 32 token rows, each
 * pass serving both signs.
 * descs: host array, read before the call returns.  Everything is enqueued on `stream`.  The
 * descriptor tables of the grouped launches (forwards of a fused step; the update of every step)
 * travel through a ring of eight pinned host buffers per host thread (allocated on first use,
 * released when the thread ends); a call waits on the host only if a copy issued eight tables
 * earlier on this thread (four tiled steps) has not executed yet.  Because of those buffers NO
 * variant of this call can be captured into a HIP graph: it returns SZO_EUNSUPPORTED, with nothing
 * enqueued, while `stream` is capturing.  The single-layer calls above are plain launches and can
 * be captured.  The workspace must not be shared with a call running concurrently on another
 * stream. */
#define SZO_STEP_FUSED_LOSS 1
/* Bit 1 (with bit 0): take the slicing path of the few-token case at ANY token count.  Both forwards of
 * a layer see the same x in this call, so y(+-) = x (dq + v)^T +- eps x z^T: the dense product is
 * computed once per slice of up to 48 token rows and serves both signs, the sparse products are added.
 * Same results as two forwards; half the dense work; the weights are streamed once per slice.  Not the
 * default for many tokens because it does not carry over to a caller whose two forwards see different
 * activations (every layer of a real model but the first), who calls szo_linear_fwd per sign instead. */
#define SZO_STEP_ONE_DENSE_PASS 2
int szo_zo_step(const szo_linear_desc* descs /* host */, int n, uint64_t seed, uint64_t step,
                float eps, float lr, double* scalars, void* workspace, int flags, void* stream);

/* The same step for callers that cannot allocate: code running under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same inputs, same outputs as szo_zo_step with
 * SZO_STEP_FUSED_LOSS (scalars = (L+, L-, g); every layer's sp_val updated; desc->y is not written),
 * up to the order in which the fp64 loss partials are added.  It takes no workspace: the loss partials
 * live in a fixed array inside the library (1 MiB per GPU, kept until the process ends), and it
 * stages no descriptor table: every layer is one plain launch of the few-token kernel (when every
 * layer of the step qualifies for it and none has x_minus), else one tiled launch per sign; then one
 * reduction, and one update launch per layer.  It calls no
 * allocating routine (no hipMalloc / hipHostMalloc, no event creation unless szo_kernel_timing is
 * on) and can be captured into a HIP graph.
 * Limit: at most 65 536 workgroups per sign over the whole step (one per 256 x 256 output tile, or
 * per 128 x 128 tile for small layers, or per 256-column strip and slice of token rows of a few-token
 * layer): beyond that SZO_EUNSUPPORTED, with nothing enqueued.  A Llama-2-7B decoder block at 4096
 * tokens has 3 088 per sign.
 * All calls on one GPU share that array: calls that overlap in time on one GPU (different streams
 * or host threads) race on it.  Nothing in it needs clearing between calls (every partial that is
 * read has been written by the same call). */
int szo_zo_step_noalloc(const szo_linear_desc* descs /* host */, int n, uint64_t seed, uint64_t step,
                        float eps, float lr, double* scalars /* device double[3] */, void* stream);

/* Bytes of device workspace the loss-accumulating calls need (a constant). */
size_t szo_workspace_bytes(void);

/* Puts a freshly allocated workspace into its idle state (zeroes its header).  Needed once per
 * workspace; every loss-accumulating call leaves the workspace idle again when it completes. */
int szo_workspace_init(void* workspace, void* stream);

/* ---- one-time set-up on the host (no GPU needed; deterministic) ------------------------- */

/* Number of TCSR tiles of an [N,K] matrix: ceil(N/64) * (K/64).  0 if K % 64 != 0. */
int64_t szo_num_tiles(int64_t N, int64_t K);

/* Synthetic stand-in for the sensitive mask of Definition 3 (the real one needs gradients of
 * a trained model).  kind 0: nnz distinct positions uniform over the matrix.  kind 1: heavy
 * tail -- ceil(N/100) hot rows hold floor(nnz/2) entries, the rest is uniform.  Draw d of
 * stream s is Philox-4x32-10(key = mask_seed, counter = (lo32 d, hi32 d, s, 0)), value
 * (r0*2^32 + r1) mod range, duplicates dropped in draw order.  flat_out: host u32 [nnz],
 * ascending flat positions n*K+k. */
int szo_mask_generate(int64_t N, int64_t K, int64_t nnz, int kind, uint64_t mask_seed,
                      uint32_t* flat_out);

/* Tile-ordered layout from ascending unique flat positions.  Outputs (host): tile_ptr
 * [szo_num_tiles+1], sp_idx [nnz], perm [nnz] with sp_idx[j] == flat_sorted[perm[j]] (perm may
 * be NULL).  SZO_EINVAL if positions are not strictly ascending or out of range. */
int szo_tcsr_build(int64_t N, int64_t K, const uint32_t* flat_sorted, int64_t nnz,
                   uint32_t* tile_ptr_out, uint32_t* sp_idx_out, uint32_t* perm_out);

/* Decomposition w = w_sparse + w_dense (Section 3.4) and 4-bit quantisation of w_dense
 * (Section 3.5): masked weights are copied to sp_val_out (in the order of mask_flat) and set
 * to zero; then per row and per group of `group` columns scale = fp16(max|w|/7),
 * code = clamp(rint(w/scale),-8,7)+8 (scale 0 -> code 8).  W: host fp32 [N,K];
 * q_out: host [N,K/2]; scales_out: host fp16 bit patterns [N,K/group]. */
int szo_quantize_pack(const float* W, int64_t N, int64_t K, int group, const uint32_t* mask_flat,
                      int64_t nnz, uint8_t* q_out, uint16_t* scales_out, float* sp_val_out);

/* The same decomposition with the non-uniform format (SZO_FORMAT_LUT).  The paper fixes no
 * codebook; this one is the plainest deterministic choice: masked weights are set to zero, a
 * row's 16 centroids are its order statistics at ranks (2c+1)K/32, c = 0..15 (the medians of 16
 * equal-mass bins), rounded to fp16, and a weight's code is the index of the nearest centroid
 * (distance in fp64, ties to the lower index).  Needs K % 32 == 0.  lut_out: host fp16 bit
 * patterns [N,16], non-decreasing along a row; q_out as in szo_quantize_pack. */
int szo_quantize_pack_lut(const float* W, int64_t N, int64_t K, const uint32_t* mask_flat,
                          int64_t nnz, uint8_t* q_out, uint16_t* lut_out, float* sp_val_out);

/* Sizes of the banded device arrays: bytes of qweight, elements of scales (0 on bad shapes). */
size_t szo_qweight_bytes(int64_t N, int64_t K);
size_t szo_scales_count(int64_t N, int64_t K, int group);

/* Row-major host arrays (q [N,K/2], scales fp16 bits [N,K/group], as written by
 * szo_quantize_pack) -> banded device layout described above, into host buffers of
 * szo_qweight_bytes / szo_scales_count elements that the caller then copies to the device.
 * Pure data movement.  scales and scales_banded may both be NULL (SZO_FORMAT_LUT: codes only;
 * group is then ignored).  Errors: SZO_EINVAL on null pointers, K % 64 != 0 or K % group != 0. */
int szo_layout_weights(const uint8_t* q, const uint16_t* scales, int64_t N, int64_t K, int group,
                       uint8_t* q_banded, uint16_t* scales_banded);

/* ---- inspection ----------------------------------------------------------------------- */

/* Largest |x| of `count` bf16 values (device), written as fp32 to *absmax_out (device, 4-byte aligned);
 * NaN if any value is NaN, +inf if any is infinite, 0 for count == 0.  Enqueued on `stream`. */
int szo_activation_absmax(const void* x /* device bf16 */, int64_t count, float* absmax_out /* device */,
                          void* stream);

/* Host rule for the tile type: SZO_TILE_F16 if every activation converts to fp16 without saturating
 * (x_absmax <= 65504), else SZO_TILE_BF16; SZO_EINVAL for a negative or NaN argument. */
int szo_choose_tile_dtype(float x_absmax);

/* Timing of the forward kernels (the tiled kernel and the few-token kernel) for benchmarks.
 * szo_kernel_timing(1) makes every later forward-kernel launch record a pair of events around
 * itself on the stream it is launched on; szo_kernel_timing(0) stops that.  Either call drops
 * what was recorded.  szo_kernel_timing_read() waits for the recorded launches, returns the sum
 * of their durations in milliseconds and their number, and starts a new collection.  Process-
 * wide state, for one measuring thread; events are created on demand and kept. */
int szo_kernel_timing(int enable);
int szo_kernel_timing_read(double* total_ms /* host */, int64_t* launches /* host */);
/* The same collection split by kind: [0] the forward kernels (what szo_kernel_timing_read returns),
 * [1] the sparse update kernels, which are bracketed as well while timing is on. */
int szo_kernel_timing_read2(double total_ms[2] /* host */, int64_t launches[2] /* host */);

/* Host evaluation of Philox-4x32-10 (ten rounds; multipliers 0xD2511F53, 0xCD9E8D57; key
 * increments 0x9E3779B9, 0xBB67AE85). */
int szo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Device: for j < nnz write the four Philox words behind entry nnz_base + j to
 * words_out[4*j..4*j+3] (device u32, may be NULL) and its Gaussian to z_out[j] (device fp32,
 * may be NULL) -- the same device routine the forward and the update use. */
int szo_debug_zbar(uint64_t nnz_base, int64_t nnz, uint64_t seed, uint64_t step,
                   uint32_t* words_out, float* z_out, void* stream);

/* Tuning/testing hook: which workgroup tile the forward uses.  0 = chosen from the shape
 * (default; also enables the few-token path), 1 = 128x128 outputs with 4 waves,
 * 2 = 256x256 outputs with 8 waves, 3 = as 2 and szo_zo_step always launches all forwards of a
 * step as one grid (with 0 and 2 it does so only when the step has at least 192 tiles), 4 / 5 = as 0
 * and the few-token path takes 32 / 48 token rows per pass for every layer with more than 16 tokens
 * (by default it chooses 16, 32 or 48, the larger ones only in launches that fill the chip more than
 * twice over), 6 = as 0 and szo_zo_step always launches all forwards of a step as one grid, whatever its
 * size (with 0 only when the grid fills the chip); that grid uses dual-sign tiles -- one workgroup computes
 * both forwards of 256 x 128 outputs and dequantises the weights once -- unless a layer has x_minus,
 * 7 = as 0 and the few-token path loads its codes as a non-temporal stream in every launch with one slice
 * of token rows per strip (by default only when the launch streams more codes than the last-level cache
 * holds).
 * Process-wide, not thread-safe; results do not depend on it beyond fp32 summation order. */
int szo_set_tile_config(int config);

/* HIP error code of the most recent SZO_ELAUNCH on this thread (0 if none). */
int szo_last_hip_error(void);

/* ABI version; bumped when a signature or the descriptor changes. */
int szo_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SZO_H_ */
