/*
 * slimfit.h -- C ABI of the MI355X (gfx950) SlimFit hot-path library.
 *
 * SlimFit (arXiv 2305.18513) fine-tunes transformers under a memory budget by
 * (1) scoring every layer by how much its weights moved in the last step
 * (Eq. 1), (2) freezing the lowest-scoring layers each iteration (Alg. 1,
 * inter-layer scheduling, ILS), (3) caching the activations that cannot be
 * discarded in 8 or 4 bits (Alg. 2, Sec. 4 and 5) and (4) caching only the
 * largest 10 % of some activations as values + indices (Alg. 5).  This
 * library is that per-step path and nothing else.
 *
 * Conventions
 *  - Every function returns a slimfit_status as int32_t.  Nothing throws,
 *    nothing allocates device memory, nothing synchronises with the host.
 *  - "device pointer" = memory the GPU can address (hipMalloc / a torch CUDA
 *    tensor); "host pointer" = ordinary process memory.  Each argument says
 *    which one it is.  The caller owns every buffer and keeps it alive until
 *    the stream has passed the call.  Inputs are never written; outputs are
 *    fully overwritten for the sizes given (the one argument that is both, the
 *    weights of slimfit_apply_update_layer_delta, is marked as such).
 *  - Device pointers must be 16-byte aligned (SLIMFIT_ERR_ALIGNMENT), except
 *    where a narrower alignment is stated.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    All device work of a call is enqueued on it, in order.
 *  - Arguments are validated before anything is launched, so every error
 *    return leaves the GPU untouched.  A size of zero is SLIMFIT_OK and a
 *    no-op.  With pointer checks on (the default, see
 *    slimfit_set_pointer_checks) each device pointer is also looked up in the
 *    HIP runtime and rejected with SLIMFIT_ERR_POINTER when it is not device
 *    memory or when the bytes the call would touch run past the end of its
 *    allocation (the enclosing allocation: a caching allocator's segment may
 *    be far larger than the tensor carved out of it, so the caller still owes
 *    buffers of the stated sizes).  While `stream` is being captured into a
 *    HIP graph the look-ups are skipped for that call (the runtime does not
 *    allow them during a capture); every other check still runs.
 *  - Inputs must be finite.  NaN/Inf never fault but their results are
 *    unspecified.
 *  - dtype SLIMFIT_BF16 means raw bfloat16 bit patterns (uint16_t).
 */
#ifndef SLIMFIT_H
#define SLIMFIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SLIMFIT_OK = 0,
    SLIMFIT_ERR_INVALID_ARG = 1, /* NULL where data is required, negative size, k > cols ... */
    SLIMFIT_ERR_UNSUPPORTED = 2, /* a value outside the supported set (bits, block, cols) */
    SLIMFIT_ERR_ALIGNMENT = 3,   /* a device pointer is not aligned as required */
    SLIMFIT_ERR_WORKSPACE = 4,   /* workspace NULL or smaller than the size query says */
    SLIMFIT_ERR_HIP = 5,         /* the HIP runtime refused a launch or a query */
    SLIMFIT_ERR_POINTER = 6      /* pointer check failed: not device memory / too small */
} slimfit_status;

typedef enum { SLIMFIT_F32 = 0, SLIMFIT_BF16 = 1 } slimfit_dtype;
typedef enum { SLIMFIT_Q_FIXED = 0, SLIMFIT_Q_BLOCK = 1 } slimfit_qmode;
typedef enum { SLIMFIT_PRUNE_TOPK = 0, SLIMFIT_PRUNE_THRESHOLD = 1 } slimfit_prune_mode;

/* Static text for a status code (never NULL). */
const char *slimfit_status_string(int32_t status);

/* Library version, major*10000 + minor*100 + patch. */
int32_t slimfit_version(void);

/* Turn the run-time device-pointer checks on (non-zero, default) or off for
 * the whole process: an opt-out for callers that have validated their buffers
 * (graph capture does not need it).  Returns the previous setting.  Host-side
 * only; the checks cost about 0.3 microseconds per call when on. */
int32_t slimfit_set_pointer_checks(int32_t on);

/* Diagnostic, not part of the method: a plain streaming kernel with a chosen read : write ratio, the
 * yardstick for what a perfect kernel of a given traffic mix could reach on this GPU.  Loads are 16-byte,
 * non-temporal and coalesced.
 *  ratio 1, 2, 4, 8, 16 (a quantiser, a pruner): 16 / ratio bytes are written for every vector read, next
 *      to its neighbours'.  With source vector i = (x, y, z, w) as fp32 and s = ((x + y) + z) + w, output
 *      element i is: ratio 1 the vector itself; 2 the pair (x + y, z + w); 4 s; 8 the upper 16 bits of s;
 *      16 the upper 8 bits of s.  dst: in_vecs * 16 / ratio bytes.
 *  ratio 0 (a scoring pass): read only; wavefront g of workgroup b (1024 source vectors a workgroup, thread t
 *      reading vectors b*1024 + t + 256*j) writes the sum of its lanes' s values to the float dst[4*b + g]
 *      (lane values added over j, then butterfly over the lanes: 32, 16, ... 1).  dst: ceil(in_vecs / 1024) * 16 bytes.
 *  ratio -2, -4, -8 (a dequantiser): M = -ratio vectors are written per vector read, one thread per output
 *      vector: output vector o is (s, s + 1, s + 2, s + 3) with s the sum, as a float, of the unsigned 16-bit
 *      words of source bytes [o * 16 / M, (o + 1) * 16 / M).  dst: in_vecs * M * 16 bytes.
 *  src : DEVICE, in_vecs * 16 bytes, 16-byte aligned, read only.     dst : DEVICE, 16-byte aligned, not src. */
int32_t slimfit_stream_probe(const void *src, void *dst, int64_t in_vecs, int32_t ratio, void *stream);

/* ------------------------------------------------------------------------
 * (a) Training-dynamics freeze score -- Eq. 1 (Sec. 3.1):
 *        d_i = 1/(M*I) * || (W_i^t - W_i^{t-1}) / W_i^{t-1} ||_l1
 *     entry-wise over the M x I weights of layer i, i.e. the mean of
 *     |delta| / |w_prev|.  One call scores all L layers ("layer" = one weight
 *     tensor, the granularity of the paper's layer list).
 *
 *  w_prev, w_cur : HOST arrays of L DEVICE pointers.  w_prev[i] holds
 *                  W_i^{t-1} (numel[i] elements of prev_dt); w_cur[i] holds
 *                  W_i^t, or, when cur_is_delta != 0, the update
 *                  W_i^t - W_i^{t-1} itself (numel[i] elements of cur_dt).
 *                  The arrays are read during the call only.
 *  numel         : HOST array of L element counts, each >= 0 (0 scores 0).
 *  eps           : >= 0.  Floor on |w_prev| in the denominator; 0 gives the
 *                  literal equation (a changed weight whose old value is 0
 *                  makes the score +inf).  An unchanged element contributes 0
 *                  whatever its old value.
 *  d_out         : DEVICE float[L], 4-byte aligned.
 *  workspace     : DEVICE scratch of at least the bytes
 *                  slimfit_layer_delta_workspace reports, 256-byte aligned.
 *
 *  Arithmetic: each term is formed in fp32 (difference, IEEE division), the
 *  terms are accumulated in fp64 in a fixed order, so results are identical
 *  from run to run.  A term above FLT_MAX saturates to +inf.
 *
 *  slimfit_layer_delta       = plan + run in one call.
 *  slimfit_layer_delta_plan  writes the layer table into the workspace (the
 *                            pointers of a model do not change between
 *                            steps, so a trainer plans once).
 *  slimfit_layer_delta_run   scores the planned layers; numel, L and the
 *                            dtypes must be the ones given to the plan.  If
 *                            the workspace does not hold a matching plan,
 *                            d_out is filled with NaN and nothing else is
 *                            touched.
 * ---------------------------------------------------------------------- */
int32_t slimfit_layer_delta_workspace(int32_t L, const int64_t *numel, size_t *bytes);

int32_t slimfit_layer_delta_plan(const void *const *w_prev, int32_t prev_dt,
                                 const void *const *w_cur, int32_t cur_dt,
                                 const int64_t *numel, int32_t L,
                                 void *workspace, size_t workspace_bytes, void *stream);

int32_t slimfit_layer_delta_run(const int64_t *numel, int32_t L,
                                int32_t prev_dt, int32_t cur_dt, int32_t cur_is_delta,
                                float eps, float *d_out,
                                void *workspace, size_t workspace_bytes, void *stream);

int32_t slimfit_layer_delta(const void *const *w_prev, int32_t prev_dt,
                            const void *const *w_cur, int32_t cur_dt, int32_t cur_is_delta,
                            const int64_t *numel, int32_t L, float eps,
                            float *d_out, void *workspace, size_t workspace_bytes,
                            void *stream);

/* ------------------------------------------------------------------------
 * slimfit_layer_delta for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, arithmetic and results as slimfit_layer_delta,
 * minus the workspace: the layer table and the per-chunk partial sums live in
 * a fixed device array of SLIMFIT_LAYER_DELTA_STATIC_BYTES inside the library
 * (one copy per GPU, held until the process ends).  The call allocates
 * nothing and frees nothing.
 *
 *  - The device that is current when the call is made must be the stream's
 *    device; its copy of the array is used.
 *  - Limit: slimfit_layer_delta_workspace(L, numel) must not exceed
 *    SLIMFIT_LAYER_DELTA_STATIC_BYTES (about 2 * 10^9 weights in a few
 *    hundred layers); beyond it the call returns SLIMFIT_ERR_WORKSPACE and
 *    enqueues nothing.
 *  - Every call on a GPU uses that GPU's one array: calls whose kernels may
 *    overlap on the same GPU (different streams, or a captured graph replayed
 *    next to eager calls) race.  Nothing has to be cleared between calls: a
 *    call rewrites the table and every partial sum it later reads.
 * ---------------------------------------------------------------------- */
#define SLIMFIT_LAYER_DELTA_STATIC_BYTES (1u << 20)

int32_t slimfit_layer_delta_static(const void *const *w_prev, int32_t prev_dt,
                                   const void *const *w_cur, int32_t cur_dt, int32_t cur_is_delta,
                                   const int64_t *numel, int32_t L, float eps,
                                   float *d_out, void *stream);

/* ------------------------------------------------------------------------
 * (a') Eq. 1 measured while the optimizer's update is applied.  The paper's
 *     formulation compares W^t with a kept copy of W^{t-1}; when the optimizer
 *     hands over its update delta_i = W_i^t - W_i^{t-1} instead of applying it,
 *     one pass can do both: take the terms |delta| / |W^{t-1}| and overwrite
 *     W^{t-1} with W^t = W^{t-1} + delta.  No copy of the previous weights is
 *     kept and the update costs no pass of its own.
 *
 *  w     : HOST array of L DEVICE pointers to the weights (numel[i] elements of
 *          w_dt, 16-byte aligned); on return of the kernels they hold W^t: one
 *          fp32 addition per element on the widened operands, bf16 weights
 *          rounded to nearest even once more.
 *  delta : HOST array of L DEVICE pointers to the updates (delta_dt), read only;
 *          must not alias w.
 *  d_out, eps, workspace, numel, arithmetic of the score: as in (a) with
 *          cur_is_delta != 0.
 *
 *  slimfit_apply_update_layer_delta = plan + run.  slimfit_layer_delta_apply_run
 *  runs on a plan written by slimfit_layer_delta_plan(w as w_prev, delta as
 *  w_cur): it WRITES through the planned w_prev pointers.  Without a matching
 *  plan d_out is NaN and no weight is touched.
 * ---------------------------------------------------------------------- */
int32_t slimfit_layer_delta_apply_run(const int64_t *numel, int32_t L, int32_t w_dt, int32_t delta_dt,
                                      float eps, float *d_out,
                                      void *workspace, size_t workspace_bytes, void *stream);

int32_t slimfit_apply_update_layer_delta(void *const *w, int32_t w_dt,
                                         const void *const *delta, int32_t delta_dt,
                                         const int64_t *numel, int32_t L, float eps,
                                         float *d_out, void *workspace, size_t workspace_bytes,
                                         void *stream);

/* ------------------------------------------------------------------------
 * (b) Low-bit caching of saved activations -- Alg. 2 (appendix on the
 *     conversion between fixed point and fp32), Sec. 4 (8 bits = 4 integer +
 *     4 fractional for the imbalanced layer) and Sec. 5 (4 bits for GELU, two
 *     codes stored per byte by shifting).
 *
 *     FIXED (the paper's algorithm): b = bits, fb = frac_bits,
 *         code = clamp(round(x * 2^fb), -2^(b-1), 2^(b-1)-1),   x^ = code / 2^fb
 *       round = half-to-even.  block and scales are ignored (scales may be
 *       NULL).  -32 <= frac_bits <= 32.
 *     BLOCK (per-block scale in place of 2^fb): for each run of `block`
 *       consecutive elements of the flat tensor (the last may be short),
 *         a = max|x|, inv = qmax / a, scale = a / qmax   (qmax = 2^(b-1)-1)
 *         code = clamp(round(x * inv), -2^(b-1), qmax),         x^ = code * scale
 *       all in fp32.  A block with a == 0, or with a so small that qmax / a
 *       overflows fp32, stores scale 0 and codes 0.  block in {32,64,128,256}.
 *     bits in {4, 8}.  Codes are two's complement.  8-bit: byte j = code j.
 *     4-bit: byte m = (code[2m] & 0xF) | (code[2m+1] & 0xF) << 4; an odd n
 *     leaves the last high nibble 0.
 *
 *  x / y  : DEVICE, n elements of dtype dt (bf16 input is widened exactly;
 *           bf16 output is x^ rounded to nearest-even).
 *  codes  : DEVICE uint8[slimfit_packed_bytes(n, bits)].
 *  scales : DEVICE float[slimfit_num_blocks(n, block)] (BLOCK mode).
 * ---------------------------------------------------------------------- */
size_t slimfit_packed_bytes(int64_t n, int32_t bits);  /* ceil(n*bits/8); 0 if n<0 or bad bits */
int64_t slimfit_num_blocks(int64_t n, int32_t block);  /* ceil(n/block);  0 if n<0 or block<=0 */

int32_t slimfit_quant_pack(const void *x, int32_t dt, int64_t n,
                           int32_t mode, int32_t bits, int32_t block, int32_t frac_bits,
                           uint8_t *codes, float *scales, void *stream);

int32_t slimfit_dequant_unpack(const uint8_t *codes, const float *scales, int64_t n,
                               int32_t mode, int32_t bits, int32_t block, int32_t frac_bits,
                               void *y, int32_t dt, void *stream);

/* ------------------------------------------------------------------------
 * (b') The same cache fused into its producer and consumer -- Sec. 4: the
 *     input of GELU is a static activation kept for the backward pass in 4
 *     bits; compression does not change the forward result.
 *
 *  slimfit_gelu_quant_pack       : y = GELU(x) from the exact x, and
 *                                  (codes, scales) = slimfit_quant_pack(x), with
 *                                  x read once.
 *  slimfit_gelu_backward_dequant : dx = dy * GELU'(x^),  x^ = code * scale (the
 *                                  fp32 product slimfit_dequant_unpack forms),
 *                                  never written to memory.
 *  GELU is the exact form  x * (1 + erf(x / sqrt 2)) / 2,  its derivative
 *  (1 + erf(x / sqrt 2)) / 2 + x * exp(-x^2 / 2) / sqrt(2 pi); both in fp32
 *  (codes and scales are bit-identical to the unfused call; y within
 *  4e-7 * |x| + 1e-6 * |y| and dx within 1e-6 * |dy| of the fp64 value, bf16
 *  results within one bf16 rounding of that).
 *
 *  x, y, dy, dx : DEVICE, n elements of dt, 16-byte aligned; y must not be x
 *                 and dx must not be dy (INVALID_ARG), nor overlap them.
 *  other arguments, layouts and errors as in (b).
 * ---------------------------------------------------------------------- */
int32_t slimfit_gelu_quant_pack(const void *x, int32_t dt, int64_t n,
                                int32_t mode, int32_t bits, int32_t block, int32_t frac_bits,
                                void *y, uint8_t *codes, float *scales, void *stream);

int32_t slimfit_gelu_backward_dequant(const uint8_t *codes, const float *scales, int64_t n,
                                      int32_t mode, int32_t bits, int32_t block, int32_t frac_bits,
                                      const void *dy, void *dx, int32_t dt, void *stream);

/* ------------------------------------------------------------------------
 * (c) Pruning to values + indices -- Alg. 5 and the appendix on pruning:
 *     sort from largest to smallest with indices, keep the first k, store
 *     them with their indices (the dense size is rows x cols, which the
 *     caller keeps); restoring creates zeros and scatters the kept values.
 *     Here the algorithm is applied to each row of a row-major rows x cols
 *     matrix (attention probabilities: one row per query).
 *
 *     The kept set of a row is the first k entries of the order "value
 *     descending, then column ascending" (signed comparison; -0 equals +0);
 *     it is emitted in ascending column order.
 *     TOPK      : exactly k pairs per row.
 *     THRESHOLD : the first min(k, #{p >= tau}) pairs of the same order;
 *                 unused slots hold value 0 and index 0xFFFF.
 *
 *  p      : DEVICE, rows*cols elements of dt; alignment = element size.
 *  vals   : DEVICE, rows*k elements of dt, bit copies of the kept inputs.
 *  idx    : DEVICE uint16[rows*k], column of each kept value.
 *  counts : DEVICE int32[rows] or NULL; pairs kept per row (k in TOPK mode).
 *  1 <= k <= cols <= 65536 (else INVALID_ARG / UNSUPPORTED).
 *
 *  slimfit_restore_scores is the backward half: out (rows x cols of dt,
 *  16-byte aligned) is zero-filled and the first counts[r] (or k when counts is
 *  NULL) pairs of each row are scattered into it, in one pass that writes every
 *  output byte once.  An index >= cols is skipped; columns must be distinct
 *  within a row.
 * ---------------------------------------------------------------------- */
int32_t slimfit_keep_count(int32_t cols, int32_t keep_ppm); /* cols*keep_ppm/1e6, integer; -1 on bad input */

int32_t slimfit_prune_scores(const void *p, int32_t dt, int64_t rows, int32_t cols, int32_t k,
                             int32_t mode, float tau,
                             void *vals, uint16_t *idx, int32_t *counts, void *stream);

int32_t slimfit_restore_scores(const void *vals, const uint16_t *idx, const int32_t *counts,
                               int32_t dt, int64_t rows, int32_t cols, int32_t k,
                               void *out, void *stream);

/* ------------------------------------------------------------------------
 * (c'') Pruning fused into the Softmax that produces the probabilities -- the
 *     output of Softmax is the activation that Softmax and the following MatMul
 *     share (Sec. 4); Alg. 5 prunes it for the backward pass while the forward
 *     pass goes on with the dense row.
 *
 *     Per row of logits:  p_j = exp(l_j - max l) / sum_i exp(l_i - max l)  is
 *     written to probs (dense, for the forward MatMul), and the k pairs that
 *     slimfit_prune_scores would keep are written to vals / idx.  The kept set
 *     is decided on the logits: they order the row exactly as the probabilities
 *     do and are not subject to rounding (equal logits: lower column first);
 *     vals are the row's p_j, emitted in ascending column order.  Arithmetic is
 *     fp32 (hardware exp2, a sum in a fixed order, one IEEE division per row):
 *     p_j within p_j * (2e-6 + 2e-7 * (max l - l_j)) of the exact value (a
 *     subnormal p_j may be flushed to zero), bf16 results within one further
 *     bf16 rounding.
 *
 *  logits, probs : DEVICE, rows*cols elements of dt, distinct buffers.
 *  vals, idx     : as in (c).   1 <= k <= cols <= 2048 (wider rows: UNSUPPORTED).
 * ---------------------------------------------------------------------- */
int32_t slimfit_softmax_prune(const void *logits, int32_t dt, int64_t rows, int32_t cols, int32_t k,
                              void *probs, void *vals, uint16_t *idx, void *stream);

/* ------------------------------------------------------------------------
 * (c-back) Backward pass of Softmax straight from the pruned probabilities -- the
 *     consumer of the pairs that (c) and (c'') emit (Sec. 4 caches Softmax's
 *     output for its backward pass; Alg. 5's restoring process rebuilds it as
 *     p^ = zeros + scatter).  With p^ in place of p in the derivative of Softmax,
 *
 *         ds_j = p^_j * (dp_j - sum_i p^_i dp_i),
 *
 *     which is zero wherever nothing was kept; the dense p^ is never written.
 *     fp32 arithmetic: the sum runs over a row's pairs in a fixed order (lane
 *     partials, then the wave), ds_j within
 *     |p^_j| * ((8 + k/64) * 6e-8 * sum_i |p^_i dp_i| + 1.2e-7 * |dp_j|) + 6e-8 * |ds_j|
 *     of the exact value; bf16 results within one further bf16 rounding.
 *
 *  vals, idx, counts : DEVICE, as (c) wrote them (counts may be NULL: k pairs per
 *                      row; an index >= cols marks an unused slot).
 *  dp                : DEVICE, rows*cols elements of dt, the gradient w.r.t. the
 *                      probabilities; only the kept columns are read.
 *  ds                : DEVICE, rows*cols elements of dt, 16-byte aligned, not dp;
 *                      every element is written once.
 *  1 <= k <= cols <= 65536.
 * ---------------------------------------------------------------------- */
int32_t slimfit_softmax_backward_pruned(const void *vals, const uint16_t *idx, const int32_t *counts,
                                        const void *dp, int32_t dt, int64_t rows, int32_t cols, int32_t k,
                                        void *ds, void *stream);

/* ------------------------------------------------------------------------
 * (c') Alg. 5 on a whole flattened tensor -- the form the paper applies to the
 *     standardised input of LayerNorm: sort all n entries from largest to
 *     smallest with their indices, keep the first k = int(n * 0.1), store the
 *     values with int32 indices; restoring creates zeros(n) and scatters.
 *
 *     by_magnitude != 0 orders by |x| (discarding the small values of a signed
 *     tensor), by_magnitude == 0 by the signed value (-0 equals +0).  Equal
 *     keys go by lower index.  The k survivors are emitted in ascending index
 *     order; vals are bit copies of the (signed) inputs.  NaN inputs are
 *     outside the contract.
 *
 *  x         : DEVICE, n elements of dt, 16-byte aligned.  0 <= k <= n < 2^31
 *              (k == 0 or n == 0: nothing is written).
 *  vals, idx : DEVICE, k elements of dt / int32[k].
 *  tile_ptr  : DEVICE int32[slimfit_global_tile_ptr_len(n)] or NULL.  Optional
 *              companion of the index list, not part of the paper's format:
 *              tile_ptr[t] = number of survivors whose index is below
 *              t * SLIMFIT_GLOBAL_TILE, the last entry = k.  With it the
 *              restoring process builds every output tile once instead of
 *              filling zeros and scattering into them.
 *  workspace : DEVICE, 16-byte aligned, at least the byte count that
 *              slimfit_prune_global_workspace(n) reports (about n/2 bytes);
 *              owned by the caller, contents need not be initialised and are
 *              overwritten.  Calls that share a workspace must not overlap.
 *  slimfit_restore_global : out (n elements of dt, 16-byte aligned) = zeros,
 *              then out[idx[s]] = vals[s] for s < k; an index outside [0, n) is
 *              skipped; indices must be distinct.  tile_ptr == NULL accepts the
 *              pairs in any order.  With tile_ptr the pairs must be in ascending
 *              index order with pointers as described above (what
 *              slimfit_prune_global emits); a pair filed under the wrong tile
 *              is skipped, never written out of bounds.
 *  Errors: INVALID_ARG (dtype, sizes, null pointers), UNSUPPORTED (n >= 2^31),
 *  ALIGNMENT, WORKSPACE (too small), POINTER, HIP.
 * ---------------------------------------------------------------------- */
#define SLIMFIT_GLOBAL_TILE 4096

int32_t slimfit_prune_global_workspace(int64_t n, size_t *bytes);
int64_t slimfit_global_tile_ptr_len(int64_t n);   /* ceil(n / SLIMFIT_GLOBAL_TILE) + 1; -1 if n < 0 or n >= 2^31 */

int32_t slimfit_prune_global(const void *x, int32_t dt, int64_t n, int64_t k, int32_t by_magnitude,
                             void *vals, int32_t *idx, int32_t *tile_ptr,
                             void *workspace, size_t workspace_bytes, void *stream);

int32_t slimfit_restore_global(const void *vals, const int32_t *idx, const int32_t *tile_ptr, int64_t k,
                               int32_t dt, int64_t n, void *out, void *stream);

/* ------------------------------------------------------------------------
 * (c-ln) LayerNorm around the pruned cache of its standardised input -- Sec. 4:
 *        x~ = (x - E x) / sqrt(Var x + eps),   y = x~ * gamma + beta   per row of
 *     H elements (Var with divisor H).  A frozen LayerNorm keeps only the
 *     largest 10 % of x~ (Alg. 5) and computes its input gradient as
 *        g = gamma * y^ / (H * sqrt(Var x + eps)),
 *        x^ = H * g - sum_H g - x~ * sum_H (g * x~),
 *     every pruned x~ counting as 0.  fp32 arithmetic with fixed-order sums.
 *     gamma, beta, the statistics and the parameter gradients are always fp32;
 *     the entry points that take dt accept x / y / dy / dx as fp32 or bf16 (bf16
 *     inputs are widened exactly, bf16 outputs are the fp32 results rounded to
 *     nearest even: one further bf16 rounding on top of the tolerances below).
 *     The standardised values are fp32 numbers whatever the input's type, so
 *     the kept values (vals of slimfit_prune_global_standardized and of
 *     slimfit_layernorm_backward_pruned) are always fp32.
 *
 *  slimfit_layernorm_forward : y, and per row mean = E x and
 *        rstd = 1 / sqrt(Var x + eps).  Against the fp64 values: mean within
 *        1e-6 * max|x_row|, rstd within 2e-6 relative,
 *        |d y| <= |gamma| * (4e-6 * |x~| + 2e-6 * max|x_row| * rstd) + 1e-6 * |y|.
 *  slimfit_prune_global_standardized : slimfit_prune_global applied to x~
 *        without storing it: element j of row r enters as
 *        fl(fl(x_j - mean[r]) * rstd[r]) (two fp32 operations), vals receive
 *        those values as fp32 (x itself fp32 or bf16, widened exactly).
 *        n = rows * H; H a multiple of 4 (fp32) or 8 (bf16).
 *        mean, rstd: DEVICE float[n / H].
 *        row_ptr: DEVICE int32[n / H + 1] or NULL; row_ptr[r] = number of
 *        survivors with index below r * H, the last entry = k (the pairs of row
 *        r are [row_ptr[r], row_ptr[r+1]) of the list).
 *  slimfit_layernorm_backward_pruned : x^ from the pairs (vals, idx, row_ptr as
 *        slimfit_prune_global_standardized emits them; row_ptr is required),
 *        rstd, gamma and y^ (dy); a pair whose index does not fall in the row
 *        the pointers file it under is skipped.
 *        |d x^| <= 4e-6 * (H * |g| + sum_H |g| + |x~| * sum_H |g * x~|).
 *  x, y, dy, dx : DEVICE, rows * H elements of dt, 16-byte aligned, outputs
 *  distinct from inputs; gamma, beta : DEVICE float[H], 16-byte aligned.
 *  H <= 4096, a multiple of 4 (fp32) or 8 (bf16), rows * H < 2^31 (else
 *  INVALID_ARG / UNSUPPORTED).
 * ---------------------------------------------------------------------- */
int32_t slimfit_layernorm_forward(const void *x, int32_t dt, const float *gamma, const float *beta,
                                  int64_t rows, int64_t H, float eps, void *y, float *mean, float *rstd,
                                  void *stream);

int32_t slimfit_prune_global_standardized(const void *x, int32_t dt, int64_t n, int64_t H,
                                          const float *mean, const float *rstd, int64_t k, int32_t by_magnitude,
                                          void *vals, int32_t *idx, int32_t *tile_ptr, int32_t *row_ptr,
                                          void *workspace, size_t workspace_bytes, void *stream);

/* Input gradient of an active (not frozen) LayerNorm, Sec. 4: the formula above with every
 * x~ present, x~ = (x - mean[r]) * rstd[r] from the statistics slimfit_layernorm_forward
 * returned; same tolerance as slimfit_layernorm_backward_pruned.  dx must be neither x nor dy. */
int32_t slimfit_layernorm_backward(const void *x, int32_t dt, const float *mean, const float *rstd,
                                   const float *gamma, const void *dy, int64_t rows, int64_t H, void *dx,
                                   void *stream);

/* Parameter gradients of an active (not frozen) LayerNorm, Sec. 4:
 *   gamma^_j = sum over rows of x~_rj * y^_rj,   beta^_j = sum over rows of y^_rj,
 * x~ = (x - mean[r]) * rstd[r] from the statistics slimfit_layernorm_forward returned.
 * fp32 products and slab sums (256 rows, four interleaved quarters), fp64 across slabs, fixed order (no atomics):
 * within 4e-6 * sum_r |x~ * y^| (resp. |y^|) of the fp64 value.
 * dgamma, dbeta : DEVICE float[H].  workspace: DEVICE, 16-byte aligned, at least
 * slimfit_layernorm_param_grads_workspace(rows, H) bytes; contents overwritten. */
int32_t slimfit_layernorm_param_grads_workspace(int64_t rows, int64_t H, size_t *bytes);

int32_t slimfit_layernorm_param_grads(const void *x, int32_t dt, const float *mean, const float *rstd,
                                      const void *dy, int64_t rows, int64_t H, float *dgamma, float *dbeta,
                                      void *workspace, size_t workspace_bytes, void *stream);

int32_t slimfit_layernorm_backward_pruned(const float *vals, const int32_t *idx, const int32_t *row_ptr, int64_t k,
                                          const float *rstd, const float *gamma, const void *dy, int32_t dt,
                                          int64_t rows, int64_t H, void *dx, void *stream);

/* LayerNorm with the low-bit cache of its input (Alg. 2, one scale per block; Sec. 4 and 5) fused in.
 *   slimfit_layernorm_forward_quant_pack : slimfit_layernorm_forward and, from the same read of x,
 *        the codes and scales slimfit_quant_pack(x, dt, rows*H, BLOCK, bits, block) produces --
 *        bit for bit -- so the input is read once instead of twice.
 *   slimfit_layernorm_backward_dequant   : slimfit_layernorm_backward on x^ = code * scale (one fp32
 *        multiplication, the value slimfit_dequant_unpack would store) without storing x^:
 *        x~ = (x^ - mean[r]) * rstd[r] with the statistics the forward pass returned (those of the
 *        exact input).  Same tolerance as slimfit_layernorm_backward.
 * bits 4 | 8; block 32 | 64 | 128 | 256 and H % block == 0, so that no block straddles two rows (else
 * UNSUPPORTED).  codes: DEVICE uint8[rows*H*bits/8]; scales: DEVICE float[rows*H/block]; both 16-byte
 * aligned.  Everything else as slimfit_layernorm_forward / slimfit_layernorm_backward. */
int32_t slimfit_layernorm_forward_quant_pack(const void *x, int32_t dt, const float *gamma, const float *beta,
                                             int64_t rows, int64_t H, float eps, int32_t bits, int32_t block,
                                             void *y, float *mean, float *rstd, uint8_t *codes, float *scales,
                                             void *stream);

int32_t slimfit_layernorm_backward_dequant(const uint8_t *codes, const float *scales, int32_t bits, int32_t block,
                                           const float *mean, const float *rstd, const float *gamma,
                                           const void *dy, int32_t dt, int64_t rows, int64_t H, void *dx,
                                           void *stream);

/* ------------------------------------------------------------------------
 * (d) Inter-layer scheduling on the host -- Alg. 1 and Sec. 3.2 / Fig. 4:
 *        idx = argsort(d)[: int(L*F)]   -> these layers are frozen;
 *     afterwards only the layers that were active take their new distance,
 *     frozen layers keep the old one.  Every pointer is a HOST pointer.
 *
 *  slimfit_freeze_count : int(L*F) evaluated in double like the pseudo code;
 *                         -1 if L < 0 or F outside [0, 1].
 *  slimfit_ils_select   : frozen_idx[0..n_freeze) = the n_freeze layers with
 *                         the smallest d, smallest first; equal values go by
 *                         lower index; NaN orders after +inf.  mask (uint8[L]
 *                         or NULL) gets 1 for frozen, 0 for active.
 *  slimfit_ils_update   : d[i] = new_scores[i] where frozen_mask[i] == 0.
 *  slimfit_ils_select_blocks : the same selection at the granularity of blocks of
 *                         `group` consecutive layers (the tensors of one encoder
 *                         block; the last block may be shorter): a block's
 *                         distance is the mean of its layers' d, summed in layer
 *                         order in double; frozen_blocks[0..n_freeze) = the blocks
 *                         with the smallest means, same ordering rules; mask
 *                         (uint8[L] or NULL) gets 1 for every layer of a frozen
 *                         block.  n_freeze <= ceil(L / group).  group = 1 is
 *                         slimfit_ils_select.
 * ---------------------------------------------------------------------- */
int32_t slimfit_freeze_count(int32_t L, double F);

int32_t slimfit_ils_select(const float *d, int32_t L, int32_t n_freeze,
                           int32_t *frozen_idx, uint8_t *mask);

int32_t slimfit_ils_select_blocks(const float *d, int32_t L, int32_t group, int32_t n_freeze,
                                  int32_t *frozen_blocks, uint8_t *mask);

int32_t slimfit_ils_update(float *d, const float *new_scores,
                           const uint8_t *frozen_mask, int32_t L);

/* ------------------------------------------------------------------------
 * (d') The two schedules the paper compares ILS with (its ablation of freezing
 *     schedules): "random" draws the int(L*F) frozen layers uniformly at random
 *     at every iteration, "progressive" keeps the earliest layers frozen and
 *     updates the later ones throughout.  HOST pointers, same outputs as
 *     slimfit_ils_select.
 *
 *  slimfit_schedule_random : a function of (seed, iteration) only.  The draw is
 *     the first n_freeze steps of a Fisher-Yates shuffle of 0..L-1 (step i swaps
 *     entry i with entry i + next() mod (L - i)), next() being SplitMix64
 *     started at seed XOR (iteration * 0xD6E8FEB86659FD93).  frozen_idx lists
 *     the picks in the order drawn.
 *  slimfit_schedule_progressive : frozen_idx = 0 .. n_freeze-1.
 *  INVALID_ARG if L < 0, n_freeze outside [0, L] or frozen_idx is NULL with
 *  n_freeze > 0; mask may be NULL.
 * ---------------------------------------------------------------------- */
int32_t slimfit_schedule_random(int32_t L, int32_t n_freeze, uint64_t seed, uint64_t iteration,
                                int32_t *frozen_idx, uint8_t *mask);

int32_t slimfit_schedule_progressive(int32_t L, int32_t n_freeze, int32_t *frozen_idx, uint8_t *mask);

#ifdef __cplusplus
}
#endif
#endif /* SLIMFIT_H */
