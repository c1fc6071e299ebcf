/*
 * SlimFit hot path -- CPU oracle (TEST INFRASTRUCTURE, not a product path).
 *
 * A plain, slow, obviously-correct implementation of what the GPU library
 * computes, written from the paper's definitions.  It shares no code with the
 * HIP path: only tests, the smoke check and the benchmark's cpu_baseline leg
 * may load it.  Every pointer is a HOST pointer.  Each function runs its
 * independent units (layers, quantisation blocks, score rows) sequentially or,
 * when threads > 1, under "omp parallel for" over those units only, which
 * cannot change any result.
 *
 * Precision: the distance score (Eq. 1) is evaluated in fp64.  The quantiser
 * (Alg. 2) is evaluated in fp32 because the paper fixes that precision (all
 * tensors are single precision and the rounding decides an integer code).
 *
 * dtype codes: 0 = fp32, 1 = bf16 (raw uint16 bit patterns).
 * Return value: 0 on success, a negative number for an argument the
 * definition does not cover.
 *
 * Pins (tests/, -m "not gpu"): Fig. 4 replay for the ILS pair (and, with
 * blocks of one layer, for its block-granularity variant, which is further
 * pinned by NumPy means with a stable argsort and a worked example); closed forms,
 * scaling/sign/permutation invariants and a NumPy float64 one-liner for
 * Eq. 1; exhaustive grid against Alg. 2 in double, half-step bound,
 * idempotence and pack/unpack identity for the quantiser; brute-force
 * repeat-argmax selector and a library stable argsort for the pruner (row-wise
 * and whole-tensor forms); textbook values, the reflection identity, a library
 * normal CDF and numerical differentiation for GELU and its derivative; a
 * library layer norm and its automatic derivative (fp64) for LayerNorm, the
 * paper's input-gradient formula and the parameter gradients; a library
 * softmax and brute force on the exact probabilities for the fused softmax +
 * pruning, the automatic derivative of a library softmax for its backward
 * pass; the generator's published known answers, big-integer arithmetic
 * and a chi-square test for the random freezing schedule.
 * Parity unpinned by the paper (it prints no worked numbers for them): the
 * per-block-scale mode, the 4-bit split of integer/fraction bits, the
 * threshold pruning mode, bf16 I/O, and everything beyond its Fig. 4 example
 * (the paper prints formulas, not values, for GELU, Softmax, LayerNorm and
 * Alg. 5).  Those are pinned by brute force, closed forms, library routines
 * and invariants only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REF_OK 0
#define REF_BAD (-1)

/* ------------------------------------------------------------------ */
/* bf16 <-> fp32                                                        */
/* ------------------------------------------------------------------ */

static float bf16_widen(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even on the 16 discarded bits; NaN stays NaN */
static uint16_t bf16_narrow(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep = u >> 16;
    uint32_t rest = u & 0xffffu;
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u)))
        keep += 1u;
    return (uint16_t)keep;
}

static float load_elem(const void *p, int dt, int64_t j)
{
    if (dt == 0)
        return ((const float *)p)[j];
    return bf16_widen(((const uint16_t *)p)[j]);
}

static void store_elem(void *p, int dt, int64_t j, float v)
{
    if (dt == 0)
        ((float *)p)[j] = v;
    else
        ((uint16_t *)p)[j] = bf16_narrow(v);
}

static int dtype_ok(int dt) { return dt == 0 || dt == 1; }

/* ------------------------------------------------------------------ */
/* Eq. 1 -- training-dynamics distance of one layer                     */
/*   d_i = 1/(M*I) * sum_j | (W^t_ij - W^{t-1}_ij) / W^{t-1}_ij |       */
/* Entry-wise l1 (the 1/(M*I) normaliser makes it a mean).  Readings    */
/* where the paper is silent: an element whose weight did not change    */
/* contributes 0 even if the old weight is 0; otherwise IEEE division   */
/* (a zero old weight with a non-zero change gives +inf) unless the     */
/* caller passes eps > 0, which floors the denominator's magnitude.     */
/* An empty layer scores 0.                                             */
/* ------------------------------------------------------------------ */

static float layer_distance(const void *w_prev, int prev_dt, const void *w_cur,
                            int cur_dt, int cur_is_delta, int64_t n, float eps)
{
    if (n <= 0)
        return 0.0f;
    double sum = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        double wp = (double)load_elem(w_prev, prev_dt, j);
        double c = (double)load_elem(w_cur, cur_dt, j);
        double delta = cur_is_delta ? c : c - wp;
        if (delta == 0.0)
            continue;
        double den = fabs(wp);
        if (den < (double)eps)
            den = (double)eps;
        sum += fabs(delta) / den;
    }
    return (float)(sum / (double)n);
}

int slimfit_ref_layer_delta(const void *const *w_prev, int prev_dt,
                            const void *const *w_cur, int cur_dt,
                            int cur_is_delta, const int64_t *numel, int L,
                            float eps, float *d_out, int threads)
{
    if (L < 0 || !dtype_ok(prev_dt) || !dtype_ok(cur_dt) || !(eps >= 0.0f))
        return REF_BAD;
    if (L == 0)
        return REF_OK;
    if (!w_prev || !w_cur || !numel || !d_out)
        return REF_BAD;
    for (int i = 0; i < L; ++i)
        if (numel[i] < 0 || (numel[i] > 0 && (!w_prev[i] || !w_cur[i])))
            return REF_BAD;
    if (threads < 1)
        threads = 1;
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
    for (int i = 0; i < L; ++i)
        d_out[i] = layer_distance(w_prev[i], prev_dt, w_cur[i], cur_dt,
                                  cur_is_delta, numel[i], eps);
    return REF_OK;
}

/* Eq. 1 measured while the optimizer's update is applied: the caller   */
/* hands over W^{t-1} and the update delta = W^t - W^{t-1}; the score is */
/* that of the function above with cur_is_delta, and the weights become  */
/* W^t = W^{t-1} + delta -- one fp32 addition on the widened operands,   */
/* rounded once more to bf16 for bf16 weights.  No copy of W^{t-1} has   */
/* to be kept for the score.                                             */
int slimfit_ref_apply_update_layer_delta(void *const *w, int w_dt,
                                         const void *const *delta, int delta_dt,
                                         const int64_t *numel, int L, float eps,
                                         float *d_out, int threads)
{
    if (L < 0 || !dtype_ok(w_dt) || !dtype_ok(delta_dt) || !(eps >= 0.0f))
        return REF_BAD;
    if (L == 0)
        return REF_OK;
    if (!w || !delta || !numel || !d_out)
        return REF_BAD;
    for (int i = 0; i < L; ++i)
        if (numel[i] < 0 || (numel[i] > 0 && (!w[i] || !delta[i])))
            return REF_BAD;
    if (threads < 1)
        threads = 1;
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
    for (int i = 0; i < L; ++i) {
        d_out[i] = layer_distance(w[i], w_dt, delta[i], delta_dt, 1, numel[i], eps);
        for (int64_t j = 0; j < numel[i]; ++j) {
            volatile float sum = load_elem(w[i], w_dt, j) + load_elem(delta[i], delta_dt, j);
            store_elem(w[i], w_dt, j, sum);
        }
    }
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* Alg. 2 -- fixed-point conversion, plus the per-block-scale variant   */
/*   quantise:   y = clamp(round(x * 2^fb), -2^(b-1), 2^(b-1)-1)        */
/*   dequantise: x = y / 2^fb                                           */
/* round = half-to-even (the paper's code is PyTorch, whose round is).  */
/* mode 0 (FIXED): exactly the above, b = ib + fb total bits.           */
/* mode 1 (BLOCK): 2^fb is replaced, per run of `block` consecutive     */
/*   elements of the flattened tensor, by inv = qmax / absmax; the      */
/*   stored scale = absmax / qmax replaces 1/2^fb on the way back.      */
/*   Degenerate block (absmax == 0, or so small that qmax/absmax        */
/*   overflows fp32): scale 0 and all codes 0.                          */
/* Codes are signed two's-complement; 4-bit codes are stored two per    */
/* byte by shifting, element 2m in the low nibble, 2m+1 in the high     */
/* one; an odd tail pads the high nibble with 0.                        */
/* ------------------------------------------------------------------ */

static int quant_args_ok(int dt, int64_t n, int mode, int bits, int block,
                         int frac_bits)
{
    if (!dtype_ok(dt) || n < 0)
        return 0;
    if (bits != 4 && bits != 8)
        return 0;
    if (mode == 0)
        return frac_bits >= -32 && frac_bits <= 32;
    if (mode == 1)
        return block == 32 || block == 64 || block == 128 || block == 256;
    return 0;
}

static int quantise_one(float x, float mult, int qmin, int qmax)
{
    float q = x * mult;              /* one fp32 multiply */
    float r = nearbyintf(q);         /* half-to-even under the default mode */
    if (r != r)
        return 0;                    /* NaN is outside the contract */
    if (r < (float)qmin)
        r = (float)qmin;
    if (r > (float)qmax)
        r = (float)qmax;
    return (int)r;
}

static void put_code(uint8_t *codes, int bits, int64_t j, int c)
{
    if (bits == 8) {
        codes[j] = (uint8_t)(c & 0xff);
    } else {
        int64_t m = j >> 1;
        uint8_t nib = (uint8_t)(c & 0xf);
        if ((j & 1) == 0)
            codes[m] = nib;                       /* also zeroes the pad */
        else
            codes[m] = (uint8_t)(codes[m] | (nib << 4));
    }
}

static int get_code(const uint8_t *codes, int bits, int64_t j)
{
    if (bits == 8)
        return (int)(int8_t)codes[j];
    uint8_t byte = codes[j >> 1];
    int nib = (j & 1) ? (byte >> 4) : (byte & 0xf);
    return nib >= 8 ? nib - 16 : nib;             /* sign-extend */
}

int slimfit_ref_quant_pack(const void *x, int dt, int64_t n, int mode, int bits,
                           int block, int frac_bits, uint8_t *codes,
                           float *scales, int threads)
{
    if (!quant_args_ok(dt, n, mode, bits, block, frac_bits))
        return REF_BAD;
    if (n == 0)
        return REF_OK;
    if (!x || !codes || (mode == 1 && !scales))
        return REF_BAD;
    const int qmax = (1 << (bits - 1)) - 1;
    const int qmin = -(1 << (bits - 1));
    if (threads < 1)
        threads = 1;

    if (mode == 0) {
        const float mult = ldexpf(1.0f, frac_bits);
        /* pairs of elements: neighbouring 4-bit codes share a byte */
        const int64_t npair = (n + 1) / 2;
#pragma omp parallel for num_threads(threads) schedule(static)
        for (int64_t m = 0; m < npair; ++m)
            for (int64_t j = 2 * m; j < 2 * m + 2 && j < n; ++j)
                put_code(codes, bits, j,
                         quantise_one(load_elem(x, dt, j), mult, qmin, qmax));
        return REF_OK;
    }

    const int64_t nblk = (n + block - 1) / block;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t b = 0; b < nblk; ++b) {
        int64_t lo = b * block;
        int64_t hi = lo + block < n ? lo + block : n;
        float a = 0.0f;
        for (int64_t j = lo; j < hi; ++j) {
            float m = fabsf(load_elem(x, dt, j));
            if (m > a)
                a = m;
        }
        float inv = 0.0f, scale = 0.0f;
        if (a > 0.0f) {
            inv = (float)qmax / a;               /* one fp32 division */
            if (isinf(inv))
                inv = 0.0f;
            else
                scale = a / (float)qmax;         /* one fp32 division */
        }
        scales[b] = scale;
        /* block sizes are even, so a block never shares a byte with its
         * neighbour and blocks may run in parallel */
        for (int64_t j = lo; j < hi; ++j)
            put_code(codes, bits, j,
                     quantise_one(load_elem(x, dt, j), inv, qmin, qmax));
    }
    return REF_OK;
}

int slimfit_ref_dequant_unpack(const uint8_t *codes, const float *scales,
                               int64_t n, int mode, int bits, int block,
                               int frac_bits, void *y, int dt, int threads)
{
    if (!quant_args_ok(dt, n, mode, bits, block, frac_bits))
        return REF_BAD;
    if (n == 0)
        return REF_OK;
    if (!y || !codes || (mode == 1 && !scales))
        return REF_BAD;
    if (threads < 1)
        threads = 1;
    const float step = ldexpf(1.0f, frac_bits);
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        float c = (float)get_code(codes, bits, j);
        float v = (mode == 0) ? c / step           /* exact: power of two */
                              : c * scales[j / block];
        store_elem(y, dt, j, v);
    }
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* Alg. 5 -- pruning to (values, indices), applied to every row         */
/*   sort the row from largest to smallest with indices, keep the       */
/*   first k.  Readings: ties are broken by the lower column; the kept  */
/*   pairs are emitted in ascending column order (the set is what       */
/*   matters; restoring gives the same dense row either way).           */
/* mode 0 (TOPK): exactly k pairs.                                      */
/* mode 1 (THRESHOLD): the first min(k, #{p >= tau}) pairs of the same  */
/*   order; unused slots hold value 0 and index 0xFFFF.                 */
/* counts (optional) receives the number of pairs kept per row.         */
/* ------------------------------------------------------------------ */

typedef struct {
    float v;
    int32_t col;
} ref_pair;

static int pair_before(const void *pa, const void *pb)
{
    const ref_pair *a = (const ref_pair *)pa, *b = (const ref_pair *)pb;
    if (a->v > b->v)
        return -1;
    if (a->v < b->v)
        return 1;
    return (a->col > b->col) - (a->col < b->col);
}

int slimfit_ref_prune_scores(const void *p, int dt, int64_t rows, int cols,
                             int k, int mode, float tau, void *vals,
                             uint16_t *idx, int32_t *counts, int threads)
{
    if (!dtype_ok(dt) || rows < 0 || cols < 1 || cols > 65536 || k < 1 ||
        k > cols || (mode != 0 && mode != 1))
        return REF_BAD;
    if (rows == 0)
        return REF_OK;
    if (!p || !vals || !idx)
        return REF_BAD;
    if (threads < 1)
        threads = 1;
    int failed = 0;
#pragma omp parallel num_threads(threads)
    {
        ref_pair *buf = (ref_pair *)malloc(sizeof(ref_pair) * (size_t)cols);
        uint8_t *kept = (uint8_t *)malloc((size_t)cols);
        if (!buf || !kept) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t r = 0; r < rows; ++r) {
            if (!buf || !kept)
                continue;
            const int64_t base = r * (int64_t)cols;
            for (int c = 0; c < cols; ++c) {
                buf[c].v = load_elem(p, dt, base + c);
                buf[c].col = c;
            }
            qsort(buf, (size_t)cols, sizeof(ref_pair), pair_before);
            int take = k;
            if (mode == 1) {
                int pass = 0;
                while (pass < cols && buf[pass].v >= tau)
                    ++pass;
                if (pass < take)
                    take = pass;
            }
            memset(kept, 0, (size_t)cols);
            for (int s = 0; s < take; ++s)
                kept[buf[s].col] = 1;
            int out = 0;
            const int64_t obase = r * (int64_t)k;
            for (int c = 0; c < cols; ++c) {
                if (!kept[c])
                    continue;
                /* the stored value is a bit copy of the input element */
                if (dt == 0)
                    ((float *)vals)[obase + out] =
                        ((const float *)p)[base + c];
                else
                    ((uint16_t *)vals)[obase + out] =
                        ((const uint16_t *)p)[base + c];
                idx[obase + out] = (uint16_t)c;
                ++out;
            }
            for (; out < k; ++out) {
                if (dt == 0)
                    ((float *)vals)[obase + out] = 0.0f;
                else
                    ((uint16_t *)vals)[obase + out] = 0;
                idx[obase + out] = 0xFFFFu;
            }
            if (counts)
                counts[r] = take;
        }
        free(buf);
        free(kept);
    }
    return failed ? REF_BAD : REF_OK;
}

/* Alg. 5, restoring process: zeros(numel) then scatter the kept values.
 * counts == NULL means every row holds k pairs. */
int slimfit_ref_restore_scores(const void *vals, const uint16_t *idx,
                               const int32_t *counts, int dt, int64_t rows,
                               int cols, int k, void *out, int threads)
{
    if (!dtype_ok(dt) || rows < 0 || cols < 1 || cols > 65536 || k < 1 ||
        k > cols)
        return REF_BAD;
    if (rows == 0)
        return REF_OK;
    if (!vals || !idx || !out)
        return REF_BAD;
    if (threads < 1)
        threads = 1;
    const size_t esz = dt == 0 ? 4 : 2;
    int bad = 0;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        char *orow = (char *)out + (size_t)r * (size_t)cols * esz;
        memset(orow, 0, (size_t)cols * esz);
        int cnt = counts ? counts[r] : k;
        if (cnt < 0 || cnt > k) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        for (int s = 0; s < cnt; ++s) {
            uint16_t c = idx[r * (int64_t)k + s];
            if ((int)c >= cols) {
#pragma omp atomic write
                bad = 1;
                continue;
            }
            memcpy(orow + (size_t)c * esz,
                   (const char *)vals + ((size_t)r * (size_t)k + (size_t)s) * esz,
                   esz);
        }
    }
    return bad ? REF_BAD : REF_OK;
}

/* ------------------------------------------------------------------ */
/* GELU, whose input is the activation that Sec. 4 caches in 4 bits.    */
/* The paper names the function without printing it; this is the exact  */
/* (erf) form,  GELU(x) = x * Phi(x),  Phi(x) = (1 + erf(x / sqrt 2))/2, */
/* and its derivative  Phi(x) + x * phi(x),  phi(x) = exp(-x^2/2)/sqrt(2 pi). */
/* Evaluated in fp64 on the widened inputs, rounded once to the output  */
/* dtype.  The fused GPU entry points are this composed with the        */
/* quantiser above: forward caches quant(x) and returns GELU(x);        */
/* backward returns dy * GELU'(x^) with x^ = code * scale in fp32.      */
/* ------------------------------------------------------------------ */

/* (1 + erf(t)) / 2 written as erfc(-t) / 2, which keeps its accuracy in the left tail */
static double gelu_value(double x) { return 0.5 * x * erfc(-x * 0.70710678118654752440); }

static double gelu_slope(double x)
{
    const double cdf = 0.5 * erfc(-x * 0.70710678118654752440);
    const double pdf = exp(-0.5 * x * x) * 0.39894228040143267794;
    return cdf + x * pdf;
}

int slimfit_ref_gelu(const void *x, int dt, int64_t n, void *y)
{
    if (!dtype_ok(dt) || n < 0 || (n > 0 && (!x || !y)))
        return REF_BAD;
    for (int64_t j = 0; j < n; ++j)
        store_elem(y, dt, j, (float)gelu_value((double)load_elem(x, dt, j)));
    return REF_OK;
}

/* xhat is always fp32 (the dequantised cache); dy and dx have dtype dt */
int slimfit_ref_gelu_backward(const float *xhat, const void *dy, int dt, int64_t n, void *dx)
{
    if (!dtype_ok(dt) || n < 0 || (n > 0 && (!xhat || !dy || !dx)))
        return REF_BAD;
    for (int64_t j = 0; j < n; ++j)
        store_elem(dx, dt, j, (float)((double)load_elem(dy, dt, j) * gelu_slope((double)xhat[j])));
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* Softmax whose output Alg. 5 prunes (the attention probabilities that */
/* Softmax and the following MatMul share as their cached activation).  */
/* Per row:  p_j = exp(l_j - max_i l_i) / sum_i exp(l_i - max_i l_i),   */
/* evaluated in fp64 on the widened logits and rounded once to dt.      */
/* The kept set is decided on the logits, which order the row exactly   */
/* as the probabilities do (exp is increasing) but are not subject to   */
/* rounding: first k of "logit descending, column ascending", emitted   */
/* in ascending column order; the kept values are the row's p_j.        */
/* probs may be NULL (only the pruned form is wanted).                  */
/* ------------------------------------------------------------------ */

int slimfit_ref_softmax_prune(const void *logits, int dt, int64_t rows, int cols,
                              int k, void *probs, void *vals, uint16_t *idx,
                              int threads)
{
    if (!dtype_ok(dt) || rows < 0 || cols < 1 || cols > 65536 || k < 1 || k > cols)
        return REF_BAD;
    if (rows > 0 && (!logits || !vals || !idx))
        return REF_BAD;
    int bad = 0;
    (void)threads;
#pragma omp parallel for num_threads(threads > 1 ? threads : 1) schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t base = r * (int64_t)cols;
        double *e = (double *)malloc(sizeof(double) * (size_t)cols);
        ref_pair *buf = (ref_pair *)malloc(sizeof(ref_pair) * (size_t)cols);
        uint8_t *kept = (uint8_t *)calloc((size_t)cols, 1);
        if (!e || !buf || !kept) {
            bad = 1;
            free(e);
            free(buf);
            free(kept);
            continue;
        }
        double top = -INFINITY, sum = 0.0;
        for (int c = 0; c < cols; ++c) {
            buf[c].v = load_elem(logits, dt, base + c);
            buf[c].col = c;
            if ((double)buf[c].v > top)
                top = (double)buf[c].v;
        }
        for (int c = 0; c < cols; ++c) {
            e[c] = exp((double)buf[c].v - top);
            sum += e[c];
        }
        if (probs)
            for (int c = 0; c < cols; ++c)
                store_elem(probs, dt, base + c, (float)(e[c] / sum));
        qsort(buf, (size_t)cols, sizeof(ref_pair), pair_before);
        for (int s = 0; s < k; ++s)
            kept[buf[s].col] = 1;
        int out = 0;
        for (int c = 0; c < cols; ++c) {
            if (!kept[c])
                continue;
            store_elem(vals, dt, r * (int64_t)k + out, (float)(e[c] / sum));
            idx[r * (int64_t)k + out] = (uint16_t)c;
            ++out;
        }
        free(e);
        free(buf);
        free(kept);
    }
    return bad ? REF_BAD : REF_OK;
}

/* Backward pass of Softmax from the pruned probabilities: with p^ the row that  */
/* Alg. 5's restoring process rebuilds (the kept p_j, zeros elsewhere) and dp the */
/* gradient with respect to the probabilities,                                    */
/*     ds_j = p^_j * (dp_j - sum_i p^_i dp_i),                                     */
/* the derivative of softmax with p^ in place of p; it is zero wherever p^ is.    */
/* counts may be NULL (k pairs per row); an index 0xFFFF marks an unused slot.    */
/* fp64 on the widened inputs, rounded once to dt.                                */
int slimfit_ref_softmax_backward_pruned(const void *vals, const uint16_t *idx, const int32_t *counts,
                                        const void *dp, int dt, int64_t rows, int cols, int k,
                                        void *ds, int threads)
{
    if (!dtype_ok(dt) || rows < 0 || cols < 1 || cols > 65536 || k < 1 || k > cols)
        return REF_BAD;
    if (rows > 0 && (!vals || !idx || !dp || !ds))
        return REF_BAD;
    (void)threads;
#pragma omp parallel for num_threads(threads > 1 ? threads : 1) schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int cnt = counts ? counts[r] : k;
        double dot = 0.0;
        for (int s = 0; s < cnt && s < k; ++s) {
            const int c = idx[r * (int64_t)k + s];
            if (c < cols)
                dot += (double)load_elem(vals, dt, r * (int64_t)k + s) * (double)load_elem(dp, dt, r * (int64_t)cols + c);
        }
        for (int c = 0; c < cols; ++c)
            store_elem(ds, dt, r * (int64_t)cols + c, 0.0f);
        for (int s = 0; s < cnt && s < k; ++s) {
            const int c = idx[r * (int64_t)k + s];
            if (c < cols) {
                const double v = (double)load_elem(vals, dt, r * (int64_t)k + s);
                store_elem(ds, dt, r * (int64_t)cols + c,
                           (float)(v * ((double)load_elem(dp, dt, r * (int64_t)cols + c) - dot)));
            }
        }
    }
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* Alg. 5 as the paper states it: the whole flattened tensor is one     */
/* input vector (the paper applies it to LayerNorm's standardised input */
/* and keeps int(numel * 0.1) entries).                                 */
/*   sort all n entries from largest to smallest with their indices,    */
/*   keep the first k.  by_magnitude != 0 orders by |x| (Sec. 5 speaks  */
/*   of discarding the small values of a signed tensor), otherwise by   */
/*   the signed value (Alg. 5's plain sort).  Ties: lower index first.  */
/*   The kept pairs are emitted in ascending index order; values are    */
/*   bit copies of the (signed) inputs.                                 */
/* ------------------------------------------------------------------ */

typedef struct {
    float key;
    int64_t pos;
} ref_gpair;

static int gpair_before(const void *pa, const void *pb)
{
    const ref_gpair *a = (const ref_gpair *)pa, *b = (const ref_gpair *)pb;
    if (a->key > b->key)
        return -1;
    if (a->key < b->key)
        return 1;
    return (a->pos > b->pos) - (a->pos < b->pos);
}

int slimfit_ref_prune_global(const void *x, int dt, int64_t n, int64_t k,
                             int by_magnitude, void *vals, int32_t *idx)
{
    if (!dtype_ok(dt) || n < 1 || n > 2147483647LL || k < 1 || k > n)
        return REF_BAD;
    if (!x || !vals || !idx)
        return REF_BAD;
    ref_gpair *buf = (ref_gpair *)malloc(sizeof(ref_gpair) * (size_t)n);
    uint8_t *kept = (uint8_t *)calloc((size_t)n, 1);
    if (!buf || !kept) {
        free(buf);
        free(kept);
        return REF_BAD;
    }
    for (int64_t j = 0; j < n; ++j) {
        float v = load_elem(x, dt, j);
        buf[j].key = by_magnitude ? fabsf(v) : v;
        buf[j].pos = j;
    }
    qsort(buf, (size_t)n, sizeof(ref_gpair), gpair_before);
    for (int64_t s = 0; s < k; ++s)
        kept[buf[s].pos] = 1;
    int64_t out = 0;
    for (int64_t j = 0; j < n; ++j) {
        if (!kept[j])
            continue;
        if (dt == 0)
            ((float *)vals)[out] = ((const float *)x)[j];
        else
            ((uint16_t *)vals)[out] = ((const uint16_t *)x)[j];
        idx[out] = (int32_t)j;
        ++out;
    }
    free(buf);
    free(kept);
    return out == k ? REF_OK : REF_BAD;
}

/* restoring process for the flattened form: zeros(n), then scatter */
int slimfit_ref_restore_global(const void *vals, const int32_t *idx, int64_t k,
                               int dt, int64_t n, void *out)
{
    if (!dtype_ok(dt) || n < 1 || k < 0 || k > n)
        return REF_BAD;
    if (!out || (k > 0 && (!vals || !idx)))
        return REF_BAD;
    const size_t esz = dt == 0 ? 4 : 2;
    memset(out, 0, (size_t)n * esz);
    for (int64_t s = 0; s < k; ++s) {
        if (idx[s] < 0 || idx[s] >= n)
            return REF_BAD;
        memcpy((char *)out + (size_t)idx[s] * esz, (const char *)vals + (size_t)s * esz, esz);
    }
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* LayerNorm as Sec. 4 writes it, per row of H elements:                */
/*   x~ = (x - E x) / sqrt(Var x + eps),   y = x~ * gamma + beta,       */
/* and, for a frozen LayerNorm, the input gradient                      */
/*   g = gamma * y^ / (H * sqrt(Var x + eps)),                          */
/*   x^ = H * g - sum_H g - x~ * sum_H (g * x~),                        */
/* where x~ is what the layer keeps for the backward pass: all of it,   */
/* or the pairs Alg. 5 kept of it (every other x~ counts as 0).         */
/* Var is the mean of squared deviations (divisor H).  All in fp64 on   */
/* the fp32 inputs, rounded once to fp32.                               */
/* ------------------------------------------------------------------ */

int slimfit_ref_layernorm_forward(const float *x, const float *gamma, const float *beta,
                                  int64_t rows, int H, float eps, float *y,
                                  float *mean, float *rstd, int threads)
{
    if (rows < 0 || H < 1 || !(eps >= 0.0f))
        return REF_BAD;
    if (rows > 0 && (!x || !gamma || !beta || !y || !mean || !rstd))
        return REF_BAD;
    (void)threads;
#pragma omp parallel for num_threads(threads > 1 ? threads : 1) schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *xr = x + r * (int64_t)H;
        double mu = 0.0, var = 0.0;
        for (int j = 0; j < H; ++j)
            mu += (double)xr[j];
        mu /= (double)H;
        for (int j = 0; j < H; ++j) {
            const double d = (double)xr[j] - mu;
            var += d * d;
        }
        var /= (double)H;
        const double rs = 1.0 / sqrt(var + (double)eps);
        for (int j = 0; j < H; ++j)
            y[r * (int64_t)H + j] = (float)(((double)xr[j] - mu) * rs * (double)gamma[j] + (double)beta[j]);
        mean[r] = (float)mu;
        rstd[r] = (float)rs;
    }
    return REF_OK;
}

/* The standardised tensor as the fused pruner forms it: two fp32 operations  */
/* per element on given fp32 statistics, x~_j = fl(fl(x_j - mean_r) * rstd_r), */
/* so that the k-th largest |x~| is decided on the same bits on both sides.    */
int slimfit_ref_standardize(const float *x, const float *mean, const float *rstd,
                            int64_t rows, int H, float *xs)
{
    if (rows < 0 || H < 1 || (rows > 0 && (!x || !mean || !rstd || !xs)))
        return REF_BAD;
    for (int64_t r = 0; r < rows; ++r) {
        for (int j = 0; j < H; ++j) {
            const float d = x[r * (int64_t)H + j] - mean[r];
            xs[r * (int64_t)H + j] = d * rstd[r];
        }
    }
    return REF_OK;
}

/* vals/idx: k kept entries of the flattened x~ (flat int32 indices, any order, distinct) */
int slimfit_ref_layernorm_backward_pruned(const float *vals, const int32_t *idx, int64_t k,
                                          const float *rstd, const float *gamma,
                                          const float *dy, int64_t rows, int H, float *dx)
{
    if (rows < 0 || H < 1 || k < 0 || k > rows * (int64_t)H)
        return REF_BAD;
    if (rows > 0 && (!rstd || !gamma || !dy || !dx || (k > 0 && (!vals || !idx))))
        return REF_BAD;
    const int64_t n = rows * (int64_t)H;
    double *xt = (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double));
    if (!xt)
        return REF_BAD;
    for (int64_t s = 0; s < k; ++s) {
        if (idx[s] < 0 || idx[s] >= n) {
            free(xt);
            return REF_BAD;
        }
        xt[idx[s]] = (double)vals[s];
    }
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t base = r * (int64_t)H;
        double sum_g = 0.0, sum_gx = 0.0;
        for (int j = 0; j < H; ++j) {
            const double g = (double)gamma[j] * (double)dy[base + j] * (double)rstd[r] / (double)H;
            sum_g += g;
            sum_gx += g * xt[base + j];
        }
        for (int j = 0; j < H; ++j) {
            const double g = (double)gamma[j] * (double)dy[base + j] * (double)rstd[r] / (double)H;
            dx[base + j] = (float)((double)H * g - sum_g - xt[base + j] * sum_gx);
        }
    }
    free(xt);
    return REF_OK;
}

/* Input gradient of an active LayerNorm: the same formula with every x~ present,  */
/* x~ = (x - mean_r) * rstd_r from the given fp32 statistics, evaluated in fp64.     */
int slimfit_ref_layernorm_backward(const float *x, const float *mean, const float *rstd,
                                   const float *gamma, const float *dy, int64_t rows, int H,
                                   float *dx)
{
    if (rows < 0 || H < 1 || (rows > 0 && (!x || !mean || !rstd || !gamma || !dy || !dx)))
        return REF_BAD;
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t base = r * (int64_t)H;
        double sum_g = 0.0, sum_gx = 0.0;
        for (int j = 0; j < H; ++j) {
            const double xt = ((double)x[base + j] - (double)mean[r]) * (double)rstd[r];
            const double g = (double)gamma[j] * (double)dy[base + j] * (double)rstd[r] / (double)H;
            sum_g += g;
            sum_gx += g * xt;
        }
        for (int j = 0; j < H; ++j) {
            const double xt = ((double)x[base + j] - (double)mean[r]) * (double)rstd[r];
            const double g = (double)gamma[j] * (double)dy[base + j] * (double)rstd[r] / (double)H;
            dx[base + j] = (float)((double)H * g - sum_g - xt * sum_gx);
        }
    }
    return REF_OK;
}

/* Parameter gradients of an active LayerNorm (Sec. 4):  gamma^ = sum over rows of  */
/* x~ * y^,  beta^ = sum over rows of y^,  with x~ = (x - mean_r) * rstd_r from the   */
/* given fp32 statistics, everything else in fp64, rounded once to fp32.               */
int slimfit_ref_layernorm_param_grads(const float *x, const float *mean, const float *rstd,
                                      const float *dy, int64_t rows, int H,
                                      float *dgamma, float *dbeta)
{
    if (rows < 0 || H < 1 || !dgamma || !dbeta || (rows > 0 && (!x || !mean || !rstd || !dy)))
        return REF_BAD;
    for (int j = 0; j < H; ++j) {
        double sg = 0.0, sb = 0.0;
        for (int64_t r = 0; r < rows; ++r) {
            const double xt = ((double)x[r * (int64_t)H + j] - (double)mean[r]) * (double)rstd[r];
            sg += xt * (double)dy[r * (int64_t)H + j];
            sb += (double)dy[r * (int64_t)H + j];
        }
        dgamma[j] = (float)sg;
        dbeta[j] = (float)sb;
    }
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* Alg. 1 -- inter-layer scheduling on the host                         */
/*   idx = argsort(d)[:int(L*F)]  -> those layers are frozen            */
/* Readings: equal distances freeze the lower layer index first; NaN    */
/* orders as +inf.  Only active layers take a new distance afterwards;  */
/* a frozen layer keeps its old one (Sec. 3.2, Fig. 4).                 */
/* ------------------------------------------------------------------ */

int slimfit_ref_freeze_count(int L, double F)
{
    if (L < 0 || !(F >= 0.0) || !(F <= 1.0))
        return REF_BAD;
    return (int)((double)L * F);                   /* Python's int(L*F) */
}

int slimfit_ref_keep_count(int cols, int keep_ppm)
{
    if (cols < 0 || keep_ppm < 0 || keep_ppm > 1000000)
        return REF_BAD;
    return (int)(((int64_t)cols * (int64_t)keep_ppm) / 1000000);
}

static int dist_before(float da, int ia, float db, int ib)
{
    /* NaN behaves like +inf */
    int na = da != da, nb = db != db;
    if (na || nb) {
        if (na && nb)
            return ia < ib;
        return nb;                                 /* non-NaN first */
    }
    if (da < db)
        return 1;
    if (da > db)
        return 0;
    return ia < ib;
}

int slimfit_ref_ils_select(const float *d, int L, int n_freeze,
                           int32_t *frozen_idx, uint8_t *mask)
{
    if (L < 0 || n_freeze < 0 || n_freeze > L)
        return REF_BAD;
    if (L > 0 && !d)
        return REF_BAD;
    if (n_freeze > 0 && !frozen_idx)
        return REF_BAD;
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L > 0 ? L : 1));
    if (!order)
        return REF_BAD;
    /* insertion sort: stable, and L is about a hundred */
    for (int i = 0; i < L; ++i) {
        int pos = i;
        while (pos > 0 && dist_before(d[i], i, d[order[pos - 1]], order[pos - 1])) {
            order[pos] = order[pos - 1];
            --pos;
        }
        order[pos] = i;
    }
    if (mask)
        memset(mask, 0, (size_t)L);
    for (int s = 0; s < n_freeze; ++s) {
        frozen_idx[s] = order[s];
        if (mask)
            mask[order[s]] = 1;
    }
    free(order);
    return REF_OK;
}

/* ILS at the granularity of blocks of consecutive layers (e.g. the tensors   */
/* of one encoder block): a block's distance is the mean of its layers'       */
/* distances (Eq. 1 values), summed in layer order in double; the n_freeze    */
/* blocks with the smallest means are frozen whole.  Same order as above:     */
/* equal means by lower block index, a block holding a NaN after all others.  */
/* With group = 1 this is slimfit_ref_ils_select.                             */
int slimfit_ref_ils_select_blocks(const float *d, int L, int group, int n_freeze,
                                  int32_t *frozen_blocks, uint8_t *mask)
{
    if (L < 0 || group < 1 || n_freeze < 0)
        return REF_BAD;
    const int nb = (L + group - 1) / group;
    if (n_freeze > nb || (L > 0 && !d) || (n_freeze > 0 && !frozen_blocks))
        return REF_BAD;
    double *mean = (double *)malloc(sizeof(double) * (size_t)(nb > 0 ? nb : 1));
    char *taken = (char *)calloc((size_t)(nb > 0 ? nb : 1), 1);
    if (!mean || !taken) {
        free(mean);
        free(taken);
        return REF_BAD;
    }
    for (int b = 0; b < nb; ++b) {
        const int lo = b * group, hi = lo + group < L ? lo + group : L;
        double sum = 0.0;
        for (int i = lo; i < hi; ++i)
            sum += (double)d[i];
        mean[b] = sum / (double)(hi - lo);
    }
    if (mask)
        memset(mask, 0, (size_t)L);
    /* selection by repeated minimum: obviously the n_freeze smallest, in order */
    for (int s = 0; s < n_freeze; ++s) {
        int best = -1;
        for (int b = 0; b < nb; ++b) {
            if (taken[b])
                continue;
            if (best < 0) {
                best = b;
                continue;
            }
            const int nan_b = mean[b] != mean[b], nan_best = mean[best] != mean[best];
            if (nan_b != nan_best) {
                if (nan_best)
                    best = b;
            } else if (!nan_b && mean[b] < mean[best]) {
                best = b;
            }
        }
        taken[best] = 1;
        frozen_blocks[s] = best;
        if (mask) {
            const int lo = best * group, hi = lo + group < L ? lo + group : L;
            for (int i = lo; i < hi; ++i)
                mask[i] = 1;
        }
    }
    free(mean);
    free(taken);
    return REF_OK;
}

int slimfit_ref_ils_update(float *d, const float *new_scores,
                           const uint8_t *frozen_mask, int L)
{
    if (L < 0)
        return REF_BAD;
    if (L == 0)
        return REF_OK;
    if (!d || !new_scores || !frozen_mask)
        return REF_BAD;
    for (int i = 0; i < L; ++i)
        if (!frozen_mask[i])
            d[i] = new_scores[i];
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* The two other freezing schedules the paper compares ILS with (the    */
/* ablation on freezing schedules): "random" picks the int(L*F) frozen  */
/* layers uniformly at random at every iteration, "progressive" keeps   */
/* the earliest layers frozen and updates the later ones throughout.    */
/* The random draw is a counter-based recipe both sides implement:      */
/*   stream  SplitMix64 with state s0 = seed XOR (iteration *            */
/*           0xD6E8FEB86659FD93), each output advancing the state by     */
/*           0x9E3779B97F4A7C15 and mixing it with the 30/27/31 shifts   */
/*           and the two multipliers of that generator;                  */
/*   choice  the first n_freeze steps of a Fisher-Yates shuffle of        */
/*           0..L-1: at step i, j = i + (next() mod (L - i)), swap;       */
/*   frozen_idx lists the picks in the order they were drawn.            */
/* ------------------------------------------------------------------ */

static uint64_t splitmix64_next(uint64_t *state)
{
    uint64_t z = (*state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* n raw outputs of the stream started at `state` (for the known-answer pin) */
int slimfit_ref_splitmix64(uint64_t state, int n, uint64_t *out)
{
    if (n < 0 || (n > 0 && !out))
        return REF_BAD;
    for (int i = 0; i < n; ++i)
        out[i] = splitmix64_next(&state);
    return REF_OK;
}

int slimfit_ref_schedule_random(int L, int n_freeze, uint64_t seed, uint64_t iteration,
                                int32_t *frozen_idx, uint8_t *mask)
{
    if (L < 0 || n_freeze < 0 || n_freeze > L || (n_freeze > 0 && !frozen_idx))
        return REF_BAD;
    int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L > 0 ? L : 1));
    if (!perm)
        return REF_BAD;
    for (int i = 0; i < L; ++i) {
        perm[i] = i;
        if (mask)
            mask[i] = 0;
    }
    uint64_t state = seed ^ (iteration * 0xD6E8FEB86659FD93ull);
    for (int i = 0; i < n_freeze; ++i) {
        const int j = i + (int)(splitmix64_next(&state) % (uint64_t)(L - i));
        const int32_t t = perm[i];
        perm[i] = perm[j];
        perm[j] = t;
        frozen_idx[i] = perm[i];
        if (mask)
            mask[perm[i]] = 1;
    }
    free(perm);
    return REF_OK;
}

int slimfit_ref_schedule_progressive(int L, int n_freeze, int32_t *frozen_idx, uint8_t *mask)
{
    if (L < 0 || n_freeze < 0 || n_freeze > L || (n_freeze > 0 && !frozen_idx))
        return REF_BAD;
    for (int i = 0; i < L; ++i)
        if (mask)
            mask[i] = i < n_freeze ? 1 : 0;
    for (int i = 0; i < n_freeze; ++i)
        frozen_idx[i] = i;
    return REF_OK;
}
