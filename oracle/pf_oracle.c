/*
 * pf_oracle.c -- plain CPU oracle for the neuron-aware sparse FFN of a decode step.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may include, link or call
 * this file; only the tests, the smoke check and the benchmark's cpu_baseline leg do.
 * It shares no code, header or table with the HIP library.  (The integer-mix constants of
 * the benchmark glue's sign pattern are, necessarily, written out on both sides: they define
 * the pattern.)
 *
 * What it states (PowerInfer, arXiv 2312.12456):
 *   - A neuron is one row of FC1 (and of the gate matrix for gated FFNs) together with
 *     the matching column of FC2; a neuron is "activated" when its ReLU output is non
 *     zero and therefore contributes to the block output (Sec. 2.1, Fig. "bg-mlp";
 *     footnote in Sec. 1).
 *   - A per-layer MLP predictor with one hidden layer marks the neurons expected to
 *     fire (Sec. 5.1); the neuron-aware operator then processes, for every neuron that
 *     is marked, its FC1 row and its FC2 column and skips all others (Sec. 5.4).
 *   - Weights are FP16 or INT4, intermediate activations FP32 (Sec. 8.1).  Here every
 *     stored weight is widened exactly and all sums are carried in fp64, so that the
 *     oracle's own rounding is negligible next to an fp32-accumulating device kernel.
 *
 * Readings taken where the paper is silent (each is listed in the design notes):
 *   predictor = d -> r, ReLU, r -> ffn, optional per-neuron logit bias, logistic
 *   squashing, strict "score > threshold"; gated FFN = ReLU(gate row . x + bias) *
 *   (up row . x); INT4 = unsigned nibble u, value = scale * (u - 8), one fp16 scale per
 *   128 consecutive elements of a neuron's row, element 2j in the low nibble of byte j;
 *   FC2 is held transposed, one neuron per row, like FC1.
 *
 * Every function loops over neurons in ascending index order and adds in that order,
 * so dense, masked and index-list forms agree bit for bit whenever they cover the
 * same non-zero terms.  OpenMP only splits independent outputs across threads; the
 * order of every individual sum is fixed, so results do not depend on thread count.
 *
 * Parity pins (tests/test_oracle_*.py): all-ones mask == dense; exact ReLU-positive
 * mask == dense; brute force over all masks of tiny integer-valued layers; fp64 matmul
 * of a linear-algebra library on the widened arrays; int4 round trip over all nibbles;
 * linearity over disjoint masks; removal of one true positive changes y by exactly
 * that neuron's term.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t d;         /* model width                                              */
    int32_t ffn;       /* number of neurons F                                      */
    int32_t r;         /* predictor hidden width                                   */
    int32_t act;       /* 0: ReLU FFN with FC1 bias; 1: ReLU-gated (gate, up, down);
                          2: dReLU (ReLU on the gate and on the up branch)         */
    int32_t wtype;     /* 0: fp16 bit patterns; 1: int4, group 128, fp16 scales    */
    int32_t pad_;
    double threshold;  /* predictor score threshold tau                            */
    const void *w_up;    /* [ffn][d] fp16 bits, or [ffn][d/2] packed nibbles       */
    const void *w_gate;  /* same shape, gated FFN only                             */
    const void *w_down;  /* FC2 transposed: [ffn][d], one neuron's column per row  */
    const uint16_t *s_up, *s_gate, *s_down; /* [ffn][d/128] fp16 bits, int4 only   */
    const float *b_up;   /* [ffn] FC1 bias (gate bias when gated) or NULL          */
    const float *b_down; /* [d] or NULL                                            */
    const uint16_t *p1;  /* [r][d]   fp16 bits                                     */
    const uint16_t *p2;  /* [ffn][r] fp16 bits                                     */
    const float *p_bias; /* [ffn] added to the logit, or NULL                      */
} pfo_layer;

/* IEEE 754 binary16 bit pattern -> double, exact (subnormals, inf and nan included). */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

double pfo_half_to_double(uint16_t h) { return half_bits_to_double(h); }

int pfo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Widen columns [c0, c1) of neuron i of one stored matrix into out[0 .. c1-c0). */
static void widen_row(const pfo_layer *L, const void *w, const uint16_t *s, int i, int c0,
                      int c1, double *out)
{
    int d = L->d;
    if (L->wtype == 0) {
        const uint16_t *row = (const uint16_t *)w + (size_t)i * d;
        for (int c = c0; c < c1; ++c) out[c - c0] = half_bits_to_double(row[c]);
    } else {
        const uint8_t *row = (const uint8_t *)w + (size_t)i * (d / 2);
        const uint16_t *srow = s + (size_t)i * (d / 128);
        for (int c = c0; c < c1; ++c) {
            uint8_t byte = row[c >> 1];
            int u = (c & 1) ? (byte >> 4) : (byte & 15);
            out[c - c0] = half_bits_to_double(srow[c / 128]) * (double)(u - 8);
        }
    }
}

/* Dequantised value of one stored element (exposed for the int4 round-trip pin). */
double pfo_weight_value(const pfo_layer *L, int which, int i, int c)
{
    const void *w = which == 0 ? L->w_up : which == 1 ? L->w_gate : L->w_down;
    const uint16_t *s = which == 0 ? L->s_up : which == 1 ? L->s_gate : L->s_down;
    double v;
    widen_row(L, w, s, i, c, c + 1, &v);
    return v;
}

static double dot_row(const double *wrow, const float *x, int d)
{
    double acc = 0.0;
    for (int c = 0; c < d; ++c) acc += wrow[c] * (double)x[c];
    return acc;
}

/*
 * FC1 stage of one neuron for one token (Sec. 2.1): pre-activation, and the value the
 * neuron hands to FC2.  *pre is the quantity whose sign decides "activated":
 *   ReLU FFN : pre = w_up[i].x + b_up[i],            h = max(pre, 0)
 *   gated    : pre = w_gate[i].x + b_up[i] (gate),   h = max(pre, 0) * (w_up[i].x)
 *   dReLU    : g = w_gate[i].x + b_up[i], u = w_up[i].x,  h = max(g, 0) * max(u, 0),
 *              pre = min(g, u): the neuron contributes only when both branches are open
 *              (the activation of the Bamboo-7B row of Table "model_eval", Sec. 8.1; the
 *              paper names it without a formula, this is the reading taken)
 */
static double neuron_fc1(const pfo_layer *L, int i, const float *x, double *rowbuf, double *pre)
{
    int d = L->d;
    double bias = L->b_up ? (double)L->b_up[i] : 0.0;
    if (L->act == 0) {
        widen_row(L, L->w_up, L->s_up, i, 0, d, rowbuf);
        double z = dot_row(rowbuf, x, d) + bias;
        *pre = z;
        return z > 0.0 ? z : 0.0;
    }
    widen_row(L, L->w_gate, L->s_gate, i, 0, d, rowbuf);
    double g = dot_row(rowbuf, x, d) + bias;
    widen_row(L, L->w_up, L->s_up, i, 0, d, rowbuf);
    double u = dot_row(rowbuf, x, d);
    if (L->act == 2) {
        *pre = g < u ? g : u;
        return (g > 0.0 ? g : 0.0) * (u > 0.0 ? u : 0.0);
    }
    *pre = g;
    return (g > 0.0 ? g : 0.0) * u;
}

/* pre[b][i] for every neuron: the pre-activation that ReLU is applied to. */
void pfo_preact(const pfo_layer *L, const float *x, int B, double *pre)
{
    int d = L->d, F = L->ffn;
#pragma omp parallel
    {
        double *rowbuf = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(static)
        for (int i = 0; i < F; ++i)
            for (int b = 0; b < B; ++b) {
                double p;
                (void)neuron_fc1(L, i, x + (size_t)b * d, rowbuf, &p);
                pre[(size_t)b * F + i] = p;
            }
        free(rowbuf);
    }
}

/*
 * FC2 stage (Fig. "bg-mlp", right): y[b][c] = b_down[c] + sum over the listed neurons,
 * ascending, of h[b][i] * W_down[c][i]; W_down is stored transposed so that term reads
 * row i.  `take[i] != 0` selects the neurons summed.  Threads own disjoint column
 * blocks; each column's sum runs over i in ascending order.
 */
static void fc2_accumulate(const pfo_layer *L, const double *h /*[B][F]*/, const uint8_t *take,
                           int B, double *y)
{
    int d = L->d, F = L->ffn;
    enum { CB = 128 };
#pragma omp parallel
    {
        double colbuf[CB];
#pragma omp for schedule(static)
        for (int c0 = 0; c0 < d; c0 += CB) {
            int c1 = c0 + CB < d ? c0 + CB : d;
            for (int b = 0; b < B; ++b)
                for (int c = c0; c < c1; ++c)
                    y[(size_t)b * d + c] = L->b_down ? (double)L->b_down[c] : 0.0;
            for (int i = 0; i < F; ++i) {
                if (!take[i]) continue;
                widen_row(L, L->w_down, L->s_down, i, c0, c1, colbuf);
                for (int b = 0; b < B; ++b) {
                    double hv = h[(size_t)b * F + i];
                    double *yb = y + (size_t)b * d;
                    for (int c = c0; c < c1; ++c) yb[c] += hv * colbuf[c - c0];
                }
            }
        }
    }
}

/* Dense FFN block: every neuron is computed (Sec. 2.1). */
void pfo_dense_ffn(const pfo_layer *L, const float *x, int B, double *y)
{
    int d = L->d, F = L->ffn;
    double *h = (double *)malloc(sizeof(double) * (size_t)B * F);
    uint8_t *all = (uint8_t *)malloc((size_t)F);
    memset(all, 1, (size_t)F);
#pragma omp parallel
    {
        double *rowbuf = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(static)
        for (int i = 0; i < F; ++i)
            for (int b = 0; b < B; ++b) {
                double p;
                h[(size_t)b * F + i] = neuron_fc1(L, i, x + (size_t)b * d, rowbuf, &p);
            }
        free(rowbuf);
    }
    fc2_accumulate(L, h, all, B, y);
    free(all);
    free(h);
}

/*
 * Neuron-aware FFN for a given activation mask (Sec. 5.4): a neuron with mask[i] != 0
 * is processed -- its FC1 row (and gate row), the activation function, and its FC2
 * column -- for every token of the batch; a neuron with mask[i] == 0 is skipped
 * entirely.  With a batch the mask is the union over the tokens (Sec. 8.2, batching).
 */
void pfo_masked_ffn(const pfo_layer *L, const float *x, int B, const uint8_t *mask, double *y)
{
    int d = L->d, F = L->ffn;
    double *h = (double *)calloc((size_t)B * F, sizeof(double));
#pragma omp parallel
    {
        double *rowbuf = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 16)
        for (int i = 0; i < F; ++i) {
            if (!mask[i]) continue;
            for (int b = 0; b < B; ++b) {
                double p;
                h[(size_t)b * F + i] = neuron_fc1(L, i, x + (size_t)b * d, rowbuf, &p);
            }
        }
        free(rowbuf);
    }
    fc2_accumulate(L, h, mask, B, y);
    free(h);
}

/* Ascending list of the set entries of mask[0..F); returns its length. */
int pfo_compact(const uint8_t *mask, int F, int32_t *idx)
{
    int n = 0;
    for (int i = 0; i < F; ++i)
        if (mask[i]) idx[n++] = i;
    return n;
}

/*
 * The same operator driven by an index list instead of a mask: idx[0..count) names
 * the neurons to process, in the order given.  hbuf (optional, [B][count]) receives
 * the FC1 outputs h[b][j] of the listed neurons.
 */
void pfo_sparse_ffn_idx(const pfo_layer *L, const float *x, int B, const int32_t *idx, int count,
                        double *y, double *hbuf)
{
    int d = L->d;
    double *h = (double *)malloc(sizeof(double) * (size_t)B * (size_t)(count > 0 ? count : 1));
#pragma omp parallel
    {
        double *rowbuf = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(static)
        for (int j = 0; j < count; ++j)
            for (int b = 0; b < B; ++b) {
                double p;
                h[(size_t)b * count + j] = neuron_fc1(L, idx[j], x + (size_t)b * d, rowbuf, &p);
            }
        free(rowbuf);
    }
    enum { CB = 128 };
#pragma omp parallel
    {
        double colbuf[CB];
#pragma omp for schedule(static)
        for (int c0 = 0; c0 < d; c0 += CB) {
            int c1 = c0 + CB < d ? c0 + CB : d;
            for (int b = 0; b < B; ++b)
                for (int c = c0; c < c1; ++c)
                    y[(size_t)b * d + c] = L->b_down ? (double)L->b_down[c] : 0.0;
            for (int j = 0; j < count; ++j) {
                widen_row(L, L->w_down, L->s_down, idx[j], c0, c1, colbuf);
                for (int b = 0; b < B; ++b) {
                    double hv = h[(size_t)b * count + j];
                    double *yb = y + (size_t)b * d;
                    for (int c = c0; c < c1; ++c) yb[c] += hv * colbuf[c - c0];
                }
            }
        }
    }
    if (hbuf) memcpy(hbuf, h, sizeof(double) * (size_t)B * (size_t)count);
    free(h);
}

/*
 * Activation predictor (Sec. 5.1: input layer, one hidden layer, output layer):
 *   t[b][m]     = max(p1[m] . x[b], 0)
 *   logit[b][i] = p2[i] . t[b] + p_bias[i]
 *   score[b][i] = 1 / (1 + exp(-logit[b][i]))
 *   active[i]   = any over b of (score[b][i] > threshold)
 * Outputs are optional (NULL skips them): hidden [B][r], logits [B][F], scores [B][F],
 * active [F] (union), active_rows [B][F].
 */
void pfo_predict(const pfo_layer *L, const float *x, int B, double *hidden, double *logits,
                 double *scores, uint8_t *active, uint8_t *active_rows)
{
    int d = L->d, F = L->ffn, r = L->r;
    double *t = (double *)malloc(sizeof(double) * (size_t)B * r);
#pragma omp parallel for schedule(static)
    for (int m = 0; m < r; ++m) {
        const uint16_t *row = L->p1 + (size_t)m * d;
        for (int b = 0; b < B; ++b) {
            const float *xb = x + (size_t)b * d;
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += half_bits_to_double(row[c]) * (double)xb[c];
            t[(size_t)b * r + m] = acc > 0.0 ? acc : 0.0;
        }
    }
#pragma omp parallel for schedule(static)
    for (int i = 0; i < F; ++i) {
        const uint16_t *row = L->p2 + (size_t)i * r;
        int any = 0;
        for (int b = 0; b < B; ++b) {
            const double *tb = t + (size_t)b * r;
            double acc = 0.0;
            for (int m = 0; m < r; ++m) acc += half_bits_to_double(row[m]) * tb[m];
            if (L->p_bias) acc += (double)L->p_bias[i];
            double sc = 1.0 / (1.0 + exp(-acc));
            int on = sc > L->threshold;
            any |= on;
            if (logits) logits[(size_t)b * F + i] = acc;
            if (scores) scores[(size_t)b * F + i] = sc;
            if (active_rows) active_rows[(size_t)b * F + i] = (uint8_t)on;
        }
        if (active) active[i] = (uint8_t)any;
    }
    if (hidden) memcpy(hidden, t, sizeof(double) * (size_t)B * r);
    free(t);
}

/* Mask of the neurons that really fire for at least one token: pre-activation > 0. */
void pfo_exact_mask(const pfo_layer *L, const float *x, int B, uint8_t *mask)
{
    int F = L->ffn;
    double *pre = (double *)malloc(sizeof(double) * (size_t)B * F);
    pfo_preact(L, x, B, pre);
    for (int i = 0; i < F; ++i) {
        int any = 0;
        for (int b = 0; b < B; ++b) any |= pre[(size_t)b * F + i] > 0.0;
        mask[i] = (uint8_t)any;
    }
    free(pre);
}

/*
 * One layer of the decode step as the engine runs it (Sec. 4.2, single-layer example,
 * without the CPU half): predict, then run the neuron-aware FFN on the predicted set.
 * mask_out (optional, [F]) receives the predicted union mask.
 */
void pfo_layer_step(const pfo_layer *L, const float *x, int B, double *y, uint8_t *mask_out)
{
    int F = L->ffn;
    uint8_t *mask = (uint8_t *)malloc((size_t)F);
    pfo_predict(L, x, B, NULL, NULL, NULL, mask, NULL);
    pfo_masked_ffn(L, x, B, mask, y);
    if (mask_out) memcpy(mask_out, mask, (size_t)F);
    free(mask);
}

/*
 * Sign that the glue gives column c of batch row b: +1 for row 0, otherwise the top bit of
 * a fixed integer mix of (b, c) -- a counter-based pattern, the same for every call.
 */
static double pfo_glue_sign(uint32_t b, uint32_t c)
{
    if (b == 0) return 1.0;
    uint32_t h = b * 0x9E3779B1u + c * 0x85EBCA77u + 0x165667B1u;
    h ^= h >> 15;
    h *= 0x2C1B3C6Du;
    h ^= h >> 12;
    h *= 0x297A2D39u;
    h ^= h >> 15;
    return (h >> 31) ? -1.0 : 1.0;
}

/*
 * Glue between the layers of the synthetic FFN stack (a benchmark construction, not in
 * the paper): residual add followed by a scale-only RMS normalisation,
 *   v = x + y,  x_next = sign(b, c) * v * sqrt(d) / ||v||_2     (per token; v == 0 stays 0).
 * The fixed sign pattern of the rows b >= 1 keeps the tokens of a batch from aligning: the
 * always-active neurons add nearly the same vector to every row, and without it the rows of
 * a batch would list the same neurons after a few layers (the union over the batch, whose
 * growth is what a batched step is about, would collapse to one token's set).
 * The result is rounded to fp32 because activations travel between layers in fp32.
 */
void pfo_stack_glue(const float *x, const double *y, int d, int B, float *x_next)
{
    for (int b = 0; b < B; ++b) {
        double ss = 0.0;
        for (int c = 0; c < d; ++c) {
            double v = (double)x[(size_t)b * d + c] + y[(size_t)b * d + c];
            ss += v * v;
        }
        double scale = ss > 0.0 ? sqrt((double)d / ss) : 0.0;
        for (int c = 0; c < d; ++c) {
            double v = (double)x[(size_t)b * d + c] + y[(size_t)b * d + c];
            x_next[(size_t)b * d + c] = (float)(pfo_glue_sign((uint32_t)b, (uint32_t)c) * v * scale);
        }
    }
}
