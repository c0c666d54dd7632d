/*
 * CPU oracle for the learned-cache lookup.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, single-threaded, fp64 statement of what one lookup computes, written
 * from the paper's description of a learned cache (Section 3, "Learned Cache
 * Design"): a prediction operation followed by a selection operation, with hits
 * leaving the batch and misses continuing to the next layer (Section 1: a request
 * that misses keeps running on the base model).  It shares no code, header,
 * table or constant with the HIP library and must never be linked into or called
 * from the product path; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg use it.
 *
 * Every function is the definition written out as loops with double
 * accumulators: no blocking, no vectorisation, no reordering.
 *
 * Pins (tests/test_oracle_*.py): hand-computed cases in exact rational
 * arithmetic, closed forms (K=2 softmax = logistic; zero weights), invariants
 * (sum/count, softmax sums to 1, shift invariance, hits and misses partition the
 * batch, order preserved), brute force over all hit masks, an independent
 * library affine map as a third opinion, and the paper's printed effective
 * hit-rate example (Section 4 toy example; Appendix A.1 "effective cache-hit
 * rate" equation).  The paper prints no worked numeric lookup, so full-lookup
 * values are pinned by those hand cases, not by paper numbers.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_NCS = 0, ORACLE_NSC = 1 };

typedef struct {
    int32_t C, S, H, K;
    int32_t act_dtype;       /* ORACLE_F32 / ORACLE_BF16: element type of the activation  */
    int32_t layout;          /* ORACLE_NCS: x[(r*C+c)*S+s];  ORACLE_NSC: x[(r*S+s)*C+c]   */
    int32_t round_operands;  /* 1: bf16 cache arithmetic: W1, W2, and the FC operands p, h
                                are rounded to bf16 (nearest even) before each product;
                                0: nothing is rounded ("ideal" arithmetic)                 */
    float   threshold;       /* tau: hit iff confidence > tau (strict)                    */
    int32_t selector;        /* 0: selector network (affine map over [pooled ; prob], logistic)
                                1: no selector network: confidence = largest class probability
                                   (the softmax-threshold baseline of the design analysis)
                                2: selector network with one hidden layer of sel_hidden units
                                   (Section 3, "Selector Network Design"): affine map over
                                   [features ; prob] -> ReLU -> affine map to one score -> logistic */
    int32_t predictor;       /* 0: global average pool -> FC -> ReLU -> FC
                                1: the paper's Pool(h): adaptive average pool of the in_h x in_w
                                   map to out_h x out_w -> ReLU -> one FC over the
                                   F = C*out_h*out_w features (H, W1, b1 unused)
                                2: the paper's FC(h): the whole activation row, flattened in
                                   storage order (D = C*S values), -> FC(D->H) -> ReLU -> FC(H->K);
                                   the selector reads [hidden ; prob]
                                3: the paper's Conv(k,s): convolution of the C x in_h x in_w map with
                                   H filters of conv_k x conv_k, stride conv_s, no padding -> ReLU ->
                                   one FC over the F = H*out_h*out_w hidden values, out = (in-k)/s+1
                                   (out_h, out_w are derived, not read); W1 is [H, C, k, k], b1 [H]  */
    int32_t in_h, in_w, out_h, out_w;   /* predictor 1 only; S = in_h*in_w, layout NCS        */
    int32_t sel_hidden;      /* selector 2 only: units in the selector's hidden layer      */
    int32_t conv_k, conv_s;  /* predictor 3 only                                           */
} oracle_desc_t;

static int conv_out_h(const oracle_desc_t *d) { return (d->in_h - d->conv_k) / d->conv_s + 1; }
static int conv_out_w(const oracle_desc_t *d) { return (d->in_w - d->conv_k) / d->conv_s + 1; }

/* Number of features the pooling step produces per row. */
static int n_features(const oracle_desc_t *d)
{
    if (d->predictor == 1) return d->C * d->out_h * d->out_w;
    if (d->predictor == 2) return d->H;
    if (d->predictor == 3) return d->H * conv_out_h(d) * conv_out_w(d);
    return d->C;
}

/* ---- number formats ------------------------------------------------------------ */

/* bf16 bit pattern -> real value (exact): bf16 is the top 16 bits of an IEEE fp32. */
static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Nearest bf16 value (8 significant bits, ties to even) of a double, as a double.
 * Works on the value itself, not on fp32 bit patterns. */
double oracle_round_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);                /* x = m * 2^e with 0.5 <= |m| < 1 */
    int q = e - 8;                     /* quantum exponent for 8 significant bits */
    if (q < -133) q = -133;            /* bf16 subnormal spacing */
    double r = ldexp(nearbyint(ldexp(x, -q)), q);   /* nearbyint: ties to even */
    if (fabs(r) > 3.3895313892515355e38) r = (x > 0) ? INFINITY : -INFINITY;
    return r;
}

static double act_at(const oracle_desc_t *d, const void *act, int64_t r, int c, int s)
{
    int64_t idx = (d->layout == ORACLE_NCS)
        ? ((r * d->C + c) * (int64_t)d->S + s)
        : ((r * d->S + s) * (int64_t)d->C + c);
    if (d->act_dtype == ORACLE_BF16) return bf16_bits_to_double(((const uint16_t *)act)[idx]);
    return (double)((const float *)act)[idx];
}

/* Element e of the flattened activation row r, in storage order (no layout arithmetic: the
 * FC(h) predictor sees the hidden layer output as one vector). */
static double act_flat(const oracle_desc_t *d, const void *act, int64_t r, int64_t e)
{
    int64_t idx = r * (int64_t)d->C * d->S + e;
    if (d->act_dtype == ORACLE_BF16) return bf16_bits_to_double(((const uint16_t *)act)[idx]);
    return (double)((const float *)act)[idx];
}

typedef struct {
    const float *W1;  /* [H,C] */
    const float *b1;  /* [H]   */
    const float *W2;  /* [K,H] */
    const float *b2;  /* [K]   */
    const float *ws;  /* [C+K], pooled features first, class probabilities after */
    float bs;
    /* selector 2 (hidden layer): */
    const float *Ws;  /* [sel_hidden, F+K] first layer, features first, probabilities after */
    const float *cs;  /* [sel_hidden] first-layer bias                                      */
    const float *vs;  /* [sel_hidden] second layer; its bias is bs                          */
} oracle_weights_t;

/* ---- the steps ------------------------------------------------------------------- */

/* Global average pool: p[c] = (sum over s of x[c,s]) / S, rounded once to fp32.
 * (Pooling predictor, Table "model architectures": Input -Pool-> Hidden; here the
 * pool extent is the whole spatial / token axis.) */
void oracle_pool_row(const oracle_desc_t *d, const void *act, int64_t r, float *p)
{
    for (int c = 0; c < d->C; ++c) {
        double sum = 0.0;
        for (int s = 0; s < d->S; ++s) sum += act_at(d, act, r, c, s);
        p[c] = (float)(sum / (double)d->S);
    }
}

/* Adaptive average pool of one row: window i of an axis of length In pooled to Out covers
 * [floor(i*In/Out), ceil((i+1)*In/Out)) (windows overlap when Out does not divide In; they
 * are the plain In/Out blocks when it does).  f[(c*out_h + oy)*out_w + ox] = relu(mean over
 * the window), the mean rounded once to fp32.  (Pooling predictor, table of predictor
 * architectures: Input -Pool-> Hidden Layer(h), ReLU activation; h is the size after pooling.) */
void oracle_pool_adaptive_row(const oracle_desc_t *d, const void *act, int64_t r, float *f)
{
    for (int c = 0; c < d->C; ++c)
        for (int oy = 0; oy < d->out_h; ++oy)
            for (int ox = 0; ox < d->out_w; ++ox) {
                int y0 = (oy * d->in_h) / d->out_h, y1 = ((oy + 1) * d->in_h + d->out_h - 1) / d->out_h;
                int x0 = (ox * d->in_w) / d->out_w, x1 = ((ox + 1) * d->in_w + d->out_w - 1) / d->out_w;
                double sum = 0.0;
                for (int y = y0; y < y1; ++y)
                    for (int x = x0; x < x1; ++x) sum += act_at(d, act, r, c, y * d->in_w + x);
                float m = (float)(sum / (double)((y1 - y0) * (x1 - x0)));
                f[(c * d->out_h + oy) * d->out_w + ox] = m > 0.f ? m : 0.f;
            }
}

/* Convolution predictor, hidden layer of one row (table of predictor architectures:
 * Input -Conv-> Hidden Layer, ReLU; Conv(k,s) = kernel size k, stride s):
 *   f[(o*oh + oy)*ow + ox] = relu(b1[o] + sum_{c,dy,dx} W1[o,c,dy,dx] * x[c, oy*s+dy, ox*s+dx]),
 * no padding, rounded once to fp32.  W1op holds the filter weights as operands (rounded to bf16
 * in the bf16 cache arithmetic); activation values are exact in either element type. */
void oracle_conv_row(const oracle_desc_t *d, const double *W1op, const float *b1, const void *act,
                     int64_t r, float *f)
{
    const int k = d->conv_k, s = d->conv_s, oh = conv_out_h(d), ow = conv_out_w(d);
    for (int o = 0; o < d->H; ++o)
        for (int oy = 0; oy < oh; ++oy)
            for (int ox = 0; ox < ow; ++ox) {
                double acc = 0.0;
                for (int c = 0; c < d->C; ++c)
                    for (int dy = 0; dy < k; ++dy)
                        for (int dx = 0; dx < k; ++dx)
                            acc += W1op[(((int64_t)o * d->C + c) * k + dy) * k + dx] *
                                   act_at(d, act, r, c, (oy * s + dy) * d->in_w + ox * s + dx);
                acc += (double)b1[o];
                f[((int64_t)o * oh + oy) * ow + ox] = (float)(acc > 0.0 ? acc : 0.0);
            }
}

/* Operand preparation for the bf16 cache arithmetic: a vector rounded element by
 * element to the nearest bf16 value (or copied unchanged when nothing is rounded).
 * Rounding a weight once here or once per product gives the same number. */
static void operand_f32(const oracle_desc_t *d, const float *src, int64_t n, double *dst)
{
    for (int64_t i = 0; i < n; ++i)
        dst[i] = d->round_operands ? oracle_round_bf16((double)src[i]) : (double)src[i];
}
static void operand_f64(const oracle_desc_t *d, const double *src, int64_t n, double *dst)
{
    for (int64_t i = 0; i < n; ++i)
        dst[i] = d->round_operands ? oracle_round_bf16(src[i]) : src[i];
}

/* Hidden layer of the predictor: h[j] = max(0, b1[j] + sum_c W1[j,c] p[c]).
 * (Table "model architectures": -FC-> Hidden Layer, ReLU activation.)
 * W1op / pop are the operands after preparation. */
static void fc1_relu(const oracle_desc_t *d, const double *W1op, const float *b1,
                     const double *pop, double *h)
{
    for (int j = 0; j < d->H; ++j) {
        double acc = 0.0;
        for (int c = 0; c < d->C; ++c) acc += W1op[(int64_t)j * d->C + c] * pop[c];
        acc += (double)b1[j];
        h[j] = acc > 0.0 ? acc : 0.0;
    }
}

/* Output layer of the predictor: z[k] = b2[k] + sum_j W2[k,j] h[j].
 * (Table "model architectures": Hidden Layer -FC-> Output.) */
static void fc2(const oracle_desc_t *d, const double *W2op, const float *b2,
                const double *hop, double *z)
{
    for (int k = 0; k < d->K; ++k) {
        double acc = 0.0;
        for (int j = 0; j < d->H; ++j) acc += W2op[(int64_t)k * d->H + j] * hop[j];
        z[k] = acc + (double)b2[k];
    }
}

/* Step-level entry points for the pin tests: one row through one FC layer. */
int oracle_fc1_relu(const oracle_desc_t *d, const oracle_weights_t *w, const float *p, double *h)
{
    int64_t nw = (int64_t)d->H * d->C;
    double *W1op = (double *)malloc(sizeof(double) * (size_t)nw);
    double *pop  = (double *)malloc(sizeof(double) * (size_t)d->C);
    if (!W1op || !pop) { free(W1op); free(pop); return -1; }
    operand_f32(d, w->W1, nw, W1op);
    operand_f32(d, p, d->C, pop);
    fc1_relu(d, W1op, w->b1, pop, h);
    free(W1op); free(pop);
    return 0;
}
int oracle_fc2(const oracle_desc_t *d, const oracle_weights_t *w, const double *h, double *z)
{
    int64_t nw = (int64_t)d->K * d->H;
    double *W2op = (double *)malloc(sizeof(double) * (size_t)nw);
    double *hop  = (double *)malloc(sizeof(double) * (size_t)d->H);
    if (!W2op || !hop) { free(W2op); free(hop); return -1; }
    operand_f32(d, w->W2, nw, W2op);
    operand_f64(d, h, d->H, hop);
    fc2(d, W2op, w->b2, hop, z);
    free(W2op); free(hop);
    return 0;
}

/* Class distribution and predicted class (Section 3, "Training Learned Caches":
 * the prediction is a distribution of class probabilities whose argmax is the
 * predicted class).  The class is decided on the fp32-rounded logits, the
 * precision the library reports them in; ties go to the lowest index. */
int32_t oracle_softmax_argmax(int K, const double *z, double *q)
{
    double m = z[0];
    for (int k = 1; k < K; ++k) if (z[k] > m) m = z[k];
    double denom = 0.0;
    for (int k = 0; k < K; ++k) denom += exp(z[k] - m);
    for (int k = 0; k < K; ++k) q[k] = exp(z[k] - m) / denom;
    int32_t best = 0;
    float bestv = (float)z[0];
    for (int k = 1; k < K; ++k) {
        float v = (float)z[k];
        if (v > bestv) { bestv = v; best = k; }
    }
    return best;
}

/* Selector: u = bs + sum_c ws[c] p[c] + sum_k ws[C+k] q[k]; confidence = logistic(u).
 * (Section 3, "Selector Network Design" and T = sigma_i(PR); the input here is the
 * pooled features followed by the class distribution.) */
double oracle_selector_score(const oracle_desc_t *d, const oracle_weights_t *w,
                             const float *p, const double *q)
{
    const int F = n_features(d);
    double u = (double)w->bs;
    for (int c = 0; c < F; ++c) u += (double)w->ws[c] * (double)p[c];
    for (int k = 0; k < d->K; ++k) u += (double)w->ws[F + k] * q[k];
    return u;
}

/* Selector with one hidden layer (Section 3, "Selector Network Design": a network with one
 * hidden layer that projects the predictor's output onto a binary decision; ReLU as in every
 * hidden layer of the cache's networks):
 *   g[j] = relu(cs[j] + sum_c Ws[j,c] p[c] + sum_k Ws[j,F+k] q[k]),  u = bs + sum_j vs[j] g[j].
 * In the bf16 cache arithmetic the first layer is a matrix product like the predictor's, so
 * its weights and operands (p, q) are rounded to bf16 and so is the hidden vector g that it
 * hands on; the one-output second layer is plain fp32 arithmetic on unrounded vs. */
double oracle_selector_hidden_score(const oracle_desc_t *d, const oracle_weights_t *w,
                                    const float *p, const double *q)
{
    const int F = n_features(d), In = F + d->K;
    double u = (double)w->bs;
    for (int j = 0; j < d->sel_hidden; ++j) {
        double acc = 0.0;
        for (int c = 0; c < F; ++c) {
            double wv = (double)w->Ws[(int64_t)j * In + c], x = (double)p[c];
            if (d->round_operands) { wv = oracle_round_bf16(wv); x = oracle_round_bf16(x); }
            acc += wv * x;
        }
        for (int k = 0; k < d->K; ++k) {
            double wv = (double)w->Ws[(int64_t)j * In + F + k], x = q[k];
            if (d->round_operands) { wv = oracle_round_bf16(wv); x = oracle_round_bf16(x); }
            acc += wv * x;
        }
        acc += (double)w->cs[j];
        double g = acc > 0.0 ? acc : 0.0;
        if (d->round_operands) g = oracle_round_bf16(g);
        u += (double)w->vs[j] * g;
    }
    return u;
}

static double logistic(double u) { return 1.0 / (1.0 + exp(-u)); }

/* One lookup per active row i (source row r = row_index ? row_index[i] : i).
 * Any output pointer may be NULL.  Returns 0, or -1 on allocation failure. */
int oracle_lookup(const oracle_desc_t *d, const oracle_weights_t *w, const void *act,
                  const int32_t *row_index, int32_t n,
                  float *pooled /*[n,F]*/, float *logits /*[n,K]*/, double *probs /*[n,K]*/,
                  int32_t *pred_class /*[n]*/, double *score /*[n]*/, float *confidence /*[n]*/,
                  uint8_t *hit /*[n]*/)
{
    const int F = n_features(d);
    const int pool_fc = d->predictor == 1, flat_fc = d->predictor == 2, conv_fc = d->predictor == 3;
    const int H = (pool_fc || conv_fc) ? F : d->H;   /* width of the layer that feeds the output FC */
    const int64_t D = (int64_t)d->C * d->S;    /* inputs of the first FC of the FC(h) predictor */
    int64_t n1 = pool_fc ? 1 : (flat_fc ? (int64_t)d->H * D : (int64_t)d->H * d->C), n2 = (int64_t)d->K * H;
    if (conv_fc) n1 = (int64_t)d->H * d->C * d->conv_k * d->conv_k;
    float  *p    = (float *)malloc(sizeof(float) * (size_t)F);
    double *pop  = (double *)malloc(sizeof(double) * (size_t)F);
    double *h    = (double *)malloc(sizeof(double) * (size_t)H);
    double *hop  = (double *)malloc(sizeof(double) * (size_t)H);
    double *z    = (double *)malloc(sizeof(double) * (size_t)d->K);
    double *q    = (double *)malloc(sizeof(double) * (size_t)d->K);
    double *W1op = (double *)malloc(sizeof(double) * (size_t)n1);
    double *W2op = (double *)malloc(sizeof(double) * (size_t)n2);
    int rc = -1;
    if (!p || !pop || !h || !hop || !z || !q || !W1op || !W2op) goto done;
    if (!pool_fc) operand_f32(d, w->W1, n1, W1op);
    operand_f32(d, w->W2, n2, W2op);
    oracle_desc_t dh = *d;                     /* the output FC reads H inputs */
    dh.H = H;
    for (int32_t i = 0; i < n; ++i) {
        int64_t r = row_index ? (int64_t)row_index[i] : (int64_t)i;
        if (pool_fc) {
            oracle_pool_adaptive_row(d, act, r, p);          /* hidden layer = relu(pooled) */
            for (int c = 0; c < F; ++c) h[c] = (double)p[c];
        } else if (conv_fc) {
            oracle_conv_row(d, W1op, w->b1, act, r, p);      /* hidden layer = relu(conv) */
            for (int c = 0; c < F; ++c) h[c] = (double)p[c];
        } else if (flat_fc) {
            /* hidden[j] = relu(b1[j] + sum_e W1[j,e] x[e]) over the whole flattened row; the
             * activation values are exact in either element type, W1 is an operand (rounded
             * in the bf16 arithmetic).  The hidden layer is kept as fp32 features. */
            for (int j = 0; j < d->H; ++j) {
                double acc = 0.0;
                for (int64_t e = 0; e < D; ++e) acc += W1op[(int64_t)j * D + e] * act_flat(d, act, r, e);
                acc += (double)w->b1[j];
                p[j] = (float)(acc > 0.0 ? acc : 0.0);
                h[j] = (double)p[j];
            }
        } else {
            oracle_pool_row(d, act, r, p);
            operand_f32(d, p, d->C, pop);
            fc1_relu(d, W1op, w->b1, pop, h);
        }
        operand_f64(d, h, H, hop);
        fc2(&dh, W2op, w->b2, hop, z);
        int32_t cls = oracle_softmax_argmax(d->K, z, q);
        double u, c;
        if (d->selector == 1) {
            /* Appendix, "Decoupling prediction and selection": only the predictor, with a
             * threshold over its softmax scores.  score = confidence = max_k q[k]. */
            c = q[0];
            for (int k = 1; k < d->K; ++k) if (q[k] > c) c = q[k];
            u = c;
        } else if (d->selector == 2) {
            u = oracle_selector_hidden_score(d, w, p, q);
            c = logistic(u);
        } else {
            u = oracle_selector_score(d, w, p, q);
            c = logistic(u);
        }
        float conf = (float)c;
        if (pooled) memcpy(pooled + (int64_t)i * F, p, sizeof(float) * (size_t)F);
        if (logits) for (int k = 0; k < d->K; ++k) logits[(int64_t)i * d->K + k] = (float)z[k];
        if (probs)  memcpy(probs + (int64_t)i * d->K, q, sizeof(double) * (size_t)d->K);
        if (pred_class) pred_class[i] = cls;
        if (score) score[i] = u;
        if (confidence) confidence[i] = conf;
        if (hit) hit[i] = (conf > d->threshold) ? 1 : 0;   /* decided in fp32, strictly above */
    }
    rc = 0;
done:
    free(p); free(pop); free(h); free(hop); free(z); free(q); free(W1op); free(W2op);
    return rc;
}

/* Misses continue: the ids whose hit flag is 0, in their incoming order.
 * ids_in == NULL means the identity list 0..n-1.  Returns the miss count. */
int32_t oracle_compact_misses(const uint8_t *hit, const int32_t *ids_in, int32_t n, int32_t *ids_out)
{
    int32_t m = 0;
    for (int32_t i = 0; i < n; ++i)
        if (!hit[i]) ids_out[m++] = ids_in ? ids_in[i] : i;
    return m;
}
