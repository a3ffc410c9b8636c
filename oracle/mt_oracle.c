/*
 * Reference evaluator ("oracle") for the multi-tenant inference path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It is never linked into, imported by or called
 * from the product library; it shares no header, helper or table with it.
 *
 * What it computes follows the paper's primer on DNNs (section 1.1): a DNN is
 * a stateless, deterministic function made of a fixed sequence of layers, and
 * evaluating it means applying each layer in turn to the previous layer's
 * output.  A fully-connected layer multiplies the previous output with a
 * stored tensor of learned values.  The output is a vector of class
 * probabilities.  Every request is evaluated on its own, with the layers of
 * the model its tenant uploaded (section 3: users upload a DNN, then send
 * inference requests; a worker hosts the DNNs of many tenants).
 *
 * The paper fixes no bias, activation, convolution, pooling, softmax or number
 * format; those come from the workload definitions and are read as follows:
 *   - FC:    z[n] = b[n] + sum_k W[n][k] * h[k]            (W stored [N][K])
 *   - CONV:  3x3 cross-correlation, zero padding 1, stride s, NHWC activations,
 *            filters stored [C_out][C_in][3][3], bias per output channel
 *   - GAP:   arithmetic mean over H x W for every channel
 *   - hidden layers: h = q(act(z)), act in {none, ReLU, exact-erf GELU};
 *     q = identity (fp32 models) or round-to-nearest-even to bfloat16
 *   - last layer: logits = z (no activation, never rounded),
 *     probs = exp(z - max z) / sum, label = lowest index of the maximum
 * All sums are fp64, taken in index order.
 *
 * Parity pins (tests/test_oracle_*.py): identity / zero / diagonal weights,
 * linearity, permutation invariance, hand-computed two-tenant nets, conv delta
 * and all-ones kernels, conv == FC on an explicit im2col, GAP closed forms,
 * GELU identities, bf16 rounding against every bit pattern and against a
 * library conversion, MAC counter == closed-form cost.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_FC = 0, ORC_CONV = 1, ORC_GAP = 2 };
enum { ORC_ACT_NONE = 0, ORC_ACT_RELU = 1, ORC_ACT_GELU = 2 };

typedef struct {
    int32_t kind, act;
    int32_t in_features, out_features; /* FC: K, N.  CONV: C_in, C_out.  GAP: C, C */
    int32_t in_h, in_w;                /* CONV / GAP input height and width */
    int32_t stride;                    /* CONV */
} orc_layer;

/* ---- bfloat16 rounding of a double (round to nearest, ties to even) ------- */
/* bfloat16: 1 sign, 8 exponent, 7 fraction bits.  Normal numbers keep 8
 * significant bits; below 2^-126 the spacing is fixed at 2^-133. */
double orc_round_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);          /* |x| = f * 2^e, f in [0.5, 1)  => leading bit at e-1 */
    int lead = e - 1;
    if (lead < -126) lead = -126;
    double quantum = ldexp(1.0, lead - 7);
    double r = nearbyint(x / quantum) * quantum;   /* default mode: ties to even */
    const double max_bf16 = 3.3895313892515355e38; /* (2 - 2^-7) * 2^127 */
    if (fabs(r) > max_bf16) return x > 0 ? INFINITY : -INFINITY;
    return r;
}

static double apply_act(double z, int act)
{
    switch (act) {
    case ORC_ACT_RELU: return z > 0.0 ? z : 0.0;
    case ORC_ACT_GELU: return 0.5 * z * (1.0 + erf(z / sqrt(2.0)));
    default: return z;
    }
}
double orc_act(double z, int act) { return apply_act(z, act); }

int orc_layer_out_len(const orc_layer* L)
{
    if (L->kind == ORC_FC) return L->out_features;
    if (L->kind == ORC_GAP) return L->in_features;
    int oh = (L->in_h + 2 - 3) / L->stride + 1;
    int ow = (L->in_w + 2 - 3) / L->stride + 1;
    return oh * ow * L->out_features;
}
int orc_layer_in_len(const orc_layer* L)
{
    if (L->kind == ORC_FC) return L->in_features;
    return L->in_h * L->in_w * L->in_features;
}

/* ---- single layers ------------------------------------------------------- */
static uint64_t fc_layer(const orc_layer* L, const double* W, const double* b,
                         const double* h, double* z)
{
    const int K = L->in_features, N = L->out_features;
    uint64_t macs = 0;
    for (int n = 0; n < N; ++n) {
        double s = b ? b[n] : 0.0;
        for (int k = 0; k < K; ++k) { s += W[(size_t)n * K + k] * h[k]; ++macs; }
        z[n] = s;
    }
    return macs;
}

static uint64_t conv_layer(const orc_layer* L, const double* W, const double* b,
                           const double* h, double* z)
{
    const int Ci = L->in_features, Co = L->out_features, H = L->in_h, Wd = L->in_w, s = L->stride;
    const int OH = (H + 2 - 3) / s + 1, OW = (Wd + 2 - 3) / s + 1;
    uint64_t macs = 0;
    for (int oh = 0; oh < OH; ++oh)
        for (int ow = 0; ow < OW; ++ow)
            for (int co = 0; co < Co; ++co) {
                double acc = b ? b[co] : 0.0;
                for (int kh = 0; kh < 3; ++kh)
                    for (int kw = 0; kw < 3; ++kw) {
                        int ih = oh * s + kh - 1, iw = ow * s + kw - 1;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue; /* zero padding */
                        for (int ci = 0; ci < Ci; ++ci) {
                            acc += W[(((size_t)co * Ci + ci) * 3 + kh) * 3 + kw] *
                                   h[((size_t)ih * Wd + iw) * Ci + ci];
                            ++macs;
                        }
                    }
                z[((size_t)oh * OW + ow) * Co + co] = acc;
            }
    return macs;
}

static void gap_layer(const orc_layer* L, const double* h, double* z)
{
    const int C = L->in_features, HW = L->in_h * L->in_w;
    for (int c = 0; c < C; ++c) {
        double s = 0.0;
        for (int p = 0; p < HW; ++p) s += h[(size_t)p * C + c];
        z[c] = s / (double)HW;
    }
}

/* Second, independent loop nest for the convolution: build the im2col matrix
 * of one image explicitly (rows = output pixels, columns ordered ci,kh,kw like
 * the stored filter) and apply the filter bank as a fully-connected layer. */
uint64_t orc_conv_via_im2col(const orc_layer* L, const double* W, const double* b,
                             const double* h, double* z)
{
    const int Ci = L->in_features, Co = L->out_features, H = L->in_h, Wd = L->in_w, s = L->stride;
    const int OH = (H + 2 - 3) / s + 1, OW = (Wd + 2 - 3) / s + 1, K = Ci * 9;
    double* col = (double*)calloc((size_t)K, sizeof(double));
    orc_layer fc = {ORC_FC, ORC_ACT_NONE, K, Co, 0, 0, 0};
    uint64_t macs = 0;
    for (int p = 0; p < OH * OW; ++p) {
        int oh = p / OW, ow = p % OW;
        for (int j = 0; j < K; ++j) {
            int ci = j / 9, kh = (j % 9) / 3, kw = j % 3;
            int ih = oh * s + kh - 1, iw = ow * s + kw - 1;
            col[j] = (ih < 0 || ih >= H || iw < 0 || iw >= Wd) ? 0.0
                     : h[((size_t)ih * Wd + iw) * Ci + ci];
        }
        macs += fc_layer(&fc, W, b, col, z + (size_t)p * Co);
    }
    free(col);
    return macs;
}

/* ---- head ---------------------------------------------------------------- */
void orc_head(const double* logits, int C, double* probs, int32_t* label)
{
    int best = 0;
    for (int c = 1; c < C; ++c) if (logits[c] > logits[best]) best = c; /* lowest index on ties */
    double mx = logits[best], sum = 0.0;
    for (int c = 0; c < C; ++c) { probs[c] = exp(logits[c] - mx); sum += probs[c]; }
    for (int c = 0; c < C; ++c) probs[c] /= sum;
    *label = best;
}

/* ---- one request through one model -------------------------------------- */
/* hidden_out (optional): concatenation of every hidden layer's h (after act and
 * q), in layer order, for prefix checks.  Returns the number of MACs done. */
uint64_t orc_forward_one(const orc_layer* layers, int n_layers,
                         const double* const* weights, const double* const* biases,
                         int round_bf16, const double* x,
                         double* logits, double* probs, int32_t* label, double* hidden_out)
{
    int max_len = orc_layer_in_len(&layers[0]);
    for (int l = 0; l < n_layers; ++l) {
        int o = orc_layer_out_len(&layers[l]);
        if (o > max_len) max_len = o;
    }
    double* cur = (double*)malloc(sizeof(double) * (size_t)max_len);
    double* nxt = (double*)malloc(sizeof(double) * (size_t)max_len);
    int len = orc_layer_in_len(&layers[0]);
    for (int i = 0; i < len; ++i) cur[i] = round_bf16 ? orc_round_bf16(x[i]) : x[i];
    uint64_t macs = 0;
    size_t hid_pos = 0;
    for (int l = 0; l < n_layers; ++l) {
        const orc_layer* L = &layers[l];
        int out_len = orc_layer_out_len(L);
        if (L->kind == ORC_FC) macs += fc_layer(L, weights[l], biases[l], cur, nxt);
        else if (L->kind == ORC_CONV) macs += conv_layer(L, weights[l], biases[l], cur, nxt);
        else gap_layer(L, cur, nxt);
        if (l == n_layers - 1) {
            for (int i = 0; i < out_len; ++i) logits[i] = nxt[i];
        } else {
            for (int i = 0; i < out_len; ++i) {
                double a = apply_act(nxt[i], L->act);
                nxt[i] = round_bf16 ? orc_round_bf16(a) : a;
            }
            if (hidden_out) { memcpy(hidden_out + hid_pos, nxt, sizeof(double) * (size_t)out_len); hid_pos += (size_t)out_len; }
        }
        double* t = cur; cur = nxt; nxt = t;
        len = out_len;
    }
    orc_head(logits, len, probs, label);
    free(cur); free(nxt);
    return macs;
}

/* ---- many requests of one model, split across threads by request --------- */
typedef struct {
    const orc_layer* layers; int n_layers;
    const double* const* weights; const double* const* biases;
    int round_bf16; const double* X; int in_len; int n_classes;
    int row_begin, row_end;
    double* logits; double* probs; int32_t* labels; uint64_t macs;
} job_t;

static void* job_main(void* p)
{
    job_t* j = (job_t*)p;
    j->macs = 0;
    for (int r = j->row_begin; r < j->row_end; ++r)
        j->macs += orc_forward_one(j->layers, j->n_layers, j->weights, j->biases, j->round_bf16,
                                   j->X + (size_t)r * j->in_len,
                                   j->logits + (size_t)r * j->n_classes,
                                   j->probs + (size_t)r * j->n_classes, j->labels + r, NULL);
    return NULL;
}

uint64_t orc_forward_rows(const orc_layer* layers, int n_layers,
                          const double* const* weights, const double* const* biases,
                          int round_bf16, const double* X, int n_rows, int n_threads,
                          double* logits, double* probs, int32_t* labels)
{
    if (n_rows <= 0) return 0;
    if (n_threads < 1) n_threads = 1;
    if (n_threads > n_rows) n_threads = n_rows;
    if (n_threads > 256) n_threads = 256;
    job_t jobs[256]; pthread_t th[256];
    int in_len = orc_layer_in_len(&layers[0]);
    int n_classes = orc_layer_out_len(&layers[n_layers - 1]);
    for (int t = 0; t < n_threads; ++t) {
        job_t j = {layers, n_layers, weights, biases, round_bf16, X, in_len, n_classes,
                   (int)((long long)n_rows * t / n_threads), (int)((long long)n_rows * (t + 1) / n_threads),
                   logits, probs, labels, 0};
        jobs[t] = j;
    }
    for (int t = 1; t < n_threads; ++t) pthread_create(&th[t], NULL, job_main, &jobs[t]);
    job_main(&jobs[0]);
    uint64_t macs = jobs[0].macs;
    for (int t = 1; t < n_threads; ++t) { pthread_join(th[t], NULL); macs += jobs[t].macs; }
    return macs;
}

/* expose the single layers for the pins */
uint64_t orc_fc(const orc_layer* L, const double* W, const double* b, const double* h, double* z) { return fc_layer(L, W, b, h, z); }
uint64_t orc_conv(const orc_layer* L, const double* W, const double* b, const double* h, double* z) { return conv_layer(L, W, b, h, z); }
void orc_gap(const orc_layer* L, const double* h, double* z) { gap_layer(L, h, z); }
