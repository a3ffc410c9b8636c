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
 *   - CONV:  k x k cross-correlation (k = 1, 3 or 7), zero padding p, stride s, NHWC
 *            activations, filters stored [C_out][C_in][k][k], bias per output channel;
 *            output size floor((H + 2p - k) / s) + 1
 *   - GAP:   arithmetic mean over H x W for every channel
 *   - MAXPOOL: maximum over a k x k window, stride s, padding p; taps outside the image
 *            never win (a window always holds at least one pixel when p < k)
 *   - ADD:   elementwise sum of two earlier outputs of the same shape (a residual
 *            connection), then the activation
 *   - a layer reads the output of the layer before it unless `src` names an earlier
 *     one (src = j + 1 reads the output of layer j; 0 = the previous layer, or the
 *     request for layer 0); ADD takes its second operand from `src2` the same way
 *   - folded batch normalisation (orc_fold_bn): a convolution followed by
 *     y = gamma * (x - mean) / sqrt(var + eps) + beta per channel is one convolution
 *     with W' = q_w(W * s), b' = fl32((b - mean) * s + beta), s = gamma / sqrt(var + eps),
 *     everything in fp64 and rounded once (q_w: to bfloat16 for bf16 models, to fp32
 *     otherwise); the folded filters are the model's stored values from then on
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
 * library conversion, MAC counter == closed-form cost; 1x1 convolution == the
 * per-pixel matrix product, 7x7 against a library correlation, delta and all-ones
 * kernels at every size, max-pool against hand numbers and a library maximum
 * filter, residual models against their composition from single layers, the
 * folded normalisation against the unfolded formula.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_FC = 0, ORC_CONV = 1, ORC_GAP = 2, ORC_MAXPOOL = 3, ORC_ADD = 4 };
enum { ORC_ACT_NONE = 0, ORC_ACT_RELU = 1, ORC_ACT_GELU = 2 };

typedef struct {
    int32_t kind, act;
    int32_t in_features, out_features; /* FC: K, N.  CONV: C_in, C_out.  GAP / MAXPOOL / ADD: C, C */
    int32_t in_h, in_w;                /* input height and width of the image layers */
    int32_t stride;                    /* CONV, MAXPOOL */
    int32_t ksize, pad;                /* CONV, MAXPOOL: window k x k, padding */
    int32_t src, src2;                 /* j + 1: read the output of layer j; 0: the previous layer */
} orc_layer;

static int out_size(int in, int k, int pad, int stride) { return (in + 2 * pad - k) / stride + 1; }

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
    if (L->kind == ORC_ADD) return L->in_h * L->in_w * L->in_features;
    int oh = out_size(L->in_h, L->ksize, L->pad, L->stride);
    int ow = out_size(L->in_w, L->ksize, L->pad, L->stride);
    return oh * ow * (L->kind == ORC_MAXPOOL ? L->in_features : L->out_features);
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
    const int k = L->ksize, p = L->pad;
    const int OH = out_size(H, k, p, s), OW = out_size(Wd, k, p, s);
    uint64_t macs = 0;
    for (int oh = 0; oh < OH; ++oh)
        for (int ow = 0; ow < OW; ++ow)
            for (int co = 0; co < Co; ++co) {
                double acc = b ? b[co] : 0.0;
                for (int kh = 0; kh < k; ++kh)
                    for (int kw = 0; kw < k; ++kw) {
                        int ih = oh * s + kh - p, iw = ow * s + kw - p;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue; /* zero padding */
                        for (int ci = 0; ci < Ci; ++ci) {
                            acc += W[(((size_t)co * Ci + ci) * k + kh) * k + kw] *
                                   h[((size_t)ih * Wd + iw) * Ci + ci];
                            ++macs;
                        }
                    }
                z[((size_t)oh * OW + ow) * Co + co] = acc;
            }
    return macs;
}

/* Maximum over the window; taps outside the image are skipped, so they never win. */
static void maxpool_layer(const orc_layer* L, const double* h, double* z)
{
    const int C = L->in_features, H = L->in_h, Wd = L->in_w, s = L->stride, k = L->ksize, p = L->pad;
    const int OH = out_size(H, k, p, s), OW = out_size(Wd, k, p, s);
    for (int oh = 0; oh < OH; ++oh)
        for (int ow = 0; ow < OW; ++ow)
            for (int c = 0; c < C; ++c) {
                double best = -INFINITY;
                for (int kh = 0; kh < k; ++kh)
                    for (int kw = 0; kw < k; ++kw) {
                        int ih = oh * s + kh - p, iw = ow * s + kw - p;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                        double v = h[((size_t)ih * Wd + iw) * C + c];
                        if (v > best) best = v;
                    }
                z[((size_t)oh * OW + ow) * C + c] = best;
            }
}

static void add_layer(const orc_layer* L, const double* a, const double* b, double* z)
{
    const int n = L->in_h * L->in_w * L->in_features;
    for (int i = 0; i < n; ++i) z[i] = a[i] + b[i];
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
    const int k = L->ksize, pd = L->pad;
    const int OH = out_size(H, k, pd, s), OW = out_size(Wd, k, pd, s), K = Ci * k * k;
    double* col = (double*)calloc((size_t)K, sizeof(double));
    orc_layer fc = {ORC_FC, ORC_ACT_NONE, K, Co, 0, 0, 0, 0, 0, 0, 0};
    uint64_t macs = 0;
    for (int p = 0; p < OH * OW; ++p) {
        int oh = p / OW, ow = p % OW;
        for (int j = 0; j < K; ++j) {
            int ci = j / (k * k), kh = (j % (k * k)) / k, kw = j % k;
            int ih = oh * s + kh - pd, iw = ow * s + kw - pd;
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
    /* outs[0] = the request, outs[l + 1] = output of layer l: a later layer may name any earlier one */
    double** outs = (double**)calloc((size_t)n_layers + 1, sizeof(double*));
    int len = orc_layer_in_len(&layers[0]);
    outs[0] = (double*)malloc(sizeof(double) * (size_t)len);
    for (int i = 0; i < len; ++i) outs[0][i] = round_bf16 ? orc_round_bf16(x[i]) : x[i];
    uint64_t macs = 0;
    size_t hid_pos = 0;
    for (int l = 0; l < n_layers; ++l) {
        const orc_layer* L = &layers[l];
        const int out_len = orc_layer_out_len(L);
        const double* in = outs[L->src > 0 ? L->src : l];
        double* z = (double*)malloc(sizeof(double) * (size_t)out_len);
        outs[l + 1] = z;
        if (L->kind == ORC_FC) macs += fc_layer(L, weights[l], biases[l], in, z);
        else if (L->kind == ORC_CONV) macs += conv_layer(L, weights[l], biases[l], in, z);
        else if (L->kind == ORC_MAXPOOL) maxpool_layer(L, in, z);
        else if (L->kind == ORC_ADD) add_layer(L, in, outs[L->src2 > 0 ? L->src2 : l], z);
        else gap_layer(L, in, z);
        if (l == n_layers - 1) {
            for (int i = 0; i < out_len; ++i) logits[i] = z[i];
        } else {
            for (int i = 0; i < out_len; ++i) {
                double a = apply_act(z[i], L->act);
                z[i] = round_bf16 ? orc_round_bf16(a) : a;
            }
            if (hidden_out) { memcpy(hidden_out + hid_pos, z, sizeof(double) * (size_t)out_len); hid_pos += (size_t)out_len; }
        }
        len = out_len;
    }
    orc_head(logits, len, probs, label);
    for (int l = 0; l <= n_layers; ++l) free(outs[l]);
    free(outs);
    return macs;
}

/* ---- batch normalisation folded into the convolution before it ------------ */
/* W [Co][per] and b [Co] are replaced by the folded values (see the header).  bn = gamma, beta,
 * mean, var, each [Co].  to_bf16: round the folded filters to bfloat16, else to fp32. */
void orc_fold_bn(double* W, double* b, int Co, int per, const double* gamma, const double* beta,
                 const double* mean, const double* var, double eps, int to_bf16)
{
    for (int c = 0; c < Co; ++c) {
        const double s = gamma[c] / sqrt(var[c] + eps);
        for (int i = 0; i < per; ++i) {
            const double w = W[(size_t)c * per + i] * s;
            W[(size_t)c * per + i] = to_bf16 ? orc_round_bf16(w) : (double)(float)w;
        }
        const double shifted = (b[c] - mean[c]) * s;
        b[c] = (double)(float)(shifted + beta[c]);
    }
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
void orc_maxpool(const orc_layer* L, const double* h, double* z) { maxpool_layer(L, h, z); }
void orc_add(const orc_layer* L, const double* a, const double* b, double* z) { add_layer(L, a, b, z); }
