/*
 * CPU oracle for scheme scoring in Arithmetic-Intensity-Aware Quantization.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU path must compute; it is linked by the tests, the smoke check and the
 * CPU-baseline leg of the benchmark and by nothing else.  It shares no code
 * with the HIP library.
 *
 * What it states (paper sections in brackets):
 *  - a scheme q = (q_1..q_L) gives every layer a bit-width           [Problem Formulation]
 *  - each layer's weights are quantized to q_i bits and the model's
 *    accuracy is measured by running it                              [Introduction (ii); Search Over
 *                                                                     Mixed-Precision Schemes]
 *  - the model's global arithmetic intensity follows analytically
 *    from FLOPs and memory traffic                                   [Introduction (i)]
 * The paper fixes neither the quantizer nor the AI formula; the readings used
 * here are spelled out next to each function.
 *
 * Arithmetic: the quantizer is IEEE binary32 scalar code (its results are
 * integers and scales that must be reproducible bit for bit); everything in
 * the forward pass is binary64 direct loops.
 *
 * Activation fake-quantization (a variant; the paper gives a layer only a bit-width) is stated
 * next to quantize_activations below and pinned by tests/test_oracle_activations.py.
 *
 * Parity status: quantizer, convolution, depthwise, classifier head and the AI
 * model are pinned by tests/test_oracle_*.py (hand-worked rows, closed forms,
 * library matmul / einsum special cases, the paper's AI gains).  Trained-model
 * accuracy figures of the paper (92 %, 82.05 % ...) are "parity unpinned":
 * they need CIFAR-10 and trained weights, which do not exist here.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { F_KIND, F_CIN, F_COUT, F_KH, F_KW, F_STRIDE, F_PAD, F_HIN, F_WIN, F_INPUT, F_RESIDUAL, F_ACT,
       F_SLOT, N_FIELDS };
enum { KIND_CONV = 0, KIND_DEPTHWISE = 1, KIND_FC = 2 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2 };

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int bits_supported(int bits)
{
    return bits == 32 || bits == 16 || bits == 8 || bits == 6 || bits == 4 || bits == 2;
}

/*
 * Symmetric per-output-channel weight quantize -> dequantize   [Problem Formulation: "bit-width q_i"]
 *
 * Reading (the paper gives only the bit-width): for row c of w[cout][k],
 *   amax = max_k |w|,  qmax = 2^(b-1) - 1,  s = amax / qmax  (s = 1 if the row is all zero),
 *   code = clamp(round_half_even(w / s), -qmax, +qmax),  w_dq = code * s,
 * every step one IEEE binary32 operation.  b = 32 leaves the row unchanged with s = 1.
 * codes may be NULL.  Returns 0, or 2 for a bit-width outside {32,16,8,6,4,2}.
 */
int oracle_quantize_weights(const float *w, int cout, int k, int bits, float *w_dq, float *scales,
                            int32_t *codes)
{
    if (!bits_supported(bits)) return 2;
    if (!w || !w_dq || !scales || cout < 0 || k < 0) return 1;
    for (int c = 0; c < cout; ++c) {
        const float *row = w + (size_t)c * k;
        float *out = w_dq + (size_t)c * k;
        if (bits == 32) {
            scales[c] = 1.0f;
            for (int i = 0; i < k; ++i) out[i] = row[i];
            continue;
        }
        const int32_t qmax = (1 << (bits - 1)) - 1;
        float amax = 0.0f;
        for (int i = 0; i < k; ++i) {
            float a = fabsf(row[i]);
            if (a > amax) amax = a;
        }
        volatile float s = (amax > 0.0f) ? amax / (float)qmax : 1.0f;
        scales[c] = s;
        for (int i = 0; i < k; ++i) {
            volatile float t = row[i] / s;
            int32_t q = (int32_t)rintf(t); /* default rounding mode: to nearest, ties to even */
            if (q > qmax) q = qmax;
            if (q < -qmax) q = -qmax;
            volatile float d = (float)q * s;
            out[i] = d;
            if (codes) codes[(size_t)c * k + i] = q;
        }
    }
    return 0;
}

/*
 * Per-tensor variant: one scale for the whole weight matrix     [Conclusion: per-channel effects are
 *                                                                named as future work, so the paper's
 *                                                                own runs most likely used one scale
 *                                                                per layer]
 * Definition: the per-output-channel rule above applied to the matrix read as a single row of
 * cout * k weights; scales[c] receives that one scale for every c.
 */
int oracle_quantize_weights_per_tensor(const float *w, int cout, int k, int bits, float *w_dq, float *scales,
                                       int32_t *codes)
{
    if (!bits_supported(bits)) return 2;
    if (!w || !w_dq || !scales || cout < 0 || k < 0) return 1;
    float s = 1.0f;
    int rc = oracle_quantize_weights(w, 1, cout * k, bits, w_dq, &s, codes);
    if (rc) return rc;
    for (int c = 0; c < cout; ++c) scales[c] = s;
    return 0;
}

static int out_size(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

/*
 * Analytic arithmetic intensity of a scheme                     [Introduction (i); Search: "AI can be
 *                                                                recomputed analytically"]
 * Reading (the paper prints no formula): per layer
 *   MACs  = Hout*Wout*Cout*(Cin/groups)*kh*kw   (classifier: Cin*Cout)
 *   FLOPs = 2 * MACs * batch
 *   Bytes = n_weights * b/8 + 4 * batch * (input elements + output elements)
 * and AI = sum FLOPs / sum Bytes over all layers.  Layers outside the scheme count at 32 bits.
 * With batch = 1 this reproduces the paper's ResNet-20 gains (about +42 % at uniform 8 bits).
 */
int oracle_layer_ai_ex(const int32_t *desc, int n_layers, const uint8_t *scheme, int L, int batch, int act_quant,
                       double *flops, double *bytes, double *global_ai);

int oracle_layer_ai(const int32_t *desc, int n_layers, const uint8_t *scheme, int L, int batch,
                    double *flops, double *bytes, double *global_ai)
{
    return oracle_layer_ai_ex(desc, n_layers, scheme, L, batch, 0, flops, bytes, global_ai);
}

/*
 * The same with activation fake-quantization counted (act_quant != 0): a layer at b bits reads its
 * input activations at b bits as well, so
 *   Bytes = n_weights * b/8 + batch * (input elements * b/8 + 4 * output elements);
 * outputs are written in fp32 (the next layer quantizes what it reads to its own width).
 */
int oracle_layer_ai_ex(const int32_t *desc, int n_layers, const uint8_t *scheme, int L, int batch, int act_quant,
                       double *flops, double *bytes, double *global_ai)
{
    if (!desc || n_layers <= 0 || batch < 1 || !global_ai) return 1;
    double sum_f = 0.0, sum_b = 0.0;
    for (int l = 0; l < n_layers; ++l) {
        const int32_t *d = desc + (size_t)l * N_FIELDS;
        int bits = 32;
        if (d[F_SLOT] >= 0) {
            if (!scheme || d[F_SLOT] >= L) return 3;
            bits = scheme[d[F_SLOT]];
            if (!bits_supported(bits)) return 2;
        }
        double macs, n_w, in_e, out_e;
        if (d[F_KIND] == KIND_FC) {
            n_w = (double)d[F_CIN] * d[F_COUT];
            macs = n_w;
            in_e = d[F_CIN];
            out_e = d[F_COUT];
        } else {
            int ho = out_size(d[F_HIN], d[F_KH], d[F_STRIDE], d[F_PAD]);
            int wo = out_size(d[F_WIN], d[F_KW], d[F_STRIDE], d[F_PAD]);
            double cin_g = (d[F_KIND] == KIND_DEPTHWISE) ? 1.0 : (double)d[F_CIN];
            n_w = (double)d[F_COUT] * cin_g * d[F_KH] * d[F_KW];
            macs = (double)ho * wo * n_w;
            in_e = (double)d[F_HIN] * d[F_WIN] * d[F_CIN];
            out_e = (double)ho * wo * d[F_COUT];
        }
        double f = 2.0 * macs * batch;
        double in_bytes = act_quant ? in_e * bits / 8.0 : 4.0 * in_e;
        double b = n_w * bits / 8.0 + batch * (in_bytes + 4.0 * out_e);
        if (flops) flops[l] = f;
        if (bytes) bytes[l] = b;
        sum_f += f;
        sum_b += b;
    }
    *global_ai = sum_f / sum_b;
    return 0;
}

static double activate(double v, int act)
{
    if (act == ACT_RELU || act == ACT_RELU6) v = v > 0.0 ? v : 0.0;
    if (act == ACT_RELU6) v = v < 6.0 ? v : 6.0;
    return v;
}

/*
 * One convolution layer on one image, the textbook definition:
 *   y[oy][ox][co] = act( bias[co] + sum_{ci,ky,kx} x[oy*st+ky-pad][ox*st+kx-pad][ci] * w[co][ci][ky][kx]
 *                        (+ res[oy][ox][co]) )
 * cross-correlation, zero outside the image.  x is [hin][win][cin], w is [cout][cin][kh][kw]
 * (depthwise: [c][kh][kw], output channel c reads input channel c).  Returns the number of
 * multiply-adds performed, padded taps included.
 */
static int64_t conv_layer(const int32_t *d, const double *x, const float *w, const float *bias,
                          const double *res, double *y)
{
    const int cin = d[F_CIN], cout = d[F_COUT], kh = d[F_KH], kw = d[F_KW];
    const int st = d[F_STRIDE], pad = d[F_PAD], hin = d[F_HIN], win = d[F_WIN];
    const int ho = out_size(hin, kh, st, pad), wo = out_size(win, kw, st, pad);
    const int dw = d[F_KIND] == KIND_DEPTHWISE;
    int64_t macs = 0;
    for (int oy = 0; oy < ho; ++oy)
        for (int ox = 0; ox < wo; ++ox)
            for (int co = 0; co < cout; ++co) {
                double acc = (double)bias[co];
                const int ci0 = dw ? co : 0, ci1 = dw ? co + 1 : cin;
                for (int ci = ci0; ci < ci1; ++ci)
                    for (int ky = 0; ky < kh; ++ky)
                        for (int kx = 0; kx < kw; ++kx) {
                            int iy = oy * st + ky - pad, ix = ox * st + kx - pad;
                            double xv = 0.0;
                            if (iy >= 0 && iy < hin && ix >= 0 && ix < win)
                                xv = x[((size_t)iy * win + ix) * cin + ci];
                            size_t wi = dw ? ((size_t)co * kh + ky) * kw + kx
                                           : (((size_t)co * cin + ci) * kh + ky) * kw + kx;
                            acc += xv * (double)w[wi];
                            ++macs;
                        }
                size_t oi = ((size_t)oy * wo + ox) * cout + co;
                if (res) acc += res[oi];
                y[oi] = activate(acc, d[F_ACT]);
            }
    return macs;
}

/*
 * Activation fake-quantization (variant)                        [Problem Formulation: a layer gets a
 *                                                                bit-width; the paper does not say whether
 *                                                                that width also applies to what the layer
 *                                                                reads]
 * Reading: a layer at b < 32 bits reads its input tensor quantized to b bits, symmetric, with one
 * scale per image taken from that image's own tensor (no calibration data is needed):
 *   amax = max |x| over the tensor,  qmax = 2^(b-1) - 1,  s = amax / qmax  (1 if the tensor is zero),
 *   x_q = clamp(round_half_even(x / s), -qmax, +qmax) * s,
 * the same rule as for a weight row, every step one IEEE binary32 operation on the activation
 * rounded to binary32.  The residual input of a layer is added unquantized; the classifier reads the
 * pooled vector quantized.  b = 32: nothing happens.  x is replaced in place.
 */
static void quantize_activations(double *x, size_t n, int bits)
{
    if (bits == 32) return;
    const int32_t qmax = (1 << (bits - 1)) - 1;
    float amax = 0.0f;
    for (size_t i = 0; i < n; ++i) {
        float a = fabsf((float)x[i]);
        if (a > amax) amax = a;
    }
    volatile float s = (amax > 0.0f) ? amax / (float)qmax : 1.0f;
    for (size_t i = 0; i < n; ++i) {
        volatile float t = (float)x[i] / s;
        int32_t q = (int32_t)rintf(t);
        if (q > qmax) q = qmax;
        if (q < -qmax) q = -qmax;
        volatile float d = (float)q * s;
        x[i] = (double)d;
    }
}

/* Exposed so that tests can pin the rule on hand-worked tensors.  x: n doubles, replaced in place. */
int oracle_quantize_activations(double *x, int64_t n, int bits)
{
    if (!bits_supported(bits)) return 2;
    if (!x || n < 0) return 1;
    quantize_activations(x, (size_t)n, bits);
    return 0;
}

/* Classifier: global average pool over hin*win, then z[j] = bias[j] + sum_c p[c] * w[j][c].
 * act_bits < 32: the pooled vector is quantized before the matrix reads it. */
static int64_t fc_layer(const int32_t *d, const double *x, const float *w, const float *bias, double *z, int act_bits)
{
    const int cin = d[F_CIN], cout = d[F_COUT], hw = d[F_HIN] * d[F_WIN];
    double *p = (double *)malloc(sizeof(double) * cin);
    for (int c = 0; c < cin; ++c) {
        double s = 0.0;
        for (int i = 0; i < hw; ++i) s += x[(size_t)i * cin + c];
        p[c] = s / (double)hw;
    }
    quantize_activations(p, (size_t)cin, act_bits);
    int64_t macs = 0;
    for (int j = 0; j < cout; ++j) {
        double acc = (double)bias[j];
        for (int c = 0; c < cin; ++c) {
            acc += p[c] * (double)w[(size_t)j * cin + c];
            ++macs;
        }
        z[j] = activate(acc, d[F_ACT]);
    }
    free(p);
    return macs;
}

static size_t node_out_elems(const int32_t *d)
{
    if (d[F_KIND] == KIND_FC) return (size_t)d[F_COUT];
    int ho = out_size(d[F_HIN], d[F_KH], d[F_STRIDE], d[F_PAD]);
    int wo = out_size(d[F_WIN], d[F_KW], d[F_STRIDE], d[F_PAD]);
    return (size_t)ho * wo * d[F_COUT];
}

/* Structural check of a graph: node order, shapes of producer and consumer agree.  0 = valid. */
int oracle_check_graph(const int32_t *desc, int n_layers, int hin0, int win0, int cin0)
{
    if (!desc || n_layers <= 0) return 1;
    for (int l = 0; l < n_layers; ++l) {
        const int32_t *d = desc + (size_t)l * N_FIELDS;
        if (d[F_KIND] < 0 || d[F_KIND] > 2) return 6;
        if (d[F_INPUT] >= l || d[F_RESIDUAL] >= l || d[F_INPUT] < -1 || d[F_RESIDUAL] < -1) return 3;
        int ph, pw, pc;
        if (d[F_INPUT] < 0) {
            ph = hin0; pw = win0; pc = cin0;
        } else {
            const int32_t *p = desc + (size_t)d[F_INPUT] * N_FIELDS;
            if (p[F_KIND] == KIND_FC) return 3;
            ph = out_size(p[F_HIN], p[F_KH], p[F_STRIDE], p[F_PAD]);
            pw = out_size(p[F_WIN], p[F_KW], p[F_STRIDE], p[F_PAD]);
            pc = p[F_COUT];
        }
        if (ph != d[F_HIN] || pw != d[F_WIN] || pc != d[F_CIN]) return 3;
        if (d[F_KIND] == KIND_DEPTHWISE && d[F_CIN] != d[F_COUT]) return 3;
        if (d[F_RESIDUAL] >= 0) {
            const int32_t *r = desc + (size_t)d[F_RESIDUAL] * N_FIELDS;
            if (d[F_KIND] == KIND_FC || r[F_KIND] == KIND_FC) return 3;
            if (node_out_elems(r) != node_out_elems(d) || r[F_COUT] != d[F_COUT]) return 3;
        }
        if (d[F_KIND] == KIND_FC && l != n_layers - 1) return 6;
    }
    if (desc[(size_t)(n_layers - 1) * N_FIELDS + F_KIND] != KIND_FC) return 6;
    return 0;
}

/*
 * Forward pass of one image through the graph in binary64.  image is fp32 [hin][win][3];
 * w[l] / bias[l] are that layer's (already dequantized) fp32 tensors.  logits receives
 * n_classes doubles.  acts (nullable) receives every node's output, concatenated in node
 * order.  Returns total multiply-adds.
 */
static size_t node_out_elems(const int32_t *d);

/* act_bits: NULL, or per node the width its input activations are quantized to (32 = not at all). */
static int64_t forward_image(const int32_t *desc, int n_layers, const float *const *w,
                             const float *const *bias, const float *image, double *logits, double *acts,
                             const int *act_bits)
{
    const int32_t *d0 = desc;
    size_t in_elems = (size_t)d0[F_HIN] * d0[F_WIN] * d0[F_CIN];
    double *x0 = (double *)malloc(sizeof(double) * in_elems);
    for (size_t i = 0; i < in_elems; ++i) x0[i] = (double)image[i];
    double **out = (double **)calloc(n_layers, sizeof(double *));
    int64_t macs = 0;
    size_t acts_off = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int32_t *d = desc + (size_t)l * N_FIELDS;
        const double *x = d[F_INPUT] < 0 ? x0 : out[d[F_INPUT]];
        const double *r = d[F_RESIDUAL] < 0 ? NULL : out[d[F_RESIDUAL]];
        size_t n_out = node_out_elems(d);
        out[l] = (double *)malloc(sizeof(double) * n_out);
        const int ab = act_bits ? act_bits[l] : 32;
        if (d[F_KIND] == KIND_FC) {
            macs += fc_layer(d, x, w[l], bias[l], out[l], ab);
        } else if (ab != 32) {
            /* the layer reads a quantized copy: other readers of the same tensor see it as it is */
            size_t n_in = (size_t)d[F_HIN] * d[F_WIN] * d[F_CIN];
            double *xq = (double *)malloc(sizeof(double) * n_in);
            memcpy(xq, x, sizeof(double) * n_in);
            quantize_activations(xq, n_in, ab);
            macs += conv_layer(d, xq, w[l], bias[l], r, out[l]);
            free(xq);
        } else {
            macs += conv_layer(d, x, w[l], bias[l], r, out[l]);
        }
        if (acts) {
            memcpy(acts + acts_off, out[l], sizeof(double) * n_out);
            acts_off += n_out;
        }
    }
    const int32_t *dl = desc + (size_t)(n_layers - 1) * N_FIELDS;
    memcpy(logits, out[n_layers - 1], sizeof(double) * dl[F_COUT]);
    for (int l = 0; l < n_layers; ++l) free(out[l]);
    free(out);
    free(x0);
    return macs;
}

/* argmax with the lowest index winning ties */
static int32_t argmax(const double *z, int n)
{
    int32_t best = 0;
    for (int j = 1; j < n; ++j)
        if (z[j] > z[best]) best = j;
    return best;
}

/*
 * Forward of N images with the weights as given (no quantization).
 * logits [N][n_classes] doubles; top1 (nullable) [N]; acts (nullable) [N][sum of node outputs];
 * macs_per_image (nullable) receives the multiply-add count of one image.
 */
int oracle_forward(const int32_t *desc, int n_layers, const float *const *w, const float *const *bias,
                   const float *images, int N, double *logits, int32_t *top1, double *acts,
                   int64_t *macs_per_image)
{
    if (!desc || !w || !bias || !images || !logits || N < 0) return 1;
    const int32_t *d0 = desc;
    int rc = oracle_check_graph(desc, n_layers, d0[F_HIN], d0[F_WIN], d0[F_CIN]);
    if (rc) return rc;
    const int ncls = desc[(size_t)(n_layers - 1) * N_FIELDS + F_COUT];
    size_t img_elems = (size_t)d0[F_HIN] * d0[F_WIN] * d0[F_CIN];
    size_t acts_per = 0;
    for (int l = 0; l < n_layers; ++l) acts_per += node_out_elems(desc + (size_t)l * N_FIELDS);
    int64_t macs0 = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < N; ++n) {
        int64_t m = forward_image(desc, n_layers, w, bias, images + (size_t)n * img_elems,
                                  logits + (size_t)n * ncls, acts ? acts + (size_t)n * acts_per : NULL, NULL);
        if (top1) top1[n] = argmax(logits + (size_t)n * ncls, ncls);
        if (n == 0) macs0 = m;
    }
    if (macs_per_image) *macs_per_image = macs0;
    return 0;
}

/*
 * Score S schemes on N images                                   [Problem Formulation; Search Over
 *                                                                Mixed-Precision Schemes]
 * For each scheme: quantize-dequantize every scheme layer at its bit-width (layers with
 * scheme_slot = -1 keep their fp32 weights), run all images, take top-1.  "Accuracy" on
 * unlabeled synthetic images is agreement with the top-1 of the all-FP32 model:
 * agree[s] = #{n : top1[s][n] == top1_base[n]}.
 * w / bias: fp32 per node.  schemes uint8 [S][L].  Outputs (host, caller-allocated):
 * logits_base [N][C], top1_base [N], logits [S][N][C], top1 [S][N], agree [S]; logits, top1 nullable.
 */
int oracle_eval_schemes_ex(const int32_t *desc, int n_layers, const float *const *w, const float *const *bias,
                           const float *images, int N, const uint8_t *schemes, int S, int L, int per_tensor,
                           double *logits_base, int32_t *top1_base, double *logits, int32_t *top1,
                           int32_t *agree);

int oracle_eval_schemes(const int32_t *desc, int n_layers, const float *const *w, const float *const *bias,
                        const float *images, int N, const uint8_t *schemes, int S, int L,
                        double *logits_base, int32_t *top1_base, double *logits, int32_t *top1,
                        int32_t *agree)
{
    return oracle_eval_schemes_ex(desc, n_layers, w, bias, images, N, schemes, S, L, 0, logits_base, top1_base,
                                  logits, top1, agree);
}

int oracle_eval_schemes_aq(const int32_t *desc, int n_layers, const float *const *w, const float *const *bias,
                           const float *images, int N, const uint8_t *schemes, int S, int L, int per_tensor,
                           int act_quant, double *logits_base, int32_t *top1_base, double *logits, int32_t *top1,
                           int32_t *agree, double *acts);

/* per_tensor != 0: every scheme layer is quantized with one scale per layer instead of one per output channel. */
int oracle_eval_schemes_ex(const int32_t *desc, int n_layers, const float *const *w, const float *const *bias,
                           const float *images, int N, const uint8_t *schemes, int S, int L, int per_tensor,
                           double *logits_base, int32_t *top1_base, double *logits, int32_t *top1,
                           int32_t *agree)
{
    return oracle_eval_schemes_aq(desc, n_layers, w, bias, images, N, schemes, S, L, per_tensor, 0, logits_base,
                                  top1_base, logits, top1, agree, NULL);
}

/* act_quant != 0: a scheme layer at b bits also reads its input activations at b bits (quantize_activations).
 * acts (nullable): every node's output under every scheme, [S][N][sum of node outputs]. */
int oracle_eval_schemes_aq(const int32_t *desc, int n_layers, const float *const *w, const float *const *bias,
                           const float *images, int N, const uint8_t *schemes, int S, int L, int per_tensor,
                           int act_quant, double *logits_base, int32_t *top1_base, double *logits, int32_t *top1,
                           int32_t *agree, double *acts)
{
    if (!desc || !w || !bias || !images || !schemes || !logits_base || !top1_base || !agree) return 1;
    if (N < 0 || S < 0) return 1;
    const int32_t *d0 = desc;
    int rc = oracle_check_graph(desc, n_layers, d0[F_HIN], d0[F_WIN], d0[F_CIN]);
    if (rc) return rc;
    int max_slot = -1;
    for (int l = 0; l < n_layers; ++l) {
        int s = desc[(size_t)l * N_FIELDS + F_SLOT];
        if (s > max_slot) max_slot = s;
    }
    if (max_slot + 1 != L) return 3;
    for (int i = 0; i < S * L; ++i)
        if (!bits_supported(schemes[i])) return 2;
    const int ncls = desc[(size_t)(n_layers - 1) * N_FIELDS + F_COUT];
    if (ncls > 64) return 6;
    size_t img_elems = (size_t)d0[F_HIN] * d0[F_WIN] * d0[F_CIN];

    rc = oracle_forward(desc, n_layers, w, bias, images, N, logits_base, top1_base, NULL, NULL);
    if (rc) return rc;

    size_t acts_per = 0;
    for (int l = 0; l < n_layers; ++l) acts_per += node_out_elems(desc + (size_t)l * N_FIELDS);
    for (int s = 0; s < S; ++s) {
        float **wq = (float **)calloc(n_layers, sizeof(float *));
        int *ab = (int *)malloc(sizeof(int) * n_layers);
        for (int l = 0; l < n_layers; ++l) {
            const int32_t *d = desc + (size_t)l * N_FIELDS;
            int cout = d[F_COUT];
            int k = d[F_KIND] == KIND_FC ? d[F_CIN]
                    : (d[F_KIND] == KIND_DEPTHWISE ? 1 : d[F_CIN]) * d[F_KH] * d[F_KW];
            int bits = d[F_SLOT] >= 0 ? schemes[(size_t)s * L + d[F_SLOT]] : 32;
            ab[l] = act_quant ? bits : 32;
            wq[l] = (float *)malloc(sizeof(float) * (size_t)cout * k);
            float *sc = (float *)malloc(sizeof(float) * cout);
            if (per_tensor)
                oracle_quantize_weights_per_tensor(w[l], cout, k, bits, wq[l], sc, NULL);
            else
                oracle_quantize_weights(w[l], cout, k, bits, wq[l], sc, NULL);
            free(sc);
        }
        int32_t count = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : count)
        for (int n = 0; n < N; ++n) {
            double z[64];
            double *zp = logits ? logits + ((size_t)s * N + n) * ncls : z;
            forward_image(desc, n_layers, (const float *const *)wq, bias, images + (size_t)n * img_elems, zp,
                          acts ? acts + ((size_t)s * N + n) * acts_per : NULL, ab);
            int32_t t = argmax(zp, ncls);
            if (top1) top1[(size_t)s * N + n] = t;
            count += (t == top1_base[n]);
        }
        agree[s] = count;
        for (int l = 0; l < n_layers; ++l) free(wq[l]);
        free(wq);
        free(ab);
    }
    return 0;
}

/* Single layer on one image, exposed so that tests can pin the loops against brute force. */
int oracle_conv_layer(const int32_t *d, const double *x, const float *w, const float *bias, const double *res,
                      double *y, int64_t *macs)
{
    if (!d || !x || !w || !bias || !y) return 1;
    int64_t m = d[F_KIND] == KIND_FC ? fc_layer(d, x, w, bias, y, 32) : conv_layer(d, x, w, bias, res, y);
    if (macs) *macs = m;
    return 0;
}
