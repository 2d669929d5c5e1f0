/*
 * aiq.h - C boundary of the MI355X scheme-scoring library (libaiq.so).
 *
 * Arithmetic-Intensity-Aware Quantization searches over per-layer bit-width
 * schemes q = (q_1 .. q_L); every candidate is scored by (i) an analytic global
 * arithmetic intensity and (ii) the accuracy of the model with each layer's
 * weights quantized to q_i bits (paper: Introduction, items (i) and (ii);
 * Approach, Problem Formulation; Search Over Mixed-Precision Schemes).  This
 * library is the scoring step: weight quantize-dequantize, a batched forward
 * pass of all candidate schemes, and top-1 agreement with the FP32 model.  The
 * search loops stay with the caller.
 *
 * Conventions
 *  - Plain C ABI.  No function throws; every function returns aiq_status.
 *  - "device" pointers are HIP device memory owned by the caller; "host"
 *    pointers are ordinary memory.  The library allocates device memory only in
 *    aiq_model_create (weights and the per-bit-width weight bank) and frees it
 *    in aiq_model_destroy.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *    Device work is enqueued on it and not synchronised.
 *  - Arguments are validated before any device work; on a non-OK status found
 *    by validation no output buffer has been touched.
 *  - Small HOST arrays an entry point takes (schemes, a reference scheme) are read in full
 *    before it returns - they reach the device as kernel arguments - so the caller may reuse
 *    them at once, whatever kind of host memory they live in.
 *  - One aiq_model must not be used from two threads at once.
 *  - There is no CPU fallback: without a usable GPU every device entry point
 *    returns AIQ_DEVICE_ERROR.
 */
#ifndef AIQ_H
#define AIQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t aiq_status;
enum {
    AIQ_OK = 0,
    AIQ_INVALID_ARG = 1,        /* null pointer, negative or zero size where not allowed */
    AIQ_UNSUPPORTED_BITS = 2,   /* bit-width outside {32,16,8,6,4,2} */
    AIQ_SHAPE_MISMATCH = 3,     /* graph shapes inconsistent, scheme length != L */
    AIQ_WORKSPACE_TOO_SMALL = 4,
    AIQ_DEVICE_ERROR = 5,       /* a HIP call failed; see aiq_last_hip_error() */
    AIQ_UNSUPPORTED_LAYER = 6   /* layer kind / kernel size / stride the kernels do not cover */
};

/* Static, never NULL. */
const char *aiq_status_str(aiq_status st);
/* hipError_t (as int) of the last failed HIP call on this thread, 0 if none. */
int32_t aiq_last_hip_error(void);

/*
 * One weighted layer of a straight-line graph with residual links.  Nodes are
 * listed in execution order.  Activations are NHWC fp32.
 */
typedef struct {
    int32_t kind;        /* 0 convolution (groups = 1), 1 depthwise convolution, 2 classifier
                            (global average pool over hin x win, then a cout x cin matrix) */
    int32_t cin, cout;
    int32_t kh, kw;      /* 3x3 or 1x1 (classifier: 1, 1) */
    int32_t stride;      /* 1 or 2 */
    int32_t pad;         /* 1 for 3x3, 0 for 1x1 */
    int32_t hin, win;    /* input spatial size */
    int32_t input;       /* producing node, -1 = the network input */
    int32_t residual;    /* node whose output is added before the activation, -1 = none */
    int32_t act;         /* 0 none, 1 ReLU, 2 ReLU6 */
    int32_t scheme_slot; /* position i of this layer in a scheme (q_1..q_L), -1 = always FP32 */
} aiq_layer_desc;

/*
 * Analytic arithmetic intensity of one scheme (paper: Introduction item (i);
 * Search Over Mixed-Precision Schemes, closing paragraph).  Host only, pure.
 *   FLOPs_l = 2 * batch * Hout*Wout*Cout*(Cin/groups)*kh*kw    (classifier: 2*batch*Cin*Cout)
 *   Bytes_l = n_weights_l * bits_l / 8 + 4 * batch * (in_elems_l + out_elems_l)
 *   AI      = sum_l FLOPs_l / sum_l Bytes_l
 * layers:  host, n_layers records.  scheme: host uint8[L], values in {32,16,8,6,4,2};
 * layers with scheme_slot = -1 count at 32 bits.  flops_per_layer / bytes_per_layer:
 * host double[n_layers], either may be NULL.  global_ai: host, required.
 * Errors: INVALID_ARG (null, n_layers <= 0, batch < 1), SHAPE_MISMATCH (a scheme_slot >= L),
 * UNSUPPORTED_BITS.
 */
aiq_status aiq_layer_ai(const aiq_layer_desc *layers, int32_t n_layers, const uint8_t *scheme, int32_t L,
                        int32_t batch, double *flops_per_layer, double *bytes_per_layer, double *global_ai);
/*
 * The same for the variant in which a layer at b bits also reads its input activations at b bits
 * (AIQ_MODEL_ACT_QUANT below; the paper's Problem Formulation gives a layer one bit-width and does not
 * say what it covers).  act_quant = 1:
 *   Bytes_l = n_weights_l * bits_l / 8 + batch * (in_elems_l * bits_l / 8 + 4 * out_elems_l);
 * act_quant = 0 is aiq_layer_ai.  Errors as aiq_layer_ai; act_quant outside {0, 1}: INVALID_ARG.
 */
aiq_status aiq_layer_ai_ex(const aiq_layer_desc *layers, int32_t n_layers, const uint8_t *scheme, int32_t L,
                           int32_t batch, int32_t act_quant, double *flops_per_layer, double *bytes_per_layer,
                           double *global_ai);

/*
 * Symmetric per-output-channel quantize -> dequantize of one weight matrix
 * (paper: Problem Formulation, "bit-width q_i" per layer; the rule itself is
 * this library's reading): for row c,
 *   amax = max_k |w[c][k]|, qmax = 2^(bits-1)-1, s = amax/qmax (1 if amax = 0),
 *   code = clamp(round-half-even(w/s), -qmax, qmax), w_dq = code * s,
 * each step one IEEE binary32 operation.  bits = 32 copies w and sets s = 1.
 * w, w_dq: device fp32 [cout][k] row-major (may not alias).  scales: device fp32 [cout].
 * codes: device int32 [cout][k] or NULL; left untouched when bits = 32.
 * cout = 0 or k = 0 is a valid no-op.  Asynchronous on hip_stream.
 * Errors: INVALID_ARG, UNSUPPORTED_BITS, DEVICE_ERROR.
 */
aiq_status aiq_quantize_weights(const float *w, int32_t cout, int32_t k, int32_t bits, float *w_dq,
                                float *scales, int32_t *codes, void *hip_stream);

/*
 * Same with a choice of granularity (the paper does not say which it used; its Conclusion names
 * per-channel effects as future work).  per_tensor = 0: one scale per output channel, as above.
 * per_tensor = 1: one scale for the whole matrix, s = max_{c,k} |w| / qmax, written to every
 * scales[c].  scratch: device, 4 bytes, 4-byte aligned, required when per_tensor = 1 (the
 * matrix-wide maximum is formed there by a first launch); may be NULL otherwise.
 * Errors: INVALID_ARG, UNSUPPORTED_BITS, DEVICE_ERROR.
 */
aiq_status aiq_quantize_weights_ex(const float *w, int32_t cout, int32_t k, int32_t bits, int32_t per_tensor,
                                   float *w_dq, float *scales, int32_t *codes, void *scratch, void *hip_stream);

typedef struct aiq_model aiq_model; /* opaque */

/*
 * Builds a model: validates the graph, copies weights and biases to the device
 * and allocates the weight bank (one slot per scheme layer and bit-width).
 * layers: host.  w_host[l]: host fp32 [cout][k], k = (cin/groups)*kh*kw in (ci, ky, kx)
 * order, BN already folded.  bias_host[l]: host fp32 [cout].  The network input is
 * fp32 [hin][win][cin] of node 0 per image.  Synchronous.
 * Errors: INVALID_ARG, SHAPE_MISMATCH, UNSUPPORTED_LAYER, DEVICE_ERROR.  *out is NULL on error.
 */
aiq_status aiq_model_create(const aiq_layer_desc *layers, int32_t n_layers, const float *const *w_host,
                            const float *const *bias_host, aiq_model **out);
/*
 * Same, with flags.  AIQ_MODEL_LAYERWISE: always run layer by layer through HBM, also for
 * graphs (CIFAR-style ResNets of 16/32/64 channels) whose activations would otherwise stay
 * in LDS for the whole network.  Both strategies compute the same function.
 * AIQ_MODEL_PER_TENSOR: one quantization scale per layer instead of one per output channel.
 * AIQ_MODEL_ACT_QUANT: activation fake-quantization (a variant; the paper's Problem Formulation gives a
 * layer a bit-width and says nothing of activations).  A scheme layer at b < 32 bits reads its input
 * tensor quantized to b bits by the weight rule with one scale per image, taken from that image's own
 * tensor: amax = max |x|, s = amax / (2^(b-1)-1) (1 if the tensor is zero),
 * x_q = clamp(round-half-even(x / s)) * s, each step one IEEE binary32 operation.  The residual input
 * of a layer is added unquantized, layers outside every scheme read their input as it is, the
 * classifier reads the pooled vector quantized.  Implies AIQ_MODEL_LAYERWISE.  The search drivers then
 * count activation bytes at the layer's width (aiq_layer_ai_ex).  Rounding an activation is a
 * discontinuity: two correct implementations whose activations differ in the last bit can assign
 * neighbouring codes, so outputs of deep networks are compared layer by layer (aiq_forward_nodes).
 */
enum { AIQ_MODEL_LAYERWISE = 1, AIQ_MODEL_PER_TENSOR = 2, AIQ_MODEL_ACT_QUANT = 4 };
aiq_status aiq_model_create_ex(const aiq_layer_desc *layers, int32_t n_layers, const float *const *w_host,
                               const float *const *bias_host, uint32_t flags, aiq_model **out);
/* 1 if the model runs LDS-resident (one launch for the whole network), 0 if not, -1 for NULL. */
int32_t aiq_model_is_lds_resident(const aiq_model *m);
/* Number of inverted-residual blocks (1x1 expand, depthwise 3x3, 1x1 project) that run as one
   launch with the expanded tensor held in LDS; the other layers run layer by layer.  -1 for NULL. */
int32_t aiq_model_lds_resident_blocks(const aiq_model *m);
void aiq_model_destroy(aiq_model *m); /* NULL-safe */

/* L (number of scheme layers) and the classifier width; -1 for a NULL model. */
int32_t aiq_model_scheme_layers(const aiq_model *m);
int32_t aiq_model_classes(const aiq_model *m);

/* Device bytes aiq_eval_schemes needs for S schemes processed chunk images at a time. */
aiq_status aiq_eval_workspace_bytes(const aiq_model *m, int32_t S, int32_t chunk, size_t *bytes);

/*
 * Scores S candidate schemes on N images (paper: Search Over Mixed-Precision
 * Schemes - the candidate configurations of one greedy iteration or one
 * coordinate-descent sweep are scored together).  For every scheme s each scheme
 * layer is quantized at schemes[s][slot] bits, the network is run on all images
 * and agree[s] = #{n : argmax logits[s][n] == top1_base[n]} (lowest index wins ties).
 *
 * images:    device fp32 [N][hin][win][cin] (NHWC).
 * schemes:   HOST uint8 [S][L]; read before the call returns.
 * chunk:     images per pass through the network (>= 1); N need not be a multiple.
 * top1_base: device int32 [N].  base_valid = 0: the library also runs the all-FP32
 *            scheme and writes its top-1 here; base_valid = 1: read only.
 * logits:    device fp32 [S][N][classes] or NULL.   top1: device int32 [S][N] or NULL.
 * agree:     device int32 [S], overwritten.
 * workspace: device, >= aiq_eval_workspace_bytes(m, S, chunk), 256-byte aligned.
 * S = 0 or N = 0 is valid (agree is zero-filled).  Asynchronous on hip_stream.
 * S + 1 may not exceed 65535 (INVALID_ARG): the schemes, plus the all-FP32 pass, form one grid axis.
 * Errors: INVALID_ARG (also a workspace that is not 256-byte aligned), UNSUPPORTED_BITS,
 * WORKSPACE_TOO_SMALL, DEVICE_ERROR.
 */
aiq_status aiq_eval_schemes(aiq_model *m, const float *images, int32_t N, const uint8_t *schemes, int32_t S,
                            int32_t chunk, int32_t *top1_base, int32_t base_valid, float *logits,
                            int32_t *top1, int32_t *agree, void *workspace, size_t workspace_bytes,
                            void *hip_stream);

/*
 * aiq_eval_schemes for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * aiq_eval_schemes, minus the workspace: the library's own fixed array of
 * AIQ_NOALLOC_SCRATCH_BYTES takes its place (one copy per GPU, part of the loaded code, held until
 * the process ends; its address is looked up once per device, on the first call with that
 * device current).  The call allocates and frees nothing on the device, copies nothing from
 * host memory (the scheme table travels as kernel arguments) and does not wait for the stream.
 * It fits models whose scoring workspace is small: the LDS-resident ResNets need
 * S*L + 4*S*chunk bytes plus alignment; a model that runs layer by layer needs its activation
 * buffers and is refused.  aiq_eval_noalloc_workspace_bytes reports what a call would need
 * (needed) and what the array holds (available); either pointer may be NULL.
 * Every call on one GPU uses that GPU's one array, which keeps what the last call left there;
 * nothing in it has to start at zero (the scheme table and the per-chunk top-1 buffer are
 * written before they are read).  Calls that overlap on one GPU - two streams, two threads,
 * two models - race on it: serialise them.
 * Errors: as aiq_eval_schemes; WORKSPACE_TOO_SMALL when the need exceeds the array (nothing is
 * launched and no output is touched).
 */
#define AIQ_NOALLOC_SCRATCH_BYTES (2u << 20)
aiq_status aiq_eval_noalloc_workspace_bytes(const aiq_model *m, int32_t S, int32_t chunk, size_t *needed,
                                            size_t *available);
aiq_status aiq_eval_schemes_noalloc(aiq_model *m, const float *images, int32_t N, const uint8_t *schemes, int32_t S,
                                    int32_t chunk, int32_t *top1_base, int32_t base_valid, float *logits,
                                    int32_t *top1, int32_t *agree, void *hip_stream);

/*
 * aiq_eval_schemes with a shared forward prefix.  The schemes of one search step are all
 * derived from one scheme by changing a single layer (paper: Search Over Mixed-Precision
 * Schemes - greedy lowers one layer of the current scheme, coordinate descent varies one
 * layer with the others fixed), so up to that layer their forward passes equal the
 * current scheme's.  ref_scheme (HOST uint8 [L], read before the call returns) is that
 * scheme: it is run once per image, and scheme s resumes at its first layer whose width
 * differs from ref_scheme's.  Every output is bit for bit what aiq_eval_schemes returns
 * for the same arguments; schemes need not be related to ref_scheme (a scheme that differs
 * in its first layer simply runs whole).  The LDS-resident ResNet kernel hands its state over
 * through per-layer checkpoints of one workgroup's LDS; the layer-by-layer kernels keep the
 * reference pass's activations per layer and launch each layer only for the schemes that
 * have left the reference by then.  Models for which aiq_model_shares_prefix is 0 (none at
 * present) run every scheme whole.  Asynchronous on hip_stream like aiq_eval_schemes: the call
 * enqueues its work and does not wait for the stream.  workspace >= aiq_eval_shared_workspace_bytes(m, S, chunk); other
 * arguments, ownership and errors as for aiq_eval_schemes (ref_scheme NULL: INVALID_ARG).
 */
int32_t aiq_model_shares_prefix(const aiq_model *m); /* 1, 0, or -1 for a NULL model */
aiq_status aiq_eval_shared_workspace_bytes(const aiq_model *m, int32_t S, int32_t chunk, size_t *bytes);
aiq_status aiq_eval_schemes_shared(aiq_model *m, const float *images, int32_t N, const uint8_t *schemes, int32_t S,
                                   const uint8_t *ref_scheme, int32_t chunk, int32_t *top1_base,
                                   int32_t base_valid, float *logits, int32_t *top1, int32_t *agree,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Search drivers (paper: Approach - Problem Formulation for the loss, Search Over
 * Mixed-Precision Schemes for the two loops).  Host loops around aiq_eval_schemes: every
 * iteration scores all its candidate schemes in one scheme-batched call.
 *   loss(q) = -lambda * AI(q) + (1 - lambda) * AccLoss(q),  AccLoss = 100 * (1 - agree/N)
 * (percentage points), AI from aiq_layer_ai with params.batch.
 * greedy: start all-FP32; per iteration score every move "layer i -> lower width b in Q",
 *   accept the move with the smallest loss change if negative, else stop; at most
 *   max_iters iterations (0 = L).  only_fp32_layers = 1: a layer is a candidate only while
 *   it is still at bits[0].
 * coordinate descent: start all-FP32; for each layer in turn take argmin over Q with the
 *   other layers fixed (the current width wins ties); repeat sweeps until one changes
 *   nothing or max_iters sweeps (0 = 50) are done.
 * Ties between candidates go to the first in (layer ascending, width descending) order.
 * share_prefix = 1 scores each step through aiq_eval_schemes_shared with the current scheme
 * as the reference: same result, less work.
 *
 * params.bits: the alphabet Q, strictly descending, bits[0] = 32.  layers: the same records
 * the model was built from (for the AI model).  images: device fp32 [N][hin][win][cin].
 * workspace: device, >= aiq_search_workspace_bytes.  scheme_out: host uint8[L].
 * trace: host array of trace_cap entries or NULL; entry 0 is the all-FP32 start, then one
 * per accepted move (layer, bits, loss, AI, agreement after the move); *n_trace receives the
 * number of entries the search produced (it may exceed trace_cap; only trace_cap are stored).
 * Synchronous: returns when the search is finished.
 * Errors: INVALID_ARG, UNSUPPORTED_BITS, SHAPE_MISMATCH, WORKSPACE_TOO_SMALL, DEVICE_ERROR.
 */
typedef struct {
    double lambda;
    int32_t n_bits;
    uint8_t bits[8];
    int32_t batch;
    int32_t max_iters;
    int32_t only_fp32_layers;
    int32_t share_prefix; /* 1: the candidates of a step share the forward prefix of the current scheme */
} aiq_search_params;

typedef struct {
    int32_t layer; /* scheme slot changed by this step, -1 for the start entry */
    int32_t bits;
    int32_t agree;
    int32_t sweep; /* coordinate descent: sweep number (1-based), greedy: iteration */
    double loss, ai;
} aiq_search_step;

aiq_status aiq_search_workspace_bytes(const aiq_model *m, int32_t N, int32_t chunk, int32_t n_bits, size_t *bytes);
aiq_status aiq_search_greedy(aiq_model *m, const aiq_layer_desc *layers, int32_t n_layers, const float *images,
                             int32_t N, int32_t chunk, const aiq_search_params *params, void *workspace,
                             size_t workspace_bytes, void *hip_stream, uint8_t *scheme_out,
                             aiq_search_step *trace, int32_t trace_cap, int32_t *n_trace);
aiq_status aiq_search_coordinate_descent(aiq_model *m, const aiq_layer_desc *layers, int32_t n_layers,
                                         const float *images, int32_t N, int32_t chunk,
                                         const aiq_search_params *params, void *workspace, size_t workspace_bytes,
                                         void *hip_stream, uint8_t *scheme_out, aiq_search_step *trace,
                                         int32_t trace_cap, int32_t *n_trace);

/*
 * Per-layer sensitivity (paper: Analysis of Initial Hypotheses, Table 1 - the accuracy change when a
 * single layer is quantized to 8 or 4 bits and every other layer stays FP32).  Scores the
 * L * n_bits single-layer schemes in scheme-batched calls and returns their agreement counts:
 * agree_out[i * n_bits + k] = #{n : top-1 with only layer i at bits[k] == FP32 top-1}; the
 * sensitivity in percentage points is 100 * (1 - agree / N).
 * bits: host uint8[n_bits], each in {16,8,6,4,2}, 1 <= n_bits <= 5.  images: device fp32 [N][hin][win][cin].
 * workspace: device, >= aiq_sensitivity_workspace_bytes, 256-byte aligned.  agree_out: HOST int32 [L][n_bits].
 * Synchronous.  Errors: INVALID_ARG, UNSUPPORTED_BITS, WORKSPACE_TOO_SMALL, DEVICE_ERROR.
 */
aiq_status aiq_sensitivity_workspace_bytes(const aiq_model *m, int32_t N, int32_t chunk, int32_t n_bits, size_t *bytes);
aiq_status aiq_layer_sensitivity(aiq_model *m, const float *images, int32_t N, int32_t chunk, const uint8_t *bits,
                                 int32_t n_bits, void *workspace, size_t workspace_bytes, void *hip_stream,
                                 int32_t *agree_out);

/*
 * One scheme, every node's output (the forward pass of the scored model, paper: Introduction item (ii),
 * opened up for inspection): runs scheme (HOST uint8 [L]) on N images layer by layer and leaves node l's
 * output in node_out[l] (HOST array of aiq_model_nodes(m) DEVICE pointers, each fp32
 * [N][aiq_node_output_elems(m, l)], NHWC; the last node's are the logits).  Lets a caller check any
 * layer in isolation from the tensors it actually read, which is how results are compared where
 * activation rounding makes end-to-end outputs discontinuous.  m must run layer by layer
 * (AIQ_MODEL_LAYERWISE or AIQ_MODEL_ACT_QUANT; else UNSUPPORTED_LAYER).  workspace: device, 256-byte
 * aligned, >= aiq_eval_workspace_bytes(m, 1, N).  Asynchronous on hip_stream.
 * Errors: INVALID_ARG, UNSUPPORTED_BITS, UNSUPPORTED_LAYER, WORKSPACE_TOO_SMALL, DEVICE_ERROR.
 */
int32_t aiq_model_nodes(const aiq_model *m); /* -1 for NULL */
aiq_status aiq_node_output_elems(const aiq_model *m, int32_t node, size_t *elems);
aiq_status aiq_forward_nodes(aiq_model *m, const float *images, int32_t N, const uint8_t *scheme,
                             float *const *node_out, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Deployed inference of one scheme (paper: Implementation, experiment (3); Results, Analysis of
 * AIQ Throughput Effects - the model with the searched layers at low precision is run end to end
 * and its images/s compared with the FP32 model's).  The function computed is the scored one:
 * the forward pass with every layer's weights quantized to scheme[i] bits.  What changes is the
 * arithmetic of dense convolutions (groups = 1, not the network's first layer) of at most 8 bits:
 * their weights are integer codes times a per-channel scale, the codes are exact in bf16, and an
 * fp32 activation is exactly the sum of three bf16 terms, so the layer runs as three
 * v_mfma_f32_32x32x16_bf16 products with exact terms in place of one fp32 MFMA product, sixteen
 * times slower.  Results agree with aiq_eval_schemes to fp32 rounding (the accumulation order
 * differs and the scale multiplies the finished sum).  All other layers run on the fp32 kernels.
 *
 * aiq_deploy_create: m must outlive the deployment; scheme: host uint8[L].  A model that keeps its
 * activations in LDS (created without AIQ_MODEL_LAYERWISE: CIFAR-style ResNets, inverted-residual
 * blocks) is deployed on those kernels - the scheme runs as the single candidate of a scoring
 * call: for such models that is faster than any layer-by-layer path.  The whole-network ResNet
 * kernel stays in fp32 (bit-identical to aiq_eval_schemes, the FP32 model's own rate).  An
 * inverted-residual block whose expand or project layer carries at most 8 bits runs with
 * those 1x1 products taken from integer codes inside the block kernel (same three-term
 * arithmetic, v_mfma_f32_16x16x32_bf16 / 16x16x16_bf16; the depthwise layer, the hidden
 * tensor and a 16- or 32-bit 1x1 layer beside a low-bit one stay fp32), counted per layer in
 * aiq_deploy_code_layers; a last 1x1 layer of at
 * most 8 bits on 8x8 pixels that only the classifier reads (its epilogue forms the average pool)
 * runs from codes as well; results agree with aiq_eval_schemes to fp32 rounding.  Layer-by-layer integer-code layers need
 * AIQ_MODEL_LAYERWISE.  flags: AIQ_DEPLOY_FP32_MATRIX keeps every layer and block on the fp32
 * kernels (the same model without the bf16 path, for comparison; bit-identical to scoring).
 * Quantizes and packs the weights; allocates device memory (codes and scales), freed by
 * aiq_deploy_destroy.  Synchronous.  It fills weight-bank slots of m: do not overlap it with
 * other calls on m.  Errors: INVALID_ARG, UNSUPPORTED_BITS, UNSUPPORTED_LAYER, DEVICE_ERROR.
 *
 * aiq_deploy_forward: images: device fp32 [N][hin][win][cin].  logits: device fp32 [N][classes]
 * or NULL.  top1: device int32 [N], required.  workspace: device, 256-byte aligned, at least
 * aiq_deploy_workspace_bytes(d, chunk) bytes (activation buffers for `chunk` images at a time).
 * Asynchronous on hip_stream.  N = 0 is a valid no-op.
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, DEVICE_ERROR.
 *
 * Models created with AIQ_MODEL_ACT_QUANT: a dense convolution of at most 8 bits whose input tensor has
 * a multiple of 16 channels runs on the INT8 matrix pipe - its input is quantized to int8 codes with the
 * image's scale (the variant's own rule), the weights are stored as int8 codes, the products are summed
 * exactly in int32 and scaled once by s_w[c] * s_x[n]: the function is the one aiq_eval_schemes computes
 * for that model up to fp32 rounding of the final scaling.  Other layers run as in scoring.
 *
 * aiq_deploy_forward_nodes: like aiq_forward_nodes for a deployed scheme - every node's output on N
 * images in node_out[l] (HOST array of aiq_model_nodes(m) DEVICE pointers, fp32 [N][aiq_node_output_elems]),
 * which is how the layers of the activation variant are compared one by one.  workspace: device,
 * 256-byte aligned, >= aiq_deploy_workspace_bytes(d, N).  Not for models deployed on their LDS-resident
 * kernels (UNSUPPORTED_LAYER).  Asynchronous on hip_stream.
 * Errors: INVALID_ARG, UNSUPPORTED_LAYER, WORKSPACE_TOO_SMALL, DEVICE_ERROR.
 */
typedef struct aiq_deployed aiq_deployed; /* opaque */
enum { AIQ_DEPLOY_FP32_MATRIX = 1 };
aiq_status aiq_deploy_create(aiq_model *m, const uint8_t *scheme, uint32_t flags, aiq_deployed **out);
void aiq_deploy_destroy(aiq_deployed *d); /* NULL-safe */
/* Number of layers that run from their integer codes (bf16 or INT8 matrix pipe); -1 for NULL. */
int32_t aiq_deploy_code_layers(const aiq_deployed *d);
aiq_status aiq_deploy_workspace_bytes(const aiq_deployed *d, int32_t chunk, size_t *bytes);
aiq_status aiq_deploy_forward(aiq_deployed *d, const float *images, int32_t N, int32_t chunk, float *logits,
                              int32_t *top1, void *workspace, size_t workspace_bytes, void *hip_stream);
aiq_status aiq_deploy_forward_nodes(aiq_deployed *d, const float *images, int32_t N, float *const *node_out,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Per-kernel timing for roofline reports.  While enabled, aiq_eval_schemes and aiq_deploy_forward bracket
 * every launch with HIP events on the launch stream.  aiq_profile_read waits for the
 * recorded events, then returns for kernel class cls the number of launches, their
 * summed duration and the algorithmic FLOPs and bytes they covered, and clears the
 * record for that class.  Classes: 0 quantize, 1 dense convolution (MFMA),
 * 2 depthwise convolution, 3 classifier head, 4 agreement count, 5 LDS-resident whole network,
 * 6 LDS-resident inverted-residual block, 7 dense convolution on integer codes (bf16 MFMA,
 * deployed inference).
 */
enum { AIQ_K_QUANTIZE = 0, AIQ_K_CONV = 1, AIQ_K_DEPTHWISE = 2, AIQ_K_HEAD = 3, AIQ_K_AGREE = 4,
       AIQ_K_FUSED = 5, AIQ_K_MBCONV = 6, AIQ_K_CONV_CODES = 7, AIQ_K_CLASSES = 8 };
aiq_status aiq_profile_enable(aiq_model *m, int32_t on);
aiq_status aiq_profile_read(aiq_model *m, int32_t cls, int64_t *launches, double *total_ms, double *flops,
                            double *bytes);

#ifdef __cplusplus
}
#endif
#endif /* AIQ_H */
