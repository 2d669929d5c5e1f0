// Host side of libaiq.so: argument validation, the analytic arithmetic-intensity
// model, the per-call plan (which (layer, bit-width) bank slots to fill, which
// kernel configuration each layer gets) and the launch sequence.  Every step of the
// scored path itself runs in the kernels of the .hip files; this file holds no device code
// and compiles as plain C++ against the HIP runtime API.
#include "../../include/aiq.h"
#include "aiq_internal.h"

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

using namespace aiq;

namespace {

thread_local int32_t g_last_hip_error = 0;

inline bool hip_ok(hipError_t e)
{
    if (e == hipSuccess) return true;
    g_last_hip_error = (int32_t)e;
    (void)hipGetLastError(); // clear the sticky launch error
    return false;
}

#define AIQ_HIP(call)                               \
    do {                                            \
        if (!hip_ok(call)) return AIQ_DEVICE_ERROR; \
    } while (0)

inline int out_size(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

inline bool bits_supported(int b) { return bits_index(b) >= 0; }

struct ConvPlan {
    int nt, wave_px_split, R, G, regions_per_image, CB, CKC, RIN, LW, PS, cout_tiles, grid_y;
    size_t lds_bytes;
};

struct Node {
    aiq_layer_desc d;
    int hout, wout;
    int k;              // weights per output channel
    size_t out_elems;   // per image
    size_t in_elems;
    int layout;
    size_t bank_elems;  // elements of one bank slot (padded layout)
    float *w_plain = nullptr;
    float *bias = nullptr;
    float *bank[kNumBits] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    int buf = -1;       // activation buffer holding this node's output
    int job0 = -1;      // first quantize job (bits index 1) of this node, -1 if not a scheme layer
    ConvPlan plan;
    int mb_role = 0;    // 1: 1x1 expand heading an LDS-resident inverted-residual block, 2: its depthwise / project
    MbShape mb_shape{};
    double flops_per_image;      // 2 * multiply-adds
    double act_bytes_per_image;  // algorithmic: input + output (+ residual) activations
    bool pooled = false; // 1x1 layer feeding only the classifier: writes the per-image mean of its output instead
};

// Integer codes of a deployed inverted-residual block (at its expand node): null codes = the block runs on
// the fp32 block kernel.
struct MbCodes {
    uint16_t *codes_e = nullptr, *codes_p = nullptr;
    float *scale_e = nullptr, *scale_p = nullptr;
};

struct ProfRec {
    hipEvent_t start, stop;
    int cls;
    double flops, bytes;
};

} // namespace

struct aiq_model {
    std::vector<Node> nodes;
    int L = 0, classes = 0;
    int hin0 = 0, win0 = 0, cin0 = 0;
    int n_bufs = 0;
    size_t buf_elems = 0; // per scheme-image
    QuantJob *jobs_dev = nullptr;
    int32_t *block_job_dev = nullptr;
    int n_jobs = 0, n_quant_blocks = 0;
    std::vector<QuantJob> jobs_host;
    std::vector<void *> allocations;
    // LDS-resident path (CIFAR-style ResNets)
    bool fused = false;
    bool per_tensor = false;       // one quantization scale per layer instead of one per output channel
    bool act_quant = false;        // a layer at b bits also reads its input activations at b bits
    size_t aq_elems = 0;           // largest input tensor of a scheme layer (per image)
    float *aq_cur = nullptr;       // quantized-input buffer of the call in progress (part of its workspace)
    uint32_t *layer_amax = nullptr; // device: bit pattern of max |w| of every layer (per-tensor scales)
    int mb_blocks = 0;  // inverted-residual blocks run by the LDS-resident block kernel
    const MbCodes *mb_codes_cur = nullptr; // per node, of the deployed forward call in progress (else null)
    const uint8_t *mb_scheme_cur = nullptr; // host copy of that call's scheme
    std::vector<FusedOp> fused_ops;
    FusedOp *fused_ops_dev = nullptr;
    double fused_flops_per_image = 0.0;
    size_t fused_ckpt_floats = 0;     // checkpoint record of one image (0: prefix sharing not available)
    std::vector<int> slot_op;         // scheme slot -> op that carries it
    // layer-by-layer path: outputs of a reference pass kept per node (prefix sharing)
    std::vector<int> slot_node;       // scheme slot -> node that carries it
    std::vector<size_t> ref_node_off; // element offset of a node's output in one image's record
    size_t ref_act_elems = 0;         // elements of one image's record
    // profiling
    bool prof_on = false;
    std::vector<hipEvent_t> ev_pool;
    size_t ev_used = 0;
    std::vector<ProfRec> prof;
};

namespace {

aiq_status plan_conv(Node &nd)
{
    const aiq_layer_desc &d = nd.d;
    ConvPlan p{};
    p.cout_tiles = (d.cout + 15) / 16;
    p.CB = (d.cin + 15) / 16;
    // output-channel tiles per wavefront (nt) and wavefronts along output channels (wco): among
    // the pairs that waste at most 1/8 of the MFMAs on padding or idle wavefronts, take the one
    // covering the most output channels per workgroup (the staged input is reused most), then
    // the larger nt (each LDS read feeds more MFMAs)
    int wco = 1, best_cover = 0;
    p.nt = 1;
    for (int nt = 1; nt <= 4; ++nt)
        for (int w = 1; w <= 4; w *= 2) {
            const int per_wg = nt * w;
            const int waste = (p.cout_tiles + per_wg - 1) / per_wg * per_wg - p.cout_tiles;
            if (waste * 8 > p.cout_tiles) continue;
            if (per_wg > best_cover || (per_wg == best_cover && nt > p.nt)) {
                best_cover = per_wg;
                p.nt = nt;
                wco = w;
            }
        }
    p.wave_px_split = 4 / wco;
    p.grid_y = (p.cout_tiles + p.nt * wco - 1) / (p.nt * wco);
    const int region_px = 64 * p.wave_px_split;
    const int px_img = nd.hout * nd.wout;
    if (px_img >= region_px) {
        p.G = 1;
        p.R = region_px / nd.wout;
        if (p.R < 1) return AIQ_UNSUPPORTED_LAYER;
        p.R = std::min(p.R, nd.hout);
        p.regions_per_image = (nd.hout + p.R - 1) / p.R;
    } else {
        p.G = region_px / px_img;
        p.R = nd.hout;
        p.regions_per_image = 1;
    }
    const int cp = p.CB * 16;
    p.CKC = cp >= 64 ? 64 : (cp >= 32 ? 32 : 16);
    p.RIN = (p.R - 1) * d.stride + d.kh;
    p.LW = d.win + 2 * d.pad;
    // Channels staged per pass: as many as leave room for two workgroups per compute unit
    // (with one, its four wavefronts sit alone on their SIMDs and every staging phase and every
    // load latency idles the matrix pipe); a single workgroup only when even 16 channels need
    // more than half of the LDS.
    for (;;) {
        p.PS = p.CKC + 4;
        p.lds_bytes = sizeof(float) * (size_t)p.G * p.RIN * p.LW * p.PS;
        if (p.lds_bytes <= 76 * 1024) break;
        if (p.CKC == 16) {
            if (p.lds_bytes <= 152 * 1024) break;
            return AIQ_UNSUPPORTED_LAYER;
        }
        p.CKC /= 2;
    }
    nd.plan = p;
    return AIQ_OK;
}

// Tiling of the integer-code convolution (conv_codes_kernel): output-channel tiles are 32 wide,
// a wavefront holds one or two of them for 64 pixels.  Per pass of CKC channels the LDS holds the
// region's input rows (per pixel three bf16 planes of CKC channels, each padded by 16 bytes) and
// the codes of the workgroup's tiles for those channels; a thread stages at most kCodeStageItems
// activation items and kCodeStageChunks code chunks per pass.  False if no tiling fits.
struct CodePlan {
    int nt, mt, wave_px_split, R, G, regions_per_image, CB, CKC, RIN, LW, PSU, cout_tiles, grid_y, code_off, stage_items;
    size_t lds_bytes;
};

bool plan_code_conv(const Node &nd, CodePlan &p)
{
    const aiq_layer_desc &d = nd.d;
    const int T = d.kh * d.kw;
    // Preferred split of the four wavefronts as for the fp32 kernel (most output channels per
    // workgroup at no more than 1/8 of the MFMAs wasted); if the region that goes with it does
    // not fit, more wavefronts go along the output channels and the region shrinks.  A wavefront
    // with a single output tile takes one pixel tile instead of two where four such workgroups fit a
    // compute unit.
    for (int wco_min = 1; wco_min <= 4; wco_min *= 2) {
        const int cout_tiles = (d.cout + 31) / 32;
        int nt_sel = 1, wco = 0, best_cover = 0;
        for (int nt = 1; nt <= 2; ++nt)
            for (int w = wco_min; w <= 4; w *= 2) {
                const int per_wg = nt * w;
                const bool smallest = nt == 1 && w == wco_min;
                const int waste = (cout_tiles + per_wg - 1) / per_wg * per_wg - cout_tiles;
                if (!smallest && (waste * 8 > cout_tiles || per_wg * T * 64 > kCodeStageChunks * 256)) continue;
                if (per_wg > best_cover || (per_wg == best_cover && nt > nt_sel)) {
                    best_cover = per_wg;
                    nt_sel = nt;
                    wco = w;
                }
            }
        for (int mt = nt_sel == 1 ? 1 : 2; mt <= 2; ++mt)
        for (int ki = kCodeStageItems; ki <= 2 * kCodeStageItems; ki += kCodeStageItems) {
            p = CodePlan{};
            p.stage_items = ki;
            p.mt = mt;
            p.nt = nt_sel;
            p.cout_tiles = cout_tiles;
            p.CB = (d.cin + 15) / 16;
            p.wave_px_split = 4 / wco;
            p.grid_y = (p.cout_tiles + p.nt * wco - 1) / (p.nt * wco);
            const int region_px = 32 * mt * p.wave_px_split;
            const int px_img = nd.hout * nd.wout;
            if (px_img >= region_px) {
                p.G = 1;
                p.R = std::min(region_px / nd.wout, nd.hout);
                if (p.R < 1) continue;
                p.regions_per_image = (nd.hout + p.R - 1) / p.R;
            } else {
                p.G = region_px / px_img;
                p.R = nd.hout;
                p.regions_per_image = 1;
            }
            const int cp = p.CB * 16;
            p.CKC = cp >= 64 ? 64 : (cp >= 32 ? 32 : 16);
            p.RIN = (p.R - 1) * d.stride + d.kh;
            p.LW = d.win + 2 * d.pad;
            // three workgroups per compute unit where the region allows it (the kernel variants with
            // the longer staging list or four pixel tiles need more registers: two)
            const size_t lds_limit = (size_t)(ki != kCodeStageItems ? 80 : (mt == 1 ? 40 : 53)) * 1024;
            bool fits;
            for (;;) {
                p.PSU = p.CKC / 8;
                p.code_off = p.G * p.RIN * p.LW * 3 * p.PSU;
                const int chunks = p.nt * wco * T * (p.CKC / 16) * 64;
                // the epilogue lays every wavefront's pixels, 32 at a time, x 32 * nt channels out in LDS
                p.lds_bytes = std::max((size_t)16 * (p.code_off + chunks), (size_t)4 * 32 * 32 * p.nt * sizeof(float));
                fits = p.G * p.RIN * p.LW * (p.CKC / 8) <= ki * 256 && chunks <= kCodeStageChunks * 256;
                if ((fits && p.lds_bytes <= lds_limit) || p.CKC == 16) break;
                p.CKC /= 2;
            }
            if (fits && p.lds_bytes <= (mt == 1 ? lds_limit : (size_t)160 * 1024)) return true;
        }
    }
    return false;
}

// Tiling of the int8 convolution (conv_i8_kernel): a wavefront holds 64 pixels x one or two
// output-channel tiles of 32; all output channels go to one workgroup where four wavefronts can hold
// them, so that the region's activations are staged once.  Per pass the LDS holds the region's input
// rows (32 or 64 channels of int8 per pixel + 16 bytes of padding) and the weight codes of the
// workgroup's tiles for those channels.  False if no tiling fits.
struct I8Plan {
    int nt, wave_px_split, R, G, regions_per_image, CBK, CKB, RIN, LW, PSB, cout_tiles, tiles_per_wg, grid_y, code_off;
    size_t lds_bytes;
};

bool plan_i8_conv(const Node &nd, I8Plan &p)
{
    const aiq_layer_desc &d = nd.d;
    if (d.cin % 16 != 0 || d.cout % 4 != 0) return false;
    const int T = d.kh * d.kw;
    p = I8Plan{};
    p.cout_tiles = (d.cout + 31) / 32;
    p.nt = p.cout_tiles >= 2 ? 2 : 1;
    const int groups = (p.cout_tiles + p.nt - 1) / p.nt; // wavefronts along the output channels, if all fit
    // first choice: two workgroups or more per compute unit; regions whose input rows are long (stride 2
    // at 32x32) get what one workgroup per unit can hold
    for (size_t lds_limit : {(size_t)79 * 1024, (size_t)159 * 1024})
    for (int wco = groups >= 4 ? 4 : (groups >= 2 ? 2 : 1); wco >= 1; wco /= 2) {
        p.wave_px_split = 4 / wco;
        p.tiles_per_wg = p.nt * wco;
        p.grid_y = (p.cout_tiles + p.tiles_per_wg - 1) / p.tiles_per_wg;
        const int region_px = 64 * p.wave_px_split;
        const int px_img = nd.hout * nd.wout;
        if (px_img >= region_px) {
            p.G = 1;
            p.R = std::min(region_px / nd.wout, nd.hout);
            if (p.R < 1) continue;
            p.regions_per_image = (nd.hout + p.R - 1) / p.R;
        } else {
            p.G = std::min(region_px / px_img, 64); // the epilogue keeps one activation scale per lane
            p.R = nd.hout;
            p.regions_per_image = 1;
        }
        p.CBK = (d.cin + 31) / 32;
        p.RIN = (p.R - 1) * d.stride + d.kh;
        p.LW = d.win + 2 * d.pad;
        for (p.CKB = std::min(p.CBK, 2); p.CKB >= 1; --p.CKB) {
            p.PSB = 32 * p.CKB + 16;
            // the epilogue's tiles (4 wavefronts x 32 pixels x 32 * nt channels) lie over the activations,
            // never over the weight codes, which stay for the workgroup's next region
            p.code_off = (int)std::max<size_t>((size_t)(p.G * p.RIN * p.LW * p.PSB + 255) / 256 * 256,
                                               (size_t)4 * 32 * 32 * p.nt * sizeof(float));
            p.lds_bytes = (size_t)p.code_off + (size_t)p.tiles_per_wg * T * p.CKB * 1024;
            if (p.lds_bytes <= lds_limit) return true;
        }
    }
    return false;
}

// Recognises stem -> basic blocks (identity, or stride-2 with a 1x1 projection) -> classifier
// with 16/32/64 channels at 32/16/8 pixels, and lays the tensors out in two LDS regions:
// a block reads its input from one region, writes the intermediate to the other and the
// block output back in place.  Returns false if the graph has any other shape.
bool plan_fused(const std::vector<Node> &nodes, std::vector<FusedOp> &ops)
{
    const int n = (int)nodes.size();
    auto is_conv = [&](int i, int k, int stride, int cin, int cout, int hin) {
        const aiq_layer_desc &d = nodes[i].d;
        return d.kind == 0 && d.kh == k && d.kw == k && d.stride == stride && d.cin == cin && d.cout == cout &&
               d.hin == hin && d.win == hin;
    };
    if (n < 2 || !is_conv(0, 3, 1, 3, 16, 32) || nodes[0].d.residual >= 0) return false;
    const int R[2] = {0, kFusedRegionFloats};
    auto mk = [&](int type, int node, int src, int dst, int res, int res_padded, int zero_ring) {
        FusedOp op{};
        op.type = type;
        op.slot = nodes[node].d.scheme_slot;
        op.act = nodes[node].d.act;
        op.src_off = src;
        op.dst_off = dst;
        op.res_off = res;
        op.res_padded = res_padded;
        op.zero_ring = zero_ring;
        op.classes = nodes[node].d.cout;
        ops.push_back(op);
    };
    ops.clear();
    int reg = 0; // region holding the current block input
    mk(kOpStem, 0, R[1], R[0], -1, 0, 0);
    int cur = 0, c = 16, h = 32, i = 1;
    while (i < n && nodes[i].d.kind != 2) {
        const aiq_layer_desc &c1 = nodes[i].d;
        if (c1.input != cur || c1.residual >= 0) return false;
        const int ctype = c == 16 ? kOpC16 : (c == 32 ? kOpC32 : kOpC64);
        if (is_conv(i, 3, 1, c, c, h)) {
            if (i + 1 >= n || !is_conv(i + 1, 3, 1, c, c, h)) return false;
            const aiq_layer_desc &c2 = nodes[i + 1].d;
            if (c2.input != i || c2.residual != cur) return false;
            mk(ctype, i, R[reg], R[1 - reg], -1, 0, 0);
            mk(ctype, i + 1, R[1 - reg], R[reg], R[reg], 1, 0);
            cur = i + 1;
            i += 2;
        } else if (c < 64 && is_conv(i, 3, 2, c, 2 * c, h)) {
            if (i + 2 >= n || !is_conv(i + 1, 1, 2, c, 2 * c, h) || !is_conv(i + 2, 3, 1, 2 * c, 2 * c, h / 2))
                return false;
            const aiq_layer_desc &sc = nodes[i + 1].d, &c2 = nodes[i + 2].d;
            if (sc.input != cur || sc.residual >= 0 || c2.input != i || c2.residual != i + 1) return false;
            const int ho = h / 2, co = 2 * c;
            const int t_floats = (co / 4) * (ho + 2) * (ho + 2) * 4;
            if (t_floats + co * ho * ho > kFusedRegionFloats) return false;
            mk(c == 16 ? kOpT16_32 : kOpT32_64, i, R[reg], R[1 - reg], -1, 0, 1);
            mk(c == 16 ? kOpS16_32 : kOpS32_64, i + 1, R[reg], R[1 - reg] + t_floats, -1, 0, 0);
            mk(co == 32 ? kOpC32 : kOpC64, i + 2, R[1 - reg], R[reg], R[1 - reg] + t_floats, 0, 1);
            cur = i + 2;
            c = co;
            h = ho;
            i += 3;
        } else {
            return false;
        }
    }
    if (i != n - 1) return false;
    const aiq_layer_desc &fc = nodes[i].d;
    if (fc.kind != 2 || fc.input != cur || fc.cin != 64 || c != 64 || h != 8 || fc.hin != 8 || fc.win != 8) return false;
    mk(kOpHead, i, R[reg], R[1 - reg], -1, 0, 0);
    return true;
}

// Checkpoints for prefix sharing.  A pass that resumes at op o needs every LDS float that op o
// or a later op reads before writing it - tensors still live and the zero borders of the
// regions later ops write into.  Per region that is covered by the prefix that reaches the
// furthest read of any op >= o, which is what the reference pass stores before op o.  Only
// ops that carry a scheme layer can be the first difference between two schemes.  Returns
// the floats of one image's record, 0 if the scheme slots do not follow the op order.
size_t plan_fused_checkpoints(std::vector<FusedOp> &ops, int L, std::vector<int> &slot_op)
{
    static const int in_floats[9] = {34 * 34 * 4, 18496, 18496, 18496, 10368, 10368, 10368, 6400, 6400};
    static const int res_unpadded[9] = {0, 0, 0, 0, 32 * 16 * 16, 0, 0, 64 * 8 * 8, 0};
    const int n = (int)ops.size();
    slot_op.assign(L, -1);
    int last = -1;
    for (int o = 0; o < n; ++o) {
        if (ops[o].slot < 0) continue;
        if (ops[o].slot <= last || ops[o].slot >= L) return 0;
        last = ops[o].slot;
        slot_op[last] = o;
    }
    for (int v : slot_op)
        if (v < 0) return 0;
    int ext[2] = {0, 0};
    std::vector<int> e0(n), e1(n);
    for (int o = n - 1; o >= 0; --o) {
        auto cover = [&](int off, int len) {
            const int r = off >= kFusedRegionFloats ? 1 : 0;
            ext[r] = std::max(ext[r], off + len - r * kFusedRegionFloats);
        };
        cover(ops[o].src_off, in_floats[ops[o].type]);
        if (ops[o].res_off >= 0)
            cover(ops[o].res_off, ops[o].res_padded ? in_floats[ops[o].type] : res_unpadded[ops[o].type]);
        e0[o] = (ext[0] + 3) & ~3;
        e1[o] = (ext[1] + 3) & ~3;
    }
    size_t total = 0;
    for (int o = 0; o < n; ++o) {
        ops[o].ck_off = 0;
        ops[o].ck_ext[0] = ops[o].ck_ext[1] = 0;
        if (o == 0 || ops[o].slot < 0) continue;
        if (e0[o] > kFusedRegionFloats || e1[o] > kFusedRegionFloats) return 0;
        ops[o].ck_off = (int32_t)total;
        ops[o].ck_ext[0] = e0[o];
        ops[o].ck_ext[1] = e1[o];
        total += (size_t)e0[o] + e1[o];
    }
    return total;
}

// Marks every expand -> depthwise -> project triple whose shape the LDS-resident block kernel
// covers and whose two hidden tensors have no other reader.  Returns the number of blocks.
int plan_mbconv(std::vector<Node> &nodes)
{
    const int n = (int)nodes.size();
    std::vector<int> readers(n, 0);
    for (const Node &nd : nodes) {
        if (nd.d.input >= 0) ++readers[nd.d.input];
        if (nd.d.residual >= 0) ++readers[nd.d.residual];
    }
    int blocks = 0;
    for (int i = 0; i + 2 < n; ++i) {
        const aiq_layer_desc &e = nodes[i].d, &d = nodes[i + 1].d, &p = nodes[i + 2].d;
        if (e.kind != 0 || e.kh != 1 || e.stride != 1 || e.input < 0 || e.residual >= 0 || e.hin != e.win) continue;
        if (d.kind != 1 || d.input != i || readers[i] != 1) continue;
        if (p.kind != 0 || p.kh != 1 || p.stride != 1 || p.input != i + 1 || readers[i + 1] != 1) continue;
        if (p.residual >= 0 && p.residual != e.input) continue;
        MbShape sh{e.cin, e.cout, p.cout, e.hin, d.stride, p.residual >= 0 ? 1 : 0};
        if (!mbconv_supported(sh)) continue;
        nodes[i].mb_role = 1;
        nodes[i].mb_shape = sh;
        nodes[i + 1].mb_role = nodes[i + 2].mb_role = 2;
        ++blocks;
        i += 2;
    }
    return blocks;
}

aiq_status validate_graph(const aiq_layer_desc *layers, int n_layers)
{
    if (layers[0].input != -1) return AIQ_SHAPE_MISMATCH;
    for (int l = 0; l < n_layers; ++l) {
        const aiq_layer_desc &d = layers[l];
        if (d.kind < 0 || d.kind > 2) return AIQ_UNSUPPORTED_LAYER;
        if (d.cin <= 0 || d.cout <= 0 || d.hin <= 0 || d.win <= 0) return AIQ_INVALID_ARG;
        if (d.input < -1 || d.input >= l || d.residual < -1 || d.residual >= l) return AIQ_SHAPE_MISMATCH;
        if (d.act < 0 || d.act > 2) return AIQ_INVALID_ARG;
        if (d.kind == 2) {
            if (l != n_layers - 1) return AIQ_UNSUPPORTED_LAYER;
            if (d.cout > 64 || d.residual >= 0 || d.input < 0 || d.act != 0) return AIQ_UNSUPPORTED_LAYER;
        } else {
            const bool k3 = d.kh == 3 && d.kw == 3 && d.pad == 1;
            const bool k1 = d.kh == 1 && d.kw == 1 && d.pad == 0;
            if (!(k3 || k1) || (d.stride != 1 && d.stride != 2)) return AIQ_UNSUPPORTED_LAYER;
            if (d.kind == 1 && (!k3 || d.cin != d.cout || (d.cin & 3) || d.residual >= 0 || d.input < 0))
                return AIQ_UNSUPPORTED_LAYER;
            if (d.kind == 0 && (d.cout & 3)) return AIQ_UNSUPPORTED_LAYER;
            if (d.kind == 0 && d.input >= 0 && (d.cin & 3)) return AIQ_UNSUPPORTED_LAYER;
        }
        if (d.input >= 0) {
            const aiq_layer_desc &p = layers[d.input];
            if (p.kind == 2) return AIQ_SHAPE_MISMATCH;
            if (out_size(p.hin, p.kh, p.stride, p.pad) != d.hin || out_size(p.win, p.kw, p.stride, p.pad) != d.win ||
                p.cout != d.cin)
                return AIQ_SHAPE_MISMATCH;
        } else if (d.hin != layers[0].hin || d.win != layers[0].win || d.cin != layers[0].cin) {
            return AIQ_SHAPE_MISMATCH;
        }
        if (d.residual >= 0) {
            const aiq_layer_desc &r = layers[d.residual];
            if (r.kind == 2 || r.cout != d.cout ||
                out_size(r.hin, r.kh, r.stride, r.pad) != out_size(d.hin, d.kh, d.stride, d.pad) ||
                out_size(r.win, r.kw, r.stride, r.pad) != out_size(d.win, d.kw, d.stride, d.pad))
                return AIQ_SHAPE_MISMATCH;
        }
    }
    if (layers[n_layers - 1].kind != 2) return AIQ_UNSUPPORTED_LAYER;
    // scheme slots must be exactly 0..L-1, each used once
    int L = 0;
    for (int l = 0; l < n_layers; ++l) L = std::max(L, layers[l].scheme_slot + 1);
    std::vector<int> seen(L, 0);
    for (int l = 0; l < n_layers; ++l) {
        const int sl = layers[l].scheme_slot;
        if (sl < -1) return AIQ_INVALID_ARG;
        if (sl >= 0 && seen[sl]++) return AIQ_SHAPE_MISMATCH;
    }
    for (int i = 0; i < L; ++i)
        if (!seen[i]) return AIQ_SHAPE_MISMATCH;
    return AIQ_OK;
}

template <typename T>
aiq_status dev_alloc(aiq_model *m, T **p, size_t n)
{
    void *q = nullptr;
    AIQ_HIP(hipMalloc(&q, std::max<size_t>(n * sizeof(T), 256)));
    m->allocations.push_back(q);
    *p = reinterpret_cast<T *>(q);
    return AIQ_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct WorkspaceLayout {
    size_t schemes_off, top1_off, act_off, aq_off, amax_off, total;
    size_t buf_stride; // bytes of one activation buffer
    // prefix sharing only (0 otherwise): reference scheme, first op per scheme, the reference
    // pass's top-1, the checkpoint records of one chunk
    size_t ref_off, first_op_off, ref_top1_off, sorted_off, ckpt_off;
};

WorkspaceLayout workspace_layout(const aiq_model *m, int S, int chunk, bool shared = false)
{
    WorkspaceLayout w{};
    size_t off = 0;
    w.schemes_off = off;
    off = align_up(off + (size_t)std::max(S, 1) * std::max(m->L, 1), 256);
    w.top1_off = off;
    off = align_up(off + sizeof(int32_t) * (size_t)std::max(S, 1) * chunk, 256);
    w.act_off = off;
    w.buf_stride = align_up(sizeof(float) * m->buf_elems * (size_t)(S + 1) * chunk, 256);
    off += w.buf_stride * m->n_bufs;
    w.aq_off = off; // activation fake-quantization: the quantized copy of the input of the node being launched
    // (+ one float per image: the deployed int8 layers keep the images' activation scales behind their codes)
    if (m->act_quant)
        off += align_up(sizeof(float) * m->aq_elems * (size_t)(S + 1) * chunk, 256) +
               align_up(sizeof(float) * (size_t)(S + 1) * chunk, 256);
    // deployed int8 layers: per node and image, the absolute maximum of the node's output (float bit patterns)
    w.amax_off = off;
    if (m->act_quant) off += align_up(sizeof(uint32_t) * m->nodes.size() * (size_t)chunk, 256);
    if (shared && (m->fused_ckpt_floats > 0 || !m->fused)) {
        off = align_up(off, 256);
        w.ref_off = off;
        off = align_up(off + (size_t)std::max(m->L, 1), 256);
        w.first_op_off = off; // layer-by-layer path: the row map, S + 2 entries
        off = align_up(off + sizeof(int32_t) * (size_t)(S + 2), 256);
        w.ref_top1_off = off;
        off = align_up(off + sizeof(int32_t) * (size_t)chunk, 256);
        w.sorted_off = off;
        if (!m->fused) off = align_up(off + (size_t)(S + 1) * std::max(m->L, 1), 256);
        w.ckpt_off = off; // layer-by-layer path: the reference pass's activations
        off += align_up(sizeof(float) * (m->fused ? m->fused_ckpt_floats : m->ref_act_elems) * (size_t)chunk, 256);
    }
    w.total = off;
    return w;
}

// Brackets one launch with events when profiling is on.
struct ProfScope {
    aiq_model *m;
    hipStream_t st;
    ProfRec rec{};
    bool live = false;
    ProfScope(aiq_model *m_, hipStream_t st_, int cls, double flops, double bytes) : m(m_), st(st_)
    {
        if (!m->prof_on || m->ev_used + 2 > m->ev_pool.size()) return;
        rec.start = m->ev_pool[m->ev_used++];
        rec.stop = m->ev_pool[m->ev_used++];
        rec.cls = cls;
        rec.flops = flops;
        rec.bytes = bytes;
        live = hipEventRecord(rec.start, st) == hipSuccess;
    }
    ~ProfScope()
    {
        if (live && hipEventRecord(rec.stop, st) == hipSuccess) m->prof.push_back(rec);
    }
};

} // namespace

extern "C" {

const char *aiq_status_str(aiq_status st)
{
    switch (st) {
    case AIQ_OK: return "ok";
    case AIQ_INVALID_ARG: return "invalid argument";
    case AIQ_UNSUPPORTED_BITS: return "unsupported bit-width";
    case AIQ_SHAPE_MISMATCH: return "shape mismatch";
    case AIQ_WORKSPACE_TOO_SMALL: return "workspace too small";
    case AIQ_DEVICE_ERROR: return "device error";
    case AIQ_UNSUPPORTED_LAYER: return "unsupported layer";
    default: return "unknown status";
    }
}

int32_t aiq_last_hip_error(void) { return g_last_hip_error; }

aiq_status aiq_layer_ai(const aiq_layer_desc *layers, int32_t n_layers, const uint8_t *scheme, int32_t L,
                        int32_t batch, double *flops_per_layer, double *bytes_per_layer, double *global_ai)
{
    return aiq_layer_ai_ex(layers, n_layers, scheme, L, batch, 0, flops_per_layer, bytes_per_layer, global_ai);
}

aiq_status aiq_layer_ai_ex(const aiq_layer_desc *layers, int32_t n_layers, const uint8_t *scheme, int32_t L,
                           int32_t batch, int32_t act_quant, double *flops_per_layer, double *bytes_per_layer,
                           double *global_ai)
{
    if (!layers || n_layers <= 0 || batch < 1 || !global_ai || L < 0) return AIQ_INVALID_ARG;
    if (act_quant != 0 && act_quant != 1) return AIQ_INVALID_ARG;
    // validate everything before writing anything
    for (int l = 0; l < n_layers; ++l) {
        const aiq_layer_desc &d = layers[l];
        if (d.kind < 0 || d.kind > 2) return AIQ_UNSUPPORTED_LAYER;
        if (d.scheme_slot >= 0) {
            if (!scheme) return AIQ_INVALID_ARG;
            if (d.scheme_slot >= L) return AIQ_SHAPE_MISMATCH;
            if (!bits_supported(scheme[d.scheme_slot])) return AIQ_UNSUPPORTED_BITS;
        }
    }
    double total_flops = 0.0, total_bytes = 0.0;
    for (int l = 0; l < n_layers; ++l) {
        const aiq_layer_desc &d = layers[l];
        const double bits = d.scheme_slot >= 0 ? (double)scheme[d.scheme_slot] : 32.0;
        double weights, macs, in_e, out_e;
        if (d.kind == 2) {
            weights = (double)d.cin * d.cout;
            macs = weights;
            in_e = d.cin;
            out_e = d.cout;
        } else {
            const double ho = out_size(d.hin, d.kh, d.stride, d.pad), wo = out_size(d.win, d.kw, d.stride, d.pad);
            weights = (double)d.cout * (d.kind == 1 ? 1 : d.cin) * d.kh * d.kw;
            macs = weights * ho * wo;
            in_e = (double)d.hin * d.win * d.cin;
            out_e = ho * wo * d.cout;
        }
        const double f = 2.0 * batch * macs;
        const double in_bytes = act_quant ? in_e * bits / 8.0 : 4.0 * in_e;
        const double b = weights * bits / 8.0 + batch * (in_bytes + 4.0 * out_e);
        if (flops_per_layer) flops_per_layer[l] = f;
        if (bytes_per_layer) bytes_per_layer[l] = b;
        total_flops += f;
        total_bytes += b;
    }
    *global_ai = total_flops / total_bytes;
    return AIQ_OK;
}

aiq_status aiq_quantize_weights(const float *w, int32_t cout, int32_t k, int32_t bits, float *w_dq, float *scales,
                                int32_t *codes, void *hip_stream)
{
    if (cout < 0 || k < 0) return AIQ_INVALID_ARG;
    if (!bits_supported(bits)) return AIQ_UNSUPPORTED_BITS;
    if (cout == 0) return AIQ_OK;
    if (!scales || (k > 0 && (!w || !w_dq))) return AIQ_INVALID_ARG;
    QuantJob j{};
    j.w = w;
    j.out = w_dq;
    j.scales = scales;
    j.codes = bits == 32 ? nullptr : codes;
    j.cout = cout;
    j.k = k;
    j.bits = bits;
    j.layout = kLayoutPlain;
    j.taps = 1;
    j.cblocks = 1;
    AIQ_HIP(launch_quantize_single(j, (hipStream_t)hip_stream));
    return AIQ_OK;
}

aiq_status aiq_quantize_weights_ex(const float *w, int32_t cout, int32_t k, int32_t bits, int32_t per_tensor,
                                   float *w_dq, float *scales, int32_t *codes, void *scratch, void *hip_stream)
{
    if (per_tensor != 0 && per_tensor != 1) return AIQ_INVALID_ARG;
    if (!per_tensor) return aiq_quantize_weights(w, cout, k, bits, w_dq, scales, codes, hip_stream);
    if (cout < 0 || k < 0) return AIQ_INVALID_ARG;
    if (!bits_supported(bits)) return AIQ_UNSUPPORTED_BITS;
    if (cout == 0) return AIQ_OK;
    if (!scales || !scratch || (reinterpret_cast<uintptr_t>(scratch) & 3) || (k > 0 && (!w || !w_dq)))
        return AIQ_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    uint32_t *amax = static_cast<uint32_t *>(scratch);
    if (bits != 32) AIQ_HIP(launch_tensor_absmax(w, (size_t)cout * k, amax, st));
    QuantJob j{};
    j.w = w;
    j.out = w_dq;
    j.scales = scales;
    j.codes = bits == 32 ? nullptr : codes;
    j.cout = cout;
    j.k = k;
    j.bits = bits;
    j.layout = kLayoutPlain;
    j.taps = 1;
    j.cblocks = 1;
    j.tensor_amax = bits == 32 ? nullptr : amax;
    AIQ_HIP(launch_quantize_single(j, st));
    return AIQ_OK;
}

int32_t aiq_model_scheme_layers(const aiq_model *m) { return m ? m->L : -1; }
int32_t aiq_model_classes(const aiq_model *m) { return m ? m->classes : -1; }

void aiq_model_destroy(aiq_model *m)
{
    if (!m) return;
    for (hipEvent_t e : m->ev_pool) (void)hipEventDestroy(e);
    for (void *p : m->allocations) (void)hipFree(p);
    delete m;
}

int32_t aiq_model_is_lds_resident(const aiq_model *m) { return m ? (m->fused ? 1 : 0) : -1; }
int32_t aiq_model_lds_resident_blocks(const aiq_model *m) { return m ? m->mb_blocks : -1; }

aiq_status aiq_model_create(const aiq_layer_desc *layers, int32_t n_layers, const float *const *w_host,
                            const float *const *bias_host, aiq_model **out)
{
    return aiq_model_create_ex(layers, n_layers, w_host, bias_host, 0u, out);
}

aiq_status aiq_model_create_ex(const aiq_layer_desc *layers, int32_t n_layers, const float *const *w_host,
                               const float *const *bias_host, uint32_t flags, aiq_model **out)
{
    if (out) *out = nullptr;
    if (flags & ~(uint32_t)(AIQ_MODEL_LAYERWISE | AIQ_MODEL_PER_TENSOR | AIQ_MODEL_ACT_QUANT)) return AIQ_INVALID_ARG;
    if (flags & AIQ_MODEL_ACT_QUANT) flags |= AIQ_MODEL_LAYERWISE; // the quantized copy of a layer's input lives in memory
    if (!layers || n_layers <= 0 || !w_host || !bias_host || !out) return AIQ_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l)
        if (!w_host[l] || !bias_host[l]) return AIQ_INVALID_ARG;
    aiq_status st = validate_graph(layers, n_layers);
    if (st != AIQ_OK) return st;

    aiq_model *m = new (std::nothrow) aiq_model();
    if (!m) return AIQ_INVALID_ARG;
    m->hin0 = layers[0].hin;
    m->win0 = layers[0].win;
    m->cin0 = layers[0].cin;
    m->classes = layers[n_layers - 1].cout;
    m->nodes.resize(n_layers);
    for (int l = 0; l < n_layers; ++l) {
        Node &nd = m->nodes[l];
        nd.d = layers[l];
        const aiq_layer_desc &d = nd.d;
        m->L = std::max(m->L, d.scheme_slot + 1);
        if (d.kind == 2) {
            nd.hout = nd.wout = 1;
            nd.k = d.cin;
            nd.out_elems = d.cout;
            nd.in_elems = (size_t)d.hin * d.win * d.cin;
            nd.layout = kLayoutPlain;
            nd.bank_elems = (size_t)d.cout * d.cin;
            nd.flops_per_image = 2.0 * d.cin * d.cout + 2.0 * d.hin * d.win * d.cin;
            nd.act_bytes_per_image = 4.0 * nd.in_elems;
        } else {
            nd.hout = out_size(d.hin, d.kh, d.stride, d.pad);
            nd.wout = out_size(d.win, d.kw, d.stride, d.pad);
            nd.out_elems = (size_t)nd.hout * nd.wout * d.cout;
            nd.in_elems = (size_t)d.hin * d.win * d.cin;
            if (d.kind == 1) {
                nd.k = d.kh * d.kw;
                nd.layout = kLayoutTapMajor;
                nd.bank_elems = (size_t)d.cout * nd.k;
            } else {
                nd.k = d.cin * d.kh * d.kw;
                nd.layout = kLayoutMfma;
                nd.bank_elems = (size_t)((d.cout + 15) / 16) * 16 * d.kh * d.kw * ((d.cin + 15) / 16) * 16;
                if (d.cin <= 4 && d.kh == 3 && d.kw == 3 && d.stride == 1 && d.pad == 1 && d.residual < 0) {
                    // network stem: the input channel is the MFMA's k index (conv_stem_kernel)
                    nd.layout = kLayoutStem;
                    nd.bank_elems = (size_t)((d.cout + 15) / 16) * 9 * 64;
                }
                st = plan_conv(nd);
                if (st != AIQ_OK) {
                    delete m;
                    return st;
                }
            }
            nd.flops_per_image = 2.0 * (double)nd.out_elems * nd.k;
            nd.act_bytes_per_image = 4.0 * ((double)nd.in_elems * (d.stride == 1 ? 1.0 : 1.0) + nd.out_elems +
                                            (d.residual >= 0 ? nd.out_elems : 0));
        }
    }

    if (!(flags & AIQ_MODEL_LAYERWISE))
        m->fused = plan_fused(m->nodes, m->fused_ops) && m->fused_ops.size() <= (size_t)kFusedMaxOps;
    if (m->fused) {
        Node &stem = m->nodes[0];
        stem.layout = kLayoutStem;
        stem.bank_elems = (size_t)((stem.d.cout + 15) / 16) * 9 * 64;
        // stride-1 3x3 layers read their weights one tap column at a time
        for (size_t o = 0; o < m->fused_ops.size(); ++o) {
            const int t = m->fused_ops[o].type;
            if (t == kOpC16 || t == kOpC32 || t == kOpC64) m->nodes[o].layout = kLayoutMfmaKx;
        }
        for (const Node &nd : m->nodes) m->fused_flops_per_image += nd.flops_per_image;
        m->fused_ckpt_floats = plan_fused_checkpoints(m->fused_ops, m->L, m->slot_op);
    } else if (!(flags & AIQ_MODEL_LAYERWISE)) {
        m->mb_blocks = plan_mbconv(m->nodes);
        // A 1x1 layer whose only reader is the classifier, on 8x8 pixels: the classifier starts
        // with the mean over those pixels, which the layer's own epilogue can form (a wavefront
        // holds one whole image), so the full-resolution output never reaches memory.
        if (n_layers >= 2) {
            Node &pc = m->nodes[n_layers - 2];
            const aiq_layer_desc &d = pc.d, &fc = layers[n_layers - 1];
            int readers = 0;
            for (int l = 0; l < n_layers; ++l)
                readers += (layers[l].input == n_layers - 2) + (layers[l].residual == n_layers - 2);
            if (fc.kind == 2 && fc.input == n_layers - 2 && readers == 1 && d.kind == 0 && d.kh == 1 && d.stride == 1 &&
                d.input >= 0 && d.residual < 0 && pc.mb_role == 0 && pc.hout * pc.wout == 64 && (d.cout & 3) == 0) {
                pc.pooled = true;
                pc.out_elems = (size_t)d.cout;
                pc.act_bytes_per_image = 4.0 * ((double)pc.in_elems + d.cout);
                m->nodes[n_layers - 1].in_elems = (size_t)d.cout; // what the classifier reads per image
                m->nodes[n_layers - 1].act_bytes_per_image = 4.0 * d.cout;
            }
        }
    }

    // activation buffers: a node's output lives until its last reader has run
    std::vector<int> last_use(n_layers, -1);
    for (int l = 0; l < n_layers; ++l) {
        if (layers[l].input >= 0) last_use[layers[l].input] = l;
        if (layers[l].residual >= 0) last_use[layers[l].residual] = std::max(last_use[layers[l].residual], l);
        // a block kernel reads the block input while it writes the project output: both stay live
        if (m->nodes[l].mb_role == 1) last_use[layers[l].input] = std::max(last_use[layers[l].input], l + 2);
    }
    std::vector<int> owner; // owner[b] = node currently held by buffer b, -1 free
    for (int l = 0; l + 1 < n_layers; ++l) {
        // the hidden tensors of an LDS-resident block (expand and depthwise outputs) never reach memory
        if (m->nodes[l].mb_role == 1 || (m->nodes[l].mb_role == 2 && m->nodes[l].d.kind == 1)) continue;
        // free buffers whose tenant is no longer needed by node l or later
        for (size_t b = 0; b < owner.size(); ++b)
            if (owner[b] >= 0 && last_use[owner[b]] < l) owner[b] = -1;
        int pick = -1;
        for (size_t b = 0; b < owner.size(); ++b)
            if (owner[b] < 0) {
                pick = (int)b;
                break;
            }
        if (pick < 0) {
            owner.push_back(-1);
            pick = (int)owner.size() - 1;
        }
        owner[pick] = l;
        m->nodes[l].buf = pick;
        m->buf_elems = std::max(m->buf_elems, m->nodes[l].out_elems);
    }
    m->n_bufs = m->fused ? 0 : (int)owner.size();
    m->slot_node.assign(m->L, -1);
    m->ref_node_off.assign(n_layers, 0);
    for (int l = 0; l < n_layers; ++l) {
        if (layers[l].scheme_slot >= 0) m->slot_node[layers[l].scheme_slot] = l;
        if (!m->fused && m->nodes[l].buf >= 0) {
            m->ref_node_off[l] = m->ref_act_elems;
            m->ref_act_elems += (m->nodes[l].out_elems + 63) / 64 * 64; // 256-byte aligned records
        }
    }

    // device copies, bank slots, quantize job table
    auto fail = [&](aiq_status code) {
        aiq_model_destroy(m);
        return code;
    };
    if (!hip_ok(conv_set_lds_limits()) || !hip_ok(fused_set_lds_limit()) || !hip_ok(conv_codes_set_lds_limits()))
        return fail(AIQ_DEVICE_ERROR);
    std::vector<int32_t> block_job;
    m->per_tensor = (flags & AIQ_MODEL_PER_TENSOR) != 0;
    m->act_quant = (flags & AIQ_MODEL_ACT_QUANT) != 0;
    for (const Node &nd : m->nodes)
        if (m->act_quant && nd.d.scheme_slot >= 0 && nd.d.kind != 2) m->aq_elems = std::max(m->aq_elems, nd.in_elems);
    if (m->per_tensor && (st = dev_alloc(m, &m->layer_amax, (size_t)n_layers)) != AIQ_OK) return fail(st);
    for (int l = 0; l < n_layers; ++l) {
        Node &nd = m->nodes[l];
        const size_t wn = (size_t)nd.d.cout * nd.k;
        if ((st = dev_alloc(m, &nd.w_plain, wn)) != AIQ_OK) return fail(st);
        if ((st = dev_alloc(m, &nd.bias, (size_t)nd.d.cout)) != AIQ_OK) return fail(st);
        if (!hip_ok(hipMemcpy(nd.w_plain, w_host[l], wn * sizeof(float), hipMemcpyHostToDevice)) ||
            !hip_ok(hipMemcpy(nd.bias, bias_host[l], nd.d.cout * sizeof(float), hipMemcpyHostToDevice)))
            return fail(AIQ_DEVICE_ERROR);
        // the weights never change: the matrix-wide maximum per-tensor scales need is formed once
        if (m->per_tensor && !hip_ok(launch_tensor_absmax(nd.w_plain, wn, m->layer_amax + l, nullptr)))
            return fail(AIQ_DEVICE_ERROR);
        const int n_slots = nd.d.scheme_slot >= 0 ? kNumBits : 1;
        for (int b = 0; b < n_slots; ++b) {
            if ((st = dev_alloc(m, &nd.bank[b], nd.bank_elems)) != AIQ_OK) return fail(st);
            if (!hip_ok(hipMemset(nd.bank[b], 0, nd.bank_elems * sizeof(float)))) return fail(AIQ_DEVICE_ERROR);
            QuantJob j{};
            j.w = nd.w_plain;
            j.out = nd.bank[b];
            j.cout = nd.d.cout;
            j.k = nd.k;
            j.bits = kBitsOfIndex[b];
            j.layout = nd.layout;
            j.taps = nd.d.kind == 2 ? 1 : nd.d.kh * nd.d.kw;
            j.cblocks = (nd.d.cin + 15) / 16;
            j.tensor_amax = (m->per_tensor && b > 0) ? m->layer_amax + l : nullptr;
            if (b == 0) {
                // the FP32 copy in kernel layout is written once, here
                if (!hip_ok(launch_quantize_single(j, nullptr))) return fail(AIQ_DEVICE_ERROR);
            } else {
                if (b == 1) nd.job0 = (int)m->jobs_host.size();
                j.first_block = (int32_t)block_job.size();
                const int blocks = (j.cout + kQuantChannelsPerBlock - 1) / kQuantChannelsPerBlock;
                block_job.insert(block_job.end(), blocks, (int32_t)m->jobs_host.size());
                m->jobs_host.push_back(j);
            }
        }
    }
    m->n_jobs = (int)m->jobs_host.size();
    m->n_quant_blocks = (int)block_job.size();
    if (m->n_jobs > kMaxQuantJobs) return fail(AIQ_UNSUPPORTED_LAYER);
    if (m->n_jobs) {
        if ((st = dev_alloc(m, &m->jobs_dev, (size_t)m->n_jobs)) != AIQ_OK) return fail(st);
        if ((st = dev_alloc(m, &m->block_job_dev, block_job.size())) != AIQ_OK) return fail(st);
        if (!hip_ok(hipMemcpy(m->jobs_dev, m->jobs_host.data(), sizeof(QuantJob) * m->n_jobs,
                              hipMemcpyHostToDevice)) ||
            !hip_ok(hipMemcpy(m->block_job_dev, block_job.data(), sizeof(int32_t) * block_job.size(),
                              hipMemcpyHostToDevice)))
            return fail(AIQ_DEVICE_ERROR);
    }
    if (m->fused) {
        // ops follow the node order with projections in place, so op o describes node o
        for (size_t o = 0; o < m->fused_ops.size(); ++o) {
            const Node &nd = m->nodes[o];
            for (int b = 0; b < kNumBits; ++b) m->fused_ops[o].bank[b] = nd.bank[b] ? nd.bank[b] : nd.bank[0];
            m->fused_ops[o].bias = nd.bias;
        }
        if ((st = dev_alloc(m, &m->fused_ops_dev, m->fused_ops.size())) != AIQ_OK) return fail(st);
        if (!hip_ok(hipMemcpy(m->fused_ops_dev, m->fused_ops.data(), sizeof(FusedOp) * m->fused_ops.size(),
                              hipMemcpyHostToDevice)))
            return fail(AIQ_DEVICE_ERROR);
    }
    if (!hip_ok(hipDeviceSynchronize())) return fail(AIQ_DEVICE_ERROR);
    *out = m;
    return AIQ_OK;
}

aiq_status aiq_eval_workspace_bytes(const aiq_model *m, int32_t S, int32_t chunk, size_t *bytes)
{
    if (!m || !bytes || S < 0 || chunk < 1) return AIQ_INVALID_ARG;
    *bytes = workspace_layout(m, S, chunk).total;
    return AIQ_OK;
}

} // extern "C"

namespace {

// Checkpoints a reference pass has left in a workspace, remembered across the scoring calls of
// one search run (which owns the workspace for its duration and never changes images or
// chunking): the reference scheme they were taken under and which ops have one.  A later
// reference scheme that agrees with it on the layers before an op can reuse that op's
// checkpoint, so the reference pass of the next step continues from the deepest such
// checkpoint instead of from the image, and stops after the last checkpoint the step needs.
struct CkptCache {
    int s_layout = 0;            // scheme count the workspace is laid out for (offsets must not move between steps)
    const void *workspace = nullptr;
    std::vector<uint8_t> scheme; // empty: nothing cached
    uint64_t valid[2] = {0, 0};
    int valid_nodes = 0;         // layer-by-layer path: the reference outputs of nodes [0, valid_nodes) are good
};

// What one launch of a node reads and writes: pointers for its first scheme and the distance
// (in elements) between consecutive schemes; distance 0 = all schemes share one copy.
struct NodeIO {
    const float *in;
    size_t in_stride;
    float *out;
    size_t out_stride;
    const float *res;
    size_t res_stride;
    const uint8_t *schemes;  // device [S][L], first scheme of the launch
    int S;                   // scheme rows; launch indices >= S run all-FP32 (the base pass)
    int s_total;             // launch extent along the scheme axis
    const int32_t *row_map;  // classifier: output row of launch index i (-1: the FP32 pass), or nullptr = i
    int32_t *top1_base_out;  // classifier: where the FP32 pass writes its top-1, or nullptr
};

// Where the classifier of a call puts its results.
struct HeadOut {
    float *logits;     // nullable; [rows][N][classes]
    int32_t N;         // images of the whole call
    int32_t *top1;     // nullable: [rows][N]; else top1_tmp [rows][chunk]
    int32_t *top1_tmp;
    int32_t chunk;
};

// One node (or one LDS-resident block, at its expand node) for the schemes the launch covers.
aiq_status launch_node(aiq_model *m, hipStream_t st, const HeadOut &ho, size_t l, const NodeIO &io_in, int n, int n0)
{
    const Node &nd = m->nodes[l];
    const aiq_layer_desc &d = nd.d;
    const double work = (double)io_in.s_total * n;
    if (nd.mb_role == 2) return AIQ_OK; // computed by the block kernel launched at its expand node
    if (m->act_quant && d.scheme_slot >= 0 && d.kind != 2) {
        // the layer reads a copy of its input quantized at its own width (the classifier does the same to the
        // pooled vector inside its kernel)
        if (!m->aq_cur) return AIQ_INVALID_ARG;
        ActQuantArgs q{};
        q.in = io_in.in;
        q.out = m->aq_cur;
        q.schemes = io_in.schemes;
        q.in_scheme_stride = io_in.in_stride;
        q.out_scheme_stride = (size_t)n * nd.in_elems;
        q.S = io_in.S;
        q.L = m->L;
        q.slot = d.scheme_slot;
        q.N = n;
        q.elems = (int32_t)nd.in_elems;
        {
            ProfScope ps(m, st, AIQ_K_QUANTIZE, 0.0, 8.0 * nd.in_elems * work);
            AIQ_HIP(launch_act_quantize(q, io_in.s_total, st));
        }
    }
    NodeIO io = io_in;
    if (m->act_quant && d.scheme_slot >= 0 && d.kind != 2) {
        io.in = m->aq_cur;
        io.in_stride = (size_t)n * nd.in_elems;
    }
    if (nd.mb_role == 1 && m->mb_codes_cur && (m->mb_codes_cur[l].codes_e || m->mb_codes_cur[l].codes_p) && io.S == 1 &&
        io.s_total == 1) {
        // deployed scheme, expand and / or project at most eight bits wide: those products from integer codes
        const Node &dwn = m->nodes[l + 1], &pjn = m->nodes[l + 2];
        const MbCodes &mc = m->mb_codes_cur[l];
        auto bank_of = [&](const Node &x) {
            const int bi = x.d.scheme_slot >= 0 ? bits_index(m->mb_scheme_cur[x.d.scheme_slot]) : 0;
            return x.bank[bi] ? x.bank[bi] : x.bank[0];
        };
        MbCodeArgs a{};
        a.in = io.in;
        a.out = io.out;
        a.codes_e = mc.codes_e;
        a.codes_p = mc.codes_p;
        a.scale_e = mc.scale_e;
        a.scale_p = mc.scale_p;
        a.w_d = bank_of(dwn);
        a.w_e = bank_of(nd);
        a.w_p = bank_of(pjn);
        a.bias_e = nd.bias;
        a.bias_d = dwn.bias;
        a.bias_p = pjn.bias;
        a.N = n;
        a.act_e = d.act;
        a.act_d = dwn.d.act;
        a.act_p = pjn.d.act;
        const double flops = nd.flops_per_image + dwn.flops_per_image + pjn.flops_per_image;
        const double bytes = 4.0 * (nd.in_elems + pjn.out_elems + (pjn.d.residual >= 0 ? pjn.out_elems : 0));
        ProfScope ps(m, st, AIQ_K_MBCONV, flops * work, bytes * work);
        AIQ_HIP(launch_mbconv_codes(nd.mb_shape, a, st));
    } else if (nd.mb_role == 1) {
        const Node &dwn = m->nodes[l + 1], &pjn = m->nodes[l + 2];
        MbArgs a{};
        a.in = io.in;
        a.out = io.out;
        for (int b = 0; b < kNumBits; ++b) {
            a.bank_e[b] = nd.bank[b] ? nd.bank[b] : nd.bank[0];
            a.bank_d[b] = dwn.bank[b] ? dwn.bank[b] : dwn.bank[0];
            a.bank_p[b] = pjn.bank[b] ? pjn.bank[b] : pjn.bank[0];
        }
        a.bias_e = nd.bias;
        a.bias_d = dwn.bias;
        a.bias_p = pjn.bias;
        a.schemes = io.schemes;
        a.in_scheme_stride = io.in_stride;
        a.out_scheme_stride = io.out_stride;
        a.S = io.S;
        a.L = m->L;
        a.slot_e = d.scheme_slot;
        a.slot_d = dwn.d.scheme_slot;
        a.slot_p = pjn.d.scheme_slot;
        a.N = n;
        a.act_e = d.act;
        a.act_d = dwn.d.act;
        a.act_p = pjn.d.act;
        const double flops = nd.flops_per_image + dwn.flops_per_image + pjn.flops_per_image;
        const double bytes = 4.0 * (nd.in_elems + pjn.out_elems + (pjn.d.residual >= 0 ? pjn.out_elems : 0));
        ProfScope ps(m, st, AIQ_K_MBCONV, flops * work, bytes * work);
        AIQ_HIP(launch_mbconv(nd.mb_shape, a, io.s_total, st));
    } else if (nd.pooled && m->mb_codes_cur && m->mb_codes_cur[l].codes_e && io.S == 1 && io.s_total == 1) {
        // deployed scheme: the last 1x1 layer (with the classifier's pooling) from integer codes
        const MbCodes &mc = m->mb_codes_cur[l];
        PoolCodeArgs a{};
        a.in = io.in;
        a.out = io.out;
        a.codes = mc.codes_e;
        a.scales = mc.scale_e;
        a.bias = nd.bias;
        a.N = n;
        a.Cin = d.cin;
        a.Cout = d.cout;
        a.act = d.act;
        a.KS = (d.cin + 31) / 32;
        if (!pooled_codes_plan(d.cin, d.cout, &a.CG, &a.groups)) return AIQ_INVALID_ARG;
        ProfScope ps(m, st, AIQ_K_CONV_CODES, nd.flops_per_image * work, nd.act_bytes_per_image * work);
        AIQ_HIP(launch_pooled_codes(a, st));
    } else if (d.kind == 0 && d.kh == 1 && d.stride == 1 && d.input >= 0) {
        // 1x1 stride 1: flat pixel axis
        const ConvPlan &p = nd.plan;
        PointwiseArgs a{};
        a.in = io.in;
        a.out = io.out;
        a.res = io.res;
        a.bias = nd.bias;
        for (int b = 0; b < kNumBits; ++b) a.bank[b] = nd.bank[b] ? nd.bank[b] : nd.bank[0];
        a.schemes = io.schemes;
        a.in_scheme_stride = io.in_stride;
        a.out_scheme_stride = io.out_stride;
        a.res_scheme_stride = io.res_stride;
        a.S = io.S;
        a.L = m->L;
        a.slot = d.scheme_slot;
        a.P = n * nd.hout * nd.wout;
        a.Cin = d.cin;
        a.Cout = d.cout;
        a.act = d.act;
        a.CB = p.CB;
        a.CKC = p.CKC;
        a.PS = p.PS;
        a.wave_px_split = p.wave_px_split;
        a.cout_tiles = p.cout_tiles;
        a.pool = nd.pooled ? 1 : 0;
        a.grid_y = p.grid_y;
        const int tile_px = 64 * p.wave_px_split;
        const size_t lds = sizeof(float) * (size_t)tile_px * p.PS;
        ProfScope ps(m, st, AIQ_K_CONV, nd.flops_per_image * work, nd.act_bytes_per_image * work);
        AIQ_HIP(launch_pointwise(a, p.nt, lds,
                                 dim3((unsigned)((a.P + tile_px - 1) / tile_px), p.grid_y, io.s_total), st));
    } else if (d.kind == 0) {
        const ConvPlan &p = nd.plan;
        ConvArgs a{};
        a.in = io.in;
        a.out = io.out;
        a.res = io.res;
        a.bias = nd.bias;
        for (int b = 0; b < kNumBits; ++b) a.bank[b] = nd.bank[b] ? nd.bank[b] : nd.bank[0];
        a.schemes = io.schemes;
        a.in_scheme_stride = io.in_stride;
        a.out_scheme_stride = io.out_stride;
        a.res_scheme_stride = io.res_stride;
        a.S = io.S;
        a.L = m->L;
        a.slot = d.scheme_slot;
        a.N = n;
        a.Hin = d.hin;
        a.Win = d.win;
        a.Cin = d.cin;
        a.Hout = nd.hout;
        a.Wout = nd.wout;
        a.Cout = d.cout;
        a.act = d.act;
        a.R = p.R;
        a.G = p.G;
        a.regions_per_image = p.regions_per_image;
        a.CB = p.CB;
        a.CKC = p.CKC;
        a.RIN = p.RIN;
        a.LW = p.LW;
        a.PS = p.PS;
        a.wave_px_split = p.wave_px_split;
        a.cout_tiles = p.cout_tiles;
        a.div_lw = make_fastdiv(p.LW);
        a.div_rin = make_fastdiv(p.RIN);
        a.div_wout = make_fastdiv(nd.wout);
        a.div_rw = make_fastdiv(p.R * nd.wout);
        const unsigned gx = p.G > 1 ? (unsigned)((n + p.G - 1) / p.G) : (unsigned)(n * p.regions_per_image);
        ProfScope ps(m, st, AIQ_K_CONV, nd.flops_per_image * work, nd.act_bytes_per_image * work);
        if (nd.layout == kLayoutStem)
            AIQ_HIP(launch_conv_stem(a, p.nt, dim3(gx, p.grid_y, io.s_total), st));
        else
            AIQ_HIP(launch_conv(a, d.kh, d.stride, p.nt, p.lds_bytes, dim3(gx, p.grid_y, io.s_total), st));
    } else if (d.kind == 1) {
        DepthwiseArgs a{};
        a.in = io.in;
        a.out = io.out;
        a.bias = nd.bias;
        for (int b = 0; b < kNumBits; ++b) a.bank[b] = nd.bank[b] ? nd.bank[b] : nd.bank[0];
        a.schemes = io.schemes;
        a.in_scheme_stride = io.in_stride;
        a.out_scheme_stride = io.out_stride;
        a.S = io.S;
        a.L = m->L;
        a.slot = d.scheme_slot;
        a.N = n;
        a.Hin = d.hin;
        a.Win = d.win;
        a.C = d.cin;
        a.Hout = nd.hout;
        a.Wout = nd.wout;
        a.stride = d.stride;
        a.act = d.act;
        a.div_c4 = make_fastdiv(d.cin / 4);
        ProfScope ps(m, st, AIQ_K_DEPTHWISE, nd.flops_per_image * work, nd.act_bytes_per_image * work);
        AIQ_HIP(launch_depthwise(a, io.s_total, st));
    } else {
        HeadArgs a{};
        a.in = io.in;
        a.bias = nd.bias;
        for (int b = 0; b < kNumBits; ++b) a.bank[b] = nd.bank[b] ? nd.bank[b] : nd.bank[0];
        a.schemes = io.schemes;
        a.in_scheme_stride = io.in_stride;
        a.S = io.S;
        a.L = m->L;
        a.slot = d.scheme_slot;
        a.N = n;
        a.HW = m->nodes[d.input].pooled ? 1 : d.hin * d.win; // a pooled producer has already taken the mean
        a.C = d.cin;
        a.classes = d.cout;
        a.logits = ho.logits;
        a.logits_n = ho.N;
        a.n0 = n0;
        if (ho.top1) {
            a.top1 = ho.top1 + n0;
            a.top1_stride = ho.N;
        } else {
            a.top1 = ho.top1_tmp;
            a.top1_stride = ho.chunk;
        }
        a.top1_base = io.top1_base_out;
        a.row_map = io.row_map;
        a.act_quant = m->act_quant ? 1 : 0;
        ProfScope ps(m, st, AIQ_K_HEAD, nd.flops_per_image * work, nd.act_bytes_per_image * work);
        AIQ_HIP(launch_head(a, io.s_total, st));
    }
    return AIQ_OK;
}

// Scores S schemes.  ref = NULL: every scheme runs the whole network.  ref = host uint8[L]:
// where the model supports it, the reference scheme is run once per image and scheme s
// resumes at its first layer whose width differs from ref's; the results are the same.
aiq_status eval_impl(aiq_model *m, const float *images, int32_t N, const uint8_t *schemes, int32_t S,
                     const uint8_t *ref, int32_t chunk, int32_t *top1_base, int32_t base_valid, float *logits,
                     int32_t *top1, int32_t *agree, void *workspace, size_t workspace_bytes, void *hip_stream,
                     CkptCache *cache = nullptr, bool want_agree = true)
{
    // want_agree = false (deployed inference of one scheme): no agreement count, no FP32 reference;
    // agree and top1_base may then be null and base_valid must be 1
    if (!m || N < 0 || S < 0 || chunk < 1) return AIQ_INVALID_ARG;
    if (S > 0 && (!schemes || (want_agree && !agree))) return AIQ_INVALID_ARG;
    if (N > 0 && (!images || (want_agree && !top1_base) || !workspace)) return AIQ_INVALID_ARG;
    if (!want_agree && base_valid != 1) return AIQ_INVALID_ARG;
    if (base_valid != 0 && base_valid != 1) return AIQ_INVALID_ARG;
    if (S + 1 > 65535) return AIQ_INVALID_ARG; // the scheme axis (plus the FP32 pass) is a grid y / z extent
    for (size_t i = 0; i < (size_t)S * m->L; ++i)
        if (!bits_supported(schemes[i])) return AIQ_UNSUPPORTED_BITS;
    if (ref)
        for (int i = 0; i < m->L; ++i)
            if (!bits_supported(ref[i])) return AIQ_UNSUPPORTED_BITS;
    chunk = std::min(chunk, std::max(N, 1));
    const bool shared = ref != nullptr;
    const WorkspaceLayout wl = workspace_layout(m, cache ? std::max(cache->s_layout, S) : S, chunk, shared);
    // sharing needs a reference pass that can hand over its state, and something to share it with
    const bool resume = shared && m->fused && m->fused_ckpt_floats > 0 && S > 0;
    if (N > 0 && workspace_bytes < wl.total) return AIQ_WORKSPACE_TOO_SMALL;
    if (N > 0 && (reinterpret_cast<uintptr_t>(workspace) & 255)) return AIQ_INVALID_ARG;

    hipStream_t st = (hipStream_t)hip_stream;
    if (S > 0 && want_agree) AIQ_HIP(launch_fill_i32(agree, 0, (size_t)S, st));
    if (N == 0) return AIQ_OK;
    const bool run_base = base_valid == 0;
    const int s_total = S + (run_base ? 1 : 0);
    if (s_total == 0) return AIQ_OK;

    char *ws = static_cast<char *>(workspace);
    uint8_t *schemes_dev = reinterpret_cast<uint8_t *>(ws + wl.schemes_off);
    int32_t *top1_tmp = reinterpret_cast<int32_t *>(ws + wl.top1_off);
    m->aq_cur = m->act_quant ? reinterpret_cast<float *>(ws + wl.aq_off) : nullptr;

    // plan: which (layer, bit-width) bank slots this call reads
    QuantMask mask{};
    bool any = false;
    for (const Node &nd : m->nodes) {
        if (nd.d.scheme_slot < 0) continue;
        for (int s = 0; s < S; ++s) {
            const int bi = bits_index(schemes[(size_t)s * m->L + nd.d.scheme_slot]);
            if (bi > 0) {
                const int ji = nd.job0 + bi - 1;
                mask.word[ji >> 6] |= 1ull << (ji & 63);
                any = true;
            }
        }
    }
    if (S > 0) AIQ_HIP(upload_bytes(schemes_dev, schemes, (size_t)S * m->L, st));

    // prefix sharing: op at which every scheme leaves the reference scheme, and what the
    // passes that start there execute
    uint8_t *ref_dev = nullptr;
    int32_t *first_op_dev = nullptr, *ref_top1 = nullptr;
    float *ckpt = nullptr;
    bool ref_is_base = false;
    double resumed_flops_per_image = 0.0; // summed over the S schemes
    std::vector<int32_t> first_op;
    if (resume) {
        ref_dev = reinterpret_cast<uint8_t *>(ws + wl.ref_off);
        first_op_dev = reinterpret_cast<int32_t *>(ws + wl.first_op_off);
        ref_top1 = reinterpret_cast<int32_t *>(ws + wl.ref_top1_off);
        ckpt = reinterpret_cast<float *>(ws + wl.ckpt_off);
        ref_is_base = true;
        for (int i = 0; i < m->L; ++i) {
            ref_is_base = ref_is_base && ref[i] == 32;
            const int bi = bits_index(ref[i]);
            if (bi > 0) {
                const int ji = m->nodes[m->slot_op[i]].job0 + bi - 1;
                mask.word[ji >> 6] |= 1ull << (ji & 63);
                any = true;
            }
        }
        const int n_ops = (int)m->fused_ops.size();
        std::vector<double> suffix(n_ops + 1, 0.0);
        for (int o = n_ops - 1; o >= 0; --o) suffix[o] = suffix[o + 1] + m->nodes[o].flops_per_image;
        first_op.assign(S + 1, 0);
        for (int s_ = 0; s_ < S; ++s_) {
            int d = 0;
            while (d < m->L && schemes[(size_t)s_ * m->L + d] == ref[d]) ++d;
            first_op[s_] = d < m->L ? m->slot_op[d] : n_ops - 1; // identical to ref: only the last op runs again
            resumed_flops_per_image += suffix[first_op[s_]];
        }
        AIQ_HIP(upload_bytes(ref_dev, ref, (size_t)m->L, st));
        AIQ_HIP(upload_bytes(first_op_dev, first_op.data(), sizeof(int32_t) * (S + 1), st));
    }
    // The same on the layer-by-layer path: the rows (schemes, plus the FP32 pass when it has to
    // run and is not the reference itself) are sorted by the node at which they leave the
    // reference, so that the rows a node has to compute are always a prefix of the sorted order.
    const bool share_nodes = shared && !m->fused && S > 0;
    uint8_t *sorted_dev = nullptr;
    int32_t *row_map_dev = nullptr;
    float *ref_act = nullptr;
    int S_rows = 0, first_node_max = 0;
    std::vector<int> active;
    const std::vector<size_t> &ref_node_off = m->ref_node_off;
    if (share_nodes) {
        ref_dev = reinterpret_cast<uint8_t *>(ws + wl.ref_off);
        row_map_dev = reinterpret_cast<int32_t *>(ws + wl.first_op_off);
        sorted_dev = reinterpret_cast<uint8_t *>(ws + wl.sorted_off);
        ref_act = reinterpret_cast<float *>(ws + wl.ckpt_off);
        const int n_nodes = (int)m->nodes.size();
        ref_is_base = true;
        for (int i = 0; i < m->L; ++i) {
            ref_is_base = ref_is_base && ref[i] == 32;
            const int bi = bits_index(ref[i]);
            if (bi > 0) {
                const int ji = m->nodes[m->slot_node[i]].job0 + bi - 1;
                mask.word[ji >> 6] |= 1ull << (ji & 63);
                any = true;
            }
        }
        std::vector<std::pair<int, int>> rows; // (first node, original row; -1 = the FP32 pass)
        if (run_base && !ref_is_base) rows.emplace_back(0, -1);
        for (int s_ = 0; s_ < S; ++s_) {
            int d = 0;
            while (d < m->L && schemes[(size_t)s_ * m->L + d] == ref[d]) ++d;
            int f = d < m->L ? m->slot_node[d] : n_nodes - 1; // identical to ref: only the classifier runs again
            while (m->nodes[f].mb_role == 2) --f;             // a block runs from its expand node
            rows.emplace_back(f, s_);
        }
        std::stable_sort(rows.begin(), rows.end(),
                         [](const std::pair<int, int> &x, const std::pair<int, int> &y) { return x.first < y.first; });
        S_rows = (int)rows.size();
        first_node_max = rows.back().first; // rows are sorted by their first node
        std::vector<uint8_t> sorted((size_t)S_rows * m->L, 32);
        std::vector<int32_t> row_map(S_rows + 1, -1);
        active.assign(n_nodes, 0);
        for (int i = 0; i < S_rows; ++i) {
            row_map[i] = rows[i].second;
            if (rows[i].second >= 0)
                std::memcpy(&sorted[(size_t)i * m->L], schemes + (size_t)rows[i].second * m->L, m->L);
            ++active[rows[i].first];
        }
        for (int l = 1; l < n_nodes; ++l) active[l] += active[l - 1];
        AIQ_HIP(upload_bytes(ref_dev, ref, (size_t)m->L, st));
        AIQ_HIP(upload_bytes(sorted_dev, sorted.data(), sorted.size(), st));
        AIQ_HIP(upload_bytes(row_map_dev, row_map.data(), sizeof(int32_t) * row_map.size(), st));
    }
    if (any) {
        double qbytes = 0.0;
        for (int ji = 0; ji < m->n_jobs; ++ji)
            if ((mask.word[ji >> 6] >> (ji & 63)) & 1ull)
                qbytes += 8.0 * m->jobs_host[ji].cout * m->jobs_host[ji].k;
        ProfScope ps(m, st, AIQ_K_QUANTIZE, 0.0, qbytes);
        AIQ_HIP(launch_quantize_batch(m->jobs_dev, m->block_job_dev, m->n_quant_blocks, mask, st));
    }

    const HeadOut ho{logits, N, top1, top1_tmp, chunk};
    auto launch_node = [&](size_t l, const NodeIO &io, int n, int n0) -> aiq_status {
        return ::launch_node(m, st, ho, l, io, n, n0);
    };

    for (int n0 = 0; n0 < N; n0 += chunk) {
        const int n = std::min(chunk, N - n0);
        auto buf_ptr = [&](int b) { return reinterpret_cast<float *>(ws + wl.act_off + wl.buf_stride * b); };
        if (m->fused) {
            FusedArgs a{};
            a.ops = m->fused_ops_dev;
            a.n_ops = (int32_t)m->fused_ops.size();
            a.images = images + (size_t)n0 * m->nodes[0].in_elems;
            a.schemes = schemes_dev;
            a.S = S;
            a.L = m->L;
            a.N = n;
            a.logits = logits;
            a.logits_n = N;
            a.n0 = n0;
            if (top1) {
                a.top1 = top1 + n0;
                a.top1_stride = N;
            } else {
                a.top1 = top1_tmp;
                a.top1_stride = chunk;
            }
            a.top1_base = run_base ? top1_base + n0 : nullptr;
            const double work = (double)s_total * n;
            if (resume) {
                // reference pass: one scheme (the FP32 pass itself when ref is all-FP32)
                FusedArgs r = a;
                r.schemes = ref_dev;
                r.S = ref_is_base ? 0 : 1;
                r.logits = nullptr;
                r.top1 = ref_top1;
                r.top1_stride = chunk;
                r.top1_base = ref_is_base && run_base ? top1_base + n0 : nullptr;
                r.ckpt = ckpt;
                r.ckpt_stride = (int64_t)m->fused_ckpt_floats;
                const int n_ops = (int)m->fused_ops.size();
                const bool ref_head = ref_is_base && run_base; // the pass's own top-1 is wanted
                // checkpoints the candidates resume from
                uint64_t need[2] = {0, 0};
                for (int s_ = 0; s_ < S; ++s_)
                    if (first_op[s_] > 0) need[first_op[s_] >> 6] |= 1ull << (first_op[s_] & 63);
                // those a previous step of the same search has left behind and that are still good:
                // taken under a reference that agrees with this one on every layer before the op
                const bool cached = cache && N <= chunk && cache->workspace == workspace &&
                                    cache->scheme.size() == (size_t)m->L;
                int same_upto = 0; // ops [0, same_upto) carry the same widths in both references
                if (cached) {
                    int d = 0;
                    while (d < m->L && cache->scheme[d] == ref[d]) ++d;
                    same_upto = d < m->L ? m->slot_op[d] + 1 : n_ops; // a checkpoint precedes its op
                }
                auto have = [&](int o) { return cached && o < same_upto && ((cache->valid[o >> 6] >> (o & 63)) & 1ull); };
                r.ref_first_op = 0;
                r.ref_stop_op = ref_head ? n_ops : 0;
                double ck_floats = 0.0;
                int first_missing = n_ops;
                for (int o = 1; o < n_ops; ++o)
                    if (((need[o >> 6] >> (o & 63)) & 1ull) && !have(o)) {
                        r.ck_mask[o >> 6] |= 1ull << (o & 63);
                        ck_floats += m->fused_ops[o].ck_ext[0] + m->fused_ops[o].ck_ext[1];
                        first_missing = std::min(first_missing, o);
                        r.ref_stop_op = std::max(r.ref_stop_op, o);
                    }
                const bool run_ref = ref_head || first_missing < n_ops;
                if (run_ref && !ref_head)
                    for (int o = first_missing - 1; o > 0; --o) // deepest reusable checkpoint before the first missing one
                        if (have(o)) {
                            r.ref_first_op = o;
                            break;
                        }
                if (run_ref) {
                    double fl = 0.0;
                    for (int o = r.ref_first_op; o < std::min(r.ref_stop_op, n_ops); ++o) fl += m->nodes[o].flops_per_image;
                    ProfScope ps(m, st, AIQ_K_FUSED, fl * n,
                                 n * (4.0 * (m->nodes[0].in_elems + m->classes) + 4.0 * ck_floats));
                    AIQ_HIP(launch_fused(r, 1, kFusedReference, st));
                }
                if (cache && N <= chunk) {
                    // what the workspace now holds: the reusable part of the old set plus what this pass wrote
                    uint64_t v[2] = {0, 0};
                    for (int o = 1; o < n_ops; ++o)
                        if (have(o) || ((r.ck_mask[o >> 6] >> (o & 63)) & 1ull)) v[o >> 6] |= 1ull << (o & 63);
                    cache->workspace = workspace;
                    cache->scheme.assign(ref, ref + m->L);
                    cache->valid[0] = v[0];
                    cache->valid[1] = v[1];
                }
                a.ckpt = ckpt;
                a.ckpt_stride = r.ckpt_stride;
                a.first_op = first_op_dev;
                if (ref_is_base) a.top1_base = nullptr; // written by the reference pass
                const bool extra_base = run_base && !ref_is_base;
                double rd_bytes = 0.0;
                for (int s_ = 0; s_ < S; ++s_) {
                    const FusedOp &op = m->fused_ops[first_op[s_]];
                    rd_bytes += first_op[s_] > 0 ? 4.0 * (op.ck_ext[0] + op.ck_ext[1]) : 4.0 * m->nodes[0].in_elems;
                }
                ProfScope ps(m, st, AIQ_K_FUSED,
                             (resumed_flops_per_image + (extra_base ? m->fused_flops_per_image : 0.0)) * n,
                             n * (rd_bytes + 4.0 * m->classes * S));
                AIQ_HIP(launch_fused(a, S + (extra_base ? 1 : 0), kFusedResume, st));
            } else {
                ProfScope ps(m, st, AIQ_K_FUSED, m->fused_flops_per_image * work,
                             work * 4.0 * (m->nodes[0].in_elems + m->classes));
                AIQ_HIP(launch_fused(a, s_total, kFusedPlain, st));
            }
            if (want_agree) {
                AgreeArgs g{};
                g.top1 = a.top1;
                g.top1_stride = a.top1_stride;
                g.top1_base = top1_base + n0;
                g.agree = agree;
                g.N = n;
                g.S = S;
                ProfScope ps(m, st, AIQ_K_AGREE, 0.0, 8.0 * S * n);
                AIQ_HIP(launch_agree(g, st));
            }
            continue;
        }
        if (!share_nodes) {
            NodeIO io{};
            io.schemes = schemes_dev;
            io.S = S;
            io.s_total = s_total;
            io.top1_base_out = run_base ? top1_base + n0 : nullptr;
            for (size_t l = 0; l < m->nodes.size(); ++l) {
                const Node &nd = m->nodes[l];
                io.in = nd.d.input < 0 ? images + (size_t)n0 * nd.in_elems : buf_ptr(m->nodes[nd.d.input].buf);
                io.in_stride = nd.d.input < 0 ? 0 : (size_t)n * nd.in_elems;
                const Node &on = nd.mb_role == 1 ? m->nodes[l + 2] : nd; // a block writes its project node's output
                io.out = on.buf >= 0 ? buf_ptr(on.buf) : nullptr;
                io.out_stride = (size_t)n * on.out_elems;
                io.res = nd.d.residual >= 0 ? buf_ptr(m->nodes[nd.d.residual].buf) : nullptr;
                io.res_stride = io.out_stride;
                aiq_status rc = launch_node(l, io, n, n0);
                if (rc != AIQ_OK) return rc;
            }
        } else {
            // ---- reference pass: every node once, outputs kept per node
            auto ref_ptr = [&](int node) { return ref_act + ref_node_off[node] * (size_t)chunk; };
            const bool ref_head = ref_is_base && run_base; // its top-1 is the FP32 pass's
            NodeIO io{};
            io.schemes = ref_dev;
            io.S = 1;
            io.s_total = 1;
            io.row_map = row_map_dev + S_rows; // a single -1: the row of the FP32 pass
            io.top1_base_out = ref_head ? top1_base + n0 : nullptr;
            // Rows only read reference outputs of nodes before the node they start at, so the pass
            // ends at the last row's first node (unless its own top-1 is wanted); and it begins
            // where the outputs a previous step of the same search left behind stop being good:
            // at the first node whose layer differs between the two references.
            const int n_nodes = (int)m->nodes.size();
            int ref_lo = 0, ref_hi = ref_head ? n_nodes : first_node_max;
            const bool caching = cache && N <= chunk;
            if (caching && cache->workspace == workspace && cache->scheme.size() == (size_t)m->L) {
                int d = 0;
                while (d < m->L && cache->scheme[d] == ref[d]) ++d;
                int changed = d < m->L ? m->slot_node[d] : n_nodes;
                while (changed < n_nodes && m->nodes[changed].mb_role == 2) --changed; // a block is recomputed whole
                ref_lo = std::min(cache->valid_nodes, changed);
            }
            if (caching) {
                cache->workspace = workspace;
                cache->scheme.assign(ref, ref + m->L);
                cache->valid_nodes = std::max(ref_lo, ref_hi);
            }
            for (int l = ref_lo; l < ref_hi; ++l) {
                const Node &nd = m->nodes[l];
                if (nd.d.kind == 2 && !ref_head) continue;
                io.in = nd.d.input < 0 ? images + (size_t)n0 * nd.in_elems : ref_ptr(nd.d.input);
                io.in_stride = 0;
                const int on = nd.mb_role == 1 ? (int)l + 2 : (int)l;
                io.out = m->nodes[on].buf >= 0 ? ref_ptr(on) : nullptr;
                io.out_stride = 0;
                io.res = nd.d.residual >= 0 ? ref_ptr(nd.d.residual) : nullptr;
                io.res_stride = 0;
                aiq_status rc = launch_node(l, io, n, n0);
                if (rc != AIQ_OK) return rc;
            }
            // ---- candidates, sorted by the node they leave the reference at: node l runs rows
            // [0, active[l]); a row reads its own copy of an input it has computed itself and the
            // reference pass's copy otherwise
            for (size_t l = 0; l < m->nodes.size(); ++l) {
                const Node &nd = m->nodes[l];
                if (nd.mb_role == 2) continue;
                const int na = active[l];
                const int own_in = nd.d.input < 0 ? na : std::min(na, active[nd.d.input]);
                const int own_res = nd.d.residual < 0 ? na : std::min(na, active[nd.d.residual]);
                const int cuts[4] = {0, std::min(own_in, own_res), std::max(own_in, own_res), na};
                const int on = nd.mb_role == 1 ? (int)l + 2 : (int)l;
                for (int c = 0; c < 3; ++c) {
                    const int b0 = cuts[c], b1 = cuts[c + 1];
                    if (b1 <= b0) continue;
                    io = NodeIO{};
                    io.schemes = sorted_dev + (size_t)b0 * m->L;
                    io.S = b1 - b0;
                    io.s_total = b1 - b0;
                    io.row_map = row_map_dev + b0;
                    io.top1_base_out = top1_base + n0; // only the FP32 row (row_map < 0) writes it
                    if (nd.d.input < 0) {
                        io.in = images + (size_t)n0 * nd.in_elems;
                    } else if (b0 < own_in) {
                        io.in_stride = (size_t)n * nd.in_elems;
                        io.in = buf_ptr(m->nodes[nd.d.input].buf) + (size_t)b0 * io.in_stride;
                    } else {
                        io.in = ref_ptr(nd.d.input);
                    }
                    io.out_stride = (size_t)n * m->nodes[on].out_elems;
                    io.out = m->nodes[on].buf >= 0 ? buf_ptr(m->nodes[on].buf) + (size_t)b0 * io.out_stride : nullptr;
                    if (nd.d.residual >= 0) {
                        if (b0 < own_res) {
                            io.res_stride = io.out_stride;
                            io.res = buf_ptr(m->nodes[nd.d.residual].buf) + (size_t)b0 * io.res_stride;
                        } else {
                            io.res = ref_ptr(nd.d.residual);
                        }
                    }
                    aiq_status rc = launch_node(l, io, n, n0);
                    if (rc != AIQ_OK) return rc;
                }
            }
        }
        if (S > 0 && want_agree) {
            AgreeArgs g{};
            g.top1 = top1 ? top1 + n0 : top1_tmp;
            g.top1_stride = top1 ? N : chunk;
            g.top1_base = top1_base + n0;
            g.agree = agree;
            g.N = n;
            g.S = S;
            ProfScope ps(m, st, AIQ_K_AGREE, 0.0, 8.0 * S * n);
            AIQ_HIP(launch_agree(g, st));
        }
    }
    return AIQ_OK;
}

} // namespace

extern "C" {

aiq_status aiq_eval_schemes(aiq_model *m, const float *images, int32_t N, const uint8_t *schemes, int32_t S,
                            int32_t chunk, int32_t *top1_base, int32_t base_valid, float *logits, int32_t *top1,
                            int32_t *agree, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return eval_impl(m, images, N, schemes, S, nullptr, chunk, top1_base, base_valid, logits, top1, agree, workspace,
                     workspace_bytes, hip_stream);
}

aiq_status aiq_eval_noalloc_workspace_bytes(const aiq_model *m, int32_t S, int32_t chunk, size_t *needed,
                                            size_t *available)
{
    if (!m || S < 0 || chunk < 1 || (!needed && !available)) return AIQ_INVALID_ARG;
    if (needed) *needed = workspace_layout(m, S, chunk).total;
    if (available) *available = AIQ_NOALLOC_SCRATCH_BYTES;
    return AIQ_OK;
}

aiq_status aiq_eval_schemes_noalloc(aiq_model *m, const float *images, int32_t N, const uint8_t *schemes, int32_t S,
                                    int32_t chunk, int32_t *top1_base, int32_t base_valid, float *logits,
                                    int32_t *top1, int32_t *agree, void *hip_stream)
{
    if (!m || N < 0 || S < 0 || chunk < 1) return AIQ_INVALID_ARG;
    // the size check uses the chunk the scoring will really use
    const int32_t eff_chunk = std::min(chunk, std::max(N, 1));
    if (workspace_layout(m, S, eff_chunk).total > (size_t)AIQ_NOALLOC_SCRATCH_BYTES) return AIQ_WORKSPACE_TOO_SMALL;
    void *ws = nullptr;
    size_t ws_bytes = 0;
    AIQ_HIP(noalloc_scratch(&ws, &ws_bytes));
    return eval_impl(m, images, N, schemes, S, nullptr, chunk, top1_base, base_valid, logits, top1, agree, ws, ws_bytes,
                     hip_stream);
}

int32_t aiq_model_shares_prefix(const aiq_model *m)
{
    if (!m) return -1;
    return !m->fused || m->fused_ckpt_floats > 0 ? 1 : 0;
}

aiq_status aiq_eval_shared_workspace_bytes(const aiq_model *m, int32_t S, int32_t chunk, size_t *bytes)
{
    if (!m || !bytes || S < 0 || chunk < 1) return AIQ_INVALID_ARG;
    *bytes = workspace_layout(m, S, chunk, true).total;
    return AIQ_OK;
}

aiq_status aiq_eval_schemes_shared(aiq_model *m, const float *images, int32_t N, const uint8_t *schemes, int32_t S,
                                   const uint8_t *ref_scheme, int32_t chunk, int32_t *top1_base, int32_t base_valid,
                                   float *logits, int32_t *top1, int32_t *agree, void *workspace,
                                   size_t workspace_bytes, void *hip_stream)
{
    if (!m || !ref_scheme) return AIQ_INVALID_ARG;
    return eval_impl(m, images, N, schemes, S, ref_scheme, chunk, top1_base, base_valid, logits, top1, agree,
                     workspace, workspace_bytes, hip_stream);
}

// ---------------------------------------------------------------- one scheme, every node's output

int32_t aiq_model_nodes(const aiq_model *m) { return m ? (int32_t)m->nodes.size() : -1; }

aiq_status aiq_node_output_elems(const aiq_model *m, int32_t node, size_t *elems)
{
    if (!m || !elems || node < 0 || node >= (int32_t)m->nodes.size()) return AIQ_INVALID_ARG;
    *elems = m->nodes[node].out_elems;
    return AIQ_OK;
}

aiq_status aiq_forward_nodes(aiq_model *m, const float *images, int32_t N, const uint8_t *scheme,
                             float *const *node_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!m || N < 0 || !node_out || (m->L > 0 && !scheme)) return AIQ_INVALID_ARG;
    if (N > 0 && (!images || !workspace)) return AIQ_INVALID_ARG;
    for (int i = 0; i < m->L; ++i)
        if (!bits_supported(scheme[i])) return AIQ_UNSUPPORTED_BITS;
    if (m->fused || m->mb_blocks > 0) return AIQ_UNSUPPORTED_LAYER;
    for (const Node &nd : m->nodes)
        if (nd.pooled) return AIQ_UNSUPPORTED_LAYER;
    for (size_t l = 0; l < m->nodes.size(); ++l)
        if (N > 0 && !node_out[l]) return AIQ_INVALID_ARG;
    if (N == 0) return AIQ_OK;
    const WorkspaceLayout wl = workspace_layout(m, 1, N);
    if (workspace_bytes < wl.total) return AIQ_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return AIQ_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = static_cast<char *>(workspace);
    uint8_t *schemes_dev = reinterpret_cast<uint8_t *>(ws + wl.schemes_off);
    if (m->L > 0) AIQ_HIP(upload_bytes(schemes_dev, scheme, (size_t)m->L, st));
    // the layers read the weight bank: fill the slots this scheme uses
    QuantMask mask{};
    bool any = false;
    for (const Node &nd : m->nodes) {
        if (nd.d.scheme_slot < 0) continue;
        const int bi = bits_index(scheme[nd.d.scheme_slot]);
        if (bi > 0) {
            const int ji = nd.job0 + bi - 1;
            mask.word[ji >> 6] |= 1ull << (ji & 63);
            any = true;
        }
    }
    if (any) AIQ_HIP(launch_quantize_batch(m->jobs_dev, m->block_job_dev, m->n_quant_blocks, mask, st));
    m->aq_cur = m->act_quant ? reinterpret_cast<float *>(ws + wl.aq_off) : nullptr;
    const size_t last = m->nodes.size() - 1;
    const HeadOut ho{node_out[last], N, nullptr, reinterpret_cast<int32_t *>(ws + wl.top1_off), N};
    for (size_t l = 0; l < m->nodes.size(); ++l) {
        const Node &nd = m->nodes[l];
        NodeIO io{};
        io.schemes = schemes_dev;
        io.S = 1;
        io.s_total = 1;
        io.in = nd.d.input < 0 ? images : node_out[nd.d.input];
        io.out = node_out[l];
        io.res = nd.d.residual >= 0 ? node_out[nd.d.residual] : nullptr;
        aiq_status rc = launch_node(m, st, ho, l, io, N, 0);
        if (rc != AIQ_OK) return rc;
    }
    return AIQ_OK;
}

// ---------------------------------------------------------------- deployed inference

struct aiq_deployed {
    aiq_model *m = nullptr;
    std::vector<uint8_t> scheme;
    uint8_t *scheme_dev = nullptr;
    struct Layer {
        uint16_t *codes = nullptr; // non-null: this node runs from its integer codes on the bf16 pipe
        int8_t *codes8 = nullptr;  // non-null: activation variant, weights and activations as int8 codes
        float *scales = nullptr;
        CodePlan plan{};
        I8Plan plan8{};
        int bits = 32;
    };
    std::vector<Layer> layer; // per node
    std::vector<char> amax_ok; // per node: its kernel leaves max |output| per image for the int8 layers that read it
    std::vector<void *> allocations;
    int n_code_layers = 0;
    bool resident = false; // the model keeps activations in LDS: the scheme runs on those kernels
    std::vector<MbCodes> mb; // per node; filled at the expand node of every block that runs from integer codes
};

void aiq_deploy_destroy(aiq_deployed *d)
{
    if (!d) return;
    for (void *p : d->allocations) (void)hipFree(p);
    delete d;
}

int32_t aiq_deploy_code_layers(const aiq_deployed *d) { return d ? d->n_code_layers : -1; }

aiq_status aiq_deploy_create(aiq_model *m, const uint8_t *scheme, uint32_t flags, aiq_deployed **out)
{
    if (out) *out = nullptr;
    if (!m || !out || (m->L > 0 && !scheme) || (flags & ~(uint32_t)AIQ_DEPLOY_FP32_MATRIX)) return AIQ_INVALID_ARG;
    for (int i = 0; i < m->L; ++i)
        if (!bits_supported(scheme[i])) return AIQ_UNSUPPORTED_BITS;
    bool resident = m->fused || m->mb_blocks > 0;
    for (const Node &nd : m->nodes) resident = resident || nd.pooled;

    aiq_deployed *d = new (std::nothrow) aiq_deployed();
    if (!d) return AIQ_INVALID_ARG;
    d->m = m;
    d->scheme.assign(scheme, scheme + m->L);
    d->layer.resize(m->nodes.size());
    d->amax_ok.assign(m->nodes.size(), 0);
    auto fail = [&](aiq_status code) {
        aiq_deploy_destroy(d);
        return code;
    };
    auto alloc = [&](void **p, size_t bytes) {
        if (!hip_ok(hipMalloc(p, std::max<size_t>(bytes, 256)))) return false;
        d->allocations.push_back(*p);
        return true;
    };
    if (resident) {
        // A model whose activations stay in LDS (whole CIFAR-style ResNets, inverted-residual blocks) is
        // deployed on those kernels, the scheme being the one "candidate" of a scoring call: the layer-by-layer
        // integer-code kernels work through HBM and are slower than that for such models.  The weight bank
        // slots are filled by the forward call.  Inverted-residual blocks whose expand or project layer carries
        // at most eight bits run on the block kernel that takes those matrix products from integer codes (a
        // 16- or 32-bit layer beside one keeps the fp32 MFMA), and so does a last 1x1 layer of at most eight bits that forms the classifier's pooling in its
        // epilogue; what is prepared here are those codes and scales.
        d->resident = true;
        d->mb.resize(m->nodes.size());
        // layers to prepare: node, k step of the operand layout, rows the packed buffer is padded to,
        // destination (expand / pooled layer: codes_e of its own node; project: codes_p of the block's expand node)
        struct CodeJob {
            size_t node, owner;
            int kstep, tiles;
            bool project;
        };
        std::vector<CodeJob> jobs;
        if (!m->act_quant && !(flags & AIQ_DEPLOY_FP32_MATRIX))
            for (size_t l = 0; l < m->nodes.size(); ++l) {
                const Node &e = m->nodes[l];
                if (e.mb_role == 1 && l + 2 < m->nodes.size()) {
                    const Node &pj = m->nodes[l + 2];
                    const bool ec = e.d.scheme_slot >= 0 && scheme[e.d.scheme_slot] <= 8;
                    const bool pc = pj.d.scheme_slot >= 0 && scheme[pj.d.scheme_slot] <= 8;
                    if (!mbconv_codes_supported(e.mb_shape, ec, pc)) continue;
                    if (ec) jobs.push_back({l, l, 32, (e.d.cout + 15) / 16, false});
                    if (pc) jobs.push_back({l + 2, l, 16, (pj.d.cout + 15) / 16, true});
                } else if (e.pooled && e.d.scheme_slot >= 0 && scheme[e.d.scheme_slot] <= 8) {
                    int cg = 0, groups = 0;
                    if (!pooled_codes_plan(e.d.cin, e.d.cout, &cg, &groups)) continue;
                    jobs.push_back({l, l, 32, cg * groups, false});
                }
            }
        if (jobs.empty()) {
            *out = d;
            return AIQ_OK;
        }
        size_t tmp_elems = 0;
        for (const CodeJob &cj : jobs) tmp_elems = std::max(tmp_elems, (size_t)m->nodes[cj.node].d.cout * m->nodes[cj.node].k);
        void *tmp_codes = nullptr, *tmp_out = nullptr;
        bool ok = hip_ok(hipMalloc(&tmp_codes, tmp_elems * sizeof(int32_t))) && hip_ok(hipMalloc(&tmp_out, tmp_elems * sizeof(float)));
        for (size_t ji = 0; ok && ji < jobs.size(); ++ji) {
            const CodeJob &cj = jobs[ji];
            const Node &nd = m->nodes[cj.node];
            MbCodes &mc = d->mb[cj.owner];
            const size_t code_elems = (size_t)cj.tiles * ((nd.k + cj.kstep - 1) / cj.kstep) * 64 * (cj.kstep / 4);
            uint16_t *&codes = cj.project ? mc.codes_p : mc.codes_e;
            float *&scales = cj.project ? mc.scale_p : mc.scale_e;
            ok = alloc(reinterpret_cast<void **>(&codes), code_elems * sizeof(uint16_t)) &&
                 alloc(reinterpret_cast<void **>(&scales), (size_t)nd.d.cout * sizeof(float)) &&
                 hip_ok(hipMemset(codes, 0, code_elems * sizeof(uint16_t)));
            if (!ok) break;
            QuantJob j = m->jobs_host[nd.job0 + bits_index(scheme[nd.d.scheme_slot]) - 1];
            j.out = static_cast<float *>(tmp_out);
            j.layout = kLayoutPlain;
            j.scales = scales;
            j.codes = static_cast<int32_t *>(tmp_codes);
            ok = hip_ok(launch_quantize_single(j, nullptr)) &&
                 hip_ok(launch_pack_mb_codes(j.codes, codes, nd.d.cout, nd.k, cj.kstep, nullptr));
            ++d->n_code_layers;
        }
        ok = hip_ok(hipDeviceSynchronize()) && ok;
        if (tmp_codes) (void)hipFree(tmp_codes);
        if (tmp_out) (void)hipFree(tmp_out);
        if (!ok) return fail(AIQ_DEVICE_ERROR);
        *out = d;
        return AIQ_OK;
    }
    if (!alloc(reinterpret_cast<void **>(&d->scheme_dev), (size_t)std::max(m->L, 1))) return fail(AIQ_DEVICE_ERROR);
    if (m->L && !hip_ok(hipMemcpy(d->scheme_dev, scheme, (size_t)m->L, hipMemcpyHostToDevice)))
        return fail(AIQ_DEVICE_ERROR);

    // fp32-path layers read the weight bank: fill the slots this scheme uses (their content
    // depends on nothing but the weights, so other calls on the model rewrite the same values)
    QuantMask mask{};
    bool any = false;
    size_t tmp_elems = 0;
    for (size_t l = 0; l < m->nodes.size(); ++l) {
        const Node &nd = m->nodes[l];
        if (nd.d.scheme_slot < 0) continue;
        const int bits = scheme[nd.d.scheme_slot], bi = bits_index(bits);
        if (bi == 0) continue;
        const bool dense = !(flags & AIQ_DEPLOY_FP32_MATRIX) && bits <= 8 && nd.d.kind == 0 && nd.d.input >= 0 &&
                           nd.layout == kLayoutMfma;
        const bool on_codes = dense && !m->act_quant && plan_code_conv(nd, d->layer[l].plan);
        const bool on_int8 = dense && m->act_quant && nd.in_elems % 16 == 0 && plan_i8_conv(nd, d->layer[l].plan8);
        d->layer[l].bits = bits;
        if (on_int8) {
            const I8Plan &p = d->layer[l].plan8;
            const size_t code_bytes = (size_t)p.cout_tiles * nd.d.kh * nd.d.kw * p.CBK * 1024;
            if (!alloc(reinterpret_cast<void **>(&d->layer[l].codes8), code_bytes) ||
                !alloc(reinterpret_cast<void **>(&d->layer[l].scales), (size_t)nd.d.cout * sizeof(float)) ||
                !hip_ok(hipMemset(d->layer[l].codes8, 0, code_bytes)))
                return fail(AIQ_DEVICE_ERROR);
            tmp_elems = std::max(tmp_elems, (size_t)nd.d.cout * nd.k);
            ++d->n_code_layers;
            // the 32 pixels of an output tile lie in one image: one maximum per tile
            d->amax_ok[l] = p.G == 1 || (nd.hout * nd.wout) % 32 == 0;
        } else if (on_codes) {
            const CodePlan &p = d->layer[l].plan;
            const size_t code_elems = (size_t)p.cout_tiles * nd.d.kh * nd.d.kw * p.CB * 512;
            if (!alloc(reinterpret_cast<void **>(&d->layer[l].codes), code_elems * sizeof(uint16_t)) ||
                !alloc(reinterpret_cast<void **>(&d->layer[l].scales), (size_t)nd.d.cout * sizeof(float)) ||
                !hip_ok(hipMemset(d->layer[l].codes, 0, code_elems * sizeof(uint16_t))))
                return fail(AIQ_DEVICE_ERROR);
            tmp_elems = std::max(tmp_elems, (size_t)nd.d.cout * nd.k);
            ++d->n_code_layers;
        } else {
            const int ji = nd.job0 + bi - 1;
            mask.word[ji >> 6] |= 1ull << (ji & 63);
            any = true;
        }
    }
    if (any && !hip_ok(launch_quantize_batch(m->jobs_dev, m->block_job_dev, m->n_quant_blocks, mask, nullptr)))
        return fail(AIQ_DEVICE_ERROR);
    if (d->n_code_layers) {
        // quantizer -> integer codes and scales -> codes in the matrix pipe's operand order
        void *tmp_codes = nullptr, *tmp_out = nullptr;
        bool ok = hip_ok(hipMalloc(&tmp_codes, tmp_elems * sizeof(int32_t))) &&
                  hip_ok(hipMalloc(&tmp_out, tmp_elems * sizeof(float)));
        for (size_t l = 0; ok && l < m->nodes.size(); ++l) {
            const Node &nd = m->nodes[l];
            if (!d->layer[l].codes && !d->layer[l].codes8) continue;
            QuantJob j = m->jobs_host[nd.job0 + bits_index(scheme[nd.d.scheme_slot]) - 1];
            j.out = static_cast<float *>(tmp_out);
            j.layout = kLayoutPlain;
            j.scales = d->layer[l].scales;
            j.codes = static_cast<int32_t *>(tmp_codes);
            ok = hip_ok(launch_quantize_single(j, nullptr)) &&
                 hip_ok(d->layer[l].codes8
                            ? launch_pack_codes_i8(j.codes, d->layer[l].codes8, nd.d.cout, nd.d.cin, nd.d.kh * nd.d.kw, nullptr)
                            : launch_pack_codes(j.codes, d->layer[l].codes, nd.d.cout, nd.d.cin, nd.d.kh * nd.d.kw, nullptr));
        }
        ok = hip_ok(hipDeviceSynchronize()) && ok;
        if (tmp_codes) (void)hipFree(tmp_codes);
        if (tmp_out) (void)hipFree(tmp_out);
        if (!ok) return fail(AIQ_DEVICE_ERROR);
    } else if (!hip_ok(hipDeviceSynchronize())) {
        return fail(AIQ_DEVICE_ERROR);
    }
    *out = d;
    return AIQ_OK;
}

aiq_status aiq_deploy_workspace_bytes(const aiq_deployed *d, int32_t chunk, size_t *bytes)
{
    if (!d || !bytes || chunk < 1) return AIQ_INVALID_ARG;
    *bytes = workspace_layout(d->m, d->resident ? 1 : 0, chunk).total;
    return AIQ_OK;
}

namespace {

// One node of a deployed scheme on n images: from integer codes where the layer has them, else on the
// scoring kernels.  aq: the activation variant's scratch area (room for the fp32 copy of the largest
// input tensor of a scheme layer, per image); the int8 path keeps its activation codes in the first
// quarter of it and the images' scales behind them.
aiq_status deploy_node(aiq_deployed *d, hipStream_t st, const HeadOut &ho, size_t l, const NodeIO &io, int n, int n0,
                       char *aq, uint32_t *amax, size_t amax_stride)
{
    aiq_model *m = d->m;
    const Node &nd = m->nodes[l];
    const aiq_deployed::Layer &cl = d->layer[l];
    const aiq_layer_desc &ld = nd.d;
    if (cl.codes8) {
        const I8Plan &p = cl.plan8;
        int8_t *xcodes = reinterpret_cast<int8_t *>(aq);
        float *xscale = reinterpret_cast<float *>(aq + align_up(nd.in_elems * (size_t)n, 256));
        {
            ProfScope ps(m, st, AIQ_K_QUANTIZE, 0.0, 5.0 * nd.in_elems * n); // one read, one byte written per value
            const uint32_t *in_amax = ld.input >= 0 && d->amax_ok[ld.input] ? amax + amax_stride * ld.input : nullptr;
            AIQ_HIP(launch_act_codes(io.in, in_amax, xcodes, xscale, n, (int)nd.in_elems, cl.bits, st));
        }
        I8ConvArgs a{};
        a.in = xcodes;
        a.xscale = xscale;
        a.out = io.out;
        a.res = io.res;
        a.bias = nd.bias;
        a.codes = cl.codes8;
        a.scales = cl.scales;
        a.amax_out = d->amax_ok[l] ? amax + amax_stride * l : nullptr;
        a.N = n;
        a.Hin = ld.hin;
        a.Win = ld.win;
        a.Cin = ld.cin;
        a.Hout = nd.hout;
        a.Wout = nd.wout;
        a.Cout = ld.cout;
        a.act = ld.act;
        a.R = p.R;
        a.G = p.G;
        a.regions_per_image = p.regions_per_image;
        a.CBK = p.CBK;
        a.CKB = p.CKB;
        a.RIN = p.RIN;
        a.LW = p.LW;
        a.PSB = p.PSB;
        a.wave_px_split = p.wave_px_split;
        a.cout_tiles = p.cout_tiles;
        a.tiles_per_wg = p.tiles_per_wg;
        a.code_off = p.code_off;
        a.div_rin = make_fastdiv(p.RIN);
        a.div_wout = make_fastdiv(nd.wout);
        a.div_rw = make_fastdiv(p.R * nd.wout);
        a.div_per_row = make_fastdiv(p.LW * 2 * p.CKB);
        a.div_pximg = make_fastdiv(nd.hout * nd.wout);
        a.total_regions = p.G > 1 ? (n + p.G - 1) / p.G : n * p.regions_per_image;
        // single-pass layers: a workgroup keeps the weight codes for several regions, as long as about a
        // thousand workgroups remain
        a.RPW = p.CBK <= p.CKB ? std::max(1, std::min(8, a.total_regions / 1024)) : 1;
        const unsigned gx = (unsigned)((a.total_regions + a.RPW - 1) / a.RPW);
        ProfScope ps(m, st, AIQ_K_CONV_CODES, nd.flops_per_image * n,
                     ((double)nd.in_elems + 4.0 * nd.out_elems * (ld.residual >= 0 ? 2 : 1)) * n);
        AIQ_HIP(launch_conv_i8(a, ld.kh, ld.stride, p.nt, p.lds_bytes, dim3(gx, p.grid_y, 1), st));
        return AIQ_OK;
    }
    if (!cl.codes) return launch_node(m, st, ho, l, io, n, n0);
    const CodePlan &p = cl.plan;
    CodeConvArgs a{};
    a.in = io.in;
    a.out = io.out;
    a.res = io.res;
    a.bias = nd.bias;
    a.codes = cl.codes;
    a.scales = cl.scales;
    a.N = n;
    a.Hin = ld.hin;
    a.Win = ld.win;
    a.Cin = ld.cin;
    a.Hout = nd.hout;
    a.Wout = nd.wout;
    a.Cout = ld.cout;
    a.act = ld.act;
    a.R = p.R;
    a.G = p.G;
    a.regions_per_image = p.regions_per_image;
    a.CB = p.CB;
    a.CKC = p.CKC;
    a.RIN = p.RIN;
    a.LW = p.LW;
    a.PSU = p.PSU;
    a.wave_px_split = p.wave_px_split;
    a.cout_tiles = p.cout_tiles;
    a.tiles_per_wg = p.nt * (4 / p.wave_px_split);
    a.code_off = p.code_off;
    a.div_rin = make_fastdiv(p.RIN);
    a.div_wout = make_fastdiv(nd.wout);
    a.div_rw = make_fastdiv(p.R * nd.wout);
    a.div_per_row = make_fastdiv(p.LW * (p.CKC / 8));
    const unsigned gx = p.G > 1 ? (unsigned)((n + p.G - 1) / p.G) : (unsigned)(n * p.regions_per_image);
    ProfScope ps(m, st, AIQ_K_CONV_CODES, nd.flops_per_image * n, nd.act_bytes_per_image * n);
    AIQ_HIP(launch_conv_codes(a, ld.kh, ld.stride, p.nt, p.stage_items, p.mt, p.lds_bytes, dim3(gx, p.grid_y, 1), st));
    return AIQ_OK;
}

} // namespace

aiq_status aiq_deploy_forward(aiq_deployed *d, const float *images, int32_t N, int32_t chunk, float *logits,
                              int32_t *top1, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!d || N < 0 || chunk < 1) return AIQ_INVALID_ARG;
    if (N > 0 && (!images || !top1 || !workspace)) return AIQ_INVALID_ARG;
    if (N == 0) return AIQ_OK;
    aiq_model *m = d->m;
    chunk = std::min(chunk, N);
    if (d->resident) {
        m->mb_codes_cur = d->n_code_layers ? d->mb.data() : nullptr;
        m->mb_scheme_cur = d->scheme.data();
        const aiq_status rc = eval_impl(m, images, N, d->scheme.data(), 1, nullptr, chunk, nullptr, 1, logits, top1, nullptr,
                                        workspace, workspace_bytes, hip_stream, nullptr, false);
        m->mb_codes_cur = nullptr;
        m->mb_scheme_cur = nullptr;
        return rc;
    }
    const WorkspaceLayout wl = workspace_layout(m, 0, chunk);
    if (workspace_bytes < wl.total) return AIQ_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return AIQ_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = static_cast<char *>(workspace);
    auto buf_ptr = [&](int b) { return reinterpret_cast<float *>(ws + wl.act_off + wl.buf_stride * b); };
    m->aq_cur = m->act_quant ? reinterpret_cast<float *>(ws + wl.aq_off) : nullptr;
    const HeadOut ho{logits, N, top1, nullptr, chunk};
    uint32_t *amax = reinterpret_cast<uint32_t *>(ws + wl.amax_off);
    const bool any_amax = std::any_of(d->amax_ok.begin(), d->amax_ok.end(), [](char c) { return c != 0; });
    for (int n0 = 0; n0 < N; n0 += chunk) {
        const int n = std::min(chunk, N - n0);
        if (any_amax) AIQ_HIP(launch_fill_i32(reinterpret_cast<int32_t *>(amax), 0, m->nodes.size() * (size_t)chunk, st));
        for (size_t l = 0; l < m->nodes.size(); ++l) {
            const Node &nd = m->nodes[l];
            NodeIO io{};
            io.schemes = d->scheme_dev;
            io.S = 1;
            io.s_total = 1;
            io.in = nd.d.input < 0 ? images + (size_t)n0 * nd.in_elems : buf_ptr(m->nodes[nd.d.input].buf);
            io.out = nd.buf >= 0 ? buf_ptr(nd.buf) : nullptr;
            io.res = nd.d.residual >= 0 ? buf_ptr(m->nodes[nd.d.residual].buf) : nullptr;
            aiq_status rc = deploy_node(d, st, ho, l, io, n, n0, ws + wl.aq_off, amax, (size_t)chunk);
            if (rc != AIQ_OK) return rc;
        }
    }
    return AIQ_OK;
}

aiq_status aiq_deploy_forward_nodes(aiq_deployed *d, const float *images, int32_t N, float *const *node_out,
                                    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!d || N < 0 || !node_out) return AIQ_INVALID_ARG;
    if (N > 0 && (!images || !workspace)) return AIQ_INVALID_ARG;
    aiq_model *m = d->m;
    if (d->resident) return AIQ_UNSUPPORTED_LAYER;
    for (size_t l = 0; l < m->nodes.size(); ++l)
        if (N > 0 && !node_out[l]) return AIQ_INVALID_ARG;
    if (N == 0) return AIQ_OK;
    const WorkspaceLayout wl = workspace_layout(m, 0, N);
    if (workspace_bytes < wl.total) return AIQ_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return AIQ_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = static_cast<char *>(workspace);
    m->aq_cur = m->act_quant ? reinterpret_cast<float *>(ws + wl.aq_off) : nullptr;
    const size_t last = m->nodes.size() - 1;
    const HeadOut ho{node_out[last], N, nullptr, reinterpret_cast<int32_t *>(ws + wl.top1_off), N};
    uint32_t *amax = reinterpret_cast<uint32_t *>(ws + wl.amax_off);
    if (m->act_quant) AIQ_HIP(launch_fill_i32(reinterpret_cast<int32_t *>(amax), 0, m->nodes.size() * (size_t)N, st));
    for (size_t l = 0; l < m->nodes.size(); ++l) {
        const Node &nd = m->nodes[l];
        NodeIO io{};
        io.schemes = d->scheme_dev;
        io.S = 1;
        io.s_total = 1;
        io.in = nd.d.input < 0 ? images : node_out[nd.d.input];
        io.out = node_out[l];
        io.res = nd.d.residual >= 0 ? node_out[nd.d.residual] : nullptr;
        aiq_status rc = deploy_node(d, st, ho, l, io, N, 0, ws + wl.aq_off, amax, (size_t)N);
        if (rc != AIQ_OK) return rc;
    }
    return AIQ_OK;
}

namespace {

// Shared state of one search run: device buffers carved out of the workspace and the
// scoring of a batch of candidate schemes.
struct SearchCtx {
    aiq_model *m;
    const aiq_layer_desc *layers;
    int32_t n_layers;
    const float *images;
    int32_t N, chunk, L;
    const aiq_search_params *p;
    hipStream_t st;
    int32_t *top1_base, *agree_dev;
    void *eval_ws;
    size_t eval_ws_bytes;
    int32_t s_max;
    bool base_valid = false;
    std::vector<int32_t> agree_host;
    CkptCache ckpt_cache; // the workspace is this run's alone: checkpoints stay good from step to step

    double ai(const uint8_t *q, aiq_status *err) const
    {
        double v = 0.0;
        aiq_status st_ = aiq_layer_ai_ex(layers, n_layers, q, L, p->batch, m->act_quant ? 1 : 0, nullptr, nullptr, &v);
        if (st_ != AIQ_OK) *err = st_;
        return v;
    }
    double loss(double ai_v, int32_t agree) const
    {
        const double acc_loss = N > 0 ? 100.0 * (1.0 - (double)agree / (double)N) : 0.0;
        return -p->lambda * ai_v + (1.0 - p->lambda) * acc_loss;
    }
    // scores S schemes (host [S][L]); agree_host[0..S) filled on return.  With prefix sharing the
    // schemes of one batch resume from the forward pass of ref (host [L]), the scheme they all
    // were derived from by changing one layer.
    aiq_status score(const std::vector<uint8_t> &schemes, int32_t S, const uint8_t *ref)
    {
        if (S > s_max) return AIQ_WORKSPACE_TOO_SMALL;
        aiq_status rc = eval_impl(m, images, N, schemes.data(), S, p->share_prefix ? ref : nullptr, chunk, top1_base,
                                  base_valid ? 1 : 0, nullptr, nullptr, agree_dev, eval_ws, eval_ws_bytes, st,
                                  &ckpt_cache);
        if (rc != AIQ_OK) return rc;
        base_valid = true;
        agree_host.assign(S, 0);
        if (S > 0)
            AIQ_HIP(hipMemcpyAsync(agree_host.data(), agree_dev, sizeof(int32_t) * S, hipMemcpyDeviceToHost, st));
        AIQ_HIP(hipStreamSynchronize(st));
        return AIQ_OK;
    }
};

struct SearchLayout {
    size_t top1_off, agree_off, eval_off, total;
    int32_t s_max;
};

SearchLayout search_layout(const aiq_model *m, int32_t N, int32_t chunk, int32_t n_bits)
{
    SearchLayout l{};
    l.s_max = std::max(1, m->L * std::max(1, n_bits - 1));
    size_t off = 0;
    l.top1_off = off;
    off = align_up(off + sizeof(int32_t) * (size_t)std::max(N, 1), 256);
    l.agree_off = off;
    off = align_up(off + sizeof(int32_t) * (size_t)l.s_max, 256);
    l.eval_off = off;
    off += workspace_layout(m, l.s_max, std::min(chunk, std::max(N, 1)), true).total;
    l.total = off;
    return l;
}

aiq_status search_setup(SearchCtx &c, aiq_model *m, const aiq_layer_desc *layers, int32_t n_layers,
                        const float *images, int32_t N, int32_t chunk, const aiq_search_params *p, void *workspace,
                        size_t workspace_bytes, void *hip_stream, uint8_t *scheme_out, int32_t *n_trace)
{
    if (!m || !layers || !p || !scheme_out || !n_trace || N < 1 || chunk < 1 || !images || !workspace)
        return AIQ_INVALID_ARG;
    if (n_layers != (int32_t)m->nodes.size()) return AIQ_SHAPE_MISMATCH;
    if (!(p->lambda >= 0.0 && p->lambda <= 1.0) || p->n_bits < 1 || p->n_bits > 8 || p->batch < 1 || p->max_iters < 0)
        return AIQ_INVALID_ARG;
    for (int i = 0; i < p->n_bits; ++i) {
        if (!bits_supported(p->bits[i])) return AIQ_UNSUPPORTED_BITS;
        if (i > 0 && p->bits[i] >= p->bits[i - 1]) return AIQ_INVALID_ARG;
    }
    if (p->bits[0] != 32) return AIQ_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l)
        if (std::memcmp(&layers[l], &m->nodes[l].d, sizeof(aiq_layer_desc)) != 0) return AIQ_SHAPE_MISMATCH;
    const SearchLayout lay = search_layout(m, N, chunk, p->n_bits);
    if (workspace_bytes < lay.total) return AIQ_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return AIQ_INVALID_ARG;
    char *ws = static_cast<char *>(workspace);
    c.m = m;
    c.layers = layers;
    c.n_layers = n_layers;
    c.images = images;
    c.N = N;
    c.chunk = chunk;
    c.L = m->L;
    c.p = p;
    c.st = (hipStream_t)hip_stream;
    c.top1_base = reinterpret_cast<int32_t *>(ws + lay.top1_off);
    c.agree_dev = reinterpret_cast<int32_t *>(ws + lay.agree_off);
    c.eval_ws = ws + lay.eval_off;
    c.eval_ws_bytes = workspace_bytes - lay.eval_off;
    c.s_max = lay.s_max;
    c.ckpt_cache.s_layout = lay.s_max;
    return AIQ_OK;
}

void push_trace(aiq_search_step *trace, int32_t cap, int32_t &n, int32_t layer, int32_t bits, int32_t agree,
                int32_t sweep, double loss, double ai)
{
    if (trace && n < cap) trace[n] = aiq_search_step{layer, bits, agree, sweep, loss, ai};
    ++n;
}

} // namespace

aiq_status aiq_search_workspace_bytes(const aiq_model *m, int32_t N, int32_t chunk, int32_t n_bits, size_t *bytes)
{
    if (!m || !bytes || N < 1 || chunk < 1 || n_bits < 1 || n_bits > 8) return AIQ_INVALID_ARG;
    *bytes = search_layout(m, N, chunk, n_bits).total;
    return AIQ_OK;
}

aiq_status aiq_search_greedy(aiq_model *m, const aiq_layer_desc *layers, int32_t n_layers, const float *images,
                             int32_t N, int32_t chunk, const aiq_search_params *params, void *workspace,
                             size_t workspace_bytes, void *hip_stream, uint8_t *scheme_out, aiq_search_step *trace,
                             int32_t trace_cap, int32_t *n_trace)
{
    SearchCtx c;
    aiq_status rc = search_setup(c, m, layers, n_layers, images, N, chunk, params, workspace, workspace_bytes,
                                 hip_stream, scheme_out, n_trace);
    if (rc != AIQ_OK) return rc;
    const int L = c.L, nb = params->n_bits;
    std::vector<uint8_t> q(L, params->bits[0]);
    aiq_status err = AIQ_OK;
    // start: the all-FP32 scheme agrees with itself on every image
    std::vector<uint8_t> batch(q);
    if ((rc = c.score(batch, 1, nullptr)) != AIQ_OK) return rc;
    double cur_ai = c.ai(q.data(), &err);
    double cur = c.loss(cur_ai, c.agree_host[0]);
    int32_t nt = 0;
    push_trace(trace, trace_cap, nt, -1, params->bits[0], c.agree_host[0], 0, cur, cur_ai);
    const int iters = params->max_iters > 0 ? params->max_iters : L;
    for (int it = 1; it <= iters; ++it) {
        std::vector<std::pair<int, int>> moves;
        batch.clear();
        for (int i = 0; i < L; ++i) {
            if (params->only_fp32_layers && q[i] != params->bits[0]) continue;
            for (int b = 0; b < nb; ++b)
                if (params->bits[b] < q[i]) {
                    moves.emplace_back(i, params->bits[b]);
                    batch.insert(batch.end(), q.begin(), q.end());
                    batch[batch.size() - L + i] = params->bits[b];
                }
        }
        if (moves.empty()) break;
        if ((rc = c.score(batch, (int32_t)moves.size(), q.data())) != AIQ_OK) return rc;
        int best = -1;
        double best_delta = 0.0, best_ai = 0.0;
        for (size_t k = 0; k < moves.size(); ++k) {
            const double ai_v = c.ai(batch.data() + k * L, &err);
            const double delta = c.loss(ai_v, c.agree_host[k]) - cur;
            if (best < 0 || delta < best_delta) {
                best = (int)k;
                best_delta = delta;
                best_ai = ai_v;
            }
        }
        if (err != AIQ_OK) return err;
        if (!(best_delta < 0.0)) break;
        q[moves[best].first] = (uint8_t)moves[best].second;
        cur += best_delta;
        push_trace(trace, trace_cap, nt, moves[best].first, moves[best].second, c.agree_host[best], it, cur, best_ai);
    }
    std::memcpy(scheme_out, q.data(), L);
    *n_trace = nt;
    return err;
}

aiq_status aiq_search_coordinate_descent(aiq_model *m, const aiq_layer_desc *layers, int32_t n_layers,
                                         const float *images, int32_t N, int32_t chunk,
                                         const aiq_search_params *params, void *workspace, size_t workspace_bytes,
                                         void *hip_stream, uint8_t *scheme_out, aiq_search_step *trace,
                                         int32_t trace_cap, int32_t *n_trace)
{
    SearchCtx c;
    aiq_status rc = search_setup(c, m, layers, n_layers, images, N, chunk, params, workspace, workspace_bytes,
                                 hip_stream, scheme_out, n_trace);
    if (rc != AIQ_OK) return rc;
    const int L = c.L, nb = params->n_bits;
    std::vector<uint8_t> q(L, params->bits[0]);
    aiq_status err = AIQ_OK;
    std::vector<uint8_t> batch(q);
    if ((rc = c.score(batch, 1, nullptr)) != AIQ_OK) return rc;
    double cur_ai = c.ai(q.data(), &err);
    double cur = c.loss(cur_ai, c.agree_host[0]);
    int32_t nt = 0;
    push_trace(trace, trace_cap, nt, -1, params->bits[0], c.agree_host[0], 0, cur, cur_ai);
    const int sweeps = params->max_iters > 0 ? params->max_iters : 50;
    for (int sweep = 1; sweep <= sweeps; ++sweep) {
        bool updated = false;
        for (int i = 0; i < L && nb > 1; ++i) {
            std::vector<int> others;
            batch.clear();
            for (int b = 0; b < nb; ++b)
                if (params->bits[b] != q[i]) {
                    others.push_back(params->bits[b]);
                    batch.insert(batch.end(), q.begin(), q.end());
                    batch[batch.size() - L + i] = params->bits[b];
                }
            if ((rc = c.score(batch, (int32_t)others.size(), q.data())) != AIQ_OK) return rc;
            int best = -1;
            double best_val = 0.0, best_ai = 0.0;
            for (size_t k = 0; k < others.size(); ++k) {
                const double ai_v = c.ai(batch.data() + k * L, &err);
                const double v = c.loss(ai_v, c.agree_host[k]);
                if (best < 0 || v < best_val) {
                    best = (int)k;
                    best_val = v;
                    best_ai = ai_v;
                }
            }
            if (err != AIQ_OK) return err;
            if (best >= 0 && best_val < cur) {
                q[i] = (uint8_t)others[best];
                cur = best_val;
                updated = true;
                push_trace(trace, trace_cap, nt, i, others[best], c.agree_host[best], sweep, cur, best_ai);
            }
        }
        if (!updated) break;
    }
    std::memcpy(scheme_out, q.data(), L);
    *n_trace = nt;
    return err;
}

aiq_status aiq_sensitivity_workspace_bytes(const aiq_model *m, int32_t N, int32_t chunk, int32_t n_bits, size_t *bytes)
{
    if (!m || !bytes || N < 1 || chunk < 1 || n_bits < 1 || n_bits > 5) return AIQ_INVALID_ARG;
    *bytes = search_layout(m, N, chunk, n_bits + 1).total; // as a search over {32} + bits: L * n_bits schemes at most
    return AIQ_OK;
}

aiq_status aiq_layer_sensitivity(aiq_model *m, const float *images, int32_t N, int32_t chunk, const uint8_t *bits,
                                 int32_t n_bits, void *workspace, size_t workspace_bytes, void *hip_stream,
                                 int32_t *agree_out)
{
    if (!m || !images || !bits || !workspace || !agree_out || N < 1 || chunk < 1 || n_bits < 1 || n_bits > 5)
        return AIQ_INVALID_ARG;
    for (int k = 0; k < n_bits; ++k)
        if (!bits_supported(bits[k]) || bits[k] == 32) return AIQ_UNSUPPORTED_BITS;
    const SearchLayout lay = search_layout(m, N, chunk, n_bits + 1);
    if (workspace_bytes < lay.total) return AIQ_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return AIQ_INVALID_ARG;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = (hipStream_t)hip_stream;
    int32_t *top1_base = reinterpret_cast<int32_t *>(ws + lay.top1_off);
    int32_t *agree_dev = reinterpret_cast<int32_t *>(ws + lay.agree_off);
    const int L = m->L, S = L * n_bits;
    std::vector<uint8_t> schemes((size_t)S * L, 32);
    for (int i = 0; i < L; ++i)
        for (int k = 0; k < n_bits; ++k) schemes[((size_t)i * n_bits + k) * L + i] = bits[k];
    // every candidate differs from the all-FP32 scheme in one layer: share its forward prefix
    const std::vector<uint8_t> ref(L, 32);
    aiq_status rc = eval_impl(m, images, N, schemes.data(), S, ref.data(), chunk, top1_base, 0, nullptr, nullptr,
                              agree_dev, ws + lay.eval_off, workspace_bytes - lay.eval_off, st);
    if (rc != AIQ_OK) return rc;
    AIQ_HIP(hipMemcpyAsync(agree_out, agree_dev, sizeof(int32_t) * S, hipMemcpyDeviceToHost, st));
    AIQ_HIP(hipStreamSynchronize(st));
    return AIQ_OK;
}

aiq_status aiq_profile_enable(aiq_model *m, int32_t on)
{
    if (!m) return AIQ_INVALID_ARG;
    if (on && m->ev_pool.empty()) {
        const size_t want = 16384;
        m->ev_pool.reserve(want);
        for (size_t i = 0; i < want; ++i) {
            hipEvent_t e;
            AIQ_HIP(hipEventCreate(&e));
            m->ev_pool.push_back(e);
        }
    }
    m->prof_on = on != 0;
    return AIQ_OK;
}

aiq_status aiq_profile_read(aiq_model *m, int32_t cls, int64_t *launches, double *total_ms, double *flops,
                            double *bytes)
{
    if (!m || cls < 0 || cls >= AIQ_K_CLASSES) return AIQ_INVALID_ARG;
    int64_t cnt = 0;
    double ms = 0.0, fl = 0.0, by = 0.0;
    std::vector<ProfRec> keep;
    for (const ProfRec &r : m->prof) {
        if (r.cls != cls) {
            keep.push_back(r);
            continue;
        }
        AIQ_HIP(hipEventSynchronize(r.stop));
        float t = 0.0f;
        AIQ_HIP(hipEventElapsedTime(&t, r.start, r.stop));
        ++cnt;
        ms += t;
        fl += r.flops;
        by += r.bytes;
    }
    m->prof.swap(keep);
    if (m->prof.empty()) m->ev_used = 0;
    if (launches) *launches = cnt;
    if (total_ms) *total_ms = ms;
    if (flops) *flops = fl;
    if (bytes) *bytes = by;
    return AIQ_OK;
}

} // extern "C"
