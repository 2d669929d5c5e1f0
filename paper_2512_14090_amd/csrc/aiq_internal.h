// Internal declarations shared by the host planner (aiq_host.cpp) and the gfx950
// kernels (aiq_kernels.hip).  Not part of the public boundary.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace aiq {

// Bit-width alphabet in bank order: index 0 is the FP32 copy.
constexpr int kNumBits = 6;
__host__ __device__ inline int bits_index(int bits)
{
    switch (bits) {
    case 32: return 0;
    case 16: return 1;
    case 8: return 2;
    case 6: return 3;
    case 4: return 4;
    case 2: return 5;
    default: return -1;
    }
}
constexpr int kBitsOfIndex[kNumBits] = {32, 16, 8, 6, 4, 2};

// Weight layouts the quantizer can write.
enum WeightLayout : int32_t {
    kLayoutPlain = 0,   // [cout][k]
    kLayoutMfma = 1,    // dense convolution: [cout/16][tap][cin/16][64 lanes][4], zero padded
    kLayoutTapMajor = 2, // depthwise: [tap][channels]
    kLayoutStem = 3,     // dense convolution with cin <= 4: [cout/16][tap][64 lanes], lane = ci*16 + co
    kLayoutMfmaKx = 4    // dense 3x3 convolution: [cout/16][kx][cin/16][ky][64 lanes][4] (column-major taps)
};

// One (weight matrix, bit-width) quantization job.
struct QuantJob {
    const float *w;   // [cout][k] source
    float *out;       // destination in `layout`
    float *scales;    // [cout] or nullptr
    int32_t *codes;   // [cout][k] or nullptr
    int32_t cout, k;
    int32_t bits;
    int32_t layout;
    int32_t taps;     // kh*kw (mfma / tap-major layouts)
    int32_t cblocks;  // ceil(cin/16) (mfma layout)
    int32_t first_block; // first grid block of this job in a batched launch
    int32_t pad_;
    const uint32_t *tensor_amax; // per-tensor scale: bit pattern of the whole matrix's largest |w|; nullptr: per channel
};

constexpr int kQuantChannelsPerBlock = 4; // one wavefront per output channel
constexpr int kMaxQuantJobs = 512;        // bits of QuantMask

struct QuantMask {
    uint64_t word[kMaxQuantJobs / 64];
};

// Exact division of small non-negative integers by a runtime constant:
// q = (n * magic) >> 32 with magic = floor(2^32 / d) + 1 is exact for n * d < 2^32.
struct FastDiv {
    uint32_t d, magic;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    f.magic = d <= 1 ? 0u : (uint32_t)((0x100000000ull / d) + 1ull);
    return f;
}
#ifdef __HIPCC__
__device__ inline uint32_t fd_div(uint32_t n, FastDiv f) { return f.d <= 1 ? n : __umulhi(n, f.magic); }
#endif

// Arguments of the dense (3x3 / 1x1) MFMA convolution.
struct ConvArgs {
    const float *in;          // [S?][N][Hin][Win][Cin]
    float *out;               // [S][N][Hout][Wout][Cout]
    const float *res;         // like out, or nullptr
    const float *bias;        // [Cout]
    const float *bank[kNumBits];
    const uint8_t *schemes;   // device [S][L]
    size_t in_scheme_stride;  // elements between schemes of `in` (0: shared network input)
    size_t out_scheme_stride; // elements between schemes of out
    size_t res_scheme_stride; // elements between schemes of res (0: one copy for all schemes)
    int32_t S, L, slot;       // schemes with index >= S (the base pass) and slot < 0 use FP32
    int32_t N;                // images in this chunk
    int32_t Hin, Win, Cin, Hout, Wout, Cout;
    int32_t act;
    int32_t R;                // output rows per workgroup region
    int32_t G;                // images per workgroup (R == Hout when G > 1)
    int32_t regions_per_image;
    int32_t CB;               // ceil(Cin/16)
    int32_t CKC;              // channels staged per pass (16, 32 or 64)
    int32_t RIN, LW, PS;      // LDS tile: rows, row width (pixels), pixel stride (floats)
    int32_t wave_px_split;    // waves along pixels (4, 2 or 1); 4/wave_px_split along couts
    int32_t cout_tiles;       // ceil(Cout/16)
    FastDiv div_lw, div_rin, div_wout, div_rw; // LW, RIN, Wout, R*Wout
};

// Arguments of the 1x1 stride-1 convolution (pixels form one flat axis).
struct PointwiseArgs {
    const float *in;          // [S?][P][Cin]
    float *out;               // [S][P][Cout]
    const float *res;         // like out, or nullptr
    const float *bias;
    const float *bank[kNumBits];
    const uint8_t *schemes;
    size_t in_scheme_stride, out_scheme_stride, res_scheme_stride;
    int32_t S, L, slot;
    int32_t P;                // pixels of this chunk: images * H * W
    int32_t Cin, Cout, act;
    int32_t CB, CKC, PS;      // ceil(Cin/16), channels staged per pass, LDS pixel stride (floats)
    int32_t wave_px_split, cout_tiles;
    int32_t grid_y;           // output-channel blocks (the launcher folds them into the block axis)
    int32_t pool;             // 1: images of 64 pixels (one per wavefront), no residual; out = [S][images][Cout],
                              // the mean of the activated outputs over each image's pixels
};

struct DepthwiseArgs {
    const float *in;
    float *out;
    const float *bias;
    const float *bank[kNumBits]; // tap-major [9][C]
    const uint8_t *schemes;
    size_t in_scheme_stride, out_scheme_stride;
    int32_t S, L, slot;
    int32_t N, Hin, Win, C, Hout, Wout, stride, act;
    FastDiv div_c4;
};

// Activation fake-quantization of one node's input: every (scheme, image) tensor of `elems` floats gets one
// symmetric scale from its own largest magnitude and is rewritten at the width the scheme gives the node.
struct ActQuantArgs {
    const float *in;           // [S?][N][elems]
    float *out;                // [s_total][N][elems]
    const uint8_t *schemes;
    size_t in_scheme_stride, out_scheme_stride;
    int32_t S, L, slot;        // launch indices >= S (the FP32 pass) and width 32 copy
    int32_t N, elems;
};

struct HeadArgs {
    const float *in;           // [S][N][HW][C]
    const float *bias;         // [classes]
    const float *bank[kNumBits]; // plain [classes][C]
    const uint8_t *schemes;
    size_t in_scheme_stride;
    int32_t S, L, slot;
    int32_t N;                 // images in this chunk
    int32_t HW, C, classes;
    float *logits;             // nullable; element (s, n) at logits + (s*logits_n + n0 + n)*classes
    int64_t logits_n, n0;
    int32_t *top1;             // (s, n) at top1 + s*top1_stride + n
    int64_t top1_stride;
    int32_t *top1_base;        // the FP32 pass writes top1_base[n]; may be nullptr when there is none
    const int32_t *row_map;    // device: output row of launch index s, < 0 = the FP32 pass; nullptr: row s, and
                               // indices >= S are the FP32 pass
    int32_t act_quant;         // 1: the pooled vector is quantized at the classifier's width before the matrix reads it
};

struct AgreeArgs {
    const int32_t *top1;
    int64_t top1_stride;
    const int32_t *top1_base;
    int32_t *agree;
    int32_t N, S;
};

// Launchers (aiq_kernels.hip).  All return the launch's hipError_t.
hipError_t launch_quantize_single(const QuantJob &job, hipStream_t st);
// out = bit pattern of max |w[i]| over n elements (out is cleared first); non-negative floats order like integers
hipError_t launch_tensor_absmax(const float *w, size_t n, uint32_t *out, hipStream_t st);
hipError_t launch_quantize_batch(const QuantJob *jobs_dev, const int32_t *block_job_dev, int n_blocks,
                                 const QuantMask &mask, hipStream_t st);
hipError_t launch_conv(const ConvArgs &a, int ks, int stride, int nt, size_t lds_bytes, dim3 grid,
                       hipStream_t st);
// 3x3 stride-1 convolution with at most four input channels and no residual (bank layout kLayoutStem)
hipError_t launch_conv_stem(const ConvArgs &a, int nt, dim3 grid, hipStream_t st);
hipError_t launch_pointwise(const PointwiseArgs &a, int nt, size_t lds_bytes, dim3 grid, hipStream_t st);
hipError_t launch_depthwise(const DepthwiseArgs &a, int s_total, hipStream_t st);
hipError_t launch_head(const HeadArgs &a, int s_total, hipStream_t st);
hipError_t launch_act_quantize(const ActQuantArgs &a, int s_total, hipStream_t st);
hipError_t launch_agree(const AgreeArgs &a, hipStream_t st);
hipError_t launch_fill_i32(int32_t *p, int32_t v, size_t n, hipStream_t st);
// Small host tables (schemes, row maps) to device memory as kernel arguments, 2 KB per launch: the bytes are
// taken when the launch is enqueued, so the host buffer is free again when the call returns, nothing waits
// for the stream, and the step can be captured in a HIP graph.
hipError_t upload_bytes(void *dst_dev, const void *src_host, size_t nbytes, hipStream_t st);
// The library's own fixed workspace for aiq_eval_schemes_noalloc: address of the current device's copy and its size.
hipError_t noalloc_scratch(void **ptr, size_t *bytes);
hipError_t conv_set_lds_limits();

} // namespace aiq

// ---------------------------------------------------------------- LDS-resident path
//
// CIFAR-style ResNets (3x3 convolutions of 16/32/64 channels at 32/16/8 pixels, basic
// blocks, 1x1 stride-2 projections) keep every activation of one image in LDS.  One
// workgroup scores one (scheme, image) pair: the op list below is interpreted in order,
// each op reads and writes LDS regions, only the image, the weights and the logits touch
// global memory.
namespace aiq {

enum FusedOpType : int32_t {
    kOpStem = 0,     // 3x3, 3 -> 16, 32x32, image plane -> padded planes
    kOpC16 = 1,      // 3x3, 16 -> 16 at 32x32
    kOpT16_32 = 2,   // 3x3 stride 2, 16 -> 32, 32x32 -> 16x16
    kOpS16_32 = 3,   // 1x1 stride 2, 16 -> 32 (projection, unpadded destination)
    kOpC32 = 4,      // 3x3, 32 -> 32 at 16x16
    kOpT32_64 = 5,   // 3x3 stride 2, 32 -> 64, 16x16 -> 8x8
    kOpS32_64 = 6,   // 1x1 stride 2, 32 -> 64
    kOpC64 = 7,      // 3x3, 64 -> 64 at 8x8
    kOpHead = 8      // global average pool + classifier + argmax
};

struct FusedOp {
    const float *bank[kNumBits];
    const float *bias;
    int32_t type;
    int32_t slot;      // scheme slot or -1
    int32_t act;
    int32_t src_off;   // LDS offsets in floats
    int32_t dst_off;
    int32_t res_off;   // -1: no residual
    int32_t res_padded; // residual region has the padded layout of the destination
    int32_t zero_ring; // destination gets a new layout: clear its border first
    int32_t classes;   // head only
    // Checkpoint taken before this op in a reference pass and restored by a pass that starts
    // here: the first ck_ext[r] floats of LDS region r, stored back to back at float offset
    // ck_off of the image's checkpoint record.  ck_ext = {0, 0}: no checkpoint for this op.
    int32_t ck_off;
    int32_t ck_ext[2];
};

constexpr int kFusedThreads = 512;
constexpr int kFusedMaxOps = 128; // rows of the per-workgroup op table in LDS
constexpr int kFusedRegionFloats = 18560; // 74 240 bytes: a padded 34x34x16 tensor, or 18x18x32 + 16x16x32
constexpr int kFusedLdsBytes = 2 * kFusedRegionFloats * 4;

struct FusedArgs {
    const FusedOp *ops; // device
    int32_t n_ops;
    const float *images; // [N][32][32][3]
    const uint8_t *schemes;
    int32_t S, L, N;
    float *logits;
    int64_t logits_n, n0;
    int32_t *top1;
    int64_t top1_stride;
    int32_t *top1_base;
    float *ckpt;               // checkpoint records [N][ckpt_stride] (reference and resumed passes)
    int64_t ckpt_stride;       // floats per image
    const int32_t *first_op;   // resumed pass: [S] op at which scheme s starts (0 = from the image)
    uint64_t ck_mask[2];       // reference pass: bit o set = write the checkpoint of op o
    int32_t ref_first_op;      // reference pass: op to start at, from its own checkpoint (0 = from the image)
    int32_t ref_stop_op;       // reference pass: stop before this op, after its checkpoint (n_ops = run to the end)
};

// How a launch of the LDS-resident kernel treats the checkpoints.
enum FusedMode : int32_t {
    kFusedPlain = 0,     // every (scheme, image) runs the whole network
    kFusedReference = 1, // whole network, LDS state written out before every op that has a checkpoint
    kFusedResume = 2     // scheme s starts at op first_op[s] from the reference pass's checkpoint
};

hipError_t launch_fused(const FusedArgs &a, int s_total, FusedMode mode, hipStream_t st);
hipError_t fused_set_lds_limit();

} // namespace aiq

// ---------------------------------------------------------------- inverted-residual blocks
//
// 1x1 expand -> depthwise 3x3 -> 1x1 project with the expanded tensor held in LDS
// (aiq_mbconv.hip).  Only the shapes listed there are covered; everything else runs layer
// by layer.
namespace aiq {


struct MbShape {
    int32_t cin, hid, cout, h, stride, res;
};

struct MbArgs {
    const float *in;  // [S?][N][H][W][CIN]
    float *out;       // [S][N][HO][WO][COUT]
    const float *bank_e[kNumBits], *bank_d[kNumBits], *bank_p[kNumBits]; // expand (MFMA layout), depthwise (tap-major), project
    const float *bias_e, *bias_d, *bias_p;
    const uint8_t *schemes;
    size_t in_scheme_stride, out_scheme_stride;
    int32_t S, L, slot_e, slot_d, slot_p;
    int32_t N;
    int32_t act_e, act_d, act_p;
};

bool mbconv_supported(const MbShape &sh);
hipError_t launch_mbconv(const MbShape &sh, const MbArgs &a, int s_total, hipStream_t st);

// The same blocks for one deployed scheme whose expand and / or project layer carries at most eight bits: those
// matrix products from integer codes on the bf16 matrix pipe (aiq_mbconv_codes.hip).
struct MbCodeArgs {
    const float *in;         // [N][H][W][CIN]
    float *out;              // [N][HO][WO][COUT]
    const uint16_t *codes_e; // bf16 bit patterns [HID/16][ceil(CIN/32)][64 lanes][8], zero padded; null: expand in fp32 from w_e
    const uint16_t *codes_p; // bf16 bit patterns [ceil(COUT/16)][HID/16][64 lanes][4], zero padded; null: project in fp32 from w_p
    const float *scale_e;    // [HID] (with codes_e)
    const float *scale_p;    // [COUT] (with codes_p)
    const float *w_e, *w_p;  // fp32 weights of a layer without codes, at its width, in the scoring kernel's MFMA layout
    const float *w_d;        // depthwise weights at the width the scheme gives them, tap-major [9][HID]
    const float *bias_e, *bias_d, *bias_p;
    int32_t N;
    int32_t act_e, act_d, act_p;
};

// at least one of the two layers on codes; a block with one fp32 layer is covered where the tiling keeps the block
// input in registers
bool mbconv_codes_supported(const MbShape &sh, bool expand_codes, bool project_codes);
hipError_t launch_mbconv_codes(const MbShape &sh, const MbCodeArgs &a, hipStream_t st);
// A 1x1 layer on 8x8 pixels that writes the per-image mean of its activated outputs (the classifier's pooling),
// from integer codes.
struct PoolCodeArgs {
    const float *in;       // [N][64][Cin]
    float *out;            // [N][Cout]
    const uint16_t *codes; // bf16 bit patterns [groups * CG][KS][64 lanes][8], zero padded
    const float *scales;   // [Cout]
    const float *bias;     // [Cout]
    int32_t N, Cin, Cout, act;
    int32_t KS;            // ceil(Cin/32)
    int32_t CG, groups;    // tiles of 16 output channels a wavefront takes at a time; ceil(tiles / CG)
};
// false: the layer does not fit (Cin % 8, Cout % 4, LDS); else the tile grouping the kernel will use
bool pooled_codes_plan(int cin, int cout, int *cg, int *groups);
hipError_t launch_pooled_codes(const PoolCodeArgs &a, hipStream_t st);
// codes: int32 [rows][k]; out: cleared buffer [ceil(rows/16)][ceil(k/kstep)][64 lanes][kstep/4], kstep 32 or 16
hipError_t launch_pack_mb_codes(const int32_t *codes, uint16_t *out, int rows, int k, int kstep, hipStream_t st);

} // namespace aiq

// ---------------------------------------------------------------- deployed inference
//
// Dense convolution of a layer of at most eight bits from its integer codes on the bf16
// matrix pipe (aiq_deploy.hip).  One scheme, so there is no scheme axis.
namespace aiq {

constexpr int kCodeStageItems = 3;  // items (eight channels of one pixel) a thread stages per pass; twice that in the
                                    // kernel variant for long regions
constexpr int kCodeStageChunks = 5; // 16-byte chunks of codes a thread stages per pass, at most

struct CodeConvArgs {
    const float *in;       // [N][Hin][Win][Cin]
    float *out;            // [N][Hout][Wout][Cout]
    const float *res;      // like out, or nullptr
    const float *bias;     // [Cout]
    const uint16_t *codes; // bf16 bit patterns, [ceil(Cout/32)][tap][ceil(Cin/16)][64 lanes][8], zero padded
    const float *scales;   // [Cout]
    int32_t N;
    int32_t Hin, Win, Cin, Hout, Wout, Cout;
    int32_t act;
    int32_t R;             // output rows per workgroup region
    int32_t G;             // images per workgroup (R == Hout when G > 1)
    int32_t regions_per_image;
    int32_t CB;            // ceil(Cin/16)
    int32_t CKC;           // channels staged per pass (16, 32 or 64)
    int32_t RIN, LW;       // LDS tile: rows, row width (pixels)
    int32_t PSU;           // eight-channel units of one staged pixel: CKC / 8 (each holds its hi, mid, lo pieces: 48 bytes)
    int32_t wave_px_split; // waves along pixels (4, 2 or 1); 4/wave_px_split along output channels
    int32_t cout_tiles;    // ceil(Cout/32)
    int32_t tiles_per_wg;  // output-channel tiles of one workgroup: NT * 4 / wave_px_split
    int32_t code_off;      // LDS unit where the pass's codes start (after the activations)
    FastDiv div_rin, div_wout, div_rw, div_per_row; // RIN, Wout, R*Wout, LW * CKC / 8
};

// codes: int32 [cout][cin][taps]; out: cleared buffer in the layout above
hipError_t launch_pack_codes(const int32_t *codes, uint16_t *out, int cout, int cin, int taps, hipStream_t st);
hipError_t launch_conv_codes(const CodeConvArgs &a, int ks, int stride, int nt, int stage_items, int mt, size_t lds_bytes,
                             dim3 grid, hipStream_t st);
hipError_t conv_codes_set_lds_limits();

// Dense convolution of a layer of at most eight bits whose input tensor is quantized as well
// (activation variant), from int8 codes on both sides on the INT8 matrix pipe (aiq_int8.hip).
struct I8ConvArgs {
    const int8_t *in;      // activation codes [N][Hin][Win][Cin], Cin % 16 == 0
    const float *xscale;   // [N]: the images' activation scales
    float *out;            // [N][Hout][Wout][Cout]
    const float *res;      // like out, or nullptr
    const float *bias;     // [Cout]
    const int8_t *codes;   // weight codes [ceil(Cout/32)][tap][ceil(Cin/32)][64 lanes][16], zero padded
    const float *scales;   // [Cout]: weight scales
    uint32_t *amax_out;    // nullable: [N], cleared by the caller; receives max |out| per image as float bit patterns
    int32_t N;
    int32_t Hin, Win, Cin, Hout, Wout, Cout;
    int32_t act;
    int32_t R;             // output rows per workgroup region
    int32_t G;             // images per workgroup (R == Hout when G > 1)
    int32_t regions_per_image;
    int32_t CBK;           // ceil(Cin/32)
    int32_t CKB;           // blocks of 32 channels staged per pass (1 or 2)
    int32_t RIN, LW;       // LDS tile: rows, row width (pixels)
    int32_t PSB;           // bytes of one staged pixel: 32 * CKB + 16
    int32_t wave_px_split; // waves along pixels (4, 2 or 1); 4/wave_px_split along output channels
    int32_t cout_tiles;    // ceil(Cout/32)
    int32_t tiles_per_wg;  // output-channel tiles of one workgroup: NT * 4 / wave_px_split
    int32_t code_off;      // LDS byte where the pass's weight codes start (after the activations and the epilogue's tiles)
    int32_t RPW;           // consecutive regions one workgroup works through (1 unless the layer needs a single pass)
    int32_t total_regions; // regions (G == 1) or image groups (G > 1) of the launch
    FastDiv div_rin, div_wout, div_rw, div_per_row, div_pximg; // RIN, Wout, R*Wout, LW * 2 * CKB, Hout*Wout
};

// in: fp32 [n][elems] (elems % 16 == 0) -> codes int8 [n][elems], xscale[n]; bits in {8, 6, 4, 2}.
// amax_bits: nullable, [n]: the images' absolute maxima as float bit patterns, if the producer has left them
hipError_t launch_act_codes(const float *in, const uint32_t *amax_bits, int8_t *codes, float *xscale, int n, int elems,
                            int bits, hipStream_t st);
// codes: int32 [cout][cin][taps]; out: cleared buffer in the layout above
hipError_t launch_pack_codes_i8(const int32_t *codes, int8_t *out, int cout, int cin, int taps, hipStream_t st);
hipError_t launch_conv_i8(const I8ConvArgs &a, int ks, int stride, int nt, size_t lds_bytes, dim3 grid, hipStream_t st);

} // namespace aiq
