// LDS-resident scoring of CIFAR-style ResNets on gfx950: one workgroup runs the whole
// network for one (scheme, image) pair without writing an activation to HBM.
//
// What is computed is unchanged - the forward pass of the model whose layer i carries
// weights quantized at q_i bits (paper: Problem Formulation; Introduction item (ii)) - only
// where the intermediate tensors live differs from the layer-by-layer kernels.
//
// LDS layout of a tensor with C channels and H x H pixels: C/4 planes of (H+2) x (H+2)
// pixels x 4 floats, border zero.  In the 16x16x4 fp32 MFMA a lane (pixel p = lane%16,
// kq = lane/16) needs channels 16*cb + 4*kq .. +3 of its pixel: exactly one 16-byte element
// of plane 4*cb + kq, and the 16 lanes of equal kq read 256 contiguous bytes (no bank
// conflicts for stride-1 layers).  The same lane's four accumulators are output channels
// 16*ct + 4*kq .. +3 of its pixel: one 16-byte write into plane 4*ct + kq.
#include "aiq_internal.h"

namespace aiq {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Weight and bias pointers come out of the op table, so the compiler only knows them as
// generic pointers; loading through an explicit global address space gives global_load
// (counted by vmcnt only) instead of flat_load (which also holds up LDS waits).
typedef const __attribute__((address_space(1))) floatx4 *gvec4_ptr;
typedef const __attribute__((address_space(1))) float *gfloat_ptr;
__device__ __forceinline__ floatx4 gload4(const float *p) { return *(gvec4_ptr)(p); }
__device__ __forceinline__ float gload1(const float *p) { return *(gfloat_ptr)(p); }

// Activation as a clamp to [lo, hi]: none = (-inf, inf), ReLU = (0, inf), ReLU6 = (0, 6).
__device__ __forceinline__ floatx4 clamp4(floatx4 v, float lo, float hi)
{
    // one v_med3_f32 per element: the median of (v, lo, hi) is v clamped to [lo, hi]
    v.x = __builtin_amdgcn_fmed3f(v.x, lo, hi);
    v.y = __builtin_amdgcn_fmed3f(v.y, lo, hi);
    v.z = __builtin_amdgcn_fmed3f(v.z, lo, hi);
    v.w = __builtin_amdgcn_fmed3f(v.w, lo, hi);
    return v;
}
__device__ __forceinline__ float act_lo(int act) { return act >= 1 ? 0.0f : -__builtin_inff(); }
__device__ __forceinline__ float act_hi(int act) { return act == 2 ? 6.0f : __builtin_inff(); }

// Shape constants of the dense ops, indexed by FusedOpType (0 where not a dense convolution):
// reduction steps (taps x 16-channel blocks) and output-channel tiles.  Used to prefetch the
// first weights of the next op while the current one finishes.
__device__ constexpr int kOpSteps[9] = {0, 9, 9, 1, 18, 18, 2, 36, 0};
__device__ constexpr int kOpCoutTiles[9] = {0, 1, 2, 2, 2, 4, 4, 4, 0};
constexpr int kWeightRing = 6; // weight chunks in flight per wavefront (two tap columns of a 3x3 layer)

// One dense convolution, LDS -> LDS.  NW wavefronts; wavefront w owns output-channel tile
// w % CT and MT pixel tiles.  The reduction is a straight line of STEPS = taps x CB steps;
// step k's activations (one 16-byte LDS read per pixel tile) are issued before step k-1's
// MFMAs, its weights (one 16-byte global read, L2-resident, MFMA operand order) kWeightRing
// steps ahead.  Weight chunk c always lives in ring slot c % kWeightRing; wr[] arrives holding
// this op's first chunks (loaded while the previous op ran) and leaves holding those of the
// next op (next_w; next_last = index of its last chunk), so no wavefront waits on L2 right after a barrier.
template <int CIN, int COUT, int HIN, int STRIDE, int KS, bool DST_PADDED, int NW>
__device__ __forceinline__ void fused_conv(const float *src, float *dst, const float *res, bool res_padded,
                                           const float *__restrict__ wq, const floatx4 bv, int act,
                                           bool zero_ring, int tid, floatx4 (&wr)[kWeightRing],
                                           const float *__restrict__ next_w, int next_last)
{
    constexpr int CB = CIN / 16, CT = COUT / 16, HO = HIN / STRIDE, PT = HO * HO / 16, T = KS * KS;
    constexpr int STEPS = T * CB;
    constexpr int WPC = NW / CT;   // wavefronts per output-channel tile
    constexpr int MT = PT / WPC;   // pixel tiles per wavefront
    static_assert(NW % CT == 0 && PT % WPC == 0 && MT >= 1, "tiles must divide evenly");
    constexpr int PIN = HIN + 2, POUT = HO + 2;
    constexpr int SRC_PLANE = PIN * PIN * 4, DST_PLANE = (DST_PADDED ? POUT * POUT : HO * HO) * 4;
    // the per-lane index arithmetic below depends only on tid; without this the compiler
    // hoists it for every op type out of the op loop and runs out of registers
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = tid >> 6, p = lane & 15, kq = lane >> 4;
    const int ct = wave % CT, pg = wave / CT;

    if (zero_ring) {
        // border of the destination's padded layout: COUT/4 planes x (4*POUT - 4) pixels
        constexpr int RING = 4 * POUT - 4;
        for (int i = tid; i < (COUT / 4) * RING; i += NW * 64) {
            const int plane = i / RING, r = i - plane * RING;
            int y, x;
            if (r < POUT) { y = 0; x = r; }
            else if (r < 2 * POUT) { y = POUT - 1; x = r - POUT; }
            else { const int q = r - 2 * POUT; y = 1 + (q >> 1); x = (q & 1) ? POUT - 1 : 0; }
            *reinterpret_cast<floatx4 *>(dst + plane * DST_PLANE + (y * POUT + x) * 4) = floatx4{0.f, 0.f, 0.f, 0.f};
        }
    }

    // per pixel tile: source offset of the lane's pixel; destination / residual offsets are
    // recomputed where they are used (cheap shifts) rather than held across the reduction
    int src_off[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int P = (pg + i * WPC) * 16 + p;
        const int oy = P / HO, ox = P % HO;
        src_off[i] = kq * SRC_PLANE + ((oy * STRIDE) * PIN + ox * STRIDE) * 4 + (KS == 1 ? (PIN + 1) * 4 : 0);
    }
    auto out_index = [&](int i, bool padded) {
        const int P = (pg + i * WPC) * 16 + p;
        const int oy = P / HO, ox = P % HO;
        const int plane = ct * 4 + kq;
        return padded ? plane * (POUT * POUT * 4) + ((oy + 1) * POUT + ox + 1) * 4
                      : plane * (HO * HO * 4) + (oy * HO + ox) * 4;
    };
    const float *wbase = wq + ((size_t)ct * STEPS * 64 + lane) * 4;
    const float lo = act_lo(act), hi = act_hi(act);

    floatx4 acc[MT]; // start from the bias: nothing to add in the epilogue
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = bv;

    floatx4 xb[2][MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) xb[0][i] = *reinterpret_cast<const floatx4 *>(src + src_off[i]);

#pragma unroll
    for (int k = 0; k < STEPS; ++k) {
        // keep each step's prefetches in that step: nothing is scheduled across this point
        __builtin_amdgcn_sched_barrier(0);
        const int cur = k & 1;
        if (k + 1 < STEPS) {
            const int t = (k + 1) / CB, cb = (k + 1) % CB;
            const int off = ((t / KS) * PIN + (t % KS)) * 4 + cb * 4 * SRC_PLANE;
#pragma unroll
            for (int i = 0; i < MT; ++i)
                xb[cur ^ 1][i] = *reinterpret_cast<const floatx4 *>(src + src_off[i] + off);
        } else if (res) {
            // last step: the idle activation buffer receives the residual values
#pragma unroll
            for (int i = 0; i < MT; ++i)
                xb[cur ^ 1][i] = *reinterpret_cast<const floatx4 *>(res + out_index(i, res_padded));
        }
        const floatx4 w = wr[k % kWeightRing];
        if (k + kWeightRing < STEPS) {
            wr[k % kWeightRing] = gload4(wbase + (k + kWeightRing) * 256);
        } else {
            // this ring slot is free from here on: fetch the next op's chunk that lives in it
            // (branch-free: a chunk index past the next op's last one re-reads its last chunk)
            wr[k % kWeightRing] = gload4(next_w + min(k % kWeightRing, next_last) * 256);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < MT; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[j], xb[cur][i][j], acc[i], 0, 0, 0);
        // issue order inside the step: the weight fetch, then one LDS read per two MFMAs (all
        // reads of the next step are in flight by mid-step), then the remaining MFMAs
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * MT, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // ops with fewer steps than ring slots (1x1 projections) never used the upper slots
#pragma unroll
    for (int nk = STEPS; nk < kWeightRing; ++nk) wr[nk] = gload4(next_w + min(nk, next_last) * 256);

    constexpr int RB = (STEPS & 1); // buffer that received the residual: (STEPS-1)&1 ^ 1
    if (res) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
            *reinterpret_cast<floatx4 *>(dst + out_index(i, DST_PADDED)) = clamp4(acc[i] + xb[RB][i], lo, hi);
    } else {
#pragma unroll
        for (int i = 0; i < MT; ++i)
            *reinterpret_cast<floatx4 *>(dst + out_index(i, DST_PADDED)) = clamp4(acc[i], lo, hi);
    }
}

// Stride-1 3x3 convolution with vertical operand reuse.  A wavefront owns output-channel tile
// w % CT and a strip of MT vertically adjacent pixel tiles.  For one tap column kx and one
// 16-channel block the strip's inputs are NR = RPT*(MT-1) + 3 window rows (RPT image rows per
// pixel tile); the row a tile needs for tap row ky is the one its lower neighbour needs for
// ky-1, so each 16-byte LDS read feeds up to three tiles (12 MFMAs) instead of one (4): 10 reads
// instead of 24 per 96 MFMAs at 32x32.  Weights come one tap column at a time (three chunks:
// ky = 0, 1, 2; bank layout [kx][channel block][ky]) through the same register ring as
// fused_conv, including the hand-over of the next op's first chunks.
template <int CIN, int COUT, int HIN, int NW>
__device__ __forceinline__ void fused_conv3s1(const float *src, float *dst, const float *res, bool res_padded,
                                              const float *__restrict__ wq, const floatx4 bv, int act,
                                              bool zero_ring, int tid, floatx4 (&wr)[kWeightRing],
                                              const float *__restrict__ next_w, int next_last)
{
    constexpr int CB = CIN / 16, CT = COUT / 16, HO = HIN, PT = HO * HO / 16, STEPS = 9 * CB;
    constexpr int WPC = NW / CT, MT = PT / WPC;
    constexpr int RPT = HO >= 16 ? 1 : 16 / HO; // image rows per pixel tile
    constexpr int TPR = HO >= 16 ? HO / 16 : 1; // pixel tiles per image row
    constexpr int NR = RPT * (MT - 1) + 3;      // window rows of a strip
    constexpr int NG = 3 * CB;                  // (tap column, channel block) groups of three weight chunks
    constexpr int PIN = HIN + 2, PLANE = PIN * PIN * 4;
    static_assert(NW % CT == 0 && PT % WPC == 0 && WPC % TPR == 0 && STEPS >= kWeightRing, "strips must tile the image");
    // (no barrier against hoisting here: the three strip geometries' lane offsets are computed
    // once per kernel and kept in registers, which shortens every op's prologue)
    const int lane = tid & 63, wave = tid >> 6, p = lane & 15, kq = lane >> 4;
    const int ct = wave % CT, pg = wave / CT;
    const int oy0 = (pg / TPR) * MT * RPT + (RPT > 1 ? p / HO : 0);
    const int ox = (pg % TPR) * 16 + (RPT > 1 ? p % HO : p);
    const int src_base = kq * PLANE + (oy0 * PIN + ox) * 4;

    if (zero_ring) {
        constexpr int RING = 4 * PIN - 4;
        for (int i = tid; i < (COUT / 4) * RING; i += NW * 64) {
            const int plane = i / RING, r = i - plane * RING;
            int y, x;
            if (r < PIN) { y = 0; x = r; }
            else if (r < 2 * PIN) { y = PIN - 1; x = r - PIN; }
            else { const int q = r - 2 * PIN; y = 1 + (q >> 1); x = (q & 1) ? PIN - 1 : 0; }
            *reinterpret_cast<floatx4 *>(dst + plane * PLANE + (y * PIN + x) * 4) = floatx4{0.f, 0.f, 0.f, 0.f};
        }
    }
    auto out_index = [&](int i, bool padded) {
        const int oy = oy0 + i * RPT, plane = ct * 4 + kq;
        return padded ? plane * PLANE + ((oy + 1) * PIN + ox + 1) * 4 : plane * (HO * HO * 4) + (oy * HO + ox) * 4;
    };
    const float *wbase = wq + ((size_t)ct * STEPS * 64 + lane) * 4;
    const float lo = act_lo(act), hi = act_hi(act);

    floatx4 acc[MT]; // start from the bias: nothing to add in the epilogue
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = bv;

    // window rows are read two ahead of their use; q = g * NR + r runs over (group, row)
    constexpr int NQ = NG * NR, DEPTH = 2;
    auto row_addr = [&](int q) {
        const int g = q / NR, r = q - g * NR;
        const int kx = g / CB, cb = g - kx * CB;
        return src + src_base + (kx + r * PIN) * 4 + cb * 4 * PLANE;
    };
    floatx4 xb[DEPTH + 1];
#pragma unroll
    for (int q = 0; q < DEPTH; ++q) xb[q] = *reinterpret_cast<const floatx4 *>(row_addr(q));
    floatx4 rv[MT]; // residual values, fetched during the last group
    floatx4 w0, w1, w2;

#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        __builtin_amdgcn_sched_barrier(0);
        const int g = q / NR, r = q - g * NR;
        if (q + DEPTH < NQ) xb[(q + DEPTH) % (DEPTH + 1)] = *reinterpret_cast<const floatx4 *>(row_addr(q + DEPTH));
        if (r == 0) {
            // this group's three chunks leave the ring; their slots are refilled at once, with this
            // op's chunks two groups on or, at the end, with the next op's first chunks
            w0 = wr[(3 * g) % kWeightRing];
            w1 = wr[(3 * g + 1) % kWeightRing];
            w2 = wr[(3 * g + 2) % kWeightRing];
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int c = 3 * g + j, slot = c % kWeightRing;
                wr[slot] = c + kWeightRing < STEPS ? gload4(wbase + (c + kWeightRing) * 256)
                                                   : gload4(next_w + min(slot, next_last) * 256);
            }
            if (g == NG - 1 && res) {
#pragma unroll
                for (int i = 0; i < MT; ++i) rv[i] = *reinterpret_cast<const floatx4 *>(res + out_index(i, res_padded));
            }
        }
        const floatx4 x = xb[q % (DEPTH + 1)];
        // the (up to three) tiles this row feeds take turns, so that consecutive MFMAs never
        // accumulate into the same registers
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const int d = r - ky;
            if (d < 0 || d % RPT != 0 || d / RPT >= MT) continue;
            const floatx4 w = ky == 0 ? w0 : (ky == 1 ? w1 : w2);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[d / RPT] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[j], x[j], acc[d / RPT], 0, 0, 0);
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    if (res) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
            *reinterpret_cast<floatx4 *>(dst + out_index(i, true)) = clamp4(acc[i] + rv[i], lo, hi);
    } else {
#pragma unroll
        for (int i = 0; i < MT; ++i)
            *reinterpret_cast<floatx4 *>(dst + out_index(i, true)) = clamp4(acc[i], lo, hi);
    }
}

// Stem: 3 input channels held as one plane of (r, g, b, 0) pixels; one MFMA per tap
// (reduction = the 4 floats of a pixel).  Weights: [tap][64 lanes], lane = kq*16 + co.
template <int NW>
__device__ __forceinline__ void fused_stem(const float *src, float *dst, const float *__restrict__ wq,
                                           const float *__restrict__ bias, int act, int tid)
{
    // A wavefront owns a strip of MT vertically adjacent pixel tiles (half an image row wide), so a
    // window row read for tap column kx serves tap row ky of tile r - ky: 3 * (MT + 2) four-byte
    // LDS reads instead of 9 * MT.
    constexpr int H = 32, PIN = 34, PT = H * H / 16, MT = PT / NW, PLANE = PIN * PIN * 4, NR = MT + 2;
    static_assert(NW % 2 == 0 && PT % NW == 0, "strips must tile the image");
    asm volatile("" : "+v"(tid)); // keep the index arithmetic inside the op (see fused_conv)
    const int lane = tid & 63, wave = tid >> 6, p = lane & 15, kq = lane >> 4;
    const int oy0 = (wave >> 1) * MT, ox = (wave & 1) * 16 + p;
    const float *base = src + (oy0 * PIN + ox) * 4 + kq;
    float w[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) w[t] = gload1(wq + t * 64 + lane);
    const floatx4 bv = gload4(bias + kq * 4);
    float x[3][NR];
#pragma unroll
    for (int kx = 0; kx < 3; ++kx)
#pragma unroll
        for (int r = 0; r < NR; ++r) x[kx][r] = base[(r * PIN + kx) * 4];
    floatx4 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = bv;
#pragma unroll
    for (int kx = 0; kx < 3; ++kx)
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
            for (int i = 0; i < MT; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[ky * 3 + kx], x[kx][i + ky], acc[i], 0, 0, 0);
    const float lo = act_lo(act), hi = act_hi(act);
#pragma unroll
    for (int i = 0; i < MT; ++i)
        *reinterpret_cast<floatx4 *>(dst + kq * PLANE + ((oy0 + i + 1) * PIN + ox + 1) * 4) = clamp4(acc[i], lo, hi);
}

__device__ inline float fused_wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Per-op record for THIS workgroup's scheme, built once at kernel start so that the op loop
// never chases pointers through global memory right after a barrier.
struct OpRT {
    uint32_t w_lo, w_hi;     // weights of the scheme's bit-width, kernel layout
    uint32_t b_lo, b_hi;     // bias
    int32_t type, act, src_off, dst_off;
    int32_t res_off, flags, classes;
    int32_t shape;           // dense ops: (reduction steps << 8) | (output-channel tiles - 1); 0 otherwise
};

__device__ __forceinline__ OpRT uniform_op(const OpRT &v)
{
    OpRT r;
    r.w_lo = __builtin_amdgcn_readfirstlane(v.w_lo);
    r.w_hi = __builtin_amdgcn_readfirstlane(v.w_hi);
    r.b_lo = __builtin_amdgcn_readfirstlane(v.b_lo);
    r.b_hi = __builtin_amdgcn_readfirstlane(v.b_hi);
    r.type = __builtin_amdgcn_readfirstlane(v.type);
    r.act = __builtin_amdgcn_readfirstlane(v.act);
    r.src_off = __builtin_amdgcn_readfirstlane(v.src_off);
    r.dst_off = __builtin_amdgcn_readfirstlane(v.dst_off);
    r.res_off = __builtin_amdgcn_readfirstlane(v.res_off);
    r.flags = __builtin_amdgcn_readfirstlane(v.flags);
    r.classes = __builtin_amdgcn_readfirstlane(v.classes);
    r.shape = __builtin_amdgcn_readfirstlane(v.shape);
    return r;
}
__device__ __forceinline__ const float *op_ptr(uint32_t lo, uint32_t hi)
{
    return reinterpret_cast<const float *>(((uint64_t)hi << 32) | lo);
}

// Copies between the two LDS regions and an image's checkpoint record: the first e0 floats of
// region 0 and the first e1 of region 1, back to back in global memory (all multiples of 4).
// kBatch 16-byte transfers are in flight per thread.  The caller synchronises.
template <int NW, bool RESTORE>
__device__ __forceinline__ void fused_checkpoint_copy(float *lds, float *g, int e0, int e1, int tid)
{
    constexpr int kBatch = 8;
    floatx4 *lds4 = reinterpret_cast<floatx4 *>(lds);
    floatx4 *g4 = reinterpret_cast<floatx4 *>(g);
    const int n0 = e0 >> 2, n4 = (e0 + e1) >> 2;
    for (int base = tid; base < n4; base += NW * 64 * kBatch) {
        floatx4 v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = base + u * NW * 64;
            const int l = i < n0 ? i : i - n0 + kFusedRegionFloats / 4;
            if (i < n4) v[u] = RESTORE ? gload4(g + (size_t)i * 4) : lds4[l];
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = base + u * NW * 64;
            const int l = i < n0 ? i : i - n0 + kFusedRegionFloats / 4;
            if (i < n4) {
                if (RESTORE) lds4[l] = v[u];
                else g4[i] = v[u];
            }
        }
    }
}

// MODE (FusedMode): the plain kernel runs every op; the reference pass also writes the LDS
// state out before each op whose checkpoint is asked for (and may itself continue from one of
// its earlier checkpoints and stop once the last one asked for is written); a resumed pass
// starts scheme s at op first_op[s] from that state.  Ops before first_op[s] carry the same bit-widths in scheme s
// and in the reference scheme, so the restored state is bit for bit what the full run of
// scheme s would hold there and the result does not depend on the mode.
template <int NW, int MODE>
__global__ __launch_bounds__(NW * 64) void resnet_fused_kernel(FusedArgs a)
{
    extern __shared__ float lds[];
    __shared__ OpRT s_ops[kFusedMaxOps];
    const int tid = threadIdx.x;
    const int n = blockIdx.x, s = blockIdx.y;
    int o0 = 0;
    if (MODE == kFusedResume && s < a.S) o0 = __builtin_amdgcn_readfirstlane(a.first_op[s]);
    if (MODE == kFusedReference) o0 = a.ref_first_op; // a reference pass may continue from its own checkpoint
    const bool from_image = o0 == 0;

    // the image goes to registers first so that its HBM latency overlaps the LDS clear
    constexpr int IMG_PER_THREAD = 3072 / (NW * 64);
    static_assert(3072 % (NW * 64) == 0, "image elements must divide among the threads");
    float img_r[IMG_PER_THREAD];
    if (from_image) {
        const float *img = a.images + (size_t)n * 3072;
#pragma unroll
        for (int q = 0; q < IMG_PER_THREAD; ++q) img_r[q] = img[tid + q * NW * 64];
    }
    if (tid < a.n_ops) {
        const FusedOp &op = a.ops[tid];
        int bi = 0;
        if (op.slot >= 0 && s < a.S) bi = bits_index(a.schemes[(size_t)s * a.L + op.slot]);
        const uint64_t w = reinterpret_cast<uint64_t>(op.bank[bi]), bptr = reinterpret_cast<uint64_t>(op.bias);
        OpRT r;
        r.w_lo = (uint32_t)w;
        r.w_hi = (uint32_t)(w >> 32);
        r.b_lo = (uint32_t)bptr;
        r.b_hi = (uint32_t)(bptr >> 32);
        r.type = op.type;
        r.act = op.act;
        r.src_off = op.src_off;
        r.dst_off = op.dst_off;
        r.res_off = op.res_off;
        r.flags = (op.res_padded ? 1 : 0) | (op.zero_ring ? 2 : 0);
        r.classes = op.classes;
        r.shape = kOpSteps[op.type] > 0 ? (kOpSteps[op.type] << 8) | (kOpCoutTiles[op.type] - 1) : 0;
        s_ops[tid] = r;
    }
    __syncthreads();
    OpRT cur = uniform_op(s_ops[o0]);
    // What has to be zero before the first read: the image plane (border and fourth component)
    // and the borders of the 34 x 34 planes the first stage writes - four in the stem's
    // destination region, the other three of the image's region.  Interiors are always written
    // before they are read; later layouts clear their own borders (zero_ring).
    if (from_image) {
        constexpr int PIN = 34, PLANE = PIN * PIN * 4, RING = 4 * PIN - 4;
        const floatx4 zero = floatx4{0.f, 0.f, 0.f, 0.f};
        floatx4 *img4 = reinterpret_cast<floatx4 *>(lds + cur.src_off);
        for (int i = tid; i < PIN * PIN; i += NW * 64) img4[i] = zero;
        for (int i = tid; i < 7 * RING; i += NW * 64) {
            const int q = i / RING, r = i - q * RING;
            float *plane = q < 4 ? lds + cur.dst_off + q * PLANE : lds + cur.src_off + (q - 3) * PLANE;
            int y, x;
            if (r < PIN) { y = 0; x = r; }
            else if (r < 2 * PIN) { y = PIN - 1; x = r - PIN; }
            else { const int e = r - 2 * PIN; y = 1 + (e >> 1); x = (e & 1) ? PIN - 1 : 0; }
            *reinterpret_cast<floatx4 *>(plane + (y * PIN + x) * 4) = zero;
        }
    }
    __syncthreads();
    if (from_image) {
        float *plane = lds + cur.src_off;
#pragma unroll
        for (int q = 0; q < IMG_PER_THREAD; ++q) {
            const int e = tid + q * NW * 64;
            const int pix = e / 3, c = e - pix * 3;
            const int y = pix >> 5, x = pix & 31;
            plane[((y + 1) * 34 + x + 1) * 4 + c] = img_r[q];
        }
    } else {
        const FusedOp &op = a.ops[o0];
        fused_checkpoint_copy<NW, true>(lds, a.ckpt + (size_t)n * a.ckpt_stride + op.ck_off, op.ck_ext[0],
                                        op.ck_ext[1], tid);
    }
    OpRT nxt_raw = s_ops[o0 + 1 < a.n_ops ? o0 + 1 : o0]; // stays in flight until the next iteration needs it
    __syncthreads();

    floatx4 wr[kWeightRing];
#pragma unroll
    for (int j = 0; j < kWeightRing; ++j) wr[j] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int lane = tid & 63, wave = tid >> 6;
    // bias of the current dense op for this lane's four output channels; like the first weight
    // chunks it is fetched while the previous op runs (the stem reads its own)
    floatx4 bcur = floatx4{0.f, 0.f, 0.f, 0.f};
    if (!from_image && cur.shape != 0) {
        // no previous op has fetched the first weights and the bias of the op resumed at
        const int ns = cur.shape >> 8;
        const int nct = wave & (cur.shape & 255);
        const float *w0 = op_ptr(cur.w_lo, cur.w_hi) + ((size_t)nct * ns * 64 + lane) * 4;
#pragma unroll
        for (int j = 0; j < kWeightRing; ++j) wr[j] = gload4(w0 + min(j, ns - 1) * 256);
        bcur = gload4(op_ptr(cur.b_lo, cur.b_hi) + nct * 16 + (lane >> 4) * 4);
    }

    for (int o = o0; o < a.n_ops; ++o) {
        if (MODE == kFusedReference && o > 0) {
            const FusedOp &op = a.ops[o];
            if (o > o0 && ((a.ck_mask[o >> 6] >> (o & 63)) & 1ull)) {
                fused_checkpoint_copy<NW, false>(lds, a.ckpt + (size_t)n * a.ckpt_stride + op.ck_off, op.ck_ext[0],
                                                 op.ck_ext[1], tid);
                __syncthreads(); // the op below overwrites what other wavefronts may still be copying
            }
            if (o >= a.ref_stop_op) break; // only the checkpoints were wanted
        }
        const OpRT nxt = uniform_op(nxt_raw);
        nxt_raw = s_ops[o + 2 < a.n_ops ? o + 2 : a.n_ops - 1];
        const float *wq = op_ptr(cur.w_lo, cur.w_hi);
        const float *bias = op_ptr(cur.b_lo, cur.b_hi);
        const float *src = lds + cur.src_off;
        float *dst = lds + cur.dst_off;
        const float *res = cur.res_off >= 0 ? lds + cur.res_off : nullptr;
        const bool rp = (cur.flags & 1) != 0, zr = (cur.flags & 2) != 0;
        // first weight chunks of the next dense op, fetched while this op runs; when there is
        // none the prefetch harmlessly re-reads chunk 0 of this op's own weights
        const float *next_w = wq + lane * 4;
        const float *next_b = bias;
        int next_last = 0;
        if (o + 1 < a.n_ops && nxt.shape != 0) {
            // the next op's shape comes with its table row: no dependent constant-memory reads here
            const int ns = nxt.shape >> 8;
            const int nct = wave & (nxt.shape & 255);
            next_w = op_ptr(nxt.w_lo, nxt.w_hi) + ((size_t)nct * ns * 64 + lane) * 4;
            next_b = op_ptr(nxt.b_lo, nxt.b_hi) + nct * 16 + (lane >> 4) * 4;
            next_last = ns - 1;
        }
        const floatx4 bnxt = gload4(next_b); // every bias array holds at least four values
        switch (cur.type) {
        case kOpStem:
#pragma unroll
            for (int j = 0; j < kWeightRing; ++j) wr[j] = gload4(next_w + min(j, next_last) * 256);
            fused_stem<NW>(src, dst, wq, bias, cur.act, tid);
            break;
        case kOpC16: fused_conv3s1<16, 16, 32, NW>(src, dst, res, rp, wq, bcur, cur.act, zr, tid, wr, next_w, next_last); break;
        case kOpT16_32: fused_conv<16, 32, 32, 2, 3, true, NW>(src, dst, res, rp, wq, bcur, cur.act, zr, tid, wr, next_w, next_last); break;
        case kOpS16_32: fused_conv<16, 32, 32, 2, 1, false, NW>(src, dst, res, rp, wq, bcur, cur.act, zr, tid, wr, next_w, next_last); break;
        case kOpC32: fused_conv3s1<32, 32, 16, NW>(src, dst, res, rp, wq, bcur, cur.act, zr, tid, wr, next_w, next_last); break;
        case kOpT32_64: fused_conv<32, 64, 16, 2, 3, true, NW>(src, dst, res, rp, wq, bcur, cur.act, zr, tid, wr, next_w, next_last); break;
        case kOpS32_64: fused_conv<32, 64, 16, 2, 1, false, NW>(src, dst, res, rp, wq, bcur, cur.act, zr, tid, wr, next_w, next_last); break;
        case kOpC64: fused_conv3s1<64, 64, 8, NW>(src, dst, res, rp, wq, bcur, cur.act, zr, tid, wr, next_w, next_last); break;
        case kOpHead: {
            // 64 channels x 8x8 pixels (padded 10x10 planes): pool, classifier, argmax.  The
            // classifier rows of this wavefront are requested first, so that they arrive while
            // the pooling runs.
            constexpr int JW = (16 + NW - 1) / NW; // classes per wavefront (at most 16 classes per round)
            float wrow[JW], brow[JW];
#pragma unroll
            for (int q = 0; q < JW; ++q) {
                const int j = min(wave + q * NW, cur.classes - 1);
                wrow[q] = gload1(wq + j * 64 + lane);
                brow[q] = gload1(bias + j);
            }
            float *scratch = dst;            // [NW][64] partial sums, then pooled[64], then z[classes]
            const int c = tid & 63, part = tid >> 6;
            float acc = 0.0f;
            for (int px = part; px < 64; px += NW) {
                const int y = px >> 3, x = px & 7;
                acc += src[(c >> 2) * 400 + ((y + 1) * 10 + x + 1) * 4 + (c & 3)];
            }
            scratch[part * 64 + c] = acc;
            __syncthreads();
            float *pooled = scratch + NW * 64;
            if (tid < 64) {
                float t = 0.0f;
                for (int q = 0; q < NW; ++q) t += scratch[q * 64 + tid];
                pooled[tid] = t * (1.0f / 64.0f);
            }
            __syncthreads();
            float *z = pooled + 64;
            const float pl = pooled[lane];
#pragma unroll
            for (int q = 0; q < JW; ++q) {
                const int j = wave + q * NW;
                const float t = fused_wave_sum(pl * wrow[q]);
                if (lane == 0 && j < cur.classes) z[j] = t + brow[q];
            }
            for (int j = JW * NW + wave; j < cur.classes; j += NW) { // more than 16 classes: the rest, unprefetched
                const float t = fused_wave_sum(pl * gload1(wq + j * 64 + lane));
                if (lane == 0) z[j] = t + gload1(bias + j);
            }
            __syncthreads();
            if (tid == 0) {
                int best = 0;
                for (int j = 1; j < cur.classes; ++j)
                    if (z[j] > z[best]) best = j;
                if (s < a.S) a.top1[(size_t)s * a.top1_stride + n] = best;
                else if (a.top1_base) a.top1_base[n] = best;
            }
            if (a.logits && s < a.S && tid < cur.classes)
                a.logits[((size_t)s * a.logits_n + a.n0 + n) * cur.classes + tid] = z[tid];
            break;
        }
        default: break;
        }
        __syncthreads();
        cur = nxt;
        bcur = bnxt;
    }
}

hipError_t fused_set_lds_limit()
{
    constexpr int NW = kFusedThreads / 64;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&resnet_fused_kernel<NW, kFusedPlain>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLdsBytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&resnet_fused_kernel<NW, kFusedReference>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLdsBytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&resnet_fused_kernel<NW, kFusedResume>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLdsBytes);
    return e;
}

hipError_t launch_fused(const FusedArgs &a, int s_total, FusedMode mode, hipStream_t st)
{
    constexpr int NW = kFusedThreads / 64;
    if (a.N == 0 || s_total == 0) return hipSuccess;
    if (mode != kFusedPlain && !a.ckpt) return hipErrorInvalidValue;
    if (mode == kFusedResume && !a.first_op) return hipErrorInvalidValue;
    const dim3 grid(a.N, s_total), block(kFusedThreads);
    switch (mode) {
    case kFusedPlain:
        hipLaunchKernelGGL((resnet_fused_kernel<NW, kFusedPlain>), grid, block, kFusedLdsBytes, st, a);
        break;
    case kFusedReference:
        hipLaunchKernelGGL((resnet_fused_kernel<NW, kFusedReference>), grid, block, kFusedLdsBytes, st, a);
        break;
    case kFusedResume:
        hipLaunchKernelGGL((resnet_fused_kernel<NW, kFusedResume>), grid, block, kFusedLdsBytes, st, a);
        break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace aiq
