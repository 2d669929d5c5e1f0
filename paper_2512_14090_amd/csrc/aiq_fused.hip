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

__device__ inline float fused_act(float v, int act)
{
    if (act >= 1) v = fmaxf(v, 0.0f);
    if (act == 2) v = fminf(v, 6.0f);
    return v;
}

// One dense convolution, LDS -> LDS.  NW wavefronts; wavefront w owns output-channel tile
// w % CT and MT pixel tiles; weights stream from global memory (L2-resident, MFMA operand
// order) one tap ahead of their use.
template <int CIN, int COUT, int HIN, int STRIDE, int KS, bool DST_PADDED, int NW>
__device__ __forceinline__ void fused_conv(const float *src, float *dst,
                                           const float *res, bool res_padded,
                                           const float *__restrict__ wq, const float *__restrict__ bias, int act,
                                           bool zero_ring, int tid)
{
    constexpr int CB = CIN / 16, CT = COUT / 16, HO = HIN / STRIDE, PT = HO * HO / 16, T = KS * KS;
    constexpr int WPC = NW / CT;   // wavefronts per output-channel tile
    constexpr int MT = PT / WPC;   // pixel tiles per wavefront
    static_assert(NW % CT == 0 && PT % WPC == 0 && MT >= 1, "tiles must divide evenly");
    constexpr int PIN = HIN + 2, POUT = HO + 2;
    constexpr int SRC_PLANE = PIN * PIN * 4, DST_PLANE = (DST_PADDED ? POUT * POUT : HO * HO) * 4;
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

    int src_off[MT], out_y[MT], out_x[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int P = (pg + i * WPC) * 16 + p;
        const int oy = P / HO, ox = P % HO;
        out_y[i] = oy;
        out_x[i] = ox;
        src_off[i] = kq * SRC_PLANE + ((oy * STRIDE) * PIN + ox * STRIDE) * 4 + (KS == 1 ? (PIN + 1) * 4 : 0);
    }

    floatx4 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    const float *wbase = wq + ((size_t)ct * T * CB * 64 + lane) * 4;
    const floatx4 bv = *reinterpret_cast<const floatx4 *>(bias + ct * 16 + kq * 4);
    floatx4 wcur[CB], wnext[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) wcur[cb] = *reinterpret_cast<const floatx4 *>(wbase + cb * 256);

#pragma unroll 1
    for (int t = 0; t < T; ++t) {
        if (t + 1 < T) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
                wnext[cb] = *reinterpret_cast<const floatx4 *>(wbase + ((t + 1) * CB + cb) * 256);
        }
        const int ky = t / KS, kx = t - ky * KS;
        const int tapoff = (ky * PIN + kx) * 4;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            floatx4 xb[MT];
#pragma unroll
            for (int i = 0; i < MT; ++i)
                xb[i] = *reinterpret_cast<const floatx4 *>(src + src_off[i] + tapoff + cb * 4 * SRC_PLANE);
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < MT; ++i)
                    acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(wcur[cb][j], xb[i][j], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) wcur[cb] = wnext[cb];
    }

#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int plane = ct * 4 + kq;
        const int didx = plane * DST_PLANE +
                         (DST_PADDED ? ((out_y[i] + 1) * POUT + out_x[i] + 1) : (out_y[i] * HO + out_x[i])) * 4;
        floatx4 v = acc[i] + bv;
        if (res) {
            const int ridx = res_padded ? plane * (POUT * POUT * 4) + ((out_y[i] + 1) * POUT + out_x[i] + 1) * 4
                                        : plane * (HO * HO * 4) + (out_y[i] * HO + out_x[i]) * 4;
            v += *reinterpret_cast<const floatx4 *>(res + ridx);
        }
        v.x = fused_act(v.x, act);
        v.y = fused_act(v.y, act);
        v.z = fused_act(v.z, act);
        v.w = fused_act(v.w, act);
        *reinterpret_cast<floatx4 *>(dst + didx) = v;
    }
}

// Stem: 3 input channels held as one plane of (r, g, b, 0) pixels; one MFMA per tap
// (reduction = the 4 floats of a pixel).  Weights: [tap][64 lanes], lane = kq*16 + co.
template <int NW>
__device__ __forceinline__ void fused_stem(const float *__restrict__ src, float *__restrict__ dst,
                                           const float *__restrict__ wq, const float *__restrict__ bias, int act,
                                           int tid)
{
    constexpr int H = 32, PIN = 34, PT = H * H / 16, MT = PT / NW, DST_PLANE = PIN * PIN * 4;
    const int lane = tid & 63, wave = tid >> 6, p = lane & 15, kq = lane >> 4;
    float w[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) w[t] = wq[t * 64 + lane];
    const floatx4 bv = *reinterpret_cast<const floatx4 *>(bias + kq * 4);
#pragma unroll 2
    for (int i = 0; i < MT; ++i) {
        const int P = (wave + i * NW) * 16 + p;
        const int oy = P / H, ox = P % H;
        floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const float x = src[((oy + t / 3) * PIN + ox + t % 3) * 4 + kq];
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w[t], x, acc, 0, 0, 0);
        }
        floatx4 v = acc + bv;
        v.x = fused_act(v.x, act);
        v.y = fused_act(v.y, act);
        v.z = fused_act(v.z, act);
        v.w = fused_act(v.w, act);
        *reinterpret_cast<floatx4 *>(dst + kq * DST_PLANE + ((oy + 1) * PIN + ox + 1) * 4) = v;
    }
}

__device__ inline float fused_wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <int NW>
__global__ __launch_bounds__(NW * 64) void resnet_fused_kernel(FusedArgs a)
{
    extern __shared__ float lds[];
    const int tid = threadIdx.x;
    const int n = blockIdx.x, s = blockIdx.y;

    // clear both regions (borders must be zero), then bring in the image as (r, g, b, 0) pixels
    for (int i = tid; i < kFusedLdsBytes / 16; i += NW * 64)
        reinterpret_cast<floatx4 *>(lds)[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    {
        const float *img = a.images + (size_t)n * 3072;
        float *plane = lds + a.ops[0].src_off;
        for (int e = tid; e < 3072; e += NW * 64) {
            const int pix = e / 3, c = e - pix * 3;
            const int y = pix >> 5, x = pix & 31;
            plane[((y + 1) * 34 + x + 1) * 4 + c] = img[e];
        }
    }
    __syncthreads();

    for (int o = 0; o < a.n_ops; ++o) {
        const FusedOp &op = a.ops[o];
        int bi = 0;
        if (op.slot >= 0 && s < a.S) bi = bits_index(a.schemes[(size_t)s * a.L + op.slot]);
        const float *wq = op.bank[bi];
        const float *src = lds + op.src_off;
        float *dst = lds + op.dst_off;
        const float *res = op.res_off >= 0 ? lds + op.res_off : nullptr;
        const bool rp = op.res_padded != 0, zr = op.zero_ring != 0;
        switch (op.type) {
        case kOpStem: fused_stem<NW>(src, dst, wq, op.bias, op.act, tid); break;
        case kOpC16: fused_conv<16, 16, 32, 1, 3, true, NW>(src, dst, res, rp, wq, op.bias, op.act, zr, tid); break;
        case kOpT16_32: fused_conv<16, 32, 32, 2, 3, true, NW>(src, dst, res, rp, wq, op.bias, op.act, zr, tid); break;
        case kOpS16_32: fused_conv<16, 32, 32, 2, 1, false, NW>(src, dst, res, rp, wq, op.bias, op.act, zr, tid); break;
        case kOpC32: fused_conv<32, 32, 16, 1, 3, true, NW>(src, dst, res, rp, wq, op.bias, op.act, zr, tid); break;
        case kOpT32_64: fused_conv<32, 64, 16, 2, 3, true, NW>(src, dst, res, rp, wq, op.bias, op.act, zr, tid); break;
        case kOpS32_64: fused_conv<32, 64, 16, 2, 1, false, NW>(src, dst, res, rp, wq, op.bias, op.act, zr, tid); break;
        case kOpC64: fused_conv<64, 64, 8, 1, 3, true, NW>(src, dst, res, rp, wq, op.bias, op.act, zr, tid); break;
        case kOpHead: {
            // 64 channels x 8x8 pixels (padded 10x10 planes): pool, classifier, argmax
            float *scratch = dst;            // [8][64] partial sums, then pooled[64], then z[classes]
            const int c = tid & 63, part = tid >> 6; // NW parts
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
            const int lane = tid & 63, wave = tid >> 6;
            for (int j = wave; j < op.classes; j += NW) {
                float t = fused_wave_sum(pooled[lane] * wq[j * 64 + lane]);
                if (lane == 0) z[j] = t + op.bias[j];
            }
            __syncthreads();
            if (tid == 0) {
                int best = 0;
                for (int j = 1; j < op.classes; ++j)
                    if (z[j] > z[best]) best = j;
                if (s < a.S) a.top1[(size_t)s * a.top1_stride + n] = best;
                else if (a.top1_base) a.top1_base[n] = best;
            }
            if (a.logits && s < a.S && tid < op.classes)
                a.logits[((size_t)s * a.logits_n + a.n0 + n) * op.classes + tid] = z[tid];
            break;
        }
        default: break;
        }
        __syncthreads();
    }
}

hipError_t fused_set_lds_limit()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&resnet_fused_kernel<kFusedThreads / 64>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLdsBytes);
}

hipError_t launch_fused(const FusedArgs &a, int s_total, hipStream_t st)
{
    if (a.N == 0 || s_total == 0) return hipSuccess;
    hipLaunchKernelGGL((resnet_fused_kernel<kFusedThreads / 64>), dim3(a.N, s_total), dim3(kFusedThreads),
                       kFusedLdsBytes, st, a);
    return hipGetLastError();
}

} // namespace aiq
