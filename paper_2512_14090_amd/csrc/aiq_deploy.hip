// gfx950 (CDNA4) kernels of the deployed-inference path: dense convolutions whose weights
// are the integer codes of a low-bit layer, on the bf16 matrix pipe.
//
// The paper deploys the model with the layers its search chose held at low precision and
// compares end-to-end throughput with the FP32 model (Implementation, experiment (3);
// Results, Analysis of AIQ Throughput Effects).  On this machine the lever is the matrix
// pipe's rate, not weight traffic: v_mfma_f32_32x32x16_bf16 runs sixteen times faster than
// the fp32 MFMA.
//
// A layer quantized to b <= 8 bits has weights w = code * s with |code| <= 127, so the code is
// exact in bf16.  A finite fp32 activation x is exactly hi + mid + lo, three bf16 terms (its 24
// significand bits cut into three groups of eight).  Hence
//     sum_k w_k x_k = s * (sum_k code_k hi_k + sum_k code_k mid_k + sum_k code_k lo_k),
// every product exact in the MFMA's fp32 accumulator: three bf16 MFMAs replace one fp32 MFMA
// and the result differs from the fp32 path only in the rounding of the accumulation and of
// the one multiplication by s.  Activations stay NHWC fp32 in memory, so layers on this path
// and layers on the fp32 path mix freely.
#include "aiq_internal.h"

#include <algorithm>

namespace aiq {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// hardware block b runs on XCD b % 8; XCD k gets the k-th contiguous stretch of logical blocks,
// so that regions sharing halo rows meet in one L2
__device__ inline uint32_t xcd_stretch_block(uint32_t b, uint32_t n)
{
    const uint32_t per = n >> 3, rem = n & 7u, xcd = b & 7u, idx = b >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

__device__ __forceinline__ floatx4 global_load4(const float *p)
{
    return *(const __attribute__((address_space(1))) floatx4 *)(p);
}

// x = hi + mid + lo exactly for finite x; each term is a bf16 value held in the upper half of
// an fp32 bit pattern (both subtractions are exact: they only clear leading significand bits)
__device__ __forceinline__ void split3(float x, uint32_t &hi, uint32_t &mid, uint32_t &lo)
{
    hi = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(hi);
    mid = __float_as_uint(r1) & 0xffff0000u;
    lo = __float_as_uint(r1 - __uint_as_float(mid));
}

// two bf16 values (upper halves of a and b) as one dword, a first
__device__ __forceinline__ uint32_t pack2(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

} // namespace

// ------------------------------------------------------------------ code packing
//
// int32 codes [cout][cin][taps] -> bf16 in the order the MFMA's A operand wants:
// [cout/32][tap][cin/16][64 lanes][8], lane = 32 * (k / 8) + row, element = k % 8, where row is
// the output channel within its tile of 32 and k the input channel within its block of 16.
// The destination has been cleared: padding rows and channels stay zero.
__global__ __launch_bounds__(256) void pack_codes_kernel(const int32_t *__restrict__ codes, uint16_t *__restrict__ out,
                                                         int cout, int cin, int taps, int cblocks)
{
    const int k = cin * taps;
    const size_t total = (size_t)cout * k;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int c = (int)(i / k), r = (int)(i - (size_t)c * k);
        const int ci = r / taps, t = r - ci * taps;
        const int ct = c >> 5, row = c & 31, cb = ci >> 4, kk = ci & 15;
        const size_t o = ((((size_t)ct * taps + t) * cblocks + cb) * 64 + (kk >> 3) * 32 + row) * 8 + (kk & 7);
        out[o] = (uint16_t)(__float_as_uint((float)codes[i]) >> 16); // |code| <= 127: exact
    }
}

hipError_t launch_pack_codes(const int32_t *codes, uint16_t *out, int cout, int cin, int taps, hipStream_t st)
{
    const size_t total = (size_t)cout * cin * taps;
    if (total == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(pack_codes_kernel, dim3(blocks), dim3(256), 0, st, codes, out, cout, cin, taps, (cin + 15) / 16);
    return hipGetLastError();
}

// ------------------------------------------------------------------ convolution on integer codes
//
// Implicit GEMM on v_mfma_f32_32x32x16_bf16: A = codes (rows = 32 output channels), B = 32
// output pixels, k = 16 input channels of one tap.  A lane's sixteen accumulator values are
// four groups of four consecutive output channels of one pixel: four 16-byte NHWC stores.
//
// Workgroup = 4 wavefronts; it stages the input rows of its region in LDS already split: per
// pixel three planes (hi, mid, lo) of CKC bf16 channels.  A wavefront owns 64 pixels x 32*NT
// output channels and issues, per tap and block of 16 channels, 2 * NT * 3 MFMAs from NT
// 16-byte global reads (codes, L2-resident) and six 16-byte LDS reads.

// Stages channels [c0, c0 + CKC) of the region's input rows, zero outside the image and past
// Cin.  One item = eight channels of one pixel: two 16-byte global reads, three 16-byte LDS
// writes.  Three items per thread are in flight before the first is split.
template <int STRIDE, int PAD>
__device__ __forceinline__ void stage_split_rows(const CodeConvArgs &a, uintx4 *lds4, int c0, int c8shift, int img0,
                                                 int oy0, int tid)
{
    constexpr int UB = 3;
    const int c8n = 1 << c8shift;
    const int per_row = a.LW << c8shift;
    const int total = a.G * a.RIN * per_row;
    for (int base = tid; base < total; base += 256 * UB) {
        floatx4 v[UB][2];
        int dst[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int it = base + u * 256;
            v[u][0] = v[u][1] = floatx4{0.f, 0.f, 0.f, 0.f};
            dst[u] = -1;
            if (it < total) {
                const int row = (int)fd_div((uint32_t)it, a.div_per_row);
                const int rem = it - row * per_row;
                const int col = rem >> c8shift, c8 = rem & (c8n - 1);
                const int g = (int)fd_div((uint32_t)row, a.div_rin);
                const int r = row - g * a.RIN;
                const int iy = oy0 * STRIDE - PAD + r, ix = col - PAD, img = img0 + g;
                const int c = c0 + c8 * 8;
                dst[u] = (row * a.LW + col) * 3 * a.PSU + c8;
                if (iy >= 0 && iy < a.Hin && ix >= 0 && ix < a.Win && img < a.N && c < a.Cin) { // Cin % 4 == 0
                    const float *src = a.in + (((size_t)img * a.Hin + iy) * a.Win + ix) * a.Cin + c;
                    v[u][0] = global_load4(src);
                    if (c + 4 < a.Cin) v[u][1] = global_load4(src + 4);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            if (dst[u] < 0) continue;
            uint32_t hi[8], mid[8], lo[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                split3(v[u][0][e], hi[e], mid[e], lo[e]);
                split3(v[u][1][e], hi[4 + e], mid[4 + e], lo[4 + e]);
            }
            lds4[dst[u]] = uintx4{pack2(hi[0], hi[1]), pack2(hi[2], hi[3]), pack2(hi[4], hi[5]), pack2(hi[6], hi[7])};
            lds4[dst[u] + a.PSU] =
                uintx4{pack2(mid[0], mid[1]), pack2(mid[2], mid[3]), pack2(mid[4], mid[5]), pack2(mid[6], mid[7])};
            lds4[dst[u] + 2 * a.PSU] =
                uintx4{pack2(lo[0], lo[1]), pack2(lo[2], lo[3]), pack2(lo[4], lo[5]), pack2(lo[6], lo[7])};
        }
    }
}

template <int KS, int STRIDE, int NT>
__global__ __launch_bounds__(256, 2) void conv_codes_kernel(CodeConvArgs a)
{
    extern __shared__ float lds_raw[];
    uintx4 *lds4 = reinterpret_cast<uintx4 *>(lds_raw);
    constexpr int T = KS * KS;
    constexpr int PAD = KS == 3 ? 1 : 0;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // uniform: tile and code addresses stay scalar

    const int bx = (int)xcd_stretch_block(blockIdx.x, gridDim.x);
    int img0, oy0;
    if (a.G > 1) {
        img0 = bx * a.G;
        oy0 = 0;
    } else {
        img0 = bx / a.regions_per_image;
        oy0 = (bx - img0 * a.regions_per_image) * a.R;
    }

    const int wpx = wave % a.wave_px_split;
    const int wco = wave / a.wave_px_split;
    const int wco_count = 4 / a.wave_px_split;
    const int ct0 = (blockIdx.y * wco_count + wco) * NT;
    const int p = lane & 31, kh = lane >> 5; // pixel within the tile of 32; which eight of the 16 channels

    const int pix_units = 3 * a.PSU; // 16-byte units per staged pixel
    int lds_base[2];
    int out_img[2], out_y[2], out_x[2];
    const int rw = a.R * a.Wout;
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const uint32_t P = (uint32_t)(wpx * 64 + m * 32 + p);
        const uint32_t g = fd_div(P, a.div_rw);
        const uint32_t rem = P - g * rw;
        const uint32_t oy = fd_div(rem, a.div_wout);
        const uint32_t ox = rem - oy * a.Wout;
        const bool in_region = g < (uint32_t)a.G; // lanes past the region's last pixel compute nothing useful
        lds_base[m] = in_region ? ((g * a.RIN + oy * STRIDE) * a.LW + ox * STRIDE) * pix_units + kh : kh;
        out_img[m] = in_region ? img0 + (int)g : a.N;
        out_y[m] = oy0 + oy;
        out_x[m] = ox;
    }

    floatx16 acc[2][NT];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[m][n][e] = 0.0f;

    const int c8shift = __ffs(a.CKC >> 3) - 1; // CKC is 16, 32 or 64
    const bool active = ct0 < a.cout_tiles;    // wavefronts past the last output-channel tile only help staging

    for (int c0 = 0; c0 < a.CB * 16; c0 += a.CKC) {
        if (c0) __syncthreads();
        stage_split_rows<STRIDE, PAD>(a, lds4, c0, c8shift, img0, oy0, tid);
        __syncthreads();

        if (active) {
            // one flat sequence of (tap, channel block) steps; step k+1's codes and activations are
            // requested before step k's MFMAs, alternating between two register sets
            const int ncb = min(a.CKC, a.CB * 16 - c0) >> 4;
            const int cb0 = c0 >> 4;
            const int steps = T * ncb;
            int lt = 0, lc = 0;
            auto load_step = [&](uintx4 (&wa)[NT], uintx4 (&xb)[2][3]) {
                const int t = lt, cbl = lc;
                if (++lc == ncb) {
                    lc = 0;
                    ++lt;
                }
                const int ky = t / KS, kx = t - ky * KS;
                const int tapoff = (ky * a.LW + kx) * pix_units + cbl * 2;
#pragma unroll
                for (int n = 0; n < NT; ++n) {
                    const int ct = min(ct0 + n, a.cout_tiles - 1);
                    const uint16_t *wrow = a.codes + (((size_t)ct * T + t) * a.CB + cb0 + cbl) * 512; // uniform
                    wa[n] = *reinterpret_cast<const uintx4 *>(wrow + lane * 8);
                }
#pragma unroll
                for (int m = 0; m < 2; ++m)
#pragma unroll
                    for (int pc = 0; pc < 3; ++pc) xb[m][pc] = lds4[lds_base[m] + tapoff + pc * a.PSU];
            };
            auto mma_step = [&](const uintx4 (&wa)[NT], const uintx4 (&xb)[2][3]) {
#pragma unroll
                for (int pc = 2; pc >= 0; --pc) // smallest terms first
#pragma unroll
                    for (int m = 0; m < 2; ++m)
#pragma unroll
                        for (int n = 0; n < NT; ++n)
                            acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8, wa[n]), __builtin_bit_cast(bf16x8, xb[m][pc]), acc[m][n], 0, 0, 0);
            };
            uintx4 wa0[NT], xb0[2][3], wa1[NT], xb1[2][3];
            load_step(wa0, xb0);
            int k = 0;
#pragma unroll 1
            for (; k + 2 <= steps; k += 2) {
                load_step(wa1, xb1);
                mma_step(wa0, xb0);
                if (k + 2 < steps) load_step(wa0, xb0);
                mma_step(wa1, xb1);
            }
            if (k < steps) mma_step(wa0, xb0); // odd number of steps: the last one is already loaded
        }
    }

    if (!active) return;
    // ---- epilogue: scale, bias, residual, activation.  Accumulator e of a lane is output channel
    // 8 * (e / 4) + 4 * kh + e % 4 of its tile
    const float lo = a.act >= 1 ? 0.0f : -__builtin_inff(), hi = a.act == 2 ? 6.0f : __builtin_inff();
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        if (out_img[m] >= a.N || out_y[m] >= a.Hout) continue;
        const size_t pix = (((size_t)out_img[m] * a.Hout + out_y[m]) * a.Wout + out_x[m]) * a.Cout;
        float *out_p = a.out + pix;
        const float *res_p = a.res ? a.res + pix : nullptr;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int co = (ct0 + n) * 32 + g4 * 8 + kh * 4;
                if (co >= a.Cout) continue; // Cout % 4 == 0
                const floatx4 sc = *reinterpret_cast<const floatx4 *>(a.scales + co);
                const floatx4 bi = *reinterpret_cast<const floatx4 *>(a.bias + co);
                floatx4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = __fmaf_rn(acc[m][n][g4 * 4 + e], sc[e], bi[e]);
                if (res_p) v += *reinterpret_cast<const floatx4 *>(res_p + co);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = __builtin_amdgcn_fmed3f(v[e], lo, hi);
                *reinterpret_cast<floatx4 *>(out_p + co) = v;
            }
        }
    }
}

template <int KS, int STRIDE>
static hipError_t launch_codes_nt(const CodeConvArgs &a, int nt, size_t lds_bytes, dim3 grid, hipStream_t st)
{
    switch (nt) {
    case 1: hipLaunchKernelGGL((conv_codes_kernel<KS, STRIDE, 1>), grid, dim3(256), lds_bytes, st, a); break;
    case 2: hipLaunchKernelGGL((conv_codes_kernel<KS, STRIDE, 2>), grid, dim3(256), lds_bytes, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_conv_codes(const CodeConvArgs &a, int ks, int stride, int nt, size_t lds_bytes, dim3 grid,
                             hipStream_t st)
{
    if (ks == 3 && stride == 1) return launch_codes_nt<3, 1>(a, nt, lds_bytes, grid, st);
    if (ks == 3 && stride == 2) return launch_codes_nt<3, 2>(a, nt, lds_bytes, grid, st);
    if (ks == 1 && stride == 1) return launch_codes_nt<1, 1>(a, nt, lds_bytes, grid, st);
    if (ks == 1 && stride == 2) return launch_codes_nt<1, 2>(a, nt, lds_bytes, grid, st);
    return hipErrorInvalidValue;
}

template <int KS, int STRIDE, int NT>
static hipError_t codes_lds_t()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_codes_kernel<KS, STRIDE, NT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

// Dynamic LDS above 64 KB has to be allowed per kernel.
hipError_t conv_codes_set_lds_limits()
{
    hipError_t e = hipSuccess;
#define AIQ_SET(KS, ST)                                  \
    if (e == hipSuccess) e = codes_lds_t<KS, ST, 1>();   \
    if (e == hipSuccess) e = codes_lds_t<KS, ST, 2>();
    AIQ_SET(3, 1)
    AIQ_SET(3, 2)
    AIQ_SET(1, 1)
    AIQ_SET(1, 2)
#undef AIQ_SET
    return e;
}

} // namespace aiq
