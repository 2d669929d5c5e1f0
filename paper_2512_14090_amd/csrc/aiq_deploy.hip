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

// two bf16 values (upper halves of a and b) as one dword, a first: bytes {a2, a3, b2, b3}
__device__ __forceinline__ uint32_t pack2(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

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
// pixel three planes (hi, mid, lo) of CKC bf16 channels, CKC channels per pass.  A wavefront
// owns 64 pixels x 32*NT output channels and issues, per tap and block of 16 channels,
// 2 * NT * 3 MFMAs from NT 16-byte global reads (codes, L2-resident) and six 16-byte LDS reads.

// Staging.  One item = eight channels of one staged pixel: two 16-byte global reads, three 16-byte
// LDS writes (the hi, mid and lo planes).  Item tid + 256 * i belongs to thread tid; which pixel
// and which eight channels of the pass it is does not change from pass to pass, so its LDS unit
// and its element offset from the workgroup's first image are formed once (kStageItems of them
// per thread; the host keeps a region's item count within that).  Per pass the reads of all items
// are issued first (stage_fetch), then split and written to LDS (stage_store).
constexpr int kStageItems = kCodeStageItems;

struct StageItems {
    int dst[kStageItems]; // LDS unit of the hi plane, -1: no such item
    int src[kStageItems]; // element offset of channel c0 + 8 * c8 at the pixel, -1: outside the image
};

template <int STRIDE, int PAD>
__device__ __forceinline__ void stage_plan(const CodeConvArgs &a, StageItems &it, int c8shift, int img0, int oy0, int tid)
{
    const int c8n = 1 << c8shift;
    const int per_row = a.LW << c8shift;
    const int total = a.G * a.RIN * per_row;
    const int g_lim = min(a.G, a.N - img0); // images of the group that exist
    const int iy0 = oy0 * STRIDE - PAD;
#pragma unroll
    for (int i = 0; i < kStageItems; ++i) {
        const int e = tid + i * 256;
        it.dst[i] = it.src[i] = -1;
        if (e < total) {
            const int row = (int)fd_div((uint32_t)e, a.div_per_row);
            const int rem = e - row * per_row;
            const int col = rem >> c8shift, c8 = rem & (c8n - 1);
            const int g = (int)fd_div((uint32_t)row, a.div_rin);
            const int iy = iy0 + row - g * a.RIN, ix = col - PAD;
            it.dst[i] = (row * a.LW + col) * 3 * a.PSU + c8;
            if ((unsigned)iy < (unsigned)a.Hin && (unsigned)ix < (unsigned)a.Win && g < g_lim)
                it.src[i] = ((g * a.Hin + iy) * a.Win + ix) * a.Cin + c8 * 8;
        }
    }
}

// in0: the workgroup's first image; offsets within its own images fit 32 bits whatever the batch
__device__ __forceinline__ void stage_fetch(const CodeConvArgs &a, const StageItems &it, floatx4 (&v)[kStageItems][2],
                                            const float *in0, int c0, int c8shift, int n_items, int tid)
{
    const int c = c0 + (tid & ((1 << c8shift) - 1)) * 8; // 256 is a multiple of the items per pixel: one c8 per thread
    const bool ok0 = c < a.Cin, ok1 = c + 4 < a.Cin;     // Cin % 4 == 0
#pragma unroll
    for (int i = 0; i < kStageItems; ++i) {
        v[i][0] = v[i][1] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (i < n_items && it.src[i] >= 0) {
            const float *src = in0 + it.src[i] + c0;
            if (ok0) v[i][0] = global_load4(src);
            if (ok1) v[i][1] = global_load4(src + 4);
        }
    }
}

__device__ __forceinline__ void stage_store(const CodeConvArgs &a, const StageItems &it, const floatx4 (&v)[kStageItems][2],
                                            uintx4 *lds4, int n_items)
{
#pragma unroll
    for (int i = 0; i < kStageItems; ++i) {
        if (i >= n_items || it.dst[i] < 0) continue;
        uint32_t hi[8], mid[8], lo[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            split3(v[i][0][e], hi[e], mid[e], lo[e]);
            split3(v[i][1][e], hi[4 + e], mid[4 + e], lo[4 + e]);
        }
        uintx4 *d = lds4 + it.dst[i];
        d[0] = uintx4{pack2(hi[0], hi[1]), pack2(hi[2], hi[3]), pack2(hi[4], hi[5]), pack2(hi[6], hi[7])};
        d[a.PSU] = uintx4{pack2(mid[0], mid[1]), pack2(mid[2], mid[3]), pack2(mid[4], mid[5]), pack2(mid[6], mid[7])};
        d[2 * a.PSU] = uintx4{pack2(lo[0], lo[1]), pack2(lo[2], lo[3]), pack2(lo[4], lo[5]), pack2(lo[6], lo[7])};
        __builtin_amdgcn_sched_barrier(0); // one item's 24 temporaries at a time: the accumulators are live here
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
    const uint16_t *wbase[NT];                 // the wavefront's code tiles (uniform)
#pragma unroll
    for (int n = 0; n < NT; ++n) wbase[n] = a.codes + (size_t)min(ct0 + n, a.cout_tiles - 1) * T * a.CB * 512;

    StageItems items;
    stage_plan<STRIDE, PAD>(a, items, c8shift, img0, oy0, tid);
    const int n_items = (a.G * a.RIN * (a.LW << c8shift) + 255) >> 8; // <= kStageItems (host)
    const float *in0 = a.in + (size_t)img0 * a.Hin * a.Win * a.Cin;

    for (int c0 = 0; c0 < a.CB * 16; c0 += a.CKC) {
        {
            // The pass's activations: all reads first, then split and written.  (Holding the next
            // pass's reads in registers across the MFMA loop does not pay: memory reads return in
            // order, so the loop's code reads would wait behind them.)  The other workgroup of the
            // compute unit computes meanwhile.
            floatx4 staged[kStageItems][2];
            stage_fetch(a, items, staged, in0, c0, c8shift, n_items, tid);
            if (c0) __syncthreads(); // the previous pass's LDS reads are done
            stage_store(a, items, staged, lds4, n_items);
        }
        __syncthreads();

        if (active) {
            // One flat sequence of (tap, channel block) steps, channel block fastest.  The codes of
            // step k+2 are requested during step k (three register sets in rotation: they come from
            // L2, about two steps away); the activations of step k+1 replace those of step k plane by
            // plane, each plane as soon as the MFMAs that read it have been issued.  Both addresses
            // advance by increments.
            const int ncb = min(a.CKC, a.CB * 16 - c0) >> 4;
            const int steps = T * ncb;
            const int w_tap_step = (a.CB - ncb + 1) * 512; // last block of a tap -> first block of the next
            int woff = (c0 >> 4) * 512, wc = 0;            // codes: element offset in the tile, block within the pass
            auto load_codes = [&](uintx4 (&wa)[NT]) {
#pragma unroll
                for (int n = 0; n < NT; ++n) wa[n] = *reinterpret_cast<const uintx4 *>(wbase[n] + woff + lane * 8);
                if (++wc == ncb) {
                    wc = 0;
                    woff += w_tap_step;
                } else {
                    woff += 512;
                }
            };
            const int a_tap_step = pix_units - (ncb - 1) * 2, a_row_step = (a.LW - KS) * pix_units;
            int tapoff = 0, ac = 0, akx = 0; // activations: LDS offset of the step's tap and block
            uintx4 xb[2][3];
            auto load_plane = [&](int pc) {
#pragma unroll
                for (int m = 0; m < 2; ++m) xb[m][pc] = lds4[lds_base[m] + tapoff + pc * a.PSU];
            };
            auto next_acts = [&]() {
                if (++ac == ncb) {
                    ac = 0;
                    tapoff += a_tap_step;
                    if (++akx == KS) {
                        akx = 0;
                        tapoff += a_row_step;
                    }
                } else {
                    tapoff += 2;
                }
            };
            auto mma_plane = [&](const uintx4 (&wa)[NT], int pc) {
#pragma unroll
                for (int m = 0; m < 2; ++m)
#pragma unroll
                    for (int n = 0; n < NT; ++n)
                        acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, wa[n]), __builtin_bit_cast(bf16x8, xb[m][pc]), acc[m][n], 0, 0, 0);
            };
            // step k: wa holds its codes, xb its activations; wa_later receives the codes of step k+2
            auto step = [&](int k, const uintx4 (&wa)[NT], uintx4 (&wa_later)[NT]) {
                if (k + 2 < steps) load_codes(wa_later);
                __builtin_amdgcn_sched_barrier(0); // the request stays ahead of the step's MFMAs
                const bool more = k + 1 < steps;
                if (more) next_acts();
#pragma unroll
                for (int pc = 2; pc >= 0; --pc) { // smallest terms first
                    mma_plane(wa, pc);
                    if (more) load_plane(pc);
                }
            };
            uintx4 w0[NT], w1[NT], w2[NT];
            load_codes(w0);
            if (steps > 1) load_codes(w1);
#pragma unroll
            for (int pc = 0; pc < 3; ++pc) load_plane(pc);
            int k = 0;
#pragma unroll 1
            for (; k + 3 <= steps; k += 3) {
                step(k, w0, w2);
                step(k + 1, w1, w0);
                step(k + 2, w2, w1);
            }
            if (k < steps) step(k, w0, w2);
            if (k + 1 < steps) step(k + 1, w1, w0);
        }
    }

    if (!active) return;
    // ---- epilogue: scale, bias, residual, activation.  Accumulator e of a lane is output channel
    // 8 * (e / 4) + 4 * kh + e % 4 of its tile.  Everything a pixel's stores need is read before its
    // first store, so the reads are in flight together instead of one round trip per store.
    const float lo = a.act >= 1 ? 0.0f : -__builtin_inff(), hi = a.act == 2 ? 6.0f : __builtin_inff();
    floatx4 sc[NT][4], bi[NT][4];
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const int co = (ct0 + n) * 32 + g4 * 8 + kh * 4;
            sc[n][g4] = bi[n][g4] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (co < a.Cout) { // Cout % 4 == 0
                sc[n][g4] = *reinterpret_cast<const floatx4 *>(a.scales + co);
                bi[n][g4] = *reinterpret_cast<const floatx4 *>(a.bias + co);
            }
        }
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        if (out_img[m] >= a.N || out_y[m] >= a.Hout) continue;
        const size_t pix = (((size_t)out_img[m] * a.Hout + out_y[m]) * a.Wout + out_x[m]) * a.Cout;
        float *out_p = a.out + pix;
        floatx4 rv[NT][4];
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int co = (ct0 + n) * 32 + g4 * 8 + kh * 4;
                rv[n][g4] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (a.res && co < a.Cout) rv[n][g4] = global_load4(a.res + pix + co);
            }
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int co = (ct0 + n) * 32 + g4 * 8 + kh * 4;
                if (co >= a.Cout) continue;
                floatx4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    v[e] = __builtin_amdgcn_fmed3f(__fmaf_rn(acc[m][n][g4 * 4 + e], sc[n][g4][e], bi[n][g4][e]) + rv[n][g4][e], lo, hi);
                *reinterpret_cast<floatx4 *>(out_p + co) = v;
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
