// Deployed inference of the activation-quantization variant on the INT8 matrix pipe of gfx950.
//
// In that variant a scheme layer at b <= 8 bits reads its input tensor quantized to b bits with
// one scale per image (paper: Problem Formulation gives a layer its bit-width; the reading of it
// for activations is the one the scoring path implements).  Then both factors of every product
// are integer codes: w = q_w * s_w[c], x = q_x * s_x[n], |q| <= 127, and
//     sum_k w_k x_k = s_w[c] * s_x[n] * sum_k q_w,k q_x,k
// with the integer sum exact in the MFMA's int32 accumulator.  The layer is two launches:
//   act_codes_kernel   the producer's fp32 tensor -> int8 codes and the image's scale (the scoring
//                      path's quantizer, step for step; what it would multiply back is never formed);
//   conv_i8_kernel     implicit GEMM on v_mfma_i32_32x32x32_i8: A = weight codes (rows = 32 output
//                      channels), B = 32 output pixels, k = 32 input channels of one tap; epilogue
//                      float(acc) * (s_w * s_x) + bias (+ residual, read unquantized), activation.
// One int8 MFMA stands where the fp32 kernels issue 32 and the bf16-code kernels 6, and the consumer
// reads one byte per activation: the layer is bound by its fp32 output and by the quantizer's pass.
#include "aiq_internal.h"

#include <algorithm>

namespace aiq {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

// hardware block b runs on XCD b % 8; XCD k gets the k-th contiguous stretch of logical blocks,
// so that regions sharing halo rows meet in one L2
__device__ inline uint32_t xcd_stretch(uint32_t b, uint32_t n)
{
    const uint32_t per = n >> 3, rem = n & 7u, xcd = b & 7u, idx = b >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

__device__ inline float wave_max_f(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// Maximum of a non-negative value over the wavefront, left in lane 63, by data-parallel-primitive moves
// (no LDS traffic): shifts within rows of 16 lanes give lane 15 of each row its row's maximum, the two
// row broadcasts carry it on to lane 63.  Lanes shifted in from outside a row read 0, the identity here.
template <int CTRL>
__device__ __forceinline__ float dpp_max_step(float x)
{
    return fmaxf(x, __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), CTRL, 0xf, 0xf, true)));
}
__device__ __forceinline__ float wave_max_nonneg(float v)
{
    v = dpp_max_step<0x111>(v); // row_shr:1
    v = dpp_max_step<0x112>(v); // row_shr:2
    v = dpp_max_step<0x114>(v); // row_shr:4
    v = dpp_max_step<0x118>(v); // row_shr:8
    v = dpp_max_step<0x142>(v); // row_bcast:15
    v = dpp_max_step<0x143>(v); // row_bcast:31
    return v;
}

// 16 bytes through an explicit global address (global_load, not flat_load)
__device__ __forceinline__ uintx4 gload16(const void *p)
{
    return *(const __attribute__((address_space(1))) uintx4 *)(p);
}

// code of one value: IEEE division, round half to even, clamp (the quantizer's first three steps)
__device__ __forceinline__ int code_of(float x, float s, int qmax)
{
    const int q = (int)rintf(__fdiv_rn(x, s));
    return min(max(q, -qmax), qmax);
}

// four values -> four codes in one dword, first value in the low byte
__device__ __forceinline__ uint32_t pack_codes4(floatx4 f, float s, int qmax)
{
    return (uint32_t)(code_of(f.x, s, qmax) & 255) | ((uint32_t)(code_of(f.y, s, qmax) & 255) << 8) |
           ((uint32_t)(code_of(f.z, s, qmax) & 255) << 16) | ((uint32_t)(code_of(f.w, s, qmax) & 255) << 24);
}

} // namespace

// ------------------------------------------------------------------ activation codes
//
// One workgroup per image: absolute maximum of the image's tensor (exact in any order), scale
// = amax / qmax (1 for a zero tensor), then sixteen codes per 16-byte store.  elems % 16 == 0.
__global__ __launch_bounds__(256) void act_codes_kernel(const float *__restrict__ in, int8_t *__restrict__ codes,
                                                        float *__restrict__ xscale, int elems, int bits)
{
    __shared__ float wmax[4];
    const int n = blockIdx.x, tid = threadIdx.x;
    const float *x = in + (size_t)n * elems;
    const int n4 = elems >> 2;
    // eight 16-byte reads in flight per thread: the pass is a chain of memory latencies otherwise
    constexpr int kDepth = 8;
    float amax = 0.0f;
    for (int base = tid; base < n4; base += 256 * kDepth) {
        uintx4 v[kDepth];
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int i = base + u * 256;
            v[u] = i < n4 ? gload16(x + (size_t)i * 4) : uintx4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const floatx4 f = __builtin_bit_cast(floatx4, v[u]);
            amax = fmaxf(fmaxf(amax, fmaxf(fabsf(f.x), fabsf(f.y))), fmaxf(fabsf(f.z), fabsf(f.w)));
        }
    }
    amax = wave_max_f(amax);
    if ((tid & 63) == 0) wmax[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    const int qmax = (1 << (bits - 1)) - 1;
    const float sc = amax > 0.0f ? __fdiv_rn(amax, (float)qmax) : 1.0f;
    if (tid == 0) xscale[n] = sc;
    // second pass: a lane turns one 16-byte read into four codes, one 4-byte store; consecutive lanes
    // on consecutive addresses both ways
    uint32_t *out32 = reinterpret_cast<uint32_t *>(codes + (size_t)n * elems);
    for (int base = tid; base < n4; base += 256 * kDepth) {
        uintx4 v[kDepth];
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int i = base + u * 256;
            v[u] = i < n4 ? gload16(x + (size_t)i * 4) : uintx4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int i = base + u * 256;
            if (i < n4) out32[i] = pack_codes4(__builtin_bit_cast(floatx4, v[u]), sc, qmax);
        }
    }
}

// The same codes when the producing kernel has left the images' absolute maxima (bit patterns of
// non-negative floats, combined by integer atomic maxima: exact in any order): one streaming pass,
// blockIdx.y = image, a thread converts kPieces 16-byte pieces.
constexpr int kCodeReads = 8; // 16-byte reads in flight per thread

__global__ __launch_bounds__(256) void act_codes_known_amax_kernel(const float *__restrict__ in,
                                                                   const uint32_t *__restrict__ amax_bits,
                                                                   int8_t *__restrict__ codes, float *__restrict__ xscale,
                                                                   int elems, int bits)
{
    const int n = blockIdx.y, tid = threadIdx.x;
    const uintx4 *x4 = reinterpret_cast<const uintx4 *>(in + (size_t)n * elems);
    const float amax = __uint_as_float(amax_bits[n]);
    const int qmax = (1 << (bits - 1)) - 1;
    const float sc = amax > 0.0f ? __fdiv_rn(amax, (float)qmax) : 1.0f;
    if (blockIdx.x == 0 && tid == 0) xscale[n] = sc;
    uint32_t *out32 = reinterpret_cast<uint32_t *>(codes + (size_t)n * elems);
    const int n4 = elems >> 2;
    const int base = blockIdx.x * (256 * kCodeReads) + tid;
    uintx4 v[kCodeReads];
#pragma unroll
    for (int u = 0; u < kCodeReads; ++u) {
        const int i = base + u * 256;
        v[u] = i < n4 ? __builtin_nontemporal_load(x4 + i) : uintx4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < kCodeReads; ++u) {
        const int i = base + u * 256;
        if (i < n4) out32[i] = pack_codes4(__builtin_bit_cast(floatx4, v[u]), sc, qmax);
    }
}

hipError_t launch_act_codes(const float *in, const uint32_t *amax_bits, int8_t *codes, float *xscale, int n, int elems,
                            int bits, hipStream_t st)
{
    if (n == 0 || elems == 0) return hipSuccess;
    if (amax_bits) {
        const unsigned bx = (unsigned)(((elems >> 2) + 256 * kCodeReads - 1) / (256 * kCodeReads));
        hipLaunchKernelGGL(act_codes_known_amax_kernel, dim3(bx, n), dim3(256), 0, st, in, amax_bits, codes, xscale, elems, bits);
    } else {
        hipLaunchKernelGGL(act_codes_kernel, dim3(n), dim3(256), 0, st, in, codes, xscale, elems, bits);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ weight code packing
//
// int32 codes [cout][cin][taps] -> int8 in the order the MFMA's A operand wants:
// [cout/32][tap][cin/32][64 lanes][16], lane = 32 * (k / 16) + row, byte = k % 16, where row is the
// output channel within its tile of 32 and k the input channel within its block of 32.
// The destination has been cleared: padding rows and channels stay zero.
__global__ __launch_bounds__(256) void pack_codes_i8_kernel(const int32_t *__restrict__ codes, int8_t *__restrict__ out,
                                                            int cout, int cin, int taps, int kblocks)
{
    const int k = cin * taps;
    const size_t total = (size_t)cout * k;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int c = (int)(i / k), r = (int)(i - (size_t)c * k);
        const int ci = r / taps, t = r - ci * taps;
        const int ct = c >> 5, row = c & 31, kb = ci >> 5, kk = ci & 31;
        const size_t o = ((((size_t)ct * taps + t) * kblocks + kb) * 64 + (kk >> 4) * 32 + row) * 16 + (kk & 15);
        out[o] = (int8_t)codes[i]; // |code| <= 127
    }
}

hipError_t launch_pack_codes_i8(const int32_t *codes, int8_t *out, int cout, int cin, int taps, hipStream_t st)
{
    const size_t total = (size_t)cout * cin * taps;
    if (total == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(pack_codes_i8_kernel, dim3(blocks), dim3(256), 0, st, codes, out, cout, cin, taps, (cin + 31) / 32);
    return hipGetLastError();
}

// ------------------------------------------------------------------ convolution on int8 codes
//
// Workgroup = 4 wavefronts; a wavefront owns 64 pixels (two MFMA tiles) x 32*NT output channels of a
// region (whole rows of one image, or whole small images).  Per pass of CKB blocks of 32 channels the
// workgroup stages in LDS the region's input rows (one 16-byte piece = 16 channels of a pixel, copied
// as it is; pixels outside the image are code 0; the pixel stride carries 16 bytes of padding so that
// the 32 pixels of an operand read spread over the banks) and the weight codes of its output tiles for
// those channels.  The taps are unrolled; every operand read is the lane's base address plus an
// immediate.
//
// The MFMA work is small (one instruction where the fp32 kernels issue 32), so the kernel is a data
// mover: where a layer needs a single pass, a workgroup keeps the weight codes in LDS for RPW
// consecutive regions and requests the next region's activations (registers) before it computes and
// stores the current one, so that reads, MFMAs and the fp32 stores of neighbouring regions overlap.
template <int KS, int STRIDE, int NT>
__global__ __launch_bounds__(256, 2) void conv_i8_kernel(I8ConvArgs a)
{
    extern __shared__ float lds_raw[];
    char *ldsb = reinterpret_cast<char *>(lds_raw);
    constexpr int T = KS * KS;
    constexpr int PAD = KS == 3 ? 1 : 0;
    constexpr int MT = 2;
    constexpr int KI = 6; // 16-byte pieces a thread holds for the next region
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wpx = wave % a.wave_px_split;
    const int wco = wave / a.wave_px_split;
    const int first_tile = blockIdx.y * a.tiles_per_wg;
    const int ct0 = first_tile + wco * NT;
    const int p = lane & 31, kh = lane >> 5;

    uint32_t lds_base[MT];
    const int rw = a.R * a.Wout;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const uint32_t P = (uint32_t)(wpx * (32 * MT) + m * 32 + p);
        const uint32_t g = fd_div(P, a.div_rw);
        const uint32_t rem = P - g * rw;
        const uint32_t oy = fd_div(rem, a.div_wout);
        const uint32_t ox = rem - oy * a.Wout;
        const bool in_region = g < (uint32_t)a.G; // lanes past the region's last pixel compute nothing useful
        lds_base[m] = (in_region ? ((g * a.RIN + oy * STRIDE) * a.LW + ox * STRIDE) * (uint32_t)a.PSB : 0u) + kh * 16u;
    }

    const bool active = ct0 < a.cout_tiles; // wavefronts past the last output-channel tile only help staging
    const int upp = a.CKB * 2;              // 16-byte pieces of one staged pixel (2 or 4)
    const int upp_shift = upp == 2 ? 1 : 2;
    const int per_row = a.LW * upp;
    const int act_items = a.G * a.RIN * per_row;
    const int code_run = 64 * a.CKB;        // pieces of one (tile, tap)
    const int code_items = a.tiles_per_wg * T * code_run;
    const bool single = a.CBK <= a.CKB;     // one pass: the weight codes stay in LDS from region to region
    const bool ahead = single && act_items <= KI * 256;
    const size_t img_bytes = (size_t)a.Hin * a.Win * a.Cin;

    // where piece e of a pass comes from and goes to; -1: no such piece / always outside the image
    auto item_plan = [&](int e, int kb0, int &dst, int &src, int &rl, int &g) {
        dst = src = -1;
        rl = g = 0;
        if (e >= act_items) return;
        const int row = (int)fd_div((uint32_t)e, a.div_per_row);
        const int rem = e - row * per_row;
        const int col = rem >> upp_shift, u = rem & (upp - 1);
        g = (int)fd_div((uint32_t)row, a.div_rin);
        rl = row - g * a.RIN;
        const int ix = col - PAD, c = kb0 * 32 + u * 16;
        dst = (row * a.LW + col) * a.PSB + u * 16;
        if ((unsigned)ix < (unsigned)a.Win && c < a.Cin) src = (g * a.Hin * a.Win + ix) * a.Cin + c;
    };
    // weight codes of a pass: piece j goes to code_off + 16 * j, order [tile][tap][block][lane]
    auto stage_codes = [&](int kb0, int ncb) {
        constexpr int kBatch = 6;
        for (int base = tid; base < code_items; base += 256 * kBatch) {
            uintx4 v[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const int j = base + i * 256;
                v[i] = uintx4{0u, 0u, 0u, 0u};
                if (j < code_items) {
                    const int r = j / code_run, q = j - r * code_run;
                    const int ctl = r / T, t = r - ctl * T;
                    const int kbl = q >> 6, ln = q & 63;
                    const int ct = min(first_tile + ctl, a.cout_tiles - 1);
                    if (kbl < ncb) v[i] = gload16(a.codes + ((((size_t)ct * T + t) * a.CBK + kb0 + kbl) * 64 + ln) * 16);
                }
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const int j = base + i * 256;
                if (j < code_items) *reinterpret_cast<uintx4 *>(ldsb + a.code_off + j * 16) = v[i];
            }
        }
    };

    // this thread's pieces of a single-pass region, the same from region to region
    int it_dst[KI], it_src[KI], it_rg[KI];
    if (ahead) {
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            int rl, g;
            item_plan(tid + i * 256, 0, it_dst[i], it_src[i], rl, g);
            it_rg[i] = rl | (g << 16);
        }
    }
    // region index -> first image, first output row
    auto region_at = [&](int region, int &img0, int &oy0) {
        if (a.G > 1) {
            img0 = region * a.G;
            oy0 = 0;
        } else {
            img0 = region / a.regions_per_image;
            oy0 = (region - img0 * a.regions_per_image) * a.R;
        }
    };
    auto fetch_ahead = [&](int region, uintx4 (&v)[KI]) {
        int img0, oy0;
        region_at(region, img0, oy0);
        const int iy0 = oy0 * STRIDE - PAD, g_lim = min(a.G, a.N - img0);
        const int8_t *in0 = a.in + (size_t)img0 * img_bytes;
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            v[i] = uintx4{0u, 0u, 0u, 0u};
            const int iy = iy0 + (it_rg[i] & 0xffff), g = it_rg[i] >> 16;
            if (it_src[i] >= 0 && (unsigned)iy < (unsigned)a.Hin && g < g_lim)
                v[i] = gload16(in0 + it_src[i] + (size_t)iy * a.Win * a.Cin);
        }
    };

    const int bx = (int)xcd_stretch(blockIdx.x, gridDim.x);
    const int r_begin = bx * a.RPW, r_end = min(r_begin + a.RPW, a.total_regions);
    if (r_begin >= r_end) return;
    if (single) stage_codes(0, a.CBK);
    // per-channel scale and bias of the chunk this lane stores in the epilogue: the same for every region
    floatx4 sc = {0.f, 0.f, 0.f, 0.f}, bi = {0.f, 0.f, 0.f, 0.f};
    {
        const int co = ct0 * 32 + (lane & (8 * NT - 1)) * 4;
        if (active && co < a.Cout) {
            sc = __builtin_bit_cast(floatx4, gload16(a.scales + co));
            bi = __builtin_bit_cast(floatx4, gload16(a.bias + co));
        }
    }
    uintx4 ahead_v[KI];
    if (ahead) fetch_ahead(r_begin, ahead_v);

    for (int region = r_begin; region < r_end; ++region) {
        int img0, oy0;
        region_at(region, img0, oy0);
        const int iy0 = oy0 * STRIDE - PAD, g_lim = min(a.G, a.N - img0);
        const int8_t *in0 = a.in + (size_t)img0 * img_bytes;

        intx16 acc[MT][NT];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int n = 0; n < NT; ++n)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[m][n][e] = 0;
        // The activation scales the epilogue multiplies by are requested here, so that they arrive during
        // the MFMA loop: a region of one image has one (uniform), a region of several small images one per
        // image (lane g holds image g's; the epilogue picks by pixel).
        float xs_img = 0.0f;
        if (a.G == 1) xs_img = a.xscale[img0];
        else if (lane < g_lim) xs_img = a.xscale[img0 + lane];

        for (int kb0 = 0; kb0 < a.CBK; kb0 += a.CKB) {
            const int ncb = min(a.CKB, a.CBK - kb0);
            if (kb0) __syncthreads(); // the previous pass's LDS reads are done
            if (ahead) {
#pragma unroll
                for (int i = 0; i < KI; ++i)
                    if (it_dst[i] >= 0) *reinterpret_cast<uintx4 *>(ldsb + it_dst[i]) = ahead_v[i];
            } else {
                constexpr int kBatch = 6;
                for (int base = tid; base < act_items; base += 256 * kBatch) {
                    uintx4 v[kBatch];
                    int dst[kBatch];
#pragma unroll
                    for (int i = 0; i < kBatch; ++i) {
                        int src, rl, g;
                        item_plan(base + i * 256, kb0, dst[i], src, rl, g);
                        v[i] = uintx4{0u, 0u, 0u, 0u};
                        const int iy = iy0 + rl;
                        if (src >= 0 && (unsigned)iy < (unsigned)a.Hin && g < g_lim)
                            v[i] = gload16(in0 + src + (size_t)iy * a.Win * a.Cin);
                    }
#pragma unroll
                    for (int i = 0; i < kBatch; ++i)
                        if (dst[i] >= 0) *reinterpret_cast<uintx4 *>(ldsb + dst[i]) = v[i];
                }
            }
            if (!single) stage_codes(kb0, ncb);
            __syncthreads();
            if (ahead && region + 1 < r_end) fetch_ahead(region + 1, ahead_v); // travels while this region computes and stores

            const uint32_t wbase = (uint32_t)a.code_off + (uint32_t)(wco * NT * T * code_run + lane) * 16u;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                // a tap's operand reads stay inside the tap: hoisted over the unrolled taps they would take
                // more registers than the kernel has, and the wavefronts of the other workgroup cover the wait
                __builtin_amdgcn_sched_barrier(0);
                const uint32_t xoff = (uint32_t)((t / KS) * a.LW + (t % KS)) * (uint32_t)a.PSB;
#pragma unroll 1
                for (int kbl = 0; kbl < ncb; ++kbl) {
                    intx4 wa[NT], xb[MT];
#pragma unroll
                    for (int n = 0; n < NT; ++n)
                        wa[n] = *reinterpret_cast<const intx4 *>(ldsb + wbase + (uint32_t)(((n * T + t) * a.CKB + kbl) * 1024));
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        xb[m] = *reinterpret_cast<const intx4 *>(ldsb + lds_base[m] + xoff + (uint32_t)kbl * 32u);
#pragma unroll
                    for (int m = 0; m < MT; ++m)
#pragma unroll
                        for (int n = 0; n < NT; ++n)
                            acc[m][n] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wa[n], xb[m], acc[m][n], 0, 0, 0);
                }
            }
        }

        // ---- epilogue: through LDS (a lane's accumulators are four groups of four consecutive output
        // channels of one pixel; consecutive lanes then store consecutive 16-byte chunks of a pixel: whole
        // lines), scale, bias, residual, activation.  Chunk c of row r lives in unit r * U + (c ^ (r % U)).
        // The tiles lie over the staged activations (never over the weight codes).
        __syncthreads();
        if (active) {
            constexpr int U = 8 * NT;
            // the lane arithmetic of the epilogue is redone per region: kept across the region loop it
            // would push the accumulators out of the register file
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int p = ln & 31, kh = ln >> 5;
            uintx4 *tile = reinterpret_cast<uintx4 *>(ldsb) + wave * 32 * U;
            const float lo = a.act >= 1 ? 0.0f : -__builtin_inff(), hi = a.act == 2 ? 6.0f : __builtin_inff();
            const int px_img = a.Hout * a.Wout;
            const size_t first_px = a.G > 1 ? (size_t)img0 * px_img : ((size_t)img0 * a.Hout + oy0) * a.Wout;
            const int valid_px = a.G > 1 ? g_lim * px_img : min(a.R, a.Hout - oy0) * a.Wout;
            float *out0 = a.out + first_px * a.Cout;
            const float *res0 = a.res ? a.res + first_px * a.Cout : nullptr;
            constexpr int ROWS = 64 / U, ITS = 32 / ROWS;
            const int chunk = ln & (U - 1), sub = ln / U;
            const int co = ct0 * 32 + chunk * 4;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float vmax = 0.0f; // largest magnitude this lane stores of tile m
                // accumulator e of a lane is output channel 8 * (e / 4) + 4 * kh + e % 4 of its tile
#pragma unroll
                for (int n = 0; n < NT; ++n)
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4) {
                        const int c = n * 8 + g4 * 2 + kh;
                        const floatx4 v = {(float)acc[m][n][g4 * 4], (float)acc[m][n][g4 * 4 + 1],
                                           (float)acc[m][n][g4 * 4 + 2], (float)acc[m][n][g4 * 4 + 3]};
                        tile[p * U + (c ^ (p & (U - 1)))] = __builtin_bit_cast(uintx4, v);
                    }
                floatx4 rv[ITS];
                float xs[ITS];
#pragma unroll
                for (int it = 0; it < ITS; ++it) {
                    const int P = wpx * (32 * MT) + m * 32 + it * ROWS + sub;
                    rv[it] = floatx4{0.f, 0.f, 0.f, 0.f};
                    // every lane takes part in the shuffle; images past the group's last give 0 and are not stored
                    const int g = a.G > 1 ? min((int)fd_div((uint32_t)P, a.div_pximg), 63) : 0;
                    xs[it] = a.G > 1 ? __shfl(xs_img, g, 64) : xs_img;
                    if (res0 && co < a.Cout && P < valid_px)
                        rv[it] = __builtin_bit_cast(floatx4, gload16(res0 + (size_t)P * a.Cout + co));
                }
#pragma unroll
                for (int it = 0; it < ITS; ++it) {
                    const int row = it * ROWS + sub, P = wpx * (32 * MT) + m * 32 + row;
                    floatx4 v = __builtin_bit_cast(floatx4, tile[row * U + (chunk ^ (row & (U - 1)))]);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        v[e] = __builtin_amdgcn_fmed3f(__fmaf_rn(v[e], __fmul_rn(sc[e], xs[it]), bi[e]) + rv[it][e], lo, hi);
                    if (co < a.Cout && P < valid_px) {
                        __builtin_nontemporal_store(v, reinterpret_cast<floatx4 *>(out0 + (size_t)P * a.Cout + co));
                        vmax = fmaxf(fmaxf(vmax, fmaxf(fabsf(v[0]), fabsf(v[1]))), fmaxf(fabsf(v[2]), fabsf(v[3])));
                    }
                }
                // The image's absolute maximum for the layer that reads this output quantized: the host asks
                // for it only where the 32 pixels of a tile lie in one image.  Bit patterns of non-negative
                // floats order like the floats, and an integer maximum does not depend on the order.
                if (a.amax_out) {
                    vmax = wave_max_nonneg(vmax); // in lane 63
                    const int P0 = wpx * (32 * MT) + m * 32;
                    if (lane == 63 && P0 < valid_px) {
                        const int g = a.G > 1 ? (int)fd_div((uint32_t)P0, a.div_pximg) : 0;
                        atomicMax(a.amax_out + img0 + g, __float_as_uint(vmax));
                    }
                }
            }
        }
        if (region + 1 < r_end) __syncthreads(); // the tiles are read before the next region's activations land on them
    }
}

template <int KS, int STRIDE, int NT>
static hipError_t i8_launch(const I8ConvArgs &a, size_t lds_bytes, dim3 grid, hipStream_t st)
{
    static bool lds_set = false;
    if (!lds_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_i8_kernel<KS, STRIDE, NT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 159 * 1024);
        if (e != hipSuccess) return e;
        lds_set = true;
    }
    hipLaunchKernelGGL((conv_i8_kernel<KS, STRIDE, NT>), grid, dim3(256), lds_bytes, st, a);
    return hipGetLastError();
}

hipError_t launch_conv_i8(const I8ConvArgs &a, int ks, int stride, int nt, size_t lds_bytes, dim3 grid, hipStream_t st)
{
    if (a.N == 0) return hipSuccess;
#define AIQ_I8(KS_, ST_)                                                                          \
    if (ks == KS_ && stride == ST_) {                                                             \
        if (nt == 1) return i8_launch<KS_, ST_, 1>(a, lds_bytes, grid, st);                       \
        if (nt == 2) return i8_launch<KS_, ST_, 2>(a, lds_bytes, grid, st);                       \
    }
    AIQ_I8(3, 1)
    AIQ_I8(3, 2)
    AIQ_I8(1, 1)
    AIQ_I8(1, 2)
#undef AIQ_I8
    return hipErrorInvalidValue;
}

} // namespace aiq
