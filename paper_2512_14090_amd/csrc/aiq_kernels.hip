// gfx950 (CDNA4) kernels of the scheme-scoring path: weight quantize-dequantize,
// dense convolution on fp32 MFMA, depthwise convolution, classifier head, agreement.
//
// The operation each kernel performs is the plain definition of a convolutional
// forward pass with per-layer quantized weights (paper: Problem Formulation - a
// scheme assigns a bit-width to each layer; Introduction item (ii) - the model's
// accuracy under the scheme is measured by running it).  The scheme axis is a grid
// dimension: block z scores scheme z, picking each layer's weights from the bank
// slot of that scheme's bit-width.
#include "../../include/aiq.h"
#include "aiq_internal.h"

#include <algorithm>
#include <cstring>

namespace aiq {

typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kStageBatch = 8; // 16-byte global reads a thread keeps in flight while staging

// ------------------------------------------------------------------ helpers

// 16-byte read through an explicit global address space: global_load (vmcnt only) rather than
// flat_load, whose LDS-side counter would make waits on LDS reads wait for weights as well.
__device__ __forceinline__ floatx4 gload4(const float *p)
{
    return *(const __attribute__((address_space(1))) floatx4 *)(p);
}

__device__ inline int scheme_bits_index(const uint8_t *schemes, int s, int S, int L, int slot)
{
    if (slot < 0 || s >= S) return 0;
    return bits_index(schemes[(size_t)s * L + slot]);
}

__device__ inline int bits_of_index(int bi)
{
    switch (bi) {
    case 1: return 16;
    case 2: return 8;
    case 3: return 6;
    case 4: return 4;
    case 5: return 2;
    default: return 32;
    }
}

// One value through the quantizer: IEEE division, round half to even, clamp, one multiplication.
__device__ inline float quantize_value(float x, float s, int qmax)
{
    int q = (int)rintf(__fdiv_rn(x, s));
    q = min(max(q, -qmax), qmax);
    return __fmul_rn((float)q, s);
}

__device__ inline float apply_act(float v, int act)
{
    if (act >= 1) v = fmaxf(v, 0.0f);
    if (act == 2) v = fminf(v, 6.0f);
    return v;
}

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Logical block index for launches whose neighbouring blocks share data: hardware block b runs
// on XCD b % 8; XCD k is given the k-th contiguous stretch of n / 8 (one more for the first
// n % 8) logical blocks.  A permutation of [0, n), whatever the dispatch order really is.
__device__ inline uint32_t xcd_contiguous_block(uint32_t b, uint32_t n)
{
    const uint32_t per = n >> 3, rem = n & 7u, xcd = b & 7u, idx = b >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

// ------------------------------------------------------------------ quantizer
//
// One wavefront per output channel.  Pass 1: absmax of the row by a cross-lane
// butterfly.  Pass 2: w/s (IEEE binary32 division), round-half-even, clamp, code*s,
// written straight into the layout the consuming kernel wants.

__device__ inline size_t quant_out_index(const QuantJob &j, int c, int i)
{
    if (j.layout == kLayoutPlain) return (size_t)c * j.k + i;
    const int t = i % j.taps;
    const int ci = i / j.taps;
    if (j.layout == kLayoutTapMajor) return (size_t)t * j.cout + c; // depthwise: k == taps, ci == 0
    if (j.layout == kLayoutStem) return (((size_t)(c >> 4) * j.taps + t) * 64) + ci * 16 + (c & 15);
    const int ct = c >> 4, co = c & 15;
    const int cb = ci >> 4, kq = (ci & 15) >> 2, jj = ci & 3;
    if (j.layout == kLayoutMfmaKx) { // taps == 9: t = ky * 3 + kx
        const int ky = t / 3, kx = t - ky * 3;
        return (((((size_t)ct * 3 + kx) * j.cblocks + cb) * 3 + ky) * 64 + (kq * 16 + co)) * 4 + jj;
    }
    return ((((size_t)ct * j.taps + t) * j.cblocks + cb) * 64 + (kq * 16 + co)) * 4 + jj;
}

__device__ inline void quantize_channel(const QuantJob &j, int c, int lane)
{
    const float *row = j.w + (size_t)c * j.k;
    if (j.bits == 32) {
        for (int i = lane; i < j.k; i += 64) j.out[quant_out_index(j, c, i)] = row[i];
        if (lane == 0 && j.scales) j.scales[c] = 1.0f;
        return;
    }
    float amax = 0.0f;
    if (j.tensor_amax) {
        amax = __uint_as_float(*j.tensor_amax);
    } else {
        for (int i = lane; i < j.k; i += 64) amax = fmaxf(amax, fabsf(row[i]));
        amax = wave_max(amax);
    }
    const int qmax = (1 << (j.bits - 1)) - 1;
    const float s = amax > 0.0f ? __fdiv_rn(amax, (float)qmax) : 1.0f;
    if (lane == 0 && j.scales) j.scales[c] = s;
    for (int i = lane; i < j.k; i += 64) {
        const float t = __fdiv_rn(row[i], s);
        int q = (int)rintf(t);
        q = min(max(q, -qmax), qmax);
        j.out[quant_out_index(j, c, i)] = __fmul_rn((float)q, s);
        if (j.codes) j.codes[(size_t)c * j.k + i] = q;
    }
}

__global__ __launch_bounds__(256) void quantize_single_kernel(QuantJob j)
{
    const int c = blockIdx.x * kQuantChannelsPerBlock + (threadIdx.x >> 6);
    if (c < j.cout) quantize_channel(j, c, threadIdx.x & 63);
}

// Batched form: a static job table for every (layer, bit-width) of a model; the
// mask says which jobs this call needs, all others exit at once.
__global__ __launch_bounds__(256) void quantize_batch_kernel(const QuantJob *jobs, const int32_t *block_job,
                                                             QuantMask mask)
{
    const int ji = block_job[blockIdx.x];
    if (!((mask.word[ji >> 6] >> (ji & 63)) & 1ull)) return;
    const QuantJob j = jobs[ji];
    const int c = (blockIdx.x - j.first_block) * kQuantChannelsPerBlock + (threadIdx.x >> 6);
    if (c < j.cout) quantize_channel(j, c, threadIdx.x & 63);
}

// Plain [cout][k] rows with k % 4 == 0 and 16-byte aligned pointers: the WPR wavefronts that share
// a row keep it in registers (NV 16-byte elements per lane), so every weight is read from memory
// once and written once, 16 bytes per lane per access, all reads of a workgroup in flight before
// its first write.  Long rows take a whole workgroup (WPR = 4, absmax combined through LDS): a
// workgroup then lives for one short burst of reads and one of writes and makes room for the next,
// which the memory system rewards (5.2 -> 5.9 TB/s on 8192 x 4608 against one wavefront per row;
// a copy kernel shows the same preference for short-lived workgroups over looping ones).
// Same arithmetic, step for step, as quantize_channel.
template <int NV, int WPR>
__global__ __launch_bounds__(256) void quantize_rows_kernel(QuantJob j)
{
    __shared__ float wave_amax[4];
    constexpr int RPB = kQuantChannelsPerBlock / WPR; // rows per workgroup
    const int wave = threadIdx.x >> 6;
    const int c = blockIdx.x * RPB + wave / WPR;
    const bool live = c < j.cout; // (with WPR > 1 every wavefront reaches the barrier below)
    if (WPR == 1 && !live) return;
    const int lane = (wave % WPR) * 64 + (threadIdx.x & 63); // position among the row's 64 * WPR lanes
    const int k4 = j.k >> 2;
    const floatx4 *row = reinterpret_cast<const floatx4 *>(j.w + (size_t)(live ? c : 0) * j.k);
    floatx4 *out = reinterpret_cast<floatx4 *>(j.out + (size_t)(live ? c : 0) * j.k);
    floatx4 v[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int i = u * (64 * WPR) + lane;
        v[u] = (live && i < k4) ? __builtin_nontemporal_load(row + i) : floatx4{0.f, 0.f, 0.f, 0.f};
    }
    if (j.bits == 32) {
        if (!live) return; // no barrier on this path
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int i = u * (64 * WPR) + lane;
            if (i < k4) __builtin_nontemporal_store(v[u], out + i);
        }
        if (lane == 0 && j.scales) j.scales[c] = 1.0f;
        return;
    }
    float amax = 0.0f;
    if (j.tensor_amax) {
        amax = __uint_as_float(*j.tensor_amax);
    } else {
#pragma unroll
        for (int u = 0; u < NV; ++u)
            amax = fmaxf(fmaxf(amax, fmaxf(fabsf(v[u].x), fabsf(v[u].y))), fmaxf(fabsf(v[u].z), fabsf(v[u].w)));
        amax = wave_max(amax);
        if (WPR > 1) { // the maximum is exact whatever the order: combine the row's wavefronts through LDS
            if ((threadIdx.x & 63) == 0) wave_amax[wave] = amax;
            __syncthreads();
            const int w0 = (wave / WPR) * WPR;
#pragma unroll
            for (int q = 0; q < WPR; ++q) amax = fmaxf(amax, wave_amax[w0 + q]);
        }
    }
    if (!live) return;
    const int qmax = (1 << (j.bits - 1)) - 1;
    const float s = amax > 0.0f ? __fdiv_rn(amax, (float)qmax) : 1.0f;
    if (lane == 0 && j.scales) j.scales[c] = s;
    typedef int intx4 __attribute__((ext_vector_type(4)));
    intx4 *codes = j.codes ? reinterpret_cast<intx4 *>(j.codes + (size_t)c * j.k) : nullptr;
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int i = u * (64 * WPR) + lane;
        if (i >= k4) continue;
        intx4 q;
        floatx4 d;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int qe = (int)rintf(__fdiv_rn(v[u][e], s));
            qe = min(max(qe, -qmax), qmax);
            q[e] = qe;
            d[e] = __fmul_rn((float)qe, s);
        }
        __builtin_nontemporal_store(d, out + i);
        if (codes) codes[i] = q;
    }
}

template <int NV, int WPR>
static hipError_t launch_quantize_rows(const QuantJob &job, hipStream_t st)
{
    constexpr int RPB = kQuantChannelsPerBlock / WPR;
    hipLaunchKernelGGL((quantize_rows_kernel<NV, WPR>), dim3((job.cout + RPB - 1) / RPB), dim3(256), 0, st, job);
    return hipGetLastError();
}

hipError_t launch_quantize_single(const QuantJob &job, hipStream_t st)
{
    if (job.cout == 0) return hipSuccess; // k == 0 still writes s = 1 for every (empty) row
    const int blocks = (job.cout + kQuantChannelsPerBlock - 1) / kQuantChannelsPerBlock;
    const bool aligned = ((reinterpret_cast<uintptr_t>(job.w) | reinterpret_cast<uintptr_t>(job.out) |
                           reinterpret_cast<uintptr_t>(job.codes)) & 15) == 0;
    if (job.layout == kLayoutPlain && job.k > 0 && (job.k & 3) == 0 && aligned && job.k <= 4 * 256 * 20) {
        const int k4 = job.k / 4;
        // rows of up to 64 / 128 16-byte elements: one / two wavefronts per row; longer rows: the workgroup
        if (k4 <= 64) return launch_quantize_rows<1, 1>(job, st);
        if (k4 <= 128) return launch_quantize_rows<1, 2>(job, st);
        const int nv = (k4 + 255) / 256;
        if (nv <= 1) return launch_quantize_rows<1, 4>(job, st);
        if (nv <= 2) return launch_quantize_rows<2, 4>(job, st);
        if (nv <= 3) return launch_quantize_rows<3, 4>(job, st);
        if (nv <= 5) return launch_quantize_rows<5, 4>(job, st);
        if (nv <= 10) return launch_quantize_rows<10, 4>(job, st);
        return launch_quantize_rows<20, 4>(job, st);
    }
    hipLaunchKernelGGL(quantize_single_kernel, dim3(blocks), dim3(256), 0, st, job);
    return hipGetLastError();
}

// Largest magnitude of a whole matrix (per-tensor scales): wavefront butterfly, then one integer
// atomic per wavefront - the bit patterns of non-negative floats order like unsigned integers,
// so the result does not depend on the order of arrival.
__global__ __launch_bounds__(256) void tensor_absmax_kernel(const float *__restrict__ w, size_t n, uint32_t *out)
{
    float amax = 0.0f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        amax = fmaxf(amax, fabsf(w[i]));
    amax = wave_max(amax);
    if ((threadIdx.x & 63) == 0) atomicMax(out, __float_as_uint(amax));
}

hipError_t launch_tensor_absmax(const float *w, size_t n, uint32_t *out, hipStream_t st)
{
    hipError_t e = launch_fill_i32(reinterpret_cast<int32_t *>(out), 0, 1, st);
    if (e != hipSuccess || n == 0) return e;
    const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 2048);
    hipLaunchKernelGGL(tensor_absmax_kernel, dim3(blocks), dim3(256), 0, st, w, n, out);
    return hipGetLastError();
}

hipError_t launch_quantize_batch(const QuantJob *jobs_dev, const int32_t *block_job_dev, int n_blocks,
                                 const QuantMask &mask, hipStream_t st)
{
    if (n_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(quantize_batch_kernel, dim3(n_blocks), dim3(256), 0, st, jobs_dev, block_job_dev, mask);
    return hipGetLastError();
}

// ------------------------------------------------------------------ dense convolution
//
// Implicit GEMM on v_mfma_f32_16x16x4_f32 with the weights as the A operand
// (rows = 16 output channels) and 16 output pixels as the B operand, so that a
// lane's four accumulator values are four consecutive output channels of one pixel:
// one 16-byte NHWC store.  The reduction index is (tap, input channel); within a
// block of 16 input channels lane (p, kq) supplies channels 4*kq+j to MFMA j, so a
// lane's activations for four MFMAs are one 16-byte LDS read and its weights one
// 16-byte global read from the pre-packed bank.
//
// Workgroup = 4 wavefronts.  It stages the input rows its region needs (with the
// zero border) in LDS, CKC channels at a time; every wavefront owns a tile of 64
// pixels x 16*NT output channels and keeps its accumulators across channel passes.

// Stages channels [c0, c0 + 4*c4n) of the region's input rows into LDS, zero outside the
// image.  One wavefront takes NR rows at a time (rows wave, wave+4, ...): a row's image,
// position and validity are uniform, so per element only the column and the channel chunk
// are lane arithmetic.  All B*NR 16-byte loads of a round are issued before the first LDS
// store, so a lane has that many reads in flight.
template <int STRIDE, int PAD, int B, int NR>
__device__ __forceinline__ void conv_stage_rows(const ConvArgs &a, const float *in_s, floatx4 *lds4, int ps4, int c0,
                                                int c4n, int c4shift, int img0, int oy0, int wave_u, int lane)
{
    const int stage_rows = a.G * a.RIN;
    const int per_row = a.LW << c4shift; // 16-byte chunks of one staged row
    const bool vec_ok = (a.Cin & 3) == 0;
    for (int row0 = wave_u; row0 < stage_rows; row0 += 4 * NR) {
        for (int base = lane; base < per_row; base += 64 * B) {
            floatx4 v[NR][B];
#pragma unroll
            for (int rr = 0; rr < NR; ++rr) {
                const int row = row0 + 4 * rr;
                const int g = (int)fd_div((uint32_t)row, a.div_rin);
                const int r = row - g * a.RIN;
                const int iy = oy0 * STRIDE - PAD + r;
                const int img = img0 + g;
                const bool row_ok = row < stage_rows && iy >= 0 && iy < a.Hin && img < a.N;
                // dereferenced only when row_ok
                const float *src_row =
                    in_s + (((size_t)(row_ok ? img : 0) * a.Hin + (row_ok ? iy : 0)) * a.Win) * a.Cin + c0;
#pragma unroll
                for (int u = 0; u < B; ++u) {
                    const int e = base + u * 64;
                    const int c = (e & (c4n - 1)) * 4;
                    const int ix = (e >> c4shift) - PAD;
                    v[rr][u] = floatx4{0.f, 0.f, 0.f, 0.f};
                    if (row_ok && e < per_row && ix >= 0 && ix < a.Win && c0 + c < a.Cin) {
                        const float *src = src_row + ix * a.Cin + c;
                        if (vec_ok) {
                            v[rr][u] = *reinterpret_cast<const floatx4 *>(src);
                        } else {
                            v[rr][u].x = src[0];
                            if (c0 + c + 1 < a.Cin) v[rr][u].y = src[1];
                            if (c0 + c + 2 < a.Cin) v[rr][u].z = src[2];
                            if (c0 + c + 3 < a.Cin) v[rr][u].w = src[3];
                        }
                    }
                }
            }
#pragma unroll
            for (int rr = 0; rr < NR; ++rr) {
                const int row = row0 + 4 * rr;
                if (row >= stage_rows) continue;
                floatx4 *dst_row = lds4 + row * a.LW * ps4;
#pragma unroll
                for (int u = 0; u < B; ++u) {
                    const int e = base + u * 64;
                    if (e < per_row) dst_row[(e >> c4shift) * ps4 + (e & (c4n - 1))] = v[rr][u];
                }
            }
        }
    }
}

template <int KS, int STRIDE, int NT>
__global__ __launch_bounds__(256, 2) void conv_mfma_kernel(ConvArgs a)
{
    extern __shared__ float lds[];
    constexpr int T = KS * KS;
    constexpr int PAD = KS == 3 ? 1 : 0;
    const int tid = threadIdx.x, lane = tid & 63;
    // the wavefront index is uniform; saying so keeps everything derived from it (output-channel
    // tile, weight addresses) in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s = blockIdx.z;

    // neighbouring regions share halo rows: keep them on one XCD
    const int bx = (int)xcd_contiguous_block(blockIdx.x, gridDim.x);
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
    const int p = lane & 15, kq = lane >> 4;

    floatx4 *lds4 = reinterpret_cast<floatx4 *>(lds); // LDS is addressed in 16-byte units (PS % 4 == 0)
    const int ps4 = a.PS >> 2;
    // per pixel tile: LDS base offset (16-byte units) of the lane's pixel, and its output position
    int lds_base[4];
    int out_img[4], out_y[4], out_x[4];
    const int rw = a.R * a.Wout;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const uint32_t P = (uint32_t)(wpx * 64 + m * 16 + p);
        const uint32_t g = fd_div(P, a.div_rw);
        const uint32_t rem = P - g * rw;
        const uint32_t oy = fd_div(rem, a.div_wout);
        const uint32_t ox = rem - oy * a.Wout;
        const bool in_region = g < (uint32_t)a.G; // lanes past the region's last pixel compute nothing useful
        lds_base[m] = in_region ? ((g * a.RIN + oy * STRIDE) * a.LW + ox * STRIDE) * ps4 + kq : kq;
        out_img[m] = in_region ? img0 + (int)g : a.N;
        out_y[m] = oy0 + oy;
        out_x[m] = ox;
    }

    const float *wq = a.bank[scheme_bits_index(a.schemes, s, a.S, a.L, a.slot)];
    const float *in_s = a.in + (size_t)s * a.in_scheme_stride;

    floatx4 acc[4][NT];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[m][n] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int c4n = a.CKC >> 2;            // 16-byte chunks per staged pixel
    const int c4shift = __ffs(c4n) - 1;    // CKC is 16, 32 or 64
    const bool active = ct0 < a.cout_tiles; // wavefronts past the last output-channel tile only help staging

    const int wave_u = wave;
    const int per_row = a.LW << c4shift; // 16-byte chunks of one staged row

    for (int c0 = 0; c0 < a.CB * 16; c0 += a.CKC) {
        if (c0) __syncthreads();
        // ---- stage channels [c0, c0+CKC) of the region's input rows: about nine 16-byte reads in
        // flight per lane whatever the row length
        if (per_row <= 64)
            conv_stage_rows<STRIDE, PAD, 1, 8>(a, in_s, lds4, ps4, c0, c4n, c4shift, img0, oy0, wave_u, lane);
        else if (per_row <= 128)
            conv_stage_rows<STRIDE, PAD, 2, 4>(a, in_s, lds4, ps4, c0, c4n, c4shift, img0, oy0, wave_u, lane);
        else if (per_row <= 192)
            conv_stage_rows<STRIDE, PAD, 3, 3>(a, in_s, lds4, ps4, c0, c4n, c4shift, img0, oy0, wave_u, lane);
        else if (per_row <= 320)
            conv_stage_rows<STRIDE, PAD, 5, 2>(a, in_s, lds4, ps4, c0, c4n, c4shift, img0, oy0, wave_u, lane);
        else
            conv_stage_rows<STRIDE, PAD, 9, 1>(a, in_s, lds4, ps4, c0, c4n, c4shift, img0, oy0, wave_u, lane);
        __syncthreads();

        if (active) {
            // The reduction over (tap, channel block) is one flat sequence of steps; step k+1's
            // weights (16-byte global reads, L2-resident) and activations (16-byte LDS reads) are
            // requested before step k's MFMAs, alternating between two register sets.
            const int ncb = min(a.CKC, a.CB * 16 - c0) >> 4;
            const int cb0 = c0 >> 4;
            const int steps = T * ncb;
            // Addresses of the next step to load, as byte offsets that advance by one of a few uniform
            // increments (next block of the tap, next tap of the window row, next window row): a
            // counter and two selects per step instead of divisions and 64-bit products.
            const uint32_t x_tap = (uint32_t)a.PS * 4u - (uint32_t)(ncb - 1) * 64u;
            const uint32_t x_row = x_tap + (uint32_t)(a.LW - KS) * (uint32_t)a.PS * 4u;
            const uint32_t w_tap = (uint32_t)(a.CB - ncb + 1) * 1024u;
            const char *ldsb = reinterpret_cast<const char *>(lds);
            const char *wbase[NT]; // uniform: weights of tile n, tap 0, first block of the pass
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                const int ct = min(ct0 + n, a.cout_tiles - 1);
                wbase[n] = reinterpret_cast<const char *>(wq + ((size_t)ct * T * a.CB + cb0) * 256);
            }
            uint32_t wv = (uint32_t)lane * 16u, xv[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) xv[m] = (uint32_t)lds_base[m] * 16u;
            int lc = 0, lkx = 0; // channel block and tap column of the next step to load
            auto load_step = [&](floatx4 (&wa)[NT], floatx4 (&xb)[4]) {
#pragma unroll
                for (int n = 0; n < NT; ++n) wa[n] = *reinterpret_cast<const floatx4 *>(wbase[n] + wv);
#pragma unroll
                for (int m = 0; m < 4; ++m) xb[m] = *reinterpret_cast<const floatx4 *>(ldsb + xv[m]);
                uint32_t dx = 64u, dw = 1024u;
                if (++lc == ncb) { // uniform
                    lc = 0;
                    dw = w_tap;
                    dx = x_tap;
                    if (++lkx == KS) {
                        lkx = 0;
                        dx = x_row;
                    }
                }
                wv += dw;
#pragma unroll
                for (int m = 0; m < 4; ++m) xv[m] += dx;
            };
            auto mma_step = [&](const floatx4 (&wa)[NT], const floatx4 (&xb)[4]) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int m = 0; m < 4; ++m)
#pragma unroll
                        for (int n = 0; n < NT; ++n)
                            acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[n][j], xb[m][j], acc[m][n], 0, 0, 0);
            };
            floatx4 wa0[NT], xb0[4], wa1[NT], xb1[4];
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
    // ---- epilogue: bias, residual, activation, 16-byte NHWC stores
    const float lo = a.act >= 1 ? 0.0f : -__builtin_inff(), hi = a.act == 2 ? 6.0f : __builtin_inff();
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        if (out_img[m] >= a.N || out_y[m] >= a.Hout) continue;
        const size_t pix = (((size_t)out_img[m] * a.Hout + out_y[m]) * a.Wout + out_x[m]) * a.Cout;
        float *out_p = a.out + (size_t)s * a.out_scheme_stride + pix;
        const float *res_p = a.res ? a.res + (size_t)s * a.res_scheme_stride + pix : nullptr;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            const int co = (ct0 + n) * 16 + kq * 4;
            if (co >= a.Cout) continue;
            floatx4 v = acc[m][n] + *reinterpret_cast<const floatx4 *>(a.bias + co);
            if (res_p) v += *reinterpret_cast<const floatx4 *>(res_p + co);
            v.x = __builtin_amdgcn_fmed3f(v.x, lo, hi);
            v.y = __builtin_amdgcn_fmed3f(v.y, lo, hi);
            v.z = __builtin_amdgcn_fmed3f(v.z, lo, hi);
            v.w = __builtin_amdgcn_fmed3f(v.w, lo, hi);
            *reinterpret_cast<floatx4 *>(out_p + co) = v;
        }
    }
}

// ------------------------------------------------------------------ network stems
//
// 3x3 stride-1 convolution of an input with at most four channels.  In the general kernel a
// block of 16 input channels is the unit of the reduction, so three channels would waste
// 13/16 of the MFMAs; here the MFMA's k index is the input channel itself (lane (p, kq)
// supplies channel kq of its pixel, one 4-byte LDS read, and the weight of (output channel,
// tap, channel kq), one register), one MFMA per tap.  Same output tiling and epilogue as
// conv_mfma_kernel; the weights of the wavefront's NT tiles stay in registers.

template <int NT>
__global__ __launch_bounds__(256, 2) void conv_stem_kernel(ConvArgs a)
{
    extern __shared__ float lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // uniform: keeps the tile indices scalar
    const int s = blockIdx.z;
    const int bx = (int)xcd_contiguous_block(blockIdx.x, gridDim.x); // halo rows meet in one XCD's L2
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
    const int ct0 = (blockIdx.y * (4 / a.wave_px_split) + wco) * NT;
    const int p = lane & 15, kq = lane >> 4;
    const bool active = ct0 < a.cout_tiles;

    // weights first: their latency overlaps the staging
    const float *wq = a.bank[scheme_bits_index(a.schemes, s, a.S, a.L, a.slot)];
    float w[NT][9];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int ct = min(ct0 + n, a.cout_tiles - 1);
#pragma unroll
        for (int t = 0; t < 9; ++t) w[n][t] = wq[((size_t)ct * 9 + t) * 64 + lane];
    }

    // stage the region's input rows as one 16-byte element per pixel (channels past Cin and
    // pixels outside the image are zero)
    const float *in_s = a.in + (size_t)s * a.in_scheme_stride;
    floatx4 *lds4 = reinterpret_cast<floatx4 *>(lds);
    const int n_pix = a.G * a.RIN * a.LW;
    for (int pix = tid; pix < n_pix; pix += 256) {
        const uint32_t row = fd_div((uint32_t)pix, a.div_lw);
        const int x = pix - row * a.LW;
        const uint32_t g = fd_div(row, a.div_rin);
        const int r = row - g * a.RIN;
        const int iy = oy0 - 1 + r, ix = x - 1, img = img0 + g;
        floatx4 v = floatx4{0.f, 0.f, 0.f, 0.f};
        if (iy >= 0 && iy < a.Hin && ix >= 0 && ix < a.Win && img < a.N) {
            const float *src = in_s + (((size_t)img * a.Hin + iy) * a.Win + ix) * a.Cin;
            v.x = src[0];
            if (a.Cin > 1) v.y = src[1];
            if (a.Cin > 2) v.z = src[2];
            if (a.Cin > 3) v.w = src[3];
        }
        lds4[pix] = v;
    }

    int lds_base[4], out_img[4], out_y[4], out_x[4];
    const int rw = a.R * a.Wout;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const uint32_t P = (uint32_t)(wpx * 64 + m * 16 + p);
        const uint32_t g = fd_div(P, a.div_rw);
        const uint32_t rem = P - g * rw;
        const uint32_t oy = fd_div(rem, a.div_wout);
        const uint32_t ox = rem - oy * a.Wout;
        const bool in_region = g < (uint32_t)a.G;
        lds_base[m] = in_region ? ((g * a.RIN + oy) * a.LW + ox) * 4 + kq : kq;
        out_img[m] = in_region ? img0 + (int)g : a.N;
        out_y[m] = oy0 + oy;
        out_x[m] = ox;
    }
    __syncthreads();
    if (!active) return;

    floatx4 acc[4][NT];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[m][n] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int tapoff = ((t / 3) * a.LW + (t % 3)) * 4;
        float xb[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) xb[m] = lds[lds_base[m] + tapoff];
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int n = 0; n < NT; ++n)
                acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[n][t], xb[m], acc[m][n], 0, 0, 0);
    }

    const float lo = a.act >= 1 ? 0.0f : -__builtin_inff(), hi = a.act == 2 ? 6.0f : __builtin_inff();
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        if (out_img[m] >= a.N || out_y[m] >= a.Hout) continue;
        const size_t pix = (((size_t)out_img[m] * a.Hout + out_y[m]) * a.Wout + out_x[m]) * a.Cout;
        float *out_p = a.out + (size_t)s * a.out_scheme_stride + pix;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            const int co = (ct0 + n) * 16 + kq * 4;
            if (co >= a.Cout) continue;
            floatx4 v = acc[m][n] + *reinterpret_cast<const floatx4 *>(a.bias + co);
            v.x = __builtin_amdgcn_fmed3f(v.x, lo, hi);
            v.y = __builtin_amdgcn_fmed3f(v.y, lo, hi);
            v.z = __builtin_amdgcn_fmed3f(v.z, lo, hi);
            v.w = __builtin_amdgcn_fmed3f(v.w, lo, hi);
            __builtin_nontemporal_store(v, reinterpret_cast<floatx4 *>(out_p + co));
        }
    }
}

hipError_t launch_conv_stem(const ConvArgs &a, int nt, dim3 grid, hipStream_t st)
{
    if (a.Cin > 4 || a.res) return hipErrorInvalidValue;
    const size_t lds_bytes = sizeof(float) * 4 * (size_t)a.G * a.RIN * a.LW;
    if (lds_bytes > 64 * 1024) return hipErrorInvalidValue;
    switch (nt) {
    case 1: hipLaunchKernelGGL((conv_stem_kernel<1>), grid, dim3(256), lds_bytes, st, a); break;
    case 2: hipLaunchKernelGGL((conv_stem_kernel<2>), grid, dim3(256), lds_bytes, st, a); break;
    case 3: hipLaunchKernelGGL((conv_stem_kernel<3>), grid, dim3(256), lds_bytes, st, a); break;
    case 4: hipLaunchKernelGGL((conv_stem_kernel<4>), grid, dim3(256), lds_bytes, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int KS, int STRIDE, int NT>
static hipError_t launch_conv_t(const ConvArgs &a, size_t lds_bytes, dim3 grid, hipStream_t st)
{
    hipLaunchKernelGGL((conv_mfma_kernel<KS, STRIDE, NT>), grid, dim3(256), lds_bytes, st, a);
    return hipGetLastError();
}

template <int KS, int STRIDE>
static hipError_t launch_conv_nt(const ConvArgs &a, int nt, size_t lds_bytes, dim3 grid, hipStream_t st)
{
    switch (nt) {
    case 1: return launch_conv_t<KS, STRIDE, 1>(a, lds_bytes, grid, st);
    case 2: return launch_conv_t<KS, STRIDE, 2>(a, lds_bytes, grid, st);
    case 3: return launch_conv_t<KS, STRIDE, 3>(a, lds_bytes, grid, st);
    case 4: return launch_conv_t<KS, STRIDE, 4>(a, lds_bytes, grid, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_conv(const ConvArgs &a, int ks, int stride, int nt, size_t lds_bytes, dim3 grid, hipStream_t st)
{
    if (ks == 3 && stride == 1) return launch_conv_nt<3, 1>(a, nt, lds_bytes, grid, st);
    if (ks == 3 && stride == 2) return launch_conv_nt<3, 2>(a, nt, lds_bytes, grid, st);
    if (ks == 1 && stride == 1) return launch_conv_nt<1, 1>(a, nt, lds_bytes, grid, st);
    if (ks == 1 && stride == 2) return launch_conv_nt<1, 2>(a, nt, lds_bytes, grid, st);
    return hipErrorInvalidValue;
}

template <int KS, int STRIDE, int NT>
static hipError_t set_lds_t()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_kernel<KS, STRIDE, NT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

// Dynamic LDS above 64 KB has to be allowed per kernel.
hipError_t conv_set_lds_limits()
{
    hipError_t e = hipSuccess;
#define AIQ_SET(KS, ST)                                             \
    if (e == hipSuccess) e = set_lds_t<KS, ST, 1>();                \
    if (e == hipSuccess) e = set_lds_t<KS, ST, 2>();                \
    if (e == hipSuccess) e = set_lds_t<KS, ST, 3>();                \
    if (e == hipSuccess) e = set_lds_t<KS, ST, 4>();
    AIQ_SET(3, 1)
    AIQ_SET(3, 2)
    AIQ_SET(1, 1)
    AIQ_SET(1, 2)
#undef AIQ_SET
    return e;
}

// ------------------------------------------------------------------ 1x1 stride-1 convolution
//
// Same MFMA tiling as conv_mfma_kernel, but a 1x1 stride-1 convolution has no spatial
// structure: the pixels of all images form one flat axis, so staging is a strided copy and
// no per-pixel (image, row, column) arithmetic or border handling is needed.  That matters
// for the narrow layers (16..32 input channels), where a wavefront tile holds only a few
// dozen MFMAs and index arithmetic would otherwise outweigh them.

template <int NT>
__global__ __launch_bounds__(256, 2) void pointwise_mfma_kernel(PointwiseArgs a)
{
    extern __shared__ float lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // uniform: keeps the tile indices scalar
    const int s = blockIdx.z;
    const int tile_px = 64 * a.wave_px_split;
    // One flat block axis, output-channel block fastest: the blocks that read the same pixel tile
    // follow each other, and the XCD-contiguous order puts them behind one L2 (with the
    // output-channel blocks on a second grid axis every one of them fetched the tile from HBM).
    const uint32_t lb = xcd_contiguous_block(blockIdx.x, gridDim.x);
    const int bx = (int)(lb / (uint32_t)a.grid_y), by = (int)(lb - (uint32_t)bx * a.grid_y);
    const int P0 = bx * tile_px;
    const int wpx = wave % a.wave_px_split;
    const int wco = wave / a.wave_px_split;
    const int ct0 = (by * (4 / a.wave_px_split) + wco) * NT;
    const int p = lane & 15, kq = lane >> 4;
    const bool active = ct0 < a.cout_tiles;

    const float *wq = a.bank[scheme_bits_index(a.schemes, s, a.S, a.L, a.slot)];
    const float *in_s = a.in + (size_t)s * a.in_scheme_stride + (size_t)P0 * a.Cin;
    const int px_here = min(tile_px, a.P - P0);

    floatx4 acc[4][NT];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[m][n] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int c4n = a.CKC >> 2;
    const int c4shift = __ffs(c4n) - 1;
    const int n_chunks = tile_px << c4shift;
    floatx4 *lds4 = reinterpret_cast<floatx4 *>(lds); // LDS is addressed in 16-byte units (PS % 4 == 0)
    const int ps4 = a.PS >> 2;
    const int lds_lane = (wpx * 64 + p) * ps4 + kq;

    for (int c0 = 0; c0 < a.CB * 16; c0 += a.CKC) {
        if (c0) __syncthreads();
        // batches of kStageBatch 16-byte loads are issued before their LDS stores, so that a
        // thread has several global reads in flight instead of one
        for (int base = tid; base < n_chunks; base += 256 * kStageBatch) {
            floatx4 v[kStageBatch];
#pragma unroll
            for (int u = 0; u < kStageBatch; ++u) {
                const int idx = base + u * 256;
                const int c4 = idx & (c4n - 1);
                const int pix = idx >> c4shift;
                const int c = c0 + c4 * 4;
                v[u] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (idx < n_chunks && pix < px_here && c < a.Cin)
                    v[u] = *reinterpret_cast<const floatx4 *>(in_s + (size_t)pix * a.Cin + c);
            }
#pragma unroll
            for (int u = 0; u < kStageBatch; ++u) {
                const int idx = base + u * 256;
                if (idx < n_chunks) lds4[(idx >> c4shift) * ps4 + (idx & (c4n - 1))] = v[u];
            }
        }
        __syncthreads();
        if (active) {
            const int ncb = min(a.CKC, a.CB * 16 - c0) >> 4;
            const int cb0 = c0 >> 4;
#pragma unroll 1
            for (int cbl = 0; cbl < ncb; ++cbl) {
                floatx4 wa[NT], xb[4];
#pragma unroll
                for (int n = 0; n < NT; ++n) {
                    const int ct = min(ct0 + n, a.cout_tiles - 1);
                    const float *wrow = wq + ((size_t)ct * a.CB + cb0 + cbl) * 256; // uniform
                    wa[n] = *reinterpret_cast<const floatx4 *>(wrow + lane * 4);
                }
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    xb[m] = lds4[lds_lane + m * 16 * ps4 + cbl * 4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int m = 0; m < 4; ++m)
#pragma unroll
                        for (int n = 0; n < NT; ++n)
                            acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[n][j], xb[m][j], acc[m][n], 0, 0, 0);
            }
        }
    }
    if (!active) return;

    const float lo = a.act >= 1 ? 0.0f : -__builtin_inff(), hi = a.act == 2 ? 6.0f : __builtin_inff();
    if (a.pool) {
        // Global average pooling fused into the layer: the 64 pixels of this wavefront are one
        // whole image, so the mean over them is the sum of the lane's four tiles followed by a
        // butterfly over the 16 lanes that share kq - a fixed order, hence run-to-run identical.
        // Only the [image][Cout] means reach memory.
        const int img = (P0 >> 6) + wpx;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            const int co = (ct0 + n) * 16 + kq * 4;
            const floatx4 b = co < a.Cout ? *reinterpret_cast<const floatx4 *>(a.bias + co) : floatx4{0.f, 0.f, 0.f, 0.f};
            floatx4 sum = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                floatx4 v = acc[m][n] + b;
                v.x = fminf(fmaxf(v.x, lo), hi);
                v.y = fminf(fmaxf(v.y, lo), hi);
                v.z = fminf(fmaxf(v.z, lo), hi);
                v.w = fminf(fmaxf(v.w, lo), hi);
                sum += v;
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) {
                sum.x += __shfl_xor(sum.x, off);
                sum.y += __shfl_xor(sum.y, off);
                sum.z += __shfl_xor(sum.z, off);
                sum.w += __shfl_xor(sum.w, off);
            }
            if (p == 0 && co < a.Cout && img * 64 < a.P)
                *reinterpret_cast<floatx4 *>(a.out + (size_t)s * a.out_scheme_stride + (size_t)img * a.Cout + co) =
                    sum * (1.0f / 64.0f);
        }
        return;
    }
    const size_t obase = (size_t)s * a.out_scheme_stride + (size_t)P0 * a.Cout;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int co = (ct0 + n) * 16 + kq * 4;
        if (co >= a.Cout) continue;
        const floatx4 b = *reinterpret_cast<const floatx4 *>(a.bias + co);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int pl = wpx * 64 + m * 16 + p;
            if (pl >= px_here) continue;
            const size_t o = obase + (size_t)pl * a.Cout + co;
            floatx4 v = acc[m][n] + b;
            if (a.res)
                v += *reinterpret_cast<const floatx4 *>(a.res + (o - (size_t)s * a.out_scheme_stride) +
                                                        (size_t)s * a.res_scheme_stride);
            v.x = fminf(fmaxf(v.x, lo), hi);
            v.y = fminf(fmaxf(v.y, lo), hi);
            v.z = fminf(fmaxf(v.z, lo), hi);
            v.w = fminf(fmaxf(v.w, lo), hi);
            *reinterpret_cast<floatx4 *>(a.out + o) = v;
        }
    }
}

template <int NT>
static hipError_t launch_pointwise_t(const PointwiseArgs &a, size_t lds_bytes, dim3 grid, hipStream_t st)
{
    static bool lds_set = false;
    if (!lds_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pointwise_mfma_kernel<NT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        lds_set = true;
    }
    if (a.grid_y < 1 || (int)grid.y != a.grid_y) return hipErrorInvalidValue;
    hipLaunchKernelGGL((pointwise_mfma_kernel<NT>), dim3(grid.x * grid.y, 1, grid.z), dim3(256), lds_bytes, st, a);
    return hipGetLastError();
}

hipError_t launch_pointwise(const PointwiseArgs &a, int nt, size_t lds_bytes, dim3 grid, hipStream_t st)
{
    switch (nt) {
    case 1: return launch_pointwise_t<1>(a, lds_bytes, grid, st);
    case 2: return launch_pointwise_t<2>(a, lds_bytes, grid, st);
    case 3: return launch_pointwise_t<3>(a, lds_bytes, grid, st);
    case 4: return launch_pointwise_t<4>(a, lds_bytes, grid, st);
    default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------------------ depthwise 3x3
//
// Bandwidth-bound: 18 FLOP per output element.  One thread owns four consecutive channels
// (16 bytes along the NHWC channel axis) of XG adjacent output columns in a band of RB output
// rows and walks down the band with the 3-row window in registers: the nine filter taps are loaded
// once, every input row of the band once per thread ((XG-1)*STRIDE + 3 16-byte loads for XG outputs,
// the two outer ones shared with the neighbouring threads through L1), rows are requested PF output
// rows ahead of their use, results leave with nontemporal 16-byte stores.  With PF = RB every load
// of the band is in flight before the first store: a workgroup lives for one burst of reads and one
// of writes and then makes room for the next, which this memory system serves faster than long-lived
// workgroups that alternate (5.14 -> 5.7 TB/s over MobileNetV2's depthwise layers against threads that
// walk the whole image height).  The two halo rows a band shares with its neighbours come from L2:
// the (image, band, column group, channel group) positions of the chunk form one flat thread axis in
// memory order, and one XCD takes a contiguous stretch of it.

template <int STRIDE, int XG, int PF, int RB>
__global__ __launch_bounds__(256) void depthwise3x3_kernel(DepthwiseArgs a)
{
    constexpr int WIN = (XG - 1) * STRIDE + 3; // input columns per window row
    constexpr int NB = 3 + PF * STRIDE;        // row buffers: the window plus the rows in flight
    const int s = blockIdx.z;
    const int c4n = a.C >> 2;
    const uint32_t P = (uint32_t)(a.Wout / XG) * c4n;
    const uint32_t bands = (uint32_t)(a.Hout + RB - 1) / RB;
    // Workgroups are handed to the eight XCDs in turn, each with its own L2.  Neighbouring
    // workgroups share halo columns and rows, so each XCD gets one contiguous eighth of the flat axis
    // instead of every eighth workgroup: the shared pixels then meet in one L2.
    const uint32_t gidx = xcd_contiguous_block(blockIdx.x, gridDim.x) * 256u + threadIdx.x;
    if (gidx >= (uint32_t)a.N * bands * P) return;
    const uint32_t ib = gidx / P, pos = gidx - ib * P;
    const uint32_t img = ib / bands, band = ib - img * bands;
    const int oy0 = band * RB;
    const uint32_t xg = fd_div(pos, a.div_c4);
    const int c = (pos - xg * c4n) * 4, ox0 = xg * XG;
    const float *wq = a.bank[scheme_bits_index(a.schemes, s, a.S, a.L, a.slot)];
    const float *__restrict__ in = a.in + (size_t)s * a.in_scheme_stride + (size_t)img * a.Hin * a.Win * a.C + c;
    float *__restrict__ out =
        a.out + (size_t)s * a.out_scheme_stride + ((size_t)img * a.Hout * a.Wout + ox0) * a.C + c;

    floatx4 w[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) w[t] = *reinterpret_cast<const floatx4 *>(wq + (size_t)t * a.C + c);
    const floatx4 bias = *reinterpret_cast<const floatx4 *>(a.bias + c);
    const float lo = a.act >= 1 ? 0.0f : -__builtin_inff(), hi = a.act == 2 ? 6.0f : __builtin_inff();
    const floatx4 zero = floatx4{0.f, 0.f, 0.f, 0.f};
    const int ix0 = ox0 * STRIDE - 1;
    const bool ok_first = ix0 >= 0, ok_last = ix0 + WIN - 1 < a.Win; // only the outer columns can fall outside
    // last input row this band reads: rows beyond it (or beyond the image) are never fetched
    const int iy_end = min(a.Hin - 1, (min(oy0 + RB, a.Hout) - 1) * STRIDE + 1);
    auto load_row = [&](int iy, floatx4 (&r)[WIN]) {
        if (iy < 0 || iy > iy_end) {
#pragma unroll
            for (int k = 0; k < WIN; ++k) r[k] = zero;
            return;
        }
        const float *row = in + ((size_t)iy * a.Win + ix0) * a.C;
        r[0] = ok_first ? *reinterpret_cast<const floatx4 *>(row) : zero;
#pragma unroll
        for (int k = 1; k < WIN - 1; ++k) r[k] = *reinterpret_cast<const floatx4 *>(row + (size_t)k * a.C);
        r[WIN - 1] = ok_last ? *reinterpret_cast<const floatx4 *>(row + (size_t)(WIN - 1) * a.C) : zero;
    };

    // r[q] holds input row oy*STRIDE - 1 + q
    floatx4 r[NB][WIN];
#pragma unroll
    for (int q = 0; q < NB; ++q) load_row(oy0 * STRIDE - 1 + q, r[q]);
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        const int oy = oy0 + i;
        if (oy < a.Hout) {
#pragma unroll
            for (int x = 0; x < XG; ++x) {
                floatx4 acc = bias;
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    acc += r[0][x * STRIDE + k] * w[k];
                    acc += r[1][x * STRIDE + k] * w[3 + k];
                    acc += r[2][x * STRIDE + k] * w[6 + k];
                }
                acc.x = __builtin_amdgcn_fmed3f(acc.x, lo, hi);
                acc.y = __builtin_amdgcn_fmed3f(acc.y, lo, hi);
                acc.z = __builtin_amdgcn_fmed3f(acc.z, lo, hi);
                acc.w = __builtin_amdgcn_fmed3f(acc.w, lo, hi);
                __builtin_nontemporal_store(acc, reinterpret_cast<floatx4 *>(out + ((size_t)oy * a.Wout + x) * a.C));
            }
        }
        if (i + 1 < RB) {
#pragma unroll
            for (int q = 0; q + STRIDE < NB; ++q)
#pragma unroll
                for (int k = 0; k < WIN; ++k) r[q][k] = r[q + STRIDE][k];
            if (i + 1 + PF < RB) { // the band's last output row is i = RB - 1
#pragma unroll
                for (int j = 0; j < STRIDE; ++j) load_row((oy + 1) * STRIDE - 1 + NB - STRIDE + j, r[NB - STRIDE + j]);
            }
        }
    }
}

template <int STRIDE, int XG, int PF, int RB>
static hipError_t launch_depthwise_t(const DepthwiseArgs &a, int s_total, hipStream_t st)
{
    const size_t threads = (size_t)a.N * ((a.Hout + RB - 1) / RB) * (a.Wout / XG) * (a.C >> 2);
    if (threads > 0xffffffffull) return hipErrorInvalidValue;
    hipLaunchKernelGGL((depthwise3x3_kernel<STRIDE, XG, PF, RB>), dim3((unsigned)((threads + 255) / 256), 1, s_total),
                       dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_depthwise(const DepthwiseArgs &a, int s_total, hipStream_t st)
{
    if (a.N == 0 || s_total == 0) return hipSuccess;
    // bands of eight output rows with every row of the band requested up front (stride 2: two rows
    // of outputs ahead, the window being twice as tall); narrower column groups for odd widths
    if (a.stride == 1) {
        if (a.Wout % 4 == 0) return launch_depthwise_t<1, 4, 8, 8>(a, s_total, st);
        if (a.Wout % 2 == 0) return launch_depthwise_t<1, 2, 8, 8>(a, s_total, st);
        return launch_depthwise_t<1, 1, 8, 8>(a, s_total, st);
    }
    if (a.Wout % 2 == 0) return launch_depthwise_t<2, 2, 4, 8>(a, s_total, st);
    return launch_depthwise_t<2, 1, 4, 8>(a, s_total, st);
}

// ------------------------------------------------------------------ activation fake-quantization
//
// Variant in which a layer at b bits also reads its input at b bits: one workgroup per (scheme, image)
// tensor takes the tensor's largest magnitude (exact in any order), forms the scale and rewrites the
// tensor by the weight rule - same arithmetic, step for step, as quantize_channel.  The quantized copy
// goes to a buffer of its own, since other readers of the tensor (residual links, layers of another
// width) see it as it is; the consuming kernel is launched on the copy.  The second pass over the
// tensor comes from L2.

__global__ __launch_bounds__(256) void act_quantize_kernel(ActQuantArgs a)
{
    __shared__ float wmax[4];
    const int n = blockIdx.x, s = blockIdx.y, tid = threadIdx.x;
    const float *x = a.in + (size_t)s * a.in_scheme_stride + (size_t)n * a.elems;
    float *y = a.out + (size_t)s * a.out_scheme_stride + (size_t)n * a.elems;
    const int bits = bits_of_index(scheme_bits_index(a.schemes, s, a.S, a.L, a.slot));
    const bool vec = (a.elems & 3) == 0 && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y)) & 15) == 0;
    const int n4 = vec ? a.elems >> 2 : 0;
    const floatx4 *x4 = reinterpret_cast<const floatx4 *>(x);
    floatx4 *y4 = reinterpret_cast<floatx4 *>(y);
    if (bits == 32) {
        for (int i = tid; i < n4; i += 256) y4[i] = x4[i];
        for (int i = n4 * 4 + tid; i < a.elems; i += 256) y[i] = x[i];
        return;
    }
    float amax = 0.0f;
    for (int i = tid; i < n4; i += 256) {
        const floatx4 v = x4[i];
        amax = fmaxf(fmaxf(amax, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
    for (int i = n4 * 4 + tid; i < a.elems; i += 256) amax = fmaxf(amax, fabsf(x[i]));
    amax = wave_max(amax);
    if ((tid & 63) == 0) wmax[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    const int qmax = (1 << (bits - 1)) - 1;
    const float sc = amax > 0.0f ? __fdiv_rn(amax, (float)qmax) : 1.0f;
    for (int i = tid; i < n4; i += 256) {
        const floatx4 v = x4[i];
        floatx4 d;
#pragma unroll
        for (int e = 0; e < 4; ++e) d[e] = quantize_value(v[e], sc, qmax);
        y4[i] = d;
    }
    for (int i = n4 * 4 + tid; i < a.elems; i += 256) y[i] = quantize_value(x[i], sc, qmax);
}

hipError_t launch_act_quantize(const ActQuantArgs &a, int s_total, hipStream_t st)
{
    if (a.N == 0 || s_total == 0 || a.elems == 0) return hipSuccess;
    hipLaunchKernelGGL(act_quantize_kernel, dim3(a.N, s_total), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------ classifier head
//
// One workgroup per (scheme, image): global average pool, the classes x C matrix,
// argmax with the lowest index winning ties.

constexpr int kMaxClasses = 64;

__global__ __launch_bounds__(256) void head_kernel(HeadArgs a)
{
    extern __shared__ float sm[]; // pooled[C], then partial sums [256] x 16 bytes, then z[classes]
    const int s = blockIdx.y, n = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *x = a.in + (size_t)s * a.in_scheme_stride + (size_t)n * a.HW * a.C;
    float *pooled = sm;
    float *partial = sm + a.C;
    float *z = partial + 1024;

    // Pooling with 16-byte loads (C is a multiple of 4 for every producer): threads are laid out
    // [pixel group][4-channel lane]; the pixel groups split the positions when C / 4 < 256, four
    // independent partial sums per thread keep several loads in flight.
    const floatx4 *x4 = reinterpret_cast<const floatx4 *>(x);
    floatx4 *partial4 = reinterpret_cast<floatx4 *>(partial);
    const int c4n = a.C >> 2;
    const int cw = c4n < 256 ? c4n : 256;
    const int groups = 256 / cw;
    const int grp = tid / cw, cl = tid - grp * cw;
    const float inv = 1.0f / (float)a.HW;
    for (int c4 = cl; c4 < c4n; c4 += cw) {
        floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = acc0, acc2 = acc0, acc3 = acc0;
        if (grp < groups) {
            int i = grp;
            for (; i + 3 * groups < a.HW; i += 4 * groups) {
                acc0 += x4[(size_t)i * c4n + c4];
                acc1 += x4[(size_t)(i + groups) * c4n + c4];
                acc2 += x4[(size_t)(i + 2 * groups) * c4n + c4];
                acc3 += x4[(size_t)(i + 3 * groups) * c4n + c4];
            }
            for (; i < a.HW; i += groups) acc0 += x4[(size_t)i * c4n + c4];
        }
        floatx4 acc = (acc0 + acc1) + (acc2 + acc3);
        if (groups > 1) {
            __syncthreads();
            partial4[tid] = acc;
            __syncthreads();
            if (grp == 0) {
                for (int g = 1; g < groups; ++g) acc += partial4[g * cw + cl];
                *reinterpret_cast<floatx4 *>(pooled + c4 * 4) = acc * inv;
            }
        } else if (grp == 0) {
            *reinterpret_cast<floatx4 *>(pooled + c4 * 4) = acc * inv; // threads past the last whole group hold nothing
        }
    }
    __syncthreads();

    // activation fake-quantization: the pooled vector is rewritten at the classifier's width (one scale
    // for the vector) before the matrix reads it
    const int act_bits = a.act_quant ? bits_of_index(scheme_bits_index(a.schemes, s, a.S, a.L, a.slot)) : 32;
    if (act_bits != 32) { // uniform over the workgroup
        float amax = 0.0f;
        for (int c = tid; c < a.C; c += 256) amax = fmaxf(amax, fabsf(pooled[c]));
        amax = wave_max(amax);
        if (lane == 0) partial[wave] = amax; // the partial-sum area is free again
        __syncthreads();
        amax = fmaxf(fmaxf(partial[0], partial[1]), fmaxf(partial[2], partial[3]));
        const int qmax = (1 << (act_bits - 1)) - 1;
        const float sc = amax > 0.0f ? __fdiv_rn(amax, (float)qmax) : 1.0f;
        for (int c = tid; c < a.C; c += 256) pooled[c] = quantize_value(pooled[c], sc, qmax);
        __syncthreads();
    }

    // output row of this launch index: itself, unless the caller maps it; < 0 = the FP32 pass
    const int row = a.row_map ? a.row_map[s] : (s < a.S ? s : -1);
    const float *w = a.bank[scheme_bits_index(a.schemes, s, a.S, a.L, a.slot)];
    for (int j = wave; j < a.classes; j += 4) {
        float acc = 0.0f;
        for (int c = lane; c < a.C; c += 64) acc += pooled[c] * w[(size_t)j * a.C + c];
        acc = wave_sum(acc);
        if (lane == 0) z[j] = acc + a.bias[j];
    }
    __syncthreads();
    if (tid == 0) {
        int best = 0;
        for (int j = 1; j < a.classes; ++j)
            if (z[j] > z[best]) best = j;
        if (row >= 0) {
            a.top1[(size_t)row * a.top1_stride + n] = best;
        } else if (a.top1_base) {
            a.top1_base[n] = best;
        }
    }
    if (a.logits && row >= 0 && tid < a.classes)
        a.logits[((size_t)row * a.logits_n + a.n0 + n) * a.classes + tid] = z[tid];
}

hipError_t launch_head(const HeadArgs &a, int s_total, hipStream_t st)
{
    if (a.N == 0 || s_total == 0) return hipSuccess;
    if (a.C & 3) return hipErrorInvalidValue;
    const size_t sm = sizeof(float) * ((size_t)a.C + 1024 + kMaxClasses);
    hipLaunchKernelGGL(head_kernel, dim3(a.N, s_total), dim3(256), sm, st, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------ agreement

__global__ __launch_bounds__(256) void agree_kernel(AgreeArgs a)
{
    const int s = blockIdx.y;
    const int n = blockIdx.x * 256 + threadIdx.x;
    int hit = 0;
    if (n < a.N) hit = a.top1[(size_t)s * a.top1_stride + n] == a.top1_base[n];
    const int cnt = __popcll(__ballot(hit));
    __shared__ int wsum[4];
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int tot = wsum[0] + wsum[1] + wsum[2] + wsum[3];
        if (tot) atomicAdd(a.agree + s, tot);
    }
}

hipError_t launch_agree(const AgreeArgs &a, hipStream_t st)
{
    if (a.N == 0 || a.S == 0) return hipSuccess;
    hipLaunchKernelGGL(agree_kernel, dim3((a.N + 255) / 256, a.S), dim3(256), 0, st, a);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t *p, int32_t v, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

hipError_t launch_fill_i32(int32_t *p, int32_t v, size_t n, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
    return hipGetLastError();
}

// ------------------------------------------------------------------ fixed workspace (no-allocation entry point)
//
// One copy per GPU, part of the loaded code object, held until the process ends.  In host code the
// array's name is only a handle for the runtime, never an address: noalloc_scratch() asks the
// runtime, once per device and with that device current, where that device keeps its copy, and
// everything else (kernel arguments included) uses the pointer it returns.

static __device__ __align__(256) unsigned char scratch[AIQ_NOALLOC_SCRATCH_BYTES];

hipError_t noalloc_scratch(void **ptr, size_t *bytes)
{
    constexpr int kMaxDevices = 64;
    static void *per_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!per_device[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255)) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    *bytes = sizeof(scratch);
    return hipSuccess;
}

// ------------------------------------------------------------------ host tables as kernel arguments

constexpr int kUploadWords = 512;
struct UploadSlice {
    uint32_t w[kUploadWords];
};

__global__ __launch_bounds__(256) void upload_kernel(UploadSlice src, uint8_t *dst, int nbytes)
{
    // byte by byte: the destination needs no alignment
    const uint8_t *b = reinterpret_cast<const uint8_t *>(src.w);
    for (int i = threadIdx.x; i < nbytes; i += 256) dst[i] = b[i];
}

hipError_t upload_bytes(void *dst_dev, const void *src_host, size_t nbytes, hipStream_t st)
{
    const uint8_t *src = static_cast<const uint8_t *>(src_host);
    uint8_t *dst = static_cast<uint8_t *>(dst_dev);
    for (size_t off = 0; off < nbytes; off += sizeof(UploadSlice)) {
        UploadSlice sl;
        const size_t n = std::min(sizeof(UploadSlice), nbytes - off);
        std::memcpy(sl.w, src + off, n);
        hipLaunchKernelGGL(upload_kernel, dim3(1), dim3(256), 0, st, sl, dst + off, (int)n);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

} // namespace aiq
