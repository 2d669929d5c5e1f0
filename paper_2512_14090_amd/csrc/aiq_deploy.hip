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
// four groups of four consecutive output channels of one pixel; the epilogue passes them through
// LDS so that the NHWC stores cover whole lines.
//
// Workgroup = 4 wavefronts; per pass of CKC channels it stages in LDS the input rows of its
// region, already split (per pixel and eight-channel unit three neighbouring 16-byte pieces - hi,
// mid, lo - of bf16 values), and the codes of its output-channel tiles for those channels.  A wavefront owns 32*MT pixels x 32*NT
// output channels (MT = 2; 1 for layers of at most 32 output channels: short workgroups whose
// fixed latencies only more workgroups in flight can cover - four per compute unit) and issues, per tap and block of 16 channels,
// MT * NT * 3 MFMAs from 3 * MT + NT 16-byte LDS reads.

// Staging.  One item = eight channels of one staged pixel: two 16-byte global reads, three 16-byte
// LDS writes (the hi, mid and lo planes).  Item tid + 256 * i belongs to thread tid; which pixel
// and which eight channels of the pass it is does not change from pass to pass, so its LDS unit
// and its element offset from the workgroup's first image are formed once (kStageItems of them
// per thread; the host keeps a region's item count within that).  Per pass the reads of all items
// are issued first (stage_fetch), then split and written to LDS (stage_store).
constexpr int kChunks = kCodeStageChunks;

template <int kStageItems> // activation items per thread: kCodeStageItems, or twice that for long regions
struct StageItems {
    int dst[kStageItems]; // LDS unit of the hi plane, -1: no such item
    int src[kStageItems]; // element offset of channel c0 + 8 * c8 at the pixel, -1: outside the image
    // The pass's codes, 16 bytes per chunk: chunk tid + 256 * i goes to LDS unit code_off + tid + 256 * i;
    // the units are ordered [tile of the workgroup][tap][block of the pass][lane].
    int csrc[kChunks];    // element offset of the chunk in the codes for the pass that starts at block 0,
                          // plus the chunk's block within the pass in the low three bits; -1: no such chunk
};

template <int STRIDE, int PAD, int T, int kStageItems>
__device__ __forceinline__ void stage_plan(const CodeConvArgs &a, StageItems<kStageItems> &it, int c8shift, int img0, int oy0, int tid,
                                           int first_tile)
{
    {
        const int bshift = c8shift - 1;            // blocks of 16 channels per full pass: CKC / 16
        const int run = 64 << bshift;              // chunks of one (tile, tap)
        const int total = a.tiles_per_wg * T * run;
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            const int j = tid + i * 256;
            it.csrc[i] = -1;
            if (j < total) {
                const int r = j >> (6 + bshift), q = j & (run - 1);
                const int ctl = r / T, t = r - ctl * T;
                const int ct = min(first_tile + ctl, a.cout_tiles - 1);
                it.csrc[i] = ((ct * T + t) * a.CB) * 512 + q * 8 + (q >> 6);
            }
        }
    }
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
            it.dst[i] = (row * a.LW + col) * 3 * a.PSU + c8 * 3;
            if ((unsigned)iy < (unsigned)a.Hin && (unsigned)ix < (unsigned)a.Win && g < g_lim)
                it.src[i] = ((g * a.Hin + iy) * a.Win + ix) * a.Cin + c8 * 8;
        }
    }
}

// in0: the workgroup's first image; offsets within its own images fit 32 bits whatever the batch
template <int kStageItems>
__device__ __forceinline__ void stage_fetch(const CodeConvArgs &a, const StageItems<kStageItems> &it, floatx4 (&v)[kStageItems][2],
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

// chunk i of the pass that starts at channel block cb0 and has ncb blocks
template <int kStageItems>
__device__ __forceinline__ void code_fetch(const CodeConvArgs &a, const StageItems<kStageItems> &it, uintx4 (&cv)[kChunks], int cb0,
                                           int ncb)
{
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
        cv[i] = uintx4{0u, 0u, 0u, 0u};
        if (it.csrc[i] >= 0 && (it.csrc[i] & 7) < ncb)
            cv[i] = *(const __attribute__((address_space(1))) uintx4 *)(a.codes + (it.csrc[i] & ~7) + cb0 * 512);
    }
}

template <int kStageItems>
__device__ __forceinline__ void code_store(const CodeConvArgs &a, const StageItems<kStageItems> &it, const uintx4 (&cv)[kChunks],
                                           uintx4 *lds4, int tid)
{
#pragma unroll
    for (int i = 0; i < kChunks; ++i)
        if (it.csrc[i] >= 0) lds4[a.code_off + tid + i * 256] = cv[i];
}

template <int kStageItems>
__device__ __forceinline__ void stage_store(const CodeConvArgs &a, const StageItems<kStageItems> &it, const floatx4 (&v)[kStageItems][2],
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
        d[1] = uintx4{pack2(mid[0], mid[1]), pack2(mid[2], mid[3]), pack2(mid[4], mid[5]), pack2(mid[6], mid[7])};
        d[2] = uintx4{pack2(lo[0], lo[1]), pack2(lo[2], lo[3]), pack2(lo[4], lo[5]), pack2(lo[6], lo[7])};
        __builtin_amdgcn_sched_barrier(0); // one item's 24 temporaries at a time: the accumulators are live here
    }
}

// ONE: every pass stages a single block of 16 channels (CKC == 16)
template <int KS, int STRIDE, int NT, int KI, int MT, bool ONE>
__global__ __launch_bounds__(256, KI > kCodeStageItems ? 2 : (MT == 1 ? 4 : 3)) void conv_codes_kernel(CodeConvArgs a)
{
    constexpr int kStageItems = KI;
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
    int lds_base[MT];
    const int rw = a.R * a.Wout;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const uint32_t P = (uint32_t)(wpx * (32 * MT) + m * 32 + p);
        const uint32_t g = fd_div(P, a.div_rw);
        const uint32_t rem = P - g * rw;
        const uint32_t oy = fd_div(rem, a.div_wout);
        const uint32_t ox = rem - oy * a.Wout;
        const bool in_region = g < (uint32_t)a.G; // lanes past the region's last pixel compute nothing useful
        lds_base[m] = in_region ? ((g * a.RIN + oy * STRIDE) * a.LW + ox * STRIDE) * pix_units + kh * 3 : kh * 3;
    }

    floatx16 acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[m][n][e] = 0.0f;

    const int c8shift = __ffs(a.CKC >> 3) - 1; // CKC is 16, 32 or 64
    const bool active = ct0 < a.cout_tiles;    // wavefronts past the last output-channel tile only help staging
    StageItems<KI> items;
    stage_plan<STRIDE, PAD, T, KI>(a, items, c8shift, img0, oy0, tid, blockIdx.y * a.tiles_per_wg);
    const int n_items = (a.G * a.RIN * (a.LW << c8shift) + 255) >> 8; // <= kStageItems (host)
    const float *in0 = a.in + (size_t)img0 * a.Hin * a.Win * a.Cin;
    const int ncbf = a.CKC >> 4; // blocks of a full pass

    // The next pass's activations are requested before the current pass's MFMA loop and travel
    // while it runs; the loop itself reads LDS only, so it never waits behind these reads.  The
    // pass's codes (L2-resident) are requested at its start and arrive while the activations are
    // split: holding them a pass ahead as well would cost the registers that let three workgroups
    // share a compute unit.
    floatx4 staged[kStageItems][2];
    stage_fetch(a, items, staged, in0, 0, c8shift, n_items, tid);

    for (int c0 = 0; c0 < a.CB * 16; c0 += a.CKC) {
        const int ncb = min(a.CKC, a.CB * 16 - c0) >> 4;
        {
            uintx4 cstaged[kChunks];
            code_fetch(a, items, cstaged, c0 >> 4, ncb);
            if (c0) __syncthreads(); // the previous pass's LDS reads are done
            stage_store(a, items, staged, lds4, n_items);
            code_store(a, items, cstaged, lds4, tid);
        }
        __syncthreads();
        if (c0 + a.CKC < a.CB * 16) stage_fetch(a, items, staged, in0, c0 + a.CKC, c8shift, n_items, tid);

        {
            // The reduction runs over (tap, channel block) steps, channel block fastest.  The operands of
            // the next step are read from LDS during the current one: the codes into a second register
            // set, the activations plane by plane into the set in use, each plane as soon as the MFMAs
            // that read it have been issued.  The taps are unrolled, so which increment takes a lane's
            // two kinds of LDS address to the next step (next block, next tap, next window row) is one
            // scalar select on "last block of the tap"; the three planes of an eight-channel unit are
            // neighbours, so they are reached by immediate offsets.  The last step reads its own
            // operands again instead of running past the end.  (Wavefronts without an output tile of
            // their own run the loop on the last tile and store nothing.)
            // (addresses below are byte offsets into LDS)
            const int w_tap_step = (ncbf - ncb + 1) * 1024; // last block of a tap -> first block of the next
            const int a_tap_step = (pix_units - (ncb - 1) * 6) * 16, a_row_step = (a.LW - KS) * pix_units * 16;
            const char *ldsb = reinterpret_cast<const char *>(lds_raw);
            auto lds_at = [&](uint32_t off, int imm) { return *reinterpret_cast<const uintx4 *>(ldsb + off + imm); };
            uint32_t wv[NT], xv[MT];
#pragma unroll
            for (int n = 0; n < NT; ++n) wv[n] = (uint32_t)(a.code_off + ((wco * NT + n) * T * ncbf) * 64 + lane) * 16u;
#pragma unroll
            for (int m = 0; m < MT; ++m) xv[m] = (uint32_t)lds_base[m] * 16u;
            uintx4 xb[MT][3], wcur[NT], wnext[NT];
#pragma unroll
            for (int n = 0; n < NT; ++n) wcur[n] = lds_at(wv[n], 0);
#pragma unroll
            for (int pc = 0; pc < 3; ++pc)
#pragma unroll
                for (int m = 0; m < MT; ++m) xb[m][pc] = lds_at(xv[m], pc * 16);
            if constexpr (ONE) {
                // Passes of one channel block (the staging of long regions allows no more): a pixel is 96
                // bytes and a tap's codes 1024, so with the taps unrolled every operand sits at an
                // immediate offset from the lane's code address or from its window row's address, and
                // the two code register sets simply alternate: the loop issues no address arithmetic
                // and no register copies between its MFMAs.
                uint32_t xrow[MT][KS];
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int ky = 0; ky < KS; ++ky) xrow[m][ky] = xv[m] + (uint32_t)(ky * a.LW) * 96u;
                uintx4 wset[2][NT];
#pragma unroll
                for (int n = 0; n < NT; ++n) wset[0][n] = wcur[n];
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    __builtin_amdgcn_sched_barrier(0); // a tap's prefetches stay inside the tap
                    const int tn = t + 1, kyn = tn / KS, kxn = tn % KS;
                    if (tn < T) {
#pragma unroll
                        for (int n = 0; n < NT; ++n) wset[tn & 1][n] = lds_at(wv[n], tn * 1024);
                    }
#pragma unroll
                    for (int pc = 2; pc >= 0; --pc) { // smallest terms first
#pragma unroll
                        for (int m = 0; m < MT; ++m)
#pragma unroll
                            for (int n = 0; n < NT; ++n)
                                acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                    __builtin_bit_cast(bf16x8, wset[t & 1][n]), __builtin_bit_cast(bf16x8, xb[m][pc]), acc[m][n], 0, 0, 0);
                        if (tn < T) {
#pragma unroll
                            for (int m = 0; m < MT; ++m) xb[m][pc] = lds_at(xrow[m][tn < T ? kyn : 0], kxn * 96 + pc * 16);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            } else
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int x_last = t + 1 == T ? 0 : ((t % KS) == KS - 1 ? a_tap_step + a_row_step : a_tap_step);
                const int w_last = t + 1 == T ? 0 : w_tap_step;
#pragma unroll 1
                for (int cb = 0; cb < ncb; ++cb) {
                    const bool last = cb + 1 == ncb; // uniform
                    const uint32_t dw = last ? w_last : 1024, dx = last ? x_last : 96;
#pragma unroll
                    for (int n = 0; n < NT; ++n) wv[n] += dw;
#pragma unroll
                    for (int m = 0; m < MT; ++m) xv[m] += dx;
#pragma unroll
                    for (int n = 0; n < NT; ++n) wnext[n] = lds_at(wv[n], 0);
#pragma unroll
                    for (int pc = 2; pc >= 0; --pc) { // smallest terms first
#pragma unroll
                        for (int m = 0; m < MT; ++m)
#pragma unroll
                            for (int n = 0; n < NT; ++n)
                                acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                    __builtin_bit_cast(bf16x8, wcur[n]), __builtin_bit_cast(bf16x8, xb[m][pc]), acc[m][n], 0, 0, 0);
#pragma unroll
                        for (int m = 0; m < MT; ++m) xb[m][pc] = lds_at(xv[m], pc * 16);
                    }
#pragma unroll
                    for (int n = 0; n < NT; ++n) wcur[n] = wnext[n];
                }
            }
        }
    }

    // ---- epilogue: through LDS, then scale, bias, residual, activation.  A lane's accumulators are four
    // consecutive output channels of one pixel at a time, and a store of those would put sixteen
    // 16-byte pieces of sixteen different lines into every quarter of a store instruction; the
    // memory system takes such pieces one request each.  So the wavefront lays its pixels (32 at a
    // time) x 32*NT channels out in LDS (its own stretch of it: the staged tensors are dead once every
    // wavefront has left the last MFMA loop), then reads them back with consecutive lanes on
    // consecutive 16-byte chunks of one pixel and stores whole lines.  Chunk c of row r lives in
    // unit r * U + (c ^ (r % U)), which keeps both directions free of bank conflicts.
    __syncthreads();
    if (!active) return;
    constexpr int U = 8 * NT; // 16-byte chunks of one pixel's channels in this wavefront's tile
    uintx4 *tile = lds4 + wave * 32 * U; // 32 pixels at a time (one MFMA tile row), twice
    // The region's pixels are consecutive in memory (whole rows of one image, or whole images):
    // pixel P of the region is pixel first_px + P of the chunk.
    const float lo = a.act >= 1 ? 0.0f : -__builtin_inff(), hi = a.act == 2 ? 6.0f : __builtin_inff();
    const int px_img = a.Hout * a.Wout;
    const size_t first_px = a.G > 1 ? (size_t)img0 * px_img : ((size_t)img0 * a.Hout + oy0) * a.Wout;
    const int valid_px = a.G > 1 ? min(a.G, a.N - img0) * px_img : min(a.R, a.Hout - oy0) * a.Wout;
    float *out0 = a.out + first_px * a.Cout;
    const float *res0 = a.res ? a.res + first_px * a.Cout : nullptr;
    constexpr int ROWS = 64 / U;            // pixels one instruction covers
    constexpr int ITS = 32 / ROWS;          // instructions per half
    const int chunk = lane & (U - 1), sub = lane / U;
    const int co = ct0 * 32 + chunk * 4;    // Cout % 4 == 0; in the read-back a lane keeps one chunk: one scale, one bias
    floatx4 sc = {0.f, 0.f, 0.f, 0.f}, bi = {0.f, 0.f, 0.f, 0.f};
    if (co < a.Cout) {
        sc = *reinterpret_cast<const floatx4 *>(a.scales + co);
        bi = *reinterpret_cast<const floatx4 *>(a.bias + co);
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        // accumulator e of a lane is output channel 8 * (e / 4) + 4 * kh + e % 4 of its tile
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int c = n * 8 + g4 * 2 + kh;
                const floatx4 v = {acc[m][n][g4 * 4], acc[m][n][g4 * 4 + 1], acc[m][n][g4 * 4 + 2], acc[m][n][g4 * 4 + 3]};
                tile[p * U + (c ^ (p & (U - 1)))] = __builtin_bit_cast(uintx4, v);
            }
        floatx4 rv[ITS];
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int P = wpx * (32 * MT) + m * 32 + it * ROWS + sub;
            rv[it] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (res0 && co < a.Cout && P < valid_px) rv[it] = global_load4(res0 + P * a.Cout + co);
        }
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int row = it * ROWS + sub, P = wpx * (32 * MT) + m * 32 + row;
            floatx4 v = __builtin_bit_cast(floatx4, tile[row * U + (chunk ^ (row & (U - 1)))]);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = __builtin_amdgcn_fmed3f(__fmaf_rn(v[e], sc[e], bi[e]) + rv[it][e], lo, hi);
            if (co < a.Cout && P < valid_px) *reinterpret_cast<floatx4 *>(out0 + P * a.Cout + co) = v;
        }
    }
}

template <int KS, int STRIDE>
static hipError_t launch_codes_nt(const CodeConvArgs &a, int nt, int ki, int mt, size_t lds_bytes, dim3 grid, hipStream_t st)
{
    constexpr int K1 = kCodeStageItems, K2 = 2 * kCodeStageItems;
#define AIQ_LAUNCH(NT_, KI_, MT_)                                                                                     \
    if (nt == NT_ && ki == KI_ && mt == MT_) {                                                                       \
        if (a.CKC == 16)                                                                                             \
            hipLaunchKernelGGL((conv_codes_kernel<KS, STRIDE, NT_, KI_, MT_, true>), grid, dim3(256), lds_bytes, st, a);  \
        else                                                                                                         \
            hipLaunchKernelGGL((conv_codes_kernel<KS, STRIDE, NT_, KI_, MT_, false>), grid, dim3(256), lds_bytes, st, a); \
        return hipGetLastError();                                                                                    \
    }
    AIQ_LAUNCH(1, K1, 2)
    AIQ_LAUNCH(2, K1, 2)
    AIQ_LAUNCH(1, K2, 2)
    AIQ_LAUNCH(2, K2, 2)
    AIQ_LAUNCH(1, K1, 1)
    AIQ_LAUNCH(1, K2, 1)
#undef AIQ_LAUNCH
    return hipErrorInvalidValue;
}

hipError_t launch_conv_codes(const CodeConvArgs &a, int ks, int stride, int nt, int stage_items, int mt, size_t lds_bytes,
                             dim3 grid, hipStream_t st)
{
    if (ks == 3 && stride == 1) return launch_codes_nt<3, 1>(a, nt, stage_items, mt, lds_bytes, grid, st);
    if (ks == 3 && stride == 2) return launch_codes_nt<3, 2>(a, nt, stage_items, mt, lds_bytes, grid, st);
    if (ks == 1 && stride == 1) return launch_codes_nt<1, 1>(a, nt, stage_items, mt, lds_bytes, grid, st);
    if (ks == 1 && stride == 2) return launch_codes_nt<1, 2>(a, nt, stage_items, mt, lds_bytes, grid, st);
    return hipErrorInvalidValue;
}

template <int KS, int STRIDE, int NT, int KI, int MT>
static hipError_t codes_lds_t()
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_codes_kernel<KS, STRIDE, NT, KI, MT, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_codes_kernel<KS, STRIDE, NT, KI, MT, false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

// Dynamic LDS above 64 KB has to be allowed per kernel.
hipError_t conv_codes_set_lds_limits()
{
    hipError_t e = hipSuccess;
#define AIQ_SET(KS, ST)                                                                 \
    if (e == hipSuccess) e = codes_lds_t<KS, ST, 1, kCodeStageItems, 2>();              \
    if (e == hipSuccess) e = codes_lds_t<KS, ST, 2, kCodeStageItems, 2>();              \
    if (e == hipSuccess) e = codes_lds_t<KS, ST, 1, 2 * kCodeStageItems, 2>();          \
    if (e == hipSuccess) e = codes_lds_t<KS, ST, 2, 2 * kCodeStageItems, 2>();          \
    if (e == hipSuccess) e = codes_lds_t<KS, ST, 1, kCodeStageItems, 1>();              \
    if (e == hipSuccess) e = codes_lds_t<KS, ST, 1, 2 * kCodeStageItems, 1>();
    AIQ_SET(3, 1)
    AIQ_SET(3, 2)
    AIQ_SET(1, 1)
    AIQ_SET(1, 2)
#undef AIQ_SET
    return e;
}

} // namespace aiq
