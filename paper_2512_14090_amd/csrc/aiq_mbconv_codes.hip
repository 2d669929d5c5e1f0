// Deployed inverted-residual blocks (1x1 expand -> depthwise 3x3 -> 1x1 project, MobileNetV2)
// with 1x1 layers of at most eight bits: the block kernel of aiq_mbconv.hip with the matrix
// products of those layers taken from integer codes on the bf16 matrix pipe (a 16- or 32-bit
// 1x1 layer beside a low-bit one keeps the fp32 MFMA of the scoring kernel).
//
// The paper deploys the searched scheme and compares end-to-end throughput with the FP32 model,
// MobileNetV2 being its headline case (Implementation, experiment (3); Results, Analysis of AIQ
// Throughput Effects).  As in aiq_deploy.hip a weight of a layer at b <= 8 bits is code * s with
// |code| <= 127, exact in bf16, and a finite fp32 activation is exactly hi + mid + lo, three bf16
// terms, so
//     sum_k w_k x_k = s * (sum_k code_k hi_k + sum_k code_k mid_k + sum_k code_k lo_k)
// with every product exact in the MFMA's fp32 accumulator: the block computes the function of
// the weight-quantized FP32 model, up to the rounding order of the sums and one multiplication
// by s.  The depthwise layer stays on the vector ALU in fp32 with its quantize-dequantized
// weights (any width), and the hidden tensor stays in LDS in fp32.
//
// Differences from the fp32 block kernel:
//   expand   v_mfma_f32_16x16x32_bf16: A = codes of 16 hidden channels x 32 input channels,
//            B = 16 pixels x 32 input channels, once per term.  The block input is split once
//            per workgroup, either into registers (ready-made B operands of the pixel tiles a
//            wavefront owns) or into LDS planes of 64 bytes per pixel, 32-channel step and term.
//   project  v_mfma_f32_16x16x16_bf16: a lane's four depthwise outputs (hidden channels
//            16*hb + 4*kq .. +3 of its pixel) are split into three pairs of dwords - exactly the
//            B operands of that instruction - so the depthwise output still never leaves
//            registers.
//   scales   one multiplication per hidden value (folded with the bias into one FMA) and per
//            output value.
// The residual is re-read from global memory (it is in L2: the workgroup has just read it).
#include "aiq_internal.h"

#include <algorithm>

namespace aiq {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ floatx4 mc_gload4(const float *p)
{
    return *(const __attribute__((address_space(1))) floatx4 *)(p);
}
__device__ __forceinline__ uintx4 mc_gload_u4(const uint16_t *p)
{
    return *(const __attribute__((address_space(1))) uintx4 *)(p);
}
__device__ __forceinline__ uintx2 mc_gload_u2(const uint16_t *p)
{
    return *(const __attribute__((address_space(1))) uintx2 *)(p);
}
__device__ __forceinline__ floatx4 mc_clamp4(floatx4 v, float lo, float hi)
{
    v.x = __builtin_amdgcn_fmed3f(v.x, lo, hi);
    v.y = __builtin_amdgcn_fmed3f(v.y, lo, hi);
    v.z = __builtin_amdgcn_fmed3f(v.z, lo, hi);
    v.w = __builtin_amdgcn_fmed3f(v.w, lo, hi);
    return v;
}
__device__ __forceinline__ float mc_lo(int act) { return act >= 1 ? 0.0f : -__builtin_inff(); }
__device__ __forceinline__ float mc_hi(int act) { return act == 2 ? 6.0f : __builtin_inff(); }

// x = hi + mid + lo exactly for finite x, each a bf16 value in the upper half of an fp32 bit
// pattern; both subtractions only clear leading significand bits and are exact
__device__ __forceinline__ void mc_split(float x, uint32_t &hi, uint32_t &mid, uint32_t &lo)
{
    hi = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(hi);
    mid = __float_as_uint(r1) & 0xffff0000u;
    lo = __float_as_uint(r1 - __uint_as_float(mid));
}
// upper halves of a and b as one dword, a in the low half
__device__ __forceinline__ uint32_t mc_pack(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// four values -> their three terms, each as four bf16 in two dwords
__device__ __forceinline__ void mc_split4(floatx4 v, uintx2 t[3])
{
    uint32_t h[4], m[4], l[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) mc_split(v[j], h[j], m[j], l[j]);
    t[0] = uintx2{mc_pack(h[0], h[1]), mc_pack(h[2], h[3])};
    t[1] = uintx2{mc_pack(m[0], m[1]), mc_pack(m[2], m[3])};
    t[2] = uintx2{mc_pack(l[0], l[1]), mc_pack(l[2], l[3])};
}
// eight values (two groups of four consecutive channels) -> three terms of eight bf16
__device__ __forceinline__ void mc_split8(floatx4 v0, floatx4 v1, uintx4 t[3])
{
    uintx2 a[3], b[3];
    mc_split4(v0, a);
    mc_split4(v1, b);
#pragma unroll
    for (int i = 0; i < 3; ++i) t[i] = uintx4{a[i].x, a[i].y, b[i].x, b[i].y};
}

// Block shape (CIN, HID, COUT, H, STRIDE, RES) and tiling: R output rows per workgroup, G images
// per workgroup (whole images only), HC hidden channels per chunk, NW wavefronts per workgroup,
// XREG: split block input in registers instead of LDS, WGS: workgroups meant to share a compute
// unit, EPRE / DPRE: the expand codes of a chunk / the depthwise and project weights of a hidden
// block are fetched into registers one step ahead.
template <int CIN_, int HID_, int COUT_, int H_, int STRIDE_, bool RES_, int R_, int G_, int HC_, int NW_, bool XREG_,
          int WGS_, bool EPRE_, bool DPRE_>
struct McCfg {
    static constexpr int CIN = CIN_, HID = HID_, COUT = COUT_, H = H_, STRIDE = STRIDE_, R = R_, G = G_, HC = HC_;
    static constexpr bool RES = RES_, XREG = XREG_, EPRE = EPRE_, DPRE = DPRE_;
    static constexpr int NW = NW_, THREADS = NW_ * 64, WGS = WGS_;
    static constexpr int WAVES_PER_SIMD = NW * WGS / 4;
    static constexpr int W = H, HO = H / STRIDE, WO = HO;
    static constexpr int RI = (R - 1) * STRIDE + 3;  // E rows: input rows a band of R output rows needs
    static constexpr bool WHOLE = (R == HO);         // the band is the whole image: E row 0 is always padding
    static constexpr int XOFF = WHOLE ? 1 : 0;       // E row of X row 0
    static constexpr int XROWS = WHOLE ? H : RI;     // most rows of X a band can hold
    static constexpr int KS = (CIN + 31) / 32;       // 32-channel steps of the expand product
    static constexpr int UNITS = KS * 4;             // eight-channel units of a pixel
    static constexpr int NPX = G * XROWS * W;        // pixels of X
    static constexpr int HT = HC / 16, HB = HID / 16, NCH = HID / HC;
    static constexpr int CT = (COUT + 15) / 16;
    static constexpr int EW = W + 1, EPIX = RI * EW + 1;
    static constexpr int EPL = G * EPIX * 4;          // floats per E plane
    static constexpr int X_BYTES = XREG ? 0 : KS * 3 * NPX * 64;
    static constexpr int E_FLOATS = (HC / 4) * EPL;
    static constexpr int LDS_BYTES = X_BYTES + 2 * E_FLOATS * 4;
    static constexpr int PTE = G * XROWS * W / 16;
    static constexpr int XT = PTE >= NW ? (PTE + NW - 1) / NW : 1;
    static constexpr int HS = PTE >= NW ? 1 : NW / PTE;
    static constexpr int HTW = HT / HS;
    static constexpr int PTO = G * R * WO / 16;
    static constexpr int MT = PTO >= NW ? PTO / NW : 1;
    static constexpr int WPP = PTO >= NW ? 1 : NW / PTO;
    static constexpr int CTW = CT / WPP;
    static constexpr int BANDS = HO / R;
    static constexpr int TPR = WO >= 16 ? WO / 16 : 1;
    static constexpr int NRW = (MT - 1) * STRIDE + 3;
    static_assert(CIN % 8 == 0 && HID % HC == 0 && HC % 16 == 0 && COUT % 4 == 0, "channel counts");
    static_assert(HO % R == 0 && (G == 1 || WHOLE), "bands tile the image; several images only as whole images");
    static_assert((G * XROWS * W) % 16 == 0 && (PTE >= NW || (NW % PTE == 0 && HT % HS == 0)), "expand tiles");
    static_assert(!WHOLE || PTE < NW || PTE % NW == 0, "whole images: every wavefront has all its expand tiles");
    static_assert((G * R * WO) % 16 == 0 && (PTO >= NW ? PTO % NW == 0 : NW % PTO == 0), "pixel tiles per wavefront");
    static_assert(CT % WPP == 0, "output-channel tiles per wavefront");
    static_assert(MT == 1 || (WO >= 16 && NW % TPR == 0 && G == 1), "strips of tiles need whole 16-pixel row segments");
    static_assert((W & (W - 1)) == 0 && ((R * WO) & (R * WO - 1)) == 0, "powers of two");
    static_assert(!RES || (CIN == COUT && STRIDE == 1), "residual needs matching shapes");
    static_assert(X_BYTES % 16 == 0 && LDS_BYTES * WGS <= 160 * 1024, "LDS budget");
};

} // namespace

// ------------------------------------------------------------------ code packing
//
// int32 codes [rows][k] -> bf16 in the order an MFMA's A operand wants for steps of KSTEP = 32 or
// 16 along k: [rows/16][ceil(k/KSTEP)][64 lanes][KSTEP/4], lane = 16 * (position in step / (KSTEP/4))
// + row within its tile of 16, element = position % (KSTEP/4).  The destination has been cleared:
// padding rows and positions stay zero.
__global__ __launch_bounds__(256) void pack_mb_codes_kernel(const int32_t *__restrict__ codes, uint16_t *__restrict__ out,
                                                            int rows, int k, int kstep)
{
    const size_t total = (size_t)rows * k;
    const int per = kstep >> 2, steps = (k + kstep - 1) / kstep;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int r = (int)(i / k), kk = (int)(i - (size_t)r * k);
        const int ks = kk / kstep, pos = kk - ks * kstep;
        const size_t o = ((((size_t)(r >> 4) * steps + ks) * 64) + (pos / per) * 16 + (r & 15)) * per + pos % per;
        out[o] = (uint16_t)(__float_as_uint((float)codes[i]) >> 16); // |code| <= 127: exact
    }
}

hipError_t launch_pack_mb_codes(const int32_t *codes, uint16_t *out, int rows, int k, int kstep, hipStream_t st)
{
    const size_t total = (size_t)rows * k;
    if (total == 0) return hipSuccess;
    if (kstep != 16 && kstep != 32) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(pack_mb_codes_kernel, dim3(blocks), dim3(256), 0, st, codes, out, rows, k, kstep);
    return hipGetLastError();
}

// ------------------------------------------------------------------ the block kernel

// EC / PC: the expand / project layer runs from codes; a layer of 16 or 32 bits beside a low-bit one keeps its
// quantize-dequantized fp32 weights and the fp32 MFMA of the scoring kernel (its operand then needs no split).
template <class C, bool EC, bool PC>
__global__ __launch_bounds__(C::THREADS) __attribute__((amdgpu_waves_per_eu(C::WAVES_PER_SIMD, C::WAVES_PER_SIMD)))
void mbconv_codes_kernel(MbCodeArgs a)
{
    static_assert(EC || PC, "at least one layer on codes");
    static_assert(EC || C::XREG, "an fp32 expand layer keeps the block input in registers");
    constexpr int CB = (C::CIN + 15) / 16; // 16-channel steps of an fp32 expand product
    extern __shared__ float lds[];
    char *X = reinterpret_cast<char *>(lds);
    float *E = lds + C::X_BYTES / 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, p = lane & 15, kq = lane >> 4;
    const int band = blockIdx.x % C::BANDS;
    const int img0 = (blockIdx.x / C::BANDS) * C::G;

    // valid E rows of this band: E row r holds image row iy0 + r
    const int iy0 = band * C::R * C::STRIDE - 1;
    const int r_lo = iy0 < 0 ? -iy0 : 0;
    const int r_hi = min(C::RI, C::H - iy0);
    const int nrows = r_hi - r_lo;
    const int n_exp_tiles = (C::G * nrows * C::W) >> 4;

    // ---- expand tiles of this wavefront: E offset of the lane's pixel, and X as split B operands
    const int h0 = C::HS > 1 ? (wave % C::HS) * C::HTW : 0;
    bool x_ok[C::XT];
    int e_off[C::XT], x_pix[C::XT];
    uintx4 xr[(C::XREG && EC) ? C::XT : 1][(C::XREG && EC) ? C::KS : 1][3];
    floatx4 xf[EC ? 1 : C::XT][EC ? 1 : CB];
#pragma unroll
    for (int k = 0; k < C::XT; ++k) {
        const int e = C::HS > 1 ? wave / C::HS : wave + k * C::NW;
        const int f = e * 16 + p;
        int g = 0, rem = f;
        if (C::G > 1) {
            g = f / (C::H * C::W); // several images only as whole images: nrows == H
            rem = f % (C::H * C::W);
        }
        const int rr = rem / C::W, x = rem % C::W;
        const int r = r_lo + rr;
        x_ok[k] = e < n_exp_tiles;
        e_off[k] = (g * C::EPIX + r * C::EW + x + 1) * 4 + kq * C::EPL;
        x_pix[k] = (g * C::XROWS + (r - C::XOFF)) * C::W + x;
        if (!EC) {
            const int img = img0 + g;
            const float *px = a.in + (((size_t)img * C::H + (iy0 + r)) * C::W + x) * C::CIN;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const int ch = cb * 16 + kq * 4;
                xf[EC ? 0 : k][EC ? 0 : cb] = (x_ok[k] && img < a.N && ch < C::CIN) ? mc_gload4(px + ch) : floatx4{0.f, 0.f, 0.f, 0.f};
            }
        } else if (C::XREG) {
            const int img = img0 + g;
            const float *px = a.in + (((size_t)img * C::H + (iy0 + r)) * C::W + x) * C::CIN;
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) {
                const int ch = ks * 32 + kq * 8;
                floatx4 v0 = floatx4{0.f, 0.f, 0.f, 0.f}, v1 = v0;
                if (x_ok[k] && img < a.N && ch < C::CIN) {
                    v0 = mc_gload4(px + ch);
                    v1 = mc_gload4(px + ch + 4);
                }
                mc_split8(v0, v1, xr[(C::XREG && EC) ? k : 0][(C::XREG && EC) ? ks : 0]);
            }
        }
    }

    // ---- clear E (borders and out-of-image rows stay zero for good); stage X unless it is in registers
    for (int i = tid; i < 2 * C::E_FLOATS / 4; i += C::THREADS)
        reinterpret_cast<floatx4 *>(E)[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (!C::XREG && EC) {
        // item = eight channels of one pixel: two 16-byte global reads, one 16-byte LDS write per term;
        // units past CIN are written as zeros (they meet zero codes, but must not hold NaN patterns)
        const int per_img = nrows * C::W * C::UNITS;
        const int xrow = r_lo - C::XOFF; // X row of the first valid E row
        for (int g = 0; g < C::G; ++g) {
            const int img = img0 + g;
            const float *src = a.in + (((size_t)img * C::H + (iy0 + r_lo)) * C::W) * C::CIN;
            constexpr int UN = 2;
            for (int base = tid; base < per_img; base += C::THREADS * UN) {
                floatx4 v[UN][2];
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int idx = base + u * C::THREADS;
                    const int unit = idx % C::UNITS, pix = idx / C::UNITS;
                    v[u][0] = v[u][1] = floatx4{0.f, 0.f, 0.f, 0.f};
                    if (idx < per_img && img < a.N && unit * 8 < C::CIN) {
                        v[u][0] = mc_gload4(src + (size_t)pix * C::CIN + unit * 8);
                        v[u][1] = mc_gload4(src + (size_t)pix * C::CIN + unit * 8 + 4);
                    }
                }
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int idx = base + u * C::THREADS;
                    if (idx < per_img) {
                        const int unit = idx % C::UNITS, pix = idx / C::UNITS; // pix = rr * W + x
                        const int xp = (g * C::XROWS + xrow) * C::W + pix;
                        uintx4 t[3];
                        mc_split8(v[u][0], v[u][1], t);
#pragma unroll
                        for (int i = 0; i < 3; ++i)
                            *reinterpret_cast<uintx4 *>(X + ((size_t)((unit >> 2) * 3 + i) * C::NPX + xp) * 64 + (unit & 3) * 16) = t[i];
                    }
                }
            }
        }
    }

    const float lo_e = mc_lo(a.act_e), hi_e = mc_hi(a.act_e), lo_d = mc_lo(a.act_d), hi_d = mc_hi(a.act_d);

    // ---- output tiles of this wavefront
    const int ct0 = (C::WPP > 1 ? (wave % C::WPP) : 0) * C::CTW;
    int e_base[C::MT], o_g[C::MT], o_y[C::MT], o_x[C::MT];
#pragma unroll
    for (int m = 0; m < C::MT; ++m) {
        const int t = C::WPP > 1 ? wave / C::WPP : ((wave / C::TPR) * C::MT + m) * C::TPR + wave % C::TPR;
        const int o = t * 16 + p;
        const int g = o / (C::R * C::WO), rem = o % (C::R * C::WO);
        const int oy = rem / C::WO, ox = rem % C::WO;
        o_g[m] = g;
        o_y[m] = oy;
        o_x[m] = ox;
        e_base[m] = (g * C::EPIX + oy * C::STRIDE * C::EW + ox * C::STRIDE) * 4 + kq * C::EPL;
    }

    floatx4 acc[C::MT][C::CTW];
#pragma unroll
    for (int m = 0; m < C::MT; ++m)
#pragma unroll
        for (int i = 0; i < C::CTW; ++i) acc[m][i] = floatx4{0.f, 0.f, 0.f, 0.f};

    // Weights of one expand step of this wavefront: bias, scale and the code operands of its hidden tiles.
    constexpr bool EPRE = C::EPRE;
    struct ExpW {
        floatx4 be[C::HTW], se[EC ? C::HTW : 1];
        uintx4 wa[(EPRE && EC) ? C::HTW : 1][(EPRE && EC) ? C::KS : 1];
        floatx4 wf[(EPRE && !EC) ? C::HTW : 1][(EPRE && !EC) ? CB : 1];
    };
    auto load_expw = [&](int c, ExpW &w) {
#pragma unroll
        for (int h = 0; h < C::HTW; ++h) {
            w.be[h] = mc_gload4(a.bias_e + (c * C::HT + h0 + h) * 16 + kq * 4);
            if (EC) w.se[EC ? h : 0] = mc_gload4(a.scale_e + (c * C::HT + h0 + h) * 16 + kq * 4);
        }
        if (EPRE && !EC) {
            const float *wc = a.w_e + ((size_t)(c * C::HT + h0) * CB * 64 + lane) * 4;
#pragma unroll
            for (int h = 0; h < C::HTW; ++h)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    w.wf[(EPRE && !EC) ? h : 0][(EPRE && !EC) ? cb : 0] = mc_gload4(wc + (size_t)((h * CB + cb) * 64) * 4);
        }
        if (EPRE && EC) {
            const uint16_t *wc = a.codes_e + ((size_t)(c * C::HT + h0) * C::KS * 64 + lane) * 8;
#pragma unroll
            for (int h = 0; h < C::HTW; ++h)
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks)
                    w.wa[(EPRE && EC) ? h : 0][(EPRE && EC) ? ks : 0] = mc_gload_u4(wc + (size_t)((h * C::KS + ks) * 64) * 8);
        }
    };
    // expand of hidden chunk c into E buffer eb
    auto expand = [&](int c, int eb, const ExpW &w) {
        float *Eb = E + eb * C::E_FLOATS + h0 * 4 * C::EPL;
        const uint16_t *wc = a.codes_e + ((size_t)(c * C::HT + h0) * C::KS * 64 + lane) * 8;
#pragma unroll
        for (int k = 0; k < C::XT; ++k) {
            if (!C::WHOLE && !x_ok[k]) continue; // uniform per wavefront; whole images have every tile
            floatx4 ea[C::HTW];
#pragma unroll
            for (int h = 0; h < C::HTW; ++h) ea[h] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (!EC) {
                const float *wcf = a.w_e + ((size_t)(c * C::HT + h0) * CB * 64 + lane) * 4;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    const floatx4 xb = xf[EC ? 0 : k][EC ? 0 : cb];
                    floatx4 wa[C::HTW];
#pragma unroll
                    for (int h = 0; h < C::HTW; ++h)
                        wa[h] = EPRE ? w.wf[(EPRE && !EC) ? h : 0][(EPRE && !EC) ? cb : 0] : mc_gload4(wcf + (size_t)((h * CB + cb) * 64) * 4);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int h = 0; h < C::HTW; ++h)
                            ea[h] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[h][j], xb[j], ea[h], 0, 0, 0);
                }
#pragma unroll
                for (int h = 0; h < C::HTW; ++h)
                    *reinterpret_cast<floatx4 *>(Eb + h * 4 * C::EPL + e_off[k]) = mc_clamp4(ea[h] + w.be[h], lo_e, hi_e);
                continue;
            }
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) {
                uintx4 xb[3];
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    if (C::XREG)
                        xb[t] = xr[(C::XREG && EC) ? k : 0][(C::XREG && EC) ? ks : 0][t];
                    else
                        xb[t] = *reinterpret_cast<const uintx4 *>(X + ((size_t)(ks * 3 + t) * C::NPX + x_pix[k]) * 64 + kq * 16);
                }
                uintx4 wa[C::HTW];
#pragma unroll
                for (int h = 0; h < C::HTW; ++h)
                    wa[h] = EPRE ? w.wa[(EPRE && EC) ? h : 0][(EPRE && EC) ? ks : 0] : mc_gload_u4(wc + (size_t)((h * C::KS + ks) * 64) * 8);
#pragma unroll
                for (int t = 0; t < 3; ++t)
#pragma unroll
                    for (int h = 0; h < C::HTW; ++h)
                        ea[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[h]),
                                                                        __builtin_bit_cast(bf16x8, xb[t]), ea[h], 0, 0, 0);
            }
#pragma unroll
            for (int h = 0; h < C::HTW; ++h)
                *reinterpret_cast<floatx4 *>(Eb + h * 4 * C::EPL + e_off[k]) = mc_clamp4(ea[h] * w.se[EC ? h : 0] + w.be[h], lo_e, hi_e);
        }
    };

    // Weights of one 16-channel hidden block for the depthwise + project step.
    struct DwW {
        floatx4 wd[9], bd;
        uintx2 wp[PC ? C::CTW : 1];
        floatx4 wpf[PC ? 1 : C::CTW];
    };
    auto load_dww = [&](int hb, DwW &w) {
#pragma unroll
        for (int t = 0; t < 9; ++t) w.wd[t] = mc_gload4(a.w_d + (size_t)t * C::HID + hb * 16 + kq * 4);
        w.bd = mc_gload4(a.bias_d + hb * 16 + kq * 4);
#pragma unroll
        for (int i = 0; i < C::CTW; ++i) {
            if (PC)
                w.wp[PC ? i : 0] = mc_gload_u2(a.codes_p + (((size_t)(ct0 + i) * C::HB + hb) * 64 + lane) * 4);
            else
                w.wpf[PC ? 0 : i] = mc_gload4(a.w_p + (((size_t)(ct0 + i) * C::HB + hb) * 64 + lane) * 4);
        }
    };
    auto dw_project = [&](int sb, int eb, const DwW &w) {
        const float *Eb = E + eb * C::E_FLOATS + sb * 4 * C::EPL + e_base[0];
        floatx4 d[C::MT];
#pragma unroll
        for (int m = 0; m < C::MT; ++m) d[m] = w.bd;
#pragma unroll
        for (int kx = 0; kx < 3; ++kx)
#pragma unroll
            for (int r = 0; r < C::NRW; ++r) {
                const floatx4 v = *reinterpret_cast<const floatx4 *>(Eb + (r * C::EW + kx) * 4);
#pragma unroll
                for (int ky = 0; ky < 3; ++ky) {
                    const int dd = r - ky;
                    if (dd < 0 || dd % C::STRIDE != 0 || dd / C::STRIDE >= C::MT) continue;
                    d[dd / C::STRIDE] += v * w.wd[ky * 3 + kx];
                }
            }
#pragma unroll
        for (int m = 0; m < C::MT; ++m) {
            const floatx4 dc = mc_clamp4(d[m], lo_d, hi_d);
            if (!PC) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < C::CTW; ++i)
                        acc[m][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(w.wpf[PC ? 0 : i][j], dc[j], acc[m][i], 0, 0, 0);
                continue;
            }
            uintx2 t[3];
            mc_split4(dc, t);
#pragma unroll
            for (int j = 0; j < 3; ++j)
#pragma unroll
                for (int i = 0; i < C::CTW; ++i)
                    acc[m][i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, w.wp[PC ? i : 0]),
                                                                          __builtin_bit_cast(shortx4, t[j]), acc[m][i], 0, 0, 0);
        }
    };
    // consumes chunk c; with DPRE w0 arrives holding the weights of its first hidden block
    auto consume = [&](int c, int eb, DwW &w0) {
#pragma unroll
        for (int sb = 0; sb < C::HT; ++sb) {
            if (C::DPRE) {
                DwW w1;
                if (sb + 1 < C::HT) load_dww(c * C::HT + sb + 1, w1);
                dw_project(sb, eb, w0);
                if (sb + 1 < C::HT) w0 = w1;
            } else {
                load_dww(c * C::HT + sb, w0);
                dw_project(sb, eb, w0);
            }
        }
    };

    // Inside a barrier interval chunk c is consumed and chunk c+1 expanded; the two are independent.
    DwW w0;
    ExpW ew;
    if (C::DPRE) load_dww(0, w0);
    load_expw(0, ew);
    __syncthreads();
    expand(0, 0, ew);
    __syncthreads();
#pragma unroll 1
    for (int c = 0; c < C::NCH; ++c) {
        const int eb = c & 1;
        const bool more = c + 1 < C::NCH;
        if (more) load_expw(c + 1, ew);
        consume(c, eb, w0);
        if (more) {
            if (C::DPRE) load_dww((c + 1) * C::HT, w0);
            expand(c + 1, eb ^ 1, ew);
        }
        __syncthreads();
    }

    // ---- epilogue: scale, bias, residual (the block input), activation, 16-byte NHWC stores
    const float lo_p = mc_lo(a.act_p), hi_p = mc_hi(a.act_p);
#pragma unroll
    for (int i = 0; i < C::CTW; ++i) {
        const int co = (ct0 + i) * 16 + kq * 4;
        if (co >= C::COUT) continue;
        const floatx4 bp = mc_gload4(a.bias_p + co);
        const floatx4 sp = PC ? mc_gload4(a.scale_p + co) : floatx4{1.f, 1.f, 1.f, 1.f};
#pragma unroll
        for (int m = 0; m < C::MT; ++m) {
            const int img = img0 + o_g[m];
            if (img >= a.N) continue;
            const int oy = band * C::R + o_y[m];
            const size_t o = (((size_t)img * C::HO + oy) * C::WO + o_x[m]) * C::COUT + co;
            floatx4 v = PC ? acc[m][i] * sp + bp : acc[m][i] + bp;
            if (C::RES) v += mc_gload4(a.in + o); // same shape as the output
            *reinterpret_cast<floatx4 *>(a.out + o) = mc_clamp4(v, lo_p, hi_p);
        }
    }
}

// ------------------------------------------------------------------ last 1x1 layer with the classifier's pooling
//
// A 1x1 layer on 8x8 pixels whose only reader is the classifier (MobileNetV2's last convolution)
// writes the mean of its activated outputs over the image instead of the outputs.  From integer
// codes: one workgroup of 8 wavefronts per image; the image's 64 pixels x Cin values are split once
// into LDS planes (64 bytes per pixel, 32-channel step and term); a wavefront takes groups of CG
// tiles of 16 output channels, each against the four pixel tiles of the image (A operands from
// global memory one step ahead, 12 LDS reads per 12 * CG MFMAs), then applies scale, bias and
// activation, adds the four tiles in registers and the 16 pixels of a tile across lanes.
template <int CG>
__global__ __launch_bounds__(512) void pooled_codes_kernel(PoolCodeArgs a)
{
    extern __shared__ float lds[];
    char *X = reinterpret_cast<char *>(lds);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, p = lane & 15, kq = lane >> 4;
    const int img = blockIdx.x;
    const int KS = a.KS, units = KS * 4, items = 64 * units;
    const float *src = a.in + (size_t)img * 64 * a.Cin;
    constexpr int UN = 2;
    for (int base = tid; base < items; base += 512 * UN) {
        floatx4 v[UN][2];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int idx = base + u * 512;
            const int unit = idx % units, pix = idx / units;
            v[u][0] = v[u][1] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (idx < items && unit * 8 < a.Cin) {
                v[u][0] = mc_gload4(src + (size_t)pix * a.Cin + unit * 8);
                v[u][1] = mc_gload4(src + (size_t)pix * a.Cin + unit * 8 + 4);
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int idx = base + u * 512;
            if (idx < items) {
                const int unit = idx % units, pix = idx / units;
                uintx4 t[3];
                mc_split8(v[u][0], v[u][1], t);
#pragma unroll
                for (int i = 0; i < 3; ++i)
                    *reinterpret_cast<uintx4 *>(X + ((size_t)((unit >> 2) * 3 + i) * 64 + pix) * 64 + (unit & 3) * 16) = t[i];
            }
        }
    }
    __syncthreads();

    const float lo = mc_lo(a.act), hi = mc_hi(a.act);
    const char *xl = X + p * 64 + kq * 16;
    for (int g = wave; g < a.groups; g += 8) {
        floatx4 acc[CG][4];
#pragma unroll
        for (int i = 0; i < CG; ++i)
#pragma unroll
            for (int pt = 0; pt < 4; ++pt) acc[i][pt] = floatx4{0.f, 0.f, 0.f, 0.f};
        const uint16_t *wc = a.codes + ((size_t)(g * CG) * KS * 64 + lane) * 8;
        uintx4 wa[CG], wn[CG];
#pragma unroll
        for (int i = 0; i < CG; ++i) wa[i] = mc_gload_u4(wc + (size_t)(i * KS) * 512);
        for (int ks = 0; ks < KS; ++ks) {
            const int kn = ks + 1 < KS ? ks + 1 : ks;
#pragma unroll
            for (int i = 0; i < CG; ++i) wn[i] = mc_gload_u4(wc + (size_t)(i * KS + kn) * 512);
#pragma unroll
            for (int t = 0; t < 3; ++t)
#pragma unroll
                for (int pt = 0; pt < 4; ++pt) {
                    const uintx4 xb = *reinterpret_cast<const uintx4 *>(xl + ((size_t)(ks * 3 + t) * 64 + pt * 16) * 64);
#pragma unroll
                    for (int i = 0; i < CG; ++i)
                        acc[i][pt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[i]),
                                                                             __builtin_bit_cast(bf16x8, xb), acc[i][pt], 0, 0, 0);
                }
#pragma unroll
            for (int i = 0; i < CG; ++i) wa[i] = wn[i];
        }
#pragma unroll
        for (int i = 0; i < CG; ++i) {
            const int co = (g * CG + i) * 16 + kq * 4; // uniform over the 16 lanes that are reduced together
            floatx4 sum = floatx4{0.f, 0.f, 0.f, 0.f};
            if (co < a.Cout) {
                const floatx4 sc = mc_gload4(a.scales + co), bi = mc_gload4(a.bias + co);
#pragma unroll
                for (int pt = 0; pt < 4; ++pt) sum += mc_clamp4(acc[i][pt] * sc + bi, lo, hi);
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) {
                sum.x += __shfl_xor(sum.x, off);
                sum.y += __shfl_xor(sum.y, off);
                sum.z += __shfl_xor(sum.z, off);
                sum.w += __shfl_xor(sum.w, off);
            }
            if (p == 0 && co < a.Cout) *reinterpret_cast<floatx4 *>(a.out + (size_t)img * a.Cout + co) = sum * (1.0f / 64.0f);
        }
    }
}

template <int CG>
static hipError_t pooled_launch(const PoolCodeArgs &a, size_t lds_bytes, hipStream_t st)
{
    static bool lds_set = false;
    if (!lds_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pooled_codes_kernel<CG>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        lds_set = true;
    }
    hipLaunchKernelGGL((pooled_codes_kernel<CG>), dim3((unsigned)a.N), dim3(512), lds_bytes, st, a);
    return hipGetLastError();
}

bool pooled_codes_plan(int cin, int cout, int *cg, int *groups)
{
    const int ks = (cin + 31) / 32, tiles = (cout + 15) / 16;
    if (cin % 8 != 0 || cout % 4 != 0 || ks * 12288 > 160 * 1024) return false;
    *cg = tiles % 5 == 0 ? 5 : 2;
    *groups = (tiles + *cg - 1) / *cg;
    return true;
}

hipError_t launch_pooled_codes(const PoolCodeArgs &a, hipStream_t st)
{
    if (a.N == 0) return hipSuccess;
    int cg = 0, groups = 0;
    if (!pooled_codes_plan(a.Cin, a.Cout, &cg, &groups) || cg != a.CG || groups != a.groups || a.KS != (a.Cin + 31) / 32)
        return hipErrorInvalidValue;
    const size_t lds_bytes = (size_t)a.KS * 12288;
    return cg == 5 ? pooled_launch<5>(a, lds_bytes, st) : pooled_launch<2>(a, lds_bytes, st);
}

// ------------------------------------------------------------------ configurations
//
// One instantiation per block shape of MobileNetV2 for 32x32 inputs.  The split block input needs
// 6 bytes per value; it lives in registers as ready-made operands wherever a wavefront's share
// fits beside the accumulators, and in LDS for the last block (320 output channels).  Measured
// choices (2048 images, one launch, best of the tilings tried per shape): as for the fp32 kernel,
// several small workgroups per compute unit beat one large one with larger hidden chunks (at
// 32x32: 4 wavefronts x 2 workgroups 254 - 500 us against 330 - 660 us for 8 wavefronts with
// chunks of 32 - 48 channels); the stride-2 block at 32x32 does best with bands of 4 output rows.

namespace {

#ifndef AIQ_MC_TABLE
//                CIN  HID  COUT  H  S  RES    R  G  HC NW XREG WGS EPRE DPRE
typedef McCfg<16, 96, 24, 32, 1, false, 8, 1, 16, 4, true, 2, true, true> Mc0;
typedef McCfg<24, 144, 24, 32, 1, true, 8, 1, 16, 4, true, 2, true, true> Mc1;
typedef McCfg<24, 144, 32, 32, 1, false, 8, 1, 16, 4, true, 2, true, true> Mc2;
typedef McCfg<32, 192, 32, 32, 1, true, 8, 1, 16, 4, true, 2, true, true> Mc3;
typedef McCfg<32, 192, 64, 32, 2, false, 4, 1, 32, 4, true, 2, true, true> Mc4;
typedef McCfg<64, 384, 64, 16, 1, true, 16, 1, 16, 8, true, 1, true, true> Mc5;
typedef McCfg<64, 384, 96, 16, 1, false, 16, 1, 32, 8, true, 1, true, true> Mc6;
typedef McCfg<96, 576, 96, 16, 1, true, 16, 1, 16, 8, true, 1, false, true> Mc7;
typedef McCfg<96, 576, 160, 16, 2, false, 8, 1, 16, 8, true, 1, true, true> Mc8;
typedef McCfg<160, 960, 160, 8, 1, true, 8, 1, 16, 4, true, 2, true, true> Mc9;
typedef McCfg<160, 960, 320, 8, 1, false, 8, 1, 16, 4, false, 2, true, true> Mc10;
#else
AIQ_MC_TABLE
#endif

template <class C>
bool mc_matches(const MbShape &sh)
{
    return sh.cin == C::CIN && sh.hid == C::HID && sh.cout == C::COUT && sh.h == C::H && sh.stride == C::STRIDE &&
           (sh.res != 0) == C::RES;
}

template <class C, bool EC, bool PC>
hipError_t mc_launch_as(const MbCodeArgs &a, hipStream_t st)
{
    static bool lds_set = false;
    if (!lds_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&mbconv_codes_kernel<C, EC, PC>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        lds_set = true;
    }
    const unsigned gx = (unsigned)((a.N + C::G - 1) / C::G) * C::BANDS;
    hipLaunchKernelGGL((mbconv_codes_kernel<C, EC, PC>), dim3(gx), dim3(C::THREADS), C::LDS_BYTES, st, a);
    return hipGetLastError();
}

// a block with one fp32 layer needs the block input in registers
template <class C>
constexpr bool mc_mixed_ok() { return C::XREG; }

template <class C>
hipError_t mc_launch(const MbCodeArgs &a, hipStream_t st)
{
    const bool ec = a.codes_e != nullptr, pc = a.codes_p != nullptr;
    if (ec && pc) return mc_launch_as<C, true, true>(a, st);
    if constexpr (C::XREG) {
        if (ec) return mc_launch_as<C, true, false>(a, st);
        if (pc) return mc_launch_as<C, false, true>(a, st);
    }
    return hipErrorInvalidValue;
}

} // namespace

#define AIQ_MC_CONFIGS(F) F(Mc0) F(Mc1) F(Mc2) F(Mc3) F(Mc4) F(Mc5) F(Mc6) F(Mc7) F(Mc8) F(Mc9) F(Mc10)

bool mbconv_codes_supported(const MbShape &sh, bool expand_codes, bool project_codes)
{
    if (!expand_codes && !project_codes) return false;
#define AIQ_MC_MATCH(C) if (mc_matches<C>(sh)) return (expand_codes && project_codes) || mc_mixed_ok<C>();
    AIQ_MC_CONFIGS(AIQ_MC_MATCH)
#undef AIQ_MC_MATCH
    return false;
}

hipError_t launch_mbconv_codes(const MbShape &sh, const MbCodeArgs &a, hipStream_t st)
{
    if (a.N == 0) return hipSuccess;
#define AIQ_MC_LAUNCH(C) if (mc_matches<C>(sh)) return mc_launch<C>(a, st);
    AIQ_MC_CONFIGS(AIQ_MC_LAUNCH)
#undef AIQ_MC_LAUNCH
    return hipErrorInvalidValue;
}

} // namespace aiq
