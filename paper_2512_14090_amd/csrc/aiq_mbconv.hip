// Inverted-residual blocks (1x1 expand -> depthwise 3x3 -> 1x1 project, MobileNetV2) on
// gfx950 with the expanded tensor held in LDS: one workgroup computes a band of output rows
// of one (scheme, image) pair and only the narrow block input and output touch HBM.
//
// What is computed is the plain forward pass of the three layers, each with the weights of
// the bit-width its scheme entry names (paper: Problem Formulation; Introduction item (ii));
// only where the hidden activations live differs from the layer-by-layer kernels.
//
// The hidden channels are processed HC at a time.  Per chunk:
//   expand   X (LDS, block input rows incl. the halo) x W_e -> E (LDS), fp32 MFMA 16x16x4:
//            A = 16 hidden channels, B = 16 pixels; bias + activation; pixels outside the
//            image stay zero (they are the depthwise layer's zero padding).
//   depthwise + project   lane (pixel p, kq) forms the depthwise output of its pixel for
//            hidden channels 16*hb + 4*kq .. +3 (nine 16-byte LDS reads, 36 FMAs) - exactly
//            the B operand of the project MFMAs for that 16-channel block - and accumulates
//            into the block output tile it owns.  The depthwise output never leaves registers.
// E is double buffered: chunk c+1 is expanded in the same barrier interval in which chunk c
// is consumed.
//
// LDS layouts.  X: CIN/4 planes of [image][row][column] pixels x 4 floats.  E (one buffer):
// HC/4 planes; pixel (row r, column x), x in [-1, W], sits at r*(W+1) + x + 1, so that the
// right border of a row and the left border of the next share one zero pixel.
#include "aiq_internal.h"

namespace aiq {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ floatx4 mb_gload4(const float *p)
{
    return *(const __attribute__((address_space(1))) floatx4 *)(p);
}
__device__ __forceinline__ floatx4 mb_clamp4(floatx4 v, float lo, float hi)
{
    v.x = fminf(fmaxf(v.x, lo), hi);
    v.y = fminf(fmaxf(v.y, lo), hi);
    v.z = fminf(fmaxf(v.z, lo), hi);
    v.w = fminf(fmaxf(v.w, lo), hi);
    return v;
}
__device__ __forceinline__ float mb_lo(int act) { return act >= 1 ? 0.0f : -__builtin_inff(); }
__device__ __forceinline__ float mb_hi(int act) { return act == 2 ? 6.0f : __builtin_inff(); }

template <int CIN_, int HID_, int COUT_, int H_, int STRIDE_, bool RES_, int R_, int G_, int HC_>
struct MbCfg {
    static constexpr int CIN = CIN_, HID = HID_, COUT = COUT_, H = H_, STRIDE = STRIDE_, R = R_, G = G_, HC = HC_;
    static constexpr bool RES = RES_;
    static constexpr int NW = kMbThreads / 64;
    static constexpr int W = H, HO = H / STRIDE, WO = HO;
    static constexpr int RI = (R - 1) * STRIDE + 3;  // E rows: input rows a band of R output rows needs
    static constexpr bool WHOLE = (R == HO);         // the band is the whole image: E row 0 is always padding
    static constexpr int XOFF = WHOLE ? 1 : 0;       // E row of X row 0
    static constexpr int XROWS = WHOLE ? H : RI;
    static constexpr int CB = (CIN + 15) / 16, XPLANES = CIN / 4;
    static constexpr int HT = HC / 16, HB = HID / 16, NCH = HID / HC;
    static constexpr int CT = (COUT + 15) / 16;
    static constexpr int EW = W + 1, EPIX = RI * EW + 1;
    static constexpr int XPL = G * XROWS * W * 4 + 4; // floats per X plane (+16 bytes: planes start in different banks)
    static constexpr int EPL = G * EPIX * 4;          // floats per E plane
    static constexpr int X_FLOATS = XPLANES * XPL;
    static constexpr int E_FLOATS = (HC / 4) * EPL;
    static constexpr int LDS_BYTES = (X_FLOATS + 2 * E_FLOATS) * 4;
    static constexpr int PTO = G * R * WO / 16;       // output pixel tiles of the workgroup
    static constexpr int MT = PTO >= NW ? PTO / NW : 1;  // pixel tiles per wavefront
    static constexpr int WPP = PTO >= NW ? 1 : NW / PTO; // wavefronts sharing a pixel tile (they split the output channels)
    static constexpr int CTW = CT / WPP;
    static constexpr int BANDS = HO / R;
    static_assert(CIN % 4 == 0 && HID % HC == 0 && HC % 16 == 0 && COUT % 4 == 0, "channel counts");
    static_assert(HO % R == 0 && (G == 1 || WHOLE), "bands tile the image; several images only as whole images");
    static_assert((G * R * WO) % 16 == 0 && (PTO >= NW ? PTO % NW == 0 : NW % PTO == 0), "pixel tiles per wavefront");
    static_assert(CT % WPP == 0, "output-channel tiles per wavefront");
    static_assert((W & (W - 1)) == 0 && ((R * WO) & (R * WO - 1)) == 0, "powers of two");
    static_assert(!RES || (CIN == COUT && STRIDE == 1), "residual needs matching shapes");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

} // namespace

template <class C>
__global__ __launch_bounds__(kMbThreads) void mbconv_kernel(MbArgs a)
{
    extern __shared__ float lds[];
    float *X = lds;
    float *E = lds + C::X_FLOATS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, p = lane & 15, kq = lane >> 4;
    const int s = blockIdx.y;
    const int band = blockIdx.x % C::BANDS;
    const int img0 = (blockIdx.x / C::BANDS) * C::G;

    int bi_e = 0, bi_d = 0, bi_p = 0;
    if (s < a.S) {
        const uint8_t *q = a.schemes + (size_t)s * a.L;
        if (a.slot_e >= 0) bi_e = bits_index(q[a.slot_e]);
        if (a.slot_d >= 0) bi_d = bits_index(q[a.slot_d]);
        if (a.slot_p >= 0) bi_p = bits_index(q[a.slot_p]);
    }
    const float *w_e = a.bank_e[bi_e], *w_d = a.bank_d[bi_d], *w_p = a.bank_p[bi_p];

    // valid E rows of this band: E row r holds image row iy0 + r
    const int iy0 = band * C::R * C::STRIDE - 1;
    const int r_lo = iy0 < 0 ? -iy0 : 0;
    const int r_hi = min(C::RI, C::H - iy0);
    const int nrows = r_hi - r_lo;

    // ---- clear E (borders and out-of-image rows stay zero for good), load the X tile
    for (int i = tid; i < 2 * C::E_FLOATS / 4; i += kMbThreads)
        reinterpret_cast<floatx4 *>(E)[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    {
        const float *in_s = a.in + (size_t)s * a.in_scheme_stride;
        constexpr int C4 = C::CIN / 4;
        const int per_img = nrows * C::W * C4;
        for (int g = 0; g < C::G; ++g) {
            const int img = img0 + g;
            const float *src = in_s + (((size_t)img * C::H + (iy0 + r_lo)) * C::W) * C::CIN;
            constexpr int UN = 4;
            for (int base = tid; base < per_img; base += kMbThreads * UN) {
                floatx4 v[UN];
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int idx = base + u * kMbThreads;
                    v[u] = (idx < per_img && img < a.N) ? mb_gload4(src + (size_t)idx * 4) : floatx4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int idx = base + u * kMbThreads;
                    if (idx < per_img) {
                        const int c4 = idx % C4, pix = idx / C4; // pix = rr * W + x
                        const int xr = r_lo - C::XOFF;           // X row of the first valid E row
                        *reinterpret_cast<floatx4 *>(X + c4 * C::XPL + ((g * C::XROWS + xr) * C::W + pix) * 4) = v[u];
                    }
                }
            }
        }
    }

    // ---- per-lane constants
    const float lo_e = mb_lo(a.act_e), hi_e = mb_hi(a.act_e), lo_d = mb_lo(a.act_d), hi_d = mb_hi(a.act_d);
    const int n_exp_tiles = (C::G * nrows * C::W) >> 4;

    // output tiles of this wavefront
    const int ct0 = (C::WPP > 1 ? (wave % C::WPP) : 0) * C::CTW;
    int e_base[C::MT], o_g[C::MT], o_y[C::MT], o_x[C::MT];
#pragma unroll
    for (int m = 0; m < C::MT; ++m) {
        const int t = C::WPP > 1 ? wave / C::WPP : wave * C::MT + m;
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

    // expand of hidden chunk c into E buffer eb
    auto expand = [&](int c, int eb) {
        float *Eb = E + eb * C::E_FLOATS;
        floatx4 be[C::HT];
#pragma unroll
        for (int h = 0; h < C::HT; ++h) be[h] = mb_gload4(a.bias_e + (c * C::HT + h) * 16 + kq * 4);
        const float *wc = w_e + ((size_t)c * C::HT * C::CB * 64 + lane) * 4;
#pragma unroll 1
        for (int e = wave; e < n_exp_tiles; e += C::NW) {
            const int f = e * 16 + p;
            int g = 0, rem = f;
            if (C::G > 1) {
                g = f / (C::H * C::W); // several images only as whole images: nrows == H
                rem = f % (C::H * C::W);
            }
            const int rr = rem / C::W, x = rem % C::W;
            const int r = r_lo + rr;
            const int x_off = ((g * C::XROWS + (r - C::XOFF)) * C::W + x) * 4;
            floatx4 ea[C::HT];
#pragma unroll
            for (int h = 0; h < C::HT; ++h) ea[h] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int cb = 0; cb < C::CB; ++cb) {
                // channels past CIN (CIN not a multiple of 16) meet zero weights; read any valid plane
                const int plane = min(cb * 4 + kq, C::XPLANES - 1);
                const floatx4 xb = *reinterpret_cast<const floatx4 *>(X + plane * C::XPL + x_off);
                floatx4 wa[C::HT];
#pragma unroll
                for (int h = 0; h < C::HT; ++h) wa[h] = mb_gload4(wc + (size_t)((h * C::CB + cb) * 64) * 4);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int h = 0; h < C::HT; ++h)
                        ea[h] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[h][j], xb[j], ea[h], 0, 0, 0);
            }
            const int e_off = (g * C::EPIX + r * C::EW + x + 1) * 4;
#pragma unroll
            for (int h = 0; h < C::HT; ++h)
                *reinterpret_cast<floatx4 *>(Eb + (h * 4 + kq) * C::EPL + e_off) = mb_clamp4(ea[h] + be[h], lo_e, hi_e);
        }
    };

    struct DwW {
        floatx4 wd[9], bd, wp[C::CTW];
    };
    auto load_dww = [&](int hb, DwW &w) {
#pragma unroll
        for (int t = 0; t < 9; ++t) w.wd[t] = mb_gload4(w_d + (size_t)t * C::HID + hb * 16 + kq * 4);
        w.bd = mb_gload4(a.bias_d + hb * 16 + kq * 4);
#pragma unroll
        for (int i = 0; i < C::CTW; ++i)
            w.wp[i] = mb_gload4(w_p + (((size_t)(ct0 + i) * C::HB + hb) * 64 + lane) * 4);
    };
    auto dw_project = [&](int sb, int eb, const DwW &w) {
        const float *Eb = E + eb * C::E_FLOATS + sb * 4 * C::EPL;
#pragma unroll
        for (int m = 0; m < C::MT; ++m) {
            floatx4 d = w.bd;
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const floatx4 v = *reinterpret_cast<const floatx4 *>(Eb + e_base[m] + ((t / 3) * C::EW + (t % 3)) * 4);
                d += v * w.wd[t];
            }
            d = mb_clamp4(d, lo_d, hi_d);
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < C::CTW; ++i)
                    acc[m][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(w.wp[i][j], d[j], acc[m][i], 0, 0, 0);
        }
    };

    __syncthreads();
    expand(0, 0);
    __syncthreads();
#pragma unroll 1
    for (int c = 0; c < C::NCH; ++c) {
        const int eb = c & 1;
        DwW w0;
        load_dww(c * C::HT, w0);
        if (c + 1 < C::NCH) expand(c + 1, eb ^ 1);
#pragma unroll
        for (int sb = 0; sb < C::HT; ++sb) {
            DwW w1;
            if (sb + 1 < C::HT) load_dww(c * C::HT + sb + 1, w1);
            dw_project(sb, eb, w0);
            if (sb + 1 < C::HT) w0 = w1;
        }
        __syncthreads();
    }

    // ---- epilogue: bias, residual (the block input, still in X), activation, 16-byte NHWC stores
    const float lo_p = mb_lo(a.act_p), hi_p = mb_hi(a.act_p);
    float *out_s = a.out + (size_t)s * a.out_scheme_stride;
#pragma unroll
    for (int i = 0; i < C::CTW; ++i) {
        const int co = (ct0 + i) * 16 + kq * 4;
        if (co >= C::COUT) continue;
        const floatx4 bp = mb_gload4(a.bias_p + co);
#pragma unroll
        for (int m = 0; m < C::MT; ++m) {
            const int img = img0 + o_g[m];
            if (img >= a.N) continue;
            floatx4 v = acc[m][i] + bp;
            if (C::RES) {
                const int xr = o_y[m] + 1 - C::XOFF;
                v += *reinterpret_cast<const floatx4 *>(X + (co >> 2) * C::XPL +
                                                        ((o_g[m] * C::XROWS + xr) * C::W + o_x[m]) * 4);
            }
            v = mb_clamp4(v, lo_p, hi_p);
            const int oy = band * C::R + o_y[m];
            *reinterpret_cast<floatx4 *>(out_s + (((size_t)img * C::HO + oy) * C::WO + o_x[m]) * C::COUT + co) = v;
        }
    }
}

// ------------------------------------------------------------------ configurations
//
// One instantiation per block shape of MobileNetV2 for 32x32 inputs; band height R, images
// per workgroup G and hidden chunk HC are chosen so that X plus two E buffers fill most of
// the 160 KB of LDS (longer barrier intervals, less halo recomputation).

namespace {

//                CIN  HID  COUT  H  S  RES    R  G  HC
typedef MbCfg<16, 96, 24, 32, 1, false, 8, 1, 48> Mb0;
typedef MbCfg<24, 144, 24, 32, 1, true, 8, 1, 48> Mb1;
typedef MbCfg<24, 144, 32, 32, 1, false, 8, 1, 48> Mb2;
typedef MbCfg<32, 192, 32, 32, 1, true, 8, 1, 32> Mb3;
typedef MbCfg<32, 192, 64, 32, 2, false, 4, 1, 48> Mb4;
typedef MbCfg<64, 384, 64, 16, 1, true, 16, 1, 32> Mb5;
typedef MbCfg<64, 384, 96, 16, 1, false, 16, 1, 32> Mb6;
typedef MbCfg<96, 576, 96, 16, 1, true, 16, 1, 16> Mb7;
typedef MbCfg<96, 576, 160, 16, 2, false, 8, 1, 16> Mb8;
typedef MbCfg<160, 960, 160, 8, 1, true, 8, 2, 32> Mb9;
typedef MbCfg<160, 960, 320, 8, 1, false, 8, 1, 64> Mb10;

template <class C>
bool mb_matches(const MbShape &sh)
{
    return sh.cin == C::CIN && sh.hid == C::HID && sh.cout == C::COUT && sh.h == C::H && sh.stride == C::STRIDE &&
           (sh.res != 0) == C::RES;
}

template <class C>
hipError_t mb_launch(const MbArgs &a, int s_total, hipStream_t st)
{
    static bool lds_set = false;
    if (!lds_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&mbconv_kernel<C>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        lds_set = true;
    }
    const unsigned gx = (unsigned)((a.N + C::G - 1) / C::G) * C::BANDS;
    hipLaunchKernelGGL((mbconv_kernel<C>), dim3(gx, s_total), dim3(kMbThreads), C::LDS_BYTES, st, a);
    return hipGetLastError();
}

} // namespace

#define AIQ_MB_CONFIGS(F) F(Mb0) F(Mb1) F(Mb2) F(Mb3) F(Mb4) F(Mb5) F(Mb6) F(Mb7) F(Mb8) F(Mb9) F(Mb10)

bool mbconv_supported(const MbShape &sh)
{
#define AIQ_MB_MATCH(C) if (mb_matches<C>(sh)) return true;
    AIQ_MB_CONFIGS(AIQ_MB_MATCH)
#undef AIQ_MB_MATCH
    return false;
}

hipError_t launch_mbconv(const MbShape &sh, const MbArgs &a, int s_total, hipStream_t st)
{
    if (a.N == 0 || s_total == 0) return hipSuccess;
#define AIQ_MB_LAUNCH(C) if (mb_matches<C>(sh)) return mb_launch<C>(a, s_total, st);
    AIQ_MB_CONFIGS(AIQ_MB_LAUNCH)
#undef AIQ_MB_LAUNCH
    return hipErrorInvalidValue;
}

} // namespace aiq
