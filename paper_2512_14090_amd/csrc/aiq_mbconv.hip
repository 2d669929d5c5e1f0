// Inverted-residual blocks (1x1 expand -> depthwise 3x3 -> 1x1 project, MobileNetV2) on
// gfx950 with the expanded tensor held in LDS: one workgroup computes a band of output rows
// of one (scheme, image) pair and only the narrow block input and output touch HBM.
//
// What is computed is the plain forward pass of the three layers, each with the weights of
// the bit-width its scheme entry names (paper: Problem Formulation; Introduction item (ii));
// only where the hidden activations live differs from the layer-by-layer kernels.
//
// The hidden channels are processed HC at a time.  Per chunk:
//   expand   X (block input rows incl. the halo) x W_e -> E (LDS), fp32 MFMA 16x16x4:
//            A = 16 hidden channels, B = 16 pixels; bias + activation; pixels outside the
//            image stay zero (they are the depthwise layer's zero padding).  Every wavefront
//            owns fixed pixel tiles of X for the whole kernel, so X is either held in its
//            registers as ready-made B operands (XREG) or staged once in LDS.
//   depthwise + project   lane (pixel p, kq) forms the depthwise output of its pixel for
//            hidden channels 16*hb + 4*kq .. +3 (nine 16-byte LDS reads, 36 FMAs) - exactly
//            the B operand of the project MFMAs for that 16-channel block - and accumulates
//            into the block output tile it owns.  The depthwise output never leaves registers.
//            A wavefront's tiles are vertically adjacent, so a window row read for one tile
//            also serves its neighbours (3 * (MT + 2) reads for MT tiles at stride 1).
// E is double buffered: chunk c+1 is expanded in the same barrier interval in which chunk c
// is consumed.  With X in registers E alone occupies LDS and two workgroups share a compute
// unit, so that one's barriers, prologue and epilogue are covered by the other's MFMAs.
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
    // one v_med3_f32 per element: the median of (v, lo, hi) is v clamped to [lo, hi]
    v.x = __builtin_amdgcn_fmed3f(v.x, lo, hi);
    v.y = __builtin_amdgcn_fmed3f(v.y, lo, hi);
    v.z = __builtin_amdgcn_fmed3f(v.z, lo, hi);
    v.w = __builtin_amdgcn_fmed3f(v.w, lo, hi);
    return v;
}
__device__ __forceinline__ float mb_lo(int act) { return act >= 1 ? 0.0f : -__builtin_inff(); }
__device__ __forceinline__ float mb_hi(int act) { return act == 2 ? 6.0f : __builtin_inff(); }

// Block shape (CIN, HID, COUT, H, STRIDE, RES) and tiling: R output rows per workgroup, G images
// per workgroup (whole images only), HC hidden channels per chunk, NW wavefronts per workgroup,
// XREG: block input in registers instead of LDS, WGS: workgroups meant to share a compute unit,
// EPRE: the expand weights of a chunk are fetched into registers one step ahead.
template <int CIN_, int HID_, int COUT_, int H_, int STRIDE_, bool RES_, int R_, int G_, int HC_, int NW_, bool XREG_,
          int WGS_, bool EPRE_>
struct MbCfg {
    static constexpr int CIN = CIN_, HID = HID_, COUT = COUT_, H = H_, STRIDE = STRIDE_, R = R_, G = G_, HC = HC_;
    static constexpr bool RES = RES_, XREG = XREG_, EPRE = EPRE_;
    static constexpr int NW = NW_, THREADS = NW_ * 64, WGS = WGS_;
    static constexpr int WAVES_PER_SIMD = NW * WGS / 4;
    static constexpr int W = H, HO = H / STRIDE, WO = HO;
    static constexpr int RI = (R - 1) * STRIDE + 3;  // E rows: input rows a band of R output rows needs
    static constexpr bool WHOLE = (R == HO);         // the band is the whole image: E row 0 is always padding
    static constexpr int XOFF = WHOLE ? 1 : 0;       // E row of X row 0
    static constexpr int XROWS = WHOLE ? H : RI;     // most rows of X a band can hold
    static constexpr int CB = (CIN + 15) / 16, XPLANES = CIN / 4;
    static constexpr int HT = HC / 16, HB = HID / 16, NCH = HID / HC;
    static constexpr int CT = (COUT + 15) / 16;
    static constexpr int EW = W + 1, EPIX = RI * EW + 1;
    static constexpr int XPL = G * XROWS * W * 4 + 4; // floats per X plane (+16 bytes: planes start in different banks)
    static constexpr int EPL = G * EPIX * 4;          // floats per E plane
    static constexpr int X_FLOATS = XREG ? 0 : XPLANES * XPL;
    static constexpr int E_FLOATS = (HC / 4) * EPL;
    static constexpr int LDS_BYTES = (X_FLOATS + 2 * E_FLOATS) * 4;
    // expand: pixel tiles of X (at most PTE of them), XT per wavefront; with fewer tiles than
    // wavefronts, HS wavefronts share a tile and split the chunk's hidden-channel tiles
    static constexpr int PTE = G * XROWS * W / 16;
    static constexpr int XT = PTE >= NW ? (PTE + NW - 1) / NW : 1;
    static constexpr int HS = PTE >= NW ? 1 : NW / PTE;
    static constexpr int HTW = HT / HS;
    // project: PTO output pixel tiles, MT per wavefront; with fewer tiles than wavefronts,
    // WPP wavefronts share a tile and split the output-channel tiles
    static constexpr int PTO = G * R * WO / 16;
    static constexpr int MT = PTO >= NW ? PTO / NW : 1;
    static constexpr int WPP = PTO >= NW ? 1 : NW / PTO;
    static constexpr int CTW = CT / WPP;
    static constexpr int BANDS = HO / R;
    static constexpr int TPR = WO >= 16 ? WO / 16 : 1;   // output pixel tiles per image row
    static constexpr int NRW = (MT - 1) * STRIDE + 3;    // depthwise window rows of a strip of MT tiles
    static_assert(CIN % 4 == 0 && HID % HC == 0 && HC % 16 == 0 && COUT % 4 == 0, "channel counts");
    static_assert(HO % R == 0 && (G == 1 || WHOLE), "bands tile the image; several images only as whole images");
    static_assert((G * XROWS * W) % 16 == 0 && (PTE >= NW || (NW % PTE == 0 && HT % HS == 0)), "expand tiles");
    static_assert(!WHOLE || PTE < NW || PTE % NW == 0, "whole images: every wavefront has all its expand tiles");
    static_assert((G * R * WO) % 16 == 0 && (PTO >= NW ? PTO % NW == 0 : NW % PTO == 0), "pixel tiles per wavefront");
    static_assert(CT % WPP == 0, "output-channel tiles per wavefront");
    static_assert(MT == 1 || (WO >= 16 && NW % TPR == 0 && G == 1), "strips of tiles need whole 16-pixel row segments");
    static_assert((W & (W - 1)) == 0 && ((R * WO) & (R * WO - 1)) == 0, "powers of two");
    static_assert(!RES || (CIN == COUT && STRIDE == 1), "residual needs matching shapes");
    static_assert(LDS_BYTES * WGS <= 160 * 1024, "LDS budget");
};

} // namespace

template <class C>
__global__ __launch_bounds__(C::THREADS) __attribute__((amdgpu_waves_per_eu(C::WAVES_PER_SIMD, C::WAVES_PER_SIMD)))
void mbconv_kernel(MbArgs a)
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
    const float *in_s = a.in + (size_t)s * a.in_scheme_stride;

    // valid E rows of this band: E row r holds image row iy0 + r
    const int iy0 = band * C::R * C::STRIDE - 1;
    const int r_lo = iy0 < 0 ? -iy0 : 0;
    const int r_hi = min(C::RI, C::H - iy0);
    const int nrows = r_hi - r_lo;
    const int n_exp_tiles = (C::G * nrows * C::W) >> 4;

    // ---- expand tiles of this wavefront: E offset of the lane's pixel, and X as B operands
    const int h0 = C::HS > 1 ? (wave % C::HS) * C::HTW : 0; // first hidden tile (within a chunk) of this wavefront
    bool x_ok[C::XT];
    int e_off[C::XT], x_off[C::XT];
    floatx4 xr[C::XREG ? C::XT : 1][C::XREG ? C::CB : 1];
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
        x_off[k] = ((g * C::XROWS + (r - C::XOFF)) * C::W + x) * 4;
        if (C::XREG) {
            const int img = img0 + g;
            const float *px = in_s + (((size_t)img * C::H + (iy0 + r)) * C::W + x) * C::CIN;
#pragma unroll
            for (int cb = 0; cb < C::CB; ++cb) {
                const int ch = cb * 16 + kq * 4;
                xr[k][cb] = (x_ok[k] && img < a.N && ch < C::CIN) ? mb_gload4(px + ch) : floatx4{0.f, 0.f, 0.f, 0.f};
            }
        }
    }

    // ---- clear E (borders and out-of-image rows stay zero for good); stage X unless it is in registers
    for (int i = tid; i < 2 * C::E_FLOATS / 4; i += C::THREADS)
        reinterpret_cast<floatx4 *>(E)[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (!C::XREG) {
        constexpr int C4 = C::CIN / 4;
        const int per_img = nrows * C::W * C4;
        for (int g = 0; g < C::G; ++g) {
            const int img = img0 + g;
            const float *src = in_s + (((size_t)img * C::H + (iy0 + r_lo)) * C::W) * C::CIN;
            constexpr int UN = 4;
            for (int base = tid; base < per_img; base += C::THREADS * UN) {
                floatx4 v[UN];
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int idx = base + u * C::THREADS;
                    v[u] = (idx < per_img && img < a.N) ? mb_gload4(src + (size_t)idx * 4) : floatx4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int idx = base + u * C::THREADS;
                    if (idx < per_img) {
                        const int c4 = idx % C4, pix = idx / C4; // pix = rr * W + x
                        const int xrow = r_lo - C::XOFF;         // X row of the first valid E row
                        *reinterpret_cast<floatx4 *>(X + c4 * C::XPL + ((g * C::XROWS + xrow) * C::W + pix) * 4) = v[u];
                    }
                }
            }
        }
    }

    const float lo_e = mb_lo(a.act_e), hi_e = mb_hi(a.act_e), lo_d = mb_lo(a.act_d), hi_d = mb_hi(a.act_d);

    // ---- output tiles of this wavefront
    const int ct0 = (C::WPP > 1 ? (wave % C::WPP) : 0) * C::CTW;
    int e_base[C::MT], o_g[C::MT], o_y[C::MT], o_x[C::MT];
#pragma unroll
    for (int m = 0; m < C::MT; ++m) {
        // a wavefront's MT tiles are vertically adjacent (a strip TPR-th of the width wide), so
        // that the depthwise window rows of one tile are shared with the tiles above and below
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

    // Weights of one expand step of this wavefront: bias and the A operands of its hidden tiles.
    // Where the registers allow it they are fetched one step ahead (EPRE), which hides their
    // L2 latency behind the consumption of the previous chunk (measured: 6-25 % per block);
    // otherwise they are read where they are used.
    constexpr bool EPRE = C::EPRE;
    struct ExpW {
        floatx4 be[C::HTW], wa[EPRE ? C::HTW : 1][EPRE ? C::CB : 1];
    };
    auto load_expw = [&](int c, ExpW &w) {
#pragma unroll
        for (int h = 0; h < C::HTW; ++h) w.be[h] = mb_gload4(a.bias_e + (c * C::HT + h0 + h) * 16 + kq * 4);
        if (EPRE) {
            const float *wc = w_e + ((size_t)(c * C::HT + h0) * C::CB * 64 + lane) * 4;
#pragma unroll
            for (int h = 0; h < C::HTW; ++h)
#pragma unroll
                for (int cb = 0; cb < C::CB; ++cb)
                    w.wa[EPRE ? h : 0][EPRE ? cb : 0] = mb_gload4(wc + (size_t)((h * C::CB + cb) * 64) * 4);
        }
    };
    // expand of hidden chunk c into E buffer eb
    auto expand = [&](int c, int eb, const ExpW &w) {
        float *Eb = E + eb * C::E_FLOATS + h0 * 4 * C::EPL;
        const float *wc = w_e + ((size_t)(c * C::HT + h0) * C::CB * 64 + lane) * 4;
#pragma unroll
        for (int k = 0; k < C::XT; ++k) {
            if (!C::WHOLE && !x_ok[k]) continue; // uniform per wavefront; whole images have every tile
            floatx4 ea[C::HTW];
#pragma unroll
            for (int h = 0; h < C::HTW; ++h) ea[h] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int cb = 0; cb < C::CB; ++cb) {
                floatx4 xb;
                if (C::XREG) {
                    xb = xr[C::XREG ? k : 0][C::XREG ? cb : 0];
                } else {
                    // channels past CIN (CIN not a multiple of 16) meet zero weights; read any valid plane
                    const int plane = min(cb * 4 + kq, C::XPLANES - 1);
                    xb = *reinterpret_cast<const floatx4 *>(X + plane * C::XPL + x_off[k]);
                }
                floatx4 wa[C::HTW];
#pragma unroll
                for (int h = 0; h < C::HTW; ++h)
                    wa[h] = EPRE ? w.wa[EPRE ? h : 0][EPRE ? cb : 0] : mb_gload4(wc + (size_t)((h * C::CB + cb) * 64) * 4);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int h = 0; h < C::HTW; ++h)
                        ea[h] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[h][j], xb[j], ea[h], 0, 0, 0);
            }
#pragma unroll
            for (int h = 0; h < C::HTW; ++h)
                *reinterpret_cast<floatx4 *>(Eb + h * 4 * C::EPL + e_off[k]) = mb_clamp4(ea[h] + w.be[h], lo_e, hi_e);
        }
    };

    // Weights of one 16-channel hidden block for the depthwise + project step.
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
        const float *Eb = E + eb * C::E_FLOATS + sb * 4 * C::EPL + e_base[0];
        // depthwise: window row r of tap column kx serves tap row ky of tile (r - ky) / STRIDE, so a
        // strip of MT tiles needs 3 * NRW reads instead of 9 * MT
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
            d[m] = mb_clamp4(d[m], lo_d, hi_d);
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < C::CTW; ++i)
                    acc[m][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(w.wp[i][j], d[m][j], acc[m][i], 0, 0, 0);
        }
    };
    // consumes chunk c; w0 arrives holding the weights of its first hidden block
    auto consume = [&](int c, int eb, DwW &w0) {
#pragma unroll
        for (int sb = 0; sb < C::HT; ++sb) {
            DwW w1;
            if (sb + 1 < C::HT) load_dww(c * C::HT + sb + 1, w1);
            dw_project(sb, eb, w0);
            if (sb + 1 < C::HT) w0 = w1;
        }
    };

    // Inside a barrier interval chunk c is consumed and chunk c+1 expanded; the two are
    // independent.  Each step's weights are fetched while the other step runs: the expand
    // weights before the consumption, the next chunk's depthwise / project weights (into the
    // registers the consumption has just finished with) before the expansion.
    DwW w0;
    ExpW ew;
    load_dww(0, w0);
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
            load_dww((c + 1) * C::HT, w0);
            expand(c + 1, eb ^ 1, ew);
        }
        __syncthreads();
    }

    // ---- epilogue: bias, residual (the block input), activation, 16-byte NHWC stores
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
            const int oy = band * C::R + o_y[m];
            const size_t o = (((size_t)img * C::HO + oy) * C::WO + o_x[m]) * C::COUT + co;
            floatx4 v = acc[m][i] + bp;
            if (C::RES) {
                if (C::XREG) {
                    v += mb_gload4(in_s + o); // same shape as the output
                } else {
                    const int xrow = o_y[m] + 1 - C::XOFF;
                    v += *reinterpret_cast<const floatx4 *>(X + (co >> 2) * C::XPL +
                                                            ((o_g[m] * C::XROWS + xrow) * C::W + o_x[m]) * 4);
                }
            }
            *reinterpret_cast<floatx4 *>(out_s + o) = mb_clamp4(v, lo_p, hi_p);
        }
    }
}

// ------------------------------------------------------------------ configurations
//
// One instantiation per block shape of MobileNetV2 for 32x32 inputs.  Measured choices: at
// 32x32 pixels small workgroups (4 wavefronts, X in registers, 2-3 workgroups per compute
// unit) beat one large one by 20-40 % - independent barrier domains keep the matrix pipe fed;
// at 16x16 and 8x8 the input has too many channels for registers and one workgroup of 8
// wavefronts with X in LDS does best.  The hidden chunk HC is the largest whose expand weights
// still fit in registers one step ahead (the last block's do not at any chunk size).

namespace {

#ifndef AIQ_MB_TABLE
//                CIN  HID  COUT  H  S  RES    R  G  HC NW XREG WGS EPRE
typedef MbCfg<16, 96, 24, 32, 1, false, 8, 1, 16, 4, true, 3, true> Mb0;
typedef MbCfg<24, 144, 24, 32, 1, true, 8, 1, 16, 4, true, 2, false> Mb1;
typedef MbCfg<24, 144, 32, 32, 1, false, 8, 1, 16, 4, true, 2, false> Mb2;
typedef MbCfg<32, 192, 32, 32, 1, true, 8, 1, 16, 4, true, 2, true> Mb3;
typedef MbCfg<32, 192, 64, 32, 2, false, 8, 1, 16, 4, true, 2, true> Mb4;
typedef MbCfg<64, 384, 64, 16, 1, true, 16, 1, 32, 8, false, 1, true> Mb5;
typedef MbCfg<64, 384, 96, 16, 1, false, 16, 1, 32, 8, false, 1, true> Mb6;
typedef MbCfg<96, 576, 96, 16, 1, true, 16, 1, 16, 8, false, 1, true> Mb7;
typedef MbCfg<96, 576, 160, 16, 2, false, 8, 1, 16, 8, false, 1, true> Mb8;
typedef MbCfg<160, 960, 160, 8, 1, true, 8, 2, 16, 8, false, 1, true> Mb9;
typedef MbCfg<160, 960, 320, 8, 1, false, 8, 1, 64, 8, false, 1, false> Mb10;
#else
AIQ_MB_TABLE
#endif

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
    hipLaunchKernelGGL((mbconv_kernel<C>), dim3(gx, s_total), dim3(C::THREADS), C::LDS_BYTES, st, a);
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
