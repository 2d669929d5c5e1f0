// TEST INFRASTRUCTURE ONLY (never part of libaiq.so): stand-ins that let the host side of the library -
// argument validation, graph planning, workspace layout, launch sequencing (aiq_host.cpp) - run on a CPU
// under AddressSanitizer / UndefinedBehaviorSanitizer.
//
// "Device" memory is host memory, so every pointer the planner derives can be checked: each launcher
// stand-in touches the first and the last element of every region its kernel would read or write, for
// every scheme of the launch.  A workspace layout that is too small, a stride or an offset that is
// wrong, or a launch extent that runs past a buffer shows up as a sanitizer report.  Nothing of the
// scored method is computed here (small outputs are filled with zeros, activation tensors only touched).
#include "../../paper_2512_14090_amd/csrc/aiq_internal.h"

#include <cstdlib>
#include <cstring>

namespace {

volatile float g_sink;
long g_launches = 0;

template <typename T>
void touch_read(const T *p, size_t n)
{
    if (!p || n == 0) return;
    const volatile unsigned char *b = reinterpret_cast<const volatile unsigned char *>(p);
    g_sink = g_sink + (float)b[0] + (float)b[n * sizeof(T) - 1];
}
template <typename T>
void touch_write(T *p, size_t n)
{
    if (!p || n == 0) return;
    p[0] = T(0);
    p[n - 1] = T(0);
}
template <typename T>
void fill_zero(T *p, size_t n)
{
    if (p && n) std::memset(p, 0, n * sizeof(T));
}

int out_dim(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

} // namespace

extern "C" long aiq_stub_launch_count() { return g_launches; }

// ---------------------------------------------------------------- HIP runtime stand-ins
extern "C" {
hipError_t hipMalloc(void **p, size_t n)
{
    *p = std::malloc(n ? n : 1); // exact size: the sanitizer's red zones sit right behind it
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void *p)
{
    std::free(p);
    return hipSuccess;
}
hipError_t hipMemcpy(void *d, const void *s, size_t n, hipMemcpyKind)
{
    std::memcpy(d, s, n);
    return hipSuccess;
}
hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, hipMemcpyKind, hipStream_t)
{
    std::memcpy(d, s, n);
    return hipSuccess;
}
hipError_t hipMemset(void *d, int v, size_t n)
{
    std::memset(d, v, n);
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipDeviceSynchronize(void) { return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t *e)
{
    *e = reinterpret_cast<hipEvent_t>(std::malloc(8));
    return hipSuccess;
}
hipError_t hipEventDestroy(hipEvent_t e)
{
    std::free(e);
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t)
{
    *ms = 1.0f;
    return hipSuccess;
}
}

// ---------------------------------------------------------------- launcher stand-ins
namespace aiq {

hipError_t conv_set_lds_limits() { return hipSuccess; }
hipError_t fused_set_lds_limit() { return hipSuccess; }
hipError_t conv_codes_set_lds_limits() { return hipSuccess; }

hipError_t launch_fill_i32(int32_t *p, int32_t v, size_t n, hipStream_t)
{
    ++g_launches;
    for (size_t i = 0; i < n; ++i) p[i] = v;
    return hipSuccess;
}

hipError_t upload_bytes(void *dst, const void *src, size_t n, hipStream_t)
{
    ++g_launches;
    std::memcpy(dst, src, n);
    return hipSuccess;
}

hipError_t noalloc_scratch(void **ptr, size_t *bytes)
{
    static void *p = std::malloc(2u << 20);
    *ptr = p;
    *bytes = 2u << 20;
    return hipSuccess;
}

static size_t job_out_elems(const QuantJob &j)
{
    switch (j.layout) {
    case kLayoutPlain:
    case kLayoutTapMajor: return (size_t)j.cout * j.k;
    case kLayoutStem: return (size_t)((j.cout + 15) / 16) * j.taps * 64;
    default: return (size_t)((j.cout + 15) / 16) * 16 * j.taps * j.cblocks * 16;
    }
}

hipError_t launch_quantize_single(const QuantJob &j, hipStream_t)
{
    ++g_launches;
    touch_read(j.w, (size_t)j.cout * j.k);
    fill_zero(j.out, job_out_elems(j));
    fill_zero(j.scales, (size_t)j.cout);
    if (j.bits != 32) fill_zero(j.codes, (size_t)j.cout * j.k);
    if (j.tensor_amax) touch_read(j.tensor_amax, 1);
    return hipSuccess;
}

hipError_t launch_tensor_absmax(const float *w, size_t n, uint32_t *out, hipStream_t)
{
    ++g_launches;
    touch_read(w, n);
    *out = 0x3f800000u;
    return hipSuccess;
}

hipError_t launch_quantize_batch(const QuantJob *jobs, const int32_t *block_job, int n_blocks, const QuantMask &mask,
                                 hipStream_t st)
{
    ++g_launches;
    int last = -1;
    for (int b = 0; b < n_blocks; ++b) {
        const int ji = block_job[b];
        if (ji == last) continue;
        last = ji;
        if (ji < 0 || ji >= kMaxQuantJobs) return hipErrorInvalidValue;
        if (!((mask.word[ji >> 6] >> (ji & 63)) & 1ull)) continue;
        if (jobs[ji].first_block != b) return hipErrorInvalidValue;
        (void)launch_quantize_single(jobs[ji], st);
    }
    return hipSuccess;
}

static void touch_schemes(const uint8_t *schemes, int S, int L)
{
    if (S > 0) touch_read(schemes, (size_t)S * L);
}

hipError_t launch_conv(const ConvArgs &a, int ks, int stride, int nt, size_t lds_bytes, dim3 grid, hipStream_t)
{
    ++g_launches;
    if (lds_bytes > 160 * 1024 || nt < 1 || nt > 4 || grid.x == 0 || grid.y == 0) return hipErrorInvalidValue;
    if (out_dim(a.Hin, ks, stride, ks == 3 ? 1 : 0) != a.Hout) return hipErrorInvalidValue;
    touch_schemes(a.schemes, a.S, a.L);
    touch_read(a.bias, (size_t)a.Cout);
    for (unsigned s = 0; s < grid.z; ++s) {
        touch_read(a.in + s * a.in_scheme_stride, (size_t)a.N * a.Hin * a.Win * a.Cin);
        touch_write(a.out + s * a.out_scheme_stride, (size_t)a.N * a.Hout * a.Wout * a.Cout);
        if (a.res) touch_read(a.res + s * a.res_scheme_stride, (size_t)a.N * a.Hout * a.Wout * a.Cout);
    }
    for (int b = 0; b < kNumBits; ++b) touch_read(a.bank[b], (size_t)a.cout_tiles * 16 * ks * ks * a.CB * 16);
    return hipSuccess;
}

hipError_t launch_conv_stem(const ConvArgs &a, int nt, dim3 grid, hipStream_t)
{
    ++g_launches;
    if (a.Cin > 4 || a.res || nt < 1 || nt > 4) return hipErrorInvalidValue;
    touch_schemes(a.schemes, a.S, a.L);
    for (unsigned s = 0; s < grid.z; ++s) {
        touch_read(a.in + s * a.in_scheme_stride, (size_t)a.N * a.Hin * a.Win * a.Cin);
        touch_write(a.out + s * a.out_scheme_stride, (size_t)a.N * a.Hout * a.Wout * a.Cout);
    }
    for (int b = 0; b < kNumBits; ++b) touch_read(a.bank[b], (size_t)a.cout_tiles * 9 * 64);
    return hipSuccess;
}

hipError_t launch_pointwise(const PointwiseArgs &a, int nt, size_t lds_bytes, dim3 grid, hipStream_t)
{
    ++g_launches;
    if (lds_bytes > 160 * 1024 || nt < 1 || nt > 4 || (int)grid.y != a.grid_y) return hipErrorInvalidValue;
    touch_schemes(a.schemes, a.S, a.L);
    const size_t out_per = a.pool ? (size_t)(a.P / 64) * a.Cout : (size_t)a.P * a.Cout;
    for (unsigned s = 0; s < grid.z; ++s) {
        touch_read(a.in + s * a.in_scheme_stride, (size_t)a.P * a.Cin);
        touch_write(a.out + s * a.out_scheme_stride, out_per);
        if (a.res) touch_read(a.res + s * a.res_scheme_stride, (size_t)a.P * a.Cout);
    }
    for (int b = 0; b < kNumBits; ++b) touch_read(a.bank[b], (size_t)a.cout_tiles * 16 * a.CB * 16);
    return hipSuccess;
}

hipError_t launch_depthwise(const DepthwiseArgs &a, int s_total, hipStream_t)
{
    ++g_launches;
    touch_schemes(a.schemes, a.S, a.L);
    for (int s = 0; s < s_total; ++s) {
        touch_read(a.in + s * a.in_scheme_stride, (size_t)a.N * a.Hin * a.Win * a.C);
        touch_write(a.out + s * a.out_scheme_stride, (size_t)a.N * a.Hout * a.Wout * a.C);
    }
    for (int b = 0; b < kNumBits; ++b) touch_read(a.bank[b], (size_t)9 * a.C);
    return hipSuccess;
}

hipError_t launch_head(const HeadArgs &a, int s_total, hipStream_t)
{
    ++g_launches;
    touch_schemes(a.schemes, a.S, a.L);
    for (int s = 0; s < s_total; ++s) {
        touch_read(a.in + s * a.in_scheme_stride, (size_t)a.N * a.HW * a.C);
        const int row = a.row_map ? a.row_map[s] : (s < a.S ? s : -1);
        if (row >= 0) {
            fill_zero(a.top1 + (size_t)row * a.top1_stride, (size_t)a.N);
            if (a.logits) fill_zero(a.logits + ((size_t)row * a.logits_n + a.n0) * a.classes, (size_t)a.N * a.classes);
        } else if (a.top1_base) {
            fill_zero(a.top1_base, (size_t)a.N);
        }
    }
    for (int b = 0; b < kNumBits; ++b) touch_read(a.bank[b], (size_t)a.classes * a.C);
    return hipSuccess;
}

hipError_t launch_act_quantize(const ActQuantArgs &a, int s_total, hipStream_t)
{
    ++g_launches;
    touch_schemes(a.schemes, a.S, a.L);
    for (int s = 0; s < s_total; ++s) {
        touch_read(a.in + s * a.in_scheme_stride, (size_t)a.N * a.elems);
        touch_write(a.out + s * a.out_scheme_stride, (size_t)a.N * a.elems);
    }
    return hipSuccess;
}

hipError_t launch_agree(const AgreeArgs &a, hipStream_t)
{
    ++g_launches;
    for (int s = 0; s < a.S; ++s) {
        touch_read(a.top1 + (size_t)s * a.top1_stride, (size_t)a.N);
        a.agree[s] += a.N;
    }
    touch_read(a.top1_base, (size_t)a.N);
    return hipSuccess;
}

hipError_t launch_fused(const FusedArgs &a, int s_total, FusedMode mode, hipStream_t)
{
    ++g_launches;
    if (mode != kFusedPlain && !a.ckpt) return hipErrorInvalidValue;
    if (mode == kFusedResume && !a.first_op) return hipErrorInvalidValue;
    touch_read(a.ops, (size_t)a.n_ops);
    touch_read(a.images, (size_t)a.N * 3072);
    touch_schemes(a.schemes, a.S, a.L);
    const int classes = a.ops[a.n_ops - 1].classes;
    if (mode == kFusedResume) touch_read(a.first_op, (size_t)a.S);
    for (int s = 0; s < s_total; ++s) {
        if (s < a.S) {
            fill_zero(a.top1 + (size_t)s * a.top1_stride, (size_t)a.N);
            if (a.logits) fill_zero(a.logits + ((size_t)s * a.logits_n + a.n0) * classes, (size_t)a.N * classes);
            if (mode == kFusedResume && a.first_op[s] > 0) {
                const FusedOp &op = a.ops[a.first_op[s]];
                for (int n = 0; n < a.N; n += (a.N > 1 ? a.N - 1 : 1))
                    touch_read(a.ckpt + (size_t)n * a.ckpt_stride + op.ck_off, (size_t)op.ck_ext[0] + op.ck_ext[1]);
            }
        } else if (a.top1_base) {
            fill_zero(a.top1_base, (size_t)a.N);
        }
    }
    if (mode == kFusedReference)
        for (int o = 1; o < a.n_ops; ++o)
            if ((a.ck_mask[o >> 6] >> (o & 63)) & 1ull)
                for (int n = 0; n < a.N; n += (a.N > 1 ? a.N - 1 : 1))
                    touch_write(a.ckpt + (size_t)n * a.ckpt_stride + a.ops[o].ck_off,
                                (size_t)a.ops[o].ck_ext[0] + a.ops[o].ck_ext[1]);
    return hipSuccess;
}

// the block shapes the LDS-resident block kernel is instantiated for (shapes only)
bool mbconv_supported(const MbShape &sh)
{
    static const int t[][6] = {{16, 96, 24, 32, 1, 0},   {24, 144, 24, 32, 1, 1},  {24, 144, 32, 32, 1, 0},
                               {32, 192, 32, 32, 1, 1},  {32, 192, 64, 32, 2, 0},  {64, 384, 64, 16, 1, 1},
                               {64, 384, 96, 16, 1, 0},  {96, 576, 96, 16, 1, 1},  {96, 576, 160, 16, 2, 0},
                               {160, 960, 160, 8, 1, 1}, {160, 960, 320, 8, 1, 0}};
    for (const auto &r : t)
        if (sh.cin == r[0] && sh.hid == r[1] && sh.cout == r[2] && sh.h == r[3] && sh.stride == r[4] && (sh.res != 0) == (r[5] != 0))
            return true;
    return false;
}

hipError_t launch_mbconv(const MbShape &sh, const MbArgs &a, int s_total, hipStream_t)
{
    ++g_launches;
    if (!mbconv_supported(sh)) return hipErrorInvalidValue;
    touch_schemes(a.schemes, a.S, a.L);
    const int ho = sh.h / sh.stride;
    for (int s = 0; s < s_total; ++s) {
        touch_read(a.in + s * a.in_scheme_stride, (size_t)a.N * sh.h * sh.h * sh.cin);
        touch_write(a.out + s * a.out_scheme_stride, (size_t)a.N * ho * ho * sh.cout);
    }
    for (int b = 0; b < kNumBits; ++b) {
        touch_read(a.bank_e[b], (size_t)((sh.hid + 15) / 16) * 16 * ((sh.cin + 15) / 16) * 16);
        touch_read(a.bank_d[b], (size_t)9 * sh.hid);
        touch_read(a.bank_p[b], (size_t)((sh.cout + 15) / 16) * 16 * ((sh.hid + 15) / 16) * 16);
    }
    return hipSuccess;
}

bool mbconv_codes_supported(const MbShape &sh, bool expand_codes, bool project_codes)
{
    if (!expand_codes && !project_codes) return false;
    return mbconv_supported(sh) && ((expand_codes && project_codes) || sh.cout != 320);
}

hipError_t launch_mbconv_codes(const MbShape &sh, const MbCodeArgs &a, hipStream_t)
{
    ++g_launches;
    if (!mbconv_codes_supported(sh, a.codes_e != nullptr, a.codes_p != nullptr)) return hipErrorInvalidValue;
    const int ho = sh.h / sh.stride;
    touch_read(a.in, (size_t)a.N * sh.h * sh.h * sh.cin);
    touch_write(a.out, (size_t)a.N * ho * ho * sh.cout);
    if (a.codes_e) {
        touch_read(a.codes_e, (size_t)(sh.hid / 16) * ((sh.cin + 31) / 32) * 512);
        touch_read(a.scale_e, (size_t)sh.hid);
    } else {
        touch_read(a.w_e, (size_t)((sh.hid + 15) / 16) * 16 * ((sh.cin + 15) / 16) * 16);
    }
    if (a.codes_p) {
        touch_read(a.codes_p, (size_t)((sh.cout + 15) / 16) * (sh.hid / 16) * 256);
        touch_read(a.scale_p, (size_t)sh.cout);
    } else {
        touch_read(a.w_p, (size_t)((sh.cout + 15) / 16) * 16 * ((sh.hid + 15) / 16) * 16);
    }
    touch_read(a.w_d, (size_t)9 * sh.hid);
    touch_read(a.bias_e, (size_t)sh.hid);
    touch_read(a.bias_d, (size_t)sh.hid);
    touch_read(a.bias_p, (size_t)sh.cout);
    return hipSuccess;
}

bool pooled_codes_plan(int cin, int cout, int *cg, int *groups)
{
    const int ks = (cin + 31) / 32, tiles = (cout + 15) / 16;
    if (cin % 8 != 0 || cout % 4 != 0 || ks * 12288 > 160 * 1024) return false;
    *cg = tiles % 5 == 0 ? 5 : 2;
    *groups = (tiles + *cg - 1) / *cg;
    return true;
}

hipError_t launch_pooled_codes(const PoolCodeArgs &a, hipStream_t)
{
    ++g_launches;
    int cg = 0, groups = 0;
    if (!pooled_codes_plan(a.Cin, a.Cout, &cg, &groups) || cg != a.CG || groups != a.groups || a.KS != (a.Cin + 31) / 32)
        return hipErrorInvalidValue;
    touch_read(a.in, (size_t)a.N * 64 * a.Cin);
    touch_write(a.out, (size_t)a.N * a.Cout);
    touch_read(a.codes, (size_t)a.groups * a.CG * a.KS * 512);
    touch_read(a.scales, (size_t)a.Cout);
    touch_read(a.bias, (size_t)a.Cout);
    return hipSuccess;
}

hipError_t launch_pack_mb_codes(const int32_t *codes, uint16_t *out, int rows, int k, int kstep, hipStream_t)
{
    ++g_launches;
    if (kstep != 16 && kstep != 32) return hipErrorInvalidValue;
    touch_read(codes, (size_t)rows * k);
    touch_write(out, (size_t)((rows + 15) / 16) * ((k + kstep - 1) / kstep) * 64 * (kstep / 4));
    return hipSuccess;
}

hipError_t launch_pack_codes(const int32_t *codes, uint16_t *out, int cout, int cin, int taps, hipStream_t)
{
    ++g_launches;
    touch_read(codes, (size_t)cout * cin * taps);
    touch_write(out, (size_t)((cout + 31) / 32) * taps * ((cin + 15) / 16) * 512);
    return hipSuccess;
}

hipError_t launch_conv_codes(const CodeConvArgs &a, int ks, int stride, int nt, int stage_items, int mt, size_t lds_bytes,
                             dim3 grid, hipStream_t)
{
    ++g_launches;
    if (lds_bytes > 160 * 1024 || nt < 1 || nt > 2 || mt < 1 || mt > 2 || grid.x == 0) return hipErrorInvalidValue;
    touch_read(a.in, (size_t)a.N * a.Hin * a.Win * a.Cin);
    touch_write(a.out, (size_t)a.N * a.Hout * a.Wout * a.Cout);
    if (a.res) touch_read(a.res, (size_t)a.N * a.Hout * a.Wout * a.Cout);
    touch_read(a.codes, (size_t)a.cout_tiles * ks * ks * a.CB * 512);
    touch_read(a.scales, (size_t)a.Cout);
    touch_read(a.bias, (size_t)a.Cout);
    return hipSuccess;
}

hipError_t launch_act_codes(const float *in, const uint32_t *amax_bits, int8_t *codes, float *xscale, int n, int elems,
                            int bits, hipStream_t)
{
    ++g_launches;
    if (bits < 2 || bits > 8 || (elems & 15)) return hipErrorInvalidValue;
    if (amax_bits) touch_read(amax_bits, (size_t)n);
    touch_read(in, (size_t)n * elems);
    touch_write(codes, (size_t)n * elems);
    touch_write(xscale, (size_t)n);
    return hipSuccess;
}

hipError_t launch_pack_codes_i8(const int32_t *codes, int8_t *out, int cout, int cin, int taps, hipStream_t)
{
    ++g_launches;
    touch_read(codes, (size_t)cout * cin * taps);
    touch_write(out, (size_t)((cout + 31) / 32) * taps * ((cin + 31) / 32) * 1024);
    return hipSuccess;
}

hipError_t launch_conv_i8(const I8ConvArgs &a, int ks, int stride, int nt, size_t lds_bytes, dim3 grid, hipStream_t)
{
    ++g_launches;
    if (lds_bytes > 159 * 1024 || nt < 1 || nt > 2 || grid.x == 0 || (a.Cin & 15)) return hipErrorInvalidValue;
    touch_read(a.in, (size_t)a.N * a.Hin * a.Win * a.Cin);
    touch_read(a.xscale, (size_t)a.N);
    if (a.amax_out) touch_write(a.amax_out, (size_t)a.N);
    touch_write(a.out, (size_t)a.N * a.Hout * a.Wout * a.Cout);
    if (a.res) touch_read(a.res, (size_t)a.N * a.Hout * a.Wout * a.Cout);
    touch_read(a.codes, (size_t)a.cout_tiles * ks * ks * a.CBK * 1024);
    touch_read(a.scales, (size_t)a.Cout);
    touch_read(a.bias, (size_t)a.Cout);
    return hipSuccess;
}

} // namespace aiq
