// Stand-alone probe, not part of the library: what instructions issued between fp32 MFMAs cost on gfx950.
// A loop of 64 independent v_mfma_f32_16x16x4_f32 per iteration with PER other instructions per 16 MFMAs,
// placed after every G-th MFMA by scheduling barriers (runs of PER * G / 16).  Prints SIMD cycles per MFMA
// at 2.4 GHz.  The figures bound what a kernel that mixes MFMAs with vector work can reach.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef float floatx4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("hip error %d at %d\n", (int)e_, __LINE__); return 1; } } while (0)

// KIND 0: v_fma_f32, 1: s_mul_i32 + s_add_i32, 2: v_med3_f32
template <int NWAVES, int KIND, int PER, int G>
__global__ __launch_bounds__(NWAVES * 64) void mix_kernel(float *out, int iters, float c1, float c2, int sa)
{
    floatx4 acc[16];
#pragma unroll
    for (int m = 0; m < 16; ++m) acc[m] = floatx4{0.f, 0.f, 0.f, 0.f};
    floatx4 wa[4], xb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        wa[i] = floatx4{threadIdx.x * 1e-3f, 0.5f, 0.25f, i * 1.f};
        xb[i] = floatx4{1.f + threadIdx.x * 1e-4f, 2.f, i * 1.f, 3.f};
    }
    float x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = threadIdx.x * 0.01f + i;
    int sx[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) sx[i] = __builtin_amdgcn_readfirstlane(sa + i);
    constexpr int RUN = PER * G / 16;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int m = 0; m < 16; ++m)
                acc[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[m & 3][j], xb[m >> 2][j], acc[m], 0, 0, 0);
#pragma unroll
            for (int v = 0; v < PER; ++v) {
                if (KIND == 0) x[v & 15] = __builtin_fmaf(x[v & 15], c1, c2);
                if (KIND == 1) sx[v & 7] = sx[v & 7] * 3 + sa;
                if (KIND == 2) x[v & 15] = __builtin_amdgcn_fmed3f(x[v & 15], c1, c2);
            }
            constexpr int mask = KIND == 1 ? 0x004 : 0x002; // SALU : VALU
#pragma unroll
            for (int m = 0; m < 16 / G; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, G, 0);
                if (RUN > 0) __builtin_amdgcn_sched_group_barrier(mask, RUN, 0);
            }
        }
    }
    floatx4 s = {0, 0, 0, 0};
#pragma unroll
    for (int m = 0; m < 16; ++m) s += acc[m];
    float t = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += x[i];
    int u = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) u += sx[i];
    if (s.x + s.y + s.z + s.w + t + u == 12345.f) out[0] = s.x;
}

template <int NWAVES, int KIND, int PER, int G>
int run(float *out)
{
    const int wgs = 256 * 4, iters = 4000 / (NWAVES / 4);
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    static const char *names[] = {"v_fma_f32", "s_mul+s_add", "v_med3_f32"};
    printf("wavefronts/SIMD %d  %-12s %2d per 16 MFMAs, in runs of %2d:", NWAVES / 4, names[KIND], PER, PER * G / 16);
    for (int r = 0; r < 2; ++r) {
        CK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL((mix_kernel<NWAVES, KIND, PER, G>), dim3(wgs), dim3(NWAVES * 64), 0, 0, out, iters, 1.0001f, 0.5f, 3);
        CK(hipEventRecord(e1, 0));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        const double mfmas_per_simd = (double)wgs * NWAVES * iters * 64 / 1024.0;
        printf("  %.1f cycles per MFMA (%.1f %% of the fp32 MFMA peak)", ms * 1e-3 * 2.4e9 / mfmas_per_simd,
               (double)wgs * NWAVES * iters * 64 * 2048 / ms / 1e9 / 157.3 * 100);
        fflush(stdout);
    }
    printf("\n");
    return 0;
}

int main()
{
    float *out;
    CK(hipMalloc(&out, 256));
#define R(NW, K, P, G) if (run<NW, K, P, G>(out)) return 1;
    R(8, 0, 0, 16)
    R(8, 0, 16, 1) R(8, 0, 16, 2) R(8, 0, 16, 4) R(8, 0, 16, 8) R(8, 0, 16, 16)
    R(8, 0, 32, 1) R(8, 0, 32, 4) R(8, 0, 32, 16)
    R(8, 0, 64, 1) R(8, 0, 64, 4) R(8, 0, 64, 16)
    R(8, 2, 16, 1) R(8, 2, 16, 16)
    R(8, 1, 16, 1) R(8, 1, 16, 16) R(8, 1, 32, 1)
    R(4, 0, 16, 1) R(4, 0, 16, 16) R(16, 0, 16, 1) R(16, 0, 16, 16)
    CK(hipDeviceSynchronize());
    CK(hipFree(out));
    return 0;
}
