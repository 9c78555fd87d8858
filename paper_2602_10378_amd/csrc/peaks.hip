// sdkde_peaks: measures, on the GPU it runs on, the instruction rates the SD-KDE pair kernels are
// bounded by: fp32 MFMA (16x16x4 and 32x32x2), v_exp_f32, v_fma_f32, and how fp32 MFMA and VALU
// work share a SIMD (NM MFMAs per iteration with NE exps and NA adds, all mutually independent), and
// the same for the fp16 MFMAs of the lower-precision input modes.
// Cycle figures assume the nominal 2.4 GHz engine clock.
#include <hip/hip_runtime.h>
#include <cstdio>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int kIters = 20000;
constexpr int kBlock = 256;
constexpr int kCUs = 256;
constexpr double kClockHz = 2.4e9;

__global__ __launch_bounds__(kBlock) void mfma16_kernel(float* out, int iters, float a, float b)
{
    f32x4 acc[4];
    for (int c = 0; c < 4; ++c) acc[c] = f32x4{0, 0, 0, 0};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[c], 0, 0, 0);
    }
    float s = 0;
    for (int c = 0; c < 4; ++c) s += acc[c].x + acc[c].y + acc[c].z + acc[c].w;
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(kBlock) void mfma32_kernel(float* out, int iters, float a, float b)
{
    f32x16 acc[2];
    for (int c = 0; c < 2; ++c)
        for (int k = 0; k < 16; ++k) acc[c][k] = 0;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < 2; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
    }
    float s = 0;
    for (int c = 0; c < 2; ++c)
        for (int k = 0; k < 16; ++k) s += acc[c][k];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <bool EXP>
__global__ __launch_bounds__(kBlock) void valu_kernel(float* out, int iters, float a, float b)
{
    float v[8];
    for (int c = 0; c < 8; ++c) v[c] = -0.001f * (threadIdx.x + c);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] = EXP ? __builtin_amdgcn_exp2f(v[c]) : fmaf(v[c], a, b);
    }
    float s = 0;
    for (int c = 0; c < 8; ++c) s += v[c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// NM MFMAs, NE exps, NA adds per iteration; the VALU work is dealt evenly over the MFMA slots
// (SPREAD) or issued as one clump after all MFMAs.
template <int NM, int NE, int NA, bool SPREAD>
__global__ __launch_bounds__(kBlock) void mix_kernel(float* out, int iters, float a, float b)
{
    f32x4 acc[4];
    float e[8], s[8];
    for (int c = 0; c < 4; ++c) acc[c] = f32x4{0, 0, 0, 0};
    for (int c = 0; c < 8; ++c) {
        e[c] = -0.001f * (threadIdx.x + c);
        s[c] = c;
    }
    for (int i = 0; i < iters; ++i) {
        if (SPREAD) {
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                acc[k % 4] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[k % 4], 0, 0, 0);
#pragma unroll
                for (int q = k * NE / NM; q < (k + 1) * NE / NM; ++q) e[q % 8] = __builtin_amdgcn_exp2f(e[q % 8]);
#pragma unroll
                for (int q = k * NA / NM; q < (k + 1) * NA / NM; ++q) s[q % 8] = s[q % 8] + a;
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int k = 0; k < NM; ++k) acc[k % 4] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[k % 4], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < NE; ++q) e[q % 8] = __builtin_amdgcn_exp2f(e[q % 8]);
#pragma unroll
            for (int q = 0; q < NA; ++q) s[q % 8] = s[q % 8] + a;
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float r = 0;
    for (int c = 0; c < 4; ++c) r += acc[c].x + acc[c].y + acc[c].z + acc[c].w;
    for (int c = 0; c < 8; ++c) r += e[c] + s[c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

// fp16 MFMAs: K32 ? v_mfma_f32_16x16x32_f16 : v_mfma_f32_16x16x16_f16; NM of them, then NE exps and NA adds as one clump.
template <bool K32, int NM, int NE, int NA>
__global__ __launch_bounds__(kBlock) void mix_f16_kernel(float* out, int iters, float a, float b)
{
    f32x4 acc[4];
    float e[8], s[8];
    for (int c = 0; c < 4; ++c) acc[c] = f32x4{0, 0, 0, 0};
    for (int c = 0; c < 8; ++c) {
        e[c] = -0.001f * (threadIdx.x + c);
        s[c] = c;
    }
    const _Float16 ha = (_Float16)a, hb = (_Float16)b;
    const f16x4 a4 = {ha, hb, ha, hb};
    const f16x8 a8 = {ha, hb, ha, hb, ha, hb, ha, hb};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            if (K32) acc[k % 4] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a8, a8, acc[k % 4], 0, 0, 0);
            else acc[k % 4] = __builtin_amdgcn_mfma_f32_16x16x16f16(a4, a4, acc[k % 4], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < NE; ++q) e[q % 8] = __builtin_amdgcn_exp2f(e[q % 8]);
#pragma unroll
        for (int q = 0; q < NA; ++q) s[q % 8] = s[q % 8] + a;
        __builtin_amdgcn_sched_barrier(0);
    }
    float r = 0;
    for (int c = 0; c < 4; ++c) r += acc[c].x + acc[c].y + acc[c].z + acc[c].w;
    for (int c = 0; c < 8; ++c) r += e[c] + s[c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

hipEvent_t g_e0, g_e1;
float* g_out;

template <typename Launch>
float time_ms(Launch launch)
{
    launch();
    if (hipDeviceSynchronize() != hipSuccess) return -1.0f;
    if (hipEventRecord(g_e0) != hipSuccess) return -1.0f;
    launch();
    if (hipEventRecord(g_e1) != hipSuccess || hipEventSynchronize(g_e1) != hipSuccess) return -1.0f;
    float ms = -1.0f;
    if (hipEventElapsedTime(&ms, g_e0, g_e1) != hipSuccess) return -1.0f;
    return ms;
}

template <int NM, int NE, int NA, bool SPREAD>
void run_mix(int waves_per_simd)
{
    const int blocks = kCUs * waves_per_simd;
    float ms = time_ms([&] {
        hipLaunchKernelGGL((mix_kernel<NM, NE, NA, SPREAD>), dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 1.0f, 0.5f);
    });
    const double clk = ms * 1e-3 * kClockHz / kIters / waves_per_simd;
    const double tflops = NM * 32.0 * kIters * (double)blocks * kBlock / (ms * 1e-3) / 1e12;
    printf("  %d MFMA + %2d exp + %2d add, %-11s %d waves/SIMD: %6.1f clk per iteration per wave, MFMA %6.1f TFLOP/s\n", NM,
           NE, NA, SPREAD ? "interleaved" : "one clump", waves_per_simd, clk, tflops);
}

template <bool K32, int NM, int NE, int NA>
void run_mix_f16(int waves_per_simd)
{
    const int blocks = kCUs * waves_per_simd;
    float ms = time_ms([&] {
        hipLaunchKernelGGL((mix_f16_kernel<K32, NM, NE, NA>), dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 1.0f, 0.5f);
    });
    const double clk = ms * 1e-3 * kClockHz / kIters / waves_per_simd;
    printf("  %d x %s + %2d exp + %2d add, one clump, %d waves/SIMD: %6.1f clk per iteration per wave\n", NM,
           K32 ? "16x16x32_f16" : "16x16x16_f16", NE, NA, waves_per_simd, clk);
}

}  // namespace

int main()
{
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, 0) != hipSuccess) {
        fprintf(stderr, "no HIP device\n");
        return 1;
    }
    printf("device: %s, %d CUs, %d kHz\n", prop.gcnArchName, prop.multiProcessorCount, prop.clockRate);
    if (hipMalloc(&g_out, sizeof(float) * kBlock * kCUs * 4) != hipSuccess) return 1;
    if (hipEventCreate(&g_e0) != hipSuccess || hipEventCreate(&g_e1) != hipSuccess) return 1;

    printf("instruction peaks (4 waves per SIMD):\n");
    const int blocks = kCUs * 4;
    const double lanes = (double)blocks * kBlock * kIters;
    float ms = time_ms([&] { hipLaunchKernelGGL(mfma16_kernel, dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 1.0f, 0.5f); });
    printf("  v_mfma_f32_16x16x4_f32 : %7.1f TFLOP/s\n", lanes * 4 * 32.0 / (ms * 1e-3) / 1e12);
    ms = time_ms([&] { hipLaunchKernelGGL(mfma32_kernel, dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 1.0f, 0.5f); });
    printf("  v_mfma_f32_32x32x2_f32 : %7.1f TFLOP/s\n", lanes * 2 * 64.0 / (ms * 1e-3) / 1e12);
    ms = time_ms([&] { hipLaunchKernelGGL(valu_kernel<true>, dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 0.999f, 0.001f); });
    printf("  v_exp_f32              : %7.2f T lane-ops/s\n", lanes * 8 / (ms * 1e-3) / 1e12);
    ms = time_ms([&] { hipLaunchKernelGGL(valu_kernel<false>, dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 0.999f, 0.001f); });
    printf("  v_fma_f32              : %7.2f T lane-ops/s\n", lanes * 8 / (ms * 1e-3) / 1e12);

    printf("fp32 MFMA and VALU on one SIMD (8 MFMAs = 256 clk if they overlapped perfectly):\n");
    for (int w : {1, 4}) {
        run_mix<8, 0, 0, true>(w);
        run_mix<8, 0, 8, true>(w);
        run_mix<8, 0, 16, true>(w);
        run_mix<8, 0, 32, true>(w);
        run_mix<8, 8, 0, true>(w);
        run_mix<8, 16, 0, true>(w);
        run_mix<8, 4, 8, true>(w);
        run_mix<8, 4, 8, false>(w);
        run_mix<8, 8, 16, false>(w);
    }

    printf("fp16 MFMA and VALU on one SIMD (the 16x16x16 and 16x16x32 forms take the same time per instruction):\n");
    for (int w : {2, 4}) {
        run_mix_f16<false, 8, 0, 0>(w);
        run_mix_f16<true, 8, 0, 0>(w);
        run_mix_f16<true, 0, 8, 8>(w);
        run_mix_f16<true, 4, 8, 8>(w);
        run_mix_f16<true, 4, 4, 16>(w);
    }
    return 0;
}
