// sdkde_peaks: measures, on the GPU it runs on, the instruction rates the SD-KDE pair kernels are
// bounded by: fp32 MFMA (16x16x4 and 32x32x2), the issue rates of v_fma_f32 / v_add_f32 / v_exp_f32 and of
// their mix in different orders, how fp32 MFMA and VALU
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

// Sustained issue rate of one VALU instruction (WHAT 0: v_fma_f32, 1: v_add_f32, 2: v_exp_f32): 128 independent
// instructions per iteration over 16 registers, pinned with volatile asm so that none is merged or reordered.
#define SDKDE_FMA(k) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(s[(k) % 16]) : "v"(a), "v"(b))
#define SDKDE_ADD(k) asm volatile("v_add_f32 %0, %0, %1" : "+v"(s[(k) % 16]) : "v"(a))
#define SDKDE_EXP(k) asm volatile("v_exp_f32 %0, %0" : "+v"(e[(k) % 16]))
#define SDKDE_R16(OP) OP(0); OP(1); OP(2); OP(3); OP(4); OP(5); OP(6); OP(7); OP(8); OP(9); OP(10); OP(11); OP(12); OP(13); OP(14); OP(15);
#define SDKDE_R128(OP) SDKDE_R16(OP) SDKDE_R16(OP) SDKDE_R16(OP) SDKDE_R16(OP) SDKDE_R16(OP) SDKDE_R16(OP) SDKDE_R16(OP) SDKDE_R16(OP)
template <int WHAT>
__global__ __launch_bounds__(kBlock) void issue_kernel(float* out, int iters, float a, float b)
{
    float s[16], e[16];
    for (int c = 0; c < 16; ++c) s[c] = e[c] = -0.001f * (threadIdx.x + c);
    for (int i = 0; i < iters; ++i) {
        if (WHAT == 0) { SDKDE_R128(SDKDE_FMA) }
        if (WHAT == 1) { SDKDE_R128(SDKDE_ADD) }
        if (WHAT == 2) { SDKDE_R128(SDKDE_EXP) }
    }
    float r = 0;
    for (int c = 0; c < 16; ++c) r += s[c] + e[c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

// The thin path's mix, 16 v_exp_f32 and 64 independent v_fma_f32 per iteration, in three orders:
// ORDER 0: (exp, 4 fma) x 16; 1: 16 exp, then 64 fma; 2: (4 exp, 16 fma) x 4.
#define SDKDE_F4(k) SDKDE_FMA(4 * (k)); SDKDE_FMA(4 * (k) + 1); SDKDE_FMA(4 * (k) + 2); SDKDE_FMA(4 * (k) + 3);
#define SDKDE_E4(k) SDKDE_EXP(4 * (k)); SDKDE_EXP(4 * (k) + 1); SDKDE_EXP(4 * (k) + 2); SDKDE_EXP(4 * (k) + 3);
template <int ORDER>
__global__ __launch_bounds__(kBlock) void exp_order_kernel(float* out, int iters, float a, float b)
{
    float s[16], e[16];
    for (int c = 0; c < 16; ++c) s[c] = e[c] = -0.001f * (threadIdx.x + c);
    for (int i = 0; i < iters; ++i) {
        if (ORDER == 0) {
#define SDKDE_G(k) SDKDE_EXP(k); SDKDE_F4(k)
            SDKDE_G(0) SDKDE_G(1) SDKDE_G(2) SDKDE_G(3) SDKDE_G(4) SDKDE_G(5) SDKDE_G(6) SDKDE_G(7)
            SDKDE_G(8) SDKDE_G(9) SDKDE_G(10) SDKDE_G(11) SDKDE_G(12) SDKDE_G(13) SDKDE_G(14) SDKDE_G(15)
#undef SDKDE_G
        }
        if (ORDER == 1) {
            SDKDE_E4(0) SDKDE_E4(1) SDKDE_E4(2) SDKDE_E4(3)
            SDKDE_F4(0) SDKDE_F4(1) SDKDE_F4(2) SDKDE_F4(3) SDKDE_F4(4) SDKDE_F4(5) SDKDE_F4(6) SDKDE_F4(7)
            SDKDE_F4(8) SDKDE_F4(9) SDKDE_F4(10) SDKDE_F4(11) SDKDE_F4(12) SDKDE_F4(13) SDKDE_F4(14) SDKDE_F4(15)
        }
        if (ORDER == 2) {
#define SDKDE_G(k) SDKDE_E4(k) SDKDE_F4(4 * (k)) SDKDE_F4(4 * (k) + 1) SDKDE_F4(4 * (k) + 2) SDKDE_F4(4 * (k) + 3)
            SDKDE_G(0) SDKDE_G(1) SDKDE_G(2) SDKDE_G(3)
#undef SDKDE_G
        }
    }
    float r = 0;
    for (int c = 0; c < 16; ++c) r += s[c] + e[c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

// fp16 MFMAs: K32 ? v_mfma_f32_16x16x32_f16 : v_mfma_f32_16x16x16_f16; NM of them and NF fp32 MFMAs (16x16x4), then NE
// exps and NA adds as one clump.
template <bool K32, int NM, int NE, int NA, int NF = 0>
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
#pragma unroll
        for (int k = 0; k < NF; ++k) acc[k % 4] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[k % 4], 0, 0, 0);
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

template <bool K32, int NM, int NE, int NA, int NF = 0>
void run_mix_f16(int waves_per_simd)
{
    const int blocks = kCUs * waves_per_simd;
    float ms = time_ms([&] {
        hipLaunchKernelGGL((mix_f16_kernel<K32, NM, NE, NA, NF>), dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 1.0f, 0.5f);
    });
    const double clk = ms * 1e-3 * kClockHz / kIters / waves_per_simd;
    printf("  %d x %s + %d x 16x16x4_f32 + %2d exp + %2d add, one clump, %d waves/SIMD: %6.1f clk per iteration per wave\n", NM,
           K32 ? "16x16x32_f16" : "16x16x16_f16", NF, NE, NA, waves_per_simd, clk);
}

// NM x v_mfma_f32_32x32x2_f32, then NE exps and NA adds as one clump.
template <int NM, int NE, int NA>
__global__ __launch_bounds__(kBlock) void mix32_kernel(float* out, int iters, float a, float b)
{
    f32x16 acc[2];
    float e[16], s[16];
    for (int c = 0; c < 2; ++c)
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.0f;
    for (int c = 0; c < 16; ++c) {
        e[c] = -0.001f * (threadIdx.x + c);
        s[c] = c;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int k = 0; k < NM; ++k) acc[k % 2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[k % 2], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < NE; ++q) e[q % 16] = __builtin_amdgcn_exp2f(e[q % 16]);
#pragma unroll
        for (int q = 0; q < NA; ++q) s[q % 16] = s[q % 16] + a;
        __builtin_amdgcn_sched_barrier(0);
    }
    float r = 0;
    for (int c = 0; c < 2; ++c)
        for (int v = 0; v < 16; ++v) r += acc[c][v];
    for (int c = 0; c < 16; ++c) r += e[c] + s[c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

template <int NM, int NE, int NA>
void run_mix32(int waves_per_simd)
{
    const int blocks = kCUs * waves_per_simd;
    float ms = time_ms([&] { hipLaunchKernelGGL((mix32_kernel<NM, NE, NA>), dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 1.0f, 0.5f); });
    const double clk = ms * 1e-3 * kClockHz / kIters / waves_per_simd;
    printf("  %d x 32x32x2_f32 + %2d exp + %2d add, one clump   %d waves/SIMD: %6.1f clk per iteration per wave\n", NM, NE, NA,
           waves_per_simd, clk);
}

template <int WHAT>
void run_issue(const char* what)
{
    constexpr int iters = 4000;
    for (int w : {1, 2, 4, 8}) {
        const int blocks = kCUs * w;
        float ms = time_ms([&] { hipLaunchKernelGGL(issue_kernel<WHAT>, dim3(blocks), dim3(kBlock), 0, 0, g_out, iters, 0.999f, 0.001f); });
        printf("  %-10s %d waves/SIMD: %5.2f clk per wave instruction per SIMD, %6.2f T lane-ops/s\n", what, w,
               ms * 1e-3 * kClockHz / iters / w / 128, 128.0 * iters * (double)blocks * kBlock / (ms * 1e-3) / 1e12);
    }
}

template <int ORDER>
void run_exp_order(const char* what)
{
    constexpr int iters = 10000;
    for (int w : {4, 8}) {
        const int blocks = kCUs * w;
        float ms = time_ms([&] { hipLaunchKernelGGL(exp_order_kernel<ORDER>, dim3(blocks), dim3(kBlock), 0, 0, g_out, iters, 0.999f, 0.001f); });
        printf("  %-22s %d waves/SIMD: %5.2f clk per (exp + 4 fma)\n", what, w, ms * 1e-3 * kClockHz / iters / w / 16);
    }
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
    if (hipMalloc(&g_out, sizeof(float) * kBlock * kCUs * 8) != hipSuccess) return 1;
    if (hipEventCreate(&g_e0) != hipSuccess || hipEventCreate(&g_e1) != hipSuccess) return 1;

    printf("instruction peaks (4 waves per SIMD):\n");
    const int blocks = kCUs * 4;
    const double lanes = (double)blocks * kBlock * kIters;
    float ms = time_ms([&] { hipLaunchKernelGGL(mfma16_kernel, dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 1.0f, 0.5f); });
    printf("  v_mfma_f32_16x16x4_f32 : %7.1f TFLOP/s\n", lanes * 4 * 32.0 / (ms * 1e-3) / 1e12);
    ms = time_ms([&] { hipLaunchKernelGGL(mfma32_kernel, dim3(blocks), dim3(kBlock), 0, 0, g_out, kIters, 1.0f, 0.5f); });
    printf("  v_mfma_f32_32x32x2_f32 : %7.1f TFLOP/s\n", lanes * 2 * 64.0 / (ms * 1e-3) / 1e12);

    printf("VALU issue, independent instructions (fp32 vector peak 157.3 TFLOP/s = 78.6 T FMA lane-ops/s = one wave instruction per 2 clk per SIMD):\n");
    run_issue<0>("v_fma_f32");
    run_issue<1>("v_add_f32");
    run_issue<2>("v_exp_f32");
    printf("16 v_exp_f32 and 64 v_fma_f32 per iteration, by order of issue (the thin path's mix):\n");
    run_exp_order<0>("(exp, 4 fma) x 16");
    run_exp_order<1>("16 exp, then 64 fma");
    run_exp_order<2>("(4 exp, 16 fma) x 4");

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

    printf("the eval kernels' mix by MFMA shape: per 256 pairs 4 x 16x16x4 + 4 exp + 8 add, per 1024 pairs 8 x 32x32x2 + 16 exp + 32 add:\n");
    for (int w : {2, 4}) {
        run_mix<4, 4, 8, false>(w);
        run_mix32<8, 16, 32>(w);
    }

    printf("fp16 MFMA and VALU on one SIMD (the 16x16x16 and 16x16x32 forms take the same time per instruction):\n");
    for (int w : {2, 4}) {
        run_mix_f16<false, 8, 0, 0>(w);
        run_mix_f16<true, 8, 0, 0>(w);
        run_mix_f16<true, 0, 8, 8>(w);
        run_mix_f16<true, 4, 8, 8>(w);
        run_mix_f16<true, 4, 4, 16>(w);
        run_mix_f16<true, 2, 4, 8, 4>(w);        // the fp16x2 input mode's score mix: cross term on fp16, Phi X on fp32 MFMAs
        run_mix_f16<true, 2, 4, 8>(w);           // its eval mix
        run_mix_f16<true, 3, 4, 10>(w);          // single-fp16-weights mode: 3 fp16 MFMAs, 4 exp, 4 add + 2 cvt + 2 dot2 + 2 mov
    }
    return 0;
}
