// Measurement aid: what clock and rate the chip sustains on bf16 matrix instructions alone, as a function of how
// busy the matrix pipe is kept.  Every wave runs a register-only loop of v_mfma_f32_32x32x16_bf16 (or
// v_mfma_f32_16x16x32_bf16) on N(0,1) operands that change from one instruction to the next, with `gap` times
// eight idle cycles (s_nop 7) behind each instruction; 512 workgroups of 8 waves fill the 256 compute units at two
// waves per SIMD for two rounds.  The program prints the rate of each configuration from HIP events; run under
//     rocprofv3 --pmc SQ_BUSY_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_MFMA --kernel-trace -- wk_mfma_duty_probe
// the counters give the cycles of each launch (SQ_BUSY_CYCLES / 32 shader engines), hence the clock over the
// launch's duration, and the share of cycles the matrix pipe was busy.  It is the context for the attention
// kernel's roofline fraction: no arithmetic of the library is in here.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// WIDE: 32x32x16 with four accumulators; otherwise 16x16x32 with sixteen.  Both issue 16 x 32,768 flop per wave and
// loop iteration; the A operand changes every instruction, the B operand every second one.
template <bool WIDE, int GAP>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_mfma_duty(const float *in, float *out,
                                                                                             int iters) {
    const float *pin = in + (threadIdx.x & 63);
    bf16x8 a[8], b[4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) a[i][e] = (__bf16)pin[(i * 8 + e) * 64];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) b[i][e] = (__bf16)pin[8192 + (i * 8 + e) * 64];
    float s = 0.f;
    if constexpr (WIDE) {
        f32x16 acc[4];
        for (int c = 0; c < 4; ++c)
            for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u * 3) & 7], b[(u >> 1) & 3], acc[u & 3], 0, 0, 0);
                for (int g = 0; g < GAP; ++g) asm volatile("s_nop 7");
            }
        }
        for (int c = 0; c < 4; ++c)
            for (int r = 0; r < 16; ++r) s += acc[c][r];
    } else {
        f32x4 acc[16];
        for (int c = 0; c < 16; ++c)
            for (int r = 0; r < 4; ++r) acc[c][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                acc[u & 15] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[(u * 3) & 7], b[(u >> 1) & 3], acc[u & 15], 0, 0, 0);
                for (int g = 0; g < GAP; ++g) asm volatile("s_nop 7");
            }
        }
        for (int c = 0; c < 16; ++c)
            for (int r = 0; r < 4; ++r) s += acc[c][r];
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <bool WIDE, int GAP>
static void run(const float *in, float *out) {
    const int blocks = 512, iters = 40000;
    hipEvent_t e0, e1;
    hipEventCreate(&e0);
    hipEventCreate(&e1);
    hipLaunchKernelGGL((k_mfma_duty<WIDE, GAP>), dim3(blocks), dim3(512), 0, 0, in, out, 2000);   // warm-up
    hipDeviceSynchronize();
    hipEventRecord(e0);
    hipLaunchKernelGGL((k_mfma_duty<WIDE, GAP>), dim3(blocks), dim3(512), 0, 0, in, out, iters);
    hipEventRecord(e1);
    hipDeviceSynchronize();
    float ms = 0.f;
    hipEventElapsedTime(&ms, e0, e1);
    const double flop = (double)blocks * 8 * iters * 16 * 32768.0;
    std::printf("%s, %2d idle cycles behind each instruction: %7.3f ms  %6.1f TFLOP/s (%4.1f %% of 2500)\n",
                WIDE ? "32x32x16" : "16x16x32", 8 * GAP, ms, flop / ms / 1e9, flop / ms / 1e9 / 25.0);
    std::fflush(stdout);
}

int main() {
    float *in, *out;
    if (hipMalloc(&in, 1 << 20) != hipSuccess || hipMalloc(&out, 1 << 24) != hipSuccess) return 2;
    std::vector<float> h(1 << 18);
    unsigned long long s = 88172645463325252ull;   // xorshift64 -> Box-Muller
    for (size_t i = 0; i < h.size(); i += 2) {
        s ^= s << 13; s ^= s >> 7; s ^= s << 17;
        const float u1 = ((s >> 11) & 0xFFFFFF) / 16777216.0f + 1e-7f, u2 = ((s >> 35) & 0xFFFFFF) / 16777216.0f;
        const float r = std::sqrt(-2.f * std::log(u1));
        h[i] = r * std::cos(6.2831853f * u2);
        h[i + 1] = r * std::sin(6.2831853f * u2);
    }
    if (hipMemcpy(in, h.data(), 1 << 20, hipMemcpyHostToDevice) != hipSuccess) return 2;
    run<true, 0>(in, out);
    run<true, 1>(in, out);
    run<true, 2>(in, out);
    run<true, 4>(in, out);
    run<false, 0>(in, out);
    run<false, 1>(in, out);
    run<false, 2>(in, out);
    return 0;
}
