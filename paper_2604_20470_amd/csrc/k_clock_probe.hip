// Measurement aid: average shader clock over a time window.  One wavefront polls the constant-rate
// 100 MHz counter (s_memrealtime) until the window has elapsed and reports how far the shader-clock
// counter (s_memtime) advanced meanwhile.  Launched on a side stream while other kernels run, it shows
// the frequency the chip actually sustains under that load (the matrix-core peak is quoted at 2.4 GHz).
#include "dr_internal.h"

namespace dr {
namespace {

__global__ __launch_bounds__(64) void k_clock_probe(unsigned long long window_ticks, unsigned long long* out) {
    const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();
    const unsigned long long s0 = __builtin_amdgcn_s_memtime();
    unsigned long long r = r0;
    // bounded twice: by the window, and by an iteration count that no real window reaches
    for (int i = 0; i < (1 << 24) && r - r0 < window_ticks; ++i) {
        __builtin_amdgcn_s_sleep(64);
        r = __builtin_amdgcn_s_memrealtime();
    }
    const unsigned long long s1 = __builtin_amdgcn_s_memtime();
    if (threadIdx.x == 0) {
        out[0] = s1 - s0;
        out[1] = r - r0;
    }
}

// Measurement aid: what the matrix cores sustain with nothing else going on.  Every wavefront keeps eight A and eight
// B fragments in registers and issues matrix instructions on eight independent accumulators; the fragments are
// either one repeated value (little switching activity) or pseudo-random bf16 numbers in [-1, 1) (the activity of
// real operands).  SHAPE 32: v_mfma_f32_32x32x16_bf16 (32768 flop), SHAPE 16: v_mfma_f32_16x16x32_bf16 (16384 flop);
// 8 instructions per wavefront and iteration.
typedef __bf16 pv8bf __attribute__((ext_vector_type(8)));
typedef float pv16f __attribute__((ext_vector_type(16)));
typedef float pv4f __attribute__((ext_vector_type(4)));

template <int SHAPE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_mfma_probe(int iters, int random_operands,
                                                                                                float* sink) {
    pv8bf a[8], b[8];
    uint32_t x = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    for (int f = 0; f < 8; ++f)
        for (int i = 0; i < 8; ++i) {
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;                        // xorshift32
            const float u = random_operands ? ((x & 0xffff) / 32768.0f - 1.0f) : 0.5f;
            a[f][i] = (__bf16)u;
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            const float w = random_operands ? ((x & 0xffff) / 32768.0f - 1.0f) : 0.5f;
            b[f][i] = (__bf16)w;
        }
    float t = 0.f;
    if (SHAPE == 32) {
        pv16f acc[8];
        for (int c = 0; c < 8; ++c)
            for (int j = 0; j < 16; ++j) acc[c][j] = 0.f;
        for (int it = 0; it < iters; it += 8) {          // iters is a multiple of 8 (checked on the host)
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int f = 0; f < 8; ++f)
                    acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], b[(f + j) & 7], acc[f], 0, 0, 0);
        }
        for (int c = 0; c < 8; ++c)
            for (int j = 0; j < 16; ++j) t += acc[c][j];
    } else {
        pv4f acc[8];
        for (int c = 0; c < 8; ++c)
            for (int j = 0; j < 4; ++j) acc[c][j] = 0.f;
        for (int it = 0; it < iters; it += 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int f = 0; f < 8; ++f)
                    acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[f], b[(f + j) & 7], acc[f], 0, 0, 0);
        }
        for (int c = 0; c < 8; ++c)
            for (int j = 0; j < 4; ++j) t += acc[c][j];
    }
    if (t == 1.2345e-30f) sink[0] = t;                                      // keeps the loop alive
}

// Measurement aid: the matrix instruction with the attention loop's kind of company.  One wavefront per SIMD, as in the
// attention kernels; per slot one v_mfma_f32_32x32x16_bf16 on pseudo-random bf16 operands, one v_exp_f32 and two
// v_fma_f32 on live fp32 registers (the attention loop has per slot 0.9 exponentials, 0.45 packs to bf16, 0.65 LDS
// fragment reads and about one scalar instruction).  8 slots per iteration; the scheduling barriers keep each slot's
// instructions where they are written.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_mfma_mix_probe(int iters, float* sink) {
    pv8bf a[8], b[8];
    uint32_t x = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    for (int f = 0; f < 8; ++f)
        for (int i = 0; i < 8; ++i) {
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            a[f][i] = (__bf16)((x & 0xffff) / 32768.0f - 1.0f);
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            b[f][i] = (__bf16)((x & 0xffff) / 32768.0f - 1.0f);
        }
    float e[8], y[8];
    for (int i = 0; i < 8; ++i) { e[i] = 0.f; y[i] = 0.5f + 0.001f * (float)(i + (threadIdx.x & 63)); }
    pv16f acc[4];
    for (int c = 0; c < 4; ++c)
        for (int j = 0; j < 16; ++j) acc[c][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            // written out so that the accumulators stay in AGPRs and no copy joins the slot
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[g & 3]) : "v"(a[g]), "v"(b[(g + 3) & 7]));
            e[g] = __builtin_amdgcn_exp2f(y[(g + 3) & 7]);
            asm volatile("" : "+v"(e[g]));
            y[g] = __builtin_fmaf(y[g], 0.999f, 0.001f);
            asm volatile("" : "+v"(y[g]));
            y[(g + 1) & 7] = __builtin_fmaf(y[(g + 1) & 7], 0.999f, 0.001f);
            asm volatile("" : "+v"(y[(g + 1) & 7]));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float t = 0.f;
    for (int c = 0; c < 4; ++c)
        for (int j = 0; j < 16; ++j) t += acc[c][j];
    for (int i = 0; i < 8; ++i) t += e[i] + y[i];
    if (t == 1.2345e-30f) sink[0] = t;                                      // keeps the loop alive
}

}  // namespace

hipError_t launch_mfma_mix_probe(int workgroups, int iters, float* sink, hipStream_t s) {
    hipLaunchKernelGGL(k_mfma_mix_probe, dim3(workgroups), dim3(256), 0, s, iters, sink);
    return hipGetLastError();
}

hipError_t launch_mfma_probe(int shape, int workgroups, int iters, int random_operands, float* sink, hipStream_t s) {
    if (shape == 32) hipLaunchKernelGGL(k_mfma_probe<32>, dim3(workgroups), dim3(256), 0, s, iters, random_operands, sink);
    else hipLaunchKernelGGL(k_mfma_probe<16>, dim3(workgroups), dim3(256), 0, s, iters, random_operands, sink);
    return hipGetLastError();
}

hipError_t launch_clock_probe(unsigned long long window_ticks, unsigned long long* out, hipStream_t s) {
    hipLaunchKernelGGL(k_clock_probe, dim3(1), dim3(64), 0, s, window_ticks, out);
    return hipGetLastError();
}

}  // namespace dr
