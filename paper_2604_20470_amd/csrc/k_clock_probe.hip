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

}  // namespace

hipError_t launch_clock_probe(unsigned long long window_ticks, unsigned long long* out, hipStream_t s) {
    hipLaunchKernelGGL(k_clock_probe, dim3(1), dim3(64), 0, s, window_ticks, out);
    return hipGetLastError();
}

}  // namespace dr
