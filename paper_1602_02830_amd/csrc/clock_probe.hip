// Measurement aid of the benchmark, not part of the library's C ABI: built into a library of its
// own (libbnn_clock_probe.so) that only bench.py loads.
//
// One wavefront samples the shader-clock counter next to the constant-rate (100 MHz) counter while
// other kernels run on the rest of the chip; the ratio of the two differences is the clock the
// compute units actually ran at, which turns a throughput into a fraction of the peak at the
// measured clock instead of the nominal 2.4 GHz.  The loop is bounded by `n`, so the kernel always ends.
#include <hip/hip_runtime.h>
#include <stdint.h>

__global__ void clock_probe_kernel(long long* samples, int n, int sleeps) {
    if (threadIdx.x != 0) return;
    for (int i = 0; i < n; ++i) {
        samples[2 * i] = clock64();            // shader clock cycles
        samples[2 * i + 1] = wall_clock64();   // 100 MHz, independent of the shader clock
        for (int s = 0; s < sleeps; ++s) __builtin_amdgcn_s_sleep(127);
    }
}

// samples: DEVICE array of 2*n int64, pair i = (shader cycles, 100 MHz ticks) of sample i.
// Returns 0 or the hipError_t of the launch; n and sleeps must be in [1, 1 << 20].
extern "C" int bnn_clock_probe(long long* samples, int n, int sleeps, void* stream) {
    if (!samples || n < 1 || sleeps < 1 || n > (1 << 20) || sleeps > (1 << 20)) return int(hipErrorInvalidValue);
    hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), samples, n,
                       sleeps);
    return int(hipGetLastError());
}
