// Measurement aid of bench.py, built into its own shared object (libbench_mfma_probe.so), not part of the library:
// a register-resident INT8 MFMA loop (no memory traffic in the loop).  Its rate is the ceiling the chip's matrix cores
// reach at the clock they settle on under load, which bench.py reports the GEMM's rate against beside the datasheet peak.
#include <hip/hip_runtime.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256, 2) void mfma_i8_loop(int iters, int *sink)
{
    const int t = threadIdx.x;
    const v4i a = {t, t + 1, t + 2, t + 3}, b = {t * 3, t * 5, t * 7, t * 11};
    v16i c0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
    if (s == 0x7fffffff) sink[0] = s;   // keeps the loop alive; practically never taken
}

// Enqueues on `stream` a kernel of `blocks` workgroups x 4 wavefronts, each wavefront issuing 4*iters 32x32x32 INT8
// MFMAs on registers only: 2*32*32*32 * 4*iters * 4*blocks operations in all.  sink: device int (4 bytes, never written
// in practice).  Returns 0, -1 for bad arguments, or the HIP error code of the launch.
extern "C" int bench_mfma_probe(int iters, int blocks, void *sink, void *stream)
{
    if (!sink || (reinterpret_cast<uintptr_t>(sink) & 3) || iters < 1 || blocks < 1 || blocks > 65535) return -1;
    hipLaunchKernelGGL(mfma_i8_loop, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), iters, static_cast<int *>(sink));
    return static_cast<int>(hipGetLastError());
}
