// Measurement aid (no part of the library): the rate of back-to-back independent
// v_mfma_f32_32x32x2_f32 with no memory traffic at all, for 1 to 7 accumulator tiles per wavefront
// and 1 to 4 blocks of 4 wavefronts per CU: what the matrix cores deliver for fp32 operands on
// this chip, against which the dense route's contraction is judged in the design notes.
// Build: hipcc --offload-arch=gfx950 -O3 -shared -fPIC probe_mfma.hip -o libprobe_mfma.so; call probe_mfma().
#include <hip/hip_runtime.h>
#include <cstdio>
typedef float f32x16 __attribute__((ext_vector_type(16)));
template <int NACC>
__global__ void __launch_bounds__(256) rate(float* out, int iters, float a0, float b0)
{
    f32x16 acc[NACC];
    for (int i = 0; i < NACC; ++i) for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    float a = a0 + threadIdx.x, b = b0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
#pragma unroll
            for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
        }
    }
    float s = 0.0f;
    for (int i = 0; i < NACC; ++i) for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
template <int NACC> double run(int blocks, int iters, float* d)
{
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    hipLaunchKernelGGL(rate<NACC>, dim3(blocks), dim3(256), 0, 0, d, 10, 1.0f, 0.5f);
    hipDeviceSynchronize();
    hipEventRecord(e0);
    hipLaunchKernelGGL(rate<NACC>, dim3(blocks), dim3(256), 0, 0, d, iters, 1.0f, 0.5f);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    const double mfmas = (double)blocks * 4 * iters * 16 * NACC;
    const double flops = mfmas * 4096;
    printf("NACC=%d blocks=%d: %.3f ms, %.1f TFLOP/s, %.1f clk/MFMA/SIMD at 2.4 GHz (if 1 block per CU)\n", NACC, blocks, ms,
           flops / ms / 1e9, ms * 1e-3 * 2.4e9 / (mfmas / (blocks < 256 ? blocks : 256) / 4));
    hipEventDestroy(e0); hipEventDestroy(e1);
    return flops / ms / 1e9;
}
// rates[i] = TFLOP/s of variant i (accumulator tiles per wavefront x blocks); returns the number of variants, < 0 on error
extern "C" int probe_mfma(double* rates, int cap)
{
    float* d; if (hipMalloc(&d, 4096 * 256 * 4)) return -2;
    const double r[6] = { run<4>(256, 2000, d), run<7>(256, 1000, d), run<1>(256, 4000, d),
                          run<2>(256, 4000, d), run<4>(512, 2000, d), run<4>(1024, 1000, d) };
    for (int i = 0; i < 6 && i < cap; ++i) rates[i] = r[i];
    if (hipDeviceSynchronize() != hipSuccess) return -3;
    hipFree(d);
    return 6;
}
