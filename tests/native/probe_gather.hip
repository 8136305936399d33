// Measurement aid (no part of the library): the rate at which the vector memory path delivers the
// access pattern of the batch kernels' multiply phase and nothing else -- 16 (or 8) wavefronts per
// CU, 8-lane groups fetching random 128-byte rows of one 3.2 MB panel that stays in L2, row numbers
// read from LDS, 4 / 10 / 20 fetches in flight per group.  All addresses are in bounds by
// construction (row numbers are drawn below n).  Prints one line per variant; the design notes
// quote the best of them as the ceiling of that phase.
// Build: hipcc --offload-arch=gfx950 -O3 -shared -fPIC probe_gather.hip -o libprobe_gather.so; call probe_gather().
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <random>
#include <vector>
template <int PIPE>
__global__ void __launch_bounds__(1024) gather(const float* __restrict__ panel, const uint32_t* __restrict__ rows, int per_wave, int reps, float* out)
{
    const uint32_t lane = threadIdx.x & 63, wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const uint32_t grp = lane >> 3, lig = lane & 7;
    __shared__ uint32_t lrows[16][512];
    uint32_t* my = lrows[threadIdx.x >> 6];
    for (int i = lane; i < per_wave; i += 64) my[i] = rows[(size_t)wave * per_wave + i];
    __syncthreads();
    float4 acc = make_float4(0, 0, 0, 0);
    for (int r = 0; r < reps; ++r) {
        for (int i = grp; i + 8 * (PIPE - 1) < per_wave; i += 8 * PIPE) {
            float4 v[PIPE];
#pragma unroll
            for (int k = 0; k < PIPE; ++k) v[k] = *reinterpret_cast<const float4*>(panel + (size_t)my[i + 8 * k] * 32 + lig * 4);
#pragma unroll
            for (int k = 0; k < PIPE; ++k) { acc.x += v[k].x; acc.y += v[k].y; acc.z += v[k].z; acc.w += v[k].w; }
        }
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc.x + acc.y + acc.z + acc.w;
}
// rates[i] = TB/s of variant i (waves per block 16, 8 x fetches in flight 4, 10, 20); returns the number of variants, < 0 on error
extern "C" int probe_gather(double* rates, int cap)
{
    int count = 0;
    const int n = 25088, waves = 4096, per_wave = 480, reps = 8;
    std::vector<uint32_t> rows((size_t)waves * per_wave);
    std::mt19937 rng(1);
    for (int w = 0; w < waves; ++w) {                      // ascending random rows, like a sparse column
        std::vector<uint32_t> r(per_wave);
        for (auto& x : r) x = rng() % n;
        std::sort(r.begin(), r.end());
        std::copy(r.begin(), r.end(), rows.begin() + (size_t)w * per_wave);
    }
    float *panel, *out; uint32_t* drows;
    if (hipMalloc(&panel, (size_t)n * 128) || hipMalloc(&out, (size_t)waves * 64 * 4) || hipMalloc(&drows, rows.size() * 4)) return -2;
    hipMemset(panel, 0, (size_t)n * 128);
    hipMemcpy(drows, rows.data(), rows.size() * 4, hipMemcpyHostToDevice);
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    for (int wpb : {16, 8}) {
        for (int variant = 0; variant < 3; ++variant) {
            auto launch = [&]() {
                dim3 grid(waves / wpb), block(wpb * 64);
                if (variant == 0) hipLaunchKernelGGL(gather<4>, grid, block, 0, 0, panel, drows, per_wave, reps, out);
                else if (variant == 1) hipLaunchKernelGGL(gather<10>, grid, block, 0, 0, panel, drows, per_wave, reps, out);
                else hipLaunchKernelGGL(gather<20>, grid, block, 0, 0, panel, drows, per_wave, reps, out);
            };
            launch(); hipDeviceSynchronize();
            hipEventRecord(e0); launch(); hipEventRecord(e1); hipEventSynchronize(e1);
            float ms; hipEventElapsedTime(&ms, e0, e1);
            const int pipe = variant == 0 ? 4 : variant == 1 ? 10 : 20;
            const double bytes = (double)waves * (per_wave / (8 * pipe)) * (8 * pipe) * 128.0 * reps;
            printf("waves/block=%d pipe=%d: %.3f ms, %.1f TB/s\n", wpb, pipe, ms, bytes / ms / 1e9);
            if (count < cap) rates[count] = bytes / ms / 1e9;
            ++count;
        }
    }
    if (hipDeviceSynchronize() != hipSuccess) return -3;
    hipEventDestroy(e0); hipEventDestroy(e1);
    hipFree(panel); hipFree(out); hipFree(drows);
    return count;
}
