// Measurement helper of bench.py, built into a shared object of its own (libfscnn_bench_probe.so):
// not part of the library, its header or its binding.
//
// Ceiling probe for the hot loop's instruction mix, with no sparsity, staging or barriers: every
// wave repeats {1 address add, 4 x ds_read_b128 (conflict-free, 16 words per lane), 16 FMAs with a
// scalar weight} at full occupancy.  What it reports is the rate at which gfx950 sustains one LDS
// word per fused multiply-add; bench.py prints it beside the kernel's achieved rate.
#include <hip/hip_runtime.h>

namespace {
__global__ void __launch_bounds__(256) gather_fma_probe_kernel(float *out, int iters)
{
    __shared__ __align__(16) float tile[8192];  // 32 KB
    for (int i = threadIdx.x; i < 8192; i += 256) tile[i] = 1.0f + i * 1e-6f;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const char *base = reinterpret_cast<const char *>(tile) + lane * 16 + wave * 2048;
    float acc[16];
#pragma unroll
    for (int p = 0; p < 16; ++p) acc[p] = 0.0f;
    const float w = out[0];
    for (int it = 0; it < iters; ++it) {
        const char *p = base + ((it & 7) << 8);  // stays inside the tile: < 8 KB + 2 KB + 4 x 1 KB + 1 KB
        float4 in[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) in[v] = *reinterpret_cast<const float4 *>(p + v * 1056);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            acc[v * 4 + 0] = __builtin_fmaf(w, in[v].x, acc[v * 4 + 0]);
            acc[v * 4 + 1] = __builtin_fmaf(w, in[v].y, acc[v * 4 + 1]);
            acc[v * 4 + 2] = __builtin_fmaf(w, in[v].z, acc[v * 4 + 2]);
            acc[v * 4 + 3] = __builtin_fmaf(w, in[v].w, acc[v * 4 + 3]);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int p = 0; p < 16; ++p) s += acc[p];
    if (s == 123.456f) out[1] = s;  // keeps the loop alive; never true for the values used
}
}  // namespace

// Launches `work_groups` groups of 256 threads that each repeat the mix `iters` times; the caller
// times it (flop count: work_groups * 256 * iters * 32).  scratch_dev: device, at least 2 floats,
// the first one is read as the weight.  Asynchronous on `stream`.  Returns 0, or 1 for bad
// arguments, or 2 for a launch error.
extern "C" int bench_probe_gather_fma(float *scratch_dev, int iters, int work_groups, void *stream)
{
    if (!scratch_dev || iters <= 0 || work_groups <= 0 || work_groups > (1 << 20)) return 1;
    hipLaunchKernelGGL(gather_fma_probe_kernel, dim3(work_groups), dim3(256), 0, (hipStream_t)stream,
                       scratch_dev, iters);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
