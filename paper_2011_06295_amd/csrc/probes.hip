// Roof probes: two small kernels of known work whose measured rates stand beside the published peaks
// that the benchmark's roofline fractions are quoted against.
//   * LDS read rate: every wavefront reads 64 consecutive 16-byte elements (ds_read_b128, the access
//     pattern of the convolution kernel's gather) at changing offsets and does nothing else.
//   * Memory copy rate: a grid-stride copy of 16-byte words (read once, written once).
#include <hip/hip_runtime.h>

#include "internal.h"

namespace sc {

namespace {

constexpr int kProbeThreads = 1024;
constexpr int kProbeLdsBytes = 64 * 1024;
constexpr int kProbeReadsPerIter = 8;

__global__ __launch_bounds__(kProbeThreads) void lds_read_probe(int iterations, float* sink)
{
    __shared__ __attribute__((aligned(16))) float lds[kProbeLdsBytes / 4];
    for (int i = threadIdx.x; i < kProbeLdsBytes / 4; i += kProbeThreads) lds[i] = 1.0f;
    __syncthreads();
    typedef float vec4 __attribute__((ext_vector_type(4)));
    const vec4* t = reinterpret_cast<const vec4*>(lds);
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    float acc = 0.f;
    for (int it = 0; it < iterations; ++it) {
        vec4 x[kProbeReadsPerIter];
#pragma unroll
        for (int u = 0; u < kProbeReadsPerIter; ++u)   // 64 consecutive elements, start changing from read to read
            x[u] = t[(lane + wave * 64 + (it * kProbeReadsPerIter + u) * 37) & (kProbeLdsBytes / 16 - 1)];
#pragma unroll
        for (int u = 0; u < kProbeReadsPerIter; ++u) acc += x[u][0];
    }
    sink[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = acc;
}

__global__ __launch_bounds__(256) void copy_probe(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t words)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride) dst[i] = src[i];
}

}  // namespace

int launch_lds_read_probe(void* sink, int workgroups, int iterations, void* stream, long long* bytes_read)
{
    hipLaunchKernelGGL(lds_read_probe, dim3(workgroups), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                       iterations, static_cast<float*>(sink));
    if (bytes_read) *bytes_read = (long long)workgroups * kProbeThreads * 16ll * kProbeReadsPerIter * iterations;
    return (int)hipGetLastError();
}

int launch_copy_probe(void* dst, const void* src, long long bytes, void* stream)
{
    const size_t words = (size_t)bytes / 16;
    hipLaunchKernelGGL(copy_probe, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint4*>(dst), static_cast<const uint4*>(src), words);
    return (int)hipGetLastError();
}

}  // namespace sc
