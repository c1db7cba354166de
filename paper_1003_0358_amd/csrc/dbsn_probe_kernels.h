// Measurement aid of libdbsn, not part of the method: the memory traffic of a streamed on-line
// back-propagation step with no arithmetic to speak of.  A step reads every weight in the forward
// sweep and reads and rewrites it in the backward sweep (12 bytes per float32 weight); the two
// kernels here do exactly that over a buffer of n floats, one sweep each, with 128-bit accesses.
// What they sustain over a footprint is the ceiling a streaming training kernel can approach on
// that footprint (inside the memory-side cache or out of it).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dbsn {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 4;

// read sweep: every float4 is loaded once; the sums only keep the loads alive (one float per wavefront)
__global__ __launch_bounds__(kProbeThreads) void k_probe_read(const float4* __restrict__ w, long long n4,
                                                              float* __restrict__ sink) {
    const long long stride = (long long)gridDim.x * kProbeThreads;
    long long i = (long long)blockIdx.x * kProbeThreads + threadIdx.x;
    float4 acc[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) acc[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (; i + (kProbeUnroll - 1) * stride < n4; i += kProbeUnroll * stride) {
        float4 v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) v[u] = w[i + u * stride];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            acc[u].x += v[u].x; acc[u].y += v[u].y; acc[u].z += v[u].z; acc[u].w += v[u].w;
        }
    }
    for (; i < n4; i += stride) {
        const float4 v = w[i];
        acc[0].x += v.x; acc[0].y += v.y; acc[0].z += v.z; acc[0].w += v.w;
    }
    float s = 0.0f;
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) s += (acc[u].x + acc[u].y) + (acc[u].z + acc[u].w);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if ((threadIdx.x & 63) == 0) sink[blockIdx.x * (kProbeThreads / 64) + (threadIdx.x >> 6)] = s;
}

// update sweep: every float4 is loaded, changed and stored back
__global__ __launch_bounds__(kProbeThreads) void k_probe_update(float4* __restrict__ w, long long n4, float c) {
    const long long stride = (long long)gridDim.x * kProbeThreads;
    long long i = (long long)blockIdx.x * kProbeThreads + threadIdx.x;
    for (; i + (kProbeUnroll - 1) * stride < n4; i += kProbeUnroll * stride) {
        float4 v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) v[u] = w[i + u * stride];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            v[u].x += c; v[u].y += c; v[u].z += c; v[u].w += c;
            w[i + u * stride] = v[u];
        }
    }
    for (; i < n4; i += stride) {
        float4 v = w[i];
        v.x += c; v.y += c; v.z += c; v.w += c;
        w[i] = v;
    }
}

}  // namespace dbsn
