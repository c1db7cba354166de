// Small reductions of libdbsn for the passes around training (section "Results": the error count of
// a validation or test pass; the mean loss of an epoch).  One workgroup each, sums in a fixed
// order, so the results are reproducible from run to run; the inputs are at most a few hundred
// thousand values, which one workgroup reads in microseconds.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dbsn {

constexpr int kReduceThreads = 1024;

// *out = number of positions s < n with a[s] != b[s]
__global__ __launch_bounds__(kReduceThreads) void k_count_errors(const int* __restrict__ a, const int* __restrict__ b,
                                                                 long long n, long long* __restrict__ out) {
    __shared__ long long part[kReduceThreads];
    long long c = 0;
    for (long long s = threadIdx.x; s < n; s += kReduceThreads) c += (a[s] != b[s]) ? 1 : 0;
    part[threadIdx.x] = c;
    __syncthreads();
    for (int w = kReduceThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = part[0];
}

// *out = (float)(sum of v[0 .. n) in double / n): thread t adds v[t], v[t + 1024], ... in index order,
// then the 1024 sums are added pairwise in a fixed tree
__global__ __launch_bounds__(kReduceThreads) void k_mean(const float* __restrict__ v, long long n,
                                                         float* __restrict__ out) {
    __shared__ double part[kReduceThreads];
    double s = 0.0;
    for (long long i = threadIdx.x; i < n; i += kReduceThreads) s += (double)v[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = kReduceThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = (float)(part[0] / (double)n);
}

// plain fill with zeros (instead of a memset node, for callers that record the stream into a graph)
__global__ void k_zero(float4* __restrict__ p, long long n4) {
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (long long)gridDim.x * blockDim.x)
        p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

__global__ void k_zero_int(int* __restrict__ p, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

}  // namespace dbsn
