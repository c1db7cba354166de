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

// The bare hand-over of the persistent training kernel, without its arithmetic: in every round each
// of the 256 workgroups publishes 64 tagged 64-bit words and then polls 8 words of 8 other
// workgroups until they carry the round's number.  ACROSS: the partners are spread over the chip,
// stores and loads of device scope.  WITHIN_DIE: the partners are the workgroups of the same die
// (workgroup g runs on die g % 8), the stores of workgroup scope, which stop in the die's L2, where
// the device-scope loads of the pollers find them.  A poll gives up after `limit` rounds of loads
// and counts itself in *gave_up (so a wrong assumption about the dies ends, it does not hang).
constexpr int kHandoverGroups = 256, kHandoverWords = 64, kHandoverFan = 8;
template <bool WITHIN_DIE>
__global__ __launch_bounds__(64) void k_probe_handover(unsigned long long* buf, int rounds, unsigned limit, int* gave_up) {
    typedef __attribute__((address_space(1))) unsigned long long gu64;
    constexpr int ngroups = WITHIN_DIE ? 8 : 1;
    const int grp = blockIdx.x % ngroups, me = blockIdx.x / ngroups, gsz = kHandoverGroups / ngroups;
    const int lane = threadIdx.x;
    bool ok = true;
    for (int it = 1; it <= rounds && ok; ++it) {
        unsigned long long* cur = buf + (size_t)(it & 1) * kHandoverGroups * kHandoverWords;
        const unsigned long long word = ((unsigned long long)(unsigned)it << 32) | (unsigned)lane;
        if (WITHIN_DIE) __hip_atomic_store((gu64*)(cur + (size_t)blockIdx.x * kHandoverWords + lane), word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        else __hip_atomic_store((gu64*)(cur + (size_t)blockIdx.x * kHandoverWords + lane), word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        for (;;) {
            bool pending = false;
#pragma unroll
            for (int k = 0; k < kHandoverFan; ++k) {
                const int prod = ((me + 1 + k * (gsz / kHandoverFan)) % gsz) * ngroups + grp;
                const unsigned long long v = __hip_atomic_load((const gu64*)(cur + (size_t)prod * kHandoverWords + lane),
                                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                pending |= (int)((unsigned)(v >> 32) - (unsigned)it) < 0;   // (a partner may be a round ahead)
            }
            if (!__any(pending)) break;
            if (++spins > limit) { ok = false; break; }
        }
    }
    if (!ok && lane == 0) atomicAdd(gave_up, 1);
}

}  // namespace dbsn
