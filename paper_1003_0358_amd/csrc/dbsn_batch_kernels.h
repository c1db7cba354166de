// Forward-only propagation of a BATCH of samples through one layer, for the classification passes
// over validation and test sets (sections "Data" and "Results"; appendix "Forward propagation").
// With many samples at once the layer is a dense contraction Y = X W^T, so unlike the on-line
// training step it belongs on the matrix cores: fp32 MFMA (products and sums in binary32, as
// everywhere in this library), each weight tile read from memory once per 128 samples.
//
// One workgroup of 4 wavefronts computes a tile of 128 samples x 128 neurons; wavefront w owns the
// 64 x 64 quadrant (w & 1, w >> 1) as 2 x 2 v_mfma_f32_32x32x2 accumulators (64 registers).  The k
// dimension is walked in chunks of 16 staged in LDS (pitch 17: the operand reads, row = lane % 32,
// k = lane / 32, fall in distinct banks), in two buffers used in turn: while the matrix
// instructions work on one chunk, the next one is written to the other buffer and the one after
// that is on its way from memory into registers, so a chunk costs one barrier and memory latency
// hides behind the arithmetic.  Operand layout of the instruction: lane t supplies
// A[i = t % 32][k = t / 32] and B[k = t / 32][j = t % 32]; result register r of lane t is
// D[i = r % 4 + 4 (t / 32) + 8 (r / 4)][j = t % 32].
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dbsn_mlp_kernels.h"

namespace dbsn {

typedef float floatx16 __attribute__((ext_vector_type(16)));
constexpr int kBatchTile = 128;         // samples and neurons per workgroup tile
constexpr int kBatchK = 16;             // k-chunk staged in LDS
constexpr int kBatchPitch = kBatchK + 1;
constexpr int kBatchThreads = 256;
constexpr int kBatchRows = kBatchTile * kBatchK / kBatchThreads;   // elements of each operand tile a thread stages per chunk
constexpr int kBatchSamples = 8192;     // samples per pass through the layers (sizes the activation buffers)

// Y[s][j] = f(b[j] + sum_i W[j][i] X[s][i]) for s < S, j < n_out; f = scaled tanh (ACT) or identity
// (the output layer's pre-activations, whose largest entry is the class).  X: [S][ldx], W: [n_out][ldw],
// Y: [S][ldy].
template <bool ACT>
__global__ __launch_bounds__(kBatchThreads) void k_layer_batch(const float* __restrict__ X, int ldx, int S,
                                                                const float* __restrict__ W, int ldw,
                                                                const float* __restrict__ b, int n_in, int n_out,
                                                                float* __restrict__ Y, int ldy) {
    __shared__ float Xs[2][kBatchTile * kBatchPitch];
    __shared__ float Ws[2][kBatchTile * kBatchPitch];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s0 = blockIdx.y * kBatchTile, j0 = blockIdx.x * kBatchTile;
    const int sw = (wave & 1) * 64, jw = (wave >> 1) * 64;
    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;
    // staging: column tk of rows tr, tr + 16, ...
    const int tk = threadIdx.x & (kBatchK - 1), tr = threadIdx.x / kBatchK;
    constexpr int kRowStep = kBatchThreads / kBatchK;
    float xr[kBatchRows], wrg[kBatchRows];
    // element offsets of this thread's first staged row (32-bit: a pass holds fewer than 2^31 floats);
    // rows further down are a uniform stride away, the chunk moves the uniform base
    const unsigned xoff = (unsigned)(s0 + tr) * (unsigned)ldx + (unsigned)tk;
    const unsigned woff = (unsigned)(j0 + tr) * (unsigned)ldw + (unsigned)tk;
    const unsigned xstep = (unsigned)kRowStep * (unsigned)ldx, wstep = (unsigned)kRowStep * (unsigned)ldw;
    auto fetch = [&](int k0) {
        const bool kin = k0 + tk < n_in;
        const float* __restrict__ Xk = X + k0;
        const float* __restrict__ Wk = W + k0;
#pragma unroll
        for (int r = 0; r < kBatchRows; ++r) {
            const int row = tr + kRowStep * r;
            xr[r] = (kin && s0 + row < S) ? Xk[xoff + (unsigned)r * xstep] : 0.0f;
            wrg[r] = (kin && j0 + row < n_out) ? Wk[woff + (unsigned)r * wstep] : 0.0f;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int r = 0; r < kBatchRows; ++r) {
            const int row = tr + kRowStep * r;
            Xs[buf][row * kBatchPitch + tk] = xr[r];
            Ws[buf][row * kBatchPitch + tk] = wrg[r];
        }
    };
    const int nchunks = (n_in + kBatchK - 1) / kBatchK;
    fetch(0);
    stage(0);
    __syncthreads();
    if (nchunks > 1) fetch(kBatchK);
    for (int c = 0; c < nchunks; ++c) {
        const int cur = c & 1;
        // the other buffer was last read one chunk ago, before the barrier every wavefront has passed
        if (c + 1 < nchunks) stage(cur ^ 1);
        if (c + 2 < nchunks) fetch((c + 2) * kBatchK);   // in flight during the matrix instructions below
        const float* xs = Xs[cur];
        const float* ws = Ws[cur];
#pragma unroll
        for (int kk = 0; kk < kBatchK; kk += 2) {
            const int kc = kk + (lane >> 5);
            const float a0 = xs[(sw + (lane & 31)) * kBatchPitch + kc];
            const float a1 = xs[(sw + 32 + (lane & 31)) * kBatchPitch + kc];
            const float w0 = ws[(jw + (lane & 31)) * kBatchPitch + kc];
            const float w1 = ws[(jw + 32 + (lane & 31)) * kBatchPitch + kc];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, w0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, w1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, w0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, w1, acc[1][1], 0, 0, 0);
        }
        __syncthreads();
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int j = j0 + jw + 32 * c + (lane & 31);
        if (j < n_out) {
            const float bj = b[j];
#pragma unroll
            for (int a = 0; a < 2; ++a) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int s = s0 + sw + 32 * a + (r & 3) + 4 * (lane >> 5) + 8 * (r >> 2);
                    if (s < S) {
                        const float v = acc[a][c][r] + bj;
                        Y[(size_t)s * ldy + j] = ACT ? act_fast(v) : v;
                    }
                }
            }
        }
    }
}

// Output layer of the classification pass: labels[s] = index of the largest pre-activation
// b[c] + sum_i W[c][i] X[s][i] over the classes (the lowest index on ties).  The layer has only a
// few rows, so it is no job for 128-wide tiles: one wavefront per sample, lanes over the inputs,
// classes 16 at a time in registers, sums over the lanes on the vector ALU.
__global__ __launch_bounds__(kBatchThreads) void k_top_batch(const float* __restrict__ X, int ldx, int S,
                                                              const float* __restrict__ W, int ldw,
                                                              const float* __restrict__ b, int n_in, int n_out,
                                                              int* __restrict__ labels) {
    const int lane = threadIdx.x & 63;
    const int s = blockIdx.x * (kBatchThreads / 64) + (threadIdx.x >> 6);
    if (s >= S) return;
    const float* x = X + (size_t)s * ldx;
    int best = 0;
    float bv = 0.0f;
    for (int c0 = 0; c0 < n_out; c0 += 16) {
        float acc[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) acc[c] = 0.0f;
        for (int i = lane; i < n_in; i += 64) {
            const float xi = x[i];
#pragma unroll
            for (int c = 0; c < 16; ++c)
                if (c0 + c < n_out) acc[c] = fmaf(W[(size_t)(c0 + c) * ldw + i], xi, acc[c]);
        }
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            if (c0 + c < n_out) {   // (uniform)
                float v = acc[c];
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
                v += b[c0 + c];
                if ((c0 + c == 0) || v > bv) { bv = v; best = c0 + c; }
            }
        }
    }
    if (lane == 0) labels[s] = best;
}

}  // namespace dbsn
