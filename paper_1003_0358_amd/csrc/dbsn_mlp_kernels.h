// MLP kernels of libdbsn for gfx950: forward mat-vec + activation, fused backward
// (W^T delta + rank-1 update in one sweep) and output layer, one launch per layer phase.  (The
// persistent kernel that runs whole calls in one launch is in dbsn_persistent_kernel.h.)
//
// Layout.  Layer l (1..L) keeps W_l output-major: row j = the n_{l-1} incoming weights of
// neuron j, rows padded to `ld` (a multiple of 4 floats, so every row starts 16-byte aligned and
// is read with 128-bit loads); pad columns hold 0 and stay 0.  Biases live in their own vector.
//
// Work split.  The launch has G workgroups of kThreads threads (8 wavefronts of 64 lanes).
// Workgroup g owns the contiguous rows [g*n/G, (g+1)*n/G) of every layer, in the forward AND in
// the backward sweep, so a weight is only ever touched by one workgroup (hence one XCD's L2).
// Inside a workgroup rows are dealt round-robin to wavefronts; a wavefront handles one row at a
// time, lane t holding columns 256k + 4t .. 4t+3 (k = 0 .. NCH-1).  Because a lane always sees
// the same columns, its slice of the input vector x_{l-1} and its slice of the W^T delta
// accumulator stay in registers for the whole phase; the forward sweep needs one wavefront
// reduction per row, the backward sweep none.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dbsn_plan.h"
#include "dbsn_rng.h"

namespace dbsn {

constexpr float kA = 1.7159f;  // y(a) = A tanh(B a), section "Architectures"
constexpr float kB = 0.6666f;

struct Layer {
    float* W;   // [n_out][ld]
    float* b;   // [n_out]
    float* x;   // [n_out] outputs of this layer (activations; softmax probabilities for layer L)
    float* d;   // [n_out] deltas of the last bp step
    int n_in, n_out, ld, nch;
};

struct Net {
    Layer lay[kMaxLayers + 1];  // 1 .. L
    float* gpart[2];            // partial W^T delta rows, [G][gld] each; layer l reads gpart[l & 1]
    int L, G, gld;
};

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ inline float act(float a) { return kA * tanhf(kB * a); }
// y(a) = A tanh(B a) without the library routine: tanh(t) = 1 - 2 / (exp(2t) + 1) away from zero,
// the odd Taylor polynomial up to t^7 below |t| = 0.125 (where the first form would cancel); the
// quotient through the hardware reciprocal (one ulp, a tenth of the instructions of a division).
// Absolute error below 4e-7 on the whole axis.
__device__ inline float act_fast(float a) {
    const float t = kB * a;
    const float at = fabsf(t);
    const float e = __expf(2.0f * at);
    const float big = fmaf(-2.0f, __builtin_amdgcn_rcpf(e + 1.0f), 1.0f);
    const float t2 = t * t;
    const float small = at * fmaf(t2, fmaf(t2, fmaf(t2, -17.0f / 315.0f, 2.0f / 15.0f), -1.0f / 3.0f), 1.0f);
    const float r = (at < 0.125f) ? small : big;
    return kA * copysignf(r, t);
}

// derivative from the stored output, as the appendix's delta kernel takes it from the state
__device__ inline float dact_from_y(float y) { return (kB / kA) * (kA * kA - y * y); }
__device__ inline int row_begin(int g, int n, int G) { return (int)(((long long)g * n) / G); }

template <int NCH>
__device__ inline void stage_x(float* xs, const float* __restrict__ xin, int n_in) {
    for (int i = threadIdx.x; i < NCH * 256; i += kThreads) xs[i] = (i < n_in) ? xin[i] : 0.0f;
}

template <int NCH>
__device__ inline void load_row(float4 (&w)[NCH], const float* __restrict__ wrow, int ld, int lane) {
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        const int col = k * 256 + lane * 4;
        w[k] = (col < ld) ? *reinterpret_cast<const float4*>(wrow + col) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// Forward propagation of one hidden layer (appendix "Forward propagation"):
// x_l[j] = A tanh(B (b_l[j] + sum_i W_l[j][i] x_{l-1}[i])) for the rows of workgroup g.
template <int NCH>
__device__ void fwd_phase(const Layer& Ly, const float* __restrict__ xin, float* lds, int g, int G) {
    float* xs = lds;
    stage_x<NCH>(xs, xin, Ly.n_in);
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float4 xr[NCH];
#pragma unroll
    for (int k = 0; k < NCH; ++k) xr[k] = *reinterpret_cast<const float4*>(xs + k * 256 + lane * 4);
    const int re = row_begin(g + 1, Ly.n_out, G);
    int r = row_begin(g, Ly.n_out, G) + wave;
    float4 wa[NCH], wb[NCH];
    if (r < re) load_row<NCH>(wa, Ly.W + (size_t)r * Ly.ld, Ly.ld, lane);
    for (; r < re; r += kWaves) {
        const int rn = r + kWaves;
        if (rn < re) load_row<NCH>(wb, Ly.W + (size_t)rn * Ly.ld, Ly.ld, lane);
        float acc = 0.0f;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            acc = fmaf(wa[k].x, xr[k].x, acc);
            acc = fmaf(wa[k].y, xr[k].y, acc);
            acc = fmaf(wa[k].z, xr[k].z, acc);
            acc = fmaf(wa[k].w, xr[k].w, acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) Ly.x[r] = act(acc + Ly.b[r]);
#pragma unroll
        for (int k = 0; k < NCH; ++k) wa[k] = wb[k];
    }
    __syncthreads();  // xs is reused by the next phase
}

// Fused backward sweep of layer l (appendix "Backward propagation" and "Weight updating", done in
// one pass): for the rows j of workgroup g
//   delta_l[j]   = (sum_p gsrc[p][j]) * f'(x_l[j])          (partials of the layer above)
//   gacc[i]     += W_l[j][i] * delta_l[j]                   (old weight, before the update)
//   W_l[j][i]   -= eta * delta_l[j] * x_{l-1}[i];  b_l[j] -= eta * delta_l[j]
// and the workgroup's partial row gdst[i] = sum over its rows of W_l[j][i] delta_l[j]
// (gdst == nullptr for the first layer, which has nothing below it).
template <int NCH>
__device__ void bwd_phase(const Layer& Ly, const float* __restrict__ xin, float eta, const float* gsrc, int P,
                          int gsrc_ld, float* __restrict__ gdst, float* lds, int g, int G) {
    float* xs = lds;
    float* dl = xs + NCH * 256;
    float* gred = dl + kMaxRowsPerGroup;  // [kWaves][NCH*256]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    stage_x<NCH>(xs, xin, Ly.n_in);
    const int rb = row_begin(g, Ly.n_out, G), re = row_begin(g + 1, Ly.n_out, G);
    for (int r = rb + wave; r < re; r += kWaves) {
        float s = 0.0f;
        for (int p = lane; p < P; p += 64) s += gsrc[(size_t)p * gsrc_ld + r];
        s = wave_sum(s);
        if (lane == 0) {
            const float d = s * dact_from_y(Ly.x[r]);
            dl[r - rb] = d;
            Ly.d[r] = d;
        }
    }
    __syncthreads();
    float4 xr[NCH], gacc[NCH];
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        xr[k] = *reinterpret_cast<const float4*>(xs + k * 256 + lane * 4);
        gacc[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    int r = rb + wave;
    float4 wa[NCH], wb[NCH];
    if (r < re) load_row<NCH>(wa, Ly.W + (size_t)r * Ly.ld, Ly.ld, lane);
    for (; r < re; r += kWaves) {
        const int rn = r + kWaves;
        if (rn < re) load_row<NCH>(wb, Ly.W + (size_t)rn * Ly.ld, Ly.ld, lane);
        const float d = dl[r - rb];
        const float ed = eta * d;
        float* wrow = Ly.W + (size_t)r * Ly.ld;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            const int col = k * 256 + lane * 4;
            float4 w = wa[k];
            gacc[k].x = fmaf(w.x, d, gacc[k].x);
            gacc[k].y = fmaf(w.y, d, gacc[k].y);
            gacc[k].z = fmaf(w.z, d, gacc[k].z);
            gacc[k].w = fmaf(w.w, d, gacc[k].w);
            w.x = fmaf(-ed, xr[k].x, w.x);
            w.y = fmaf(-ed, xr[k].y, w.y);
            w.z = fmaf(-ed, xr[k].z, w.z);
            w.w = fmaf(-ed, xr[k].w, w.w);
            if (col < Ly.ld) *reinterpret_cast<float4*>(wrow + col) = w;
        }
        if (lane == 0) Ly.b[r] -= ed;
#pragma unroll
        for (int k = 0; k < NCH; ++k) wa[k] = wb[k];
    }
    if (gdst != nullptr) {
#pragma unroll
        for (int k = 0; k < NCH; ++k)
            *reinterpret_cast<float4*>(gred + wave * (NCH * 256) + k * 256 + lane * 4) = gacc[k];
        __syncthreads();
        for (int i = threadIdx.x; i < Ly.n_in; i += kThreads) {
            float s = 0.0f;
#pragma unroll
            for (int v = 0; v < kWaves; ++v) s += gred[v * (NCH * 256) + i];
            gdst[i] = s;
        }
    }
    __syncthreads();
}

// LDS words a phase of chunk count NCH needs.
__host__ __device__ constexpr int phase_lds_floats(int nch) {
    return nch * 256 + kMaxRowsPerGroup + kWaves * nch * 256 + 2 * kMaxClasses + 16;
}

// Output layer (the 10-way softmax the project fixes for the paper's unnamed output unit):
// logits a = W_L x + b, p = softmax(a), loss = -log p[label], delta_L = p - onehot(label),
// g[i] = sum_j W_L[j][i] delta_L[j] for the layer below, and (do_update) the rank-1 update of W_L.
// Runs in ONE workgroup; `top` points at 2*kMaxClasses floats of LDS that keep delta_L afterwards.
__device__ void top_phase(const Layer& Ly, const float* __restrict__ xin, int label, float eta, bool do_update,
                          bool publish, float* loss_out, int* label_out, float* gdst, float* xs, float* top) {
    float* logit = top;
    float* dL = top + kMaxClasses;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_in = Ly.n_in, n_out = Ly.n_out, ld = Ly.ld;
    for (int i = threadIdx.x; i < n_in; i += kThreads) xs[i] = xin[i];
    __syncthreads();
    for (int j = wave; j < n_out; j += kWaves) {
        const float* wrow = Ly.W + (size_t)j * ld;
        float acc = 0.0f;
        for (int i = lane; i < n_in; i += 64) acc = fmaf(wrow[i], xs[i], acc);
        acc = wave_sum(acc);
        if (lane == 0) logit[j] = acc + Ly.b[j];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = logit[0];
        int best = 0;
        for (int k = 1; k < n_out; ++k)
            if (logit[k] > m) { m = logit[k]; best = k; }
        float s = 0.0f;
        for (int k = 0; k < n_out; ++k) { dL[k] = expf(logit[k] - m); s += dL[k]; }
        float pl = 0.0f;
        for (int k = 0; k < n_out; ++k) {
            const float p = dL[k] / s;
            if (k == label) pl = p;
            if (publish) Ly.x[k] = p;
            dL[k] = p - (k == label ? 1.0f : 0.0f);
            if (publish && do_update) Ly.d[k] = dL[k];   // (a forward-only call leaves the last step's deltas alone)
        }
        if (publish && loss_out) *loss_out = -logf(pl);
        if (publish && label_out) *label_out = best;
    }
    __syncthreads();
    if (gdst != nullptr || do_update) {
        for (int i = threadIdx.x; i < n_in; i += kThreads) {
            float gsum = 0.0f;
            const float xi = xs[i];
            for (int j = 0; j < n_out; ++j) {
                const float w = Ly.W[(size_t)j * ld + i];
                gsum = fmaf(w, dL[j], gsum);
                if (do_update) Ly.W[(size_t)j * ld + i] = fmaf(-(eta * dL[j]), xi, w);
            }
            if (gdst != nullptr) gdst[i] = gsum;
        }
        if (do_update && (int)threadIdx.x < n_out) Ly.b[threadIdx.x] -= eta * dL[threadIdx.x];
    }
    __syncthreads();
}

#define DBSN_NCH_SWITCH(MAXNCH, nch, CALL)                          \
    switch (nch) {                                                  \
        case 1:  { constexpr int N = 1;  CALL; } break;             \
        case 2:  { constexpr int N = 2;  CALL; } break;             \
        case 3:  { constexpr int N = 3;  CALL; } break;             \
        case 4:  { constexpr int N = 4;  CALL; } break;             \
        case 5:  if constexpr (MAXNCH >= 5)  { constexpr int N = 5;  CALL; } break;  \
        case 6:  if constexpr (MAXNCH >= 6)  { constexpr int N = 6;  CALL; } break;  \
        case 8:  if constexpr (MAXNCH >= 8)  { constexpr int N = 8;  CALL; } break;  \
        case 10: if constexpr (MAXNCH >= 10) { constexpr int N = 10; CALL; } break;  \
        case 12: if constexpr (MAXNCH >= 12) { constexpr int N = 12; CALL; } break;  \
        case 16: if constexpr (MAXNCH >= 16) { constexpr int N = 16; CALL; } break;  \
        default: break;                                             \
    }

// ---- one kernel per phase (DBSN_MODE_LAUNCHES) --------------------------------------------

template <int NCH>
__global__ __launch_bounds__(kThreads) void k_fwd(Net net, int l, const float* x0) {
    extern __shared__ float lds[];
    const float* xin = (l == 1) ? x0 : net.lay[l - 1].x;
    fwd_phase<NCH>(net.lay[l], xin, lds, blockIdx.x, gridDim.x);
}

__global__ __launch_bounds__(kThreads) void k_top(Net net, const float* x0, const int* label_ptr, int label_val,
                                                   float eta, int train, float* loss_out, int* label_out) {
    extern __shared__ float lds[];
    const int L = net.L;
    const Layer& Ly = net.lay[L];
    int label = label_ptr ? *label_ptr : label_val;
    label = label < 0 ? 0 : (label >= Ly.n_out ? Ly.n_out - 1 : label);
    const float* xin = (L == 1) ? x0 : net.lay[L - 1].x;
    float* xs = lds;
    float* top = lds + Ly.ld + 4;
    float* gdst = (train && L > 1) ? net.gpart[(L - 1) & 1] : nullptr;
    top_phase(Ly, xin, label, eta, train != 0, true, loss_out, label_out, gdst, xs, top);
}

template <int NCH>
__global__ __launch_bounds__(kThreads) void k_bwd(Net net, int l, const float* x0, float eta) {
    extern __shared__ float lds[];
    const float* xin = (l == 1) ? x0 : net.lay[l - 1].x;
    const int P = (l == net.L - 1) ? 1 : net.G;  // the output layer leaves a single row
    float* gdst = (l > 1) ? net.gpart[(l - 1) & 1] + (size_t)blockIdx.x * net.gld : nullptr;
    bwd_phase<NCH>(net.lay[l], xin, eta, net.gpart[l & 1], P, net.gld, gdst, lds, blockIdx.x, gridDim.x);
}

// ---- initialisation (section "Architectures": weights uniform in [-0.05, 0.05)) ------------
// Layer l uses stream l; W[j][i] takes counter j*(n_in+1)+i, the bias b[j] counter j*(n_in+1)+n_in.
__global__ void k_init_layer(Layer Ly, uint64_t key) {
    const float scale = 0.05f / 8388608.0f;
    const long long total = (long long)Ly.n_out * (Ly.ld + 1);
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (long long)gridDim.x * blockDim.x) {
        const int j = (int)(t / (Ly.ld + 1)), i = (int)(t % (Ly.ld + 1));
        if (i == Ly.ld) {
            const uint64_t r = rng_draw(key, (uint64_t)j * (uint64_t)(Ly.n_in + 1) + (uint64_t)Ly.n_in);
            Ly.b[j] = (float)rng_i24(r) * scale;
        } else if (i < Ly.n_in) {
            const uint64_t r = rng_draw(key, (uint64_t)j * (uint64_t)(Ly.n_in + 1) + (uint64_t)i);
            Ly.W[(size_t)j * Ly.ld + i] = (float)rng_i24(r) * scale;
        } else {
            Ly.W[(size_t)j * Ly.ld + i] = 0.0f;
        }
    }
}

}  // namespace dbsn
