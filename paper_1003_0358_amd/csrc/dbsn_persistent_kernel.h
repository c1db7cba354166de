// Persistent on-line back-propagation kernel of libdbsn for gfx950: n strictly sequential
// batch-size-1 steps in ONE launch, with no grid barrier and no kernel boundary between layers.
//
// Why it looks like this.  A step of the paper's big nets moves 144 MB of weights but is a chain
// of 2L dependent mat-vec phases; on this chip a kernel boundary or a grid-wide barrier costs
// 2-4 us, as much as streaming a whole layer.  So the phases are connected by DATAFLOW instead:
//
//  * Every layer l is cut into tiles of R_l rows x C_l <= 256 columns; tile (cb, rb) belongs to
//    workgroup g = rb * nCB_l + cb for the whole life of the network, forward and backward, so a
//    weight is only ever touched by one workgroup (plain cached loads and stores, one XCD's L2).
//  * What crosses workgroups is small: forward, a tile publishes its R partial dot products
//    yp_l[cb][rows]; backward, its C partial sums gp_{l-1}[rb][cols] of W^T delta.  Each value
//    travels as ONE 64-bit word {step tag, float} written with a device-scope atomic store, and a
//    consumer simply polls the words it needs until they carry the current step's tag: the data
//    is its own flag.  No fence, no L2 write-back, no counter that 256 workgroups hammer.
//  * A consumer adds the partials in index order (deterministic, bit-reproducible), applies the
//    activation (forward) or its derivative (backward) itself, and goes on.
//  * Buffers alternate with the parity of the step tag; the output layer needs all of x_{L-1},
//    hence every tile of the step, which keeps any workgroup from running two steps ahead.
//  * The 10 x n_{L-1} output layer lives in every workgroup's LDS; each workgroup evaluates it
//    and applies the same update to its private copy (same code, same inputs, same bits), so the
//    deltas of the last hidden layer are available everywhere without communication.
//  * A wavefront holds all its rows of a tile in registers (one 128-bit load per row and lane,
//    issued BEFORE the wait for the inputs, so the weight stream overlaps the wait).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dbsn_mlp_kernels.h"

namespace dbsn {

typedef unsigned long long u64;

constexpr int kPGroups = 256;        // workgroups of the persistent kernel (tile geometry is fixed for it)
constexpr int kKR = 12;              // rows a wavefront keeps in registers at a time
constexpr int kStageFloats = 8192;   // LDS staging for polled partials
constexpr int kTopWMax = 12288;      // floats of W_L kept in LDS
constexpr int kTopXMax = 4096;

struct PLayer {
    float* W; float* b; float* x; float* d;
    u64* yp;          // [2][nCB][n_out]   forward partial sums of this layer's rows
    u64* gp;          // [2][gP][n_out]    partial W^T delta for this layer's neurons (from layer l+1)
    int n_in, n_out, ld;
    int nCB, nRB, C, R;
    int gP;           // number of partial rows in gp = nRB of layer l+1
};

struct PNet {
    PLayer lay[kMaxLayers + 1];
    int* err;
    int L;
    unsigned spin_limit;
};

// LDS map (floats)
struct PLds {
    static constexpr int WL = 0;                                  // [kTopWMax]
    static constexpr int bL = WL + kTopWMax;                      // [kMaxClasses]
    static constexpr int logit = bL + kMaxClasses;                // [kMaxClasses]
    static constexpr int dL = logit + kMaxClasses;                // [kMaxClasses]
    static constexpr int xkeep = dL + kMaxClasses;                // [kMaxLayers + 1][256]
    static constexpr int stage = xkeep + (kMaxLayers + 1) * 256;  // [kStageFloats]
    static constexpr int dl = stage + kStageFloats;               // [256]
    static constexpr int ysum = dl + 256;                         // [256]
    static constexpr int gred = ysum + 256;                       // [kWaves][256]
    static constexpr int xtop = gred + kWaves * 256;              // [kTopXMax]
    static constexpr int dtop = xtop + kTopXMax;                  // [kTopXMax]
    static constexpr int total = dtop + kTopXMax;
};

__device__ inline u64 pack_tagged(float v, unsigned tag) { return ((u64)tag << 32) | (u64)__float_as_uint(v); }

// Wait for P x len tagged words src[p * stride + j] (p < P, j < len) of step `tag` and put their
// float payloads at stage[p * len + j].  Each thread keeps up to 4 loads in flight and re-reads
// only what was not there yet.  Returns false when the spin limit ran out.
__device__ inline bool poll_to_lds(const u64* src, int P, int len, size_t stride, unsigned tag, float* stage,
                                   unsigned limit) {
    const int total = P * len;
    bool ok = true;
    for (int e0 = threadIdx.x; e0 < total && ok; e0 += kThreads * 4) {
        const u64* a[4];
        int e[4];
        bool need[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            e[k] = e0 + k * kThreads;
            need[k] = e[k] < total;
            const int p = need[k] ? e[k] / len : 0;
            const int j = need[k] ? e[k] - p * len : 0;
            a[k] = src + (size_t)p * stride + j;
        }
        unsigned spins = 0;
        for (;;) {
            u64 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (need[k]) v[k] = __hip_atomic_load(a[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            bool pending = false;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (need[k]) {
                    if ((unsigned)(v[k] >> 32) == tag) {
                        stage[e[k]] = __uint_as_float((unsigned)v[k]);
                        need[k] = false;
                    } else {
                        pending = true;
                    }
                }
            if (!pending) break;
            if (++spins > limit) { ok = false; break; }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    return ok;
}

// true when every thread of the workgroup succeeded; otherwise raises the error flag
__device__ inline bool all_ok(bool ok, int* err) {
    const int r = __syncthreads_and(ok ? 1 : 0);
    if (!r && threadIdx.x == 0) __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return r != 0;
}

struct TileCtx {
    int cb, rb, c0, r0, Ceff, Reff;
    bool lane_on;
    const float* wbase;   // &W[r0][c0 + 4 * lane]
};

__device__ inline bool tile_ctx(const PLayer& Ly, int g, TileCtx& t) {
    if (g >= Ly.nCB * Ly.nRB) return false;
    const int lane = threadIdx.x & 63;
    t.cb = g % Ly.nCB;
    t.rb = g / Ly.nCB;
    t.c0 = t.cb * Ly.C;
    t.r0 = t.rb * Ly.R;
    t.Ceff = min(Ly.C, Ly.n_in - t.c0);
    t.Reff = min(Ly.R, Ly.n_out - t.r0);
    t.lane_on = (4 * lane < Ly.C) && (t.c0 + 4 * lane < Ly.ld);
    t.wbase = Ly.W + (size_t)t.r0 * Ly.ld + t.c0 + 4 * lane;
    return true;
}

// rows [first, first + 8 * kKR) of the tile, dealt round-robin to the 8 wavefronts
__device__ inline void load_rows(float4 (&w)[kKR], const TileCtx& t, int ld, int first) {
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < kKR; ++k) {
        const int rl = first + wave + kWaves * k;
        w[k] = (rl < t.Reff && t.lane_on) ? *reinterpret_cast<const float4*>(t.wbase + (size_t)rl * ld)
                                          : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// Forward propagation of this workgroup's tile of layer l (appendix "Forward propagation"):
// partial sums of the rows over the tile's columns, the bias riding on column block 0.
__device__ bool p_fwd_tile(const PNet& net, int l, int g, const float* __restrict__ x0, unsigned tag, float* lds) {
    const PLayer& Ly = net.lay[l];
    TileCtx t;
    if (!tile_ctx(Ly, g, t)) return true;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    float4 w[kKR];
    load_rows(w, t, Ly.ld, 0);  // in flight while the inputs are awaited

    float* xk = lds + PLds::xkeep + l * 256;
    if (l == 1) {
        if (threadIdx.x < 256) xk[threadIdx.x] = (threadIdx.x < t.Ceff) ? x0[t.c0 + threadIdx.x] : 0.0f;
    } else {
        const PLayer& Lp = net.lay[l - 1];
        float* stage = lds + PLds::stage;
        const u64* src = Lp.yp + (size_t)par * Lp.nCB * Lp.n_out + t.c0;
        const bool ok = poll_to_lds(src, Lp.nCB, t.Ceff, (size_t)Lp.n_out, tag, stage, net.spin_limit);
        if (!all_ok(ok, net.err)) return false;
        if (threadIdx.x < 256) {
            float s = 0.0f;
            if (threadIdx.x < t.Ceff) {
                for (int p = 0; p < Lp.nCB; ++p) s += stage[p * t.Ceff + threadIdx.x];
                s = act(s);
            }
            xk[threadIdx.x] = s;
        }
    }
    __syncthreads();
    const float4 x4 = *reinterpret_cast<const float4*>(xk + 4 * lane);
    float* ysum = lds + PLds::ysum;
    for (int first = 0; first < t.Reff; first += kWaves * kKR) {
        if (first > 0) load_rows(w, t, Ly.ld, first);
#pragma unroll
        for (int k = 0; k < kKR; ++k) {
            const int rl = first + wave + kWaves * k;
            float acc = w[k].x * x4.x;
            acc = fmaf(w[k].y, x4.y, acc);
            acc = fmaf(w[k].z, x4.z, acc);
            acc = fmaf(w[k].w, x4.w, acc);
            acc = wave_sum(acc);
            if (lane == 0 && rl < t.Reff) ysum[rl] = (t.cb == 0) ? acc + Ly.b[t.r0 + rl] : acc;
        }
    }
    __syncthreads();
    u64* dst = Ly.yp + (size_t)par * Ly.nCB * Ly.n_out + (size_t)t.cb * Ly.n_out + t.r0;
    for (int j = threadIdx.x; j < t.Reff; j += kThreads)
        __hip_atomic_store(dst + j, pack_tagged(ysum[j], tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// Fused backward sweep of this workgroup's tile of layer l (appendix "Backward propagation" and
// "Weight updating" in one pass over the tile): deltas of the tile's rows, partial W^T delta of
// its columns from the OLD weights, rank-1 update of the tile.
__device__ bool p_bwd_tile(const PNet& net, int l, int g, float eta, unsigned tag, float* lds) {
    const PLayer& Ly = net.lay[l];
    TileCtx t;
    if (!tile_ctx(Ly, g, t)) return true;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    float4 w[kKR];
    load_rows(w, t, Ly.ld, 0);

    float* dl = lds + PLds::dl;
    if (l == net.L - 1) {
        // the output layer was evaluated in this workgroup: its deltas are already in LDS
        for (int j = threadIdx.x; j < t.Reff; j += kThreads) {
            dl[j] = lds[PLds::dtop + t.r0 + j];
            if (t.cb == 0) {
                Ly.x[t.r0 + j] = lds[PLds::xtop + t.r0 + j];
                Ly.d[t.r0 + j] = dl[j];
            }
        }
    } else {
        float* sg = lds + PLds::stage;
        float* sy = lds + PLds::stage + kStageFloats / 2;
        const u64* gsrc = Ly.gp + (size_t)par * Ly.gP * Ly.n_out + t.r0;
        const u64* ysrc = Ly.yp + (size_t)par * Ly.nCB * Ly.n_out + t.r0;
        bool ok = poll_to_lds(gsrc, Ly.gP, t.Reff, (size_t)Ly.n_out, tag, sg, net.spin_limit);
        ok = poll_to_lds(ysrc, Ly.nCB, t.Reff, (size_t)Ly.n_out, tag, sy, net.spin_limit) && ok;
        if (!all_ok(ok, net.err)) return false;
        for (int j = threadIdx.x; j < t.Reff; j += kThreads) {
            float gs = 0.0f, ys = 0.0f;
            for (int p = 0; p < Ly.gP; ++p) gs += sg[p * t.Reff + j];
            for (int p = 0; p < Ly.nCB; ++p) ys += sy[p * t.Reff + j];
            const float y = act(ys);
            const float d = gs * dact_from_y(y);
            dl[j] = d;
            if (t.cb == 0) {
                Ly.x[t.r0 + j] = y;
                Ly.d[t.r0 + j] = d;
            }
        }
    }
    __syncthreads();
    const float* xk = lds + PLds::xkeep + l * 256;
    const float4 x4 = *reinterpret_cast<const float4*>(xk + 4 * lane);
    float4 gacc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int first = 0; first < t.Reff; first += kWaves * kKR) {
        if (first > 0) load_rows(w, t, Ly.ld, first);
#pragma unroll
        for (int k = 0; k < kKR; ++k) {
            const int rl = first + wave + kWaves * k;
            if (rl < t.Reff) {
                const float d = dl[rl];
                const float ed = eta * d;
                float4 v = w[k];
                gacc.x = fmaf(v.x, d, gacc.x);
                gacc.y = fmaf(v.y, d, gacc.y);
                gacc.z = fmaf(v.z, d, gacc.z);
                gacc.w = fmaf(v.w, d, gacc.w);
                v.x = fmaf(-ed, x4.x, v.x);
                v.y = fmaf(-ed, x4.y, v.y);
                v.z = fmaf(-ed, x4.z, v.z);
                v.w = fmaf(-ed, x4.w, v.w);
                if (t.lane_on)
                    *reinterpret_cast<float4*>(const_cast<float*>(t.wbase) + (size_t)rl * Ly.ld) = v;
            }
        }
    }
    if (t.cb == 0)
        for (int j = threadIdx.x; j < t.Reff; j += kThreads) Ly.b[t.r0 + j] -= eta * dl[j];
    if (l > 1) {
        float* gred = lds + PLds::gred;
        *reinterpret_cast<float4*>(gred + wave * 256 + 4 * lane) = gacc;
        __syncthreads();
        const PLayer& Lp = net.lay[l - 1];
        u64* dst = Lp.gp + (size_t)par * Lp.gP * Lp.n_out + (size_t)t.rb * Lp.n_out + t.c0;
        if (threadIdx.x < t.Ceff) {
            float s = 0.0f;
#pragma unroll
            for (int v = 0; v < kWaves; ++v) s += gred[v * 256 + threadIdx.x];
            __hip_atomic_store(dst + threadIdx.x, pack_tagged(s, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    return true;
}

// Output layer in every workgroup, on its private LDS copy of W_L: x_{L-1} from the partials,
// logits, softmax, loss, delta_L, the deltas of layer L-1 and the rank-1 update of the copy.
__device__ bool p_top(const PNet& net, int g, int label, float eta, unsigned tag, float* loss_out, float* lds) {
    const int L = net.L;
    const PLayer& Ly = net.lay[L];
    const PLayer& Lp = net.lay[L - 1];
    const int n = Ly.n_in, nc = Ly.n_out;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    float* stage = lds + PLds::stage;
    float* xtop = lds + PLds::xtop;
    float* dtop = lds + PLds::dtop;
    float* WL = lds + PLds::WL;
    float* bL = lds + PLds::bL;
    float* logit = lds + PLds::logit;
    float* dL = lds + PLds::dL;

    const u64* src = Lp.yp + (size_t)par * Lp.nCB * Lp.n_out;
    const bool ok = poll_to_lds(src, Lp.nCB, n, (size_t)Lp.n_out, tag, stage, net.spin_limit);
    if (!all_ok(ok, net.err)) return false;
    for (int i = threadIdx.x; i < n; i += kThreads) {
        float s = 0.0f;
        for (int p = 0; p < Lp.nCB; ++p) s += stage[p * n + i];
        xtop[i] = act(s);
    }
    __syncthreads();
    for (int j = wave; j < nc; j += kWaves) {
        float acc = 0.0f;
        for (int i = lane; i < n; i += 64) acc = fmaf(WL[j * n + i], xtop[i], acc);
        acc = wave_sum(acc);
        if (lane == 0) logit[j] = acc + bL[j];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = logit[0];
        for (int k = 1; k < nc; ++k) m = logit[k] > m ? logit[k] : m;
        float s = 0.0f;
        for (int k = 0; k < nc; ++k) { dL[k] = expf(logit[k] - m); s += dL[k]; }
        float pl = 0.0f;
        for (int k = 0; k < nc; ++k) {
            const float p = dL[k] / s;
            if (k == label) pl = p;
            dL[k] = p - (k == label ? 1.0f : 0.0f);
            if (g == 0) { Ly.x[k] = p; Ly.d[k] = dL[k]; }
        }
        if (g == 0 && loss_out) *loss_out = -logf(pl);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += kThreads) {
        float gs = 0.0f;
        const float xi = xtop[i];
        for (int j = 0; j < nc; ++j) {
            const float wv = WL[j * n + i];
            gs = fmaf(wv, dL[j], gs);
            WL[j * n + i] = fmaf(-(eta * dL[j]), xi, wv);
        }
        dtop[i] = gs * dact_from_y(xi);
    }
    if (threadIdx.x < nc) bL[threadIdx.x] -= eta * dL[threadIdx.x];
    __syncthreads();
    return true;
}

__global__ __launch_bounds__(kThreads) void k_bp_dataflow(PNet net, const float* samples, const int* labels,
                                                           int label_val, long long n, float eta, float* loss_out,
                                                           unsigned tag_base) {
    extern __shared__ float lds[];
    const int g = blockIdx.x, L = net.L;
    const PLayer& LyL = net.lay[L];
    const int n0 = net.lay[1].n_in;
    // private copy of the output layer
    for (int e = threadIdx.x; e < LyL.n_out * LyL.n_in; e += kThreads) {
        const int j = e / LyL.n_in, i = e - j * LyL.n_in;
        lds[PLds::WL + e] = LyL.W[(size_t)j * LyL.ld + i];
    }
    if (threadIdx.x < LyL.n_out) lds[PLds::bL + threadIdx.x] = LyL.b[threadIdx.x];
    for (int e = threadIdx.x; e < (kMaxLayers + 1) * 256; e += kThreads) lds[PLds::xkeep + e] = 0.0f;
    __syncthreads();

    bool alive = true;
    for (long long s = 0; s < n && alive; ++s) {
        const unsigned tag = tag_base + (unsigned)s + 1u;
        const float* x0 = samples + s * n0;
        int label = labels ? labels[s] : label_val;
        label = label < 0 ? 0 : (label >= LyL.n_out ? LyL.n_out - 1 : label);
        for (int l = 1; l < L && alive; ++l) alive = p_fwd_tile(net, l, g, x0, tag, lds);
        if (alive) alive = p_top(net, g, label, eta, tag, loss_out ? loss_out + s : nullptr, lds);
        for (int l = L - 1; l >= 1 && alive; --l) alive = p_bwd_tile(net, l, g, eta, tag, lds);
    }
    if (g == 0) {
        __syncthreads();
        for (int e = threadIdx.x; e < LyL.n_out * LyL.n_in; e += kThreads) {
            const int j = e / LyL.n_in, i = e - j * LyL.n_in;
            LyL.W[(size_t)j * LyL.ld + i] = lds[PLds::WL + e];
        }
        if (threadIdx.x < LyL.n_out) LyL.b[threadIdx.x] = lds[PLds::bL + threadIdx.x];
    }
}

}  // namespace dbsn
