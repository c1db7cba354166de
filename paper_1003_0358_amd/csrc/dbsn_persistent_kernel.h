// Persistent on-line back-propagation kernel of libdbsn for gfx950: n strictly sequential
// batch-size-1 steps in ONE launch, with no grid barrier and no kernel boundary between layers.
//
// Why it looks like this.  A step of the paper's big nets touches 144 MB of weights but is a chain
// of 2L dependent mat-vec phases; on this chip a kernel boundary or a grid-wide barrier costs
// 2-4 us, as much as streaming a whole layer.  So the phases are connected by DATAFLOW instead:
//
//  * Every hidden layer l is cut into tiles of R_l rows x C_l <= 256 columns; tile (cb, rb)
//    belongs to workgroup g = rb * nCB_l + cb for the whole life of the network, forward and
//    backward, so a weight is only ever touched by one workgroup (plain cached loads and stores).
//  * What crosses workgroups is small: forward, a tile publishes its R partial dot products
//    yp_l[cb][rows]; backward, its C partial sums gp_{l-1}[rb][cols] of W^T delta.  Each value
//    travels as ONE 64-bit word {step tag, float} written with a device-scope atomic store, and a
//    consumer polls the words it needs until they carry the current step's tag: the data is its
//    own flag.  No fence, no L2 write-back, no counter that 256 workgroups hammer.
//  * A consumer adds the partials in index order (deterministic, bit-reproducible), applies the
//    activation (forward) or its derivative (backward) itself, and goes on.
//  * Buffers alternate with the parity of the step tag; the output layer needs all of x_{L-1},
//    hence every tile of the step, which keeps any workgroup from running two steps ahead.
//  * The 10 x n_{L-1} output layer lives in every workgroup's LDS; each workgroup evaluates it
//    and applies the same update to its private copy (same code, same inputs, same bits), so the
//    deltas of the last hidden layer are available everywhere without communication.
//  * Weights live in REGISTERS.  A wavefront owns rows wave, wave+8, ... of a tile, one 128-bit
//    register quadruple per row and lane, in groups of four rows.  The 256 workgroups x 8
//    wavefronts x 36 quadruples hold 75 MB: when all tiles of a workgroup fit (they do for every
//    net of the paper, 48 MB at most) the weights are loaded once per launch, updated in place
//    for n steps and written back at the end ("stationary"); the memory system then carries
//    only the small tagged words, and a step costs its chain of hand-overs, not its bytes.
//    Otherwise each phase loads its tile into the same registers (the loads are issued before
//    the wait for the inputs, so they overlap it) and the backward phase stores it back.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dbsn_mlp_kernels.h"

namespace dbsn {

typedef unsigned long long u64;

// Optional per-phase time stamps for tuning (compiled out unless DBSN_PROFILE is defined).
#ifdef DBSN_PROFILE
__device__ unsigned long long* g_prof;     // [steps][slots][workgroups]
__device__ int g_prof_steps, g_prof_slots;
#define DBSN_PROF(step, slot)                                                                        \
    do {                                                                                             \
        if (threadIdx.x == 0 && (step) < g_prof_steps && (slot) < g_prof_slots)                      \
            g_prof[((size_t)(step) * g_prof_slots + (slot)) * gridDim.x + blockIdx.x] = wall_clock64(); \
    } while (0)
#define DBSN_PROF_VAL(step, slot, val)                                                               \
    do {                                                                                             \
        if (threadIdx.x == 0 && (step) < g_prof_steps && (slot) < g_prof_slots)                      \
            g_prof[((size_t)(step) * g_prof_slots + (slot)) * gridDim.x + blockIdx.x] = (val);       \
    } while (0)
#else
#define DBSN_PROF(step, slot) do { } while (0)
#define DBSN_PROF_VAL(step, slot, val) do { } while (0)
#endif
#define DBSN_PROF_SUB(step, phase, sub) DBSN_PROF(step, (phase) * 4 + (sub))

constexpr int kPGroups = 256;        // workgroups of the persistent kernel (tile geometry is fixed for it)
constexpr int kNG = 9;               // register groups of 4 rows per wavefront
constexpr int kSlots = 4 * kNG;      // rows a wavefront holds: 36 (a tile has at most 8 * 36 = 288 rows)
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
    int g0, ng;       // register groups [g0, g0 + ng) hold this layer's tile
};

struct PNet {
    PLayer lay[kMaxLayers + 1];
    int* err;
    int L;
    unsigned spin_limit;
    int backoff;      // pause between two polls of the same words, in units of 64 clocks
    int stationary;   // 1: every layer has its own register groups for the whole launch
};

// LDS map (floats)
struct PLds {
    static constexpr int WL = 0;                                  // [kTopWMax]
    static constexpr int bL = WL + kTopWMax;                      // [kMaxClasses]
    static constexpr int logit = bL + kMaxClasses;                // [kMaxClasses]
    static constexpr int dL = logit + kMaxClasses;                // [kMaxClasses]
    static constexpr int xkeep = dL + kMaxClasses;                // [kMaxLayers + 1][256]
    static constexpr int stage = xkeep + (kMaxLayers + 1) * 256;  // [kStageFloats]
    static constexpr int dl = stage + kStageFloats;               // [kSlots * kWaves]
    static constexpr int ysum = dl + kSlots * kWaves;             // [4][kSlots * kWaves]
    static constexpr int gred = ysum + 4 * kSlots * kWaves;       // [kWaves][256]
    static constexpr int xtop = gred + kWaves * 256;              // [kTopXMax]
    static constexpr int dtop = xtop + kTopXMax;                  // [kTopXMax]
    static constexpr int total = dtop + kTopXMax;
};

__device__ inline u64 pack_tagged(float v, unsigned tag) { return ((u64)tag << 32) | (u64)__float_as_uint(v); }

// Wait for tagged words of step `tag` and put their float payloads into LDS.  The words come from
// two strided sources that share the row length `len` <= 512: srcA[p * stride + j] (p < PA) lands
// at stage[p * pitch + j], srcB[p * stride + j] (p < PB) behind them at stage[(PA + p) * pitch + j]
// (PB may be 0).  Threads are laid out as rows of 2^lg >= len lanes over consecutive j, so that no
// division is needed and a wavefront reads runs of consecutive words; every thread keeps up to 8
// loads in flight, and a wavefront re-reads its batch until all of it carries the tag (the loop
// is wavefront-uniform: no divergent control flow around the loads).  Returns false when the
// spin limit ran out.
__device__ inline bool poll_to_lds(const u64* srcA, int PA, const u64* srcB, int PB, int len, size_t stride,
 unsigned tag, float* stage, int pitch, unsigned limit, int backoff,
                                   unsigned* rounds = nullptr) {
    int lg = 5;                                   // rows of 32, 64, 128 or 256 lanes
    while ((1 << lg) < len) ++lg;
    const int j = (int)threadIdx.x & ((1 << lg) - 1);
    const int prow = (int)threadIdx.x >> lg;      // first partial this thread reads
    const int pstep = kThreads >> lg;             // partials covered by one pass of the workgroup
    const int P = PA + PB;
    const bool jon = j < len;
    bool ok = true;
    for (int p0 = 0; p0 < P; p0 += 8 * pstep) {
        const u64* a[8];
        bool valid[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int p = p0 + prow + k * pstep;
            valid[k] = jon && p < P;
            const u64* base = (p < PA || !valid[k]) ? srcA : srcB;
            const int pp = !valid[k] ? 0 : (p < PA ? p : p - PA);
            a[k] = base + (size_t)pp * stride + (valid[k] ? j : 0);
        }
        u64 v[8];
        unsigned spins = 0;
        for (;;) {
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = __hip_atomic_load(a[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            bool pending = false;
#pragma unroll
            for (int k = 0; k < 8; ++k) pending |= valid[k] && ((unsigned)(v[k] >> 32) != tag);
            if (!__any(pending)) break;
            if (++spins > limit) { ok = false; break; }
            for (int z = 0; z < backoff; ++z) __builtin_amdgcn_s_sleep(1);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (valid[k]) stage[(p0 + prow + k * pstep) * pitch + j] = __uint_as_float((unsigned)v[k]);
        if (rounds) *rounds += spins + 1;
        if (!ok) break;
    }
    return ok;
}

// true when every thread of the workgroup succeeded; otherwise raises the error flag
__device__ inline bool all_ok(bool ok, int* err) {
    const int r = __syncthreads_and(ok ? 1 : 0);
    if (!r && threadIdx.x == 0) __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return r != 0;
}

// Cross-lane data movement on the vector ALU (DPP), no LDS traffic.
template <int CTRL>
__device__ inline float dpp_mov(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;   // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int kDppRor8 = 0x128;  // rotate within a row of 16 lanes by 8
constexpr int kDppRor4 = 0x124;  // ... by 4

// Sum of one value over the 64 lanes, result in every lane.
__device__ inline float wave_sum_dpp(float v) {
    v += dpp_mov<kDppXor1>(v);
    v += dpp_mov<kDppXor2>(v);
    v += dpp_mov<kDppRor4>(v);
    v += dpp_mov<kDppRor8>(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}

// Sums of four values over the 64 lanes at once: two halving steps inside every quad of lanes
// leave value (t & 3) in lane t, the remaining steps add over the 16 quads.  On return lane t
// holds the sum of a[t & 3] over its row of 16 lanes; the caller adds the four rows with two LDS
// permutes (xor 16, xor 32), which it can overlap across several groups.  13 vector ops.
__device__ inline float quad_sum4(float a0, float a1, float a2, float a3) {
    const int lane = threadIdx.x & 63;
    const bool b0 = (lane & 1) != 0, b1 = (lane & 2) != 0;
    const float s0 = (b0 ? a1 : a0) + dpp_mov<kDppXor1>(b0 ? a0 : a1);
    const float s1 = (b0 ? a3 : a2) + dpp_mov<kDppXor1>(b0 ? a2 : a3);
    float v = (b1 ? s1 : s0) + dpp_mov<kDppXor2>(b1 ? s0 : s1);
    v += dpp_mov<kDppRor4>(v);
    v += dpp_mov<kDppRor8>(v);
    return v;   // sum over this row of 16 lanes; the caller adds the four rows (xor 16, xor 32)
}

// sum over p < P of stage[p * len + j], in index order; the LDS reads go out eight at a time
__device__ inline float sum_partials(const float* stage, int P, int len, int j) {
    float s = 0.0f;
    int p = 0;
    for (; p + 8 <= P; p += 8) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = stage[(p + k) * len + j];
#pragma unroll
        for (int k = 0; k < 8; ++k) s += v[k];
    }
    if (p < P) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = (p + k < P) ? stage[(p + k) * len + j] : 0.0f;
#pragma unroll
        for (int k = 0; k < 8; ++k) s += v[k];   // adding the zeros of the tail changes nothing
    }
    return s;
}

// y(a) = A tanh(B a) without the library routine: tanh(t) = 1 - 2 / (exp(2t) + 1) away from zero,
// the odd Taylor polynomial up to t^7 below |t| = 0.125 (where the first form would cancel).
// Absolute error below 3e-7 on the whole axis.
__device__ inline float act_fast(float a) {
    const float t = kB * a;
    const float at = fabsf(t);
    const float e = __expf(2.0f * at);
    const float big = 1.0f - __fdividef(2.0f, e + 1.0f);
    const float t2 = t * t;
    const float small = at * fmaf(t2, fmaf(t2, fmaf(t2, -17.0f / 315.0f, 2.0f / 15.0f), -1.0f / 3.0f), 1.0f);
    const float r = (at < 0.125f) ? small : big;
    return kA * copysignf(r, t);
}

__device__ inline float dot4(const float4& w, const float4& x) {
    float acc = w.x * x.x;
    acc = fmaf(w.y, x.y, acc);
    acc = fmaf(w.z, x.z, acc);
    return fmaf(w.w, x.w, acc);
}

struct TileCtx {
    int cb, rb, c0, r0, Ceff, Reff;
    bool lane_on;
    float* wbase;   // &W[r0][c0 + 4 * lane]
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

// Register slot s of group G = g0 + s / 4 holds tile row wave + 8 * s.
#define DBSN_FOR_LAYER_SLOTS(Ly, BODY)                                  \
    _Pragma("unroll") for (int G_ = 0; G_ < kNG; ++G_) {                 \
        if (G_ >= g0_ && G_ < g0_ + ng_) {                               \
            const int sbase_ = 4 * (G_ - g0_);                           \
            BODY                                                         \
        }                                                                \
    }
#define DBSN_LAYER_GROUPS(Ly) const int g0_ = (Ly).g0, ng_ = (Ly).ng

__device__ __forceinline__ void load_tile(float4 (&wr)[kSlots], const PLayer& Ly, const TileCtx& t) {
    const int wave = threadIdx.x >> 6;
    DBSN_LAYER_GROUPS(Ly);
    DBSN_FOR_LAYER_SLOTS(Ly, {
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {
            const int rl = wave + kWaves * (sbase_ + q);
            wr[4 * G_ + q] = (rl < t.Reff && t.lane_on)
                                 ? *reinterpret_cast<const float4*>(t.wbase + (size_t)rl * Ly.ld)
                                 : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    })
}

__device__ __forceinline__ void store_tile(const float4 (&wr)[kSlots], const PLayer& Ly, const TileCtx& t) {
    const int wave = threadIdx.x >> 6;
    DBSN_LAYER_GROUPS(Ly);
    DBSN_FOR_LAYER_SLOTS(Ly, {
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {
            const int rl = wave + kWaves * (sbase_ + q);
            if (rl < t.Reff && t.lane_on) *reinterpret_cast<float4*>(t.wbase + (size_t)rl * Ly.ld) = wr[4 * G_ + q];
        }
    })
}

// Forward propagation of this workgroup's tile of layer l (appendix "Forward propagation"):
// partial sums of the rows over the tile's columns, the bias riding on column block 0.
__device__ __forceinline__ bool p_fwd_tile(float4 (&wr)[kSlots], const PNet& net, int l, int g,
                                           const float* __restrict__ x0, unsigned tag, float* lds, long long ps,
                                           int ph) {
    const PLayer& Ly = net.lay[l];
    TileCtx t;
    if (!tile_ctx(Ly, g, t)) return true;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    DBSN_LAYER_GROUPS(Ly);
    DBSN_PROF_SUB(ps, ph, 0);
    if (!net.stationary) load_tile(wr, Ly, t);  // in flight while the inputs are awaited

    float* xk = lds + PLds::xkeep + l * 256;
    if (l == 1) {
        if (threadIdx.x < 256) xk[threadIdx.x] = (threadIdx.x < t.Ceff) ? x0[t.c0 + threadIdx.x] : 0.0f;
    } else {
        const PLayer& Lp = net.lay[l - 1];
        float* stage = lds + PLds::stage;
        const u64* src = Lp.yp + (size_t)par * Lp.nCB * Lp.n_out + t.c0;
        unsigned rounds = 0;
        const bool ok = poll_to_lds(src, Lp.nCB, nullptr, 0, t.Ceff, (size_t)Lp.n_out, tag, stage, t.Ceff,
                                    net.spin_limit, net.backoff, &rounds);
        DBSN_PROF_VAL(ps, (2 * net.L - 1) * 4 + ph, rounds);
        DBSN_PROF(ps, (2 * net.L - 1) * 5 + ph * 3 + 0);
        if (!all_ok(ok, net.err)) return false;
        DBSN_PROF(ps, (2 * net.L - 1) * 5 + ph * 3 + 1);
        if (threadIdx.x < 256) {
            float s = 0.0f;
            if (threadIdx.x < t.Ceff) {
                s = act_fast(sum_partials(stage, Lp.nCB, t.Ceff, threadIdx.x));
                if (t.rb == 0) Lp.x[t.c0 + threadIdx.x] = s;   // state read-out (dbsn_mlp_get_activations)
            }
            xk[threadIdx.x] = s;
        }
    }
    __syncthreads();
    DBSN_PROF_SUB(ps, ph, 1);
    const float4 x4 = *reinterpret_cast<const float4*>(xk + 4 * lane);
    float* ysum = lds + PLds::ysum;
    // per group: 4 row sums transposed onto the quads, reduced inside each row of 16 lanes on the
    // vector ALU; the four rows of 16 park their sums in LDS and the publishing thread adds them
    const int lrow = lane >> 4;
    DBSN_FOR_LAYER_SLOTS(Ly, {
        const float v = quad_sum4(dot4(wr[4 * G_ + 0], x4), dot4(wr[4 * G_ + 1], x4), dot4(wr[4 * G_ + 2], x4),
                                  dot4(wr[4 * G_ + 3], x4));
        const int rl = wave + kWaves * (sbase_ + (lane & 3));
        if ((lane & 12) == 0) ysum[lrow * (kSlots * kWaves) + rl] = v;
    })
    __syncthreads();
    DBSN_PROF_SUB(ps, ph, 2);
    u64* dst = Ly.yp + (size_t)par * Ly.nCB * Ly.n_out + (size_t)t.cb * Ly.n_out + t.r0;
    for (int j = threadIdx.x; j < t.Reff; j += kThreads) {
        constexpr int kYS = kSlots * kWaves;
        float v = (ysum[j] + ysum[kYS + j]) + (ysum[2 * kYS + j] + ysum[3 * kYS + j]);
        if (t.cb == 0) v += Ly.b[t.r0 + j];
        __hip_atomic_store(dst + j, pack_tagged(v, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    DBSN_PROF_SUB(ps, ph, 3);
    return true;
}

// Fused backward sweep of this workgroup's tile of layer l (appendix "Backward propagation" and
// "Weight updating" in one pass over the tile): deltas of the tile's rows, partial W^T delta of
// its columns from the OLD weights (published first, it is what other workgroups wait for), then
// the rank-1 update of the tile.
__device__ __forceinline__ bool p_bwd_tile(float4 (&wr)[kSlots], const PNet& net, int l, int g, float eta,
                                           unsigned tag, float* lds, long long ps, int ph) {
    const PLayer& Ly = net.lay[l];
    TileCtx t;
    if (!tile_ctx(Ly, g, t)) return true;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    DBSN_LAYER_GROUPS(Ly);
    DBSN_PROF_SUB(ps, ph, 0);
    if (!net.stationary) load_tile(wr, Ly, t);

    float* dl = lds + PLds::dl;
    float* sg = lds + PLds::stage;
    if (l == net.L - 1) {
        // the output layer was evaluated in this workgroup: its deltas are already in LDS
        for (int j = threadIdx.x; j < t.Reff; j += kThreads) dl[j] = lds[PLds::dtop + t.r0 + j];
    } else {
        const u64* gsrc = Ly.gp + (size_t)par * Ly.gP * Ly.n_out + t.r0;
        unsigned rounds = 0;
        const bool ok = poll_to_lds(gsrc, Ly.gP, nullptr, 0, t.Reff, (size_t)Ly.n_out, tag, sg, t.Reff,
                                    net.spin_limit, net.backoff, &rounds);
        DBSN_PROF_VAL(ps, (2 * net.L - 1) * 4 + ph, rounds);
        if (!all_ok(ok, net.err)) return false;
        // the producers multiplied their partial sums by f'(x_l) already (they hold x_l, see below)
        for (int j = threadIdx.x; j < t.Reff; j += kThreads) dl[j] = sum_partials(sg, Ly.gP, t.Reff, j);
    }
    __syncthreads();
    DBSN_PROF_SUB(ps, ph, 1);
    const float* xk = lds + PLds::xkeep + l * 256;
    const float4 x4 = *reinterpret_cast<const float4*>(xk + 4 * lane);
    // lane s of a wavefront fetches the delta of the wavefront's s-th row; slots read it by lane index
    const int myrow = wave + kWaves * lane;
    const float dlane = (lane < kSlots && myrow < t.Reff) ? dl[myrow] : 0.0f;
    if (l > 1) {
        float4 gacc = make_float4(0.f, 0.f, 0.f, 0.f);
        DBSN_FOR_LAYER_SLOTS(Ly, {
            _Pragma("unroll") for (int q = 0; q < 4; ++q) {
                const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dlane), sbase_ + q));
                const float4 v = wr[4 * G_ + q];
                gacc.x = fmaf(v.x, d, gacc.x);
                gacc.y = fmaf(v.y, d, gacc.y);
                gacc.z = fmaf(v.z, d, gacc.z);
                gacc.w = fmaf(v.w, d, gacc.w);
            }
        })
        float* gred = lds + PLds::gred;
        *reinterpret_cast<float4*>(gred + wave * 256 + 4 * lane) = gacc;
        __syncthreads();
        const PLayer& Lp = net.lay[l - 1];
        u64* dst = Lp.gp + (size_t)par * Lp.gP * Lp.n_out + (size_t)t.rb * Lp.n_out + t.c0;
        if (threadIdx.x < t.Ceff) {
            float v[kWaves];
#pragma unroll
            for (int k = 0; k < kWaves; ++k) v[k] = gred[k * 256 + threadIdx.x];
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < kWaves; ++k) s += v[k];
            // this tile's columns are neurons of layer l-1 whose outputs it holds: fold f' in here,
            // so that the consumer's sum over row blocks is delta_{l-1} itself
            s *= dact_from_y(xk[threadIdx.x]);
            __hip_atomic_store(dst + threadIdx.x, pack_tagged(s, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    DBSN_PROF_SUB(ps, ph, 2);
    // rank-1 update w -= eta * delta_j * x_i (rows beyond the tile hold zeros and stay zero)
    DBSN_FOR_LAYER_SLOTS(Ly, {
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {
            const float ed = eta * __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dlane), sbase_ + q));
            float4 v = wr[4 * G_ + q];
            v.x = fmaf(-ed, x4.x, v.x);
            v.y = fmaf(-ed, x4.y, v.y);
            v.z = fmaf(-ed, x4.z, v.z);
            v.w = fmaf(-ed, x4.w, v.w);
            wr[4 * G_ + q] = v;
        }
    })
    if (!net.stationary) store_tile(wr, Ly, t);
    if (t.cb == 0) {
        // bias update, and the layer's deltas for dbsn_mlp_get_deltas
        for (int j = threadIdx.x; j < t.Reff; j += kThreads) {
            const float d = dl[j];
            Ly.b[t.r0 + j] -= eta * d;
            Ly.d[t.r0 + j] = d;
        }
    }
    __syncthreads();
    DBSN_PROF_SUB(ps, ph, 3);
    return true;
}

// Output layer in every workgroup, on its private LDS copy of W_L: x_{L-1} from the partials,
// logits, softmax, loss, delta_L, the deltas of layer L-1 and the rank-1 update of the copy.
// Thread i owns column i (input neuron i) of W_L: it forms the products W_L[j][i] x_i, the
// workgroup adds them per class (quads -> rows of 16 lanes on the vector ALU, then through LDS),
// and after the softmax the same thread back-propagates and updates its column.
__device__ __forceinline__ bool p_top(const PNet& net, int g, int label, float eta, unsigned tag, float* loss_out,
                                      float* lds, long long ps, int ph) {
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
    float* part = lds + PLds::gred;   // [kMaxClasses][32] partial logits: 8 wavefronts x 4 rows of 16 lanes

    DBSN_PROF_SUB(ps, ph, 0);
    const u64* src = Lp.yp + (size_t)par * Lp.nCB * Lp.n_out;
    unsigned rounds = 0;
    bool ok = true;
    for (int j0 = 0; j0 < n && ok; j0 += kThreads)
        ok = poll_to_lds(src + j0, Lp.nCB, nullptr, 0, min(kThreads, n - j0), (size_t)Lp.n_out, tag, stage + j0, n,
                         net.spin_limit, net.backoff, &rounds);
    DBSN_PROF_VAL(ps, (2 * net.L - 1) * 4 + ph, rounds);
    if (!all_ok(ok, net.err)) return false;
    DBSN_PROF_SUB(ps, ph, 1);

    // products per class, 16 classes at a time; columns beyond 512 are folded into the same thread
    for (int j0 = 0; j0 < nc; j0 += 16) {
        float acc[16];
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) acc[jj] = 0.0f;
        for (int i = threadIdx.x; i < n; i += kThreads) {
            const float xi = act_fast(sum_partials(stage, Lp.nCB, n, i));
            if (j0 == 0) {
                xtop[i] = xi;
                if (g == 0) Lp.x[i] = xi;   // state read-out (dbsn_mlp_get_activations)
            }
            float wv[16];
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) wv[jj] = (j0 + jj < nc) ? WL[(j0 + jj) * n + i] : 0.0f;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) acc[jj] = fmaf(wv[jj], xi, acc[jj]);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float v = quad_sum4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
            const int cls = j0 + 4 * q + (lane & 3);
            if ((lane & 12) == 0 && cls < nc) part[cls * 32 + wave * 4 + (lane >> 4)] = v;
        }
    }
    __syncthreads();
    DBSN_PROF_SUB(ps, ph, 2);
    if (wave == 0) {
        // logits and softmax over nc <= 64 classes, one class per lane
        float a = -3.0e38f;
        if (lane < nc) a = sum_partials(part + lane * 32, 32, 1, 0) + bL[lane];
        float m = a;
        m = fmaxf(m, dpp_mov<kDppXor1>(m));
        m = fmaxf(m, dpp_mov<kDppXor2>(m));
        m = fmaxf(m, dpp_mov<kDppRor4>(m));
        m = fmaxf(m, dpp_mov<kDppRor8>(m));
        m = fmaxf(m, __shfl_xor(m, 16, 64));
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        const float e = (lane < nc) ? expf(a - m) : 0.0f;
        if (lane < nc) logit[lane] = e;       // scratch: exponentials
        // (LDS serves one wavefront's accesses in program order: the reads below see these writes)
        const float s = sum_partials(logit, nc, 1, 0);   // index order
        const float p = e / s;
        const float d = p - (lane == label ? 1.0f : 0.0f);
        const float pl = __shfl(p, label, 64);
        if (lane < nc) {
            dL[lane] = d;
            if (g == 0) { Ly.x[lane] = p; Ly.d[lane] = d; }
        }
        if (g == 0 && lane == 0 && loss_out) *loss_out = -logf(pl);
    }
    __syncthreads();
    // deltas of layer L-1 and update of the private W_L, 16 classes at a time from registers
    for (int i = threadIdx.x; i < n; i += kThreads) {
        const float xi = xtop[i];
        float gs = 0.0f;
        for (int j0 = 0; j0 < nc; j0 += 16) {
            float wv[16], dj[16];
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const bool on = j0 + jj < nc;
                wv[jj] = on ? WL[(j0 + jj) * n + i] : 0.0f;
                dj[jj] = on ? dL[j0 + jj] : 0.0f;
            }
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                gs = fmaf(wv[jj], dj[jj], gs);
                if (j0 + jj < nc) WL[(j0 + jj) * n + i] = fmaf(-(eta * dj[jj]), xi, wv[jj]);
            }
        }
        dtop[i] = gs * dact_from_y(xi);
    }
    if (threadIdx.x < nc) bL[threadIdx.x] -= eta * dL[threadIdx.x];
    __syncthreads();
    DBSN_PROF_SUB(ps, ph, 3);
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

    float4 wr[kSlots];
#pragma unroll
    for (int s = 0; s < kSlots; ++s) wr[s] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (net.stationary) {
        for (int l = 1; l < L; ++l) {
            TileCtx t;
            if (tile_ctx(net.lay[l], g, t)) load_tile(wr, net.lay[l], t);
        }
    }
    __syncthreads();

    bool alive = true;
    for (long long s = 0; s < n && alive; ++s) {
        const unsigned tag = tag_base + (unsigned)s + 1u;
        const float* x0 = samples + s * n0;
        int label = labels ? labels[s] : label_val;
        label = label < 0 ? 0 : (label >= LyL.n_out ? LyL.n_out - 1 : label);
        for (int l = 1; l < L && alive; ++l) alive = p_fwd_tile(wr, net, l, g, x0, tag, lds, s, l - 1);
        if (alive) alive = p_top(net, g, label, eta, tag, loss_out ? loss_out + s : nullptr, lds, s, L - 1);
        for (int l = L - 1; l >= 1 && alive; --l) alive = p_bwd_tile(wr, net, l, g, eta, tag, lds, s, L + (L - 1 - l));
    }
    if (net.stationary) {
        for (int l = 1; l < L; ++l) {
            TileCtx t;
            if (tile_ctx(net.lay[l], g, t)) store_tile(wr, net.lay[l], t);
        }
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
