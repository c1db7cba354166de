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
//    register quadruple per row and lane (a lane holds four consecutive columns), in groups of
//    kGR rows.  The 256 workgroups x 8 wavefronts x kSlots quadruples hold 58 MB: when all tiles
//    of a workgroup fit (they do for every net of the paper, 48 MB at most) the weights are
//    loaded once per launch, updated in place for n steps and written back at the end
//    ("stationary"); the memory system then carries only the small tagged words, and a step
//    costs its chain of hand-overs, not its bytes.  Otherwise each phase loads its tile into the
//    same registers (the loads are issued before the wait for the inputs, so they overlap it)
//    and the backward phase stores it back.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dbsn_mlp_kernels.h"

namespace dbsn {

typedef unsigned long long u64;

// Optional per-phase time stamps for tuning (compiled out unless DBSN_PROFILE is defined): thread 0
// of every workgroup notes the shader clock in LDS for kProfSteps consecutive steps and copies the
// notes to global memory when the kernel ends, so that taking a stamp costs no memory traffic.
#ifdef DBSN_PROFILE
constexpr int kProfSteps = 4, kProfSlots = 128, kProfSubs = 8;
__device__ unsigned long long* g_prof;     // [kProfSteps][kProfSlots][workgroups]
__device__ long long g_prof_first;         // first step to record
#define DBSN_PROF_DECL unsigned long long* prof_lds_ = reinterpret_cast<unsigned long long*>(lds + PLds::total); \
                       for (int e_ = threadIdx.x; e_ < kProfSteps * kProfSlots; e_ += kThreads) prof_lds_[e_] = 0; \
                       const long long prof_first_ = g_prof_first
#define DBSN_PROF_ARGS , unsigned long long* prof_lds_, long long prof_first_
#define DBSN_PROF_PASS , prof_lds_, prof_first_
#define DBSN_PROF_VAL(step, slot, val)                                                                  \
    do {                                                                                                \
        const long long ps_ = (long long)(step) - prof_first_;                                          \
        if (threadIdx.x == 0 && ps_ >= 0 && ps_ < kProfSteps && (slot) < kProfSlots)                    \
            prof_lds_[ps_ * kProfSlots + (slot)] = (val);                                               \
    } while (0)
#define DBSN_PROF(step, slot) DBSN_PROF_VAL(step, slot, clock64())
#define DBSN_PROF_FLUSH()                                                                               \
    do {                                                                                                \
        __syncthreads();                                                                                \
        for (int e_ = threadIdx.x; e_ < kProfSteps * kProfSlots; e_ += kThreads)                        \
            g_prof[(size_t)e_ * gridDim.x + blockIdx.x] = prof_lds_[e_];                                \
    } while (0)
constexpr int kProfLdsFloats = 2 * kProfSteps * kProfSlots;
#else
#define DBSN_PROF_DECL do { } while (0)
#define DBSN_PROF_ARGS
#define DBSN_PROF_PASS
#define DBSN_PROF(step, slot) do { } while (0)
#define DBSN_PROF_VAL(step, slot, val) do { } while (0)
#define DBSN_PROF_FLUSH() do { } while (0)
constexpr int kProfLdsFloats = 0;
#endif
// (tuning only) a spin limit of all ones makes every wait accept whatever it reads: the results are
// then meaningless, the time per step is that of the local work plus one round trip per hand-over
#ifdef DBSN_PROFILE
#define DBSN_WAITING(limit) ((limit) != 0xFFFFFFFFu)
#else
#define DBSN_WAITING(limit) true
#endif
#define DBSN_PROF_SUB(step, phase, sub) DBSN_PROF(step, (phase) * 8 + (sub))

constexpr int kPGroups = 256;        // workgroups of the persistent kernel (tile geometry is fixed for it)
constexpr int kGR = 2;               // rows per register group
constexpr int kNG = 14;              // register groups per wavefront
constexpr int kSlots = kGR * kNG;    // rows a wavefront holds: 28 (a tile has at most 8 * 28 = 224 rows)
constexpr int kMaxTileRows = kSlots * kWaves;   // 224
constexpr int kTopWMax = 10240;      // floats of W_L kept in LDS
constexpr int kTopXMax = 2048;       // neurons of layer L-1 the output phase can take
constexpr int kStageFloats = 7168 - kProfLdsFloats;   // LDS staging for the partials a backward tile gathers

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
    static constexpr int WL = 0;                                  // [kTopWMax]  private copy of W_L
    static constexpr int bL = WL + kTopWMax;                      // [kMaxClasses]
    static constexpr int xkeep = bL + kMaxClasses;                // [2][kMaxLayers + 1][256] inputs of each tile, by step parity
    static constexpr int bias = xkeep + 2 * (kMaxLayers + 1) * 256;       // [kMaxLayers + 1][kMaxTileRows] (column block 0)
    static constexpr int dkeep = bias + (kMaxLayers + 1) * kMaxTileRows;  // [kMaxLayers + 1][kMaxTileRows] deltas of each tile's rows
    static constexpr int stage = dkeep + (kMaxLayers + 1) * kMaxTileRows; // [kStageFloats]
    static constexpr int ysum = stage + kStageFloats;             // [4][kMaxTileRows]; delta_L and probabilities
    static constexpr int gred = ysum + 4 * kMaxTileRows;          // [kWaves][256]; [class][33] partial logits
    static constexpr int xtop = gred + kWaves * 264;              // [kTopXMax]
    static constexpr int dtop = xtop + kTopXMax;                  // [kTopXMax]
    static constexpr int fail = dtop + kTopXMax;                  // [1] set when a wait gave up
    static constexpr int total = fail + 16;
};
static_assert(PLds::total * 4 <= 160 * 1024, "LDS map exceeds 160 KB");
static_assert(kMaxClasses * 33 <= kWaves * 264, "partial logits do not fit");

__device__ inline u64 pack_tagged(float v, unsigned tag) { return ((u64)tag << 32) | (u64)__float_as_uint(v); }
__device__ inline u64 ld_tagged(const u64* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_tagged(u64* p, float v, unsigned tag) {
    __hip_atomic_store(p, pack_tagged(v, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Workgroup barrier that orders LDS traffic only.  The workgroup's wavefronts talk to each other
// through LDS alone, so a barrier need not wait for outstanding global stores (__syncthreads()
// would, and the tagged words published for other workgroups take long to be acknowledged).
__device__ inline void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Barrier + agreement: true when every thread of the workgroup succeeded; otherwise raises the
// error flag.  (The LDS flag is never cleared: a failure ends the kernel.)
__device__ inline bool all_ok(bool ok, int* err, float* lds) {
    int* fail = reinterpret_cast<int*>(lds + PLds::fail);
    if (!ok) *fail = 1;
    lds_barrier();
    const bool bad = *fail != 0;
    if (bad && threadIdx.x == 0) __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return !bad;
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

// Gathering the partial sums a thread needs: P tagged words of step `tag`, word k at
// base + off(k), with `base` the same for the whole wavefront and off(k) a 32-bit element offset
// per lane (so that the loads can take a scalar base and one vector offset register).
// poll_issue sends the first batch of up to 16 loads; the caller may then do unrelated work while
// they are in flight; poll_finish waits until every word carries the tag (re-reading as long as
// necessary, batch after batch when P > 16) and returns the sum of the payloads of the first
// `np` <= P words in index order.  P must be the same for all lanes of a wavefront (the re-read
// loop is wavefront-uniform), np may differ: a lane that needs fewer words than its neighbours
// lets off() repeat a word it does need.
template <class OffF>
__device__ __forceinline__ void poll_issue(u64 (&v)[16], int P, const u64* base, OffF off) {
    const int nb = min(16, P);
#pragma unroll
    for (int k = 0; k < 16; ++k)
        if (k < nb) v[k] = ld_tagged(base + off(k));
}
template <class OffF>
__device__ __forceinline__ float poll_finish(u64 (&v)[16], int P, int np, const u64* base, OffF off, unsigned tag,
                                             unsigned limit, bool& ok) {
    float s = 0.0f;
    for (int p0 = 0; p0 < P; p0 += 16) {
        const int nb = min(16, P - p0);
        unsigned spins = 0;
        for (;;) {
            if (p0 > 0 || spins > 0) {
#pragma unroll
                for (int k = 0; k < 16; ++k)
                    if (k < nb) v[k] = ld_tagged(base + off(p0 + k));
            }
            bool pending = false;
#pragma unroll
            for (int k = 0; k < 16; ++k)
                if (k < nb) pending |= ((unsigned)(v[k] >> 32) != tag);
            if (!__any(pending && DBSN_WAITING(limit))) break;
            if (++spins > limit) { ok = false; break; }
        }
#pragma unroll
        for (int k = 0; k < 16; ++k)
            if (k < nb) s += (p0 + k < np) ? __uint_as_float((unsigned)v[k]) : 0.0f;
        if (!ok) break;
    }
    return s;
}

// Row layout of the staging area used by the backward phase: row j holds its P partials
// contiguously, P rounded up to a multiple of 4 and padded with zeros, rows PP floats apart with
// PP odd (bank-conflict-free both for the scattered writes and for the reads).
__device__ inline int stage_quarter(int P) { return (P + 3) >> 2; }
__device__ inline int stage_pitch(int P) { return (4 * stage_quarter(P)) | 1; }

// Wait for the tagged words src[p * stride + j] (p < P, j < len <= 256) of step `tag` and put their
// payloads at stage[j * PP + p].  NT threads (the first NT of the workgroup) form rows of
// 2^lg >= len lanes over consecutive j, so that a wavefront reads runs of consecutive words;
// NB loads in flight per thread.  A word that has arrived is not read again.
template <int NT, int NB>
__device__ __forceinline__ bool poll_rows_to_lds(const u64* src, int P, int len, unsigned stride, unsigned tag,
                                                 float* stage, unsigned limit) {
    int lg = 5;
    while ((1 << lg) < len) ++lg;
    const int j = (int)threadIdx.x & ((1 << lg) - 1);
    const int prow = (int)threadIdx.x >> lg;
    const int pstep = NT >> lg;
    const int PP = stage_pitch(P), Ppad = 4 * stage_quarter(P);
    const bool jon = j < len;
    const u64* col = src + (jon ? j : 0);
    float* row = stage + j * PP;
    bool ok = true;
    for (int p0 = prow; p0 - prow < Ppad; p0 += NB * pstep) {   // (uniform trip count over the wavefront)
        u64 v[NB];
        bool pend[NB];
        unsigned o[NB];
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int p = p0 + k * pstep;
            pend[k] = jon && p < P;
            o[k] = (unsigned)(pend[k] ? p : 0) * stride;
            v[k] = 0;
        }
        unsigned spins = 0;
        for (;;) {
#pragma unroll
            for (int k = 0; k < NB; ++k)
                if (pend[k]) v[k] = ld_tagged(col + o[k]);
            bool pending = false;
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                pend[k] = pend[k] && ((unsigned)(v[k] >> 32) != tag);
                pending |= pend[k];
            }
            if (!__any(pending && DBSN_WAITING(limit))) break;
            if (++spins > limit) { ok = false; break; }
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int p = p0 + k * pstep;
            if (jon && p < Ppad) row[p] = (p < P) ? __uint_as_float((unsigned)v[k]) : 0.0f;
        }
        if (!ok) break;
    }
    return ok;
}

// Thread (j, q), q = 0..3, adds quarter q of row j of the staging area in index order; the four
// quarter sums are then combined inside the quad of lanes as (q0 + q1) + (q2 + q3).  All four
// lanes of a quad (lanes 4a .. 4a+3 hold the same j) return the row sum.
__device__ inline float sum_row4(const float* stage, int P, int j, int q) {
    const int P4 = stage_quarter(P);
    const float* r = stage + j * stage_pitch(P) + q * P4;
    float s = 0.0f;
    for (int k0 = 0; k0 < P4; k0 += 8) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (k0 + k < P4) v[k] = r[k0 + k];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (k0 + k < P4) s += v[k];
    }
    s += dpp_mov<kDppXor1>(s);
    s += dpp_mov<kDppXor2>(s);
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

// Same idea for two values: on return lane t holds the sum of a[t & 1] over the 8 lanes of its
// row of 16 that share its parity.
__device__ inline float pair_sum2(float a0, float a1) {
    const bool b0 = (threadIdx.x & 1) != 0;
    float v = (b0 ? a1 : a0) + dpp_mov<kDppXor1>(b0 ? a0 : a1);
    v += dpp_mov<kDppXor2>(v);
    v += dpp_mov<kDppRor4>(v);
    v += dpp_mov<kDppRor8>(v);
    return v;
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

// Register slot s of group G = g0 + s / kGR holds tile row wave + 8 * s.
#define DBSN_FOR_LAYER_SLOTS(Ly, BODY)                                  \
    _Pragma("unroll") for (int G_ = 0; G_ < kNG; ++G_) {                 \
        if (G_ >= g0_ && G_ < g0_ + ng_) {                               \
            const int sbase_ = kGR * (G_ - g0_);                         \
            BODY                                                         \
        }                                                                \
    }
#define DBSN_LAYER_GROUPS(Ly) const int g0_ = (Ly).g0, ng_ = (Ly).ng

__device__ __forceinline__ void load_tile(float4 (&wr)[kSlots], const PLayer& Ly, const TileCtx& t) {
    const int wave = threadIdx.x >> 6;
    DBSN_LAYER_GROUPS(Ly);
    DBSN_FOR_LAYER_SLOTS(Ly, {
        _Pragma("unroll") for (int q = 0; q < kGR; ++q) {
            const int rl = wave + kWaves * (sbase_ + q);
            wr[kGR * G_ + q] = (rl < t.Reff && t.lane_on)
                                 ? *reinterpret_cast<const float4*>(t.wbase + (size_t)rl * Ly.ld)
                                 : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    })
}

__device__ __forceinline__ void store_tile(const float4 (&wr)[kSlots], const PLayer& Ly, const TileCtx& t) {
    const int wave = threadIdx.x >> 6;
    DBSN_LAYER_GROUPS(Ly);
    DBSN_FOR_LAYER_SLOTS(Ly, {
        _Pragma("unroll") for (int q = 0; q < kGR; ++q) {
            const int rl = wave + kWaves * (sbase_ + q);
            if (rl < t.Reff && t.lane_on) *reinterpret_cast<float4*>(t.wbase + (size_t)rl * Ly.ld) = wr[kGR * G_ + q];
        }
    })
}

// Rank-1 update of the tile held in registers, w[j][i] -= eta * delta_j * x_i (appendix "Weight
// updating").  Lane s < kSlots of the wavefront holds in `dlane` the delta of the wavefront's s-th row;
// rows beyond the tile hold zeros and get a zero delta, so they stay zero.
__device__ __forceinline__ void update_tile(float4 (&wr)[kSlots], const PLayer& Ly, const float4& x4, float dlane,
                                            float eta) {
    DBSN_LAYER_GROUPS(Ly);
    DBSN_FOR_LAYER_SLOTS(Ly, {
        _Pragma("unroll") for (int q = 0; q < kGR; ++q) {
            const float ed = eta * __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dlane), sbase_ + q));
            float4 v = wr[kGR * G_ + q];
            v.x = fmaf(-ed, x4.x, v.x);
            v.y = fmaf(-ed, x4.y, v.y);
            v.z = fmaf(-ed, x4.z, v.z);
            v.w = fmaf(-ed, x4.w, v.w);
            wr[kGR * G_ + q] = v;
        }
    })
}

// deltas of the rows of this workgroup's tile of layer l, as left by the backward phase
__device__ inline const float* tile_deltas(const PNet& net, int l, const TileCtx& t, const float* lds) {
    return (l == net.L - 1) ? lds + PLds::dtop + t.r0 : lds + PLds::dkeep + l * kMaxTileRows;
}

// Forward propagation of this workgroup's tile of layer l (appendix "Forward propagation"):
// partial sums of the rows over the tile's columns, the bias riding on column block 0.
template <bool ST>
__device__ __forceinline__ bool p_fwd_tile(float4 (&wr)[kSlots], const PNet& net, int l, int g, float x0pre,
                                           unsigned tag, bool last, float* lds, long long ps, int ph DBSN_PROF_ARGS) {
    const PLayer& Ly = net.lay[l];
    TileCtx t;
    if (!tile_ctx(Ly, g, t)) return true;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    DBSN_LAYER_GROUPS(Ly);
    DBSN_PROF_SUB(ps, ph, 0);
    if (!ST) load_tile(wr, Ly, t);  // in flight while the inputs are awaited

    float* xk = lds + PLds::xkeep + (par * (kMaxLayers + 1) + l) * 256;
    if (l == 1) {
        // the caller fetched this thread's input pixel ahead of time
        if (threadIdx.x < 256) xk[threadIdx.x] = (threadIdx.x < t.Ceff) ? x0pre : 0.0f;
        lds_barrier();
    } else {
        // thread j < Ceff gathers the nCB partial sums of its input column j, adds them in index
        // order and applies the activation: x_{l-1}[c0 + j]
        const PLayer& Lp = net.lay[l - 1];
        const bool poller = threadIdx.x < 256;
        const bool on = (int)threadIdx.x < t.Ceff;
        const u64* base = Lp.yp + (size_t)par * Lp.nCB * Lp.n_out + t.c0;
        const unsigned stride = (unsigned)Lp.n_out, col = on ? threadIdx.x : 0u;
        auto off = [=](int k) { return (unsigned)k * stride + col; };
        u64 v[16];
        bool ok = true;
        if (poller) {
            poll_issue(v, Lp.nCB, base, off);
            DBSN_PROF_SUB(ps, ph, 1);
            const float a = poll_finish(v, Lp.nCB, Lp.nCB, base, off, tag, net.spin_limit, ok);
            xk[threadIdx.x] = on ? act_fast(a) : 0.0f;
            DBSN_PROF_SUB(ps, ph, 2);
        }
        if (!all_ok(ok, net.err, lds)) return false;
    }
    DBSN_PROF_SUB(ps, ph, 3);
    const float4 x4 = *reinterpret_cast<const float4*>(xk + 4 * lane);
    float* ysum = lds + PLds::ysum;
    // per group: 2 row sums transposed onto pairs of lanes, reduced inside each row of 16 lanes on
    // the vector ALU; the four rows of 16 park their sums in LDS and the publishing thread adds them
    const int lrow = lane >> 4;
    DBSN_FOR_LAYER_SLOTS(Ly, {
        const float v2 = pair_sum2(dot4(wr[kGR * G_ + 0], x4), dot4(wr[kGR * G_ + 1], x4));
        const int rl = wave + kWaves * (sbase_ + (lane & 1));
        if ((lane & 14) == 0) ysum[lrow * kMaxTileRows + rl] = v2;
    })
    DBSN_PROF_SUB(ps, ph, 4);
    lds_barrier();
    DBSN_PROF_SUB(ps, ph, 5);
    if (threadIdx.x >= 256) {   // the upper four wavefronts publish
        u64* dst = Ly.yp + (size_t)par * Ly.nCB * Ly.n_out + (size_t)t.cb * Ly.n_out + t.r0;
        for (int j = threadIdx.x - 256; j < t.Reff; j += 256) {
            constexpr int kYS = kMaxTileRows;
            float y = (ysum[j] + ysum[kYS + j]) + (ysum[2 * kYS + j] + ysum[3 * kYS + j]);
            if (t.cb == 0) y += lds[PLds::bias + l * kMaxTileRows + j];
            st_tagged(dst + j, y, tag);
        }
        // state read-out after the last step (dbsn_mlp_get_activations): row block 0 writes the
        // inputs it gathered
        if (last && l > 1 && t.rb == 0 && (int)threadIdx.x - 256 < t.Ceff)
            net.lay[l - 1].x[t.c0 + threadIdx.x - 256] = xk[threadIdx.x - 256];
    }
    DBSN_PROF_SUB(ps, ph, 7);
    return true;
}

// Fused backward sweep of this workgroup's tile of layer l (appendix "Backward propagation" and
// "Weight updating" over the same registers): deltas of the tile's rows, partial W^T delta of its
// columns from the OLD weights, published at once (it is what other workgroups wait for), then
// the rank-1 update of the tile.
template <bool ST>
__device__ __forceinline__ bool p_bwd_tile(float4 (&wr)[kSlots], const PNet& net, int l, int g, float eta,
                                           unsigned tag, bool last, float* lds, long long ps,
                                           int ph DBSN_PROF_ARGS) {
    const PLayer& Ly = net.lay[l];
    TileCtx t;
    if (!tile_ctx(Ly, g, t)) return true;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    DBSN_LAYER_GROUPS(Ly);
    DBSN_PROF_SUB(ps, ph, 0);
    if (!ST) load_tile(wr, Ly, t);

    // Deltas of the tile's rows.  For the last hidden layer they are in LDS already (the output
    // layer was evaluated in this workgroup).  Otherwise the workgroup gathers the gP partials of
    // each of its rows from the layer above into LDS (the producers have multiplied them by
    // f'(x_l) already, see below) and four threads per row add a quarter each in index order.
    const float* dl = tile_deltas(net, l, t, lds);
    if (l < net.L - 1) {
        float* dw = lds + PLds::dkeep + l * kMaxTileRows;
        float* sg = lds + PLds::stage;
        const u64* gsrc = Ly.gp + (size_t)par * Ly.gP * Ly.n_out + t.r0;
        const bool ok = poll_rows_to_lds<kThreads, 8>(gsrc, Ly.gP, t.Reff, (unsigned)Ly.n_out, tag, sg,
                                                      net.spin_limit);
        DBSN_PROF_SUB(ps, ph, 1);
        if (!all_ok(ok, net.err, lds)) return false;
        DBSN_PROF_SUB(ps, ph, 2);
        for (int t4 = threadIdx.x; (t4 >> 2) - (lane >> 2) < t.Reff; t4 += kThreads) {
            // (trip count uniform over the wavefront: sum_row4 exchanges data inside quads)
            const int j = t4 >> 2;
            const float d = sum_row4(sg, Ly.gP, min(j, t.Reff - 1), t4 & 3);
            if ((t4 & 3) == 0 && j < t.Reff) dw[j] = d;
        }
        lds_barrier();
    }
    const int myrow = wave + kWaves * lane;
    const float dlane = (lane < kSlots && myrow < t.Reff) ? dl[myrow] : 0.0f;
    DBSN_PROF_SUB(ps, ph, 3);
    const float* xk = lds + PLds::xkeep + (par * (kMaxLayers + 1) + l) * 256;
    const float4 x4 = *reinterpret_cast<const float4*>(xk + 4 * lane);
    if (l > 1) {
        float4 gacc = make_float4(0.f, 0.f, 0.f, 0.f);
        DBSN_FOR_LAYER_SLOTS(Ly, {
            _Pragma("unroll") for (int q = 0; q < kGR; ++q) {
                const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dlane), sbase_ + q));
                const float4 w4 = wr[kGR * G_ + q];
                gacc.x = fmaf(w4.x, d, gacc.x);
                gacc.y = fmaf(w4.y, d, gacc.y);
                gacc.z = fmaf(w4.z, d, gacc.z);
                gacc.w = fmaf(w4.w, d, gacc.w);
            }
        })
        float* gred = lds + PLds::gred;
        *reinterpret_cast<float4*>(gred + wave * 264 + 4 * lane) = gacc;
        DBSN_PROF_SUB(ps, ph, 4);
        lds_barrier();
        DBSN_PROF_SUB(ps, ph, 5);
        const PLayer& Lp = net.lay[l - 1];
        u64* dst = Lp.gp + (size_t)par * Lp.gP * Lp.n_out + (size_t)t.rb * Lp.n_out + t.c0;
        const int i = (int)threadIdx.x - 256;   // the upper four wavefronts publish
        if (i >= 0 && i < t.Ceff) {
            float v8[kWaves];
#pragma unroll
            for (int k = 0; k < kWaves; ++k) v8[k] = gred[k * 264 + i];
            float s8 = 0.0f;
#pragma unroll
            for (int k = 0; k < kWaves; ++k) s8 += v8[k];
            // this tile's columns are neurons of layer l-1 whose outputs it holds: fold f' in here,
            // so that the consumer's sum over row blocks is delta_{l-1} itself
            st_tagged(dst + i, s8 * dact_from_y(xk[i]), tag);
        }
    }
    DBSN_PROF_SUB(ps, ph, 6);
    update_tile(wr, Ly, x4, dlane, eta);
    if (!ST) store_tile(wr, Ly, t);
    if (t.cb == 0) {
        // bias update (the biases of this tile's rows live in LDS for the whole launch), and after
        // the last step the layer's deltas for dbsn_mlp_get_deltas
        for (int j = threadIdx.x; j < t.Reff; j += kThreads) {
            const float d = dl[j];
            lds[PLds::bias + l * kMaxTileRows + j] -= eta * d;
            if (last) Ly.d[t.r0 + j] = d;
        }
    }
    DBSN_PROF_SUB(ps, ph, 7);
    return true;
}

// Output layer in every workgroup, on its private LDS copy of W_L: x_{L-1} from the partials,
// logits, softmax, loss, delta_L, the deltas of layer L-1 and the rank-1 update of the copy.
// Thread i owns column i (input neuron i) of W_L: it gathers x_i and forms the products
// W_L[j][i] x_i; the workgroup adds them per class (quads -> rows of 16 lanes on the vector ALU,
// then 32 partial sums per class through LDS); wavefront 0 does the softmax, and each thread
// back-propagates through and updates its column.
__device__ __forceinline__ bool p_top(const PNet& net, int g, int label, float eta, unsigned tag, float* loss_out,
                                      bool last, float* lds, long long ps, int ph DBSN_PROF_ARGS) {
    const int L = net.L;
    const PLayer& Ly = net.lay[L];
    const PLayer& Lp = net.lay[L - 1];
    const int n = Ly.n_in, nc = Ly.n_out;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    float* xtop = lds + PLds::xtop;
    float* dtop = lds + PLds::dtop;
    float* WL = lds + PLds::WL;
    float* bL = lds + PLds::bL;
    float* part = lds + PLds::gred;    // [class][33]: 8 wavefronts x 4 rows of 16 lanes (pitch 33: no bank conflicts)
    float* dL = lds + PLds::ysum;      // [kMaxClasses] delta_L

    DBSN_PROF_SUB(ps, ph, 0);
    bool ok = true;
    {
        // thread i gathers x_{L-1}[i] (and i + 512, ...): the nCB partial sums in index order
        const u64* base = Lp.yp + (size_t)par * Lp.nCB * Lp.n_out;
        const unsigned stride = (unsigned)Lp.n_out;
        for (int i0 = 0; i0 < n; i0 += kThreads) {
            const int i = i0 + (int)threadIdx.x;
            const bool on = i < n;
            const unsigned col = on ? (unsigned)i : 0u;
            auto off = [=](int k) { return (unsigned)k * stride + col; };
            u64 v[16];
            poll_issue(v, Lp.nCB, base, off);
            const float a = poll_finish(v, Lp.nCB, Lp.nCB, base, off, tag, net.spin_limit, ok);
            if (on) xtop[i] = act_fast(a);
        }
    }
    DBSN_PROF_SUB(ps, ph, 2);
    // products per class, four classes at a time; a thread folds its columns i, i + 512, ... together
    for (int j0 = 0; j0 < nc; j0 += 4) {
        float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
        const int j1 = min(j0 + 1, nc - 1), j2 = min(j0 + 2, nc - 1), j3 = min(j0 + 3, nc - 1);
        for (int i = threadIdx.x; i < n; i += kThreads) {
            const float xi = xtop[i];   // this thread's own write
            a0 = fmaf(WL[j0 * n + i], xi, a0);
            a1 = fmaf(WL[j1 * n + i], xi, a1);
            a2 = fmaf(WL[j2 * n + i], xi, a2);
            a3 = fmaf(WL[j3 * n + i], xi, a3);
        }
        const float v = quad_sum4(a0, a1, a2, a3);
        const int cls = j0 + (lane & 3);
        if ((lane & 12) == 0 && cls < nc) part[cls * 33 + wave * 4 + (lane >> 4)] = v;
    }
    DBSN_PROF_SUB(ps, ph, 3);
    if (!all_ok(ok, net.err, lds)) return false;
    DBSN_PROF_SUB(ps, ph, 4);
    if (wave == 0) {
        // class c = lane: logit, softmax (the sum of the exponentials is taken in index order)
        float a = -3.0e38f;
        if (lane < nc) {
            float v[32];
#pragma unroll
            for (int r = 0; r < 32; ++r) v[r] = part[lane * 33 + r];
            float acc = 0.0f;
#pragma unroll
            for (int r = 0; r < 32; ++r) acc += v[r];
            a = acc + bL[lane];
        }
        float m = a;
        m = fmaxf(m, dpp_mov<kDppXor1>(m));
        m = fmaxf(m, dpp_mov<kDppXor2>(m));
        m = fmaxf(m, dpp_mov<kDppRor4>(m));
        m = fmaxf(m, dpp_mov<kDppRor8>(m));
        if (nc > 16) {
            m = fmaxf(m, __shfl_xor(m, 16, 64));
            m = fmaxf(m, __shfl_xor(m, 32, 64));
        } else {
            m = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(m)));   // row 0 holds all classes
        }
        const float e = (lane < nc) ? expf(a - m) : 0.0f;
        float ssum = 0.0f;
        for (int c = 0; c < nc; ++c) ssum += __int_as_float(__builtin_amdgcn_readlane(__float_as_int(e), c));
        const float p = e / ssum;
        if (lane < nc) {
            dL[lane] = p - (lane == label ? 1.0f : 0.0f);
            dL[kMaxClasses + lane] = p;
        }
    }
    DBSN_PROF_SUB(ps, ph, 5);
    lds_barrier();
    DBSN_PROF_SUB(ps, ph, 6);
    if (g == 0 && wave == kWaves - 1) {
        // results for the host: the loss of every step; after the last step also the probabilities,
        // the output deltas and x_{L-1}
        if (lane == 0 && loss_out) *loss_out = -logf(dL[kMaxClasses + label]);
        if (last) {
            if (lane < nc) { Ly.x[lane] = dL[kMaxClasses + lane]; Ly.d[lane] = dL[lane]; }
            for (int i = lane; i < n; i += 64) Lp.x[i] = xtop[i];
        }
    }
    // deltas of layer L-1 and update of the private W_L
    for (int i = threadIdx.x; i < n; i += kThreads) {
        const float xi = xtop[i];
        float gs = 0.0f;
        for (int j0 = 0; j0 < nc; j0 += 4) {
            const int j1 = min(j0 + 1, nc - 1), j2 = min(j0 + 2, nc - 1), j3 = min(j0 + 3, nc - 1);
            const float w0 = WL[j0 * n + i], w1 = WL[j1 * n + i], w2 = WL[j2 * n + i], w3 = WL[j3 * n + i];
            const float d0 = dL[j0], d1 = dL[j1], d2 = dL[j2], d3 = dL[j3];
            gs = fmaf(w0, d0, gs);
            WL[j0 * n + i] = fmaf(-(eta * d0), xi, w0);
            if (j0 + 1 < nc) { gs = fmaf(w1, d1, gs); WL[j1 * n + i] = fmaf(-(eta * d1), xi, w1); }
            if (j0 + 2 < nc) { gs = fmaf(w2, d2, gs); WL[j2 * n + i] = fmaf(-(eta * d2), xi, w2); }
            if (j0 + 3 < nc) { gs = fmaf(w3, d3, gs); WL[j3 * n + i] = fmaf(-(eta * d3), xi, w3); }
        }
        dtop[i] = gs * dact_from_y(xi);
    }
    if (threadIdx.x < nc) bL[threadIdx.x] -= eta * dL[threadIdx.x];
    lds_barrier();
    DBSN_PROF_SUB(ps, ph, 7);
    return true;
}

template <bool ST>
__global__ __launch_bounds__(kThreads) void k_bp_dataflow(PNet net, const float* samples, const int* labels,
                                                           int label_val, long long n, float eta, float* loss_out,
                                                           unsigned tag_base) {
    extern __shared__ float lds[];
    DBSN_PROF_DECL;
    const int g = blockIdx.x, L = net.L;
    const PLayer& LyL = net.lay[L];
    const int n0 = net.lay[1].n_in;
    // private copy of the output layer
    for (int e = threadIdx.x; e < LyL.n_out * LyL.n_in; e += kThreads) {
        const int j = e / LyL.n_in, i = e - j * LyL.n_in;
        lds[PLds::WL + e] = LyL.W[(size_t)j * LyL.ld + i];
    }
    if (threadIdx.x < LyL.n_out) lds[PLds::bL + threadIdx.x] = LyL.b[threadIdx.x];
    for (int e = threadIdx.x; e < 2 * (kMaxLayers + 1) * 256; e += kThreads) lds[PLds::xkeep + e] = 0.0f;
    if (threadIdx.x == 0) *reinterpret_cast<int*>(lds + PLds::fail) = 0;

    for (int l = 1; l < L; ++l) {
        TileCtx t;
        if (tile_ctx(net.lay[l], g, t) && t.cb == 0)
            for (int j = threadIdx.x; j < t.Reff; j += kThreads)
                lds[PLds::bias + l * kMaxTileRows + j] = net.lay[l].b[t.r0 + j];
    }
    float4 wr[kSlots];
#pragma unroll
    for (int s = 0; s < kSlots; ++s) wr[s] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (ST) {
        for (int l = 1; l < L; ++l) {
            TileCtx t;
            if (tile_ctx(net.lay[l], g, t)) load_tile(wr, net.lay[l], t);
        }
    }
    __syncthreads();

    // this thread's input pixel of the first layer's tile, fetched one sample ahead
    TileCtx t1;
    const bool has1 = tile_ctx(net.lay[1], g, t1) && (int)threadIdx.x < t1.Ceff;
    float x0pre = (has1 && n > 0) ? samples[t1.c0 + threadIdx.x] : 0.0f;
    int labpre = (labels && n > 0) ? labels[0] : label_val;

    bool alive = true;
    for (long long s = 0; s < n && alive; ++s) {
        const unsigned tag = tag_base + (unsigned)s + 1u;
        int label = labpre;
        label = label < 0 ? 0 : (label >= LyL.n_out ? LyL.n_out - 1 : label);
        const float x0cur = x0pre;
        if (s + 1 < n) {
            if (has1) x0pre = samples[(s + 1) * n0 + t1.c0 + threadIdx.x];
            if (labels) labpre = labels[s + 1];
        }
        const bool last = (s + 1 == n);
        for (int l = 1; l < L && alive; ++l)
            alive = p_fwd_tile<ST>(wr, net, l, g, x0cur, tag, last, lds, s, l - 1 DBSN_PROF_PASS);
        if (alive)
            alive = p_top(net, g, label, eta, tag, loss_out ? loss_out + s : nullptr, last, lds, s, L - 1 DBSN_PROF_PASS);
        for (int l = L - 1; l >= 1 && alive; --l)
            alive = p_bwd_tile<ST>(wr, net, l, g, eta, tag, last, lds, s, L + (L - 1 - l) DBSN_PROF_PASS);
    }
    if (ST) {
        for (int l = 1; l < L; ++l) {
            TileCtx t;
            if (tile_ctx(net.lay[l], g, t)) store_tile(wr, net.lay[l], t);
        }
    }
    __syncthreads();
    for (int l = 1; l < L; ++l) {
        TileCtx t;
        if (tile_ctx(net.lay[l], g, t) && t.cb == 0)
            for (int j = threadIdx.x; j < t.Reff; j += kThreads)
                net.lay[l].b[t.r0 + j] = lds[PLds::bias + l * kMaxTileRows + j];
    }
    DBSN_PROF_FLUSH();
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
