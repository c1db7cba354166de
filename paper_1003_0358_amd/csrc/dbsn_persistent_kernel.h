// Persistent on-line back-propagation kernel of libdbsn for gfx950: n strictly sequential
// batch-size-1 steps in ONE launch, with no grid barrier and no kernel boundary between layers.
//
// Why it looks like this.  A step of the paper's big nets touches 144 MB of weights but is a chain
// of 2L dependent mat-vec phases; on this chip a kernel boundary or a grid-wide barrier costs
// 2-4 us, as much as streaming a whole layer.  So the phases are connected by DATAFLOW instead:
//
//  * Every hidden layer l is cut into tiles of R_l rows x C_l <= 256 columns (dbsn_plan.h); a tile
//    belongs to one workgroup number g for the whole life of the network, forward and backward,
//    so a weight is only ever touched by one workgroup.  Where two hidden layers follow each
//    other the cut goes in bands per die of the chip, so that what those two layers hand to each
//    other never leaves a die's L2 (stores of workgroup scope there, which cost half); the
//    workgroups take their numbers g by the die they find themselves on.
//  * What crosses workgroups is small: forward, a tile publishes its R partial dot products
//    yp_l[cb][rows]; backward, its C partial sums of W^T delta.  Each value travels as ONE 64-bit
//    word {step tag, float} written with a device-scope atomic store, and a consumer polls the
//    words it needs until they carry the current step's tag: the data is its own flag.  No fence,
//    no L2 write-back, no counter that 256 workgroups hammer.
//  * A consumer adds the partials in a fixed order (bit-reproducible), applies the activation
//    (forward) itself, and goes on.
//  * Buffers alternate with the parity of the step tag; the output layer needs all of x_{L-1},
//    hence every tile of the step, which keeps any workgroup from running two steps ahead.
//  * The 10 x n_{L-1} output layer lives in every workgroup's LDS; each workgroup evaluates it
//    and applies the same update to its private copy (same code, same inputs, same bits), so the
//    deltas of the last hidden layer are available everywhere without communication.
//  * Weights live in REGISTERS.  A wavefront owns ns consecutive rows of a tile, one 128-bit
//    register quadruple ("slot") per row and lane (a lane holds four consecutive columns),
//    processed in groups of kGR slots.  The 256 workgroups x 8 wavefronts x kSlots quadruples hold
//    58 MB: when all tiles of a workgroup fit (they do for every net of the paper, 48 MB at most) the weights are
//    loaded once per launch, updated in place for n steps and written back at the end
//    ("stationary"); the memory system then carries only the small tagged words, and a step
//    costs its chain of hand-overs, not its bytes.  Otherwise each phase loads its tile into the
//    same registers (the loads are issued before the wait for the inputs, so they overlap it)
//    and the backward phase stores it back.
//  * With the weights on chip a step costs INSTRUCTIONS and load round trips, so everything a
//    phase needs that does not change from step to step (tile bounds, word offsets, register
//    group ranges) is worked out once per launch into a small per-layer table in LDS, the
//    register groups of a layer are entered by one switch instead of a test per group, and
//    reductions stay on the vector ALU (DPP inside rows of 16 lanes, lane-row swaps across them).
//    A forward phase has one workgroup barrier (the tile's inputs go through LDS to all
//    wavefronts), a backward phase one (the column sums of W^T delta over the eight wavefronts;
//    every wavefront gathers the deltas of its own rows by itself), the output phase three.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

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
#ifdef DBSN_PROFILE_WALL   // the 100 MHz counter all compute units share, for comparing workgroups
#define DBSN_PROF(step, slot) DBSN_PROF_VAL(step, slot, wall_clock64())
#else
#define DBSN_PROF(step, slot) DBSN_PROF_VAL(step, slot, clock64())
#endif
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
#define DBSN_PROF(step, slot) do { (void)(step); (void)(slot); } while (0)
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

static_assert(kGR == 2, "the forward reduction pairs the two rows of a register group");
static_assert(kSlots <= 32, "one lane per row slot, two blocks of 16");

struct PLayer {
    float* W; float* b; float* x; float* d;
    u64* yp;          // [2][nCB][n_out]            forward partial sums of this layer's rows
    u64* gp;          // [2][nRB] chunks            partial delta of this layer's neurons, one chunk per row block: for
                      //                            every row of the block gP words (one per row block of layer l+1),
                      //                            arranged by the consumer's wavefronts (gp_word_in_chunk)
    int n_in, n_out, ld;
    TileShape shape;  // how the layer is cut into tiles (dbsn_plan.h)
    int gP;           // number of partial rows in gp = row blocks of layer l+1
    int s0, ns;       // row slots [s0, s0 + ns) of a wavefront hold this layer's tile
    int fwd_local;    // 1: the forward partial sums this layer publishes are read on the publisher's die only
    int bwd_local;    // 1: the backward partial sums this layer publishes (for the layer below) likewise
};

struct PNet {
    PLayer lay[kMaxLayers + 1];
    int* err;
    int L;
    unsigned spin_limit;
    int stationary;   // 1: every layer has its own register slots for the whole launch
    int any_local;    // 1: some hand-over stays inside a die: workgroups number themselves by the die they run on
    // pause of each (direction, layer) before its first look at the partials, in units of 64 clocks
    // ([0]: forward, index L the output layer; [1]: backward)
    unsigned char pace[2][kMaxLayers + 1];
};

// Per-layer table of this workgroup (32-bit words in LDS), filled once per launch.
constexpr int kPlanInts = 32;
enum : int {
    PL_FLAGS = 0,   // bit 0: the workgroup has a tile of this layer; bit 1: column block 0; bit 2: row block 0;
                    // bit 3: the layer above it in which the workgroup has its next tile has the same parity
    PL_CEFF, PL_REFF, PL_R0, PL_C0, PL_S0, PL_SEND,   // (slots [S0, SEND) of a wavefront hold the tile's rows)
    PL_PF,          // forward: partials per input column = nCB of the layer below
    PL_FSTRIDE,     // forward: words between two partials of one column = n of the layer below
    PL_FPAR,        // forward source: words between the two parity buffers
    PL_FDPAR,       // forward destination: words between the two parity buffers
    PL_GP,          // backward: partials per row
    PL_BPAR,        // backward source: words between the parity buffers
    PL_BDPAR,       // backward destination (gp of the layer below): words between the parity buffers
    PL_FLOCAL,      // forward: 1 when every reader of the words published here runs on this die
    PL_BLOCAL,      // backward: likewise for the words published for the layer below
    PL_RB,          // row block of this tile
    PL_FSRC = 20,   // (2 words each) pointers: forward source of parity 0 at this tile's first column,
    PL_FDST = 22,   //   forward destination at this tile's first row,
    PL_BSRC = 24,   //   this tile's chunk of gp,
    PL_BDST = 26    //   gp of the layer below
};

// LDS map (floats)
struct PLds {
    static constexpr int WL = 0;                                  // [kTopWMax]  private copy of W_L, [padded classes][n]
    static constexpr int bL = WL + kTopWMax;                      // [kMaxClasses]
    static constexpr int xkeep = bL + kMaxClasses;                // [kMaxLayers + 1][256] inputs of each tile (rows 0 and 1:
                                                                  //   the first layer's, by the parity of the step)
    static constexpr int bias = xkeep + (kMaxLayers + 1) * 256;   // [kMaxLayers + 1][kMaxTileRows] (column block 0)
    static constexpr int dLp = bias + (kMaxLayers + 1) * kMaxTileRows;   // [2][kMaxClasses] delta_L (padded with zeros), probabilities
    static constexpr int gred = dLp + 2 * kMaxClasses;            // [2][kWaves][264] (by the parity of the layer); [class][8] partial logits
    static constexpr int xtop = gred + 2 * kWaves * 264;          // [kTopXMax]
    static constexpr int dtop = xtop + kTopXMax;                  // [kTopXMax]
    static constexpr int plan = dtop + kTopXMax;                  // [kMaxLayers + 1][kPlanInts]
    static constexpr int fail = plan + (kMaxLayers + 1) * kPlanInts;   // [1] set when a wait gave up
    static constexpr int pace = fail + 16;                        // [2][kMaxLayers + 1] pauses before polling
    static constexpr int bdst = pace + 2 * (kMaxLayers + 1) + 14; // [kMaxLayers + 1][256] where column i of the layer's tile
                                                                  //   publishes its backward partial sum (word offset in gp)
    static constexpr int total = bdst + (kMaxLayers + 1) * 256;
};
static_assert((PLds::total + kProfLdsFloats) * 4 <= 160 * 1024, "LDS map exceeds 160 KB");
static_assert(kMaxClasses * kWaves <= kWaves * 264, "partial logits do not fit");

__device__ inline u64 pack_tagged(float v, unsigned tag) { return ((u64)tag << 32) | (u64)__float_as_uint(v); }
// (the words are in device memory: saying so keeps the compiler from emitting generic-address loads
// for pointers it has seen rebuilt from integers)
typedef __attribute__((address_space(1))) u64 global_u64;
__device__ inline u64 ld_tagged(const u64* p) {
    return __hip_atomic_load((const global_u64*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_tagged(u64* p, float v, unsigned tag) {
    __hip_atomic_store((global_u64*)p, pack_tagged(v, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The same for words whose readers all run on the publisher's die (`local`, uniform): the store
// then stops at the die's L2, where the readers' device-scope loads find it, in half the time of a
// store that has to become visible to the other dies.  (Were the word ever evicted, it would reach
// memory, where those loads look next: visibility never depends on luck, only speed does.)
__device__ inline void st_tagged(u64* p, float v, unsigned tag, bool local) {
    if (local) __hip_atomic_store((global_u64*)p, pack_tagged(v, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else __hip_atomic_store((global_u64*)p, pack_tagged(v, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

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
    if (bad && threadIdx.x == 0) __hip_atomic_fetch_max(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // (keeps a 2)
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

// v[t] + v[t ^ 16] + v[t ^ 32] + v[t ^ 48] in every lane: adds the four rows of 16 lanes as
// (row0 + row1) + (row2 + row3) with the lane-row swap instructions of gfx950.
__device__ inline float rows_sum(float v) {
    const unsigned a = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane16_swap(a, a, false, false);
    const float s = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    const unsigned b = __float_as_uint(s);
    const auto q = __builtin_amdgcn_permlane32_swap(b, b, false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// Sums of four values over the 64 lanes at once: two halving steps inside every quad of lanes
// leave value (t & 3) in lane t, the remaining steps add over the quads of the row of 16 lanes.
__device__ inline float quad_sum4(float a0, float a1, float a2, float a3) {
    const int lane = threadIdx.x & 63;
    const bool b0 = (lane & 1) != 0, b1 = (lane & 2) != 0;
    const float s0 = (b0 ? a1 : a0) + dpp_mov<kDppXor1>(b0 ? a0 : a1);
    const float s1 = (b0 ? a3 : a2) + dpp_mov<kDppXor1>(b0 ? a2 : a3);
    float v = (b1 ? s1 : s0) + dpp_mov<kDppXor2>(b1 ? s0 : s1);
    v += dpp_mov<kDppRor4>(v);
    v += dpp_mov<kDppRor8>(v);
    return v;   // sum over this row of 16 lanes; the caller adds the four rows
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

// Gathering the partial sums of one input column: P <= N tagged words of step `tag`, word k at
// row_k[col] with row_k = base + k * stride the same for the whole wavefront (scalar address
// arithmetic) and col the lane's column.  All N loads are in flight together; the batch is read
// again until every word carries the tag.  Slots beyond P repeat word P - 1 and are left out of the
// sum, which adds the payloads in index order.
template <int N>
__device__ __forceinline__ float poll_sum_n(const u64* base, unsigned col, int P, unsigned stride, unsigned tag,
                                            unsigned limit, bool& ok, float s) {
    u64 v[N];
    unsigned spins = 0;
    for (;;) {
#pragma unroll
        for (int k = 0; k < N; ++k) {
            const u64* row = base + (size_t)((unsigned)min(k, P - 1) * stride);
            v[k] = ld_tagged(row + col);
        }
        bool pending = false;
#pragma unroll
        for (int k = 0; k < N; ++k) pending |= ((unsigned)(v[k] >> 32) != tag);
        if (!__any(pending && DBSN_WAITING(limit))) break;
        if (++spins > limit) { ok = false; break; }
    }
#pragma unroll
    for (int k = 0; k < N; ++k) s += (k < P) ? __uint_as_float((unsigned)v[k]) : 0.0f;
    return s;
}
// (more than 12 partials take batches of 8 one after the other)
__device__ __forceinline__ float poll_sum(const u64* base, unsigned col, int P, unsigned stride, unsigned tag,
                                          unsigned limit, bool& ok) {
    float s = 0.0f;
    while (P > 12 && ok) {
        s = poll_sum_n<8>(base, col, 8, stride, tag, limit, ok, s);
        base += (size_t)(8u * stride);
        P -= 8;
    }
    if (P <= 4) return poll_sum_n<4>(base, col, P, stride, tag, limit, ok, s);
    if (P <= 8) return poll_sum_n<8>(base, col, P, stride, tag, limit, ok, s);
    return poll_sum_n<12>(base, col, P, stride, tag, limit, ok, s);
}

// Two columns at once (col0, col1 of the same rows): all 2 N loads in flight together, one wait for
// both.  P <= N.
template <int N>
__device__ __forceinline__ void poll_sum_pair(const u64* base, unsigned col0, unsigned col1, int P, unsigned stride,
                                              unsigned tag, unsigned limit, bool& ok, float& s0, float& s1) {
    u64 v0[N], v1[N];
    unsigned spins = 0;
    for (;;) {
#pragma unroll
        for (int k = 0; k < N; ++k) {
            const u64* row = base + (size_t)((unsigned)min(k, P - 1) * stride);
            v0[k] = ld_tagged(row + col0);
            v1[k] = ld_tagged(row + col1);
        }
        bool pending = false;
#pragma unroll
        for (int k = 0; k < N; ++k) pending |= ((unsigned)(v0[k] >> 32) != tag) | ((unsigned)(v1[k] >> 32) != tag);
        if (!__any(pending && DBSN_WAITING(limit))) break;
        if (++spins > limit) { ok = false; break; }
    }
    s0 = 0.0f; s1 = 0.0f;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        s0 += (k < P) ? __uint_as_float((unsigned)v0[k]) : 0.0f;
        s1 += (k < P) ? __uint_as_float((unsigned)v1[k]) : 0.0f;
    }
}

// Gathering a wavefront's own share of a chunk of backward partial sums (layout: dbsn_plan.h): lane
// t reads the words p[64 k], k < K (K uniform), of which its first Pl (0 for a lane with no row)
// belong to its row; all loads of a batch are in flight together, the batch is read again until the
// lane's words carry the tag, and the payloads are added in index order.
template <int N>
__device__ __forceinline__ float poll_lanes_n(const u64* p, int Pl, int K, unsigned tag, unsigned limit, bool& ok, float s) {
    u64 v[N];
    unsigned spins = 0;
    for (;;) {
#pragma unroll
        for (int k = 0; k < N; ++k) v[k] = ld_tagged(p + 64 * min(k, K - 1));
        bool pending = false;
#pragma unroll
        for (int k = 0; k < N; ++k) pending |= (k < Pl) && ((unsigned)(v[k] >> 32) != tag);
        if (!__any(pending && DBSN_WAITING(limit))) break;
        if (++spins > limit) { ok = false; break; }
    }
#pragma unroll
    for (int k = 0; k < N; ++k) s += (k < Pl) ? __uint_as_float((unsigned)v[k]) : 0.0f;
    return s;
}
// (the last of the K loads may run past the wavefront's share, by less than 64 words: the buffer ends
// with kGpTailWords spare ones; more than 12 words per lane take batches of 8 one after the other)
__device__ __forceinline__ float poll_lanes(const u64* p, int Pl, int K, unsigned tag, unsigned limit, bool& ok) {
    float s = 0.0f;
    while (K > 12 && ok) {
        s = poll_lanes_n<8>(p, Pl, 8, tag, limit, ok, s);
        p += 8 * 64;
        Pl -= 8;
        K -= 8;
    }
    if (K <= 2) return poll_lanes_n<2>(p, Pl, K, tag, limit, ok, s);
    if (K <= 4) return poll_lanes_n<4>(p, Pl, K, tag, limit, ok, s);
    if (K <= 8) return poll_lanes_n<8>(p, Pl, K, tag, limit, ok, s);
    return poll_lanes_n<12>(p, Pl, K, tag, limit, ok, s);
}
// Sum over the lanes t, t + span, t + 2 span, ... of the wavefront (span a power of two up to 32,
// uniform), left in every one of them: fixed tree, vector ALU only.
__device__ __forceinline__ float span_sum(float v, int span) {
    if (span <= 1) v += dpp_mov<kDppXor1>(v);
    if (span <= 2) v += dpp_mov<kDppXor2>(v);
    if (span <= 4) v += dpp_mov<kDppRor4>(v);
    if (span <= 8) v += dpp_mov<kDppRor8>(v);
    if (span <= 16) {
        const unsigned a = __float_as_uint(v);
        const auto r = __builtin_amdgcn_permlane16_swap(a, a, false, false);
        v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    const unsigned b = __float_as_uint(v);
    const auto q = __builtin_amdgcn_permlane32_swap(b, b, false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// Pacing of the polls.  A batch of loads that comes back without the data costs a full round trip
// before the next one can be judged, so it pays to look a little later and find the data at the
// first look.  How much later depends on the layer, the direction and the machine: one pause per
// (direction, layer), in units of 64 clocks, set by the host (defaults, or the search of
// dbsn_mlp_autotune).  Results do not depend on it.
constexpr int kPaceMax = 48;
__device__ __forceinline__ void pace_begin(const float* lds, int dir, int l) {
    const int* tab = reinterpret_cast<const int*>(lds + PLds::pace);
    const int d = uniform(tab[dir * (kMaxLayers + 1) + l]);
    for (int w = 0; w < d; ++w) __builtin_amdgcn_s_sleep(1);
}

__device__ inline float dot4(const float4& w, const float4& x) {
    float acc = w.x * x.x;
    acc = fmaf(w.y, x.y, acc);
    acc = fmaf(w.z, x.z, acc);
    return fmaf(w.w, x.w, acc);
}

// Runs f(G) for the register groups G = g0 .. gend - 1 of one layer, G a compile-time constant
// inside f (register indices must be): one switch to enter, one compare per group to leave.
#define DBSN_GROUP_CASE(G)                                   \
    case G:                                                  \
        f(std::integral_constant<int, G>{});                 \
        if (gend == G + 1) break;                            \
        [[fallthrough]];
template <class F>
__device__ __forceinline__ void for_layer_groups(int g0, int gend, F&& f) {
    static_assert(kNG == 14, "one case per register group");
    switch (g0) {
        DBSN_GROUP_CASE(0) DBSN_GROUP_CASE(1) DBSN_GROUP_CASE(2) DBSN_GROUP_CASE(3) DBSN_GROUP_CASE(4)
        DBSN_GROUP_CASE(5) DBSN_GROUP_CASE(6) DBSN_GROUP_CASE(7) DBSN_GROUP_CASE(8) DBSN_GROUP_CASE(9)
        DBSN_GROUP_CASE(10) DBSN_GROUP_CASE(11) DBSN_GROUP_CASE(12)
        case 13: f(std::integral_constant<int, 13>{}); break;
        default: break;
    }
}

// Entering the groups through that switch costs a few dozen scalar instructions per loop, as much
// as the work of a small layer.  Networks whose layers fit a register LAYOUT fixed at compile time
// (layer l owns the groups [g0(l), g0(l) + ngmax(l)), of which it uses its first ng) skip it: the
// loops below then see constant group numbers, selected by one plain switch on the layer.
// (the layouts are tabulated in dbsn_plan.h; the host takes the first one a network fits)
// (All groups of the layer's static range run, used or not: an unused group holds zero weights and
// meets zero deltas, so it publishes nothing and stays zero, and the code has no branch to merge.)
template <int G, int GEND, class F>
__device__ __forceinline__ void run_groups(F&& f) {
    if constexpr (G < GEND) {
        f(std::integral_constant<int, G>{});
        run_groups<G + 1, GEND>(f);
    }
}
// POS = 0: the layer is known at run time only (LAYOUT 0); POS = 1 .. kLayoutDepth[LAYOUT]: the
// phase is compiled for hidden layer POS of that layout.
// (s0, send: the layer's slots; the groups that hold any of them run.  A group shared with a
// neighbouring layer runs for both: the foreign row's dot product is never published, and in the
// backward sweep it meets a zero delta.)
template <int LAYOUT, int POS, class F>
__device__ __forceinline__ void layer_groups(int s0, int send, F&& f) {
    if constexpr (POS == 0) for_layer_groups(s0 / kGR, (send + kGR - 1) / kGR, f);
    else {
        static_assert(POS <= kLayoutDepth[LAYOUT] && kLayoutS0[LAYOUT][POS - 1] + kLayoutNS[LAYOUT][POS - 1] <= kSlots,
                      "the layout has this layer and its slots exist");
        run_groups<kLayoutS0[LAYOUT][POS - 1] / kGR,
                   (kLayoutS0[LAYOUT][POS - 1] + kLayoutNS[LAYOUT][POS - 1] + kGR - 1) / kGR>(f);
    }
}

// Register slot a of a wavefront holds tile row wave * ns + (a - s0) of the layer whose ns slots start
// at s0 ("absolute" slot a, the same index in every per-slot register; group G = slots 2 G, 2 G + 1).
struct TileGeom {
    float* wbase;   // &W[r0][c0 + 4 * lane]
    int ld, Reff, s0, send;
    bool lane_on;
};
__device__ inline bool tile_geom(const PLayer& Ly, int g, TileGeom& t) {
    TileAt at;
    if (!tile_at(Ly.shape, Ly.n_in, Ly.n_out, g, at)) return false;
    const int lane = threadIdx.x & 63;
    t.ld = Ly.ld;
    t.Reff = at.Reff;
    t.s0 = Ly.s0;
    t.send = Ly.s0 + Ly.ns;
    t.lane_on = (4 * lane < at.Ceff);   // (row pitch and column starts are multiples of 4: a float4 never leaves the row)
    t.wbase = Ly.W + (size_t)at.r0 * Ly.ld + at.c0 + 4 * lane;
    return true;
}

// KEEP = true (weights stationary: the layers share the registers for the whole launch): slots
// outside [s0, send) belong to other layers and are left alone.  KEEP = false (streaming: the phase
// has the registers to itself, s0 = 0): every slot of the groups is assigned, rows past the tile
// get zeros, and the loads carry no condition that would keep them from being in flight together.
template <bool KEEP>
__device__ __forceinline__ void load_tile(float4 (&wr)[kSlots], const TileGeom& t) {
    const int wave = threadIdx.x >> 6;
    // (the wavefront's rows end where the next wavefront's begin, or with the tile: one bound per
    // wavefront, so that a slot past the layer's last one - the second of an odd layer's last group -
    // reads as a row past the tile)
    const int lim = min(t.Reff, (wave + 1) * (t.send - t.s0));
    for_layer_groups(t.s0 / kGR, (t.send + kGR - 1) / kGR, [&](auto Gc) {
        constexpr int G = decltype(Gc)::value;
#pragma unroll
        for (int q = 0; q < kGR; ++q) {
            const int a = kGR * G + q;
            const int rl = wave * (t.send - t.s0) + (a - t.s0);
            if (!KEEP || (a >= t.s0 && a < t.send))
                wr[a] = (rl < lim && t.lane_on) ? *reinterpret_cast<const float4*>(t.wbase + (size_t)rl * t.ld)
                                                : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    });
}
__device__ __forceinline__ void store_tile(const float4 (&wr)[kSlots], const TileGeom& t) {
    const int wave = threadIdx.x >> 6;
    for_layer_groups(t.s0 / kGR, (t.send + kGR - 1) / kGR, [&](auto Gc) {
        constexpr int G = decltype(Gc)::value;
#pragma unroll
        for (int q = 0; q < kGR; ++q) {
            const int a = kGR * G + q;
            const int rl = wave * (t.send - t.s0) + (a - t.s0);
            if (a >= t.s0 && a < t.send && rl < t.Reff && t.lane_on)
                *reinterpret_cast<float4*>(t.wbase + (size_t)rl * t.ld) = wr[a];
        }
    });
}

__device__ inline const int* plan_of(const float* lds, int l) {
    return reinterpret_cast<const int*>(lds + PLds::plan) + l * kPlanInts;
}
// The whole table row of layer l into scalar registers with 128-bit LDS reads issued back to back
// (one wait for all of them); what a phase does not use is dropped by the compiler.  Kernels with
// a compile-time layout fetch the rows once, before the step loop.
struct PlanRow {
    int v[kPlanInts];
    __device__ __forceinline__ int operator[](int i) const { return v[i]; }
};
__device__ __forceinline__ PlanRow load_plan(const float* lds, int l) {
    PlanRow r;
    const int4* src = reinterpret_cast<const int4*>(plan_of(lds, l));
#pragma unroll
    for (int k = 0; k < kPlanInts / 4; ++k) {
        const int4 q = src[k];
        r.v[4 * k + 0] = uniform(q.x); r.v[4 * k + 1] = uniform(q.y);
        r.v[4 * k + 2] = uniform(q.z); r.v[4 * k + 3] = uniform(q.w);
    }
    return r;
}
__device__ __forceinline__ u64* plan_ptr(const PlanRow& pl, int at) {
    return reinterpret_cast<u64*>(((u64)(unsigned)uniform(pl[at + 1]) << 32) | (u64)(unsigned)uniform(pl[at]));
}

// Fills this workgroup's table (called by one thread per layer at kernel start).
__device__ inline void make_plan(const PNet& net, int l, int g, float* lds) {
    int* pl = reinterpret_cast<int*>(lds + PLds::plan) + l * kPlanInts;
    const int L = net.L;
    const PLayer& Ly = net.lay[l];
    for (int e = 0; e < kPlanInts; ++e) pl[e] = 0;
    auto put_ptr = [&](int at, const u64* p) {
        pl[at] = (int)(unsigned)((u64)p & 0xFFFFFFFFull);
        pl[at + 1] = (int)(unsigned)((u64)p >> 32);
    };
    if (l == L) {   // output layer: only the gathering of x_{L-1}
        const PLayer& Lp = net.lay[L - 1];
        pl[PL_FLAGS] = 1;
        pl[PL_PF] = Lp.shape.nCB;
        pl[PL_FSTRIDE] = Lp.n_out;
        pl[PL_FPAR] = Lp.shape.nCB * Lp.n_out;
        put_ptr(PL_FSRC, Lp.yp);
        return;
    }
    TileAt at;
    if (!tile_at(Ly.shape, Ly.n_in, Ly.n_out, g, at)) return;
    pl[PL_FLAGS] = 1 | (at.cb == 0 ? 2 : 0) | (at.rb == 0 ? 4 : 0);
    // (the backward phases of layers 2 .. L-1 use two LDS copies of their column sums by layer parity,
    // see p_bwd_tile: does the phase this workgroup runs before this one use the same copy?)
    if (l > 1)
        for (int k = l + 1; k < L; ++k) {
            TileAt above;
            if (tile_at(net.lay[k].shape, net.lay[k].n_in, net.lay[k].n_out, g, above)) {
                if (((k - l) & 1) == 0) pl[PL_FLAGS] |= 8;
                break;
            }
        }
    pl[PL_CEFF] = at.Ceff;
    pl[PL_REFF] = at.Reff;
    pl[PL_R0] = at.r0;
    pl[PL_C0] = at.c0;
    pl[PL_S0] = Ly.s0;
    pl[PL_SEND] = Ly.s0 + Ly.ns;
    pl[PL_RB] = at.rb;
    pl[PL_FLOCAL] = Ly.fwd_local;
    pl[PL_BLOCAL] = Ly.bwd_local;
    pl[PL_FDPAR] = Ly.shape.nCB * Ly.n_out;
    put_ptr(PL_FDST, Ly.yp + (size_t)at.cb * Ly.n_out + at.r0);
    if (l > 1) {
        const PLayer& Lp = net.lay[l - 1];
        pl[PL_PF] = Lp.shape.nCB;
        pl[PL_FSTRIDE] = Lp.n_out;
        pl[PL_FPAR] = Lp.shape.nCB * Lp.n_out;
        put_ptr(PL_FSRC, Lp.yp + at.c0);
        pl[PL_BDPAR] = Lp.shape.nRB * gp_chunk_words(Lp.ns, Lp.gP);
        put_ptr(PL_BDST, Lp.gp);
    }
    if (l < L - 1) {
        pl[PL_GP] = Ly.gP;
        pl[PL_BPAR] = Ly.shape.nRB * gp_chunk_words(Ly.ns, Ly.gP);
        put_ptr(PL_BSRC, Ly.gp + (size_t)at.rb * gp_chunk_words(Ly.ns, Ly.gP));
    }
}

// Where column i of this workgroup's tile of layer l publishes its backward partial sum: neuron
// c = c0 + i of layer l-1 is row j' of that layer's row block rb', and the word is the one of this
// tile's row block in row j' of chunk rb' (gp_word_in_chunk).  Worked out once per launch (thread i
// of the workgroup).
__device__ inline void make_bdst(const PNet& net, int l, int g, int i, float* lds) {
    int* tab = reinterpret_cast<int*>(lds + PLds::bdst) + l * 256;
    tab[i] = 0;
    if (l < 2 || l >= net.L) return;
    TileAt at;
    if (!tile_at(net.lay[l].shape, net.lay[l].n_in, net.lay[l].n_out, g, at) || i >= at.Ceff) return;
    const PLayer& Lp = net.lay[l - 1];
    int rbp, jp, reffp;
    row_block_at(Lp.shape, Lp.n_out, at.c0 + i, rbp, jp, reffp);
    tab[i] = rbp * gp_chunk_words(Lp.ns, Lp.gP) + gp_word_in_chunk(Lp.ns, Lp.gP, jp, at.rb);
}

// Forward propagation of this workgroup's tile of layer l (appendix "Forward propagation"):
// partial sums of the rows over the tile's columns, the bias riding on column block 0.
template <bool ST, int LAYOUT, int POS>
__device__ __forceinline__ bool p_fwd_tile(float4 (&wr)[kSlots], const PNet& net, int l, int g, float x0pre,
                                           unsigned tag, bool last, float* lds, const PlanRow& pl, long long ps, int ph DBSN_PROF_ARGS) {
    const int flags = uniform(pl[PL_FLAGS]);
    if (!(flags & 1)) return true;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    const int Ceff = uniform(pl[PL_CEFF]), Reff = uniform(pl[PL_REFF]);
    const int s0 = uniform(pl[PL_S0]), send = uniform(pl[PL_SEND]);
    DBSN_PROF_SUB(ps, ph, 0);
    if (!ST) {   // in flight while the inputs are awaited
        TileGeom tg;
        if (tile_geom(net.lay[l], g, tg)) load_tile<false>(wr, tg);
    }

    // (the first layer keeps its inputs by the parity of the step: its backward phase has no barrier
    // between reading them and the next step's forward phase, which writes the other copy)
    float* xk = lds + PLds::xkeep + (l == 1 ? (int)par : l) * 256;
    if (l == 1) {
        // the caller fetched this thread's input pixel ahead of time
        if (threadIdx.x < 256) xk[threadIdx.x] = ((int)threadIdx.x < Ceff) ? x0pre : 0.0f;
        lds_barrier();
    } else {
        // thread j < Ceff of the lower four wavefronts gathers the partial sums of its input column j,
        // adds them in index order and applies the activation: x_{l-1}[c0 + j]
        bool ok = true;
        if (threadIdx.x < 256) {
            const int P = uniform(pl[PL_PF]);
            const unsigned stride = (unsigned)uniform(pl[PL_FSTRIDE]);
            const u64* base = plan_ptr(pl, PL_FSRC) + (size_t)(par * (unsigned)uniform(pl[PL_FPAR]));
            const unsigned col = min(threadIdx.x, (unsigned)Ceff - 1u);
            pace_begin(lds, 0, l);
            DBSN_PROF_SUB(ps, ph, 1);
            const float a = poll_sum(base, col, P, stride, tag, net.spin_limit, ok);
            const float x = ((int)threadIdx.x < Ceff) ? act_fast(a) : 0.0f;
            xk[threadIdx.x] = x;
            // state read-out after the last step (dbsn_mlp_get_activations): row block 0 writes the
            // inputs it gathered
            if (last && (flags & 4) && (int)threadIdx.x < Ceff) net.lay[l - 1].x[uniform(pl[PL_C0]) + threadIdx.x] = x;
            DBSN_PROF_SUB(ps, ph, 2);
        }
        if (!all_ok(ok, net.err, lds)) return false;
    }
    DBSN_PROF_SUB(ps, ph, 3);
    const float4 x4 = *reinterpret_cast<const float4*>(xk + 4 * lane);
    // the lane that will publish absolute slot a = lane (lanes 0 .. 31): tile row and bias
    const int myrow = wave * (send - s0) + (lane - s0);
    const bool pub = lane >= s0 && lane < send && myrow < Reff;
    const float mybias = (pub && (flags & 2)) ? lds[PLds::bias + l * kMaxTileRows + myrow] : 0.0f;
    // per group: the two row sums transposed onto the even and odd lanes and reduced inside each row
    // of 16 lanes; lane 16 r + (a & 15) keeps the sum of slot a over lane row r
    float res0 = 0.0f, res1 = 0.0f;
    const int lane14 = lane & 14;
    layer_groups<LAYOUT, POS>(s0, send, [&](auto Gc) {
        constexpr int G = decltype(Gc)::value;
        const float v2 = pair_sum2(dot4(wr[kGR * G + 0], x4), dot4(wr[kGR * G + 1], x4));
        if (kGR * G < 16) res0 = (lane14 == ((kGR * G) & 14)) ? v2 : res0;
        else res1 = (lane14 == ((kGR * G) & 14)) ? v2 : res1;
    });
    res0 = rows_sum(res0);
    if (send > 16) res1 = rows_sum(res1);
    DBSN_PROF_SUB(ps, ph, 4);
    if (pub) {
        u64* dst = plan_ptr(pl, PL_FDST) + (size_t)(par * (unsigned)uniform(pl[PL_FDPAR]));
        st_tagged(dst + myrow, ((lane < 16) ? res0 : res1) + mybias, tag, uniform(pl[PL_FLOCAL]) != 0);
    }
    DBSN_PROF_SUB(ps, ph, 7);
    return true;
}

// Fused backward sweep of this workgroup's tile of layer l (appendix "Backward propagation" and
// "Weight updating" over the same registers): deltas of the tile's rows, partial W^T delta of its
// columns from the OLD weights, published at once (it is what other workgroups wait for), then
// the rank-1 update of the tile.
template <bool ST, int LAYOUT, int POS>
__device__ __forceinline__ bool p_bwd_tile(float4 (&wr)[kSlots], const PNet& net, int l, int g, float eta,
                                           unsigned tag, bool last, float* lds, const PlanRow& pl, long long ps,
                                           int ph DBSN_PROF_ARGS) {
    const int flags = uniform(pl[PL_FLAGS]);
    if (!(flags & 1)) return true;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    const int Ceff = uniform(pl[PL_CEFF]), Reff = uniform(pl[PL_REFF]);
    const int s0 = uniform(pl[PL_S0]), send = uniform(pl[PL_SEND]);
    DBSN_PROF_SUB(ps, ph, 0);
    TileGeom tg;
    if (!ST) { tile_geom(net.lay[l], g, tg); load_tile<false>(wr, tg); }   // (flags & 1: the tile exists)
    // the tile's inputs, kept since the forward sweep
    const float* xk = lds + PLds::xkeep + (l == 1 ? (int)par : l) * 256;
    const float4 x4 = *reinterpret_cast<const float4*>(xk + 4 * lane);

    // Deltas of the wavefront's rows, lane a <-> absolute slot a.  For the last hidden layer they
    // are in LDS already (the output layer was evaluated in this workgroup).  Otherwise every
    // wavefront gathers the partial sums of its own rows, gP per row, which the producers have
    // multiplied by f'(x_l) already (see below): its share of the tile's chunk is one run of words
    // that the 64 lanes read side by side, lane t the words of slot (t - s0) mod span and of the
    // partial sums p = t / span, t / span + 64 / span, ...; a lane adds its words in index order, and
    // the lanes of a slot are added by a fixed tree, which leaves the row's delta in the lane of its
    // absolute slot.  No LDS, no barrier: a wavefront goes on as soon as its own rows are there.
    const int ns = send - s0;
    const int srel = lane - s0;   // slot of this lane within the layer
    const int myrow = wave * ns + srel;
    const bool rowon = srel >= 0 && lane < send && myrow < Reff;
    float dlane = 0.0f;
    if (l == net.L - 1) {
        if (rowon) dlane = lds[PLds::dtop + uniform(pl[PL_R0]) + myrow];
    } else {
        const int gP = uniform(pl[PL_GP]);
        const int span = slot_span(ns), nc = 64 / span;   // lanes per partial sum, partial sums per load
        const int arel = srel & (span - 1), c = lane / span;
        const int wv = uniform(wave);
        const bool mine = arel < ns && wv * ns + arel < Reff;
        const int Pl = (mine && c < gP) ? (gP - c + nc - 1) / nc : 0;
        const int K = (gP + nc - 1) / nc;
        const u64* src = plan_ptr(pl, PL_BSRC) + (size_t)(par * (unsigned)uniform(pl[PL_BPAR])) +
                         (size_t)(unsigned)(wv * gP * span);
        bool ok = true;
        float part = 0.0f;
        if (wv * ns < Reff) {   // (a wavefront past the tile's last row has nothing to wait for)
            pace_begin(lds, 1, l);
            part = poll_lanes(src + (c * span + arel), Pl, K, tag, net.spin_limit, ok);
        }
        DBSN_PROF_SUB(ps, ph, 1);
        // (a wait that gave up: the next agreement of the workgroup, or the end of the launch, reports it)
        if (!ok) *reinterpret_cast<int*>(lds + PLds::fail) = 1;
        part = span_sum(part, span);
        dlane = rowon ? part : 0.0f;
        DBSN_PROF_SUB(ps, ph, 2);
    }
    DBSN_PROF_SUB(ps, ph, 3);
    if (l > 1) {
        float4 gacc = make_float4(0.f, 0.f, 0.f, 0.f);
        layer_groups<LAYOUT, POS>(s0, send, [&](auto Gc) {
            constexpr int G = decltype(Gc)::value;
#pragma unroll
            for (int q = 0; q < kGR; ++q) {
                const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dlane), kGR * G + q));
                const float4 w4 = wr[kGR * G + q];
                gacc.x = fmaf(w4.x, d, gacc.x);
                gacc.y = fmaf(w4.y, d, gacc.y);
                gacc.z = fmaf(w4.z, d, gacc.z);
                gacc.w = fmaf(w4.w, d, gacc.w);
            }
        });
        // (two copies used in turn by the layers: this phase's only barrier lies between writing and
        // reading, so the next phase's writes must not land where this one's readers may still look;
        // the phase after that has the next phase's barrier behind it.  A workgroup skips the layers it
        // has no tile of: where that brings two layers of the same parity together, the second one
        // waits for the first one's readers here - flag 8, worked out with the table)
        if (flags & 8) lds_barrier();
        float* gred = lds + PLds::gred + (l & 1) * (kWaves * 264);
        *reinterpret_cast<float4*>(gred + wave * 264 + 4 * lane) = gacc;
        DBSN_PROF_SUB(ps, ph, 4);
        lds_barrier();
        DBSN_PROF_SUB(ps, ph, 5);
        const int i = (int)threadIdx.x;   // the lower four wavefronts publish, one column each
        if (i < Ceff) {
            float v8[kWaves];
#pragma unroll
            for (int k = 0; k < kWaves; ++k) v8[k] = gred[k * 264 + i];
            const float xi = xk[i];
            float s8 = 0.0f;
#pragma unroll
            for (int k = 0; k < kWaves; ++k) s8 += v8[k];
            // where the word goes (see make_bdst)
            const unsigned at = (unsigned)reinterpret_cast<const int*>(lds + PLds::bdst)[l * 256 + i];
            u64* dst = plan_ptr(pl, PL_BDST) + (size_t)(par * (unsigned)uniform(pl[PL_BDPAR]));
            // this tile's columns are neurons of layer l-1 whose outputs it holds: fold f' in here,
            // so that the consumer's sum over row blocks is delta_{l-1} itself
            st_tagged(dst + at, s8 * dact_from_y(xi), tag, uniform(pl[PL_BLOCAL]) != 0);
        }
    }
    DBSN_PROF_SUB(ps, ph, 6);
    // rank-1 update of the tile held in registers, w[j][i] -= eta * delta_j * x_i; rows beyond the
    // tile hold zeros and get a zero delta, so they stay zero
    layer_groups<LAYOUT, POS>(s0, send, [&](auto Gc) {
        constexpr int G = decltype(Gc)::value;
#pragma unroll
        for (int q = 0; q < kGR; ++q) {
            const float ed = eta * __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dlane), kGR * G + q));
            float4 v = wr[kGR * G + q];
            v.x = fmaf(-ed, x4.x, v.x);
            v.y = fmaf(-ed, x4.y, v.y);
            v.z = fmaf(-ed, x4.z, v.z);
            v.w = fmaf(-ed, x4.w, v.w);
            wr[kGR * G + q] = v;
        }
    });
    if (!ST) store_tile(wr, tg);
    if ((flags & 2) && rowon) {
        // bias update (the biases of this tile's rows live in LDS for the whole launch), and after
        // the last step the layer's deltas for dbsn_mlp_get_deltas
        lds[PLds::bias + l * kMaxTileRows + myrow] -= eta * dlane;
        if (last) net.lay[l].d[uniform(pl[PL_R0]) + myrow] = dlane;
    }
    DBSN_PROF_SUB(ps, ph, 7);
    return true;
}

// Registers of the output phase when a thread owns TC columns of W_L (i, i + 512, ...) and there
// are at most 16 classes (the paper's nets): the columns themselves, for the whole launch, and what
// their update needs, which is applied after the backward phase that follows has published its
// partial sums.  TC = 1 covers last hidden layers of up to 512 neurons, TC = 2 up to 1024.
template <int TC>
struct TopRegs {
    float w[TC][16];    // W_L[c][i] of this thread's columns, classes padded with zeros
    float xi[TC];       // x_{L-1}[i] of the step in flight
};
// (delta_L of the step is still in LDS, padded with zeros up to 16 classes)
template <int TC>
__device__ __forceinline__ void top_update(TopRegs<TC>& tr, float eta, const float* lds) {
    const float4* dL = reinterpret_cast<const float4*>(lds + PLds::dLp);
#pragma unroll
    for (int jq = 0; jq < 4; ++jq) {
        const float4 d4 = dL[jq];
#pragma unroll
        for (int c = 0; c < TC; ++c) {
            tr.w[c][4 * jq + 0] = fmaf(-(eta * d4.x), tr.xi[c], tr.w[c][4 * jq + 0]);
            tr.w[c][4 * jq + 1] = fmaf(-(eta * d4.y), tr.xi[c], tr.w[c][4 * jq + 1]);
            tr.w[c][4 * jq + 2] = fmaf(-(eta * d4.z), tr.xi[c], tr.w[c][4 * jq + 2]);
            tr.w[c][4 * jq + 3] = fmaf(-(eta * d4.w), tr.xi[c], tr.w[c][4 * jq + 3]);
        }
    }
}

// Output layer in every workgroup, on its private LDS copy of W_L (classes padded to a multiple of
// four with zero rows): x_{L-1} from the partials, logits, softmax, loss, delta_L, the deltas of
// layer L-1 and the rank-1 update of the copy.  Thread i owns column i (input neuron i) of W_L
// (and i + 512, ...): it gathers x_i and forms the products W_L[j][i] x_i; the workgroup adds them
// per class (quads -> rows of 16 lanes on the vector ALU, then 32 partial sums per class through
// LDS); wavefront 0 does the softmax, and each thread back-propagates through and updates its columns.
template <int TC>
__device__ __forceinline__ bool p_top(const PNet& net, int g, int label, float eta, unsigned tag, float* loss_out,
                                      bool last, float* lds, const PlanRow& pl, TopRegs<TC>& tr, long long ps,
                                      int ph DBSN_PROF_ARGS) {
    const int L = net.L;
    const PLayer& Ly = net.lay[L];
    const int n = Ly.n_in, nc = Ly.n_out, ncq = (nc + 3) >> 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned par = tag & 1u;
    float* xtop = lds + PLds::xtop;
    float* dtop = lds + PLds::dtop;
    float* WL = lds + PLds::WL;
    float* bL = lds + PLds::bL;
    float* part = lds + PLds::gred;    // [class][8 wavefronts] partial logits
    float* dL = lds + PLds::dLp;       // [kMaxClasses] delta_L, then [kMaxClasses] probabilities

    DBSN_PROF_SUB(ps, ph, 0);
    bool ok = true;
    const int P = uniform(pl[PL_PF]);
    const unsigned stride = (unsigned)uniform(pl[PL_FSTRIDE]);
    const u64* base = plan_ptr(pl, PL_FSRC) + (size_t)(par * (unsigned)uniform(pl[PL_FPAR]));
    pace_begin(lds, 0, L);
    // At most TC columns per thread and at most 16 classes (the paper's nets): the columns of W_L stay
    // in registers from the products to the update.  Otherwise the same steps with loops over the
    // thread's columns and the classes.
    const bool small = n <= TC * kThreads && ncq <= 4;
    if (small) {
        const int i = (int)threadIdx.x;
        if constexpr (TC == 1) {
            const float a = poll_sum(base, (unsigned)min(i, n - 1), P, stride, tag, net.spin_limit, ok);
            tr.xi[0] = (i < n) ? act_fast(a) : 0.0f;
        } else {
            static_assert(TC == 2, "one or two columns per thread");
            const unsigned c0 = (unsigned)min(i, n - 1), c1 = (unsigned)min(i + kThreads, n - 1);
            float a0, a1;
            if (n <= kThreads) {   // (a narrow layer under a kernel compiled for two columns: the second is not there)
                a0 = poll_sum(base, c0, P, stride, tag, net.spin_limit, ok);
                a1 = 0.0f;
            } else if (P <= 4) {
                poll_sum_pair<4>(base, c0, c1, P, stride, tag, net.spin_limit, ok, a0, a1);
            } else {   // (more words per column than registers for both columns at once: one after the other)
                a0 = poll_sum(base, c0, P, stride, tag, net.spin_limit, ok);
                a1 = poll_sum(base, c1, P, stride, tag, net.spin_limit, ok);
            }
            tr.xi[0] = (i < n) ? act_fast(a0) : 0.0f;
            tr.xi[1] = (i + kThreads < n) ? act_fast(a1) : 0.0f;
        }
        DBSN_PROF_SUB(ps, ph, 2);
#pragma unroll
        for (int jq = 0; jq < 4; ++jq) {
            if (jq < ncq) {
                float p4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    p4[e] = tr.w[0][4 * jq + e] * tr.xi[0];
#pragma unroll
                    for (int c = 1; c < TC; ++c) p4[e] = fmaf(tr.w[c][4 * jq + e], tr.xi[c], p4[e]);
                }
                float v = quad_sum4(p4[0], p4[1], p4[2], p4[3]);
                v = rows_sum(v);   // lanes 0 .. 3 hold the wavefront's sums of classes 4 jq .. 4 jq + 3
                if (lane < 4) part[(4 * jq + lane) * kWaves + wave] = v;
            }
        }
    } else {
        // thread i gathers x_{L-1}[i] (and i + 512, ...): the partial sums in index order
        for (int i0 = 0; i0 < n; i0 += kThreads) {
            const int i = i0 + (int)threadIdx.x;
            const float a = poll_sum(base, (unsigned)min(i, n - 1), P, stride, tag, net.spin_limit, ok);
            if (i < n) xtop[i] = act_fast(a);
        }
        DBSN_PROF_SUB(ps, ph, 2);
        // products per class, four classes at a time; a thread folds its columns i, i + 512, ... together
        for (int jq = 0; jq < ncq; ++jq) {
            float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
            const float* w = WL + 4 * jq * n;
            for (int i = threadIdx.x; i < n; i += kThreads) {
                const float xv = xtop[i];   // this thread's own write
                a0 = fmaf(w[i], xv, a0);
                a1 = fmaf(w[n + i], xv, a1);
                a2 = fmaf(w[2 * n + i], xv, a2);
                a3 = fmaf(w[3 * n + i], xv, a3);
            }
            float v = quad_sum4(a0, a1, a2, a3);
            v = rows_sum(v);
            if (lane < 4) part[(4 * jq + lane) * kWaves + wave] = v;
        }
    }
    DBSN_PROF_SUB(ps, ph, 3);
    if (!all_ok(ok, net.err, lds)) return false;
    DBSN_PROF_SUB(ps, ph, 4);
    if (wave == 0) {
        // class c = lane: logit (the eight wavefronts' sums added pairwise in a fixed tree), softmax
        float a = -3.0e38f;
        if (lane < nc) {
            const float4 p0 = *reinterpret_cast<const float4*>(part + lane * kWaves);
            const float4 p1 = *reinterpret_cast<const float4*>(part + lane * kWaves + 4);
            a = ((p0.x + p0.y) + (p0.z + p0.w)) + ((p1.x + p1.y) + (p1.z + p1.w)) + bL[lane];
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
        const float e = (lane < nc) ? __expf(a - m) : 0.0f;
        // sum of the exponentials: fixed tree inside the rows of 16 lanes, then the four rows
        float ssum = e;
        ssum += dpp_mov<kDppXor1>(ssum);
        ssum += dpp_mov<kDppXor2>(ssum);
        ssum += dpp_mov<kDppRor4>(ssum);
        ssum += dpp_mov<kDppRor8>(ssum);
        if (nc > 16) ssum = rows_sum(ssum);
        else ssum = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(ssum)));
        const float p = __fdividef(e, ssum);
        // classes nc .. 4 ncq - 1 are padding: zero delta keeps their zero weights zero
        dL[lane] = (lane < nc) ? p - (lane == label ? 1.0f : 0.0f) : 0.0f;
        dL[kMaxClasses + lane] = p;
    }
    DBSN_PROF_SUB(ps, ph, 5);
    lds_barrier();
    DBSN_PROF_SUB(ps, ph, 6);
    if (g == 0 && wave == kWaves - 1) {
        // results for the host: the loss of every step; after the last step also the probabilities
        // and the output deltas
        if (lane == 0 && loss_out) *loss_out = -logf(dL[kMaxClasses + label]);
        if (last && lane < nc) { Ly.x[lane] = dL[kMaxClasses + lane]; Ly.d[lane] = dL[lane]; }
    }
    // deltas of layer L-1 (and, with many columns per thread, the update of the private W_L)
    if (small) {
#pragma unroll
        for (int c = 0; c < TC; ++c) {
            const int i = (int)threadIdx.x + c * kThreads;
            float gs = 0.0f;
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) {
                if (jq < ncq) {
                    const float4 d4 = *reinterpret_cast<const float4*>(dL + 4 * jq);
                    gs = fmaf(tr.w[c][4 * jq + 0], d4.x, gs);
                    gs = fmaf(tr.w[c][4 * jq + 1], d4.y, gs);
                    gs = fmaf(tr.w[c][4 * jq + 2], d4.z, gs);
                    gs = fmaf(tr.w[c][4 * jq + 3], d4.w, gs);
                }
            }
            if (i < n) {
                dtop[i] = gs * dact_from_y(tr.xi[c]);
                if (last && g == 0) net.lay[L - 1].x[i] = tr.xi[c];   // x_{L-1} for the host
            }
        }
    } else {
        for (int i = threadIdx.x; i < n; i += kThreads) {
            const float xv = xtop[i];
            float gs = 0.0f;
            for (int jq = 0; jq < ncq; ++jq) {
                float* w = WL + 4 * jq * n + i;
                const float4 d4 = *reinterpret_cast<const float4*>(dL + 4 * jq);
                const float w0 = w[0], w1 = w[n], w2 = w[2 * n], w3 = w[3 * n];
                gs = fmaf(w0, d4.x, gs);
                gs = fmaf(w1, d4.y, gs);
                gs = fmaf(w2, d4.z, gs);
                gs = fmaf(w3, d4.w, gs);
                w[0] = fmaf(-(eta * d4.x), xv, w0);
                w[n] = fmaf(-(eta * d4.y), xv, w1);
                w[2 * n] = fmaf(-(eta * d4.z), xv, w2);
                w[3 * n] = fmaf(-(eta * d4.w), xv, w3);
            }
            dtop[i] = gs * dact_from_y(xv);
            if (last && g == 0) net.lay[L - 1].x[i] = xv;
        }
    }
    if ((int)threadIdx.x < nc) bL[threadIdx.x] -= eta * dL[threadIdx.x];
    lds_barrier();
    DBSN_PROF_SUB(ps, ph, 7);
    return true;
}

// The die (XCD) this wavefront runs on: bits 3:0 of the hardware register XCC_ID.
__device__ inline int die_id() { return (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u); }

// Notes, for every workgroup of a launch shaped like the training kernel's, the die it runs on.
__global__ __launch_bounds__(kThreads) void k_die_probe(int* ids) {
    if (threadIdx.x == 0) ids[blockIdx.x] = die_id();
}

template <bool ST, int LAYOUT>
__global__ __launch_bounds__(kThreads) void k_bp_dataflow(PNet net, const float* samples, const int* labels,
                                                           int label_val, long long n, float eta, float* loss_out,
                                                           unsigned tag_base, unsigned launch_seq) {
    extern __shared__ float lds[];
    DBSN_PROF_DECL;
    const int L = net.L;
    // Which tiles this workgroup owns follows from its number g.  With hand-overs inside a die, g
    // must say where the workgroup really runs: die g % 8.  The hardware deals workgroups to the
    // dies in turn only while nothing else occupies the chip (a kernel on another stream moves
    // them), so the workgroup asks: it reads the die it is on and takes the next free rank among the
    // workgroups of that die (one counter per die in the network's flag block, 32 tickets per die
    // and launch since every compute unit holds exactly one workgroup of this kernel), g = die + 8
    // rank.  Which workgroup gets which number varies from launch to launch; what number g
    // computes does not, so results do not depend on it.
    if (threadIdx.x == 0) {
        int v = blockIdx.x;
        if (net.any_local) {
            const int die = die_id();
            unsigned rank = kPGroups;
            if (die < kXcds)
                rank = __hip_atomic_fetch_add(reinterpret_cast<unsigned*>(net.err) + kDieTicketsAt + die, 1u, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT) - (unsigned)(kPGroups / kXcds) * launch_seq;
            if (rank < (unsigned)(kPGroups / kXcds)) v = die + kXcds * (int)rank;
            else __hip_atomic_store(net.err, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // not eight dies of 32: the waits will give up
        }
        *reinterpret_cast<int*>(lds + PLds::fail + 1) = v;
    }
    __syncthreads();
    const int g = uniform(*reinterpret_cast<const int*>(lds + PLds::fail + 1));
    // A workgroup that owns no tile of any layer leaves at once.  It has nothing to contribute (every
    // workgroup that owns one evaluates the output layer for itself), and nobody would ever wait
    // for it: left in, it could fall two steps behind the others (it may start late, when another
    // kernel still holds its compute unit) and then look for tags that have been overwritten.  An
    // owner cannot be left behind: every output of the last hidden layer depends on every tile of
    // every layer, so no workgroup passes the output phase of a step before all owners have
    // published in it.  (Workgroup 0, which reports losses and the final state, owns the first
    // tile of every layer.)
    {
        bool owns = false;
        for (int l = 1; l < L; ++l) {
            TileAt at;
            owns = owns || tile_at(net.lay[l].shape, net.lay[l].n_in, net.lay[l].n_out, g, at);
        }
        if (!owns) return;
    }
    const PLayer& LyL = net.lay[L];
    const int n0 = net.lay[1].n_in;
    // The tiles first: their loads are the long part of starting up (all workgroups together read
    // every weight once), and what follows until the barrier needs none of them: the tables and the
    // cleared LDS regions are worked out while they are in flight, the small reads from memory
    // (output layer, biases) come last.
    float4 wr[kSlots];
#pragma unroll
    for (int s = 0; s < kSlots; ++s) wr[s] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (ST) {
        for (int l = 1; l < L; ++l) {
            TileGeom tg;
            if (tile_geom(net.lay[l], g, tg)) load_tile<true>(wr, tg);
        }
    }
    for (int e = threadIdx.x; e < 2 * kMaxClasses; e += kThreads) lds[PLds::dLp + e] = 0.0f;
    for (int e = threadIdx.x; e < (kMaxLayers + 1) * 256; e += kThreads) lds[PLds::xkeep + e] = 0.0f;
    if (threadIdx.x == 0) *reinterpret_cast<int*>(lds + PLds::fail) = 0;
    for (int e = threadIdx.x; e < 2 * (kMaxLayers + 1); e += kThreads)
        reinterpret_cast<int*>(lds + PLds::pace)[e] = net.pace[e / (kMaxLayers + 1)][e % (kMaxLayers + 1)];
    if ((int)threadIdx.x >= 1 && (int)threadIdx.x <= L) make_plan(net, threadIdx.x, g, lds);
    for (int l = 1; l < L; ++l)   // (layers 2 .. L-1 have such a table; the kernel reads no other)
        if (threadIdx.x < 256) make_bdst(net, l, g, threadIdx.x, lds);
    // private copy of the output layer, classes padded to a multiple of four with zero rows (four
    // elements per thread at a time, so that their loads are in flight together)
    {
        const int nL = LyL.n_in, ncp = ((LyL.n_out + 3) >> 2) << 2, total = ncp * nL;
        for (int e0 = threadIdx.x; e0 < total; e0 += 4 * kThreads) {
            float v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int e = e0 + k * kThreads, j = e / nL, i = e - j * nL;
                v[k] = (e < total && j < LyL.n_out) ? LyL.W[(size_t)j * LyL.ld + i] : 0.0f;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (e0 + k * kThreads < total) lds[PLds::WL + e0 + k * kThreads] = v[k];
        }
    }
    if (threadIdx.x < kMaxClasses) lds[PLds::bL + threadIdx.x] = ((int)threadIdx.x < LyL.n_out) ? LyL.b[threadIdx.x] : 0.0f;
    for (int l = 1; l < L; ++l) {
        const PLayer& Ly = net.lay[l];
        TileAt at;
        if (tile_at(Ly.shape, Ly.n_in, Ly.n_out, g, at) && at.cb == 0) {
            for (int j = threadIdx.x; j < at.Reff; j += kThreads) lds[PLds::bias + l * kMaxTileRows + j] = Ly.b[at.r0 + j];
        }
    }
    __syncthreads();

    // this thread's input pixel of the first layer's tile, fetched one sample ahead
    const int* pl1 = plan_of(lds, 1);
    const bool has1 = (pl1[PL_FLAGS] & 1) && (int)threadIdx.x < pl1[PL_CEFF];
    const int c01 = pl1[PL_C0];
    float x0pre = (has1 && n > 0) ? samples[c01 + threadIdx.x] : 0.0f;
    int labpre = (labels && n > 0) ? labels[0] : label_val;

    // this thread's columns of the output layer, when they live in registers (see TopRegs): two per
    // thread in the kernels for deep narrow nets and for any net, one in those of the paper's nets of
    // up to five hidden layers, whose last hidden layer has 500 neurons
    constexpr int TC = (LAYOUT == 0 || LAYOUT == 3) ? 2 : 1;
    TopRegs<TC> tr;
    const bool top_small = LyL.n_in <= TC * kThreads && LyL.n_out <= 16;
#pragma unroll
    for (int k = 0; k < TC; ++k) {
        const int i = (int)threadIdx.x + k * kThreads;
#pragma unroll
        for (int c = 0; c < 16; ++c)
            tr.w[k][c] = (top_small && i < LyL.n_in && c < LyL.n_out) ? lds[PLds::WL + c * LyL.n_in + i] : 0.0f;
        tr.xi[k] = 0.0f;
    }
    // the table rows of the layers: fetched once here when the layout is fixed at compile time
    const PlanRow rowL = load_plan(lds, L);
    const PlanRow row1 = load_plan(lds, 1), row2 = load_plan(lds, LAYOUT ? min(2, L) : 1),
                  row3 = load_plan(lds, LAYOUT ? min(3, L) : 1), row4 = load_plan(lds, LAYOUT ? min(4, L) : 1),
                  row5 = load_plan(lds, LAYOUT ? min(5, L) : 1);
    bool alive = true;
    for (long long s = 0; s < n && alive; ++s) {
        const unsigned tag = tag_base + (unsigned)s + 1u;
        int label = labpre;
        label = label < 0 ? 0 : (label >= LyL.n_out ? LyL.n_out - 1 : label);
        const float x0cur = x0pre;
        if (s + 1 < n) {
            if (has1) x0pre = samples[(s + 1) * n0 + c01 + threadIdx.x];
            if (labels) labpre = labels[s + 1];
        }
        const bool last = (s + 1 == n);
#define DBSN_FWD(POS, l, row) p_fwd_tile<ST, ((POS) ? LAYOUT : 0), POS>(wr, net, l, g, x0cur, tag, last, lds, row, s, (l) - 1 DBSN_PROF_PASS)
#define DBSN_BWD(POS, l, row) p_bwd_tile<ST, ((POS) ? LAYOUT : 0), POS>(wr, net, l, g, eta, tag, last, lds, row, s, L + (L - 1 - (l)) DBSN_PROF_PASS)
        if constexpr (LAYOUT == 0) {
            for (int l = 1; l < L && alive; ++l) alive = DBSN_FWD(0, l, load_plan(lds, l));
        } else {
            static_assert(kLayoutDepth[LAYOUT] == 5 || kLayoutDepth[LAYOUT] == 9, "one line per hidden layer of the layout");
            alive = DBSN_FWD(1, 1, row1);
            if (L > 2 && alive) alive = DBSN_FWD(2, 2, row2);
            if (L > 3 && alive) alive = DBSN_FWD(3, 3, row3);
            if (L > 4 && alive) alive = DBSN_FWD(4, 4, row4);
            if (L > 5 && alive) alive = DBSN_FWD(5, 5, row5);
            if constexpr (kLayoutDepth[LAYOUT] > 5) {   // (table rows of the deeper layers: fetched at each phase)
                if (L > 6 && alive) alive = DBSN_FWD(6, 6, load_plan(lds, 6));
                if (L > 7 && alive) alive = DBSN_FWD(7, 7, load_plan(lds, 7));
                if (L > 8 && alive) alive = DBSN_FWD(8, 8, load_plan(lds, 8));
                if (L > 9 && alive) alive = DBSN_FWD(9, 9, load_plan(lds, 9));
            }
        }
        if (alive)
            alive = p_top(net, g, label, eta, tag, loss_out ? loss_out + s : nullptr, last, lds, rowL, tr, s, L - 1 DBSN_PROF_PASS);
        // (the update of the register-held column of W_L waits until the first backward phase has
        // published: it is nobody's input before the next step's output phase)
        if constexpr (LAYOUT == 0) {
            for (int l = L - 1; l >= 1 && alive; --l) {
                alive = DBSN_BWD(0, l, load_plan(lds, l));
                if (l == L - 1) top_update(tr, eta, lds);
            }
        } else {
            if constexpr (kLayoutDepth[LAYOUT] > 5) {
                if (L > 9 && alive) alive = DBSN_BWD(9, 9, load_plan(lds, 9));
                if (L == 10) top_update(tr, eta, lds);
                if (L > 8 && alive) alive = DBSN_BWD(8, 8, load_plan(lds, 8));
                if (L == 9) top_update(tr, eta, lds);
                if (L > 7 && alive) alive = DBSN_BWD(7, 7, load_plan(lds, 7));
                if (L == 8) top_update(tr, eta, lds);
                if (L > 6 && alive) alive = DBSN_BWD(6, 6, load_plan(lds, 6));
                if (L == 7) top_update(tr, eta, lds);
            }
            if (L > 5 && alive) alive = DBSN_BWD(5, 5, row5);
            if (L == 6) top_update(tr, eta, lds);
            if (L > 4 && alive) alive = DBSN_BWD(4, 4, row4);
            if (L == 5) top_update(tr, eta, lds);
            if (L > 3 && alive) alive = DBSN_BWD(3, 3, row3);
            if (L == 4) top_update(tr, eta, lds);
            if (L > 2 && alive) alive = DBSN_BWD(2, 2, row2);
            if (L == 3) top_update(tr, eta, lds);
            if (alive) alive = DBSN_BWD(1, 1, row1);
            if (L == 2) top_update(tr, eta, lds);
        }
#undef DBSN_FWD
#undef DBSN_BWD
    }
    if (ST) {
        for (int l = 1; l < L; ++l) {
            TileGeom tg;
            if (tile_geom(net.lay[l], g, tg)) store_tile(wr, tg);
        }
    }
    __syncthreads();
    // (a backward wait that gave up in the last steps has met no agreement of the workgroup yet)
    if (threadIdx.x == 0 && *reinterpret_cast<const int*>(lds + PLds::fail) != 0)
        __hip_atomic_fetch_max(net.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int l = 1; l < L; ++l) {
        const PLayer& Ly = net.lay[l];
        TileAt at;
        if (tile_at(Ly.shape, Ly.n_in, Ly.n_out, g, at) && at.cb == 0) {
            for (int j = threadIdx.x; j < at.Reff; j += kThreads) Ly.b[at.r0 + j] = lds[PLds::bias + l * kMaxTileRows + j];
        }
    }
    DBSN_PROF_FLUSH();
    if (g == 0) {
        if (top_small) {
#pragma unroll
            for (int k = 0; k < TC; ++k) {
                const int i = (int)threadIdx.x + k * kThreads;
#pragma unroll
                for (int c = 0; c < 16; ++c)
                    if (i < LyL.n_in && c < LyL.n_out) lds[PLds::WL + c * LyL.n_in + i] = tr.w[k][c];
            }
        }
        __syncthreads();
        for (int e = threadIdx.x; e < LyL.n_out * LyL.n_in; e += kThreads) {
            const int j = e / LyL.n_in, i = e - j * LyL.n_in;
            LyL.W[(size_t)j * LyL.ld + i] = lds[PLds::WL + e];
        }
        if ((int)threadIdx.x < LyL.n_out) LyL.b[threadIdx.x] = lds[PLds::bL + threadIdx.x];
    }
}

}  // namespace dbsn
