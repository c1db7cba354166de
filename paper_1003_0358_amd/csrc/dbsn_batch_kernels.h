// Forward-only propagation of a BATCH of samples through one layer, for the classification passes
// over validation and test sets (sections "Data" and "Results"; appendix "Forward propagation").
// With many samples at once the layer is a dense contraction Y = X W^T, so unlike the on-line
// training step it belongs on the matrix cores: fp32 MFMA (products and sums in binary32, as
// everywhere in this library), each weight tile read from memory once per 128 samples.
//
// Two kernels compute it.  k_layer_batch_dma is the fast one and needs aligned rows;
// k_layer_batch takes anything: one workgroup of 4 wavefronts per tile of 128 samples x 128
// neurons, wavefront w on the 64 x 64 quadrant (w & 1, w >> 1) as 2 x 2 v_mfma_f32_32x32x2
// accumulators, the k dimension in chunks of 16 staged element by element through two LDS buffers
// (pitch 17: the operand reads, row = lane % 32, k = lane / 32, fall in distinct banks).
// Operand layout of the instruction: lane t supplies A[i = t % 32][k = t / 32] and
// B[k = t / 32][j = t % 32]; result register r of lane t is
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

// End of a tile for one wavefront: its quadrant of 32 NA samples x 64 neurons (NA x 2 accumulators,
// first sample s_base, first neuron j_base) gets bias and activation and goes to Y.  The two bias values are pinned in
// registers before the first guarded store: a guard that were the first to touch them would make
// every later one wait for all memory operations in flight, the stores before it included, since
// the compiler cannot know which guards were taken.  Addresses are 32-bit byte offsets from Y (a
// pass's activations stay far below 4 GB): one addition per store.
template <bool ACT, int NA>
__device__ __forceinline__ void store_quadrant(const floatx16 (&acc)[NA][2], const float* __restrict__ b,
                                               float* __restrict__ Y, int ldy, int S, int n_out, int s_base,
                                               int j_base, int lane) {
    const int jl = j_base + (lane & 31);
    const int sl = s_base + 4 * (lane >> 5);
    float bj[2] = {b[min(jl, n_out - 1)], b[min(jl + 32, n_out - 1)]};
    asm volatile("" : "+v"(bj[0]), "+v"(bj[1]));
    char* Yb = reinterpret_cast<char*>(Y);
    const unsigned pitch = 4u * (unsigned)ldy;
    const unsigned at = (unsigned)sl * pitch + 4u * (unsigned)jl;
    if (s_base + 32 * NA <= S && j_base + 64 <= n_out) {
        // the quadrant lies inside the matrix (a uniform test): no guards, one basic block, so the 64
        // independent activations interleave instead of each waiting out its own latencies
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ds = 32 * a + (r & 3) + 8 * (r >> 2);   // sample of this element, from the lane's first
                    const float v = acc[a][c][r] + bj[c];
                    *reinterpret_cast<float*>(Yb + (at + (unsigned)ds * pitch + 128u * c)) = ACT ? act_fast(v) : v;
                }
        return;
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int j = jl + 32 * c;
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ds = 32 * a + (r & 3) + 8 * (r >> 2);
                if (j < n_out && sl + ds < S) {
                    const float v = acc[a][c][r] + bj[c];
                    *reinterpret_cast<float*>(Yb + (at + (unsigned)ds * pitch + 128u * c)) = ACT ? act_fast(v) : v;
                }
            }
    }
}

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
    store_quadrant<ACT, 2>(acc, b, Y, ldy, S, n_out, s0 + sw, j0 + jw, lane);
}

// The same layer at speed, for operands whose rows start on 16-byte boundaries and n_in % 4 == 0
// (every activation buffer of the library; the caller's samples when their length is a multiple of
// four).  A persistent workgroup per compute unit walks tiles blockIdx.x, + gridDim.x, ... of
// 128 samples x 128 neurons, the k dimension in chunks of 32, and is WAVE-SPECIALISED: four
// CONSUMER wavefronts (one per SIMD) only read operands from LDS and issue matrix instructions,
// each on a 64 x 64 quadrant (2 x 2 accumulators of v_mfma_f32_32x32x2); four PRODUCER wavefronts
// only move chunks from memory into a ring of four LDS stages.  Both choices come from
// measurements on this chip: a wavefront issues in order, so every memory instruction that waits
// for its queue holds back the matrix instructions behind it, and while the matrix instructions
// of a SIMD run, loads that return into vector registers of that SIMD take three to four times
// as long.  So the producers' loads never touch registers: global_load_lds_dwordx4 writes the
// 64 x 16 bytes of a wavefront's load to 1 KB of consecutive LDS, with a scalar base and a
// constant 32-bit offset per lane (no vector arithmetic in the steady state).
//
// That fixes the LDS layout: rows of 32 floats without padding, eight rows per load.  Bank
// conflicts are avoided by permuting the float4 inside each row instead: slot p of row r holds the
// chunk's float4 number p ^ ((r >> 1) & 7), which each lane arranges by the global address it
// supplies; a consumer reads float4 q of row r at slot q ^ ((r >> 1) & 7), and the 16 rows
// r .. r + 15 that neighbouring lanes read then fall in 16 different bank groups.  The matrix
// instruction sums over two k per issue, one from each half of the wavefront; which two is free as
// long as both operands agree, so lanes 0..31 walk the first 16 k of the chunk and lanes 32..63
// the second 16, and one float4 read per operand quadrant feeds four instructions: per chunk and
// consumer 16 LDS reads for 64 matrix instructions, each read issued one group of 16 ahead.
//
// Pipeline: chunks are numbered straight through the tiles of a workgroup.  In iteration i the
// consumers work on chunk i in stage i % 4 (and, at its end, read the first operands of chunk
// i + 1); the producers start the loads of chunk i + 3 into the stage that chunk i - 1 left at the
// last barrier, wait for those of chunk i + 2, issued an iteration earlier, and join the barrier
// that closes the iteration.  So the ring is already filling for the next tile while the
// consumers store the current one.  A float4 of the weights past n_in comes from 16 zero bytes at
// `zeros`, the matching one of the other operand from the start of its row (finite, times zero).
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kDmaThreads = 512;
constexpr int kDmaK = 32;            // k-chunk of a stage
constexpr int kDmaStages = 4;
// floats of a stage: TM sample rows and 128 weight rows of 32, unpadded
constexpr int dma_stage_floats(int TM) { return (TM + kBatchTile) * kDmaK; }
constexpr size_t dma_lds_bytes(int TM) { return sizeof(float) * kDmaStages * dma_stage_floats(TM); }

// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding and for
// nothing else
constexpr int vmcnt_only(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// TM = samples per tile: 128, or 64 for layers whose 128-sample tiles would leave the last round of
// the persistent workgroups mostly empty (the host chooses).  With 64 a consumer's quadrant is
// 32 x 64 (1 x 2 accumulators), everything else alike.
template <bool ACT, int TM>
__global__ __launch_bounds__(kDmaThreads) void k_layer_batch_dma(const float* __restrict__ X, int ldx, int S,
                                                                 const float* __restrict__ W, int ldw,
                                                                 const float* __restrict__ b, int n_in, int n_out,
                                                                 float* __restrict__ Y, int ldy, int nx, int ntiles,
                                                                 const float* __restrict__ zeros) {
    static_assert(TM == 128 || TM == 64, "two or one 32-row block per consumer");
    constexpr int NA = TM / 64;                     // 32-row blocks of samples per consumer
    constexpr int kXLoads = TM / 32;                // loads of eight sample rows per producer and chunk
    constexpr int kWLoads = kBatchTile / 32;        // loads of eight weight rows per producer and chunk
    constexpr int kLoads = kXLoads + kWLoads;
    constexpr int kXop = TM * kDmaK;                // floats of the sample rows of a stage
    constexpr int kStage = dma_stage_floats(TM);
    extern __shared__ __attribute__((aligned(16))) float lds_batch[];
    typedef const __attribute__((address_space(1))) void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform: the roles branch on the scalar unit)
    const int nchunks = (n_in + kDmaK - 1) / kDmaK;
    const int my_tiles = ((int)blockIdx.x < ntiles) ? (ntiles - 1 - (int)blockIdx.x) / (int)gridDim.x + 1 : 0;
    const int total = my_tiles * nchunks;   // iterations of this workgroup
    if (total == 0) return;                 // (the whole workgroup: no barrier is left behind)

    if (wave >= 4) {
        // ---- producer: wavefront pw brings a quarter of the rows of both operands, eight rows a load
        const int pw = wave - 4;
        const int prow = lane >> 3, pslot = lane & 7;
        int ptile = 0, pchunk = 0, pleft = total;   // next chunk to load; chunks not loaded yet
        // byte offsets from the (uniform) operand pointers: 32 bits each, so that a load is one
        // instruction with a scalar base and no address arithmetic on the vector unit
        unsigned xoff[kXLoads], xrow[kXLoads], xq[kXLoads], woff[kWLoads], wq[kWLoads];
        auto tile_offsets = [&]() {
            const int tile = (int)blockIdx.x + ptile * (int)gridDim.x;
            const int s0 = (tile / nx) * TM, j0 = (tile % nx) * kBatchTile;
#pragma unroll
            for (int r = 0; r < kXLoads; ++r) {
                const int row = 8 * kXLoads * pw + 8 * r + prow;
                xq[r] = 4u * (unsigned)(pslot ^ ((row >> 1) & 7));   // first k of this lane's float4 in the chunk
                xrow[r] = 4u * (unsigned)min(s0 + row, S - 1) * (unsigned)ldx;
                xoff[r] = xrow[r] + 4u * xq[r];
            }
#pragma unroll
            for (int r = 0; r < kWLoads; ++r) {
                const int row = 8 * kWLoads * pw + 8 * r + prow;
                wq[r] = 4u * (unsigned)(pslot ^ ((row >> 1) & 7));
                woff[r] = 4u * ((unsigned)min(j0 + row, n_out - 1) * (unsigned)ldw + wq[r]);
            }
        };
        auto load_next = [&](int stage) {
            const int k0 = pchunk * kDmaK;
            float* xs = lds_batch + stage * kStage + (8 * kXLoads * pw) * kDmaK;
            float* ws = lds_batch + stage * kStage + kXop + (8 * kWLoads * pw) * kDmaK;
            const char* Xk = reinterpret_cast<const char*>(X + k0);
            const char* Wk = reinterpret_cast<const char*>(W + k0);
            if (k0 + kDmaK <= n_in) {
#pragma unroll
                for (int r = 0; r < kXLoads; ++r)
                    __builtin_amdgcn_global_load_lds((gptr)(Xk + xoff[r]), (lptr)(xs + 8 * r * kDmaK), 16, 0, 0);
#pragma unroll
                for (int r = 0; r < kWLoads; ++r)
                    __builtin_amdgcn_global_load_lds((gptr)(Wk + woff[r]), (lptr)(ws + 8 * r * kDmaK), 16, 0, 0);
            } else {
#pragma unroll
                for (int r = 0; r < kXLoads; ++r) {
                    const char* xp = k0 + (int)xq[r] < n_in ? Xk + xoff[r] : reinterpret_cast<const char*>(X) + xrow[r];
                    __builtin_amdgcn_global_load_lds((gptr)xp, (lptr)(xs + 8 * r * kDmaK), 16, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < kWLoads; ++r) {
                    const char* wp = k0 + (int)wq[r] < n_in ? Wk + woff[r] : reinterpret_cast<const char*>(zeros);
                    __builtin_amdgcn_global_load_lds((gptr)wp, (lptr)(ws + 8 * r * kDmaK), 16, 0, 0);
                }
            }
            // on to the next chunk; past the end the last chunk is loaded again, into stages nobody reads
            if (pleft > 1) {
                --pleft;
                if (++pchunk == nchunks) {
                    pchunk = 0;
                    ++ptile;
                    tile_offsets();
                }
            }
        };
        tile_offsets();
        load_next(0);
        load_next(1);
        load_next(2);
        __builtin_amdgcn_s_waitcnt(vmcnt_only(kLoads));   // chunks 0 and 1 have landed
        __builtin_amdgcn_s_barrier();
        int stage = 3;   // (i + 3) % 4
        for (int i = 0; i < total; ++i) {
            load_next(stage);
            __builtin_amdgcn_s_waitcnt(vmcnt_only(kLoads));   // all but the loads just issued: chunk i + 2 has landed
            stage = (stage + 1) & (kDmaStages - 1);
            __builtin_amdgcn_s_barrier();
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_only(0));   // nothing may land in LDS after the workgroup has gone
        return;
    }

    // ---- consumer: quadrant (wave & 1, wave >> 1) of 32 NA samples x 64 neurons
    const int sw = (wave & 1) * (32 * NA), jw = ((wave >> 1) & 1) * 64;
    const int lrow = lane & 31, half = lane >> 5, swz = (lrow >> 1) & 7;
    int slot[kDmaK / 8];   // float offset, inside a row, of the float4 this lane feeds to group m
#pragma unroll
    for (int m = 0; m < kDmaK / 8; ++m) slot[m] = 4 * ((m + 4 * half) ^ swz);
    const float* xs0 = lds_batch + (sw + lrow) * kDmaK;
    const float* ws0 = lds_batch + kXop + (jw + lrow) * kDmaK;
    __syncthreads();
    // operands of the next group of matrix instructions, read one group ahead
    floatx4 pa[NA], pw0, pw1;
#pragma unroll
    for (int a = 0; a < NA; ++a) pa[a] = *reinterpret_cast<const floatx4*>(xs0 + 32 * a * kDmaK + slot[0]);
    pw0 = *reinterpret_cast<const floatx4*>(ws0 + slot[0]);
    pw1 = *reinterpret_cast<const floatx4*>(ws0 + 32 * kDmaK + slot[0]);
    int stage = 0;   // i % 4 of iteration i
    for (int t = 0; t < my_tiles; ++t) {
        floatx16 acc[NA][2];
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;
        // nothing is outstanding on the LDS / scalar-memory counter when the chunk loop is entered:
        // with scalar loads possibly in flight the compiler would have to drain the counter before
        // the first matrix instruction of every chunk, the reads just issued included
        __builtin_amdgcn_s_waitcnt(0xc07f);
        for (int cc = 0; cc < nchunks; ++cc) {
            const int stage1 = (stage + 1) & (kDmaStages - 1);
            // the first group of the next chunk sits in the next stage, complete since the last barrier
            const float* xs = xs0 + stage * kStage;
            const float* ws = ws0 + stage * kStage;
            const float* xn = xs0 + stage1 * kStage;
            const float* wn = ws0 + stage1 * kStage;
#pragma unroll
            for (int m = 0; m < kDmaK / 8; ++m) {
                floatx4 av[NA];
#pragma unroll
                for (int a = 0; a < NA; ++a) av[a] = pa[a];
                const floatx4 w0 = pw0, w1 = pw1;
                const float* xr = (m + 1 < kDmaK / 8) ? xs : xn;
                const float* wr = (m + 1 < kDmaK / 8) ? ws : wn;
                const int sl = slot[(m + 1) % (kDmaK / 8)];
#pragma unroll
                for (int a = 0; a < NA; ++a) pa[a] = *reinterpret_cast<const floatx4*>(xr + 32 * a * kDmaK + sl);
                pw0 = *reinterpret_cast<const floatx4*>(wr + sl);
                pw1 = *reinterpret_cast<const floatx4*>(wr + 32 * kDmaK + sl);
                __builtin_amdgcn_sched_barrier(0);   // the reads go out before the matrix instructions, not after
#pragma unroll
                for (int e = 0; e < 4; ++e) {
#pragma unroll
                    for (int a = 0; a < NA; ++a) {
                        acc[a][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[a][e], w0[e], acc[a][0], 0, 0, 0);
                        acc[a][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[a][e], w1[e], acc[a][1], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            stage = stage1;
            __syncthreads();
        }
        // the tile is complete: bias, activation, store (the producers are already filling the ring
        // for the next tile)
        const int tile = (int)blockIdx.x + t * (int)gridDim.x;
        const int s0 = (tile / nx) * TM, j0 = (tile % nx) * kBatchTile;
        store_quadrant<ACT, NA>(acc, b, Y, ldy, S, n_out, s0 + sw, j0 + jw, lane);
    }
}

// Output layer of the classification pass: labels[s] = index of the largest pre-activation
// b[c] + sum_i W[c][i] X[s][i] over the classes (the lowest index on ties).  The layer has only a
// few rows, so it is no job for 128-wide tiles: one wavefront per sample, lanes over the inputs,
// classes 16 at a time in registers, sums over the lanes on the vector ALU.  This form takes any
// strides and alignment (a network without hidden layers classifies the caller's samples with it).
__global__ __launch_bounds__(kBatchThreads) void k_top_batch_any(const float* __restrict__ X, int ldx, int S,
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

// The same for rows that start on 16-byte boundaries (the activation buffers): a wavefront takes
// four samples at once and reads float4, so a weight row is fetched once per four samples and a
// 500-input layer is two rounds of loads instead of eight per sample.  A float4 that straddles
// n_in meets the zero padding of the weight rows.
constexpr int kTopPerWave = 4;
__global__ __launch_bounds__(kBatchThreads) void k_top_batch(const float* __restrict__ X, int ldx, int S,
                                                              const float* __restrict__ W, int ldw,
                                                              const float* __restrict__ b, int n_in, int n_out,
                                                              int* __restrict__ labels) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x & 63;
    const int s0 = (blockIdx.x * (kBatchThreads / 64) + (threadIdx.x >> 6)) * kTopPerWave;
    if (s0 >= S) return;
    const float* xrow[kTopPerWave];
#pragma unroll
    for (int q = 0; q < kTopPerWave; ++q) xrow[q] = X + (size_t)min(s0 + q, S - 1) * ldx;
    int best[kTopPerWave];
    float bv[kTopPerWave];
#pragma unroll
    for (int q = 0; q < kTopPerWave; ++q) { best[q] = 0; bv[q] = 0.0f; }
    for (int c0 = 0; c0 < n_out; c0 += 16) {
        float acc[kTopPerWave][16];
#pragma unroll
        for (int q = 0; q < kTopPerWave; ++q)
#pragma unroll
            for (int c = 0; c < 16; ++c) acc[q][c] = 0.0f;
        for (int i = 4 * lane; i < n_in; i += 256) {
            f4 x[kTopPerWave];
#pragma unroll
            for (int q = 0; q < kTopPerWave; ++q) x[q] = *reinterpret_cast<const f4*>(xrow[q] + i);
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                if (c0 + c < n_out) {   // (uniform)
                    const f4 w = *reinterpret_cast<const f4*>(W + (size_t)(c0 + c) * ldw + i);
#pragma unroll
                    for (int q = 0; q < kTopPerWave; ++q)
                        acc[q][c] = fmaf(w[3], x[q][3], fmaf(w[2], x[q][2], fmaf(w[1], x[q][1], fmaf(w[0], x[q][0], acc[q][c]))));
                }
            }
        }
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            if (c0 + c < n_out) {   // (uniform)
                const float bc = b[c0 + c];
#pragma unroll
                for (int q = 0; q < kTopPerWave; ++q) {
                    float v = acc[q][c];
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
                    v += bc;
                    if ((c0 + c == 0) || v > bv[q]) { bv[q] = v; best[q] = c0 + c; }
                }
            }
        }
    }
    if (lane < kTopPerWave && s0 + lane < S) {
        int out = best[0];
#pragma unroll
        for (int q = 1; q < kTopPerWave; ++q) out = lane == q ? best[q] : out;
        labels[s0 + lane] = out;
    }
}

}  // namespace dbsn
