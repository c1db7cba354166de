// Host-side planning of libdbsn: limits shared by the kernels and the host code, the layout of a
// network's arena and the tile geometry of the persistent training kernel.  Plain C++ with no HIP
// in it, so that it can also be compiled and exercised on a machine without a GPU.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "dbsn.h"

namespace dbsn {

// ---- limits of the kernels ------------------------------------------------------------------
constexpr int kMaxLayers = DBSN_MAX_LAYERS;
constexpr int kThreads = 512;                     // threads of a training workgroup
constexpr int kWaves = kThreads / 64;
constexpr int kMaxRowsPerGroup = 256;             // rows a workgroup of the launch-per-phase kernels may own
constexpr int kMaxClasses = DBSN_MAX_CLASSES;
constexpr int kArenaGroups = 512;                 // partial-sum rows the arena is sized for (>= workgroups launched)
constexpr int kZerosAt = 16;                      // four ints of the flag block that stay zero (a float4 of zeros)
constexpr int kBatchSamples = 16384;              // samples per pass of the batched classification (sizes its buffers)

// persistent kernel
constexpr int kPGroups = 256;        // workgroups (the tile geometry is fixed for this number)
constexpr int kGR = 2;               // rows per register group
constexpr int kNG = 14;              // register groups per wavefront
constexpr int kSlots = kGR * kNG;    // rows a wavefront holds: 28 (a tile has at most 8 * 28 = 224 rows)
constexpr int kMaxTileRows = kSlots * kWaves;   // 224
constexpr int kMaxTileCols = 256;    // a lane holds four consecutive columns of a row
constexpr int kTopWMax = 16384;      // floats of W_L kept in LDS (rows padded to a multiple of four classes)
constexpr int kTopXMax = 2048;       // neurons of layer L-1 the output phase can take

// Register layouts of the persistent kernel that are fixed at compile time (layer l owns the
// groups [g0(l), g0(l) + ngmax(l)), of which it uses its first ng):
// 0: groups packed in layer order at run time (any network);
// 1: up to four hidden layers of at most 2, 3, 2, 1 groups (1000-500, 1500-1000-500, 2000-1500-1000-500);
// 2: up to five hidden layers of at most 3, 5, 3, 2, 1 groups (2500-2000-1500-1000-500);
// 3: up to nine hidden layers of one group each (nine hidden layers of 1000 units, other deep narrow nets).
constexpr int kLayouts = 4;
constexpr int kLayoutMaxDepth = 9;
constexpr int kLayoutDepth[kLayouts] = {0, 5, 5, 9};
constexpr int kLayoutG0[kLayouts][kLayoutMaxDepth] = {{0, 0, 0, 0, 0, 0, 0, 0, 0},
                                                      {0, 2, 5, 7, 8, 8, 8, 8, 8},
                                                      {0, 3, 8, 11, 13, 14, 14, 14, 14},
                                                      {0, 1, 2, 3, 4, 5, 6, 7, 8}};
constexpr int kLayoutNG[kLayouts][kLayoutMaxDepth] = {{0, 0, 0, 0, 0, 0, 0, 0, 0},
                                                      {2, 3, 2, 1, 0, 0, 0, 0, 0},
                                                      {3, 5, 3, 2, 1, 0, 0, 0, 0},
                                                      {1, 1, 1, 1, 1, 1, 1, 1, 1}};

constexpr size_t kArenaAlign = 256;
inline size_t align_up(size_t v, size_t a = kArenaAlign) { return (v + a - 1) / a * a; }

inline bool shape_ok(const int32_t* sizes, int32_t n_sizes) {
    if (!sizes || n_sizes < 2 || n_sizes > DBSN_MAX_LAYERS + 1) return false;
    for (int i = 0; i < n_sizes; ++i)
        if (sizes[i] < 1 || sizes[i] > DBSN_MAX_WIDTH) return false;
    return sizes[n_sizes - 1] <= DBSN_MAX_CLASSES;
}

// column chunks of 256 a launch-per-phase kernel is compiled for
inline int nch_for(int ld) {
    const int need = (ld + 255) / 256;
    const int opts[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
    for (int o : opts)
        if (o >= need) return o;
    return -1;
}

// Byte offsets of everything a network keeps in its arena, and the tile geometry of the persistent
// kernel (hidden layers 1 .. L-1).
struct ArenaPlan {
    size_t W[kMaxLayers + 1], b[kMaxLayers + 1], x[kMaxLayers + 1], d[kMaxLayers + 1];
    size_t yp[kMaxLayers + 1], gp[kMaxLayers + 1];
    size_t gpart[2], flags, act[2], total;
    int ld[kMaxLayers + 1], gld, ldact;
    int nCB[kMaxLayers + 1], nRB[kMaxLayers + 1], C[kMaxLayers + 1], R[kMaxLayers + 1];
    int g0[kMaxLayers + 1], ng[kMaxLayers + 1];   // register groups of each layer's tile
    bool persistent_ok, stationary;
};

inline ArenaPlan plan_arena(const int32_t* sizes, int32_t n_sizes) {
    ArenaPlan p{};
    size_t off = 0;
    int maxw = 0;
    for (int l = 1; l < n_sizes; ++l) {
        const int nin = sizes[l - 1], nout = sizes[l];
        p.ld[l] = (nin + 3) / 4 * 4;
        p.W[l] = off; off = align_up(off + sizeof(float) * (size_t)nout * p.ld[l]);
        p.b[l] = off; off = align_up(off + sizeof(float) * (size_t)nout);
        p.x[l] = off; off = align_up(off + sizeof(float) * (size_t)nout);
        p.d[l] = off; off = align_up(off + sizeof(float) * (size_t)nout);
        if (nin > maxw) maxw = nin;
    }
    p.gld = (maxw + 63) / 64 * 64;
    for (int k = 0; k < 2; ++k) {
        p.gpart[k] = off;
        off = align_up(off + sizeof(float) * (size_t)kArenaGroups * p.gld);
    }
    // error word of the training kernels; ints kZerosAt .. kZerosAt + 3 stay zero for good
    p.flags = off; off = align_up(off + 256);
    // activations of a batch of samples for the forward-only classification passes, two buffers
    // that the layers use in turn
    int maxo = 0;
    for (int l = 1; l < n_sizes; ++l) maxo = sizes[l] > maxo ? sizes[l] : maxo;
    p.ldact = (maxo + 3) / 4 * 4;
    for (int k = 0; k < 2; ++k) {
        p.act[k] = off;
        off = align_up(off + sizeof(float) * (size_t)kBatchSamples * p.ldact);
    }

    // Persistent kernel: layer l is cut into nRB x nCB tiles of R rows x C <= 256 columns, one per
    // workgroup; yp_l holds the forward partial sums [2][nCB][n_l], gp_l the backward ones
    // [2][nRB_l][nRB_{l+1}][R_l], as 64-bit {tag, float} words.
    const int L = n_sizes - 1;
    p.persistent_ok = (L >= 2);
    for (int l = 1; l < L; ++l) {
        const int nin = sizes[l - 1], nout = sizes[l];
        p.nCB[l] = (nin + kMaxTileCols - 1) / kMaxTileCols;
        p.C[l] = ((nin + p.nCB[l] - 1) / p.nCB[l] + 3) / 4 * 4;
        const int rb_max = kPGroups / p.nCB[l];
        p.R[l] = (nout + rb_max - 1) / rb_max;
        p.nRB[l] = (nout + p.R[l] - 1) / p.R[l];
        if (p.R[l] > kMaxTileRows || p.C[l] > kMaxTileCols) p.persistent_ok = false;
    }
    for (int l = 1; l < L; ++l) {
        p.yp[l] = off; off = align_up(off + sizeof(uint64_t) * 2 * (size_t)p.nCB[l] * sizes[l]);
        if (l <= L - 2) {
            // one chunk of nRB_{l+1} x R_l words per row block
            p.gp[l] = off; off = align_up(off + sizeof(uint64_t) * 2 * (size_t)p.nRB[l] * p.R[l] * p.nRB[l + 1]);
        }
    }
    // register groups of kGR rows per wavefront: stationary when every layer gets groups of its own
    int groups = 0;
    for (int l = 1; l < L; ++l) {
        p.ng[l] = ((p.R[l] + kWaves - 1) / kWaves + kGR - 1) / kGR;
        if (p.ng[l] > kNG) p.persistent_ok = false;
        groups += p.ng[l];
    }
    p.stationary = groups <= kNG;
    for (int l = 1, at = 0; l < L; ++l) {
        p.g0[l] = p.stationary ? at : 0;
        at += p.ng[l];
    }
    if (L >= 2) {
        // W_L lives in LDS with its classes padded to a multiple of four
        if ((size_t)((sizes[L] + 3) / 4 * 4) * sizes[L - 1] > (size_t)kTopWMax || sizes[L - 1] > kTopXMax)
            p.persistent_ok = false;
    }
    p.total = off;
    return p;
}

// The first compile-time register layout the network's tiles fit (0: none, pack at run time).
inline int choose_layout(const ArenaPlan& p, int L) {
    if (!p.stationary || !p.persistent_ok) return 0;
    for (int cand = 1; cand < kLayouts; ++cand) {
        bool fits = L - 1 <= kLayoutDepth[cand];
        for (int l = 1; l < L && fits; ++l) fits = p.ng[l] <= kLayoutNG[cand][l - 1];
        if (fits) return cand;
    }
    return 0;
}

}  // namespace dbsn
