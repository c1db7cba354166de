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
constexpr int kDieTicketsAt = 32;                 // eight ints of the flag block: workgroups of the persistent kernel per die so far
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

// Register layouts of the persistent kernel that are fixed at compile time, in row slots of a
// wavefront (layer l owns the slots [s0(l), s0(l) + nsmax(l)), of which it uses its first ns):
// 0: slots packed in layer order at run time (any network);
// 1: up to four hidden layers of at most 4, 6, 4, 2 slots (1000-500, 1500-1000-500, 2000-1500-1000-500);
// 2: up to five hidden layers of at most 5, 11, 6, 4, 2 slots (2500-2000-1500-1000-500: all 28 slots);
// 3: up to nine hidden layers of 2, 4, 2, 4, ... slots (nine hidden layers of 1000 units, other deep narrow nets).
constexpr int kLayouts = 4;
constexpr int kLayoutMaxDepth = 9;
constexpr int kLayoutDepth[kLayouts] = {0, 5, 5, 9};   // (layout 1 lists a fifth layer of no slots: the kernel has one line per layer of 5 or of 9)
constexpr int kLayoutS0[kLayouts][kLayoutMaxDepth] = {{0, 0, 0, 0, 0, 0, 0, 0, 0},
                                                      {0, 4, 10, 14, 16, 16, 16, 16, 16},
                                                      {0, 5, 16, 22, 26, 28, 28, 28, 28},
                                                      {0, 2, 6, 8, 12, 14, 18, 20, 24}};
constexpr int kLayoutNS[kLayouts][kLayoutMaxDepth] = {{0, 0, 0, 0, 0, 0, 0, 0, 0},
                                                      {4, 6, 4, 2, 0, 0, 0, 0, 0},
                                                      {5, 11, 6, 4, 2, 0, 0, 0, 0},
                                                      {2, 4, 2, 4, 2, 4, 2, 4, 2}};

#if defined(__HIPCC__)
#define DBSN_HD __host__ __device__
#else
#define DBSN_HD
#endif

// ---- tiles of the persistent kernel ------------------------------------------------------------
// The weight matrix [n_out][n_in] of a hidden layer is cut into at most kPGroups tiles of at most
// kMaxTileRows x kMaxTileCols, tile <-> workgroup number g for the life of the network.  The chip is
// eight dies (XCDs) with an L2 each, and the training kernel numbers its workgroups so that g runs
// on die g % 8; a hand-over between workgroups of one die costs half of one across dies.  So besides the PLAIN cut (column blocks x
// row blocks, tile (cb, rb) on workgroup rb * nCB + cb) two layers that follow each other can be cut
// in BANDS: the neurons between them (rows of the lower layer = columns of the upper) are split
// into eight bands of B, band k living on die k on both sides: the lower layer ROW-banded (its tiles
// of band k: all column blocks x the row blocks of the band), the upper COLUMN-banded (its tiles of
// band k: the column blocks of the band x all row blocks).  Everything the upper layer needs of the
// lower one in the forward sweep, and the lower of the upper in the backward sweep, then comes from
// the same die.
constexpr int kXcds = 8;
enum : int { TILE_PLAIN = 0, TILE_ROWBAND = 1, TILE_COLBAND = 2 };
struct TileShape {
    int kind;
    int C, R;         // columns / rows of a full tile (C a multiple of 4)
    int nCBq, nRBq;   // column / row blocks: of the layer (plain axis) or of one band (banded axis)
    int B;            // rows (ROWBAND) or columns (COLBAND) of a band, a multiple of 4; 0 for PLAIN
    int nCB, nRB;     // non-empty column / row blocks of the whole layer; blocks are numbered band after band,
                      // and empty ones only come last
};
struct TileAt { int cb, rb, c0, Ceff, r0, Reff; };   // block numbers (layer-wide), first column / row, extent

DBSN_HD inline int imin(int a, int b) { return a < b ? a : b; }

// The tile of workgroup g, if it has one.
DBSN_HD inline bool tile_at(const TileShape& s, int n_in, int n_out, int g, TileAt& t) {
    if (s.kind == TILE_PLAIN) {
        if (g >= s.nCBq * s.nRBq) return false;
        t.cb = g % s.nCBq; t.rb = g / s.nCBq;
        t.c0 = t.cb * s.C; t.r0 = t.rb * s.R;
        if (t.c0 >= n_in || t.r0 >= n_out) return false;
        t.Ceff = imin(s.C, n_in - t.c0); t.Reff = imin(s.R, n_out - t.r0);
        return true;
    }
    const int k = g % kXcds, q = g / kXcds;
    if (q >= s.nCBq * s.nRBq) return false;
    if (s.kind == TILE_ROWBAND) {
        const int cbq = q % s.nCBq, j = q / s.nCBq;
        const int bend = imin((k + 1) * s.B, n_out);
        t.r0 = k * s.B + j * s.R;
        t.c0 = cbq * s.C;
        if (t.r0 >= bend || t.c0 >= n_in) return false;
        t.Reff = imin(s.R, bend - t.r0); t.Ceff = imin(s.C, n_in - t.c0);
        t.cb = cbq; t.rb = k * s.nRBq + j;
        return true;
    }
    const int cbq = q % s.nCBq, rbq = q / s.nCBq;
    const int bend = imin((k + 1) * s.B, n_in);
    t.c0 = k * s.B + cbq * s.C;
    t.r0 = rbq * s.R;
    if (t.c0 >= bend || t.r0 >= n_out) return false;
    t.Ceff = imin(s.C, bend - t.c0); t.Reff = imin(s.R, n_out - t.r0);
    t.cb = k * s.nCBq + cbq; t.rb = rbq;
    return true;
}

// Row r of the layer: its row block, its place in it and the rows of that block.
DBSN_HD inline void row_block_at(const TileShape& s, int n_out, int r, int& rb, int& j, int& reff) {
    if (s.kind == TILE_ROWBAND) {
        const int k = r / s.B, rr = r - k * s.B, jb = rr / s.R;
        const int bend = imin((k + 1) * s.B, n_out);
        rb = k * s.nRBq + jb;
        j = rr - jb * s.R;
        reff = imin(s.R, bend - (k * s.B + jb * s.R));
        return;
    }
    rb = r / s.R;
    j = r - rb * s.R;
    reff = imin(s.R, n_out - rb * s.R);
}

inline int round_up4(int v) { return (v + 3) / 4 * 4; }
// Rows of a tile are dealt to the kWaves wavefronts of its workgroup, so a tile costs as much as the
// next multiple of kWaves rows would: take that many, and the layer has fewer row blocks, hence
// fewer partial sums for the layer below to gather.
inline int whole_slots(int rows) { return (rows + kWaves - 1) / kWaves * kWaves; }

// PLAIN cut: as few column blocks as the 256-column limit allows, as many row blocks as fill the workgroups.
inline TileShape plain_shape(int n_in, int n_out) {
    TileShape s{};
    s.kind = TILE_PLAIN;
    s.nCBq = (n_in + kMaxTileCols - 1) / kMaxTileCols;
    s.C = round_up4((n_in + s.nCBq - 1) / s.nCBq);
    s.nCBq = (n_in + s.C - 1) / s.C;
    const int rb_max = kPGroups / s.nCBq;
    s.R = whole_slots((n_out + rb_max - 1) / rb_max);
    s.nRBq = (n_out + s.R - 1) / s.R;
    s.nCB = s.nCBq; s.nRB = s.nRBq;
    return s;
}
// Band size for n neurons between two banded layers.
inline int band_size(int n) { return round_up4((n + kXcds - 1) / kXcds); }
inline int bands_blocks(int n, int B, int blk) {   // non-empty blocks of `blk` over the bands of B that cover n
    int c = 0;
    for (int k = 0; k < kXcds; ++k) {
        const int len = imin((k + 1) * B, n) - k * B;
        if (len > 0) c += (len + blk - 1) / blk;
    }
    return c;
}
inline TileShape rowband_shape(int n_in, int n_out) {
    TileShape s{};
    s.kind = TILE_ROWBAND;
    s.B = band_size(n_out);
    s.nCBq = (n_in + kMaxTileCols - 1) / kMaxTileCols;
    s.C = round_up4((n_in + s.nCBq - 1) / s.nCBq);
    s.nCBq = (n_in + s.C - 1) / s.C;
    const int per_die = kPGroups / kXcds;
    const int rb_max = per_die / s.nCBq > 0 ? per_die / s.nCBq : 1;
    s.R = whole_slots((s.B + rb_max - 1) / rb_max);
    s.nRBq = (s.B + s.R - 1) / s.R;
    s.nCB = s.nCBq;
    s.nRB = bands_blocks(n_out, s.B, s.R);
    return s;
}
inline TileShape colband_shape(int n_in, int n_out) {
    TileShape s{};
    s.kind = TILE_COLBAND;
    s.B = band_size(n_in);
    s.nCBq = (s.B + kMaxTileCols - 1) / kMaxTileCols;
    s.C = round_up4((s.B + s.nCBq - 1) / s.nCBq);
    s.nCBq = (s.B + s.C - 1) / s.C;
    const int per_die = kPGroups / kXcds;
    const int rb_max = per_die / s.nCBq > 0 ? per_die / s.nCBq : 1;
    s.R = whole_slots((n_out + rb_max - 1) / rb_max);
    s.nRBq = (n_out + s.R - 1) / s.R;
    s.nRB = s.nRBq;
    s.nCB = bands_blocks(n_in, s.B, s.C);
    return s;
}

// ---- backward hand-over of the persistent kernel ------------------------------------------------
// A wavefront w of a tile's workgroup owns the ns consecutive tile rows [w ns, (w + 1) ns), one per
// register slot.  The partial deltas that the tiles of layer l + 1 publish for the rows of one tile
// of layer l (a "chunk": one per row block of layer l, gP = row blocks of layer l + 1 partial sums
// per row) are laid out so that each wavefront of the consumer finds its own rows' words side by
// side and reads them with whole-wavefront loads, no word twice and none for another wavefront:
//     word(w, p, a) = (w gP + p) span + a,    span = the power of two >= ns, a < ns the slot.
// Lane t of the wavefront then takes slot t % span and the partial sums p = t / span, t / span +
// 64 / span, ...: its k-th word is word 64 k + t of the wavefront's gP span words.
DBSN_HD inline int slot_span(int ns) {
    int a = 1;
    while (a < ns) a <<= 1;
    return a;
}
DBSN_HD inline int gp_chunk_words(int ns, int gP) { return kWaves * gP * slot_span(ns); }
// j: row within the tile (row block), p: row block of layer l + 1 that publishes
DBSN_HD inline int gp_word_in_chunk(int ns, int gP, int j, int p) {
    const int w = j / ns, a = j - w * ns;
    return (w * gP + p) * slot_span(ns) + a;
}
constexpr int kGpTailWords = 64;   // a wavefront's last load may run up to 63 words past its share: the buffer ends with spare words

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

// Tiles of the hidden layers 1 .. L-1 for one choice of banding, and what follows from them.
struct TilePlan {
    TileShape shape[kMaxLayers + 1];
    int ns[kMaxLayers + 1];       // row slots a wavefront needs for the layer's tile: ceil(R / kWaves)
    int s0[kMaxLayers + 1];       // first slot of the layer when every layer has slots of its own (packed in layer order)
    int gP[kMaxLayers + 1];       // backward partial sums per row of layer l = row blocks of layer l + 1
    bool fwd_local[kMaxLayers + 1];   // the forward partial sums layer l publishes are only read on the publisher's die
    bool bwd_local[kMaxLayers + 1];   // the backward partial sums layer l publishes (for layer l - 1) likewise
    size_t yp_words[kMaxLayers + 1], gp_words[kMaxLayers + 1];   // 64-bit words of the hand-over buffers
    int pairs;                    // banded pairs of layers
    bool ok;                      // every tile within the kernel's limits, output layer included
    bool stationary;              // all tiles of a workgroup fit its registers together
};

// first_pair: 0 = every layer PLAIN; 1 or 2 = layers (first_pair, first_pair + 1), (first_pair + 2, ...) banded
// where both are hidden layers and the neurons between them are at least 256.
inline TilePlan plan_tiles(const int32_t* sizes, int32_t n_sizes, int first_pair) {
    TilePlan t{};
    const int L = n_sizes - 1;
    t.ok = (L >= 2);
    for (int l = 1; l < L; ++l) t.shape[l] = plain_shape(sizes[l - 1], sizes[l]);
    if (first_pair > 0) {
        for (int a = first_pair; a + 1 < L; a += 2) {
            if (sizes[a] < 256) continue;
            t.shape[a] = rowband_shape(sizes[a - 1], sizes[a]);
            t.shape[a + 1] = colband_shape(sizes[a], sizes[a + 1]);
            t.fwd_local[a] = true;
            t.bwd_local[a + 1] = true;
            ++t.pairs;
        }
    }
    int slots = 0;
    for (int l = 1; l < L; ++l) {
        const TileShape& s = t.shape[l];
        if (s.R > kMaxTileRows || s.C > kMaxTileCols) t.ok = false;
        t.ns[l] = (s.R + kWaves - 1) / kWaves;
        if (t.ns[l] > kSlots) t.ok = false;
        slots += t.ns[l];
    }
    t.stationary = slots <= kSlots;
    for (int l = 1, at = 0; l < L; ++l) {
        t.s0[l] = t.stationary ? at : 0;
        at += t.ns[l];
    }
    for (int l = 1; l < L; ++l) {
        t.yp_words[l] = 2 * (size_t)t.shape[l].nCB * sizes[l];
        if (l <= L - 2) {
            t.gP[l] = t.shape[l + 1].nRB;
            t.gp_words[l] = 2 * (size_t)t.shape[l].nRB * gp_chunk_words(t.ns[l], t.gP[l]) + kGpTailWords;   // one chunk per row block
        }
    }
    if (L >= 2) {
        // W_L lives in LDS with its classes padded to a multiple of four
        if ((size_t)((sizes[L] + 3) / 4 * 4) * sizes[L - 1] > (size_t)kTopWMax || sizes[L - 1] > kTopXMax) t.ok = false;
    }
    return t;
}

// The first compile-time register layout the tiles fit (0: none, pack at run time).
inline int choose_layout(const TilePlan& t, int L) {
    if (!t.stationary || !t.ok) return 0;
    for (int cand = 1; cand < kLayouts; ++cand) {
        bool fits = L - 1 <= kLayoutDepth[cand];
        for (int l = 1; l < L && fits; ++l) fits = t.ns[l] <= kLayoutNS[cand][l - 1];
        if (fits) return cand;
    }
    return 0;
}

// Byte offsets of everything a network keeps in its arena.  tiles[0] is the PLAIN cut of every
// layer, tiles[1] the banded cut the library prefers on a chip of eight dies (the one of
// first_pair 1 or 2 that is within the limits, fits the registers and bands more pairs of layers;
// equal to tiles[0] when neither does); the hand-over buffers are sized for the larger of the two.
struct ArenaPlan {
    size_t W[kMaxLayers + 1], b[kMaxLayers + 1], x[kMaxLayers + 1], d[kMaxLayers + 1];
    size_t yp[kMaxLayers + 1], gp[kMaxLayers + 1];
    size_t gpart[2], flags, act[2], total;
    int ld[kMaxLayers + 1], gld, ldact;
    TilePlan tiles[2];
    bool persistent_ok, stationary;   // of tiles[0]
    bool banded;                      // tiles[1] bands at least one pair of layers
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

    // Persistent kernel: yp_l holds the forward partial sums [2][nCB_l][n_l], gp_l the backward ones
    // [2][nRB_l] chunks (see gp_word_in_chunk), as 64-bit {tag, float} words.
    const int L = n_sizes - 1;
    p.tiles[0] = plan_tiles(sizes, n_sizes, 0);
    p.tiles[1] = p.tiles[0];
    // more banded pairs first; between equals the cut that fits a compile-time register layout, then
    // the one whose last pair ends at the last hidden layer (measured a little faster)
    bool has_layout = false;
    for (int first = 1; first <= 2; ++first) {
        const TilePlan t = plan_tiles(sizes, n_sizes, first);
        if (!t.ok || !t.stationary || t.pairs == 0) continue;
        const bool lay = choose_layout(t, L) != 0;
        if (t.pairs > p.tiles[1].pairs || (t.pairs == p.tiles[1].pairs && lay >= has_layout)) {
            p.tiles[1] = t;
            has_layout = lay;
        }
    }
    p.banded = p.tiles[1].pairs > 0;
    p.persistent_ok = p.tiles[0].ok;
    p.stationary = p.tiles[0].stationary;
    for (int l = 1; l < L; ++l) {
        const size_t yw = p.tiles[0].yp_words[l] > p.tiles[1].yp_words[l] ? p.tiles[0].yp_words[l] : p.tiles[1].yp_words[l];
        const size_t gw = p.tiles[0].gp_words[l] > p.tiles[1].gp_words[l] ? p.tiles[0].gp_words[l] : p.tiles[1].gp_words[l];
        p.yp[l] = off; off = align_up(off + sizeof(uint64_t) * yw);
        if (l <= L - 2) { p.gp[l] = off; off = align_up(off + sizeof(uint64_t) * gw); }
    }
    p.total = off;
    return p;
}

}  // namespace dbsn
