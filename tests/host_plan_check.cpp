// Host-side planning of libdbsn (csrc/dbsn_plan.h, plain C++) exercised without a GPU, meant to be
// built with -fsanitize=address,undefined: random layer shapes, the invariants of the arena layout
// and of the persistent kernel's tile geometry.  Prints "ok <cases>" or the first violation.
#include <cstdio>
#include <algorithm>
#include <cstdlib>
#include <random>
#include <vector>

#include "dbsn_plan.h"

using namespace dbsn;

#define CHECK(cond)                                                                     \
    do {                                                                                \
        if (!(cond)) {                                                                  \
            std::printf("violated: %s (line %d), sizes:", #cond, __LINE__);             \
            for (int v : sizes) std::printf(" %d", v);                                  \
            std::printf("\n");                                                          \
            return 1;                                                                   \
        }                                                                               \
    } while (0)

static int check(const std::vector<int32_t>& sizes) {
    const int n_sizes = (int)sizes.size(), L = n_sizes - 1;
    CHECK(shape_ok(sizes.data(), n_sizes));
    const ArenaPlan p = plan_arena(sizes.data(), n_sizes);
    // arena: blocks in order, 256-byte aligned, none overlapping, all inside `total`
    std::vector<std::pair<size_t, size_t>> blocks;   // (offset, bytes)
    for (int l = 1; l <= L; ++l) {
        CHECK(p.ld[l] % 4 == 0 && p.ld[l] >= sizes[l - 1] && p.ld[l] < sizes[l - 1] + 4);
        blocks.push_back({p.W[l], sizeof(float) * (size_t)sizes[l] * p.ld[l]});
        blocks.push_back({p.b[l], sizeof(float) * (size_t)sizes[l]});
        blocks.push_back({p.x[l], sizeof(float) * (size_t)sizes[l]});
        blocks.push_back({p.d[l], sizeof(float) * (size_t)sizes[l]});
    }
    for (int k = 0; k < 2; ++k) blocks.push_back({p.gpart[k], sizeof(float) * (size_t)kArenaGroups * p.gld});
    blocks.push_back({p.flags, 256});
    for (int k = 0; k < 2; ++k) blocks.push_back({p.act[k], sizeof(float) * (size_t)kBatchSamples * p.ldact});
    for (int l = 1; l < L; ++l) {   // the hand-over buffers hold either cut
        const size_t yw = std::max(p.tiles[0].yp_words[l], p.tiles[1].yp_words[l]);
        blocks.push_back({p.yp[l], sizeof(uint64_t) * yw});
        if (l <= L - 2) blocks.push_back({p.gp[l], sizeof(uint64_t) * std::max(p.tiles[0].gp_words[l], p.tiles[1].gp_words[l])});
    }
    size_t at = 0;
    for (auto& b : blocks) {
        CHECK(b.first % kArenaAlign == 0);
        CHECK(b.first >= at);
        at = b.first + b.second;
    }
    CHECK(p.total >= at && p.total % kArenaAlign == 0);
    CHECK(p.gld % 64 == 0);
    CHECK(p.ldact % 4 == 0);
    for (int l = 1; l <= L; ++l) CHECK(p.gld >= sizes[l - 1] && p.ldact >= sizes[l]);
    CHECK(nch_for(p.gld) >= 1 && nch_for(p.gld) * 256 >= p.gld);
    CHECK(p.persistent_ok == p.tiles[0].ok && p.stationary == p.tiles[0].stationary);
    CHECK(p.tiles[0].pairs == 0);
    CHECK(p.banded == (p.tiles[1].pairs > 0));
    if (p.banded) CHECK(p.tiles[1].ok && p.tiles[1].stationary);

    // tiles of the persistent kernel, both cuts: every weight of a hidden layer in exactly one tile, at most
    // one tile per workgroup; blocks numbered without holes; banded pairs keep their hand-overs on one die
    for (int v = 0; v < 2; ++v) {
        const TilePlan& t = p.tiles[v];
        int slots = 0;
        bool fits = L >= 2;
        for (int l = 1; l < L; ++l) {
            const int nin = sizes[l - 1], nout = sizes[l];
            const TileShape& s = t.shape[l];
            CHECK(s.C % 4 == 0 && s.C >= 4 && s.R >= 1 && s.B % 4 == 0);
            CHECK(s.nCB >= 1 && s.nRB >= 1);
            // (weight by weight for layers up to 2^20 weights; for all layers through the blocks: tiles =
            // every column block x every row block, each once, the blocks of either axis end to end)
            const bool exhaustive = (size_t)nin * nout <= (1u << 20);
            std::vector<int> own(exhaustive ? (size_t)nin * nout : 0, 0);
            std::vector<int> cb_seen(s.nCB, 0), rb_seen(s.nRB, 0), cb_c0(s.nCB, -1), cb_ce(s.nCB, -1), rb_r0(s.nRB, -1), rb_re(s.nRB, -1);
            std::vector<int> pair_seen((size_t)s.nCB * s.nRB, 0);
            int tiles = 0;
            for (int g = 0; g < kPGroups; ++g) {
                TileAt a;
                if (!tile_at(s, nin, nout, g, a)) continue;
                ++tiles;
                CHECK(a.cb >= 0 && a.cb < s.nCB && a.rb >= 0 && a.rb < s.nRB);
                CHECK(a.Ceff >= 1 && a.Ceff <= s.C && a.Reff >= 1 && a.Reff <= s.R);
                CHECK(a.c0 % 4 == 0 && a.c0 >= 0 && a.c0 + a.Ceff <= nin && a.r0 >= 0 && a.r0 + a.Reff <= nout);
                cb_seen[a.cb] = 1; rb_seen[a.rb] = 1;
                CHECK(cb_c0[a.cb] == -1 || (cb_c0[a.cb] == a.c0 && cb_ce[a.cb] == a.Ceff));
                CHECK(rb_r0[a.rb] == -1 || (rb_r0[a.rb] == a.r0 && rb_re[a.rb] == a.Reff));
                cb_c0[a.cb] = a.c0; cb_ce[a.cb] = a.Ceff; rb_r0[a.rb] = a.r0; rb_re[a.rb] = a.Reff;
                CHECK(++pair_seen[(size_t)a.rb * s.nCB + a.cb] == 1);
                for (int r = 0; r < a.Reff; ++r) {
                    int rb, j, reff;
                    row_block_at(s, nout, a.r0 + r, rb, j, reff);
                    CHECK(rb == a.rb && j == r && reff == a.Reff);
                    if (exhaustive)
                        for (int c = 0; c < a.Ceff; ++c) ++own[(size_t)(a.r0 + r) * nin + a.c0 + c];
                }
                if (s.kind == TILE_ROWBAND) CHECK(a.r0 / s.B == g % kXcds && (a.r0 + a.Reff - 1) / s.B == g % kXcds);
                if (s.kind == TILE_COLBAND) CHECK(a.c0 / s.B == g % kXcds && (a.c0 + a.Ceff - 1) / s.B == g % kXcds);
            }
            for (int e : own) CHECK(e == 1);
            for (int e : cb_seen) CHECK(e == 1);
            for (int e : rb_seen) CHECK(e == 1);
            for (int e : pair_seen) CHECK(e == 1);
            CHECK(tiles == s.nCB * s.nRB && tiles <= kPGroups);
            for (int c = 0, at = 0; c < s.nCB; ++c) { CHECK(cb_c0[c] == at); at += cb_ce[c]; if (c == s.nCB - 1) CHECK(at == nin); }
            for (int r = 0, at = 0; r < s.nRB; ++r) { CHECK(rb_r0[r] == at); at += rb_re[r]; if (r == s.nRB - 1) CHECK(at == nout); }
            CHECK(t.ns[l] * kWaves == s.R);   // tiles take whole slots
            if (s.R > kMaxTileRows || s.C > kMaxTileCols || t.ns[l] > kSlots) fits = false;
            slots += t.ns[l];
            CHECK(t.yp_words[l] == 2 * (size_t)s.nCB * nout);
            if (l <= L - 2) {
                const int gP = t.gP[l], ns = t.ns[l], span = slot_span(ns), chunk = gp_chunk_words(ns, gP);
                CHECK(gP == t.shape[l + 1].nRB && t.gp_words[l] == 2 * (size_t)s.nRB * chunk + kGpTailWords);
                CHECK(span >= ns && span < 2 * ns + 1 && (span & (span - 1)) == 0 && 64 % span == 0 && chunk == kWaves * gP * span);
                // backward hand-over: every (row of a tile, publishing row block) has a word of its own in the
                // chunk, inside the share of the wavefront that owns the row, and a wavefront that reads its
                // share 64 words at a time stays within the spare words behind the last chunk
                std::vector<char> used(chunk, 0);
                for (int j = 0; j < s.R; ++j)
                    for (int q = 0; q < gP; ++q) {
                        const int wd = gp_word_in_chunk(ns, gP, j, q);
                        CHECK(wd >= 0 && wd < chunk && !used[wd]);
                        used[wd] = 1;
                        const int w = j / ns;
                        CHECK(w < kWaves && wd >= w * gP * span && wd < (w + 1) * gP * span);
                        // the lane and load that read it: lane t = (p % nc) span + a, load k = p / nc
                        const int nc = 64 / span, a = j - w * ns;
                        CHECK(wd == w * gP * span + 64 * (q / nc) + (q % nc) * span + a);
                    }
                const int nc = 64 / span, K = (gP + nc - 1) / nc;
                CHECK((kWaves - 1) * gP * span + 64 * K <= chunk + kGpTailWords);
            }
            // a banded pair: the lower layer row-banded, the upper column-banded with the same bands
            if (t.fwd_local[l]) {
                CHECK(l + 1 < L && s.kind == TILE_ROWBAND && t.shape[l + 1].kind == TILE_COLBAND && t.bwd_local[l + 1]);
                CHECK(s.B == t.shape[l + 1].B);
            }
            if (s.kind == TILE_ROWBAND) CHECK(t.fwd_local[l]);
            if (s.kind == TILE_COLBAND) CHECK(t.bwd_local[l] && l >= 2 && t.shape[l - 1].kind == TILE_ROWBAND);
            if (s.kind == TILE_PLAIN) CHECK(!t.fwd_local[l] && !t.bwd_local[l]);
        }
        if (L >= 2 && ((size_t)((sizes[L] + 3) / 4 * 4) * sizes[L - 1] > (size_t)kTopWMax || sizes[L - 1] > kTopXMax)) fits = false;
        CHECK(t.ok == fits);
        CHECK(t.stationary == (slots <= kSlots));
        if (t.ok && t.stationary) {
            int next = 0;
            for (int l = 1; l < L; ++l) {
                CHECK(t.s0[l] == next);   // slots of the layers packed one after the other, disjoint
                next += t.ns[l];
            }
            CHECK(next <= kSlots);
        }
        const int lay = choose_layout(t, L);
        CHECK(lay >= 0 && lay < kLayouts);
        if (lay) {
            CHECK(t.stationary && t.ok && L - 1 <= kLayoutDepth[lay]);
            for (int l = 1; l < L; ++l) {
                CHECK(t.ns[l] <= kLayoutNS[lay][l - 1]);
                CHECK(kLayoutS0[lay][l - 1] + kLayoutNS[lay][l - 1] <= kSlots);
                if (l > 1) CHECK(kLayoutS0[lay][l - 1] >= kLayoutS0[lay][l - 2] + kLayoutNS[lay][l - 2]);
            }
        }
    }
    return 0;
}

int main(int argc, char** argv) {
    const int cases = argc > 1 ? std::atoi(argv[1]) : 20000;
    std::mt19937 rng(12345);
    std::vector<int32_t> sizes;
    // the paper's nets first
    const std::vector<std::vector<int32_t>> fixed = {
        {784, 1000, 500, 10}, {784, 1500, 1000, 500, 10}, {784, 2000, 1500, 1000, 500, 10},
        {784, 2500, 2000, 1500, 1000, 500, 10}, {784, 1000, 1000, 1000, 1000, 1000, 1000, 1000, 1000, 1000, 10},
        {784, 10}, {1, 1}, {4096, 4096, 64}, {784, 3584, 3584, 3584, 1000, 10}};
    for (auto& f : fixed) {
        sizes = f;
        if (check(sizes)) return 1;
    }
    {
        sizes = {784, 2500, 2000, 1500, 1000, 500, 10};
        const ArenaPlan p = plan_arena(sizes.data(), 7);
        if (!(p.persistent_ok && p.stationary && choose_layout(p.tiles[0], 6) == 2 && p.banded && p.tiles[1].pairs == 2 &&
              choose_layout(p.tiles[1], 6) == 2)) { std::printf("benchmark net: wrong plan\n"); return 1; }
        sizes = {784, 1000, 500, 10};
        const ArenaPlan q = plan_arena(sizes.data(), 4);
        if (!(q.persistent_ok && q.stationary && choose_layout(q.tiles[0], 3) == 1 && q.banded && q.tiles[1].pairs == 1 &&
              choose_layout(q.tiles[1], 3) == 1)) { std::printf("config 0: wrong plan\n"); return 1; }
        sizes = {784, 1000, 1000, 1000, 1000, 1000, 1000, 1000, 1000, 1000, 10};
        const ArenaPlan r = plan_arena(sizes.data(), 11);
        if (!(r.banded && r.tiles[1].pairs == 4 && choose_layout(r.tiles[0], 10) == 3 && choose_layout(r.tiles[1], 10) == 3)) {
            std::printf("nine hidden layers: wrong plan\n"); return 1; }
    }
    for (int c = 0; c < cases; ++c) {
        const int L = 1 + (int)(rng() % DBSN_MAX_LAYERS);
        sizes.assign(L + 1, 0);
        for (int i = 0; i <= L; ++i) {
            const int kind = (int)(rng() % 4);
            const int hi = i == L ? DBSN_MAX_CLASSES : DBSN_MAX_WIDTH;
            int v = kind == 0 ? 1 + (int)(rng() % 8) : kind == 1 ? hi - (int)(rng() % 8) : 1 + (int)(rng() % hi);
            sizes[i] = v < 1 ? 1 : (v > hi ? hi : v);
        }
        if (check(sizes)) return 1;
    }
    // shapes the library must refuse
    const int32_t too_wide[] = {784, DBSN_MAX_WIDTH + 1, 10}, zero[] = {784, 0, 10}, classes[] = {784, 100, DBSN_MAX_CLASSES + 1};
    std::vector<int32_t> deep(DBSN_MAX_LAYERS + 2, 10);
    if (shape_ok(too_wide, 3) || shape_ok(zero, 3) || shape_ok(classes, 3) || shape_ok(deep.data(), (int)deep.size()) ||
        shape_ok(too_wide, 1) || shape_ok(nullptr, 3)) {
        std::printf("a bad shape was accepted\n");
        return 1;
    }
    std::printf("ok %d\n", cases);
    return 0;
}
