// Host-side planning of libdbsn (csrc/dbsn_plan.h, plain C++) exercised without a GPU, meant to be
// built with -fsanitize=address,undefined: random layer shapes, the invariants of the arena layout
// and of the persistent kernel's tile geometry.  Prints "ok <cases>" or the first violation.
#include <cstdio>
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
    for (int l = 1; l < L; ++l) {
        blocks.push_back({p.yp[l], sizeof(uint64_t) * 2 * (size_t)p.nCB[l] * sizes[l]});
        if (l <= L - 2) blocks.push_back({p.gp[l], sizeof(uint64_t) * 2 * (size_t)p.nRB[l] * p.R[l] * p.nRB[l + 1]});
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

    // tiles of the persistent kernel: every weight of a hidden layer in exactly one tile, one tile per workgroup
    int groups = 0;
    bool fits = L >= 2;
    for (int l = 1; l < L; ++l) {
        const int nin = sizes[l - 1], nout = sizes[l];
        CHECK(p.nCB[l] >= 1 && p.nRB[l] >= 1 && p.nCB[l] * p.nRB[l] <= kPGroups);
        CHECK(p.C[l] % 4 == 0 && p.C[l] >= 1 && p.R[l] >= 1);
        CHECK((long long)p.nCB[l] * p.C[l] >= nin && (long long)(p.nCB[l] - 1) * p.C[l] < nin);   // columns: covered, no empty block
        CHECK((long long)p.nRB[l] * p.R[l] >= nout && (long long)(p.nRB[l] - 1) * p.R[l] < nout);  // rows likewise
        CHECK(p.ng[l] * kGR * kWaves >= p.R[l] && (p.ng[l] - 1) * kGR * kWaves < p.R[l]);          // register groups hold the rows
        if (p.R[l] > kMaxTileRows || p.C[l] > kMaxTileCols || p.ng[l] > kNG) fits = false;
        groups += p.ng[l];
    }
    if (L >= 2 && ((size_t)((sizes[L] + 3) / 4 * 4) * sizes[L - 1] > (size_t)kTopWMax || sizes[L - 1] > kTopXMax)) fits = false;
    CHECK(p.persistent_ok == fits);
    CHECK(p.stationary == (groups <= kNG));
    if (p.persistent_ok) {
        for (int l = 1; l < L; ++l) CHECK(p.R[l] <= kMaxTileRows && p.C[l] <= kMaxTileCols && p.ng[l] <= kNG);
        if (p.stationary) {
            int next = 0;
            for (int l = 1; l < L; ++l) {
                CHECK(p.g0[l] == next);   // groups of the layers packed one after the other, disjoint
                next += p.ng[l];
            }
            CHECK(next <= kNG);
        }
    }
    const int lay = choose_layout(p, L);
    CHECK(lay >= 0 && lay < kLayouts);
    if (lay) {
        CHECK(p.stationary && p.persistent_ok && L - 1 <= kLayoutDepth[lay]);
        for (int l = 1; l < L; ++l) {
            CHECK(p.ng[l] <= kLayoutNG[lay][l - 1]);
            CHECK(kLayoutG0[lay][l - 1] + kLayoutNG[lay][l - 1] <= kNG);
            if (l > 1) CHECK(kLayoutG0[lay][l - 1] >= kLayoutG0[lay][l - 2] + kLayoutNG[lay][l - 2]);
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
        if (!(p.persistent_ok && p.stationary && choose_layout(p, 6) == 2)) { std::printf("benchmark net: wrong plan\n"); return 1; }
        sizes = {784, 1000, 500, 10};
        const ArenaPlan q = plan_arena(sizes.data(), 4);
        if (!(q.persistent_ok && q.stationary && choose_layout(q, 3) == 1)) { std::printf("config 0: wrong plan\n"); return 1; }
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
