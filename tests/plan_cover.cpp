// Host-only check of the planner (no HIP): for a list of problems, every (worker, layer) pair
// with edges is covered exactly once by its row tiles (rows x column segments) and by its
// column tiles (columns x row blocks), tiles respect what their kernel family assumes, and the
// workspace sections hold the partial sums.  Prints "ok <name>" per problem; exit status 1 on
// the first violation.  Built and run by tests/test_host_api.py.
#include <cstdio>
#include <cstdint>
#include <algorithm>
#include <map>
#include <vector>

#include "../include/powergossip.h"
#include "../paper_2008_01425_amd/csrc/pg_plan.hpp"

using namespace pg;

#define REQUIRE(cond, ...)                       \
    do {                                         \
        if (!(cond)) {                           \
            printf("FAIL %s: ", name);           \
            printf(__VA_ARGS__);                 \
            printf(" [%s]\n", #cond);            \
            return 1;                            \
        }                                        \
    } while (0)

static void ring(int n, std::vector<int32_t> &e) {
    for (int i = 0; i < n; ++i) {
        e.push_back(i);
        e.push_back((i + 1) % n);
    }
}
static void torus(int R, int C, std::vector<int32_t> &e) {
    for (int r = 0; r < R; ++r)
        for (int c = 0; c < C; ++c) {
            int v = r * C + c;
            e.push_back(v);
            e.push_back(r * C + (c + 1) % C);
            e.push_back(v);
            e.push_back(((r + 1) % R) * C + c);
        }
}

static int check(const char *name, int n, const std::vector<int32_t> &e, const std::vector<float> &ew,
                 const std::vector<int32_t> &rows, const std::vector<int32_t> &cols, int rank, int steps,
                 const Tuning &tune) {
    Plan P;
    int rc = build_plan(P, n, (int)ew.size(), e.data(), ew.data(), (int)rows.size(), rows.data(), cols.data(),
                        rank, steps, tune);
    REQUIRE(rc == PG_OK, "build_plan returned %d", rc);
    const int L = (int)rows.size();

    // ---- row tiles: per (pair, segment) the row intervals tile [0, p) ----
    std::map<std::pair<int, int>, std::vector<std::pair<int, int>>> rcover;
    for (const RowClass &c : P.row_classes)
        for (const RowTile &t : c.tiles) {
            REQUIRE(t.pair >= 0 && t.pair < (int)P.pairs.size(), "row tile pair %d", t.pair);
            const PairDesc &pd = P.pairs[t.pair];
            REQUIRE(compiled_cols(pd.R) == c.RC, "pair %d with R=%d in class RC=%d", t.pair, pd.R, c.RC);
            REQUIRE(t.nrows >= 1 && t.row0 >= 0 && t.row0 + t.nrows <= pd.p, "row tile rows %d+%d of %d", t.row0, t.nrows, pd.p);
            REQUIRE(t.seg >= 0 && t.seg < pd.nseg && (int64_t)t.seg * pd.seg_len < pd.q, "segment %d", t.seg);
            if (c.RC >= kWideCols) REQUIRE(c.V == pd.V, "class V=%d, layer V=%d", c.V, pd.V);
            if (c.vec) REQUIRE(pd.q == 1 && c.RC < kWideCols && t.nrows <= 256, "vector tile: q=%d, RC=%d, %d rows", pd.q, c.RC, t.nrows);
            if (tune.vec_kernels == 2 && c.RC < kWideCols) REQUIRE(c.vec == (pd.q == 1), "vector layer outside the vector classes (q=%d)", pd.q);
            if (tune.vec_kernels == 0) REQUIRE(!c.vec, "vector class although switched off");
            if (c.mfma) {
                REQUIRE(pd.wc == 1 || pd.wc == 2 || pd.wc == 4, "wc=%d", pd.wc);
                REQUIRE(pd.seg_len % 64 == 0, "seg_len=%d", pd.seg_len);
                REQUIRE(t.nrows <= 16 * kMfmaRowBlocks * (4 / pd.wc), "matrix-core tile of %d rows, wc=%d", t.nrows, pd.wc);
                REQUIRE((int64_t)pd.p * pd.q < ((int64_t)1 << 30), "layer too large for 32-bit offsets");
            } else if (c.RC >= kWideCols) {
                REQUIRE((int64_t)c.RC * pd.seg_len * 4 <= kWideLdsBytes, "Q slice of %d x %d floats", c.RC, pd.seg_len);
                REQUIRE(c.max_seg >= pd.seg_len, "max_seg");
                REQUIRE(pd.seg_len % (pd.lpr * pd.V) == 0, "seg_len %d, lpr %d, V %d", pd.seg_len, pd.lpr, pd.V);
            } else {
                REQUIRE(pd.lpr >= 1 && pd.lpr <= 64 && (pd.lpr & (pd.lpr - 1)) == 0, "lpr=%d", pd.lpr);
                REQUIRE(pd.seg_len % pd.V == 0, "seg_len %d V %d", pd.seg_len, pd.V);
            }
            rcover[{t.pair, t.seg}].push_back({t.row0, t.row0 + t.nrows});
        }
    // ---- column tiles: per (pair, row block) the column intervals tile [0, q) ----
    std::map<std::pair<int, int>, std::vector<std::pair<int, int>>> ccover;
    for (const ColClass &c : P.col_classes)
        for (const ColTile &t : c.tiles) {
            REQUIRE(t.pair >= 0 && t.pair < (int)P.pairs.size(), "col tile pair %d", t.pair);
            const PairDesc &pd = P.pairs[t.pair];
            REQUIRE(compiled_cols(pd.R) == c.RC, "pair %d with R=%d in column class RC=%d", t.pair, pd.R, c.RC);
            REQUIRE(t.blk >= 0 && t.blk < pd.nblk && (int64_t)t.blk * pd.blk_rows < pd.p, "row block %d", t.blk);
            if (c.vec) REQUIRE(pd.q == 1 && c.RC < kWideCols, "vector column tile: q=%d, RC=%d", pd.q, c.RC);
            if (tune.vec_kernels == 2 && c.RC < kWideCols) REQUIRE(c.vec == (pd.q == 1), "vector layer outside the vector column classes (q=%d)", pd.q);
            const int cw = (c.RC >= kWideCols && P.mfma_cols) ? kMfmaTileCols : pd.lg * pd.V;
            REQUIRE(t.c0 >= 0 && t.c0 < pd.q && t.c0 % cw == 0, "column tile at %d, width %d", t.c0, cw);
            if (!(c.RC >= kWideCols && P.mfma_cols)) {
                REQUIRE(c.max_rows >= pd.blk_rows, "max_rows");
                REQUIRE((int64_t)(pd.blk_rows + 1) * c.RC * 4 <= kColLdsBytes, "Phat slice of %d rows x %d columns", pd.blk_rows, c.RC);
            }
            ccover[{t.pair, t.blk}].push_back({t.c0, std::min(pd.q, t.c0 + cw)});
        }
    auto tiles_exactly = [](std::vector<std::pair<int, int>> v, int end) {
        std::sort(v.begin(), v.end());
        int at = 0;
        for (auto &iv : v) {
            if (iv.first != at) return false;
            at = iv.second;
        }
        return at == end;
    };
    int64_t pw_need = 0, qw_need = 0;
    REQUIRE((int)P.pair_first.size() == L * n && (int)P.pair_count.size() == L * n, "pair index tables");
    int next_pair = 0;
    for (int l = 0; l < L; ++l)
        for (int i = 0; i < n; ++i) {
            const int first = P.pair_first[l * n + i], count = P.pair_count[l * n + i];
            REQUIRE(first == next_pair && count >= 1 && count <= P.max_groups, "groups of layer %d worker %d", l, i);
            next_pair += count;
            int Rsum = 0;
            for (int gi = 0; gi < count; ++gi) {
                const int pair = first + gi;
                const PairDesc &pd = P.pairs[pair];
                REQUIRE(pd.p == rows[l] && pd.q == cols[l] && pd.worker == i, "pair %d fields", pair);
                REQUIRE(P.pair_group[pair] == gi && P.pair_layer[pair] == l, "pair %d group/layer", pair);
                REQUIRE(pd.R <= kMaxCols && pd.R % P.layers[l].r == 0, "R=%d of pair %d", pd.R, pair);
                REQUIRE(pd.ld >= pd.q && (pd.ld == pd.q || pd.ld % 32 == 0), "row stride %d of pair %d", pd.ld, pair);
                Rsum += pd.R;
                if (pd.R == 0) {
                    REQUIRE(count == 1, "empty group beside others");
                    REQUIRE(!rcover.count({pair, 0}) && !ccover.count({pair, 0}), "tiles for a worker without edges");
                    continue;
                }
                REQUIRE((int64_t)pd.nseg * pd.seg_len >= pd.q && (int64_t)(pd.nseg - 1) * pd.seg_len < pd.q, "segments of pair %d", pair);
                REQUIRE((int64_t)pd.nblk * pd.blk_rows >= pd.p && (int64_t)(pd.nblk - 1) * pd.blk_rows < pd.p, "blocks of pair %d", pair);
                for (int sg = 0; sg < pd.nseg; ++sg)
                    REQUIRE(tiles_exactly(rcover[{pair, sg}], pd.p), "rows of pair %d (layer %d, worker %d), segment %d", pair, l, i, sg);
                for (int b = 0; b < pd.nblk; ++b)
                    REQUIRE(tiles_exactly(ccover[{pair, b}], pd.q), "columns of pair %d, block %d", pair, b);
                REQUIRE(pd.pw_off == pw_need && pd.qw_off == qw_need, "partial-sum offsets of pair %d", pair);
                pw_need += (int64_t)pd.nseg * pd.R * pd.p;
                qw_need += (int64_t)pd.nblk * pd.R * pd.q;
            }
            REQUIRE(Rsum == (int)P.incident[i].size() * P.layers[l].r, "stacked columns of layer %d worker %d", l, i);
        }
    REQUIRE(next_pair == (int)P.pairs.size(), "pair count");
    // a row class holds tiles of one column group only (groups of one matrix never share a launch)
    for (const RowClass &c : P.row_classes)
        for (const RowTile &t : c.tiles) REQUIRE(P.pair_group[t.pair] == c.group, "tile of group %d in class of group %d", P.pair_group[t.pair], c.group);
    REQUIRE(P.ws_qw >= P.ws_pw + (size_t)pw_need * 8, "P partial sums do not fit their section");
    REQUIRE(P.ws_pd >= P.ws_qw + (size_t)qw_need * 8, "Q partial sums do not fit their section");
    REQUIRE(P.ws_bytes >= P.ws_uq, "workspace size");
    if (name[0] != 'r' || name[1] != 'a') printf("ok %s\n", name);  // the random problems stay quiet
    return 0;
}

int main() {
    int bad = 0;
    std::vector<Tuning> tunings(4);
    tunings[1].mfma_rows = false;
    tunings[1].vec_kernels = 0;
    tunings[2].mfma_rows = false;
    tunings[2].mfma_cols = false;
    tunings[3].vec_kernels = 2;
    for (const Tuning &tn : tunings) {
        std::vector<int32_t> e;
        ring(4, e);
        bad |= check("tiny", 4, e, std::vector<float>(4, 1 / 3.f), {64, 32, 16}, {32, 16, 1}, 1, 1, tn);
        e.clear();
        ring(16, e);
        bad |= check("vgg16 r=2", 16, e, std::vector<float>(16, 1 / 3.f),
                     {64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512, 10},
                     {27, 576, 576, 1152, 1152, 2304, 2304, 2304, 4608, 4608, 4608, 4608, 4608, 512}, 2, 1, tn);
        e.clear();
        torus(4, 4, e);
        bad |= check("lstm", 16, e, std::vector<float>(32, 0.2f), {33278, 2600, 2600, 2600, 2600},
                     {650, 650, 650, 650, 650}, 4, 2, tn);
        e.clear();
        torus(8, 8, e);
        {
            std::vector<int32_t> r, c;
            for (int i = 0; i < 161; ++i) {
                r.push_back(64 + i * 13 % 2000);
                c.push_back(i % 3 == 0 ? 1 : (i % 5 == 0 ? 147 : 64 * (1 + i % 70)));
            }
            bad |= check("resnet50-like", 64, e, std::vector<float>(128, 0.2f), r, c, 2, 2, tn);
        }
        e.clear();
        ring(3, e);
        bad |= check("odd shapes", 3, e, std::vector<float>(3, 1 / 3.f), {1, 7, 33278, 5, 4099}, {1, 3, 650, 100003, 68}, 3, 1, tn);
        // star with a chord, rank 4: 16, 8, 8, 4 and 4 stacked columns in every layer; one worker without edges
        e = {0, 1, 0, 2, 3, 0, 0, 4, 2, 1};
        bad |= check("mixed degrees", 6, e, {0.2f, 0.2f, 0.2f, 0.2f, 0.15f},
                     {50, 17, 100, 9, 33, 16, 1, 300, 2}, {131, 70, 64, 3, 200, 65, 40, 5000, 9}, 4, 2, tn);
        e.clear();
        torus(3, 3, e);
        bad |= check("torus 3x3 rank 2", 9, e, std::vector<float>(18, 0.2f), {120, 33, 40, 2600}, {260, 12, 1, 63}, 2, 1, tn);
        bad |= check("extreme aspect ratios", 9, e, std::vector<float>(18, 0.2f), {5, 300001, 1, 2, 70001, 33278},
                     {100003, 3, 1, 65537, 1, 1}, 4, 1, tn);
        // more than 16 stacked columns: rank 8 (two groups of two edges), rank 6 (two of two), rank 16 (four of one)
        bad |= check("torus 3x3 rank 8", 9, e, std::vector<float>(18, 0.2f), {120, 33, 40, 8, 700}, {260, 12, 1, 100, 650}, 8, 2, tn);
        bad |= check("torus 3x3 rank 6", 9, e, std::vector<float>(18, 0.2f), {120, 33, 5}, {260, 12, 64}, 6, 1, tn);
        bad |= check("torus 3x3 rank 16", 9, e, std::vector<float>(18, 0.2f), {120, 16, 40}, {260, 300, 1}, 16, 1, tn);
    }
    // seeded random problems: graphs with isolated and high-degree workers, layer shapes from 1 x 1 to
    // very tall and very wide, ranks 1..16, every kernel-family setting
    uint64_t state = 0x9E3779B97F4A7C15ull;
    auto rnd = [&](int lo, int hi) {  // uniform in [lo, hi]
        state ^= state << 13;
        state ^= state >> 7;
        state ^= state << 17;
        return lo + (int)(state % (uint64_t)(hi - lo + 1));
    };
    int nrandom = 0;
    for (int trial = 0; trial < 240 && !bad; ++trial) {
        const int n = rnd(1, 12);
        std::vector<int32_t> e;
        std::vector<int> deg(n, 0);
        for (int a = 0; a < n; ++a)
            for (int b = a + 1; b < n; ++b)
                if (rnd(0, 99) < (trial % 3 == 0 ? 70 : 25)) {
                    if (rnd(0, 1)) { e.push_back(a); e.push_back(b); } else { e.push_back(b); e.push_back(a); }
                    ++deg[a]; ++deg[b];
                }
        const int ne = (int)e.size() / 2;
        const int dmax = std::max(1, *std::max_element(deg.begin(), deg.end()));
        std::vector<float> w(ne, 1.0f / dmax);
        std::vector<int32_t> r, c;
        const int nl = rnd(1, 6);
        for (int l = 0; l < nl; ++l) {
            switch (rnd(0, 5)) {
                case 0: r.push_back(rnd(1, 40)); c.push_back(rnd(1, 40)); break;
                case 1: r.push_back(rnd(1, 90000)); c.push_back(1); break;
                case 2: r.push_back(rnd(1, 8)); c.push_back(rnd(1, 120000)); break;
                case 3: r.push_back(rnd(1, 40000)); c.push_back(rnd(1, 12)); break;
                default: r.push_back(rnd(16, 3000)); c.push_back(rnd(16, 5000)); break;
            }
        }
        char label[64];
        snprintf(label, sizeof(label), "random %d", trial);
        bad |= check(label, n, e, w, r, c, rnd(1, 16), rnd(1, 3), tunings[trial % tunings.size()]);
        ++nrandom;
    }
    if (!bad) printf("ok %d random problems\n", nrandom);
    return bad;
}
