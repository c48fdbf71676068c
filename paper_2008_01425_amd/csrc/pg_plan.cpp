#include "pg_plan.hpp"

#include <algorithm>
#include <cmath>
#include <set>
#include <utility>

#include "../../include/powergossip.h"

namespace pg {

static inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
static inline int pow2_ceil(int v) {
    int r = 1;
    while (r < v) r <<= 1;
    return r;
}

int compiled_cols(int R) {
    int rc = 1;
    while (rc < R) rc <<= 1;
    return rc;
}

int rows_unroll(int RC, bool light) {
    if (RC < kWideCols) return light ? 4 : 8;
    return 4;
}

int build_plan(Plan &P, int n_workers, int n_edges, const int32_t *edges, const float *edge_w,
               int n_layers, const int32_t *rows, const int32_t *cols, int rank, int power_steps,
               const Tuning &tune) {
    if (n_workers < 1 || n_edges < 0 || n_layers < 1 || rank < 1 || power_steps < 1) return PG_ERR_ARG;
    if ((n_edges > 0 && (!edges || !edge_w)) || !rows || !cols) return PG_ERR_ARG;

    P.n = n_workers;
    P.n_edges = n_edges;
    P.n_layers = n_layers;
    P.rank = rank;
    P.steps = power_steps;
    P.mfma_cols = tune.mfma_cols;
    P.edges.assign(edges, edges + 2 * (size_t)n_edges);
    P.edge_w.assign(edge_w, edge_w + n_edges);

    // ---- topology (graph G and mixing weights W, assumption A4) ----
    std::set<std::pair<int, int>> seen;
    P.incident.assign(n_workers, {});
    std::vector<double> wsum(n_workers, 0.0);
    for (int e = 0; e < n_edges; ++e) {
        int a = edges[2 * e], b = edges[2 * e + 1];
        if (a < 0 || b < 0 || a >= n_workers || b >= n_workers || a == b) return PG_ERR_TOPOLOGY;
        if (!seen.insert({std::min(a, b), std::max(a, b)}).second) return PG_ERR_TOPOLOGY;
        float w = edge_w[e];
        if (!std::isfinite(w) || w < 0.0f) return PG_ERR_ARG;
        wsum[a] += w;
        wsum[b] += w;
        P.incident[a].push_back(e);
        P.incident[b].push_back(e);
    }
    for (int i = 0; i < n_workers; ++i)
        if (wsum[i] > 1.0 + 1e-6) return PG_ERR_ARG;  // the self-weight W_ii would be negative

    size_t max_deg = 0;
    for (int i = 0; i < n_workers; ++i) max_deg = std::max(max_deg, P.incident[i].size());

    // ---- layers: every weight and bias is its own matrix (Section 2) ----
    P.layers.resize(n_layers);
    int64_t off = 0;
    P.elems_per_worker = 0;
    P.message_floats = 0;
    for (int l = 0; l < n_layers; ++l) {
        int p = rows[l], q = cols[l];
        if (p < 1 || q < 1) return PG_ERR_SHAPE;
        LayerInfo &L = P.layers[l];
        L.p = p;
        L.q = q;
        L.r = std::min(rank, std::min(p, q));
        P.max_layer_rank = std::max(P.max_layer_rank, L.r);
        P.max_rows = std::max(P.max_rows, p);
        L.V = (q % 4 == 0) ? 4 : (q % 2 == 0 ? 2 : 1);
        // Row stride.  With 8 or more stacked columns a tile's wavefronts work side by side on
        // 64-column (256-byte) pieces of the same rows; when rows start at arbitrary addresses every
        // piece ends inside a 128-byte line that the neighbouring wavefront touches at another time,
        // and the line crosses the memory interface twice (measured on 650-float rows: a third more
        // bytes read, a quarter more written).  Rows of such layers start on line boundaries.
        const int per_pass = std::min<int>((int)max_deg, std::max(1, kMaxCols / L.r));  // edges one pass takes
        const bool shared_rows = compiled_cols(std::max(1, per_pass * L.r)) >= kWideCols;
        L.ld = (shared_rows && q >= 64) ? (int)round_up(q, 32) : q;
        L.x_off = off;
        off = round_up(off + (int64_t)p * L.ld, 32);
        P.elems_per_worker += (double)p * q;
        P.message_floats += (size_t)L.r * ((size_t)p + q);
    }
    P.param_floats = (size_t)off;
    for (int l = 0; l < n_layers; ++l)
        if (P.layers[l].r > kMaxCols) return PG_ERR_ARG;  // one edge's columns must fit one pass

    // ---- projection state: edge-major, then layer, r_l columns of q_l floats ----
    P.q_off.resize((size_t)n_edges * n_layers);
    P.ph_off.resize((size_t)n_edges * n_layers);
    P.flag_off.resize((size_t)n_edges * n_layers);
    int64_t qo = 0, pho = 0, flo = 0, pdo = 0;
    std::vector<int64_t> pd_off((size_t)n_edges * n_layers);
    for (int e = 0; e < n_edges; ++e)
        for (int l = 0; l < n_layers; ++l) {
            const LayerInfo &L = P.layers[l];
            size_t id = (size_t)e * n_layers + l;
            P.q_off[id] = qo;
            qo = round_up(qo + (int64_t)L.q * L.r, 4);
            P.ph_off[id] = pho;
            pho = round_up(pho + (int64_t)L.p * L.r, 4);
            pd_off[id] = pdo;
            pdo += (int64_t)L.p * L.r;
            P.flag_off[id] = flo;
            flo += L.r;
        }
    P.qstate_floats = (size_t)qo;
    P.pstate_floats = (size_t)pho;

    // ---- tile sizes: the byte targets suit workloads that fill the chip many times over; small
    // parameter sets are cut finer so that every SIMD still gets a tile ----
    Tuning tn = tune;
    {
        const double total_bytes = 4.0 * n_workers * P.elems_per_worker;
        const double slots = 4096.0;  // 256 CUs x 4 SIMDs x a few wavefronts
        P.light = tune.light < 0 ? total_bytes <= (double)kLightBytes : tune.light != 0;
        tn.row_tile_bytes = (int)std::max((P.light ? 4.0 : 8.0) * 1024, std::min((double)tune.row_tile_bytes, total_bytes / slots));
        tn.col_tile_bytes = (int)std::max(32.0 * 1024, std::min((double)tune.col_tile_bytes, 4.0 * total_bytes / slots));
        tn.wide_tile_bytes = (int)std::max(32.0 * 1024, std::min((double)tune.wide_tile_bytes, 4.0 * total_bytes / slots));
        tn.mcol_tile_bytes = (int)std::max(64.0 * 1024, std::min((double)tune.mcol_tile_bytes, 8.0 * total_bytes / slots));
    }

    // ---- per-layer launch geometry ----
    struct Geo {
        int lpr, nseg, seg_len, rows_iter_base;  // row-owner
        int wc;                                  // matrix-core row tiles: wavefronts across the column steps
        bool wide;                               // row-owner: many stacked columns, Q slice in LDS
        bool mrow;                               // row-owner: matrix-core tiles
        int lg, nblk, blk_rows;                  // column-owner
    };
    std::vector<Geo> geo(n_layers);
    constexpr int kColUnroll = 8;
    for (int l = 0; l < n_layers; ++l) {
        const LayerInfo &L = P.layers[l];
        Geo &g = geo[l];
        int nv = L.q / L.V;  // vector loads per row
        // The row blocking depends on the stacked column count; size for the best-connected worker.
        // (a worker with more than kMaxCols stacked columns takes several passes of whole edges)
        const int per_pass = std::min<int>((int)max_deg, std::max(1, kMaxCols / L.r));
        int rc_max = compiled_cols(std::max(1, per_pass * L.r));
        g.wide = rc_max >= kWideCols;
        // Row passes on the matrix cores pay from 16 stacked columns on (measured: at 8 the vector
        // kernels' P-sweep is the faster one) and address a layer with 32-bit byte offsets.
        g.mrow = tune.mfma_rows && rc_max >= tune.mfma_row_cols && (int64_t)L.p * L.ld < ((int64_t)1 << 30);
        // Lanes per row: a whole wavefront for few stacked columns; 16 for many, where the
        // per-row lane reduction (RC values per row) would otherwise rival the products.
        g.lpr = std::min((g.wide && !g.mrow) ? 16 : 64, pow2_ceil(nv));
        int chunk = g.lpr * L.V;  // floats one lane group covers per step
        int nchunks = (L.q + chunk - 1) / chunk;
        int seg_chunks;
        if (!g.wide) {
            // one wavefront per tile: column segments keep a tile near the byte target when a
            // single row is long
            int rows_iter = (64 / g.lpr) * rows_unroll(rc_max, P.light);
            int64_t chunk_bytes = (int64_t)rows_iter * chunk * 4;
            seg_chunks = (int)std::max<int64_t>(1, tn.row_tile_bytes / chunk_bytes);
            g.rows_iter_base = 64 / g.lpr;
        } else if (g.mrow) {
            // matrix cores: steps of 64 columns; a row is cut only when it is very long
            chunk = 64;
            nchunks = (L.q + chunk - 1) / chunk;
            seg_chunks = kMfmaSegCols / chunk;
            g.rows_iter_base = 64 / g.lpr;  // for this layer's workers with few stacked columns
        } else {
            // four wavefronts per tile share the Q slice in LDS: RC * seg_len floats must fit
            seg_chunks = std::max(1, kWideLdsBytes / (rc_max * 4) / chunk);
            g.rows_iter_base = (kThreads / 64) * (64 / g.lpr);
        }
        g.nseg = (nchunks + seg_chunks - 1) / seg_chunks;
        seg_chunks = (nchunks + g.nseg - 1) / g.nseg;
        g.nseg = (nchunks + seg_chunks - 1) / seg_chunks;
        g.seg_len = seg_chunks * chunk;
        g.wc = 1;
        if (g.mrow) g.wc = seg_chunks >= 4 ? 4 : (seg_chunks >= 2 ? 2 : 1);

        // Column-owner kernel: lanes side by side over columns; pick the lane-group width that
        // wastes the fewest lanes on the ragged end of a row (ties go to the wider group).
        int best = 64;
        double best_util = -1;
        for (int lg : {64, 32, 16}) {
            int lgc = std::min(lg, pow2_ceil(nv));
            int groups = (nv + lgc - 1) / lgc;
            double util = (double)nv / ((double)groups * lgc);
            if (util > best_util + 0.05) {
                best_util = util;
                best = lgc;
            }
        }
        // With many stacked columns the kernel is bound by arithmetic and LDS reads of Phat, and
        // one row per wavefront (all 64 lanes side by side) with shorter row blocks measures best.
        const bool col_heavy = rc_max >= 16;
        if (col_heavy && (double)nv / ((double)((nv + 63) / 64) * 64) > 0.6) best = std::min(64, pow2_ceil(nv));
        g.lg = best;
        int row_groups = 4 * (64 / g.lg);
        int64_t row_bytes = (int64_t)g.lg * L.V * 4;
        int64_t want = std::max<int64_t>(1, tn.col_tile_bytes / row_bytes);
        int64_t unit = (int64_t)row_groups * kColUnroll;
        if (g.wide && tune.mfma_cols) {
            // four wavefronts per tile of kMfmaTileCols columns
            want = std::max<int64_t>(16, tn.mcol_tile_bytes / (kMfmaTileCols * 4));
            unit = 16;
        }
        int64_t br = round_up(want, unit);
        if (!(g.wide && tune.mfma_cols)) {
            // the vector column kernel stages the block's Phat slice in LDS: (rows + 1) x columns floats
            const int64_t cap = kColLdsBytes / (4 * rc_max) - 1;
            if (br > cap) br = cap >= unit ? cap / unit * unit : cap;
        }
        if (br >= L.p) br = L.p;
        g.blk_rows = (int)br;
        g.nblk = (L.p + g.blk_rows - 1) / g.blk_rows;
    }

    // ---- (worker, layer) pairs with their stacked columns ----
    // A worker multiplies its matrix by the columns of all its incident edges in one pass when
    // they number at most kMaxCols; otherwise its edges are split into groups of whole edges,
    // one PairDesc (one pass over the matrix) per group.
    P.pairs.clear();
    P.pair_first.assign((size_t)n_layers * n_workers, 0);
    P.pair_count.assign((size_t)n_layers * n_workers, 0);
    P.max_groups = 1;
    P.cols.clear();
    int64_t pwo = 0, qwo = 0;
    // per (layer, worker, incident slot): which group the edge is in, and its first column there
    std::vector<std::vector<std::pair<int, int>>> slot_home((size_t)n_layers * n_workers);
    for (int l = 0; l < n_layers; ++l) {
        const LayerInfo &L = P.layers[l];
        const Geo &g = geo[l];
        const int epg = std::max(1, kMaxCols / L.r);  // edges per group
        for (int i = 0; i < n_workers; ++i) {
            const auto &inc = P.incident[i];
            const size_t li = (size_t)l * n_workers + i;
            const int ngroups = std::max<int>(1, ((int)inc.size() + epg - 1) / epg);
            P.pair_first[li] = (int)P.pairs.size();
            P.pair_count[li] = ngroups;
            P.max_groups = std::max(P.max_groups, ngroups);
            slot_home[li].resize(inc.size());
            for (int gi = 0; gi < ngroups; ++gi) {
                const int s0 = gi * epg, s1 = std::min<int>((int)inc.size(), s0 + epg);
                PairDesc pd;
                pd.worker = i;
                pd.p = L.p;
                pd.q = L.q;
                pd.R = (s1 - s0) * L.r;
                pd.x_off = L.x_off;
                pd.pw_off = pwo;
                pd.qw_off = qwo;
                pd.col0 = (int)P.cols.size();
                pd.lpr = g.lpr;
                pd.nseg = g.nseg;
                pd.seg_len = g.seg_len;
                pd.lg = g.lg;
                pd.nblk = g.nblk;
                pd.blk_rows = g.blk_rows;
                pd.V = L.V;
                pd.wc = g.wc;
                pd.ld = L.ld;
                pwo += (int64_t)g.nseg * pd.R * L.p;
                qwo += (int64_t)g.nblk * pd.R * L.q;
                for (int sl = s0; sl < s1; ++sl) {
                    const int e = inc[sl];
                    slot_home[li][sl] = {(int)P.pairs.size(), (sl - s0) * L.r};
                    for (int k = 0; k < L.r; ++k) {
                        ColDesc c;
                        size_t id = (size_t)e * n_layers + l;
                        c.q_off = P.q_off[id] + (int64_t)k * L.q;
                        c.ph_off = P.ph_off[id] + (int64_t)k * L.p;
                        c.coef = (P.edges[2 * e] == i) ? P.edge_w[e] : -P.edge_w[e];
                        c.pad = 0;
                        P.cols.push_back(c);
                    }
                }
                P.pairs.push_back(pd);
                P.pair_group.push_back(gi);
                P.pair_layer.push_back(l);
            }
        }
    }

    // ---- (edge, layer) records ----
    P.els.resize((size_t)n_layers * n_edges);
    P.comb_tiles.clear();
    for (int l = 0; l < n_layers; ++l) {
        const LayerInfo &L = P.layers[l];
        const Geo &g = geo[l];
        for (int e = 0; e < n_edges; ++e) {
            EdgeLayerDesc &d = P.els[(size_t)l * n_edges + e];
            int a = P.edges[2 * e], b = P.edges[2 * e + 1];
            auto home = [&](int w) {
                const auto &inc = P.incident[w];
                const int sl = (int)(std::find(inc.begin(), inc.end(), e) - inc.begin());
                return slot_home[(size_t)l * n_workers + w][sl];
            };
            const std::pair<int, int> ha = home(a), hb = home(b);
            const PairDesc &pa = P.pairs[ha.first];
            const PairDesc &pb = P.pairs[hb.first];
            const int ja = ha.second, jb = hb.second;
            size_t id = (size_t)e * n_layers + l;
            d.p = L.p;
            d.q = L.q;
            d.r = L.r;
            d.nseg = g.nseg;
            d.nblk = g.nblk;
            d.pad = 0;
            d.pwa_off = pa.pw_off + (int64_t)ja * L.p;
            d.pwb_off = pb.pw_off + (int64_t)jb * L.p;
            d.pwa_seg = (int64_t)pa.R * L.p;
            d.pwb_seg = (int64_t)pb.R * L.p;
            d.qwa_off = pa.qw_off + (int64_t)ja * L.q;
            d.qwb_off = pb.qw_off + (int64_t)jb * L.q;
            d.qwa_blk = (int64_t)pa.R * L.q;
            d.qwb_blk = (int64_t)pb.R * L.q;
            d.pd_off = pd_off[id];
            d.ph_off = P.ph_off[id];
            d.q_off = P.q_off[id];
            d.flag_off = P.flag_off[id];
            int64_t total = (int64_t)L.r * L.q;
            for (int64_t f = 0; f < total; f += kThreads)
                P.comb_tiles.push_back({(int32_t)((size_t)l * n_edges + e), (int32_t)f});
        }
    }

    // ---- workspace sections ----
    size_t o = 0;
    P.ws_pw = o;
    o = (size_t)round_up(o + (size_t)pwo * 8, 256);
    P.ws_qw = o;
    o = (size_t)round_up(o + (size_t)qwo * 8, 256);
    P.ws_pd = o;
    o = (size_t)round_up(o + (size_t)pdo * 8, 256);
    P.ws_ph = o;
    o = (size_t)round_up(o + (size_t)pho * 4, 256);
    P.ws_flag = o;
    o = (size_t)round_up(o + (size_t)flo * 4, 256);
    // tall layers: row chunks for the two-kernel orthonormalisation (36 Gram sums per chunk)
    P.orth_tiles.clear();
    bool tall = false;
    for (int l = 0; l < n_layers; ++l) tall = tall || P.layers[l].p > kOrthTallRows;
    if (tall) {
        for (size_t el = 0; el < P.els.size(); ++el) {
            const int p = P.els[el].p;
            const int nch = (p + kOrthChunkRows - 1) / kOrthChunkRows;
            for (int ch = 0; ch < nch; ++ch)
                P.orth_tiles.push_back({(int32_t)el, ch * kOrthChunkRows,
                                        std::min(kOrthChunkRows, p - ch * kOrthChunkRows), ch, nch, 0});
        }
    }
    P.ws_gpart = o;
    o = (size_t)round_up(o + P.orth_tiles.size() * 36 * 8, 256);
    // unit vectors in R^q of Algorithm 2's odd iterations (state layout)
    P.ws_uq = o;
    o = (size_t)round_up(o + (size_t)qo * 4, 256);
    P.ws_bytes = std::max<size_t>(o, 256);

    // ---- tiles, grouped by kernel instantiation, in address order ----
    P.row_classes.clear();
    P.col_classes.clear();
    P.isolated_pairs.clear();
    P.isolated_elems = 0;
    P.pass_elems = 0;
    // many stacked columns: one class (one kernel instantiation) per vector width
    // (tiles of different column groups of one matrix must not update it at the same time: every
    // group index has launches of its own)
    auto row_class = [&](int RC, int V, bool mfma, int group, bool vec) -> size_t {
        if (RC < kWideCols) V = 0;
        for (size_t k = 0; k < P.row_classes.size(); ++k)
            if (P.row_classes[k].RC == RC && P.row_classes[k].V == V && P.row_classes[k].mfma == mfma &&
                P.row_classes[k].group == group && P.row_classes[k].vec == vec)
                return k;
        P.row_classes.push_back({RC, V, mfma, {}, 0, 0, 0, group, vec});
        return P.row_classes.size() - 1;
    };
    auto col_class = [&](int RC, int V, bool vec) -> size_t {
        if (RC < kWideCols) V = 0;
        for (size_t k = 0; k < P.col_classes.size(); ++k)
            if (P.col_classes[k].RC == RC && P.col_classes[k].V == V && P.col_classes[k].vec == vec) return k;
        P.col_classes.push_back({RC, V, {}, 0, 0, 0, vec});
        return P.col_classes.size() - 1;
    };
    // Vector layers (biases, normalisation scales) are a sliver of the bytes; as tiles of the matrix
    // kernels they run at those kernels' low occupancy, one short latency-bound wavefront after the
    // other.  Where there are many of them they get launches of their own with a kernel that needs
    // few registers; where there are few, another launch would cost more than it saves.
    int64_t vec_pairs = 0;
    for (int l = 0; l < n_layers; ++l)
        if (P.layers[l].q == 1)
            for (int i = 0; i < n_workers; ++i) vec_pairs += P.pair_count[(size_t)l * n_workers + i];
    const bool split_vec = tune.vec_kernels >= 2 || (tune.vec_kernels == 1 && vec_pairs >= kVecClassPairs);
    for (int l = 0; l < n_layers; ++l) {
        const LayerInfo &L = P.layers[l];
        const Geo &g = geo[l];
        for (int i = 0; i < n_workers; ++i)
          for (int gi = 0; gi < P.pair_count[(size_t)l * n_workers + i]; ++gi) {
            int pair = P.pair_first[(size_t)l * n_workers + i] + gi;
            const PairDesc &pd = P.pairs[pair];
            if (pd.R == 0) {  // isolated worker: nothing to multiply, no gossip term
                P.isolated_pairs.push_back(pair);
                P.isolated_elems += (double)L.p * L.q;
                continue;
            }
            int RC = compiled_cols(pd.R);
            const bool mrow = g.mrow && RC >= kWideCols;
            const bool vec = split_vec && L.q == 1 && RC < kWideCols;
            RowClass &rc = P.row_classes[row_class(RC, L.V, mrow, gi, vec)];
            int rows_iter = g.rows_iter_base * rows_unroll(RC, P.light);
            int tile_rows;
            if (RC < kWideCols) {
                int iters = 1;
                if (g.nseg == 1) {
                    int64_t bytes_iter = (int64_t)rows_iter * L.q * 4;
                    iters = (int)std::max<int64_t>(1, tn.row_tile_bytes / bytes_iter);
                }
                tile_rows = rows_iter * iters;
                // the vector kernel: one step (four entries per lane) per tile, so that a long vector
                // is several short independent tiles and not one latency-bound loop
                if (vec) tile_rows = 256;
            } else if (mrow) {
                tile_rows = 16 * kMfmaRowBlocks * (4 / g.wc);
            } else {
                // enough rows that staging the Q slice (RC rows' worth of traffic) is amortised
                int64_t seg_bytes = (int64_t)std::min(g.seg_len, L.q) * 4;
                int64_t want = std::max<int64_t>(8 * RC, tn.wide_tile_bytes / seg_bytes);
                tile_rows = (int)(round_up(want, rows_iter));
                rc.max_seg = std::max(rc.max_seg, g.seg_len);
            }
            for (int r0 = 0; r0 < L.p; r0 += tile_rows)
                for (int sg = 0; sg < g.nseg; ++sg)
                    rc.tiles.push_back({pair, r0, std::min(tile_rows, L.p - r0), sg});
            rc.elems += (double)L.p * L.q;
            P.pass_elems += (double)L.p * L.q;

            ColClass &cc = P.col_classes[col_class(RC, L.V, vec)];
            int cw = (RC >= kWideCols && tune.mfma_cols) ? kMfmaTileCols : g.lg * L.V;
            for (int b = 0; b < g.nblk; ++b)
                for (int c0 = 0; c0 < L.q; c0 += cw) cc.tiles.push_back({pair, c0, b, 0});
            cc.elems += (double)L.p * L.q;
            cc.max_rows = std::max(cc.max_rows, g.blk_rows);
        }
    }
    return PG_OK;
}

}  // namespace pg
