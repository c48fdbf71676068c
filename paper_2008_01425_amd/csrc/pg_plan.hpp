// Host-side planning of a PowerGossip context: validation, buffer layouts, per-worker
// stacked-column tables and the tile lists the kernels are launched over.  No HIP here.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "pg_desc.h"

namespace pg {

struct LayerInfo {
    int p, q, r;        // r = min(rank, p, q)
    int V;              // floats per vector load: 4, 2 or 1 (largest that divides q)
    int ld;             // row stride in a worker buffer, floats: q, or q rounded up to a whole number of
                        // 128-byte lines where several wavefronts share the rows of a tile
    int64_t x_off;      // float offset inside a worker buffer
};

// Tiles of one kernel instantiation: compiled column count RC >= R.  Tiles keep the order
// layer, worker, rows: the address order every pass walks (forwards or backwards).
struct RowClass {
    int RC;
    int V;                  // 0: any vector width (RC < kWideCols); else the one width of this class
    bool mfma;              // tiles cut for the matrix-core row kernel
    std::vector<RowTile> tiles;
    size_t dev_first = 0;   // index of the first tile in the uploaded table
    double elems = 0;       // parameter elements covered (for byte accounting)
    int max_seg = 0;        // RC >= kWideCols: longest column segment (sizes the Q slice in LDS)
    int group = 0;          // which of a worker's column groups these tiles belong to (0 unless a worker
                            // has more than kMaxCols stacked columns)
    bool vec = false;       // vector layers (q = 1) only, run by the light-weight vector kernel
};
struct ColClass {
    int RC;
    int V;                  // as in RowClass
    std::vector<ColTile> tiles;
    size_t dev_first = 0;
    double elems = 0;
    int max_rows = 0;       // largest row block (sizes the staged Phat slice in LDS)
    bool vec = false;       // as in RowClass
};

struct Tuning {
    int row_tile_bytes = 72 * 1024;  // target parameter bytes per row-owner tile (one wavefront)
    int col_tile_bytes = 512 * 1024; // target parameter bytes per column-owner tile (four wavefronts)
    int wide_tile_bytes = 256 * 1024; // target parameter bytes per wide row-owner tile (four wavefronts)
    int mcol_tile_bytes = 512 * 1024; // target parameter bytes per matrix-core column tile (256 columns x a row block)
    // 8-16 stacked columns: which passes run on the matrix cores
    bool mfma_cols = true;            // Q-sweep
    bool mfma_rows = true;            // P-sweep and update ...
    int mfma_row_cols = kMfmaRowCols; // ... of layers with at least this many stacked columns (8 or 16)
    int light = -1;                   // blocking for small parameter sets: -1 by size, 0 never, 1 always
    int vec_kernels = 1;              // vector layers in launches of their own (light-weight kernels):
                                      // 0 never, 1 where there are many of them, 2 always
};

struct Plan {
    int n = 0, n_edges = 0, n_layers = 0, rank = 0, steps = 0;
    bool mfma_cols = true;                   // Q-sweep over 8-16 stacked columns runs on the matrix cores
    std::vector<int32_t> edges;   // 2 * n_edges
    std::vector<float> edge_w;
    std::vector<LayerInfo> layers;
    std::vector<std::vector<int>> incident;  // per worker: edge ids in edge-list order

    size_t param_floats = 0, qstate_floats = 0, pstate_floats = 0, message_floats = 0;
    double elems_per_worker = 0;             // N = sum p*q
    std::vector<int64_t> q_off;              // [e * L + l]

    // workspace sections (byte offsets) and their sizes
    size_t ws_pw = 0, ws_qw = 0, ws_pd = 0, ws_ph = 0, ws_flag = 0, ws_gpart = 0, ws_uq = 0, ws_bytes = 0;
    std::vector<int64_t> ph_off;             // [e * L + l] float offset inside the Phat section
    std::vector<int64_t> flag_off;           // [e * L + l] int32 index inside the flag section

    std::vector<PairDesc> pairs;             // one per (layer, worker, column group)
    std::vector<int> pair_first, pair_count; // [l * n + i]: that worker's groups in `pairs`
    std::vector<int> pair_group, pair_layer; // per pair: its group index and layer
    int max_groups = 1;                      // most column groups any (worker, layer) has
    double pass_elems = 0;                   // elements one sweep reads: sum of p * q over all pairs with edges
    std::vector<ColDesc> cols;
    std::vector<EdgeLayerDesc> els;          // [l * n_edges + e]
    std::vector<CombTile> comb_tiles;
    std::vector<int32_t> isolated_pairs;     // (worker, layer) pairs of workers without edges
    double isolated_elems = 0;               // their parameter count
    std::vector<OrthTile> orth_tiles;        // filled only when some layer has more than one row chunk
    std::vector<RowClass> row_classes;
    std::vector<ColClass> col_classes;
    // A small parameter set (all workers together at most kLightBytes) does not fill the chip with
    // the tiles that serve a large one: a pass is then as long as one wavefront's chain of
    // dependent loads, so the narrow row kernels block fewer rows per lane group (half the
    // registers, twice the wavefronts per SIMD) over tiles half as large.
    bool light = false;
    int max_layer_rank = 1;                  // largest r_l
    int max_rows = 1;                        // largest p_l
};

// Rows one lane group covers per step for a compiled column count (register blocking); `light`:
// the blocking for small parameter sets (see Plan::light).
int rows_unroll(int RC, bool light = false);
// Smallest compiled column count >= R (1, 2, 4, 8, 16).
int compiled_cols(int R);

// Returns PG_OK or a negative status; on success `plan` is complete.
int build_plan(Plan &plan, int n_workers, int n_edges, const int32_t *edges, const float *edge_w,
               int n_layers, const int32_t *rows, const int32_t *cols, int rank, int power_steps,
               const Tuning &tune);

}  // namespace pg
