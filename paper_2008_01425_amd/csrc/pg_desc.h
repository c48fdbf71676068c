// Descriptor records shared by the host planner and the gfx950 kernels.
//
// Notation follows the paper: workers i, edges e = (a, b), layers l with X^l in R^{p x q},
// rank r_l, projection state Q_e^l (q x r_l), P_e^l = D_e Q_e (p x r_l), Phat = orth(P).
// A worker multiplies its matrix ONCE per sweep by the stacked columns of all its incident
// edges ("Linearity", Section 3.1): R = deg(i) * r_l stacked columns j = slot * r_l + k.
#pragma once
#include <stdint.h>

namespace pg {

constexpr int kMaxCols = 16;   // largest R = deg(i) * r_l one pass supports
constexpr int kThreads = 256;  // work-group size of the column-owner and combine kernels (4 wavefronts)
constexpr int kRowThreads = 64;  // narrow row-owner kernels: one wavefront per tile
constexpr int64_t kLightBytes = 64ll << 20;  // parameter bytes (all workers) up to which the narrow row kernels block 4 rows, not 8
constexpr int kVecClassPairs = 1024;  // (worker, vector layer) pairs from which vector layers get kernels of their own
constexpr int kWideCols = 8;     // from this many compiled columns on, row tiles stage Q in LDS
constexpr int kWideLdsBytes = 48 * 1024;  // LDS budget of a wide row tile's Q slice
constexpr int kColLdsBytes = 48 * 1024;   // LDS budget of a (vector) column tile's Phat slice
constexpr int kMfmaRowBlocks = 2;  // matrix-core row tiles: blocks of 16 rows per wavefront
constexpr int kMfmaRowCols = 16;    // stacked columns from which row passes run on the matrix cores
constexpr int kMfmaSegCols = 2048;  // matrix-core row tiles: longest column segment
constexpr int kMfmaTileCols = 256;  // matrix-core column tiles: columns per tile (four wavefronts)

// One stacked column of a (worker, layer) pair.
struct ColDesc {
    int64_t q_off;   // float offset of the Q column (edge, layer, k) in the state buffer
    int64_t ph_off;  // float offset of the Phat column (edge, layer, k) in the workspace
    float coef;      // +w_e when the worker is the edge's first endpoint, -w_e otherwise:
                     // X_i -= coef * Phat Q'^T   (Eq. (2); equal and opposite on the two ends)
    int32_t pad;
};

// One (worker, layer) pair.
struct PairDesc {
    int32_t worker, p, q, R;
    int64_t x_off;     // float offset of the layer inside a worker buffer (rows are ld floats apart)
    int64_t pw_off;    // double offset of this pair's partial products X_i S: [seg][j][row]
    int64_t qw_off;    // double offset of this pair's partial products X_i^T T: [blk][j][c]
    int32_t col0;      // first ColDesc of the pair (R consecutive entries)
    int32_t lpr;       // row-owner kernels: lanes that share one row (power of two <= 64)
    int32_t nseg;      // row-owner kernels: column segments a row is split into
    int32_t seg_len;   // floats per segment (multiple of lpr * V; the last one may be shorter)
    int32_t lg;        // column-owner kernel: lanes side by side over columns (power of two <= 64)
    int32_t nblk;      // column-owner kernel: row blocks
    int32_t blk_rows;  // rows per block
    int32_t V;         // floats per vector load on this layer: 4, 2 or 1 (largest that divides q)
    int32_t wc;        // matrix-core row tiles: wavefronts side by side over the column steps (1, 2 or 4)
    int32_t ld;        // floats from one row of the layer to the next in a worker buffer (>= q)
};

// Row-owner tile: rows [row0, row0 + nrows) x column segment seg of one pair.
struct RowTile {
    int32_t pair, row0, nrows, seg;
};

// Column-owner tile: columns [c0, c0 + lg * V) x row block blk of one pair.
struct ColTile {
    int32_t pair, c0, blk, pad;
};

// One (edge, layer): where its partial products, Phat, state and flags live.
struct EdgeLayerDesc {
    int32_t p, q, r, nseg;
    int32_t nblk, pad;
    int64_t pwa_off, pwb_off;  // double offsets of this edge's column 0, segment 0, in worker a / b
    int64_t pwa_seg, pwb_seg;  // stride between segments (R_a * p, R_b * p)
    int64_t qwa_off, qwb_off;  // double offsets of this edge's column 0, block 0, in worker a / b
    int64_t qwa_blk, qwb_blk;  // stride between blocks (R_a * q, R_b * q)
    int64_t pd_off;            // double offset of the Gram-Schmidt scratch: r columns of p
    int64_t ph_off;            // float offset of Phat: r columns of p
    int64_t q_off;             // float offset of the state block: r columns of q
    int64_t flag_off;          // int32 index of the r dropped-column flags
};

// Row chunk of one (edge, layer) for the two-kernel orthonormalisation of tall layers; the
// chunks of an (edge, layer) are consecutive tiles.
struct OrthTile {
    int32_t el, row0, nrows, chunk, nchunks, pad;
};
constexpr int kOrthTallRows = 4096;   // layers taller than this are orthonormalised chunk by chunk
constexpr int kCombPRows = 2048;      // rows per work-group of the p-side combine of single iterations
constexpr int kOrthChunkRows = 1024;  // rows per chunk (one work-group of 256 threads)

// combine_q tile: 256 consecutive elements of the r*q block of one (edge, layer).
struct CombTile {
    int32_t el, first;
};

}  // namespace pg
