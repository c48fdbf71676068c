// gfx950 kernels of the PowerGossip round.  Wavefronts are 64 lanes; every kernel is bound by
// HBM traffic on the parameter matrices, so the design goals are: each X_i is read once per
// sweep for ALL of worker i's edges (the stacked right-hand sides), loads are 128-bit and
// coalesced, and sums are carried in double so that the two large products X_a v and X_b v can
// be subtracted without losing the (much smaller) difference.
//
// Two streaming kernel families cover the passes over X:
//   row_kernel  -- a lane group owns rows: P-sweep (X S), rank-r update, or both fused;
//   col_kernel  -- a lane owns columns:    Q-sweep (X^T T).
// Two small kernels work per edge: orth_kernel (combine + Gram-Schmidt) and comb_kernel.
#include <hip/hip_runtime.h>
#include <float.h>

#include "pg_desc.h"

namespace pg {

template <int V>
struct alignas(4 * V) FV {
    float a[V];
};

template <int V>
__device__ __forceinline__ FV<V> ldv(const float *p) {
    return *reinterpret_cast<const FV<V> *>(p);
}
template <int V>
__device__ __forceinline__ void stv(float *p, const FV<V> &v) {
    *reinterpret_cast<FV<V> *>(p) = v;
}

// Sum over the `width` (power of two) consecutive lanes that contain this lane.
__device__ __forceinline__ double group_sum(double v, int width) {
    for (int o = width >> 1; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// ---------------------------------------------------------------------------------------
// Row-owner kernel.  A group of `lpr` lanes walks along M rows of X_i at once with vector
// loads; per column step it holds the RC stacked right-hand-side columns for its slice.
//   SWEEP : Pw[j][row] = sum_c X[row, c] * Q_j[c]            (Algorithm 2, odd iteration:
//           p_i = X_i v for every incident edge's v in one read of X_i)
//   UPDATE: X[row, c] -= sum_j coef_j * Phat_j[row] * Q'_j[c] (Eq. (2) summed over the edges)
//   both  : the update, then the next round's sweep on the updated values -- the next
//           round's right-hand side is exactly the Q' just applied (warm start).
// ---------------------------------------------------------------------------------------
template <int V, int RC, int M, bool UPDATE, bool SWEEP>
__global__ void __launch_bounds__(kThreads)
row_kernel(const RowTile *__restrict__ tiles, const PairDesc *__restrict__ pairs,
           const ColDesc *__restrict__ cols, float *const *__restrict__ xs,
           const float *__restrict__ qstate, const float *__restrict__ phat,
           double *__restrict__ pw) {
    const RowTile t = tiles[blockIdx.x];
    const PairDesc pd = pairs[t.pair];
    float *__restrict__ X = xs[pd.worker] + pd.x_off;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lpr = pd.lpr;
    const int lpr_shift = __ffs(lpr) - 1;
    const int sub = lane & (lpr - 1);
    const int grp = wave * (64 >> lpr_shift) + (lane >> lpr_shift);
    const int ngrp = (kThreads / 64) * (64 >> lpr_shift);
    const int q = pd.q, R = pd.R;
    const int c_begin = t.seg * pd.seg_len;
    const int c_end = min(q, c_begin + pd.seg_len);
    const int row_end = t.row0 + t.nrows;

    const float *qcol[RC];
    const float *phc[RC];
    float coef[RC];
#pragma unroll
    for (int j = 0; j < RC; ++j) {
        const ColDesc cd = cols[pd.col0 + min(j, R - 1)];
        qcol[j] = qstate + cd.q_off;
        phc[j] = phat + cd.ph_off;
        coef[j] = (j < R) ? cd.coef : 0.0f;
    }

    for (int rbase = t.row0 + grp * M; rbase < row_end; rbase += ngrp * M) {
        int rowi[M];
        bool ok[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            ok[m] = rbase + m < row_end;
            rowi[m] = ok[m] ? rbase + m : row_end - 1;
        }
        double cp[M][RC];
        if (UPDATE) {
#pragma unroll
            for (int m = 0; m < M; ++m)
#pragma unroll
                for (int j = 0; j < RC; ++j) cp[m][j] = (double)coef[j] * (double)phc[j][rowi[m]];
        }
        double acc[M][RC];
#pragma unroll
        for (int m = 0; m < M; ++m)
#pragma unroll
            for (int j = 0; j < RC; ++j) acc[m][j] = 0.0;

        for (int c = c_begin + sub * V; c < c_end; c += lpr * V) {
            FV<V> qv[RC];
#pragma unroll
            for (int j = 0; j < RC; ++j) qv[j] = ldv<V>(qcol[j] + c);
            FV<V> xv[M];
#pragma unroll
            for (int m = 0; m < M; ++m) xv[m] = ldv<V>(X + (int64_t)rowi[m] * q + c);
            if (UPDATE) {
#pragma unroll
                for (int m = 0; m < M; ++m) {
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        double x = (double)xv[m].a[v];
#pragma unroll
                        for (int j = 0; j < RC; ++j) x = fma(-cp[m][j], (double)qv[j].a[v], x);
                        xv[m].a[v] = (float)x;
                    }
                    if (ok[m]) stv<V>(X + (int64_t)rowi[m] * q + c, xv[m]);
                }
            }
            if (SWEEP) {
#pragma unroll
                for (int m = 0; m < M; ++m)
#pragma unroll
                    for (int j = 0; j < RC; ++j)
#pragma unroll
                        for (int v = 0; v < V; ++v)
                            acc[m][j] = fma((double)xv[m].a[v], (double)qv[j].a[v], acc[m][j]);
            }
        }
        if (SWEEP) {
#pragma unroll
            for (int m = 0; m < M; ++m)
#pragma unroll
                for (int j = 0; j < RC; ++j) {
                    double s = group_sum(acc[m][j], lpr);
                    if (sub == 0 && ok[m] && j < R)
                        pw[pd.pw_off + ((int64_t)t.seg * R + j) * pd.p + rowi[m]] = s;
                }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Column-owner kernel.  A lane owns V adjacent columns of X_i and runs down a block of rows;
// `lg` lanes sit side by side, the other lanes of the wavefront (and the other wavefronts)
// take interleaved rows of the same columns and are summed at the end.
//   Qw[blk][j][c] = sum_{row in blk} X[row, c] * Phat_j[row]   (Algorithm 2, even iteration:
//   the product with X^T, for every incident edge in one read of X_i)
// ---------------------------------------------------------------------------------------
template <int V, int RC, int U>
__global__ void __launch_bounds__(kThreads)
col_kernel(const ColTile *__restrict__ tiles, const PairDesc *__restrict__ pairs,
           const ColDesc *__restrict__ cols, float *const *__restrict__ xs,
           const float *__restrict__ phat, double *__restrict__ qw) {
    __shared__ double red[kThreads / 64 - 1][64][V];
    const ColTile t = tiles[blockIdx.x];
    const PairDesc pd = pairs[t.pair];
    const float *__restrict__ X = xs[pd.worker] + pd.x_off;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lg = pd.lg;
    const int lg_shift = __ffs(lg) - 1;
    const int cg = lane & (lg - 1);
    const int rg = wave * (64 >> lg_shift) + (lane >> lg_shift);
    const int RG = (kThreads / 64) * (64 >> lg_shift);
    const int q = pd.q, R = pd.R;
    int c = t.c0 + cg * V;
    const bool cok = c < q;
    if (!cok) c = q - V;
    const int rb = t.blk * pd.blk_rows;
    const int re = min(pd.p, rb + pd.blk_rows);

    const float *phc[RC];
#pragma unroll
    for (int j = 0; j < RC; ++j) phc[j] = phat + cols[pd.col0 + min(j, R - 1)].ph_off;

    double acc[RC][V];
#pragma unroll
    for (int j = 0; j < RC; ++j)
#pragma unroll
        for (int v = 0; v < V; ++v) acc[j][v] = 0.0;

    for (int row = rb + rg; row < re; row += RG * U) {
        FV<V> xv[U];
        float tv[U][RC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int rr = row + u * RG;
            const bool ok = rr < re;
            const int rc = ok ? rr : row;
            xv[u] = ldv<V>(X + (int64_t)rc * q + c);
#pragma unroll
            for (int j = 0; j < RC; ++j) tv[u][j] = ok ? phc[j][rc] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < RC; ++j)
#pragma unroll
                for (int v = 0; v < V; ++v)
                    acc[j][v] = fma((double)xv[u].a[v], (double)tv[u][j], acc[j][v]);
    }
    // lanes of one wavefront that hold the same columns
    for (int o = lg; o < 64; o <<= 1)
#pragma unroll
        for (int j = 0; j < RC; ++j)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[j][v] += __shfl_xor(acc[j][v], o);
    // the four wavefronts, one stacked column at a time
#pragma unroll
    for (int j = 0; j < RC; ++j) {
        if (j < R) {
            if (wave > 0 && lane < lg)
#pragma unroll
                for (int v = 0; v < V; ++v) red[wave - 1][lane][v] = acc[j][v];
            __syncthreads();
            if (wave == 0 && lane < lg && cok) {
                double *dst = qw + pd.qw_off + ((int64_t)t.blk * R + j) * q + c;
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    double s = acc[j][v];
#pragma unroll
                    for (int w = 0; w < kThreads / 64 - 1; ++w) s += red[w][lane][v];
                    dst[v] = s;
                }
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------
// Per (edge, layer): P = Pw_a - Pw_b, then modified Gram-Schmidt over the r columns, left to
// right, in double; Phat is rounded to float when stored.  One work-group per (edge, layer).
// (Eq. (3): normalisation for r = 1; orthogonalisation for r > 1, appendix on rank.)
// ---------------------------------------------------------------------------------------
template <int NT>
__device__ __forceinline__ double block_sum(double v, double *sh) {
    v = group_sum(v, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) s += sh[w];
    __syncthreads();
    return s;
}

template <int NT>
__global__ void __launch_bounds__(NT)
orth_kernel(const EdgeLayerDesc *__restrict__ els, const double *__restrict__ pw,
            double *__restrict__ pdbuf, float *__restrict__ phat, int32_t *__restrict__ flags) {
    __shared__ double sh[NT / 64];
    const EdgeLayerDesc d = els[blockIdx.x];
    const int p = d.p;
    const int tid = threadIdx.x;
    for (int k = 0; k < d.r; ++k) {
        double *col = pdbuf + d.pd_off + (int64_t)k * p;
        double loc = 0.0;
        for (int row = tid; row < p; row += NT) {
            double sa = 0.0, sb = 0.0;
            for (int s = 0; s < d.nseg; ++s) {
                sa += pw[d.pwa_off + s * d.pwa_seg + (int64_t)k * p + row];
                sb += pw[d.pwb_off + s * d.pwb_seg + (int64_t)k * p + row];
            }
            const double v = sa - sb;
            col[row] = v;
            loc += v * v;
        }
        const double norm2_in = block_sum<NT>(loc, sh);
        double norm2 = norm2_in;
        if (k > 0) {
            for (int j = 0; j < k; ++j) {
                const double *prev = pdbuf + d.pd_off + (int64_t)j * p;
                loc = 0.0;
                for (int row = tid; row < p; row += NT) loc += prev[row] * col[row];
                const double dot = block_sum<NT>(loc, sh);
                for (int row = tid; row < p; row += NT) col[row] -= dot * prev[row];
            }
            loc = 0.0;
            for (int row = tid; row < p; row += NT) loc += col[row] * col[row];
            norm2 = block_sum<NT>(loc, sh);
        }
        double floor2 = 1e-10 * norm2_in;
        if (floor2 < (double)FLT_MIN) floor2 = (double)FLT_MIN;
        const bool dropped = !(norm2 >= floor2);
        const double nrm = sqrt(norm2);
        float *dst = phat + d.ph_off + (int64_t)k * p;
        for (int row = tid; row < p; row += NT) {
            const double v = dropped ? 0.0 : col[row] / nrm;
            col[row] = v;
            dst[row] = (float)v;
        }
        if (tid == 0) flags[d.flag_off + k] = dropped ? 1 : 0;
    }
}

// Per (edge, layer): Q' = (sum of worker a's row-block partials) - (worker b's), rounded to
// float into the state buffer; the column of a dropped Phat keeps its old state.
// (Algorithm 2: v_ij <- p_j - p_i, unnormalised.)
__global__ void __launch_bounds__(kThreads)
comb_kernel(const CombTile *__restrict__ tiles, const EdgeLayerDesc *__restrict__ els,
            const double *__restrict__ qw, const int32_t *__restrict__ flags,
            float *__restrict__ qstate) {
    const CombTile t = tiles[blockIdx.x];
    const EdgeLayerDesc d = els[t.el];
    const int64_t idx = (int64_t)t.first + threadIdx.x;  // k * q + c
    if (idx >= (int64_t)d.r * d.q) return;
    const int k = (int)(idx / d.q);
    if (flags[d.flag_off + k]) return;
    double sa = 0.0, sb = 0.0;
    for (int b = 0; b < d.nblk; ++b) {
        sa += qw[d.qwa_off + b * d.qwa_blk + idx];
        sb += qw[d.qwb_off + b * d.qwb_blk + idx];
    }
    qstate[d.q_off + idx] = (float)(sa - sb);
}

}  // namespace pg
