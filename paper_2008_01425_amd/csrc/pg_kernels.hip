// gfx950 kernels of the PowerGossip round.  Wavefronts are 64 lanes; every kernel is bound by
// HBM traffic on the parameter matrices, so the design goals are: each X_i is read once per
// sweep for ALL of worker i's edges (the stacked right-hand sides), loads are 128-bit and
// coalesced, and sums are carried in double so that the two large products X_a v and X_b v can
// be subtracted without losing the (much smaller) difference.
//
// Two streaming kernel families cover the passes over X:
//   row_kernel  -- a lane group owns rows: P-sweep (X S), rank-r update, or both fused;
//   col_kernel  -- a lane owns columns:    Q-sweep (X^T T).
// With up to 4 stacked columns the vector ALUs keep up with HBM.  From 8 on (row_wide_kernel)
// they fall behind, and at 8 (Q-sweep) or 16 (all passes) the contraction moves to the double
// precision matrix cores: mrow_kernel, mcol_kernel.
// Small kernels work per edge: orth_gram_kernel / orth_kernel (combine + Gram-Schmidt) and comb_kernel.
#include <hip/hip_runtime.h>
#include <float.h>

#include "pg_desc.h"

namespace pg {

#define PG_GLOBAL __attribute__((address_space(1)))
// Instruction-scheduling fence: nothing is moved across it.
#define PG_FENCE() __builtin_amdgcn_sched_barrier(0)

// V floats moved by one load / store instruction (128, 64 or 32 bits).
template <int V>
struct VecT {
    typedef float T __attribute__((ext_vector_type(V)));
};

// Loads and stores through explicitly global pointers: parameter buffers are reached through a
// pointer table, so the compiler cannot see that they are global and would emit flat accesses.
template <int V>
__device__ __forceinline__ typename VecT<V>::T ldg(const float *p) {
    return *(const PG_GLOBAL typename VecT<V>::T *)p;
}
template <int V>
__device__ __forceinline__ void stg(float *p, typename VecT<V>::T v) {
    *(PG_GLOBAL typename VecT<V>::T *)p = v;
}
__device__ __forceinline__ float ldg1(const float *p) { return *(const PG_GLOBAL float *)p; }

// Which tile this work-group takes: the tile list in order, or backwards, so that a pass can start
// on the data the previous pass touched last (still resident in the memory-side cache).
__device__ __forceinline__ int tile_index(int ntiles, int reverse) {
    return reverse ? ntiles - 1 - (int)blockIdx.x : (int)blockIdx.x;
}

// ---- wavefront reductions on the DPP / swizzle network --------------------------------
template <int CTRL>
__device__ __forceinline__ double dpp_mov(double v) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    // every lane has a valid source lane under these controls, so no `old` value is needed
    lo = __builtin_amdgcn_mov_dpp(lo, CTRL, 0xf, 0xf, false);
    hi = __builtin_amdgcn_mov_dpp(hi, CTRL, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double swizzle_xor16(double v) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_ds_swizzle(lo, 0x401f);  // bit mode: and 0x1f, or 0, xor 0x10
    hi = __builtin_amdgcn_ds_swizzle(hi, 0x401f);
    return __hiloint2double(hi, lo);
}
// Sum over the `width` (power of two) consecutive lanes that contain this lane; every lane of
// the group receives the sum.  Lane exchanges: quad permutes (1, 2), mirror within 8 and within
// 16 lanes (each lane of a quad / octet already holds that quad's / octet's sum), swizzle across
// 16, and a cross-half shuffle for 64.
__device__ __forceinline__ double group_sum(double v, int width) {
    if (width > 1) v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
    if (width > 2) v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
    if (width > 4) v += dpp_mov<0x141>(v);  // row_half_mirror
    if (width > 8) v += dpp_mov<0x140>(v);  // row_mirror
    if (width > 16) v += swizzle_xor16(v);
    if (width > 32) v += __shfl_xor(v, 32);
    return v;
}

// The same for N values at once, exchange step outermost (one branch per step, not per value).
template <int N>
__device__ __forceinline__ void group_sum_all(double (&v)[N], int width) {
    if (width > 1) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_mov<0xB1>(v[i]);
    }
    if (width > 2) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_mov<0x4E>(v[i]);
    }
    if (width > 4) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_mov<0x141>(v[i]);
    }
    if (width > 8) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_mov<0x140>(v[i]);
    }
    if (width > 16) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += swizzle_xor16(v[i]);
    }
    if (width > 32) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += __shfl_xor(v[i], 32);
    }
}

// ---------------------------------------------------------------------------------------
// Row-owner kernel for few stacked columns (RC <= 4): one wavefront per tile.  A group of `lpr`
// lanes walks along M rows of X_i at once with vector loads; per column step it holds the RC
// stacked right-hand-side columns for its slice in registers (they come from L1/L2).  The
// loads of step c + D are issued before the arithmetic of step c.
//   SWEEP : Pw[j][row] = sum_c X[row, c] * Q_j[c]            (Algorithm 2, odd iteration:
//           p_i = X_i v for every incident edge's v in one read of X_i)
//   UPDATE: X[row, c] -= sum_j coef_j * Phat_j[row] * Q'_j[c] (Eq. (2) summed over the edges)
//   both  : the update, then the next round's sweep on the updated values -- the next
//           round's right-hand side is exactly the Q' just applied (warm start).
// ---------------------------------------------------------------------------------------
template <int V, int RC, int M, int D, bool UPDATE, bool SWEEP, bool GRAD>
__device__ __forceinline__ void row_body(const RowTile &t, const PairDesc &pd,
                                         const ColDesc *__restrict__ cols, float *X,
                                         const float *__restrict__ qstate,
                                         const float *__restrict__ phat, double *__restrict__ pw,
                                         const float *Gp, double eta) {
    typedef typename VecT<V>::T vec;
    const int lane = threadIdx.x;
    const int lpr = pd.lpr;
    const int lpr_shift = __ffs(lpr) - 1;
    const int sub = lane & (lpr - 1);
    const int grp = lane >> lpr_shift;
    const int ngrp = 64 >> lpr_shift;
    const int q = pd.q, R = pd.R;
    const int c_begin = t.seg * pd.seg_len;
    const int c_end = min(q, c_begin + pd.seg_len);
    const int row_end = t.row0 + t.nrows;
    const int step = lpr * V;

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
        float *xrow[M];
        const float *grow[M];
        bool ok[M];
        int rowi[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            ok[m] = rbase + m < row_end;
            rowi[m] = ok[m] ? rbase + m : row_end - 1;
            xrow[m] = X + (int64_t)rowi[m] * pd.ld;
            grow[m] = GRAD ? Gp + (int64_t)rowi[m] * pd.ld : nullptr;
        }
        double cp[M][RC];
        if (UPDATE) {
#pragma unroll
            for (int m = 0; m < M; ++m)
#pragma unroll
                for (int j = 0; j < RC; ++j)
                    cp[m][j] = (double)coef[j] * (double)ldg1(phc[j] + rowi[m]);
        }
        double acc[M][RC];
#pragma unroll
        for (int m = 0; m < M; ++m)
#pragma unroll
            for (int j = 0; j < RC; ++j) acc[m][j] = 0.0;

        auto load = [&](int c, vec(&xv)[M], vec(&qv)[RC], vec(&gv)[GRAD ? M : 1]) {
#pragma unroll
            for (int j = 0; j < RC; ++j) qv[j] = ldg<V>(qcol[j] + c);
#pragma unroll
            for (int m = 0; m < M; ++m) xv[m] = ldg<V>(xrow[m] + c);
            if (GRAD) {
#pragma unroll
                for (int m = 0; m < M; ++m) gv[GRAD ? m : 0] = ldg<V>(grow[m] + c);
            }
        };
        auto process = [&](int c, vec(&xv)[M], vec(&qv)[RC], vec(&gv)[GRAD ? M : 1]) {
            double qd[RC][V];
#pragma unroll
            for (int j = 0; j < RC; ++j)
#pragma unroll
                for (int v = 0; v < V; ++v) qd[j][v] = (double)qv[j][v];
#pragma unroll
            for (int m = 0; m < M; ++m) {
                double xd[V];
#pragma unroll
                for (int v = 0; v < V; ++v) xd[v] = (double)xv[m][v];
                if (UPDATE) {
#pragma unroll
                    for (int v = 0; v < V; ++v) {
#pragma unroll
                        for (int j = 0; j < RC; ++j) xd[v] = fma(-cp[m][j], qd[j][v], xd[v]);
                        if (GRAD) xd[v] = fma(-eta, (double)gv[GRAD ? m : 0][v], xd[v]);
                        xv[m][v] = (float)xd[v];
                        xd[v] = (double)xv[m][v];  // the sweep uses the stored (rounded) value
                    }
                    if (ok[m]) stg<V>(xrow[m] + c, xv[m]);
                }
                if (SWEEP) {
#pragma unroll
                    for (int j = 0; j < RC; ++j)
#pragma unroll
                        for (int v = 0; v < V; ++v) acc[m][j] = fma(xd[v], qd[j][v], acc[m][j]);
                }
            }
        };

        const int c0 = c_begin + sub * V;
        if (c0 < c_end) {
            // Software pipeline over the column steps: the loads of step s + D are issued before
            // the arithmetic of step s, through a ring of D + 1 register buffers (indices are
            // compile-time after unrolling).  PG_FENCE keeps the compiler from sinking a prefetch
            // below the arithmetic it overlaps.
            constexpr int NB = D + 1;
            vec xb[NB][M], qb[NB][RC], gb[NB][GRAD ? M : 1];
            const int nsteps = (c_end - c0 - 1) / step + 1;
#pragma unroll
            for (int k = 0; k < D; ++k)
                if (k < nsteps) load(c0 + k * step, xb[k], qb[k], gb[k]);
            int s = 0;
            for (; s + NB + D <= nsteps; s += NB) {
#pragma unroll
                for (int k = 0; k < NB; ++k) {
                    load(c0 + (s + k + D) * step, xb[(k + D) % NB], qb[(k + D) % NB], gb[(k + D) % NB]);
                    PG_FENCE();
                    process(c0 + (s + k) * step, xb[k], qb[k], gb[k]);
                    PG_FENCE();
                }
            }
#pragma unroll
            for (int k = 0; k < NB + D - 1; ++k) {
                if (s + k < nsteps) {
                    if (s + k + D < nsteps)
                        load(c0 + (s + k + D) * step, xb[(k + D) % NB], qb[(k + D) % NB], gb[(k + D) % NB]);
                    PG_FENCE();
                    process(c0 + (s + k) * step, xb[k % NB], qb[k % NB], gb[k % NB]);
                    PG_FENCE();
                }
            }
        }
        if (SWEEP) {
            double(&flat)[M * RC] = reinterpret_cast<double(&)[M * RC]>(acc);
            group_sum_all<M * RC>(flat, lpr);
            if (sub == 0) {
#pragma unroll
                for (int m = 0; m < M; ++m)
#pragma unroll
                    for (int j = 0; j < RC; ++j)
                        if (ok[m] && j < R)
                            pw[pd.pw_off + ((int64_t)t.seg * R + j) * pd.p + rowi[m]] = acc[m][j];
            }
        }
    }
}

// The same pass for a vector layer (p x 1: a bias, a normalisation scale).  Its "rows" are single
// floats next to each other in memory, so lanes take consecutive rows (coalesced) instead of one
// lane group per row; every product is a scalar multiple, with the same operations in the same
// order as the general body performs for q = 1.
template <int RC, bool UPDATE, bool SWEEP, bool GRAD>
__device__ __forceinline__ void vec_row_body(const RowTile &t, const PairDesc &pd,
                                             const ColDesc *__restrict__ cols, float *X,
                                             const float *__restrict__ qstate,
                                             const float *__restrict__ phat, double *__restrict__ pw,
                                             const float *Gp, double eta) {
    constexpr int U = 4;  // rows in flight per lane
    const int R = pd.R;
    const int row_end = t.row0 + t.nrows;
    double qd[RC];
    const float *phc[RC];
    float coef[RC];
#pragma unroll
    for (int j = 0; j < RC; ++j) {
        const ColDesc cd = cols[pd.col0 + min(j, R - 1)];
        qd[j] = (double)ldg1(qstate + cd.q_off);
        phc[j] = phat + cd.ph_off;
        coef[j] = (j < R) ? cd.coef : 0.0f;
    }
    for (int base = t.row0 + (int)threadIdx.x; base < row_end; base += 64 * U) {
        int row[U];
        bool ok[U];
        double x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            ok[u] = base + 64 * u < row_end;
            row[u] = ok[u] ? base + 64 * u : row_end - 1;
            x[u] = (double)ldg1(X + row[u]);
        }
        if (UPDATE) {
            float ph[U][RC], g[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int j = 0; j < RC; ++j) ph[u][j] = ldg1(phc[j] + row[u]);
                g[u] = GRAD ? ldg1(Gp + row[u]) : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int j = 0; j < RC; ++j) x[u] = fma(-((double)coef[j] * (double)ph[u][j]), qd[j], x[u]);
                if (GRAD) x[u] = fma(-eta, (double)g[u], x[u]);
                const float xf = (float)x[u];
                if (ok[u]) *(PG_GLOBAL float *)(X + row[u]) = xf;
                x[u] = (double)xf;  // the sweep uses the stored (rounded) value
            }
        }
        if (SWEEP) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int j = 0; j < RC; ++j)
                    if (ok[u] && j < R) pw[pd.pw_off + (int64_t)j * pd.p + row[u]] = fma(x[u], qd[j], 0.0);
        }
    }
}

// One wavefront per tile; `reverse` walks the tile list backwards so that a pass can start on
// the data the previous pass touched last (still resident in the memory-side cache).
//   GRAD  : (with UPDATE) also subtract eta * G[row, c]: the update step of Algorithm 1 in one pass.
template <int RC, int M, int D, bool UPDATE, bool SWEEP, bool GRAD>
__global__ void __launch_bounds__(kRowThreads)
row_kernel(const RowTile *__restrict__ tiles, int ntiles, int reverse,
           const PairDesc *__restrict__ pairs, const ColDesc *__restrict__ cols,
           float *const *__restrict__ xs, const float *__restrict__ qstate,
           const float *__restrict__ phat, double *__restrict__ pw,
           const float *const *__restrict__ gs, double eta) {
    const RowTile t = tiles[tile_index(ntiles, reverse)];
    const PairDesc pd = pairs[t.pair];
    float *X = xs[pd.worker] + pd.x_off;
    const float *Gp = GRAD ? gs[pd.worker] + pd.x_off : nullptr;
    if (pd.q == 1) vec_row_body<RC, UPDATE, SWEEP, GRAD>(t, pd, cols, X, qstate, phat, pw, Gp, eta);
    else if (pd.V == 4) row_body<4, RC, M, D, UPDATE, SWEEP, GRAD>(t, pd, cols, X, qstate, phat, pw, Gp, eta);
    else if (pd.V == 2) row_body<2, RC, M, D, UPDATE, SWEEP, GRAD>(t, pd, cols, X, qstate, phat, pw, Gp, eta);
    else row_body<1, RC, M, D, UPDATE, SWEEP, GRAD>(t, pd, cols, X, qstate, phat, pw, Gp, eta);
}

// The row passes over vector layers alone (one wavefront per tile): the same arithmetic as the
// vector branch above in a kernel that needs few registers, so that many short tiles are
// resident at once.
template <int RC, bool UPDATE, bool SWEEP, bool GRAD>
__global__ void __launch_bounds__(kRowThreads)
vec_row_kernel(const RowTile *__restrict__ tiles, int ntiles, int reverse,
               const PairDesc *__restrict__ pairs, const ColDesc *__restrict__ cols,
               float *const *__restrict__ xs, const float *__restrict__ qstate,
               const float *__restrict__ phat, double *__restrict__ pw,
               const float *const *__restrict__ gs, double eta) {
    const RowTile t = tiles[tile_index(ntiles, reverse)];
    const PairDesc pd = pairs[t.pair];
    float *X = xs[pd.worker] + pd.x_off;
    const float *Gp = GRAD ? gs[pd.worker] + pd.x_off : nullptr;
    vec_row_body<RC, UPDATE, SWEEP, GRAD>(t, pd, cols, X, qstate, phat, pw, Gp, eta);
}

// ---------------------------------------------------------------------------------------
// Row-owner kernel for many stacked columns (RC >= 8): four wavefronts per tile share the
// tile's Q slice, staged once in LDS (RC x segment floats), so each loaded X value meets all
// RC columns without the Q slice being re-fetched per row.  Lane groups own M rows each as in
// the narrow kernel; only X is prefetched a step ahead, in registers.
// ---------------------------------------------------------------------------------------
template <int V, int RC, int M, bool UPDATE, bool SWEEP, bool GRAD>
__device__ __forceinline__ void row_wide_body(const RowTile &t, const PairDesc &pd,
                                              const ColDesc *__restrict__ cols, float *X,
                                              const float *__restrict__ qstate,
                                              const float *__restrict__ phat,
                                              double *__restrict__ pw, float *sQ,
                                              const float *Gp, double eta) {
    typedef typename VecT<V>::T vec;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lpr = pd.lpr;
    const int lpr_shift = __ffs(lpr) - 1;
    const int sub = lane & (lpr - 1);
    const int grp = wave * (64 >> lpr_shift) + (lane >> lpr_shift);
    const int ngrp = (kThreads / 64) * (64 >> lpr_shift);
    const int q = pd.q, R = pd.R;
    const int c_begin = t.seg * pd.seg_len;
    const int c_end = min(q, c_begin + pd.seg_len);
    const int seg_cols = c_end - c_begin;
    const int sstride = pd.seg_len;  // multiple of lpr * V: every column slice starts V-aligned
    const int row_end = t.row0 + t.nrows;
    const int step = lpr * V;

    // stage Q[c_begin:c_end, 0:R) as sQ[j][c]; unused columns j >= R read as zero
#pragma unroll 1
    for (int j = 0; j < RC; ++j) {
        if (j < R) {
            const float *src = qstate + cols[pd.col0 + j].q_off + c_begin;
            for (int cc = tid * V; cc < seg_cols; cc += kThreads * V)
                *reinterpret_cast<vec *>(sQ + j * sstride + cc) = ldg<V>(src + cc);
        } else {
            vec z;
#pragma unroll
            for (int v = 0; v < V; ++v) z[v] = 0.0f;
            for (int cc = tid * V; cc < seg_cols; cc += kThreads * V)
                *reinterpret_cast<vec *>(sQ + j * sstride + cc) = z;
        }
    }
    const float *phc[RC];
    float coef[RC];
    if (UPDATE) {
#pragma unroll
        for (int j = 0; j < RC; ++j) {
            const ColDesc cd = cols[pd.col0 + min(j, R - 1)];
            phc[j] = phat + cd.ph_off;
            coef[j] = (j < R) ? cd.coef : 0.0f;
        }
    }
    __syncthreads();

    for (int rbase = t.row0 + grp * M; rbase < row_end; rbase += ngrp * M) {
        float *xrow[M];
        const float *grow[M];
        bool ok[M];
        int rowi[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            ok[m] = rbase + m < row_end;
            rowi[m] = ok[m] ? rbase + m : row_end - 1;
            xrow[m] = X + (int64_t)rowi[m] * pd.ld;
            grow[m] = GRAD ? Gp + (int64_t)rowi[m] * pd.ld : nullptr;
        }
        double cp[M][RC];
        if (UPDATE) {
#pragma unroll
            for (int m = 0; m < M; ++m)
#pragma unroll
                for (int j = 0; j < RC; ++j)
                    cp[m][j] = (double)coef[j] * (double)ldg1(phc[j] + rowi[m]);
        }
        double acc[M][RC];
#pragma unroll
        for (int m = 0; m < M; ++m)
#pragma unroll
            for (int j = 0; j < RC; ++j) acc[m][j] = 0.0;

        auto load = [&](int c, vec(&xv)[M], vec(&gv)[GRAD ? M : 1]) {
#pragma unroll
            for (int m = 0; m < M; ++m) xv[m] = ldg<V>(xrow[m] + c);
            if (GRAD) {
#pragma unroll
                for (int m = 0; m < M; ++m) gv[GRAD ? m : 0] = ldg<V>(grow[m] + c);
            }
        };
        auto process = [&](int c, vec(&xv)[M], vec(&gv)[GRAD ? M : 1]) {
            const float *sq = sQ + (c - c_begin);
            double xd[M][V];
#pragma unroll
            for (int m = 0; m < M; ++m)
#pragma unroll
                for (int v = 0; v < V; ++v) xd[m][v] = (double)xv[m][v];
            if (UPDATE) {
#pragma unroll
                for (int j = 0; j < RC; ++j) {
                    const vec qv = *reinterpret_cast<const vec *>(sq + j * sstride);
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const double qd = (double)qv[v];
#pragma unroll
                        for (int m = 0; m < M; ++m) xd[m][v] = fma(-cp[m][j], qd, xd[m][v]);
                    }
                    // keep the compiler from hoisting all RC slices (and their conversions) at once
                    if ((j & 3) == 3) PG_FENCE();
                }
#pragma unroll
                for (int m = 0; m < M; ++m) {
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        if (GRAD) xd[m][v] = fma(-eta, (double)gv[GRAD ? m : 0][v], xd[m][v]);
                        xv[m][v] = (float)xd[m][v];
                        xd[m][v] = (double)xv[m][v];  // the sweep uses the stored (rounded) value
                    }
                    if (ok[m]) stg<V>(xrow[m] + c, xv[m]);
                }
            }
            if (SWEEP) {
#pragma unroll
                for (int j = 0; j < RC; ++j) {
                    const vec qv = *reinterpret_cast<const vec *>(sq + j * sstride);
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const double qd = (double)qv[v];
#pragma unroll
                        for (int m = 0; m < M; ++m) acc[m][j] = fma(xd[m][v], qd, acc[m][j]);
                    }
                    if ((j & 3) == 3) PG_FENCE();
                }
            }
        };

        int c = c_begin + sub * V;
        if (c < c_end) {
            vec xa[M], xb[M], ga[GRAD ? M : 1], gb[GRAD ? M : 1];
            int rem = (c_end - c - 1) / step;  // steps after the first one
            load(c, xa, ga);
#pragma unroll 1
            for (; rem > 0; --rem) {
                load(c + step, xb, gb);
                PG_FENCE();
                process(c, xa, ga);
                PG_FENCE();
#pragma unroll
                for (int m = 0; m < M; ++m) xa[m] = xb[m];
                if (GRAD) {
#pragma unroll
                    for (int m = 0; m < M; ++m) ga[GRAD ? m : 0] = gb[GRAD ? m : 0];
                }
                c += step;
            }
            process(c, xa, ga);
        }
        if (SWEEP) {
            double(&flat)[M * RC] = reinterpret_cast<double(&)[M * RC]>(acc);
            group_sum_all<M * RC>(flat, lpr);
            if (sub == 0) {
#pragma unroll
                for (int m = 0; m < M; ++m)
#pragma unroll
                    for (int j = 0; j < RC; ++j)
                        if (ok[m] && j < R)
                            pw[pd.pw_off + ((int64_t)t.seg * R + j) * pd.p + rowi[m]] = acc[m][j];
            }
        }
    }
}

// One instantiation per vector width V: with 8-16 stacked columns a kernel that carried all
// three widths would be allocated the registers of its widest body and lose occupancy.
template <int V, int RC, int M, bool UPDATE, bool SWEEP, bool GRAD>
__global__ void __launch_bounds__(kThreads)
row_wide_kernel(const RowTile *__restrict__ tiles, int ntiles, int reverse,
                const PairDesc *__restrict__ pairs, const ColDesc *__restrict__ cols,
                float *const *__restrict__ xs, const float *__restrict__ qstate,
                const float *__restrict__ phat, double *__restrict__ pw,
                const float *const *__restrict__ gs, double eta) {
    extern __shared__ double smem[];
    float *sQ = reinterpret_cast<float *>(smem);
    const RowTile t = tiles[tile_index(ntiles, reverse)];
    const PairDesc pd = pairs[t.pair];
    float *X = xs[pd.worker] + pd.x_off;
    const float *Gp = GRAD ? gs[pd.worker] + pd.x_off : nullptr;
    row_wide_body<V, RC, M, UPDATE, SWEEP, GRAD>(t, pd, cols, X, qstate, phat, pw, sQ, Gp, eta);
}

// ---------------------------------------------------------------------------------------
// Matrix-core kernels for many stacked columns (8 or 16).  With 16 right-hand sides a pass is a
// p x q by q x 16 contraction: on the vector ALUs its 16 double multiply-adds per loaded float
// (plus operand conversions and lane reductions) take longer than the HBM read.  The double
// precision matrix instruction V_MFMA_F64_16X16X4_F64 does the same 1024 multiply-adds in one
// issue slot, sums over lanes inside the instruction and keeps a 16 x 16 accumulator in eight
// registers, which leaves the vector ALUs to the float -> double conversions and the memory
// pipeline to the loads.  Lane layout of D = A B + C (lo = lane % 16, hi = lane / 16):
//   A[i][k]: lane (lo = i, hi = k);   B[k][j]: lane (hi = k, lo = j);
//   D[i][j]: lane (lo = j, hi = i % 4), register i / 4.
// ---------------------------------------------------------------------------------------
typedef double mfma_acc __attribute__((ext_vector_type(4)));
__device__ __forceinline__ mfma_acc mfma16(double a, double b, mfma_acc c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// Four consecutive floats of a row as 4 / V vector loads.  `nvalid` (a multiple of V) floats
// from p on are inside the row; units past them re-read the last valid unit and come back as
// zeros.  nvalid >= 4 is the plain case.
// Four consecutive floats in one 16-byte load at any 4-byte aligned address (global memory
// takes under-aligned vector accesses; rows of a matrix with q % 4 != 0 start at such addresses).
typedef float float4_any __attribute__((ext_vector_type(4), aligned(4)));
__device__ __forceinline__ void ld4(const float *p, float (&x)[4]) {
    const float4_any t = *(const PG_GLOBAL float4_any *)p;
#pragma unroll
    for (int v = 0; v < 4; ++v) x[v] = t[v];
}
// The 64 columns of one row step as the 16 lanes lo see them: 4 / V loads of V floats in which
// the lanes sit side by side; a lane's float t is column 16 V (t / V) + V lo + t % V of the step.
// Addresses are a wavefront-uniform base plus a 32-bit byte offset per lane (a layer is smaller
// than 4 GB), which is the form a load takes its base from scalar registers in.  `off` is the
// byte offset of the step's first column in the row (always inside the row).  FULL: all 64
// columns exist.  Otherwise `nvalid` columns are left in the row: units at or past that re-read
// the first column (the caller discards or zeroes them) and are not stored.
template <int V>
__device__ __forceinline__ typename VecT<V>::T ldg_at(const float *base, uint32_t byte_off) {
    return *(const PG_GLOBAL typename VecT<V>::T *)((const PG_GLOBAL char *)base + byte_off);
}
template <int V>
__device__ __forceinline__ void stg_at(float *base, uint32_t byte_off, typename VecT<V>::T v) {
    *(PG_GLOBAL typename VecT<V>::T *)((PG_GLOBAL char *)base + byte_off) = v;
}
template <int V, bool FULL>
__device__ __forceinline__ void ldrow(const float *base, uint32_t off, int lo, int nvalid, float (&x)[4]) {
#pragma unroll
    for (int u = 0; u < 4 / V; ++u) {
        const int c = 16 * V * u + V * lo;
        const typename VecT<V>::T t = ldg_at<V>(base, off + 4u * (uint32_t)((FULL || c < nvalid) ? c : 0));
#pragma unroll
        for (int e = 0; e < V; ++e) x[V * u + e] = t[e];
    }
}
template <int V, bool FULL>
__device__ __forceinline__ void strow(float *base, uint32_t off, int lo, int nvalid, const float (&x)[4]) {
#pragma unroll
    for (int u = 0; u < 4 / V; ++u) {
        const int c = 16 * V * u + V * lo;
        typename VecT<V>::T t;
#pragma unroll
        for (int e = 0; e < V; ++e) t[e] = x[V * u + e];
        if (FULL || c < nvalid) stg_at<V>(base, off + 4u * (uint32_t)c, t);
    }
}
// The same lane-to-column map into an LDS row of 64 floats.
template <int V>
__device__ __forceinline__ void lds_put_row(float *row, int lo, const float (&x)[4]) {
#pragma unroll
    for (int u = 0; u < 4 / V; ++u) {
        typename VecT<V>::T t;
#pragma unroll
        for (int e = 0; e < V; ++e) t[e] = x[V * u + e];
        *reinterpret_cast<typename VecT<V>::T *>(row + 16 * V * u + V * lo) = t;
    }
}
// Orders one wavefront's LDS writes before its later LDS reads of other lanes' data (the LDS
// serves a wavefront's instructions in order; this keeps the compiler from reordering them).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Row-owner pass on the matrix cores.  A tile is a block of rows by one column segment; it is
// walked in steps of 64 columns.  Its four wavefronts are arranged WR x WC (WC = pd.wc): wavefront
// (wr, wc) owns MB blocks of 16 rows and every WC-th step, so that the WC wavefronts of a row
// group read adjacent 256-byte pieces of the same rows.  Loads and stores are coalesced: lane
// (lo, hi) holds, for v = 0..3, four floats of row 4 v + hi of a block (column map of ldrow).
//   UPDATE: D_t[row][slot] = X - sum_j (coef_j Phat_j[row]) Q'_j[col(slot, t)], four stacked
//           columns j = 4 m + hi per instruction (A = coef * Phat, B = -Q', C = X); the result
//           comes back in exactly the layout the values were loaded in (register v = row / 4);
//   SWEEP : needs rows across the lanes lo, so the (updated, rounded) block goes through a
//           private LDS buffer, 16 x 64 floats, and comes back as A[row][k]: lane (lo = row,
//           hi = k) reads the four floats at column 16 s2 + 4 hi; the step's 64 x 16 slice of
//           the right-hand sides is staged the same way as B[k][j] (layout [column / 4][j][4]).
//           D[row][j] += X[row][c] Q_j[c], 16 instructions per block and step.
// Partial sums of the WC wavefronts of a row group meet in LDS, in a fixed order.  Steps with
// all 64 columns of a wavefront whose rows all exist run a body without any bounds handling.
// RCM = compiled stacked columns / 4 (2 or 4): the instructions one update block takes per t.
constexpr int kMrowXStride = 68;  // floats per LDS row: 64 + 4 keeps 128-bit reads down a column of lanes conflict-free
// The Q slice of a step, [column / 4][j][4]: 64 floats per group of four columns plus a pad that
// spreads the lanes' staging writes over the banks (measured with a plain 64-float stride: 60 % of
// the LDS cycles of the sweep were bank conflicts, all 64 lanes of a write landing on 16 banks).
// 8-byte writes (rows of even length) want a shift of 8 banks per group, the others 4.
constexpr int kMrowQStrideMax = 72;
template <int V>
struct MrowQStride {
    static constexpr int value = V == 2 ? 72 : 68;
};
constexpr int kMrowWaveFloats = 2 * 16 * kMrowXStride + 16 * kMrowQStrideMax;  // two X buffers and the Q slice of a step
constexpr size_t kMrowLdsBytes = (size_t)(kThreads / 64) * kMrowWaveFloats * sizeof(float);
template <bool B>
struct BoolTag {
    static constexpr bool value = B;
};
// Two work-groups per CU: left alone the compiler takes every register it can (one work-group).
// (measured: the sweep alone is 11 % faster at three wavefronts per SIMD, one register spilled).
template <int V, int RCM, int MB, int D, bool UPDATE, bool SWEEP, bool GRAD>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu((UPDATE || GRAD) ? 2 : 3)))
mrow_kernel(const RowTile *__restrict__ tiles, int ntiles, int reverse, const PairDesc *__restrict__ pairs,
            const ColDesc *__restrict__ cols, float *const *__restrict__ xs,
            const float *__restrict__ qstate, const float *__restrict__ phat,
            double *__restrict__ pw, const float *const *__restrict__ gs, double eta) {
    extern __shared__ double smem[];
    const RowTile t = tiles[tile_index(ntiles, reverse)];
    const PairDesc pd = pairs[t.pair];
    float *X = xs[pd.worker] + pd.x_off;
    const float *Gp = GRAD ? gs[pd.worker] + pd.x_off : nullptr;
    const int tid = threadIdx.x, lane = tid & 63, lo = lane & 15, hi = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // the same for the whole wavefront: keep it scalar
    float *lds = reinterpret_cast<float *>(smem) + wave * kMrowWaveFloats;
    float *qbuf = lds + 2 * 16 * kMrowXStride;
    const int q = pd.q, R = pd.R;
    const int WC = pd.wc;  // 1, 2 or 4
    const int wcol = wave & (WC - 1);
    const int wr = wave >> (WC == 4 ? 2 : (WC == 2 ? 1 : 0));
    const int c_begin = t.seg * pd.seg_len;
    const int c_end = min(q, c_begin + pd.seg_len);
    const int nst_all = (c_end - c_begin + 63) >> 6;
    const int row_end = t.row0 + t.nrows;
    const int row0w = t.row0 + wr * 16 * MB;  // this wavefront's first row; none left: no steps
    const int nsteps = (row0w < row_end && nst_all > wcol) ? (nst_all - wcol + WC - 1) / WC : 0;

    // byte offsets of this lane's rows (a row past the tile's end stands in for by the last one)
    uint32_t roff[MB][4];
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            roff[b][v] = 4u * (uint32_t)min(row0w + 16 * b + 4 * v + hi, row_end - 1) * (uint32_t)pd.ld;

    // update operand A: coef_j * Phat_j[row lo of the block], j = 4 m + hi
    const float *qup[UPDATE ? RCM : 1];
    double cp[UPDATE ? MB : 1][UPDATE ? RCM : 1];
    if (UPDATE) {
#pragma unroll
        for (int m = 0; m < RCM; ++m) {
            const int j = 4 * m + hi;
            const ColDesc cd = cols[pd.col0 + min(j, R - 1)];
            qup[m] = qstate + cd.q_off;
            const double coef = (j < R) ? (double)cd.coef : 0.0;
#pragma unroll
            for (int b = 0; b < MB; ++b)
                cp[b][m] = coef * (double)ldg1(phat + cd.ph_off + min(row0w + 16 * b + lo, row_end - 1));
        }
    }
    // sweep: this lane stages the right-hand sides j = hi + 4 i (the update's j = 4 m + hi: when
    // both run, one set of loads serves the two)
    const float *qsp[SWEEP ? 4 : 1];
    if (SWEEP && !UPDATE) {
#pragma unroll
        for (int i = 0; i < 4; ++i) qsp[i] = qstate + cols[pd.col0 + min(hi + 4 * i, R - 1)].q_off;
    }
    mfma_acc acc[MB];
#pragma unroll
    for (int b = 0; b < MB; ++b) acc[b] = mfma_acc{0.0, 0.0, 0.0, 0.0};

    struct Buf {
        float x[MB][4][4];
        float g[GRAD ? MB : 1][4][4];
        float qu[UPDATE ? RCM : 1][4];
        float qs[(SWEEP && !UPDATE) ? 4 : 1][4];  // fused: the update's Q' slices are the same data, same lanes
    };
    auto load = [&](auto full, int s, Buf &f) {
        constexpr bool FULL = decltype(full)::value;
        const int cs = c_begin + 64 * (wcol + WC * s);
        const int nvalid = c_end - cs;
        const uint32_t cso = 4u * (uint32_t)cs;
#pragma unroll
        for (int b = 0; b < MB; ++b) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                ldrow<V, FULL>(X, roff[b][v] + cso, lo, nvalid, f.x[b][v]);
                if (GRAD) ldrow<V, FULL>(Gp, roff[b][v] + cso, lo, nvalid, f.g[GRAD ? b : 0][v]);
            }
        }
        if (UPDATE) {
#pragma unroll
            for (int m = 0; m < RCM; ++m) ldrow<V, FULL>(qup[m], cso, lo, nvalid, f.qu[UPDATE ? m : 0]);
        }
        if (SWEEP && !UPDATE) {
#pragma unroll
            for (int i = 0; i < 4; ++i) ldrow<V, FULL>(qsp[i], cso, lo, nvalid, f.qs[(SWEEP && !UPDATE) ? i : 0]);
        }
    };
    auto process = [&](auto full, int s, Buf &f) {
        constexpr bool FULL = decltype(full)::value;
        const int cs = c_begin + 64 * (wcol + WC * s);
        const int nvalid = c_end - cs;
        const uint32_t cso = 4u * (uint32_t)cs;
        if (SWEEP) {
            // B[k][j]: layout [column / 4][j][4]; a unit of V floats stays inside one group of 4
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int u = 0; u < 4 / V; ++u) {
                    const int c = 16 * V * u + V * lo;
                    typename VecT<V>::T tv;
#pragma unroll
                    for (int e = 0; e < V; ++e)
                        tv[e] = UPDATE ? f.qu[UPDATE ? (i < RCM ? i : RCM - 1) : 0][V * u + e]
                                       : f.qs[(SWEEP && !UPDATE) ? i : 0][V * u + e];
                    *reinterpret_cast<typename VecT<V>::T *>(qbuf + (c >> 2) * MrowQStride<V>::value + (hi + 4 * i) * 4 + (c & 3)) = tv;
                }
            }
            wave_lds_sync();
        }
        // columns past the row's end: the sweep must see zeros there
        bool cok[4];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) cok[tt] = FULL || 16 * V * (tt / V) + V * lo < nvalid;
#pragma unroll
        for (int b = 0; b < MB; ++b) {
            if (UPDATE) {
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) {
                    mfma_acc d;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        d[v] = (double)f.x[b][v][tt];
                        if (GRAD) d[v] = fma(-eta, (double)f.g[GRAD ? b : 0][v][tt], d[v]);
                    }
#pragma unroll
                    for (int m = 0; m < RCM; ++m) d = mfma16(cp[b][m], -(double)f.qu[UPDATE ? m : 0][tt], d);
#pragma unroll
                    for (int v = 0; v < 4; ++v) f.x[b][v][tt] = cok[tt] ? (float)d[v] : 0.0f;
                    PG_FENCE();  // keeps the conversions of later groups from being hoisted (registers)
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (FULL || row0w + 16 * b + 4 * v + hi < row_end)
                        strow<V, FULL>(X, roff[b][v] + cso, lo, nvalid, f.x[b][v]);
                }
            }
            if (SWEEP) {
                if (!UPDATE && !FULL) {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
#pragma unroll
                        for (int tt = 0; tt < 4; ++tt) f.x[b][v][tt] = cok[tt] ? f.x[b][v][tt] : 0.0f;
                }
                float *xb = lds + (b & 1) * 16 * kMrowXStride;
#pragma unroll
                for (int v = 0; v < 4; ++v) lds_put_row<V>(xb + (4 * v + hi) * kMrowXStride, lo, f.x[b][v]);
                wave_lds_sync();
                // the B operand is read back per block rather than kept across the blocks of a step:
                // 16 registers less, which the fused pass would otherwise spill
#pragma unroll
                for (int s2 = 0; s2 < 4; ++s2) {
                    const VecT<4>::T av =
                        *reinterpret_cast<const VecT<4>::T *>(xb + lo * kMrowXStride + 16 * s2 + 4 * hi);
                    const VecT<4>::T bv = *reinterpret_cast<const VecT<4>::T *>(qbuf + (4 * s2 + hi) * MrowQStride<V>::value + lo * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[b] = mfma16((double)av[e], (double)bv[e], acc[b]);
                    PG_FENCE();
                }
            }
        }
    };
    // software pipeline over steps [0, n): loads of step s + D are issued before the arithmetic of step s
    auto pipeline = [&](auto full, int n) {
        constexpr int NB = D + 1;
        Buf ring[NB];
#pragma unroll
        for (int k = 0; k < D; ++k)
            if (k < n) load(full, k, ring[k]);
        int s = 0;
        for (; s + NB + D <= n; s += NB) {
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                load(full, s + k + D, ring[(k + D) % NB]);
                PG_FENCE();
                process(full, s + k, ring[k]);
                PG_FENCE();
            }
        }
#pragma unroll
        for (int k = 0; k < NB + D - 1; ++k) {
            if (s + k < n) {
                if (s + k + D < n) load(full, s + k + D, ring[(k + D) % NB]);
                PG_FENCE();
                process(full, s + k, ring[k % NB]);
                PG_FENCE();
            }
        }
    };

    // The segment's last step may be ragged; it is the last step of the wavefront that owns it.
    const bool ragged_mine = ((c_end - c_begin) & 63) != 0 && ((nst_all - 1) & (WC - 1)) == wcol;
    if (row0w + 16 * MB <= row_end) {
        const int nfull = ragged_mine ? nsteps - 1 : nsteps;
        pipeline(BoolTag<true>(), nfull);
        if (nfull < nsteps) {
            Buf last;
            load(BoolTag<false>(), nsteps - 1, last);
            process(BoolTag<false>(), nsteps - 1, last);
        }
    } else {
        // a wavefront with rows past the tile's end: a few tiles per layer, no prefetch ring
        for (int s = 0; s < nsteps; ++s) {
            Buf one;
            load(BoolTag<false>(), s, one);
            process(BoolTag<false>(), s, one);
        }
    }

    if (SWEEP) {
        // D[row][j] sits in lane (lo = j, hi = row % 4), register row / 4
        if (WC > 1) {
            double *mine = reinterpret_cast<double *>(lds);
            wave_lds_sync();
            if (wcol != 0) {
#pragma unroll
                for (int b = 0; b < MB; ++b)
#pragma unroll
                    for (int w = 0; w < 4; ++w) mine[(b * 4 + w) * 64 + lane] = acc[b][w];
            }
            __syncthreads();
            if (wcol == 0) {
                for (int o = 1; o < WC; ++o) {
                    const double *other = reinterpret_cast<const double *>(lds + o * kMrowWaveFloats);
#pragma unroll
                    for (int b = 0; b < MB; ++b)
#pragma unroll
                        for (int w = 0; w < 4; ++w) acc[b][w] += other[(b * 4 + w) * 64 + lane];
                }
            }
        }
        if (wcol == 0 && lo < R) {
            double *dst = pw + pd.pw_off + ((int64_t)t.seg * R + lo) * pd.p;
#pragma unroll
            for (int b = 0; b < MB; ++b)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const int r = row0w + 16 * b + 4 * w + hi;
                    if (r < row_end) dst[r] = acc[b][w];
                }
        }
    }
}

// Column-owner pass (Q-sweep) on the matrix cores: four wavefronts per tile, each on its own
// 64 adjacent columns of one row block (side by side, so that the four read the same DRAM pages
// at about the same time; they share nothing and never wait for each other), 16 rows per step.
// Lane (lo, hi) holds, for u = 0..3, four floats of row r + 4 hi + u, fetched as 4 / V loads of
// V floats in which the 16 lanes lo sit side by side: float v is column c0 + V lo + v % V +
// 16 V (v / V).  The instruction for (u, v) adds X^T Phat over the rows r + 4 hi + u, hi = 0..3:
// D_v[col][j] += X[row][col] * Phat_j[row] (A = X^T, B = the stacked Phat columns, j = lo); a
// lane's four Phat values of a step are consecutive in memory and come in one load.
// STAGE: the row block's Phat entries, all 16 stacked columns, are staged in LDS once per tile
// ([j][row], rows past the block's end and columns j >= R as zeros) and the four wavefronts take
// their B operands from there; otherwise every wavefront fetches them from global memory step by step.
__host__ __device__ constexpr int mcol_stage_stride(int blk_rows) { return ((blk_rows + 31) & ~31) + 4; }
template <int V, int D, bool STAGE>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2)))
mcol_kernel(const ColTile *__restrict__ tiles, int ntiles, int reverse,
            const PairDesc *__restrict__ pairs, const ColDesc *__restrict__ cols,
            float *const *__restrict__ xs, const float *__restrict__ phat,
            double *__restrict__ qw) {
    extern __shared__ double smem[];
    float *sP = reinterpret_cast<float *>(smem);
    const ColTile t = tiles[tile_index(ntiles, reverse)];
    const PairDesc pd = pairs[t.pair];
    const float *X = xs[pd.worker] + pd.x_off;
    const int lane = threadIdx.x & 63, lo = lane & 15, hi = lane >> 4;
    const int q = pd.q, R = pd.R;
    const int c0 = t.c0 + 64 * __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool mine = c0 < q;  // a wavefront past the matrix's last column only helps staging
    if (!STAGE && !mine) return;
    const int ncols = mine ? min(64, q - c0) : V;  // this wavefront's columns inside the matrix
    const int rb = t.blk * pd.blk_rows;
    const int re = min(pd.p, rb + pd.blk_rows);
    const int nsteps = (re - rb + 15) >> 4;
    const bool ragged = ((re - rb) & 15) != 0;
    const float *ph = phat + cols[pd.col0 + min(lo, R - 1)].ph_off;
    const bool jok = lo < R;
    const float *xt = X + (mine ? c0 : 0);
    const int stride = mcol_stage_stride(pd.blk_rows);
    if (STAGE) {
        const float *src[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) src[j] = phat + cols[pd.col0 + min(j, R - 1)].ph_off + rb;
        for (int r = threadIdx.x; r < 16 * nsteps; r += kThreads) {
#pragma unroll
            for (int j = 0; j < 16; ++j) sP[j * stride + r] = (j < R && r < re - rb) ? ldg1(src[j] + r) : 0.0f;
        }
    }

    mfma_acc acc[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[v] = mfma_acc{0.0, 0.0, 0.0, 0.0};

    struct Buf {
        float x[4][4];
        float t[4];
    };
    auto load = [&](int s, Buf &f) {
        const int r0 = rb + 16 * s + 4 * hi;
        const bool last = ragged && s == nsteps - 1;
        if (!STAGE && !last) ld4(ph + r0, f.t);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = last ? min(r0 + u, re - 1) : r0 + u;
            if (!STAGE && last) f.t[u] = ldg1(ph + r);
            const float *xr = xt + (int64_t)r * pd.ld;
#pragma unroll
            for (int w = 0; w < 4 / V; ++w) {
                const int cw = 16 * V * w + V * lo;
                // a lane past the row's end re-reads the row's last unit (a line the valid lanes
                // fetch anyway): that sum is not stored
                const typename VecT<V>::T xv = ldg<V>(xr + (cw < ncols ? cw : ncols - V));
#pragma unroll
                for (int e = 0; e < V; ++e) f.x[u][V * w + e] = xv[e];
            }
        }
    };
    auto process = [&](int s, Buf &f) {
        const int r0 = rb + 16 * s + 4 * hi;
        if (STAGE) {
            const VecT<4>::T tv = *reinterpret_cast<const VecT<4>::T *>(sP + lo * stride + 16 * s + 4 * hi);
#pragma unroll
            for (int u = 0; u < 4; ++u) f.t[u] = tv[u];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const double td = (STAGE || (jok && r0 + u < re)) ? (double)f.t[u] : 0.0;
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[v] = mfma16((double)f.x[u][v], td, acc[v]);
        }
    };

    constexpr int NB = D + 1;
    Buf ring[NB];
    if (mine) {
#pragma unroll
        for (int k = 0; k < D; ++k)
            if (k < nsteps) load(k, ring[k]);
    }
    if (STAGE) {
        __syncthreads();  // Phat staged (the first loads of X are already under way)
        if (!mine) return;
    }
    int s = 0;
    for (; s + NB + D <= nsteps; s += NB) {
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            load(s + k + D, ring[(k + D) % NB]);
            PG_FENCE();
            process(s + k, ring[k]);
            PG_FENCE();
        }
    }
#pragma unroll
    for (int k = 0; k < NB + D - 1; ++k) {
        if (s + k < nsteps) {
            if (s + k + D < nsteps) load(s + k + D, ring[(k + D) % NB]);
            PG_FENCE();
            process(s + k, ring[k % NB]);
            PG_FENCE();
        }
    }

    // D_v[i][j] sits in lane (lo = j, hi = i % 4), register i / 4; i stands for column
    // c0 + V i + v % V + 16 V (v / V)
    if (jok) {
        double *dst = qw + pd.qw_off + ((int64_t)t.blk * R + lo) * q + c0;
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int cc = V * (4 * w + hi) + v % V + 16 * V * (v / V);
                if (cc < ncols) dst[cc] = acc[v][w];
            }
    }
}

// Workers without any edge receive no gossip term; with a gradient their step is plain SGD,
// X -= eta * G, elementwise over the listed (worker, layer) pairs.
__global__ void __launch_bounds__(kThreads)
sgd_only_kernel(const int32_t *__restrict__ pair_ids, const PairDesc *__restrict__ pairs,
                float *const *__restrict__ xs, const float *const *__restrict__ gs, double eta) {
    // 64 work-groups per listed pair (a one-dimensional grid: the list may be longer than a grid's y range)
    const PairDesc pd = pairs[pair_ids[blockIdx.x >> 6]];
    float *X = xs[pd.worker] + pd.x_off;
    const float *G = gs[pd.worker] + pd.x_off;
    const int64_t total = (int64_t)pd.p * pd.q;
    for (int64_t i = (int64_t)(blockIdx.x & 63) * kThreads + threadIdx.x; i < total;
         i += (int64_t)64 * kThreads) {
        const int64_t at = (i / pd.q) * pd.ld + i % pd.q;
        X[at] = (float)fma(-eta, (double)G[at], (double)X[at]);
    }
}

// ---------------------------------------------------------------------------------------
// Column-owner kernel.  A lane owns V adjacent columns of X_i and runs down a block of rows;
// `lg` lanes sit side by side, the other lanes of the wavefront (and the other wavefronts)
// take interleaved rows of the same columns and are summed at the end.  The block's Phat
// entries are staged in LDS once; the loads of the next U rows are issued before the
// arithmetic of the current U rows.
//   Qw[blk][j][c] = sum_{row in blk} X[row, c] * Phat_j[row]   (Algorithm 2, even iteration:
//   the product with X^T, for every incident edge in one read of X_i)
// ---------------------------------------------------------------------------------------
template <int V, int RC, int U>
__device__ __forceinline__ void col_body(const ColTile &t, const PairDesc &pd,
                                         const ColDesc *__restrict__ cols, const float *X,
                                         const float *__restrict__ phat, double *__restrict__ qw,
                                         float *sT) {
    typedef typename VecT<V>::T vec;
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
    const int nrows = re - rb;

    // stage Phat[rb:re, 0:R) as sT[row][j]; columns j >= R and the extra row `nrows` are zero
    // (rows past the block's end are pointed at that zero row)
    const float *src[RC];
#pragma unroll
    for (int j = 0; j < RC; ++j) src[j] = phat + cols[pd.col0 + min(j, R - 1)].ph_off + rb;
    for (int rr = threadIdx.x; rr <= nrows; rr += kThreads) {
#pragma unroll
        for (int j = 0; j < RC; ++j) sT[rr * RC + j] = (j < R && rr < nrows) ? ldg1(src[j] + rr) : 0.0f;
    }

    double acc[RC][V];
#pragma unroll
    for (int j = 0; j < RC; ++j)
#pragma unroll
        for (int v = 0; v < V; ++v) acc[j][v] = 0.0;

    const float *xcol = X + c;
    auto load = [&](int row, vec(&xv)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int rr = min(row + u * RG, re - 1);
            xv[u] = ldg<V>(xcol + (int64_t)rr * pd.ld);
        }
    };
    auto process = [&](int row, vec(&xv)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int li = (min(row + u * RG, re) - rb) * RC;
            double xd[V];
#pragma unroll
            for (int v = 0; v < V; ++v) xd[v] = (double)xv[u][v];
#pragma unroll
            for (int j = 0; j < RC; ++j) {
                const double td = (double)sT[li + j];
#pragma unroll
                for (int v = 0; v < V; ++v) acc[j][v] = fma(xd[v], td, acc[j][v]);
            }
        }
    };

    int row = rb + rg;
    const int stride = RG * U;
    vec xa[U], xb[U];
    const bool active = row < re;
    int rem = active ? (re - row - 1) / stride : 0;
    if (active) load(row, xa);
    __syncthreads();  // Phat staged
    if (active) {
#pragma unroll 1
        for (; rem > 0; --rem) {
            load(row + stride, xb);
            PG_FENCE();
            process(row, xa);
            PG_FENCE();
#pragma unroll
            for (int u = 0; u < U; ++u) xa[u] = xb[u];
            row += stride;
        }
        process(row, xa);
    }
    // lanes of one wavefront that hold the same columns
    for (int o = lg; o < 64; o <<= 1)
#pragma unroll
        for (int j = 0; j < RC; ++j)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[j][v] += __shfl_xor(acc[j][v], o);
    // the four wavefronts, one stacked column at a time, through LDS
    __syncthreads();  // everyone is done with sT
    double(*red)[64][V] = reinterpret_cast<double(*)[64][V]>(sT);
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

// V = 0: tiles of any vector width (few stacked columns); V = 1, 2, 4: one width only.
template <int V, int RC, int U>
__global__ void __launch_bounds__(kThreads)
col_kernel(const ColTile *__restrict__ tiles, int ntiles, int reverse,
           const PairDesc *__restrict__ pairs, const ColDesc *__restrict__ cols,
           float *const *__restrict__ xs, const float *__restrict__ phat,
           double *__restrict__ qw) {
    extern __shared__ double smem[];  // [blk_rows][RC] Phat floats, then reused for the reduction
    float *sT = reinterpret_cast<float *>(smem);
    const ColTile t = tiles[tile_index(ntiles, reverse)];
    const PairDesc pd = pairs[t.pair];
    const float *X = xs[pd.worker] + pd.x_off;
    if constexpr (V != 0) {
        col_body<V, RC, U>(t, pd, cols, X, phat, qw, sT);
    } else {
        if (pd.V == 4) col_body<4, RC, U>(t, pd, cols, X, phat, qw, sT);
        else if (pd.V == 2) col_body<2, RC, U>(t, pd, cols, X, phat, qw, sT);
        else col_body<1, RC, U>(t, pd, cols, X, phat, qw, sT);
    }
}

// The Q-sweep of vector layers alone: X_i^T Phat_j is a dot product per stacked column.  One
// wavefront per (worker, layer, row block), lanes on consecutive entries, U of them in flight per lane.
//   Qw[blk][j] = sum_{row in blk} X[row] * Phat_j[row]
template <int RC>
__global__ void __launch_bounds__(kRowThreads)
vec_col_kernel(const ColTile *__restrict__ tiles, int ntiles, int reverse,
               const PairDesc *__restrict__ pairs, const ColDesc *__restrict__ cols,
               float *const *__restrict__ xs, const float *__restrict__ phat,
               double *__restrict__ qw) {
    constexpr int U = 4;
    const ColTile t = tiles[tile_index(ntiles, reverse)];
    const PairDesc pd = pairs[t.pair];
    const float *X = xs[pd.worker] + pd.x_off;
    const int R = pd.R;
    const int rb = t.blk * pd.blk_rows;
    const int re = min(pd.p, rb + pd.blk_rows);
    const float *ph[RC];
    double acc[RC];
#pragma unroll
    for (int j = 0; j < RC; ++j) {
        ph[j] = phat + cols[pd.col0 + min(j, R - 1)].ph_off;
        acc[j] = 0.0;
    }
    for (int base = rb + (int)threadIdx.x; base < re; base += 64 * U) {
        float x[U], f[U][RC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = min(base + 64 * u, re - 1);
            x[u] = ldg1(X + row);
#pragma unroll
            for (int j = 0; j < RC; ++j) f[u][j] = ldg1(ph[j] + row);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const double xd = base + 64 * u < re ? (double)x[u] : 0.0;
#pragma unroll
            for (int j = 0; j < RC; ++j) acc[j] = fma(xd, (double)f[u][j], acc[j]);
        }
    }
    group_sum_all<RC>(acc, 64);
    if (threadIdx.x == 0) {
#pragma unroll
        for (int j = 0; j < RC; ++j)
            if (j < R) qw[pd.qw_off + (int64_t)t.blk * R + j] = acc[j];
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

// The same orthonormalisation for r <= RMAX <= 8 in two passes over P instead of O(r^2):
// pass 1 forms the Gram matrix G = P^T P; one thread factors it, G = R^T R (R upper
// triangular: R_jk is the Gram-Schmidt coefficient of column k on the orthonormal column j,
// R_kk the norm of its residual, so the dropped-column test reads d_k = G_kk - sum_j R_jk^2
// against max(FLT_MIN, 1e-10 G_kk)); pass 2 applies Phat = P R^-1 row by row by forward
// substitution.  Same columns as the left-to-right Gram-Schmidt up to rounding in double.
// What is orthonormalised and where the result goes: either the difference of the two workers'
// partial products (P = sum Pw_a - sum Pw_b, `st` null), or r stored float columns of `len`
// entries (one of Algorithm 2's vectors v_ij per column).
struct GramIO {
    const double *pw;
    const float *st;
    int64_t st_off;
    int len;
    float *out;
    int64_t out_off;
};

template <int RMAX>
__device__ __forceinline__ void gram_load_row(const EdgeLayerDesc &d, const GramIO &io, int row,
                                              double (&v)[RMAX]) {
    if (io.st) {
#pragma unroll
        for (int k = 0; k < RMAX; ++k)
            v[k] = (k < d.r) ? (double)io.st[io.st_off + (int64_t)k * io.len + row] : 0.0;
        return;
    }
#pragma unroll
    for (int k = 0; k < RMAX; ++k) {
        double sa = 0.0, sb = 0.0;
        if (k < d.r) {
            for (int s = 0; s < d.nseg; ++s) {
                sa += io.pw[d.pwa_off + s * d.pwa_seg + (int64_t)k * d.p + row];
                sb += io.pw[d.pwb_off + s * d.pwb_seg + (int64_t)k * d.p + row];
            }
        }
        v[k] = sa - sb;
    }
}

// Pass 1 over rows [row0, row1): the work-group's Gram sums, packed G[j][k] (j <= k) at
// k (k + 1) / 2 + j, left in sG.
template <int NT, int RMAX>
__device__ __forceinline__ void gram_rows(const EdgeLayerDesc &d, const GramIO &io,
                                          int row0, int row1,
                                          double (*sRed)[RMAX * (RMAX + 1) / 2], double *sG) {
    constexpr int NG = RMAX * (RMAX + 1) / 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double g[NG];
#pragma unroll
    for (int i = 0; i < NG; ++i) g[i] = 0.0;
#pragma unroll 2
    for (int row = row0 + tid; row < row1; row += NT) {
        double v[RMAX];
        gram_load_row<RMAX>(d, io, row, v);
        int idx = 0;
#pragma unroll
        for (int k = 0; k < RMAX; ++k)
#pragma unroll
            for (int j = 0; j <= k; ++j) {
                g[idx] = fma(v[j], v[k], g[idx]);
                ++idx;
            }
    }
    group_sum_all<NG>(g, 64);
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < NG; ++i) sRed[wave][i] = g[i];
    }
    __syncthreads();
    if (tid < NG) {
        double s = 0.0;
        for (int w = 0; w < NT / 64; ++w) s += sRed[w][tid];
        sG[tid] = s;
    }
    __syncthreads();
}

// One thread factors G = R^T R with the dropped-column rule; everyone waits for it.
template <int RMAX>
__device__ __forceinline__ void gram_factor(const EdgeLayerDesc &d, const double *G,
                                            double (*sR)[RMAX], int *sDrop,
                                            int32_t *__restrict__ flags, bool write_flags) {
    if (threadIdx.x == 0) {
        for (int k = 0; k < d.r; ++k) {
            const double gkk = G[k * (k + 1) / 2 + k];
            double dk = gkk;
            for (int j = 0; j < k; ++j) {
                double rjk = 0.0;
                if (!sDrop[j]) {
                    double t = G[k * (k + 1) / 2 + j];
                    for (int i = 0; i < j; ++i)
                        if (!sDrop[i]) t -= sR[i][j] * sR[i][k];
                    rjk = t / sR[j][j];
                }
                sR[j][k] = rjk;
                dk -= rjk * rjk;
            }
            double floor2 = 1e-10 * gkk;
            if (floor2 < (double)FLT_MIN) floor2 = (double)FLT_MIN;
            const int dropped = !(dk >= floor2);
            sDrop[k] = dropped;
            sR[k][k] = dropped ? 1.0 : sqrt(dk);
            if (write_flags) flags[d.flag_off + k] = dropped;
        }
    }
    __syncthreads();
}

// Pass 2 over rows [row0, row1): Phat = P R^-1 by forward substitution, rounded to float.
template <int NT, int RMAX>
__device__ __forceinline__ void gram_apply_rows(const EdgeLayerDesc &d, const GramIO &io,
                                                int row0, int row1,
                                                const double (*sR)[RMAX], const int *sDrop) {
#pragma unroll 2
    for (int row = row0 + (int)threadIdx.x; row < row1; row += NT) {
        double v[RMAX], ph[RMAX];
        gram_load_row<RMAX>(d, io, row, v);
#pragma unroll
        for (int k = 0; k < RMAX; ++k) {
            if (k < d.r) {
                double t = v[k];
#pragma unroll
                for (int j = 0; j < k; ++j) t -= sR[j][k] * ph[j];
                ph[k] = sDrop[k] ? 0.0 : t / sR[k][k];
                io.out[io.out_off + (int64_t)k * io.len + row] = (float)ph[k];
            } else {
                ph[k] = 0.0;
            }
        }
    }
}

// Whole (edge, layer) in one work-group: used when every layer has few rows.
template <int NT, int RMAX>
__global__ void __launch_bounds__(NT)
orth_gram_kernel(const EdgeLayerDesc *__restrict__ els, const double *__restrict__ pw,
                 float *__restrict__ phat, int32_t *__restrict__ flags) {
    constexpr int NG = RMAX * (RMAX + 1) / 2;
    __shared__ double sRed[NT / 64][NG];
    __shared__ double sG[NG];
    __shared__ double sR[RMAX][RMAX];
    __shared__ int sDrop[RMAX];
    const EdgeLayerDesc d = els[blockIdx.x];
    const GramIO io{pw, nullptr, 0, d.p, phat, d.ph_off};
    gram_rows<NT, RMAX>(d, io, 0, d.p, sRed, sG);
    gram_factor<RMAX>(d, sG, sR, sDrop, flags, true);
    gram_apply_rows<NT, RMAX>(d, io, 0, d.p, sR, sDrop);
}

// Orthonormalise the r stored columns of every (edge, layer) -- Algorithm 2's vhat = v / |v|,
// Gram-Schmidt for r > 1 -- from `src` into `dst` (same offsets).  in_q = 1: the vectors live
// in R^q (state layout), 0: in R^p (Phat layout).
template <int NT, int RMAX>
__global__ void __launch_bounds__(NT)
orth_state_kernel(const EdgeLayerDesc *__restrict__ els, const float *__restrict__ src,
                  float *__restrict__ dst, int in_q, int32_t *__restrict__ flags) {
    constexpr int NG = RMAX * (RMAX + 1) / 2;
    __shared__ double sRed[NT / 64][NG];
    __shared__ double sG[NG];
    __shared__ double sR[RMAX][RMAX];
    __shared__ int sDrop[RMAX];
    const EdgeLayerDesc d = els[blockIdx.x];
    const int len = in_q ? d.q : d.p;
    const int64_t off = in_q ? d.q_off : d.ph_off;
    const GramIO io{nullptr, src, off, len, dst, off};
    gram_rows<NT, RMAX>(d, io, 0, len, sRed, sG);
    gram_factor<RMAX>(d, sG, sR, sDrop, flags, true);
    gram_apply_rows<NT, RMAX>(d, io, 0, len, sR, sDrop);
}

// Algorithm 2, odd iteration: v_ij <- p_j - p_i, the difference of the two workers' products,
// stored unnormalised as float columns of length p; columns whose unit vector was dropped keep
// their old content.
// Grid: (edge, layer) x chunks of chunk_rows rows (sized for the tallest layer; chunks past a
// layer's end leave at once).
__global__ void __launch_bounds__(kThreads)
comb_p_kernel(const EdgeLayerDesc *__restrict__ els, const double *__restrict__ pw,
              const int32_t *__restrict__ flags, float *__restrict__ pstate, int chunk_rows) {
    const EdgeLayerDesc d = els[blockIdx.x];
    const int64_t first = (int64_t)blockIdx.y * chunk_rows;
    const int row0 = (int)min<int64_t>(first, d.p);
    const int row1 = (int)min<int64_t>(first + chunk_rows, d.p);
    for (int k = 0; k < d.r; ++k) {
        if (row0 >= row1 || flags[d.flag_off + k]) continue;
        for (int row = row0 + (int)threadIdx.x; row < row1; row += kThreads) {
            double sa = 0.0, sb = 0.0;
            for (int s = 0; s < d.nseg; ++s) {
                sa += pw[d.pwa_off + s * d.pwa_seg + (int64_t)k * d.p + row];
                sb += pw[d.pwb_off + s * d.pwb_seg + (int64_t)k * d.p + row];
            }
            pstate[d.ph_off + (int64_t)k * d.p + row] = (float)(sa - sb);
        }
    }
}

// Tall layers: the rows of an (edge, layer) are cut into chunks, one work-group each.  The first
// kernel leaves each chunk's Gram sums in gpart; the second adds an (edge, layer)'s chunks in
// order, factors (every chunk redoes this tiny step) and applies R^-1 to its own rows.
template <int NT, int RMAX>
__global__ void __launch_bounds__(NT)
orth_gram_part_kernel(const OrthTile *__restrict__ tiles, const EdgeLayerDesc *__restrict__ els,
                      const double *__restrict__ pw, double *__restrict__ gpart,
                      const float *__restrict__ st) {
    constexpr int NG = RMAX * (RMAX + 1) / 2;
    __shared__ double sRed[NT / 64][NG];
    __shared__ double sG[NG];
    const OrthTile t = tiles[blockIdx.x];
    const EdgeLayerDesc d = els[t.el];
    // st: the stored float columns of length p to normalise (Algorithm 2's vectors) instead of
    // the difference of the partial products
    const GramIO io{pw, st, d.ph_off, d.p, nullptr, 0};
    gram_rows<NT, RMAX>(d, io, t.row0, t.row0 + t.nrows, sRed, sG);
    if (threadIdx.x < NG) gpart[(int64_t)blockIdx.x * NG + threadIdx.x] = sG[threadIdx.x];
}

template <int NT, int RMAX>
__global__ void __launch_bounds__(NT)
orth_gram_apply_kernel(const OrthTile *__restrict__ tiles, const EdgeLayerDesc *__restrict__ els,
                       const double *__restrict__ pw, const double *__restrict__ gpart,
                       float *__restrict__ phat, int32_t *__restrict__ flags,
                       const float *__restrict__ st) {
    constexpr int NG = RMAX * (RMAX + 1) / 2;
    __shared__ double sG[NG];
    __shared__ double sR[RMAX][RMAX];
    __shared__ int sDrop[RMAX];
    const OrthTile t = tiles[blockIdx.x];
    const EdgeLayerDesc d = els[t.el];
    if (threadIdx.x < NG) {
        double s = 0.0;
        const int64_t first = (int64_t)blockIdx.x - t.chunk;  // chunk 0 of this (edge, layer)
        for (int c = 0; c < t.nchunks; ++c) s += gpart[(first + c) * NG + threadIdx.x];
        sG[threadIdx.x] = s;
    }
    __syncthreads();
    gram_factor<RMAX>(d, sG, sR, sDrop, flags, t.chunk == 0);
    const GramIO io{pw, st, d.ph_off, d.p, phat, d.ph_off};
    gram_apply_rows<NT, RMAX>(d, io, t.row0, t.row0 + t.nrows, sR, sDrop);
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
    // four interleaved running sums keep several loads in flight; the order is fixed
    double sa[4] = {0.0, 0.0, 0.0, 0.0}, sb[4] = {0.0, 0.0, 0.0, 0.0};
    int b = 0;
    for (; b + 4 <= d.nblk; b += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            sa[u] += qw[d.qwa_off + (b + u) * d.qwa_blk + idx];
            sb[u] += qw[d.qwb_off + (b + u) * d.qwb_blk + idx];
        }
    }
    for (; b < d.nblk; ++b) {
        sa[0] += qw[d.qwa_off + b * d.qwa_blk + idx];
        sb[0] += qw[d.qwb_off + b * d.qwb_blk + idx];
    }
    qstate[d.q_off + idx] = (float)(((sa[0] + sa[1]) + (sa[2] + sa[3])) - ((sb[0] + sb[1]) + (sb[2] + sb[3])));
}

}  // namespace pg
