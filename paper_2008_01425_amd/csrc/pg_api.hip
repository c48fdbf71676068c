// C ABI of the PowerGossip library: context life cycle, layout queries, launch sequencing.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/powergossip.h"
#include "pg_kernels.hip"
#include "pg_plan.hpp"

using namespace pg;

namespace {

constexpr int kOrthThreads = 1024;

// Workspace of pg_round_static: device memory that exists from the moment the library's code
// object is loaded on a GPU (one copy per GPU, at its own address, held until the process
// ends), so that a round can run without any allocation.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels and copies take the address that call returns.
static __device__ __align__(256) unsigned char scratch[PG_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];  // per device: address of `scratch` there (null = not asked yet)

enum Kind { K_SWEEP_P = 0, K_ORTH_P, K_SWEEP_Q, K_COMBINE_Q, K_UPDATE, K_UPDATE_SWEEP_P, K_UPDATE_SGD,
            K_ORTH_V, K_COMBINE_P, K_COUNT };
const char *const kKindName[K_COUNT] = {"sweep_p", "orth_p", "sweep_q", "combine_q", "update",
                                        "update_sweep_p", "update_sgd", "orth_v", "combine_p"};

struct ProfRec {
    int kind;
    double bytes;
    hipEvent_t t0, t1;
};

}  // namespace

struct pg_ctx {
    Plan plan;
    bool uploaded = false;
    bool touched_device = false;  // some HIP allocation was attempted: pg_destroy has things to free
    PairDesc *d_pairs = nullptr;
    ColDesc *d_cols = nullptr;
    RowTile *d_row_tiles = nullptr;
    ColTile *d_col_tiles = nullptr;
    EdgeLayerDesc *d_els = nullptr;
    CombTile *d_comb = nullptr;
    OrthTile *d_orth = nullptr;
    int32_t *d_iso = nullptr;
    float **d_xs = nullptr;
    std::vector<float *> xs_cached;
    float **d_gs = nullptr;
    std::vector<const float *> gs_cached;
    bool mcol_stage = true;  // matrix-core Q-sweep: Phat of a tile's row block staged in LDS
    bool profiling = false;
    // Passes alternate direction through the parameters: each starts where the one before it
    // (also the last one of an earlier call) ended, on data still in the memory-side cache.
    bool alternate = true;
    int reverse = 0;  // direction of the next pass
    std::vector<ProfRec> recs;
    std::vector<hipEvent_t> free_events;
};

namespace {

#define PG_HIP(call)                                 \
    do {                                             \
        hipError_t err__ = (call);                   \
        if (err__ != hipSuccess) {                   \
            (void)hipGetLastError();                 \
            if (getenv("PG_VERBOSE"))                \
                fprintf(stderr, "powergossip: %s: %s\n", #call, hipGetErrorString(err__)); \
            return err__ == hipErrorOutOfMemory ? PG_ERR_NOMEM : PG_ERR_DEVICE; \
        }                                            \
    } while (0)

template <typename T>
int upload_vec(T **dst, const std::vector<T> &src) {
    size_t bytes = std::max<size_t>(src.size(), 1) * sizeof(T);
    PG_HIP(hipMalloc((void **)dst, bytes));
    if (!src.empty()) PG_HIP(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
    return PG_OK;
}

// Address of the static workspace on the current device (asked once per device).
int static_scratch(void **out) {
    int dev = -1;
    PG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return PG_ERR_DEVICE;
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        PG_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PG_OK;
}

int do_upload(pg_ctx *c) {
    if (c->uploaded) return PG_OK;
    c->touched_device = true;
    Plan &P = c->plan;
    std::vector<RowTile> rt;
    for (auto &rc : P.row_classes) {
        rc.dev_first = rt.size();
        rt.insert(rt.end(), rc.tiles.begin(), rc.tiles.end());
    }
    std::vector<ColTile> ct;
    for (auto &cc : P.col_classes) {
        cc.dev_first = ct.size();
        ct.insert(ct.end(), cc.tiles.begin(), cc.tiles.end());
    }
    int rc;
    if ((rc = upload_vec(&c->d_pairs, P.pairs))) return rc;
    if ((rc = upload_vec(&c->d_cols, P.cols))) return rc;
    if ((rc = upload_vec(&c->d_row_tiles, rt))) return rc;
    if ((rc = upload_vec(&c->d_col_tiles, ct))) return rc;
    if ((rc = upload_vec(&c->d_els, P.els))) return rc;
    if ((rc = upload_vec(&c->d_comb, P.comb_tiles))) return rc;
    if ((rc = upload_vec(&c->d_orth, P.orth_tiles))) return rc;
    if ((rc = upload_vec(&c->d_iso, P.isolated_pairs))) return rc;
    PG_HIP(hipMalloc((void **)&c->d_xs, sizeof(float *) * (size_t)P.n));
    PG_HIP(hipMalloc((void **)&c->d_gs, sizeof(float *) * (size_t)P.n));
    void *unused = nullptr;
    if ((rc = static_scratch(&unused))) return rc;
    c->uploaded = true;
    return PG_OK;
}

// Register blocking of the narrow row-owner kernel: M rows per lane group, loads issued D column
// steps ahead (M * D vector loads per lane in flight).  Measured on VGG-16 shapes, eight rows one
// step ahead beat fewer rows with a deeper pipeline for every mode and column count, also where
// part of the M * RC accumulators and update coefficients then lives in accumulation registers.
constexpr int kRowsPerGroup = 8;
constexpr int kRowsPerGroupLight = 4;  // small parameter sets (Plan::light)
constexpr int kPrefetchSteps = 1;
// Matrix-core kernels: steps a row tile and a column tile load ahead (measured on the
// LSTM-shaped torus: deeper rings only cost registers).
constexpr int kMfmaRowPrefetch = 1;
constexpr int kMfmaColPrefetch = 2;

struct Launcher {
    pg_ctx *c;
    hipStream_t st;
    float *qstate;
    char *ws;
    double eta = 0.0;  // learning rate of the fused gradient term
    // Algorithm 2 one iteration at a time: the right-hand vectors (length q) and the left-hand
    // vectors (length p) the sweeps and the update read, when they are not the state / Phat
    const float *rhs = nullptr;
    const float *lhs = nullptr;
    bool quiet = false;  // never record timing events (creating an event allocates)
    int status = PG_OK;

    const float *right() const { return rhs ? rhs : qstate; }
    const float *left() const { return lhs ? lhs : ph(); }
    float *uq() const { return (float *)(ws + c->plan.ws_uq); }

    double *pw() const { return (double *)(ws + c->plan.ws_pw); }
    double *qw() const { return (double *)(ws + c->plan.ws_qw); }
    double *pdb() const { return (double *)(ws + c->plan.ws_pd); }
    float *ph() const { return (float *)(ws + c->plan.ws_ph); }
    int32_t *flags() const { return (int32_t *)(ws + c->plan.ws_flag); }
    double *gpart() const { return (double *)(ws + c->plan.ws_gpart); }

    hipEvent_t get_event() {
        if (!c->free_events.empty()) {
            hipEvent_t e = c->free_events.back();
            c->free_events.pop_back();
            return e;
        }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) status = PG_ERR_DEVICE;
        return e;
    }
    void begin(int kind, double bytes) {
        if (!c->profiling || quiet || status) return;
        ProfRec r{kind, bytes, get_event(), get_event()};
        if (status) return;
        if (hipEventRecord(r.t0, st) != hipSuccess) status = PG_ERR_DEVICE;
        c->recs.push_back(r);
    }
    void end() {
        if (!c->profiling || quiet || status) return;
        if (hipEventRecord(c->recs.back().t1, st) != hipSuccess) status = PG_ERR_DEVICE;
    }
    void check() {
        if (hipGetLastError() != hipSuccess) status = PG_ERR_DEVICE;
    }

    template <int RC, bool UPD, bool SWP, bool GRAD = false>
    void row_launch(const RowClass &rc) {
        const int n = (int)rc.tiles.size();
        const RowTile *tiles = c->d_row_tiles + rc.dev_first;
        if constexpr (RC < kWideCols) {
            if (rc.vec)
                vec_row_kernel<RC, UPD, SWP, GRAD><<<dim3((unsigned)n), dim3(kRowThreads), 0, st>>>(
                    tiles, n, c->reverse, c->d_pairs, c->d_cols, c->d_xs, right(), left(), pw(), c->d_gs, eta);
            else if (c->plan.light)
                row_kernel<RC, kRowsPerGroupLight, kPrefetchSteps, UPD, SWP, GRAD><<<dim3((unsigned)n), dim3(kRowThreads), 0, st>>>(
                    tiles, n, c->reverse, c->d_pairs, c->d_cols, c->d_xs, right(), left(), pw(), c->d_gs, eta);
            else
                row_kernel<RC, kRowsPerGroup, kPrefetchSteps, UPD, SWP, GRAD><<<dim3((unsigned)n), dim3(kRowThreads), 0, st>>>(
                    tiles, n, c->reverse, c->d_pairs, c->d_cols, c->d_xs, right(), left(), pw(), c->d_gs, eta);
        } else if (rc.mfma) {
#define PG_MROW(VV) mrow_kernel<VV, RC / 4, kMfmaRowBlocks, kMfmaRowPrefetch, UPD, SWP, GRAD> \
                <<<dim3((unsigned)n), dim3(kThreads), kMrowLdsBytes, st>>>( \
                tiles, n, c->reverse, c->d_pairs, c->d_cols, c->d_xs, right(), left(), pw(), c->d_gs, eta)
            if (rc.V == 4) PG_MROW(4);
            else if (rc.V == 2) PG_MROW(2);
            else PG_MROW(1);
#undef PG_MROW
        } else {
            // register budget: RC accumulators and RC update coefficients per row
            constexpr int M = ((UPD && SWP) || GRAD || (RC > 8 && UPD)) ? 2 : 4;
            size_t lds = (size_t)RC * rc.max_seg * sizeof(float);
#define PG_WIDE(VV) row_wide_kernel<VV, RC, M, UPD, SWP, GRAD><<<dim3((unsigned)n), dim3(kThreads), lds, st>>>( \
                tiles, n, c->reverse, c->d_pairs, c->d_cols, c->d_xs, right(), left(), pw(), c->d_gs, eta)
            if (rc.V == 4) PG_WIDE(4);
            else if (rc.V == 2) PG_WIDE(2);
            else PG_WIDE(1);
#undef PG_WIDE
        }
    }
    template <int RC>
    void row_mode(const RowClass &rc, bool upd, bool swp, bool grad) {
        if (grad) {
            row_launch<RC, true, false, true>(rc);
        } else if (upd && swp) {
            if (RC <= kWideCols || rc.mfma) {
                row_launch<RC, true, true>(rc);
            } else {
                // with many stacked columns the fused pass does not fit in registers and is bound
                // by arithmetic, not memory: two passes are faster
                row_launch<RC, true, false>(rc);
                row_launch<RC, false, true>(rc);
            }
        } else if (upd) {
            row_launch<RC, true, false>(rc);
        } else {
            row_launch<RC, false, true>(rc);
        }
    }
    // One pass of the row-owner kernels over every parameter: sweep, update, or
    // both; `grad` = update with the gradient term (X -= eta * G) in the same pass.
    void rows(bool upd, bool swp, bool grad = false) {
        if (status) return;
        int kind = grad ? K_UPDATE_SGD : (upd ? (swp ? K_UPDATE_SWEEP_P : K_UPDATE) : K_SWEEP_P);
        const auto &classes = c->plan.row_classes;
        for (size_t k = 0; k < classes.size(); ++k) {
            const RowClass &rc = classes[c->reverse ? classes.size() - 1 - k : k];
            if (rc.tiles.empty()) continue;
            // a worker with several column groups: the gradient enters with the first group only
            const bool g = grad && rc.group == 0;
            begin(kind, rc.elems * 4.0 * (g ? 3.0 : (upd ? 2.0 : 1.0)));
            switch (rc.RC) {
                case 1: row_mode<1>(rc, upd, swp, g); break;
                case 2: row_mode<2>(rc, upd, swp, g); break;
                case 4: row_mode<4>(rc, upd, swp, g); break;
                case 8: row_mode<8>(rc, upd, swp, g); break;
                default: row_mode<16>(rc, upd, swp, g); break;
            }
            check();
            end();
        }
        turn();
    }
    // The next pass walks the parameters the other way.
    void turn() {
        if (c->alternate) c->reverse ^= 1;
    }
    // Workers without edges: their whole step is X -= eta * G.
    void sgd_isolated() {
        const Plan &P = c->plan;
        if (status || P.isolated_pairs.empty()) return;
        begin(K_UPDATE_SGD, P.isolated_elems * 12.0);
        sgd_only_kernel<<<dim3(64u * (unsigned)P.isolated_pairs.size()), dim3(kThreads), 0, st>>>(
            c->d_iso, c->d_pairs, c->d_xs, c->d_gs, eta);
        check();
        end();
    }

    template <int RC>
    void col_launch(const ColClass &cc) {
        constexpr int U = (RC <= 4) ? 8 : 4;  // rows in flight per lane
        const int n = (int)cc.tiles.size();
        // LDS: the staged Phat slice plus one zero row, later reused for the cross-wavefront sums
        size_t lds = std::max((size_t)(cc.max_rows + 1) * RC * sizeof(float),
                              (size_t)(kThreads / 64 - 1) * 64 * 4 * sizeof(double));
#define PG_COL(VV) col_kernel<VV, RC, U><<<dim3((unsigned)n), dim3(kThreads), lds, st>>>( \
            c->d_col_tiles + cc.dev_first, n, c->reverse, c->d_pairs, c->d_cols, \
            c->d_xs, left(), qw())
        if constexpr (RC < kWideCols) {
            if (cc.vec)
                vec_col_kernel<RC><<<dim3((unsigned)n), dim3(kRowThreads), 0, st>>>(
                    c->d_col_tiles + cc.dev_first, n, c->reverse, c->d_pairs, c->d_cols, c->d_xs, left(), qw());
            else
                PG_COL(0);
        } else if (c->plan.mfma_cols) {
#define PG_MCOL(VV, STAGE, LDS) mcol_kernel<VV, kMfmaColPrefetch, STAGE><<<dim3((unsigned)n), dim3(kThreads), LDS, st>>>( \
            c->d_col_tiles + cc.dev_first, n, c->reverse, c->d_pairs, c->d_cols, \
            c->d_xs, left(), qw())
            // The row block's Phat slice in LDS, where it fits beside a second work-group's.  Measured:
            // with 16 stacked columns the Q-sweep of the LSTM-shaped torus gains 5 % (430 -> 410 us);
            // with 8 (half of the staged slice zeros, many short layers) it loses 0.5 %.
            const size_t stage = (size_t)16 * mcol_stage_stride(cc.max_rows) * sizeof(float);
            if (c->mcol_stage && RC >= 16 && stage <= 64 * 1024) {
                if (cc.V == 4) PG_MCOL(4, true, stage);
                else if (cc.V == 2) PG_MCOL(2, true, stage);
                else PG_MCOL(1, true, stage);
            } else {
                if (cc.V == 4) PG_MCOL(4, false, 0);
                else if (cc.V == 2) PG_MCOL(2, false, 0);
                else PG_MCOL(1, false, 0);
            }
#undef PG_MCOL
        } else {
            if (cc.V == 4) PG_COL(4);
            else if (cc.V == 2) PG_COL(2);
            else PG_COL(1);
        }
#undef PG_COL
    }
    void sweep_q() {
        if (status) return;
        const auto &classes = c->plan.col_classes;
        for (size_t k = 0; k < classes.size(); ++k) {
            const ColClass &cc = classes[c->reverse ? classes.size() - 1 - k : k];
            if (cc.tiles.empty()) continue;
            begin(K_SWEEP_Q, cc.elems * 4.0);
            switch (cc.RC) {
                case 1: col_launch<1>(cc); break;
                case 2: col_launch<2>(cc); break;
                case 4: col_launch<4>(cc); break;
                case 8: col_launch<8>(cc); break;
                default: col_launch<16>(cc); break;
            }
            check();
            end();
        }
        turn();
    }
    template <int NT, int RMAX>
    void orth_launch() {
        const Plan &P = c->plan;
        if (P.orth_tiles.empty()) {
            orth_gram_kernel<NT, RMAX><<<dim3((unsigned)P.els.size()), dim3(NT), 0, st>>>(
                c->d_els, pw(), ph(), flags());
        } else {
            dim3 grid((unsigned)P.orth_tiles.size());
            orth_gram_part_kernel<NT, RMAX><<<grid, dim3(NT), 0, st>>>(c->d_orth, c->d_els, pw(), gpart(), nullptr);
            orth_gram_apply_kernel<NT, RMAX><<<grid, dim3(NT), 0, st>>>(c->d_orth, c->d_els, pw(), gpart(),
                                                                        ph(), flags(), nullptr);
        }
    }
    void orth_p() {
        if (status || c->plan.els.empty()) return;
        begin(K_ORTH_P, 0.0);
        const int rmax = c->plan.max_layer_rank;
        // short layers: small work-groups, so that many (edge, layer) pairs share a CU
        // (row chunks of tall layers are sized for 256 threads as well)
        const bool small = c->plan.max_rows <= 2048 || !c->plan.orth_tiles.empty();
        if (rmax <= 1) small ? orth_launch<256, 1>() : orth_launch<kOrthThreads, 1>();
        else if (rmax <= 2) small ? orth_launch<256, 2>() : orth_launch<kOrthThreads, 2>();
        else if (rmax <= 4) small ? orth_launch<256, 4>() : orth_launch<kOrthThreads, 4>();
        else if (rmax <= 8) small ? orth_launch<256, 8>() : orth_launch<512, 8>();
        else orth_kernel<kOrthThreads><<<dim3((unsigned)c->plan.els.size()), dim3(kOrthThreads), 0, st>>>(
            c->d_els, pw(), pdb(), ph(), flags());
        check();
        end();
    }
    // Algorithm 2's normalisation of the stored vectors (Gram-Schmidt for r > 1): src -> dst.
    template <int RMAX>
    void orth_v_launch(const float *src, float *dst, int in_q) {
        const Plan &P = c->plan;
        if (!in_q && !P.orth_tiles.empty()) {
            // vectors of length p with tall layers among them: chunk by chunk, like the round's own
            // orthonormalisation
            dim3 grid((unsigned)P.orth_tiles.size());
            orth_gram_part_kernel<256, RMAX><<<grid, dim3(256), 0, st>>>(c->d_orth, c->d_els, nullptr, gpart(), src);
            orth_gram_apply_kernel<256, RMAX><<<grid, dim3(256), 0, st>>>(c->d_orth, c->d_els, nullptr, gpart(),
                                                                          dst, flags(), src);
            return;
        }
        constexpr int NT = RMAX <= 4 ? 1024 : 512;
        orth_state_kernel<NT, RMAX><<<dim3((unsigned)P.els.size()), dim3(NT), 0, st>>>(
            c->d_els, src, dst, in_q, flags());
    }
    void orth_v(const float *src, float *dst, int in_q) {
        if (status || c->plan.els.empty()) return;
        begin(K_ORTH_V, 0.0);
        const int rmax = c->plan.max_layer_rank;
        if (rmax <= 1) orth_v_launch<1>(src, dst, in_q);
        else if (rmax <= 2) orth_v_launch<2>(src, dst, in_q);
        else if (rmax <= 4) orth_v_launch<4>(src, dst, in_q);
        else if (rmax <= 8) orth_v_launch<8>(src, dst, in_q);
        else status = PG_ERR_ARG;
        check();
        end();
    }
    void combine_p(float *pstate) {
        if (status || c->plan.els.empty()) return;
        begin(K_COMBINE_P, 0.0);
        // a grid's second dimension holds at most 65535 chunks
        const int chunk_rows = std::max(kCombPRows, (c->plan.max_rows + 65534) / 65535);
        const unsigned chunks = (unsigned)((c->plan.max_rows + chunk_rows - 1) / chunk_rows);
        comb_p_kernel<<<dim3((unsigned)c->plan.els.size(), chunks), dim3(kThreads), 0, st>>>(c->d_els, pw(), flags(), pstate,
                                                                                             chunk_rows);
        check();
        end();
    }
    void combine_q() {
        if (status || c->plan.comb_tiles.empty()) return;
        begin(K_COMBINE_Q, 0.0);
        comb_kernel<<<dim3((unsigned)c->plan.comb_tiles.size()), dim3(kThreads), 0, st>>>(
            c->d_comb, c->d_els, qw(), flags(), qstate);
        check();
        end();
    }
};

int prepare(pg_ctx *c, float *const *worker_params, float *q_state, void *workspace, hipStream_t st,
            bool may_allocate = true) {
    if (!c || !worker_params || !workspace) return PG_ERR_ARG;
    const Plan &P = c->plan;
    if (P.qstate_floats > 0 && !q_state) return PG_ERR_ARG;
    if (((uintptr_t)q_state & 15) || ((uintptr_t)workspace & 255)) return PG_ERR_ARG;
    for (int i = 0; i < P.n; ++i)
        if (!worker_params[i] || ((uintptr_t)worker_params[i] & 15)) return PG_ERR_ARG;
    if (!c->uploaded && !may_allocate) return PG_ERR_ARG;
    int rc = do_upload(c);
    if (rc) return rc;
    bool same = c->xs_cached.size() == (size_t)P.n;
    for (int i = 0; same && i < P.n; ++i) same = c->xs_cached[i] == worker_params[i];
    if (!same) {
        // Kernels already queued may still read the old table: drain the stream first.
        PG_HIP(hipStreamSynchronize(st));
        c->xs_cached.assign(worker_params, worker_params + P.n);
        PG_HIP(hipMemcpy(c->d_xs, c->xs_cached.data(), sizeof(float *) * (size_t)P.n, hipMemcpyHostToDevice));
    }
    return PG_OK;
}

int prepare_grads(pg_ctx *c, const float *const *worker_grads, hipStream_t st) {
    const Plan &P = c->plan;
    if (!worker_grads) return PG_ERR_ARG;
    for (int i = 0; i < P.n; ++i)
        if (!worker_grads[i] || ((uintptr_t)worker_grads[i] & 15)) return PG_ERR_ARG;
    bool same = c->gs_cached.size() == (size_t)P.n;
    for (int i = 0; same && i < P.n; ++i) same = c->gs_cached[i] == worker_grads[i];
    if (!same) {
        PG_HIP(hipStreamSynchronize(st));
        c->gs_cached.assign(worker_grads, worker_grads + P.n);
        PG_HIP(hipMemcpy(c->d_gs, c->gs_cached.data(), sizeof(float *) * (size_t)P.n, hipMemcpyHostToDevice));
    }
    return PG_OK;
}

int run_rounds(pg_ctx *c, float *const *worker_params, float *q_state, void *workspace,
               void *hip_stream, int rounds, bool fuse, bool may_allocate = true) {
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = prepare(c, worker_params, q_state, workspace, st, may_allocate);
    if (rc) return rc;
    if (c->plan.n_edges == 0 || rounds == 0) return PG_OK;
    Launcher L{c, st, q_state, (char *)workspace};
    L.quiet = !may_allocate;
    const int s = c->plan.steps;
    // Several column groups per worker: the update takes one pass per group, so no single pass
    // sees the finished parameters together with all of a worker's columns; rounds run unfused.
    if (c->plan.max_groups > 1) fuse = false;
    // Measured: with the passes that write (update + sweep) walking forwards and the Q-sweeps
    // backwards a run of fused rounds is 4 % faster than its mirror image, so a run starts forwards.
    if (fuse) c->reverse = 0;
    for (int t = 0; t < rounds; ++t) {
        for (int step = 0; step < s; ++step) {
            // the first product of a later round was already formed by the fused update pass
            if (!(fuse && t > 0 && step == 0)) L.rows(false, true);
            L.orth_p();
            L.sweep_q();
            L.combine_q();
        }
        L.rows(true, fuse && t + 1 < rounds);
    }
    return L.status;
}

}  // namespace

extern "C" {

const char *pg_strerror(int status) {
    switch (status) {
        case PG_OK: return "ok";
        case PG_ERR_ARG: return "invalid argument";
        case PG_ERR_TOPOLOGY: return "invalid topology (index out of range, self-loop or duplicate edge)";
        case PG_ERR_SHAPE: return "invalid layer shape";
        case PG_ERR_NOMEM: return "out of memory";
        case PG_ERR_DEVICE: return "HIP call failed";
        case PG_ERR_TOO_LARGE: return "problem needs more workspace than the static one holds";
        default: return "unknown status";
    }
}

int pg_init(pg_ctx **out, int n_workers, int n_edges, const int32_t *edges, const float *edge_w,
            int n_layers, const int32_t *rows, const int32_t *cols, int rank, int power_steps) {
    if (!out) return PG_ERR_ARG;
    pg_ctx *c = new (std::nothrow) pg_ctx();
    if (!c) return PG_ERR_NOMEM;
    Tuning tune;
    if (const char *e = getenv("PG_ROW_TILE_BYTES")) tune.row_tile_bytes = std::max(1024, atoi(e));
    if (const char *e = getenv("PG_ALTERNATE")) c->alternate = atoi(e) != 0;
    if (const char *e = getenv("PG_COL_TILE_BYTES")) tune.col_tile_bytes = std::max(1024, atoi(e));
    if (const char *e = getenv("PG_WIDE_TILE_BYTES")) {
        tune.wide_tile_bytes = std::max(1024, atoi(e));
        tune.mcol_tile_bytes = 2 * tune.wide_tile_bytes;
    }
    if (const char *e = getenv("PG_MCOL_TILE_BYTES")) tune.mcol_tile_bytes = std::max(1024, atoi(e));
    if (const char *e = getenv("PG_MFMA_ROWS")) tune.mfma_rows = atoi(e) != 0;
    if (const char *e = getenv("PG_MFMA_COLS")) tune.mfma_cols = atoi(e) != 0;
    if (const char *e = getenv("PG_MCOL_STAGE")) c->mcol_stage = atoi(e) != 0;
    if (const char *e = getenv("PG_LIGHT")) tune.light = atoi(e) != 0;
    if (const char *e = getenv("PG_VEC_KERNELS")) tune.vec_kernels = std::min(2, std::max(0, atoi(e)));
    if (const char *e = getenv("PG_MFMA_ROW_COLS")) tune.mfma_row_cols = atoi(e) <= 8 ? 8 : 16;
    int rc;
    try {
        rc = build_plan(c->plan, n_workers, n_edges, edges, edge_w, n_layers, rows, cols, rank,
                        power_steps, tune);
    } catch (const std::bad_alloc &) {
        rc = PG_ERR_NOMEM;
    }
    if (rc) {
        delete c;
        return rc;
    }
    *out = c;
    return PG_OK;
}

int pg_destroy(pg_ctx *c) {
    if (!c) return PG_ERR_ARG;
    if (c->touched_device) {  // also after an upload that failed half way: free what it got
        (void)hipDeviceSynchronize();
        for (auto &r : c->recs) {
            (void)hipEventDestroy(r.t0);
            (void)hipEventDestroy(r.t1);
        }
        for (auto e : c->free_events) (void)hipEventDestroy(e);
        (void)hipFree(c->d_pairs);
        (void)hipFree(c->d_cols);
        (void)hipFree(c->d_row_tiles);
        (void)hipFree(c->d_col_tiles);
        (void)hipFree(c->d_els);
        (void)hipFree(c->d_comb);
        (void)hipFree(c->d_orth);
        (void)hipFree(c->d_xs);
        (void)hipFree(c->d_gs);
        (void)hipFree(c->d_iso);
    }
    delete c;
    return PG_OK;
}

size_t pg_param_floats(const pg_ctx *c) { return c ? c->plan.param_floats : (size_t)-1; }
size_t pg_layer_offset(const pg_ctx *c, int l) {
    if (!c || l < 0 || l >= c->plan.n_layers) return (size_t)-1;
    return (size_t)c->plan.layers[l].x_off;
}
size_t pg_layer_stride(const pg_ctx *c, int l) {
    if (!c || l < 0 || l >= c->plan.n_layers) return (size_t)-1;
    return (size_t)c->plan.layers[l].ld;
}
int pg_layer_rank(const pg_ctx *c, int l) {
    if (!c || l < 0 || l >= c->plan.n_layers) return -1;
    return c->plan.layers[l].r;
}
size_t pg_qstate_floats(const pg_ctx *c) { return c ? c->plan.qstate_floats : (size_t)-1; }
size_t pg_q_offset(const pg_ctx *c, int e, int l) {
    if (!c || l < 0 || l >= c->plan.n_layers || e < 0 || e >= c->plan.n_edges) return (size_t)-1;
    return (size_t)c->plan.q_off[(size_t)e * c->plan.n_layers + l];
}
size_t pg_pstate_floats(const pg_ctx *c) { return c ? c->plan.pstate_floats : (size_t)-1; }
size_t pg_p_offset(const pg_ctx *c, int e, int l) {
    if (!c || l < 0 || l >= c->plan.n_layers || e < 0 || e >= c->plan.n_edges) return (size_t)-1;
    return (size_t)c->plan.ph_off[(size_t)e * c->plan.n_layers + l];
}
size_t pg_workspace_bytes(const pg_ctx *c) { return c ? c->plan.ws_bytes : (size_t)-1; }
size_t pg_ws_phat_offset(const pg_ctx *c, int e, int l) {
    if (!c || l < 0 || l >= c->plan.n_layers || e < 0 || e >= c->plan.n_edges) return (size_t)-1;
    return c->plan.ws_ph + 4 * (size_t)c->plan.ph_off[(size_t)e * c->plan.n_layers + l];
}
size_t pg_ws_flag_offset(const pg_ctx *c, int e, int l) {
    if (!c || l < 0 || l >= c->plan.n_layers || e < 0 || e >= c->plan.n_edges) return (size_t)-1;
    return c->plan.ws_flag + 4 * (size_t)c->plan.flag_off[(size_t)e * c->plan.n_layers + l];
}
size_t pg_message_floats(const pg_ctx *c) { return c ? c->plan.message_floats : (size_t)-1; }
double pg_round_bytes(const pg_ctx *c, int fused) {
    if (!c) return -1.0;
    if (c->plan.max_groups > 1)  // one pass per column group, never fused
        return 4.0 * c->plan.pass_elems * (2 * c->plan.steps + 2);
    int passes = 2 * c->plan.steps + (fused ? 1 : 2);
    return 4.0 * c->plan.n * c->plan.elems_per_worker * passes;
}

int pg_upload(pg_ctx *c) {
    if (!c) return PG_ERR_ARG;
    return do_upload(c);
}

int pg_round(pg_ctx *c, float *const *worker_params, float *q_state, void *workspace, void *hip_stream) {
    return run_rounds(c, worker_params, q_state, workspace, hip_stream, 1, false);
}

int pg_round_static(pg_ctx *c, float *const *worker_params, float *q_state, void *hip_stream) {
    if (!c) return PG_ERR_ARG;
    if (!c->uploaded) return PG_ERR_ARG;  // uploading allocates: pg_upload comes first
    if (c->plan.ws_bytes > (size_t)PG_STATIC_WORKSPACE_BYTES) return PG_ERR_TOO_LARGE;
    void *ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc) return rc;
    // Nothing in the workspace has to start at zero: every section is written by the round's own
    // kernels before it is read, so whatever an earlier call (of any context) left is harmless.
    return run_rounds(c, worker_params, q_state, ws, hip_stream, 1, false, /*may_allocate=*/false);
}

int pg_round_sgd(pg_ctx *c, float *const *worker_params, const float *const *worker_grads, float eta,
                 float *q_state, void *workspace, void *hip_stream) {
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = prepare(c, worker_params, q_state, workspace, st);
    if (rc) return rc;
    if (!std::isfinite(eta)) return PG_ERR_ARG;
    if ((rc = prepare_grads(c, worker_grads, st))) return rc;
    Launcher L{c, st, q_state, (char *)workspace};
    L.eta = (double)eta;
    const int s = c->plan.steps;
    if (c->plan.n_edges > 0) {
        for (int step = 0; step < s; ++step) {
            L.rows(false, true);
            L.orth_p();
            L.sweep_q();
            L.combine_q();
        }
        L.rows(true, false, /*grad=*/true);
    }
    L.sgd_isolated();
    return L.status;
}

int pg_iterate(pg_ctx *c, float *const *worker_params, float *q_state, float *p_state, long long k_done,
               int iterations, const float *const *worker_grads, float eta, void *workspace,
               void *hip_stream) {
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = prepare(c, worker_params, q_state, workspace, st);
    if (rc) return rc;
    if (k_done < 0 || iterations < 1 || (worker_grads && !std::isfinite(eta))) return PG_ERR_ARG;
    if (c->plan.pstate_floats > 0 && (!p_state || ((uintptr_t)p_state & 15))) return PG_ERR_ARG;
    if (c->plan.max_layer_rank > 8) return PG_ERR_ARG;
    if (worker_grads && (rc = prepare_grads(c, worker_grads, st))) return rc;
    Launcher L{c, st, q_state, (char *)workspace};
    L.eta = (double)eta;
    if (c->plan.n_edges > 0) {
        for (int it = 1; it <= iterations; ++it) {
            if ((k_done + it) & 1) {
                // odd: vhat = v / |v| in R^q, p = X_a vhat - X_b vhat, v <- p (in R^p)
                L.orth_v(q_state, L.uq(), 1);
                L.rhs = L.uq();
                L.rows(false, true);
                L.combine_p(p_state);
                L.lhs = p_state;  // approximation p vhat^T
            } else {
                // even: vhat = v / |v| in R^p, p' = X_a^T vhat - X_b^T vhat, v <- p' (in R^q)
                L.orth_v(p_state, L.ph(), 0);
                L.lhs = nullptr;  // the unit vectors sit where Phat sits
                L.sweep_q();
                L.combine_q();
                L.rhs = nullptr;  // approximation vhat p'^T
            }
        }
        L.rows(true, false, worker_grads != nullptr);
    }
    if (worker_grads) L.sgd_isolated();
    return L.status;
}

int pg_run(pg_ctx *c, float *const *worker_params, float *q_state, void *workspace,
           void *hip_stream, int rounds) {
    if (rounds < 0) return PG_ERR_ARG;
    return run_rounds(c, worker_params, q_state, workspace, hip_stream, rounds, true);
}

int pg_profile_enable(pg_ctx *c, int on) {
    if (!c) return PG_ERR_ARG;
    c->profiling = on != 0;
    return PG_OK;
}

int pg_profile_collect(pg_ctx *c, pg_kernel_time *out, int max_out, int *n_out) {
    if (!c || !out || !n_out || max_out < 0) return PG_ERR_ARG;
    pg_kernel_time acc[K_COUNT];
    for (int k = 0; k < K_COUNT; ++k) {
        memset(&acc[k], 0, sizeof(acc[k]));
        strncpy(acc[k].name, kKindName[k], sizeof(acc[k].name) - 1);
    }
    int status = PG_OK;
    for (auto &r : c->recs) {
        float ms = 0.0f;
        if (hipEventSynchronize(r.t1) != hipSuccess || hipEventElapsedTime(&ms, r.t0, r.t1) != hipSuccess) {
            (void)hipGetLastError();
            status = PG_ERR_DEVICE;
        }
        acc[r.kind].launches += 1;
        acc[r.kind].ms += ms;
        acc[r.kind].bytes += r.bytes;
        c->free_events.push_back(r.t0);
        c->free_events.push_back(r.t1);
    }
    c->recs.clear();
    int n = 0;
    for (int k = 0; k < K_COUNT && n < max_out; ++k)
        if (acc[k].launches > 0) out[n++] = acc[k];
    *n_out = n;
    return status;
}

}  // extern "C"
