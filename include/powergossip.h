/*
 * powergossip.h -- C ABI of the PowerGossip hot path for one MI355X (gfx950).
 *
 * The library runs simulated gossip rounds of PowerGossip (Vogels, Karimireddy, Jaggi,
 * "Practical Low-Rank Communication Compression in Decentralized Deep Learning",
 * arXiv 2008.01425) with all n workers' parameters resident in one GPU's memory.
 *
 * What one round computes (paper notation; Section 3, Eq. (2), Eq. (3), Algorithm 2;
 * the gradient-free consensus form is Eq. (4) of Section 4.2):
 *   - the model is a list of L matrices X^l in R^{p_l x q_l}, one copy X_i^l per worker i;
 *     convolution weights are reshaped to (output channels) x (inputs x kernel size) and
 *     vectors are p x 1 matrices (Section 2); every matrix is handled on its own;
 *   - the workers form an undirected graph with a symmetric mixing weight w_e = W_ab on
 *     each edge e = (a, b) (assumption A4); each edge and matrix owns a projection state
 *     Q_e^l in R^{q_l x r_l}, r_l = min(rank, p_l, q_l), initialised by the CALLER with
 *     N(0, 1) entries (initialisation of Algorithm 2);
 *   - with D_e = X_a - X_b taken at the start of the round, repeated `power_steps` times on
 *     the unchanged parameters:
 *         P_e    = X_a Q_e - X_b Q_e              (the products are formed per worker and
 *                                                  subtracted: "Linearity", Section 3.1)
 *         Phat_e = orthonormalise(P_e)            (2-norm for r = 1, Eq. (3); Gram-Schmidt over
 *                                                  the columns, left to right, for r > 1:
 *                                                  appendix "Changing rank vs ...")
 *         Q_e   <- X_a^T Phat_e - X_b^T Phat_e    (not normalised; Algorithm 2 stores p_j - p_i)
 *     One such pair is TWO of the paper's "iterations" (its odd and its even one);
 *   - then every worker applies, once, X_a -= w_e Phat_e Q_e^T and X_b += w_e Phat_e Q_e^T
 *     summed over its edges (Eq. (2); equal and opposite, so the mean is kept: Lemma 1);
 *   - Q_e is left in the state buffer as the warm start of the next round.
 *   A column of P_e whose Gram-Schmidt residual vanishes (squared norm below
 *   max(FLT_MIN, 1e-10 x its squared norm before projection)) is dropped for that step:
 *   zero Phat column, no contribution, its Q column kept (Section 3.1: a zero difference
 *   gives a zero update).
 *
 * Arithmetic: parameters, Q and Phat are stored as IEEE float; every sum (the products, the
 * norms, the Gram-Schmidt, the update of an element) is accumulated in double and rounded
 * to float once when stored.
 *
 * Conventions.  Every function returns an int status (0 = PG_OK, negative = error) unless it
 * is a size query.  Nothing throws or aborts.  "host" / "device" below says where a pointer
 * must point.  The caller owns the parameter buffers, the state buffer and the workspace
 * (plain device allocations); the library owns only the context and its descriptor tables.
 * Work is enqueued on the caller's HIP stream and the call returns without waiting; results
 * are defined once the stream has reached that point.  Calls on one context must not overlap.
 */
#ifndef POWERGOSSIP_H
#define POWERGOSSIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pg_ctx pg_ctx; /* opaque */

enum {
    PG_OK = 0,
    PG_ERR_ARG = -1,      /* null pointer, rank < 1, power_steps < 1, bad weight, unsupported size */
    PG_ERR_TOPOLOGY = -2, /* worker index out of range, self-loop, duplicate edge (either orientation) */
    PG_ERR_SHAPE = -3,    /* a layer with p < 1 or q < 1 */
    PG_ERR_NOMEM = -4,    /* host or device allocation failed */
    PG_ERR_DEVICE = -5,   /* a HIP call failed (no device, launch error, ...) */
    PG_ERR_TOO_LARGE = -6 /* pg_round_static: the problem needs more than PG_STATIC_WORKSPACE_BYTES */
};

/* Static, NUL-terminated description of a status code.  Never NULL. */
const char *pg_strerror(int status);

/*
 * Build a context: validate the problem and plan the launches.  Host work only -- no HIP
 * call is made, so this succeeds without a GPU; the descriptor tables are uploaded by
 * pg_upload() or by the first round.
 *
 *   out          host; receives the context (unchanged on error)
 *   n_workers    n >= 1
 *   n_edges      |E| >= 0
 *   edges        host, [2*n_edges] int32: pairs (a, b), a != b, each undirected edge once
 *   edge_w       host, [n_edges] float: w_e = W_ab = W_ba, finite and >= 0; for every worker the
 *                sum over its edges must be <= 1 + 1e-6 (its self-weight W_ii stays >= 0, A4)
 *   n_layers     L >= 1
 *   rows, cols   host, [n_layers] int32: p_l, q_l (q_l = 1 for vectors)
 *   rank         r >= 1 (r_l = min(r, p_l, q_l)); r_l must be <= 16.  A worker whose stacked
 *                columns deg(i) * r_l exceed 16 is handled in groups of whole edges, one pass over
 *                its matrix per group and product; its update is then applied group by group,
 *                each pass rounding the parameters to float once, and pg_run does not fuse
 *   power_steps  s >= 1
 * All host arrays are copied; the caller may free them on return.
 */
int pg_init(pg_ctx **out, int n_workers, int n_edges, const int32_t *edges, const float *edge_w,
            int n_layers, const int32_t *rows, const int32_t *cols, int rank, int power_steps);

/* Free the context and its device tables (synchronises the device if tables were uploaded). */
int pg_destroy(pg_ctx *ctx);

/*
 * Layout queries (host, no HIP call).
 *
 * A worker's parameter buffer is `pg_param_floats` floats; layer l is a row-major p_l x q_l
 * matrix starting at float `pg_layer_offset(l)` whose rows are `pg_layer_stride(l)` >= q_l floats
 * apart: element (row, c) is float offset + row * stride + c.  The stride is q_l, except for
 * layers that run with 8 or more stacked columns (deg(i) * r_l), whose rows are padded to whole
 * 128-byte lines (stride = q_l rounded up to a multiple of 32).  Offsets are multiples of 32
 * floats; padding, between rows or between layers, is never read or written.  Gradient buffers
 * (pg_round_sgd, pg_iterate) use the same layout.
 *
 * The state buffer is `pg_qstate_floats` floats; the block of edge e, layer l starts at float
 * `pg_q_offset(e, l)` (a multiple of 4) and holds r_l columns of q_l floats each, column k at
 * +k*q_l: one of Algorithm 2's vectors v_ij per column.
 *
 * Out-of-range indices give (size_t)-1 (pg_layer_rank: -1).
 */
size_t pg_param_floats(const pg_ctx *ctx);
size_t pg_layer_offset(const pg_ctx *ctx, int layer);
size_t pg_layer_stride(const pg_ctx *ctx, int layer);
int pg_layer_rank(const pg_ctx *ctx, int layer);
size_t pg_qstate_floats(const pg_ctx *ctx);
size_t pg_q_offset(const pg_ctx *ctx, int edge, int layer);

/* Bytes of device scratch the caller lends to every round (256-byte aligned). */
size_t pg_workspace_bytes(const pg_ctx *ctx);

/*
 * Where the last power step's Phat_e^l (r_l float columns of length p_l, column k at +k*p_l)
 * and its dropped-column flags (r_l int32, 1 = dropped) sit inside the workspace, as BYTE
 * offsets; valid after a round, until the next one.  For inspection and tests.
 */
size_t pg_ws_phat_offset(const pg_ctx *ctx, int edge, int layer);
size_t pg_ws_flag_offset(const pg_ctx *ctx, int edge, int layer);

/*
 * Floats one endpoint of an edge would send per power step if the workers sat on different
 * devices: sum over layers of r_l * (p_l + q_l) -- a length-p then a length-q vector per
 * matrix and rank column (Algorithm 2; the "Compression" column of the paper's parameter
 * tables is p*q / ((p+q)/2) per iteration).
 */
size_t pg_message_floats(const pg_ctx *ctx);

/*
 * Algorithmic bytes of parameter traffic of one round: 4 * n * N * passes, N = sum p_l q_l,
 * passes = 2*power_steps + 2 for pg_round (each product reads every X once, the update reads
 * and writes it), 2*power_steps + 1 per round inside pg_run (the update also feeds the next
 * round's first product).
 */
double pg_round_bytes(const pg_ctx *ctx, int fused);

/* Upload the descriptor tables to the current device now (otherwise the first round does it).
   Allocates device memory and synchronises. */
int pg_upload(pg_ctx *ctx);

/*
 * One gossip round.
 *   worker_params  host array of n_workers DEVICE pointers, each to pg_param_floats floats,
 *                  16-byte aligned (128-byte alignment lets padded rows start on cache lines);
 *                  updated in place.  The pointer values are cached; a call
 *                  with different values re-uploads the table (a synchronous copy).
 *   q_state        device, pg_qstate_floats floats, 16-byte aligned; in: Q, out: Q'
 *   workspace      device, pg_workspace_bytes bytes, 256-byte aligned; contents need not persist
 *   hip_stream     a hipStream_t (NULL = the default stream)
 * Errors: PG_ERR_ARG for null or misaligned pointers, PG_ERR_DEVICE / PG_ERR_NOMEM from HIP.
 */
int pg_round(pg_ctx *ctx, float *const *worker_params, float *q_state, void *workspace,
             void *hip_stream);

/*
 * pg_round for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same round, same results bit for bit, but the
 * workspace is a fixed array of PG_STATIC_WORKSPACE_BYTES that lives inside the library's code
 * object on every GPU it is loaded on (held until the process ends), and the call makes no
 * hipMalloc, hipFree or other allocating call: no table upload (the context must have been
 * through pg_upload, else PG_ERR_ARG), no timing events (pg_profile_enable is ignored).  A new
 * set of worker_params pointers is still copied to the device table (a synchronous copy).
 * A problem with pg_workspace_bytes > PG_STATIC_WORKSPACE_BYTES is refused with
 * PG_ERR_TOO_LARGE and nothing is launched.  All contexts and calls on one GPU share the one
 * array: calls that overlap on a GPU (different streams or threads) race; calls ordered on one
 * stream, or separated by a synchronisation, do not.  Phat and the flags of the round are not
 * reachable through pg_ws_*_offset for this call.  Other arguments and errors as pg_round.
 */
#define PG_STATIC_WORKSPACE_BYTES (32u << 20)
int pg_round_static(pg_ctx *ctx, float *const *worker_params, float *q_state, void *hip_stream);

/*
 * One step of decentralized SGD with edge-wise compression (the update step of Algorithm 1):
 *     X_i <- X_i + sum_j W_ij C(X_j - X_i) - eta * G_i
 * i.e. pg_round with the stochastic-gradient term folded into the update pass (the update then
 * reads X and G and writes X once: 12 instead of 8 + 12 bytes per parameter for a separate
 * SGD step).  Both terms enter one double-precision sum that is rounded to float once.
 *   worker_grads   host array of n_workers DEVICE pointers, laid out like the parameter
 *                  buffers (pg_param_floats floats, same layer offsets), 16-byte aligned;
 *                  read only.  Cached like worker_params.  Any update direction may stand
 *                  here: with momentum (the Cifar-10 settings of the appendix use 0.9) the
 *                  caller keeps the momentum buffer and passes it as G.
 *   eta            learning rate (finite, else PG_ERR_ARG)
 * Workers without edges get X_i -= eta * G_i.  Other arguments and errors as pg_round.
 */
int pg_round_sgd(pg_ctx *ctx, float *const *worker_params, const float *const *worker_grads,
                 float eta, float *q_state, void *workspace, void *hip_stream);

/*
 * Algorithm 2 taken literally, one mat-vec iteration at a time.  `iterations` iterations,
 * numbered k_done + 1 ... k_done + iterations, run on the unchanged parameters and the
 * approximation of the LAST one is applied (the procedure overwrites its approximation in the
 * loop and returns it once); with `worker_grads` the step is the update step of Algorithm 1.
 *   odd k : vhat = v / |v| in R^q;  p  = X_a vhat - X_b vhat;      approximation p vhat^T;   v <- p
 *   even k: vhat = v / |v| in R^p;  p' = X_a^T vhat - X_b^T vhat;  approximation vhat p'^T;  v <- p'
 * The vector alternates between the two spaces: in R^q it lives in q_state (layout above), in
 * R^p in p_state: pg_pstate_floats floats, the block of edge e, layer l at float pg_p_offset(e, l)
 * (a multiple of 4), r_l columns of p_l floats.  The space of the current iteration is read, the
 * other written; the caller keeps k (pass the number of iterations already done) and both
 * buffers.  rank > 1 (at most 8 here) orthonormalises the r columns instead of normalising one.
 * A column whose normalisation fails by the dropped-column rule contributes nothing and leaves
 * the buffer it would have written untouched.  One iteration sends one vector per matrix --
 * the paper's "PowerGossip (1 iteration)"; k_done even with iterations = 2 applies the same
 * approximation as one power step of pg_round.
 *   p_state        device, 16-byte aligned, in/out
 *   worker_grads   NULL, or as in pg_round_sgd;  eta ignored when NULL
 * Other arguments and errors as pg_round.
 */
size_t pg_pstate_floats(const pg_ctx *ctx);
size_t pg_p_offset(const pg_ctx *ctx, int edge, int layer);
int pg_iterate(pg_ctx *ctx, float *const *worker_params, float *q_state, float *p_state,
               long long k_done, int iterations, const float *const *worker_grads, float eta,
               void *workspace, void *hip_stream);

/*
 * `rounds` consecutive gossip rounds with nothing touching the parameters in between
 * (the pure consensus iteration, Eq. (4)).  Same result as calling pg_round `rounds` times;
 * the update of round t and the first product of round t+1 share one pass over the
 * parameters.  rounds >= 0.  Once a call has seen the same worker_params pointers (the first
 * call with a new set copies the pointer table to the device and waits for the stream), a call
 * with profiling off only launches kernels: it may be recorded into a HIP graph on a capturing
 * stream and replayed.
 */
int pg_run(pg_ctx *ctx, float *const *worker_params, float *q_state, void *workspace,
           void *hip_stream, int rounds);

/*
 * Per-kernel timing.  While enabled, every kernel launched by pg_round / pg_run is bracketed
 * by HIP events on the caller's stream.  pg_profile_collect waits for the recorded events,
 * adds them up per kernel kind since the previous collect, and clears the record.
 */
typedef struct pg_kernel_time {
    char name[32];   /* "sweep_p", "orth_p", "sweep_q", "combine_q", "update", "update_sweep_p", "update_sgd",
                        "orth_v", "combine_p" */
    int launches;    /* kernel launches of this kind */
    double ms;       /* summed duration */
    double bytes;    /* summed algorithmic bytes of parameter traffic (4 B per element read or written) */
} pg_kernel_time;

int pg_profile_enable(pg_ctx *ctx, int on);
/* out: host array of `max_out` entries; *n_out receives how many were filled. */
int pg_profile_collect(pg_ctx *ctx, pg_kernel_time *out, int max_out, int *n_out);

#ifdef __cplusplus
}
#endif
#endif /* POWERGOSSIP_H */
