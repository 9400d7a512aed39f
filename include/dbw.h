/*
 * dbw - consensus-based distributed SGD with dynamic backup workers, one training round
 * for all N simulated workers at once on one AMD MI355X (gfx950).
 *
 * C ABI.  Pointers are tagged "host" or "dev" (device memory, HIP).  `stream` is a
 * hipStream_t passed as void* (NULL = the default stream).  Every function returns an
 * int: DBW_OK or a negative DBW_ERR_* code; nothing throws across this boundary.  No
 * function synchronises the stream unless its comment says so.  The library never frees
 * or keeps caller memory except where stated; caller arrays must stay valid until the
 * stream work that uses them has completed.
 *
 * Concurrency.  A context holds the state of one run (selection, weights, threshold-rule
 * epoch, gradient scratch) in device memory that its kernels read and write: calls on one
 * context must be ordered, i.e. issued from one host thread at a time and on one stream
 * (or on streams the caller orders with events).  Different contexts are independent.
 * The device that is current when dbw_create is called owns the context; make it current
 * again for every later call on that context.
 *
 * Layout (the default, DBW_LAYOUT_ROWS; see DBW_LAYOUT_TILES for the alternative).
 * Worker i's parameter vector is row i of a row-major [N][ld] float array,
 * d <= ld; columns [d, ld) are padding that the library never reads into results and
 * never writes.  This is the transpose of the paper's d x N matrix W(k) (Section 2.2),
 * so the paper's right-multiplication by the consensus matrix P(k) becomes a
 * left-multiplication: X' = P X with row i of P holding worker i's weights.
 * Inside a row the model parameters are stored layer by layer, weight [out][in]
 * (convolutions [Cout][Cin][kh][kw]) followed by the bias [out].
 *
 * Graph.  The communication graph G = (N, E) of Section 2.1 is given in CSR form
 * without self loops: the neighbours of worker i are colidx[rowptr[i] .. rowptr[i+1]),
 * strictly ascending; the graph must be symmetric and connected.  deg_i is the row
 * length; the paper's neighbourhood N_i is that row plus i itself.
 */
#ifndef DBW_H
#define DBW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dbw_ctx dbw_ctx; /* opaque, owned by the library */

enum {
    DBW_OK = 0,
    DBW_ERR_NULL = -1,        /* a required pointer is NULL */
    DBW_ERR_INVALID = -2,     /* bad N, d, ld, model description, or b_i outside [0, deg_i] */
    DBW_ERR_GRAPH = -3,       /* CSR unsorted / asymmetric / self loop / out of range / disconnected */
    DBW_ERR_ALIAS = -4,       /* params_in overlaps params_out */
    DBW_ERR_STATE = -5,       /* dbw_round or dbw_get_selection before any dbw_select */
    DBW_ERR_ALLOC = -6,       /* device or host allocation failed */
    DBW_ERR_HIP = -7,         /* a HIP call failed */
    DBW_ERR_UNSUPPORTED = -8, /* combination not implemented (e.g. dense mixing for N > 256) */
    /* Deferred warning (positive, reported by dbw_check / dbw_get_selection like the deferred
     * errors, never by the call itself): dbw_dtur_b found no link of its set that can still be
     * established in this round (a worker with an infinite response time on every unvisited
     * link), so theta = +inf.  The backup counts it wrote are still the rule's. */
    DBW_WARN_THETA_INF = 1
};

/* Order of averaging and local step inside one round. */
enum {
    /* x_i' = sum_j P_ij x_j - lr g(x_i): average the neighbours' estimates, then correct
     * with the gradient taken at the pre-average point (Section 2.1, the
     * full-participation update; the abstract describes the same order). */
    DBW_ORDER_CTA = 0,
    /* x~_j = x_j - lr g(x_j) for all j, then x_i' = sum_j P_ij x~_j (Section 2.2, the
     * local update followed by the partial consensus update; Algorithm 1). */
    DBW_ORDER_ATC = 1
};

/* How the masked consensus average is evaluated. */
enum {
    DBW_MIX_AUTO = 0,  /* dense when it is supported and the graph holds more than N*N/4 links */
    DBW_MIX_CSR = 1,   /* gather over the selected neighbours only (HBM bound) */
    DBW_MIX_DENSE = 2  /* materialise P(k) as N x N and multiply on the matrix cores; needs N <= 256
                        * and ld <= 26 843 545 (DBW_ERR_UNSUPPORTED from dbw_create otherwise).
                        * Every worker's row enters every product, backup workers with weight 0:
                        * if a worker's parameters or gradients hold inf or NaN, every output row
                        * becomes NaN (0 x inf), whereas the sparse path, which reads selected rows
                        * only, keeps the rows that do not wait for that worker finite.  The same
                        * holds for dbw_consensus_rounds.  Use DBW_MIX_CSR where diverged workers
                        * must stay contained. */
};

/* How the N parameter vectors are laid out in a [N * ld] float array. */
enum {
    /* worker i's vector is row i: element (i, c) at i * ld + c */
    DBW_LAYOUT_ROWS = 0,
    /* tile-major: the columns are cut into tiles of DBW_TILE_COLUMNS, and the pieces of all
     * N workers for one tile are stored together: element (i, c) at
     * (c / 64) * N * 64 + i * 64 + c % 64.  ld must be a multiple of 64.  The masked average
     * needs every worker's values of a column range at the same time; this layout turns that
     * into linear memory streams (about 15-20 % faster on MI355X than rows that lie a whole row
     * apart).  Available without a model (gradients supplied by the caller in the same
     * layout), N <= 256, sparse mixing path; dbw_convert_layout moves between the two. */
    DBW_LAYOUT_TILES = 1
};
#define DBW_TILE_COLUMNS 64

enum {
    DBW_MODEL_NONE = 0,    /* gradients are supplied by the caller (ext_grads) */
    DBW_MODEL_SOFTMAX = 1, /* multinomial logistic regression dims[0] -> dims[1] (the LRM of
                              Section 5): the fully connected model with one layer; n_layers is
                              ignored */
    DBW_MODEL_MLP = 2,     /* fully connected dims[0] -> ... -> dims[n_layers], ReLU between
                              layers, softmax on top */
    DBW_MODEL_CNN = 3      /* conv KxK (C0->C1, same padding) ReLU maxpool2, conv KxK (C1->C2)
                              ReLU maxpool2, flatten, FC F ReLU, FC classes, cross-entropy;
                              dims = {C0, H, W, C1, C2, K, F, classes} */
};

/* Loss on top of the model's outputs. */
enum {
    DBW_LOSS_XENT = 0, /* softmax cross-entropy (Section 5) */
    DBW_LOSS_MSE = 1   /* squared error of the softmax outputs against the one-hot label, summed
                          over classes (the 2NN of Appendix B); fully connected models only */
};

/* How the gradient of a fully connected model is launched.  The results agree to rounding (the
 * products are summed in different orders). */
enum {
    DBW_GRAD_AUTO = 0,   /* the library picks: the chain where it applies, else per-layer launches, which
                            may share one weight-gradient launch and take the kernels for batches of at
                            most 64 samples */
    DBW_GRAD_LAYERS = 1, /* one batched GEMM launch per layer and pass */
    DBW_GRAD_CHAIN = 2   /* forward pass, loss and data gradients of all layers in one launch, a
                            workgroup per block of samples with the activations in LDS; for
                            DBW_MODEL_MLP with at least two layers, equal hidden widths of 128, 256
                            or 512, dims[0] a multiple of 16 and at most 16 classes
                            (DBW_ERR_UNSUPPORTED from dbw_create otherwise, or from dbw_round when
                            batch_x or the parameter rows do not start on 16-byte boundaries) */
};

typedef struct {
    int32_t kind;     /* DBW_MODEL_* */
    int32_t batch;    /* samples per worker per round (|C_j(k)| of Section 2.1) */
    int32_t n_layers; /* MLP only */
    int32_t loss;     /* DBW_LOSS_*; the mean over the batch is taken */
    int32_t dims[9];
    int32_t grad_path; /* DBW_GRAD_*; fully connected models only */
} dbw_model;

typedef struct {
    int64_t ld;       /* row stride in floats, >= d; 0 means d */
    int32_t order;    /* DBW_ORDER_* */
    int32_t mix_path; /* DBW_MIX_* */
    int32_t layout;   /* DBW_LAYOUT_*: applies to params_in, params_out and ext_grads of dbw_round */
    dbw_model model;
} dbw_opts;

/* Create a context for N workers with d parameters each on the current HIP device.
 * rowptr [host, N+1] and colidx [host, rowptr[N]] are validated (DBW_ERR_GRAPH) and
 * copied; the caller may free them afterwards.  opts may be NULL (ld = d, CTA order,
 * automatic mixing path, no model).  With a model, d must equal the model's parameter
 * count.  The link set for dbw_dtur_b (a breadth-first spanning tree from worker 0,
 * neighbours in ascending index, N - 1 links; Section 4.1) is built here.  Allocates the
 * context's device scratch; synchronous. */
int dbw_create(dbw_ctx **out, int32_t N, int64_t d, const int32_t *rowptr, const int32_t *colidx,
               const dbw_opts *opts);

/* Fastest-neighbour selection for one round (Section 1 "Dynamic Backup Workers",
 * Section 2.2): worker i waits for the p_i = deg_i - b_i neighbours with the smallest
 * response times and treats the other b_i as backups.  Neighbours are ordered by
 * (time, index) under IEEE comparison, NaN counting as +inf, so ties go to the lower
 * index.  Also prepares the Metropolis weights of Assumption 1,
 * P_ij = 1 / (1 + max(p_i, p_j)) for selected j, P_ii = 1 - sum_j P_ij, for the next
 * dbw_round.  resp_times [dev, N] float, b [dev, N] int32.  A b_i outside [0, deg_i] is
 * clamped for memory safety and recorded; dbw_get_selection / dbw_check report it as
 * DBW_ERR_INVALID.  Asynchronous on `stream`. */
int dbw_select(dbw_ctx *ctx, const float *resp_times, const int32_t *b, void *stream);

/* Backup counts from the distributed threshold-based update rule (Section 4.1,
 * Algorithm 2): theta = the earliest time max(t_u, t_v) at which a link (u, v) of the
 * link set that was not yet visited in the current epoch is established (lowest link id
 * on ties); that link is marked visited, and after all N - 1 links have been visited the
 * set is emptied.  A worker with t_j <= theta waits for exactly its neighbours with
 * t_i <= theta, any other worker for nobody: b_out[j] = deg_j - |S_j|.  Feed b_out to
 * dbw_select.  The epoch state lives in the context (dbw_dtur_reset empties it).
 * resp_times [dev, N], b_out [dev, N], theta_out [dev, 1] or NULL.  Asynchronous. */
int dbw_dtur_b(dbw_ctx *ctx, const float *resp_times, int32_t *b_out, float *theta_out, void *stream);

/* dbw_dtur_b followed by dbw_select with the backup counts it wrote (Algorithm 2, then
 * Section 2.2), as one call: the same state change, the same outputs.  For graphs of up to
 * 256 workers whose rows have at most 64 neighbours it is a single launch; otherwise the two
 * launches of the separate calls.  resp_times [dev, N], b_out [dev, N] (required),
 * theta_out [dev, 1] or NULL.  Asynchronous. */
int dbw_dtur_select(dbw_ctx *ctx, const float *resp_times, int32_t *b_out, float *theta_out, void *stream);
/* Empty the visited set: the next dbw_dtur_b starts a fresh epoch.  Asynchronous on `stream`. */
int dbw_dtur_reset(dbw_ctx *ctx, void *stream);
/* The epoch state of the threshold rule, for checkpoint and resume (everything else a run needs
 * to resume is caller-owned: parameters, round number).  visited [host, N-1] uint8: 1 for the
 * links of the link set already visited in the current epoch; n_visited [host, 1] / value: their
 * number (N - 1 with every link marked = the epoch is complete, the next call starts a new one).
 * dbw_dtur_set_state checks that the two agree (DBW_ERR_INVALID).  Both synchronise the stream. */
int dbw_dtur_get_state(dbw_ctx *ctx, uint8_t *visited, int32_t *n_visited, void *stream);
int dbw_dtur_set_state(dbw_ctx *ctx, const uint8_t *visited, int32_t n_visited, void *stream);

/* Copy out the last selection: p [dev, N] int32 (number of neighbours waited for),
 * mask [dev, nnz] uint8 aligned with colidx (1 = selected), wait_time [dev, N] float
 * (T_i = max(t_i, max over selected t_j), Section 3.2.2); each may be NULL.
 * Synchronises the stream and returns DBW_ERR_INVALID if the last dbw_select saw an
 * out-of-range b_i. */
int dbw_get_selection(dbw_ctx *ctx, int32_t *p, uint8_t *mask, float *wait_time, void *stream);

/* Duration of the round implied by the last selection (Section 3.2.2, T(k)):
 * T_out [dev, 2] float; T_out[0] = max over all workers i of T_i, T_out[1] = max of T_j over
 * the workers j that some worker waits for (the paper's set V'; 0 if nobody is waited
 * for).  With b = 0 this is the duration of a full-participation round, so calling
 * dbw_select twice on the same response times compares the two (Corollary 4).
 * Asynchronous on `stream`. */
int dbw_round_time(dbw_ctx *ctx, float *T_out, void *stream);

/* Write the dense consensus matrix P(k) [dev, N*N] float, row i = worker i's weights, built
 * from the last selection.  Asynchronous on `stream`. */
int dbw_get_weights(dbw_ctx *ctx, float *P, void *stream);

/* One training round for all N workers (Algorithm 1, one pass of its loop body):
 * mini-batch gradient of every worker at its own parameters (Section 2.1), masked
 * consensus average with the weights of the last dbw_select (Assumption 1, Section 2.2)
 * and the local SGD step, in the order chosen at create.
 *   params_in  [dev, N*ld]  read only
 *   params_out [dev, N*ld]  written in columns [0, d); must not overlap params_in
 *   batch_x    [dev, N*batch*in] float, batch_y [dev, N*batch] int32 labels in
 *              [0, classes) (a label outside is clamped and reported by dbw_check as
 *              DBW_ERR_INVALID): used iff the context has a model
 *   ext_grads  [dev, N*ld]: used iff the context has no model; NULL there means a
 *              gradient-free consensus round (the truncated model of Section 3.2.1)
 *   loss_out   [dev, N] float mean loss per worker, or NULL
 * Asynchronous on `stream`. */
int dbw_round(dbw_ctx *ctx, const float *params_in, float *params_out, const float *batch_x,
              const int32_t *batch_y, const float *ext_grads, float *loss_out, float lr, void *stream);

/* dbw_round with a learning rate of its own for every worker, eta [dev, N] float: eta_j(k) of
 * Section 2.1 and the diagonal matrix eta(k) of Section 2.2.  Average-then-correct order:
 * worker i subtracts eta_i g_i from its average; local-step-first order: worker j steps
 * with eta_j g_j before the averaging.  eta must stay valid until the stream work is done.
 * Everything else as dbw_round. */
int dbw_round_eta(dbw_ctx *ctx, const float *params_in, float *params_out, const float *batch_x,
                  const int32_t *batch_y, const float *ext_grads, float *loss_out, const float *eta,
                  void *stream);

/* r consecutive gradient-free rounds in one pass over the parameters: the consensus-only
 * iterations that follow the gradient phase (Section 3.2.1, the remark after the corollary on
 * the number of iterations), evaluated through the product of their consensus matrices
 * (Phi of Section 3.1): params_out = P(k+r-1) ... P(k+1) P(k) params_in in this library's
 * row convention.  resp_times [dev, r*N] and b [dev, r*N]: row q holds round q's response
 * times and backup counts, used as by dbw_select.  The result equals r times (dbw_select,
 * dbw_round with ext_grads = NULL) up to fp32 rounding; the parameters are read and written
 * once instead of r times.  Needs N <= 256, ld <= 26 843 545 and the rows layout
 * (DBW_ERR_UNSUPPORTED otherwise).  Leaves the
 * selection state of the last of the r rounds; out-of-range b is reported as by dbw_select.
 * params_out must not overlap params_in.  Asynchronous on `stream`. */
int dbw_consensus_rounds(dbw_ctx *ctx, const float *params_in, float *params_out, const float *resp_times,
                         const int32_t *b, int32_t r, void *stream);

/* dbw_consensus_rounds for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  No context and no dbw_create:
 * the graph is passed with every call, as device CSR arrays (same form as dbw_create's host
 * arrays: rowptr [dev, N+1], colidx [dev, nnz], nnz = rowptr[N] given by the host as well), and
 * all working memory (a checked copy of the graph, the selection state of each round, the product
 * of the consensus matrices) is a fixed array of about 1.7 MB inside the library's device image,
 * which every GPU the library runs on holds until the process ends.  The call allocates and frees
 * nothing, records no memset, and does not synchronise.
 *   Limits: N <= 256, nnz <= 256 * 255, ld <= 26 843 545 (DBW_ERR_UNSUPPORTED beyond them); ld = 0
 *   means d; rows layout only.
 *   params_in / params_out [dev, N*ld], resp_times [dev, r*N], b [dev, r*N]: as dbw_consensus_rounds;
 *   the result is the same, bit for bit, as that of dbw_consensus_rounds on a context of this graph.
 *   status_out [dev, 1] int32 or NULL: receives DBW_OK, DBW_ERR_GRAPH (the graph is checked on the
 *   device for everything dbw_create checks except connectivity; a graph that fails is treated
 *   as the graph without links, so params_out = params_in) or DBW_ERR_INVALID (some b_i outside
 *   [0, deg_i], clamped as by dbw_select) when the stream work has run.
 * All calls on one GPU share the one array, which keeps the previous call's contents (the call
 * itself clears what must start at zero): calls that overlap in time on one GPU, on whatever
 * streams, race with each other.  Asynchronous on `stream`. */
int dbw_consensus_rounds_static(int32_t N, int64_t d, int64_t ld, int32_t nnz, const int32_t *rowptr,
                                const int32_t *colidx, const float *params_in, float *params_out,
                                const float *resp_times, const int32_t *b, int32_t r, int32_t *status_out,
                                void *stream);

/* Copy a [N * ld] array from one layout to the other (all ld columns): to_tiles != 0 reads src
 * in row layout and writes dst tile-major, to_tiles == 0 the reverse.  ld must be a multiple
 * of 64 and both pointers 16-byte aligned (DBW_ERR_INVALID otherwise); src and dst must not
 * overlap.  Works on any context, whatever its own layout.  Asynchronous on `stream`. */
int dbw_convert_layout(dbw_ctx *ctx, const float *src, float *dst, int32_t to_tiles, void *stream);

/* Mini-batch gradients only (the first step of dbw_round), written to grads [dev, N*ld]
 * in columns [0, d).  Needs a model.  Asynchronous. */
int dbw_grad(dbw_ctx *ctx, const float *params, const float *batch_x, const int32_t *batch_y,
             float *grads, float *loss_out, void *stream);

/* Synchronise `stream` and return the deferred device-side status, clearing it: DBW_OK,
 * DBW_ERR_INVALID (a backup count outside [0, deg_i] in dbw_select / dbw_consensus_rounds, or a
 * label outside [0, classes) in dbw_round / dbw_grad; both are clamped for memory safety and the
 * round's results are then those of the clamped values), or DBW_WARN_THETA_INF. */
int dbw_check(dbw_ctx *ctx, void *stream);

/* Link set used by dbw_dtur_b: edges [host, 2*(N-1)] int32 as (u, v) pairs in link-id
 * order.  Returns N - 1 (or a negative error). */
int dbw_get_links(dbw_ctx *ctx, int32_t *edges);

/* Which mixing path the context resolved to (DBW_MIX_CSR or DBW_MIX_DENSE). */
int dbw_mix_path(const dbw_ctx *ctx);

/* Release the context and its device memory.  NULL is a no-op returning DBW_OK.
 * Synchronises the device. */
int dbw_destroy(dbw_ctx *ctx);

const char *dbw_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DBW_H */
