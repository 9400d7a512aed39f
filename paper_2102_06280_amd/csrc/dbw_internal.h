// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "dbw.h"
#include "dbw_measure.h"

#define DBW_HIP(call)                                   \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) return DBW_ERR_HIP;       \
    } while (0)

constexpr int DBW_DENSE_MAX_N = 256;   // the dense mixing kernel keeps all of P(k) in registers
// the dense mixing kernel adds 32-bit per-lane byte offsets of up to 40 rows to 64-bit uniform bases
constexpr int64_t DBW_DENSE_MAX_LD = (int64_t)UINT32_MAX / (40 * 4);
constexpr int DBW_SELECT_LDS_KEYS = 2048;
constexpr int DBW_FUSED_SELECT_MAX_N = 256;   // threshold rule + selection in one workgroup up to this many workers
constexpr int DBW_LOSS_CHUNKS = 16;     // workgroups per worker in the loss kernel, at most
constexpr int DBW_TILES_MAX_N = 256;   // the tile-major mixing kernel holds one 256-byte piece per worker in LDS

struct dbw_timing_slot {
    const char *name;
    hipEvent_t start, stop;
};

struct dbw_ctx {
    int32_t N = 0;
    int64_t d = 0, ld = 0;
    int32_t nnz = 0, max_deg = 0;
    int32_t order = DBW_ORDER_CTA;
    int32_t mix = DBW_MIX_CSR;
    int32_t layout = DBW_LAYOUT_ROWS;
    int32_t Npad = 0;                 // N rounded up to a power of two >= 32 (dense path)
    dbw_model model{};
    int64_t in_dim = 0;               // floats per sample
    bool selected = false;

    std::vector<int32_t> h_rowptr, h_colidx, h_links;

    // device: graph
    int32_t *rowptr = nullptr, *colidx = nullptr;
    // device: selection state of the current round
    int32_t *p = nullptr;             // [N]
    uint8_t *mask = nullptr;          // [nnz]
    float *wait = nullptr;            // [N]
    uint8_t *listed = nullptr;        // [N] scratch of the round-time kernel
    int32_t *sel_idx = nullptr;       // [nnz] row i: first p_i entries = selected neighbours, ascending
    float *sel_w = nullptr;           // [nnz] their weights
    float *self_w = nullptr;          // [N]
    float *Wdense = nullptr;          // [Npad*Npad] in MFMA A-fragment order (dense path only)
    float *phi[2] = {nullptr, nullptr};   // [Npad*Npad] running product of consensus matrices (N <= 256)
    float *phi_frag = nullptr;        // the product in MFMA A-fragment order
    int32_t *err = nullptr;           // [1] deferred status
    // device: threshold rule
    int32_t *links = nullptr;         // [2*(N-1)]
    uint8_t *visited = nullptr;       // [N-1]
    int32_t *n_visited = nullptr;     // [1]
    // device: model scratch
    float *grads = nullptr;           // [N*ld] when a model is attached
    float *act = nullptr;             // activations / deltas
    float *loss_part = nullptr;       // [N][DBW_LOSS_CHUNKS] partial loss sums of the loss kernel
    uint32_t *loss_ticket = nullptr;  // [N] arrival counters of the loss kernel, zero between launches
    size_t act_floats = 0;

    // timing
    bool timing = false;
    std::vector<dbw_timing_slot> slots;
    std::vector<hipEvent_t> free_events;
};

struct dbw_timer {
    dbw_ctx *c;
    hipStream_t s;
    hipEvent_t stop = nullptr;
    dbw_timer(dbw_ctx *ctx, const char *name, hipStream_t st);
    ~dbw_timer();
};

// api.hip: CSR rows strictly ascending, in range, loop-free, symmetric (DBW_ERR_GRAPH otherwise)
int dbw_validate_graph(int32_t N, const int32_t *rowptr, const int32_t *colidx);
// select.hip
int dbw_launch_select(dbw_ctx *c, const float *t, const int32_t *b, hipStream_t s);
int dbw_launch_round_time(dbw_ctx *c, float *out, hipStream_t s);
int dbw_launch_dtur(dbw_ctx *c, const float *t, int32_t *b_out, float *theta_out, hipStream_t s);
bool dbw_fused_dtur_select_fits(const dbw_ctx *c);
int dbw_launch_dtur_select(dbw_ctx *c, const float *t, int32_t *b_out, float *theta_out, hipStream_t s);
int dbw_launch_dtur_reset(dbw_ctx *c, hipStream_t s);
int dbw_launch_dense_weights(dbw_ctx *c, float *P, hipStream_t s);
// mix_csr.hip
// Learning rate of a round as the mixing kernels see it: one value for all workers, or
// eta_j per worker read from device memory (Section 2.1).
struct dbw_lr_scalar {
    float v;
    __device__ __forceinline__ float at(int) const { return v; }
};
struct dbw_lr_vector {
    const float *v;
    __device__ __forceinline__ float at(int j) const { return v[j]; }
};

// lr_vec (device, N) overrides lr when it is not null.
int dbw_launch_mix_csr(dbw_ctx *c, const float *x, const float *g, float *out, float lr, const float *lr_vec,
                       hipStream_t s);
// mix_dense.hip
// Columns [0, dbw_dense_columns) are the ones the matrix-core kernel covers (0 when rows are not
// 16-byte aligned).  W (A-fragment order, Npad x Npad) defaults to the matrix of the last
// selection; with a W of the caller's the remaining columns are left to the caller.
int64_t dbw_dense_columns(const dbw_ctx *c, const float *x, const float *g, const float *out);
int dbw_launch_mix_dense(dbw_ctx *c, const float *x, const float *g, float *out, float lr, const float *lr_vec,
                         hipStream_t s, const float *W = nullptr);
// mix_tiles.hip (tile-major layout)
int dbw_launch_mix_tiles(dbw_ctx *c, const float *x, const float *g, float *out, float lr, const float *lr_vec,
                         hipStream_t s);
int dbw_launch_layout_convert(dbw_ctx *c, const float *src, float *dst, int to_tiles, hipStream_t s);
// consensus.hip
int dbw_launch_consensus_rounds(dbw_ctx *c, const float *x, float *out, const float *t, const int32_t *b, int r,
                                hipStream_t s);
// grad_mlp.hip / grad_cnn.hip
// A stack of fully connected layers dims[0] -> ... -> dims[L] with ReLU between layers and
// softmax cross-entropy on top, for all workers.  Parameters of the stack start at float
// offset param_off inside each worker's row (row stride c->ld); gradients go to the same
// offsets of `grads`.  `in` is the stack's input [B][in_ld] per worker; `act` is scratch of
// act_stride floats per worker (see dbw_fc_scratch_per_worker); `din`, if not null,
// receives the gradient with respect to the input.
struct dbw_fc_args {
    int L, B, loss_kind;
    const int32_t *dims;
    const float *params;
    float *grads;
    int64_t param_off;
    const float *in;
    int64_t in_ld, in_stride;
    float *act;
    int64_t act_stride;
    float *din;
    int64_t din_ld, din_stride;
    const int32_t *y;
    float *loss;
    int grad_path;          // DBW_GRAD_*
};
int64_t dbw_fc_scratch_per_worker(int L, const int32_t *dims, int B);
bool dbw_fc_chain_shape_ok(int L, const int32_t *dims, int B, int workers);   // DBW_GRAD_CHAIN can take this model
int dbw_fc_prepare();   // one-time kernel attributes of the fully connected path
int dbw_fc_forward_backward(dbw_ctx *c, const dbw_fc_args &a, hipStream_t s);
size_t dbw_mlp_scratch_floats(const dbw_ctx *c);
int dbw_launch_grad_mlp(dbw_ctx *c, const float *params, const float *bx, const int32_t *by, float *grads,
                        float *loss, hipStream_t s);
size_t dbw_cnn_scratch_floats(const dbw_ctx *c);
int dbw_launch_grad_cnn(dbw_ctx *c, const float *params, const float *bx, const int32_t *by, float *grads,
                        float *loss, hipStream_t s);
