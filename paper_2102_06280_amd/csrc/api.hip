// C-ABI entry points: argument validation, context life cycle, and the order in which a
// round's kernels are put on the caller's stream.  All arithmetic lives in the kernels.
#include <algorithm>
#include <cstring>
#include <new>
#include <queue>

#include "dbw_internal.h"

int dbw_validate_graph(int32_t N, const int32_t *rowptr, const int32_t *colidx)
{
    if (rowptr[0] != 0) return DBW_ERR_GRAPH;
    for (int i = 0; i < N; ++i)
        if (rowptr[i + 1] < rowptr[i]) return DBW_ERR_GRAPH;
    for (int i = 0; i < N; ++i) {
        for (int e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int j = colidx[e];
            if (j < 0 || j >= N || j == i) return DBW_ERR_GRAPH;
            if (e > rowptr[i] && colidx[e - 1] >= j) return DBW_ERR_GRAPH;
            // symmetry: i must appear in row j
            if (!std::binary_search(colidx + rowptr[j], colidx + rowptr[j + 1], i)) {
                // row j may itself be unsorted; fall back to a linear scan before deciding
                if (std::find(colidx + rowptr[j], colidx + rowptr[j + 1], i) == colidx + rowptr[j + 1])
                    return DBW_ERR_GRAPH;
            }
        }
    }
    return DBW_OK;
}

namespace {

// Breadth-first spanning tree from worker 0, neighbours in ascending index; the order of
// discovery numbers the links.  Returns false if some worker is unreachable.
bool spanning_links(int32_t N, const int32_t *rowptr, const int32_t *colidx, std::vector<int32_t> &links)
{
    std::vector<char> seen(N, 0);
    std::queue<int> q;
    q.push(0);
    seen[0] = 1;
    links.clear();
    while (!q.empty()) {
        const int u = q.front();
        q.pop();
        for (int e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            const int v = colidx[e];
            if (!seen[v]) {
                seen[v] = 1;
                links.push_back(u);
                links.push_back(v);
                q.push(v);
            }
        }
    }
    return (int)links.size() == 2 * (N - 1);
}

int64_t model_param_count(const dbw_model &m, int64_t *in_dim)
{
    if (m.kind == DBW_MODEL_MLP) {
        if (m.n_layers < 1 || m.n_layers > 8) return -1;
        int64_t n = 0;
        for (int l = 0; l <= m.n_layers; ++l)
            if (m.dims[l] < 1) return -1;
        for (int l = 0; l < m.n_layers; ++l) n += (int64_t)m.dims[l + 1] * m.dims[l] + m.dims[l + 1];
        *in_dim = m.dims[0];
        return n;
    }
    if (m.kind == DBW_MODEL_CNN) {
        const int64_t C0 = m.dims[0], H = m.dims[1], W = m.dims[2], C1 = m.dims[3], C2 = m.dims[4], K = m.dims[5],
                      F = m.dims[6], NC = m.dims[7];
        if (C0 < 1 || H < 4 || W < 4 || H % 4 || W % 4 || C1 < 1 || C2 < 1 || K < 1 || K % 2 == 0 || F < 1 || NC < 1)
            return -1;
        *in_dim = C0 * H * W;
        const int64_t flat = C2 * (H / 4) * (W / 4);
        return C1 * C0 * K * K + C1 + C2 * C1 * K * K + C2 + F * flat + F + NC * F + NC;
    }
    return -1;
}

template <typename T>
int dev_alloc(T **p, size_t n)
{
    *p = nullptr;
    if (n == 0) n = 1;
    return hipMalloc((void **)p, n * sizeof(T)) == hipSuccess ? DBW_OK : DBW_ERR_ALLOC;
}

void free_ctx(dbw_ctx *c)
{
    if (!c) return;
    void *ptrs[] = {c->rowptr, c->colidx, c->p, c->mask, c->wait, c->listed, c->sel_idx, c->sel_w, c->self_w, c->Wdense,
                    c->phi[0], c->phi[1], c->phi_frag,
                    c->err, c->links, c->visited, c->n_visited, c->grads, c->act, c->loss_part, c->loss_ticket};
    for (void *q : ptrs)
        if (q) (void)hipFree(q);
    for (auto &sl : c->slots) {
        (void)hipEventDestroy(sl.start);
        (void)hipEventDestroy(sl.stop);
    }
    for (auto e : c->free_events) (void)hipEventDestroy(e);
    delete c;
}

bool overlaps(const void *a, size_t na, const void *b, size_t nb)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

// Everything of dbw_create after the graph has been validated; the caller frees `c` on any
// error return (host containers may throw: the caller turns that into DBW_ERR_ALLOC).
int fill_ctx(dbw_ctx *c, int32_t N, int64_t d, int64_t nnz64, const int32_t *rowptr, const int32_t *colidx,
             const dbw_opts *opts)
{
    c->N = N;
    c->d = d;
    c->ld = d;
    c->nnz = (int32_t)nnz64;
    if (opts) {
        if (opts->ld != 0) c->ld = opts->ld;
        c->order = opts->order;
        c->mix = opts->mix_path;
        c->layout = opts->layout;
        c->model = opts->model;
        if (c->model.kind == DBW_MODEL_SOFTMAX) {       // multinomial logistic regression dims[0] -> dims[1]
            c->model.kind = DBW_MODEL_MLP;
            c->model.n_layers = 1;
        }
    }
    if (c->ld < d || (c->order != DBW_ORDER_CTA && c->order != DBW_ORDER_ATC) || c->mix < DBW_MIX_AUTO ||
        c->mix > DBW_MIX_DENSE)
        return DBW_ERR_INVALID;
    if (c->layout != DBW_LAYOUT_ROWS && c->layout != DBW_LAYOUT_TILES) return DBW_ERR_INVALID;
    if (c->layout == DBW_LAYOUT_TILES) {
        if (c->ld % DBW_TILE_COLUMNS) return DBW_ERR_INVALID;
        if (c->model.kind != DBW_MODEL_NONE || N > DBW_TILES_MAX_N || c->mix == DBW_MIX_DENSE)
            return DBW_ERR_UNSUPPORTED;
        c->mix = DBW_MIX_CSR;
    }
    if (c->model.kind != DBW_MODEL_NONE) {
        const int64_t want = model_param_count(c->model, &c->in_dim);
        const bool loss_ok = c->model.loss == DBW_LOSS_XENT ||
                             (c->model.loss == DBW_LOSS_MSE && c->model.kind == DBW_MODEL_MLP);
        if (want != d || c->model.batch < 1 || !loss_ok) return DBW_ERR_INVALID;
        if (c->model.grad_path < DBW_GRAD_AUTO || c->model.grad_path > DBW_GRAD_CHAIN) return DBW_ERR_INVALID;
        if (c->model.grad_path == DBW_GRAD_CHAIN &&
            (c->model.kind != DBW_MODEL_MLP || !dbw_fc_chain_shape_ok(c->model.n_layers, c->model.dims, c->model.batch, N)))
            return DBW_ERR_UNSUPPORTED;
    }
    c->h_rowptr.assign(rowptr, rowptr + N + 1);
    c->h_colidx.assign(colidx, colidx + c->nnz);
    for (int i = 0; i < N; ++i) c->max_deg = std::max(c->max_deg, rowptr[i + 1] - rowptr[i]);
    if (!spanning_links(N, rowptr, colidx, c->h_links)) return DBW_ERR_GRAPH;
    const bool dense_fits = N <= DBW_DENSE_MAX_N && c->ld <= DBW_DENSE_MAX_LD;
    if (c->mix == DBW_MIX_AUTO)
        c->mix = (dense_fits && (int64_t)c->nnz * 4 > (int64_t)N * N) ? DBW_MIX_DENSE : DBW_MIX_CSR;
    if (c->mix == DBW_MIX_DENSE && !dense_fits) return DBW_ERR_UNSUPPORTED;
    c->Npad = 32;                                   // dense path: padded to a power of two
    while (c->Npad < N) c->Npad *= 2;

    int rc = DBW_OK;
    auto A = [&](int r) { if (rc == DBW_OK) rc = r; };
    A(dev_alloc(&c->rowptr, (size_t)N + 1));
    A(dev_alloc(&c->colidx, (size_t)c->nnz));
    A(dev_alloc(&c->p, (size_t)N));
    A(dev_alloc(&c->mask, (size_t)c->nnz));
    A(dev_alloc(&c->wait, (size_t)N));
    A(dev_alloc(&c->listed, (size_t)N));
    A(dev_alloc(&c->sel_idx, (size_t)c->nnz));
    A(dev_alloc(&c->sel_w, (size_t)c->nnz));
    A(dev_alloc(&c->self_w, (size_t)N));
    A(dev_alloc(&c->err, 1));
    A(dev_alloc(&c->links, c->h_links.size()));
    A(dev_alloc(&c->visited, (size_t)std::max(N - 1, 1)));
    A(dev_alloc(&c->n_visited, 1));
    if (c->mix == DBW_MIX_DENSE) A(dev_alloc(&c->Wdense, (size_t)c->Npad * c->Npad));
    if (N <= DBW_DENSE_MAX_N) {
        A(dev_alloc(&c->phi[0], (size_t)c->Npad * c->Npad));
        A(dev_alloc(&c->phi[1], (size_t)c->Npad * c->Npad));
        A(dev_alloc(&c->phi_frag, (size_t)c->Npad * c->Npad));
    }
    if (c->model.kind != DBW_MODEL_NONE) {
        A(dbw_fc_prepare());
        A(dev_alloc(&c->grads, (size_t)N * c->ld));
        c->act_floats = c->model.kind == DBW_MODEL_MLP ? dbw_mlp_scratch_floats(c) : dbw_cnn_scratch_floats(c);
        A(dev_alloc(&c->act, c->act_floats));
        A(dev_alloc(&c->loss_part, (size_t)N * DBW_LOSS_CHUNKS));
        A(dev_alloc(&c->loss_ticket, (size_t)N));
    }
    if (rc != DBW_OK) return rc;
    auto H = [&](hipError_t e) { if (rc == DBW_OK && e != hipSuccess) rc = DBW_ERR_HIP; };
    H(hipMemcpy(c->rowptr, rowptr, sizeof(int32_t) * ((size_t)N + 1), hipMemcpyHostToDevice));
    if (c->nnz) H(hipMemcpy(c->colidx, colidx, sizeof(int32_t) * (size_t)c->nnz, hipMemcpyHostToDevice));
    if (!c->h_links.empty())
        H(hipMemcpy(c->links, c->h_links.data(), sizeof(int32_t) * c->h_links.size(), hipMemcpyHostToDevice));
    H(hipMemset(c->err, 0, sizeof(int32_t)));
    H(hipMemset(c->visited, 0, (size_t)std::max(N - 1, 1)));
    H(hipMemset(c->n_visited, 0, sizeof(int32_t)));
    if (c->Wdense) H(hipMemset(c->Wdense, 0, sizeof(float) * (size_t)c->Npad * c->Npad));
    if (c->grads) H(hipMemset(c->grads, 0, sizeof(float) * (size_t)N * c->ld));
    // Scratch starts as NaN (all bits set), so that a kernel reading a value no kernel wrote shows
    // up in every result instead of depending on what the allocation happened to hold.
    if (c->act) H(hipMemset(c->act, 0xFF, sizeof(float) * c->act_floats));
    if (c->loss_ticket) H(hipMemset(c->loss_ticket, 0, sizeof(uint32_t) * (size_t)N));
    H(hipDeviceSynchronize());
    return rc;
}

}  // namespace

dbw_timer::dbw_timer(dbw_ctx *ctx, const char *name, hipStream_t st) : c(ctx), s(st)
{
    if (!c->timing) return;
    hipEvent_t ev[2];
    for (auto &e : ev) {
        if (!c->free_events.empty()) {
            e = c->free_events.back();
            c->free_events.pop_back();
        } else if (hipEventCreate(&e) != hipSuccess) {
            return;
        }
    }
    (void)hipEventRecord(ev[0], s);
    stop = ev[1];
    c->slots.push_back({name, ev[0], ev[1]});
}

dbw_timer::~dbw_timer()
{
    if (stop) (void)hipEventRecord(stop, s);
}

extern "C" {

int dbw_create(dbw_ctx **out, int32_t N, int64_t d, const int32_t *rowptr, const int32_t *colidx,
               const dbw_opts *opts)
{
    if (!out || !rowptr) return DBW_ERR_NULL;
    *out = nullptr;
    if (N < 1 || d < 1) return DBW_ERR_INVALID;
    const int64_t nnz64 = rowptr[N];
    if (nnz64 < 0) return DBW_ERR_GRAPH;
    if (nnz64 > 0 && !colidx) return DBW_ERR_NULL;
    int rc = dbw_validate_graph(N, rowptr, colidx);
    if (rc != DBW_OK) return rc;

    dbw_ctx *c = new (std::nothrow) dbw_ctx();
    if (!c) return DBW_ERR_ALLOC;
    try {
        rc = fill_ctx(c, N, d, nnz64, rowptr, colidx, opts);
    } catch (const std::bad_alloc &) {
        rc = DBW_ERR_ALLOC;
    }
    if (rc != DBW_OK) {
        free_ctx(c);
        return rc;
    }
    *out = c;
    return DBW_OK;
}

int dbw_select(dbw_ctx *c, const float *resp_times, const int32_t *b, void *stream)
{
    if (!c || !resp_times || !b) return DBW_ERR_NULL;
    const int rc = dbw_launch_select(c, resp_times, b, (hipStream_t)stream);
    if (rc == DBW_OK) c->selected = true;
    return rc;
}

int dbw_dtur_b(dbw_ctx *c, const float *resp_times, int32_t *b_out, float *theta_out, void *stream)
{
    if (!c || !resp_times || !b_out) return DBW_ERR_NULL;
    return dbw_launch_dtur(c, resp_times, b_out, theta_out, (hipStream_t)stream);
}

int dbw_dtur_select(dbw_ctx *c, const float *resp_times, int32_t *b_out, float *theta_out, void *stream)
{
    if (!c || !resp_times || !b_out) return DBW_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    int rc;
    if (dbw_fused_dtur_select_fits(c)) {
        rc = dbw_launch_dtur_select(c, resp_times, b_out, theta_out, s);
    } else {
        rc = dbw_launch_dtur(c, resp_times, b_out, theta_out, s);
        if (rc == DBW_OK) rc = dbw_launch_select(c, resp_times, b_out, s);
    }
    if (rc == DBW_OK) c->selected = true;
    return rc;
}

int dbw_dtur_reset(dbw_ctx *c, void *stream)
{
    if (!c) return DBW_ERR_NULL;
    return dbw_launch_dtur_reset(c, (hipStream_t)stream);
}

int dbw_dtur_get_state(dbw_ctx *c, uint8_t *visited, int32_t *n_visited, void *stream)
{
    if (!c || !visited || !n_visited) return DBW_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (c->N > 1) DBW_HIP(hipMemcpyAsync(visited, c->visited, (size_t)(c->N - 1), hipMemcpyDeviceToHost, s));
    DBW_HIP(hipMemcpyAsync(n_visited, c->n_visited, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    DBW_HIP(hipStreamSynchronize(s));
    return DBW_OK;
}

int dbw_dtur_set_state(dbw_ctx *c, const uint8_t *visited, int32_t n_visited, void *stream)
{
    if (!c || !visited) return DBW_ERR_NULL;
    int count = 0;
    for (int e = 0; e < c->N - 1; ++e) {
        if (visited[e] > 1) return DBW_ERR_INVALID;
        count += visited[e];
    }
    // n_visited = N - 1 with every link marked is the state after a completed epoch
    if (n_visited != count) return DBW_ERR_INVALID;
    hipStream_t s = (hipStream_t)stream;
    if (c->N > 1) DBW_HIP(hipMemcpyAsync(c->visited, visited, (size_t)(c->N - 1), hipMemcpyHostToDevice, s));
    DBW_HIP(hipMemcpyAsync(c->n_visited, &n_visited, sizeof(int32_t), hipMemcpyHostToDevice, s));
    DBW_HIP(hipStreamSynchronize(s));
    return DBW_OK;
}

int dbw_check(dbw_ctx *c, void *stream)
{
    if (!c) return DBW_ERR_NULL;
    int32_t e = 0;
    DBW_HIP(hipMemcpyAsync(&e, c->err, sizeof(int32_t), hipMemcpyDeviceToHost, (hipStream_t)stream));
    DBW_HIP(hipStreamSynchronize((hipStream_t)stream));
    if (e != 0) {
        DBW_HIP(hipMemsetAsync(c->err, 0, sizeof(int32_t), (hipStream_t)stream));
        DBW_HIP(hipStreamSynchronize((hipStream_t)stream));
    }
    return e;
}

int dbw_get_selection(dbw_ctx *c, int32_t *p, uint8_t *mask, float *wait_time, void *stream)
{
    if (!c) return DBW_ERR_NULL;
    if (!c->selected) return DBW_ERR_STATE;
    hipStream_t s = (hipStream_t)stream;
    if (p) DBW_HIP(hipMemcpyAsync(p, c->p, sizeof(int32_t) * (size_t)c->N, hipMemcpyDeviceToDevice, s));
    if (mask && c->nnz) DBW_HIP(hipMemcpyAsync(mask, c->mask, (size_t)c->nnz, hipMemcpyDeviceToDevice, s));
    if (wait_time) DBW_HIP(hipMemcpyAsync(wait_time, c->wait, sizeof(float) * (size_t)c->N, hipMemcpyDeviceToDevice, s));
    return dbw_check(c, stream);
}

int dbw_round_time(dbw_ctx *c, float *T_out, void *stream)
{
    if (!c || !T_out) return DBW_ERR_NULL;
    if (!c->selected) return DBW_ERR_STATE;
    return dbw_launch_round_time(c, T_out, (hipStream_t)stream);
}

int dbw_get_weights(dbw_ctx *c, float *P, void *stream)
{
    if (!c || !P) return DBW_ERR_NULL;
    if (!c->selected) return DBW_ERR_STATE;
    return dbw_launch_dense_weights(c, P, (hipStream_t)stream);
}

int dbw_grad(dbw_ctx *c, const float *params, const float *batch_x, const int32_t *batch_y, float *grads,
             float *loss_out, void *stream)
{
    if (!c || !params || !batch_x || !batch_y || !grads) return DBW_ERR_NULL;
    if (c->model.kind == DBW_MODEL_MLP)
        return dbw_launch_grad_mlp(c, params, batch_x, batch_y, grads, loss_out, (hipStream_t)stream);
    if (c->model.kind == DBW_MODEL_CNN)
        return dbw_launch_grad_cnn(c, params, batch_x, batch_y, grads, loss_out, (hipStream_t)stream);
    return DBW_ERR_STATE;
}

static int round_impl(dbw_ctx *c, const float *params_in, float *params_out, const float *batch_x,
                      const int32_t *batch_y, const float *ext_grads, float *loss_out, float lr, const float *lr_vec,
                      void *stream)
{
    if (!c || !params_in || !params_out) return DBW_ERR_NULL;
    if (!c->selected) return DBW_ERR_STATE;
    const size_t bytes = sizeof(float) * (size_t)c->N * (size_t)c->ld;
    if (overlaps(params_in, bytes, params_out, bytes)) return DBW_ERR_ALIAS;
    hipStream_t s = (hipStream_t)stream;
    const float *g = ext_grads;
    if (c->model.kind != DBW_MODEL_NONE) {
        const int rc = dbw_grad(c, params_in, batch_x, batch_y, c->grads, loss_out, stream);
        if (rc != DBW_OK) return rc;
        g = c->grads;
    } else if (g && overlaps(g, bytes, params_out, bytes)) {
        return DBW_ERR_ALIAS;
    }
    if (c->layout == DBW_LAYOUT_TILES) return dbw_launch_mix_tiles(c, params_in, g, params_out, lr, lr_vec, s);
    if (c->mix == DBW_MIX_DENSE) return dbw_launch_mix_dense(c, params_in, g, params_out, lr, lr_vec, s);
    return dbw_launch_mix_csr(c, params_in, g, params_out, lr, lr_vec, s);
}

int dbw_convert_layout(dbw_ctx *c, const float *src, float *dst, int32_t to_tiles, void *stream)
{
    if (!c || !src || !dst) return DBW_ERR_NULL;
    if (c->ld % DBW_TILE_COLUMNS || (uintptr_t)src % 16 || (uintptr_t)dst % 16) return DBW_ERR_INVALID;
    const size_t bytes = sizeof(float) * (size_t)c->N * (size_t)c->ld;
    if (overlaps(src, bytes, dst, bytes)) return DBW_ERR_ALIAS;
    return dbw_launch_layout_convert(c, src, dst, to_tiles != 0, (hipStream_t)stream);
}

int dbw_round(dbw_ctx *c, const float *params_in, float *params_out, const float *batch_x,
              const int32_t *batch_y, const float *ext_grads, float *loss_out, float lr, void *stream)
{
    return round_impl(c, params_in, params_out, batch_x, batch_y, ext_grads, loss_out, lr, nullptr, stream);
}

int dbw_round_eta(dbw_ctx *c, const float *params_in, float *params_out, const float *batch_x,
                  const int32_t *batch_y, const float *ext_grads, float *loss_out, const float *eta, void *stream)
{
    if (!eta) return DBW_ERR_NULL;
    return round_impl(c, params_in, params_out, batch_x, batch_y, ext_grads, loss_out, 0.f, eta, stream);
}

int dbw_consensus_rounds(dbw_ctx *c, const float *params_in, float *params_out, const float *resp_times,
                         const int32_t *b, int32_t r, void *stream)
{
    if (!c || !params_in || !params_out || !resp_times || !b) return DBW_ERR_NULL;
    if (r < 1) return DBW_ERR_INVALID;
    if (c->N > DBW_DENSE_MAX_N || c->ld > DBW_DENSE_MAX_LD || c->layout != DBW_LAYOUT_ROWS)
        return DBW_ERR_UNSUPPORTED;
    const size_t bytes = sizeof(float) * (size_t)c->N * (size_t)c->ld;
    if (overlaps(params_in, bytes, params_out, bytes)) return DBW_ERR_ALIAS;
    const int rc = dbw_launch_consensus_rounds(c, params_in, params_out, resp_times, b, r, (hipStream_t)stream);
    if (rc == DBW_OK) c->selected = true;
    return rc;
}

int dbw_get_links(dbw_ctx *c, int32_t *edges)
{
    if (!c || !edges) return DBW_ERR_NULL;
    std::memcpy(edges, c->h_links.data(), sizeof(int32_t) * c->h_links.size());
    return c->N - 1;
}

int dbw_mix_path(const dbw_ctx *c) { return c ? c->mix : DBW_ERR_NULL; }

int dbw_destroy(dbw_ctx *c)
{
    if (!c) return DBW_OK;
    (void)hipDeviceSynchronize();
    free_ctx(c);
    return DBW_OK;
}

const char *dbw_strerror(int code)
{
    switch (code) {
    case DBW_OK: return "ok";
    case DBW_ERR_NULL: return "required pointer is NULL";
    case DBW_ERR_INVALID: return "invalid argument (N, d, ld, model, or b_i outside [0, deg_i])";
    case DBW_ERR_GRAPH: return "graph must be CSR, sorted, symmetric, loop-free and connected";
    case DBW_ERR_ALIAS: return "params_in / gradients overlap params_out";
    case DBW_ERR_STATE: return "call out of order (dbw_select first; model needed for dbw_grad)";
    case DBW_ERR_ALLOC: return "allocation failed";
    case DBW_ERR_HIP: return "HIP call failed";
    case DBW_ERR_UNSUPPORTED: return "combination not supported";
    case DBW_WARN_THETA_INF: return "warning: threshold rule found no link that can be established (theta = +inf)";
    default: return "unknown error";
    }
}

int dbw_set_timing(dbw_ctx *c, int32_t on)
{
    if (!c) return DBW_ERR_NULL;
    (void)hipDeviceSynchronize();
    for (auto &sl : c->slots) {
        c->free_events.push_back(sl.start);
        c->free_events.push_back(sl.stop);
    }
    c->slots.clear();
    c->timing = on != 0;
    return DBW_OK;
}

int dbw_get_timing(dbw_ctx *c, dbw_kernel_time *out, int32_t cap)
{
    if (!c || (!out && cap > 0)) return DBW_ERR_NULL;
    DBW_HIP(hipDeviceSynchronize());
    int n = 0;
    for (auto &sl : c->slots) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sl.start, sl.stop) != hipSuccess) continue;
        int k = 0;
        for (; k < n; ++k)
            if (std::strcmp(out[k].name, sl.name) == 0) break;
        if (k == n) {
            if (n >= cap) continue;
            out[n++] = {sl.name, 0.0, 0};
        }
        out[k].ms_total += ms;
        out[k].launches += 1;
    }
    return n;
}

}  // extern "C"
