/*
 * CPU oracle for one training round of consensus SGD with dynamic backup workers.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker that the GPU library is compared
 * against; it is never part of the product path and shares no code with it.  Everything
 * is written directly from the paper's definitions, slowly and plainly: double-precision
 * accumulation, results rounded to float only when stored, no blocking, no fusion.
 *
 * What each function follows:
 *   orc_select         Section 1 ("Dynamic Backup Workers": wait for the fastest p_j
 *                      neighbours, the other b_j = n_j - p_j are backups), Section 2.2
 *                      (sets S_j(k), B_j(k)), Section 3.2.2 (wait time T_j(k)).
 *   orc_round_time     Section 3.2.2 (duration T(k) of a round).
 *   orc_weights        Assumption 1 (Metropolis weights on the time-varying graph).
 *   orc_dense_P        the same weights laid out as the N x N consensus matrix P(k).
 *   orc_round          Section 2.1, the full-participation update (average, then correct
 *                      with the gradient taken at the pre-average point) and Section 2.2,
 *                      the local update followed by the partial consensus update (local
 *                      step first, then average the stepped parameters).
 *   orc_round_eta      the same with a learning rate per worker (eta_j(k), Sections 2.1, 2.2).
 *   orc_spanning_tree  Section 4.1: the link set P that connects all nodes, length d.
 *   orc_dtur           Section 4.1: threshold rule and the d-iteration procedure (Alg. 2).
 *   orc_grad_mlp       Section 2.1, the mini-batch stochastic gradient, for fully connected models
 *                      with the cross-entropy loss of Section 5.
 *   orc_grad_cnn       the same for a two-convolution network on 3 x 32 x 32 inputs.
 *   orc_decision /     diagnostics for the tests, not part of the method: which ReLU / pooling
 *   orc_branch         decisions of a gradient lie within rounding of turning (where the gradient
 *                      of Section 2.1 is not unique), and the gradient with such decisions turned.
 *
 * Pins (tests/test_oracle_*.py): brute force over all neighbour subsets, Metropolis
 * invariants, b = 0 reduction to full participation with static Metropolis-Hastings
 * weights, closed forms on ring / regular / complete graphs, the worker-mean recursion,
 * the unrolled product recursion, consensus limit, threshold-rule connectivity,
 * finite differences and PyTorch-CPU autograd for the gradients (also with forced branches),
 * NumPy recomputation of the listed near decisions.  No function here is "parity unpinned".
 *
 * Conventions: worker i's vector is row i of a row-major [N][ld] float array, d <= ld.
 * The graph is CSR without self loops; deg_i = rowptr[i+1] - rowptr[i].
 * mask is aligned with colidx: mask[e] = 1 iff colidx[e] is in S_i for the row i of e.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Threads for the loops over workers (the only parallelism here); 1 unless a timing run
 * asks for more. */
static int orc_threads = 1;
void orc_set_threads(int n) { orc_threads = n > 0 ? n : 1; }
int orc_get_threads(void) { return orc_threads; }

#define ORC_OK 0
#define ORC_ERR_INVALID (-2)
#define ORC_ERR_GRAPH (-3)

/* Response times order as (t, index) pairs under IEEE comparison; NaN counts as +inf,
 * and -0.0 == +0.0 so such a pair ties and the lower index goes first. */
static float canon_time(float t) { return isnan(t) ? INFINITY : t; }

static int key_before(float ta, int a, float tb, int b)
{
    return ta < tb || (ta == tb && a < b);
}

int orc_select(int N, const int32_t *rowptr, const int32_t *colidx, const float *t,
               const int32_t *b, uint8_t *mask, int32_t *p, float *wait /* nullable */)
{
    for (int i = 0; i < N; ++i) {
        int deg = rowptr[i + 1] - rowptr[i];
        if (b[i] < 0 || b[i] > deg) return ORC_ERR_INVALID;
    }
    for (int i = 0; i < N; ++i) {
        int beg = rowptr[i], deg = rowptr[i + 1] - beg;
        int pi = deg - b[i];
        p[i] = pi;
        int *order = (int *)malloc(sizeof(int) * (size_t)(deg > 0 ? deg : 1));
        for (int k = 0; k < deg; ++k) order[k] = beg + k;
        /* insertion sort of the row's edge positions by the neighbour's (time, index) */
        for (int k = 1; k < deg; ++k) {
            int e = order[k], m = k;
            while (m > 0 && key_before(canon_time(t[colidx[e]]), colidx[e],
                                       canon_time(t[colidx[order[m - 1]]]), colidx[order[m - 1]])) {
                order[m] = order[m - 1];
                --m;
            }
            order[m] = e;
        }
        float w = canon_time(t[i]); /* a worker cannot finish before its own gradient */
        for (int k = 0; k < deg; ++k) {
            mask[order[k]] = (uint8_t)(k < pi);
            if (k < pi && canon_time(t[colidx[order[k]]]) > w) w = canon_time(t[colidx[order[k]]]);
        }
        if (wait) wait[i] = w;
        free(order);
    }
    return ORC_OK;
}

/* Duration of the round (Section 3.2.2): out[0] = max over all workers of their wait time
 * T_i; out[1] = the paper's literal T(k), the max of T_j over the workers j that appear in
 * some worker's selected set (0 when nobody is waited for). */
void orc_round_time(int N, const int32_t *rowptr, const int32_t *colidx, const uint8_t *mask,
                    const float *wait, float *out)
{
    uint8_t *listed = (uint8_t *)calloc((size_t)N, 1);
    for (int e = 0; e < rowptr[N]; ++e)
        if (mask[e]) listed[colidx[e]] = 1;
    float all = 0.0f, sel = 0.0f;
    for (int i = 0; i < N; ++i) {
        if (wait[i] > all) all = wait[i];
        if (listed[i] && wait[i] > sel) sel = wait[i];
    }
    out[0] = all;
    out[1] = sel;
    free(listed);
}

/* Assumption 1: P_ij = 1 / (1 + max(p_i, p_j)) for j in S_i, P_ii = 1 - sum_j P_ij. */
void orc_weights(int N, const int32_t *rowptr, const int32_t *colidx, const uint8_t *mask,
                 const int32_t *p, double *w_edge /* nnz */, double *w_self /* N */)
{
    for (int i = 0; i < N; ++i) {
        double s = 0.0;
        for (int e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int j = colidx[e];
            w_edge[e] = 0.0;
            if (mask[e]) {
                int m = p[i] > p[j] ? p[i] : p[j];
                w_edge[e] = 1.0 / (1.0 + (double)m);
                s += w_edge[e];
            }
        }
        w_self[i] = 1.0 - s;
    }
}

/* Row i of P holds worker i's weights (row-stochastic by construction). */
void orc_dense_P(int N, const int32_t *rowptr, const int32_t *colidx, const uint8_t *mask,
                 const int32_t *p, double *P /* N*N row-major */)
{
    int nnz = rowptr[N];
    double *we = (double *)malloc(sizeof(double) * (size_t)(nnz > 0 ? nnz : 1));
    double *ws = (double *)malloc(sizeof(double) * (size_t)N);
    orc_weights(N, rowptr, colidx, mask, p, we, ws);
    memset(P, 0, sizeof(double) * (size_t)N * (size_t)N);
    for (int i = 0; i < N; ++i) {
        P[(size_t)i * N + i] = ws[i];
        for (int e = rowptr[i]; e < rowptr[i + 1]; ++e) P[(size_t)i * N + colidx[e]] = we[e];
    }
    free(we);
    free(ws);
}

/* One mixing + correction pass over supplied gradients (g may be NULL: gradient-free
 * consensus round).
 *   order 0: out_i = sum_j P_ij x_j - lr g_i     (Section 2.1, full-participation form)
 *   order 1: out_i = sum_j P_ij (x_j - lr g_j)   (Section 2.2, local update then consensus)
 * Columns are independent, so any column slice is an exact sub-problem. */
void orc_round(int N, int64_t d, int64_t ld, const int32_t *rowptr, const int32_t *colidx,
               const uint8_t *mask, const int32_t *p, const float *x, const float *g,
               float lr, int order, float *out)
{
    int nnz = rowptr[N];
    double *we = (double *)malloc(sizeof(double) * (size_t)(nnz > 0 ? nnz : 1));
    double *ws = (double *)malloc(sizeof(double) * (size_t)N);
    orc_weights(N, rowptr, colidx, mask, p, we, ws);
    const double eta = (double)lr;
#pragma omp parallel for schedule(static) num_threads(orc_threads)
    for (int i = 0; i < N; ++i) {
        const float *xi = x + (size_t)i * ld;
        const float *gi = g ? g + (size_t)i * ld : NULL;
        float *oi = out + (size_t)i * ld;
        for (int64_t c = 0; c < d; ++c) {
            double acc;
            if (order == 0) {
                acc = ws[i] * (double)xi[c];
                for (int e = rowptr[i]; e < rowptr[i + 1]; ++e)
                    if (mask[e]) acc += we[e] * (double)x[(size_t)colidx[e] * ld + c];
                if (gi) acc -= eta * (double)gi[c];
            } else {
                acc = ws[i] * ((double)xi[c] - (gi ? eta * (double)gi[c] : 0.0));
                for (int e = rowptr[i]; e < rowptr[i + 1]; ++e)
                    if (mask[e]) {
                        size_t o = (size_t)colidx[e] * ld + c;
                        acc += we[e] * ((double)x[o] - (g ? eta * (double)g[o] : 0.0));
                    }
            }
            oi[c] = (float)acc;
        }
    }
    free(we);
    free(ws);
}

/* The same round with a learning rate of its own for every worker, eta_j(k) of Section 2.1
 * and of the diagonal matrix eta(k) of Section 2.2.  Order 0: worker i corrects its average
 * with eta_i g_i.  Order 1: worker j steps with eta_j g_j before anybody averages. */
void orc_round_eta(int N, int64_t d, int64_t ld, const int32_t *rowptr, const int32_t *colidx,
                   const uint8_t *mask, const int32_t *p, const float *x, const float *g,
                   const float *eta, int order, float *out)
{
    int nnz = rowptr[N];
    double *we = (double *)malloc(sizeof(double) * (size_t)(nnz > 0 ? nnz : 1));
    double *ws = (double *)malloc(sizeof(double) * (size_t)N);
    orc_weights(N, rowptr, colidx, mask, p, we, ws);
#pragma omp parallel for schedule(static) num_threads(orc_threads)
    for (int i = 0; i < N; ++i) {
        for (int64_t c = 0; c < d; ++c) {
            size_t own = (size_t)i * ld + c;
            double acc;
            if (order == 0) {
                acc = ws[i] * (double)x[own];
                for (int e = rowptr[i]; e < rowptr[i + 1]; ++e)
                    if (mask[e]) acc += we[e] * (double)x[(size_t)colidx[e] * ld + c];
                acc -= (double)eta[i] * (double)g[own];
            } else {
                acc = ws[i] * ((double)x[own] - (double)eta[i] * (double)g[own]);
                for (int e = rowptr[i]; e < rowptr[i + 1]; ++e)
                    if (mask[e]) {
                        int j = colidx[e];
                        size_t o = (size_t)j * ld + c;
                        acc += we[e] * ((double)x[o] - (double)eta[j] * (double)g[o]);
                    }
            }
            out[own] = (float)acc;
        }
    }
    free(we);
    free(ws);
}

/* Link set P: breadth-first spanning tree from node 0, neighbours in ascending index;
 * edge id = order of discovery.  Returns the number of links (N - 1) or ORC_ERR_GRAPH
 * when the graph is not connected. */
int orc_spanning_tree(int N, const int32_t *rowptr, const int32_t *colidx, int32_t *edges /* (N-1)*2 */)
{
    int *queue = (int *)malloc(sizeof(int) * (size_t)N);
    uint8_t *seen = (uint8_t *)calloc((size_t)N, 1);
    int head = 0, tail = 0, ne = 0;
    queue[tail++] = 0;
    seen[0] = 1;
    while (head < tail) {
        int u = queue[head++];
        for (int e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            int v = colidx[e];
            if (!seen[v]) {
                seen[v] = 1;
                edges[2 * ne] = u;
                edges[2 * ne + 1] = v;
                ++ne;
                queue[tail++] = v;
            }
        }
    }
    free(queue);
    free(seen);
    return ne == N - 1 ? ne : ORC_ERR_GRAPH;
}

/* One iteration of the d-iteration procedure.  A link (u, v) is established when both
 * ends have finished, at time max(t_u, t_v).  theta = the earliest establishment time
 * among links of P not yet in P' (lowest edge id on ties); that link joins P'.  P' is
 * emptied once all d links have been visited.  Then the threshold rule: a worker with
 * t_j <= theta waits for exactly its neighbours with t_i <= theta, any other worker for
 * none, expressed as backup counts b_j = deg_j - |S_j|. */
void orc_dtur(int N, const int32_t *rowptr, const int32_t *colidx, int n_edges,
              const int32_t *edges, uint8_t *visited, int32_t *n_visited, const float *t,
              int32_t *b, float *theta_out)
{
    if (*n_visited >= n_edges) {
        memset(visited, 0, (size_t)n_edges);
        *n_visited = 0;
    }
    int best = -1;
    float theta = INFINITY;
    for (int e = 0; e < n_edges; ++e) {
        if (visited[e]) continue;
        float tu = canon_time(t[edges[2 * e]]), tv = canon_time(t[edges[2 * e + 1]]);
        float est = tu > tv ? tu : tv;
        if (best < 0 || est < theta) {
            best = e;
            theta = est;
        }
    }
    if (best >= 0) {
        visited[best] = 1;
        *n_visited += 1;
    }
    for (int j = 0; j < N; ++j) {
        int deg = rowptr[j + 1] - rowptr[j];
        if (canon_time(t[j]) <= theta) {
            int cnt = 0;
            for (int e = rowptr[j]; e < rowptr[j + 1]; ++e)
                if (canon_time(t[colidx[e]]) <= theta) ++cnt;
            b[j] = deg - cnt;
        } else {
            b[j] = deg;
        }
    }
    if (theta_out) *theta_out = theta;
}

/* ------------------------------------------------------------------ gradients */

/* Branch decisions.  The models are piecewise linear up to the loss: a ReLU unit is active or
 * not, a pooling window hands its gradient to one of its four positions or (when no value is
 * positive) to none.  Where a ReLU input is zero or two pooled values tie, the mini-batch
 * gradient of Section 2.1 is not unique: either branch gives a valid subgradient, and an
 * evaluation in another precision or summation order may take the other one.  For the tests,
 * and not as part of the method, the gradient routines can (a) list every decision that lies
 * within `near_scale` rounding units of turning, and (b) evaluate the gradient with listed
 * decisions taken the other way.  The rounding unit of a pre-activation z = bias + sum_k w_k a_k
 * is u * (|bias| + sum_k |w_k a_k|) with u = 2^-24: a float evaluation of the sum in any order
 * is off by at most the number of terms times that, and typically by a fraction of it.
 *   stage  0, 1: ReLU + pooling window of the first / second convolutional stage;
 *          16 + l: ReLU after fully connected layer l (CNN: l = 0 is the layer after flatten)
 *   sample index inside the mini-batch
 *   unit   pooled output index (c * Ho + oh) * Wo + ow, or the unit's index in its layer
 *   alt    the outcome on the other side: pooling 0..3 = the window position (dh * 2 + dw) that
 *          receives the gradient, 4 = none; ReLU 1 = active, 0 = inactive
 *   gap    distance from turning, in rounding units */
typedef struct {
    int32_t stage, sample, unit, alt;
    double gap;
} orc_decision;

typedef struct {
    const orc_decision *flips; /* decisions to take as their `alt` says (gap ignored) */
    int32_t n_flips;
    orc_decision *near;        /* out: decisions with gap < near_scale, first near_cap of them */
    int32_t near_cap;
    int32_t n_near;            /* out: how many there were */
    double near_scale;
} orc_branch;

#define ORC_U 5.9604644775390625e-08 /* 2^-24 */

static const orc_decision *find_flip(const orc_branch *br, int stage, int sample, int unit)
{
    if (!br) return NULL;
    for (int f = 0; f < br->n_flips; ++f)
        if (br->flips[f].stage == stage && br->flips[f].sample == sample && br->flips[f].unit == unit)
            return &br->flips[f];
    return NULL;
}

static void note_near(orc_branch *br, int stage, int sample, int unit, int alt, double gap)
{
    if (!br || !br->near || !(gap < br->near_scale)) return;
    if (br->n_near < br->near_cap) {
        orc_decision *e = &br->near[br->n_near];
        e->stage = stage; e->sample = sample; e->unit = unit; e->alt = alt; e->gap = gap;
    }
    br->n_near += 1;
}

/* Softmax cross-entropy on one sample: fills dz = (softmax(z) - onehot(y)) * scale and
 * returns -log softmax(z)[y]. */
static double softmax_xent(int C, const double *z, int y, double scale, double *dz)
{
    double m = z[0];
    for (int c = 1; c < C; ++c)
        if (z[c] > m) m = z[c];
    double s = 0.0;
    for (int c = 0; c < C; ++c) s += exp(z[c] - m);
    for (int c = 0; c < C; ++c) dz[c] = (exp(z[c] - m) / s - (c == y ? 1.0 : 0.0)) * scale;
    return -(z[y] - m - log(s));
}

/* Squared error of the softmax outputs on one sample (the loss of the 2NN experiment of
 * Appendix B: a softmax output layer trained with the MSE loss):
 *   f = sum_c (p_c - onehot_c)^2,   df/dz_k = 2 p_k ((p_k - o_k) - sum_c p_c (p_c - o_c)).
 * Fills dz = df/dz * scale and returns f. */
static double softmax_mse(int C, const double *z, int y, double scale, double *dz)
{
    double m = z[0];
    for (int c = 1; c < C; ++c)
        if (z[c] > m) m = z[c];
    double s = 0.0;
    for (int c = 0; c < C; ++c) s += exp(z[c] - m);
    double f = 0.0, inner = 0.0;
    for (int c = 0; c < C; ++c) {
        double p = exp(z[c] - m) / s, e = p - (c == y ? 1.0 : 0.0);
        f += e * e;
        inner += p * e;
    }
    for (int c = 0; c < C; ++c) {
        double p = exp(z[c] - m) / s, e = p - (c == y ? 1.0 : 0.0);
        dz[c] = 2.0 * p * (e - inner) * scale;
    }
    return f;
}

/* Fully connected network dims[0] -> dims[1] -> ... -> dims[L], ReLU after every layer
 * but the last, mean cross-entropy over the B samples.  params / grad: per layer
 * W[out][in] then bias[out].  x: [B][dims[0]], y: [B]. */
void orc_grad_mlp_loss(int L, const int32_t *dims, int B, const float *params, const float *x,
                       const int32_t *y, int loss_kind /* 0 cross-entropy, 1 MSE on softmax outputs */,
                       float *grad, double *loss_out, orc_branch *br /* nullable */);

void orc_grad_mlp(int L, const int32_t *dims, int B, const float *params, const float *x,
                  const int32_t *y, float *grad, double *loss_out, orc_branch *br /* nullable */)
{
    orc_grad_mlp_loss(L, dims, B, params, x, y, 0, grad, loss_out, br);
}

void orc_grad_mlp_loss(int L, const int32_t *dims, int B, const float *params, const float *x,
                       const int32_t *y, int loss_kind, float *grad, double *loss_out, orc_branch *br)
{
    if (br) br->n_near = 0;
    size_t total = 0, maxw = 0;
    for (int l = 0; l < L; ++l) {
        total += (size_t)dims[l + 1] * dims[l] + dims[l + 1];
        if ((size_t)dims[l + 1] > maxw) maxw = dims[l + 1];
        if ((size_t)dims[l] > maxw) maxw = dims[l];
    }
    double *acc = (double *)calloc(total, sizeof(double));
    /* activations a[l] (input of layer l), pre-activations z[l] (output of layer l) */
    double **a = (double **)malloc(sizeof(double *) * (size_t)(L + 1));
    double **z = (double **)malloc(sizeof(double *) * (size_t)L);
    for (int l = 0; l <= L; ++l) a[l] = (double *)malloc(sizeof(double) * (size_t)dims[l]);
    for (int l = 0; l < L; ++l) z[l] = (double *)malloc(sizeof(double) * (size_t)dims[l + 1]);
    /* on[l][o]: unit o of hidden layer l is active for the current sample */
    uint8_t **on = (uint8_t **)malloc(sizeof(uint8_t *) * (size_t)L);
    for (int l = 0; l < L; ++l) on[l] = (uint8_t *)malloc((size_t)dims[l + 1]);
    double *dz = (double *)malloc(sizeof(double) * maxw);
    double *da = (double *)malloc(sizeof(double) * maxw);
    double loss = 0.0;
    for (int s = 0; s < B; ++s) {
        for (int k = 0; k < dims[0]; ++k) a[0][k] = (double)x[(size_t)s * dims[0] + k];
        size_t off = 0;
        for (int l = 0; l < L; ++l) {
            int in = dims[l], out = dims[l + 1];
            const float *W = params + off, *bias = params + off + (size_t)out * in;
            for (int o = 0; o < out; ++o) {
                double v = (double)bias[o];
                for (int k = 0; k < in; ++k) v += (double)W[(size_t)o * in + k] * a[l][k];
                z[l][o] = v;
                if (l + 1 < L) {
                    on[l][o] = v > 0.0;
                    if (br && br->near) {
                        double mag = fabs((double)bias[o]);
                        for (int k = 0; k < in; ++k) mag += fabs((double)W[(size_t)o * in + k] * a[l][k]);
                        note_near(br, 16 + l, s, o, !on[l][o], fabs(v) / (ORC_U * mag));
                    }
                    const orc_decision *f = find_flip(br, 16 + l, s, o);
                    if (f) on[l][o] = f->alt != 0;
                    a[l + 1][o] = on[l][o] && v > 0.0 ? v : 0.0;
                }
            }
            off += (size_t)out * in + out;
        }
        loss += loss_kind == 1 ? softmax_mse(dims[L], z[L - 1], y[s], 1.0 / (double)B, dz)
                               : softmax_xent(dims[L], z[L - 1], y[s], 1.0 / (double)B, dz);
        for (int l = L - 1; l >= 0; --l) {
            int in = dims[l], out = dims[l + 1];
            off -= (size_t)out * in + out;
            const float *W = params + off;
            double *gW = acc + off, *gb = acc + off + (size_t)out * in;
            for (int k = 0; k < in; ++k) da[k] = 0.0;
            for (int o = 0; o < out; ++o) {
                gb[o] += dz[o];
                for (int k = 0; k < in; ++k) {
                    gW[(size_t)o * in + k] += dz[o] * a[l][k];
                    da[k] += (double)W[(size_t)o * in + k] * dz[o];
                }
            }
            if (l > 0)
                for (int k = 0; k < in; ++k) dz[k] = on[l - 1][k] ? da[k] : 0.0;
        }
    }
    for (size_t k = 0; k < total; ++k) grad[k] = (float)acc[k];
    if (loss_out) *loss_out = loss / (double)B;
    for (int l = 0; l <= L; ++l) free(a[l]);
    for (int l = 0; l < L; ++l) { free(z[l]); free(on[l]); }
    free(a); free(z); free(on); free(dz); free(da); free(acc);
}

/* Direct 'same' convolution, stride 1, odd K, zero padding K/2:
 * out[co][oh][ow] = bias[co] + sum_{ci,kh,kw} W[co][ci][kh][kw] in[ci][oh+kh-pad][ow+kw-pad]. */
static void conv_fwd(int Ci, int Co, int H, int Wd, int K, const float *W, const float *bias,
                     const double *in, double *out)
{
    int pad = K / 2;
    for (int co = 0; co < Co; ++co) {
        double *o = out + (size_t)co * H * Wd;
        for (int q = 0; q < H * Wd; ++q) o[q] = (double)bias[co];
        for (int ci = 0; ci < Ci; ++ci)
            for (int kh = 0; kh < K; ++kh)
                for (int kw = 0; kw < K; ++kw) {
                    double w = (double)W[(((size_t)co * Ci + ci) * K + kh) * K + kw];
                    for (int oh = 0; oh < H; ++oh) {
                        int ih = oh + kh - pad;
                        if (ih < 0 || ih >= H) continue;
                        for (int ow = 0; ow < Wd; ++ow) {
                            int iw = ow + kw - pad;
                            if (iw < 0 || iw >= Wd) continue;
                            o[oh * Wd + ow] += w * in[((size_t)ci * H + ih) * Wd + iw];
                        }
                    }
                }
    }
}

/* Adjoint of conv_fwd: accumulates gW, gb; writes din when it is not NULL. */
static void conv_bwd(int Ci, int Co, int H, int Wd, int K, const float *W, const double *in,
                     const double *dout, double *gW, double *gb, double *din)
{
    int pad = K / 2;
    if (din) memset(din, 0, sizeof(double) * (size_t)Ci * H * Wd);
    for (int co = 0; co < Co; ++co) {
        const double *go = dout + (size_t)co * H * Wd;
        for (int q = 0; q < H * Wd; ++q) gb[co] += go[q];
        for (int ci = 0; ci < Ci; ++ci)
            for (int kh = 0; kh < K; ++kh)
                for (int kw = 0; kw < K; ++kw) {
                    size_t wi = (((size_t)co * Ci + ci) * K + kh) * K + kw;
                    double w = (double)W[wi], gw = 0.0;
                    for (int oh = 0; oh < H; ++oh) {
                        int ih = oh + kh - pad;
                        if (ih < 0 || ih >= H) continue;
                        for (int ow = 0; ow < Wd; ++ow) {
                            int iw = ow + kw - pad;
                            if (iw < 0 || iw >= Wd) continue;
                            size_t ii = ((size_t)ci * H + ih) * Wd + iw;
                            gw += go[oh * Wd + ow] * in[ii];
                            if (din) din[ii] += w * go[oh * Wd + ow];
                        }
                    }
                    gW[wi] += gw;
                }
    }
}

/* The rounding unit of every output of conv_fwd: |bias| + sum of |W in| over the same taps. */
static void conv_magnitude(int Ci, int Co, int H, int Wd, int K, const float *W, const float *bias,
                           const double *in, double *out)
{
    int pad = K / 2;
    for (int co = 0; co < Co; ++co) {
        double *o = out + (size_t)co * H * Wd;
        for (int q = 0; q < H * Wd; ++q) o[q] = fabs((double)bias[co]);
        for (int ci = 0; ci < Ci; ++ci)
            for (int kh = 0; kh < K; ++kh)
                for (int kw = 0; kw < K; ++kw) {
                    double w = (double)W[(((size_t)co * Ci + ci) * K + kh) * K + kw];
                    for (int oh = 0; oh < H; ++oh) {
                        int ih = oh + kh - pad;
                        if (ih < 0 || ih >= H) continue;
                        for (int ow = 0; ow < Wd; ++ow) {
                            int iw = ow + kw - pad;
                            if (iw < 0 || iw >= Wd) continue;
                            o[oh * Wd + ow] += fabs(w * in[((size_t)ci * H + ih) * Wd + iw]);
                        }
                    }
                }
    }
}

/* ReLU then 2x2/stride-2 max pooling; arg[] keeps the flat input index of the first
 * maximum in window order (0,0),(0,1),(1,0),(1,1), pass[] whether that value is positive
 * (only then does the window hand its gradient on).  mag (rounding units of z) is needed
 * only when near decisions are listed. */
static void relu_pool_fwd(int C, int H, int Wd, const double *z, double *out, int *arg, uint8_t *pass,
                          int stage, int sample, orc_branch *br, const double *mag)
{
    int Ho = H / 2, Wo = Wd / 2;
    for (int c = 0; c < C; ++c)
        for (int oh = 0; oh < Ho; ++oh)
            for (int ow = 0; ow < Wo; ++ow) {
                double best = 0.0;
                int bi = -1;
                for (int dh = 0; dh < 2; ++dh)
                    for (int dw = 0; dw < 2; ++dw) {
                        int ii = (c * H + 2 * oh + dh) * Wd + 2 * ow + dw;
                        double v = z[ii] > 0.0 ? z[ii] : 0.0;
                        if (bi < 0 || v > best) { best = v; bi = ii; }
                    }
                int q = (c * Ho + oh) * Wo + ow;
                out[q] = best;
                arg[q] = bi;
                pass[q] = z[bi] > 0.0;
                if (br && br->near && mag) {
                    for (int w = 0; w < 4; ++w) {
                        int ii = (c * H + 2 * oh + w / 2) * Wd + 2 * ow + w % 2;
                        if (pass[q] && ii != bi)       /* another position overtakes the maximum */
                            note_near(br, stage, sample, q, w, (z[bi] - z[ii]) / (ORC_U * (mag[bi] + mag[ii])));
                        else if (!pass[q])             /* a non-positive value turns positive */
                            note_near(br, stage, sample, q, w, -z[ii] / (ORC_U * mag[ii]));
                    }
                    if (pass[q])                       /* the maximum turns non-positive */
                        note_near(br, stage, sample, q, 4, z[bi] / (ORC_U * mag[bi]));
                }
                const orc_decision *f = find_flip(br, stage, sample, q);
                if (f) {
                    pass[q] = f->alt != 4;
                    if (pass[q]) arg[q] = (c * H + 2 * oh + f->alt / 2) * Wd + 2 * ow + f->alt % 2;
                    out[q] = pass[q] && z[arg[q]] > 0.0 ? z[arg[q]] : 0.0;
                }
            }
}

static void relu_pool_bwd(int C, int H, int Wd, const int *arg, const uint8_t *pass,
                          const double *dout, double *dz)
{
    int Ho = H / 2, Wo = Wd / 2;
    memset(dz, 0, sizeof(double) * (size_t)C * H * Wd);
    for (int q = 0; q < C * Ho * Wo; ++q)
        if (pass[q]) dz[arg[q]] += dout[q];
}

/* conv KxK (C0->C1, same) ReLU pool2 -> conv KxK (C1->C2, same) ReLU pool2 -> flatten
 * [C2][H/4][W/4] -> FC F ReLU -> FC classes -> mean cross-entropy.
 * shape = {C0, H, W, C1, C2, K, F, classes}.  Parameter order: conv1 W,b; conv2 W,b;
 * fc1 W,b; fc2 W,b. */
void orc_grad_cnn(const int32_t *shape, int B, const float *params, const float *x,
                  const int32_t *y, float *grad, double *loss_out, orc_branch *br /* nullable */)
{
    if (br) br->n_near = 0;
    int C0 = shape[0], H = shape[1], Wd = shape[2], C1 = shape[3], C2 = shape[4], K = shape[5],
        F = shape[6], NC = shape[7];
    int H2 = H / 2, W2 = Wd / 2, H4 = H / 4, W4 = Wd / 4, flat = C2 * H4 * W4;
    size_t o_w1 = 0, o_b1 = o_w1 + (size_t)C1 * C0 * K * K, o_w2 = o_b1 + C1,
           o_b2 = o_w2 + (size_t)C2 * C1 * K * K, o_w3 = o_b2 + C2, o_b3 = o_w3 + (size_t)F * flat,
           o_w4 = o_b3 + F, o_b4 = o_w4 + (size_t)NC * F, total = o_b4 + NC;
    double *acc = (double *)calloc(total, sizeof(double));
    double *a0 = (double *)malloc(sizeof(double) * (size_t)C0 * H * Wd);
    double *z1 = (double *)malloc(sizeof(double) * (size_t)C1 * H * Wd);
    double *dz1 = (double *)malloc(sizeof(double) * (size_t)C1 * H * Wd);
    double *p1 = (double *)malloc(sizeof(double) * (size_t)C1 * H2 * W2);
    double *dp1 = (double *)malloc(sizeof(double) * (size_t)C1 * H2 * W2);
    int *arg1 = (int *)malloc(sizeof(int) * (size_t)C1 * H2 * W2);
    double *z2 = (double *)malloc(sizeof(double) * (size_t)C2 * H2 * W2);
    double *dz2 = (double *)malloc(sizeof(double) * (size_t)C2 * H2 * W2);
    double *p2 = (double *)malloc(sizeof(double) * (size_t)flat);
    double *dp2 = (double *)malloc(sizeof(double) * (size_t)flat);
    int *arg2 = (int *)malloc(sizeof(int) * (size_t)flat);
    uint8_t *pass1 = (uint8_t *)malloc((size_t)C1 * H2 * W2);
    uint8_t *pass2 = (uint8_t *)malloc((size_t)flat);
    uint8_t *on3 = (uint8_t *)malloc((size_t)F);
    int listing = br && br->near;
    double *mag1 = listing ? (double *)malloc(sizeof(double) * (size_t)C1 * H * Wd) : NULL;
    double *mag2 = listing ? (double *)malloc(sizeof(double) * (size_t)C2 * H2 * W2) : NULL;
    double *z3 = (double *)malloc(sizeof(double) * (size_t)F);
    double *a3 = (double *)malloc(sizeof(double) * (size_t)F);
    double *dz3 = (double *)malloc(sizeof(double) * (size_t)F);
    double *z4 = (double *)malloc(sizeof(double) * (size_t)NC);
    double *dz4 = (double *)malloc(sizeof(double) * (size_t)NC);
    double loss = 0.0;
    for (int s = 0; s < B; ++s) {
        for (int q = 0; q < C0 * H * Wd; ++q) a0[q] = (double)x[(size_t)s * C0 * H * Wd + q];
        conv_fwd(C0, C1, H, Wd, K, params + o_w1, params + o_b1, a0, z1);
        if (listing) conv_magnitude(C0, C1, H, Wd, K, params + o_w1, params + o_b1, a0, mag1);
        relu_pool_fwd(C1, H, Wd, z1, p1, arg1, pass1, 0, s, br, mag1);
        conv_fwd(C1, C2, H2, W2, K, params + o_w2, params + o_b2, p1, z2);
        if (listing) conv_magnitude(C1, C2, H2, W2, K, params + o_w2, params + o_b2, p1, mag2);
        relu_pool_fwd(C2, H2, W2, z2, p2, arg2, pass2, 1, s, br, mag2);
        for (int o = 0; o < F; ++o) {
            double v = (double)params[o_b3 + o];
            for (int k = 0; k < flat; ++k) v += (double)params[o_w3 + (size_t)o * flat + k] * p2[k];
            z3[o] = v;
            on3[o] = v > 0.0;
            if (listing) {
                double mag = fabs((double)params[o_b3 + o]);
                for (int k = 0; k < flat; ++k) mag += fabs((double)params[o_w3 + (size_t)o * flat + k] * p2[k]);
                note_near(br, 16, s, o, !on3[o], fabs(v) / (ORC_U * mag));
            }
            const orc_decision *f = find_flip(br, 16, s, o);
            if (f) on3[o] = f->alt != 0;
            a3[o] = on3[o] && v > 0.0 ? v : 0.0;
        }
        for (int o = 0; o < NC; ++o) {
            double v = (double)params[o_b4 + o];
            for (int k = 0; k < F; ++k) v += (double)params[o_w4 + (size_t)o * F + k] * a3[k];
            z4[o] = v;
        }
        loss += softmax_xent(NC, z4, y[s], 1.0 / (double)B, dz4);
        /* fc2 */
        for (int k = 0; k < F; ++k) dz3[k] = 0.0;
        for (int o = 0; o < NC; ++o) {
            acc[o_b4 + o] += dz4[o];
            for (int k = 0; k < F; ++k) {
                acc[o_w4 + (size_t)o * F + k] += dz4[o] * a3[k];
                dz3[k] += (double)params[o_w4 + (size_t)o * F + k] * dz4[o];
            }
        }
        for (int k = 0; k < F; ++k)
            if (!on3[k]) dz3[k] = 0.0;
        /* fc1 */
        for (int k = 0; k < flat; ++k) dp2[k] = 0.0;
        for (int o = 0; o < F; ++o) {
            acc[o_b3 + o] += dz3[o];
            for (int k = 0; k < flat; ++k) {
                acc[o_w3 + (size_t)o * flat + k] += dz3[o] * p2[k];
                dp2[k] += (double)params[o_w3 + (size_t)o * flat + k] * dz3[o];
            }
        }
        relu_pool_bwd(C2, H2, W2, arg2, pass2, dp2, dz2);
        conv_bwd(C1, C2, H2, W2, K, params + o_w2, p1, dz2, acc + o_w2, acc + o_b2, dp1);
        relu_pool_bwd(C1, H, Wd, arg1, pass1, dp1, dz1);
        conv_bwd(C0, C1, H, Wd, K, params + o_w1, a0, dz1, acc + o_w1, acc + o_b1, NULL);
    }
    for (size_t k = 0; k < total; ++k) grad[k] = (float)acc[k];
    if (loss_out) *loss_out = loss / (double)B;
    free(acc); free(a0); free(z1); free(dz1); free(p1); free(dp1); free(arg1);
    free(z2); free(dz2); free(p2); free(dp2); free(arg2); free(z3); free(a3); free(dz3);
    free(z4); free(dz4); free(pass1); free(pass2); free(on3); free(mag1); free(mag2);
}

/* Gradients of all workers: worker i uses row i of params [N][ld], its own batch, and
 * writes row i of grad [N][ld] (padding columns zeroed).  kind 0: fully connected
 * (desc = {L, dims[0..L]}), kind 1: convolutional (desc = shape[8]), kind 2: fully connected
 * with the MSE-on-softmax loss.  With near != NULL every worker's decisions closer than
 * near_scale rounding units to turning are listed: worker i's in near[i * near_cap ...], their
 * number (also beyond near_cap) in n_near[i]. */
void orc_grad_all(int kind, const int32_t *desc, int N, int64_t d, int64_t ld, int B,
                  int64_t in_dim, const float *params, const float *x, const int32_t *y,
                  float *grad, double *loss /* N, nullable */, orc_decision *near /* nullable */,
                  int32_t near_cap, int32_t *n_near /* N */, double near_scale)
{
#pragma omp parallel for schedule(dynamic, 1) num_threads(orc_threads)
    for (int i = 0; i < N; ++i) {
        float *gi = grad + (size_t)i * ld;
        double li = 0.0;
        orc_branch br = {NULL, 0, near ? near + (size_t)i * near_cap : NULL, near_cap, 0, near_scale};
        orc_branch *bp = near ? &br : NULL;
        if (kind == 0 || kind == 2)
            orc_grad_mlp_loss(desc[0], desc + 1, B, params + (size_t)i * ld,
                              x + (size_t)i * B * in_dim, y + (size_t)i * B, kind == 2, gi, &li, bp);
        else
            orc_grad_cnn(desc, B, params + (size_t)i * ld, x + (size_t)i * B * in_dim,
                         y + (size_t)i * B, gi, &li, bp);
        for (int64_t c = d; c < ld; ++c) gi[c] = 0.0f;
        if (loss) loss[i] = li;
        if (near) n_near[i] = br.n_near;
    }
}
