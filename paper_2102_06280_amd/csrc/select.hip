// Fastest-neighbour selection, Metropolis weights and the threshold rule.
//
// Selection (Section 1 "Dynamic Backup Workers", Section 2.2): worker i waits for the
// p_i = deg_i - b_i neighbours that answer first; the rest are backups.  One 64-lane
// wavefront per worker ranks the row's neighbours by the 64-bit key (time, index): a
// neighbour is selected iff fewer than p_i keys in the row are smaller than its own (rows
// longer than 64 neighbours are shared by four wavefronts).
// Keys are distinct (indices are), so the ranks form a permutation and the result does
// not depend on any scheduling order.
//
// Weights (Assumption 1): P_ij = 1/(1 + max(p_i, p_j)) for selected j, P_ii = 1 - sum.
#include "dbw_internal.h"

namespace {

// Monotone map from float to uint32 under IEEE ordering, with NaN -> +inf and -0 -> +0.
__device__ __forceinline__ float canon_time(float t)
{
    return (t != t) ? __builtin_inff() : (t == 0.0f ? 0.0f : t);
}

__device__ __forceinline__ uint32_t sortable(float t)
{
    uint32_t u = __float_as_uint(canon_time(t));
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t make_key(float t, int32_t j)
{
    return ((uint64_t)sortable(t) << 32) | (uint32_t)j;
}

__device__ __forceinline__ int clamp_b(int b, int deg) { return b < 0 ? 0 : (b > deg ? deg : b); }

__device__ __forceinline__ float wave_sum(float v)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// A row group = WAVES wavefronts that share one worker's row.  With one wavefront the group needs no
// workgroup barrier: LDS operations of one wavefront complete in order, only the compiler has to keep them
// in order too.
template <int WAVES>
__device__ __forceinline__ void group_sync()
{
    if (WAVES > 1) {
        __syncthreads();
    } else {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// LDS of one row group.
template <int WAVES, int KEYS>
struct SelectLds {
    uint64_t keys[KEYS];
    float wrow[DBW_DENSE_MAX_N];
    int slice_cnt[WAVES];
    float red[2][WAVES];
};

// Selection, weights and wait time of worker i by a row group of WAVES wavefronts (tid = thread index inside
// the group).  Each wave ranks one 64-wide slice of the row at a time; slices are compacted in ascending order
// through per-wave counts.  b may point to global memory or to LDS.
template <int WAVES, int KEYS>
__device__ __forceinline__ void select_row(
    int i, int tid, SelectLds<WAVES, KEYS> &L, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ t, const int32_t *b, int32_t *__restrict__ p_out, uint8_t *__restrict__ mask,
    float *__restrict__ wait, int32_t *__restrict__ sel_idx, float *__restrict__ sel_w, float *__restrict__ self_w,
    float *__restrict__ Wdense, int Npad, int32_t *__restrict__ err)
{
    constexpr int T = 64 * WAVES;
    uint64_t *keys = L.keys;
    float *wrow = L.wrow;
    const int lane = tid & 63, wave = tid >> 6;
    const int beg = rowptr[i], deg = rowptr[i + 1] - beg;
    const int bi_raw = b[i];
    if ((bi_raw < 0 || bi_raw > deg) && tid == 0) *err = DBW_ERR_INVALID;
    const int pi = deg - clamp_b(bi_raw, deg);
    const bool in_lds = deg <= KEYS;

    if (in_lds)
        for (int k = tid; k < deg; k += T) {
            int j = colidx[beg + k];
            keys[k] = make_key(t[j], j);
        }
    if (Wdense)
        for (int c = tid; c < Npad; c += T) wrow[c] = 0.0f;
    group_sync<WAVES>();

    float wsum = 0.0f, tmax = canon_time(t[i]);
    int base = 0;
    for (int k0 = 0; k0 < deg; k0 += T) {
        const int k = k0 + tid;
        bool sel = false;
        int j = 0;
        float w = 0.0f;
        if (k < deg) {
            j = colidx[beg + k];
            const float tj = t[j];
            const uint64_t mine = make_key(tj, j);
            int rank = 0;
            if (in_lds) {
                for (int m = 0; m < deg; ++m) rank += keys[m] < mine ? 1 : 0;
            } else {
                for (int m = 0; m < deg; ++m) {
                    int jm = colidx[beg + m];
                    rank += make_key(t[jm], jm) < mine ? 1 : 0;
                }
            }
            sel = rank < pi;
            mask[beg + k] = sel ? 1 : 0;
            if (sel) {
                const int degj = rowptr[j + 1] - rowptr[j];
                const int pj = degj - clamp_b(b[j], degj);
                w = 1.0f / (1.0f + (float)(pi > pj ? pi : pj));
                wsum += w;
                tmax = fmaxf(tmax, canon_time(tj));
            }
        }
        // compact the selected neighbours of this slice, keeping ascending order
        const uint64_t ballot = __ballot(sel);
        int before = 0, total = __popcll(ballot);
        if (WAVES > 1) {
            if (lane == 0) L.slice_cnt[wave] = total;
            __syncthreads();
            total = 0;
#pragma unroll
            for (int q = 0; q < WAVES; ++q) {
                before += q < wave ? L.slice_cnt[q] : 0;
                total += L.slice_cnt[q];
            }
            __syncthreads();                          // slice_cnt is rewritten in the next pass
        }
        if (sel) {
            const int pos = base + before + __popcll(ballot & ((1ull << lane) - 1ull));
            sel_idx[beg + pos] = j;
            sel_w[beg + pos] = w;
            if (Wdense) wrow[j] = w;
        }
        base += total;
    }
    wsum = wave_sum(wsum);
    tmax = wave_max(tmax);
    if (WAVES > 1) {
        if (lane == 0) {
            L.red[0][wave] = wsum;
            L.red[1][wave] = tmax;
        }
        __syncthreads();
        wsum = 0.0f;
#pragma unroll
        for (int q = 0; q < WAVES; ++q) {
            wsum += L.red[0][q];
            tmax = fmaxf(tmax, L.red[1][q]);
        }
    }
    const float ws = 1.0f - wsum;
    if (tid == 0) {
        p_out[i] = pi;
        wait[i] = tmax;
        self_w[i] = ws;
    }
    if (Wdense) {
        group_sync<WAVES>();
        if (tid == 0) wrow[i] = ws;
        group_sync<WAVES>();
        // A-operand fragment order of the dense kernel: [row block][k-step][lane], with
        // lane = (k % 2) * 32 + row % 32 holding P[row][k]
        const int KB = Npad / 2;
        for (int c = tid; c < Npad; c += T)
            Wdense[((size_t)(i >> 5) * KB + (c >> 1)) * 64 + (c & 1) * 32 + (i & 31)] = wrow[c];
    }
}

// grid = N blocks of WAVES wavefronts: one block per worker.
template <int WAVES>
__global__ __launch_bounds__(64 * WAVES) void select_kernel(
    int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ t, const int32_t *__restrict__ b, int32_t *__restrict__ p_out,
    uint8_t *__restrict__ mask, float *__restrict__ wait, int32_t *__restrict__ sel_idx,
    float *__restrict__ sel_w, float *__restrict__ self_w, float *__restrict__ Wdense, int Npad,
    int32_t *__restrict__ err)
{
    __shared__ SelectLds<WAVES, DBW_SELECT_LDS_KEYS> L;
    select_row<WAVES, DBW_SELECT_LDS_KEYS>(blockIdx.x, threadIdx.x, L, rowptr, colidx, t, b, p_out, mask, wait, sel_idx,
                                           sel_w, self_w, Wdense, Npad, err);
}

// Rows [N, Npad) of the padded dense matrix stay zero: cleared once at create.

// Threshold rule and the d-iteration procedure (Section 4.1, Algorithm 2); one block of T threads.
// A link (u, v) is established at max(t_u, t_v).  theta = the smallest establishment
// time over links not yet visited in this epoch, lowest link id on ties.  b_lds (nullable) receives a
// copy of the backup counts in LDS.
template <int T>
__device__ __forceinline__ void dtur_body(
    uint64_t *red /* LDS [T] */, int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    int n_links, const int32_t *__restrict__ links, uint8_t *__restrict__ visited, int32_t *__restrict__ n_visited,
    const float *__restrict__ t, int32_t *__restrict__ b_out, int32_t *b_lds, float *__restrict__ theta_out,
    int32_t *__restrict__ err)
{
    const int tid = threadIdx.x;
    const bool fresh = *n_visited >= n_links;   // previous epoch complete: P' starts empty
    uint64_t best = ~0ull;
    for (int e = tid; e < n_links; e += T) {
        if (!fresh && visited[e]) continue;
        const float est = fmaxf(canon_time(t[links[2 * e]]), canon_time(t[links[2 * e + 1]]));
        const uint64_t key = make_key(est, e);
        best = key < best ? key : best;
    }
    red[tid] = best;
    __syncthreads();
    for (int o = T / 2; o > 0; o >>= 1) {
        if (tid < o) red[tid] = red[tid + o] < red[tid] ? red[tid + o] : red[tid];
        __syncthreads();
    }
    best = red[0];
    float theta = __builtin_inff();
    int chosen = -1;
    if (best != ~0ull) {
        chosen = (int)(uint32_t)best;
        theta = fmaxf(canon_time(t[links[2 * chosen]]), canon_time(t[links[2 * chosen + 1]]));
    }
    __syncthreads();    // every thread has read n_visited / visited before they change
    if (fresh)
        for (int e = tid; e < n_links; e += T) visited[e] = 0;
    __syncthreads();
    if (tid == 0) {
        if (chosen >= 0) visited[chosen] = 1;
        *n_visited = (fresh ? 0 : *n_visited) + (chosen >= 0 ? 1 : 0);
        if (theta_out) *theta_out = theta;
        // no link of the set can be established (a dead worker on every unvisited link): every
        // worker keeps to itself this round.  Recorded as a warning unless an error is pending.
        if (n_links > 0 && theta == __builtin_inff() && *err == 0) *err = DBW_WARN_THETA_INF;
    }
    for (int j = tid; j < N; j += T) {
        const int beg = rowptr[j], end = rowptr[j + 1];
        int bj = end - beg;
        if (canon_time(t[j]) <= theta) {
            int cnt = 0;
            for (int e = beg; e < end; ++e) cnt += canon_time(t[colidx[e]]) <= theta ? 1 : 0;
            bj -= cnt;
        }
        b_out[j] = bj;
        if (b_lds) b_lds[j] = bj;
    }
}

__global__ __launch_bounds__(256) void dtur_kernel(
    int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx, int n_links,
    const int32_t *__restrict__ links, uint8_t *__restrict__ visited, int32_t *__restrict__ n_visited,
    const float *__restrict__ t, int32_t *__restrict__ b_out, float *__restrict__ theta_out,
    int32_t *__restrict__ err)
{
    __shared__ uint64_t red[256];
    dtur_body<256>(red, N, rowptr, colidx, n_links, links, visited, n_visited, t, b_out, nullptr, theta_out, err);
}

// The threshold rule and the selection it leads to in one launch, for graphs of up to DBW_FUSED_SELECT_MAX_N
// workers with rows of at most 64 neighbours: one workgroup of 16 wavefronts runs the rule, then every
// wavefront takes workers i = wave, wave + 16, ... through select_row.  Two launches of 4-8 us each become one;
// the selection is the same code, so the results are identical.
constexpr int FUSED_WAVES = 16;
__global__ __launch_bounds__(64 * FUSED_WAVES) void dtur_select_kernel(
    int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx, int n_links,
    const int32_t *__restrict__ links, uint8_t *__restrict__ visited, int32_t *__restrict__ n_visited,
    const float *__restrict__ t, int32_t *__restrict__ b_out, float *__restrict__ theta_out,
    int32_t *__restrict__ p_out, uint8_t *__restrict__ mask, float *__restrict__ wait, int32_t *__restrict__ sel_idx,
    float *__restrict__ sel_w, float *__restrict__ self_w, float *__restrict__ Wdense, int Npad, int32_t *__restrict__ err)
{
    __shared__ uint64_t red[64 * FUSED_WAVES];
    __shared__ int32_t b_lds[DBW_FUSED_SELECT_MAX_N];
    __shared__ SelectLds<1, 64> L[FUSED_WAVES];
    dtur_body<64 * FUSED_WAVES>(red, N, rowptr, colidx, n_links, links, visited, n_visited, t, b_out, b_lds, theta_out, err);
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    for (int i = wave; i < N; i += FUSED_WAVES)
        select_row<1, 64>(i, lane, L[wave], rowptr, colidx, t, b_lds, p_out, mask, wait, sel_idx, sel_w, self_w, Wdense,
                          Npad, err);
}

// The next call of the threshold rule starts a fresh epoch.
__global__ void dtur_reset_kernel(int n_links, int32_t *__restrict__ n_visited) { *n_visited = n_links; }

// Dense consensus matrix P(k), row-major N x N, from the compacted selection.  grid = N.
__global__ __launch_bounds__(256) void dense_weights_kernel(int N, const int32_t *__restrict__ rowptr,
                                                            const int32_t *__restrict__ p,
                                                            const int32_t *__restrict__ sel_idx,
                                                            const float *__restrict__ sel_w,
                                                            const float *__restrict__ self_w, float *__restrict__ P)
{
    const int i = blockIdx.x, beg = rowptr[i], cnt = p[i];
    float *row = P + (size_t)i * N;
    for (int c = threadIdx.x; c < N; c += 256) row[c] = c == i ? self_w[i] : 0.0f;
    __syncthreads();
    for (int k = threadIdx.x; k < cnt; k += 256) row[sel_idx[beg + k]] = sel_w[beg + k];
}

// Round duration (Section 3.2.2): max of the wait times over all workers and over the
// workers that appear in some selected set.  One block of 1024 threads; the mask is read four
// entries at a time; `listed` is context scratch [N].
__global__ __launch_bounds__(1024) void round_time_kernel(int N, int nnz, const int32_t *__restrict__ colidx,
                                                          const uint8_t *__restrict__ mask,
                                                          const float *__restrict__ wait, uint8_t *__restrict__ listed,
                                                          float *__restrict__ out)
{
    __shared__ float red[2][1024];
    const int tid = threadIdx.x;
    for (int i = tid; i < N; i += 1024) listed[i] = 0;
    __syncthreads();
    const int words = nnz / 4;
    for (int q = tid; q < words; q += 1024) {
        const uint32_t m = ((const uint32_t *)mask)[q];
        if (m) {
            // benign race: every writer stores the same value
            if (m & 0x000000ffu) listed[colidx[4 * q]] = 1;
            if (m & 0x0000ff00u) listed[colidx[4 * q + 1]] = 1;
            if (m & 0x00ff0000u) listed[colidx[4 * q + 2]] = 1;
            if (m & 0xff000000u) listed[colidx[4 * q + 3]] = 1;
        }
    }
    for (int e = 4 * words + tid; e < nnz; e += 1024)
        if (mask[e]) listed[colidx[e]] = 1;
    __syncthreads();
    float all = 0.f, sel = 0.f;
    for (int i = tid; i < N; i += 1024) {
        const float t = wait[i];
        all = fmaxf(all, t);
        if (listed[i]) sel = fmaxf(sel, t);
    }
    red[0][tid] = all;
    red[1][tid] = sel;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (tid < o) {
            red[0][tid] = fmaxf(red[0][tid], red[0][tid + o]);
            red[1][tid] = fmaxf(red[1][tid], red[1][tid + o]);
        }
        __syncthreads();
    }
    if (tid == 0) {
        out[0] = red[0][0];
        out[1] = red[1][0];
    }
}

}  // namespace

int dbw_launch_round_time(dbw_ctx *c, float *out, hipStream_t s)
{
    dbw_timer tm(c, "round_time_kernel", s);
    hipLaunchKernelGGL(round_time_kernel, dim3(1), dim3(1024), 0, s, c->N, c->nnz, c->colidx, c->mask, c->wait,
                       c->listed, out);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

int dbw_launch_select(dbw_ctx *c, const float *t, const int32_t *b, hipStream_t s)
{
    dbw_timer tm(c, "select_kernel", s);
    // rows longer than one wavefront are ranked by four wavefronts side by side
    if (c->max_deg > 64)
        hipLaunchKernelGGL(select_kernel<4>, dim3(c->N), dim3(256), 0, s, c->N, c->rowptr, c->colidx, t, b, c->p,
                           c->mask, c->wait, c->sel_idx, c->sel_w, c->self_w, c->Wdense, c->Npad, c->err);
    else
        hipLaunchKernelGGL(select_kernel<1>, dim3(c->N), dim3(64), 0, s, c->N, c->rowptr, c->colidx, t, b, c->p,
                           c->mask, c->wait, c->sel_idx, c->sel_w, c->self_w, c->Wdense, c->Npad, c->err);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

int dbw_launch_dtur(dbw_ctx *c, const float *t, int32_t *b_out, float *theta_out, hipStream_t s)
{
    dbw_timer tm(c, "dtur_kernel", s);
    hipLaunchKernelGGL(dtur_kernel, dim3(1), dim3(256), 0, s, c->N, c->rowptr, c->colidx, c->N - 1, c->links,
                       c->visited, c->n_visited, t, b_out, theta_out, c->err);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

bool dbw_fused_dtur_select_fits(const dbw_ctx *c) { return c->N <= DBW_FUSED_SELECT_MAX_N && c->max_deg <= 64; }

int dbw_launch_dtur_select(dbw_ctx *c, const float *t, int32_t *b_out, float *theta_out, hipStream_t s)
{
    dbw_timer tm(c, "dtur_select_kernel", s);
    hipLaunchKernelGGL(dtur_select_kernel, dim3(1), dim3(64 * FUSED_WAVES), 0, s, c->N, c->rowptr, c->colidx, c->N - 1,
                       c->links, c->visited, c->n_visited, t, b_out, theta_out, c->p, c->mask, c->wait, c->sel_idx, c->sel_w,
                       c->self_w, c->Wdense, c->Npad, c->err);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

int dbw_launch_dtur_reset(dbw_ctx *c, hipStream_t s)
{
    hipLaunchKernelGGL(dtur_reset_kernel, dim3(1), dim3(1), 0, s, c->N - 1, c->n_visited);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

int dbw_launch_dense_weights(dbw_ctx *c, float *P, hipStream_t s)
{
    hipLaunchKernelGGL(dense_weights_kernel, dim3(c->N), dim3(256), 0, s, c->N, c->rowptr, c->p, c->sel_idx, c->sel_w,
                       c->self_w, P);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}
