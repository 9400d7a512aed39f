// Masked consensus average over the selected neighbours, fused with the local SGD step
// (Section 2.1 full-participation update; Section 2.2 local update + partial consensus).
//
//   CTA: out_i = P_ii x_i + sum_{j in S_i} P_ij x_j - lr g_i
//   ATC: out_i = P_ii (x_i - lr g_i) + sum_{j in S_i} P_ij (x_j - lr g_j)
//
// The work is a pure HBM stream: every parameter and gradient has to come in once and
// every result go out once.  A neighbour's row is needed by several workers, so all
// workers of one column chunk are scheduled next to each other on the same XCD: the
// chunk (N rows x chunk bytes) then sits in that XCD's L2 while its readers run, and
// HBM sees each row once.  Workgroup ids are dealt round-robin to the 8 XCDs, hence the
// id -> (chunk, worker) map below.  The summation order is fixed (self, then selected
// neighbours in ascending index), so results are bit-reproducible.
#include "dbw_internal.h"

namespace {

constexpr int MIX_THREADS = 256;
constexpr int MIX_XCDS = 8;

__device__ __forceinline__ float4 fma4(float w, float4 a, float4 acc)
{
    acc.x = fmaf(w, a.x, acc.x);
    acc.y = fmaf(w, a.y, acc.y);
    acc.z = fmaf(w, a.z, acc.z);
    acc.w = fmaf(w, a.w, acc.w);
    return acc;
}

// One workgroup = one worker x one chunk of MIX_THREADS*UNROLL float4 columns.
template <int ORDER, bool HAS_G, int UNROLL>
__global__ __launch_bounds__(MIX_THREADS) void mix_csr_vec4(
    int N, int64_t n_vec /* float4 columns per row */, int64_t ld4 /* row stride in float4 */,
    int n_chunks, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ p,
    const int32_t *__restrict__ sel_idx, const float *__restrict__ sel_w,
    const float *__restrict__ self_w, const float4 *__restrict__ x, const float4 *__restrict__ g,
    float4 *__restrict__ out, float lr)
{
    const int64_t L = blockIdx.x;
    const int xcd = (int)(L % MIX_XCDS);
    const int64_t slot = L / MIX_XCDS;
    const int i = (int)(slot % N);
    const int64_t chunk = (slot / N) * MIX_XCDS + xcd;
    if (chunk >= n_chunks) return;

    const int beg = rowptr[i], cnt = p[i];
    const float ws = self_w[i];
    const int64_t c0 = chunk * (int64_t)(MIX_THREADS * UNROLL) + threadIdx.x;
    const float4 *xi = x + (int64_t)i * ld4;

    float4 acc[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t c = c0 + (int64_t)u * MIX_THREADS;
        acc[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c < n_vec) {
            float4 v = xi[c];
            if (ORDER == DBW_ORDER_ATC && HAS_G) v = fma4(-lr, g[(int64_t)i * ld4 + c], v);
            acc[u] = make_float4(ws * v.x, ws * v.y, ws * v.z, ws * v.w);
        }
    }
    for (int k = 0; k < cnt; ++k) {
        const int j = sel_idx[beg + k];
        const float w = sel_w[beg + k];
        const float4 *xj = x + (int64_t)j * ld4;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t c = c0 + (int64_t)u * MIX_THREADS;
            if (c < n_vec) {
                float4 v = xj[c];
                if (ORDER == DBW_ORDER_ATC && HAS_G) v = fma4(-lr, g[(int64_t)j * ld4 + c], v);
                acc[u] = fma4(w, v, acc[u]);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t c = c0 + (int64_t)u * MIX_THREADS;
        if (c < n_vec) {
            float4 r = acc[u];
            if (ORDER == DBW_ORDER_CTA && HAS_G) r = fma4(-lr, g[(int64_t)i * ld4 + c], r);
            out[(int64_t)i * ld4 + c] = r;
        }
    }
}

// Scalar columns [c_begin, d): the ragged tail of a row, or everything when rows are
// not 16-byte aligned.  grid = (ceil(cols / 256), N).
template <int ORDER, bool HAS_G>
__global__ __launch_bounds__(256) void mix_csr_scalar(
    int N, int64_t c_begin, int64_t d, int64_t ld, const int32_t *__restrict__ rowptr,
    const int32_t *__restrict__ p, const int32_t *__restrict__ sel_idx,
    const float *__restrict__ sel_w, const float *__restrict__ self_w, const float *__restrict__ x,
    const float *__restrict__ g, float *__restrict__ out, float lr)
{
    const int i = blockIdx.y;
    const int64_t c = c_begin + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= d) return;
    const int beg = rowptr[i], cnt = p[i];
    float v = x[(int64_t)i * ld + c];
    if (ORDER == DBW_ORDER_ATC && HAS_G) v = fmaf(-lr, g[(int64_t)i * ld + c], v);
    float acc = self_w[i] * v;
    for (int k = 0; k < cnt; ++k) {
        const int j = sel_idx[beg + k];
        float vj = x[(int64_t)j * ld + c];
        if (ORDER == DBW_ORDER_ATC && HAS_G) vj = fmaf(-lr, g[(int64_t)j * ld + c], vj);
        acc = fmaf(sel_w[beg + k], vj, acc);
    }
    if (ORDER == DBW_ORDER_CTA && HAS_G) acc = fmaf(-lr, g[(int64_t)i * ld + c], acc);
    out[(int64_t)i * ld + c] = acc;
}

template <int ORDER, bool HAS_G>
int launch_scalar(dbw_ctx *c, const float *x, const float *g, float *out, float lr, int64_t c_begin, hipStream_t s)
{
    const int64_t cols = c->d - c_begin;
    dbw_timer tm(c, "mix_csr_scalar", s);
    hipLaunchKernelGGL((mix_csr_scalar<ORDER, HAS_G>), dim3((unsigned)((cols + 255) / 256), c->N), dim3(256), 0, s,
                       c->N, c_begin, c->d, c->ld, c->rowptr, c->p, c->sel_idx, c->sel_w, c->self_w, x, g, out, lr);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

template <int ORDER, bool HAS_G>
int launch(dbw_ctx *c, const float *x, const float *g, float *out, float lr, hipStream_t s)
{
    constexpr int UNROLL = 2;
    const bool aligned = (c->ld % 4 == 0) && ((uintptr_t)x % 16 == 0) && ((uintptr_t)out % 16 == 0) &&
                         (!HAS_G || (uintptr_t)g % 16 == 0);
    int64_t n_vec = aligned ? c->d / 4 : 0;
    if (n_vec > 0) {
        const int64_t per = (int64_t)MIX_THREADS * UNROLL;
        const int64_t n_chunks = (n_vec + per - 1) / per;
        const int64_t per_xcd = (n_chunks + MIX_XCDS - 1) / MIX_XCDS;
        const int64_t blocks = per_xcd * MIX_XCDS * c->N;
        if (n_chunks > INT32_MAX || blocks > INT32_MAX) return DBW_ERR_UNSUPPORTED;
        dbw_timer tm(c, "mix_csr_vec4", s);
        hipLaunchKernelGGL((mix_csr_vec4<ORDER, HAS_G, UNROLL>), dim3((unsigned)blocks), dim3(MIX_THREADS), 0, s,
                           c->N, n_vec, c->ld / 4, (int)n_chunks, c->rowptr, c->p, c->sel_idx, c->sel_w,
                           c->self_w, (const float4 *)x, (const float4 *)g, (float4 *)out, lr);
        DBW_HIP(hipGetLastError());
    }
    if (n_vec * 4 < c->d) return launch_scalar<ORDER, HAS_G>(c, x, g, out, lr, n_vec * 4, s);
    return DBW_OK;
}

}  // namespace

int dbw_launch_mix_csr(dbw_ctx *c, const float *x, const float *g, float *out, float lr, hipStream_t s)
{
    if (g == nullptr) return launch<DBW_ORDER_CTA, false>(c, x, g, out, lr, s);
    if (c->order == DBW_ORDER_ATC) return launch<DBW_ORDER_ATC, true>(c, x, g, out, lr, s);
    return launch<DBW_ORDER_CTA, true>(c, x, g, out, lr, s);
}

// Scalar evaluation of columns [c_begin, d) only (the ragged tail left by a vector path).
int dbw_launch_mix_csr_range(dbw_ctx *c, const float *x, const float *g, float *out, float lr, int64_t c_begin,
                             hipStream_t s)
{
    if (g == nullptr) return launch_scalar<DBW_ORDER_CTA, false>(c, x, g, out, lr, c_begin, s);
    if (c->order == DBW_ORDER_ATC) return launch_scalar<DBW_ORDER_ATC, true>(c, x, g, out, lr, c_begin, s);
    return launch_scalar<DBW_ORDER_CTA, true>(c, x, g, out, lr, c_begin, s);
}
