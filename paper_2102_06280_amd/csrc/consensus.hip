// Several gradient-free consensus rounds in one pass over the parameters.
//
// Without gradients, r rounds are X' = P(k+r-1) ... P(k+1) P(k) X (rows are workers): the product
// Phi of the consensus matrices (Section 3.1) is N x N, so it is formed first, with one tiny
// kernel per round that applies that round's selected-neighbour lists to the running product, and
// the N x d parameter matrix is then multiplied once on the matrix cores instead of being
// streamed r times.
#include "dbw_internal.h"

namespace {

// Phi = identity on the first N rows, zero elsewhere.  grid = Npad, block = Npad.
__global__ void phi_identity_kernel(int N, int Npad, float *__restrict__ phi)
{
    const int i = blockIdx.x, c = threadIdx.x;
    phi[(size_t)i * Npad + c] = (i == c && i < N) ? 1.0f : 0.0f;
}

// next = P(k) prev with row i of P(k) given by self_w[i] and the first p[i] entries of row i of
// (sel_idx, sel_w), summed in that fixed order.  grid = N, block = Npad.
__global__ void phi_step_kernel(int Npad, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ p,
                                const int32_t *__restrict__ sel_idx, const float *__restrict__ sel_w,
                                const float *__restrict__ self_w, const float *__restrict__ prev,
                                float *__restrict__ next)
{
    __shared__ int32_t s_idx[DBW_DENSE_MAX_N];
    __shared__ float s_w[DBW_DENSE_MAX_N];
    const int i = blockIdx.x, c = threadIdx.x;
    const int beg = rowptr[i], cnt = p[i];
    if (c < cnt) {                                     // cnt <= N - 1 < Npad = blockDim.x
        s_idx[c] = sel_idx[beg + c];
        s_w[c] = sel_w[beg + c];
    }
    __syncthreads();
    float acc = self_w[i] * prev[(size_t)i * Npad + c];
    // the loads of eight neighbours are in flight together; the sum keeps its order
    int k = 0;
    for (; k + 8 <= cnt; k += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = prev[(size_t)s_idx[k + u] * Npad + c];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc = fmaf(s_w[k + u], v[u], acc);
    }
    for (; k < cnt; ++k) acc = fmaf(s_w[k], prev[(size_t)s_idx[k] * Npad + c], acc);
    next[(size_t)i * Npad + c] = acc;
}

// Row-major Phi -> the A-fragment order of the 32x32x2 matrix instruction that the dense mixing
// kernel reads: [row block of 32][k-step][lane], lane = 32 (column & 1) + (row & 31).  Padding
// rows [N, Npad) become zero whatever the buffer holds there.  grid = Npad, block = Npad.
__global__ void phi_fragment_kernel(int N, int Npad, const float *__restrict__ phi, float *__restrict__ frag)
{
    const int i = blockIdx.x, c = threadIdx.x;
    const int KB = Npad / 2;
    frag[((size_t)(i >> 5) * KB + (c >> 1)) * 64 + (c & 1) * 32 + (i & 31)] = i < N ? phi[(size_t)i * Npad + c] : 0.0f;
}

// out[i][c] = sum_j Phi[i][j] x[j][c] for the columns [c_begin, d) that the matrix-core kernel
// leaves out (a ragged tail, or rows that are not 16-byte aligned).  grid = (ceil(cols / 256), N).
__global__ __launch_bounds__(256) void phi_apply_scalar_kernel(int N, int Npad, int64_t c_begin, int64_t d, int64_t ld,
                                                               const float *__restrict__ phi,
                                                               const float *__restrict__ x, float *__restrict__ out)
{
    const int i = blockIdx.y;
    const int64_t c = c_begin + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= d) return;
    float acc = 0.f;
    for (int j = 0; j < N; ++j) acc = fmaf(phi[(size_t)i * Npad + j], x[(int64_t)j * ld + c], acc);
    out[(int64_t)i * ld + c] = acc;
}

}  // namespace

int dbw_launch_consensus_rounds(dbw_ctx *c, const float *x, float *out, const float *t, const int32_t *b, int r,
                                hipStream_t s)
{
    const int Npad = c->Npad;
    float *cur = c->phi[0], *nxt = c->phi[1];
    {
        dbw_timer tm(c, "phi_identity_kernel", s);
        hipLaunchKernelGGL(phi_identity_kernel, dim3(Npad), dim3(Npad), 0, s, c->N, Npad, cur);
        DBW_HIP(hipGetLastError());
    }
    for (int q = 0; q < r; ++q) {
        const int rc = dbw_launch_select(c, t + (size_t)q * c->N, b + (size_t)q * c->N, s);
        if (rc != DBW_OK) return rc;
        dbw_timer tm(c, "phi_step_kernel", s);
        hipLaunchKernelGGL(phi_step_kernel, dim3(c->N), dim3(Npad), 0, s, Npad, c->rowptr, c->p, c->sel_idx, c->sel_w,
                           c->self_w, cur, nxt);
        DBW_HIP(hipGetLastError());
        float *tmp = cur;
        cur = nxt;
        nxt = tmp;
    }
    {
        dbw_timer tm(c, "phi_fragment_kernel", s);
        hipLaunchKernelGGL(phi_fragment_kernel, dim3(Npad), dim3(Npad), 0, s, c->N, Npad, cur, c->phi_frag);
        DBW_HIP(hipGetLastError());
    }
    const int rc = dbw_launch_mix_dense(c, x, nullptr, out, 0.f, nullptr, s, c->phi_frag);
    if (rc != DBW_OK) return rc;
    const int64_t done = dbw_dense_columns(c, x, nullptr, out);
    if (done < c->d) {
        dbw_timer tm(c, "phi_apply_scalar_kernel", s);
        hipLaunchKernelGGL(phi_apply_scalar_kernel, dim3((unsigned)((c->d - done + 255) / 256), c->N), dim3(256), 0, s,
                           c->N, Npad, done, c->d, c->ld, cur, x, out);
        DBW_HIP(hipGetLastError());
    }
    return DBW_OK;
}
