// Mini-batch gradients of fully connected models for all workers at once (Section 2.1,
// stochastic gradient of the local loss; cross-entropy as in Section 5).  Worker w uses
// row w of the parameter matrix and its own batch: every GEMM below is batched over
// workers with per-worker operands.
//
// Parameter row layout: per layer l, W_l [out][in] then b_l [out].
// Scratch per worker: activations a_1..a_L ([B][dims[l]], a_L = logits) followed by the
// deltas dz_1..dz_L of the same shapes.
#include <algorithm>

#include "bgemm.h"
#include "fc_batch32.h"
#include "fc_head.h"
#include "mlp_chain.h"
#include "mlp_thin.h"
#include "mlp_wgrad.h"
#include "dbw_internal.h"

namespace {

using bgemm::Dense;
using bgemm::Epilogue;

// Softmax, mean loss over the batch and its gradient with respect to the logits; one thread per
// sample, grid = (chunks, workers) with 256 samples per workgroup.  Cross-entropy:
// dz = (p - onehot(y)) / B.  MSE on the softmax outputs (Appendix B, 2NN): f = sum_c (p_c - o_c)^2,
// dz_k = 2 p_k ((p_k - o_k) - sum_c p_c (p_c - o_c)) / B.
// The loss of a worker is the sum of its workgroups' partial sums: each writes its own to
// loss_part[worker][chunk] and takes a ticket; the last one to arrive adds them in chunk order (so
// the result does not depend on the order of arrival) and puts the ticket counter back to zero.
template <int LOSS>
__global__ __launch_bounds__(256) void softmax_loss_kernel(
    int B, int C, const float *__restrict__ logits, int64_t stride_logits, const int32_t *__restrict__ y,
    float *__restrict__ dz, int64_t stride_dz, float *__restrict__ loss, float *__restrict__ loss_part,
    uint32_t *__restrict__ ticket, int32_t *__restrict__ err)
{
    __shared__ float red[256];
    const int chunk = blockIdx.x, chunks = gridDim.x, w = blockIdx.y, tid = threadIdx.x;
    const float *z = logits + w * stride_logits;
    float *d = dz + w * stride_dz;
    const float inv_b = 1.0f / (float)B;
    float part = 0.f;
    for (int s = chunk * 256 + tid; s < B; s += chunks * 256) {
        const float *zs = z + (int64_t)s * C;
        float m = zs[0];
        for (int c = 1; c < C; ++c) m = fmaxf(m, zs[c]);
        float sum = 0.f;
        for (int c = 0; c < C; ++c) sum += expf(zs[c] - m);
        int label = y[(int64_t)w * B + s];
        if (label < 0 || label >= C) {                  // clamped for memory safety, reported by dbw_check
            *err = DBW_ERR_INVALID;
            label = label < 0 ? 0 : C - 1;
        }
        const float inv = 1.0f / sum;
        if (LOSS == DBW_LOSS_XENT) {
            for (int c = 0; c < C; ++c)
                d[(int64_t)s * C + c] = (expf(zs[c] - m) * inv - (c == label ? 1.f : 0.f)) * inv_b;
            part += logf(sum) + m - zs[label];
        } else {
            float f = 0.f, inner = 0.f;
            for (int c = 0; c < C; ++c) {
                const float p = expf(zs[c] - m) * inv, e = p - (c == label ? 1.f : 0.f);
                f += e * e;
                inner += p * e;
            }
            for (int c = 0; c < C; ++c) {
                const float p = expf(zs[c] - m) * inv, e = p - (c == label ? 1.f : 0.f);
                d[(int64_t)s * C + c] = 2.f * p * (e - inner) * inv_b;
            }
            part += f;
        }
    }
    if (!loss) return;                                  // uniform: nobody asked for the loss
    red[tid] = part;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (tid < o) red[tid] += red[tid + o];
        __syncthreads();
    }
    if (chunks == 1) {
        if (tid == 0) loss[w] = red[0] * inv_b;
        return;
    }
    if (tid == 0) {
        __hip_atomic_store(&loss_part[w * chunks + chunk], red[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();                                // the partial sum is visible before the ticket is taken
        if (atomicAdd(&ticket[w], 1u) == (uint32_t)(chunks - 1)) {
            __threadfence();
            float sum = 0.f;
            for (int k = 0; k < chunks; ++k)
                sum += __hip_atomic_load(&loss_part[w * chunks + k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            loss[w] = sum * inv_b;
            ticket[w] = 0;                              // ready for the next launch
        }
    }
}

// Bias gradient: db[o] = sum over the batch of dz[s][o].  grid = (ceil(C / 32), workers); a
// workgroup covers 32 columns with RG groups of 32 threads that stride over the batch, four
// independent partial sums each, combined in a fixed order.
template <int RG>
__global__ __launch_bounds__(32 * RG) void colsum_kernel(int B, int C, const float *__restrict__ dz, int64_t stride_dz,
                                                         float *__restrict__ db, int64_t stride_db)
{
    __shared__ float part[RG][32];
    const int w = blockIdx.y, cl = threadIdx.x & 31, rg = threadIdx.x >> 5;
    const int o = blockIdx.x * 32 + cl;
    const float *d = dz + w * stride_dz;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (o < C) {
        int b = rg;
        for (; b + 3 * RG < B; b += 4 * RG) {
            s0 += d[(int64_t)b * C + o];
            s1 += d[(int64_t)(b + RG) * C + o];
            s2 += d[(int64_t)(b + 2 * RG) * C + o];
            s3 += d[(int64_t)(b + 3 * RG) * C + o];
        }
        for (; b < B; b += RG) s0 += d[(int64_t)b * C + o];
    }
    part[rg][cl] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (rg == 0 && o < C) {
        float s = part[0][cl];
        for (int r = 1; r < RG; ++r) s += part[r][cl];
        db[w * stride_db + o] = s;
    }
}

// Partial sums of a split-k forward GEMM: part[worker][split][m][n].
struct SplitOut {
    float *part;
    int64_t stride;
    int M, N;
    __device__ __forceinline__ void store(int w, int split, int m, int n, float v) const
    {
        part[w * stride + ((int64_t)split * M + m) * N + n] = v;
    }
};

// C[m][n] = act(sum over splits of part[split][m][n] + bias[n]) (bias may be NULL); grid = (ceil(M N / 256), workers).
__global__ __launch_bounds__(256) void fc_reduce_kernel(const float *__restrict__ part, int64_t pstride, int splits,
                                                        int M, int N, const float *__restrict__ bias,
                                                        int64_t bias_stride, int relu, float *__restrict__ C,
                                                        int64_t ldc, int64_t cstride)
{
    const int w = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    if (i >= M * N) return;
    const int m = i / N, n = i - m * N;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp) s += part[w * pstride + (int64_t)sp * M * N + i];
    if (bias) s += bias[w * bias_stride + n];
    if (relu) s = s > 0.f ? s : 0.f;
    C[w * cstride + (int64_t)m * ldc + n] = s;
}

// A long reduction with few output tiles (e.g. batch 32 x 512 outputs over k = 4096, or any
// small model) leaves most of the chip idle and each workgroup waiting on its own chain of
// loads; split k then, up to MAX_SPLITS ways, keeping at least two k-steps per split.
constexpr int MAX_SPLITS = 16;          // partial-sum slots per output in the scratch block
constexpr int GEMM_MAX_SPLITS = 8;
int forward_splits(int M, int N, int K, int workers)
{
    const int64_t tiles = (int64_t)((M + 63) / 64) * ((N + 63) / 64) * workers;
    int splits = 1;
    while (splits < GEMM_MAX_SPLITS && tiles * splits < 640 && K / (splits * 2) >= 2 * bgemm::BK) splits *= 2;
    return splits;
}

// The streaming kernels for a batch of exactly 32 apply to a layer in -> out when the shapes
// divide evenly and every operand row starts on a 16-byte boundary.
bool batch32_layer(int B, int in, int out, int64_t ld_params, int64_t w_off, const float *params, const float *grads)
{
    return B == 32 && in % 512 == 0 && out % 32 == 0 && ld_params % 4 == 0 && w_off % 4 == 0 &&
           fc32::aligned16(params) && fc32::aligned16(grads);
}

// The fused classifier head (fc_head.h) takes the last layer when it is narrow enough.
struct HeadPlan {
    bool use;
    int chunks, S;
    int64_t part;          // floats of partial sums per worker
};
HeadPlan head_plan(int L, const int32_t *dims, int B, int workers)
{
    const int H = dims[L - 1], C = dims[L];
    HeadPlan hp{false, 0, 0, 0};
    if (C > fchead::MAX_C || fchead::lds_bytes(H, C, 16) > fchead::LDS_LIMIT) return hp;
    auto fits = [&](int S) { return fchead::lds_bytes(H, C, S) <= fchead::LDS_LIMIT; };
    int S;
    const int whole = B <= 16 ? 16 : (B <= 32 ? 32 : 64);
    if (B <= 64 && fits(whole))
        S = whole;                                   // one chunk per worker: no partial sums at all
    else                                             // 32 samples per workgroup when that still fills the chip, else 16
        S = (fits(32) && (int64_t)((B + 31) / 32) * workers >= 256) ? 32 : 16;
    const int chunks = (B + S - 1) / S;
    if (chunks > fchead::MAX_CHUNKS) return hp;
    hp.use = true;
    hp.chunks = chunks;
    hp.S = S;
    hp.part = chunks > 1 ? (int64_t)chunks * fchead::partial_floats(H, C, L > 1) : 0;
    return hp;
}

// The whole chain of layers in one launch (mlp_chain.h) applies to equal hidden widths of 128, 256 or 512, an
// input width that divides by 16, at most 16 classes, and operands on 16-byte boundaries.  S = samples per
// workgroup: the one that needs the least time when every CU takes one workgroup at a time (ties: the larger).
struct ChainPlan {
    bool use;
    int S, chunks;
    size_t lds;
};
ChainPlan chain_plan(int L, const int32_t *dims, int B, int workers, int grad_path)
{
    ChainPlan cp{false, 0, 0, 0};
    if (grad_path == DBW_GRAD_LAYERS || L < 2 || L > mlpchain::MAX_L || dims[L] > fchead::MAX_C) return cp;
    const int H = dims[1];
    if (H != 128 && H != 256 && H != 512) return cp;
    for (int l = 2; l < L; ++l)
        if (dims[l] != H) return cp;
    if (dims[0] % 16 != 0 || dims[0] <= 0) return cp;
    int64_t best = 0;
    for (int S = 64; S >= 16; S -= 16) {
        if (mlpchain::lds_bytes(dims[0], H, dims[L], S, L) > fchead::LDS_LIMIT) continue;
        const int chunks = (B + S - 1) / S;
        if (chunks > fchead::MAX_CHUNKS) continue;
        const int64_t cost = ((int64_t)chunks * workers + 255) / 256 * S;
        if (cp.S == 0 || cost < best) {
            best = cost;
            cp.S = S;
            cp.chunks = chunks;
        }
    }
    if (cp.S == 0) return cp;
    // worth it when the workgroups keep at least half of the chip busy; otherwise the layered path, which
    // splits its products over all CUs, wins
    if (grad_path != DBW_GRAD_CHAIN && (int64_t)B * workers * 2 < best * 256) return cp;
    cp.lds = mlpchain::lds_bytes(dims[0], H, dims[L], cp.S, L);
    cp.use = true;
    return cp;
}

// Weight and bias gradients of layers 1 .. layers in one launch (mlp_wgrad.h), from the deltas and activations
// in the workers' scratch blocks; extra workgroups add the head's per-chunk sums when it has any.
struct WgradPlan {
    int layers;                 // dW_l and db_l for l = 1 .. layers
    bool last_db;               // false: somebody else (the head) computes db of layer `layers`
    const int64_t *a_off, *dz_off, *w_off;
    int64_t w_end;              // end of b_layers in the parameter row
    int64_t per, split_floats;
};
int launch_grouped_wgrad(dbw_ctx *c, const dbw_fc_args &a, const WgradPlan &wp, const fchead::Args &h, int head_chunks,
                         hipStream_t s)
{
    const int B = a.B, N = c->N;
    const int32_t *dims = a.dims;
    const int64_t wstride = a.act_stride;
    mlpwgrad::Args q{};
    q.B = B; q.layers = wp.layers; q.workers = N;
    // 64 x 64 tiles when they alone give every CU two workgroups, else 64 x 32; if that still leaves CUs idle, the
    // batch is split as well (partial tiles to scratch, one more launch to add them)
    auto count_tiles = [&](int tm, int tn, int *begin) {
        int t = 0;
        for (int l = 1; l <= wp.layers; ++l) {
            if (begin) begin[l] = t;
            t += ((dims[l] + tm - 1) / tm) * ((dims[l - 1] + tn - 1) / tn);
        }
        if (begin) begin[wp.layers + 1] = t;
        return t;
    };
    const bool thin = B <= mlpthin::MAX_B;        // one wavefront per 32 x 64 tile, no split (mlp_thin.h)
    const int tn = !thin && (int64_t)count_tiles(64, 64, nullptr) * N >= 512 ? 64 : 32;
    const int tiles = thin ? count_tiles(mlpthin::WG_TM, mlpthin::WG_TN, q.tile_begin) : count_tiles(64, tn, q.tile_begin);
    for (int l = 1; l <= wp.layers; ++l) {
        q.n_rows[l] = dims[l];
        q.n_cols[l] = dims[l - 1];
        q.want_db[l] = l < wp.layers || wp.last_db;
        q.dz_off[l] = wp.dz_off[l];
        q.a[l] = l == 1 ? a.in : a.act + wp.a_off[l - 1];
        q.a_ld[l] = l == 1 ? a.in_ld : dims[l - 1];
        q.a_stride[l] = l == 1 ? a.in_stride : wstride;
        q.w_off[l] = wp.w_off[l];
    }
    q.w_off[wp.layers + 1] = wp.w_end;
    q.dz = a.act; q.dz_stride = wstride;
    q.grads = a.grads; q.g_stride = c->ld;
    q.part = a.act + 2 * wp.per; q.part_stride = wstride;
    const int64_t len = wp.w_end - wp.w_off[1];
    int splits = (int)std::min<int64_t>(8, std::max<int64_t>(1, 512 / ((int64_t)tiles * N)));
    splits = std::min(splits, (B + 63) / 64);
    splits = (int)std::min<int64_t>(splits, std::max<int64_t>(1, wp.split_floats / len));
    if (thin) splits = 1;
    q.splits = splits;
    q.kper = ((B + splits - 1) / splits + 15) / 16 * 16;
    const int head_blocks = head_chunks > 1 ? (int)((fchead::partial_floats(h.H, h.C, h.bprev_off >= 0) + 255) / 256) : 0;
    {
        dbw_timer tm(c, "mlp_wgrad_kernel", s);
        auto whole_xcds = [](int n) { return (n + mlpwgrad::XCDS - 1) / mlpwgrad::XCDS * mlpwgrad::XCDS; };
        const int tile_wgs = thin ? (tiles * N + mlpwgrad::WAVES - 1) / mlpwgrad::WAVES : tiles * N * splits;
        const dim3 grid(whole_xcds(head_blocks * N) + whole_xcds(tile_wgs));
        if (thin && B <= 16)
            hipLaunchKernelGGL(mlpthin::wgrad_kernel<4>, grid, dim3(mlpwgrad::THREADS), 0, s, q, h, head_chunks, head_blocks);
        else if (thin && B <= 32)
            hipLaunchKernelGGL(mlpthin::wgrad_kernel<8>, grid, dim3(mlpwgrad::THREADS), 0, s, q, h, head_chunks, head_blocks);
        else if (thin)
            hipLaunchKernelGGL(mlpthin::wgrad_kernel<16>, grid, dim3(mlpwgrad::THREADS), 0, s, q, h, head_chunks, head_blocks);
        else if (tn == 64)
            hipLaunchKernelGGL(mlpwgrad::kernel<4>, grid, dim3(mlpwgrad::THREADS), 0, s, q, h, head_chunks, head_blocks);
        else
            hipLaunchKernelGGL(mlpwgrad::kernel<2>, grid, dim3(mlpwgrad::THREADS), 0, s, q, h, head_chunks, head_blocks);
        DBW_HIP(hipGetLastError());
    }
    if (splits > 1) {
        dbw_timer tm(c, "mlp_reduce_kernel", s);
        hipLaunchKernelGGL(mlpwgrad::reduce_kernel, dim3((unsigned)((len / 4 + 255) / 256), N), dim3(256), 0, s, q);
        DBW_HIP(hipGetLastError());
    }
    return DBW_OK;
}

int64_t act_floats(int L, const int32_t *dims, int B)
{
    int64_t n = 0;
    for (int l = 1; l <= L; ++l) n += (int64_t)B * dims[l];
    return (n + 3) / 4 * 4;          // the deltas and the partial sums behind them keep the 16-byte alignment
}

}  // namespace

int64_t dbw_fc_scratch_per_worker(int L, const int32_t *dims, int B)
{
    int64_t part = 0;
    for (int l = 1; l <= L; ++l) part = std::max<int64_t>(part, (int64_t)MAX_SPLITS * B * dims[l]);
    part = (part + 3) / 4 * 4;
    if (dims[L] <= fchead::MAX_C)      // partial sums of the fused head, at its smaller chunk size, behind the split partials
        part += (int64_t)((B + 15) / 16) * fchead::partial_floats(dims[L - 1], dims[L], L > 1);
    return 2 * act_floats(L, dims, B) + (part + 3) / 4 * 4;
}

bool dbw_fc_chain_shape_ok(int L, const int32_t *dims, int B, int workers)
{
    return chain_plan(L, dims, B, workers, DBW_GRAD_CHAIN).use;
}

// Forward and backward pass of a stack of fully connected layers for all workers.
int dbw_fc_forward_backward(dbw_ctx *c, const dbw_fc_args &a, hipStream_t s)
{
    const int L = a.L, B = a.B, N = c->N;
    const int32_t *dims = a.dims;
    const int64_t per = act_floats(L, dims, B), wstride = a.act_stride;
    // offsets inside a worker's scratch block and parameter row
    int64_t a_off[9], dz_off[9], w_off[9], b_off[9];
    int64_t ao = 0, po = a.param_off;
    for (int l = 1; l <= L; ++l) {
        a_off[l] = ao;
        dz_off[l] = per + ao;
        ao += (int64_t)B * dims[l];
        w_off[l] = po;
        b_off[l] = po + (int64_t)dims[l] * dims[l - 1];
        po = b_off[l] + dims[l];
    }
    float *act = a.act;
    const float *params = a.params;
    float *grads = a.grads;

    HeadPlan head = head_plan(L, dims, B, N);
    ChainPlan chain = chain_plan(L, dims, B, N, a.grad_path);
    if (chain.use && !(a.din == nullptr && a.in_ld % 4 == 0 && a.in_stride % 4 == 0 && fc32::aligned16(a.in) &&
                       fc32::aligned16(params) && c->ld % 4 == 0 && a.param_off % 4 == 0 && fc32::aligned16(act) &&
                       wstride % 4 == 0 && per % 4 == 0))
        chain.use = false;
    if (a.grad_path == DBW_GRAD_CHAIN && !chain.use) return DBW_ERR_UNSUPPORTED;
    if (chain.use) {      // the head runs inside the chain, on the chain's chunks
        head.use = true;
        head.S = chain.S;
        head.chunks = chain.chunks;
    }
    const int L_gemm = chain.use ? 0 : (head.use ? L - 1 : L);         // layers that go through the forward GEMM kernels
    // The output of layer L - 1 feeds nothing but the head.  When its forward product is split along k, the
    // head sums the partial products itself (same order, then bias and ReLU) and the reduction launch is saved.
    int head_splits = 0;
    const bool head_can_sum = head.use && L >= 2 && dims[L - 1] % 4 == 0 && b_off[L - 1] % 4 == 0 && c->ld % 4 == 0 &&
                              fc32::aligned16(params) && wstride % 4 == 0 && fc32::aligned16(act) && (2 * per) % 4 == 0;

    // forward: a_l = relu(a_{l-1} W_l^T + b_l), no ReLU on the logits
    for (int l = 1; l <= L_gemm; ++l) {
        Dense<true> A, Bm;
        if (l == 1)
            A = {a.in, a.in_ld, a.in_stride};
        else
            A = {act + a_off[l - 1], dims[l - 1], wstride};
        Bm = {params + w_off[l], dims[l - 1], c->ld};
        if (batch32_layer(B, dims[l - 1], dims[l], c->ld, w_off[l], params, grads) && A.ld % 4 == 0 &&
            A.stride % 4 == 0 && fc32::aligned16(A.p) && wstride % 4 == 0 && a_off[l] % 4 == 0 && fc32::aligned16(act)) {
            const int slices = dims[l - 1] / fc32::KSLICE, nf = dims[l] / 128;
            if (dims[l] % 128 == 0 && nf <= 4 && slices <= MAX_SPLITS) {      // split along k, inputs read once
                float *part = act + 2 * per;
                {
                    dbw_timer tm(c, "fc32_forward", s);
                    const dim3 grid(slices, N), block(fc32::THREADS);
                    const float *Wl = params + w_off[l];
                    auto go = [&](auto kern) {
                        hipLaunchKernelGGL(kern, grid, block, 0, s, dims[l - 1], A.p, A.ld, A.stride, Wl, c->ld, part,
                                           wstride);
                    };
                    switch (nf) {
                    case 1: go(fc32::forward_ksplit_kernel<1>); break;
                    case 2: go(fc32::forward_ksplit_kernel<2>); break;
                    case 3: go(fc32::forward_ksplit_kernel<3>); break;
                    default: go(fc32::forward_ksplit_kernel<4>); break;
                    }
                    DBW_HIP(hipGetLastError());
                }
                if (head_can_sum && l == L - 1 && slices <= 16) {
                    head_splits = slices;
                    continue;
                }
                dbw_timer tm(c, "fc_reduce_kernel", s);
                hipLaunchKernelGGL(fc_reduce_kernel, dim3((B * dims[l] + 255) / 256, N), dim3(256), 0, s, part, wstride,
                                   slices, B, dims[l], params + b_off[l], c->ld, l < L ? 1 : 0, act + a_off[l],
                                   (int64_t)dims[l], wstride);
                DBW_HIP(hipGetLastError());
                continue;
            }
            const int blocks = (N + fc32::XCDS - 1) / fc32::XCDS * fc32::XCDS * (dims[l] / 32);
            dbw_timer tm(c, "fc32_forward", s);
            hipLaunchKernelGGL(fc32::forward_kernel, dim3(blocks), dim3(fc32::THREADS), 0, s, N, dims[l], dims[l - 1],
                               A.p, A.ld, A.stride, params + w_off[l], c->ld, params + b_off[l], c->ld, l < L ? 1 : 0,
                               act + a_off[l], (int64_t)dims[l], wstride);
            DBW_HIP(hipGetLastError());
            continue;
        }
        // short batches: operands straight from global memory into matrix-instruction fragments (mlp_thin.h)
        if (a.grad_path == DBW_GRAD_AUTO && B <= mlpthin::MAX_B && dims[l - 1] % 4 == 0 && dims[l] % 4 == 0 &&
            A.ld % 4 == 0 && A.stride % 4 == 0 && fc32::aligned16(A.p) && fc32::aligned16(params) && c->ld % 4 == 0 &&
            w_off[l] % 4 == 0 && fc32::aligned16(act) && wstride % 4 == 0 && a_off[l] % 4 == 0) {
            mlpthin::FwdArgs f{};
            f.B = B; f.K = dims[l - 1]; f.N = dims[l]; f.workers = N; f.relu = l < L ? 1 : 0;
            f.a = A.p; f.a_ld = A.ld; f.a_stride = A.stride;
            f.params = params; f.p_stride = c->ld; f.w_off = w_off[l]; f.b_off = b_off[l];
            f.out = act + a_off[l]; f.out_stride = wstride;
            const int wgs = (dims[l] + 16 * mlpthin::FWD_CB - 1) / (16 * mlpthin::FWD_CB) * N;
            const dim3 grid((wgs + mlpthin::XCDS - 1) / mlpthin::XCDS * mlpthin::XCDS), block(mlpthin::FWD_THREADS);
            dbw_timer tm(c, "mlp_thin_forward", s);
            switch ((B + 15) / 16) {
            case 1: hipLaunchKernelGGL(mlpthin::forward_kernel<1>, grid, block, 0, s, f); break;
            case 2: hipLaunchKernelGGL(mlpthin::forward_kernel<2>, grid, block, 0, s, f); break;
            case 3: hipLaunchKernelGGL(mlpthin::forward_kernel<3>, grid, block, 0, s, f); break;
            default: hipLaunchKernelGGL(mlpthin::forward_kernel<4>, grid, block, 0, s, f); break;
            }
            DBW_HIP(hipGetLastError());
            continue;
        }
        const int splits = forward_splits(B, dims[l], dims[l - 1], N);
        if (splits > 1) {
            float *part = act + 2 * per;
            {
                dbw_timer tm(c, "mlp_forward_gemm", s);
                DBW_HIP(bgemm::launch<64>(A, Bm, SplitOut{part, wstride, B, dims[l]}, B, dims[l], dims[l - 1], N, s,
                                          splits));
            }
            if (head_can_sum && l == L - 1) {
                head_splits = splits;
                continue;
            }
            dbw_timer tm(c, "fc_reduce_kernel", s);
            hipLaunchKernelGGL(fc_reduce_kernel, dim3((B * dims[l] + 255) / 256, N), dim3(256), 0, s, part, wstride,
                               splits, B, dims[l], params + b_off[l], c->ld, l < L ? 1 : 0, act + a_off[l],
                               (int64_t)dims[l], wstride);
            DBW_HIP(hipGetLastError());
            continue;
        }
        Epilogue E{act + a_off[l], dims[l], wstride, params + b_off[l], c->ld, nullptr, 0, 0, l < L ? 1 : 0};
        dbw_timer tm(c, "mlp_forward_gemm", s);
        DBW_HIP(bgemm::launch<64>(A, Bm, E, B, dims[l], dims[l - 1], N, s));
    }
    // Weight gradients of the layers the GEMM kernels would take: all of them in one launch when the library may
    // choose and every operand allows 128-bit accesses.  Batches of 256 and more: mlp_wgrad.h, four wavefronts per
    // tile, which share the samples.  Batches of at most 64: mlp_thin.h, a tile per wavefront.  In between the GEMM
    // kernel, whose wavefronts share the tile, stays (784-200-10 with 64 samples on 32 workers: the four-wavefront
    // kernel 26 us, the GEMM kernel 21 us, a tile per wavefront 18 us).  The batch-32 streaming kernels keep their layers.
    const int Lw = head.use ? L - 1 : L;
    bool grouped = !chain.use && a.grad_path == DBW_GRAD_AUTO && Lw >= 1 && (B >= 256 || B <= mlpthin::MAX_B) &&
                   a.in_ld % 4 == 0 && a.in_stride % 4 == 0 && fc32::aligned16(a.in) && fc32::aligned16(grads) &&
                   c->ld % 4 == 0 && a.param_off % 4 == 0 && fc32::aligned16(act) && wstride % 4 == 0;
    for (int l = 0; l <= Lw && grouped; ++l) grouped = dims[l] % 4 == 0;
    for (int l = 1; l <= Lw && grouped; ++l)
        grouped = !batch32_layer(B, dims[l - 1], dims[l], c->ld, w_off[l], params, grads);
    // A short batch is one chunk of the head per worker, so that its sums over the batch are final.  When the grouped
    // launch follows, which adds per-chunk sums on the side, smaller chunks cost nothing and put the head on more CUs
    // (784-200-10, 64 samples, 32 workers: 16.1 -> 10.9 us with four chunks of 16).
    if (grouped && head.use && B <= 64)
        while (head.S > 16 && (int64_t)head.chunks * N < 256) {
            head.S /= 2;
            head.chunks = (B + head.S - 1) / head.S;
        }
    int64_t split_floats = 0;                            // the split partials of the layers, which the head's own follow
    for (int q = 1; q <= L; ++q) split_floats = std::max<int64_t>(split_floats, (int64_t)MAX_SPLITS * B * dims[q]);
    fchead::Args h{};
    if (head.use) {
        // last layer, loss and its whole backward pass in one launch (with the chain: the layers below as well)
        h.B = B; h.H = dims[L - 1]; h.C = dims[L]; h.S = head.S;
        if (L == 1) {
            h.a = a.in; h.a_ld = a.in_ld; h.a_stride = a.in_stride;
            h.da = a.din; h.da_ld = a.din_ld; h.da_stride = a.din_stride;
            h.mask = 0;
            h.bprev_off = -1;
        } else {
            h.a = act + a_off[L - 1]; h.a_ld = dims[L - 1]; h.a_stride = wstride;
            if (head_splits > 0) {      // partial products [split][B][H] instead of the finished activations
                h.a = act + 2 * per;
                h.splits = head_splits;
                h.in_bias_off = b_off[L - 1];
            }
            h.da = act + dz_off[L - 1]; h.da_ld = dims[L - 1]; h.da_stride = wstride;
            h.mask = 1;
            h.bprev_off = b_off[L - 1];
        }
        h.params = params; h.grads = grads; h.p_stride = c->ld; h.w_off = w_off[L]; h.b_off = b_off[L];
        h.y = a.y; h.loss = a.loss;
        h.part = act + 2 * per + (split_floats + 3) / 4 * 4; h.part_stride = wstride;
        h.err = c->err;
        if (chain.use) {
            mlpchain::Args g{};
            g.B = B; g.L = L; g.K0 = dims[0]; g.H = dims[1]; g.C = dims[L];
            g.chunks = chain.chunks; g.workers = N; g.loss_kind = a.loss_kind;
            g.x = a.in; g.x_ld = a.in_ld; g.x_stride = a.in_stride;
            g.params = params; g.p_stride = c->ld;
            g.act = act; g.act_stride = wstride;
            for (int l = 1; l <= L; ++l) {
                g.w_off[l] = w_off[l]; g.b_off[l] = b_off[l]; g.a_off[l] = a_off[l]; g.dz_off[l] = dz_off[l];
            }
            h.a = nullptr; h.da = nullptr;
            g.head = h;
            const int total = chain.chunks * N;
            const dim3 grid((total + mlpchain::XCDS - 1) / mlpchain::XCDS * mlpchain::XCDS);
            auto go = [&](auto kern) -> int {
                dbw_timer tm(c, "mlp_chain_kernel", s);
                hipLaunchKernelGGL(kern, grid, dim3(mlpchain::THREADS), chain.lds, s, g);
                DBW_HIP(hipGetLastError());
                return DBW_OK;
            };
            const int rb = chain.S / 16, cb = dims[1] / 128;
            int rc = DBW_ERR_UNSUPPORTED;
            switch (rb * 8 + cb) {
            case 1 * 8 + 1: rc = go(mlpchain::kernel<1, 1>); break;
            case 1 * 8 + 2: rc = go(mlpchain::kernel<1, 2>); break;
            case 1 * 8 + 4: rc = go(mlpchain::kernel<1, 4>); break;
            case 2 * 8 + 1: rc = go(mlpchain::kernel<2, 1>); break;
            case 2 * 8 + 2: rc = go(mlpchain::kernel<2, 2>); break;
            case 2 * 8 + 4: rc = go(mlpchain::kernel<2, 4>); break;
            case 3 * 8 + 1: rc = go(mlpchain::kernel<3, 1>); break;
            case 3 * 8 + 2: rc = go(mlpchain::kernel<3, 2>); break;
            case 3 * 8 + 4: rc = go(mlpchain::kernel<3, 4>); break;
            case 4 * 8 + 1: rc = go(mlpchain::kernel<4, 1>); break;
            case 4 * 8 + 2: rc = go(mlpchain::kernel<4, 2>); break;
            case 4 * 8 + 4: rc = go(mlpchain::kernel<4, 4>); break;
            }
            if (rc != DBW_OK) return rc;

            // weight and bias gradients of the layers below the head, and the head's per-chunk sums
            const WgradPlan wp{L - 1, false, a_off, dz_off, w_off, w_off[L], per, split_floats};
            const int rc2 = launch_grouped_wgrad(c, a, wp, h, head.chunks, s);
            if (rc2 != DBW_OK) return rc2;
            return DBW_OK;
        } else {
        const dim3 grid(head.chunks, N);
        const size_t lds = fchead::lds_bytes(h.H, h.C, h.S);
        const bool vec = h.H % 4 == 0 && h.a_ld % 4 == 0 && h.a_stride % 4 == 0 && (uintptr_t)h.a % 16 == 0;
        const bool mse = a.loss_kind == DBW_LOSS_MSE;
        auto go = [&](auto kern) -> int {
            dbw_timer tm(c, "fc_head_kernel", s);
            hipLaunchKernelGGL(kern, grid, dim3(fchead::THREADS), lds, s, h);
            DBW_HIP(hipGetLastError());
            return DBW_OK;
        };
        int rc;
        if (head_splits > 0) rc = mse ? go(fchead::kernel<DBW_LOSS_MSE, true, true>) : go(fchead::kernel<DBW_LOSS_XENT, true, true>);
        else if (mse) rc = vec ? go(fchead::kernel<DBW_LOSS_MSE, true>) : go(fchead::kernel<DBW_LOSS_MSE, false>);
        else rc = vec ? go(fchead::kernel<DBW_LOSS_XENT, true>) : go(fchead::kernel<DBW_LOSS_XENT, false>);
        if (rc != DBW_OK) return rc;
        }
        if (head.chunks > 1 && !grouped) {          // (the grouped weight-gradient launch adds them otherwise)
            const int64_t E = fchead::partial_floats(h.H, h.C, L > 1);
            dbw_timer tm(c, "fc_head_reduce", s);
            hipLaunchKernelGGL(fchead::reduce_kernel, dim3((unsigned)((E + 255) / 256), N), dim3(256), 0, s, h, head.chunks);
            DBW_HIP(hipGetLastError());
        }
    } else {
        const int chunks = std::min((B + 255) / 256, DBW_LOSS_CHUNKS);
        const dim3 grid(chunks, N);
        dbw_timer tm(c, "softmax_loss_kernel", s);
        if (a.loss_kind == DBW_LOSS_MSE)
            hipLaunchKernelGGL(softmax_loss_kernel<DBW_LOSS_MSE>, grid, dim3(256), 0, s, B, dims[L], act + a_off[L], wstride,
                               a.y, act + dz_off[L], wstride, a.loss, c->loss_part, c->loss_ticket, c->err);
        else
            hipLaunchKernelGGL(softmax_loss_kernel<DBW_LOSS_XENT>, grid, dim3(256), 0, s, B, dims[L], act + a_off[L], wstride,
                               a.y, act + dz_off[L], wstride, a.loss, c->loss_part, c->loss_ticket, c->err);
        DBW_HIP(hipGetLastError());
    }
    // backward
    for (int l = Lw; l >= 1; --l) {
        const bool fast = batch32_layer(B, dims[l - 1], dims[l], c->ld, w_off[l], params, grads) && wstride % 4 == 0 &&
                          dz_off[l] % 4 == 0 && fc32::aligned16(act);
        if (!grouped) {   // dW_l = dz_l^T a_{l-1}
            Dense<false> A{act + dz_off[l], dims[l], wstride}, Bm;
            if (l == 1)
                Bm = {a.in, a.in_ld, a.in_stride};
            else
                Bm = {act + a_off[l - 1], dims[l - 1], wstride};
            if (fast && Bm.ld % 4 == 0 && Bm.stride % 4 == 0 && fc32::aligned16(Bm.p)) {
                dbw_timer tm(c, "fc32_wgrad", s);
                hipLaunchKernelGGL(fc32::wgrad_kernel, dim3(dims[l - 1] / 512, dims[l] / 32, N), dim3(fc32::THREADS), 0, s,
                                   dims[l], dims[l - 1], act + dz_off[l], (int64_t)dims[l], wstride, Bm.p, Bm.ld, Bm.stride,
                                   grads + w_off[l], c->ld);
                DBW_HIP(hipGetLastError());
            } else {
                // few output tiles and a long batch: split the reduction like the forward pass does
                int splits = forward_splits(dims[l], dims[l - 1], B, N);
                int64_t part_cap = 0;
                for (int q = 1; q <= L; ++q) part_cap = std::max<int64_t>(part_cap, (int64_t)MAX_SPLITS * B * dims[q]);
                if ((int64_t)splits * dims[l] * dims[l - 1] > part_cap) splits = 1;
                if (splits > 1) {
                    float *part = act + 2 * per;
                    {
                        dbw_timer tm(c, "mlp_wgrad_gemm", s);
                        DBW_HIP(bgemm::launch<64>(A, Bm, SplitOut{part, wstride, dims[l], dims[l - 1]}, dims[l], dims[l - 1],
                                                  B, N, s, splits));
                    }
                    dbw_timer tm(c, "fc_reduce_kernel", s);
                    hipLaunchKernelGGL(fc_reduce_kernel, dim3((dims[l] * dims[l - 1] + 255) / 256, N), dim3(256), 0, s, part,
                                       wstride, splits, dims[l], dims[l - 1], (const float *)nullptr, (int64_t)0, 0,
                                       grads + w_off[l], (int64_t)dims[l - 1], c->ld);
                    DBW_HIP(hipGetLastError());
                } else {
                    Epilogue E{grads + w_off[l], dims[l - 1], c->ld, nullptr, 0, nullptr, 0, 0, 0};
                    dbw_timer tm(c, "mlp_wgrad_gemm", s);
                    DBW_HIP(bgemm::launch<64>(A, Bm, E, dims[l], dims[l - 1], B, N, s));
                }
            }
        }
        if (!grouped && !(head.use && l == L - 1)) {       // the head has written the bias gradient of the layer below it
            dbw_timer tm(c, "colsum_kernel", s);
            if (B >= 512)    // long batches: 32 row groups per workgroup
                hipLaunchKernelGGL(colsum_kernel<32>, dim3((dims[l] + 31) / 32, N), dim3(1024), 0, s, B, dims[l],
                                   act + dz_off[l], wstride, grads + b_off[l], c->ld);
            else
                hipLaunchKernelGGL(colsum_kernel<8>, dim3((dims[l] + 31) / 32, N), dim3(256), 0, s, B, dims[l],
                                   act + dz_off[l], wstride, grads + b_off[l], c->ld);
            DBW_HIP(hipGetLastError());
        }
        if (l > 1 && fast && a_off[l - 1] % 4 == 0 && dz_off[l - 1] % 4 == 0) {
            dbw_timer tm(c, "fc32_dgrad", s);
            hipLaunchKernelGGL(fc32::dgrad_kernel<4>, dim3(dims[l - 1] / 128, N), dim3(fc32::THREADS), 0, s, dims[l],
                               dims[l - 1], act + dz_off[l], (int64_t)dims[l], wstride, params + w_off[l], c->ld,
                               act + a_off[l - 1], (int64_t)dims[l - 1], wstride, act + dz_off[l - 1],
                               (int64_t)dims[l - 1], wstride);
            DBW_HIP(hipGetLastError());
        } else if (l == 1 && a.din && fast && a.din_ld % 4 == 0 && a.din_stride % 4 == 0 && fc32::aligned16(a.din)) {
            dbw_timer tm(c, "fc32_dgrad", s);
            hipLaunchKernelGGL(fc32::dgrad_kernel<1>, dim3(dims[0] / 512, N), dim3(fc32::THREADS), 0, s, dims[1], dims[0],
                               act + dz_off[1], (int64_t)dims[1], wstride, params + w_off[1], c->ld,
                               (const float *)nullptr, (int64_t)0, (int64_t)0, a.din, a.din_ld, a.din_stride);
            DBW_HIP(hipGetLastError());
        } else if (l > 1) {   // dz_{l-1} = (dz_l W_l) masked by a_{l-1} > 0
            Dense<true> A{act + dz_off[l], dims[l], wstride};
            Dense<false> Bm{params + w_off[l], dims[l - 1], c->ld};
            Epilogue E{act + dz_off[l - 1], dims[l - 1], wstride, nullptr, 0, act + a_off[l - 1], dims[l - 1],
                       wstride, 0};
            dbw_timer tm(c, "mlp_dgrad_gemm", s);
            DBW_HIP(bgemm::launch<64>(A, Bm, E, B, dims[l - 1], dims[l], N, s));
        } else if (a.din) {   // gradient with respect to the stack's input, unmasked
            Dense<true> A{act + dz_off[1], dims[1], wstride};
            Dense<false> Bm{params + w_off[1], dims[0], c->ld};
            Epilogue E{a.din, a.din_ld, a.din_stride, nullptr, 0, nullptr, 0, 0, 0};
            dbw_timer tm(c, "mlp_dgrad_gemm", s);
            DBW_HIP(bgemm::launch<64>(A, Bm, E, B, dims[0], dims[1], N, s));
        }
    }
    if (grouped) {
        const WgradPlan wp{Lw, !head.use, a_off, dz_off, w_off, b_off[Lw] + dims[Lw], per, split_floats};
        return launch_grouped_wgrad(c, a, wp, h, head.use ? head.chunks : 1, s);
    }
    return DBW_OK;
}

// The fused head uses up to 159 KB of dynamic LDS: allow that once, at create, so that no
// attribute call falls into a stream capture of the first round.
int dbw_fc_prepare()
{
    static bool done = false;
    if (done) return DBW_OK;
    const void *kernels[] = {(const void *)fchead::kernel<DBW_LOSS_MSE, true>, (const void *)fchead::kernel<DBW_LOSS_MSE, false>,
                             (const void *)fchead::kernel<DBW_LOSS_XENT, true>,
                             (const void *)fchead::kernel<DBW_LOSS_XENT, false>,
                             (const void *)fchead::kernel<DBW_LOSS_MSE, true, true>,
                             (const void *)fchead::kernel<DBW_LOSS_XENT, true, true>,
                             (const void *)mlpchain::kernel<1, 1>, (const void *)mlpchain::kernel<1, 2>,
                             (const void *)mlpchain::kernel<1, 4>, (const void *)mlpchain::kernel<2, 1>,
                             (const void *)mlpchain::kernel<2, 2>, (const void *)mlpchain::kernel<2, 4>,
                             (const void *)mlpchain::kernel<3, 1>, (const void *)mlpchain::kernel<3, 2>,
                             (const void *)mlpchain::kernel<3, 4>, (const void *)mlpchain::kernel<4, 1>,
                             (const void *)mlpchain::kernel<4, 2>, (const void *)mlpchain::kernel<4, 4>};
    for (const void *k : kernels)
        DBW_HIP(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fchead::LDS_LIMIT));
    done = true;
    return DBW_OK;
}

size_t dbw_mlp_scratch_floats(const dbw_ctx *c)
{
    return (size_t)dbw_fc_scratch_per_worker(c->model.n_layers, c->model.dims, c->model.batch) * c->N;
}

int dbw_launch_grad_mlp(dbw_ctx *c, const float *params, const float *bx, const int32_t *by, float *grads,
                        float *loss, hipStream_t s)
{
    const dbw_model &m = c->model;
    dbw_fc_args a{};
    a.L = m.n_layers;
    a.dims = m.dims;
    a.B = m.batch;
    a.loss_kind = m.loss;
    a.params = params;
    a.grads = grads;
    a.param_off = 0;
    a.in = bx;
    a.in_ld = m.dims[0];
    a.in_stride = (int64_t)m.batch * m.dims[0];
    a.act = c->act;
    a.act_stride = dbw_fc_scratch_per_worker(m.n_layers, m.dims, m.batch);
    a.y = by;
    a.loss = loss;
    a.grad_path = m.grad_path;
    return dbw_fc_forward_backward(c, a, s);
}
