// The classifier head of a model in one launch: last fully connected layer (H -> C, C <= 16),
// softmax, loss, and everything of the backward pass that hangs on it (Section 2.1, stochastic
// gradient of the local loss; cross-entropy as in Section 5, squared error of the softmax outputs
// as for the 2NN of Appendix B):
//   z = a W^T + b,  p = softmax(z),  loss,  dz = dloss/dz / B
//   dW = dz^T a,  db = column sums of dz
//   da = dz W, masked by a > 0 when a is the output of a ReLU layer (then also its column sums, the
//        bias gradient of the layer below), unmasked when a is the model's input
// As separate launches these thin products cost five to eight kernels of 4-13 us each, mostly
// latency.  Here one workgroup takes S = 16, 32 or 64 samples of one worker, keeps them and W in LDS
// and runs the three products on the matrix cores with the class dimension padded to the 16
// columns of v_mfma_f32_16x16x4_f32 (true fp32):
//   A fragment: lane l holds A[m = l % 16][k = l / 16], B fragment: B[k = l / 16][n = l % 16],
//   D: d[v] = D[m = 4 * (l / 16) + v][n = l % 16].
//
// grid = (chunks, workers).  With one chunk per worker (batches up to 64) the sums over the batch
// (dW, db, the bias gradient below, the loss) are final.  Otherwise they are written as per-chunk
// partials and added in chunk order by reduce_kernel, a second launch: a "last workgroup to arrive
// adds them" scheme inside one launch was measured and rejected, because the memory fence every
// workgroup needs before it takes its ticket writes back its XCD's whole L2 (46 us for 384
// workgroups against 6 us of arithmetic).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dbw.h"

namespace fchead {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int THREADS = 512, WAVES = THREADS / 64;
constexpr int MAX_C = 16;            // classes, padded to 16
constexpr int MAX_S = 64;            // samples per workgroup: 16, 32 or 64
constexpr int MAX_CHUNKS = 256;
constexpr size_t LDS_LIMIT = 159 * 1024;     // dynamic part; the kernel also has a few bytes of static LDS

// Element i of a small table that sits in the kernel arguments.  Indexing such a table with a run-time value
// makes the compiler copy the whole argument block into vector registers; a chain of selects over constant
// indices stays on the scalar unit.
template <class T, int N>
__device__ __forceinline__ T pick(const T (&a)[N], int i)
{
    T r = a[0];
#pragma unroll
    for (int k = 1; k < N; ++k) r = i == k ? a[k] : r;
    return r;
}

// A wave-uniform address, pinned to scalar registers: global loads then take this base plus a 32-bit lane
// offset.  Without the pin the compiler folds the lane offset into one loop-invariant 64-bit vector address per
// load, and dozens of such register pairs crowd out the accumulators.
__device__ __forceinline__ const char *uniform_base(const void *p)
{
    const uint64_t a = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    uint64_t v = ((uint64_t)hi << 32) | lo;
    asm volatile("" : "+s"(v));
    return (const char *)v;
}

struct Args {
    int B, H, C, S;                  // batch, inputs, classes, samples per chunk (16, 32 or 64)
    const float *a;                  // [B][a_ld] per worker (stride a_stride): the head's input
    int64_t a_ld, a_stride;
    int splits;                      // > 0: the input is still the partial sums of a forward product split along k,
                                     // a[split][B][H] per worker (a_ld = H): the head's input is
                                     // relu(sum over splits, in order, + the bias of that layer)
    int64_t in_bias_off;             // offset of that bias [H] in the worker's parameter row
    const float *params;             // worker rows of stride p_stride; W [C][H] at w_off, bias [C] at b_off
    float *grads;                    // same offsets and stride: receives dW and db
    int64_t p_stride, w_off, b_off;
    const int32_t *y;                // [workers][B]
    float *da;                       // [B][da_ld] per worker, or nullptr
    int64_t da_ld, da_stride;
    int mask;                        // 1: da is kept only where a > 0
    int64_t bprev_off;               // >= 0: column sums of da go to grads at this offset
    float *loss;                     // [workers] or nullptr
    float *part;                     // [workers][part_stride] scratch for the per-chunk partial sums
    int64_t part_stride;
    int32_t *err;                    // deferred status word
};

// Row pitch of the LDS images of a and W: H rounded up to 4 (the k-step of the matrix instruction;
// the extra columns are zero), made an odd multiple of 4 so that the 16 rows x 4 columns a fragment
// read touches fall into 64 different banks.
__host__ __device__ inline int row_pitch(int H)
{
    const int h4 = (H + 3) / 4 * 4;
    return (h4 / 4) % 2 ? h4 : h4 + 4;
}
__host__ __device__ inline size_t lds_floats(int H, int C, int S)
{
    // dz / logits [64][16], partial logits [8 waves][16][16], W image [C + 1][pitch] (the last row is zero and
    // stands for the padding classes), a image [S][pitch], 16 floats of slack behind each image (fragment
    // reads of the last, partly filled 16-column block run past the row)
    return (size_t)MAX_S * MAX_C + (size_t)WAVES * 16 * 16 + (size_t)(C + 1 + S) * row_pitch(H) + 32;
}
__host__ __device__ inline size_t lds_bytes(int H, int C, int S) { return sizeof(float) * lds_floats(H, C, S); }
__host__ __device__ inline int64_t partial_floats(int H, int C, bool bprev) { return (int64_t)C * H + C + (bprev ? H : 0) + 1; }

// (row, column) of the flat index e in rows of P elements, for e = tid, tid + THREADS, ...: one division per thread,
// then additions.  With a division per element the staging loops below spent more time on them than on their loads.
struct RowWalk {
    int r, k, dr, dk, P;
    __device__ __forceinline__ RowWalk(int tid, int P_) : P(P_)
    {
        r = tid / P_;
        k = tid - r * P_;
        dr = THREADS / P_;
        dk = THREADS - dr * P_;
    }
    __device__ __forceinline__ void next()
    {
        r += dr;
        k += dk;
        if (k >= P) {
            k -= P;
            ++r;
        }
    }
};

// W [C][H] of worker w -> its LDS image [C + 1][pitch]; row C, the columns >= H and the slack behind are zero.
__device__ __forceinline__ void stage_w(const Args &g, int w, float *Wl, int tid)
{
    const int H = g.H, C = g.C, HP = row_pitch(H);
    const float *__restrict__ Wg = g.params + w * g.p_stride + g.w_off;
    if (H % 4 == 0 && g.w_off % 4 == 0 && g.p_stride % 4 == 0 && (uintptr_t)g.params % 16 == 0) {
        // rows of W start on 16-byte boundaries: 128-bit loads, a quarter of the instructions
        const int q4 = HP / 4, total = (C + 1) * q4 + 4;
        RowWalk rw(tid, q4);
        for (int e0 = 0; e0 < total; e0 += 4 * THREADS) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool ok = e0 + tid + u * THREADS < total && rw.r < C && 4 * rw.k < H;
                v[u] = *(const float4 *)(Wg + (ok ? rw.r * H + 4 * rw.k : 0));
                if (!ok) v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                rw.next();
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + tid + u * THREADS;
                if (e < total) *(float4 *)(Wl + 4 * e) = v[u];
            }
        }
        return;
    }
    const int total = (C + 1) * HP + 16;
    RowWalk rw(tid, HP);
    for (int e0 = 0; e0 < total; e0 += 8 * THREADS) {       // eight loads in flight per thread
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            v[u] = (e0 + tid + u * THREADS < total && rw.r < C && rw.k < H) ? Wg[rw.r * H + rw.k] : 0.f;
            rw.next();
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int e = e0 + tid + u * THREADS;
            if (e < total) Wl[e] = v[u];
        }
    }
}

// What the body needs from global memory besides the images: the caller fetches it before its own staging, so that
// the latency passes there and not between two barriers of the body.
struct Early {
    float bias;      // b[tid % 16] (0 for the padding classes)
    int label[2];    // y of samples tid / 16 and 32 + tid / 16 of the chunk (0 beyond it)
};
__device__ __forceinline__ Early fetch_early(const Args &g, int w, int s0, int ns, int tid)
{
    Early e;
    const int c = tid & 15, s = tid >> 4;
    e.bias = c < g.C ? g.params[w * g.p_stride + g.b_off + c] : 0.f;
    const int32_t *__restrict__ y = g.y + (int64_t)w * g.B + s0;
    e.label[0] = s < ns ? y[s] : 0;
    e.label[1] = s + 32 < ns ? y[s + 32] : 0;
    return e;
}

// Everything after the staging: al [S][pitch] holds the chunk's input (rows beyond the batch, the columns >= H and 16
// floats behind the image zero), Wl the image stage_w makes.  S is a multiple of 16 up to MAX_S.  With da_to_lds the
// (masked) input gradient replaces the input in al instead of going to g.da.  All THREADS threads call this after a
// barrier that makes al and Wl visible.
template <int LOSS>
__device__ __forceinline__ void body(const Args &g, float *zl, float *zp, float *Wl, float *al, int S, int w, int chunk,
                                     int chunks, bool da_to_lds, const Early &early)
{
    const int H = g.H, C = g.C, HP = row_pitch(H);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // on the scalar unit: loops and branches on it are uniform
    const int l16 = lane & 15, lq = lane >> 4;
    const int s0 = chunk * S, ns = min(S, g.B - s0);

    // ---- logits z = a W^T: wavefront = (16-sample block, slice of k); partial sums meet in LDS.
    // A lane reads four consecutive k of its row with one 128-bit LDS read; lane group q of both operands then
    // carries k = 16 g + 4 q + e in instruction e, which is all the matrix instruction asks for.  Two
    // accumulators halve the chain of dependent instructions.
    {
        const int MB = S / 16, KS = WAVES / MB;
        const int mb = wave % MB, ks = wave / MB;
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = acc0;
        if (ks < KS) {
            const int G = HP / 16, per = (G + KS - 1) / KS, g_end = min(G, (ks + 1) * per);
            const float *ap = al + (16 * mb + l16) * HP + 4 * lq, *wp = Wl + min(l16, C) * HP + 4 * lq;
#pragma unroll 2
            for (int gk = ks * per; gk < g_end; ++gk) {
                const f32x4 a4 = *(const f32x4 *)(ap + 16 * gk), w4 = *(const f32x4 *)(wp + 16 * gk);
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[0], w4[0], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[1], w4[1], acc1, 0, 0, 0);
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[2], w4[2], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[3], w4[3], acc1, 0, 0, 0);
            }
            if (ks == KS - 1) {     // the columns behind the last whole group of 16
                const float *a1 = al + (16 * mb + l16) * HP + lq, *w1 = Wl + min(l16, C) * HP + lq;
                for (int q = 4 * G; q < HP / 4; ++q)
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[4 * q], w1[4 * q], acc0, 0, 0, 0);
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) zp[(wave * 16 + 4 * lq + v) * 16 + l16] = acc0[v] + acc1[v];
        __syncthreads();
        // sample s, class c: the slices in order, then the bias
        for (int e = tid; e < S * 16; e += THREADS) {
            const int s = e >> 4, c = e & 15;
            float z = 0.f;
            for (int q = 0; q < KS; ++q) z += zp[((q * MB + (s >> 4)) * 16 + (s & 15)) * 16 + c];
            zl[e] = c < C ? z + early.bias : 0.f;              // c == tid % 16: the stride of e is a multiple of 16
        }
    }
    __syncthreads();

    // ---- softmax, loss and dz: 16 lanes per sample, one class each; maxima and sums by butterflies over the 16
    // lanes, so that every lane holds them.  Rows of samples beyond the batch become zero.  The per-sample losses
    // go to red[0 .. 63] (the partial logits are dead) for the tree at the end.
    float *red = zp;
    {
        const float inv_b = 1.0f / (float)g.B;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int s = (tid >> 4) + 32 * pass, c = tid & 15;
            float *zs = zl + s * MAX_C;
            float dzv = 0.f, lossv = 0.f;
            if (s < ns) {                                       // the same for the 16 lanes of a sample
                const bool real = c < C;
                const float z = real ? zs[c] : -INFINITY;
                float m = z;
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) m = fmaxf(m, __shfl_xor(m, o, 16));
                const float ex = real ? expf(z - m) : 0.f;
                float sum = ex;
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) sum += __shfl_xor(sum, o, 16);
                int label = early.label[pass];
                if (label < 0 || label >= C) {              // clamped for memory safety, reported by dbw_check
                    *g.err = DBW_ERR_INVALID;
                    label = label < 0 ? 0 : C - 1;
                }
                const float pr = ex * (1.0f / sum), hot = c == label ? 1.f : 0.f;
                if (LOSS == DBW_LOSS_XENT) {
                    float zl_ = c == label ? z : 0.f;           // z of the label's class, to every lane
#pragma unroll
                    for (int o = 1; o < 16; o <<= 1) zl_ += __shfl_xor(zl_, o, 16);
                    lossv = logf(sum) + m - zl_;
                    dzv = real ? (pr - hot) * inv_b : 0.f;
                } else {
                    const float er = real ? pr - hot : 0.f;
                    float f = er * er, inner = pr * er;
#pragma unroll
                    for (int o = 1; o < 16; o <<= 1) {
                        f += __shfl_xor(f, o, 16);
                        inner += __shfl_xor(inner, o, 16);
                    }
                    lossv = f;
                    dzv = 2.f * pr * (er - inner) * inv_b;
                }
            }
            zs[c] = dzv;
            if (c == 0) red[s] = lossv;
        }
    }
    __syncthreads();

    float *__restrict__ part = g.part + w * g.part_stride + (int64_t)chunk * partial_floats(H, C, g.bprev_off >= 0);
    float *__restrict__ out_w = chunks == 1 ? g.grads + w * g.p_stride + g.w_off : part;
    float *__restrict__ out_b = chunks == 1 ? g.grads + w * g.p_stride + g.b_off : part + (size_t)C * H;
    float *__restrict__ out_bprev = g.bprev_off < 0 ? nullptr
                                    : (chunks == 1 ? g.grads + w * g.p_stride + g.bprev_off : part + (size_t)C * H + C);
    float *__restrict__ da = (g.da && !da_to_lds) ? g.da + w * g.da_stride + (int64_t)s0 * g.da_ld : nullptr;
    const int NB = (H + 15) / 16;                       // 16-column blocks of the input dimension

    // Two 16-column blocks per pass (nb and nb + WAVES): their chains of dependent instructions and LDS reads overlap.
    // A pass whose second block does not exist computes it on the first one's columns and stores nothing for it.
    for (int nb0 = wave; nb0 < NB; nb0 += 2 * WAVES) {
        const bool two = nb0 + WAVES < NB;
        int col[2];
        col[0] = 16 * nb0 + l16;
        col[1] = two ? col[0] + 16 * WAVES : col[0];
        // ---- dW[class][col] = sum over samples of dz[sample][class] a[sample][col]: the operands of 16 samples are
        // read before their instructions, two accumulators per block
        {
            f32x4 acc[2][2];
#pragma unroll
            for (int p = 0; p < 2; ++p) acc[p][0] = acc[p][1] = f32x4{0.f, 0.f, 0.f, 0.f};
            for (int k0 = 0; k0 < S; k0 += 16) {
                float zv[4], av[2][4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    zv[u] = zl[(k0 + 4 * u + lq) * MAX_C + l16];
#pragma unroll
                    for (int p = 0; p < 2; ++p) av[p][u] = al[(k0 + 4 * u + lq) * HP + col[p]];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int p = 0; p < 2; ++p)
                        acc[p][u & 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(zv[u], av[p][u], acc[p][u & 1], 0, 0, 0);
            }
#pragma unroll
            for (int p = 0; p < 2; ++p)
                if (col[p] < H && (p == 0 || two)) {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (4 * lq + v < C) out_w[(4 * lq + v) * H + col[p]] = acc[p][0][v] + acc[p][1][v];
                }
        }
        // ---- da[sample][col] = sum over classes of dz[sample][class] W[class][col], masked; its column sums.
        // Lane group q carries the classes 4 q + j in instruction j: one 128-bit read of dz per 16 samples.
        if (da || da_to_lds) {
            float wv[2][4];
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int j = 0; j < 4; ++j) wv[p][j] = Wl[min(4 * lq + j, C) * HP + col[p]];
            float colsum[2] = {0.f, 0.f};
            for (int mb = 0; mb < S / 16; ++mb) {
                const f32x4 zq = *(const f32x4 *)(zl + (16 * mb + l16) * MAX_C + 4 * lq);
                float keep[2][4];
#pragma unroll
                for (int p = 0; p < 2; ++p)
#pragma unroll
                    for (int v = 0; v < 4; ++v) keep[p][v] = al[(16 * mb + 4 * lq + v) * HP + col[p]];
                f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int p = 0; p < 2; ++p) acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(zq[j], wv[p][j], acc[p], 0, 0, 0);
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    if (p == 1 && !two) continue;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int s = 16 * mb + 4 * lq + v;
                        float d = acc[p][v];
                        if (g.mask && !(keep[p][v] > 0.f)) d = 0.f;
                        if (da_to_lds) al[s * HP + col[p]] = d;       // this wavefront alone reads and writes these columns
                        else if (s < ns && col[p] < H) da[(int64_t)s * g.da_ld + col[p]] = d;
                        colsum[p] += d;                        // rows beyond the batch have dz = 0
                    }
                }
            }
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                colsum[p] += __shfl_xor(colsum[p], 16, 64);
                colsum[p] += __shfl_xor(colsum[p], 32, 64);
                if (out_bprev && lq == 0 && col[p] < H && (p == 0 || two)) out_bprev[col[p]] = colsum[p];
            }
        }
    }
    if (tid < C) {
        float sum = 0.f;
        for (int s = 0; s < ns; ++s) sum += zl[s * MAX_C + tid];
        out_b[tid] = sum;
    }
    // ---- the chunk's loss: its samples in a fixed order (tree in LDS)
    if (g.loss) {
        for (int o = MAX_S / 2; o > 0; o >>= 1) {
            if (tid < o) red[tid] += red[tid + o];
            __syncthreads();
        }
        if (tid == 0) {
            if (chunks == 1) g.loss[w] = red[0] / (float)g.B;
            else part[partial_floats(H, C, g.bprev_off >= 0) - 1] = red[0];
        }
    }
}

// Sum of the first `splits` (<= NQ) of the float4s at src + q * plane, in order, all NQ loads in flight.  A slot
// beyond the splits re-reads the last one and adds zero: loads under a condition each would be merged back into
// one register array with a move per element.
template <int NQ>
__device__ __forceinline__ float4 split_sum(const float *src, int64_t plane, int splits)
{
    float4 v[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) v[q] = *(const float4 *)(src + min(q, splits - 1) * plane);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const bool on = q < splits;
        acc.x += on ? v[q].x : 0.f; acc.y += on ? v[q].y : 0.f;
        acc.z += on ? v[q].z : 0.f; acc.w += on ? v[q].w : 0.f;
    }
    return acc;
}

// VEC: the input rows start on 16-byte boundaries and H divides by 4 (128-bit staging loads).
// SPLIT: the input arrives as split-k partial sums (Args::splits).
template <int LOSS, bool VEC, bool SPLIT = false>
__global__ __launch_bounds__(THREADS) void kernel(Args g)
{
    extern __shared__ __attribute__((aligned(16))) float sm[];
    const int H = g.H, C = g.C, S = g.S, HP = row_pitch(H);
    float *zl = sm;                                  // [64][16]: logits, then dz
    float *zp = zl + MAX_S * MAX_C;                  // [8][16][16]: partial logits of the wavefronts
    float *Wl = zp + WAVES * 16 * 16;                // [C + 1][HP]: row C and the columns >= H are zero
    float *al = Wl + (C + 1) * HP + 16;              // [S][HP], rows >= ns and columns >= H zero
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x, chunks = gridDim.x, w = blockIdx.y;
    const int s0 = chunk * S, ns = min(S, g.B - s0);
    const float *__restrict__ a = g.a + w * g.a_stride + (int64_t)s0 * g.a_ld;

    const Early early = fetch_early(g, w, s0, ns, tid);
    // ---- stage W and this chunk of a; everything the fragments may touch beyond them is zero
    stage_w(g, w, Wl, tid);
    if (SPLIT) {
        // a = relu(sum of the partial sums + bias): one float4 per thread at a time, all splits in flight
        const int q4 = HP / 4, total = S * q4;
        const float *__restrict__ bin = g.params + w * g.p_stride + g.in_bias_off;
        const int64_t plane = (int64_t)g.B * H;
        RowWalk rw(tid, q4);
        for (int e = tid; e < total; e += THREADS, rw.next()) {
            const int r = rw.r, k = 4 * rw.k;
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < ns && k < H) {
                const float *src = g.a + w * g.a_stride + (int64_t)(s0 + r) * H + k;
                if (g.splits <= 2) acc = split_sum<2>(src, plane, g.splits);
                else if (g.splits <= 4) acc = split_sum<4>(src, plane, g.splits);
                else if (g.splits <= 8) acc = split_sum<8>(src, plane, g.splits);
                else acc = split_sum<16>(src, plane, g.splits);
                const float4 bv = *(const float4 *)(bin + k);
                acc.x = fmaxf(acc.x + bv.x, 0.f); acc.y = fmaxf(acc.y + bv.y, 0.f);
                acc.z = fmaxf(acc.z + bv.z, 0.f); acc.w = fmaxf(acc.w + bv.w, 0.f);
            }
            *(float4 *)(al + 4 * e) = acc;
        }
    } else if (VEC) {
        const int q4 = HP / 4, total = S * q4;
        RowWalk rw(tid, q4);
        for (int e0 = 0; e0 < total; e0 += 8 * THREADS) {
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (e0 + tid + u * THREADS < total && rw.r < ns && 4 * rw.k < H)
                    v[u] = *(const float4 *)(a + (int64_t)rw.r * g.a_ld + 4 * rw.k);
                rw.next();
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + tid + u * THREADS;
                if (e < total) *(float4 *)(al + 4 * e) = v[u];
            }
        }
    } else {
        const int total = S * HP;
        RowWalk rw(tid, HP);
        for (int e0 = 0; e0 < total; e0 += 8 * THREADS) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                v[u] = (e0 + tid + u * THREADS < total && rw.r < ns && rw.k < H) ? a[(int64_t)rw.r * g.a_ld + rw.k] : 0.f;
                rw.next();
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + tid + u * THREADS;
                if (e < total) al[e] = v[u];
            }
        }
    }
    if (tid < 16) al[S * HP + tid] = 0.f;
    __syncthreads();

    body<LOSS>(g, zl, zp, Wl, al, S, w, chunk, chunks, false, early);
}

// Sum of the per-chunk partials in chunk order -> dW, db, the bias gradient below, the loss.
// Blocks bx = 0 .. ceil(E / 256) - 1 of 256 threads per worker w, E = partial_floats.
__device__ __forceinline__ void reduce_body(const Args &g, int chunks, int bx, int w)
{
    const int H = g.H, C = g.C;
    const int n_w = C * H, n_b = C, n_p = g.bprev_off >= 0 ? H : 0;
    const int64_t E = partial_floats(H, C, g.bprev_off >= 0);
    const int e = bx * 256 + threadIdx.x;
    if (e >= E || (e == E - 1 && !g.loss)) return;
    const float *__restrict__ all = g.part + w * g.part_stride;
    float *__restrict__ gw = g.grads + w * g.p_stride;
    float sum = 0.f;
    for (int q0 = 0; q0 < chunks; q0 += 16) {           // sixteen loads in flight, added in chunk order
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = q0 + u < chunks ? all[(int64_t)(q0 + u) * E + e] : 0.f;
#pragma unroll
        for (int u = 0; u < 16; ++u) sum += v[u];
    }
    if (e < n_w) gw[g.w_off + e] = sum;
    else if (e < n_w + n_b) gw[g.b_off + (e - n_w)] = sum;
    else if (e < n_w + n_b + n_p) gw[g.bprev_off + (e - n_w - n_b)] = sum;
    else g.loss[w] = sum / (float)g.B;
}

// grid = (ceil(E / 256), workers)
__global__ __launch_bounds__(256) void reduce_kernel(Args g, int chunks) { reduce_body(g, chunks, blockIdx.x, blockIdx.y); }

}  // namespace fchead
