// Forward pass, loss and the data-gradient half of the backward pass of a small multilayer
// perceptron in one launch (Section 2.1, stochastic gradient of the local loss; the 2NN of
// Appendix B: equal hidden widths, batch 1 024 per worker).
//
// As one GEMM launch per layer these products are short (1.3 GFLOP each for the 2NN on 10 workers):
// every launch pays its own ramp-up, first-tile latency and tail, and the matrix cores sit idle for a
// third of it.  Nothing but the weight gradients needs more than one sample at a time, so a workgroup
// here takes S = 16 RB samples of one worker through the whole chain with the activations in LDS:
//   a_l = relu(a_{l-1} W_l^T + b_l), l = 1 .. L - 1     (a_0 = the batch)
//   head (fc_head.h): logits, loss, dz_L, dW_L, db_L, dz_{L-1} = (dz_L W_L) masked by a_{L-1} > 0, db_{L-1}
//   dz_{l-1} = (dz_l W_l) masked by a_{l-1} > 0, l = L - 1 .. 2, in place over a_{l-1}
// and writes a_1 .. a_{L-2} and dz_1 .. dz_{L-1} to the worker's scratch block, from where the weight
// gradients dW_l = dz_l^T a_{l-1} (sums over the whole batch) are taken by the GEMM kernels.
//
// Products run on v_mfma_f32_16x16x4_f32 (true fp32).  A wavefront owns 16 CB output columns of all
// S rows, worked off 32 columns at a time: RB x min(CB, 2) accumulator tiles.  Its A fragments come from the LDS image of the layer's input
// (one 128-bit read per 16 rows and 16 k), its B fragments straight from the weights in global
// memory (L2), since no other wavefront of the workgroup wants the same ones; they are fetched one
// 64-wide k-chunk ahead, spread over the matrix instructions of the chunk before.  The matrix instruction only asks that lane group q of A and of B carry the
// same k, not which one, so a lane's four values of a 128-bit read serve four instructions:
//   forward, W_l [out][in], a lane reads W[n][k0 + 4 q .. + 4]: instruction e takes k = k0 + 4 q + e;
//   backward, a lane reads the CB consecutive columns W[k0 + 4 q + j][n0 + CB c .. + CB] for
//   j = 0 .. 3: instruction (j, cb) takes k = k0 + 4 q + j and output column n0 + CB c + cb.
// Workgroup ids are renumbered so that the ids one XCD receives cover consecutive chunks of few
// workers, whose weights then stay in that XCD's L2.
#pragma once

#include "fc_head.h"

namespace mlpchain {

using fchead::f32x4;
using fchead::pick;
using fchead::uniform_base;
constexpr int THREADS = fchead::THREADS, WAVES = THREADS / 64;
constexpr int XCDS = 8;
constexpr int MAX_L = 8;

struct Args {
    int B, L, K0, H, C;              // batch, layers (the head is layer L), input width, hidden width, classes
    int chunks, workers, loss_kind;
    const float *x;                  // [B][x_ld] per worker (stride x_stride)
    int64_t x_ld, x_stride;
    const float *params;             // worker rows of stride p_stride; W_l [out][in] at w_off[l], b_l at b_off[l]
    int64_t p_stride;
    int64_t w_off[MAX_L + 1], b_off[MAX_L + 1];
    float *act;                      // per-worker scratch (stride act_stride): a_l [B][H] at a_off[l], dz_l at dz_off[l]
    int64_t act_stride;
    int64_t a_off[MAX_L + 1], dz_off[MAX_L + 1];
    fchead::Args head;               // the head's arguments; its a and da are not used (both stay in LDS)
};

// LDS: the head's logits, partial logits and W_L image, then max(L - 1, 2) activation slots of
// S x max(pitch(H), pitch(K0)) floats (+ 16 of slack): a_l in slot l - 1, the batch chunk in slot 1
// (a_2 replaces it once layer 1 is done).
__host__ __device__ inline int64_t slot_floats(int K0, int H, int S)
{
    const int hp = fchead::row_pitch(H), p0 = fchead::row_pitch(K0);
    return (int64_t)S * (hp > p0 ? hp : p0) + 16;
}
__host__ __device__ inline size_t lds_bytes(int K0, int H, int C, int S, int L)
{
    const int slots = L - 1 > 2 ? L - 1 : 2;
    return sizeof(float) * ((size_t)fchead::MAX_S * fchead::MAX_C + (size_t)WAVES * 256 +
                            (size_t)(C + 1) * fchead::row_pitch(H) + 16 + (size_t)slots * slot_floats(K0, H, S));
}

template <int N>
struct alignas(4 * N) Vec {
    float v[N];
};

// The B values of one 64-wide k-chunk for a wavefront: 16 CB floats per lane.
//   forward:  v[u][4 cb + e] = W[n0 + 16 cb + l16][k0 + 16 u + 4 lq + e]
//   backward: v[u][CB j + cb] = W[k0 + 16 u + 4 lq + j][n0 + CB l16 + cb]
template <int CB>
struct BRegs {
    float v[4][4 * CB];
};

// Both loaders split an address into a wave-uniform base (scalar registers) and one 32-bit lane offset that is
// the same for every load of the product.  A chunk is fetched in four units of 16 k, so that the loads can be
// spread over the matrix instructions of the chunk before.
template <int CB>
__device__ __forceinline__ void load_fwd_unit(BRegs<CB> &b, const float *__restrict__ Wg, int K, int k0, int n0, int lane, int u)
{
    const uint32_t lane_off = 4u * ((uint32_t)(lane & 15) * (uint32_t)K + 4u * (uint32_t)(lane >> 4));
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const char *base = uniform_base(Wg + (int64_t)(n0 + 16 * cb) * K + k0 + 16 * u);
        const f32x4 q = *(const f32x4 *)(base + lane_off);
#pragma unroll
        for (int e = 0; e < 4; ++e) b.v[u][4 * cb + e] = q[e];
    }
}

template <int CB>
__device__ __forceinline__ void load_bwd_unit(BRegs<CB> &b, const float *__restrict__ Wg, int ldw, int k0, int n0, int lane, int u)
{
    const uint32_t lane_off = 4u * (4u * (uint32_t)(lane >> 4) * (uint32_t)ldw + (uint32_t)CB * (uint32_t)(lane & 15));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const char *base = uniform_base(Wg + (int64_t)(k0 + 16 * u + j) * ldw + n0);
        const Vec<CB> q = *(const Vec<CB> *)(base + lane_off);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) b.v[u][CB * j + cb] = q.v[cb];
    }
}

template <int CB>
__device__ __forceinline__ void load_fwd(BRegs<CB> &b, const float *__restrict__ Wg, int K, int k0, int n0, int lane)
{
#pragma unroll
    for (int u = 0; u < 4; ++u) load_fwd_unit<CB>(b, Wg, K, k0, n0, lane, u);
}

template <int CB>
__device__ __forceinline__ void load_bwd(BRegs<CB> &b, const float *__restrict__ Wg, int ldw, int k0, int n0, int lane)
{
#pragma unroll
    for (int u = 0; u < 4; ++u) load_bwd_unit<CB>(b, Wg, ldw, k0, n0, lane, u);
}

// acc += A(rows of `in`, k0 .. k0 + 63) x (the chunk in b); FWD tells which of the two layouts b has.  next(u) is
// called before the multiplies of unit u and issues the loads of unit u of the chunk after: a wavefront that issues all
// loads of a chunk in one burst waits at the memory pipeline's queue with its matrix instructions behind them, and so
// does its partner on the SIMD, which runs the same code (a register-resident loop of 96 matrix instructions per 8
// loads: +19 % time with the loads in a burst, +9 % with one load per 12 instructions).
template <int RB, int CB, bool FWD, class Next>
__device__ __forceinline__ void chunk_mfma(f32x4 (&acc)[RB][CB], const float *ap, int pitch, int k0, const BRegs<CB> &b, Next next)
{
    // the A fragments of the next 16 k are requested before the multiplies of the current ones
    f32x4 av[2][RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) av[0][rb] = *(const f32x4 *)(ap + 16 * rb * pitch + k0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        next(u);
        if (u + 1 < 4) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) av[(u + 1) & 1][rb] = *(const f32x4 *)(ap + 16 * rb * pitch + k0 + 16 * (u + 1));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u & 1][rb][e], FWD ? b.v[u][4 * cb + e] : b.v[u][CB * e + cb],
                                                                       acc[rb][cb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The k loop of one product.  b0 holds chunk 0 on entry (when K >= 64); the chunks alternate between b0 and a
// second set, each fetched while the other is multiplied, so that a fetch has a whole chunk of matrix
// instructions (of both wavefronts of the SIMD) to arrive.  K is a multiple of 16; the 16-wide groups behind the
// last whole chunk are fetched and multiplied one by one.
template <int RB, int CB, bool FWD>
__device__ __forceinline__ void product(f32x4 (&acc)[RB][CB], const float *in, int pitch, int K, const float *__restrict__ Wg,
                                        int ldw, int n0, int lane, BRegs<CB> &b0)
{
    const int l16 = lane & 15, lq = lane >> 4;
    const float *ap = in + l16 * pitch + 4 * lq;
    const int nch = K / 64;
    BRegs<CB> b1;
    auto load_unit = [&](BRegs<CB> &b, int kc, int u) {
        if (FWD) load_fwd_unit<CB>(b, Wg, ldw, 64 * kc, n0, lane, u);
        else load_bwd_unit<CB>(b, Wg, ldw, 64 * kc, n0, lane, u);
    };
    for (int kc = 0; kc < nch; kc += 2) {
        const bool two = kc + 1 < nch, three = kc + 2 < nch;
        chunk_mfma<RB, CB, FWD>(acc, ap, pitch, 64 * kc, b0, [&](int u) {
            if (two) load_unit(b1, kc + 1, u);
        });
        if (two)
            chunk_mfma<RB, CB, FWD>(acc, ap, pitch, 64 * (kc + 1), b1, [&](int u) {
                if (three) load_unit(b0, kc + 2, u);
            });
    }
    for (int k = 64 * nch; k < K; k += 16) {
        f32x4 av[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) av[rb] = *(const f32x4 *)(ap + 16 * rb * pitch + k);
        if (FWD) {
            f32x4 bv[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
                bv[cb] = *(const f32x4 *)(uniform_base(Wg + (int64_t)(n0 + 16 * cb) * ldw + k) + 4u * ((uint32_t)l16 * (uint32_t)ldw + 4u * (uint32_t)lq));
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[rb][e], bv[cb][e], acc[rb][cb], 0, 0, 0);
        } else {
            Vec<CB> bv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                bv[j] = *(const Vec<CB> *)(uniform_base(Wg + (int64_t)(k + j) * ldw + n0) + 4u * (4u * (uint32_t)lq * (uint32_t)ldw + (uint32_t)CB * (uint32_t)l16));
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[rb][j], bv[j].v[cb], acc[rb][cb], 0, 0, 0);
        }
    }
}

template <int RB, int CB>
__device__ __forceinline__ void zero(f32x4 (&acc)[RB][CB])
{
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
}

// Forward epilogue: out[s][n] = relu(acc + bias[n]) for this wavefront's columns n = n0 + 16 cb + l16.
// D: register r of lane (l16, lq) is row 4 lq + r, column l16 of the 16 x 16 tile.
template <int RB, int CB>
__device__ __forceinline__ void store_forward(const f32x4 (&acc)[RB][CB], const float (&bcol)[CB], float *out, int HP, int n0,
                                              int lane)
{
    const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const int col = n0 + 16 * cb + l16;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float v = acc[rb][cb][r] + bcol[cb];
                out[(16 * rb + 4 * lq + r) * HP + col] = v > 0.f ? v : 0.f;
            }
    }
}

// Backward epilogue: prev[s][n] = acc where prev[s][n] > 0, else 0, columns n = n0 + CB l16 + cb.
template <int RB, int CB>
__device__ __forceinline__ void store_backward(const f32x4 (&acc)[RB][CB], float *prev, int HP, int n0, int lane)
{
    typedef Vec<CB> vec;
    const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            vec *p = (vec *)(prev + (16 * rb + 4 * lq + r) * HP + n0 + CB * l16);
            const vec a = *p;
            vec d;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) d.v[cb] = a.v[cb] > 0.f ? acc[rb][cb][r] : 0.f;
            *p = d;
        }
}

// rows x 4 Q4 floats from an LDS image to global rows of 4 Q4 floats, 128 bits per thread and step (Q4 is a
// compile-time constant: the index arithmetic is shifts, not divisions).
template <int Q4>
__device__ __forceinline__ void copy_out(const float *src, int pitch, float *__restrict__ dst, int rows, int tid)
{
    const int total = rows * Q4;
    for (int e0 = 0; e0 < total; e0 += 4 * THREADS) {       // four LDS reads in flight, then their stores
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = min(e0 + tid + u * THREADS, total - 1), r = e / Q4;
            v[u] = *(const float4 *)(src + r * pitch + 4 * (e - r * Q4));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + tid + u * THREADS, r = e / Q4;
            // streaming stores: 30 MB of copies per launch must not push the 8 MB of weights, which every workgroup
            // reads over and over, out of the L2
            if (e < total) {
                const f32x4 t = {v[u].x, v[u].y, v[u].z, v[u].w};
                __builtin_nontemporal_store(t, (f32x4 *)(dst + (int64_t)r * (4 * Q4) + 4 * (e - r * Q4)));
            }
        }
    }
}

// grid = workers x chunks rounded up to a multiple of XCDS; dynamic LDS = lds_bytes(...).
template <int RB, int CB>
__global__ __launch_bounds__(THREADS) void kernel(Args g)
{
    extern __shared__ __attribute__((aligned(16))) float sm[];
    constexpr int S = 16 * RB;
    const int H = g.H, C = g.C, K0 = g.K0, HP = fchead::row_pitch(H), P0 = fchead::row_pitch(K0), Lh = g.L - 1;
    const int per = gridDim.x / XCDS, id = (blockIdx.x % XCDS) * per + blockIdx.x / XCDS;
    if (id >= g.workers * g.chunks) return;                // the whole workgroup: no barrier is left waiting
    const int w = id / g.chunks, chunk = id - w * g.chunks;
    const int s0 = chunk * S, ns = min(S, g.B - s0);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // on the scalar unit

    float *zl = sm;
    float *zp = zl + fchead::MAX_S * fchead::MAX_C;
    float *Wl = zp + WAVES * 256;
    float *slots = Wl + (C + 1) * HP + 16;
    const int64_t Z = slot_floats(K0, H, S);
    float *xl = slots + Z;
    const float *__restrict__ pw = g.params + w * g.p_stride;
    float *__restrict__ sw = g.act + w * g.act_stride;

    // A wavefront's 16 CB columns are worked off in blocks of 16 CBI: with four 16-column blocks at once the
    // accumulators and the two sets of weight registers no longer fit the register file.
    // The first chunk of W_1 is on its way while the batch is staged; likewise every later product's first chunk
    // is requested before the epilogue of the product before it.
    constexpr int CBI = CB > 2 ? 2 : CB, NSUB = CB / CBI;
    const int n0 = wave * 16 * CB;
    BRegs<CBI> b0;
    if (K0 >= 64) load_fwd<CBI>(b0, pw + pick(g.w_off, 1), K0, 0, n0, lane);
    const fchead::Early early = fchead::fetch_early(g.head, w, s0, ns, tid);
    fchead::stage_w(g.head, w, Wl, tid);
    {   // the chunk of the batch, rows beyond it zero
        const float *__restrict__ x = g.x + w * g.x_stride + (int64_t)s0 * g.x_ld;
        const int q4 = K0 / 4, total = S * q4;
        fchead::RowWalk rw(tid, q4);
        for (int e0 = 0; e0 < total; e0 += 8 * THREADS) {
            float4 v[8];
            int at[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (e0 + tid + u * THREADS < total && rw.r < ns) v[u] = *(const float4 *)(x + (int64_t)rw.r * g.x_ld + 4 * rw.k);
                at[u] = rw.r * P0 + 4 * rw.k;
                rw.next();
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (e0 + tid + u * THREADS < total) *(float4 *)(xl + at[u]) = v[u];
        }
    }
    __syncthreads();

    f32x4 acc[RB][CBI];
    for (int l = 1; l <= Lh; ++l) {
        const float *in = l == 1 ? xl : slots + (l - 2) * Z;
        float *out = slots + (l - 1) * Z;
        // what the head reads beyond the H columns of a row and behind the image must be zero (nobody reads this
        // slot during this layer; the batch chunk that lay in slot 1 is dead from layer 2 on)
        for (int e = tid; e < S * 4; e += THREADS) out[(e >> 2) * HP + H + (e & 3)] = 0.f;     // HP = H + 4 for these widths
        if (tid < 16) out[S * HP + tid] = 0.f;
        const int K = l == 1 ? K0 : H;
        const float *__restrict__ Wl_ = pw + pick(g.w_off, l);
        for (int sub = 0; sub < NSUB; ++sub) {
            const int n0s = n0 + 16 * CBI * sub;
            float bcol[CBI];
#pragma unroll
            for (int cb = 0; cb < CBI; ++cb) bcol[cb] = pw[pick(g.b_off, l) + n0s + 16 * cb + (lane & 15)];
            zero<RB, CBI>(acc);
            product<RB, CBI, true>(acc, in, l == 1 ? P0 : HP, K, Wl_, K, n0s, lane, b0);
            if (sub + 1 < NSUB) {
                if (K >= 64) load_fwd<CBI>(b0, Wl_, K, 0, n0s + 16 * CBI, lane);
            } else if (l < Lh) {
                load_fwd<CBI>(b0, pw + pick(g.w_off, l + 1), H, 0, n0, lane);
            } else if (Lh >= 2) {
                load_bwd<CBI>(b0, pw + pick(g.w_off, Lh), H, 0, n0, lane);     // waits in registers through the head
            }
            // a_{l-1} goes to scratch here, behind this product's last loads: a wavefront's loads and stores complete
            // in order, so stores issued before a product hold up the wait for its second chunk until they are
            // acknowledged (this product's phase was 1.4 us longer with the copy in front of it)
            if (sub + 1 == NSUB && l >= 2) copy_out<32 * CB>(in, HP, sw + pick(g.a_off, l - 1) + (int64_t)s0 * H, ns, tid);
            store_forward<RB, CBI>(acc, bcol, out, HP, n0s, lane);
        }
        __syncthreads();
    }

    float *top = slots + (Lh - 1) * Z;                     // a_{L-1}, then dz_{L-1}
    if (g.loss_kind == DBW_LOSS_MSE)
        fchead::body<DBW_LOSS_MSE>(g.head, zl, zp, Wl, top, S, w, chunk, g.chunks, true, early);
    else
        fchead::body<DBW_LOSS_XENT>(g.head, zl, zp, Wl, top, S, w, chunk, g.chunks, true, early);
    __syncthreads();

    for (int l = Lh; l >= 2; --l) {
        float *prev = slots + (l - 2) * Z;
        const float *__restrict__ Wl_ = pw + pick(g.w_off, l);
        for (int sub = 0; sub < NSUB; ++sub) {
            const int n0s = n0 + 16 * CBI * sub;
            zero<RB, CBI>(acc);
            product<RB, CBI, false>(acc, slots + (l - 1) * Z, HP, H, Wl_, H, n0s, lane, b0);
            if (sub + 1 < NSUB) load_bwd<CBI>(b0, Wl_, H, 0, n0s + 16 * CBI, lane);
            else if (l > 2) load_bwd<CBI>(b0, pw + pick(g.w_off, l - 1), H, 0, n0, lane);
            if (sub + 1 == NSUB) copy_out<32 * CB>(slots + (l - 1) * Z, HP, sw + pick(g.dz_off, l) + (int64_t)s0 * H, ns, tid);
            store_backward<RB, CBI>(acc, prev, HP, n0s, lane);
        }
        __syncthreads();
    }
    copy_out<32 * CB>(slots, HP, sw + pick(g.dz_off, 1) + (int64_t)s0 * H, ns, tid);      // dz_1 (with one hidden layer: the head's)
}

}  // namespace mlpchain
