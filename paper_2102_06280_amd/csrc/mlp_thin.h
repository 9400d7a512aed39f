// Fully connected layers on short batches (up to 64 samples per worker), all workers in one launch
// (Section 2.1, stochastic gradient of the local loss):
//   forward_kernel   a_l[s][n] = act(sum_k a_{l-1}[s][k] W_l[n][k] + b_l[n])
//   wgrad_kernel     dW_l[m][n] = sum_s dz_l[s][m] a_{l-1}[s][n],   db_l[m] = sum_s dz_l[s][m]
// With so few samples the tiled GEMM kernel (bgemm.h) spends its time on LDS round trips and
// barriers: a 64 x 784 x 200 product per worker reached a fifth of the matrix rate.  Here every
// operand goes from global memory straight into matrix-instruction fragments
// (v_mfma_f32_16x16x4_f32; A: lane l holds A[m = l % 16][k = l / 16], B: B[k = l / 16][n = l % 16],
// D: d[v] = D[m = 4 (l / 16) + v][n = l % 16]) with 128-bit loads:
//
// forward: both operands are contiguous along k.  The instruction does not care which four k a
// step stands for, so lane (l16, lq) loads k = 16 c + 4 lq .. + 3 of its row with one load, and
// element t of that load feeds step t of chunk c (that step then covers k = 16 c + 4 lq' + t for
// lq' = 0..3).  A workgroup owns all samples x 32 outputs of one worker; its eight wavefronts
// take every eighth chunk of 16 k, and their accumulators are added through LDS in a fixed order.
//
// wgrad: both operands are contiguous along their output index; the layout trick of mlp_wgrad.h
// (a lane's four consecutive outputs go to four different tiles) applies, but with at most 16 groups
// of four samples a tile is too little work to share: every wavefront owns a 32 x 64 tile, fetches
// all its samples at once, multiplies and stores, with no LDS and no barrier.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fc_head.h"
#include "mlp_wgrad.h"

namespace mlpthin {

using fchead::f32x4;
using fchead::pick;
constexpr int XCDS = 8;
constexpr int FWD_WAVES = 8, FWD_THREADS = 64 * FWD_WAVES, FWD_CB = 2, FWD_PF = 1;
constexpr int MAX_B = 64;

struct FwdArgs {
    int B, K, N, workers, relu;          // samples (<= 16 RB), inputs and outputs (multiples of 4)
    const float *a;                      // a_{l-1} [B][a_ld] at a + w * a_stride
    int64_t a_ld, a_stride;
    const float *params;                 // worker rows of stride p_stride; W [N][K] at w_off, b [N] at b_off
    int64_t p_stride, w_off, b_off;
    float *out;                          // a_l [B][N] at out + w * out_stride
    int64_t out_stride;
};

// grid = tiles of 32 outputs x workers, rounded up to a multiple of XCDS and renumbered so that one XCD
// receives consecutive tiles: the tiles of a worker read the same samples through the same L2.
template <int RB>
__global__ __launch_bounds__(FWD_THREADS) void forward_kernel(FwdArgs g)
{
    constexpr int CB = FWD_CB, WAVES = FWD_WAVES, PF = FWD_PF;
    constexpr int TM = 16 * RB, TN = 16 * CB, TP = TN + 4;
    __shared__ __attribute__((aligned(16))) float red[WAVES / 2][TM * TP];
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles = (g.N + TN - 1) / TN;
    const int per = gridDim.x / XCDS, id = (blockIdx.x % XCDS) * per + blockIdx.x / XCDS;
    if (id >= tiles * g.workers) return;
    const int t = id % tiles, w = id / tiles, n0 = TN * t;

    // rows beyond the batch and outputs beyond the layer: any valid row instead, never stored
    const float *pa[RB], *pb[CB];
#pragma unroll
    for (int i = 0; i < RB; ++i) pa[i] = g.a + w * g.a_stride + (int64_t)min(16 * i + l16, g.B - 1) * g.a_ld + 4 * lq;
#pragma unroll
    for (int j = 0; j < CB; ++j)
        pb[j] = g.params + w * g.p_stride + g.w_off + (int64_t)min(n0 + 16 * j + l16, g.N - 1) * g.K + 4 * lq;

    f32x4 acc[RB][CB];
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int j = 0; j < CB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](const f32x4 (&x)[RB], const f32x4 (&y)[CB]) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int j = 0; j < CB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[i][e], y[j][e], acc[i][j], 0, 0, 0);
    };

    // whole chunks of 16 k: number wave, wave + WAVES, ... are this wavefront's, the next one in flight
    // while one is multiplied (deeper prefetch was slower: 24 loads per wavefront queued before the first multiply took
    // 6 us to issue, and the products then ran behind the transfers instead of under them)
    const int whole = g.K / 16, mine = whole > wave ? (whole - wave + WAVES - 1) / WAVES : 0;
    f32x4 ra[PF][RB], rb[PF][CB];
    auto fetch = [&](int u, int n) {          // this wavefront's n-th chunk into slot u
        const int k = 16 * (wave + WAVES * n);
#pragma unroll
        for (int i = 0; i < RB; ++i) ra[u][i] = *(const f32x4 *)(pa[i] + k);
#pragma unroll
        for (int j = 0; j < CB; ++j) rb[u][j] = *(const f32x4 *)(pb[j] + k);
    };
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (u < mine) fetch(u, u);
    for (int it = 0; it < mine; it += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            if (it + u < mine) {
                f32x4 x[RB], y[CB];
#pragma unroll
                for (int i = 0; i < RB; ++i) x[i] = ra[u][i];
#pragma unroll
                for (int j = 0; j < CB; ++j) y[j] = rb[u][j];
                if (it + u + PF < mine) fetch(u, it + u + PF);
                multiply(x, y);
            }
        }
    }
    // the last, partial chunk (K divides by 4, so a lane's four k are all inside or all outside)
    if (g.K % 16 != 0 && whole % WAVES == wave) {
        const bool ok = 16 * whole + 4 * lq < g.K;
        const int k = ok ? 16 * whole : -4 * lq;                 // outside: the row's first four, zeroed
        f32x4 x[RB], y[CB];
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            x[i] = *(const f32x4 *)(pa[i] + k);
            if (!ok) x[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            y[j] = *(const f32x4 *)(pb[j] + k);
            if (!ok) y[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        multiply(x, y);
    }

    // ---- the eight partial tiles: wavefronts 4..7 hand theirs to 0..3 through LDS, which add them and put
    // the sums back; then all threads add the four sums in order, bias, ReLU, 128-bit stores.
    // Register v of accumulator (i, j), lane (l16, lq): row 16 i + 4 lq + v, column 16 j + l16.
    auto slot = [&](int i, int j, int v) { return (16 * i + 4 * lq + v) * TP + 16 * j + l16; };
    if (wave >= WAVES / 2) {
        float *dst = red[wave - WAVES / 2];
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
            for (int j = 0; j < CB; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) dst[slot(i, j, v)] = acc[i][j][v];
    }
    __syncthreads();
    if (wave < WAVES / 2) {          // reads and writes the same words of its own slot: no other wavefront touches them
        float *dst = red[wave];
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
            for (int j = 0; j < CB; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) dst[slot(i, j, v)] += acc[i][j][v];
    }
    __syncthreads();
    float *__restrict__ out = g.out + w * g.out_stride;
    const float *__restrict__ bias = g.params + w * g.p_stride + g.b_off;
    for (int e = tid; e < TM * (TN / 4); e += FWD_THREADS) {
        const int row = e / (TN / 4), c4 = e % (TN / 4), col = n0 + 4 * c4;
        if (row >= g.B || col >= g.N) continue;
        f32x4 v = *(const f32x4 *)&red[0][row * TP + 4 * c4];
#pragma unroll
        for (int q = 1; q < WAVES / 2; ++q) v += *(const f32x4 *)&red[q][row * TP + 4 * c4];
        v += *(const f32x4 *)(bias + col);
        if (g.relu) {
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = fmaxf(v[c], 0.f);
        }
        *(f32x4 *)(out + (int64_t)row * g.N + col) = v;
    }
}

// Weight (and bias) gradients for batches of at most 4 GROUPS <= 64 samples: mlpwgrad::Args with splits = 1 and
// tiles of 32 rows x 64 columns, one tile per wavefront (a lane loads two consecutive outputs of dz and four of a:
// narrow layers lose less to padding on the row side than with mlp_wgrad.h's 64 x 32, and a lane's four columns
// leave as one 128-bit store).  grid = head_blocks x workers + ceil(tiles x workers / 4) workgroups of four
// wavefronts, each part rounded up to a multiple of XCDS; the workgroups in front of the tiles add the head's
// per-chunk sums as in mlp_wgrad.h.
constexpr int WG_TM = 32, WG_TN = 64;
template <int GROUPS>
__global__ __launch_bounds__(mlpwgrad::THREADS) void wgrad_kernel(mlpwgrad::Args g, fchead::Args h, int chunks, int head_blocks)
{
    constexpr int TM = WG_TM, TN = WG_TN, WAVES = mlpwgrad::WAVES;
    typedef mlpwgrad::Vec<2> vec2;
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles = pick(g.tile_begin, g.layers + 1);
    const int wave_tiles = tiles * g.workers, tile_wgs = (wave_tiles + WAVES - 1) / WAVES;
    const int head_grid = gridDim.x - (tile_wgs + XCDS - 1) / XCDS * XCDS;
    if ((int)blockIdx.x < head_grid) {                          // the whole workgroup
        const int hid = blockIdx.x;
        if (hid < head_blocks * g.workers) fchead::reduce_body(h, chunks, hid % head_blocks, hid / head_blocks);
        return;
    }
    const int b = blockIdx.x - head_grid, per = (gridDim.x - head_grid) / XCDS, id = (b % XCDS) * per + b / XCDS;
    if (id >= tile_wgs) return;
    const int wt = id * WAVES + wave;
    if (wt >= wave_tiles) return;                               // no barrier below
    const int bx = wt % tiles, w = wt / tiles;
    int l = 1;
    while (l < g.layers && bx >= pick(g.tile_begin, l + 1)) ++l;
    const int N = pick(g.n_cols, l), H = pick(g.n_rows, l), ntn = (N + TN - 1) / TN;
    const int t = bx - pick(g.tile_begin, l), m0 = TM * (t / ntn), n0 = TN * (t % ntn);
    const bool bias = pick(g.want_db, l) && n0 == 0;
    // a row pair or column group beyond the matrix (H and N divide by 4): any valid one instead, never stored
    const bool rows_ok = m0 + 2 * l16 < H, cols_ok = n0 + 4 * l16 < N;
    const float *__restrict__ dz = g.dz + w * g.dz_stride + pick(g.dz_off, l) + (rows_ok ? m0 + 2 * l16 : 0);
    const float *__restrict__ av = pick(g.a, l) + w * pick(g.a_stride, l) + (cols_ok ? n0 + 4 * l16 : 0);
    const int64_t a_ld = pick(g.a_ld, l);

    // group u = samples 4 u .. 4 u + 3, lane group lq takes sample 4 u + lq; a sample beyond the batch: a valid
    // row, zeroed (every load unconditional: loads under a condition each cost a register move per element)
    vec2 x[GROUPS];
    f32x4 y[GROUPS];
#pragma unroll
    for (int u = 0; u < GROUPS; ++u) {
        const int sm = 4 * u + lq, sl = sm < g.B ? sm : 0;
        x[u] = *(const vec2 *)(dz + (int64_t)sl * H);
        y[u] = *(const f32x4 *)(av + (int64_t)sl * a_ld);
    }
    __builtin_amdgcn_sched_barrier(0);     // every load in flight before the first multiply (left alone, the compiler
                                           // saves registers by fetching a few groups at a time: 18.1 against 17.6 us)
    // row block i, column block j: tile row 2 m + i, tile column 4 n + j for the instruction's indices m, n
    f32x4 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    float dsum[2] = {0.f, 0.f};
#pragma unroll
    for (int u = 0; u < GROUPS; ++u) {
        vec2 xv = x[u];
        f32x4 yv = y[u];
        if (4 * u + lq >= g.B) {
            xv.v[0] = xv.v[1] = 0.f;
            yv = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            dsum[i] += xv.v[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(xv.v[i], yv[j], acc[i][j], 0, 0, 0);
        }
    }
    // register r of (i, j), lane (l16, lq): tile row 2 (4 lq + r) + i, tile column 4 l16 + j
    float *__restrict__ out = g.grads + w * g.g_stride + pick(g.w_off, l);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 2 * (4 * lq + r) + i;
            const f32x4 v = {acc[i][0][r], acc[i][1][r], acc[i][2][r], acc[i][3][r]};
            if (cols_ok && m0 + row < H) *(f32x4 *)(out + (int64_t)(m0 + row) * N + n0 + 4 * l16) = v;
        }
    if (bias) {
        vec2 v;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            dsum[i] += __shfl_xor(dsum[i], 16, 64);
            dsum[i] += __shfl_xor(dsum[i], 32, 64);
            v.v[i] = dsum[i];
        }
        if (lq == 0 && rows_ok) *(vec2 *)(out + (int64_t)H * N + m0 + 2 * l16) = v;
    }
}

}  // namespace mlpthin
