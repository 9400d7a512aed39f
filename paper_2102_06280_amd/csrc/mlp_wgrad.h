// Weight and bias gradients of all hidden layers of a multilayer perceptron, all workers, in
// one launch (Section 2.1, stochastic gradient of the local loss):
//   dW_l[m][n] = sum over the batch of dz_l[s][m] a_{l-1}[s][n],   db_l[m] = sum over the batch of dz_l[s][m]
// for the layers below the head (or all layers, when the model has no fused head), reading the deltas
// and activations that the chain kernel (mlp_chain.h) or the per-layer kernels left in the worker's
// scratch block (a_0 = the batch itself).  Widths must divide by 4; tiles of rows or columns that
// stick out over a matrix are computed on any valid data and not stored.
//
// Both operands are stored sample-major, i.e. contiguous along their output index, and the matrix
// instruction v_mfma_f32_16x16x4_f32 leaves open which 16 outputs a tile's rows stand for.  So a lane
// fetches four consecutive outputs of one sample with one 128-bit load straight from global
// memory (the chain kernel wrote them a moment ago: L2 / Infinity Cache), and its four values
// feed four different tiles: tile row i of row block e is output m0 + 4 i + e.  One load of dz
// and one of a per four samples give a wavefront the 16 products of its 64 x 64 output tile; no LDS
// on the way in.  The four wavefronts of a workgroup share the tile and take every fourth group of
// four samples; their accumulators meet in LDS and are added in wavefront order.  Long batches
// are also split over workgroups (blockIdx.z); the partial tiles then go to scratch in the very
// layout of the parameter row (W_1 b_1 W_2 b_2 ...), and reduce_kernel adds them in split order.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "fc_head.h"

namespace mlpwgrad {

using fchead::f32x4;
using fchead::pick;
constexpr int THREADS = 256, WAVES = 4, MAX_L = 8, XCDS = 8;
constexpr int PF = 8;                 // groups of four samples a wavefront keeps in flight

template <int N>
struct alignas(4 * N) Vec {
    float v[N];
};

struct Args {
    int B, layers, workers;                  // batch; l = 1 .. layers
    int n_rows[MAX_L + 1];                   // rows of dW_l = width of layer l, a multiple of 4
    int n_cols[MAX_L + 1];                   // columns of dW_l = width of a_{l-1}, a multiple of 4
    int tile_begin[MAX_L + 2];               // blockIdx.x of layer l's first tile
    int want_db[MAX_L + 1];                  // 0: somebody else computes db_l
    const float *dz;                         // dz_l [B][n_rows] at dz + w * dz_stride + dz_off[l]
    int64_t dz_off[MAX_L + 1], dz_stride;
    const float *a[MAX_L + 1];               // a_{l-1} [B][a_ld] at a[l] + w * a_stride[l]
    int64_t a_ld[MAX_L + 1], a_stride[MAX_L + 1];
    float *grads;                            // worker rows of stride g_stride; W_l [n_rows][n_cols] at w_off[l], then b_l
    int64_t g_stride, w_off[MAX_L + 2];      // w_off[layers + 1] = end of b_layers
    float *part;                             // [worker][split][w_off[layers + 1] - w_off[1]] when splits > 1
    int64_t part_stride;
    int splits, kper;                        // samples per split, a multiple of 4
};

// grid = (head_blocks x workers) + (tiles of all layers x workers x splits), each rounded up to a multiple of XCDS.
// The tile workgroups are renumbered so that the ids one XCD receives are consecutive tiles: the tiles that read
// the same samples of the same worker and layer then share that XCD's L2 instead of fetching them into all eight
// (the head's workgroups stay out of that numbering: as its last ids they would be two whole XCDs' share, and
// the tiles would run on the other six).
// CBK = column blocks of a tile: 64 x 64 tiles (4) or 64 x 32 (2, twice as many workgroups, for launches that
// would otherwise have to split the batch to fill the chip).  The workgroups in front of the tiles add the per-chunk
// sums of the head (fc_head.h), which the chain kernel left before this launch: head_blocks of them per worker.
template <int CBK>
__global__ __launch_bounds__(THREADS, 2) void kernel(Args g, fchead::Args h, int chunks, int head_blocks)
{
    constexpr int TN = 16 * CBK, TP = TN + 4;
    typedef Vec<CBK> vec;
    __shared__ __attribute__((aligned(16))) float red[WAVES - 1][64 * TP];
    __shared__ __attribute__((aligned(16))) float bred[WAVES][64];
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // on the scalar unit: the loops below branch on it
    const int tiles = pick(g.tile_begin, g.layers + 1);
    const int tile_wgs = tiles * g.workers * g.splits;
    const int head_grid = gridDim.x - (tile_wgs + XCDS - 1) / XCDS * XCDS;
    if ((int)blockIdx.x < head_grid) {                          // the whole workgroup, before any barrier
        const int hid = blockIdx.x;
        if (hid < head_blocks * g.workers) fchead::reduce_body(h, chunks, hid % head_blocks, hid / head_blocks);
        return;
    }
    const int b = blockIdx.x - head_grid, per = (gridDim.x - head_grid) / XCDS, id = (b % XCDS) * per + b / XCDS;
    if (id >= tile_wgs) return;
    const int bx = id % tiles, w = (id / tiles) % g.workers, split = id / (tiles * g.workers);
    int l = 1;
    while (l < g.layers && bx >= pick(g.tile_begin, l + 1)) ++l;
    const int N = pick(g.n_cols, l), H = pick(g.n_rows, l), ntn = (N + TN - 1) / TN;
    const int t = bx - pick(g.tile_begin, l), m0 = 64 * (t / ntn), n0 = TN * (t % ntn);
    const int s_begin = split * g.kper, s_end = min(g.B, s_begin + g.kper);
    const bool bias = pick(g.want_db, l) && n0 == 0;

    // a row or column group beyond the matrix (H and N divide by 4): any valid one instead, never stored
    const bool rows_ok = m0 + 4 * l16 < H, cols_ok = n0 + CBK * l16 < N;
    const float *__restrict__ dz = g.dz + w * g.dz_stride + pick(g.dz_off, l) + (rows_ok ? m0 + 4 * l16 : 0);
    const int ncol = cols_ok ? n0 + CBK * l16 : 0;
    const float *__restrict__ av = pick(g.a, l) + w * pick(g.a_stride, l) + ncol;
    const int64_t a_ld = pick(g.a_ld, l);

    f32x4 acc[4][CBK];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < CBK; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 dsum = {0.f, 0.f, 0.f, 0.f};

    // This wavefront's groups of four samples: number wave, wave + 4, ... of the split; lane group lq takes sample lq
    // of a group.  Whole groups run in the main loop, PF of them in flight; the split's last, partial group (if any)
    // belongs to one wavefront and is masked per lane.
    const int len = max(s_end - s_begin, 0), whole = len / 4;
    const int mine = whole > wave ? (whole - wave + WAVES - 1) / WAVES : 0;
    const float *pa = dz + (int64_t)(s_begin + 4 * wave + lq) * H;
    const float *pb = av + (int64_t)(s_begin + 4 * wave + lq) * a_ld;
    const int64_t step_a = (int64_t)4 * WAVES * H, step_b = (int64_t)4 * WAVES * a_ld;
    auto multiply = [&](const f32x4 &x, const vec &y) {
        dsum += x;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < CBK; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[i], y.v[j], acc[i][j], 0, 0, 0);
    };
    f32x4 ra[PF];
    vec rb[PF];
    auto fetch = [&](int u) {
        ra[u] = *(const f32x4 *)(pa + u * step_a);
        rb[u] = *(const vec *)(pb + u * step_b);
    };
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (u < mine) fetch(u);
    pa += PF * step_a;
    pb += PF * step_b;
    // A taken branch costs a stream of matrix instructions about 40 idle cycles (a register-resident loop of 6
    // instructions per iteration runs at 83 % of the rate of the same loop unrolled), so the stretch where all PF
    // groups and their successors exist runs without conditions; the scheduling barriers keep each group's loads next
    // to its multiplies (without them the compiler gathers the loads at the top and the wave waits there).
    int it = 0;
    for (; it + 2 * PF <= mine; it += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const f32x4 x = ra[u];
            const vec y = rb[u];
            fetch(u);
            __builtin_amdgcn_sched_barrier(0);
            multiply(x, y);
            __builtin_amdgcn_sched_barrier(0);
        }
        pa += PF * step_a;
        pb += PF * step_b;
    }
    for (; it < mine; it += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            if (it + u < mine) {
                const f32x4 x = ra[u];
                const vec y = rb[u];
                if (it + u + PF < mine) fetch(u);
                multiply(x, y);
            }
        }
        pa += PF * step_a;
        pb += PF * step_b;
    }
    if (len % 4 != 0 && whole % WAVES == wave) {
        const bool ok = lq < len % 4;
        const int64_t sl = s_begin + 4 * whole + (ok ? lq : 0);      // a lane beyond the batch: a valid row, zeroed
        f32x4 x = *(const f32x4 *)(dz + sl * H);
        vec y = *(const vec *)(av + sl * a_ld);
        if (!ok) {
            x = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < CBK; ++j) y.v[j] = 0.f;
        }
        multiply(x, y);
    }

    // ---- the four wavefronts' tiles: 1, 2, 3 through LDS, added to wavefront 0's in that order.
    // Register r of row block i, lane (l16, lq): output row 4 (4 lq + r) + i, columns CBK l16 .. CBK l16 + CBK - 1.
    if (wave > 0) {
        float *mine_t = red[wave - 1];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                vec v;
#pragma unroll
                for (int j = 0; j < CBK; ++j) v.v[j] = acc[i][j][r];
                *(vec *)&mine_t[(4 * (4 * lq + r) + i) * TP + CBK * l16] = v;
            }
    }
    if (bias) {     // sums over this wavefront's samples: lane groups first
        f32x4 v = dsum;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[e] += __shfl_xor(v[e], 16, 64);
            v[e] += __shfl_xor(v[e], 32, 64);
        }
        if (lq == 0) *(f32x4 *)&bred[wave][4 * l16] = v;
    }
    __syncthreads();
    float *__restrict__ out = g.splits == 1 ? g.grads + w * g.g_stride + pick(g.w_off, l)
                                            : g.part + w * g.part_stride +
                                                  (int64_t)split * (pick(g.w_off, g.layers + 1) - pick(g.w_off, 1)) + (pick(g.w_off, l) - pick(g.w_off, 1));
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 4 * (4 * lq + r) + i;
                vec v;
#pragma unroll
                for (int j = 0; j < CBK; ++j) v.v[j] = acc[i][j][r];
#pragma unroll
                for (int q = 0; q < WAVES - 1; ++q) {
                    const vec o = *(const vec *)&red[q][row * TP + CBK * l16];
#pragma unroll
                    for (int j = 0; j < CBK; ++j) v.v[j] += o.v[j];
                }
                if (cols_ok && m0 + row < H) *(vec *)(out + (int64_t)(m0 + row) * N + n0 + CBK * l16) = v;
            }
    } else if (wave == 1 && bias && lane < 16 && m0 + 4 * lane < H) {
        f32x4 v = *(const f32x4 *)&bred[0][4 * lane];
#pragma unroll
        for (int q = 1; q < WAVES; ++q) v += *(const f32x4 *)&bred[q][4 * lane];
        *(f32x4 *)(out + (int64_t)H * N + m0 + 4 * lane) = v;
    }
}

// grads[w_off[1] .. w_off[layers + 1]) = sum over the splits, in split order, except the bias ranges
// that are somebody else's.  grid = (ceil(length / 4 / 256), workers).
__device__ __forceinline__ void reduce_body(const Args &g, int bx, int w)
{
    const int64_t len = pick(g.w_off, g.layers + 1) - pick(g.w_off, 1);
    const int64_t e = 4 * ((int64_t)bx * 256 + threadIdx.x);
    if (e >= len) return;
    const float *__restrict__ p = g.part + w * g.part_stride + e;
    // all loads in flight; a slot beyond the splits re-reads the last one and adds zero (loads under a condition
    // each would be merged back into one register array with a move per element)
    auto add = [&](auto nq) {
        constexpr int NQ = decltype(nq)::value;
        f32x4 v[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) v[q] = *(const f32x4 *)(p + min(q, g.splits - 1) * len);
        f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < NQ; ++q) t += q < g.splits ? v[q] : f32x4{0.f, 0.f, 0.f, 0.f};
        return t;
    };
    const f32x4 sum = g.splits <= 2 ? add(std::integral_constant<int, 2>{})
                                    : (g.splits <= 4 ? add(std::integral_constant<int, 4>{}) : add(std::integral_constant<int, 8>{}));
    // a group of four lies inside one W_l or one b_l: every boundary is a multiple of 4
    const int64_t pos = pick(g.w_off, 1) + e;
    bool keep = true;
#pragma unroll
    for (int l = 1; l <= MAX_L; ++l)
        if (l <= g.layers && !pick(g.want_db, l) && pos >= pick(g.w_off, l) + (int64_t)pick(g.n_rows, l) * pick(g.n_cols, l) && pos < pick(g.w_off, l + 1))
            keep = false;
    if (keep) *(f32x4 *)(g.grads + w * g.g_stride + pos) = sum;
}

// grid = (ceil(length / 4 / 256), workers)
__global__ __launch_bounds__(256) void reduce_kernel(Args g) { reduce_body(g, blockIdx.x, blockIdx.y); }

}  // namespace mlpwgrad
