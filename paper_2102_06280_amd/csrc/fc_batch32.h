// Fully connected layer for a mini-batch of exactly 32 samples per worker, as three streaming
// kernels (forward, data gradient, weight gradient).
//
// With 32 samples the three products of a wide layer (say 4096 -> 512: 8.4 MB of weights per
// worker) do 64 FLOP per weight byte at most and are bound by reading, or writing, the weight
// matrix once.  The batch is exactly the 32 rows of v_mfma_f32_32x32x2_f32, so every wave
// works on whole 32 x 32 fragments, and all traffic on the weight matrix is 128-bit per lane
// in runs of 512 bytes or more per row.
//
// Fragment layout of v_mfma_f32_32x32x2_f32, lane l: A[m = l % 32][k = l / 32],
// B[k = l / 32][n = l % 32], D: d[v] = D[m = 8 (v / 4) + 4 (l / 32) + v % 4][n = l % 32].
// Which k a given (instruction, k-slot) pair stands for is free as long as A and B agree, and so
// is which output column a (fragment, lane) pair stands for; both freedoms are used to let a
// lane load and store contiguous floats.
//
// All kernels: 256 threads = 4 waves; W is [N][K] row-major per worker (row stride K), worker
// stride w_stride; pointers 16-byte aligned, K and all leading dimensions multiples of 4.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fc32 {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int THREADS = 256;
constexpr int XCDS = 8;

__device__ __forceinline__ int d_row(int v, int lane) { return 8 * (v / 4) + 4 * (lane >> 5) + (v & 3); }

// ---------------------------------------------------------------------------------------------
// out[m][n] = act( sum_k x[m][k] W[n][k] + bias[n] ),  m < 32.
// A workgroup owns 32 output units and the whole k range: its slab of W is 32 full rows, one
// contiguous block.  Wave q takes the q-th quarter of k in windows of 32: lane (r, slot) holds
// the 16 floats k = window + 16 slot + t of row r of both operands, instruction t uses element
// t.  The four partial sums meet in LDS and are added in wave order.
// Workgroup ids are dealt round-robin to the 8 XCDs; the map below keeps all workgroups of one
// worker on one XCD, so that the worker's inputs (read by each of them) stay in that L2.
// Needs K % 128 == 0, N % 32 == 0.  grid = ceil(workers / 8) * 8 * (N / 32).
__global__ __launch_bounds__(THREADS) void forward_kernel(
    int workers, int N, int K, const float *__restrict__ x, int64_t ldx, int64_t x_stride,
    const float *__restrict__ W, int64_t w_stride, const float *__restrict__ bias, int64_t bias_stride, int relu,
    float *__restrict__ out, int64_t ldo, int64_t out_stride)
{
    __shared__ float red[4][32 * 33];
    const int nblk = N / 32;
    const int xcd = blockIdx.x % XCDS, slot_id = blockIdx.x / XCDS;
    const int w = (slot_id / nblk) * XCDS + xcd, n0 = (slot_id % nblk) * 32;
    if (w >= workers) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int q = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, ks = lane >> 5;
    const int kper = K / 4;
    const float *xr = x + w * x_stride + (int64_t)r * ldx + q * kper + 16 * ks;
    const float *wr = W + w * w_stride + (int64_t)(n0 + r) * K + q * kper + 16 * ks;

    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    f32x4 xa[2][4], wb[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        xa[0][j] = *(const f32x4 *)(xr + 4 * j);
        wb[0][j] = __builtin_nontemporal_load((const f32x4 *)(wr + 4 * j));
    }
    const int windows = kper / 32;
    for (int i = 0; i < windows; i += 2) {
        // two windows per trip so that the register buffers are indexed by constants
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int nxt = i + h + 1;
            if (nxt < windows) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    xa[h ^ 1][j] = *(const f32x4 *)(xr + 32 * nxt + 4 * j);
                    wb[h ^ 1][j] = __builtin_nontemporal_load((const f32x4 *)(wr + 32 * nxt + 4 * j));
                }
            }
            if (i + h < windows) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[h][j][e], wb[h][j][e], acc, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) red[q][d_row(v, lane) * 33 + r] = acc[v];
    __syncthreads();
    for (int e = tid; e < 32 * 32; e += THREADS) {
        const int m = e >> 5, n = e & 31;
        float s = red[0][m * 33 + n];
        s += red[1][m * 33 + n];
        s += red[2][m * 33 + n];
        s += red[3][m * 33 + n];
        if (bias) s += bias[w * bias_stride + n0 + n];
        if (relu) s = s > 0.f ? s : 0.f;
        out[w * out_stride + (int64_t)m * ldo + n0 + n] = s;
    }
}

// ---------------------------------------------------------------------------------------------
// The same product split along k: workgroup (slice, worker) multiplies the 256 columns
// k0 = 256 slice .. of x (held in LDS, read from memory once) with the matching 1 KB piece of
// every row of W and writes the partial sums part[worker][slice][m][n]; a separate pass adds the
// slices in order, then bias and activation.  Wave q owns the output units [q N / 4, (q + 1) N / 4)
// as NF fragments of 32; a step is one (32-wide k window, fragment) pair = 16 instructions.
// The B operand wants lane (r, slot) to hold 16 consecutive floats of row r, which as a load
// touches only 32 bytes of each 128-byte line per instruction.  Instead the wave fetches the
// step's 32 x 128 B block of W with whole lines per instruction (lane l: row 8 i + l / 8,
// 16-byte piece l % 8, for i = 0..3), requested two steps ahead, and turns it through a
// 4 KB LDS area of its own (no barrier: one wave writes and reads it, in order).  Piece p of
// row r sits at position p ^ (r % 8) of the row, which spreads both access patterns over all
// banks.
// Compared with forward_kernel the inputs are fetched once instead of once per 32 output units.
// Needs N == 128 NF, K % 256 == 0.  grid = (K / 256, workers).
constexpr int KSLICE = 256;
template <int NF>
__global__ __launch_bounds__(THREADS) void forward_ksplit_kernel(
    int K, const float *__restrict__ x, int64_t ldx, int64_t x_stride, const float *__restrict__ W, int64_t w_stride,
    float *__restrict__ part, int64_t part_stride)
{
    constexpr int LDX = KSLICE + 4, N = 128 * NF, WINDOWS = KSLICE / 32, STEPS = WINDOWS * NF;
    __shared__ __attribute__((aligned(16))) float xs[32 * LDX];
    __shared__ __attribute__((aligned(16))) float turn[4][32 * 32];
    const int slice = blockIdx.x, w = blockIdx.y, k0 = slice * KSLICE;
    const int tid = threadIdx.x, lane = tid & 63;
    const int q = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, ks = lane >> 5;
    for (int e = tid; e < 32 * (KSLICE / 4); e += THREADS) {
        const int m = e / (KSLICE / 4), c4 = e % (KSLICE / 4);
        *(f32x4 *)&xs[m * LDX + 4 * c4] = *(const f32x4 *)(x + w * x_stride + (int64_t)m * ldx + k0 + 4 * c4);
    }
    const int lrow = lane >> 3, piece = lane & 7;
    const float *wl = W + w * w_stride + (int64_t)(q * (N / 4) + lrow) * K + k0 + 4 * piece;
    auto request = [&](int step, f32x4 (&b)[4]) {
        const int win = step / NF, f = step % NF;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            b[i] = __builtin_nontemporal_load((const f32x4 *)(wl + (int64_t)(32 * f + 8 * i) * K + 32 * win));
    };
    float *mine = turn[q];
    const int put = lrow * 32 + 4 * (piece ^ lrow);                  // + 256 i: row 8 i + lrow
    int get[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) get[j] = r * 32 + 4 * ((4 * ks + j) ^ (r & 7));
    f32x16 acc[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[f][v] = 0.f;
    constexpr int AHEAD = 2;                                          // steps requested before they are used
    f32x4 st[AHEAD + 1][4], wb[4], xa[4];
#pragma unroll
    for (int a = 0; a < AHEAD; ++a)
        if (a < STEPS) request(a, st[a]);
    __syncthreads();
#pragma unroll
    for (int step = 0; step < STEPS; ++step) {
        const int win = step / NF, f = step % NF;
        if (step + AHEAD < STEPS) request(step + AHEAD, st[(step + AHEAD) % (AHEAD + 1)]);
#pragma unroll
        for (int i = 0; i < 4; ++i) *(f32x4 *)&mine[put + 256 * i] = st[step % (AHEAD + 1)][i];
#pragma unroll
        for (int j = 0; j < 4; ++j) wb[j] = *(const f32x4 *)&mine[get[j]];
        if (f == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) xa[j] = *(const f32x4 *)&xs[r * LDX + 32 * win + 16 * ks + 4 * j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc[f] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[j][e], wb[j][e], acc[f], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    float *pb = part + w * part_stride + (int64_t)slice * 32 * N + q * (N / 4) + r;
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int v = 0; v < 16; ++v) pb[(int64_t)d_row(v, lane) * N + 32 * f] = acc[f][v];
}

// ---------------------------------------------------------------------------------------------
// dx[m][k] = sum_n dz[m][n] W[n][k]   (kept only where mask[m][k] > 0 when mask is given).
// A wave owns 128 columns k and one of NSPLIT parts of n; a workgroup's four waves cover
// 4 / NSPLIT adjacent column groups, so that NSPLIT = 1 reads 2 KB runs of every row of W (the
// four waves walk down the same rows side by side) and needs no reduction, while NSPLIT = 4
// gives four times as many workgroups for small layers.  Lane (c, slot) loads
// W[n][k0 + 4 c .. + 3] as one 128-bit value and feeds four column fragments with it
// (fragment f, lane column c <-> k = k0 + 4 c + f), so a wave instruction reads 512 contiguous
// bytes of each of two rows and the result leaves as 128-bit stores.  The reduction index of
// instruction (step, j) and slot is n = base + 8 step + 4 slot + j, which makes dz a 128-bit
// load too.  Partial sums of the other parts go through LDS; part 0 adds them in order and stores.
// Needs N % (8 NSPLIT) == 0, K % (512 / NSPLIT) == 0.  grid = (K / (512 / NSPLIT), workers).
template <int NSPLIT>
__global__ __launch_bounds__(THREADS) void dgrad_kernel(
    int N, int K, const float *__restrict__ dz, int64_t lddz, int64_t dz_stride, const float *__restrict__ W,
    int64_t w_stride, const float *__restrict__ mask, int64_t ldmask, int64_t mask_stride, float *__restrict__ dx,
    int64_t lddx, int64_t dx_stride)
{
    constexpr int CW = 4 / NSPLIT;                                   // column groups per workgroup
    __shared__ __attribute__((aligned(16))) float red[NSPLIT > 1 ? (NSPLIT - 1) * CW : 1][NSPLIT > 1 ? 32 * 132 : 4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int q = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int part = q % NSPLIT, cgp = q / NSPLIT;
    const int w = blockIdx.y, k0 = (blockIdx.x * CW + cgp) * 128;
    const int c = lane & 31, ks = lane >> 5;
    const int nper = N / NSPLIT, nb = part * nper;
    const float *zr = dz + w * dz_stride + (int64_t)c * lddz + nb + 4 * ks;            // row m = c
    const float *wc = W + w * w_stride + (int64_t)(nb + 4 * ks) * K + k0 + 4 * c;

    f32x16 acc[4];
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[f][v] = 0.f;
    f32x4 za[2], wb[2][4];
    za[0] = *(const f32x4 *)zr;
#pragma unroll
    for (int j = 0; j < 4; ++j) wb[0][j] = __builtin_nontemporal_load((const f32x4 *)(wc + (int64_t)j * K));
    const int steps = nper / 8;
    for (int i = 0; i < steps; i += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int nxt = i + h + 1;
            if (nxt < steps) {
                za[h ^ 1] = *(const f32x4 *)(zr + 8 * nxt);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    wb[h ^ 1][j] = __builtin_nontemporal_load((const f32x4 *)(wc + (int64_t)(8 * nxt + j) * K));
            }
            if (i + h < steps) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int f = 0; f < 4; ++f)
                        acc[f] = __builtin_amdgcn_mfma_f32_32x32x2f32(za[h][j], wb[h][j][f], acc[f], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (NSPLIT > 1) {
        if (part > 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                f32x4 t = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
                *(f32x4 *)&red[(part - 1) * CW + cgp][d_row(v, lane) * 132 + 4 * c] = t;
            }
        }
        __syncthreads();
    }
    if (part == 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = d_row(v, lane);
            f32x4 t = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
#pragma unroll
            for (int o = 1; o < NSPLIT; ++o) t += *(const f32x4 *)&red[(o - 1) * CW + cgp][m * 132 + 4 * c];
            if (mask) {
                const f32x4 a = *(const f32x4 *)(mask + w * mask_stride + (int64_t)m * ldmask + k0 + 4 * c);
#pragma unroll
                for (int e = 0; e < 4; ++e) t[e] = a[e] > 0.f ? t[e] : 0.f;
            }
            *(f32x4 *)(dx + w * dx_stride + (int64_t)m * lddx + k0 + 4 * c) = t;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// dW[n][k] = sum_m dz[m][n] x[m][k],  m < 32.
// Pure output stream: a wave owns a 32 x 128 block of dW (rows n, columns k = k0 + 4 c + f as
// above), does the 16 reduction steps on values it loads once, and writes 128-bit per lane, 512
// contiguous bytes per row.  Needs N % 32 == 0, K % 512 == 0.  grid = (K / 512, N / 32, workers).
__global__ __launch_bounds__(THREADS) void wgrad_kernel(
    int N, int K, const float *__restrict__ dz, int64_t lddz, int64_t dz_stride, const float *__restrict__ x,
    int64_t ldx, int64_t x_stride, float *__restrict__ dW, int64_t dw_stride)
{
    const int w = blockIdx.z, n0 = blockIdx.y * 32;
    const int tid = threadIdx.x, lane = tid & 63;
    const int q = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int k0 = blockIdx.x * 512 + q * 128;
    const int c = lane & 31, ks = lane >> 5;
    const float *zc = dz + w * dz_stride + (int64_t)ks * lddz + n0 + c;                // A[n = c][m = 2 i + slot]
    const float *xc = x + w * x_stride + (int64_t)ks * ldx + k0 + 4 * c;               // B[m = 2 i + slot][4 columns]

    float za[16];
    f32x4 xb[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        za[i] = zc[(int64_t)(2 * i) * lddz];
        xb[i] = *(const f32x4 *)(xc + (int64_t)(2 * i) * ldx);
    }
    f32x16 acc[4];
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[f][v] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[f] = __builtin_amdgcn_mfma_f32_32x32x2f32(za[i], xb[i][f], acc[f], 0, 0, 0);
    float *ob = dW + w * dw_stride + (int64_t)n0 * K + k0 + 4 * c;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const f32x4 t = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
        __builtin_nontemporal_store(t, (f32x4 *)(ob + (int64_t)d_row(v, lane) * K));
    }
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace fc32
