// Batched fp32 GEMM on the matrix cores, one independent problem per worker:
//   C_w[m][n] = epilogue( sum_k A_w(m, k) * B_w(k, n) ),   w = blockIdx.z / splits
// Every worker has its own operands (its own parameters, its own mini-batch), which is
// what the per-worker gradient of Section 2.1 needs.
//
// Operands are described by small loader structs.  A loader splits the address of element
// (row, k) into a part that depends on the row only (`row_ctx`), a part that depends on k
// only (`k_ctx`) and a cheap combination (`load`), all in 32-bit arithmetic relative to
// the worker's base pointer, and states whether its elements are contiguous along k (KC)
// or along the row index.
// The global -> LDS copy assigns work so that one of the two indices is the same for a
// whole wavefront and the other runs with the lane: for a KC operand a wavefront reads 64
// consecutive k of one row, otherwise 64 consecutive rows of one k.  Loads are therefore
// coalesced; the context of the wave-uniform index is computed on the scalar unit, the
// per-lane context once per k-step (KC) or once per kernel (otherwise).
// The tile keeps the operand's natural layout in LDS.
//
// Workgroup: 256 threads = 4 wavefronts, tile BM x BN (64 x 64 or 32 x 128), k-step 64.
// Each wavefront owns a 32 x 32 part as 2 x 2 fragments of v_mfma_f32_16x16x4_f32 (true fp32):
//   A fragment: lane l holds A[m = l % 16][slot l / 16], B fragment: B[slot l / 16][n = l % 16]
//   D: 4 floats, d[v] = D[m = 4 * (l / 16) + v][n = l % 16]
// The four k-slots of instruction j (0..3) of a 16-wide k group are k = 4 * slot + j for
// both operands, which lets a k-contiguous operand fetch four instructions' worth of
// values with one 128-bit LDS read.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bgemm {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64, THREADS = 256;
constexpr int LDS_KC = BK + 4;                       // row stride of a k-contiguous tile [rows][68]
constexpr int lds_rc(int rows) { return rows + 4; }  // row stride of a row-contiguous tile [64][rows + 4]
constexpr int lds_floats(bool kc, int rows) { return kc ? rows * LDS_KC : BK * lds_rc(rows); }

// Dense operand.  KC: element (r, k) at p[w * stride + r * ld + k]; otherwise at
// p[w * stride + k * ld + r].  Offsets inside one worker's block fit 32 bits.
// `vec` (set by launch() when every row of the operand starts on a 16-byte boundary and the
// extents divide by 4) lets the tile be fetched with 128-bit loads.
template <bool KC_>
struct Dense {
    static constexpr bool KC = KC_;
    static constexpr bool CAN_VEC = true;
    const float *p;
    int64_t ld, stride;
    bool vec;
    struct RowCtx { int off; bool ok; };
    struct KCtx { int off; bool ok; };
    __device__ __forceinline__ RowCtx row_ctx(int r, bool ok) const { return {KC ? r * (int)ld : r, ok}; }
    __device__ __forceinline__ KCtx k_ctx(int k, bool ok) const { return {KC ? k : k * (int)ld, ok}; }
    __device__ __forceinline__ float load(int w, const RowCtx &r, const KCtx &k) const
    {
        const bool ok = r.ok && k.ok;
        const float v = (p + w * stride)[ok ? r.off + k.off : 0];
        return ok ? v : 0.f;
    }
};

// Epilogue: optional per-column bias, ReLU, or masking by the sign of another matrix.
struct Epilogue {
    float *C;
    int64_t ldc, strideC;
    const float *bias;      // [n], per worker stride strideBias; nullptr = none
    int64_t strideBias;
    const float *mask;      // keep C[m][n] only where mask[m][n] > 0; nullptr = none
    int64_t ldmask, strideMask;
    int relu;
    __device__ __forceinline__ void store(int w, int /*split*/, int m, int n, float v) const
    {
        if (bias) v += bias[w * strideBias + n];
        if (relu) v = v > 0.f ? v : 0.f;
        if (mask) v = mask[w * strideMask + (int64_t)m * ldmask + n] > 0.f ? v : 0.f;
        C[w * strideC + (int64_t)m * ldc + n] = v;
    }
};

// Global -> registers for a ROWS x 64 operand tile (ROWS / 4 elements per thread).
//   KC: element j of the thread is (row = wave + 4 j, k = lane)
//   RC: ROWS >= 64; element j is (row = lane + 64 (j % (ROWS / 64)), k = wave + 4 (j / (ROWS / 64)))
// `rows` holds the per-lane row contexts of an RC operand (computed once per kernel).
template <class L, int ROWS>
struct RowCache {
    typename L::RowCtx c[L::KC ? 1 : ROWS / 64];
};

template <class L, int ROWS>
__device__ __forceinline__ void make_rows(const L &op, int r0, int R, int lane, RowCache<L, ROWS> &rows)
{
    if (!L::KC) {
#pragma unroll
        for (int g = 0; g < ROWS / 64; ++g) {
            const int r = r0 + lane + 64 * g;
            rows.c[g] = op.row_ctx(r < R ? r : 0, r < R);
        }
    }
}

template <class L, int ROWS>
__device__ __forceinline__ void fetch_tile(const L &op, int w, int r0, int R, int k0, int K, int wave, int lane,
                                           const RowCache<L, ROWS> &rows, float (&v)[ROWS / 4])
{
    static_assert(L::KC || ROWS >= 64, "a row-contiguous operand needs at least 64 tile rows");
    if (L::KC) {
        const int k = k0 + lane;
        const typename L::KCtx kc = op.k_ctx(k < K ? k : 0, k < K);      // per lane, shared by all rows
#pragma unroll
        for (int j = 0; j < ROWS / 4; ++j) {
            const int r = r0 + wave + 4 * j;                                 // wave-uniform
            v[j] = op.load(w, op.row_ctx(r < R ? r : 0, r < R), kc);
        }
    } else {
        constexpr int RG = ROWS / 64;
#pragma unroll
        for (int j = 0; j < ROWS / 4; ++j) {
            const int k = k0 + wave + 4 * (j / RG);                          // wave-uniform
            v[j] = op.load(w, rows.c[j % RG], op.k_ctx(k < K ? k : 0, k < K));
        }
    }
}

// 128-bit variants for dense operands (ROWS / 16 float4 per thread, float4 index f = tid + 256 j):
//   KC: (row = f / 16, k = 4 (f % 16)): a wave instruction reads 256 contiguous bytes of four rows
//   RC: (k = f / (ROWS / 4), row = 4 (f % (ROWS / 4))): ROWS contiguous floats of one k
// A float4 outside the operand is read from offset 0 instead and its bit in `okbits` stays clear;
// the value is only replaced by zero when the tile is written to LDS (commit_tile_vec).  Masking
// right after the load would make the wave wait for the load before its matrix instructions, and
// the point of fetching one k-step ahead is that the loads are in flight during them.
template <class L, int ROWS>
__device__ __forceinline__ void fetch_tile_vec(const L &op, int w, int r0, int R, int k0, int K, int tid,
                                               float (&v)[ROWS / 4], uint32_t &okbits)
{
    okbits = 0;
    const float *base = op.p + w * op.stride;
#pragma unroll
    for (int j = 0; j < ROWS / 16; ++j) {
        const int f = tid + 256 * j;
        int r, k;
        if (L::KC) {
            r = r0 + (f >> 4);
            k = k0 + 4 * (f & 15);
        } else {
            r = r0 + 4 * (f % (ROWS / 4));
            k = k0 + f / (ROWS / 4);
        }
        const bool ok = r < R && k < K;
        const int off = ok ? (L::KC ? r * (int)op.ld + k : k * (int)op.ld + r) : 0;
        const f32x4 q = *(const f32x4 *)(base + off);
        okbits |= (ok ? 1u : 0u) << j;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[4 * j + e] = q[e];
    }
}

template <class L, int ROWS>
__device__ __forceinline__ void commit_tile_vec(float *lds, int tid, const float (&v)[ROWS / 4], uint32_t okbits)
{
#pragma unroll
    for (int j = 0; j < ROWS / 16; ++j) {
        const int f = tid + 256 * j;
        const bool ok = (okbits >> j) & 1u;
        const f32x4 q = {ok ? v[4 * j] : 0.f, ok ? v[4 * j + 1] : 0.f, ok ? v[4 * j + 2] : 0.f, ok ? v[4 * j + 3] : 0.f};
        if (L::KC)
            *(f32x4 *)&lds[(f >> 4) * LDS_KC + 4 * (f & 15)] = q;
        else
            *(f32x4 *)&lds[(f / (ROWS / 4)) * lds_rc(ROWS) + 4 * (f % (ROWS / 4))] = q;
    }
}

template <class L>
struct can_vec {
    template <class T> static constexpr auto test(int) -> decltype(T::CAN_VEC, true) { return T::CAN_VEC; }
    template <class T> static constexpr bool test(...) { return false; }
    static constexpr bool value = test<L>(0);
};
template <class L>
__host__ __device__ __forceinline__ bool use_vec(const L &op)
{
    if constexpr (can_vec<L>::value) return op.vec;
    else return false;
}

template <class L, int ROWS>
__device__ __forceinline__ void commit_tile(float *lds, int wave, int lane, const float (&v)[ROWS / 4])
{
#pragma unroll
    for (int j = 0; j < ROWS / 4; ++j) {
        if (L::KC)
            lds[(wave + 4 * j) * LDS_KC + lane] = v[j];
        else
            lds[(wave + 4 * (j / (ROWS / 64))) * lds_rc(ROWS) + lane + 64 * (j % (ROWS / 64))] = v[j];
    }
}

// Values of the four instructions of k group `kg` for the 16-row fragment at row `rbase`.
template <class L, int ROWS>
__device__ __forceinline__ f32x4 frag(const float *lds, int rbase, int kg, int lane)
{
    f32x4 f;
    if (L::KC) {
        f = *(const f32x4 *)&lds[(rbase + (lane & 15)) * LDS_KC + kg * 16 + 4 * (lane >> 4)];
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = lds[(kg * 16 + 4 * (lane >> 4) + j) * lds_rc(ROWS) + rbase + (lane & 15)];
    }
    return f;
}

// blockIdx.z = worker * splits + split; a split covers k in [split * kper, (split + 1) * kper)
// (kper a multiple of BK) and hands its partial sum to the epilogue, which decides where it
// goes; with splits == 1 the result is final.
// VA / VB: fetch the A / B tile with 128-bit loads (see mark_vec).
template <class LA, class LB, class EP, int BM, int BN, bool VA, bool VB>
__global__ __launch_bounds__(THREADS) void kernel(LA A, LB B, EP E, int M, int N, int K, int splits, int kper)
{
    static_assert((BM == 64 && BN == 64) || (BM == 32 && BN == 128), "supported tiles: 64 x 64, 32 x 128");
    static_assert(BM == 64 || LA::KC, "the 32-row tile needs a k-contiguous A operand");
    __shared__ __attribute__((aligned(16))) float As[lds_floats(LA::KC, BM)];
    __shared__ __attribute__((aligned(16))) float Bs[lds_floats(LB::KC, BN)];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int w = blockIdx.z / splits, split = blockIdx.z % splits;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int kbeg = split * kper, kend = min(K, kbeg + kper);
    constexpr int WM = BM / 32;                          // waves along m
    const int wm = (wave % WM) * 32, wn = (wave / WM) * 32;

    f32x4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    RowCache<LA, BM> arows;
    RowCache<LB, BN> brows;
    make_rows<LA, BM>(A, m0, M, lane, arows);
    make_rows<LB, BN>(B, n0, N, lane, brows);
    float ra[BM / 4], rb[BN / 4];
    uint32_t oka = 0, okb = 0;
    auto fetch = [&](int k0) {
        if constexpr (VA) fetch_tile_vec<LA, BM>(A, w, m0, M, k0, kend, tid, ra, oka);
        else fetch_tile<LA, BM>(A, w, m0, M, k0, kend, wave, lane, arows, ra);
        if constexpr (VB) fetch_tile_vec<LB, BN>(B, w, n0, N, k0, kend, tid, rb, okb);
        else fetch_tile<LB, BN>(B, w, n0, N, k0, kend, wave, lane, brows, rb);
    };
    fetch(kbeg);
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();                       // previous tile fully consumed
        if constexpr (VA) commit_tile_vec<LA, BM>(As, tid, ra, oka); else commit_tile<LA, BM>(As, wave, lane, ra);
        if constexpr (VB) commit_tile_vec<LB, BN>(Bs, tid, rb, okb); else commit_tile<LB, BN>(Bs, wave, lane, rb);
        __syncthreads();
        if (k0 + BK < kend) fetch(k0 + BK);    // next tile's loads fly during the MFMAs
        if constexpr (VA || VB) __builtin_amdgcn_sched_barrier(0);   // nothing that consumes them moves up here
#pragma unroll
        for (int kg = 0; kg < BK / 16; ++kg) {
            f32x4 fa[2], fb[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) fa[a] = frag<LA, BM>(As, wm + 16 * a, kg, lane);
#pragma unroll
            for (int b = 0; b < 2; ++b) fb[b] = frag<LB, BN>(Bs, wn + 16 * b, kg, lane);
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[a][j], fb[b][j], acc[a][b], 0, 0, 0);
        }
    }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int n = n0 + wn + 16 * b + (lane & 15);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = m0 + wm + 16 * a + 4 * (lane >> 4) + v;
                if (m < M && n < N) E.store(w, split, m, n, acc[a][b][v]);
            }
        }
}

// 128-bit tile fetches need every row of the operand on a 16-byte boundary and the contiguous
// extent (k for a k-contiguous operand, rows otherwise) divisible by 4.  The choice is a template
// parameter of the kernel: as a run-time branch inside it, it cost the 32-bit path 15-20 %.
template <class L>
inline void mark_vec(L &op, int rows, int K)
{
    if constexpr (can_vec<L>::value) {
        const int contiguous = L::KC ? K : rows;
        op.vec = ((uintptr_t)op.p % 16 == 0) && op.ld % 4 == 0 && op.stride % 4 == 0 && contiguous % 4 == 0;
    }
}

// BM = 32 uses 32 x 128 tiles (for problems with at most 32 rows), otherwise 64 x 64.
template <int BM, class LA, class LB, class EP>
inline hipError_t launch(const LA &A, const LB &B, const EP &E, int M, int N, int K, int batch, hipStream_t s,
                         int splits = 1)
{
    constexpr int BN = BM == 32 ? 128 : 64;
    int kper = (K + splits - 1) / splits;
    kper = (kper + BK - 1) / BK * BK;
    dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM, batch * splits);
    LA a = A;
    LB b = B;
    mark_vec(a, M, K);
    mark_vec(b, N, K);
    const bool va = use_vec(a), vb = use_vec(b);
    auto go = [&](auto kern) { hipLaunchKernelGGL(kern, grid, dim3(THREADS), 0, s, a, b, E, M, N, K, splits, kper); };
    constexpr bool CA = can_vec<LA>::value, CB = can_vec<LB>::value;
    if constexpr (CA && CB) {
        if (va && vb) go(kernel<LA, LB, EP, BM, BN, true, true>);
        else if (va) go(kernel<LA, LB, EP, BM, BN, true, false>);
        else if (vb) go(kernel<LA, LB, EP, BM, BN, false, true>);
        else go(kernel<LA, LB, EP, BM, BN, false, false>);
    } else if constexpr (CA) {
        if (va) go(kernel<LA, LB, EP, BM, BN, true, false>);
        else go(kernel<LA, LB, EP, BM, BN, false, false>);
    } else if constexpr (CB) {
        if (vb) go(kernel<LA, LB, EP, BM, BN, false, true>);
        else go(kernel<LA, LB, EP, BM, BN, false, false>);
    } else {
        go(kernel<LA, LB, EP, BM, BN, false, false>);
    }
    return hipGetLastError();
}

}  // namespace bgemm
