// Batched fp32 GEMM on the matrix cores, one independent problem per worker:
//   C_w[m][n] = epilogue( sum_k A_w(m, k) * B_w(k, n) ),   w = blockIdx.z
// Every worker has its own operands (its own parameters, its own mini-batch), which is
// what the per-worker gradient of Section 2.1 needs.
//
// Operands are described by small loader structs.  A loader states whether its elements
// are contiguous along k (KC) or along the row index, so that the 64 lanes of a wavefront
// always read consecutive addresses, and the tile keeps that natural layout in LDS.
//
// Workgroup: 256 threads = 4 wavefronts, tile 64 x 64, k-step 32.  Each wavefront owns a
// 32 x 32 quarter as 2 x 2 fragments of v_mfma_f32_16x16x4_f32 (true fp32):
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

constexpr int BM = 64, BN = 64, BK = 32, THREADS = 256;
constexpr int LDS_KC = BK + 4;    // row stride of a k-contiguous tile  [64][36]
constexpr int LDS_RC = 64 + 4;    // row stride of a row-contiguous tile [32][68]

// Dense operand.  KC: element (r, k) at p[w * stride + r * ld + k]; otherwise at
// p[w * stride + k * ld + r].
template <bool KC_>
struct Dense {
    static constexpr bool KC = KC_;
    const float *p;
    int64_t ld, stride;
    __device__ __forceinline__ float load(int w, int r, int k) const
    {
        return KC ? p[w * stride + (int64_t)r * ld + k] : p[w * stride + (int64_t)k * ld + r];
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

// Global -> registers for a 64 x 32 operand tile (8 elements per thread).
template <class L>
__device__ __forceinline__ void fetch_tile(const L &op, int w, int r0, int R, int k0, int K, int tid, float (&v)[8])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int r, k;
        if (L::KC) {
            k = tid % BK;
            r = tid / BK + 8 * j;
        } else {
            r = tid % 64;
            k = tid / 64 + 4 * j;
        }
        v[j] = (r0 + r < R && k0 + k < K) ? op.load(w, r0 + r, k0 + k) : 0.f;
    }
}

template <class L>
__device__ __forceinline__ void commit_tile(float *lds, int tid, const float (&v)[8])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (L::KC)
            lds[(tid / BK + 8 * j) * LDS_KC + tid % BK] = v[j];
        else
            lds[(tid / 64 + 4 * j) * LDS_RC + tid % 64] = v[j];
    }
}

// Values of the four instructions of k group `kg` for the 16-row fragment at row `rbase`.
template <class L>
__device__ __forceinline__ f32x4 frag(const float *lds, int rbase, int kg, int lane)
{
    f32x4 f;
    if (L::KC) {
        f = *(const f32x4 *)&lds[(rbase + (lane & 15)) * LDS_KC + kg * 16 + 4 * (lane >> 4)];
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = lds[(kg * 16 + 4 * (lane >> 4) + j) * LDS_RC + rbase + (lane & 15)];
    }
    return f;
}

constexpr int lds_floats(bool kc) { return kc ? 64 * LDS_KC : BK * LDS_RC; }

// blockIdx.z = worker * splits + split; a split covers k in [split * kper, (split + 1) * kper)
// (kper a multiple of BK) and hands its partial sum to the epilogue, which decides where it
// goes; with splits == 1 the result is final.
template <class LA, class LB, class EP>
__global__ __launch_bounds__(THREADS) void kernel(LA A, LB B, EP E, int M, int N, int K, int splits, int kper)
{
    __shared__ __attribute__((aligned(16))) float As[lds_floats(LA::KC)];
    __shared__ __attribute__((aligned(16))) float Bs[lds_floats(LB::KC)];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int w = blockIdx.z / splits, split = blockIdx.z % splits;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int kbeg = split * kper, kend = min(K, kbeg + kper);
    const int wm = (wave & 1) * 32, wn = (wave >> 1) * 32;

    f32x4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    float ra[8], rb[8];
    fetch_tile(A, w, m0, M, kbeg, kend, tid, ra);
    fetch_tile(B, w, n0, N, kbeg, kend, tid, rb);
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();                       // previous tile fully consumed
        commit_tile<LA>(As, tid, ra);
        commit_tile<LB>(Bs, tid, rb);
        __syncthreads();
        if (k0 + BK < kend) {                  // next tile's loads fly during the MFMAs
            fetch_tile(A, w, m0, M, k0 + BK, kend, tid, ra);
            fetch_tile(B, w, n0, N, k0 + BK, kend, tid, rb);
        }
#pragma unroll
        for (int kg = 0; kg < BK / 16; ++kg) {
            f32x4 fa[2], fb[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) fa[a] = frag<LA>(As, wm + 16 * a, kg, lane);
#pragma unroll
            for (int b = 0; b < 2; ++b) fb[b] = frag<LB>(Bs, wn + 16 * b, kg, lane);
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

template <class LA, class LB, class EP>
inline hipError_t launch(const LA &A, const LB &B, const EP &E, int M, int N, int K, int batch, hipStream_t s,
                         int splits = 1)
{
    int kper = (K + splits - 1) / splits;
    kper = (kper + BK - 1) / BK * BK;
    dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM, batch * splits);
    hipLaunchKernelGGL((kernel<LA, LB, EP>), grid, dim3(THREADS), 0, s, A, B, E, M, N, K, splits, kper);
    return hipGetLastError();
}

}  // namespace bgemm
