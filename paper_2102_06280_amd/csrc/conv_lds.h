// Stride-1 'same' convolution on the matrix cores with the input image resident in LDS.
//
// One workgroup computes all output channels of one sample of one worker:
//   out[co][y][x] = bias[co] + sum_{c, kh, kw} Wt[co][c][kh][kw] * in[c][y + kh - pad][x + kw - pad]
// as the GEMM  out[co][pix] = sum_k Wt[co][k] * patch[k][pix],  k = (c, kh, kw).
// The patch matrix repeats every input value KS * KS times, so it is never built and never
// fetched: a group of CG input channels is copied once into LDS with a zero halo
// ([CG][H + 2 pad][W + 2 pad]; 160 KB of LDS per CU make a whole 32-channel 16 x 16 image
// fit), and the B fragment of v_mfma_f32_16x16x4_f32 is read straight from it at
// address  pixel_offset(lane) + tap_offset(k)  with no bounds checks.  Tap offsets come
// from a small LDS table, the weights stream through LDS in 64-wide k chunks (double
// buffered).  Accumulators stay in registers across channel groups.
//
// The data gradient of a convolution is the same operation applied to the output deltas
// with the filters transposed and rotated by 180 degrees (see flip_filters_kernel).
//
// Fragment layout of v_mfma_f32_16x16x4_f32, lane l: A[m = l % 16][slot l / 16],
// B[slot l / 16][n = l % 16], D: d[v] = D[m = 4 (l / 16) + v][n = l % 16]; instruction j of a
// 16-wide k group uses k = 4 slot + j.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace convlds {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// Four horizontally adjacent pixels (x = 4 x4 .. 4 x4 + 3 of image row y) of a map that is stored
// as its 2 x 2 max-pooled gradient plus the window codes written by the POOL epilogue: a pixel
// holds the pooled gradient of its window if it was the window's first maximum, else zero.
// `pooled` / `code` point at the plane [H/2][W/2] of one (sample, channel).
__device__ __forceinline__ float4 expand_pooled(const float *pooled, const uint8_t *code, int y, int x4, int W)
{
    const int o = (y >> 1) * (W >> 1) + 2 * x4;
    const float2 g = *(const float2 *)&pooled[o];
    const uint32_t c = *(const uint16_t *)&code[o];
    const uint32_t c0 = c & 0xffu, c1 = c >> 8, pos = (uint32_t)(y & 1) * 2u;
    return make_float4(c0 == pos ? g.x : 0.f, c0 == pos + 1 ? g.x : 0.f, c1 == pos ? g.y : 0.f, c1 == pos + 1 ? g.y : 0.f);
}

// CG: input channels per LDS fill; MT: 16-row output-channel fragments (all held by every
// wave); NT: 16-pixel fragments per wave; WAVES * NT * 16 = H * W pixels per sample.
template <int CG, int MT, int NT, int H, int W, int KS, int WAVES>
struct Cfg {
    static constexpr int PAD = KS / 2, HP = H + 2 * PAD, WP = W + 2 * PAD;
    static constexpr int COUT = 16 * MT, PIX = H * W, KK = KS * KS;
    static constexpr int TAPS = CG * KK;                 // k extent of one channel group
    static constexpr int KGS = (TAPS + 15) / 16;         // 16-wide k groups per channel group
    static constexpr int CHUNKS = (KGS + 3) / 4;         // 64-wide weight chunks per channel group
    static constexpr int IMG = CG * HP * WP;
    static constexpr int LDA = 68;                       // row stride of a weight chunk [COUT][64]
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int AROWS = COUT / WAVES;           // weight rows fetched per thread and chunk
    static_assert(PIX == 16 * NT * WAVES, "waves x fragments must cover the image");
    static_assert(W % 4 == 0 && COUT % WAVES == 0, "shape not supported");
    static constexpr size_t lds_bytes = sizeof(float) * (IMG + 2 * COUT * LDA) + sizeof(int) * KGS * 16;
};

// The value of the horizontally adjacent lane (lane ^ 1) as one data-parallel move (quad permutation 1, 0, 3, 2)
// instead of a round trip through the LDS crossbar.
__device__ __forceinline__ float neighbour_lane(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
}

// The bias values of the output channels a lane's accumulator registers stand for (channel 16 mt + 4 (lane / 16) + v),
// fetched once, ahead of the multiplies.  Loaded inside the epilogue instead, each of them made the wave wait for the
// load and for every store issued before it (one counter covers both), eight times per sample.
template <int MT>
__device__ __forceinline__ void load_bias(float (&bv)[MT][4], const float *bias, int lane)
{
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 4; ++v) bv[mt][v] = bias ? bias[16 * mt + 4 * (lane >> 4) + v] : 0.f;
}

// ReLU + 2 x 2 max pooling of one sample's accumulators, written as the pooled map ob [COUT][H/2][W/2]
// and the window codes cb of the same shape (see conv_forward_kernel).  A wave's fragments cover
// whole pairs of image rows, so a window is two accumulators of one lane and of its neighbour.
template <int MT, int NT, int H, int W>
__device__ __forceinline__ void relu_pool_store(const f32x4 (&acc)[MT][NT], const float (&bv)[MT][4], float *ob, uint8_t *cb,
                                                int wave, int lane)
{
    constexpr int FR = W / 16;                       // fragments per image row
    static_assert((NT * 16) % (2 * W) == 0 && H % 2 == 0, "a wave must cover whole pairs of rows");
    constexpr int PP = (H / 2) * (W / 2);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int co = 16 * mt + 4 * (lane >> 4) + v;
#pragma unroll
            for (int nf = 0; nf < NT; ++nf) {
                if ((nf / FR) % 2) continue;         // lower row of a pair: handled with the upper one
                const int p = (wave * NT + nf) * 16 + (lane & 15);
                const int y = p / W, x = p % W;
                const float a = acc[mt][nf][v] + bv[mt][v], c = acc[mt][nf + FR][v] + bv[mt][v];
                const float a1 = neighbour_lane(a), c1 = neighbour_lane(c);
                // window (y, x) (y, x+1) (y+1, x) (y+1, x+1): the first element that attains the maximum, as selects
                const float m = fmaxf(fmaxf(a, a1), fmaxf(c, c1));
                int arg = c == m ? 2 : 3;
                arg = a1 == m ? 1 : arg;
                arg = a == m ? 0 : arg;
                arg = m > 0.f ? arg : 4;
                if ((lane & 1) == 0) {               // even x
                    const int o = co * PP + (y / 2) * (W / 2) + x / 2;
                    ob[o] = fmaxf(m, 0.f);
                    cb[o] = (uint8_t)arg;
                }
            }
        }
}

// in  [worker][B][Cin][H][W]   (worker stride in_stride)
// wgt [worker][COUT][ldw]      (row co holds its Cin * KK filter taps, worker stride w_stride)
// out [worker][B][COUT][H][W]  (worker stride out_stride);  grid = (B, workers)
// POOL: the epilogue applies ReLU and 2 x 2 max pooling and writes out [worker][B][COUT][H/2][W/2]
// together with code [worker][B][COUT][H/2][W/2] (one byte: which element of the window, in the
// order (0,0) (0,1) (1,0) (1,1), was the first to attain the maximum, or 4 when the maximum is
// not positive); the pre-activation map is not written at all.  A wave's fragments cover whole
// pairs of image rows, so a window is two accumulators of one lane and of its neighbour.
// EXPAND: the input is given as in [worker][B][Cin][H/2][W/2] (pooled gradients) with in_code of the same
// shape and is expanded to [Cin][H][W] while it is copied into LDS (see expand_pooled): the data-gradient
// convolution then needs no un-pooled delta map in memory.
template <int CG, int MT, int NT, int H, int W, int KS, int WAVES, bool POOL = false, bool EXPAND = false>
__global__ __launch_bounds__(64 * WAVES) void conv_forward_kernel(
    const float *__restrict__ in, int64_t in_stride, const float *__restrict__ wgt, int64_t w_stride, int ldw,
    const float *__restrict__ bias, int64_t bias_stride, float *__restrict__ out, int64_t out_stride, int Cin,
    uint8_t *__restrict__ code = nullptr, int64_t code_stride = 0, const uint8_t *__restrict__ in_code = nullptr,
    int64_t in_code_stride = 0)
{
    using C = Cfg<CG, MT, NT, H, W, KS, WAVES>;
    __shared__ __attribute__((aligned(16))) float img[C::IMG];
    __shared__ __attribute__((aligned(16))) float As[2][C::COUT * C::LDA];
    __shared__ __attribute__((aligned(16))) int taptab[C::KGS * 16];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = blockIdx.x, w = blockIdx.y;

    for (int k = tid; k < C::KGS * 16; k += C::THREADS) {
        const int c = k / C::KK, rr = k % C::KK, kh = rr / KS, kw = rr % KS;
        taptab[k] = k < C::TAPS ? c * C::HP * C::WP + kh * C::WP + kw : 0;
    }
    for (int e = tid; e < C::IMG; e += C::THREADS) img[e] = 0.f;     // the halo stays zero

    int pixoff[NT];
#pragma unroll
    for (int nf = 0; nf < NT; ++nf) {
        const int p = (wave * NT + nf) * 16 + (lane & 15);
        pixoff[nf] = (p / W) * C::WP + (p % W);
    }
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nf = 0; nf < NT; ++nf) acc[mt][nf] = f32x4{0.f, 0.f, 0.f, 0.f};

    float bv[MT][4];
    load_bias<MT>(bv, bias ? bias + w * bias_stride : nullptr, lane);
    const float *inb = in + w * in_stride + (int64_t)b * Cin * (EXPAND ? C::PIX / 4 : C::PIX);
    const uint8_t *icb = EXPAND ? in_code + w * in_code_stride + (int64_t)b * Cin * (C::PIX / 4) : nullptr;
    const float *ww = wgt + w * w_stride;
    const int groups = (Cin + CG - 1) / CG;

    float areg[C::AROWS];
    auto fetch_a = [&](int g, int chunk) {
        const int kloc = chunk * 64 + lane;
        const bool ok = kloc < C::TAPS && g * CG + kloc / C::KK < Cin;
        const int kglob = ok ? g * C::TAPS + kloc : 0;
#pragma unroll
        for (int j = 0; j < C::AROWS; ++j) {
            const float v = ww[(wave + WAVES * j) * ldw + kglob];
            areg[j] = ok ? v : 0.f;
        }
    };
    auto commit_a = [&](int buf) {
#pragma unroll
        for (int j = 0; j < C::AROWS; ++j) As[buf][(wave + WAVES * j) * C::LDA + lane] = areg[j];
    };

    int buf = 0;
    for (int g = 0; g < groups; ++g) {
        __syncthreads();                       // image and weight buffers of the previous group are free
        for (int e = tid; e < CG * H * (W / 4); e += C::THREADS) {
            const int c = e / (H * (W / 4)), rem = e % (H * (W / 4)), y = rem / (W / 4), x4 = rem % (W / 4);
            const int ch = g * CG + c;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (ch < Cin) {
                if (EXPAND)
                    v = expand_pooled(inb + ch * (C::PIX / 4), icb + ch * (C::PIX / 4), y, x4, W);
                else
                    v = *(const float4 *)&inb[(ch * H + y) * W + 4 * x4];
            }
            float *dst = &img[c * C::HP * C::WP + (y + C::PAD) * C::WP + C::PAD + 4 * x4];
            dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        }
        fetch_a(g, 0);
        commit_a(buf);
        __syncthreads();
        for (int chunk = 0; chunk < C::CHUNKS; ++chunk) {
            if (chunk + 1 < C::CHUNKS) fetch_a(g, chunk + 1);
#pragma unroll
            for (int kgl = 0; kgl < 4; ++kgl) {
                const int kg = chunk * 4 + kgl;
                if (kg < C::KGS) {
                    const i32x4 tap = *(const i32x4 *)&taptab[kg * 16 + 4 * (lane >> 4)];
                    f32x4 fa[MT], fb[NT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        fa[mt] = *(const f32x4 *)&As[buf][(16 * mt + (lane & 15)) * C::LDA + kgl * 16 + 4 * (lane >> 4)];
#pragma unroll
                    for (int nf = 0; nf < NT; ++nf)
#pragma unroll
                        for (int j = 0; j < 4; ++j) fb[nf][j] = img[pixoff[nf] + tap[j]];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int nf = 0; nf < NT; ++nf)
                                acc[mt][nf] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[mt][j], fb[nf][j], acc[mt][nf], 0, 0, 0);
                }
            }
            if (chunk + 1 < C::CHUNKS) commit_a(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }

    if (POOL) {
        constexpr int PP = (H / 2) * (W / 2);
        relu_pool_store<MT, NT, H, W>(acc, bv, out + w * out_stride + (int64_t)b * C::COUT * PP,
                                      code + w * code_stride + (int64_t)b * C::COUT * PP, wave, lane);
        return;
    }
    float *ob = out + w * out_stride + (int64_t)b * C::COUT * C::PIX;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int co = 16 * mt + 4 * (lane >> 4) + v;
#pragma unroll
            for (int nf = 0; nf < NT; ++nf) {
                const int p = (wave * NT + nf) * 16 + (lane & 15);
                ob[co * C::PIX + p] = acc[mt][nf][v] + bv[mt][v];
            }
        }
}

// conv_forward_kernel with POOL for a layer whose input channels all fit one LDS fill (Cin <= CG)
// and whose filters fit the two weight buffers: a workgroup keeps the filters in LDS and runs
// through SB consecutive samples.  The next sample's image is requested before the multiplies
// of the current one and put into LDS after them, so that neither the filter fetch nor the
// image fetch is waited for more than once per workgroup.  grid = (ceil(B / SB), workers).
template <int CG, int MT, int NT, int H, int W, int KS, int WAVES, int SB>
__global__ __launch_bounds__(64 * WAVES) void conv_forward_pool_multi_kernel(
    const float *__restrict__ in, int64_t in_stride, const float *__restrict__ wgt, int64_t w_stride, int ldw,
    const float *__restrict__ bias, int64_t bias_stride, float *__restrict__ out, int64_t out_stride, int Cin, int B,
    uint8_t *__restrict__ code, int64_t code_stride)
{
    using C = Cfg<CG, MT, NT, H, W, KS, WAVES>;
    static_assert(C::CHUNKS <= 2, "the filters must fit the two weight buffers");
    constexpr int QUADS = CG * H * (W / 4), PER = (QUADS + C::THREADS - 1) / C::THREADS, PP = (H / 2) * (W / 2);
    __shared__ __attribute__((aligned(16))) float img[C::IMG];
    __shared__ __attribute__((aligned(16))) float As[2][C::COUT * C::LDA];
    __shared__ __attribute__((aligned(16))) int taptab[C::KGS * 16];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b0 = blockIdx.x * SB, w = blockIdx.y;

    for (int k = tid; k < C::KGS * 16; k += C::THREADS) {
        const int c = k / C::KK, rr = k % C::KK, kh = rr / KS, kw = rr % KS;
        taptab[k] = k < C::TAPS ? c * C::HP * C::WP + kh * C::WP + kw : 0;
    }
    for (int e = tid; e < C::IMG; e += C::THREADS) img[e] = 0.f;     // the halo stays zero

    int pixoff[NT];
#pragma unroll
    for (int nf = 0; nf < NT; ++nf) {
        const int p = (wave * NT + nf) * 16 + (lane & 15);
        pixoff[nf] = (p / W) * C::WP + (p % W);
    }
    const float *ww = wgt + w * w_stride;
#pragma unroll
    for (int chunk = 0; chunk < C::CHUNKS; ++chunk) {
        const int kloc = chunk * 64 + lane;
        const bool ok = kloc < C::TAPS && kloc / C::KK < Cin;
#pragma unroll
        for (int j = 0; j < C::AROWS; ++j) {
            const float v = ww[(wave + WAVES * j) * ldw + (ok ? kloc : 0)];
            As[chunk][(wave + WAVES * j) * C::LDA + lane] = ok ? v : 0.f;
        }
    }

    float bv[MT][4];
    load_bias<MT>(bv, bias ? bias + w * bias_stride : nullptr, lane);
    float4 iv[PER];
    auto request_image = [&](int b) {
        const float *inb = in + w * in_stride + (int64_t)b * Cin * C::PIX;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int e = tid + u * C::THREADS;
            const int c = e / (H * (W / 4)), rem = e % (H * (W / 4));
            iv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (e < QUADS && c < Cin) iv[u] = *(const float4 *)&inb[c * C::PIX + 4 * rem];
        }
    };
    auto put_image = [&]() {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int e = tid + u * C::THREADS;
            if (e < QUADS) {
                const int c = e / (H * (W / 4)), rem = e % (H * (W / 4)), y = rem / (W / 4), x4 = rem % (W / 4);
                float *dst = &img[c * C::HP * C::WP + (y + C::PAD) * C::WP + C::PAD + 4 * x4];
                dst[0] = iv[u].x; dst[1] = iv[u].y; dst[2] = iv[u].z; dst[3] = iv[u].w;
            }
        }
    };
    request_image(b0);
    __syncthreads();                                   // the zero fill is complete
    put_image();
    __syncthreads();

    for (int sidx = 0; sidx < SB; ++sidx) {
        const int b = b0 + sidx;
        const bool more = sidx + 1 < SB && b + 1 < B;  // uniform over the workgroup
        if (more) request_image(b + 1);
        f32x4 acc[MT][NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nf = 0; nf < NT; ++nf) acc[mt][nf] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
        for (int kg = 0; kg < C::KGS; ++kg) {
            const i32x4 tap = *(const i32x4 *)&taptab[kg * 16 + 4 * (lane >> 4)];
            f32x4 fa[MT], fb[NT];
            const float *ab = &As[0][0] + (kg >> 2) * (C::COUT * C::LDA) + (kg & 3) * 16;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                fa[mt] = *(const f32x4 *)&ab[(16 * mt + (lane & 15)) * C::LDA + 4 * (lane >> 4)];
#pragma unroll
            for (int nf = 0; nf < NT; ++nf)
#pragma unroll
                for (int j = 0; j < 4; ++j) fb[nf][j] = img[pixoff[nf] + tap[j]];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nf = 0; nf < NT; ++nf)
                        acc[mt][nf] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[mt][j], fb[nf][j], acc[mt][nf], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);         // keeps the LDS reads of later groups from piling up in registers
        }
        relu_pool_store<MT, NT, H, W>(acc, bv, out + w * out_stride + (int64_t)b * C::COUT * PP,
                                      code + w * code_stride + (int64_t)b * C::COUT * PP, wave, lane);
        if (!more) break;
        __syncthreads();                               // every wave has read this sample's image
        put_image();
        __syncthreads();
    }
}

// dst[ci][(co, kh, kw)] = src[co][ci][KS - 1 - kh][KS - 1 - kw] per worker: the filters of the
// data-gradient convolution.  grid = (ceil(Cin * Cout * KK / 256), workers).
__global__ __launch_bounds__(256) void flip_filters_kernel(const float *__restrict__ src, int64_t src_stride,
                                                           float *__restrict__ dst, int64_t dst_stride, int Cin,
                                                           int Cout, int KK)
{
    const int w = blockIdx.y, idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= Cin * Cout * KK) return;
    const int ci = idx / (Cout * KK), rem = idx - ci * Cout * KK, co = rem / KK, rr = rem - co * KK;
    dst[w * dst_stride + idx] = src[w * src_stride + (co * Cin + ci) * KK + (KK - 1 - rr)];
}

// Weight gradient of the same convolution: dW[co][t] = sum over samples b and pixels p of
// dz[b][co][p] * in[b][tap t shifted by p], as the GEMM with M = output channels, N = filter
// taps t = (c, kh, kw), K = pixels.  The sample's input (all CIN channels, zero halo) and a
// chunk of PC pixels of its deltas sit in LDS.  The A fragment (deltas, k = pixel) is a
// 128-bit LDS read; the B fragment is img[tap_offset(lane's tap) + pixel_offset(k)], where
// the pixel offset of k = 16 kg + 4 slot + j is a per-lane constant plus a compile-time
// immediate, so the reads need no address arithmetic at all.
// Waves are arranged WM (channels) x WN (taps) x WK (pixels); every (workgroup, wk) pair
// writes its own partial result  part[worker][split = blockIdx.x * WK + wk][co][t], which a
// separate pass sums in split order (deterministic).  grid = (ceil(B / SB), workers).
template <int CIN, int MT, int NT, int WM, int WN, int WK, int H, int W, int KS, int PC>
struct WCfg {
    static constexpr int PAD = KS / 2, HP = H + 2 * PAD, WP = W + 2 * PAD;
    static constexpr int COUT = 16 * MT * WM, PIX = H * W, KK = KS * KS, TAPS = CIN * KK;
    static constexpr int WAVES = WM * WN * WK, THREADS = 64 * WAVES;
    static constexpr int IMG = CIN * HP * WP;
    static constexpr int LDD = PC + 4;                   // row stride of the delta tile [COUT][PC]
    static constexpr int KG_CHUNK = PC / 16, KG_WAVE = KG_CHUNK / WK;
    static_assert(16 * NT * WN >= TAPS, "tap fragments must cover all taps");
    static_assert(PIX % PC == 0 && KG_CHUNK % WK == 0 && W % 16 == 0, "shape not supported");
    static constexpr size_t lds_bytes = sizeof(float) * (IMG + COUT * LDD);
};

// EXPAND: dz is given as the pooled gradients [worker][B][COUT][H/2][W/2] with dz_code of the same shape
// and is expanded while the delta tile is copied into LDS (see expand_pooled).
template <int CIN, int MT, int NT, int WM, int WN, int WK, int H, int W, int KS, int PC, bool EXPAND = false>
__global__ __launch_bounds__(64 * WM * WN * WK) void conv_wgrad_kernel(
    const float *__restrict__ in, int64_t in_stride, const float *__restrict__ dz, int64_t dz_stride,
    float *__restrict__ part, int64_t part_stride, int B, int SB, const uint8_t *__restrict__ dz_code = nullptr,
    int64_t dz_code_stride = 0)
{
    using C = WCfg<CIN, MT, NT, WM, WN, WK, H, W, KS, PC>;
    __shared__ __attribute__((aligned(16))) float img[C::IMG];
    __shared__ __attribute__((aligned(16))) float dzs[C::COUT * C::LDD];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = (wave / WM) % WN, wk = wave / (WM * WN);
    const int w = blockIdx.y, b0 = blockIdx.x * SB, b1 = min(B, b0 + SB);

    for (int e = tid; e < C::IMG; e += C::THREADS) img[e] = 0.f;     // the halo stays zero

    // per-lane LDS element index of this lane's tap (plus its k-slot) for each tap fragment
    int bbase[NT];
#pragma unroll
    for (int nf = 0; nf < NT; ++nf) {
        const int t = 16 * (wn * NT + nf) + (lane & 15);
        const int c = t / C::KK, rr = t % C::KK, kh = rr / KS, kw = rr % KS;
        bbase[nf] = (t < C::TAPS ? c * C::HP * C::WP + kh * C::WP + kw : 0) + 4 * (lane >> 4);
    }
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nf = 0; nf < NT; ++nf) acc[mt][nf] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int b = b0; b < b1; ++b) {
        const float *inb = in + w * in_stride + (int64_t)b * CIN * C::PIX;
        const float *dzb = dz + w * dz_stride + (int64_t)b * C::COUT * (EXPAND ? C::PIX / 4 : C::PIX);
        const uint8_t *dcb = EXPAND ? dz_code + w * dz_code_stride + (int64_t)b * C::COUT * (C::PIX / 4) : nullptr;
        for (int chunk = 0; chunk < C::PIX / PC; ++chunk) {
            __syncthreads();                   // previous tile fully consumed
            if (chunk == 0) {
                for (int e = tid; e < CIN * H * (W / 4); e += C::THREADS) {
                    const int c = e / (H * (W / 4)), rem = e % (H * (W / 4)), y = rem / (W / 4), x4 = rem % (W / 4);
                    const float4 v = *(const float4 *)&inb[(c * H + y) * W + 4 * x4];
                    float *dst = &img[c * C::HP * C::WP + (y + C::PAD) * C::WP + C::PAD + 4 * x4];
                    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
                }
            }
            for (int e = tid; e < C::COUT * (PC / 4); e += C::THREADS) {
                const int co = e / (PC / 4), p4 = e % (PC / 4);
                float4 v;
                if (EXPAND) {
                    const int p = chunk * PC + 4 * p4;
                    v = expand_pooled(dzb + co * (C::PIX / 4), dcb + co * (C::PIX / 4), p / W, (p % W) / 4, W);
                } else {
                    v = *(const float4 *)&dzb[co * C::PIX + chunk * PC + 4 * p4];
                }
                *(float4 *)&dzs[co * C::LDD + 4 * p4] = v;
            }
            __syncthreads();
            const int chunk_row = chunk * (PC / W);                  // first image row of the chunk
            // k runs over the wave's pixel groups i (16 pixels each) and the four k-slots j of a
            // group; the B values of step (i, j) + 1 are requested before the multiplies of step
            // (i, j), and scheduling barriers keep the compiler from requesting more than that
            // ahead (hundreds of values otherwise, which spill)
            auto pixel_offset = [&](int i) {
                const int kgl = wk * C::KG_WAVE + i;                 // k group inside the chunk (wave-uniform)
                // W % 16 == 0 keeps a group inside one image row
                return (chunk_row + (16 * kgl) / W) * C::WP + (16 * kgl) % W;
            };
            float fb[2][NT];
            {
                const int poff = pixel_offset(0);
#pragma unroll
                for (int nf = 0; nf < NT; ++nf) fb[0][nf] = img[bbase[nf] + poff];
            }
#pragma unroll
            for (int i = 0; i < C::KG_WAVE; ++i) {
                const int kgl = wk * C::KG_WAVE + i;
                f32x4 fa[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    fa[mt] = *(const f32x4 *)&dzs[(16 * (wm * MT + mt) + (lane & 15)) * C::LDD + 16 * kgl + 4 * (lane >> 4)];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int step = 4 * i + j;
                    if (step + 1 < 4 * C::KG_WAVE) {
                        const int poff = pixel_offset((step + 1) / 4) + (step + 1) % 4;
#pragma unroll
                        for (int nf = 0; nf < NT; ++nf) fb[(step + 1) & 1][nf] = img[bbase[nf] + poff];
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int nf = 0; nf < NT; ++nf)
                            acc[mt][nf] =
                                __builtin_amdgcn_mfma_f32_16x16x4f32(fa[mt][j], fb[step & 1][nf], acc[mt][nf], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }

    float *pb = part + w * part_stride + (int64_t)(blockIdx.x * WK + wk) * C::COUT * C::TAPS;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nf = 0; nf < NT; ++nf) {
            const int t = 16 * (wn * NT + nf) + (lane & 15);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int co = 16 * (wm * MT + mt) + 4 * (lane >> 4) + v;
                if (t < C::TAPS) pb[co * C::TAPS + t] = acc[mt][nf][v];
            }
        }
}

}  // namespace convlds
