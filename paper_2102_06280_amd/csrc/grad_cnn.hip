// Mini-batch gradients of the convolutional model for all workers at once (Section 2.1,
// stochastic gradient of the local loss).  Network per worker, input [B][C0][H][W]:
//   conv KxK (C0->C1, same padding) -> ReLU -> maxpool 2x2 -> conv KxK (C1->C2, same) ->
//   ReLU -> maxpool 2x2 -> flatten [C2][H/4][W/4] -> FC F -> ReLU -> FC classes -> softmax
//   cross-entropy, mean over the batch.
// Parameter row layout: conv1 W [C1][C0][K][K], b [C1]; conv2 W [C2][C1][K][K], b [C2];
// fc1 W [F][flat], b [F]; fc2 W [classes][F], b [classes].
//
// Convolutions are implicit GEMMs on the batched fp32 MFMA kernel: the patch matrix is
// never materialised, the operand loaders compute the input address of each element.
//   forward   z[co][pix]      = sum_k  W[co][k] * patch[k][pix]        k = (ci, kh, kw)
//   wgrad     dW[co][k]       = sum_pix dz[co][pix] * patch[k][pix]
//   dgrad     din[ci][pix_in] = sum_k' W[co][ci][kh][kw] * dz[co][pix_in shifted]   k' = (co, kh, kw)
// Output channels are the GEMM's M and pixels its N, so stores run along consecutive pixels.
// Max pooling keeps no index: the backward pass re-derives the first maximum of each
// window from the stored pre-activations (first in window order (0,0),(0,1),(1,0),(1,1)).
#include <algorithm>

#include "bgemm.h"
#include "conv_lds.h"
#include "dbw_internal.h"

namespace {

using bgemm::Dense;

struct ConvShape {
    int Cin, Cout, H, W, KS, pad;   // stride-1 'same' convolution
};

// Filter size as a compile-time constant where it is a common one (KS_ = 0: run time), so
// that splitting k into (channel, tap) needs no division.
template <int KS_>
__device__ __forceinline__ int filter_size(const ConvShape &s) { return KS_ > 0 ? KS_ : s.KS; }

// Contexts shared by the convolution loaders.  A pixel context addresses tensor element
// (b, channel 0, y, x) of a [B][C][H][W] tensor; a tap context adds the channel plane and
// the (dy, dx) shift of one filter tap.  Element = base + off, valid iff the shifted
// position is inside the image.
struct PixelCtx { int base, y, x; bool ok; };
struct TapCtx { int off, dy, dx; bool ok; };

__device__ __forceinline__ PixelCtx pixel_ctx(const ConvShape &s, int C, int pix, bool ok)
{
    const int HW = s.H * s.W;
    const int b = pix / HW, hw = pix - b * HW, y = hw / s.W, x = hw - y * s.W;
    return {b * C * HW + hw, y, x, ok};
}

// k = (channel, kh, kw); sign = +1 reads the input of a forward tap (y + kh - pad),
// sign = -1 the output position that used this input with that tap (y - kh + pad).
template <int KS_>
__device__ __forceinline__ TapCtx tap_ctx(const ConvShape &s, int k, int sign, bool ok)
{
    const int KS = filter_size<KS_>(s), KK = KS * KS;
    const int ch = k / KK, rr = k - ch * KK, kh = rr / KS, kw = rr - kh * KS;
    const int dy = sign * (kh - s.pad), dx = sign * (kw - s.pad);
    return {ch * s.H * s.W + dy * s.W + dx, dy, dx, ok};
}

__device__ __forceinline__ float conv_load(const float *t, const ConvShape &s, const PixelCtx &p, const TapCtx &k)
{
    const bool ok = p.ok && k.ok && (unsigned)(p.y + k.dy) < (unsigned)s.H && (unsigned)(p.x + k.dx) < (unsigned)s.W;
    const float v = t[ok ? p.base + k.off : 0];
    return ok ? v : 0.f;
}

// B operand of the forward GEMM: (k = tap, row = output pixel), contiguous along pixels.
template <int KS_>
struct PatchRC {
    static constexpr bool KC = false;
    const float *in;
    int64_t stride;
    ConvShape s;
    typedef PixelCtx RowCtx;
    typedef TapCtx KCtx;
    __device__ __forceinline__ RowCtx row_ctx(int pix, bool ok) const { return pixel_ctx(s, s.Cin, pix, ok); }
    __device__ __forceinline__ KCtx k_ctx(int k, bool ok) const { return tap_ctx<KS_>(s, k, 1, ok); }
    __device__ __forceinline__ float load(int w, const RowCtx &r, const KCtx &k) const
    {
        return conv_load(in + w * stride, s, r, k);
    }
};

// B operand of the weight-gradient GEMM: row = filter tap, reduction index = output pixel.
template <int KS_>
struct PatchKC {
    static constexpr bool KC = true;
    const float *in;
    int64_t stride;
    ConvShape s;
    typedef TapCtx RowCtx;
    typedef PixelCtx KCtx;
    __device__ __forceinline__ RowCtx row_ctx(int kf, bool ok) const { return tap_ctx<KS_>(s, kf, 1, ok); }
    __device__ __forceinline__ KCtx k_ctx(int pix, bool ok) const { return pixel_ctx(s, s.Cin, pix, ok); }
    __device__ __forceinline__ float load(int w, const RowCtx &r, const KCtx &k) const
    {
        return conv_load(in + w * stride, s, k, r);
    }
};

// A operand of the weight-gradient GEMM: dz[co][pix] stored as [B][Cout][H][W].
struct DeltaKC {
    static constexpr bool KC = true;
    const float *dz;
    int64_t stride;
    int Cout, HW;
    struct RowCtx { int off; bool ok; };
    struct KCtx { int base; bool ok; };
    __device__ __forceinline__ RowCtx row_ctx(int co, bool ok) const { return {co * HW, ok}; }
    __device__ __forceinline__ KCtx k_ctx(int pix, bool ok) const
    {
        const int b = pix / HW, hw = pix - b * HW;
        return {b * Cout * HW + hw, ok};
    }
    __device__ __forceinline__ float load(int w, const RowCtx &r, const KCtx &k) const
    {
        const bool ok = r.ok && k.ok;
        const float v = (dz + w * stride)[ok ? r.off + k.base : 0];
        return ok ? v : 0.f;
    }
};

// A operand of the data-gradient GEMM: (row = ci, k' = (co, kh, kw)) -> W[co][ci][kh][kw].
template <int KS_>
struct FilterT {
    static constexpr bool KC = true;
    const float *wgt;
    int64_t stride;
    int Cin, KKrt;
    struct RowCtx { int off; bool ok; };
    struct KCtx { int base; bool ok; };
    __device__ __forceinline__ RowCtx row_ctx(int ci, bool ok) const { return {ci * (KS_ > 0 ? KS_ * KS_ : KKrt), ok}; }
    __device__ __forceinline__ KCtx k_ctx(int k, bool ok) const
    {
        const int KK = KS_ > 0 ? KS_ * KS_ : KKrt;
        const int co = k / KK, rr = k - co * KK;
        return {co * Cin * KK + rr, ok};
    }
    __device__ __forceinline__ float load(int w, const RowCtx &r, const KCtx &k) const
    {
        const bool ok = r.ok && k.ok;
        const float v = (wgt + w * stride)[ok ? r.off + k.base : 0];
        return ok ? v : 0.f;
    }
};

// B operand of the data-gradient GEMM: (k' = (co, kh, kw), row = input pixel) -> dz at the
// output position that used this input pixel with that filter tap; zero outside.
template <int KS_>
struct DeltaShiftRC {
    static constexpr bool KC = false;
    const float *dz;
    int64_t stride;
    ConvShape s;
    typedef PixelCtx RowCtx;
    typedef TapCtx KCtx;
    __device__ __forceinline__ RowCtx row_ctx(int pix, bool ok) const { return pixel_ctx(s, s.Cout, pix, ok); }
    __device__ __forceinline__ KCtx k_ctx(int k, bool ok) const { return tap_ctx<KS_>(s, k, -1, ok); }
    __device__ __forceinline__ float load(int w, const RowCtx &r, const KCtx &k) const
    {
        return conv_load(dz + w * stride, s, r, k);
    }
};

// Store C[m = channel][n = pixel] into a [B][C][H][W] tensor, adding a per-channel bias.
struct ChannelPixelOut {
    float *out;
    int64_t stride;
    int C, HW;
    const float *bias;     // per worker at bias[w * bias_stride + channel]; nullptr = none
    int64_t bias_stride;
    __device__ __forceinline__ void store(int w, int, int ch, int pix, float v) const
    {
        if (bias) v += bias[w * bias_stride + ch];
        const int b = pix / HW, hw = pix - b * HW;
        out[w * stride + (int64_t)(b * C + ch) * HW + hw] = v;
    }
};

// Partial sums of a split-k GEMM, inside each worker's scratch block: part[split][m][n].
struct PartialOut {
    float *part;
    int64_t stride;
    int M, N;
    __device__ __forceinline__ void store(int w, int split, int m, int n, float v) const
    {
        part[w * stride + ((int64_t)split * M + m) * N + n] = v;
    }
};

// dst[w * stride + i] = sum over splits of part[w][split][i], in split order.
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float *__restrict__ part, int64_t pstride,
                                                            int splits, int MN, float *__restrict__ dst,
                                                            int64_t stride)
{
    const int w = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    if (i >= MN) return;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp) s += part[w * pstride + (int64_t)sp * MN + i];
    dst[w * stride + i] = s;
}

// ReLU + 2x2 max pooling of z [B][C][H][W] -> p [B][C][H/2][W/2]; one thread per output.
__global__ __launch_bounds__(256) void relu_pool_fwd_kernel(const float *__restrict__ z, int64_t zstride,
                                                            float *__restrict__ p, int64_t pstride, int planes, int H, int W)
{
    const int w = blockIdx.y;
    const int Ho = H / 2, Wo = W / 2, total = planes * Ho * Wo;
    const int o = blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int pl = o / (Ho * Wo), rem = o - pl * Ho * Wo, oh = rem / Wo, ow = rem - oh * Wo;
    const float *src = z + w * zstride + ((int64_t)pl * H + 2 * oh) * W + 2 * ow;
    const float m = fmaxf(fmaxf(src[0], src[1]), fmaxf(src[W], src[W + 1]));
    p[w * pstride + o] = fmaxf(m, 0.f);
}

// Backward of ReLU + max pooling: the pooled gradient goes to the first element of the
// window that attains the (positive) maximum; everything else gets zero.
__global__ __launch_bounds__(256) void relu_pool_bwd_kernel(const float *__restrict__ z, int64_t zstride,
                                                            const float *__restrict__ dp, int64_t pstride,
                                                            float *__restrict__ dz, int planes, int H, int W)
{
    const int w = blockIdx.y;
    const int Ho = H / 2, Wo = W / 2, total = planes * Ho * Wo;
    const int o = blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int pl = o / (Ho * Wo), rem = o - pl * Ho * Wo, oh = rem / Wo, ow = rem - oh * Wo;
    const int64_t base = w * zstride + ((int64_t)pl * H + 2 * oh) * W + 2 * ow;
    const float v0 = z[base], v1 = z[base + 1], v2 = z[base + W], v3 = z[base + W + 1];
    const float m = fmaxf(fmaxf(v0, v1), fmaxf(v2, v3));
    const float gsrc = dp[w * pstride + o];
    int arg = -1;
    if (m > 0.f) arg = (v0 == m) ? 0 : (v1 == m) ? 1 : (v2 == m) ? 2 : 3;
    dz[base] = arg == 0 ? gsrc : 0.f;
    dz[base + 1] = arg == 1 ? gsrc : 0.f;
    dz[base + W] = arg == 2 ? gsrc : 0.f;
    dz[base + W + 1] = arg == 3 ? gsrc : 0.f;
}

// With the window codes of the fused convolution epilogue (0..3: position of the first maximum,
// 4: maximum not positive): db[ch] = sum of dz over batch and pixels = sum of the pooled gradients
// of the windows whose maximum was positive (each passes its gradient to exactly one pixel).
// One workgroup per (channel, worker); HWo % 4 == 0 and 16-byte aligned planes: a thread takes four
// windows at a time (one 128-bit load of gradients, one 32-bit load of codes).
__global__ __launch_bounds__(256) void channel_sum_code_kernel(const uint8_t *__restrict__ code, int64_t cstride,
                                                               const float *__restrict__ dp, int64_t pstride, int B,
                                                               int C, int HWo, float *__restrict__ db, int64_t dbstride)
{
    __shared__ float red[256];
    const int ch = blockIdx.x, w = blockIdx.y, tid = threadIdx.x;
    const int quads = HWo / 4;                       // per (sample, channel) plane
    const int q = tid % quads, b0 = tid / quads, bstep = 256 / quads > 0 ? 256 / quads : 1;
    float s = 0.f;
    if (b0 < bstep) {
#pragma unroll 4
        for (int b = b0; b < B; b += bstep) {
            for (int qq = q; qq < quads; qq += 256) {    // planes wider than 1024 windows
                const int64_t o = (int64_t)(b * C + ch) * HWo + 4 * qq;
                const float4 g = *(const float4 *)&dp[w * pstride + o];
                const uint32_t cd = *(const uint32_t *)&code[w * cstride + o];
                s += (cd & 0xffu) < 4u ? g.x : 0.f;
                s += ((cd >> 8) & 0xffu) < 4u ? g.y : 0.f;
                s += ((cd >> 16) & 0xffu) < 4u ? g.z : 0.f;
                s += (cd >> 24) < 4u ? g.w : 0.f;
            }
        }
    }
    red[tid] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (tid < o) red[tid] += red[tid + o];
        __syncthreads();
    }
    if (tid == 0) db[w * dbstride + ch] = red[0];
}

// db[ch] = sum over batch and pixels of dz[b][ch][hw]; one workgroup per (channel, worker).
__global__ __launch_bounds__(256) void channel_sum_kernel(const float *__restrict__ dz, int64_t stride, int B, int C,
                                                          int HW, float *__restrict__ db, int64_t dbstride)
{
    __shared__ float red[256];
    const int ch = blockIdx.x, w = blockIdx.y, tid = threadIdx.x;
    float s = 0.f;
    for (int i = tid; i < B * HW; i += 256) {
        const int b = i / HW, hw = i - b * HW;
        s += dz[w * stride + (int64_t)(b * C + ch) * HW + hw];
    }
    red[tid] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (tid < o) red[tid] += red[tid + o];
        __syncthreads();
    }
    if (tid == 0) db[w * dbstride + ch] = red[0];
}

constexpr int WGRAD_SB = 4;     // samples per workgroup in the LDS-resident weight-gradient kernels (scratch is sized for it)
constexpr int WGRAD_SB2 = 8;    // the same for conv2: 64 workers x 4 workgroups are one per compute unit

struct cnn_layout {
    int C0, H, W, C1, C2, KS, F, NC, B;
    int H2, W2, H4, W4, flat;
    int fc_dims[3];
    // parameter offsets inside a row
    int64_t w1, b1, w2, b2, fc;
    // scratch offsets inside a worker's block (floats)
    int64_t z1, p1, z2, p2, dp2, dz2, dp1, dz1, fc_act, part, wflip, code1, code2, total;
    int splits1, splits2;
};

cnn_layout make_layout(const dbw_model &m)
{
    cnn_layout L{};
    L.C0 = m.dims[0]; L.H = m.dims[1]; L.W = m.dims[2]; L.C1 = m.dims[3]; L.C2 = m.dims[4];
    L.KS = m.dims[5]; L.F = m.dims[6]; L.NC = m.dims[7]; L.B = m.batch;
    L.H2 = L.H / 2; L.W2 = L.W / 2; L.H4 = L.H / 4; L.W4 = L.W / 4;
    L.flat = L.C2 * L.H4 * L.W4;
    L.fc_dims[0] = L.flat; L.fc_dims[1] = L.F; L.fc_dims[2] = L.NC;
    const int64_t KK = (int64_t)L.KS * L.KS;
    L.w1 = 0;
    L.b1 = L.w1 + L.C1 * L.C0 * KK;
    L.w2 = L.b1 + L.C1;
    L.b2 = L.w2 + L.C2 * L.C1 * KK;
    L.fc = L.b2 + L.C2;
    const int64_t B = L.B;
    int64_t o = 0;
    auto take = [&](int64_t n) { const int64_t at = o; o += (n + 63) / 64 * 64; return at; };
    L.z1 = take(B * L.C1 * L.H * L.W);
    L.p1 = take(B * L.C1 * L.H2 * L.W2);
    L.z2 = take(B * L.C2 * L.H2 * L.W2);
    L.p2 = take(B * L.flat);
    L.dp2 = take(B * L.flat);
    L.dz2 = take(B * L.C2 * L.H2 * L.W2);
    L.dp1 = take(B * L.C1 * L.H2 * L.W2);
    L.dz1 = take(B * L.C1 * L.H * L.W);
    L.fc_act = take(dbw_fc_scratch_per_worker(2, L.fc_dims, L.B));
    // split the long pixel reductions of the weight gradients so that the grid fills the chip
    auto pick = [&](int64_t K) { int s = 1; while (s < 32 && K / (s * 2) >= 1024) s *= 2; return s; };
    L.splits1 = pick(B * L.H * L.W);
    L.splits2 = pick(B * L.H2 * L.W2);
    // the LDS-resident weight-gradient kernels write one partial per 4 samples (conv1: x 8 waves)
    const int64_t nb = (B + WGRAD_SB - 1) / WGRAD_SB;
    const int64_t s1 = std::max<int64_t>(L.splits1, nb * 8), s2 = std::max<int64_t>(L.splits2, nb);
    const int64_t p1n = s1 * L.C1 * L.C0 * KK, p2n = s2 * L.C2 * L.C1 * KK;
    L.part = take(p1n > p2n ? p1n : p2n);
    L.wflip = take((int64_t)L.C1 * L.C2 * KK);
    L.code1 = take((B * L.C1 * L.H2 * L.W2 + 3) / 4);     // one byte per pooled element
    L.code2 = take((B * L.flat + 3) / 4);
    L.total = o;
    return L;
}

// 32 x 128 tiles when the GEMM has at most 32 rows (output channels), else 64 x 64
template <class LA, class LB, class EP>
hipError_t conv_gemm(const LA &A, const LB &B, const EP &E, int M, int N, int K, int batch, hipStream_t s,
                     int splits = 1)
{
    if (M <= 32) return bgemm::launch<32>(A, B, E, M, N, K, batch, s, splits);
    return bgemm::launch<64>(A, B, E, M, N, K, batch, s, splits);
}

template <int KS_>
int launch_grad_cnn(dbw_ctx *c, const float *params, const float *bx, const int32_t *by, float *grads,
                    float *loss, hipStream_t s)
{
    const cnn_layout L = make_layout(c->model);
    const int N = c->N, B = L.B, KK = L.KS * L.KS;
    float *A = c->act;
    const int64_t ws = L.total, ld = c->ld;
    const int64_t xstride = (int64_t)B * L.C0 * L.H * L.W;
    const ConvShape s1{L.C0, L.C1, L.H, L.W, L.KS, L.KS / 2}, s2{L.C1, L.C2, L.H2, L.W2, L.KS, L.KS / 2};
    const int pix1 = B * L.H * L.W, pix2 = B * L.H2 * L.W2;
    auto blocks = [](int64_t n) { return (unsigned)((n + 255) / 256); };
    // The LDS-resident convolution kernels are instantiated for the 5x5 / 3-32-64 channel
    // network on 32 x 32 inputs; every other shape takes the implicit-GEMM path.
    const bool fast1 = KS_ == 5 && L.C0 == 3 && L.H == 32 && L.W == 32 && L.C1 == 32 && (uintptr_t)bx % 16 == 0;
    const bool fast2 = KS_ == 5 && L.C1 == 32 && L.H2 == 16 && L.W2 == 16 && L.C2 == 64;

    uint8_t *code1 = (uint8_t *)(A + L.code1), *code2 = (uint8_t *)(A + L.code2);
    const int64_t cs = ws * 4;                         // worker stride of the code maps in bytes
    if (fast1) {   // convolution + ReLU + pooling in one kernel
        dbw_timer tm(c, "conv1_forward", s);
        constexpr int SB1 = 4;                         // samples per workgroup
        hipLaunchKernelGGL((convlds::conv_forward_pool_multi_kernel<3, 2, 4, 32, 32, 5, 16, SB1>),
                           dim3((B + SB1 - 1) / SB1, N), dim3(1024), 0, s, bx, xstride, params + L.w1, ld, L.C0 * KK,
                           params + L.b1, ld, A + L.p1, ws, L.C0, B, code1, cs);
        DBW_HIP(hipGetLastError());
    } else {   // conv1 forward
        dbw_timer tm(c, "conv1_forward", s);
        DBW_HIP(conv_gemm(Dense<true>{params + L.w1, L.C0 * KK, ld}, PatchRC<KS_>{bx, xstride, s1},
                              ChannelPixelOut{A + L.z1, ws, L.C1, L.H * L.W, params + L.b1, ld}, L.C1, pix1,
                              L.C0 * KK, N, s));
    }
    if (!fast1) {
        dbw_timer tm(c, "relu_pool_fwd_kernel", s);
        hipLaunchKernelGGL(relu_pool_fwd_kernel, dim3(blocks((int64_t)B * L.C1 * L.H2 * L.W2), N), dim3(256), 0, s,
                           A + L.z1, ws, A + L.p1, ws, B * L.C1, L.H, L.W);
        DBW_HIP(hipGetLastError());
    }
    if (fast2) {
        dbw_timer tm(c, "conv2_forward", s);
        hipLaunchKernelGGL((convlds::conv_forward_kernel<16, 4, 2, 16, 16, 5, 8, true>), dim3(B, N), dim3(512), 0, s,
                           A + L.p1, ws, params + L.w2, ld, L.C1 * KK, params + L.b2, ld, A + L.p2, ws, L.C1, code2, cs);
        DBW_HIP(hipGetLastError());
    } else {   // conv2 forward
        dbw_timer tm(c, "conv2_forward", s);
        DBW_HIP(conv_gemm(Dense<true>{params + L.w2, L.C1 * KK, ld}, PatchRC<KS_>{A + L.p1, ws, s2},
                              ChannelPixelOut{A + L.z2, ws, L.C2, L.H2 * L.W2, params + L.b2, ld}, L.C2, pix2,
                              L.C1 * KK, N, s));
    }
    if (!fast2) {
        dbw_timer tm(c, "relu_pool_fwd_kernel", s);
        hipLaunchKernelGGL(relu_pool_fwd_kernel, dim3(blocks((int64_t)B * L.flat), N), dim3(256), 0, s, A + L.z2, ws,
                           A + L.p2, ws, B * L.C2, L.H2, L.W2);
        DBW_HIP(hipGetLastError());
    }
    {   // fully connected head, forward and backward, down to the gradient of the pooled features
        dbw_fc_args a{};
        a.L = 2;
        a.B = B;
        a.dims = L.fc_dims;
        a.params = params;
        a.grads = grads;
        a.param_off = L.fc;
        a.in = A + L.p2;
        a.in_ld = L.flat;
        a.in_stride = ws;
        a.act = A + L.fc_act;
        a.act_stride = ws;
        a.din = A + L.dp2;
        a.din_ld = L.flat;
        a.din_stride = ws;
        a.y = by;
        a.loss = loss;
        const int rc = dbw_fc_forward_backward(c, a, s);
        if (rc != DBW_OK) return rc;
    }
    // with the fused pooling the un-pooled delta maps are never materialised: their consumers
    // expand the pooled gradients and the window codes on the fly
    if (!fast2) {
        dbw_timer tm(c, "relu_pool_bwd_kernel", s);
        hipLaunchKernelGGL(relu_pool_bwd_kernel, dim3(blocks((int64_t)B * L.flat), N), dim3(256), 0, s, A + L.z2, ws,
                           A + L.dp2, ws, A + L.dz2, B * L.C2, L.H2, L.W2);
        DBW_HIP(hipGetLastError());
    }
    int splits2 = L.splits2, splits1 = L.splits1;
    if (fast2) {
        splits2 = (B + WGRAD_SB2 - 1) / WGRAD_SB2;
        dbw_timer tm(c, "conv2_wgrad", s);
        hipLaunchKernelGGL((convlds::conv_wgrad_kernel<32, 2, 13, 2, 4, 1, 16, 16, 5, 256, true>), dim3(splits2, N),
                           dim3(512), 0, s, A + L.p1, ws, A + L.dp2, ws, A + L.part, ws, B, WGRAD_SB2, code2, cs);
        DBW_HIP(hipGetLastError());
    } else {   // conv2 weight gradient (split over pixels, then summed in split order) and bias gradient
        dbw_timer tm(c, "conv2_wgrad", s);
        DBW_HIP(conv_gemm(DeltaKC{A + L.dz2, ws, L.C2, L.H2 * L.W2}, PatchKC<KS_>{A + L.p1, ws, s2},
                              PartialOut{A + L.part, ws, L.C2, L.C1 * KK}, L.C2, L.C1 * KK, pix2, N, s,
                              L.splits2));
    }
    {
        dbw_timer tm(c, "reduce_splits_kernel", s);
        hipLaunchKernelGGL(reduce_splits_kernel, dim3(blocks((int64_t)L.C2 * L.C1 * KK), N), dim3(256), 0, s,
                           A + L.part, ws, splits2, L.C2 * L.C1 * KK, grads + L.w2, ld);
        DBW_HIP(hipGetLastError());
    }
    if (fast2) {
        dbw_timer tm(c, "channel_sum_code_kernel", s);
        hipLaunchKernelGGL(channel_sum_code_kernel, dim3(L.C2, N), dim3(256), 0, s, code2, cs, A + L.dp2, ws, B, L.C2,
                           L.H4 * L.W4, grads + L.b2, ld);
        DBW_HIP(hipGetLastError());
    } else {
        dbw_timer tm(c, "channel_sum_kernel", s);
        hipLaunchKernelGGL(channel_sum_kernel, dim3(L.C2, N), dim3(256), 0, s, A + L.dz2, ws, B, L.C2, L.H2 * L.W2,
                           grads + L.b2, ld);
        DBW_HIP(hipGetLastError());
    }
    if (fast2) {   // conv2 data gradient = forward convolution of the deltas with flipped filters
        {
            dbw_timer tm(c, "flip_filters_kernel", s);
            hipLaunchKernelGGL(convlds::flip_filters_kernel, dim3(blocks((int64_t)L.C1 * L.C2 * KK), N), dim3(256), 0, s,
                               params + L.w2, ld, A + L.wflip, ws, L.C1, L.C2, KK);
            DBW_HIP(hipGetLastError());
        }
        dbw_timer tm(c, "conv2_dgrad", s);
        hipLaunchKernelGGL((convlds::conv_forward_kernel<16, 2, 2, 16, 16, 5, 8, false, true>), dim3(B, N), dim3(512), 0,
                           s, A + L.dp2, ws, A + L.wflip, ws, L.C2 * KK, (const float *)nullptr, (int64_t)0, A + L.dp1,
                           ws, L.C2, (uint8_t *)nullptr, (int64_t)0, code2, cs);
        DBW_HIP(hipGetLastError());
    } else {   // conv2 data gradient -> gradient of the first pooled map
        dbw_timer tm(c, "conv2_dgrad", s);
        DBW_HIP(conv_gemm(FilterT<KS_>{params + L.w2, ld, L.C1, KK}, DeltaShiftRC<KS_>{A + L.dz2, ws, s2},
                              ChannelPixelOut{A + L.dp1, ws, L.C1, L.H2 * L.W2, nullptr, 0}, L.C1, pix2, L.C2 * KK, N,
                              s));
    }
    if (!fast1) {
        dbw_timer tm(c, "relu_pool_bwd_kernel", s);
        hipLaunchKernelGGL(relu_pool_bwd_kernel, dim3(blocks((int64_t)B * L.C1 * L.H2 * L.W2), N), dim3(256), 0, s,
                           A + L.z1, ws, A + L.dp1, ws, A + L.dz1, B * L.C1, L.H, L.W);
        DBW_HIP(hipGetLastError());
    }
    if (fast1) {
        const int nb = (B + WGRAD_SB - 1) / WGRAD_SB;
        splits1 = nb * 8;
        dbw_timer tm(c, "conv1_wgrad", s);
        hipLaunchKernelGGL((convlds::conv_wgrad_kernel<3, 2, 5, 1, 1, 8, 32, 32, 5, 512, true>), dim3(nb, N), dim3(512), 0,
                           s, bx, xstride, A + L.dp1, ws, A + L.part, ws, B, WGRAD_SB, code1, cs);
        DBW_HIP(hipGetLastError());
    } else {   // conv1 weight and bias gradients
        dbw_timer tm(c, "conv1_wgrad", s);
        DBW_HIP(conv_gemm(DeltaKC{A + L.dz1, ws, L.C1, L.H * L.W}, PatchKC<KS_>{bx, xstride, s1},
                              PartialOut{A + L.part, ws, L.C1, L.C0 * KK}, L.C1, L.C0 * KK, pix1, N, s,
                              L.splits1));
    }
    {
        dbw_timer tm(c, "reduce_splits_kernel", s);
        hipLaunchKernelGGL(reduce_splits_kernel, dim3(blocks((int64_t)L.C1 * L.C0 * KK), N), dim3(256), 0, s,
                           A + L.part, ws, splits1, L.C1 * L.C0 * KK, grads + L.w1, ld);
        DBW_HIP(hipGetLastError());
    }
    if (fast1) {
        dbw_timer tm(c, "channel_sum_code_kernel", s);
        hipLaunchKernelGGL(channel_sum_code_kernel, dim3(L.C1, N), dim3(256), 0, s, code1, cs, A + L.dp1, ws, B, L.C1,
                           L.H2 * L.W2, grads + L.b1, ld);
        DBW_HIP(hipGetLastError());
    } else {
        dbw_timer tm(c, "channel_sum_kernel", s);
        hipLaunchKernelGGL(channel_sum_kernel, dim3(L.C1, N), dim3(256), 0, s, A + L.dz1, ws, B, L.C1, L.H * L.W,
                           grads + L.b1, ld);
        DBW_HIP(hipGetLastError());
    }
    return DBW_OK;
}

}  // namespace

size_t dbw_cnn_scratch_floats(const dbw_ctx *c) { return (size_t)make_layout(c->model).total * c->N; }

int dbw_launch_grad_cnn(dbw_ctx *c, const float *params, const float *bx, const int32_t *by, float *grads,
                        float *loss, hipStream_t s)
{
    switch (c->model.dims[5]) {
    case 3: return launch_grad_cnn<3>(c, params, bx, by, grads, loss, s);
    case 5: return launch_grad_cnn<5>(c, params, bx, by, grads, loss, s);
    default: return launch_grad_cnn<0>(c, params, bx, by, grads, loss, s);
    }
}
