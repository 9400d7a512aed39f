// Masked consensus average over the selected neighbours, fused with the local SGD step
// (Section 2.1 full-participation update; Section 2.2 local update + partial consensus).
//
//   CTA: out_i = P_ii x_i + sum_{j in S_i} P_ij x_j - lr g_i
//   ATC: out_i = P_ii (x_i - lr g_i) + sum_{j in S_i} P_ij (x_j - lr g_j)
//
// The work is a pure HBM stream: every parameter and gradient has to come in once and
// every result go out once, while a neighbour's row is needed by several workers.  Two
// kernels keep the HBM traffic at that minimum:
//
//  mix_lds_tiles   (N <= 512 and short neighbour lists) one persistent workgroup per CU
//                  walks over column tiles.  A tile holds the same TC4 float4 columns of
//                  ALL N rows in LDS (64 KB), so every reuse of a neighbour's values is an
//                  LDS read; the selected-neighbour lists sit in LDS as well.  Tiles are
//                  double buffered: the global loads of the next tile are in flight while
//                  the current one is combined and stored.
//  mix_csr_vec4    (any N) one workgroup per (worker, column chunk); all workers of a
//                  chunk run next to each other on the same XCD so the chunk stays in that
//                  XCD's L2 while its readers run.  Workgroup ids are dealt round-robin to
//                  the 8 XCDs, hence the id -> (chunk, worker) map.
//
// Gradients and results are touched exactly once, so they use non-temporal accesses and
// do not push parameter rows out of the caches.  The summation order is fixed (self, then
// selected neighbours in ascending index): results are bit-reproducible and identical
// between the two kernels.
#include <algorithm>

#include "dbw_internal.h"

namespace {

constexpr int MIX_THREADS = 256;
constexpr int MIX_XCDS = 8;
constexpr int LDS_THREADS = 1024;
constexpr int LDS_PER = 4;                             // float4 per thread per tile
constexpr int LDS_TILE = LDS_THREADS * LDS_PER;        // 4096 float4 = 64 KB
constexpr int LDS_MAX_EDGES = 2048;                    // neighbour list entries staged in LDS

typedef float vf4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4 fma4(float w, float4 a, float4 acc)
{
    acc.x = fmaf(w, a.x, acc.x);
    acc.y = fmaf(w, a.y, acc.y);
    acc.z = fmaf(w, a.z, acc.z);
    acc.w = fmaf(w, a.w, acc.w);
    return acc;
}

__device__ __forceinline__ float4 load_stream(const float4 *p)
{
    const vf4 v = __builtin_nontemporal_load((const vf4 *)p);
    return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void store_stream(float4 *p, float4 v)
{
    vf4 t;
    t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_nontemporal_store(t, (vf4 *)p);
}

// Persistent workgroup, tiles of N rows x TC4 float4 columns (N * TC4 <= LDS_TILE).
// Element f of a tile is (row f / TC4, column f % TC4); thread `tid` owns elements
// tid + u * LDS_THREADS, the same (row, column offset) in every tile.
template <int ORDER, bool HAS_G, int TC4, class LR>
__global__ __launch_bounds__(LDS_THREADS) void mix_lds_tiles(
    int N, int nnz, int64_t n_vec, int64_t ld4, int64_t n_tiles, const int32_t *__restrict__ rowptr,
    const int32_t *__restrict__ p, const int32_t *__restrict__ sel_idx, const float *__restrict__ sel_w,
    const float *__restrict__ self_w, const float4 *__restrict__ x, const float4 *__restrict__ g,
    float4 *__restrict__ out, LR lr, int64_t d)
{
    extern __shared__ float4 sm[];
    float4 *tiles = sm;                                  // 2 * LDS_TILE
    int32_t *s_idx = (int32_t *)(sm + 2 * LDS_TILE);     // nnz
    float *s_w = (float *)(s_idx + nnz);                 // nnz
    const int tid = threadIdx.x;
    const int total = N * TC4;

    for (int e = tid; e < nnz; e += LDS_THREADS) {
        s_idx[e] = sel_idx[e];
        s_w[e] = sel_w[e];
    }
    int beg[LDS_PER], cnt[LDS_PER], col[LDS_PER];
    float ws[LDS_PER], eta[LDS_PER];
    int64_t rowoff[LDS_PER];
#pragma unroll
    for (int u = 0; u < LDS_PER; ++u) {
        const int f = tid + u * LDS_THREADS;
        const int r = f < total ? f / TC4 : 0;
        col[u] = f < total ? f % TC4 : TC4;              // TC4 marks an element outside the tile
        beg[u] = rowptr[r];
        cnt[u] = p[r];
        ws[u] = self_w[r];
        eta[u] = lr.at(r);
        rowoff[u] = (int64_t)r * ld4;
    }

    float4 xs[LDS_PER], gs[LDS_PER];
    auto fetch = [&](int64_t t) {
#pragma unroll
        for (int u = 0; u < LDS_PER; ++u) {
            const int64_t c = t * TC4 + col[u];
            xs[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            gs[u] = xs[u];
            if (col[u] < TC4 && c < n_vec) {
                xs[u] = load_stream(&x[rowoff[u] + c]);
                if (HAS_G) gs[u] = load_stream(&g[rowoff[u] + c]);
                if (ORDER == DBW_ORDER_ATC && HAS_G) xs[u] = fma4(-eta[u], gs[u], xs[u]);
            }
        }
    };

    int64_t t = blockIdx.x;
    if (t >= n_tiles) return;
    fetch(t);
#pragma unroll
    for (int u = 0; u < LDS_PER; ++u) tiles[tid + u * LDS_THREADS] = xs[u];
    __syncthreads();

    int buf = 0;
    for (; t < n_tiles; t += gridDim.x) {
        float4 gc[LDS_PER];
#pragma unroll
        for (int u = 0; u < LDS_PER; ++u) gc[u] = gs[u];
        const int64_t nx = t + gridDim.x;
        if (nx < n_tiles) fetch(nx);

        const float4 *tl = tiles + buf * LDS_TILE;
#pragma unroll
        for (int u = 0; u < LDS_PER; ++u) {
            const int64_t c = t * TC4 + col[u];
            if (col[u] < TC4 && c < n_vec) {
                const float4 v = tl[tid + u * LDS_THREADS];
                float4 acc = make_float4(ws[u] * v.x, ws[u] * v.y, ws[u] * v.z, ws[u] * v.w);
                for (int k = 0; k < cnt[u]; ++k)
                    acc = fma4(s_w[beg[u] + k], tl[s_idx[beg[u] + k] * TC4 + col[u]], acc);
                if (ORDER == DBW_ORDER_CTA && HAS_G) acc = fma4(-eta[u], gc[u], acc);
                if (4 * c + 4 <= d) {
                    store_stream(&out[rowoff[u] + c], acc);
                } else {                           // the float4 that straddles column d: padding stays untouched
                    float *o = (float *)&out[rowoff[u] + c];
                    o[0] = acc.x;
                    if (4 * c + 1 < d) o[1] = acc.y;
                    if (4 * c + 2 < d) o[2] = acc.z;
                }
            }
        }
        if (nx < n_tiles) {
#pragma unroll
            for (int u = 0; u < LDS_PER; ++u) tiles[(buf ^ 1) * LDS_TILE + tid + u * LDS_THREADS] = xs[u];
        }
        __syncthreads();
        buf ^= 1;
    }
}

// One workgroup = one worker x one chunk of MIX_THREADS*UNROLL float4 columns.
template <int ORDER, bool HAS_G, int UNROLL, class LR>
__global__ __launch_bounds__(MIX_THREADS) void mix_csr_vec4(
    int N, int64_t n_vec /* float4 columns per row */, int64_t ld4 /* row stride in float4 */,
    int n_chunks, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ p,
    const int32_t *__restrict__ sel_idx, const float *__restrict__ sel_w,
    const float *__restrict__ self_w, const float4 *__restrict__ x, const float4 *__restrict__ g,
    float4 *__restrict__ out, LR lr, int64_t d)
{
    const int64_t L = blockIdx.x;
    const int xcd = (int)(L % MIX_XCDS);
    const int64_t slot = L / MIX_XCDS;
    const int i = (int)(slot % N);
    const int64_t chunk = (slot / N) * MIX_XCDS + xcd;
    if (chunk >= n_chunks) return;

    const int beg = rowptr[i], cnt = p[i];
    const float ws = self_w[i], eta_i = lr.at(i);
    const int64_t c0 = chunk * (int64_t)(MIX_THREADS * UNROLL) + threadIdx.x;
    const float4 *xi = x + (int64_t)i * ld4;

    float4 acc[UNROLL], gv[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t c = c0 + (int64_t)u * MIX_THREADS;
        acc[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        gv[u] = acc[u];
        if (c < n_vec) {
            float4 v = xi[c];
            if (HAS_G) gv[u] = load_stream(&g[(int64_t)i * ld4 + c]);
            if (ORDER == DBW_ORDER_ATC && HAS_G) v = fma4(-eta_i, gv[u], v);
            acc[u] = make_float4(ws * v.x, ws * v.y, ws * v.z, ws * v.w);
        }
    }
    for (int k = 0; k < cnt; ++k) {
        const int j = sel_idx[beg + k];
        const float w = sel_w[beg + k], eta_j = lr.at(j);
        const float4 *xj = x + (int64_t)j * ld4;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t c = c0 + (int64_t)u * MIX_THREADS;
            if (c < n_vec) {
                float4 v = xj[c];
                if (ORDER == DBW_ORDER_ATC && HAS_G) v = fma4(-eta_j, g[(int64_t)j * ld4 + c], v);
                acc[u] = fma4(w, v, acc[u]);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t c = c0 + (int64_t)u * MIX_THREADS;
        if (c < n_vec) {
            float4 r = acc[u];
            if (ORDER == DBW_ORDER_CTA && HAS_G) r = fma4(-eta_i, gv[u], r);
            if (4 * c + 4 <= d) {
                store_stream(&out[(int64_t)i * ld4 + c], r);
            } else {                               // the float4 that straddles column d: padding stays untouched
                float *o = (float *)&out[(int64_t)i * ld4 + c];
                o[0] = r.x;
                if (4 * c + 1 < d) o[1] = r.y;
                if (4 * c + 2 < d) o[2] = r.z;
            }
        }
    }
}

// Scalar columns [c_begin, d): the ragged tail of a row, or everything when rows are
// not 16-byte aligned.  grid = (ceil(cols / 256), N).
template <int ORDER, bool HAS_G, class LR>
__global__ __launch_bounds__(256) void mix_csr_scalar(
    int N, int64_t c_begin, int64_t d, int64_t ld, const int32_t *__restrict__ rowptr,
    const int32_t *__restrict__ p, const int32_t *__restrict__ sel_idx,
    const float *__restrict__ sel_w, const float *__restrict__ self_w, const float *__restrict__ x,
    const float *__restrict__ g, float *__restrict__ out, LR lr)
{
    const int i = blockIdx.y;
    const int64_t c = c_begin + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= d) return;
    const int beg = rowptr[i], cnt = p[i];
    float v = x[(int64_t)i * ld + c];
    if (ORDER == DBW_ORDER_ATC && HAS_G) v = fmaf(-lr.at(i), g[(int64_t)i * ld + c], v);
    float acc = self_w[i] * v;
    for (int k = 0; k < cnt; ++k) {
        const int j = sel_idx[beg + k];
        float vj = x[(int64_t)j * ld + c];
        if (ORDER == DBW_ORDER_ATC && HAS_G) vj = fmaf(-lr.at(j), g[(int64_t)j * ld + c], vj);
        acc = fmaf(sel_w[beg + k], vj, acc);
    }
    if (ORDER == DBW_ORDER_CTA && HAS_G) acc = fmaf(-lr.at(i), g[(int64_t)i * ld + c], acc);
    out[(int64_t)i * ld + c] = acc;
}

int device_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        cus = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
                  ? prop.multiProcessorCount : 256;
    }
    return cus;
}

template <int ORDER, bool HAS_G, class LR>
int launch_scalar(dbw_ctx *c, const float *x, const float *g, float *out, LR lr, int64_t c_begin, hipStream_t s)
{
    const int64_t cols = c->d - c_begin;
    dbw_timer tm(c, "mix_csr_scalar", s);
    hipLaunchKernelGGL((mix_csr_scalar<ORDER, HAS_G, LR>), dim3((unsigned)((cols + 255) / 256), c->N), dim3(256), 0, s,
                       c->N, c_begin, c->d, c->ld, c->rowptr, c->p, c->sel_idx, c->sel_w, c->self_w, x, g, out, lr);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

template <int ORDER, bool HAS_G, int TC4, class LR>
int launch_lds(dbw_ctx *c, const float *x, const float *g, float *out, LR lr, int64_t n_vec, hipStream_t s)
{
    const int64_t n_tiles = (n_vec + TC4 - 1) / TC4;
    const size_t lds = sizeof(float4) * 2 * LDS_TILE + (size_t)c->nnz * 8;
    auto kern = mix_lds_tiles<ORDER, HAS_G, TC4, LR>;
    static bool attr_set = false;                      // per instantiation
    if (!attr_set) {
        DBW_HIP(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set = true;
    }
    const int64_t grid = std::min<int64_t>(n_tiles, device_cus());
    dbw_timer tm(c, "mix_lds_tiles", s);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(LDS_THREADS), lds, s, c->N, c->nnz, n_vec, c->ld / 4, n_tiles,
                       c->rowptr, c->p, c->sel_idx, c->sel_w, c->self_w, (const float4 *)x, (const float4 *)g,
                       (float4 *)out, lr, c->d);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

template <int ORDER, bool HAS_G, class LR>
int launch(dbw_ctx *c, const float *x, const float *g, float *out, LR lr, hipStream_t s)
{
    constexpr int UNROLL = 2;
    const bool aligned = (c->ld % 4 == 0) && ((uintptr_t)x % 16 == 0) && ((uintptr_t)out % 16 == 0) &&
                         (!HAS_G || (uintptr_t)g % 16 == 0);
    int64_t n_vec = aligned ? c->d / 4 : 0;
    if (n_vec > 0) {
        // Tile width: a power of two of float4 columns, 8..256, that holds all N rows in 64 KB.  The widest one
        // moves the longest pieces of a row (2 KB pieces run at about 70 % of the HBM peak, 1 KB 68 %, 512 B 62 %,
        // 256 B 54 %), but a short parameter vector then gives the CUs unequal numbers of tiles (d = 159 010 on 32
        // workers: 311 tiles of 128 columns on 256 CUs, two rounds for 55 of them), so the width that minimises
        // rounds x width / efficiency is taken.
        const int64_t vec_cols = (c->d + 3) / 4;
        int tc4 = 0;
        double best = 0.0;
        for (int cand = 256; cand >= 8; cand /= 2) {
            if ((int64_t)c->N * cand > LDS_TILE) continue;
            const int64_t tiles = (vec_cols + cand - 1) / cand, rounds = (tiles + device_cus() - 1) / device_cus();
            const double eff = cand >= 128 ? 0.70 : (cand == 64 ? 0.68 : (cand == 32 ? 0.62 : (cand == 16 ? 0.54 : 0.40)));
            const double cost = (double)rounds * cand / eff;
            if (tc4 == 0 || cost < best) {
                best = cost;
                tc4 = cand;
            }
        }
        const bool use_lds = tc4 >= 8 && c->nnz <= LDS_MAX_EDGES && (vec_cols + tc4 - 1) / tc4 >= device_cus() / 2;
        int rc = DBW_OK;
        if (use_lds) {
            // the LDS kernel also takes the float4 that straddles column d (rows are aligned and
            // ld is a multiple of 4, so that float4 lies inside the row): no separate tail launch
            n_vec = (c->d + 3) / 4;
            switch (tc4) {
            case 256: rc = launch_lds<ORDER, HAS_G, 256, LR>(c, x, g, out, lr, n_vec, s); break;
            case 128: rc = launch_lds<ORDER, HAS_G, 128, LR>(c, x, g, out, lr, n_vec, s); break;
            case 64: rc = launch_lds<ORDER, HAS_G, 64, LR>(c, x, g, out, lr, n_vec, s); break;
            case 32: rc = launch_lds<ORDER, HAS_G, 32, LR>(c, x, g, out, lr, n_vec, s); break;
            case 16: rc = launch_lds<ORDER, HAS_G, 16, LR>(c, x, g, out, lr, n_vec, s); break;
            default: rc = launch_lds<ORDER, HAS_G, 8, LR>(c, x, g, out, lr, n_vec, s); break;
            }
            if (rc != DBW_OK) return rc;
        } else {
            n_vec = (c->d + 3) / 4;                 // as above: the straddling float4 lies inside the aligned row
            const int64_t per = (int64_t)MIX_THREADS * UNROLL;
            const int64_t n_chunks = (n_vec + per - 1) / per;
            const int64_t per_xcd = (n_chunks + MIX_XCDS - 1) / MIX_XCDS;
            const int64_t blocks = per_xcd * MIX_XCDS * c->N;
            if (n_chunks > INT32_MAX || blocks > INT32_MAX) return DBW_ERR_UNSUPPORTED;
            dbw_timer tm(c, "mix_csr_vec4", s);
            hipLaunchKernelGGL((mix_csr_vec4<ORDER, HAS_G, UNROLL, LR>), dim3((unsigned)blocks), dim3(MIX_THREADS), 0, s,
                               c->N, n_vec, c->ld / 4, (int)n_chunks, c->rowptr, c->p, c->sel_idx, c->sel_w,
                               c->self_w, (const float4 *)x, (const float4 *)g, (float4 *)out, lr, c->d);
            DBW_HIP(hipGetLastError());
        }
    }
    if (n_vec * 4 < c->d) return launch_scalar<ORDER, HAS_G, LR>(c, x, g, out, lr, n_vec * 4, s);
    return DBW_OK;
}

}  // namespace

int dbw_launch_mix_csr(dbw_ctx *c, const float *x, const float *g, float *out, float lr, const float *lr_vec,
                       hipStream_t s)
{
    if (g == nullptr) return launch<DBW_ORDER_CTA, false>(c, x, g, out, dbw_lr_scalar{0.f}, s);
    if (lr_vec) {
        if (c->order == DBW_ORDER_ATC) return launch<DBW_ORDER_ATC, true>(c, x, g, out, dbw_lr_vector{lr_vec}, s);
        return launch<DBW_ORDER_CTA, true>(c, x, g, out, dbw_lr_vector{lr_vec}, s);
    }
    if (c->order == DBW_ORDER_ATC) return launch<DBW_ORDER_ATC, true>(c, x, g, out, dbw_lr_scalar{lr}, s);
    return launch<DBW_ORDER_CTA, true>(c, x, g, out, dbw_lr_scalar{lr}, s);
}

// Scalar evaluation of columns [c_begin, d) only (the ragged tail left by a vector path).
int dbw_launch_mix_csr_range(dbw_ctx *c, const float *x, const float *g, float *out, float lr, const float *lr_vec,
                             int64_t c_begin, hipStream_t s)
{
    if (g == nullptr) return launch_scalar<DBW_ORDER_CTA, false>(c, x, g, out, dbw_lr_scalar{0.f}, c_begin, s);
    if (lr_vec) {
        if (c->order == DBW_ORDER_ATC)
            return launch_scalar<DBW_ORDER_ATC, true>(c, x, g, out, dbw_lr_vector{lr_vec}, c_begin, s);
        return launch_scalar<DBW_ORDER_CTA, true>(c, x, g, out, dbw_lr_vector{lr_vec}, c_begin, s);
    }
    if (c->order == DBW_ORDER_ATC) return launch_scalar<DBW_ORDER_ATC, true>(c, x, g, out, dbw_lr_scalar{lr}, c_begin, s);
    return launch_scalar<DBW_ORDER_CTA, true>(c, x, g, out, dbw_lr_scalar{lr}, c_begin, s);
}
