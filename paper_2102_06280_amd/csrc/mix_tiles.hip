// Masked consensus average + local SGD step on the tile-major layout (DBW_LAYOUT_TILES).
//
// In the tile-major layout the parameters of all N workers at columns [64 t, 64 t + 64) form
// one contiguous block of N x 256 bytes, so a workgroup that needs every worker's values of a
// column range (each of them is somebody's neighbour) reads and writes plain linear streams.
// With rows stored one after the other the same workgroup touches N pieces that lie a whole
// row apart, and the device's memory channels serve that pattern 15-20 % slower.
//
// One workgroup takes G consecutive layout tiles (G N <= 128 rows of 256 bytes, or one tile for
// 128 < N <= 256), stages them in LDS together with the selected-neighbour lists, and every
// thread then combines the float4 values it loaded with its neighbours' from LDS.  Several
// workgroups are resident per CU, so loads, combines and stores of different tiles overlap.
// Every parameter, gradient and result crosses HBM exactly once (non-temporal accesses).  The
// summation order is the one of the other mixing kernels: self, then the selected neighbours in
// ascending index.
#include <algorithm>

#include "dbw_internal.h"

namespace {

constexpr int TM_THREADS = 512;
constexpr int TM_W4 = DBW_TILE_COLUMNS / 4;            // float4 per worker and layout tile
constexpr int TM_MAX_EDGES = 2048;                     // neighbour list entries staged in LDS

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

// "Virtual row" vr of a workgroup = (layout tile vr / N of the group, worker vr % N); thread
// tid owns float4 column tid % 16 of the virtual rows tid / 16 + 32 u, u < PER.
template <int ORDER, bool HAS_G, int PER, bool LISTS_LDS, class LR>
__global__ __launch_bounds__(TM_THREADS) void mix_tile_major(
    int N, int nnz, int G, int64_t n_tiles, int64_t d, const int32_t *__restrict__ rowptr,
    const int32_t *__restrict__ p, const int32_t *__restrict__ sel_idx, const float *__restrict__ sel_w,
    const float *__restrict__ self_w, const float4 *__restrict__ x, const float4 *__restrict__ g,
    float4 *__restrict__ out, LR lr)
{
    extern __shared__ float4 sm[];
    float4 *tile = sm;                                             // G * N * 16
    int32_t *s_idx = (int32_t *)(sm + (size_t)G * N * TM_W4);      // nnz (LISTS_LDS)
    float *s_w = (float *)(s_idx + nnz);                           // nnz
    const int tid = threadIdx.x, c = tid & (TM_W4 - 1);
    const int64_t t0 = (int64_t)blockIdx.x * G;
    const int64_t base = t0 * N * TM_W4;
    const int vrows = (int)std::min<int64_t>(G, n_tiles - t0) * N;

    float4 gv[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int vr = (tid >> 4) + 32 * u;
        gv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (vr < vrows) {
            const int f = vr * TM_W4 + c;
            float4 v = load_stream(&x[base + f]);
            if (HAS_G) gv[u] = load_stream(&g[base + f]);
            if (ORDER == DBW_ORDER_ATC && HAS_G) v = fma4(-lr.at(vr % N), gv[u], v);
            tile[f] = v;
        }
    }
    if (LISTS_LDS)
        for (int e = tid; e < nnz; e += TM_THREADS) {
            s_idx[e] = sel_idx[e];
            s_w[e] = sel_w[e];
        }
    __syncthreads();

#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int vr = (tid >> 4) + 32 * u;
        if (vr < vrows) {
            const int tg = vr / N, r = vr - tg * N;
            const int f = vr * TM_W4 + c;
            const int beg = rowptr[r], cnt = p[r];
            const float ws = self_w[r];
            const float4 v = tile[f];
            float4 acc = make_float4(ws * v.x, ws * v.y, ws * v.z, ws * v.w);
            const float4 *tb = tile + tg * N * TM_W4 + c;
            if (LISTS_LDS) {
                for (int k = 0; k < cnt; ++k) acc = fma4(s_w[beg + k], tb[s_idx[beg + k] * TM_W4], acc);
            } else {
                for (int k = 0; k < cnt; ++k) acc = fma4(sel_w[beg + k], tb[sel_idx[beg + k] * TM_W4], acc);
            }
            if (ORDER == DBW_ORDER_CTA && HAS_G) acc = fma4(-lr.at(r), gv[u], acc);
            const int64_t col0 = (t0 + tg) * DBW_TILE_COLUMNS + 4 * c;
            if (col0 + 4 <= d) {
                store_stream(&out[base + f], acc);
            } else {                                   // the float4 that straddles column d
                float *o = (float *)&out[base + f];
                if (col0 < d) o[0] = acc.x;
                if (col0 + 1 < d) o[1] = acc.y;
                if (col0 + 2 < d) o[2] = acc.z;
            }
        }
    }
}

// Rows <-> tiles, all ld columns.  One thread per float4, indexed in tile-major order.
__global__ __launch_bounds__(256) void layout_convert_kernel(int N, int64_t ld4, int64_t total4, int to_tiles,
                                                             const float4 *__restrict__ src, float4 *__restrict__ dst)
{
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= total4) return;
    const int64_t per = (int64_t)N * TM_W4;
    const int64_t t = q / per;
    const int rem = (int)(q - t * per);
    const int r = rem / TM_W4, c = rem % TM_W4;
    const int64_t rowmajor = (int64_t)r * ld4 + t * TM_W4 + c;
    if (to_tiles)
        dst[q] = src[rowmajor];
    else
        dst[rowmajor] = src[q];
}

template <int ORDER, bool HAS_G, int PER, bool LISTS_LDS, class LR>
int launch_one(dbw_ctx *c, int G, const float *x, const float *g, float *out, LR lr, hipStream_t s)
{
    const int64_t n_tiles = (c->d + DBW_TILE_COLUMNS - 1) / DBW_TILE_COLUMNS;
    const int64_t blocks = (n_tiles + G - 1) / G;
    if (blocks > INT32_MAX) return DBW_ERR_UNSUPPORTED;
    const size_t lds = sizeof(float4) * (size_t)G * c->N * TM_W4 + (LISTS_LDS ? (size_t)c->nnz * 8 : 0);
    auto kern = mix_tile_major<ORDER, HAS_G, PER, LISTS_LDS, LR>;
    static bool attr_set = false;                      // per instantiation
    if (!attr_set) {
        DBW_HIP(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
        attr_set = true;
    }
    dbw_timer tm(c, "mix_tile_major", s);
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(TM_THREADS), lds, s, c->N, c->nnz, G, n_tiles, c->d, c->rowptr,
                       c->p, c->sel_idx, c->sel_w, c->self_w, (const float4 *)x, (const float4 *)g, (float4 *)out, lr);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

template <int ORDER, bool HAS_G, class LR>
int launch(dbw_ctx *c, const float *x, const float *g, float *out, LR lr, hipStream_t s)
{
    const bool lists_lds = c->nnz <= TM_MAX_EDGES;
    if (c->N <= 128) {
        const int G = 128 / c->N;
        return lists_lds ? launch_one<ORDER, HAS_G, 4, true, LR>(c, G, x, g, out, lr, s)
                         : launch_one<ORDER, HAS_G, 4, false, LR>(c, G, x, g, out, lr, s);
    }
    return lists_lds ? launch_one<ORDER, HAS_G, 8, true, LR>(c, 1, x, g, out, lr, s)
                     : launch_one<ORDER, HAS_G, 8, false, LR>(c, 1, x, g, out, lr, s);
}

}  // namespace

int dbw_launch_mix_tiles(dbw_ctx *c, const float *x, const float *g, float *out, float lr, const float *lr_vec,
                         hipStream_t s)
{
    if (c->N > DBW_TILES_MAX_N || c->ld % DBW_TILE_COLUMNS) return DBW_ERR_UNSUPPORTED;
    if ((uintptr_t)x % 16 || (uintptr_t)out % 16 || (g && (uintptr_t)g % 16)) return DBW_ERR_INVALID;
    if (g == nullptr) return launch<DBW_ORDER_CTA, false>(c, x, g, out, dbw_lr_scalar{0.f}, s);
    if (lr_vec) {
        if (c->order == DBW_ORDER_ATC) return launch<DBW_ORDER_ATC, true>(c, x, g, out, dbw_lr_vector{lr_vec}, s);
        return launch<DBW_ORDER_CTA, true>(c, x, g, out, dbw_lr_vector{lr_vec}, s);
    }
    if (c->order == DBW_ORDER_ATC) return launch<DBW_ORDER_ATC, true>(c, x, g, out, dbw_lr_scalar{lr}, s);
    return launch<DBW_ORDER_CTA, true>(c, x, g, out, dbw_lr_scalar{lr}, s);
}

int dbw_launch_layout_convert(dbw_ctx *c, const float *src, float *dst, int to_tiles, hipStream_t s)
{
    const int64_t total4 = (int64_t)c->N * c->ld / 4;
    const int64_t blocks = (total4 + 255) / 256;
    if (blocks > INT32_MAX) return DBW_ERR_UNSUPPORTED;
    dbw_timer tm(c, "layout_convert_kernel", s);
    hipLaunchKernelGGL(layout_convert_kernel, dim3((unsigned)blocks), dim3(256), 0, s, c->N, c->ld / 4, total4, to_tiles,
                       (const float4 *)src, (float4 *)dst);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}
