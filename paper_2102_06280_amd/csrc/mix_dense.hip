// Dense form of the consensus update for near-complete graphs: X' = P(k) X on the matrix
// cores, fused with the local SGD step (Section 2.2, compact matrix form; rows are workers
// here, so the paper's W(k) P(k) reads P X).
//
//   CTA: out = P X - lr G            ATC: out = P (X - lr G)
//
// P (N x N, zero-padded to NPAD = 32 * MB) is tiny and lives in registers: each of the 8
// wavefronts of a workgroup keeps the A-operand fragments of one 32-row block of P for the
// whole kernel.  The workgroup walks over column tiles of X; a tile (NPAD rows x TC
// columns) is staged once through LDS, laid out so that the B-operand fragment of
// v_mfma_f32_32x32x2_f32 for k-step kk is one conflict-free 64-lane row.  The next tile is
// on its way while the current one is multiplied: when no element needs a guard (FULL
// tiles) it goes from global memory straight into LDS (global_load_lds, 16 bytes per lane),
// otherwise through registers.  With the local step first (ATC) the gradient values of the
// same elements travel in registers meanwhile, and x - lr g is formed in LDS once both have
// landed, after the multiplies: forming it in registers right behind the loads made every
// wave wait for them before it could start multiplying.  In the other order the gradient
// values of the epilogue are requested before the multiply loop so that they have arrived
// when it ends.  True fp32 MFMA: no reduced-precision input format anywhere.
//
// Fragment layout of v_mfma_f32_32x32x2_f32 (M = N = 32, K = 2), lane l in [0, 64):
//   A: a = A[m = l % 32][k = l / 32]        B: b = B[k = l / 32][n = l % 32]
//   D: 16 floats, d[v] = D[m = 8 * (v / 4) + 4 * (l / 32) + v % 4][n = l % 32]
#include <algorithm>

#include "dbw_internal.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(1))) const void *global_cptr;
typedef __attribute__((address_space(3))) void *lds_ptr;

constexpr int DENSE_THREADS = 512;

// A wave-uniform address, pinned to scalar registers.  Global loads and stores take a scalar
// base plus a 32-bit lane offset; without the pin the compiler folds the lane offset into one
// loop-invariant 64-bit vector address per row, and those dozens of register pairs push the
// P block out to scratch memory.
__device__ __forceinline__ const char *uniform_base(const void *p)
{
    const uint64_t a = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    uint64_t v = ((uint64_t)hi << 32) | lo;
    asm volatile("" : "+s"(v));
    return (const char *)v;
}

template <int MB>
struct dense_cfg {
    static constexpr int NPAD = 32 * MB;              // padded number of workers
    static constexpr int KB = NPAD / 2;               // k-steps of the 32x32x2 instruction
    static constexpr int CG = 8 / MB;                 // column groups among the 8 waves
    static constexpr int NSUB = CG > 2 ? CG : 2;      // 32-column sub-tiles per tile
    static constexpr int SPW = NSUB / CG;             // sub-tiles per wave
    static constexpr int TC = 32 * NSUB;              // tile columns
    static constexpr int TILE = NPAD * TC;            // floats per LDS buffer
    static constexpr int PASSES = TILE / 4 / DENSE_THREADS;
    static constexpr int DMA_PER_WAVE = TILE / 256 / 8;   // 1 KB blocks per wave and tile
};

// FULL: N == NPAD and every tile has all TC columns, so no access needs a guard.
template <int MB, int ORDER, bool HAS_G, bool FULL, class LR>
__global__ __launch_bounds__(DENSE_THREADS) void mix_dense_kernel(
    int N, int64_t n_vec /* float4 columns covered, the last may straddle column d */, int64_t dcols /* = d */,
    int64_t ld4, const float *__restrict__ Wsw, const float4 *__restrict__ x, const float4 *__restrict__ g,
    float *__restrict__ out, const float *__restrict__ gs, LR lr, int n_tiles)
{
    using C = dense_cfg<MB>;
    constexpr bool DMA = FULL;                                     // tiles go straight into LDS
    constexpr bool PRO = FULL && ORDER == DBW_ORDER_ATC && HAS_G;  // ... and x - lr g is formed there
    __shared__ __attribute__((aligned(16))) float lds[2 * C::TILE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave index, kept scalar
    const int rb = w % MB, cg = w / MB;
    const int64_t ld = ld4 * 4;

    float wreg[C::KB];
#pragma unroll
    for (int kk = 0; kk < C::KB; ++kk) wreg[kk] = Wsw[((size_t)(rb * C::KB + kk)) * 64 + lane];

    // ---- next-tile staging through registers (guards / ATC prologue)
    float4 stage[DMA ? 1 : C::PASSES];
    // lane offsets are kept in bytes: uniform 64-bit base + 32-bit lane offset is an addressing mode of
    // the global memory instructions, so no 64-bit address has to live in vector registers
    const uint32_t fetch_lane_off = 16u * (uint32_t)((tid / (C::TC / 4)) * ld4 + tid % (C::TC / 4));
    auto fetch = [&](int64_t tile) {
#pragma unroll
        for (int ps = 0; ps < (DMA ? 0 : C::PASSES); ++ps) {
            const int k0 = ps * (DENSE_THREADS / (C::TC / 4));                   // uniform first row of the pass
            const int k = k0 + tid / (C::TC / 4);
            const int64_t col4 = tile * (C::TC / 4) + tid % (C::TC / 4);
            const float4 *xb = x + (int64_t)k0 * ld4 + tile * (C::TC / 4);        // uniform base
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (FULL || (k < N && col4 < n_vec)) {
                v = *(const float4 *)(uniform_base(xb) + fetch_lane_off);
                if (ORDER == DBW_ORDER_ATC && HAS_G) {
                    const float4 gv =
                        *(const float4 *)(uniform_base(g + (int64_t)k0 * ld4 + tile * (C::TC / 4)) + fetch_lane_off);
                    const float eta = lr.at(k);
                    v.x = fmaf(-eta, gv.x, v.x);
                    v.y = fmaf(-eta, gv.y, v.y);
                    v.z = fmaf(-eta, gv.z, v.z);
                    v.w = fmaf(-eta, gv.w, v.w);
                }
            }
            stage[ps] = v;
        }
    };
    // registers -> LDS buffer `buf`, in B-fragment order: [sub-tile][k-step][lane]
    auto commit = [&](int buf) {
#pragma unroll
        for (int ps = 0; ps < (DMA ? 0 : C::PASSES); ++ps) {
            const int f = ps * DENSE_THREADS + tid;
            const int k = f / (C::TC / 4), c4 = f % (C::TC / 4);
            const int s = c4 / 8, l = (k & 1) * 32 + (c4 & 7) * 4;
            *(float4 *)&lds[buf * C::TILE + ((s * C::KB + (k >> 1)) * 64 + l)] = stage[ps];
        }
    };
    // ---- next-tile staging straight into LDS.  One instruction fills 1 KB = the 64-lane
    // rows of four consecutive k-steps of one sub-tile; lane -> (row, 4 columns) follows.
    const uint32_t dma_lane_off = 16u * (uint32_t)((2 * (lane >> 4) + ((lane >> 3) & 1)) * ld4 + (lane & 7));
    auto dma = [&](int64_t tile, int buf) {
#pragma unroll
        for (int i = 0; i < (DMA ? C::DMA_PER_WAVE : 0); ++i) {
            const int q = w + 8 * i;                                             // uniform block id
            const int s = q / (C::KB / 4), kq = q % (C::KB / 4);
            const float4 *src = x + (int64_t)(8 * kq) * ld4 + tile * (C::TC / 4) + s * 8;   // uniform base
            __builtin_amdgcn_global_load_lds((global_cptr)(uniform_base(src) + dma_lane_off),
                                             (lds_ptr)&lds[buf * C::TILE + q * 256], 16, 0, 0);
        }
    };

    // ---- local step first: the gradient values of the elements this lane's DMA requests bring in
    // (same blocks, same lane -> (row, 4 columns) map), and the update of those elements in LDS
    float4 gstage[PRO ? C::DMA_PER_WAVE : 1];
    auto load_gdma = [&](int64_t tile) {
#pragma unroll
        for (int i = 0; i < (PRO ? C::DMA_PER_WAVE : 0); ++i) {
            const int q = w + 8 * i;
            const int s = q / (C::KB / 4), kq = q % (C::KB / 4);
            const float4 *src = g + (int64_t)(8 * kq) * ld4 + tile * (C::TC / 4) + s * 8;   // uniform base
            gstage[i] = *(const float4 *)(uniform_base(src) + dma_lane_off);
        }
    };
    auto apply_g = [&](int buf) {
#pragma unroll
        for (int i = 0; i < (PRO ? C::DMA_PER_WAVE : 0); ++i) {
            const int q = w + 8 * i;
            const int kq = q % (C::KB / 4);
            const float eta = lr.at(8 * kq + 2 * (lane >> 4) + ((lane >> 3) & 1));
            float4 *p = (float4 *)&lds[buf * C::TILE + q * 256 + 4 * lane];
            float4 v = *p;
            v.x = fmaf(-eta, gstage[i].x, v.x);
            v.y = fmaf(-eta, gstage[i].y, v.y);
            v.z = fmaf(-eta, gstage[i].z, v.z);
            v.w = fmaf(-eta, gstage[i].w, v.w);
            *p = v;
        }
    };

    int64_t tile = blockIdx.x;
    if (tile >= n_tiles) return;
    if (DMA) {
        dma(tile, 0);
        load_gdma(tile);
        __builtin_amdgcn_s_waitcnt(0);
        asm volatile("" ::: "memory");
        apply_g(0);
    } else {
        fetch(tile);
        commit(0);
    }
    __syncthreads();

    // epilogue addressing: uniform base per (tile, row block, sub-tile, v) + one lane offset
    const uint32_t epi_lane_off = 4u * (uint32_t)(4 * (lane >> 5) * ld + (lane & 31));

    int buf = 0;
    for (; tile < n_tiles; tile += gridDim.x) {
        const int64_t next = tile + gridDim.x;
        if (next < n_tiles) {
            if (DMA) {
                dma(next, buf ^ 1);
                load_gdma(next);
            } else {
                fetch(next);
            }
        }
        if (PRO) __builtin_amdgcn_sched_barrier(0);      // nothing that consumes those values moves up here

        // Per 32-column sub-tile: request its gradient values, multiply, correct and store.  The
        // sub-tiles of a wave go one after the other so that only one accumulator and one set of
        // gradient values are live at a time (the P block already takes half of the registers);
        // the other wave of the SIMD fills the gaps of the dependent chain.  The last sub-tile's
        // stores come after the barrier and drain under the next tile's multiplies.
        float gv[C::SPW][16];
        f32x16 acc[C::SPW];
        auto load_g = [&](int sp) {
            if (ORDER == DBW_ORDER_CTA && HAS_G) {
                const int s = cg * C::SPW + sp;
                const int64_t col0 = tile * C::TC + 32 * s;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row0 = 32 * rb + 8 * (v / 4) + (v & 3);             // uniform
                    const float *gb = gs + (int64_t)row0 * ld + col0;
                    if (FULL) {
                        gv[sp][v] = *(const float *)(uniform_base(gb) + epi_lane_off);
                    } else {
                        const bool ok = row0 + 4 * (lane >> 5) < N && col0 + (lane & 31) < dcols;
                        gv[sp][v] = ok ? *(const float *)(uniform_base(gb) + epi_lane_off) : 0.f;
                    }
                }
            }
        };
        const float *bbase = &lds[buf * C::TILE + lane];
        auto multiply = [&](int sp) {
            const int s = cg * C::SPW + sp;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[sp][v] = 0.f;
            // B fragments come from LDS eight k-steps at a time, one group ahead of the multiplies;
            // the scheduling barriers keep the compiler from requesting all of them up front,
            // which would push the P block out of the registers
            float bq[2][8];
#pragma unroll
            for (int j = 0; j < 8; ++j) bq[0][j] = bbase[(s * C::KB + j) * 64];
#pragma unroll
            for (int q = 0; q < C::KB / 8; ++q) {
                if (q + 1 < C::KB / 8) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) bq[(q + 1) & 1][j] = bbase[(s * C::KB + 8 * (q + 1) + j) * 64];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[sp] = __builtin_amdgcn_mfma_f32_32x32x2f32(wreg[8 * q + j], bq[q & 1][j], acc[sp], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // local SGD correction and store, 32 consecutive columns per row
        auto epilogue = [&](int sp) {
            const int s = cg * C::SPW + sp;
            const int64_t col0 = tile * C::TC + 32 * s;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row0 = 32 * rb + 8 * (v / 4) + (v & 3);
                float r = acc[sp][v];
                if (ORDER == DBW_ORDER_CTA && HAS_G) {
                    const int row = row0 + 4 * (lane >> 5);
                    r = fmaf(-lr.at(FULL || row < N ? row : 0), gv[sp][v], r);
                }
                float *ob = out + (int64_t)row0 * ld + col0;
                if (FULL || (row0 + 4 * (lane >> 5) < N && col0 + (lane & 31) < dcols))
                    *(float *)(const_cast<char *>(uniform_base(ob)) + epi_lane_off) = r;
            }
        };

        load_g(0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int sp = 0; sp + 1 < C::SPW; ++sp) {
            multiply(sp);
            load_g(sp + 1);
            epilogue(sp);
            __builtin_amdgcn_sched_barrier(0);
        }
        multiply(C::SPW - 1);

        // the next tile is complete in LDS before anybody starts on it
        if (next < n_tiles && !DMA) commit(buf ^ 1);
        if (DMA) __builtin_amdgcn_s_waitcnt(0);      // the tile written by global_load_lds has landed
        if (PRO) {
            asm volatile("" ::: "memory");               // LDS reads below stay behind the wait
            if (next < n_tiles) apply_g(buf ^ 1);
        }
        __syncthreads();
        buf ^= 1;
        epilogue(C::SPW - 1);
    }
}

template <int MB, int ORDER, bool HAS_G, class LR>
int launch_mb(dbw_ctx *c, const float *W, const float *x, const float *g, float *out, LR lr, int64_t n_vec,
              hipStream_t s)
{
    using C = dense_cfg<MB>;
    const int64_t n_tiles = (n_vec * 4 + C::TC - 1) / C::TC;
    if (n_tiles > INT32_MAX) return DBW_ERR_UNSUPPORTED;
    if (c->ld > DBW_DENSE_MAX_LD) return DBW_ERR_UNSUPPORTED;
    int cus = 256;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
        cus = prop.multiProcessorCount;
    const int blocks_per_cu = (int)((160 * 1024) / (sizeof(float) * 2 * C::TILE));
    const int64_t grid = std::min<int64_t>(n_tiles, (int64_t)cus * std::max(1, std::min(blocks_per_cu, 4)));
    const bool full = c->N == C::NPAD && c->d % C::TC == 0;
    dbw_timer tm(c, "mix_dense_kernel", s);
    if (full)
        hipLaunchKernelGGL((mix_dense_kernel<MB, ORDER, HAS_G, true, LR>), dim3((unsigned)grid), dim3(DENSE_THREADS), 0, s,
                           c->N, n_vec, c->d, c->ld / 4, W, (const float4 *)x, (const float4 *)g, out, g, lr,
                           (int)n_tiles);
    else
        hipLaunchKernelGGL((mix_dense_kernel<MB, ORDER, HAS_G, false, LR>), dim3((unsigned)grid), dim3(DENSE_THREADS), 0,
                           s, c->N, n_vec, c->d, c->ld / 4, W, (const float4 *)x, (const float4 *)g, out, g, lr,
                           (int)n_tiles);
    DBW_HIP(hipGetLastError());
    return DBW_OK;
}

template <int ORDER, bool HAS_G, class LR>
int launch(dbw_ctx *c, const float *W, const float *x, const float *g, float *out, LR lr, int64_t n_vec,
           hipStream_t s)
{
    switch (c->Npad) {
    case 32: return launch_mb<1, ORDER, HAS_G, LR>(c, W, x, g, out, lr, n_vec, s);
    case 64: return launch_mb<2, ORDER, HAS_G, LR>(c, W, x, g, out, lr, n_vec, s);
    case 128: return launch_mb<4, ORDER, HAS_G, LR>(c, W, x, g, out, lr, n_vec, s);
    case 256: return launch_mb<8, ORDER, HAS_G, LR>(c, W, x, g, out, lr, n_vec, s);
    default: return DBW_ERR_UNSUPPORTED;
    }
}

}  // namespace

int dbw_launch_mix_csr_range(dbw_ctx *c, const float *x, const float *g, float *out, float lr, const float *lr_vec,
                             int64_t c_begin, hipStream_t s);

int64_t dbw_dense_columns(const dbw_ctx *c, const float *x, const float *g, const float *out)
{
    const bool aligned = (c->ld % 4 == 0) && ((uintptr_t)x % 16 == 0) && ((uintptr_t)out % 16 == 0) &&
                         (!g || (uintptr_t)g % 16 == 0);
    return aligned ? c->d : 0;
}

int dbw_launch_mix_dense(dbw_ctx *c, const float *x, const float *g, float *out, float lr, const float *lr_vec,
                         hipStream_t s, const float *W)
{
    const bool own_matrix = W != nullptr;
    if (!W) W = c->Wdense;
    if (!W) return DBW_ERR_STATE;
    // rows are aligned and padded to a multiple of four floats: the float4 that straddles column d is
    // read whole and stored up to d
    const int64_t covered = dbw_dense_columns(c, x, g, out), n_vec = (covered + 3) / 4;
    int rc = DBW_OK;
    if (n_vec > 0) {
        if (!g)
            rc = launch<DBW_ORDER_CTA, false>(c, W, x, g, out, dbw_lr_scalar{0.f}, n_vec, s);
        else if (lr_vec && c->order == DBW_ORDER_ATC)
            rc = launch<DBW_ORDER_ATC, true>(c, W, x, g, out, dbw_lr_vector{lr_vec}, n_vec, s);
        else if (lr_vec)
            rc = launch<DBW_ORDER_CTA, true>(c, W, x, g, out, dbw_lr_vector{lr_vec}, n_vec, s);
        else if (c->order == DBW_ORDER_ATC)
            rc = launch<DBW_ORDER_ATC, true>(c, W, x, g, out, dbw_lr_scalar{lr}, n_vec, s);
        else
            rc = launch<DBW_ORDER_CTA, true>(c, W, x, g, out, dbw_lr_scalar{lr}, n_vec, s);
        if (rc != DBW_OK) return rc;
    }
    // everything when rows are not 16-byte aligned; a caller that brought its own matrix covers
    // those columns itself
    if (covered < c->d && !own_matrix) rc = dbw_launch_mix_csr_range(c, x, g, out, lr, lr_vec, covered, s);
    return rc;
}
