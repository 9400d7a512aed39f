// Achievable ceilings of the device, measured with two plain kernels that do nothing but
// stream memory or issue matrix instructions.  They give the figure that the round's kernels
// can at best approach on this chip, next to the nominal peaks.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "dbw_measure.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// a = b + s * c over n4 float4 elements, one element per thread, streaming loads and stores:
// the access pattern of the averaging with its gradient term, minus the gather.
__global__ __launch_bounds__(256) void triad_kernel(f32x4 *__restrict__ a, const f32x4 *__restrict__ b,
                                                    const f32x4 *__restrict__ c, float s, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        const f32x4 vb = __builtin_nontemporal_load(b + i);
        const f32x4 vc = __builtin_nontemporal_load(c + i);
        __builtin_nontemporal_store(vb + s * vc, a + i);
    }
}

__global__ __launch_bounds__(256) void fill_kernel(float *p, int64_t n, float v)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v + 1e-3f * (float)(i & 1023);
}

// Four independent chains of 32x32x2 fp32 matrix instructions per wave on register operands.
__global__ __launch_bounds__(256) void mfma_loop_kernel(float *__restrict__ out, int iters, float seed)
{
    f32x16 acc0 = {0}, acc1 = {0}, acc2 = {0}, acc3 = {0};
    const float a = seed + (float)(threadIdx.x & 63) * 1e-3f, b = 1.0f - a;
    for (int k = 0; k < iters; ++k) {
        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, a, acc1, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a, acc2, 0, 0, 0);
        acc3 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, b, acc3, 0, 0, 0);
    }
    const f32x16 s = acc0 + acc1 + acc2 + acc3;
    float t = 0.f;
    for (int v = 0; v < 16; ++v) t += s[v];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = t;
}

struct events {
    hipEvent_t a = nullptr, b = nullptr;
    ~events()
    {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

struct dev_buf {
    void *p = nullptr;
    ~dev_buf()
    {
        if (p) (void)hipFree(p);
    }
};

} // namespace

extern "C" int dbw_calibrate(int32_t what, int64_t size, int32_t repeats, double *result, void *stream_)
{
    if (!result) return DBW_ERR_NULL;
    if (size < 1 || repeats < 1 || repeats > 1000) return DBW_ERR_INVALID;
    hipStream_t s = (hipStream_t)stream_;
    events ev;
    if (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess) return DBW_ERR_HIP;
    float ms = 0.f;
    if (what == DBW_CAL_HBM_TRIAD) {
        if (size % 16 || size > ((int64_t)1 << 34)) return DBW_ERR_INVALID;
        dev_buf a, b, c;
        if (hipMalloc(&a.p, size) != hipSuccess || hipMalloc(&b.p, size) != hipSuccess ||
            hipMalloc(&c.p, size) != hipSuccess) {
            (void)hipGetLastError();
            return DBW_ERR_ALLOC;
        }
        const int64_t n = size / 4, n4 = size / 16;
        const unsigned gf = (unsigned)((n + 255) / 256), g4 = (unsigned)((n4 + 255) / 256);
        hipLaunchKernelGGL(fill_kernel, dim3(gf), dim3(256), 0, s, (float *)b.p, n, 1.0f);
        hipLaunchKernelGGL(fill_kernel, dim3(gf), dim3(256), 0, s, (float *)c.p, n, 2.0f);
        hipLaunchKernelGGL(triad_kernel, dim3(g4), dim3(256), 0, s, (f32x4 *)a.p, (const f32x4 *)b.p,
                           (const f32x4 *)c.p, 0.5f, n4);   // warm-up
        if (hipEventRecord(ev.a, s) != hipSuccess) return DBW_ERR_HIP;
        for (int r = 0; r < repeats; ++r)
            hipLaunchKernelGGL(triad_kernel, dim3(g4), dim3(256), 0, s, (f32x4 *)a.p, (const f32x4 *)b.p,
                               (const f32x4 *)c.p, 0.5f, n4);
        if (hipEventRecord(ev.b, s) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess ||
            hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess)
            return DBW_ERR_HIP;
        *result = 3.0 * (double)size * repeats / (ms * 1e-3) / 1e9;            // GB/s
    } else if (what == DBW_CAL_MFMA_FP32) {
        if (size > (1 << 24)) return DBW_ERR_INVALID;
        const int blocks = 256 * 8;                       // 8 workgroups of 4 waves per compute unit
        dev_buf out;
        if (hipMalloc(&out.p, (size_t)blocks * 256 * 4) != hipSuccess) {
            (void)hipGetLastError();
            return DBW_ERR_ALLOC;
        }
        hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(256), 0, s, (float *)out.p, 16, 0.25f);
        if (hipEventRecord(ev.a, s) != hipSuccess) return DBW_ERR_HIP;
        for (int r = 0; r < repeats; ++r)
            hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(256), 0, s, (float *)out.p, (int)size, 0.25f);
        if (hipEventRecord(ev.b, s) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess ||
            hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess)
            return DBW_ERR_HIP;
        const double flops = 4.0 * 4096.0 * (double)size * 4.0 * blocks * repeats;   // 4 chains x 2*32*32*2, 4 waves
        *result = flops / (ms * 1e-3) / 1e12;                                        // TFLOP/s
    } else {
        return DBW_ERR_INVALID;
    }
    if (hipGetLastError() != hipSuccess) return DBW_ERR_HIP;
    return DBW_OK;
}
