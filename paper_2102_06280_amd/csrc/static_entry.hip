// dbw_consensus_rounds_static: the gradient-free rounds of dbw_consensus_rounds for callers that
// cannot allocate device memory.  No context: the graph comes in as device CSR arrays with every
// call, and everything the kernels need beyond the caller's inputs and outputs (a checked copy of
// the graph, the selection state of each round, the running product of the consensus matrices and
// its matrix-core fragment form, the status words) lives in one file-scope device array.
// Each GPU holds its own copy of that array; its address on a device is looked up once, with that
// device current, and only that address (never the array's name) is handed to kernels.
#include <mutex>

#include "dbw_internal.h"

namespace {

constexpr int STATIC_MAX_N = DBW_DENSE_MAX_N;                       // 256 workers
constexpr int STATIC_MAX_NNZ = STATIC_MAX_N * (STATIC_MAX_N - 1);   // complete graph
constexpr int STATIC_MAX_DEVICES = 64;

constexpr size_t align256(size_t n) { return (n + 255) / 256 * 256; }

// byte offsets of the pieces inside the array
constexpr size_t OFF_ROWPTR = 0;
constexpr size_t OFF_COLIDX = OFF_ROWPTR + align256(sizeof(int32_t) * (STATIC_MAX_N + 1));
constexpr size_t OFF_P = OFF_COLIDX + align256(sizeof(int32_t) * STATIC_MAX_NNZ);
constexpr size_t OFF_MASK = OFF_P + align256(sizeof(int32_t) * STATIC_MAX_N);
constexpr size_t OFF_WAIT = OFF_MASK + align256(STATIC_MAX_NNZ);
constexpr size_t OFF_SEL_IDX = OFF_WAIT + align256(sizeof(float) * STATIC_MAX_N);
constexpr size_t OFF_SEL_W = OFF_SEL_IDX + align256(sizeof(int32_t) * STATIC_MAX_NNZ);
constexpr size_t OFF_SELF_W = OFF_SEL_W + align256(sizeof(float) * STATIC_MAX_NNZ);
constexpr size_t OFF_ERR = OFF_SELF_W + align256(sizeof(float) * STATIC_MAX_N);
constexpr size_t OFF_PHI0 = OFF_ERR + 256;
constexpr size_t PHI_BYTES = sizeof(float) * STATIC_MAX_N * STATIC_MAX_N;
constexpr size_t OFF_PHI1 = OFF_PHI0 + PHI_BYTES;
constexpr size_t OFF_PHI_FRAG = OFF_PHI1 + PHI_BYTES;
constexpr size_t SCRATCH_BYTES = OFF_PHI_FRAG + PHI_BYTES;          // about 1.7 MB

static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

std::mutex g_lock;
unsigned char *g_scratch_ptr[STATIC_MAX_DEVICES] = {};

// Device address of this GPU's copy of the array, looked up on the first call per device.
int scratch_address(unsigned char **out)
{
    int dev = 0;
    DBW_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return DBW_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        DBW_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return DBW_ERR_HIP;
        g_scratch_ptr[dev] = (unsigned char *)ptr;
    }
    *out = g_scratch_ptr[dev];
    return DBW_OK;
}

// Checks the caller's graph and copies it into the array.  What the later kernels rely on for
// memory safety is checked here: rowptr starts at 0, never decreases and ends at nnz; every row is
// strictly ascending with entries in [0, N) other than the row's own index (so no row is longer
// than N - 1); the graph is symmetric.  A graph that fails is replaced by the graph without links
// (every worker keeps its own vector) and the failure is recorded.  One workgroup.
__global__ __launch_bounds__(1024) void stage_graph_kernel(int N, int nnz, const int32_t *__restrict__ rowptr_in,
                                                           const int32_t *__restrict__ colidx_in,
                                                           int32_t *__restrict__ rowptr, int32_t *__restrict__ colidx,
                                                           int32_t *__restrict__ err)
{
    __shared__ int32_t rp[STATIC_MAX_N + 1];
    __shared__ int bad;
    const int tid = threadIdx.x;
    if (tid == 0) bad = 0;
    __syncthreads();
    for (int i = tid; i <= N; i += 1024) rp[i] = rowptr_in[i];
    __syncthreads();
    for (int i = tid; i <= N; i += 1024) {
        const bool ok = (i == 0 ? rp[0] == 0 : rp[i] >= rp[i - 1]) && (i < N || rp[N] == nnz);
        if (!ok) bad = 1;                               // benign race: every writer stores 1
    }
    __syncthreads();
    if (!bad) {                                         // offsets are monotone in [0, nnz]: entry reads stay inside colidx_in
        for (int e = tid; e < nnz; e += 1024) {
            int lo = 0, hi = N;                         // the row i with rp[i] <= e < rp[i + 1]
            while (hi - lo > 1) {
                const int mid = (lo + hi) / 2;
                if (rp[mid] <= e) lo = mid; else hi = mid;
            }
            const int i = lo, j = colidx_in[e];
            bool ok = j >= 0 && j < N && j != i && (e == rp[i] || colidx_in[e - 1] < j);
            if (ok) {                                   // i must be listed in row j
                int a = rp[j], z = rp[j + 1];
                while (a < z) {
                    const int mid = (a + z) / 2;
                    if (colidx_in[mid] < i) a = mid + 1; else z = mid;
                }
                ok = a < rp[j + 1] && colidx_in[a] == i;
            }
            if (!ok) bad = 1;
        }
    }
    __syncthreads();
    const int broken = bad;
    for (int i = tid; i <= N; i += 1024) rowptr[i] = broken ? 0 : rp[i];
    if (!broken)
        for (int e = tid; e < nnz; e += 1024) colidx[e] = colidx_in[e];
    if (tid == 0) {
        err[0] = 0;                                     // out-of-range backup counts, set by the selection kernel
        err[1] = broken ? DBW_ERR_GRAPH : 0;
    }
}

// A bad graph takes precedence over out-of-range backup counts.
__global__ void copy_status_kernel(const int32_t *err, int32_t *status_out) { *status_out = err[1] ? err[1] : err[0]; }

bool overlap(const void *a, size_t na, const void *b, size_t nb)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

}  // namespace

extern "C" int dbw_consensus_rounds_static(int32_t N, int64_t d, int64_t ld, int32_t nnz, const int32_t *rowptr,
                                           const int32_t *colidx, const float *params_in, float *params_out,
                                           const float *resp_times, const int32_t *b, int32_t r,
                                           int32_t *status_out, void *stream)
{
    if (!rowptr || !params_in || !params_out || !resp_times || !b) return DBW_ERR_NULL;
    if (nnz > 0 && !colidx) return DBW_ERR_NULL;
    if (N < 1 || d < 1 || r < 1 || nnz < 0) return DBW_ERR_INVALID;
    if (ld == 0) ld = d;
    if (ld < d) return DBW_ERR_INVALID;
    if (N > STATIC_MAX_N || nnz > STATIC_MAX_NNZ || ld > DBW_DENSE_MAX_LD) return DBW_ERR_UNSUPPORTED;
    const size_t bytes = sizeof(float) * (size_t)N * (size_t)ld;
    if (overlap(params_in, bytes, params_out, bytes)) return DBW_ERR_ALIAS;

    unsigned char *base = nullptr;
    int rc = scratch_address(&base);
    if (rc != DBW_OK) return rc;
    hipStream_t s = (hipStream_t)stream;

    // a context whose device pointers are pieces of the array; its host members stay empty
    dbw_ctx view;
    view.N = N;
    view.d = d;
    view.ld = ld;
    view.nnz = nnz;
    view.max_deg = N - 1;                               // row lengths are known on the device only
    view.Npad = 32;
    while (view.Npad < N) view.Npad *= 2;
    view.rowptr = (int32_t *)(base + OFF_ROWPTR);
    view.colidx = (int32_t *)(base + OFF_COLIDX);
    view.p = (int32_t *)(base + OFF_P);
    view.mask = base + OFF_MASK;
    view.wait = (float *)(base + OFF_WAIT);
    view.sel_idx = (int32_t *)(base + OFF_SEL_IDX);
    view.sel_w = (float *)(base + OFF_SEL_W);
    view.self_w = (float *)(base + OFF_SELF_W);
    view.err = (int32_t *)(base + OFF_ERR);
    view.phi[0] = (float *)(base + OFF_PHI0);
    view.phi[1] = (float *)(base + OFF_PHI1);
    view.phi_frag = (float *)(base + OFF_PHI_FRAG);

    // The array keeps what the previous call left.  The status words must start at zero (the
    // staging kernel writes them; no memset, so that a caller may record this call into a graph);
    // every other piece is written by this call's kernels before it is read: the product starts
    // from the identity over the whole padded square, and the fragment form writes its padding
    // rows as zero.
    hipLaunchKernelGGL(stage_graph_kernel, dim3(1), dim3(1024), 0, s, N, nnz, rowptr, colidx, view.rowptr, view.colidx,
                       view.err);
    DBW_HIP(hipGetLastError());
    rc = dbw_launch_consensus_rounds(&view, params_in, params_out, resp_times, b, r, s);
    if (rc != DBW_OK) return rc;
    if (status_out) {
        hipLaunchKernelGGL(copy_status_kernel, dim3(1), dim3(1), 0, s, view.err, status_out);
        DBW_HIP(hipGetLastError());
    }
    return DBW_OK;
}
