// Measurement support: streaming kernels with the row path's access pattern and no arithmetic, to find
// out what the machine delivers for the traffic mixes of the fused call (reads only, writes only, and
// rows read twice and written once from the same workgroup, as a densely written gradient is).
#include "dvp_device.h"
#include "dvp_internal.h"

namespace dvp {

constexpr int kProbeThreads = 1024;
constexpr int kProbeSlots = 19;      // vectors per thread a row may take (the row kernel's largest build but one)

// every vector of both matrices read once, 8 loads per thread in flight, grid-stride over chunks
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const u32x4 *a, const u32x4 *b, int64_t n, uint32_t *sink)
{
    uint32_t acc = 0;
    const int64_t chunk = (int64_t)8 * kProbeThreads;
    for (int64_t base = (int64_t)blockIdx.x * chunk; base < n; base += (int64_t)gridDim.x * chunk) {
        u32x4 va[8], vb[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t i = base + u * kProbeThreads + threadIdx.x;
            va[u] = i < n ? __builtin_nontemporal_load(a + i) : (u32x4){0u, 0u, 0u, 0u};
            vb[u] = i < n ? __builtin_nontemporal_load(b + i) : (u32x4){0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= va[u].x ^ va[u].y ^ va[u].z ^ va[u].w ^ vb[u].x ^ vb[u].y ^ vb[u].z ^ vb[u].w;
    }
    if (acc == 0x9e3779b9u && sink) *sink = acc;     // keeps the loads alive; practically never taken
}

// (small workgroups, one nontemporal store per thread: the fastest write-only shape found on this chip, see
// the zero kernels of the row path)
constexpr int kProbeFillThreads = 256;
__global__ __launch_bounds__(kProbeFillThreads) void probe_fill_kernel(u32x4 *c, int64_t n)
{
    const u32x4 zero = {0u, 0u, 0u, 0u};
    const int64_t i = (int64_t)blockIdx.x * kProbeFillThreads + threadIdx.x;
    if (i < n) __builtin_nontemporal_store(zero, c + i);
}

// the same fill in the shape that drains worse: 1024 threads, two plain stores each
__global__ __launch_bounds__(kProbeThreads) void probe_fill_wide_kernel(u32x4 *c, int64_t n)
{
    const u32x4 zero = {0u, 0u, 0u, 0u};
    const int64_t base = (int64_t)blockIdx.x * 2 * kProbeThreads + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int64_t i = base + (int64_t)u * kProbeThreads;
        if (i < n) c[i] = zero;
    }
}

// reads by workgroups that take 16 KB each and leave (no workgroup stays to keep a row): a and b one after the other
__global__ __launch_bounds__(kProbeThreads) void probe_read_oneshot_kernel(const u32x4 *a, int64_t n, uint32_t *sink)
{
    const int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
    if (i >= n) return;
    const u32x4 v = __builtin_nontemporal_load(a + i);
    if ((v.x ^ v.w) == 0x9e3779b9u && sink) *sink = v.x;     // keeps the load alive; practically never taken
}

// per row: all of b's row into registers, then all of a's row, then a's row out to c; one workgroup per
// CU walks the rows
__global__ __launch_bounds__(kProbeThreads) void probe_rows_kernel(const u32x4 *a, const u32x4 *b, u32x4 *c, int64_t n_rows,
                                                                    int row_vec)
{
    for (int64_t r = blockIdx.x; r < n_rows; r += gridDim.x) {
        const u32x4 *pa = a + r * row_vec, *pb = b + r * row_vec;
        u32x4 *pc = c + r * row_vec;
        u32x4 v[kProbeSlots];
        uint32_t acc = 0;
#pragma unroll
        for (int j = 0; j < kProbeSlots; ++j) {
            const int i = j * kProbeThreads + threadIdx.x;
            v[j] = i < row_vec ? __builtin_nontemporal_load(pb + i) : (u32x4){0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int j = 0; j < kProbeSlots; ++j) acc |= v[j].x;
#pragma unroll
        for (int j = 0; j < kProbeSlots; ++j) {
            const int i = j * kProbeThreads + threadIdx.x;
            v[j] = i < row_vec ? __builtin_nontemporal_load(pa + i) : (u32x4){0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int j = 0; j < kProbeSlots; ++j) {
            const int i = j * kProbeThreads + threadIdx.x;
            if (acc == 0x9e3779b9u) v[j].x ^= 1u;     // b's row feeds the output, so its loads stay
            if (i < row_vec) __builtin_nontemporal_store(v[j], pc + i);
        }
    }
}

hipError_t launch_probe(int mode, const void *a, const void *b, void *c, int64_t n_rows, int64_t row_bytes, hipStream_t stream)
{
    const int64_t row_vec = row_bytes / 16, n = n_rows * row_vec;
    if (n == 0) return hipSuccess;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus < 1)
        cus = 256;
    if (mode == DVP_PROBE_READ) {
        hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)(4 * cus)), dim3(kProbeThreads), 0, stream, (const u32x4 *)a,
                           (const u32x4 *)b, n, (uint32_t *)nullptr);
    } else if (mode == DVP_PROBE_FILL) {
        const int64_t per = kProbeFillThreads;
        for (int64_t v0 = 0; v0 < n; v0 += per * 0x40000000ll) {     // a launch covers at most 2^30 workgroups
            const int64_t m = n - v0 < per * 0x40000000ll ? n - v0 : per * 0x40000000ll;
            hipLaunchKernelGGL(probe_fill_kernel, dim3((unsigned)((m + per - 1) / per)), dim3(kProbeFillThreads), 0, stream,
                               (u32x4 *)c + v0, m);
        }
    } else if (mode == DVP_PROBE_FILL_WIDE) {
        const int64_t per = 2 * kProbeThreads;
        for (int64_t v0 = 0; v0 < n; v0 += per * 0x40000000ll) {
            const int64_t m = n - v0 < per * 0x40000000ll ? n - v0 : per * 0x40000000ll;
            hipLaunchKernelGGL(probe_fill_wide_kernel, dim3((unsigned)((m + per - 1) / per)), dim3(kProbeThreads), 0, stream,
                               (u32x4 *)c + v0, m);
        }
    } else if (mode == DVP_PROBE_READ_ONESHOT) {
        const int64_t per = kProbeThreads;
        for (const void *src : {a, b})
            for (int64_t v0 = 0; v0 < n; v0 += per * 0x40000000ll) {
                const int64_t m = n - v0 < per * 0x40000000ll ? n - v0 : per * 0x40000000ll;
                hipLaunchKernelGGL(probe_read_oneshot_kernel, dim3((unsigned)((m + per - 1) / per)), dim3(kProbeThreads), 0, stream,
                                   (const u32x4 *)src + v0, m, (uint32_t *)nullptr);
            }
    } else {
        int64_t grid = cus < n_rows ? cus : n_rows;
        hipLaunchKernelGGL(probe_rows_kernel, dim3((unsigned)grid), dim3(kProbeThreads), 0, stream, (const u32x4 *)a,
                           (const u32x4 *)b, (u32x4 *)c, n_rows, (int)row_vec);
    }
    return hipGetLastError();
}

}  // namespace dvp

extern "C" dvp_status dvp_hbm_probe(int mode, const void *a, const void *b, void *c, int64_t n_rows, int64_t row_bytes,
                                    void *stream)
{
    if (mode < DVP_PROBE_READ || mode > DVP_PROBE_READ_ONESHOT) return DVP_ERR_PARAM;
    if (n_rows < 0 || row_bytes < 16 || row_bytes % 16) return DVP_ERR_SHAPE;
    if (mode == DVP_PROBE_ROWS_2R1W && row_bytes > (int64_t)dvp::kProbeSlots * dvp::kProbeThreads * 16) return DVP_ERR_UNSUPPORTED;
    if (n_rows == 0) return DVP_OK;
    const bool reads = mode != DVP_PROBE_FILL && mode != DVP_PROBE_FILL_WIDE;
    const bool writes = mode != DVP_PROBE_READ && mode != DVP_PROBE_READ_ONESHOT;
    if ((reads && (!a || !b)) || (writes && !c)) return DVP_ERR_NULL;
    if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) % 16) return DVP_ERR_ALIGN;
    return dvp::launch_probe(mode, a, b, c, n_rows, row_bytes, (hipStream_t)stream) == hipSuccess ? DVP_OK : DVP_ERR_HIP;
}
