// Streaming-bandwidth probe: what plain kernels with the access shapes of this library's hot kernels reach on the
// device at hand.  A measurement aid beside the per-kernel timing: the roofline of an HBM-bound kernel is quoted
// against the published peak, and this says how much of that peak ANY kernel of the same read/write mix gets.
#include "common.h"

typedef u64 u64x2 __attribute__((ext_vector_type(2)));

// every workgroup streams one contiguous run with 16-byte non-temporal loads, eight in flight per lane
__global__ __launch_bounds__(256) void k_probe_read(const u64x2 *__restrict__ p, size_t per_wg16, u64 *out) {
    u64 acc = 0;
    const u64x2 *q = p + (size_t)blockIdx.x * per_wg16;
    for (size_t i = threadIdx.x; i + 7 * 256 < per_wg16; i += 8 * 256) {
        u64x2 v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = __builtin_nontemporal_load(q + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; u++) acc ^= v[u].x ^ v[u].y;
    }
    if (acc == 0x0123456789ABCDEFULL) out[blockIdx.x] = acc;      // keeps the loads alive; never true for the fill pattern
}
// NR read streams of n16 words each (adjacent in src), one write stream
template <int NR>
__global__ __launch_bounds__(256) void k_probe_mix(u64x2 *__restrict__ dst, const u64x2 *__restrict__ src, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        u64x2 v = {0, 0};
#pragma unroll
        for (int r = 0; r < NR; r++) {
            const u64x2 t = __builtin_nontemporal_load(src + r * n16 + i);
            v.x ^= t.x, v.y ^= t.y;
        }
        __builtin_nontemporal_store(v, dst + i);
    }
}

extern "C" cm_status cm_hbm_probe(int32_t kind, uint64_t bytes, int32_t reps, double *gb_per_s) {
    (void)hipGetLastError();
    if (!gb_per_s || reps < 1 || reps > 100 || kind < CM_PROBE_READ || kind > CM_PROBE_READ3_WRITE1) return CM_E_INVAL;
    if (bytes < ((uint64_t)64 << 20) || bytes > ((uint64_t)16 << 30)) return CM_E_INVAL;
    const int reads = kind == CM_PROBE_READ3_WRITE1 ? 3 : 1, writes = kind == CM_PROBE_READ ? 0 : 1;
    const unsigned wgs = 8192;
    // stream length: a multiple of what one sweep of the grid covers, so that every pattern moves whole runs
    const size_t unit16 = (size_t)wgs * 256 * 8;
    size_t n16 = bytes / 16 / (size_t)(reads + writes) / unit16 * unit16;
    if (!n16) n16 = unit16;
    u64x2 *src = nullptr, *dst = nullptr;
    u64 *out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    cm_status st = CM_E_NOMEM;
    double best = 0;
    if (hipMalloc((void **)&src, n16 * 16 * reads) != hipSuccess) goto done;
    if (hipMalloc((void **)&out, wgs * sizeof(u64)) != hipSuccess) goto done;
    if (writes && hipMalloc((void **)&dst, n16 * 16) != hipSuccess) goto done;
    st = CM_E_HIP;
    if (hipMemset(src, 0x5A, n16 * 16 * reads) != hipSuccess) goto done;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto done;
    for (int r = 0; r <= reps; r++) {          // the first pass is a warm-up
        if (hipEventRecord(e0, 0) != hipSuccess) goto done;
        if (kind == CM_PROBE_READ)
            hipLaunchKernelGGL(k_probe_read, dim3(wgs), dim3(256), 0, 0, src, n16 / wgs, out);
        else if (kind == CM_PROBE_COPY)
            hipLaunchKernelGGL(k_probe_mix<1>, dim3(wgs), dim3(256), 0, 0, dst, src, n16);
        else
            hipLaunchKernelGGL(k_probe_mix<3>, dim3(wgs), dim3(256), 0, 0, dst, src, n16);
        if (hipEventRecord(e1, 0) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) goto done;
        float ms = 0;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !(ms > 0)) goto done;
        const double rate = (double)n16 * 16 * (reads + writes) / (ms * 1e-3) / 1e9;
        if (r && rate > best) best = rate;
    }
    if (hipGetLastError() != hipSuccess) goto done;
    *gb_per_s = best;
    st = CM_OK;
done:
    if (e0) hipEventDestroy(e0);
    if (e1) hipEventDestroy(e1);
    hipFree(src);
    hipFree(dst);
    hipFree(out);
    return st;
}
