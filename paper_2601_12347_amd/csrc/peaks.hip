// Rates this GPU reaches on the four things the library's kernels are bound by, measured with plain kernels of
// known size, so that a kernel's achieved figure can be set against what the chip really delivers and not only
// against its nominal peaks: a streaming copy (HBM), gathers of random 128-byte lines (what a message costs),
// float atomic additions to streaming rows (what a destination costs), and a register-only loop of matrix-core
// instructions (fp32 and bf16).
#include "common.h"
#include "kernels.h"
#include <cstring>

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void k_peak_copy(const float4 *src, float4 *dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__device__ __forceinline__ uint32_t peak_mix(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

__global__ __launch_bounds__(256) void k_peak_read(const float4 *src, size_t n, float *sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float4 v = src[i];
        acc.x += v.x;
        acc.y += v.y;
        acc.z += v.z;
        acc.w += v.w;
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[threadIdx.x] = acc.x;
}

__global__ __launch_bounds__(256) void k_peak_indices(uint32_t *idx, size_t n, uint32_t n_lines) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        idx[i] = (uint32_t)(((unsigned long long)peak_mix((uint32_t)i * 2654435761u + 99u) * n_lines) >> 32);
}

// every wavefront gathers lines of 128 bytes (32 lanes x 4 bytes) at the pseudo-random line indices it reads, 64 at
// a time, from idx; sixteen requests in flight
__global__ __launch_bounds__(256) void k_peak_gather(const float *table, const uint32_t *idx, size_t n_idx, float *sink) {
    const uint32_t lane = threadIdx.x & 63;
    const size_t gw = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = ((size_t)gridDim.x * blockDim.x) >> 6;
    float acc = 0.0f;
    for (size_t base = gw * 64; base < n_idx; base += nw * 64) {
        const uint32_t mine = idx[base + lane];              // n_idx is a multiple of 64
#pragma unroll 1
        for (int k0 = 0; k0 < 64; k0 += 16) {
            float r[16];
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                const uint32_t line = (uint32_t)__shfl((int)mine, k0 + g);
                r[g] = lane < 32 ? table[(size_t)line * 32 + lane] : 0.0f;
            }
#pragma unroll
            for (int g = 0; g < 16; ++g) acc += r[g];
        }
    }
    if (acc == 12345.678f) sink[gw] = acc;                  // keeps the loads alive
}

// one 47-lane atomic addition per row of 48 floats, rows in ascending order per wavefront
__global__ __launch_bounds__(256) void k_peak_atomic(float *rows, uint32_t n_rows) {
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    const uint32_t per = (n_rows + nw - 1) / nw;
    const uint32_t r0 = gw * per, r1 = min(n_rows, r0 + per);
    for (uint32_t r = r0; r < r1; ++r)
        if (lane < 47) unsafeAtomicAdd(&rows[(size_t)r * 48 + lane], 1.0f);
}

// four independent accumulators per wavefront, operands in registers: nothing but matrix-core instructions
template <int BF>
__global__ __launch_bounds__(256) void k_peak_mfma(float *sink, uint32_t iters, float seed) {
    floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    const float av = seed + (float)(threadIdx.x & 63), bv = seed * 0.5f;
    bf16x8 ah, bh;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        ah[k] = (__bf16)av;
        bh[k] = (__bf16)bv;
    }
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (BF) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[i], 0, 0, 0);
            else acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i], 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 12345.678f) sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <typename F>
static hipError_t timed(hipStream_t s, hipEvent_t e0, hipEvent_t e1, int reps, double *best_ms, F launch) {
    *best_ms = 1e30;
    for (int rep = 0; rep < reps + 1; ++rep) {              // the first run warms up
        hipError_t e = hipEventRecord(e0, s);
        if (e != hipSuccess) return e;
        launch();
        if ((e = hipEventRecord(e1, s)) != hipSuccess) return e;
        if ((e = hipEventSynchronize(e1)) != hipSuccess) return e;
        float ms = 0.0f;
        if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) return e;
        if (rep && ms < *best_ms) *best_ms = ms;
    }
    return hipGetLastError();
}

extern "C" ripple_status ripple_measure_peaks(ripple_peaks *out, void *hip_stream) {
    if (!out) return RIPPLE_EINVAL;
    memset(out, 0, sizeof(*out));
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t copy_bytes = (size_t)1 << 30;              // 1 GiB read and 1 GiB written
    const uint32_t n_lines = 4u << 20;                      // 512 MiB table: far beyond every cache
    const uint32_t n_rows = 2u << 20;
    float *a = nullptr, *b = nullptr, *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ripple_status rc = RIPPLE_OK;
    int cu = 0, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0)
        cu = 256;
    if (hipMalloc((void **)&a, copy_bytes) != hipSuccess || hipMalloc((void **)&b, copy_bytes) != hipSuccess ||
        hipMalloc((void **)&sink, (size_t)cu * 16 * 256 * 4) != hipSuccess) {
        (void)hipGetLastError();
        rc = RIPPLE_ENOMEM;
    }
    if (rc == RIPPLE_OK && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) rc = RIPPLE_EDEVICE;
    if (rc == RIPPLE_OK && (hipMemsetAsync(a, 0, copy_bytes, s) != hipSuccess || hipMemsetAsync(b, 0, copy_bytes, s) != hipSuccess))
        rc = RIPPLE_EDEVICE;
    double ms = 0.0;
    if (rc == RIPPLE_OK) {
        const size_t n4 = copy_bytes / 16;
        if (timed(s, e0, e1, 3, &ms, [&] { hipLaunchKernelGGL(k_peak_copy, dim3(cu * 16), dim3(256), 0, s, (const float4 *)a, (float4 *)b, n4); }) != hipSuccess)
            rc = RIPPLE_EDEVICE;
        out->hbm_copy_gbps = 2.0 * (double)copy_bytes / (ms * 1e-3) / 1e9;
    }
    if (rc == RIPPLE_OK) {
        const size_t n4 = copy_bytes / 16;
        if (timed(s, e0, e1, 3, &ms, [&] { hipLaunchKernelGGL(k_peak_read, dim3(cu * 16), dim3(256), 0, s, (const float4 *)a, n4, sink); }) != hipSuccess)
            rc = RIPPLE_EDEVICE;
        out->hbm_read_gbps = (double)copy_bytes / (ms * 1e-3) / 1e9;
    }
    if (rc == RIPPLE_OK) {
        const size_t n_idx = (size_t)32 << 20;              // 33.5 M gathers; the indices (128 MiB) sit in the second buffer
        uint32_t *idx = (uint32_t *)b;
        hipLaunchKernelGGL(k_peak_indices, dim3(cu * 8), dim3(256), 0, s, idx, n_idx, n_lines);
        if (timed(s, e0, e1, 3, &ms, [&] { hipLaunchKernelGGL(k_peak_gather, dim3(cu * 16), dim3(256), 0, s, a, idx, n_idx, sink); }) != hipSuccess)
            rc = RIPPLE_EDEVICE;
        out->gather_glines = (double)n_idx / (ms * 1e-3) / 1e9;
        if (hipMemsetAsync(b, 0, copy_bytes, s) != hipSuccess) rc = RIPPLE_EDEVICE;
    }
    if (rc == RIPPLE_OK) {
        if (timed(s, e0, e1, 3, &ms, [&] { hipLaunchKernelGGL(k_peak_atomic, dim3(cu * 8), dim3(256), 0, s, b, n_rows); }) != hipSuccess)
            rc = RIPPLE_EDEVICE;
        out->atomic_gops = (double)n_rows * 47.0 / (ms * 1e-3) / 1e9;
    }
    const uint32_t iters = 4096;
    if (rc == RIPPLE_OK) {                                  // flops per instruction: 2 * 32 * 32 * k
        const double flops = (double)cu * 8 * 4 * iters * 4.0;
        if (timed(s, e0, e1, 3, &ms, [&] { hipLaunchKernelGGL((k_peak_mfma<0>), dim3(cu * 8), dim3(256), 0, s, sink, iters, 1.0f); }) != hipSuccess)
            rc = RIPPLE_EDEVICE;
        out->mfma_f32_tflops = flops * (2.0 * 32 * 32 * 2) / (ms * 1e-3) / 1e12;
        if (rc == RIPPLE_OK &&
            timed(s, e0, e1, 3, &ms, [&] { hipLaunchKernelGGL((k_peak_mfma<1>), dim3(cu * 8), dim3(256), 0, s, sink, iters, 1.0f); }) != hipSuccess)
            rc = RIPPLE_EDEVICE;
        out->mfma_bf16_tflops = flops * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
    }
    out->compute_units = (uint32_t)cu;
    if (e0) hipEventDestroy(e0);
    if (e1) hipEventDestroy(e1);
    if (a) hipFree(a);
    if (b) hipFree(b);
    if (sink) hipFree(sink);
    return rc;
}
