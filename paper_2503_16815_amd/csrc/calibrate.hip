// Measured peaks of the device, for the benchmark's roofline report (not part of the
// paper's method): what LDS delivers for the access mix of the DP sweep, and what HBM
// delivers for a plain copy.  Each figure is bytes moved / HIP-event time of one launch
// that keeps every compute unit busy.
#include <hip/hip_runtime.h>

#include <cstring>

#include "../../include/deft_knapsack.h"

namespace {

constexpr int kLdsThreads = 256;
constexpr int kLdsBytes = 40960;   // four workgroups per compute unit, as the 40 KB rows of the sweep

// 8 conflict-free 4-byte reads per lane and iteration.
__global__ void __launch_bounds__(kLdsThreads) lds_read_kernel(int *out, int iters)
{
    extern __shared__ __align__(16) int lds[];
    const int tid = threadIdx.x;
    for (int i = tid; i < kLdsBytes / 4; i += kLdsThreads) lds[i] = i;
    __syncthreads();
    int acc = 0;
    const unsigned a = tid * 4;
    for (int it = 0; it < iters; ++it) {
        int v0, v1, v2, v3, v4, v5, v6, v7;
        asm volatile("ds_read_b32 %0, %8\n ds_read_b32 %1, %8 offset:1024\n ds_read_b32 %2, %8 offset:2048\n"
                     "ds_read_b32 %3, %8 offset:3072\n ds_read_b32 %4, %8 offset:4096\n ds_read_b32 %5, %8 offset:5120\n"
                     "ds_read_b32 %6, %8 offset:6144\n ds_read_b32 %7, %8 offset:7168\n s_waitcnt lgkmcnt(0)"
                     : "=v"(v0), "=v"(v1), "=v"(v2), "=v"(v3), "=v"(v4), "=v"(v5), "=v"(v6), "=v"(v7)
                     : "v"(a)
                     : "memory");
        acc += v0 + v1 + v2 + v3 + v4 + v5 + v6 + v7;
    }
    out[blockIdx.x * kLdsThreads + tid] = acc;
}

// The sweep's mix: per cell one 4-byte read at an arbitrary (here odd) cell shift and one
// 4-byte write back to the lane's own cell, the write without an address (M0 + offset +
// 4 * lane), four of each per lane and iteration.
__global__ void __launch_bounds__(kLdsThreads) lds_read_write_kernel(int *out, int iters)
{
    extern __shared__ __align__(16) int lds[];
    const int tid = threadIdx.x;
    for (int i = tid; i < kLdsBytes / 4; i += kLdsThreads) lds[i] = i;
    __syncthreads();
    int acc = tid;
    const unsigned a = ((tid + 4096 - 37) % 4096) * 4;   // row[c - 37]
    const int m0 = (int)(uintptr_t)(__attribute__((address_space(3))) int *)lds + (tid & ~63) * 4;
    for (int it = 0; it < iters; ++it) {
        int v0, v1, v2, v3;
        asm volatile("s_nop 0\n"
                     "ds_read_b32 %0, %4\n ds_read_b32 %1, %4 offset:4096\n ds_read_b32 %2, %4 offset:8192\n"
                     "ds_read_b32 %3, %4 offset:12288\n"
                     "ds_write_addtid_b32 %5 offset:16384\n ds_write_addtid_b32 %5 offset:20480\n"
                     "ds_write_addtid_b32 %5 offset:24576\n ds_write_addtid_b32 %5 offset:28672\n s_waitcnt lgkmcnt(0)"
                     : "=v"(v0), "=v"(v1), "=v"(v2), "=v"(v3)
                     : "v"(a), "v"(acc), "{m0}"(m0)
                     : "memory");
        acc += v0 + v1 + v2 + v3;
    }
    out[blockIdx.x * kLdsThreads + tid] = acc;
}

typedef int v4i __attribute__((ext_vector_type(4)));
constexpr int kUnroll = 4;  // 16-byte accesses in flight per lane

// Streaming copy: four 16-byte non-temporal loads, then four stores, per lane and trip.
__global__ void __launch_bounds__(256) copy_kernel(const v4i *__restrict__ src, v4i *__restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256 * kUnroll;
    for (size_t i = (size_t)blockIdx.x * 256 * kUnroll + threadIdx.x; i + 256 * (kUnroll - 1) < n; i += stride) {
        v4i v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(&src[i + 256 * u]);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) __builtin_nontemporal_store(v[u], &dst[i + 256 * u]);
    }
}

__global__ void __launch_bounds__(256) read_kernel(const v4i *__restrict__ src, int *out, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256 * kUnroll;
    int acc = 0;
    for (size_t i = (size_t)blockIdx.x * 256 * kUnroll + threadIdx.x; i + 256 * (kUnroll - 1) < n; i += stride) {
        v4i v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = src[i + 256 * u];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678) out[0] = acc;  // (keeps the loads alive; the fill pattern never sums to this)
}

__global__ void __launch_bounds__(256) fill_kernel(v4i *dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256 * kUnroll;
    for (size_t i = (size_t)blockIdx.x * 256 * kUnroll + threadIdx.x; i + 256 * (kUnroll - 1) < n; i += stride) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) dst[i + 256 * u] = v4i{1, 2, 3, 4};
    }
}

template <class F>
bool timed(F &&launch, float *ms)
{
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return false;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return false; }
    bool ok = hipEventRecord(e0, nullptr) == hipSuccess;
    launch();
    ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, nullptr) == hipSuccess &&
         hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(ms, e0, e1) == hipSuccess;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return ok;
}

}  // namespace

extern "C" deft_status_t deft_knapsack_measure_peaks(int32_t device, deft_knapsack_peaks_t *out)
{
    if (!out || device < 0) return DEFT_ERR_INVALID_ARG;
    std::memset(out, 0, sizeof(*out));
    int ndev = 0, prev = -1;
    if (hipGetDeviceCount(&ndev) != hipSuccess) { (void)hipGetLastError(); return DEFT_ERR_DEVICE; }
    if (device >= ndev) return DEFT_ERR_INVALID_ARG;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) { (void)hipGetLastError(); return DEFT_ERR_DEVICE; }
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return DEFT_ERR_DEVICE;
    if (hipGetDevice(&prev) != hipSuccess || hipSetDevice(device) != hipSuccess) { (void)hipGetLastError(); return DEFT_ERR_DEVICE; }
    const int cus = prop.multiProcessorCount;
    out->compute_units = cus;
    out->clock_mhz_reported = prop.clockRate / 1000;

    deft_status_t rc = DEFT_OK;
    int *sink = nullptr;
    v4i *a = nullptr, *b = nullptr;
    const int wgs = cus * 8;
    const size_t copy_bytes = (size_t)1 << 30, n16 = copy_bytes / 16;
    if (hipMalloc(&sink, (size_t)wgs * kLdsThreads * 4) != hipSuccess || hipMalloc(&a, copy_bytes) != hipSuccess ||
        hipMalloc(&b, copy_bytes) != hipSuccess) {
        (void)hipGetLastError();
        rc = DEFT_ERR_OOM;
    }
    if (rc == DEFT_OK) {
        const int iters = 20000;
        float ms = 0.f, best;
        bool ok = true;
        // warm-up, then the best of three (the shader clock needs a moment to rise)
        hipLaunchKernelGGL(lds_read_kernel, dim3(wgs), dim3(kLdsThreads), kLdsBytes, nullptr, sink, 200);
        best = 1e30f;
        for (int r = 0; r < 3 && ok; ++r) {
            ok = timed([&] { hipLaunchKernelGGL(lds_read_kernel, dim3(wgs), dim3(kLdsThreads), kLdsBytes, nullptr, sink, iters); }, &ms);
            if (ms < best) best = ms;
        }
        out->lds_read_gbs = (float)((double)wgs * kLdsThreads * 32.0 * iters / (best * 1e-3) / 1e9);
        hipLaunchKernelGGL(lds_read_write_kernel, dim3(wgs), dim3(kLdsThreads), kLdsBytes, nullptr, sink, 200);
        best = 1e30f;
        for (int r = 0; r < 3 && ok; ++r) {
            ok = timed([&] { hipLaunchKernelGGL(lds_read_write_kernel, dim3(wgs), dim3(kLdsThreads), kLdsBytes, nullptr, sink, iters); }, &ms);
            if (ms < best) best = ms;
        }
        out->lds_read_write_gbs = (float)((double)wgs * kLdsThreads * 32.0 * iters / (best * 1e-3) / 1e9);
        const dim3 grid((unsigned)cus * 32), block(256);
        hipLaunchKernelGGL(fill_kernel, grid, block, 0, nullptr, a, n16);
        hipLaunchKernelGGL(copy_kernel, grid, block, 0, nullptr, a, b, n16);
        best = 1e30f;
        for (int r = 0; r < 3 && ok; ++r) {
            ok = timed([&] { hipLaunchKernelGGL(copy_kernel, grid, block, 0, nullptr, a, b, n16); }, &ms);
            if (ms < best) best = ms;
        }
        out->hbm_copy_gbs = (float)(2.0 * copy_bytes / (best * 1e-3) / 1e9);
        best = 1e30f;
        for (int r = 0; r < 3 && ok; ++r) {
            ok = timed([&] { hipLaunchKernelGGL(read_kernel, grid, block, 0, nullptr, a, sink, n16); }, &ms);
            if (ms < best) best = ms;
        }
        out->hbm_read_gbs = (float)((double)copy_bytes / (best * 1e-3) / 1e9);
        best = 1e30f;
        for (int r = 0; r < 3 && ok; ++r) {
            ok = timed([&] { hipLaunchKernelGGL(fill_kernel, grid, block, 0, nullptr, b, n16); }, &ms);
            if (ms < best) best = ms;
        }
        out->hbm_write_gbs = (float)((double)copy_bytes / (best * 1e-3) / 1e9);
        if (!ok || hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); rc = DEFT_ERR_DEVICE; }
    }
    if (sink) (void)hipFree(sink);
    if (a) (void)hipFree(a);
    if (b) (void)hipFree(b);
    if (prev >= 0) (void)hipSetDevice(prev);
    return rc;
}
