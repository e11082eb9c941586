// Measurement aids (lychee_bench.h), kept apart from the decode path: a plain streaming read of a
// device buffer, so that a benchmark can report what read bandwidth this GPU reaches next to its
// published peak, and a launch of the select+attend kernel of lc_decode_step by itself.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lc_internal.h"
#include "lychee_bench.h"

#define LC_SWEEP_THREADS 256
#define LC_SWEEP_WGS 2048
#define LC_SWEEP_UNROLL 4

// Every workgroup walks the buffer with a grid stride, 16 bytes per lane and load, four loads in
// flight per lane; the loaded words are folded into one value per workgroup so the loads stay live.
__global__ void __launch_bounds__(LC_SWEEP_THREADS)
lc_read_sweep_kernel(const uint4* __restrict__ src, size_t n_vec, uint32_t* __restrict__ sink) {
    __shared__ uint32_t fold[LC_SWEEP_THREADS / 64];
    const size_t stride = (size_t)gridDim.x * LC_SWEEP_THREADS;
    size_t i = (size_t)blockIdx.x * LC_SWEEP_THREADS + threadIdx.x;
    uint32_t acc = 0u;
    for (; i + (LC_SWEEP_UNROLL - 1) * stride < n_vec; i += LC_SWEEP_UNROLL * stride) {
        uint4 v[LC_SWEEP_UNROLL];
#pragma unroll
        for (int u = 0; u < LC_SWEEP_UNROLL; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < LC_SWEEP_UNROLL; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n_vec; i += stride) {
        const uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    for (int m = 1; m < 64; m <<= 1) acc ^= __shfl_xor(acc, m);
    if ((threadIdx.x & 63) == 0) fold[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t r = 0u;
        for (int w = 0; w < LC_SWEEP_THREADS / 64; ++w) r ^= fold[w];
        sink[blockIdx.x] = r;
    }
}

extern "C" int lc_bench_read_sweep(const void* src, size_t bytes, uint32_t* sink, size_t sink_words, void* stream) {
    if (!src || !sink || bytes == 0) return LC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (bytes & 15u)) return LC_ERR_INVALID_ARG;
    if (sink_words < (size_t)LC_SWEEP_WGS) return LC_ERR_WORKSPACE_TOO_SMALL;
    hipLaunchKernelGGL(lc_read_sweep_kernel, dim3(LC_SWEEP_WGS), dim3(LC_SWEEP_THREADS), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint4*>(src), bytes / 16, sink);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}

extern "C" int lc_bench_select_attend(const lc_index* idx, const void* q, const void* K, const void* V,
                                      const int64_t kv_strides[3], int H_q, int budget, float* out, float* lse,
                                      void* ws, size_t ws_bytes, void* stream) {
    return lc_decode_step_impl(idx, q, K, V, kv_strides, H_q, budget, out, lse, nullptr, nullptr, 0, ws, ws_bytes,
                               stream, /*second_kernel_only=*/true);
}
