// Side-by-side kernels for the benchmark harness (gfx950): a dense fp16 GEMV -- the FP16
// baseline the paper's end-to-end tables compare against (Tab. 4, Tab. 13) -- and a
// read-only streaming kernel that measures the achievable HBM read rate.  They share the
// launch geometry of the GQSA kernel (one workgroup per compute unit, persistent wavefronts).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#include "gqsa_bench.h"
#include "gqsa_internal.hpp"

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kThreads = 1024;
constexpr int kGrid = 256;
constexpr int kReadGrid = 8192;
constexpr int kReadThreads = 256;

__device__ __forceinline__ float dot8(uint4 w, uint4 x, float acc)
{
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.x), __builtin_bit_cast(half2_t, x.x), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.y), __builtin_bit_cast(half2_t, x.y), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.z), __builtin_bit_cast(half2_t, x.z), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.w), __builtin_bit_cast(half2_t, x.w), acc, false);
    return acc;
}

// One wavefront per output row at a time; lanes stride over K in 16-byte pieces.
__global__ __launch_bounds__(kThreads) void dense_f16_gemv_kernel(const uint16_t* W, const uint16_t* x,
                                                                  uint16_t* y, long long N, long long K)
{
    extern __shared__ __align__(16) uint8_t lds[];
    uint4* xs = reinterpret_cast<uint4*>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const long long k8 = K / 8;
    for (long long i = tid; i < k8; i += blockDim.x) xs[i] = reinterpret_cast<const uint4*>(x)[i];
    __syncthreads();
    const long long waves = static_cast<long long>(gridDim.x) * (blockDim.x >> 6);
    for (long long row = static_cast<long long>(blockIdx.x) * (blockDim.x >> 6) + (tid >> 6); row < N;
         row += waves) {
        const uint4* wr = reinterpret_cast<const uint4*>(W + row * K);
        float acc0 = 0.0f, acc1 = 0.0f;
        long long i = lane;
        for (; i + 64 < k8; i += 128) {
            const uint4 a = wr[i], b = wr[i + 64];
            acc0 = dot8(a, xs[i], acc0);
            acc1 = dot8(b, xs[i + 64], acc1);
        }
        if (i < k8) acc0 = dot8(wr[i], xs[i], acc0);
        float acc = acc0 + acc1;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
        if (lane == 0) y[row] = __builtin_bit_cast(uint16_t, static_cast<_Float16>(acc));
    }
}

// Every workgroup reads its own contiguous share of the buffer, four 16-byte loads per thread
// in flight (the access pattern that read fastest of those tried on this GPU: 6.3 TB/s on 4 GiB).
__global__ __launch_bounds__(kReadThreads) void stream_read_kernel(const uint4* buf, size_t n16,
                                                                   uint32_t* sink)
{
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t begin = per * blockIdx.x;
    const size_t end = begin + per < n16 ? begin + per : n16;
    uint32_t acc = 0;
    size_t i = begin + threadIdx.x;
    for (; i + 3 * kReadThreads < end; i += 4 * kReadThreads) {
        const uint4 a = buf[i], b = buf[i + kReadThreads], c = buf[i + 2 * kReadThreads], d = buf[i + 3 * kReadThreads];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < end; i += kReadThreads) {
        const uint4 a = buf[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) acc ^= __shfl_xor(acc, d, 64);
    __shared__ uint32_t part[kReadThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t r = 0;
        for (int w = 0; w < kReadThreads / 64; ++w) r ^= part[w];
        sink[blockIdx.x] = r;
    }
}

// Plain copy of 16-byte words: reads n16*16 bytes and writes as many.  Calibrates the HBM
// byte counters of the profiler against a kernel whose traffic is known.
__global__ __launch_bounds__(kReadThreads) void copy_kernel(const uint4* src, uint4* dst, size_t n16)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}

// Does nothing: measures what a launch of the GEMV's geometry costs by itself.
__global__ __launch_bounds__(kThreads) void launch_floor_kernel(uint32_t* sink)
{
    extern __shared__ __align__(16) uint8_t lds[];
    if (sink == nullptr && threadIdx.x == 0) lds[0] = 1;   // never true: keeps the LDS allocation
}

}  // namespace

extern "C" {

gqsa_status_t gqsa_dense_f16_gemv(const void* W_dev, const void* x_dev, void* y_dev, int64_t N,
                                  int64_t K, int batch, void* hip_stream)
{
    if (!W_dev || !x_dev || !y_dev) return GQSA_ERR_NULL;
    if (N <= 0 || K <= 0 || K % 8 != 0) return GQSA_ERR_SHAPE;
    if (batch < 1 || batch > gqsa::kMaxBatch) return GQSA_ERR_UNSUPPORTED;
    if (K * 2 > 64 * 1024) return GQSA_ERR_UNSUPPORTED;
    if (((reinterpret_cast<uintptr_t>(W_dev) | reinterpret_cast<uintptr_t>(x_dev)) & 15u) != 0)
        return GQSA_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    for (int b = 0; b < batch; ++b) {
        hipLaunchKernelGGL(dense_f16_gemv_kernel, dim3(kGrid), dim3(kThreads), static_cast<size_t>(K) * 2, s,
                           static_cast<const uint16_t*>(W_dev),
                           static_cast<const uint16_t*>(x_dev) + static_cast<size_t>(b) * K,
                           static_cast<uint16_t*>(y_dev) + static_cast<size_t>(b) * N,
                           static_cast<long long>(N), static_cast<long long>(K));
    }
    if (hipGetLastError() != hipSuccess) return GQSA_ERR_HIP;
    return GQSA_OK;
}

gqsa_status_t gqsa_launch_floor(int n_workgroups, int lds_bytes, void* sink_dev, void* hip_stream)
{
    if (!sink_dev) return GQSA_ERR_NULL;
    if (n_workgroups < 1 || n_workgroups > 65536 || lds_bytes < 0 || lds_bytes > 64 * 1024)
        return GQSA_ERR_RANGE;
    hipLaunchKernelGGL(launch_floor_kernel, dim3(n_workgroups), dim3(kThreads), static_cast<size_t>(lds_bytes),
                       static_cast<hipStream_t>(hip_stream), static_cast<uint32_t*>(sink_dev));
    if (hipGetLastError() != hipSuccess) return GQSA_ERR_HIP;
    return GQSA_OK;
}

gqsa_status_t gqsa_copy(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream)
{
    if (!dst_dev || !src_dev) return GQSA_ERR_NULL;
    if (bytes % 16 != 0) return GQSA_ERR_SHAPE;
    if (((reinterpret_cast<uintptr_t>(dst_dev) | reinterpret_cast<uintptr_t>(src_dev)) & 15u) != 0)
        return GQSA_ERR_ALIGN;
    hipLaunchKernelGGL(copy_kernel, dim3(kReadGrid), dim3(kReadThreads), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint4*>(src_dev), static_cast<uint4*>(dst_dev), bytes / 16);
    if (hipGetLastError() != hipSuccess) return GQSA_ERR_HIP;
    return GQSA_OK;
}

int gqsa_stream_read_workgroups(void) { return kReadGrid; }

gqsa_status_t gqsa_stream_read(const void* buf_dev, size_t bytes, void* sink_dev, void* hip_stream)
{
    if (!buf_dev || !sink_dev) return GQSA_ERR_NULL;
    if (bytes % 16 != 0) return GQSA_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(buf_dev) & 15u) != 0) return GQSA_ERR_ALIGN;
    // at least four loads per thread; at most kReadGrid workgroups
    const size_t n16 = bytes / 16;
    size_t grid = n16 / (4 * kReadThreads);
    grid = grid < 1 ? 1 : (grid > kReadGrid ? kReadGrid : grid);
    hipLaunchKernelGGL(stream_read_kernel, dim3(static_cast<unsigned>(grid)), dim3(kReadThreads), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(buf_dev), n16,
                       static_cast<uint32_t*>(sink_dev));
    if (hipGetLastError() != hipSuccess) return GQSA_ERR_HIP;
    return GQSA_OK;
}

}  // extern "C"
