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
constexpr int kReadGrid = 8192;
constexpr int kReadThreads = 256;

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// 16 bytes that will not be read again: a streaming (non-temporal) load.
__device__ __forceinline__ uint4 stream_load16(const uint4* p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return uint4{v.x, v.y, v.z, v.w};
}

__device__ __forceinline__ float dot8(uint4 w, uint4 x, float acc)
{
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.x), __builtin_bit_cast(half2_t, x.x), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.y), __builtin_bit_cast(half2_t, x.y), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.z), __builtin_bit_cast(half2_t, x.z), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.w), __builtin_bit_cast(half2_t, x.w), acc, false);
    return acc;
}

// v from the lane CTRL names (DPP); lanes without a source lane, or outside ROW_MASK, read 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or_zero(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF,
                                                                 ROW_MASK == 0xF));
}

// Sum over the wavefront, in lane 63: shifts inside the rows of 16 lanes, then the row totals
// handed on (lane 15 -> row 1, lane 47 -> row 3, lane 31 -> rows 2 and 3).
__device__ __forceinline__ float wave_sum_in_last_lane(float v)
{
    v += dpp_or_zero<0x111, 0xF>(v);      // row_shr:1
    v += dpp_or_zero<0x112, 0xF>(v);      // row_shr:2
    v += dpp_or_zero<0x114, 0xF>(v);      // row_shr:4
    v += dpp_or_zero<0x118, 0xF>(v);      // row_shr:8
    v += dpp_or_zero<0x142, 0xA>(v);      // row_bcast:15
    v += dpp_or_zero<0x143, 0xC>(v);      // row_bcast:31
    return v;
}

// Dense fp16 GEMV, one output row per wavefront: x staged once per workgroup of kDenseWaves rows
// (an eighth of the bytes the workgroup streams), the row's 16-byte pieces requested eight per
// lane at a time (8 KB per wavefront under way) with streaming loads, fp32 accumulation in two
// chains, a DPP sum at the end.  Workgroups: one per kDenseWaves rows -- 512 for 4096 rows --
// so that several are resident per compute unit and one's loads run under another's arithmetic.
constexpr int kDenseWaves = 8;
constexpr int kDenseInFlight = 8;

__global__ __launch_bounds__(kDenseWaves * 64) void dense_f16_gemv_kernel(const uint16_t* W, const uint16_t* x,
                                                                          uint16_t* y, long long N, long long K)
{
    extern __shared__ __align__(16) uint8_t lds[];
    uint4* xs = reinterpret_cast<uint4*>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int k8 = static_cast<int>(K / 8);
    const long long row = static_cast<long long>(blockIdx.x) * kDenseWaves + (tid >> 6);
    const uint4* wr = reinterpret_cast<const uint4*>(W + (row < N ? row : 0) * K);
    // the row's first pieces go out before x is staged: they are the long wait
    uint4 w[kDenseInFlight];
#pragma unroll
    for (int j = 0; j < kDenseInFlight; ++j) {
        const int i = lane + 64 * j;
        w[j] = stream_load16(wr + (i < k8 ? i : 0));
    }
    for (int i = tid; i < k8; i += kDenseWaves * 64) xs[i] = reinterpret_cast<const uint4*>(x)[i];
    __syncthreads();
    float acc0 = 0.0f, acc1 = 0.0f;
    for (int base = 0; base < k8; base += 64 * kDenseInFlight) {
        uint4 cur[kDenseInFlight];
#pragma unroll
        for (int j = 0; j < kDenseInFlight; ++j) cur[j] = w[j];
        const int next = base + 64 * kDenseInFlight;
        if (next < k8) {
#pragma unroll
            for (int j = 0; j < kDenseInFlight; ++j) {
                const int i = next + lane + 64 * j;
                w[j] = stream_load16(wr + (i < k8 ? i : 0));
            }
        }
#pragma unroll
        for (int j = 0; j < kDenseInFlight; j += 2) {
            const int i0 = base + lane + 64 * j, i1 = i0 + 64;
            // (pieces past the end of the row were loaded from its start: they count as zero)
            const float a = dot8(cur[j], xs[i0 < k8 ? i0 : 0], 0.0f), b = dot8(cur[j + 1], xs[i1 < k8 ? i1 : 0], 0.0f);
            acc0 += i0 < k8 ? a : 0.0f;
            acc1 += i1 < k8 ? b : 0.0f;
        }
    }
    const float total = wave_sum_in_last_lane(acc0 + acc1);
    if (lane == 63 && row < N) y[row] = __builtin_bit_cast(uint16_t, static_cast<_Float16>(total));
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
        hipLaunchKernelGGL(dense_f16_gemv_kernel, dim3(static_cast<unsigned>((N + kDenseWaves - 1) / kDenseWaves)),
                           dim3(kDenseWaves * 64), static_cast<size_t>(K) * 2, s,
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
