// Offline pre-processing of the GQS layer on the GPU (gfx950): the same steps as the host packer
// -- group the weights along K in runs of G, score every group (Sec. 3.1 Eq. 4 with a caller-supplied
// diag(H^-1), or the group's sum of squares), prune the least salient groups of every row
// (Sec. 3.2, Fig. 3), quantise the kept ones (Eq. 1-2) -- producing the BSR arrays of the Sec. 3.2
// listing plus scales and zeros, and, in the same pass, the blocks of the device image that the
// GEMV kernel streams.  The arithmetic is the host packer's operation for operation (float64
// saliency sums in index order, single IEEE fp32 operations in the quantiser, round-half-even),
// so the results are the same bits.
//
// One workgroup per output row.  The row's saliencies live in LDS; which groups go is decided by
// counting, for every group, the groups that are pruned before it (lower saliency, or equal
// saliency and lower column): a group is pruned iff that count is below the row's pruned count.
// A prefix sum over the kept flags gives every kept group its place in the row, and with the
// row's first stream position (worked out on the host from the row pointers alone) its block and
// lane in the image.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "gqsa_internal.hpp"

namespace gqsa {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxColumns = 4096;      // group-columns of a row (the format's limit)

struct PackArgs {
    const float* W;            // [N][K]
    const float* hinv;         // [K] or nullptr
    const int32_t* rowIndex;   // [N+1]
    const int64_t* row_pos;    // [N] first stream position of every row
    int32_t* groups;           // canonical arrays (outputs)
    uint8_t* values;
    uint16_t* scales;
    uint16_t* zeros;
    uint8_t* blocks;           // device image, blocks region (zeroed beforehand)
    int* status;               // bit 0: a non-finite saliency; bit 1: a bad entry of hinv; bit 2: a scale beyond fp16
    long long K;
    int kg, G, bits, cb, U, L, bb, slots_per_group;     // (U blocks per tile, L lanes in use per block)
};

__device__ __forceinline__ uint16_t half_bits(float f) { return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f)); }
__device__ __forceinline__ float half_value(uint16_t b) { return static_cast<float>(__builtin_bit_cast(_Float16, b)); }

__global__ __launch_bounds__(kThreads) void pack_rows_kernel(PackArgs a)
{
    __shared__ double sal[kMaxColumns];
    __shared__ uint8_t kept[kMaxColumns];
    __shared__ int counts[kThreads];
    __shared__ int bad;

    const int tid = threadIdx.x;
    const long long n = blockIdx.x;
    const float* wrow = a.W + n * a.K;
    const int g0 = a.rowIndex[n];
    const int keep = a.rowIndex[n + 1] - g0;
    const int kg = a.kg, G = a.G;
    if (keep == 0) return;                                  // (uniform: the whole workgroup leaves)
    const int drop = kg - keep;
    // every thread owns a contiguous run of group-columns
    const int chunk = (kg + kThreads - 1) / kThreads;
    const int c_begin = min(kg, tid * chunk), c_end = min(kg, c_begin + chunk);

    if (tid == 0) bad = 0;
    __syncthreads();
    // saliency of a weight: w^2 / d_k^2; of a group: the sum over its members, float64, index order
    for (int c = c_begin; c < c_end; ++c) {
        const float* p = wrow + static_cast<long long>(c) * G;
        double acc = 0.0;
        if (a.hinv) {
            const float* d = a.hinv + static_cast<long long>(c) * G;
            for (int j = 0; j < G; ++j) {
                const double t = static_cast<double>(p[j]) / static_cast<double>(d[j]);
                acc += t * t;
            }
        } else {
            for (int j = 0; j < G; ++j) acc += static_cast<double>(p[j]) * static_cast<double>(p[j]);
        }
        sal[c] = acc;
        if (!(fabs(acc) <= 1.79769313486231570815e+308)) bad = 1;     // NaN or infinite
    }
    __syncthreads();
    if (bad) {
        if (tid == 0) atomicOr(a.status, 1);
        return;
    }
    // a group is pruned iff fewer than `drop` groups come before it in the order of pruning
    int mine = 0;
    for (int c = c_begin; c < c_end; ++c) {
        bool k = true;
        if (drop > 0) {
            const double s = sal[c];
            int before = 0;
            for (int o = 0; o < kg; ++o) {
                const double so = sal[o];
                before += (so < s || (so == s && o < c)) ? 1 : 0;
            }
            k = before >= drop;
        }
        kept[c] = k ? 1 : 0;
        mine += k ? 1 : 0;
    }
    counts[tid] = mine;
    __syncthreads();
    // place of this thread's first kept group in the row: kept groups of the threads before it
    int place = 0;
    for (int t = 0; t < tid; ++t) place += counts[t];

    const float levels = static_cast<float>((1 << a.bits) - 1);
    for (int c = c_begin; c < c_end; ++c) {
        if (!kept[c]) continue;
        const int i = place++;                      // the group's number inside its row
        const long long g = static_cast<long long>(g0) + i;
        const float* w = wrow + static_cast<long long>(c) * G;
        // Eq. 1: the first smallest and the last largest element, as the host's scan finds them
        float lo = w[0], hi = w[0];
        for (int j = 1; j < G; ++j) {
            if (w[j] < lo) lo = w[j];
            if (!(w[j] < hi)) hi = w[j];
        }
        float s = (hi - lo) / levels;
        uint16_t sb = half_bits(s);
        if ((sb & 0x7FFFu) >= 0x7C00u) atomicOr(a.status, 4);      // the group's range is beyond what an fp16 scale holds
        s = half_value(sb);
        const float kMinScale = 0x1p-14f;
        if (!(s >= kMinScale)) {
            s = kMinScale;
            sb = half_bits(s);
        }
        float z = __builtin_rintf(-lo / s);         // round-half-even
        z = (z < -2048.0f) ? -2048.0f : z;
        z = (2048.0f < z) ? 2048.0f : z;
        const uint16_t zb = half_bits(z);
        a.groups[g] = c;
        a.scales[g] = sb;
        a.zeros[g] = zb;
        // where the group sits in the image: tile of U blocks, lane l owns U consecutive positions
        const long long pos = a.row_pos[n] + i;
        const long long tile_groups = static_cast<long long>(a.L) * a.U;
        const long long p = pos % tile_groups;
        const long long block = pos / tile_groups * a.U + p % a.U;
        const int lane = static_cast<int>(p / a.U);
        uint8_t* base = a.blocks + block * a.bb;
        const int cb = a.cb, pb = cb < 16 ? cb : 16;
        uint8_t* vout = a.values + g * cb;
        // Eq. 2, eight codes at a time: a canonical word (two codes per byte, even element low; or
        // one byte per code) and the image's word (4-bit: element 2m at bits 4m, 2m+1 at 16+4m)
        for (int h = 0; h < G / 8 + (G < 8 ? 1 : 0); ++h) {
            uint32_t q8[8];
            for (int e = 0; e < 8; ++e) {
                float q = __builtin_rintf(w[8 * h + e] / s) + z;
                q = (0.0f < q) ? q : 0.0f;
                q = (q < levels) ? q : levels;
                q8[e] = static_cast<uint32_t>(q);
            }
            if (a.bits == 4) {
                uint32_t canon = 0, image = 0;
                for (int e = 0; e < 8; ++e) {
                    canon |= q8[e] << (4 * e);
                    image |= q8[e] << ((e & 1) ? 16 + 4 * (e >> 1) : 4 * (e >> 1));
                }
                *reinterpret_cast<uint32_t*>(vout + 4 * h) = canon;
                const int byte = 4 * h;             // of the lane's code string
                *reinterpret_cast<uint32_t*>(base + (byte / pb) * a.L * pb + lane * pb + byte % pb) = image;
            } else {
                for (int half = 0; half < 2; ++half) {
                    const uint32_t word = q8[4 * half] | (q8[4 * half + 1] << 8) | (q8[4 * half + 2] << 16) | (q8[4 * half + 3] << 24);
                    const int byte = 8 * h + 4 * half;
                    *reinterpret_cast<uint32_t*>(vout + byte) = word;
                    *reinterpret_cast<uint32_t*>(base + (byte / pb) * a.L * pb + lane * pb + byte % pb) = word;
                }
            }
        }
        *reinterpret_cast<uint32_t*>(base + a.L * cb + lane * 4) = static_cast<uint32_t>(sb) | (static_cast<uint32_t>(zb) << 16);
        *reinterpret_cast<uint16_t*>(base + a.L * (cb + 4) + lane * 2) =
            static_cast<uint16_t>(((c * a.slots_per_group) << 4) | (i == 0 ? 1 : 0));
    }
}

__global__ __launch_bounds__(kThreads) void check_hinv_kernel(const float* d, long long K, int* status)
{
    const long long k = static_cast<long long>(blockIdx.x) * kThreads + threadIdx.x;
    if (k < K && !(d[k] > 0.0f && d[k] <= 3.40282346638528859812e+38f)) atomicOr(status, 2);
}

struct DeviceBuffers {        // temporaries of one pack, freed whatever happens
    void* p[8] = {};
    ~DeviceBuffers() { for (void* q : p) if (q) (void)hipFree(q); }
};

#define GQSA_HIP(call)                                                                   \
    do {                                                                                 \
        const hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) {                                                          \
            std::fprintf(stderr, "libgqsa: %s: %s\n", #call, hipGetErrorString(e_));    \
            return GQSA_ERR_HIP;                                                         \
        }                                                                                \
    } while (0)

}  // namespace

// W_dev [N][K] fp32 and hinv_dev [K] (or nullptr) on the current GPU; m has N, K, G, bits and its
// row pointers (the kept count of every row is known beforehand).  Fills the canonical arrays and
// the device image of m -- on the GPU, then copied to the host side of the handle -- and leaves
// the handle uploaded.  Synchronises `stream`.
gqsa_status_t pack_on_device(const float* W_dev, const float* hinv_dev, gqsa_matrix* m, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t nnz = m->nnzg();
    const int cb = m->code_bytes();
    if (m->K / m->G > kMaxColumns) return GQSA_ERR_SHAPE;
    // the layout of the image follows from the row pointers alone: partition, row positions,
    // per-worker records, row tables (host), with the blocks left empty
    std::vector<int64_t> row_pos;
    if (gqsa_status_t st = build_image(m, default_partition(*m), /*fill_blocks=*/false, &row_pos)) return st;
    m->groups.assign(static_cast<size_t>(nnz), 0);
    m->values.assign(static_cast<size_t>(nnz) * cb, 0);
    m->scales.assign(static_cast<size_t>(nnz), 0);
    m->zeros.assign(static_cast<size_t>(nnz), 0);

    DeviceBuffers tmp;
    void* img = nullptr;
    GQSA_HIP(hipMalloc(&img, m->image.size()));
    struct ImageGuard { void* p; ~ImageGuard() { if (p) (void)hipFree(p); } } guard{img};
    const size_t blocks_bytes = m->map.wave_info;          // the blocks region comes first
    GQSA_HIP(hipMemsetAsync(img, 0, blocks_bytes, s));
    GQSA_HIP(hipMemcpyAsync(static_cast<uint8_t*>(img) + blocks_bytes, m->image.data() + blocks_bytes,
                            m->image.size() - blocks_bytes, hipMemcpyHostToDevice, s));
    const size_t sizes[7] = {(static_cast<size_t>(m->N) + 1) * 4, static_cast<size_t>(m->N) * 8,
                             static_cast<size_t>(nnz) * 4, static_cast<size_t>(nnz) * cb,
                             static_cast<size_t>(nnz) * 2, static_cast<size_t>(nnz) * 2, 4};
    for (int i = 0; i < 7; ++i) GQSA_HIP(hipMalloc(&tmp.p[i], sizes[i] ? sizes[i] : 4));
    GQSA_HIP(hipMemcpyAsync(tmp.p[0], m->rowIndex.data(), sizes[0], hipMemcpyHostToDevice, s));
    GQSA_HIP(hipMemcpyAsync(tmp.p[1], row_pos.data(), sizes[1], hipMemcpyHostToDevice, s));
    GQSA_HIP(hipMemsetAsync(tmp.p[6], 0, 4, s));

    PackArgs a{};
    a.W = W_dev;
    a.hinv = hinv_dev;
    a.rowIndex = static_cast<const int32_t*>(tmp.p[0]);
    a.row_pos = static_cast<const int64_t*>(tmp.p[1]);
    a.groups = static_cast<int32_t*>(tmp.p[2]);
    a.values = static_cast<uint8_t*>(tmp.p[3]);
    a.scales = static_cast<uint16_t*>(tmp.p[4]);
    a.zeros = static_cast<uint16_t*>(tmp.p[5]);
    a.blocks = static_cast<uint8_t*>(img);
    a.status = static_cast<int*>(tmp.p[6]);
    a.K = m->K;
    a.kg = static_cast<int>(m->K / m->G);
    a.G = m->G;
    a.bits = m->bits;
    a.cb = cb;
    a.U = m->tile_blocks;
    a.L = m->tile_lanes;
    a.bb = m->block_bytes();
    a.slots_per_group = m->G >= 16 ? m->G / 16 : 1;
    if (hinv_dev)
        hipLaunchKernelGGL(check_hinv_kernel, dim3(static_cast<unsigned>((m->K + kThreads - 1) / kThreads)), dim3(kThreads), 0, s,
                           hinv_dev, static_cast<long long>(m->K), a.status);
    hipLaunchKernelGGL(pack_rows_kernel, dim3(static_cast<unsigned>(m->N)), dim3(kThreads), 0, s, a);
    GQSA_HIP(hipGetLastError());
    int status = 0;
    GQSA_HIP(hipMemcpyAsync(&status, tmp.p[6], 4, hipMemcpyDeviceToHost, s));
    if (nnz > 0) {
        GQSA_HIP(hipMemcpyAsync(m->groups.data(), tmp.p[2], sizes[2], hipMemcpyDeviceToHost, s));
        GQSA_HIP(hipMemcpyAsync(m->values.data(), tmp.p[3], sizes[3], hipMemcpyDeviceToHost, s));
        GQSA_HIP(hipMemcpyAsync(m->scales.data(), tmp.p[4], sizes[4], hipMemcpyDeviceToHost, s));
        GQSA_HIP(hipMemcpyAsync(m->zeros.data(), tmp.p[5], sizes[5], hipMemcpyDeviceToHost, s));
    }
    GQSA_HIP(hipMemcpyAsync(m->image.data(), img, blocks_bytes, hipMemcpyDeviceToHost, s));
    GQSA_HIP(hipStreamSynchronize(s));
    if (status != 0) return GQSA_ERR_RANGE;                // non-finite weights, a bad diag(H^-1), or a scale beyond fp16
    // the image is where the GEMV wants it already: the handle takes it over
    if (gqsa_status_t st = device_upload(m, img)) return st;
    guard.p = nullptr;
    return GQSA_OK;
}

}  // namespace gqsa
