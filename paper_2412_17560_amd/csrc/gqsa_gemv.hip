// Device side of libgqsa for gfx950 (MI355X): the GQSA decode GEMV  y = W^ x  over the
// block-sparse, group-quantised storage of the paper's GQS layer (Sec. 3.2), i.e. the
// operator flow of Sec. 3.5 / Fig. 4 -- stream the compressed groups, fetch the activation
// group named by each stored group's real group index, dequantise in registers (Eq. 3),
// multiply-accumulate, write back -- with the work split "task-centric" (Sec. 3.5, Fig. 5):
// every wavefront owns an equal, contiguous count of stored groups regardless of row
// boundaries, reduces them with a segmented wavefront scan, and leaves the partial sums of
// the rows it shares with its neighbours to a carry fix-up.
//
// Wavefront = 64 lanes.  A block is 64 stored groups, one per lane, so that every load is
// one fully coalesced instruction; in a superblock of U blocks lane l owns the U
// consecutive stream positions U*l .. U*l+U-1, sums them serially and takes part in ONE
// cross-lane segmented scan per superblock.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#include "gqsa_internal.hpp"

namespace gqsa {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

struct GemvArgs {
    const uint8_t* blocks;
    const int32_t* wave_info;    // {rank_base, tail_closed} per worker
    const int32_t* row_of_rank;  // row index of the r-th non-empty row (nullptr: identity)
    const int32_t* empty_rows;
    CarryRecord* carry;
    const uint16_t* x;           // fp16 [K]
    uint16_t* y;                 // fp16 [N]
    long long n_blocks;
    int n_waves;
    int n_empty;
    int n_ranks;                 // non-empty rows
    int kg;                      // group-columns K/G
};

__device__ __forceinline__ float half_to_float(uint32_t bits16)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(bits16)));
}

__device__ __forceinline__ uint16_t float_to_half_bits(float v)
{
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(v));  // round-to-nearest-even
}

__device__ __forceinline__ half2_t as_half2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }

// Eight 4-bit codes of one word against eight activations (four fp16 pairs).  The word is
// nibble-permuted at pack time: element 2m sits at bits 4m, element 2m+1 at bits 16+4m, so
// one AND/OR splices a pair of codes into the mantissas of the fp16 pair (1024+q, 1024+q')
// or (1024+16q, 1024+16q'); one packed op removes the bias exactly.
__device__ __forceinline__ float dot8_w4(uint32_t w, uint4 x, float acc)
{
    const half2_t k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
    const half2_t k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t k64 = {(_Float16)64.0f, (_Float16)64.0f};
    const uint32_t w2 = w >> 8;
    half2_t q0 = as_half2((w & 0x000F000Fu) | 0x64006400u) - k1024;
    half2_t q1 = as_half2((w & 0x00F000F0u) | 0x64006400u) * k16th - k64;
    half2_t q2 = as_half2((w2 & 0x000F000Fu) | 0x64006400u) - k1024;
    half2_t q3 = as_half2((w2 & 0x00F000F0u) | 0x64006400u) * k16th - k64;
    acc = __builtin_amdgcn_fdot2(q0, as_half2(x.x), acc, false);
    acc = __builtin_amdgcn_fdot2(q1, as_half2(x.y), acc, false);
    acc = __builtin_amdgcn_fdot2(q2, as_half2(x.z), acc, false);
    acc = __builtin_amdgcn_fdot2(q3, as_half2(x.w), acc, false);
    return acc;
}

// Four 8-bit codes (bytes of w, element order) against two fp16 pairs: a byte permute
// drops each code into the mantissa of 1024.0 (0x64xx), one packed subtract removes the bias.
__device__ __forceinline__ float dot4_w8(uint32_t w, uint32_t x01, uint32_t x23, float acc)
{
    const half2_t k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
    const uint32_t k64s = 0x64646464u;
    half2_t q01 = as_half2(__builtin_amdgcn_perm(w, k64s, 0x00050004u)) - k1024;
    half2_t q23 = as_half2(__builtin_amdgcn_perm(w, k64s, 0x00070006u)) - k1024;
    acc = __builtin_amdgcn_fdot2(q01, as_half2(x01), acc, false);
    acc = __builtin_amdgcn_fdot2(q23, as_half2(x23), acc, false);
    return acc;
}

struct WaveState {
    float carry;   // sum of the groups since the last row head (or since the run began)
    int rank;      // rank (among non-empty rows) of the row that is open now
    int heads;     // row heads seen so far in this worker's run
};

__device__ __forceinline__ void store_row(const GemvArgs& a, int rank, float v)
{
    if (static_cast<unsigned>(rank) >= static_cast<unsigned>(a.n_ranks)) return;  // never for a valid image
    const int row = a.row_of_rank ? a.row_of_rank[rank] : rank;
    a.y[row] = float_to_half_bits(v);
}

template <int BITS, int U>
__device__ __forceinline__ void process_superblock(const GemvArgs& a, const uint8_t* p, int lane,
                                                   int wave, int rank_base, const uint4* x_lo,
                                                   const uint4* x_hi, const float* x_sum,
                                                   WaveState& st)
{
    constexpr int CB = 16 * BITS / 8;                 // code bytes per group
    constexpr int BB = (CB + 6) * kLanes;             // block bytes
    constexpr int SZ_OFF = CB * kLanes;
    constexpr int IX_OFF = SZ_OFF + 4 * kLanes;

    // (1) stream the compressed groups: U coalesced loads of each kind, all in flight at once
    uint32_t code[U][CB / 4];
    uint32_t sz[U];
    uint32_t ix[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint8_t* blk = p + static_cast<size_t>(u) * BB;
        if constexpr (BITS == 4) {
            const uint2 c = reinterpret_cast<const uint2*>(blk)[lane];
            code[u][0] = c.x; code[u][1] = c.y;
        } else {
            const uint4 c = reinterpret_cast<const uint4*>(blk)[lane];
            code[u][0] = c.x; code[u][1] = c.y; code[u][2] = c.z; code[u][3] = c.w;
        }
        sz[u] = reinterpret_cast<const uint32_t*>(blk + SZ_OFF)[lane];
        ix[u] = reinterpret_cast<const uint16_t*>(blk + IX_OFF)[lane];
    }

    // (2)-(4) gather the activation group by real group index, dequantise, multiply:
    //   sum_j (q_j - z) s x_j  =  s * (sum_j q_j x_j  -  z * sum_j x_j)
    float part[U];
    int heads_before = 0;   // row heads at earlier stream positions of this superblock (other lanes)
    int heads_total = 0;
    uint32_t head_bits = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int col = ix[u] & 0x7FFF;
        const uint4 xl = x_lo[col];
        const uint4 xh = x_hi[col];
        const float xs = x_sum[col];
        float d = 0.0f;
        if constexpr (BITS == 4) {
            d = dot8_w4(code[u][0], xl, d);
            d = dot8_w4(code[u][1], xh, d);
        } else {
            d = dot4_w8(code[u][0], xl.x, xl.y, d);
            d = dot4_w8(code[u][1], xl.z, xl.w, d);
            d = dot4_w8(code[u][2], xh.x, xh.y, d);
            d = dot4_w8(code[u][3], xh.z, xh.w, d);
        }
        const float s = half_to_float(sz[u] & 0xFFFFu);
        const float z = half_to_float(sz[u] >> 16);
        part[u] = s * __builtin_fmaf(-z, xs, d);

        const bool is_head = (ix[u] >> 15) != 0;
        head_bits |= is_head ? (1u << u) : 0u;
        const unsigned long long bal = __ballot(is_head);
        heads_before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(bal >> 32),
                       __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(bal), heads_before));
        heads_total += __popcll(bal);
    }

    // (5a) serial segmented sum over the lane's U consecutive groups
    float acc = 0.0f, lead = 0.0f;
    int nh = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (head_bits & (1u << u)) {
            if (nh == 0) {
                lead = acc;                       // belongs to the row entering from the left
            } else {
                store_row(a, st.rank + heads_before + nh, acc);   // a whole row inside one lane
            }
            acc = 0.0f;
            ++nh;
        }
        acc += part[u];
    }

    // (5b) cross-lane segmented inclusive scan of the lanes' open sums.  dist = how far to
    // the left the lane's segment reaches; a lane with a head starts a segment.
    const bool has = nh > 0;
    const unsigned long long hmask = __ballot(has);
    const unsigned long long upto = hmask & ((2ull << lane) - 1ull);
    const int dist = upto ? lane - (63 - __builtin_clzll(upto)) : lane;
    float v = acc;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float t = __shfl_up(v, d, 64);
        if (dist >= d) v += t;
    }
    // sum flowing into this lane from the left: previous lane's segment sum, plus the run's
    // carry if no lane before this one has a head
    const float prev = __shfl_up(v, 1, 64);
    const bool head_before = (hmask & ((1ull << lane) - 1ull)) != 0;
    float inflow = lane == 0 ? 0.0f : prev;
    if (!head_before) inflow += st.carry;

    if (has) {
        const float total = inflow + lead;
        const int r = st.rank + heads_before;     // the row this lane's first head closes
        if (r == rank_base) {
            a.carry[wave].lead = total;           // row began before this worker's run
        } else {
            store_row(a, r, total);
        }
    }
    const float last = __shfl(v, 63, 64);
    st.carry = (hmask ? 0.0f : st.carry) + last;
    st.rank += heads_total;
    st.heads += heads_total;
}

template <int BITS>
__global__ __launch_bounds__(kWavesPerWorkgroup * kLanes) void gqsa_gemv_kernel(GemvArgs a)
{
    extern __shared__ __align__(16) uint8_t lds[];
    uint4* x_lo = reinterpret_cast<uint4*>(lds);          // elements 0..7 of every group-column
    uint4* x_hi = x_lo + a.kg;                            // elements 8..15
    float* x_sum = reinterpret_cast<float*>(x_hi + a.kg); // sum of the 16 activations

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = blockIdx.x * (blockDim.x >> 6) + (tid >> 6);

    // stage x once per workgroup, split so that a gather of 16 B per lane spreads over all banks
    for (int c = tid; c < a.kg; c += blockDim.x) {
        const uint4* src = reinterpret_cast<const uint4*>(a.x + static_cast<size_t>(c) * 16);
        const uint4 lo = src[0], hi = src[1];
        x_lo[c] = lo;
        x_hi[c] = hi;
        const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            s += half_to_float(w[i] & 0xFFFFu);
            s += half_to_float(w[i] >> 16);
        }
        x_sum[c] = s;
    }
    // rows without stored groups: exactly +0
    for (int i = blockIdx.x * blockDim.x + tid; i < a.n_empty; i += gridDim.x * blockDim.x)
        a.y[a.empty_rows[i]] = 0;
    __syncthreads();

    if (wave >= a.n_waves) return;
    const long long per = a.n_blocks / a.n_waves;
    const int extra = static_cast<int>(a.n_blocks % a.n_waves);
    long long mine = per + (wave < extra ? 1 : 0);
    if (mine == 0) return;
    const long long first = per * wave + (wave < extra ? wave : extra);

    constexpr int BB = (16 * BITS / 8 + 6) * kLanes;
    const uint8_t* p = a.blocks + static_cast<size_t>(first) * BB;
    const int rank_base = a.wave_info[2 * wave];
    const int tail_closed = a.wave_info[2 * wave + 1];
    WaveState st{0.0f, rank_base, 0};

    while (mine >= 4) {
        process_superblock<BITS, 4>(a, p, lane, wave, rank_base, x_lo, x_hi, x_sum, st);
        p += 4 * BB;
        mine -= 4;
    }
    if (mine >= 2) {
        process_superblock<BITS, 2>(a, p, lane, wave, rank_base, x_lo, x_hi, x_sum, st);
        p += 2 * BB;
        mine -= 2;
    }
    if (mine >= 1) {
        process_superblock<BITS, 1>(a, p, lane, wave, rank_base, x_lo, x_hi, x_sum, st);
    }

    if (lane == 0) {
        a.carry[wave].tail = st.carry;
        a.carry[wave].heads = st.heads;
        if (tail_closed && st.heads > 0) store_row(a, st.rank, st.carry);  // last row ends with the run
    }
}

// Carry fix-up: a row whose groups continue past the end of a worker's run is completed
// here, adding in fixed order the tail of the worker that holds its head, the whole runs of
// head-less workers after it and the lead of the worker that holds the next head.
__global__ void gqsa_fixup_kernel(GemvArgs a)
{
    const int w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= a.n_waves) return;
    const long long per = a.n_blocks / a.n_waves;
    const int extra = static_cast<int>(a.n_blocks % a.n_waves);
    if (per + (w < extra ? 1 : 0) == 0) return;
    if (a.wave_info[2 * w + 1]) return;         // its last row ends with its run
    const CarryRecord me = a.carry[w];
    if (me.heads == 0) return;                  // part of an earlier worker's row
    float sum = me.tail;
    for (int b = w + 1; b < a.n_waves; ++b) {
        if (per + (b < extra ? 1 : 0) == 0) break;
        const CarryRecord o = a.carry[b];
        if (o.heads == 0) {
            sum += o.tail;
            if (a.wave_info[2 * b + 1]) break;
        } else {
            sum += o.lead;
            break;
        }
    }
    store_row(a, a.wave_info[2 * w] + me.heads, sum);
}

#define GQSA_HIP(call)                                                                      \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess) {                                                             \
            std::fprintf(stderr, "libgqsa: %s failed: %s\n", #call, hipGetErrorString(e_)); \
            return GQSA_ERR_HIP;                                                            \
        }                                                                                   \
    } while (0)

}  // namespace

gqsa_status_t device_upload(gqsa_matrix* m)
{
    const size_t lds = static_cast<size_t>(m->K / m->G) * 36;
    if (lds > 160 * 1024) return GQSA_ERR_UNSUPPORTED;
    int dev = 0;
    GQSA_HIP(hipGetDevice(&dev));
    if (lds > 64 * 1024) {
        GQSA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gqsa_gemv_kernel<4>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        GQSA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gqsa_gemv_kernel<8>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    }
    void* img = nullptr;
    void* carry = nullptr;
    GQSA_HIP(hipMalloc(&img, m->image.size()));
    const size_t carry_bytes = static_cast<size_t>(m->n_waves) * sizeof(CarryRecord);
    hipError_t e = hipMalloc(&carry, carry_bytes);
    if (e == hipSuccess) e = hipMemcpy(img, m->image.data(), m->image.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(carry, 0, carry_bytes);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        std::fprintf(stderr, "libgqsa: upload failed: %s\n", hipGetErrorString(e));
        (void)hipFree(img);
        (void)hipFree(carry);
        return GQSA_ERR_HIP;
    }
    m->d_image = img;
    m->d_carry = carry;
    m->device = dev;
    return GQSA_OK;
}

void device_release(gqsa_matrix* m)
{
    if (m->d_image) (void)hipFree(m->d_image);
    if (m->d_carry) (void)hipFree(m->d_carry);
    m->d_image = nullptr;
    m->d_carry = nullptr;
}

gqsa_status_t device_gemv(gqsa_matrix* m, const void* x, void* y, int batch, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint8_t* img = static_cast<const uint8_t*>(m->d_image);
    GemvArgs a;
    a.blocks = img + m->map.blocks;
    a.wave_info = reinterpret_cast<const int32_t*>(img + m->map.wave_info);
    a.row_of_rank = m->n_empty ? reinterpret_cast<const int32_t*>(img + m->map.row_of_rank) : nullptr;
    a.empty_rows = reinterpret_cast<const int32_t*>(img + m->map.empty_rows);
    a.carry = static_cast<CarryRecord*>(m->d_carry);
    a.n_blocks = m->n_blocks;
    a.n_waves = m->n_waves;
    a.n_empty = static_cast<int>(m->n_empty);
    a.n_ranks = static_cast<int>(m->N - m->n_empty);
    a.kg = static_cast<int>(m->K / m->G);

    const int threads = kWavesPerWorkgroup * kLanes;
    const int grid = (m->n_waves + kWavesPerWorkgroup - 1) / kWavesPerWorkgroup;
    const size_t lds = static_cast<size_t>(a.kg) * 36;
    for (int b = 0; b < batch; ++b) {
        a.x = static_cast<const uint16_t*>(x) + static_cast<size_t>(b) * m->K;
        a.y = static_cast<uint16_t*>(y) + static_cast<size_t>(b) * m->N;
        if (m->bits == 4)
            hipLaunchKernelGGL(gqsa_gemv_kernel<4>, dim3(grid), dim3(threads), lds, s, a);
        else
            hipLaunchKernelGGL(gqsa_gemv_kernel<8>, dim3(grid), dim3(threads), lds, s, a);
        if (m->needs_fixup) {
            const int ft = 256;
            hipLaunchKernelGGL(gqsa_fixup_kernel, dim3((m->n_waves + ft - 1) / ft), dim3(ft), 0, s, a);
        }
    }
    GQSA_HIP(hipGetLastError());
    return GQSA_OK;
}

}  // namespace gqsa
