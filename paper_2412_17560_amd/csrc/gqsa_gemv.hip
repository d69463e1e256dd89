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
    const int4* wave_info;       // {rank_base, tail_closed, lead_first, chain_len} per worker
    const int32_t* row_of_rank;  // row index of the r-th non-empty row (nullptr: identity)
    const int32_t* empty_rows;
    CarryRecord* carry;
    int* counters;               // arrivals per carry chain, indexed by the chain's first worker
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

// Value of v in another lane, selected by a DPP control; lanes whose source lane does not
// exist (or whose row is masked off) read 0.
// The empty asm pins the cross-lane move where it is written: it must execute with every
// lane active, so it may not be sunk into the lane-predicated addition that uses its result.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or_zero(float v)
{
    int t = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false);
    asm volatile("" : "+v"(t));
    return __builtin_bit_cast(float, t);
}

struct WaveState {
    float carry;   // sum of the groups since the last row head (or since the run began)
    float lead;    // sum of the groups before the run's first row head
    int rank;      // rank (among non-empty rows) of the row that is open now
    int heads;     // row heads seen so far in this worker's run
};

__device__ __forceinline__ void store_row(const GemvArgs& a, int rank, float v)
{
    if (static_cast<unsigned>(rank) >= static_cast<unsigned>(a.n_ranks)) return;  // never for a valid image
    const int row = a.row_of_rank ? a.row_of_rank[rank] : rank;
    a.y[row] = float_to_half_bits(v);
}

// The compressed groups of up to four blocks, as loaded (one group per lane per block).
template <int BITS>
struct Tile {
    uint32_t code[4][BITS / 2];
    uint32_t sz[4];
    uint32_t ix[4];
};

// (1) stream the compressed groups: coalesced loads, all issued before anything waits.
template <int BITS>
__device__ __forceinline__ void load_tile(Tile<BITS>& t, const uint8_t* p, int U, int lane)
{
    constexpr int CB = 16 * BITS / 8;                 // code bytes per group
    constexpr int BB = (CB + 6) * kLanes;             // block bytes
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (u < U) {
            const uint8_t* blk = p + static_cast<size_t>(u) * BB;
            if constexpr (BITS == 4) {
                const uint2 c = reinterpret_cast<const uint2*>(blk)[lane];
                t.code[u][0] = c.x; t.code[u][1] = c.y;
            } else {
                const uint4 c = reinterpret_cast<const uint4*>(blk)[lane];
                t.code[u][0] = c.x; t.code[u][1] = c.y; t.code[u][2] = c.z; t.code[u][3] = c.w;
            }
            t.sz[u] = reinterpret_cast<const uint32_t*>(blk + CB * kLanes)[lane];
            t.ix[u] = reinterpret_cast<const uint16_t*>(blk + (CB + 4) * kLanes)[lane];
        }
    }
}

template <int BITS, int U>
__device__ __forceinline__ void compute_tile(const GemvArgs& a, const Tile<BITS>& t, int lane,
                                             const uint4* x_lo, const uint4* x_hi,
                                             const float* x_sum, WaveState& st)
{
    // (2)-(4) gather the activation group by real group index, dequantise, multiply:
    //   sum_j (q_j - z) s x_j  =  s * (sum_j q_j x_j  -  z * sum_j x_j)
    float part[U];
    int heads_before = 0;   // row heads of this superblock in lower lanes
    int heads_total = 0;
    uint32_t head_bits = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int col = t.ix[u] & 0x7FFF;
        const uint4 xl = x_lo[col];
        const uint4 xh = x_hi[col];
        const float xs = x_sum[col];
        float d = 0.0f;
        if constexpr (BITS == 4) {
            d = dot8_w4(t.code[u][0], xl, d);
            d = dot8_w4(t.code[u][1], xh, d);
        } else {
            d = dot4_w8(t.code[u][0], xl.x, xl.y, d);
            d = dot4_w8(t.code[u][1], xl.z, xl.w, d);
            d = dot4_w8(t.code[u][2], xh.x, xh.y, d);
            d = dot4_w8(t.code[u][3], xh.z, xh.w, d);
        }
        const float s = half_to_float(t.sz[u] & 0xFFFFu);
        const float z = half_to_float(t.sz[u] >> 16);
        part[u] = s * __builtin_fmaf(-z, xs, d);

        const bool is_head = (t.ix[u] >> 15) != 0;
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

    // (5b) cross-lane segmented inclusive scan of the lanes' open sums with DPP.  dist = how
    // far to the left the lane's segment reaches (a lane holding a head starts a segment).
    // Four shifts inside each row of 16 lanes, then the row totals are handed to the next
    // rows (lane 15 -> row 1, lane 47 -> row 3, then lane 31 -> rows 2 and 3).
    const bool has = nh > 0;
    const unsigned long long hmask = __ballot(has);
    const unsigned long long upto = hmask & ((2ull << lane) - 1ull);
    const int dist = upto ? lane - (63 - __builtin_clzll(upto)) : lane;
    float v = acc;
    float sh;
    sh = dpp_or_zero<0x111, 0xF>(v); v += dist >= 1 ? sh : 0.0f;           // row_shr:1
    sh = dpp_or_zero<0x112, 0xF>(v); v += dist >= 2 ? sh : 0.0f;           // row_shr:2
    sh = dpp_or_zero<0x114, 0xF>(v); v += dist >= 4 ? sh : 0.0f;           // row_shr:4
    sh = dpp_or_zero<0x118, 0xF>(v); v += dist >= 8 ? sh : 0.0f;           // row_shr:8
    sh = dpp_or_zero<0x142, 0xA>(v); v += dist > (lane & 15) ? sh : 0.0f;  // row_bcast:15
    sh = dpp_or_zero<0x143, 0xC>(v); v += dist > lane - 32 ? sh : 0.0f;    // row_bcast:31
    // sum flowing into this lane from the left: the previous lane's segment sum, plus the
    // run's carry if no lower lane holds a head
    float inflow = dpp_or_zero<0x138, 0xF>(v);                          // wave_shr:1
    const bool head_before = (hmask & ((1ull << lane) - 1ull)) != 0;
    if (!head_before) inflow += st.carry;

    const float total = inflow + lead;            // the row this lane's first head closes
    int first_lane = -1;
    if (st.heads == 0 && hmask != 0) {
        // first head of the whole run: what precedes it belongs to a row that began in an
        // earlier worker's run (or to nothing, if the run starts on a head)
        first_lane = __builtin_amdgcn_readfirstlane(__builtin_ctzll(hmask));
        st.lead = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, total), first_lane));
    }
    if (has && lane != first_lane) store_row(a, st.rank + heads_before, total);

    const float last = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
    st.carry = (hmask ? 0.0f : st.carry) + last;
    st.rank += heads_total;
    st.heads += heads_total;
}

// Cross-workgroup carry chain (a row whose groups are spread over wavefronts of more than
// one workgroup).  Every holder of a piece publishes its record with device-scope stores,
// then reports to the chain's counter; the last one to report adds the pieces in worker
// order (so the sum does not depend on arrival order) and writes the row.  All accesses to
// the records and counters are device-scope atomics, ordered by program order plus a wait
// for the stores to complete -- no cache write-back or invalidate is needed.
__device__ __forceinline__ void chain_arrive(const GemvArgs& a, int first)
{
    const int4 head_info = a.wave_info[first];
    const int len = head_info.w;
    const int old = __hip_atomic_fetch_add(&a.counters[first], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old != len - 1) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const int heads0 = __hip_atomic_load(&a.carry[first].heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    float sum = __hip_atomic_load(&a.carry[first].tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int b = first + 1; b < first + len; ++b) {
        const int hb = __hip_atomic_load(&a.carry[b].heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float piece = hb == 0
            ? __hip_atomic_load(&a.carry[b].tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)   // whole run
            : __hip_atomic_load(&a.carry[b].lead, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // up to its first head
        sum += piece;
    }
    store_row(a, head_info.x + heads0, sum);
    __hip_atomic_store(&a.counters[first], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
}

// What a wavefront tells its workgroup about the rows it shares with its neighbours.
struct LdsRecord {
    float lead;
    float tail;
    int heads;
    int chain_len;
};

template <int BITS>
__global__ __launch_bounds__(kWavesPerWorkgroup * kLanes) void gqsa_gemv_kernel(GemvArgs a)
{
    extern __shared__ __align__(16) uint8_t lds[];
    uint4* x_lo = reinterpret_cast<uint4*>(lds);          // elements 0..7 of every group-column
    uint4* x_hi = x_lo + a.kg;                            // elements 8..15
    float* x_sum = reinterpret_cast<float*>(x_hi + a.kg); // sum of the 16 activations
    __shared__ LdsRecord rec[kWavesPerWorkgroup];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wpw = blockDim.x >> 6;
    const int wl = tid >> 6;
    const int wg = blockIdx.x;
    const int wave = wg * wpw + wl;
    constexpr int BB = (16 * BITS / 8 + 6) * kLanes;

    // this worker's run of blocks: the blocks are dealt evenly to the workgroups, a
    // workgroup's blocks evenly to its wavefronts (contiguous runs, equal counts)
    long long left;
    const uint8_t* p;
    {
        const long long per_wg = a.n_blocks / gridDim.x;
        const int extra_wg = static_cast<int>(a.n_blocks % gridDim.x);
        const long long in_wg = per_wg + (wg < extra_wg ? 1 : 0);
        const long long wg_first = per_wg * wg + (wg < extra_wg ? wg : extra_wg);
        const long long per_wave = in_wg / wpw;
        const int extra_wave = static_cast<int>(in_wg % wpw);
        left = per_wave + (wl < extra_wave ? 1 : 0);
        p = a.blocks + static_cast<size_t>(wg_first + per_wave * wl + (wl < extra_wave ? wl : extra_wave)) * BB;
    }
    auto next_size = [](long long n) { return n >= 4 ? 4 : (n >= 2 ? 2 : static_cast<int>(n)); };

    // issue the loads of x first and of the first superblock right behind them, so that the
    // weights are already on their way while x is staged in LDS
    auto stage = [&](int c, uint4 lo, uint4 hi) {
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
    };
    uint4 lo0 = {0, 0, 0, 0}, hi0 = {0, 0, 0, 0};
    if (tid < a.kg) {
        const uint4* src = reinterpret_cast<const uint4*>(a.x + static_cast<size_t>(tid) * 16);
        lo0 = src[0];
        hi0 = src[1];
    }
    Tile<BITS> cur, nxt;
    int u_cur = next_size(left);
    const bool active = u_cur > 0;
    load_tile<BITS>(cur, p, u_cur, lane);
    const int4 info = a.wave_info[wave];   // a worker without blocks may still sit inside a row
    if (tid < a.kg) stage(tid, lo0, hi0);
    for (int c = tid + blockDim.x; c < a.kg; c += blockDim.x) {
        const uint4* src = reinterpret_cast<const uint4*>(a.x + static_cast<size_t>(c) * 16);
        stage(c, src[0], src[1]);
    }
    // rows without stored groups: exactly +0
    for (int i = blockIdx.x * blockDim.x + tid; i < a.n_empty; i += gridDim.x * blockDim.x)
        a.y[a.empty_rows[i]] = 0;
    __syncthreads();

    WaveState st{0.0f, 0.0f, info.x, 0};
    if (active) {
        for (;;) {
            left -= u_cur;
            const uint8_t* p_next = p + static_cast<size_t>(u_cur) * BB;
            const int u_next = next_size(left);
            load_tile<BITS>(nxt, p_next, u_next, lane);   // next superblock in flight during this one
            if (u_cur == 4) compute_tile<BITS, 4>(a, cur, lane, x_lo, x_hi, x_sum, st);
            else if (u_cur == 2) compute_tile<BITS, 2>(a, cur, lane, x_lo, x_hi, x_sum, st);
            else compute_tile<BITS, 1>(a, cur, lane, x_lo, x_hi, x_sum, st);
            if (u_next == 0) break;
            cur = nxt;
            u_cur = u_next;
            p = p_next;
        }
    }

    // Carry fix-up for the rows this run shares with its neighbours.  Inside a workgroup the
    // pieces meet in LDS; only rows spread over several workgroups go through device memory.
    if (lane == 0) rec[wl] = LdsRecord{st.lead, st.carry, st.heads, info.w};
    __syncthreads();
    if (lane != 0) return;

    if (info.y != 0 && st.heads > 0) store_row(a, st.rank, st.carry);   // last row ends with the run
    bool global_tail = false, global_lead = false;
    if (info.w > 0) {                         // this worker holds the head of a row that continues
        if (wl + info.w <= wpw) {
            float sum = st.carry;
            for (int b = wl + 1; b < wl + info.w; ++b) sum += rec[b].heads == 0 ? rec[b].tail : rec[b].lead;
            store_row(a, st.rank, sum);
        } else {
            global_tail = true;
        }
    }
    if (info.z >= 0) {                        // its first groups continue a row of an earlier worker
        const int fl = info.z - wg * wpw;     // that worker's index in this workgroup (if >= 0)
        global_lead = fl < 0 || fl + rec[fl < 0 ? 0 : fl].chain_len > wpw;
    }
    if (global_tail || global_lead) {
        __hip_atomic_store(&a.carry[wave].lead, st.lead, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&a.carry[wave].tail, st.carry, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&a.carry[wave].heads, st.heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // the stores have completed
        if (global_lead) chain_arrive(a, info.z);
        if (global_tail) chain_arrive(a, wave);
    }
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
    // carry records followed by one arrival counter per worker (zero between calls)
    const size_t carry_bytes = static_cast<size_t>(m->n_waves) * (sizeof(CarryRecord) + sizeof(int));
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
    a.wave_info = reinterpret_cast<const int4*>(img + m->map.wave_info);
    a.row_of_rank = m->n_empty ? reinterpret_cast<const int32_t*>(img + m->map.row_of_rank) : nullptr;
    a.empty_rows = reinterpret_cast<const int32_t*>(img + m->map.empty_rows);
    a.carry = static_cast<CarryRecord*>(m->d_carry);
    a.counters = reinterpret_cast<int*>(a.carry + m->n_waves);
    a.n_blocks = m->n_blocks;
    a.n_waves = m->n_waves;
    a.n_empty = static_cast<int>(m->n_empty);
    a.n_ranks = static_cast<int>(m->N - m->n_empty);
    a.kg = static_cast<int>(m->K / m->G);

    const int threads = m->waves_per_workgroup * kLanes;
    const int grid = m->n_workgroups;
    const size_t lds = static_cast<size_t>(a.kg) * 36;
    for (int b = 0; b < batch; ++b) {
        a.x = static_cast<const uint16_t*>(x) + static_cast<size_t>(b) * m->K;
        a.y = static_cast<uint16_t*>(y) + static_cast<size_t>(b) * m->N;
        if (m->bits == 4)
            hipLaunchKernelGGL(gqsa_gemv_kernel<4>, dim3(grid), dim3(threads), lds, s, a);
        else
            hipLaunchKernelGGL(gqsa_gemv_kernel<8>, dim3(grid), dim3(threads), lds, s, a);
    }
    GQSA_HIP(hipGetLastError());
    return GQSA_OK;
}

}  // namespace gqsa
