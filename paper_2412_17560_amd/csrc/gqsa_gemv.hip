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
    int per_wg;                  // blocks per workgroup (the first extra_wg workgroups hold one more)
    int extra_wg;
    int n_empty;
    int n_ranks;                 // non-empty rows
    int kg;                      // group-columns K/G
    // nibble masks and the fp16 pair (1024, 1024); passed in registers so that mask-and-splice
    // is one three-operand instruction instead of two with literal operands
    uint32_t nib_lo, nib_hi, k1024x2;
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
// (w & mask) | splice in one instruction; mask is wave-uniform, splice sits in a vector register
// (the three-operand form takes a single scalar operand).
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t splice)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask), "v"(splice));
    return r;
}

__device__ __forceinline__ float dot8_w4(const GemvArgs& a, uint32_t w, uint4 x, float acc)
{
    const half2_t k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
    const half2_t k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t k64 = {(_Float16)64.0f, (_Float16)64.0f};
    const uint32_t w2 = w >> 8;
    half2_t q0 = as_half2(and_or(w, a.nib_lo, a.k1024x2)) - k1024;
    half2_t q1 = as_half2(and_or(w, a.nib_hi, a.k1024x2)) * k16th - k64;
    half2_t q2 = as_half2(and_or(w2, a.nib_lo, a.k1024x2)) - k1024;
    half2_t q3 = as_half2(and_or(w2, a.nib_hi, a.k1024x2)) * k16th - k64;
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

// v from the lane CTRL names (DPP); lanes whose source lane does not exist, or whose row is
// not in ROW_MASK, read 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or_zero(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL,
                                                                 ROW_MASK, 0xF, ROW_MASK == 0xF));
}

// t in the lanes whose bit is set in the wave-uniform mask, 0 elsewhere: one select that takes
// the lane mask straight from a scalar register pair (the masks are made with scalar ops).
__device__ __forceinline__ float keep_lanes(unsigned long long mask, float t)
{
    float r;
    asm("v_cndmask_b32_e64 %0, 0, %1, %2" : "=v"(r) : "v"(t), "s"(mask));
    return r;
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

// (1) stream the compressed groups: coalesced loads, all issued before anything waits.  The
// block pointer is wave-uniform (scalar base), the lane supplies a 32-bit byte offset.
template <typename T>
__device__ __forceinline__ T load_at(const uint8_t* base, uint32_t byte_offset)
{
    return *reinterpret_cast<const T*>(base + byte_offset);
}

template <int BITS>
__device__ __forceinline__ void load_tile(Tile<BITS>& t, const uint8_t* p, int U, int lane)
{
    constexpr int CB = 16 * BITS / 8;                 // code bytes per group
    constexpr int BB = (CB + 6) * kLanes;             // block bytes
    const uint32_t ulane = static_cast<uint32_t>(lane);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (u < U) {
            if constexpr (BITS == 4) {
                const uint2 c = load_at<uint2>(p, ulane * 8u + u * BB);
                t.code[u][0] = c.x; t.code[u][1] = c.y;
            } else {
                const uint4 c = load_at<uint4>(p, ulane * 16u + u * BB);
                t.code[u][0] = c.x; t.code[u][1] = c.y; t.code[u][2] = c.z; t.code[u][3] = c.w;
            }
            t.sz[u] = load_at<uint32_t>(p, ulane * 4u + (u * BB + CB * kLanes));
            t.ix[u] = load_at<uint16_t>(p, ulane * 2u + (u * BB + (CB + 4) * kLanes));
        }
    }
}

// x in LDS: three arrays of 16-byte slots indexed by group-column -- elements 0..7, elements
// 8..15 and (first 4 bytes) the fp32 sum of the 16 -- KGP slots apart, so that one address
// register plus immediate offsets serves all three reads of a gather, and a gather of 16 B
// per lane spreads over all banks.
template <int BITS, int KGP, int U>
__device__ __forceinline__ void compute_tile(const GemvArgs& a, const Tile<BITS>& t, int lane,
                                             const uint8_t* xlds, WaveState& st)
{
    // (2)-(4) gather the activation group by real group index, dequantise, multiply:
    //   sum_j (q_j - z) s x_j  =  s * (sum_j q_j x_j  -  z * sum_j x_j)
    float part[U];
    uint32_t head_bits = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint8_t* xg = xlds + (t.ix[u] & 0xFFF0u);      // index word = column << 4 | head
        const uint4 xl = *reinterpret_cast<const uint4*>(xg);
        const uint4 xh = *reinterpret_cast<const uint4*>(xg + 16 * KGP);
        const float xs = *reinterpret_cast<const float*>(xg + 32 * KGP);
        float d = 0.0f;
        if constexpr (BITS == 4) {
            d = dot8_w4(a, t.code[u][0], xl, d);
            d = dot8_w4(a, t.code[u][1], xh, d);
        } else {
            d = dot4_w8(t.code[u][0], xl.x, xl.y, d);
            d = dot4_w8(t.code[u][1], xl.z, xl.w, d);
            d = dot4_w8(t.code[u][2], xh.x, xh.y, d);
            d = dot4_w8(t.code[u][3], xh.z, xh.w, d);
        }
        const float s = half_to_float(t.sz[u] & 0xFFFFu);
        const float z = half_to_float(t.sz[u] >> 16);
        part[u] = s * __builtin_fmaf(-z, xs, d);
        head_bits |= (t.ix[u] & 1u) << u;
    }

    // (5a) serial segmented sum over the lane's U consecutive groups: lead = what precedes the
    // lane's first row head, acc = what follows its last one (everything, if it has none)
    const bool has = head_bits != 0;
    const unsigned long long hmask = __ballot(has);
    float acc = 0.0f, lead = 0.0f;
    int heads_before;   // row heads of this superblock in lower lanes
    int heads_total;
    if (__ballot((head_bits & (head_bits - 1u)) != 0) == 0) {
        // no lane holds two heads (rows are not shorter than U groups here): branch-free
        heads_before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(hmask >> 32),
                       __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(hmask), 0));
        heads_total = __popcll(hmask);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool before = (head_bits >> u) > 1u;      // the head comes later in this lane
            lead += before ? part[u] : 0.0f;
            acc += before ? 0.0f : part[u];
        }
    } else {
        heads_before = 0;
        heads_total = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long bal = __ballot((head_bits >> u) & 1u);
            heads_before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(bal >> 32),
                           __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(bal), heads_before));
            heads_total += __popcll(bal);
        }
        int nh = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (head_bits & (1u << u)) {
                if (nh == 0) lead = acc;
                else store_row(a, st.rank + heads_before + nh, acc);   // a whole row inside one lane
                acc = 0.0f;
                ++nh;
            }
            acc += part[u];
        }
    }

    // (5b) cross-lane segmented inclusive scan of the lanes' open sums: DPP shifts inside each
    // row of 16 lanes, then the row totals are handed on (lane 15 -> row 1, lane 47 -> row 3,
    // lane 31 -> rows 2 and 3).  A lane takes the value offered at distance d only if no lane
    // in between (itself included) starts a new segment; those lane sets are wave-uniform
    // masks, smeared from the head mask with scalar shifts that stay inside a row.
    const unsigned long long p1 = hmask;
    const unsigned long long p2 = p1 | ((p1 << 1) & 0xFFFEFFFEFFFEFFFEull);
    const unsigned long long p4 = p2 | ((p2 << 2) & 0xFFFCFFFCFFFCFFFCull);
    const unsigned long long p8 = p4 | ((p4 << 4) & 0xFFF0FFF0FFF0FFF0ull);
    const unsigned long long p16 = p8 | ((p8 << 8) & 0xFF00FF00FF00FF00ull);
    unsigned long long open31 = ~p16;                       // rows 2, 3 taking lane 31's total
    if ((hmask >> 32) & 0xFFFFull) open31 &= 0x0000FFFFFFFFFFFFull;   // a head in row 2 cuts row 3 off
    float v = acc;
    v += keep_lanes(~p1, dpp_or_zero<0x111, 0xF>(v));       // row_shr:1
    v += keep_lanes(~p2, dpp_or_zero<0x112, 0xF>(v));       // row_shr:2
    v += keep_lanes(~p4, dpp_or_zero<0x114, 0xF>(v));       // row_shr:4
    v += keep_lanes(~p8, dpp_or_zero<0x118, 0xF>(v));       // row_shr:8
    v += keep_lanes(~p16, dpp_or_zero<0x142, 0xA>(v));      // row_bcast:15
    v += keep_lanes(open31, dpp_or_zero<0x143, 0xC>(v));    // row_bcast:31
    // sum flowing into this lane from the left: the previous lane's segment sum, plus the
    // run's carry for the lanes up to and including the first one that holds a head
    const unsigned long long upto_first = hmask ? (hmask ^ (hmask - 1ull)) : ~0ull;
    const float inflow = dpp_or_zero<0x138, 0xF>(v) + keep_lanes(upto_first, st.carry);   // wave_shr:1

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

template <int BITS, int KGP>
__global__ __launch_bounds__(kWavesPerWorkgroup * kLanes) void gqsa_gemv_kernel(GemvArgs a)
{
    extern __shared__ __align__(16) uint8_t xlds[];      // x arrays (48*KGP bytes), then the records
    LdsRecord* rec = reinterpret_cast<LdsRecord*>(xlds + 48 * KGP);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wpw = blockDim.x >> 6;
    const int wl = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: scalar registers
    const int wg = blockIdx.x;
    const int wave = wg * wpw + wl;
    constexpr int BB = (16 * BITS / 8 + 6) * kLanes;

    // this worker's run of blocks: the blocks are dealt evenly to the workgroups, a
    // workgroup's blocks evenly to its wavefronts (contiguous runs, equal counts)
    const unsigned in_wg = a.per_wg + (wg < a.extra_wg ? 1 : 0);
    const unsigned wg_first = a.per_wg * wg + (wg < a.extra_wg ? wg : a.extra_wg);
    const unsigned per_wave = in_wg / static_cast<unsigned>(wpw);
    const unsigned extra_wave = in_wg - per_wave * wpw;
    int left = per_wave + (static_cast<unsigned>(wl) < extra_wave ? 1 : 0);
    const uint8_t* p = a.blocks + static_cast<size_t>(wg_first + per_wave * wl +
                                                      (static_cast<unsigned>(wl) < extra_wave ? wl : extra_wave)) * BB;
    auto next_size = [](int n) { return n >= 4 ? 4 : (n >= 2 ? 2 : n); };

    // issue the loads of x first and of the first superblock right behind them, so that the
    // weights are already on their way while x is staged in LDS
    auto stage = [&](int c, uint4 lo, uint4 hi) {
        uint8_t* slot = xlds + c * 16;
        *reinterpret_cast<uint4*>(slot) = lo;
        *reinterpret_cast<uint4*>(slot + 16 * KGP) = hi;
        const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            s += half_to_float(w[i] & 0xFFFFu);
            s += half_to_float(w[i] >> 16);
        }
        *reinterpret_cast<float*>(slot + 32 * KGP) = s;
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
            const uint8_t* p_next = p + u_cur * BB;
            const int u_next = next_size(left);
            load_tile<BITS>(nxt, p_next, u_next, lane);   // next superblock in flight during this one
            if (u_cur == 4) compute_tile<BITS, KGP, 4>(a, cur, lane, xlds, st);
            else if (u_cur == 2) compute_tile<BITS, KGP, 2>(a, cur, lane, xlds, st);
            else compute_tile<BITS, KGP, 1>(a, cur, lane, xlds, st);
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

using KernelFn = void (*)(GemvArgs);

// The kernel is compiled for group-column counts rounded up to a power of two (the LDS
// offsets between the three x arrays are immediates).
template <int BITS>
KernelFn pick_kernel(int kg, int* kgp)
{
    if (kg <= 256) { *kgp = 256; return gqsa_gemv_kernel<BITS, 256>; }
    if (kg <= 512) { *kgp = 512; return gqsa_gemv_kernel<BITS, 512>; }
    if (kg <= 1024) { *kgp = 1024; return gqsa_gemv_kernel<BITS, 1024>; }
    if (kg <= 2048) { *kgp = 2048; return gqsa_gemv_kernel<BITS, 2048>; }
    *kgp = 0;
    return nullptr;
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
    int kgp = 0;
    KernelFn fn = m->bits == 4 ? pick_kernel<4>(static_cast<int>(m->K / m->G), &kgp)
                               : pick_kernel<8>(static_cast<int>(m->K / m->G), &kgp);
    if (!fn) return GQSA_ERR_UNSUPPORTED;      // K/G above 2048: x does not fit the LDS layout
    int dev = 0;
    GQSA_HIP(hipGetDevice(&dev));
    const size_t lds = static_cast<size_t>(kgp) * 48 + kWavesPerWorkgroup * 16;
    if (lds > 64 * 1024)
        GQSA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
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
    a.per_wg = static_cast<int>(m->n_blocks / m->n_workgroups);
    a.extra_wg = static_cast<int>(m->n_blocks % m->n_workgroups);
    a.n_empty = static_cast<int>(m->n_empty);
    a.n_ranks = static_cast<int>(m->N - m->n_empty);
    a.kg = static_cast<int>(m->K / m->G);
    a.nib_lo = 0x000F000Fu;
    a.nib_hi = 0x00F000F0u;
    a.k1024x2 = 0x64006400u;

    int kgp = 0;
    KernelFn fn = m->bits == 4 ? pick_kernel<4>(a.kg, &kgp) : pick_kernel<8>(a.kg, &kgp);
    if (!fn) return GQSA_ERR_UNSUPPORTED;
    const int threads = m->waves_per_workgroup * kLanes;
    const int grid = m->n_workgroups;
    const size_t lds = static_cast<size_t>(kgp) * 48 + kWavesPerWorkgroup * 16;
    for (int b = 0; b < batch; ++b) {
        a.x = static_cast<const uint16_t*>(x) + static_cast<size_t>(b) * m->K;
        a.y = static_cast<uint16_t*>(y) + static_cast<size_t>(b) * m->N;
        hipLaunchKernelGGL(fn, dim3(grid), dim3(threads), lds, s, a);
    }
    GQSA_HIP(hipGetLastError());
    return GQSA_OK;
}

}  // namespace gqsa
