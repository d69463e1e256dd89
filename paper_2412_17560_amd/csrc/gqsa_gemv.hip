// Device side of libgqsa for gfx950 (MI355X): the GQSA decode GEMV  y = W^ x  over the
// block-sparse, group-quantised storage of the paper's GQS layer (Sec. 3.2), i.e. the
// operator flow of Sec. 3.5 / Fig. 4 -- stream the compressed groups, fetch the activation
// group named by each stored group's real group index, dequantise in registers (Eq. 3),
// multiply-accumulate, write back -- with the work split "task-centric" (Sec. 3.5, Fig. 5):
// every wavefront owns an equal, contiguous count of stored groups regardless of row
// boundaries, reduces them with a segmented wavefront scan, and settles the rows it shares
// with its neighbours in a carry fix-up at the end of the same kernel.
//
// Wavefront = 64 lanes.  A block is 64 stored groups, one per lane, so that every load is
// one fully coalesced instruction; in a superblock of U blocks lane l owns the U
// consecutive stream positions U*l .. U*l+U-1, sums them serially and takes part in ONE
// cross-lane segmented scan per superblock.
//
// Small batches: the kernel is compiled for NB = 1, 2, 4, 8 activation rows per launch; each
// decoded group is multiplied with all NB rows (weights are read and dequantised once).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#include "gqsa_internal.hpp"

namespace gqsa {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kMaxRowsPerLaunch = 8;      // NB values compiled: 1, 2, 4, 8
constexpr int kMaxLdsBytes = 160 * 1024;  // LDS of one gfx950 compute unit

struct GemvArgs {
    const uint8_t* blocks;
    const int4* wave_info;       // {rank_base, tail_closed, lead_first, chain_len} per worker
    const int32_t* row_of_rank;  // row index of the r-th non-empty row (nullptr: identity)
    const int32_t* empty_rows;
    CarryRecord* carry;          // [worker][kMaxRowsPerLaunch]
    int* counters;               // arrivals per carry chain, indexed by the chain's first worker
    const uint16_t* x;           // fp16 [NB][K]
    uint16_t* y;                 // fp16 [NB][N]
    long long N, K;
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

// (w & mask) | splice in one instruction; mask is wave-uniform, splice sits in a vector register
// (the three-operand form takes a single scalar operand).
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t splice)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask), "v"(splice));
    return r;
}

// The 16 codes of one stored group as eight fp16 pairs (element 2i, 2i+1), exact.
struct Codes {
    half2_t q[8];
};

// 4-bit: the code words are nibble-permuted at pack time (element 2m at bits 4m, element 2m+1
// at bits 16+4m), so one AND-OR splices a pair of codes into the mantissas of the fp16 pair
// (1024+q, 1024+q') or (1024+16q, 1024+16q'); one packed op removes the bias exactly.
__device__ __forceinline__ void decode_w4(const GemvArgs& a, uint32_t w, half2_t* q)
{
    const half2_t k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
    const half2_t k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t k64 = {(_Float16)64.0f, (_Float16)64.0f};
    const uint32_t w2 = w >> 8;
    q[0] = as_half2(and_or(w, a.nib_lo, a.k1024x2)) - k1024;
    q[1] = as_half2(and_or(w, a.nib_hi, a.k1024x2)) * k16th - k64;
    q[2] = as_half2(and_or(w2, a.nib_lo, a.k1024x2)) - k1024;
    q[3] = as_half2(and_or(w2, a.nib_hi, a.k1024x2)) * k16th - k64;
}

// 8-bit: a byte permute drops each code (bytes of w, element order) into the mantissa of
// 1024.0 (0x64xx), one packed subtract removes the bias.
__device__ __forceinline__ void decode_w8(uint32_t w, half2_t* q)
{
    const half2_t k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
    const uint32_t k64s = 0x64646464u;
    q[0] = as_half2(__builtin_amdgcn_perm(w, k64s, 0x00050004u)) - k1024;
    q[1] = as_half2(__builtin_amdgcn_perm(w, k64s, 0x00070006u)) - k1024;
}

__device__ __forceinline__ float dot16(const Codes& c, uint4 xl, uint4 xh)
{
    float d = 0.0f;
    d = __builtin_amdgcn_fdot2(c.q[0], as_half2(xl.x), d, false);
    d = __builtin_amdgcn_fdot2(c.q[1], as_half2(xl.y), d, false);
    d = __builtin_amdgcn_fdot2(c.q[2], as_half2(xl.z), d, false);
    d = __builtin_amdgcn_fdot2(c.q[3], as_half2(xl.w), d, false);
    d = __builtin_amdgcn_fdot2(c.q[4], as_half2(xh.x), d, false);
    d = __builtin_amdgcn_fdot2(c.q[5], as_half2(xh.y), d, false);
    d = __builtin_amdgcn_fdot2(c.q[6], as_half2(xh.z), d, false);
    d = __builtin_amdgcn_fdot2(c.q[7], as_half2(xh.w), d, false);
    return d;
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

__device__ __forceinline__ float read_lane(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

template <int NB>
struct WaveState {
    float carry[NB];   // per activation row: sum of the groups since the last row head
    float lead[NB];    // sum of the groups before the run's first row head
    int rank;          // rank (among non-empty rows) of the row that is open now
    int heads;         // row heads seen so far in this worker's run
};

__device__ __forceinline__ void store_row(const GemvArgs& a, int b, int rank, float v)
{
    if (static_cast<unsigned>(rank) >= static_cast<unsigned>(a.n_ranks)) return;  // never for a valid image
    const int row = a.row_of_rank ? a.row_of_rank[rank] : rank;
    a.y[b * a.N + row] = float_to_half_bits(v);
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

// x in LDS, per activation row: three arrays of 16-byte slots indexed by group-column --
// elements 0..7, elements 8..15 and (first 4 bytes) the fp32 sum of the 16 -- KGP slots
// apart, so that one address register plus immediate offsets serves all reads of a gather, and
// a gather of 16 B per lane spreads over all banks.  Row b starts at b * 48 * KGP.
template <int BITS, int KGP, int U, int NB>
__device__ __forceinline__ void compute_tile(const GemvArgs& a, const Tile<BITS>& t, int lane,
                                             const uint8_t* xlds, WaveState<NB>& st)
{
    uint32_t head_bits = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) head_bits |= (t.ix[u] & 1u) << u;   // index word = column << 4 | head
    const bool has = head_bits != 0;
    const unsigned long long hmask = __ballot(has);
    // no lane holds two heads (no row shorter than U groups here): branch-free serial sums
    const bool simple = __ballot((head_bits & (head_bits - 1u)) != 0) == 0;
    int heads_before = 0;   // row heads of this superblock in lower lanes
    int heads_total = 0;
    if (simple) {
        heads_before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(hmask >> 32),
                       __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(hmask), 0));
        heads_total = __popcll(hmask);
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long bal = __ballot((head_bits >> u) & 1u);
            heads_before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(bal >> 32),
                           __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(bal), heads_before));
            heads_total += __popcll(bal);
        }
    }

    // (2)-(4) gather the activation group by real group index, dequantise, multiply:
    //   sum_j (q_j - z) s x_j  =  s * (sum_j q_j x_j  -  z * sum_j x_j)
    // (5a) and add serially over the lane's U consecutive groups: lead = what precedes the
    // lane's first row head, acc = what follows its last one (everything, if it has none)
    float acc[NB], lead[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) { acc[b] = 0.0f; lead[b] = 0.0f; }
    int nh = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        Codes c;
        if constexpr (BITS == 4) {
            decode_w4(a, t.code[u][0], &c.q[0]);
            decode_w4(a, t.code[u][1], &c.q[4]);
        } else {
            decode_w8(t.code[u][0], &c.q[0]);
            decode_w8(t.code[u][1], &c.q[2]);
            decode_w8(t.code[u][2], &c.q[4]);
            decode_w8(t.code[u][3], &c.q[6]);
        }
        const float s = half_to_float(t.sz[u] & 0xFFFFu);
        const float z = half_to_float(t.sz[u] >> 16);
        const uint8_t* xg = xlds + (t.ix[u] & 0xFFF0u);
        float dotz[NB];   // sum_j q_j x_j - z sum_j x_j; times s it is the group's contribution
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const uint8_t* xb = xg + b * (48 * KGP);
            const uint4 xl = *reinterpret_cast<const uint4*>(xb);
            const uint4 xh = *reinterpret_cast<const uint4*>(xb + 16 * KGP);
            const float xs = *reinterpret_cast<const float*>(xb + 32 * KGP);
            dotz[b] = __builtin_fmaf(-z, xs, dot16(c, xl, xh));
        }
        const bool head_here = (head_bits >> u) & 1u;
        if (simple) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                lead[b] = head_here ? acc[b] : lead[b];     // the only head of this lane
                acc[b] = __builtin_fmaf(s, dotz[b], head_here ? 0.0f : acc[b]);
            }
        } else {
            if (head_here) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    if (nh == 0) lead[b] = acc[b];
                    else store_row(a, b, st.rank + heads_before + nh, acc[b]);   // a whole row inside one lane
                    acc[b] = 0.0f;
                }
                ++nh;
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[b] = __builtin_fmaf(s, dotz[b], acc[b]);
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
    // the run's carry flows into the lanes up to and including the first one that holds a head
    const unsigned long long upto_first = hmask ? (hmask ^ (hmask - 1ull)) : ~0ull;
    // first head of the whole run: what precedes it belongs to a row that began in an earlier
    // worker's run (or to nothing, if the run starts on a head)
    int first_lane = -1;
    if (st.heads == 0 && hmask != 0) first_lane = __builtin_amdgcn_readfirstlane(__builtin_ctzll(hmask));

#pragma unroll
    for (int b = 0; b < NB; ++b) {
        float v = acc[b];
        v += keep_lanes(~p1, dpp_or_zero<0x111, 0xF>(v));       // row_shr:1
        v += keep_lanes(~p2, dpp_or_zero<0x112, 0xF>(v));       // row_shr:2
        v += keep_lanes(~p4, dpp_or_zero<0x114, 0xF>(v));       // row_shr:4
        v += keep_lanes(~p8, dpp_or_zero<0x118, 0xF>(v));       // row_shr:8
        v += keep_lanes(~p16, dpp_or_zero<0x142, 0xA>(v));      // row_bcast:15
        v += keep_lanes(open31, dpp_or_zero<0x143, 0xC>(v));    // row_bcast:31
        // sum flowing into this lane from the left: the previous lane's segment sum (+ carry)
        const float inflow = dpp_or_zero<0x138, 0xF>(v) + keep_lanes(upto_first, st.carry[b]);   // wave_shr:1
        const float total = inflow + lead[b];       // the row this lane's first head closes
        if (first_lane >= 0) st.lead[b] = read_lane(total, first_lane);
        if (has && lane != first_lane) store_row(a, b, st.rank + heads_before, total);
        st.carry[b] = (hmask ? 0.0f : st.carry[b]) + read_lane(v, 63);
    }
    st.rank += heads_total;
    st.heads += heads_total;
}

// Cross-workgroup carry chain (a row whose groups are spread over wavefronts of more than
// one workgroup).  Every holder of a piece publishes its record with device-scope stores,
// then reports to the chain's counter; the last one to report adds the pieces in worker
// order (so the sum does not depend on arrival order) and writes the row.  All accesses to
// the records and counters are device-scope atomics, ordered by program order plus a wait
// for the stores to complete -- no cache write-back or invalidate is needed.
template <int NB>
__device__ __forceinline__ void chain_arrive(const GemvArgs& a, int first)
{
    const int4 head_info = a.wave_info[first];
    const int len = head_info.w;
    const int old = __hip_atomic_fetch_add(&a.counters[first], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old != len - 1) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    for (int b = 0; b < NB; ++b) {
        const CarryRecord* r0 = &a.carry[first * kMaxRowsPerLaunch + b];
        const int heads0 = __hip_atomic_load(&r0->heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        float sum = __hip_atomic_load(&r0->tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int w = first + 1; w < first + len; ++w) {
            const CarryRecord* r = &a.carry[w * kMaxRowsPerLaunch + b];
            const int hw = __hip_atomic_load(&r->heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sum += hw == 0 ? __hip_atomic_load(&r->tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)    // whole run
                           : __hip_atomic_load(&r->lead, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // up to its first head
        }
        store_row(a, b, head_info.x + heads0, sum);
    }
    __hip_atomic_store(&a.counters[first], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
}

// What a wavefront tells its workgroup about the rows it shares with its neighbours.
struct LdsSums {
    float lead;
    float tail;
};
struct LdsCounts {
    int heads;
    int chain_len;
};

template <int BITS, int KGP, int NB>
__global__ __launch_bounds__(kWavesPerWorkgroup * kLanes) void gqsa_gemv_kernel(GemvArgs a)
{
    // x arrays (NB * 48 * KGP bytes), then the wavefronts' records
    extern __shared__ __align__(16) uint8_t xlds[];
    LdsCounts* rec_n = reinterpret_cast<LdsCounts*>(xlds + NB * 48 * KGP);
    LdsSums* rec_s = reinterpret_cast<LdsSums*>(rec_n + kWavesPerWorkgroup);   // [wavefront][NB]

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
    auto stage = [&](int c, uint4 lo, uint4 hi) {   // c = slot over all rows: b * kg + column
        const int b = NB == 1 ? 0 : c / a.kg;
        uint8_t* slot = xlds + b * (48 * KGP) + (c - b * a.kg) * 16;
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
    const int n_slots = NB * a.kg;                  // x is [NB][K] contiguous: slot c holds x[16c .. 16c+15]
    uint4 lo0 = {0, 0, 0, 0}, hi0 = {0, 0, 0, 0};
    if (tid < n_slots) {
        const uint4* src = reinterpret_cast<const uint4*>(a.x + static_cast<size_t>(tid) * 16);
        lo0 = src[0];
        hi0 = src[1];
    }
    Tile<BITS> cur, nxt;
    int u_cur = next_size(left);
    const bool active = u_cur > 0;
    load_tile<BITS>(cur, p, u_cur, lane);
    const int4 info = a.wave_info[wave];   // a worker without blocks may still sit inside a row
    if (tid < n_slots) stage(tid, lo0, hi0);
    for (int c = tid + blockDim.x; c < n_slots; c += blockDim.x) {
        const uint4* src = reinterpret_cast<const uint4*>(a.x + static_cast<size_t>(c) * 16);
        stage(c, src[0], src[1]);
    }
    // rows without stored groups: exactly +0
    for (int i = blockIdx.x * blockDim.x + tid; i < a.n_empty; i += gridDim.x * blockDim.x) {
        const int row = a.empty_rows[i];
#pragma unroll
        for (int b = 0; b < NB; ++b) a.y[b * a.N + row] = 0;
    }
    __syncthreads();

    WaveState<NB> st;
#pragma unroll
    for (int b = 0; b < NB; ++b) { st.carry[b] = 0.0f; st.lead[b] = 0.0f; }
    st.rank = info.x;
    st.heads = 0;
    if (active) {
        for (;;) {
            left -= u_cur;
            const uint8_t* p_next = p + u_cur * BB;
            const int u_next = next_size(left);
            load_tile<BITS>(nxt, p_next, u_next, lane);   // next superblock in flight during this one
            if (u_cur == 4) compute_tile<BITS, KGP, 4, NB>(a, cur, lane, xlds, st);
            else if (u_cur == 2) compute_tile<BITS, KGP, 2, NB>(a, cur, lane, xlds, st);
            else compute_tile<BITS, KGP, 1, NB>(a, cur, lane, xlds, st);
            if (u_next == 0) break;
            cur = nxt;
            u_cur = u_next;
            p = p_next;
        }
    }

    // Carry fix-up for the rows this run shares with its neighbours.  Inside a workgroup the
    // pieces meet in LDS; only rows spread over several workgroups go through device memory.
    if (lane == 0) {
        rec_n[wl] = LdsCounts{st.heads, info.w};
#pragma unroll
        for (int b = 0; b < NB; ++b) rec_s[wl * NB + b] = LdsSums{st.lead[b], st.carry[b]};
    }
    __syncthreads();
    if (lane != 0) return;

    if (info.y != 0 && st.heads > 0) {        // last row ends with the run
#pragma unroll
        for (int b = 0; b < NB; ++b) store_row(a, b, st.rank, st.carry[b]);
    }
    bool global_tail = false, global_lead = false;
    if (info.w > 0) {                         // this worker holds the head of a row that continues
        if (wl + info.w <= wpw) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float sum = st.carry[b];
                for (int w = wl + 1; w < wl + info.w; ++w)
                    sum += rec_n[w].heads == 0 ? rec_s[w * NB + b].tail : rec_s[w * NB + b].lead;
                store_row(a, b, st.rank, sum);
            }
        } else {
            global_tail = true;
        }
    }
    if (info.z >= 0) {                        // its first groups continue a row of an earlier worker
        const int fl = info.z - wg * wpw;     // that worker's index in this workgroup (if >= 0)
        global_lead = fl < 0 || fl + rec_n[fl < 0 ? 0 : fl].chain_len > wpw;
    }
    if (global_tail || global_lead) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            CarryRecord* r = &a.carry[wave * kMaxRowsPerLaunch + b];
            __hip_atomic_store(&r->lead, st.lead[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&r->tail, st.carry[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&r->heads, st.heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // the stores have completed
        if (global_lead) chain_arrive<NB>(a, info.z);
        if (global_tail) chain_arrive<NB>(a, wave);
    }
}

using KernelFn = void (*)(GemvArgs);

constexpr size_t lds_bytes(int kgp, int nb)
{
    return static_cast<size_t>(nb) * 48 * kgp + kWavesPerWorkgroup * (sizeof(LdsCounts) + nb * sizeof(LdsSums));
}

template <int BITS, int KGP, int NB>
KernelFn kernel_if_it_fits()
{
    if constexpr (lds_bytes(KGP, NB) <= kMaxLdsBytes) return gqsa_gemv_kernel<BITS, KGP, NB>;
    else return nullptr;
}

template <int BITS, int KGP>
KernelFn pick_rows(int nb)
{
    switch (nb) {
        case 1: return kernel_if_it_fits<BITS, KGP, 1>();
        case 2: return kernel_if_it_fits<BITS, KGP, 2>();
        case 4: return kernel_if_it_fits<BITS, KGP, 4>();
        case 8: return kernel_if_it_fits<BITS, KGP, 8>();
    }
    return nullptr;
}

// The kernel is compiled for group-column counts rounded up to a power of two (the LDS
// offsets between the x arrays are immediates) and for 1, 2, 4 or 8 activation rows per
// launch, as far as NB copies of x fit the 160 KB of LDS.
template <int BITS>
KernelFn pick_kernel(int kg, int nb, int* kgp)
{
    if (kg <= 256) { *kgp = 256; return pick_rows<BITS, 256>(nb); }
    if (kg <= 512) { *kgp = 512; return pick_rows<BITS, 512>(nb); }
    if (kg <= 1024) { *kgp = 1024; return pick_rows<BITS, 1024>(nb); }
    if (kg <= 2048) { *kgp = 2048; return pick_rows<BITS, 2048>(nb); }
    *kgp = 0;
    return nullptr;
}

KernelFn pick(const gqsa_matrix* m, int nb, int* kgp)
{
    const int kg = static_cast<int>(m->K / m->G);
    return m->bits == 4 ? pick_kernel<4>(kg, nb, kgp) : pick_kernel<8>(kg, nb, kgp);
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
    if (!pick(m, 1, &kgp)) return GQSA_ERR_UNSUPPORTED;      // K/G above 2048: x does not fit the LDS layout
    int dev = 0;
    GQSA_HIP(hipGetDevice(&dev));
    for (int nb = 1; nb <= kMaxRowsPerLaunch; nb *= 2) {
        KernelFn fn = pick(m, nb, &kgp);
        if (fn && lds_bytes(kgp, nb) > 64 * 1024)
            GQSA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         static_cast<int>(lds_bytes(kgp, nb))));
    }
    void* img = nullptr;
    void* carry = nullptr;
    GQSA_HIP(hipMalloc(&img, m->image.size()));
    // carry records (per worker and activation row) followed by one arrival counter per worker
    const size_t carry_bytes = static_cast<size_t>(m->n_waves) *
                               (kMaxRowsPerLaunch * sizeof(CarryRecord) + sizeof(int));
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
    a.counters = reinterpret_cast<int*>(a.carry + static_cast<size_t>(m->n_waves) * kMaxRowsPerLaunch);
    a.N = m->N;
    a.K = m->K;
    a.per_wg = static_cast<int>(m->n_blocks / m->n_workgroups);
    a.extra_wg = static_cast<int>(m->n_blocks % m->n_workgroups);
    a.n_empty = static_cast<int>(m->n_empty);
    a.n_ranks = static_cast<int>(m->N - m->n_empty);
    a.kg = static_cast<int>(m->K / m->G);
    a.nib_lo = 0x000F000Fu;
    a.nib_hi = 0x00F000F0u;
    a.k1024x2 = 0x64006400u;

    const int threads = m->waves_per_workgroup * kLanes;
    const int grid = m->n_workgroups;
    // the batch goes out in launches of 8, 4, 2 or 1 rows: the most that fits LDS and is left
    int done = 0;
    while (done < batch) {
        int nb = kMaxRowsPerLaunch, kgp = 0;
        KernelFn fn = nullptr;
        for (; nb >= 1; nb /= 2) {
            if (nb > batch - done) continue;
            fn = pick(m, nb, &kgp);
            if (fn) break;
        }
        if (!fn) return GQSA_ERR_UNSUPPORTED;
        a.x = static_cast<const uint16_t*>(x) + static_cast<size_t>(done) * m->K;
        a.y = static_cast<uint16_t*>(y) + static_cast<size_t>(done) * m->N;
        hipLaunchKernelGGL(fn, dim3(grid), dim3(threads), lds_bytes(kgp, nb), s, a);
        done += nb;
    }
    GQSA_HIP(hipGetLastError());
    return GQSA_OK;
}

}  // namespace gqsa
