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

#include <cstddef>
#include <cstdint>
#include <cstdio>

#include "gqsa_internal.hpp"

namespace gqsa {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kMaxRowsPerLaunch = 8;      // NB values compiled: 1, 2, 4, 8
constexpr int kMaxLdsBytes = 160 * 1024;  // LDS of one gfx950 compute unit

constexpr int kMaxMatrices = 4;           // matrices sharing x that one launch can take

// One packed matrix as the kernel sees it, split by when it is needed.  What the first loads
// depend on (x, the first matrix's run, the slot count, the wavefronts per workgroup) is also
// passed as leading scalar kernel parameters, which arrive preloaded in scalar registers; the
// argument block below is read with scalar loads, a 64-byte line per round trip, while the first
// weights are on their way.
struct MatRun {                  // where a worker's run of blocks is (32 bytes)
    const uint8_t* blocks;
    int per_wg;                  // blocks per workgroup (the first extra_wg workgroups hold one more)
    int extra_wg;
    int per_wave[2];             // blocks per wavefront in a workgroup of per_wg (+1) blocks ...
    int extra_wave[2];           // ... of which the first extra_wave wavefronts hold one more
};

struct MatArgs {                 // where results go (64 bytes)
    const int32_t* row_of_rank;  // row index of the r-th non-empty row (nullptr: identity)
    const int32_t* empty_rows;
    CarryRecord* carry;          // [worker][kMaxRowsPerLaunch]
    int* counters;               // arrivals per carry chain, indexed by the chain's first worker
    unsigned long long* slots;   // [worker][kMaxRowsPerLaunch] meeting points of rows spread over two workgroups
    uint16_t* y;                 // fp16 [NB][N]
    long long N;
    int n_empty;
    int n_ranks;                 // non-empty rows
};

template <int NM>
struct GemvArgsT {
    // ---- first 64-byte line (x, kg, wpw and run[0] travel as scalar parameters as well)
    const uint16_t* x;           // fp16 [NB][K], shared by the matrices
    int n_mats;
    int kg;                      // 16-element activation slots K/16
    int wpw;                     // wavefronts per workgroup
    int pad0[3];
    MatRun run[NM];              // run[0] completes the first line
    // ---- later lines
    const int4* wave_info[NM];   // {rank_base, tail_closed + 2 * lead_len, lead_first, chain_len} per worker
    int n_wg;                    // workgroups
    int pad;
    MatArgs m[NM];
};
typedef GemvArgsT<kMaxMatrices> GemvArgs;     // what the host fills in; a launch passes the first NM
static_assert(offsetof(GemvArgs, run) == 32 && sizeof(MatRun) == 32, "the first matrix's run closes line 0");

// where the argument block sits in the kernel-argument segment: after the ten scalar parameters
constexpr int kArgsOffset = 48;

// run[i] / m[i] of the kernel's argument block for a wave-uniform i, read from the
// kernel-argument segment itself (scalar loads from constant memory); indexing the by-value
// argument with a run-time i would make the compiler copy the whole block to scratch.
// The block follows the kernel's ten scalar parameters (two pointers, eight ints: 48 bytes).
template <int NM>
__device__ __forceinline__ MatRun matrix_run(int i)
{
    typedef const __attribute__((address_space(4))) uint8_t* ConstBytePtr;
    typedef const __attribute__((address_space(4))) MatRun* ConstRunPtr;
    ConstRunPtr src = (ConstRunPtr)((ConstBytePtr)__builtin_amdgcn_kernarg_segment_ptr() + kArgsOffset + offsetof(GemvArgsT<NM>, run)) + i;
    MatRun r;
    r.blocks = src->blocks;
    r.per_wg = src->per_wg;
    r.extra_wg = src->extra_wg;
    r.per_wave[0] = src->per_wave[0];
    r.per_wave[1] = src->per_wave[1];
    r.extra_wave[0] = src->extra_wave[0];
    r.extra_wave[1] = src->extra_wave[1];
    return r;
}

template <int NM>
__device__ __forceinline__ MatArgs matrix_args(int i)
{
    typedef const __attribute__((address_space(4))) uint8_t* ConstBytePtr;
    typedef const __attribute__((address_space(4))) MatArgs* ConstMatPtr;
    ConstMatPtr src = (ConstMatPtr)((ConstBytePtr)__builtin_amdgcn_kernarg_segment_ptr() + kArgsOffset + offsetof(GemvArgsT<NM>, m)) + i;
    MatArgs r;
    r.row_of_rank = src->row_of_rank;
    r.empty_rows = src->empty_rows;
    r.carry = src->carry;
    r.counters = src->counters;
    r.slots = src->slots;
    r.y = src->y;
    r.N = src->N;
    r.n_empty = src->n_empty;
    r.n_ranks = src->n_ranks;
    return r;
}

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
__device__ __forceinline__ void decode_w4(uint32_t w, half2_t* q)
{
    const half2_t k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
    const half2_t k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t k64 = {(_Float16)64.0f, (_Float16)64.0f};
    // nibble masks and the fp16 pair (1024, 1024): constants kept in registers, so that
    // mask-and-splice is one three-operand instruction instead of two with literal operands
    const uint32_t nib_lo = 0x000F000Fu, nib_hi = 0x00F000F0u, k1024x2 = 0x64006400u;
    const uint32_t w2 = w >> 8;
    q[0] = as_half2(and_or(w, nib_lo, k1024x2)) - k1024;
    q[1] = __builtin_elementwise_fma(as_half2(and_or(w, nib_hi, k1024x2)), k16th, -k64);
    q[2] = as_half2(and_or(w2, nib_lo, k1024x2)) - k1024;
    q[3] = __builtin_elementwise_fma(as_half2(and_or(w2, nib_hi, k1024x2)), k16th, -k64);
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

__device__ __forceinline__ void store_row(const MatArgs& m, int b, int rank, float v)
{
    if (static_cast<unsigned>(rank) >= static_cast<unsigned>(m.n_ranks)) return;  // never for a valid image
    const int row = m.row_of_rank ? m.row_of_rank[rank] : rank;
    m.y[b * m.N + row] = float_to_half_bits(v);
}

// Storage format of a group as the kernel is compiled for it: code width and group size
// G = 16 * M.  A block holds 64 groups, one per lane: the code bytes in planes of at most
// 16 bytes per lane (each plane one coalesced load), then scale | zero << 16, then the index word.
template <int BITS_, int M_>
struct Fmt {
    static constexpr int BITS = BITS_;
    static constexpr int M = M_;                         // 16-element chunks per group
    static constexpr int CB = 16 * M_ * BITS_ / 8;       // code bytes per group
    static constexpr int CW = CB / 4;                    // code words per group
    static constexpr int CWC = CW / M_;                  // code words per chunk (2 or 4)
    static constexpr int PB = CB < 16 ? CB : 16;         // bytes per lane in one code plane
    static constexpr int PLANES = CB / PB;
    static constexpr int UMAX = CB <= 16 ? 4 : (CB <= 32 ? 2 : 1);   // blocks of the largest superblock
    static constexpr int BB = (CB + 6) * kLanes;         // block bytes
};

// The compressed groups of up to UMAX blocks, as loaded (one group per lane per block).
template <typename F>
struct Tile {
    uint32_t code[F::UMAX][F::CW];
    uint32_t sz[F::UMAX];
    uint32_t ix[F::UMAX];
};

// (1) stream the compressed groups: coalesced loads, all issued before anything waits.  The
// block pointer is wave-uniform (scalar base), the lane supplies a 32-bit byte offset.
template <typename T>
__device__ __forceinline__ T load_at(const uint8_t* base, uint32_t byte_offset)
{
    return *reinterpret_cast<const T*>(base + byte_offset);
}

template <typename F>
__device__ __forceinline__ void load_tile(Tile<F>& t, const uint8_t* p, int U, int lane)
{
    const uint32_t ulane = static_cast<uint32_t>(lane);
#pragma unroll
    for (int u = 0; u < F::UMAX; ++u) {
        if (u < U) {
#pragma unroll
            for (int pl = 0; pl < F::PLANES; ++pl) {
                if constexpr (F::PB == 8) {
                    const uint2 c = load_at<uint2>(p, ulane * 8u + u * F::BB);
                    t.code[u][0] = c.x; t.code[u][1] = c.y;
                } else {
                    const uint4 c = load_at<uint4>(p, ulane * 16u + (u * F::BB + pl * 16 * kLanes));
                    t.code[u][4 * pl + 0] = c.x; t.code[u][4 * pl + 1] = c.y;
                    t.code[u][4 * pl + 2] = c.z; t.code[u][4 * pl + 3] = c.w;
                }
            }
            t.sz[u] = load_at<uint32_t>(p, ulane * 4u + (u * F::BB + F::CB * kLanes));
            t.ix[u] = load_at<uint16_t>(p, ulane * 2u + (u * F::BB + (F::CB + 4) * kLanes));
        }
    }
}

// x in LDS, per activation row: elements 0..7 of every group-column in 16-byte slots, elements
// 8..15 in a second array of 16-byte slots 16*KGP bytes further on, and the fp32 sum of the 16
// as a dense array of floats at 32*KGP (4 bytes per column: a wavefront's 64 reads of it spread
// over all banks instead of a quarter of them).  Row b starts at b * 48 * KGP.
template <typename F, int KGP, int U, int NB, typename Args>
__device__ __forceinline__ void compute_tile(const Args& a, const MatArgs& m, const Tile<F>& t,
                                             int lane, const uint8_t* xlds, WaveState<NB>& st)
{
    // Row heads as wave-uniform lane masks, one per position of the superblock (index word =
    // column << 4 | head); counting them is scalar work.
    unsigned long long bal[U];
    unsigned long long hmask = 0;
    int heads_total = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        bal[u] = __ballot((t.ix[u] & 1u) != 0);
        hmask |= bal[u];
        heads_total += __popcll(bal[u]);
    }
    // no lane holds two heads (no row shorter than U groups here): branch-free serial sums
    const bool simple = heads_total == static_cast<int>(__popcll(hmask));
    int heads_before = 0;   // row heads of this superblock in lower lanes
    if (simple) {
        heads_before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(hmask >> 32),
                       __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(hmask), 0));
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u)
            heads_before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(bal[u] >> 32),
                           __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(bal[u]), heads_before));
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
        const float s = half_to_float(t.sz[u] & 0xFFFFu);
        const float z = half_to_float(t.sz[u] >> 16);
        const uint32_t slot = t.ix[u] & 0xFFF0u;        // byte offset of the group's first 16 activations
        float dotz[NB];   // sum_j q_j x_j - z sum_j x_j; times s it is the group's contribution
#pragma unroll
        for (int i = 0; i < F::M; ++i) {                // the group's 16-element chunks
            Codes c;
            if constexpr (F::BITS == 4) {
                decode_w4(t.code[u][2 * i], &c.q[0]);
                decode_w4(t.code[u][2 * i + 1], &c.q[4]);
            } else {
                decode_w8(t.code[u][4 * i], &c.q[0]);
                decode_w8(t.code[u][4 * i + 1], &c.q[2]);
                decode_w8(t.code[u][4 * i + 2], &c.q[4]);
                decode_w8(t.code[u][4 * i + 3], &c.q[6]);
            }
            const uint8_t* xg = xlds + slot + 16 * i;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint8_t* xb = xg + b * (48 * KGP);
                const uint4 xl = *reinterpret_cast<const uint4*>(xb);
                const uint4 xh = *reinterpret_cast<const uint4*>(xb + 16 * KGP);
                const float xs = *reinterpret_cast<const float*>(xlds + b * (48 * KGP) + 32 * KGP + (slot >> 2) + 4 * i);
                const float d = __builtin_fmaf(-z, xs, dot16(c, xl, xh));
                dotz[b] = i == 0 ? d : dotz[b] + d;
            }
        }
        const bool head_here = (t.ix[u] & 1u) != 0;
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
                    else store_row(m, b, st.rank + heads_before + nh, acc[b]);   // a whole row inside one lane
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
    if (st.heads == 0 && hmask != 0) first_lane = static_cast<int>(__builtin_ctzll(hmask));   // (uniform: a scalar)

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
        if (((hmask >> lane) & 1ull) != 0 && lane != first_lane) store_row(m, b, st.rank + heads_before, total);
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
__device__ __forceinline__ void chain_arrive(const MatArgs& m, const int4* wave_info, int first)
{
    const int4 head_info = wave_info[first];
    const int len = head_info.w;
    const int old = __hip_atomic_fetch_add(&m.counters[first], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old != len - 1) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    for (int b = 0; b < NB; ++b) {
        const CarryRecord* r0 = &m.carry[first * kMaxRowsPerLaunch + b];
        const int heads0 = __hip_atomic_load(&r0->heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        float sum = __hip_atomic_load(&r0->tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int w = first + 1; w < first + len; ++w) {
            const CarryRecord* r = &m.carry[w * kMaxRowsPerLaunch + b];
            const int hw = __hip_atomic_load(&r->heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sum += hw == 0 ? __hip_atomic_load(&r->tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)    // whole run
                           : __hip_atomic_load(&r->lead, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // up to its first head
        }
        store_row(m, b, head_info.x + heads0, sum);
    }
    __hip_atomic_store(&m.counters[first], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
}

// What a wavefront tells its workgroup about the rows it shares with its neighbours.
struct LdsSums {
    float lead;
    float tail;
};
struct LdsCounts {
    int4 info;     // the worker's record {rank_base, tail_closed + 2 * lead_len, lead_first, chain_len}
    int heads;     // row heads inside its run
    int pad[3];
};

// A row whose workers sit in two neighbouring workgroups: each side adds up its workers' pieces
// through LDS, in worker order, and the two partial sums meet in device memory -- each side
// swaps its (tagged) sum into the row's meeting point with one device-scope exchange.  The side
// that finds the slot empty is done: its sum travels inside the slot.  The side that finds the
// other's sum adds the two, writes the row and empties the slot for the next launch.  One
// round trip and no fence: nothing is read through the caches.  (Two fp32 terms: their sum
// does not depend on who adds them.)
__device__ __forceinline__ unsigned long long tagged(float v)
{
    return (static_cast<unsigned long long>(__builtin_bit_cast(uint32_t, v)) << 32) | 1ull;
}

// Swap `sum` into the meeting point; true (and the other side's sum in *other) if that was
// already there.
__device__ __forceinline__ bool meet(unsigned long long* slot, float sum, float* other)
{
    const unsigned long long got = __hip_atomic_exchange(slot, tagged(sum), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((got & 1ull) == 0) return false;
    *other = __builtin_bit_cast(float, static_cast<uint32_t>(got >> 32));
    __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// Carry fix-up of one matrix by one lane of a wavefront, after the workgroup's records are in
// LDS.  A row whose workers all sit in this workgroup is summed in worker order by the wavefront
// holding its head; one spread over two workgroups goes through a meeting point (above); only a
// row spread over three or more workgroups uses records and an arrival counter (chain_arrive).
// info = the worker's {rank_base, tail_closed + 2 * lead_len, lead_first, chain_len}; lead_len is
// the chain length of the row this run continues.
template <int NB>
__device__ __forceinline__ void fixup_matrix(const MatArgs& mo, const int4* wave_info, int4 info,
                                             int heads, const float* own_lead, const float* own_tail,
                                             const LdsCounts* cn, const LdsSums* cs, int wl, int wg, int wpw,
                                             int wave)
{
    const int rank_open = info.x + heads;
    const int head_w = info.y >> 1;
    const int wg_first = wg * wpw, wg_end = wg_first + wpw;     // this workgroup's workers
    auto piece = [&](int w, int b) {   // what local worker w adds to the row its run continues
        return cn[w].heads == 0 ? cs[w * NB + b].tail : cs[w * NB + b].lead;
    };
    if ((info.y & 1) != 0 && heads > 0) {     // last row ends with the run
#pragma unroll
        for (int b = 0; b < NB; ++b) store_row(mo, b, rank_open, own_tail[b]);
    }
    bool chain_tail = false, chain_lead = false;
    if (info.w > 0) {                         // this worker holds the head of a row that continues
        const int end = wave + info.w;        // one past the row's last worker
        if (end <= wg_end + wpw) {
            const int here = (end < wg_end ? end : wg_end) - wave;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float sum = own_tail[b], other = 0.0f;
                for (int w = wl + 1; w < wl + here; ++w) sum += piece(w, b);
                if (end <= wg_end) store_row(mo, b, rank_open, sum);
                else if (meet(&mo.slots[wave * kMaxRowsPerLaunch + b], sum, &other))
                    store_row(mo, b, rank_open, sum + other);
            }
        } else {
            chain_tail = true;
        }
    }
    if (info.z >= 0) {                        // its first groups continue a row of an earlier worker
        const int end = info.z + head_w;      // one past that row's last worker
        const bool head_here = info.z >= wg_first;
        const bool two_at_most = head_here ? end <= wg_end + wpw : (info.z >= wg_first - wpw && end <= wg_end);
        if (!two_at_most) {
            chain_lead = true;
        } else if (!head_here && wl == 0) {   // the far side's first worker speaks for all of them
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float sum = heads == 0 ? own_tail[b] : own_lead[b], other = 0.0f;
                for (int w = 1; w < end - wg_first; ++w) sum += piece(w, b);
                if (meet(&mo.slots[info.z * kMaxRowsPerLaunch + b], sum, &other))
                    store_row(mo, b, info.x, other + sum);
            }
        }                                     // (else: the worker holding the head, or the far side's first, adds this piece)
    }
    if (chain_tail || chain_lead) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            CarryRecord* r = &mo.carry[wave * kMaxRowsPerLaunch + b];
            __hip_atomic_store(&r->lead, own_lead[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&r->tail, own_tail[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&r->heads, heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // the stores have completed
        if (chain_lead) chain_arrive<NB>(mo, wave_info, info.z);
        if (chain_tail) chain_arrive<NB>(mo, wave_info, wave);
    }
}

// v_i for i < NM, chosen with scalar selects (arguments by value: an object holding them would
// be indexed in memory).
template <int NM>
__device__ __forceinline__ int pick_of(int i, int v0, int v1, int v2, int v3)
{
    int r = v0;
    if (NM > 1 && i == 1) r = v1;
    if (NM > 2 && i == 2) r = v2;
    if (NM > 3 && i == 3) r = v3;
    return r;
}

// One launch multiplies up to kMaxMatrices packed matrices that share x (q/k/v or gate/up of a
// decoder layer) -- the wavefront walks its run in the first matrix, then its run in the
// second, ... as one pipelined stream, so launch, x staging and first-byte latency are paid
// once.  With one matrix this is the plain GEMV.
struct ParkedArgs {
    MatArgs m;
    const int4* wave_info;
};

// The leading scalar parameters repeat what the first loads depend on (x, the first matrix's
// run, the slot count, the wavefronts per workgroup): the file is compiled with kernel-argument
// preloading for them, so they sit in scalar registers when a wavefront starts instead of being
// fetched from the argument block first.  The block itself follows at byte kArgsOffset.
static_assert(kArgsOffset == 2 * 8 + 8 * 4, "two pointers and eight ints precede the argument block");

template <typename F, int KGP, int NB, int NM>
__global__ __launch_bounds__(kWavesPerWorkgroup * kLanes) void gqsa_gemv_kernel(
    const uint16_t* x_first, const uint8_t* blocks_first, int per_wg_first, int extra_wg_first, int per_wave0_first,
    int per_wave1_first, int extra_wave0_first, int extra_wave1_first, int kg_first, int wpw_first, GemvArgsT<NM> a)
{
    const MatRun run_first = {blocks_first, per_wg_first, extra_wg_first, {per_wave0_first, per_wave1_first},
                              {extra_wave0_first, extra_wave1_first}};
    // x arrays (NB * 48 * KGP bytes), then the wavefronts' records per matrix
    extern __shared__ __align__(16) uint8_t xlds[];
    LdsCounts* rec_n = reinterpret_cast<LdsCounts*>(xlds + NB * 48 * KGP);            // [matrix][wavefront]
    LdsSums* rec_s = reinterpret_cast<LdsSums*>(rec_n + NM * kWavesPerWorkgroup);  // [matrix][wavefront][NB]
    // the output arguments of every matrix, parked for the fix-up at the end of the kernel (reading
    // them from the argument block there would put a round trip on the kernel's tail)
    ParkedArgs* parked = reinterpret_cast<ParkedArgs*>(rec_s + NM * kWavesPerWorkgroup * NB);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wpw = wpw_first;
    const int n_threads = wpw * kLanes;
    const int wl = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: scalar registers
    const int wg = blockIdx.x;
    const int wave = wg * wpw + wl;
    constexpr int BB = F::BB;

    // a worker's run of blocks in a matrix: the blocks are dealt evenly to the workgroups, a
    // workgroup's blocks evenly to its wavefronts (contiguous runs, equal counts)
    auto run_of = [&](const MatRun& r, int& left, const uint8_t*& p) {
        const int big = wg < r.extra_wg ? 1 : 0;              // this workgroup holds per_wg + 1 blocks
        const int wg_first = r.per_wg * wg + (big ? wg : r.extra_wg);
        const int per_wave = r.per_wave[big], extra_wave = r.extra_wave[big];
        left = per_wave + (wl < extra_wave ? 1 : 0);
        p = r.blocks + static_cast<size_t>(wg_first + per_wave * wl + (wl < extra_wave ? wl : extra_wave)) * BB;
    };
    // superblocks of 4, 2, 1 blocks (as far as the format's largest superblock allows)
    auto next_size = [](int n) { return n >= 4 && F::UMAX >= 4 ? 4 : (n >= 2 && F::UMAX >= 2 ? 2 : (n >= 1 ? 1 : 0)); };

    // issue the loads of x first and of the first superblock right behind them, so that the
    // weights are already on their way while x is staged in LDS
    auto stage = [&](int c, uint4 lo, uint4 hi) {   // c = slot over all rows: b * kg + column
        const int b = NB == 1 ? 0 : c / kg_first;
        uint8_t* slot = xlds + b * (48 * KGP) + (c - b * kg_first) * 16;
        *reinterpret_cast<uint4*>(slot) = lo;
        *reinterpret_cast<uint4*>(slot + 16 * KGP) = hi;
        const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            s += half_to_float(w[i] & 0xFFFFu);
            s += half_to_float(w[i] >> 16);
        }
        *reinterpret_cast<float*>(xlds + b * (48 * KGP) + 32 * KGP + (c - b * kg_first) * 4) = s;
    };
    const int n_slots = NB * kg_first;                  // x is [NB][K] contiguous: slot c holds x[16c .. 16c+15]

    // the first matrix in which this worker owns blocks
    int mi = 0, left = 0;
    const uint8_t* p = nullptr;
    run_of(run_first, left, p);
    while (left == 0 && mi + 1 < NM) {
        ++mi;
        run_of(matrix_run<NM>(mi), left, p);
    }
    // The first superblock's loads go out first, x right behind them (both need only the first
    // line of the argument block); then the per-matrix worker records (what the fix-up needs to
    // know about this worker; a worker without blocks may still sit inside a row) and the
    // output arguments; then x is staged in LDS.
    Tile<F> cur, nxt;
    int u_cur = next_size(left);
    load_tile<F>(cur, p, u_cur, lane);
    uint4 lo0 = {0, 0, 0, 0}, hi0 = {0, 0, 0, 0};
    if (tid < n_slots) {
        const uint4* src = reinterpret_cast<const uint4*>(x_first + static_cast<size_t>(tid) * 16);
        lo0 = src[0];
        hi0 = src[1];
    }
    // Everything else comes from later lines of the argument block and from the worker table:
    // requested now, while the weights are on their way.  (Left alone, the compiler issues these
    // loads where their results are first used -- after the wait for x -- and their latency
    // would land on the critical path; the worker record is therefore fetched with a vector
    // load through a lane offset the compiler cannot see through, and the arguments are pinned.)
    int lane_zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));
    typedef int int4_t __attribute__((ext_vector_type(4)));
    auto info_of = [&](int i) { return reinterpret_cast<const int4_t*>(a.wave_info[i])[wave + lane_zero]; };
    const int4_t info0 = info_of(0);
    const int4_t info1 = NM > 1 ? info_of(1) : int4_t{-1, 1, -1, 0};
    const int4_t info2 = NM > 2 ? info_of(2) : int4_t{-1, 1, -1, 0};
    const int4_t info3 = NM > 3 ? info_of(3) : int4_t{-1, 1, -1, 0};
    MatArgs m = a.m[0];
    if constexpr (NM > 1) m = matrix_args<NM>(mi);
    asm volatile("" ::"s"(m.row_of_rank), "s"(m.y), "s"(m.N), "s"(m.n_ranks));
#pragma unroll
    for (int i = 0; i < NM; ++i)
        asm volatile("" ::"s"(a.m[i].empty_rows), "s"(a.m[i].carry), "s"(a.m[i].counters), "s"(a.m[i].y),
                     "s"(a.m[i].n_empty), "s"(a.wave_info[i]), "s"(a.n_wg));
    if (tid < n_slots) stage(tid, lo0, hi0);
    for (int c = tid + n_threads; c < n_slots; c += n_threads) {
        const uint4* src = reinterpret_cast<const uint4*>(x_first + static_cast<size_t>(c) * 16);
        stage(c, src[0], src[1]);
    }
    // rows without stored groups: exactly +0; and this worker's records start out as "nothing"
#pragma unroll
    for (int i = 0; i < NM; ++i) {
        {
            if (NM > 1 && tid == 0) parked[i] = ParkedArgs{a.m[i], a.wave_info[i]};
            if (lane == 0) {
                rec_n[i * kWavesPerWorkgroup + wl].heads = 0;
#pragma unroll
                for (int b = 0; b < NB; ++b) rec_s[(i * kWavesPerWorkgroup + wl) * NB + b] = LdsSums{0.0f, 0.0f};
            }
            for (int e = wg * n_threads + tid; e < a.m[i].n_empty; e += a.n_wg * n_threads) {
                const int row = a.m[i].empty_rows[e];
#pragma unroll
                for (int b = 0; b < NB; ++b) a.m[i].y[b * a.m[i].N + row] = 0;
            }
        }
    }
    __syncthreads();

    WaveState<NB> st;
#pragma unroll
    for (int b = 0; b < NB; ++b) { st.carry[b] = 0.0f; st.lead[b] = 0.0f; }
    // The rank bases move to scalar registers here, where every load has arrived anyway: waiting
    // for the worker records inside the loop would also wait for the superblock prefetched
    // there, since loads complete in order.
    const int rb0 = __builtin_amdgcn_readfirstlane(info0.x);
    const int rb1 = NM > 1 ? __builtin_amdgcn_readfirstlane(info1.x) : 0;
    const int rb2 = NM > 2 ? __builtin_amdgcn_readfirstlane(info2.x) : 0;
    const int rb3 = NM > 3 ? __builtin_amdgcn_readfirstlane(info3.x) : 0;
    asm volatile("" ::"s"(rb0), "s"(rb1), "s"(rb2), "s"(rb3));
    auto rank_base_of = [=](int i) { return pick_of<NM>(i, rb0, rb1, rb2, rb3); };
    st.rank = rank_base_of(mi);
    st.heads = 0;
    WaveState<NB> fin = st;      // the finished run's sums (with one matrix the fix-up takes them from here)
    if (u_cur > 0) {
        for (;;) {
            // where the stream goes on: the next superblock of this run, or the first one of the
            // worker's run in the next matrix that has blocks for it
            left -= u_cur;
            const uint8_t* p_next = p + u_cur * BB;
            int u_next = next_size(left);
            int mi_next = mi;
            while (u_next == 0 && mi_next + 1 < NM) {
                ++mi_next;
                run_of(matrix_run<NM>(mi_next), left, p_next);
                u_next = next_size(left);
            }
            load_tile<F>(nxt, p_next, u_next, lane);   // in flight during this superblock
            if constexpr (F::UMAX >= 4) {
                if (u_cur == 4) compute_tile<F, KGP, 4, NB>(a, m, cur, lane, xlds, st);
            }
            if constexpr (F::UMAX >= 2) {
                if (u_cur == 2) compute_tile<F, KGP, 2, NB>(a, m, cur, lane, xlds, st);
            }
            if (u_cur == 1) compute_tile<F, KGP, 1, NB>(a, m, cur, lane, xlds, st);
            if (mi_next != mi || u_next == 0) {           // this matrix's run is complete
                if (lane == 0) {
                    rec_n[mi * kWavesPerWorkgroup + wl].heads = st.heads;   // (info is filled in below)
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        rec_s[(mi * kWavesPerWorkgroup + wl) * NB + b] = LdsSums{st.lead[b], st.carry[b]};
                }
                if constexpr (NM > 1) {     // (with one matrix the state stays in registers for the fix-up)
                    fin = st;
#pragma unroll
                    for (int b = 0; b < NB; ++b) { st.carry[b] = 0.0f; st.lead[b] = 0.0f; }
                    st.rank = rank_base_of(mi_next);
                    st.heads = 0;
                }
            }
            if (u_next == 0) break;
            cur = nxt;
            u_cur = u_next;
            p = p_next;
            if (mi_next != mi) m = matrix_args<NM>(mi_next);
            mi = mi_next;
        }
    }

    if constexpr (NM == 1) fin = st;
    // Carry fix-up for the rows a run shares with its neighbours.  Inside a workgroup the
    // pieces meet in LDS; only rows spread over several workgroups go through device memory.
    if (lane == 0) {
        auto park = [&](int i, int4_t v) { rec_n[i * kWavesPerWorkgroup + wl].info = int4{v.x, v.y, v.z, v.w}; };  // (lane 0's copy)
        park(0, info0);
        if (NM > 1) park(1, info1);
        if (NM > 2) park(2, info2);
        if (NM > 3) park(3, info3);
    }
    __syncthreads();
    if constexpr (NM == 1) {
        if (lane != 0) return;
        // everything this worker contributes is still in registers
        fixup_matrix<NB>(a.m[0], a.wave_info[0], int4{info0.x, info0.y, info0.z, info0.w}, fin.heads,
                         fin.lead, fin.carry, rec_n, rec_s, wl, wg, wpw, wave);
    } else {
        // lane i settles matrix i (side by side: the fix-up is a chain of dependent LDS reads)
        if (lane >= NM) return;
        const int i = lane;
        const LdsCounts* cn = rec_n + i * kWavesPerWorkgroup;
        const LdsSums* cs = rec_s + i * kWavesPerWorkgroup * NB;
        float own_lead[NB], own_tail[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) { own_lead[b] = cs[wl * NB + b].lead; own_tail[b] = cs[wl * NB + b].tail; }
        fixup_matrix<NB>(parked[i].m, parked[i].wave_info, cn[wl].info, cn[wl].heads, own_lead, own_tail, cn, cs,
                         wl, wg, wpw, wave);
    }
}

// A launchable variant: the kernel for NM matrices takes the first NM entries of the host's
// argument block.
struct Variant {
    const void* fn = nullptr;    // device function, for attribute setting
    void (*launch)(const GemvArgs&, dim3, dim3, size_t, hipStream_t) = nullptr;
    explicit operator bool() const { return fn != nullptr; }
};

constexpr size_t lds_bytes(int kgp, int nb, int nm)
{
    return static_cast<size_t>(nb) * 48 * kgp +
           nm * (kWavesPerWorkgroup * (sizeof(LdsCounts) + nb * sizeof(LdsSums)) + sizeof(ParkedArgs));
}

template <int NM>
GemvArgsT<NM> first_matrices(const GemvArgs& a)
{
    GemvArgsT<NM> r{};
    r.x = a.x; r.n_mats = NM; r.kg = a.kg;
    r.wpw = a.wpw; r.n_wg = a.n_wg;
    for (int i = 0; i < NM; ++i) { r.run[i] = a.run[i]; r.wave_info[i] = a.wave_info[i]; r.m[i] = a.m[i]; }
    return r;
}

template <typename F, int KGP, int NB, int NM>
void launch_variant(const GemvArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t s)
{
    const MatRun& r = a.run[0];
    hipLaunchKernelGGL((gqsa_gemv_kernel<F, KGP, NB, NM>), grid, block, lds, s, a.x, r.blocks, r.per_wg, r.extra_wg,
                       r.per_wave[0], r.per_wave[1], r.extra_wave[0], r.extra_wave[1], a.kg, a.wpw, first_matrices<NM>(a));
}

template <typename F, int KGP, int NB, int NM>
Variant variant_if_it_fits()
{
    Variant v;
    if constexpr (lds_bytes(KGP, NB, NM) <= kMaxLdsBytes) {
        v.fn = reinterpret_cast<const void*>(&gqsa_gemv_kernel<F, KGP, NB, NM>);
        v.launch = &launch_variant<F, KGP, NB, NM>;
    }
    return v;
}

// Compiled variants.  Group size 16: 1, 2, 4 or 8 activation rows for one matrix (as far as NB
// copies of x fit the 160 KB of LDS), and 2, 3 or 4 matrices for one activation row.  Larger
// groups: one activation row, one matrix.
template <typename F, int KGP>
Variant pick_variant(int nb, int nm)
{
    if constexpr (F::M == 1) {
        if (nm == 1) {
            switch (nb) {
                case 1: return variant_if_it_fits<F, KGP, 1, 1>();
                case 2: return variant_if_it_fits<F, KGP, 2, 1>();
                case 4: return variant_if_it_fits<F, KGP, 4, 1>();
                case 8: return variant_if_it_fits<F, KGP, 8, 1>();
            }
        } else if (nb == 1) {
            switch (nm) {
                case 2: return variant_if_it_fits<F, KGP, 1, 2>();
                case 3: return variant_if_it_fits<F, KGP, 1, 3>();
                case 4: return variant_if_it_fits<F, KGP, 1, 4>();
            }
        }
    } else {
        if (nm == 1 && nb == 1) return variant_if_it_fits<F, KGP, 1, 1>();
    }
    return Variant{};
}

// The kernel is compiled for counts of 16-element activation slots (K/16) rounded up to a power
// of two (the LDS offsets between the x arrays are immediates).
template <typename F>
Variant pick_kernel(int slots, int nb, int nm, int* kgp)
{
    if (slots <= 256) { *kgp = 256; return pick_variant<F, 256>(nb, nm); }
    if (slots <= 512) { *kgp = 512; return pick_variant<F, 512>(nb, nm); }
    if (slots <= 1024) { *kgp = 1024; return pick_variant<F, 1024>(nb, nm); }
    if (slots <= 2048) { *kgp = 2048; return pick_variant<F, 2048>(nb, nm); }
    *kgp = 0;
    return Variant{};
}

Variant pick(const gqsa_matrix* m, int nb, int nm, int* kgp)
{
    const int slots = static_cast<int>(m->K / 16);
    *kgp = 0;
    if (m->bits == 4) {
        switch (m->G) {
            case 16: return pick_kernel<Fmt<4, 1>>(slots, nb, nm, kgp);
            case 32: return pick_kernel<Fmt<4, 2>>(slots, nb, nm, kgp);
            case 64: return pick_kernel<Fmt<4, 4>>(slots, nb, nm, kgp);
            case 128: return pick_kernel<Fmt<4, 8>>(slots, nb, nm, kgp);
        }
    } else if (m->bits == 8) {
        switch (m->G) {
            case 16: return pick_kernel<Fmt<8, 1>>(slots, nb, nm, kgp);
            case 32: return pick_kernel<Fmt<8, 2>>(slots, nb, nm, kgp);
            case 64: return pick_kernel<Fmt<8, 4>>(slots, nb, nm, kgp);
        }
    }
    return Variant{};
}

constexpr size_t counters_offset(int n_waves)
{
    return static_cast<size_t>(n_waves) * kMaxRowsPerLaunch * sizeof(CarryRecord);
}
constexpr size_t slots_offset(int n_waves)
{
    return counters_offset(n_waves) + (static_cast<size_t>(n_waves) + 1) / 2 * 2 * sizeof(int);
}
constexpr size_t carry_workspace_bytes(int n_waves)
{
    return slots_offset(n_waves) + static_cast<size_t>(n_waves) * kMaxRowsPerLaunch * sizeof(unsigned long long);
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
    if (!pick(m, 1, 1, &kgp)) return GQSA_ERR_UNSUPPORTED;   // K/G above 2048: x does not fit the LDS layout
    int dev = 0;
    GQSA_HIP(hipGetDevice(&dev));
    for (int nb = 1; nb <= kMaxRowsPerLaunch; nb *= 2) {
        for (int nm = 1; nm <= kMaxMatrices; ++nm) {
            Variant v = pick(m, nb, nm, &kgp);
            if (v && lds_bytes(kgp, nb, nm) > 64 * 1024)
                GQSA_HIP(hipFuncSetAttribute(v.fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                             static_cast<int>(lds_bytes(kgp, nb, nm))));
        }
    }
    void* img = nullptr;
    void* carry = nullptr;
    GQSA_HIP(hipMalloc(&img, m->image.size()));
    // carry records (per worker and activation row), one arrival counter per worker (padded to a
    // multiple of two), then the meeting points of two-worker chains (per worker and row)
    const size_t carry_bytes = carry_workspace_bytes(m->n_waves);
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

gqsa_status_t device_gemv(gqsa_matrix* const* ms, int n_mats, const void* x, void* const* ys, int batch,
                          void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const gqsa_matrix* m0 = ms[0];
    // the device image, its workspace and the kernels' LDS attributes belong to one GPU
    int dev = -1;
    GQSA_HIP(hipGetDevice(&dev));
    for (int i = 0; i < n_mats; ++i)
        if (ms[i]->device != dev) return GQSA_ERR_HIP;
    GemvArgs a{};
    for (int i = 0; i < n_mats; ++i) {
        const gqsa_matrix* m = ms[i];
        const uint8_t* img = static_cast<const uint8_t*>(m->d_image);
        MatRun& r = a.run[i];
        r.blocks = img + m->map.blocks;
        a.wave_info[i] = reinterpret_cast<const int4*>(img + m->map.wave_info);
        r.per_wg = static_cast<int>(m->n_blocks / m->n_workgroups);
        r.extra_wg = static_cast<int>(m->n_blocks % m->n_workgroups);
        for (int big = 0; big < 2; ++big) {
            r.per_wave[big] = (r.per_wg + big) / m->waves_per_workgroup;
            r.extra_wave[big] = (r.per_wg + big) % m->waves_per_workgroup;
        }
        MatArgs& o = a.m[i];
        o.row_of_rank = m->n_empty ? reinterpret_cast<const int32_t*>(img + m->map.row_of_rank) : nullptr;
        o.empty_rows = reinterpret_cast<const int32_t*>(img + m->map.empty_rows);
        o.carry = static_cast<CarryRecord*>(m->d_carry);
        uint8_t* ws = static_cast<uint8_t*>(m->d_carry);
        o.counters = reinterpret_cast<int*>(ws + counters_offset(m->n_waves));
        o.slots = reinterpret_cast<unsigned long long*>(ws + slots_offset(m->n_waves));
        o.N = m->N;
        o.n_empty = static_cast<int>(m->n_empty);
        o.n_ranks = static_cast<int>(m->N - m->n_empty);
    }
    a.n_mats = n_mats;
    a.wpw = m0->waves_per_workgroup;
    a.n_wg = m0->n_workgroups;
    a.kg = static_cast<int>(m0->K / 16);       // 16-element activation slots

    const int threads = m0->waves_per_workgroup * kLanes;
    const int grid = m0->n_workgroups;
    int kgp_multi = 0;
    const Variant multi = (n_mats > 1 && batch == 1) ? pick(m0, 1, n_mats, &kgp_multi) : Variant{};
    if (multi) {
        // several matrices, one activation row: one launch walks them all
        const int kgp = kgp_multi;
        const Variant v = multi;
        a.x = static_cast<const uint16_t*>(x);
        for (int i = 0; i < n_mats; ++i) a.m[i].y = static_cast<uint16_t*>(ys[i]);
        v.launch(a, dim3(grid), dim3(threads), lds_bytes(kgp, 1, n_mats), s);
    } else {
        // one matrix at a time; its batch goes out in launches of 8, 4, 2 or 1 rows: the most
        // that the format has a kernel for, fits LDS and is left
        for (int i = 0; i < n_mats; ++i) {
            GemvArgs one = a;
            one.n_mats = 1;
            one.run[0] = a.run[i];
            one.wave_info[0] = a.wave_info[i];
            one.m[0] = a.m[i];
            int done = 0;
            while (done < batch) {
                int nb = kMaxRowsPerLaunch, kgp = 0;
                Variant v;
                for (; nb >= 1; nb /= 2) {
                    if (nb > batch - done) continue;
                    v = pick(m0, nb, 1, &kgp);
                    if (v) break;
                }
                if (!v) return GQSA_ERR_UNSUPPORTED;
                one.x = static_cast<const uint16_t*>(x) + static_cast<size_t>(done) * m0->K;
                one.m[0].y = static_cast<uint16_t*>(ys[i]) + static_cast<size_t>(done) * ms[i]->N;
                v.launch(one, dim3(grid), dim3(threads), lds_bytes(kgp, nb, 1), s);
                done += nb;
            }
        }
    }
    GQSA_HIP(hipGetLastError());
    return GQSA_OK;
}

}  // namespace gqsa
