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
// one fully coalesced instruction; a tile is U blocks (4 at G = 16): lane l owns the U
// consecutive stream positions U*l .. U*l+U-1, sums them serially and takes part in ONE
// cross-lane segmented scan per tile.  A wavefront owns whole tiles.  With the default partition
// it owns one on decode shapes: it requests all of its bytes before anything else and works
// through the blocks in the order in which they arrive; a run of several tiles is worked through
// with the next tile requested ahead.
//
// One launch can carry several matrices that share x (q/k/v, gate/up): the workgroups of the
// grid are dealt to the matrices, each workgroup works on one of them.
//
// Small batches: the kernel is compiled for NB = 1, 2, 4, 8 activation rows per launch; each
// decoded group is multiplied with all NB rows (weights are read and dequantised once).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cstddef>
#include <cstdint>
#include <cstdio>
#include <mutex>
#include <type_traits>

#include "gqsa_internal.hpp"

// This file is compiled several times: once whole (GQSA_GEMV_PART 0: the kernels for the formats'
// own tile sizes and all the host code) and once per further tile size (parts 1..4: tiles of 3, 4, 5 and -- 4-bit codes -- 6 and 8
// blocks with a chosen count of lanes in use, group size 16), so that the kernels build side by side.
#ifndef GQSA_GEMV_PART
#define GQSA_GEMV_PART 0
#endif

#if GQSA_GEMV_PART == 0
// Fix-up workspace of gqsa_gemv_static (at the end of this file), for callers that must not
// allocate: carry records, arrival counters and meeting points for up to kScratchWorkers wavefront
// workers -- the most a default partition deals to -- at 196 bytes each.  Every GPU the library
// runs on holds its own copy (3.1 MiB) from the first use of the library to the end of the process.
// In host code the name stands for the symbol, not for memory a kernel could address: the device
// address is asked for once per GPU (scratch_address) and only that pointer is handed to kernels.
constexpr int kScratchWorkers = 16384;
constexpr size_t kScratchBytes = static_cast<size_t>(kScratchWorkers) * 196;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
#endif

namespace gqsa {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef int int4_t __attribute__((ext_vector_type(4)));

constexpr int kMaxRowsPerLaunch = 8;      // NB values compiled: 1, 2, 4, 8
constexpr int kMaxLdsBytes = 160 * 1024;  // LDS of one gfx950 compute unit

constexpr int kMaxMatrices = 4;           // matrices sharing x that one launch can take

struct MatArgs {                 // where a matrix's results go (64 bytes)
    const int32_t* row_of_rank;  // row index of the r-th non-empty row (nullptr: identity)
    const int32_t* empty_rows;
    CarryRecord* carry;          // [worker][kMaxRowsPerLaunch]
    int* counters;               // arrivals per carry chain, indexed by the chain's first worker
    unsigned long long* slots;   // [worker][kMaxRowsPerLaunch] meeting points of rows spread over two workgroups
    uint16_t* y;                 // fp16 [rows][N]
    int N;
    int last_row;                // activation rows of this launch - 1 (a kernel for NB rows may be given fewer)
    int n_empty;
    int n_ranks;                 // non-empty rows
};

// One matrix of a launch (104 bytes of the kernel-argument block).  Its T tiles are dealt evenly
// to its W workers: worker w owns the tiles floor(w T / W) .. floor((w+1) T / W) - 1.  With
// T = base * W + extra that is base * w + floor(w * extra / W), and the division is a multiply
// by magic = ceil(2^48 / W) and a shift (exact for w <= W <= 65536, extra < W).
struct MatDesc {
    const uint8_t* blocks;
    const int4_t* wave_info;     // {rank_base, tail_closed + 2 * lead_len, lead_first, chain_len} per worker
    unsigned long long magic;
    int base, extra;
    int n_wg;                    // workgroups of the launch that work on this matrix
    int pad;
    MatArgs out;
};
struct LaunchArgs {
    MatDesc m[kMaxMatrices];
};
static_assert(sizeof(MatArgs) == 64 && sizeof(MatDesc) == 104, "argument block layout");

// A launchable variant of the kernel.
struct Variant {
    const void* fn = nullptr;    // device function, for attribute setting
    void (*launch)(const LaunchArgs&, const uint16_t*, int, const int*, dim3, dim3, size_t, hipStream_t) = nullptr;
    explicit operator bool() const { return fn != nullptr; }
};

// The variants for tiles of `u` blocks that the other compilations of this file hold (an empty
// Variant from the parts that do not have that size).
Variant tile_variant_part1(int bits, int u, int slots, int nb, int* kgp);
Variant tile_variant_part2(int bits, int u, int slots, int nb, int* kgp);
Variant tile_variant_part3(int bits, int u, int slots, int nb, int* kgp);
Variant tile_variant_part4(int bits, int u, int slots, int nb, int* kgp);

namespace {

// where the argument block sits in the kernel-argument segment: after the scalar parameters
// (three pointers, a 64-bit number and six ints: the 14 dwords that can be preloaded)
constexpr int kArgsOffset = 4 * 8 + 6 * 4;

// The descriptor of matrix i (wave-uniform), read from the kernel-argument segment itself with
// scalar loads; indexing the by-value argument with a run-time i would make the compiler copy
// the whole block to scratch.
__device__ __forceinline__ MatDesc matrix_desc(int i)
{
    typedef const __attribute__((address_space(4))) uint8_t* ConstBytePtr;
    typedef const __attribute__((address_space(4))) MatDesc* ConstDescPtr;
    ConstDescPtr src = (ConstDescPtr)((ConstBytePtr)__builtin_amdgcn_kernarg_segment_ptr() + kArgsOffset) + i;
    MatDesc r;
    r.blocks = src->blocks;
    r.wave_info = src->wave_info;
    r.magic = src->magic;
    r.base = src->base;
    r.extra = src->extra;
    r.n_wg = src->n_wg;
    r.pad = 0;
    r.out.row_of_rank = src->out.row_of_rank;
    r.out.empty_rows = src->out.empty_rows;
    r.out.carry = src->out.carry;
    r.out.counters = src->out.counters;
    r.out.slots = src->out.slots;
    r.out.y = src->out.y;
    r.out.N = src->out.N;
    r.out.last_row = src->out.last_row;
    r.out.n_empty = src->out.n_empty;
    r.out.n_ranks = src->out.n_ranks;
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

// The 16 codes of one stored group as eight fp16 pairs (element 2i, 2i+1), exact -- as fp16
// SUBNORMALS: a code q moved to bits 4..7 of an otherwise empty 16-bit half is the fp16 number
// 16 q * 2^-24 = q * 2^-20, so a group is decoded by shifting and masking alone; there is no
// exponent to splice in and no bias to take off again (14 instead of 18 vector instructions per
// group).  v_dot2_f32_f16 multiplies subnormal inputs exactly; its adder, though, aligns the
// products by the operands' nominal exponents and does not renormalise a subnormal one first,
// so every leading zero of the code's mantissa costs a bit of the sum's 24: measured on the
// device against float64, the error of a 16-term dot product relative to the sum of |terms| is
// 2.0e-8 with normal operands, 9.3e-8 with codes at bits 4..7 and 2.3e-6 with codes at bits 0..3.
// Hence all four nibbles of a 16-bit half are brought to bits 4..7 (three shifts per code word
// instead of one); left in place the low nibbles saved another 3 instructions per group and
// 1.5 % of a launch, but the worst error against the oracle rose from 4.7e-4 to 5.6-7.5e-4.
// The power of two is carried along: the staged group sums of x are scaled by it (a dot product
// with the pair (2^-20, 2^-20), itself an fp16 subnormal, instead of (1, 1)), so that
// sum_j q_j x_j - z sum_j x_j comes out in units of 2^-20, and a lane's sums are multiplied by
// 2^20 once per tile, after its groups are added up (scalings by powers of two are exact).
struct Codes {
    half2_t q[8];
};
template <int BITS> struct CodeUnit;
template <> struct CodeUnit<4> {
    static constexpr float kInverse = 1048576.0f;            // 2^20
    static constexpr uint32_t kPairOfUnits = 0x00100010u;    // the fp16 pair (2^-20, 2^-20)
};
template <> struct CodeUnit<8> {            // (8-bit codes keep the unit 1, see decode_w8)
    [[maybe_unused]] static constexpr float kInverse = 1.0f;
    [[maybe_unused]] static constexpr uint32_t kPairOfUnits = 0x3C003C00u;    // (1, 1)
};

// 4-bit: the code words are nibble-permuted at pack time (element 2m at bits 4m, element 2m+1
// at bits 16+4m), so a shift and one AND isolate a pair of codes at bits 4..7 and 20..23:
// (q, q') * 2^-20.
[[maybe_unused]] __device__ __forceinline__ void decode_w4(uint32_t w, half2_t* q)
{
    const uint32_t nib_hi = 0x00F000F0u;
    q[0] = as_half2((w << 4) & nib_hi);
    q[1] = as_half2(w & nib_hi);
    q[2] = as_half2((w >> 4) & nib_hi);
    q[3] = as_half2((w >> 8) & nib_hi);
}

// 8-bit: a byte permute drops each code (bytes of w, element order) into the mantissa of
// 1024.0 (0x64xx), one packed subtract removes the bias.  (Left as subnormals, q * 2^-24, the
// 8-bit codes gave sums that missed the error bound on activations with full mantissas -- 3.6e-3
// where this form gives 4.6e-4 -- although single products came out exact; the 4-bit form
// shows no such difference.)
[[maybe_unused]] __device__ __forceinline__ void decode_w8(uint32_t w, half2_t* q)
{
    const half2_t k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
    const uint32_t k64s = 0x64646464u;
    q[0] = as_half2(__builtin_amdgcn_perm(w, k64s, 0x00050004u)) - k1024;
    q[1] = as_half2(__builtin_amdgcn_perm(w, k64s, 0x00070006u)) - k1024;
}

// sum_j q_j x_j of four pairs of codes (one code word of 4-bit codes, two of 8-bit codes) in the
// format's unit, in two chains (4-bit codes; 8-bit codes: one chain in the unit 1).
template <int BITS>
__device__ __forceinline__ float dot8(const half2_t* q, uint4 x, float lo, float& hi)
{
    if constexpr (BITS == 4) {
        lo = __builtin_amdgcn_fdot2(q[0], as_half2(x.x), lo, false);
        hi = __builtin_amdgcn_fdot2(q[1], as_half2(x.y), hi, false);
        lo = __builtin_amdgcn_fdot2(q[2], as_half2(x.z), lo, false);
        hi = __builtin_amdgcn_fdot2(q[3], as_half2(x.w), hi, false);
    } else {
        lo = __builtin_amdgcn_fdot2(q[0], as_half2(x.x), lo, false);
        lo = __builtin_amdgcn_fdot2(q[1], as_half2(x.y), lo, false);
        lo = __builtin_amdgcn_fdot2(q[2], as_half2(x.z), lo, false);
        lo = __builtin_amdgcn_fdot2(q[3], as_half2(x.w), lo, false);
    }
    return lo;
}
// the two partial sums joined, in the format's unit (2^-20 for 4-bit codes, 1 for 8-bit codes)
template <int BITS>
__device__ __forceinline__ float join(float lo, float hi)
{
    if constexpr (BITS == 4) return lo + hi;
    else return lo;      // (one chain: hi stays 0)
}

template <int BITS>
__device__ __forceinline__ float dot16(const Codes& c, uint4 xl, uint4 xh)
{
    float lo = 0.0f, hi = 0.0f;
    lo = dot8<BITS>(&c.q[0], xl, lo, hi);
    lo = dot8<BITS>(&c.q[4], xh, lo, hi);
    return join<BITS>(lo, hi);
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

// a in the lanes whose bit is set in the wave-uniform mask, b elsewhere
__device__ __forceinline__ float select_lanes(unsigned long long mask, float a, float b)
{
    float r;
    asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(r) : "v"(b), "v"(a), "s"(mask));
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
    if ((b == 3 || b == 7) && b > m.last_row) return;     // a row the caller does not have: the 4th of 3, the 8th of 7
    m.y[static_cast<size_t>(b) * m.N + row] = float_to_half_bits(v);
}

// Storage format of a group as the kernel is compiled for it: code width, group size
// G = 16 * M, or G = 8 (M = 0: half a chunk), and blocks per tile.  U_ = 0: the format's own
// count, and a block holds 64 groups, one per lane: the code bytes in planes of at most 16 bytes
// per lane (each plane one coalesced load), then scale | zero << 16, then the index word.
// U_ > 0 (FLEX): U_ blocks of L groups each, L <= 64 given at launch -- the same three arrays
// with L entries, the lanes from L on take no group (partitions that keep whole rows inside a
// wavefront's run choose U_ and L so that the rows fill the tiles).
template <int BITS_, int M_, int U_ = 0>
struct Fmt {
    static constexpr bool FLEX = U_ != 0;
    static constexpr int BITS = BITS_;
    static constexpr int M = M_;                         // 16-element chunks per group (0: G = 8)
    static constexpr bool HALF = M_ == 0;
    static constexpr int CB = (HALF ? 8 : 16 * M_) * BITS_ / 8;   // code bytes per group
    static constexpr int CW = CB / 4;                    // code words per group
    static constexpr int CWC = HALF ? CW : CW / (M_ ? M_ : 1);    // code words per chunk (2 or 4; half chunk: 1 or 2)
    static constexpr int PB = CB < 16 ? CB : 16;         // bytes per lane in one code plane
    static constexpr int PLANES = CB / PB;
    static constexpr int UMAX = U_ ? U_ : largest_tile(CB);   // blocks of a tile
    static constexpr int BB = (CB + 6) * kLanes;         // block bytes (of a 64-lane block)
    static constexpr int TB = UMAX * BB;                 // tile bytes (of 64-lane blocks)
    static constexpr int LOADS = UMAX * (PLANES + 2);    // load instructions per tile
};

// The compressed groups of a tile, as loaded (one group per lane per block).
template <typename F>
struct Tile {
    uint32_t code[F::UMAX][F::CW];
    uint32_t sz[F::UMAX];
    uint32_t ix[F::UMAX];
};

// The fields of a group's index word and its scale, as masks.  In tiles of a chosen shape the
// lanes that take no group hold all-zero masks, so that their words read as a null group's (no
// row head, slot 0, scale 0) at no extra instruction: the masks take the place of literals.
template <bool FLEX>
struct LaneMasks {
    uint32_t head, slot, scale;
    __device__ __forceinline__ explicit LaneMasks(bool lane_in_use)
        : head(lane_in_use ? 1u : 0u), slot(lane_in_use ? 0xFFF0u : 0u), scale(lane_in_use ? 0xFFFFu : 0u) {}
};
template <>
struct LaneMasks<false> {          // every lane takes a group: the masks are literals
    [[maybe_unused]] static constexpr uint32_t head = 1u, slot = 0xFFF0u, scale = 0xFFFFu;
    __device__ __forceinline__ explicit LaneMasks(bool) {}
};

// (1) stream the compressed groups: coalesced loads, all issued before anything waits.  The
// tile pointer is wave-uniform (scalar base), the lane supplies a 32-bit byte offset.
template <typename T>
__device__ __forceinline__ T load_at(const uint8_t* base, uint32_t byte_offset)
{
    return *reinterpret_cast<const T*>(base + byte_offset);
}

// Reads from LDS at a byte address given as a number.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 lds_read16(uint32_t address)
{
    const u32x4_t v = *(const __attribute__((address_space(3))) u32x4_t*)(uintptr_t)address;
    return uint4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ float lds_read_float(uint32_t address)
{
    return *(const __attribute__((address_space(3))) float*)(uintptr_t)address;
}

// A tile's loads go out index words first (four small loads: the gathers from LDS need nothing
// else), then codes and scale/zero block by block; loads return in the order of issue, so the
// tile can be worked through while its later blocks are still on their way.
template <typename F>
__device__ __forceinline__ void load_tile(Tile<F>& t, const uint8_t* p, int lane, int lanes_in_use)
{
    const uint32_t ulane = static_cast<uint32_t>(lane);
    if constexpr (F::FLEX) {
        // blocks of L = lanes_in_use entries: block u at p + u * L * (CB + 6) (a scalar), its arrays at
        // lane offsets that depend on L.  The lanes from L on load what lane 0 loads (a stored
        // group's words: finite numbers) and mask it away when they use it (LaneMasks); all
        // lanes load, so the loads are straight-line code like any other tile's and x, requested
        // before them, can be awaited alone.
        static_assert(F::PLANES == 1, "tiles of a chosen shape: one code plane");
        const uint32_t L = static_cast<uint32_t>(lanes_in_use);
        const uint32_t bb = L * (F::CB + 6);
        const uint32_t l = ulane < L ? ulane : 0u;
        const uint32_t off_ix = l * 2u + L * (F::CB + 4), off_sz = l * 4u + L * F::CB;
#pragma unroll
        for (int u = 0; u < F::UMAX; ++u) t.ix[u] = load_at<uint16_t>(p + u * bb, off_ix);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < F::UMAX; ++u) {
            if constexpr (F::PB == 8) {
                const uint2 c = load_at<uint2>(p + u * bb, l * 8u);
                t.code[u][0] = c.x; t.code[u][1] = c.y;
            } else {
                const uint4 c = load_at<uint4>(p + u * bb, l * 16u);
                t.code[u][0] = c.x; t.code[u][1] = c.y; t.code[u][2] = c.z; t.code[u][3] = c.w;
            }
            t.sz[u] = load_at<uint32_t>(p + u * bb, off_sz);
            __builtin_amdgcn_sched_barrier(0);
        }
        return;
    }
#pragma unroll
    for (int u = 0; u < F::UMAX; ++u)
        t.ix[u] = load_at<uint16_t>(p, ulane * 2u + (u * F::BB + (F::CB + 4) * kLanes));
    __builtin_amdgcn_sched_barrier(0);      // (the order of issue is the order of arrival: keep it)
#pragma unroll
    for (int u = 0; u < F::UMAX; ++u) {
#pragma unroll
        for (int pl = 0; pl < F::PLANES; ++pl) {
            if constexpr (F::PB == 4) {
                t.code[u][0] = load_at<uint32_t>(p, ulane * 4u + u * F::BB);
            } else if constexpr (F::PB == 8) {
                const uint2 c = load_at<uint2>(p, ulane * 8u + u * F::BB);
                t.code[u][0] = c.x; t.code[u][1] = c.y;
            } else {
                const uint4 c = load_at<uint4>(p, ulane * 16u + (u * F::BB + pl * 16 * kLanes));
                t.code[u][4 * pl + 0] = c.x; t.code[u][4 * pl + 1] = c.y;
                t.code[u][4 * pl + 2] = c.z; t.code[u][4 * pl + 3] = c.w;
            }
        }
        t.sz[u] = load_at<uint32_t>(p, ulane * 4u + (u * F::BB + F::CB * kLanes));
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <typename F>
__device__ __forceinline__ void decode_chunk(const Tile<F>& t, int u, int i, Codes& c)
{
    if constexpr (F::BITS == 4) {
        decode_w4(t.code[u][2 * i], &c.q[0]);
        decode_w4(t.code[u][2 * i + 1], &c.q[4]);
    } else {
        decode_w8(t.code[u][4 * i], &c.q[0]);
        decode_w8(t.code[u][4 * i + 1], &c.q[2]);
        decode_w8(t.code[u][4 * i + 2], &c.q[4]);
        decode_w8(t.code[u][4 * i + 3], &c.q[6]);
    }
}

// x in LDS, per activation row: elements 0..7 of every group-column in 16-byte slots, elements
// 8..15 in a second array of 16-byte slots 16*KGP bytes further on, and the fp32 sum of the 16
// as a dense array of floats at 32*KGP (4 bytes per column: a wavefront's 64 reads of it spread
// over all banks instead of a quarter of them; with one 16-byte slot per sum the three reads of
// a group would share an address and save a shift, but the kernels for several activation rows,
// which LDS bounds, took 5 % longer).  Row b starts at b * 48 * KGP.  (G = 8: the same
// two arrays -- a group's 8 activations are one slot of the first or of the second -- and a sum
// per half-slot, 8 bytes per column.)
//
// EAGER: the tile's loads may still be in flight.  All gathers are issued first (they need only
// the index words, the first of the tile's loads to arrive), then the groups are decoded block
// by block as their codes come in.  Otherwise the gathers go group by group (fewer registers).
template <typename F, int KGP, int NB, bool EAGER>
__device__ __forceinline__ void compute_tile(const MatArgs& m, const Tile<F>& t, int lane, const uint8_t* xlds,
                                             WaveState<NB>& st, const LaneMasks<F::FLEX> mask)
{
    constexpr int U = F::UMAX;
    // Row heads as wave-uniform lane masks, one per position of the tile (index word =
    // column << 4 | head); counting them is scalar work.
    unsigned long long bal[U];
    unsigned long long hmask = 0;
    int heads_total = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        bal[u] = __ballot((t.ix[u] & mask.head) != 0);
        hmask |= bal[u];
        heads_total += __popcll(bal[u]);
    }
    // no lane holds two heads (no row shorter than U groups here): branch-free serial sums
    const bool simple = heads_total == static_cast<int>(__popcll(hmask));
    int heads_before = 0;   // row heads of this tile in lower lanes
    if (simple) {
        heads_before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(hmask >> 32),
                       __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(hmask), 0));
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u)
            heads_before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(bal[u] >> 32),
                           __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(bal[u]), heads_before));
    }

    // (5a) the lane's U consecutive groups are added serially: lead = what precedes the lane's
    // first row head, acc = what follows its last one (everything, if it has none).  fold() adds
    // group u, given its dotz = sum_j q_j x_j - z sum_j x_j per activation row:
    //   sum_j (q_j - z) s x_j  =  s * (sum_j q_j x_j  -  z * sum_j x_j)
    // SIMPLE (no lane holds two heads): the heads of block u are the lanes of bal[u], which
    // selects straight from its scalar register pair; a block without heads (most: a row of a
    // multiple of U groups puts all its heads into block 0) just adds.
    float acc[NB], lead[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) { acc[b] = 0.0f; lead[b] = 0.0f; }
    int nh = 0;
    // (in the loops over groups below -- several activation rows, several tiles -- the plain form:
    // per-lane selects on the head flag, no branch per block: 3 % faster there)
    auto fold_in_loop = [&](int u, const float* dotz) {
        const float s = half_to_float(t.sz[u] & mask.scale);
        const bool head_here = (t.ix[u] & mask.head) != 0;
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
                    else store_row(m, b, st.rank + heads_before + nh, acc[b] * CodeUnit<F::BITS>::kInverse);   // a whole row inside one lane
                    acc[b] = 0.0f;
                }
                ++nh;
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[b] = __builtin_fmaf(s, dotz[b], acc[b]);
        }
    };
    auto fold = [&](auto simple_tag, int u, const float* dotz) {
        const float s = half_to_float(t.sz[u] & mask.scale);
        if constexpr (decltype(simple_tag)::value) {
            if (bal[u] == 0) {
#pragma unroll
                for (int b = 0; b < NB; ++b) acc[b] = __builtin_fmaf(s, dotz[b], acc[b]);
            } else {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    lead[b] = select_lanes(bal[u], acc[b], lead[b]);     // the only head of this lane
                    acc[b] = __builtin_fmaf(s, dotz[b], keep_lanes(~bal[u], acc[b]));
                }
            }
        } else {
            if ((t.ix[u] & mask.head) != 0) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    if (nh == 0) lead[b] = acc[b];
                    else store_row(m, b, st.rank + heads_before + nh, acc[b] * CodeUnit<F::BITS>::kInverse);   // a whole row inside one lane
                    acc[b] = 0.0f;
                }
                ++nh;
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[b] = __builtin_fmaf(s, dotz[b], acc[b]);
        }
    };

    // (2)-(4) gather the activation group by real group index, dequantise, multiply.
    // (LDS addresses as plain numbers: the kernel has no static LDS, so x starts at 0 -- the host
    // checks that when the kernel is first used; written through the array's symbol every
    // address would cost an addition of that 0)
    constexpr uint32_t x0 = 0;
    if constexpr (EAGER && NB == 1 && F::M == 1) {
        // (at most four groups' activations are under way at a time: enough to cover the latency
        // of LDS, and the registers do not grow with the tile)
        constexpr int AHEAD = U < 4 ? U : 4;
        uint4 xl[U], xh[U];
        float xs[U], dotz[U];
        auto gather = [&](int u) {
            const uint32_t slot = t.ix[u] & mask.slot;        // byte offset of the group's 16 activations
            xl[u] = lds_read16(x0 + slot);
            xh[u] = lds_read16(x0 + slot + 16 * KGP);
            xs[u] = lds_read_float(x0 + 32 * KGP + (slot >> 2));
        };
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) gather(u);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            Codes c;
            decode_chunk<F>(t, u, 0, c);
            const float z = half_to_float(t.sz[u] >> 16);
            dotz[u] = __builtin_fmaf(-z, xs[u], dot16<F::BITS>(c, xl[u], xh[u]));
            if (u + AHEAD < U) {
                gather(u + AHEAD);
                __builtin_amdgcn_sched_barrier(0x47F);     // (LDS reads stay behind this point: no more than AHEAD groups under way)
            }
        }
        if (simple) {
#pragma unroll
            for (int u = 0; u < U; ++u) fold(std::true_type{}, u, &dotz[u]);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) fold(std::false_type{}, u, &dotz[u]);
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float z = half_to_float(t.sz[u] >> 16);
            const uint32_t slot = t.ix[u] & mask.slot;
            float dotz[NB];          // sum_j q_j x_j - z sum_j x_j of group u for every activation row
            if constexpr (F::HALF) {
                // G = 8: the index word counts 8-element half-slots; an even one lies in the array
                // of the slots' first halves, an odd one in the array of their second halves, and
                // the sums are kept per half-slot
                Codes c;
                if constexpr (F::BITS == 4) {
                    decode_w4(t.code[u][0], &c.q[0]);
                } else {
                    decode_w8(t.code[u][0], &c.q[0]);
                    decode_w8(t.code[u][1], &c.q[2]);
                }
                const uint32_t xoff = ((slot >> 5) << 4) + ((slot >> 4) & 1u) * (16 * KGP);
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const uint4 xl = lds_read16(x0 + xoff + b * (48 * KGP));
                    const float xs = lds_read_float(x0 + b * (48 * KGP) + 32 * KGP + (slot >> 2));
                    float lo = 0.0f, hi = 0.0f;
                    lo = dot8<F::BITS>(&c.q[0], xl, lo, hi);
                    dotz[b] = __builtin_fmaf(-z, xs, join<F::BITS>(lo, hi));
                }
            }
#pragma unroll
            for (int i = 0; i < F::M; ++i) {                // the group's 16-element chunks
                Codes c;
                decode_chunk<F>(t, u, i, c);
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const uint32_t xb = x0 + slot + 16 * i + b * (48 * KGP);
                    const uint4 xl = lds_read16(xb);
                    const uint4 xh = lds_read16(xb + 16 * KGP);
                    const float xs = lds_read_float(x0 + b * (48 * KGP) + 32 * KGP + (slot >> 2) + 4 * i);
                    const float d = __builtin_fmaf(-z, xs, dot16<F::BITS>(c, xl, xh));
                    dotz[b] = i == 0 ? d : dotz[b] + d;
                }
            }
            fold_in_loop(u, dotz);
        }
    }

    // the lane's sums leave the unit of the codes' dot products (an exact scaling)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        acc[b] *= CodeUnit<F::BITS>::kInverse;
        lead[b] *= CodeUnit<F::BITS>::kInverse;
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
        v = select_lanes(p1, v, v + dpp_or_zero<0x111, 0xF>(v));       // row_shr:1
        v = select_lanes(p2, v, v + dpp_or_zero<0x112, 0xF>(v));       // row_shr:2
        v = select_lanes(p4, v, v + dpp_or_zero<0x114, 0xF>(v));       // row_shr:4
        v = select_lanes(p8, v, v + dpp_or_zero<0x118, 0xF>(v));       // row_shr:8
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

// Cross-workgroup carry chain (a row whose groups are spread over wavefronts of three or more
// workgroups).  Every holder of a piece publishes its record with device-scope stores, then
// reports to the chain's counter; the last one to report adds the pieces in worker order (so
// the sum does not depend on arrival order) and writes the row.  The report is a device-scope
// acquire-release read-modify-write: the record stores of every reporter happen before its
// report, and the last reporter's reads of the records happen after it has seen all the others'
// reports -- the ordering is the language's, not an accident of how stores complete.  (This path
// is rare -- rows longer than a workgroup's whole share -- so the cache write-back and invalidate
// that the release and the acquire cost are paid by few wavefronts.)
template <int NB>
__device__ __forceinline__ void chain_arrive(const MatArgs& m, const int4* wave_info, int first)
{
    const int4 head_info = wave_info[first];
    const int len = head_info.w;
    const int old = __hip_atomic_fetch_add(&m.counters[first], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (old != len - 1) return;
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

// What a wavefront tells its workgroup, per activation row, about the rows it shares with its
// neighbours: one 16-byte LDS word, so that a neighbour learns it with a single read.
struct LdsRecord {
    float lead;    // sum of its groups before its first row head
    float tail;    // sum of its groups since its last row head (all of them without one)
    int heads;     // row heads inside its run
    int pad;
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

// How a worker's shared rows are settled: worked out from its record and its place in the
// workgroup as soon as the record is there -- scalar arithmetic done while the tiles are still
// on their way -- so that little is left to do once the sums are known.  A row whose workers
// all sit in one workgroup is summed by the wavefront holding its head; one spread over two
// workgroups goes through a meeting point (above); only a row spread over three or more
// workgroups uses records and an arrival counter (chain_arrive).
struct FixupPlan {
    int head_mode;   // the row this run leaves open: 0 none, 1 ends in this workgroup, 2 in the next, 3 further on
    int head_n;      // workers after this one, in this workgroup, holding pieces of it
    int lead_mode;   // the row this run continues: 0 someone else adds this piece, 2 this worker speaks
                     // for the second workgroup of two, 3 three workgroups or more
    int lead_n;      // mode 2: workers after this one holding pieces of it
};

// info = the worker's {rank_base, tail_closed + 2 * lead_len, lead_first, chain_len}; lead_len is
// the chain length of the row this run continues.
__device__ __forceinline__ FixupPlan plan_fixup(int4 info, int wl, int wg, int wpw, int wave)
{
    FixupPlan pl{0, 0, 0, 0};
    const int wg_first = wg * wpw, wg_end = wg_first + wpw;     // this workgroup's workers
    if (info.w > 0) {
        const int end = wave + info.w;        // one past the row's last worker
        pl.head_mode = end <= wg_end ? 1 : (end <= wg_end + wpw ? 2 : 3);
        pl.head_n = (end < wg_end ? end : wg_end) - wave - 1;
    }
    if (info.z >= 0) {
        const int end = info.z + (info.y >> 1);
        const bool head_here = info.z >= wg_first;
        const bool two_at_most = head_here ? end <= wg_end + wpw : (info.z >= wg_first - wpw && end <= wg_end);
        pl.lead_mode = !two_at_most ? 3 : ((!head_here && wl == 0) ? 2 : 0);
        pl.lead_n = end - wg_first - 1;
    }
    return pl;
}

// Carry fix-up of one matrix by a wavefront, after the workgroup's records are in LDS.  Lane w
// reads worker w's records -- one LDS read per activation row, all in flight together, whatever
// the number of pieces -- and the pieces are then added in worker order from the lanes.
template <int NB>
__device__ __forceinline__ void fixup_matrix(const MatArgs& mo, const int4* wave_info, int4 info, FixupPlan pl,
                                             int heads, const float* own_lead, const float* own_tail,
                                             const LdsRecord* rec, int lane, int wl, int wpw, int wave)
{
    // piece[b] in lane w: what local worker w adds to the row its run continues
    float piece[NB];
    {
        const int w = lane < wpw ? lane : 0;
        LdsRecord r[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) r[b] = rec[w * NB + b];
#pragma unroll
        for (int b = 0; b < NB; ++b) piece[b] = r[b].heads == 0 ? r[b].tail : r[b].lead;
    }
    const bool writer = lane == 0;
    const int rank_open = info.x + heads;
    if (pl.head_mode == 1 || pl.head_mode == 2) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float sum = own_tail[b], other = 0.0f;
            for (int i = 1; i <= pl.head_n; ++i) sum += read_lane(piece[b], wl + i);
            if (writer) {
                if (pl.head_mode == 1) store_row(mo, b, rank_open, sum);
                else if (meet(&mo.slots[wave * kMaxRowsPerLaunch + b], sum, &other))
                    store_row(mo, b, rank_open, sum + other);
            }
        }
    }
    if (pl.lead_mode == 2) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float sum = heads == 0 ? own_tail[b] : own_lead[b], other = 0.0f;
            for (int i = 1; i <= pl.lead_n; ++i) sum += read_lane(piece[b], i);
            if (writer && meet(&mo.slots[info.z * kMaxRowsPerLaunch + b], sum, &other))
                store_row(mo, b, info.x, other + sum);
        }
    }
    if ((pl.head_mode == 3 || pl.lead_mode == 3) && writer) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            CarryRecord* r = &mo.carry[wave * kMaxRowsPerLaunch + b];
            __hip_atomic_store(&r->lead, own_lead[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&r->tail, own_tail[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&r->heads, heads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // (the reports below release these stores at device scope)
        if (pl.lead_mode == 3) chain_arrive<NB>(mo, wave_info, info.z);
        if (pl.head_mode == 3) chain_arrive<NB>(mo, wave_info, wave);
    }
}

// Workgroup barrier for data exchanged through LDS only: the wavefront's LDS accesses have
// completed; its loads from global memory that are still in flight stay in flight (a
// __syncthreads() would wait for them too).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// The leading scalar parameters repeat what the first loads depend on (x, the first matrix's
// tile stream, worker table and deal, the slot count and the wavefronts per workgroup in one
// word, where the other matrices' workgroups begin): 14 dwords, as many as the hardware preloads;
// the file is compiled with kernel-argument preloading for them, so they sit in scalar registers
// when a wavefront starts instead of being fetched from the argument block first.  The block
// itself follows at byte kArgsOffset.
template <typename F, int KGP, int NB>
__global__ __launch_bounds__(kWavesPerWorkgroup * kLanes) void gqsa_gemv_kernel(
    const uint16_t* x, const uint8_t* blocks0, const int4_t* wave_info0, unsigned long long magic0, int base0, int extra0,
    int kg_wpw, int wg_end0, int wg_end1, int wg_end2, LaunchArgs a)
{
    // x arrays (NB * 48 * KGP bytes), then what the wavefronts tell each other about shared rows
    extern __shared__ __align__(16) uint8_t xlds[];
    LdsRecord* rec = reinterpret_cast<LdsRecord*>(xlds + NB * 48 * KGP);        // [wavefront][NB]

    const int kg = kg_wpw & 0xFFFF;       // 16-element slots of K
    const int wpw = (kg_wpw >> 16) & 0x1F;    // wavefronts per workgroup
    const int lanes_in_use = F::FLEX ? ((kg_wpw >> 21) & 0x7F) : kLanes;     // groups per block
    // slots of x that exist: the caller may have fewer than NB rows (3 for a kernel of 4, 7 for
    // one of 8); the rows beyond take the last slot's activations and their sums are never stored
    const int last_slot = (((kg_wpw >> 28) & 7) + 1) * kg - 1;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int n_threads = wpw * kLanes;
    const int wl = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: scalar registers
    const int wg = blockIdx.x;

    // x goes out first: it is small, every wavefront of the workgroup needs it before it can
    // use any weight, and loads return in the order of issue.  Slot c holds x[16c .. 16c+15]
    // (x is [NB][K] contiguous); a thread's first slot (first two for K above 8192) travels in
    // registers.
    // (one slot per thread covers K up to 4096 with one activation row; with several rows, or larger K, two:
    // what is not requested here is requested behind the tile and arrives behind it)
    constexpr int XPRE = (KGP >= 512 || NB == 2 || NB == 4 || (NB == 8 && F::BITS == 4)) ? 2 : 1;      // (8 rows of 8-bit codes: the registers are not there)
    const int n_slots = NB * kg;
    uint4 xlo[XPRE], xhi[XPRE];
#pragma unroll
    for (int j = 0; j < XPRE; ++j) {
        const int c = tid + j * n_threads;
        if (c < n_slots) {       // (the same condition guards the use)
            const uint4* src = reinterpret_cast<const uint4*>(x + static_cast<size_t>(NB > 2 ? min(c, last_slot) : c) * 16);
            xlo[j] = src[0];
            xhi[j] = src[1];
        }
    }

    // which matrix this workgroup works on, and which worker of that matrix this wavefront is
    const int mi = (wg >= wg_end0 ? 1 : 0) + (wg >= wg_end1 ? 1 : 0) + (wg >= wg_end2 ? 1 : 0);
    const int lwg = wg - (mi == 0 ? 0 : (mi == 1 ? wg_end0 : (mi == 2 ? wg_end1 : wg_end2)));
    const int worker = lwg * wpw + wl;
    const MatDesc md = matrix_desc(mi);
    const uint8_t* blocks = blocks0;
    const int4_t* wave_info = wave_info0;
    unsigned long long magic = magic0;
    int base = base0, extra = extra0;
    if (mi != 0) {      // (a branch, not a select: the first matrix's workgroups do not wait for the descriptor)
        blocks = md.blocks;
        wave_info = md.wave_info;
        magic = md.magic;
        base = md.base;
        extra = md.extra;
        asm volatile("" : "+s"(base));
    }
    // the worker's record {rank_base, tail_closed + 2 * lead_len, lead_first, chain_len}: requested
    // here, between x and the tiles (loads return in the order of issue), with a vector load
    // through a lane offset the compiler cannot see through -- a scalar load it would move to
    // the first use of the record, where its latency would be in the way
    int lane_zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));
    const int4_t info_v = wave_info[worker + lane_zero];

    // the worker's run of tiles (scalar arithmetic)
    auto first_tile = [&](int w) {
        const unsigned long long n = static_cast<unsigned long long>(static_cast<unsigned>(w)) * static_cast<unsigned>(extra);
        return base * w + static_cast<int>((n * magic) >> 48);
    };
    const int tile0 = first_tile(worker);
    const int n_tiles = first_tile(worker + 1) - tile0;
    const uint32_t tile_bytes = F::FLEX ? static_cast<uint32_t>(F::UMAX * (F::CB + 6) * lanes_in_use) : static_cast<uint32_t>(F::TB);
    const uint8_t* p = blocks + static_cast<size_t>(tile0) * tile_bytes;

    auto stage = [&](int c, uint4 lo, uint4 hi) {   // c = slot over all rows: b * kg + column
        const int b = NB == 1 ? 0 : c / kg;
        uint8_t* slot = xlds + b * (48 * KGP) + (c - b * kg) * 16;
        *reinterpret_cast<uint4*>(slot) = lo;
        *reinterpret_cast<uint4*>(slot + 16 * KGP) = hi;
        const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        const half2_t ones = as_half2(CodeUnit<F::BITS>::kPairOfUnits);     // (the sums are kept in the unit of the codes' dot products)
        if constexpr (F::HALF) {     // G = 8: a sum per half-slot
            float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                s0 = __builtin_amdgcn_fdot2(as_half2(w[i]), ones, s0, false);
                s1 = __builtin_amdgcn_fdot2(as_half2(w[4 + i]), ones, s1, false);
            }
            *reinterpret_cast<float2*>(xlds + b * (48 * KGP) + 32 * KGP + (c - b * kg) * 8) = float2{s0, s1};
        } else {
            float s = 0.0f;      // sum of the slot's 16 activations, fp32: a pair per instruction
#pragma unroll
            for (int i = 0; i < 8; ++i) s = __builtin_amdgcn_fdot2(as_half2(w[i]), ones, s, false);
            *reinterpret_cast<float*>(xlds + b * (48 * KGP) + 32 * KGP + (c - b * kg) * 4) = s;
        }
    };
    // x into LDS (the loads of the tiles are already out), then the workgroup meets
    auto stage_x_and_meet = [&]() {
#pragma unroll
        for (int j = 0; j < XPRE; ++j) {
            const int c = tid + j * n_threads;
            if (c < n_slots) stage(c, xlo[j], xhi[j]);
        }
        for (int c = tid + XPRE * n_threads; c < n_slots; c += n_threads) {
            const uint4* src = reinterpret_cast<const uint4*>(x + static_cast<size_t>(NB > 2 ? min(c, last_slot) : c) * 16);
            stage(c, src[0], src[1]);
        }
        lds_barrier();
    };
    // (after the barrier: the record is the oldest load still counted, long since there)
    auto record = [&]() {
        return int4_t{__builtin_amdgcn_readfirstlane(info_v.x), __builtin_amdgcn_readfirstlane(info_v.y),
                      __builtin_amdgcn_readfirstlane(info_v.z), __builtin_amdgcn_readfirstlane(info_v.w)};
    };
    // how the rows shared with the neighbours will be settled: decided now, not when the sums are there
    auto plan = [&](int4_t i) {
        FixupPlan pl = plan_fixup(int4{i.x, i.y, i.z, i.w}, wl, lwg, wpw, worker);
        asm volatile("" : "+s"(pl.head_mode), "+s"(pl.head_n), "+s"(pl.lead_mode), "+s"(pl.lead_n));
        return pl;
    };

    const LaneMasks<F::FLEX> mask(lane < lanes_in_use);
    WaveState<NB> st;
#pragma unroll
    for (int b = 0; b < NB; ++b) { st.carry[b] = 0.0f; st.lead[b] = 0.0f; }
    st.heads = 0;
    Tile<F> cur;
    int4_t info;
    FixupPlan pl;
    if (n_tiles == 1) {
        // the whole run is one tile (the default partition's aim): nothing else is in flight
        // behind it, and its blocks are consumed in the order in which they arrive
        load_tile<F>(cur, p, lane, lanes_in_use);
        stage_x_and_meet();
        info = record();
        st.rank = info.x;
        pl = plan(info);
        compute_tile<F, KGP, NB, true>(md.out, cur, lane, xlds, st, mask);
    } else if (F::FLEX || n_tiles == 0) {
        // a worker without tiles still helps to stage x.  (Tiles of a chosen shape come one to a
        // worker -- the host builds no other partition of them -- so that kernel has no loop over tiles.)
        stage_x_and_meet();
        info = record();
        st.rank = info.x;
        pl = plan(info);
    } else if constexpr (!F::FLEX) {
        // a run of several tiles: the next tile is requested before the current one is worked on
        // (the copy at the top of the loop is where the wavefront waits for a tile; inside
        // compute_tile nothing waits for memory)
        Tile<F> nxt;
        load_tile<F>(nxt, p, lane, lanes_in_use);
        stage_x_and_meet();
        info = record();
        st.rank = info.x;
        pl = plan(info);
        for (int left = n_tiles; left > 0; --left) {
            cur = nxt;
            p += tile_bytes;
            if (left > 1) load_tile<F>(nxt, p, lane, lanes_in_use);      // in flight during this tile
            compute_tile<F, KGP, NB, false>(md.out, cur, lane, xlds, st, mask);
        }
    }

    // rows without stored groups: exactly +0
    for (int e = lwg * n_threads + tid; e < md.out.n_empty; e += md.n_wg * n_threads) {
        const int row = md.out.empty_rows[e];
#pragma unroll
        for (int b = 0; b < NB; ++b)
            if (!((b == 3 || b == 7) && b > md.out.last_row)) md.out.y[static_cast<size_t>(b) * md.out.N + row] = 0;
    }

    // the last row of the run, if it ends there
    if (lane == 0 && (info.y & 1) != 0 && st.heads > 0) {
#pragma unroll
        for (int b = 0; b < NB; ++b) store_row(md.out, b, info.x + st.heads, st.carry[b]);
    }
    // A wavefront whose run neither continues an earlier worker's row nor leaves a row open has
    // nothing to settle with its neighbours.  (A barrier does not wait for wavefronts that have
    // ended.)
    if (info.z < 0 && info.w == 0) return;
    // Carry fix-up for the rows a run shares with its neighbours.  Inside a workgroup the
    // pieces meet in LDS; only rows spread over several workgroups go through device memory.
    if (lane == 0) {
#pragma unroll
        for (int b = 0; b < NB; ++b) rec[wl * NB + b] = LdsRecord{st.lead[b], st.carry[b], st.heads, 0};
    }
    lds_barrier();
    fixup_matrix<NB>(md.out, reinterpret_cast<const int4*>(wave_info), int4{info.x, info.y, info.z, info.w}, pl, st.heads,
                     st.lead, st.carry, rec, lane, wl, wpw, worker);
}

constexpr size_t lds_bytes(int kgp, int nb)
{
    return static_cast<size_t>(nb) * 48 * kgp + kWavesPerWorkgroup * nb * sizeof(LdsRecord);
}

// (kg_wpw_rows: slots of K | wavefronts per workgroup << 16 | lanes in use << 21 | (activation rows - 1) << 28)
template <typename F, int KGP, int NB>
void launch_variant(const LaunchArgs& a, const uint16_t* x, int kg_wpw_rows, const int* wg_end, dim3 grid, dim3 block,
                    size_t lds, hipStream_t s)
{
    const MatDesc& m0 = a.m[0];
    hipLaunchKernelGGL((gqsa_gemv_kernel<F, KGP, NB>), grid, block, lds, s, x, m0.blocks, m0.wave_info, m0.magic,
                       m0.base, m0.extra, kg_wpw_rows, wg_end[0], wg_end[1], wg_end[2], a);
}

template <typename F, int KGP, int NB>
Variant variant_if_it_fits()
{
    Variant v;
    if constexpr (lds_bytes(KGP, NB) <= kMaxLdsBytes) {
        v.fn = reinterpret_cast<const void*>(&gqsa_gemv_kernel<F, KGP, NB>);
        v.launch = &launch_variant<F, KGP, NB>;
    }
    return v;
}

// Compiled variants.  Group size 16: 1, 2, 4 or 8 activation rows per launch (as far as NB
// copies of x fit the 160 KB of LDS).  Larger groups: one activation row.
template <typename F, int KGP>
Variant pick_variant(int nb)
{
    if (nb == 1) return variant_if_it_fits<F, KGP, 1>();
    if constexpr (F::M == 1) {
        switch (nb) {
            case 2: return variant_if_it_fits<F, KGP, 2>();
            case 4: return variant_if_it_fits<F, KGP, 4>();
            case 8: return variant_if_it_fits<F, KGP, 8>();
        }
    }
    return Variant{};
}

// The kernel is compiled for counts of 16-element activation slots (K/16) rounded up to a power
// of two (the LDS offsets between the x arrays are immediates).
template <typename F>
Variant pick_kernel(int slots, int nb, int* kgp)
{
    if (slots <= 256) { *kgp = 256; return pick_variant<F, 256>(nb); }
    if (slots <= 512) { *kgp = 512; return pick_variant<F, 512>(nb); }
    if (slots <= 1024) { *kgp = 1024; return pick_variant<F, 1024>(nb); }
    if (slots <= 2048) { *kgp = 2048; return pick_variant<F, 2048>(nb); }
    *kgp = 0;
    return Variant{};
}

#if GQSA_GEMV_PART != 0
// The two (code width, blocks per tile) pairs of this compilation.
#if GQSA_GEMV_PART == 1
#define GQSA_PART_NAME tile_variant_part1
#define GQSA_PART_PAIRS {4, 3}, {8, 3}
#elif GQSA_GEMV_PART == 2
#define GQSA_PART_NAME tile_variant_part2
#define GQSA_PART_PAIRS {4, 4}, {8, 4}
#elif GQSA_GEMV_PART == 3
#define GQSA_PART_NAME tile_variant_part3
#define GQSA_PART_PAIRS {4, 5}, {8, 5}
#else
#define GQSA_PART_NAME tile_variant_part4
#define GQSA_PART_PAIRS {4, 6}, {4, 8}
#endif
struct BitsAndBlocks { int bits, u; };
constexpr BitsAndBlocks kPairs[2] = {GQSA_PART_PAIRS};

}  // namespace

Variant GQSA_PART_NAME(int bits, int u, int slots, int nb, int* kgp)
{
    if (bits == kPairs[0].bits && u == kPairs[0].u) return pick_kernel<Fmt<kPairs[0].bits, 1, kPairs[0].u>>(slots, nb, kgp);
    if (bits == kPairs[1].bits && u == kPairs[1].u) return pick_kernel<Fmt<kPairs[1].bits, 1, kPairs[1].u>>(slots, nb, kgp);
    return Variant{};
}

}  // namespace gqsa

#else   // GQSA_GEMV_PART == 0: the formats' own tile sizes, and the host side

Variant pick(const gqsa_matrix* m, int nb, int* kgp)
{
    const int slots = static_cast<int>(m->K / 16);
    *kgp = 0;
    if (m->tile_blocks != largest_tile(m->code_bytes()) || m->tile_lanes != kLanes) {     // tiles of a chosen shape
        if (m->G != 16) return Variant{};
        Variant (*const parts[4])(int, int, int, int, int*) = {tile_variant_part1, tile_variant_part2, tile_variant_part3,
                                                               tile_variant_part4};
        for (auto part : parts)
            if (Variant v = part(m->bits, m->tile_blocks, slots, nb, kgp)) return v;
        return Variant{};
    }
    if (m->bits == 4) {
        switch (m->G) {
            case 8: return pick_kernel<Fmt<4, 0>>(slots, nb, kgp);
            case 16: return pick_kernel<Fmt<4, 1>>(slots, nb, kgp);
            case 32: return pick_kernel<Fmt<4, 2>>(slots, nb, kgp);
            case 64: return pick_kernel<Fmt<4, 4>>(slots, nb, kgp);
            case 128: return pick_kernel<Fmt<4, 8>>(slots, nb, kgp);
        }
    } else if (m->bits == 8) {
        switch (m->G) {
            case 8: return pick_kernel<Fmt<8, 0>>(slots, nb, kgp);
            case 16: return pick_kernel<Fmt<8, 1>>(slots, nb, kgp);
            case 32: return pick_kernel<Fmt<8, 2>>(slots, nb, kgp);
            case 64: return pick_kernel<Fmt<8, 4>>(slots, nb, kgp);
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

gqsa_status_t scratch_address(int dev, void** out);      // (with the static workspace, below)

}  // namespace

gqsa_status_t device_upload(gqsa_matrix* m, void* filled_image)
{
    int kgp = 0;
    if (!pick(m, 1, &kgp)) return GQSA_ERR_UNSUPPORTED;   // K/16 above 2048: x does not fit the LDS layout
    int dev = 0;
    GQSA_HIP(hipGetDevice(&dev));
    for (int nb = 1; nb <= kMaxRowsPerLaunch; nb *= 2) {
        Variant v = pick(m, nb, &kgp);
        if (!v) continue;
        hipFuncAttributes attr{};
        GQSA_HIP(hipFuncGetAttributes(&attr, v.fn));
        if (attr.sharedSizeBytes != 0) return GQSA_ERR_HIP;      // the kernel addresses x from LDS offset 0
        if (lds_bytes(kgp, nb) > 64 * 1024)
            GQSA_HIP(hipFuncSetAttribute(v.fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         static_cast<int>(lds_bytes(kgp, nb))));
    }
    void* img = filled_image;
    void* carry = nullptr;
    if (!img) GQSA_HIP(hipMalloc(&img, m->image.size()));
    // carry records (per worker and activation row), one arrival counter per worker (padded to a
    // multiple of two), then the meeting points of two-worker chains (per worker and row)
    const size_t carry_bytes = carry_workspace_bytes(m->n_waves);
    hipError_t e = hipMalloc(&carry, carry_bytes);
    if (e == hipSuccess && !filled_image) e = hipMemcpy(img, m->image.data(), m->image.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(carry, 0, carry_bytes);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        std::fprintf(stderr, "libgqsa: upload failed: %s\n", hipGetErrorString(e));
        if (!filled_image) (void)hipFree(img);      // (a caller's image stays the caller's on failure)
        (void)hipFree(carry);
        return GQSA_ERR_HIP;
    }
    m->d_image = img;
    m->d_carry = carry;
    m->device = dev;
    // (the set-up call of a GPU is also where the address of the static workspace on it is learnt)
    void* unused = nullptr;
    (void)scratch_address(dev, &unused);
    return GQSA_OK;
}

void device_release(gqsa_matrix* m)
{
    if (m->d_image) (void)hipFree(m->d_image);
    if (m->d_carry) (void)hipFree(m->d_carry);
    m->d_image = nullptr;
    m->d_carry = nullptr;
}

namespace {

// Wavefronts per workgroup of a launch of nb activation rows on these matrices, 0 if they
// cannot share a launch.  One activation row: the partition's own grouping.  Several rows: x
// takes nb times the LDS, so fewer workgroups fit a compute unit; the workers are then taken 8
// or 16 to a workgroup -- as many as keep about 16 wavefronts on a compute unit -- where the
// worker counts allow and every compute unit still gets a workgroup (the deal of tiles to
// workers does not depend on the grouping).
int launch_waves_per_workgroup(gqsa_matrix* const* ms, int n_mats, int nb, size_t lds_per_workgroup)
{
    const int wpw = ms[0]->waves_per_workgroup;
    int workers = 0;
    for (int i = 0; i < n_mats; ++i) {
        if (ms[i]->waves_per_workgroup != wpw || ms[i]->tile_blocks != ms[0]->tile_blocks ||
            ms[i]->tile_lanes != ms[0]->tile_lanes)
            return 0;
        workers += ms[i]->n_waves;
    }
    if (nb == 1) return wpw;
    const int per_cu = static_cast<int>(std::max<size_t>(1, kMaxLdsBytes / lds_per_workgroup));
    int want = 1;
    while (want < kWavesPerWorkgroup && want * per_cu < kWavesPerWorkgroup) want *= 2;
    for (int bigger = want; bigger > wpw; bigger /= 2) {
        bool fits = workers / bigger >= kMaxDefaultWorkgroups;
        for (int i = 0; i < n_mats; ++i)
            if (ms[i]->n_waves % bigger != 0) fits = false;
        if (fits) return bigger;
    }
    return wpw;
}

// One launch: the kernel for nb activation rows (1, 2, 4 or 8), of which the caller has `rows`
// (nb, or one fewer), times n_mats matrices that share x and the wavefronts per workgroup.
gqsa_status_t launch(gqsa_matrix* const* ms, int n_mats, const uint16_t* x, uint16_t* const* ys, int nb, int rows, int wpw,
                     void* workspace, hipStream_t s)
{
    const gqsa_matrix* m0 = ms[0];
    int kgp = 0;
    const Variant v = pick(m0, nb, &kgp);
    if (!v) return GQSA_ERR_UNSUPPORTED;
    LaunchArgs a{};
    int wg_end[kMaxMatrices] = {INT_MAX, INT_MAX, INT_MAX, INT_MAX};
    int grid = 0;
    for (int i = 0; i < n_mats; ++i) {
        const gqsa_matrix* m = ms[i];
        const uint8_t* img = static_cast<const uint8_t*>(m->d_image);
        MatDesc& d = a.m[i];
        d.blocks = img + m->map.blocks;
        d.wave_info = reinterpret_cast<const int4_t*>(img + m->map.wave_info);
        d.magic = ((1ull << 48) + m->n_waves - 1) / m->n_waves;
        d.base = static_cast<int>(m->n_tiles / m->n_waves);
        d.extra = static_cast<int>(m->n_tiles % m->n_waves);
        d.n_wg = m->n_waves / wpw;
        MatArgs& o = d.out;
        o.row_of_rank = m->n_empty ? reinterpret_cast<const int32_t*>(img + m->map.row_of_rank) : nullptr;
        o.empty_rows = reinterpret_cast<const int32_t*>(img + m->map.empty_rows);
        uint8_t* ws = static_cast<uint8_t*>(workspace ? workspace : m->d_carry);
        o.carry = reinterpret_cast<CarryRecord*>(ws);
        o.counters = reinterpret_cast<int*>(ws + counters_offset(m->n_waves));
        o.slots = reinterpret_cast<unsigned long long*>(ws + slots_offset(m->n_waves));
        o.y = ys[i];
        o.N = static_cast<int>(m->N);
        o.last_row = rows - 1;
        o.n_empty = static_cast<int>(m->n_empty);
        o.n_ranks = static_cast<int>(m->N - m->n_empty);
        grid += d.n_wg;
        if (i + 1 < n_mats) wg_end[i] = grid;
    }
    const int kg_wpw_rows = static_cast<int>(m0->K / 16) | (wpw << 16) | (m0->tile_lanes << 21) | ((rows - 1) << 28);
    v.launch(a, x, kg_wpw_rows, wg_end, dim3(grid), dim3(wpw * kLanes), lds_bytes(kgp, nb), s);
    return GQSA_OK;
}

}  // namespace

gqsa_status_t device_gemv(gqsa_matrix* const* ms, int n_mats, const void* x, void* const* ys, int batch,
                          void* stream, void* workspace)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const gqsa_matrix* m0 = ms[0];
    // the device image, its workspace and the kernels' LDS attributes belong to one GPU
    int dev = -1;
    GQSA_HIP(hipGetDevice(&dev));
    for (int i = 0; i < n_mats; ++i)
        if (ms[i]->device != dev) return GQSA_ERR_HIP;
    // the batch goes out in launches of 8, 4, 2 or 1 rows: the most that the format has a
    // kernel for, fits LDS and is left -- except that 3 rows go to the kernel for 4 and 7 to the
    // kernel for 8 (measured: a launch for 4 rows takes less than launches for 2 and for 1;
    // with two rows missing the smaller launches win on the larger matrices)
    int done = 0;
    while (done < batch) {
        const int left = batch - done;
        int nb = kMaxRowsPerLaunch, kgp = 0, rows = 0;
        if ((left == 3 || left == 7) && pick(m0, left + 1, &kgp)) {
            nb = left + 1;
            rows = left;
        } else {
            for (; nb >= 1; nb /= 2) {
                if (nb <= left && pick(m0, nb, &kgp)) break;
            }
            rows = nb;
        }
        if (nb < 1) return GQSA_ERR_UNSUPPORTED;
        const uint16_t* xb = static_cast<const uint16_t*>(x) + static_cast<size_t>(done) * m0->K;
        uint16_t* yb[kMaxMatrices];
        for (int i = 0; i < n_mats; ++i) yb[i] = static_cast<uint16_t*>(ys[i]) + static_cast<size_t>(done) * ms[i]->N;
        const size_t lds = lds_bytes(kgp, nb);
        const int together = launch_waves_per_workgroup(ms, n_mats, nb, lds);
        if (together > 0) {
            // one launch for all the matrices
            if (gqsa_status_t st = launch(ms, n_mats, xb, yb, nb, rows, together, workspace, s)) return st;
        } else {
            for (int i = 0; i < n_mats; ++i) {
                const int wpw = launch_waves_per_workgroup(ms + i, 1, nb, lds);
                if (gqsa_status_t st = launch(ms + i, 1, xb, yb + i, nb, rows, wpw, workspace, s)) return st;
            }
        }
        done += rows;
    }
    GQSA_HIP(hipGetLastError());
    return GQSA_OK;
}

// ---------------------------------------------------------------------------------------------
// The same GEMV for callers that must not allocate (code under stream capture, serving loops,
// harnesses that forbid it): the fix-up workspace -- carry records, arrival counters, meeting
// points -- does not come from the handle's allocation but from an array that is part of the
// library's device code, one copy per GPU for the life of the process.
static_assert(kScratchBytes == carry_workspace_bytes(kScratchWorkers), "size of the static workspace");

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch[kMaxDevices];               // device address of `scratch` on every GPU seen so far
std::mutex g_scratch_mutex;

// The array's name is a host-side stand-in, not an address a kernel can use: the address on
// the current GPU is asked for once per GPU and kept.
gqsa_status_t scratch_address(int dev, void** out)
{
    if (dev < 0 || dev >= kMaxDevices) return GQSA_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch[dev]) {
        void* p = nullptr;
        GQSA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return GQSA_ERR_HIP;
        g_scratch[dev] = p;
    }
    *out = g_scratch[dev];
    return GQSA_OK;
}

__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t* p, unsigned n)
{
    for (unsigned i = blockIdx.x * 256u + threadIdx.x; i < n; i += gridDim.x * 256u) p[i] = 0u;
}

}  // namespace

gqsa_status_t device_gemv_static(gqsa_matrix* m, const void* x, void* y, int batch, void* stream)
{
    if (m->n_waves > kScratchWorkers) {
        std::fprintf(stderr, "libgqsa: gqsa_gemv_static: the handle's partition has %d wavefront workers, the static "
                             "workspace holds %d\n", m->n_waves, kScratchWorkers);
        return GQSA_ERR_BUFSIZE;
    }
    int dev = -1;
    GQSA_HIP(hipGetDevice(&dev));
    if (m->device != dev) return GQSA_ERR_HIP;
    void* ws = nullptr;
    if (gqsa_status_t st = scratch_address(dev, &ws)) return st;
    if (m->needs_fixup) {
        // The array keeps what the last call left.  A call that ran to its end leaves counters and
        // meeting points at zero, one that was cut short need not: clear this call's part of them
        // (with a kernel: a memset node must not end up in a captured graph).
        const size_t first = counters_offset(m->n_waves), bytes = carry_workspace_bytes(m->n_waves) - first;
        const unsigned words = static_cast<unsigned>(bytes / 4);
        hipLaunchKernelGGL(zero_words_kernel, dim3((words + 255u) / 256u), dim3(256), 0, static_cast<hipStream_t>(stream),
                           reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(ws) + first), words);
    }
    return device_gemv(&m, 1, x, &y, batch, stream, ws);
}

bool stream_is_capturing(void* stream)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(static_cast<hipStream_t>(stream), &st) != hipSuccess) return false;
    return st != hipStreamCaptureStatusNone;
}

}  // namespace gqsa

#endif  // GQSA_GEMV_PART == 0
