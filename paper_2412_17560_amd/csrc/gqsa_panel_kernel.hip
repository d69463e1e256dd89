// y[b, n] = sum_k W^[n, k] x[b, k] for up to 16 activation rows at once on the matrix cores, from
// the panel image (gqsa_panels.cpp): a panel's groups of one group-column, 16 rows x 16 weights
// with the pruned ones zero, times the 16 x 16 activations under them, is one 16x16x16 product.
// The dequantisation of Eq. 3 stays exact -- no weight is ever rounded to fp16 -- in both forms
// of the kernel (INTZ, chosen per matrix when the image is built):
//   - every stored zero is an integer of at most 1024 in magnitude (what Eq. 1 yields): the zero
//     is taken off the codes in fp16 before the product (q - z is an exact small integer there),
//     the matrix cores multiply it by x with fp32 accumulation, the scale is applied to the sum:
//         sum_j (q_j - z) s x_j  =  s * sum_j (q_j - z) x_j;
//   - any other zero (Sec. 3.4 trains scale and zero freely): the matrix cores multiply the codes
//     q themselves (exact in fp16) by x, a second product with a matrix of ones gives the sum of
//     the 16 activations, and scale and zero are applied to the two fp32 results per group:
//         sum_j (q_j - z) s x_j  =  s * (sum_j q_j x_j  -  z * sum_j x_j).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <type_traits>

#include "gqsa_internal.hpp"

namespace gqsa {
namespace {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kPanelsPerWorkgroup = 4;   // panels a workgroup takes at most (each needs its own sums)
constexpr int kInFlight = 4;          // group-columns whose products are under way together
constexpr int kPanelWaves = 16;      // wavefronts of a workgroup (or 8, see WAVES): each takes every 16th (8th) unit (a run of group-columns) of the panel
constexpr int kWaveLds = 9216;        // bytes of LDS a wavefront stages records in (16 x 9 KB = 144 of the 160 KB)
constexpr int kMaxUnitBytes = 3072;   // records of one panel in one unit, at most (16 rows x the unit's columns)

__device__ __forceinline__ float half_bits_to_float(uint32_t h)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
}

__device__ __forceinline__ uint16_t float_to_half_bits(float v)
{
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(v));     // round to nearest even
}

// Four codes -> four fp16 numbers, exactly: 0x6400 | q is the fp16 number 1024 + q (q < 1024), and
// 0x6400 | q << 4 is 1024 + 16 q, which one fused multiply-add turns into q (x 1/16, - 64: both
// steps exact).  `splice` = 0x64006400.  What is subtracted comes from the caller: 1024 and 64
// for the plain codes, 1024 + z and 64 + z for codes minus zero (exact for an integer z of at most
// 1024 in magnitude: every intermediate and the result are integers below 2048).
// 4-bit: `pair` holds the two bytes (e0 | e2 << 4), (e1 | e3 << 4) in bits 0..7 and 16..23;
// `nib` = 0x000F000F and `nib << 4`, kept in vector registers so that AND and OR are one instruction.
struct DecodeConstants {
    uint32_t splice, nib_lo, nib_hi;
    half2_t sixteenth;
};
__device__ __forceinline__ half4_t decode4_w4(uint32_t pair, const DecodeConstants& k, half2_t off_lo, half2_t off_hi)
{
    const uint32_t lo = (pair & k.nib_lo) | k.splice;            // 1024 + e0, 1024 + e1
    const uint32_t hi = (pair & k.nib_hi) | k.splice;            // 1024 + 16 e2, 1024 + 16 e3
    const half2_t a = __builtin_bit_cast(half2_t, lo) - off_lo;
    const half2_t b = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, hi), k.sixteenth, -off_hi);
    return half4_t{a.x, a.y, b.x, b.y};
}
// 8-bit: four bytes, one per element, in the word of the pair (upper, lower) that `sel` names:
// sel = 0x0c010c00 for the lower word, 0x0c050c04 for the upper one.
__device__ __forceinline__ half4_t decode4_w8(uint32_t upper, uint32_t lower, uint32_t sel, const DecodeConstants& k, half2_t off_lo)
{
    const uint32_t lo = __builtin_amdgcn_perm(upper, lower, sel) | k.splice;                  // bytes 0, 1
    const uint32_t hi = __builtin_amdgcn_perm(upper, lower, sel + 0x00020002u) | k.splice;    // bytes 2, 3
    const half2_t a = __builtin_bit_cast(half2_t, lo) - off_lo;
    const half2_t b = __builtin_bit_cast(half2_t, hi) - off_lo;
    return half4_t{a.x, a.y, b.x, b.y};
}

// The matrices of a launch: up to four that are multiplied with the same activations (q/k/v,
// gate/up: same K, group size and code width; N may differ).  Their panels are numbered through,
// matrix after matrix, so the panels of a workgroup (blockIdx.x, + gridDim.x, ...) may belong to
// different matrices and still share the activations they load.
// (The images themselves come as separate read-only kernel arguments: the compiler reads a
// block's header with scalar loads only from memory it knows nothing writes to.)
struct PanelTargets {
    uint16_t* y[kMaxMatricesPerLaunch];
    int N[kMaxMatricesPerLaunch];
    int first[kMaxMatricesPerLaunch];       // panels of the matrices before this one (entries past the last matrix: `total`)
    int total;                  // panels of all matrices
};

// A workgroup takes up to four panels of 16 output rows (blockIdx.x, + gridDim.x, ...); wavefront
// w takes the units w, w + 16, ... (a unit = a run of group-columns, half a slice or less) of
// every one of them, so the activations under a unit are loaded once for all of the workgroup's
// panels.  A block's header is the same for all lanes and is read with scalar loads.  The records
// of a panel in a unit are contiguous in the image; the wavefront copies them from global memory
// straight into its own part of LDS, 1 KiB per instruction with nothing passing through
// registers (all of its panels at once when they fit, else two and two), and every lane then
// reads its group's codes, scale and zero from there: which group is a lane's (its row's, in the
// column at hand) follows from the header with a masked population count.  Fetching 8 bytes per
// lane from global memory instead kept 1.5 KB per wavefront under way where this keeps 6 KB.
// No lane reads conditionally: one whose row has no group in a column reads a neighbouring
// record (or the bytes behind the last one), and what it computes from it stays in its own
// column of the product, which it then leaves out.  Likewise the activation rows beyond `batch`
// are copies of the last one: they only reach result rows that are never stored.
// Operands of v_mfma_f32_16x16x16_f16 in a wavefront: lane l holds A[l % 16][4 (l / 16) .. + 3],
// B[4 (l / 16) .. + 3][l % 16] and receives D[4 (l / 16) .. + 3][l % 16].  Here A = the
// activations (row = activation row, 16 elements of one group-column), B = the codes (column =
// output row of the panel), so a lane ends up with the sums of output row l % 16 for the
// activation rows 4 (l / 16) .. + 3 -- and the scale and zero it loaded with its codes are the
// ones those sums need.
// M = 16-element chunks per group (G = 16 M): a group-column then takes M products, chained
// through the accumulator input since they share scale and zero, and a wavefront's unit of work
// is 16 / M group-columns with 4-bit codes, 8 / M with 8-bit codes (so that 16 rows x the unit's
// columns are at most 3 KiB of records).
// INTZ: every zero of the matrix is an integer of at most 1024 in magnitude (what Eq. 1 produces,
// short of extreme groups): the zero is then taken off the codes before the product, exactly, so
// sum_j (q_j - z) x_j comes out of one product and only the scale is left to apply; otherwise the
// zero is an arbitrary fp16 number and multiplies the second product's sum of activations.
// MULTI: more than one matrix in the launch (the lookups of a panel's matrix cost scalar
// registers, which the headers of four panels already fill: one matrix keeps its own code).
// WAVES: 16 wavefronts per workgroup and one workgroup per compute unit, or -- for launches of
// more workgroups than compute units -- 8 and two: the loads of one then run under the products
// of the other (workgroups of 16 wavefronts can only follow one another, each loading, then
// computing).  Either way four wavefronts per SIMD unit, 128 vector registers each.
template <int BITS, int M, bool INTZ, bool MULTI, int WAVES>
__global__ __launch_bounds__(WAVES * kLanes, 4) void gqsa_panel_kernel(
    const uint16_t* __restrict__ x,
    const uint8_t* __restrict__ headers0, const uint8_t* __restrict__ headers1,
    const uint8_t* __restrict__ headers2, const uint8_t* __restrict__ headers3,
    const uint8_t* __restrict__ data0, const uint8_t* __restrict__ data1,
    const uint8_t* __restrict__ data2, const uint8_t* __restrict__ data3,
    const PanelTargets tgt, int K, int n_slices, int batch)
{
    constexpr int CB = 2 * BITS * M;                // code bytes per group
    constexpr bool PAIRED8 = BITS == 8 && M == 1;   // 8-bit, G = 16: quarter 0, word, quarter 1, quarter 2, word, quarter 3
    constexpr int RB = CB + (PAIRED8 ? 8 : 4);      // record: codes of quarters 0, 1 | scale, zero | codes of quarters 2, 3
    constexpr int QB = (BITS / 2) * M;              // code bytes of a lane (one quarter of every chunk)
    constexpr int QW = (QB + 3) / 4;                // ... in registers
    constexpr bool PAIRED = QB == 2;                // 4-bit, G = 16: a 12-byte record, read whole
    __shared__ __attribute__((aligned(16))) uint8_t staged[WAVES * kWaveLds];
    float* part = reinterpret_cast<float*>(staged);            // the same memory once the products are done
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wl = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint8_t* mine = staged + wl * kWaveLds;                     // this wavefront's staging area
    const int r = lane & 15;                        // activation row (A), output row of the panel (B, D)
    const int j = lane >> 4;                        // which four of a group's 16 elements
    const uint32_t below = (1u << r) - 1u;
    const uint16_t* xrow = x + static_cast<size_t>(r < batch ? r : batch - 1) * K + 8 * (j & 1);
    const int last_chunk = (K >> 4) - 1;
    DecodeConstants dk;       // (kept out of the compiler's sight as constants: it would split the AND-OR)
    asm volatile("s_mov_b32 %0, 0x64006400" : "=s"(dk.splice));
    asm volatile("v_mov_b32 %0, 0x000F000F" : "=v"(dk.nib_lo));
    asm volatile("v_mov_b32 %0, 0x00F000F0" : "=v"(dk.nib_hi));
    dk.sixteenth = half2_t{(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
    const half2_t k64 = {(_Float16)64.0f, (_Float16)64.0f};
    const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    const half4_t ones = {(_Float16)1.0f, (_Float16)1.0f, (_Float16)1.0f, (_Float16)1.0f};

    // the workgroup's panels: blockIdx.x, blockIdx.x + gridDim.x, ... (at most kPanelsPerWorkgroup),
    // each in its matrix; one past the last stands in as the last and is not computed
    const auto locate = [&](int pp, int& m, int& p) {
        const int v = static_cast<int>(blockIdx.x + pp * gridDim.x);
        const bool is_live = v < tgt.total;
        const int vc = is_live ? v : tgt.total - 1;
        if constexpr (MULTI) {
            // (selects among values at fixed places of the argument block: no load depends on another)
            static_assert(kMaxMatricesPerLaunch == 4, "written out for four matrices");
            const int f1 = tgt.first[1], f2 = tgt.first[2], f3 = tgt.first[3];
            m = (vc >= f1 ? 1 : 0) + (vc >= f2 ? 1 : 0) + (vc >= f3 ? 1 : 0);
            p = vc - (m == 0 ? 0 : m == 1 ? f1 : m == 2 ? f2 : f3);
        } else {
            m = 0;
            p = vc;
        }
        return is_live;
    };
    int mat[kPanelsPerWorkgroup], pan[kPanelsPerWorkgroup];
    bool live[kPanelsPerWorkgroup];
#pragma unroll
    for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp) live[pp] = locate(pp, mat[pp], pan[pp]);
    float acc[kPanelsPerWorkgroup][4];
#pragma unroll
    for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[pp][v] = 0.0f;
    constexpr int HC = (BITS == 4 ? 16 : 8) / M;    // group-columns of a unit: 16 rows x HC columns x RB bytes <= kMaxUnitBytes
    static_assert(HC >= 1 && kPanelRows * HC * RB <= kMaxUnitBytes, "a unit's records must fit their staging area");
    constexpr int XCH = HC * M;                     // 16-element chunks of activations under a unit
    constexpr int UPS = kSliceColumns / HC;         // units per slice
    constexpr int kFly = (INTZ || M > 1) ? kInFlight : 2;      // (two sums per column without INTZ: registers)
    constexpr int FLY = HC < kFly ? HC : kFly;
    // a lane supplies elements 0-3, 8-11, 4-7, 12-15 of every chunk for j = 0..3: quarters 0, 2, 1, 3
    const uint32_t quarter = 2u * (j & 1) + (j >> 1);
    const uint32_t code_lane = quarter * QB + (quarter >= 2 ? 4u : 0u);     // where its codes start in a record
    // PAIRED: a lane reads the whole 12-byte record (codes of quarters 0, 1 | scale, zero | codes of
    // quarters 2, 3); a byte permute with a selector that differs by lane puts the lane's two code
    // bytes, from the first or the third word, into bits 0..7 and 16..23
    // PAIRED8: a lane reads the 12 bytes (quarter, scale | zero, quarter) that hold its quarter; the
    // permutes of the decode take the code bytes from the first or the third word
    const uint32_t half_of_record = quarter >= 2 ? 12u : 0u;
    const uint32_t sel_codes = PAIRED8 ? 0x0c010c00u + (quarter & 1u) * 0x00040004u
                                       : 0x0c010c00u + (quarter & 1u) * 0x00020002u + (quarter >= 2 ? 0x00040004u : 0u);
    for (int unit = wl; unit < UPS * n_slices; unit += WAVES) {
        const int s = unit / UPS;
        const int sub = unit % UPS;
        const int col0 = s * kSliceColumns + sub * HC;
        // The activations under these columns (XCH chunks of 16), once for all panels of the
        // workgroup, with 16-byte loads: of two neighbouring chunks the lanes 0..31 load the first
        // (elements 0-7 and 8-15 of it), the lanes 32..63 the second, and a swap between the two
        // halves of the wavefront hands every lane the four elements it supplies to a product:
        // elements 0-3, 8-11, 4-7, 12-15 of the chunk for the lanes' j = 0..3 (which element sits in
        // which of the product's 16 slots does not matter as long as the codes follow suit).
        // The last slice may be short: chunks beyond K (no groups there) take the last one's.
        // (The loads are issued here, ahead of everything; the swap waits until the records' loads
        // have been issued too, so that nothing is held up by the activations' arrival.)
        uint2 xa[HC][M];
        uint4 xw[XCH / 2];
#pragma unroll
        for (int pr = 0; pr < XCH / 2; ++pr) {
            const int g = col0 * M + 2 * pr + (j >> 1);
            xw[pr] = *reinterpret_cast<const uint4*>(xrow + 16 * (g < last_chunk ? g : last_chunk));
        }
        // the headers of all the workgroup's panels at once (scalar loads; a panel beyond the
        // last one stands in as the last one and is not computed)
        // (where 4 x HC words do not fit the scalar registers -- AGAIN -- only the first and the
        // last column's word of each panel are read here, and all of a panel's words a second
        // time, from the scalar cache, when its products start)
        constexpr bool AGAIN = kPanelsPerWorkgroup * HC > 32;
        uint32_t hh_all[AGAIN ? 1 : kPanelsPerWorkgroup][AGAIN ? 1 : HC];
        uint32_t header_at[kPanelsPerWorkgroup];        // byte offset of the unit's first word in the panel's matrix's headers
        uint32_t h_first[kPanelsPerWorkgroup], h_last[kPanelsPerWorkgroup], where[kPanelsPerWorkgroup];
#pragma unroll
        for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp) {
            // (the choice is made here, at the load: a header is read with scalar loads only if the
            // compiler can trace its address to a read-only argument)
            const uint8_t* headers = !MULTI || mat[pp] == 0 ? headers0 : mat[pp] == 1 ? headers1 : mat[pp] == 2 ? headers2 : headers3;
            const uint32_t* header = reinterpret_cast<const uint32_t*>(
                headers + static_cast<size_t>(pan[pp] * n_slices + s) * kPanelHeaderBytes);
            header_at[pp] = static_cast<uint32_t>((pan[pp] * n_slices + s) * kPanelHeaderBytes + sub * HC * 4);
            if constexpr (!AGAIN) {
#pragma unroll
                for (int c = 0; c < HC; ++c) hh_all[pp][c] = header[sub * HC + c];
            }
            h_first[pp] = header[sub * HC];
            h_last[pp] = header[sub * HC + HC - 1];
            where[pp] = header[32];
        }
        // Where each panel's records of this unit lie (they are contiguous: first group of the
        // first column .. last group of the last column) and where they go in the wavefront's
        // staging area: one after the other, each rounded up to 16 bytes plus room for one more
        // record (a lane without a group may read the one behind the last).  All four panels are
        // staged at once when they fit, else two and two.
        constexpr uint32_t kSpare = (RB + 15u) & ~15u;
        static_assert(2 * (kMaxUnitBytes + kSpare) <= kWaveLds, "two panels' worth must fit a wavefront's staging area");
        uint32_t first[kPanelsPerWorkgroup], bytes[kPanelsPerWorkgroup], room[kPanelsPerWorkgroup], slot[kPanelsPerWorkgroup];
#pragma unroll
        for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp) {
            const uint32_t last = h_last[pp];
            first[pp] = h_first[pp] >> 16;
            bytes[pp] = ((last >> 16) + __builtin_popcount(last & 0xFFFFu) - first[pp]) * RB;     // <= kMaxUnitBytes
            room[pp] = ((bytes[pp] + 15u) & ~15u) + kSpare;
        }
        const bool two_and_two = room[0] + room[1] + room[2] + room[3] > static_cast<uint32_t>(kWaveLds);
        slot[0] = 0;
        slot[1] = room[0];
        slot[2] = two_and_two ? 0 : room[0] + room[1];
        slot[3] = slot[2] + room[2];
#pragma unroll
        for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp) {
            if (pp == 0 || (pp == 2 && two_and_two)) {
                // stage: every lane copies 16 bytes per KiB of a panel's records, global memory ->
                // LDS directly (lane l's bytes land at the given LDS address + 16 l), no registers
#pragma unroll
                for (int q = pp; q < kPanelsPerWorkgroup; ++q) {
                    if (live[q] && (q < pp + 2 || !two_and_two)) {
                        const uint8_t* data = !MULTI || mat[q] == 0 ? data0 : mat[q] == 1 ? data1 : mat[q] == 2 ? data2 : data3;
                        const uint8_t* from = data + static_cast<size_t>(where[q]) * 16 + first[q] * RB;
#pragma unroll
                        for (int i = 0; i < kMaxUnitBytes / 1024; ++i) {
                            const uint32_t o = 16u * lane + 1024u * i;
                            if (o < bytes[q])
                                __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(from + o),
                                                                 (__attribute__((address_space(3))) void*)(mine + slot[q] + 1024u * i),
                                                                 16, 0, 0);
                        }
                    }
                }
                if (pp == 0) {
                    uint2* flat = &xa[0][0];
#pragma unroll
                    for (int pr = 0; pr < XCH / 2; ++pr) {
                        const auto s0 = __builtin_amdgcn_permlane32_swap(xw[pr].x, xw[pr].z, false, false);
                        const auto s1 = __builtin_amdgcn_permlane32_swap(xw[pr].y, xw[pr].w, false, false);
                        flat[2 * pr] = uint2{s0[0], s1[0]};
                        flat[2 * pr + 1] = uint2{s0[1], s1[1]};
                    }
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the records are in LDS before any lane reads them
            }
            if (live[pp]) {                             // (the same for the whole workgroup)
                const uint8_t* records = mine + slot[pp];           // in LDS
                const uint32_t before0 = first[pp];
                uint32_t hh[HC];
                if constexpr (!AGAIN) {
#pragma unroll
                    for (int c = 0; c < HC; ++c) hh[c] = hh_all[pp][c];
                } else {
                    uint32_t at = header_at[pp];
                    asm volatile("" : "+s"(at));            // (a read of its own, not the values kept from above)
                    const uint8_t* headers = !MULTI || mat[pp] == 0 ? headers0 : mat[pp] == 1 ? headers1 : mat[pp] == 2 ? headers2 : headers3;
                    const uint32_t* again = reinterpret_cast<const uint32_t*>(headers + at);
#pragma unroll
                    for (int c = 0; c < HC; ++c) hh[c] = again[c];
                }
                uint32_t code[HC][(PAIRED || PAIRED8) ? 2 : QW], sz[HC];
                constexpr bool TRI = PAIRED || PAIRED8;     // three words, the middle one is scale | zero as it is: the whole 12-byte
                                                            // record, or the half of the 24-byte one that holds the lane's quarter
#pragma unroll
                for (int c = 0; c < HC; ++c) {
                    const uint32_t h = hh[c];
                    const uint32_t idx = ((h >> 16) - before0) + __builtin_popcount(h & 0xFFFFu & below);
                    if constexpr (TRI) {
                        const uint32_t* w = reinterpret_cast<const uint32_t*>(records + (idx * RB + (PAIRED8 ? half_of_record : 0u)));
                        code[c][0] = w[0];
                        sz[c] = w[1];
                        code[c][1] = w[2];
                    } else {
                        const uint32_t* w = reinterpret_cast<const uint32_t*>(records + (idx * RB + code_lane));
#pragma unroll
                        for (int t = 0; t < QW; ++t) code[c][t] = w[t];
                        sz[c] = *reinterpret_cast<const uint32_t*>(records + (idx * RB + CB / 2));
                    }
                }
                // four columns at a time: the products of the later ones are under way while the
                // first one's sums are scaled.  Which lanes have a group in a column is a lane
                // mask made from the header word with scalar arithmetic (bit r -> lanes r, r + 16, ...)
#pragma unroll
                for (int c = 0; c < HC; c += FLY) {
                    float4_t d[FLY], e[FLY];
                    uint32_t sz_word[FLY];
#pragma unroll
                    for (int i = 0; i < FLY; ++i) {
                        sz_word[i] = sz[c + i];
                        half2_t off_lo = k1024, off_hi = k64;
                        if constexpr (INTZ) {
                            const half2_t both = __builtin_bit_cast(half2_t, sz_word[i]);
                            const half2_t zz = {both.y, both.y};
                            off_lo = k1024 + zz;
                            off_hi = k64 + zz;
                        }
                        d[i] = zero4;
                        e[i] = zero4;
#pragma unroll
                        for (int k = 0; k < M; ++k) {
                            const half4_t a = __builtin_bit_cast(half4_t, xa[c + i][k]);
                            half4_t q;
                            if constexpr (PAIRED8) {
                                q = decode4_w8(code[c + i][1], code[c + i][0], sel_codes, dk, off_lo);
                            } else if constexpr (PAIRED) {
                                q = decode4_w4(__builtin_amdgcn_perm(code[c + i][1], code[c + i][0], sel_codes), dk, off_lo, off_hi);   // (same selectors: bytes 0..3 = word 0, 4..7 = word 2)
                            } else if constexpr (BITS == 4) {     // chunk k: two bytes, the lower or the upper half of a word
                                q = decode4_w4(__builtin_amdgcn_perm(0u, code[c + i][k / 2], (k & 1) ? 0x0c030c02u : 0x0c010c00u), dk, off_lo, off_hi);
                            } else {
                                q = decode4_w8(0u, code[c + i][k], 0x0c010c00u, dk, off_lo);
                            }
                            d[i] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, q, d[i], 0, 0, 0);      // sum_j q_j x_j, or sum_j (q_j - z) x_j
                            if constexpr (!INTZ) e[i] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, ones, e[i], 0, 0, 0);   // sum_j x_j
                        }
                    }
#pragma unroll
                    for (int i = 0; i < FLY; ++i) {
                        const unsigned long long lanes = static_cast<unsigned long long>(hh[c + i] & 0xFFFFu) * 0x0001000100010001ull;
                        if (__builtin_amdgcn_inverse_ballot_w64(lanes)) {
                            const float sc = half_bits_to_float(sz_word[i] & 0xFFFFu);
                            if constexpr (INTZ) {
#pragma unroll
                                for (int v = 0; v < 4; ++v) acc[pp][v] = __builtin_fmaf(sc, d[i][v], acc[pp][v]);
                            } else {
                                const float z = half_bits_to_float(sz_word[i] >> 16);
#pragma unroll
                                for (int v = 0; v < 4; ++v)
                                    acc[pp][v] = __builtin_fmaf(sc, __builtin_fmaf(-z, e[i][v], d[i][v]), acc[pp][v]);
                            }
                        }
                    }
                }
            }
        }
    }

    // The wavefronts' sums meet in LDS (the staging areas, once every wavefront is done with its
    // own): all panels' at once, then the wavefronts share out the (panel, accumulator register)
    // pairs: pair t = the activation rows 4 j + (t % 4) of panel t / 4, whose contributions are
    // added in wavefront order and stored.
    static_assert(kPanelsPerWorkgroup * WAVES * 4 * kLanes * sizeof(float) <= sizeof(staged), "the sums must fit the staging areas");
    __syncthreads();
#pragma unroll
    for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp) {
        if (!live[pp]) break;                           // (the same for the whole workgroup)
#pragma unroll
        for (int v = 0; v < 4; ++v) part[((pp * 4 + v) * WAVES + wl) * kLanes + lane] = acc[pp][v];
    }
    __syncthreads();
    for (int t = wl; t < 4 * kPanelsPerWorkgroup; t += WAVES) {      // t = (panel, accumulator register)
        const int pp = t >> 2, v = t & 3;
        int m, p;
        if (locate(pp, m, p)) {
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) sum += part[(t * WAVES + w) * kLanes + lane];
            const int b = 4 * j + v;                    // activation row
            const int row = p * kPanelRows + r;         // output row
            const int n = !MULTI || m == 0 ? tgt.N[0] : m == 1 ? tgt.N[1] : m == 2 ? tgt.N[2] : tgt.N[3];
            uint16_t* y = !MULTI || m == 0 ? tgt.y[0] : m == 1 ? tgt.y[1] : m == 2 ? tgt.y[2] : tgt.y[3];
            if (b < batch && row < n) y[static_cast<size_t>(b) * n + row] = float_to_half_bits(sum);
        }
    }
}

}  // namespace

#define GQSA_HIP(call)                                                                   \
    do {                                                                                 \
        const hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) {                                                          \
            std::fprintf(stderr, "libgqsa: %s: %s\n", #call, hipGetErrorString(e_));    \
            return GQSA_ERR_HIP;                                                         \
        }                                                                                \
    } while (0)

gqsa_status_t panels_upload(gqsa_matrix* m)
{
    if (m->panel_image.empty() || m->d_panels) return GQSA_OK;
    void* img = nullptr;
    GQSA_HIP(hipMalloc(&img, m->panel_image.size()));
    const hipError_t e = hipMemcpy(img, m->panel_image.data(), m->panel_image.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        std::fprintf(stderr, "libgqsa: upload failed: %s\n", hipGetErrorString(e));
        (void)hipFree(img);
        return GQSA_ERR_HIP;
    }
    m->d_panels = img;
    return GQSA_OK;
}

void panels_release(gqsa_matrix* m)
{
    if (m->d_panels) (void)hipFree(m->d_panels);
    m->d_panels = nullptr;
}

// Up to 16 activation rows in one launch, for up to four matrices that share them (same K, group
// size, code width and handling of the zero; the caller checks).  x [batch, K], ys[i] [batch, N_i],
// fp16, on the device.
gqsa_status_t panels_gemm(const gqsa_matrix* const* ms, int n, const void* x, void* const* ys, int batch, void* stream)
{
    if (n < 1 || n > kMaxMatricesPerLaunch || batch < 1 || batch > kPanelRows) return GQSA_ERR_UNSUPPORTED;
    // the images belong to the GPU they were uploaded on
    int dev = -1;
    GQSA_HIP(hipGetDevice(&dev));
    for (int i = 0; i < n; ++i)
        if (ms[i]->device != dev) return GQSA_ERR_HIP;
    PanelTargets tgt{};
    const uint8_t* headers[kMaxMatricesPerLaunch];
    const uint8_t* data[kMaxMatricesPerLaunch];
    int64_t total = 0;
    for (int i = 0; i < n; ++i) {
        const gqsa_matrix* m = ms[i];
        if (!m->d_panels) return GQSA_ERR_UNSUPPORTED;
        if (m->K != ms[0]->K || m->G != ms[0]->G || m->bits != ms[0]->bits || m->n_slices != ms[0]->n_slices ||
            m->panel_integer_zeros != ms[0]->panel_integer_zeros)
            return GQSA_ERR_SHAPE;
        const uint8_t* img = static_cast<const uint8_t*>(m->d_panels);
        headers[i] = img;
        data[i] = img + m->panel_blocks_offset;
        tgt.y[i] = static_cast<uint16_t*>(ys[i]);
        tgt.N[i] = static_cast<int>(m->N);
        tgt.first[i] = static_cast<int>(total);
        total += m->n_panels;
    }
    if (total > INT32_MAX) return GQSA_ERR_SHAPE;
    for (int i = n; i < kMaxMatricesPerLaunch; ++i) {
        tgt.first[i] = static_cast<int>(total);
        headers[i] = headers[0];
        data[i] = data[0];
    }
    tgt.total = static_cast<int>(total);
    const gqsa_matrix* m = ms[0];
    // one workgroup per compute unit unless that gives a workgroup more than four panels
    const int64_t wgs = std::min<int64_t>(total, std::max<int64_t>(kMaxDefaultWorkgroups,
                                                                   (total + kPanelsPerWorkgroup - 1) / kPanelsPerWorkgroup));
    // more workgroups than compute units: smaller ones, two to a compute unit (see WAVES)
    const bool halves = n == 1 && wgs > kMaxDefaultWorkgroups;
    const dim3 grid(static_cast<unsigned>(wgs)), block((halves ? kPanelWaves / 2 : kPanelWaves) * kLanes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, block, 0, s, static_cast<const uint16_t*>(x), headers[0], headers[1], headers[2],
                           headers[3], data[0], data[1], data[2], data[3], tgt, static_cast<int>(m->K),
                           static_cast<int>(m->n_slices), batch);
    };
    const auto pick = [&](auto multi, auto waves) {
        constexpr bool kMulti = decltype(multi)::value;
        constexpr int kWaves = decltype(waves)::value;
        switch (m->bits * 1000 + m->G + (m->panel_integer_zeros ? 500 : 0)) {
            case 4016: launch(gqsa_panel_kernel<4, 1, false, kMulti, kWaves>); break;
            case 4032: launch(gqsa_panel_kernel<4, 2, false, kMulti, kWaves>); break;
            case 4064: launch(gqsa_panel_kernel<4, 4, false, kMulti, kWaves>); break;
            case 4128: launch(gqsa_panel_kernel<4, 8, false, kMulti, kWaves>); break;
            case 8016: launch(gqsa_panel_kernel<8, 1, false, kMulti, kWaves>); break;
            case 8032: launch(gqsa_panel_kernel<8, 2, false, kMulti, kWaves>); break;
            case 8064: launch(gqsa_panel_kernel<8, 4, false, kMulti, kWaves>); break;
            case 4516: launch(gqsa_panel_kernel<4, 1, true, kMulti, kWaves>); break;
            case 4532: launch(gqsa_panel_kernel<4, 2, true, kMulti, kWaves>); break;
            case 4564: launch(gqsa_panel_kernel<4, 4, true, kMulti, kWaves>); break;
            case 4628: launch(gqsa_panel_kernel<4, 8, true, kMulti, kWaves>); break;
            case 8516: launch(gqsa_panel_kernel<8, 1, true, kMulti, kWaves>); break;
            case 8532: launch(gqsa_panel_kernel<8, 2, true, kMulti, kWaves>); break;
            case 8564: launch(gqsa_panel_kernel<8, 4, true, kMulti, kWaves>); break;
            default: return false;
        }
        return true;
    };
    using Whole = std::integral_constant<int, kPanelWaves>;
    using Half = std::integral_constant<int, kPanelWaves / 2>;
    const bool ok = n > 1 ? pick(std::true_type{}, Whole{})
                          : (halves ? pick(std::false_type{}, Half{}) : pick(std::false_type{}, Whole{}));
    if (!ok) return GQSA_ERR_UNSUPPORTED;
    GQSA_HIP(hipGetLastError());
    return GQSA_OK;
}

}  // namespace gqsa
