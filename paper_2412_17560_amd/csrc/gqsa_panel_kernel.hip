// y[b, n] = sum_k W^[n, k] x[b, k] for up to 16 activation rows at once on the matrix cores, from
// the panel image (gqsa_panels.cpp): a panel's groups of one group-column, 16 rows x 16 weights
// with the pruned ones zero, times the 16 x 16 activations under them, is one 16x16x16 product.
// The dequantisation of Eq. 3 stays exact: the matrix cores multiply the integer codes q (exact
// in fp16) by x with fp32 accumulation, and a second product with a matrix of ones gives the sum
// of the 16 activations; scale and zero are applied to the two fp32 results per group,
//     sum_j (q_j - z) s x_j  =  s * (sum_j q_j x_j  -  z * sum_j x_j),
// so no weight is ever rounded to fp16.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>

#include "gqsa_internal.hpp"

namespace gqsa {
namespace {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kPanelsPerWorkgroup = 4;   // panels a workgroup takes at most (each needs its own sums)
constexpr int kInFlight = 4;          // group-columns whose products are under way together
constexpr int kPanelWaves = 16;      // wavefronts of a workgroup: each takes every 16th half-slice of the panel

__device__ __forceinline__ float half_bits_to_float(uint32_t h)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
}

__device__ __forceinline__ uint16_t float_to_half_bits(float v)
{
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(v));     // round to nearest even
}

// Four codes -> four fp16 integers, exactly: 0x6400 | q is the fp16 number 1024 + q (q < 1024).
// `splice` = 0x64006400 in a register (an AND-OR takes one literal, and the nibble mask is it).
// 4-bit: `pair` holds the two bytes (e0 | e2 << 4), (e1 | e3 << 4) in bits 0..7 and 16..23.
__device__ __forceinline__ half4_t decode4_w4(uint32_t pair, uint32_t splice)
{
    const uint32_t lo = (pair & 0x000F000Fu) | splice;            // e0, e1
    const uint32_t hi = ((pair >> 4) & 0x000F000Fu) | splice;     // e2, e3
    const half2_t bias = {(_Float16)1024.0f, (_Float16)1024.0f};
    const half2_t a = __builtin_bit_cast(half2_t, lo) - bias;
    const half2_t b = __builtin_bit_cast(half2_t, hi) - bias;
    return half4_t{a.x, a.y, b.x, b.y};
}
// 8-bit: four bytes, one per element, in the word of the pair (upper, lower) that `sel` names:
// sel = 0x0c010c00 for the lower word, 0x0c050c04 for the upper one.
__device__ __forceinline__ half4_t decode4_w8(uint32_t upper, uint32_t lower, uint32_t sel, uint32_t splice)
{
    const uint32_t lo = __builtin_amdgcn_perm(upper, lower, sel) | splice;                  // bytes 0, 1
    const uint32_t hi = __builtin_amdgcn_perm(upper, lower, sel + 0x00020002u) | splice;    // bytes 2, 3
    const half2_t bias = {(_Float16)1024.0f, (_Float16)1024.0f};
    const half2_t a = __builtin_bit_cast(half2_t, lo) - bias;
    const half2_t b = __builtin_bit_cast(half2_t, hi) - bias;
    return half4_t{a.x, a.y, b.x, b.y};
}

// A workgroup takes up to four panels of 16 output rows (blockIdx.x, + gridDim.x, ...); wavefront
// w takes the half-slices w, w + 16, ... (16 group-columns each) of every one of them, so the
// activations under a half-slice are loaded once for all of the workgroup's panels.  A block's
// header is the same for all lanes and is read with scalar loads; which group is a lane's (its
// row's, in the column at hand) follows from the header with a masked population count.  Nothing is loaded
// conditionally: a lane whose row has no group in a column reads a neighbouring group (the image
// ends with spare bytes), and what it computes from it stays in its own column of the product,
// which it then leaves out.  Likewise the activation rows beyond `batch` are copies of the last
// one: they only reach result rows that are never stored.
// Operands of v_mfma_f32_16x16x16_f16 in a wavefront: lane l holds A[l % 16][4 (l / 16) .. + 3],
// B[4 (l / 16) .. + 3][l % 16] and receives D[4 (l / 16) .. + 3][l % 16].  Here A = the
// activations (row = activation row, 16 elements of one group-column), B = the codes (column =
// output row of the panel), so a lane ends up with the sums of output row l % 16 for the
// activation rows 4 (l / 16) .. + 3 -- and the scale and zero it loaded with its codes are the
// ones those sums need.
// M = 16-element chunks per group (G = 16 M): a group-column then takes M products, chained
// through the accumulator input since they share scale and zero, and a wavefront's unit of work
// is 16 / M group-columns (a slice of 32 has 2 M of them).
template <int BITS, int M>
__global__ __launch_bounds__(kPanelWaves * kLanes) void gqsa_panel_kernel(
    const uint16_t* __restrict__ x, const uint8_t* __restrict__ headers, const uint8_t* __restrict__ data,
    uint16_t* __restrict__ y, int N, int K, int n_slices, int batch, int n_panels)
{
    constexpr int CB = 2 * BITS * M;                // code bytes per group
    constexpr bool PAIRED8 = BITS == 8 && M == 1;   // 8-bit, G = 16: quarter 0, word, quarter 1, quarter 2, word, quarter 3
    constexpr int RB = CB + (PAIRED8 ? 8 : 4);      // record: codes of quarters 0, 1 | scale, zero | codes of quarters 2, 3
    constexpr int QB = (BITS / 2) * M;              // code bytes of a lane (one quarter of every chunk)
    constexpr int QW = (QB + 3) / 4;                // ... in registers
    constexpr bool PAIRED = QB == 2;                // 4-bit, G = 16: codes and scale, zero in one 8-byte load
    __shared__ float part[kPanelWaves * 4 * kLanes];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wl = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15;                        // activation row (A), output row of the panel (B, D)
    const int j = lane >> 4;                        // which four of a group's 16 elements
    const uint32_t below = (1u << r) - 1u;
    const uint16_t* xrow = x + static_cast<size_t>(r < batch ? r : batch - 1) * K + 8 * (j & 1);
    const int last_chunk = (K >> 4) - 1;
    uint32_t splice;
    asm volatile("s_mov_b32 %0, 0x64006400" : "=s"(splice));     // (kept out of the compiler's sight as a constant)
    const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    const half4_t ones = {(_Float16)1.0f, (_Float16)1.0f, (_Float16)1.0f, (_Float16)1.0f};

    // the workgroup's panels: blockIdx.x, blockIdx.x + gridDim.x, ... (at most kPanelsPerWorkgroup)
    float acc[kPanelsPerWorkgroup][4];
#pragma unroll
    for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[pp][v] = 0.0f;
    constexpr int HC = 16 / M;                      // group-columns of a unit
    constexpr int UPS = kSliceColumns / HC;         // units per slice
    constexpr int FLY = HC < kInFlight ? HC : kInFlight;
    // a lane supplies elements 0-3, 8-11, 4-7, 12-15 of every chunk for j = 0..3: quarters 0, 2, 1, 3
    const uint32_t quarter = 2u * (j & 1) + (j >> 1);
    const uint32_t code_lane = quarter * QB + (quarter >= 2 ? 4u : 0u);     // where its codes start in a record
    // PAIRED: lanes of quarters 0, 1 load bytes 0..7 of the 12-byte record (codes, then scale | zero),
    // lanes of quarters 2, 3 bytes 4..11 (scale | zero, then codes); a byte permute with a selector
    // that differs by lane puts the lane's two code bytes into bits 0..7 and 16..23, another one
    // picks the scale | zero word
    // PAIRED8: quarters 0 and 2 load (codes, word), quarters 1 and 3 (word, codes); the permutes of
    // the decode take the code bytes from whichever of the two it is
    const uint32_t pair_load = PAIRED8 ? 4u * quarter + (quarter >= 2 ? 4u : 0u) : (quarter >= 2 ? 4u : 0u);
    const uint32_t sel_codes = PAIRED8 ? 0x0c010c00u + (quarter & 1u) * 0x00040004u
                                       : 0x0c010c00u + (quarter & 1u) * 0x00020002u + (quarter >= 2 ? 0x00040004u : 0u);
    const uint32_t sel_sz = PAIRED8 ? ((quarter & 1u) ? 0x03020100u : 0x07060504u)
                                    : (quarter >= 2 ? 0x03020100u : 0x07060504u);
    for (int unit = wl; unit < UPS * n_slices; unit += kPanelWaves) {
        const int s = unit / UPS;
        const int sub = unit % UPS;
        const int col0 = s * kSliceColumns + sub * HC;
        // The activations under these columns (16 chunks of 16), once for all panels of the
        // workgroup, with 16-byte loads: of two neighbouring chunks the lanes 0..31 load the first
        // (elements 0-7 and 8-15 of it), the lanes 32..63 the second, and a swap between the two
        // halves of the wavefront hands every lane the four elements it supplies to a product:
        // elements 0-3, 8-11, 4-7, 12-15 of the chunk for the lanes' j = 0..3 (which element sits in
        // which of the product's 16 slots does not matter as long as the codes follow suit).
        // The last slice may be short: chunks beyond K (no groups there) take the last one's.
        uint2 xa[HC][M];
        {
            const int chunk0 = col0 * M;
            uint2* flat = &xa[0][0];
#pragma unroll
            for (int pr = 0; pr < 8; ++pr) {
                const int g = chunk0 + 2 * pr + (j >> 1);
                const uint4 w = *reinterpret_cast<const uint4*>(xrow + 16 * (g < last_chunk ? g : last_chunk));
                const auto s0 = __builtin_amdgcn_permlane32_swap(w.x, w.z, false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(w.y, w.w, false, false);
                flat[2 * pr] = uint2{s0[0], s1[0]};
                flat[2 * pr + 1] = uint2{s0[1], s1[1]};
            }
        }
        // the headers of all the workgroup's panels at once (scalar loads; a panel beyond the
        // last one stands in as the last one and is not computed)
        uint32_t hh[kPanelsPerWorkgroup][HC], where[kPanelsPerWorkgroup];
#pragma unroll
        for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp) {
            const int p = blockIdx.x + pp * gridDim.x;
            const uint32_t* header = reinterpret_cast<const uint32_t*>(
                headers + static_cast<size_t>((p < n_panels ? p : n_panels - 1) * n_slices + s) * kPanelHeaderBytes);
#pragma unroll
            for (int c = 0; c < HC; ++c) hh[pp][c] = header[sub * HC + c];
            where[pp] = header[32];
        }
#pragma unroll
        for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp) {
            const int p = blockIdx.x + pp * gridDim.x;
            if (p < n_panels) {                         // (the same for the whole workgroup)
                const uint8_t* records = data + static_cast<size_t>(where[pp]) * 16;
                uint32_t code[HC][(PAIRED || PAIRED8) ? 2 : QW], sz[HC];
#pragma unroll
                for (int c = 0; c < HC; ++c) {
                    const uint32_t h = hh[pp][c];
                    const uint32_t idx = (h >> 16) + __builtin_popcount(h & 0xFFFFu & below);
                    if constexpr (PAIRED || PAIRED8) {
                        const uint2 w = *reinterpret_cast<const uint2*>(records + (idx * RB + pair_load));
                        code[c][0] = w.x;
                        code[c][1] = w.y;
                    } else {
                        const uint8_t* mine = records + (idx * RB + code_lane);
                        if constexpr (QW == 1) {
                            code[c][0] = *reinterpret_cast<const uint32_t*>(mine);
                        } else if constexpr (QW == 2) {
                            const uint2 w = *reinterpret_cast<const uint2*>(mine);
                            code[c][0] = w.x; code[c][1] = w.y;
                        } else {
                            const uint4 w = *reinterpret_cast<const uint4*>(mine);
                            code[c][0] = w.x; code[c][1] = w.y; code[c][2] = w.z; code[c][3] = w.w;
                        }
                        sz[c] = *reinterpret_cast<const uint32_t*>(records + (idx * RB + CB / 2));
                    }
                }
                // four columns at a time: the products of the later ones are under way while the
                // first one's sums are scaled.  Which lanes have a group in a column is a lane
                // mask made from the header word with scalar arithmetic (bit r -> lanes r, r + 16, ...)
#pragma unroll
                for (int c = 0; c < HC; c += FLY) {
                    float4_t d[FLY], e[FLY];
#pragma unroll
                    for (int i = 0; i < FLY; ++i) {
                        d[i] = zero4;
                        e[i] = zero4;
#pragma unroll
                        for (int k = 0; k < M; ++k) {
                            const half4_t a = __builtin_bit_cast(half4_t, xa[c + i][k]);
                            half4_t q;
                            if constexpr (PAIRED8) {
                                q = decode4_w8(code[c + i][1], code[c + i][0], sel_codes, splice);
                            } else if constexpr (PAIRED) {
                                q = decode4_w4(__builtin_amdgcn_perm(code[c + i][1], code[c + i][0], sel_codes), splice);
                            } else if constexpr (BITS == 4) {     // chunk k: two bytes, the lower or the upper half of a word
                                q = decode4_w4(__builtin_amdgcn_perm(0u, code[c + i][k / 2], (k & 1) ? 0x0c030c02u : 0x0c010c00u), splice);
                            } else {
                                q = decode4_w8(0u, code[c + i][k], 0x0c010c00u, splice);
                            }
                            d[i] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, q, d[i], 0, 0, 0);      // sum_j q_j x_j
                            e[i] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, ones, e[i], 0, 0, 0);   // sum_j x_j
                        }
                    }
#pragma unroll
                    for (int i = 0; i < FLY; ++i) {
                        const unsigned long long lanes = static_cast<unsigned long long>(hh[pp][c + i] & 0xFFFFu) * 0x0001000100010001ull;
                        if (__builtin_amdgcn_inverse_ballot_w64(lanes)) {
                            uint32_t sz_word;
                            if constexpr (PAIRED || PAIRED8) sz_word = __builtin_amdgcn_perm(code[c + i][1], code[c + i][0], sel_sz);
                            else sz_word = sz[c + i];
                            const float sc = half_bits_to_float(sz_word & 0xFFFFu);
                            const float z = half_bits_to_float(sz_word >> 16);
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                acc[pp][v] = __builtin_fmaf(sc, __builtin_fmaf(-z, e[i][v], d[i][v]), acc[pp][v]);
                        }
                    }
                }
            }
        }
    }

    // the wavefronts' sums meet in LDS and are added in wavefront order
#pragma unroll
    for (int pp = 0; pp < kPanelsPerWorkgroup; ++pp) {
        const int p = blockIdx.x + pp * gridDim.x;
        if (p >= n_panels) break;                       // (the same for the whole workgroup)
#pragma unroll
        for (int v = 0; v < 4; ++v) part[(wl * 4 + v) * kLanes + lane] = acc[pp][v];
        __syncthreads();
        if (tid < 4 * kLanes) {
            const int v = tid >> 6;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < kPanelWaves; ++w) sum += part[(w * 4 + v) * kLanes + lane];
            const int b = 4 * j + v;                    // activation row
            const int row = p * kPanelRows + r;         // output row
            if (b < batch && row < N) y[static_cast<size_t>(b) * N + row] = float_to_half_bits(sum);
        }
        __syncthreads();                                // before the next panel's sums
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

// Up to 16 activation rows in one launch.  x [batch, K], y [batch, N], fp16, on the device.
gqsa_status_t panels_gemm(const gqsa_matrix* m, const void* x, void* y, int batch, void* stream)
{
    if (!m->d_panels || batch < 1 || batch > kPanelRows) return GQSA_ERR_UNSUPPORTED;
    const uint8_t* img = static_cast<const uint8_t*>(m->d_panels);
    const uint8_t* data = img + m->panel_blocks_offset;
    // one workgroup per compute unit unless that gives a workgroup more than four panels
    const int64_t wgs = std::min<int64_t>(m->n_panels, std::max<int64_t>(kMaxDefaultWorkgroups,
                                                                         (m->n_panels + kPanelsPerWorkgroup - 1) / kPanelsPerWorkgroup));
    const dim3 grid(static_cast<unsigned>(wgs)), block(kPanelWaves * kLanes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, block, 0, s, static_cast<const uint16_t*>(x), img, data,
                           static_cast<uint16_t*>(y), static_cast<int>(m->N), static_cast<int>(m->K),
                           static_cast<int>(m->n_slices), batch, static_cast<int>(m->n_panels));
    };
    switch (m->bits * 1000 + m->G) {
        case 4016: launch(gqsa_panel_kernel<4, 1>); break;
        case 4032: launch(gqsa_panel_kernel<4, 2>); break;
        case 4064: launch(gqsa_panel_kernel<4, 4>); break;
        case 4128: launch(gqsa_panel_kernel<4, 8>); break;
        case 8016: launch(gqsa_panel_kernel<8, 1>); break;
        case 8032: launch(gqsa_panel_kernel<8, 2>); break;
        case 8064: launch(gqsa_panel_kernel<8, 4>); break;
        default: return GQSA_ERR_UNSUPPORTED;
    }
    GQSA_HIP(hipGetLastError());
    return GQSA_OK;
}

}  // namespace gqsa
