// Second device image of a packed matrix, for calls with many activation rows: the stored groups
// of 16 consecutive output rows (a panel), ordered by group-column, so that one group-column of a
// panel -- up to 16 groups of 16 weights, absent ones zero -- and the 16 x 16 activations under it
// form a dense 16x16x16 product for the matrix cores (groups of 32, 64 or 128 weights: two, four
// or eight such products with one scale and zero).  The row-major stream of the GEMV kernel
// cannot feed them: there every group of a row has its own activations (the gather of Sec. 3.5).
// Only the order differs from the canonical BSR arrays of Sec. 3.2; codes, scales and zeros
// (Eq. 1-3) are the same bits.
//
// Layout (all little-endian):
//   panels      P = ceil(N / 16); panel p holds rows 16p .. 16p+15 (rows >= N: no groups)
//   slices      the K/G group-columns in runs of 32: S = ceil(K/G / 32); slice s holds columns
//               32s .. 32s+31 (columns >= K/G: no groups)
//   headers     one per block (p, s), at byte 144 (p S + s): uint32[36].  Word j < 32, for column
//               32s + j: bits 0..15 = which rows of the panel store a group in that column (bit r:
//               row 16p + r), bits 16..31 = number of groups of the block before that column.
//               Word 32 = where the block's data start, in 16-byte units from the start of the data
//               region; word 33 = number of groups of the block; words 34, 35 = 0.  The header
//               region is padded to a multiple of 256 bytes.
//   data        per block, in the order of the headers: one record per group, the block's groups
//               ordered by (column, row); the block is padded to a multiple of 16 bytes.  Record =
//               the code bytes of quarters 0 and 1, then uint32 fp16 scale | fp16 zero << 16, then
//               the code bytes of quarters 2 and 3 (with 2 code bytes per quarter the record is
//               12 bytes, which a lane reads whole).  Quarter t (t = 0..3) holds, chunk
//               after chunk of 16 elements, the codes of the elements 4t .. 4t+3 of every chunk --
//               what one lane supplies to the products -- so a lane's codes are contiguous.  A quarter of a chunk is 2 bytes of
//               4-bit codes, elements e0..e3 as (e0 | e2 << 4), (e1 | e3 << 4) (two masks split
//               them into two fp16 pairs), or 4 bytes of 8-bit codes in element order.
//               8-bit codes with G = 16 (4 code bytes per quarter): the scale | zero word is
//               stored twice, record = quarter 0, scale | zero, quarter 1, quarter 2, scale | zero,
//               quarter 3 (24 bytes), so that the 12 bytes around the word hold a lane's codes.
//               The region ends with 256 zero bytes and the image is padded to a multiple of 256
//               bytes.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "gqsa_internal.hpp"

namespace gqsa {

gqsa_status_t build_panels(gqsa_matrix* m)
{
    if (m->G < 16) return GQSA_ERR_UNSUPPORTED;
    const int cb = m->code_bytes();                  // 8 .. 64
    const int64_t kg = m->K / m->G;                  // group-columns
    const int chunks = m->G / 16;
    const bool twice = m->bits == 8 && chunks == 1;            // scale | zero stored twice (see above)
    const int rb = cb + (twice ? 8 : 4);                       // record bytes
    const int64_t P = (m->N + kPanelRows - 1) / kPanelRows;
    const int64_t S = (kg + kSliceColumns - 1) / kSliceColumns;
    auto pad16 = [](size_t v) { return (v + 15) / 16 * 16; };
    auto pad256 = [](size_t v) { return (v + kAlign - 1) / kAlign * kAlign; };

    // pass 1: groups per block -> where each block's data start
    std::vector<uint32_t> count(static_cast<size_t>(P * S), 0);
    for (int64_t n = 0; n < m->N; ++n)
        for (int64_t g = m->rowIndex[n]; g < m->rowIndex[n + 1]; ++g)
            ++count[static_cast<size_t>((n / kPanelRows) * S + m->groups[g] / kSliceColumns)];
    std::vector<uint64_t> start(static_cast<size_t>(P * S) + 1, 0);     // bytes
    for (int64_t b = 0; b < P * S; ++b)
        start[b + 1] = start[b] + pad16(static_cast<size_t>(count[b]) * rb);
    if (start.back() / 16 > UINT32_MAX) return GQSA_ERR_SHAPE;
    const size_t header_bytes = pad256(static_cast<size_t>(P * S) * kPanelHeaderBytes);
    const size_t total = pad256(header_bytes + start.back() + 256);

    std::vector<uint8_t> img;
    try {
        img.assign(total, 0);
    } catch (const std::bad_alloc&) { return GQSA_ERR_ALLOC; }

    // pass 2: per panel, walk its 16 rows side by side in column order
    for (int64_t p = 0; p < P; ++p) {
        int64_t cur[kPanelRows], end[kPanelRows];
        for (int r = 0; r < kPanelRows; ++r) {
            const int64_t n = p * kPanelRows + r;
            cur[r] = n < m->N ? m->rowIndex[n] : 0;
            end[r] = n < m->N ? m->rowIndex[n + 1] : 0;
        }
        for (int64_t s = 0; s < S; ++s) {
            const size_t b = static_cast<size_t>(p * S + s);
            uint32_t* header = reinterpret_cast<uint32_t*>(img.data() + b * kPanelHeaderBytes);
            uint8_t* records = img.data() + header_bytes + start[b];
            uint32_t k = 0;
            for (int j = 0; j < kSliceColumns; ++j) {
                const int64_t c = s * kSliceColumns + j;
                uint32_t mask = 0;
                const uint32_t before = k;
                for (int r = 0; r < kPanelRows; ++r) {
                    if (cur[r] < end[r] && m->groups[cur[r]] == c) {
                        const int64_t g = cur[r]++;
                        mask |= 1u << r;
                        const uint8_t* v = &m->values[static_cast<size_t>(g) * cb];
                        uint8_t* out = records + static_cast<size_t>(k) * rb;
                        const int qb = m->bits / 2;                 // bytes of a quarter of a chunk: 2 or 4
                        for (int t = 0; t < 4; ++t) {
                            for (int i = 0; i < chunks; ++i) {
                                const uint8_t* src = v + static_cast<size_t>(i) * 4 * qb + static_cast<size_t>(t) * qb;
                                uint8_t* dst = twice ? out + 4 * t + (t >= 1 ? 4 : 0) + (t >= 3 ? 4 : 0)
                                                     : out + (static_cast<size_t>(t) * chunks + i) * qb + (t >= 2 ? 4 : 0);
                                if (m->bits == 4) {    // (e0 | e1 << 4), (e2 | e3 << 4) -> (e0 | e2 << 4), (e1 | e3 << 4)
                                    dst[0] = static_cast<uint8_t>((src[0] & 0x0F) | ((src[1] & 0x0F) << 4));
                                    dst[1] = static_cast<uint8_t>((src[0] >> 4) | (src[1] & 0xF0));
                                } else {
                                    std::memcpy(dst, src, 4);
                                }
                            }
                        }
                        const uint32_t sz = static_cast<uint32_t>(m->scales[g]) | (static_cast<uint32_t>(m->zeros[g]) << 16);
                        if (twice) {
                            std::memcpy(out + 4, &sz, 4);
                            std::memcpy(out + 16, &sz, 4);
                        } else {
                            std::memcpy(out + cb / 2, &sz, 4);
                        }
                        ++k;
                    }
                }
                header[j] = mask | (before << 16);
            }
            header[32] = static_cast<uint32_t>(start[b] / 16);
            header[33] = k;
        }
    }
    // may the kernel subtract the zero from the codes in fp16?  Exact only for integers up to 1024
    bool integer_zeros = true;
    for (const uint16_t zb : m->zeros) {
        const float z = static_cast<float>(__builtin_bit_cast(_Float16, zb));
        if (!(z == std::nearbyint(z) && std::fabs(z) <= 1024.0f)) { integer_zeros = false; break; }
    }
    m->panel_integer_zeros = integer_zeros;
    m->panel_image.swap(img);
    m->panel_blocks_offset = header_bytes;
    m->n_panels = P;
    m->n_slices = S;
    return GQSA_OK;
}

}  // namespace gqsa
