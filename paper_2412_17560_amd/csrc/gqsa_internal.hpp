// Internal definitions shared by the host packer, the device-image builder and the
// HIP launch code of libgqsa.  Not part of the public ABI.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "gqsa.h"

namespace gqsa {

constexpr int kLanes = 64;             // one stored group per lane per block
constexpr int kWavesPerWorkgroup = 16; // the most wavefronts a workgroup can have (1024 threads)
constexpr int kMaxDefaultWorkgroups = 256;  // MI355X: 256 compute units
constexpr int kMaxWorkgroups = 4096;
constexpr int kMaxBatch = 16;
constexpr int kMaxMatricesPerLaunch = 4;
constexpr int64_t kMaxGroupColumns = 4096;  // 16-element slots of K: 12-bit slot << 4 | head flag in 16 bits
constexpr size_t kAlign = 256;
constexpr int kPanelRows = 16;         // output rows per panel of the many-row image (one side of a 16x16x16 product)
constexpr int kSliceColumns = 32;      // group-columns per block of that image
constexpr int kPanelHeaderBytes = 144; // a block's header: 32 column words, data offset, group count, 2 spare

// Blocks per tile for a format with `code_bytes` bytes of codes per group, unless the partition
// names another count.
constexpr int largest_tile(int code_bytes) { return code_bytes <= 16 ? 4 : (code_bytes <= 32 ? 2 : 1); }
// Tile shapes the GEMV kernel is compiled for: the format's own block count with all 64 lanes
// of a block in use, and for G = 16 also 3, 4 or 5 blocks per tile (4-bit codes: 6 and 8 as well)
// with any multiple of 4 lanes from 32 to 64 in use (a tile then holds lanes * blocks stream
// positions); tiles of such a chosen shape come one to a worker.
constexpr bool tile_shape_is_own(int code_bytes, int blocks, int lanes)
{
    return blocks == largest_tile(code_bytes) && lanes == kLanes;
}
constexpr bool tile_shape_supported(int code_bytes, int G, int blocks, int lanes)
{
    if (tile_shape_is_own(code_bytes, blocks, lanes)) return true;
    return G == 16 && ((blocks >= 3 && blocks <= 5) || (code_bytes == 8 && (blocks == 6 || blocks == 8))) && lanes >= 32 && lanes <= kLanes && lanes % 4 == 0;
}

// How the group stream of a matrix is laid out for the wavefront workers.
struct Partition {
    int n_workgroups = 1;
    int waves_per_workgroup = 1;
    int span_tiles = 0;          // 0: rows follow each other without gaps; else tiles per span that rows are kept inside
    int tile_blocks = 0;         // blocks per tile (0: the format's own count)
    int tile_lanes = 0;          // lanes of a block in use = stream positions per block (0: all 64)
    int span_per_worker = 0;     // 0: one span per workgroup; 1: one span per wavefront worker
};

// Offsets (bytes) of the regions inside the device image.
struct ImageMap {
    size_t blocks = 0;      // n_blocks * block_bytes
    size_t wave_info = 0;   // n_waves * int32[4] {rank_base, tail_closed + 2 * lead_len, lead_first, chain_len}
    size_t row_of_rank = 0; // int32 per non-empty row
    size_t empty_rows = 0;  // int32 per empty row
    size_t total = 0;
};

// Per-worker record the GEMV kernel publishes for the rows it shares with its neighbours.
struct CarryRecord {
    float lead;    // sum of the groups before the worker's first row head
    float tail;    // sum of the groups after its last row head (or all, if it has none)
    int32_t heads; // row heads inside the worker's run
    int32_t pad;
};

}  // namespace gqsa

struct gqsa_matrix {
    int64_t N = 0, K = 0;
    int G = 0, bits = 0;
    // canonical arrays (Sec. 3.2 listing + Eq. 1 parameters)
    std::vector<int32_t> rowIndex;
    std::vector<int32_t> groups;
    std::vector<uint8_t> values;
    std::vector<uint16_t> scales;
    std::vector<uint16_t> zeros;
    // device image (host copy) and its map
    int n_workgroups = 0;
    int waves_per_workgroup = 0;
    int span_tiles = 0;       // tiles per span that rows are kept inside; 0: rows follow each other without gaps
    int span_per_worker = 0;  // 1: a span is one wavefront worker's run (rows then never straddle workers); 0: a workgroup's
    int tile_blocks = 0;      // blocks per tile
    int tile_lanes = 0;       // stream positions per block (lanes in use), 64 unless the partition says otherwise
    int n_waves = 0;          // n_workgroups * waves_per_workgroup
    int64_t n_blocks = 0;     // blocks of the padded stream = n_tiles * tile_blocks
    int64_t n_tiles = 0;
    int64_t n_empty = 0;
    int needs_fixup = 0;
    gqsa::ImageMap map;
    std::vector<uint8_t> image;
    // optional second image for calls with many activation rows (gqsa_panels.cpp)
    std::vector<uint8_t> panel_image;
    size_t panel_blocks_offset = 0;   // where the data region starts in it (after the headers)
    int64_t n_panels = 0, n_slices = 0;
    bool panel_integer_zeros = false; // every zero an integer of magnitude <= 1024: the kernel may take it off the codes
    // device side
    int device = -1;
    void* d_panels = nullptr;
    void* d_image = nullptr;
    void* d_carry = nullptr;  // carry records, arrival counters and meeting points of the fix-up

    int64_t nnzg() const { return rowIndex.empty() ? 0 : rowIndex.back(); }
    int code_bytes() const { return G * bits / 8; }
    int group_bytes() const { return code_bytes() + 6; }     // codes, scale, zero, index word
    int block_bytes() const { return group_bytes() * (tile_lanes ? tile_lanes : gqsa::kLanes); }
};

namespace gqsa {

// host packer (gqsa_pack.cpp)
gqsa_status_t pack_dense(const float* W, int64_t N, int64_t K, int G, int bits,
                         const int32_t* keep_per_row, double sparsity, const float* hinv_diag,
                         gqsa_matrix* m);
int64_t place_rows(const gqsa_matrix& m, int64_t span_groups, std::vector<int64_t>* row_pos);
Partition default_partition(const gqsa_matrix& m);
gqsa_status_t build_image(gqsa_matrix* m, const Partition& part, bool fill_blocks = true,
                          std::vector<int64_t>* row_pos_out = nullptr);
int64_t balanced_keep(int64_t groups_per_row, double sparsity);
gqsa_status_t row_pointers(gqsa_matrix* m, const int32_t* keep_per_row, double sparsity);

// GPU packer (gqsa_pack_device.hip)
gqsa_status_t pack_on_device(const float* W_dev, const float* hinv_dev, gqsa_matrix* m, void* stream);

// many-row image (gqsa_panels.cpp) and its kernel (gqsa_panel_kernel.hip)
gqsa_status_t build_panels(gqsa_matrix* m);
gqsa_status_t panels_upload(gqsa_matrix* m);
void panels_release(gqsa_matrix* m);
gqsa_status_t panels_gemm(const gqsa_matrix* const* ms, int n, const void* x, void* const* ys, int batch, void* stream);

// device side (gqsa_gemv.hip)
gqsa_status_t device_upload(gqsa_matrix* m, void* filled_image = nullptr);   // (filled_image: a device copy of m->image that the handle takes over)
void device_release(gqsa_matrix* m);
// (workspace: nullptr = every handle's own carry workspace)
gqsa_status_t device_gemv(gqsa_matrix* const* ms, int n_mats, const void* x, void* const* ys, int batch,
                          void* stream, void* workspace = nullptr);
gqsa_status_t device_gemv_static(gqsa_matrix* m, const void* x, void* y, int batch, void* stream);
bool stream_is_capturing(void* stream);

}  // namespace gqsa
