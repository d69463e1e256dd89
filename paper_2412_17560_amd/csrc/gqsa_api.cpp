// extern "C" surface of libgqsa: argument checking, handle life-cycle, export/import.
// The arithmetic lives in gqsa_pack.cpp (host) and gqsa_gemv.hip (device).
#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <stdexcept>
#include <vector>

#include "gqsa_internal.hpp"

namespace {

// Nothing is thrown across the C boundary: whatever the host code below throws -- in practice a
// failed allocation (std::bad_alloc, std::length_error) -- becomes a status.
template <typename Body>
gqsa_status_t guarded(Body&& body) noexcept
{
    try {
        return body();
    } catch (...) {
        return GQSA_ERR_ALLOC;
    }
}

gqsa_status_t check_format(int64_t N, int64_t K, int G, int bits)
{
    if (N <= 0 || K <= 0 || G <= 0) return GQSA_ERR_SHAPE;
    if (bits != 4 && bits != 8) return GQSA_ERR_UNSUPPORTED;
    if (G != 8 && G != 16 && G != 32 && G != 64 && G != 128) return GQSA_ERR_UNSUPPORTED;
    if (G * bits / 8 > 64) return GQSA_ERR_UNSUPPORTED;       // at most 64 code bytes per group
    if (K % G != 0 || K % 16 != 0) return GQSA_ERR_SHAPE;     // (x is staged in runs of 16, also for G = 8)
    if (K / std::min(G, 16) > gqsa::kMaxGroupColumns) return GQSA_ERR_SHAPE;
    if (N > (int64_t{1} << 30)) return GQSA_ERR_SHAPE;
    return GQSA_OK;
}

// Choose the default partition and build the device image; the handle goes to the caller only
// if all of that worked (and is destroyed otherwise, also when something below throws).
gqsa_status_t finish(std::unique_ptr<gqsa_matrix> m, gqsa_status_t st, gqsa_handle_t* out)
{
    if (st != GQSA_OK) return st;
    st = gqsa::build_image(m.get(), gqsa::default_partition(*m));
    if (st != GQSA_OK) return st;
    *out = m.release();
    return GQSA_OK;
}

gqsa_status_t pack_any(const float* W, int64_t N, int64_t K, int G, int bits, const int32_t* keep_per_row,
                       double sparsity, const float* hinv_diag, gqsa_handle_t* out)
{
    return guarded([&]() -> gqsa_status_t {
        std::unique_ptr<gqsa_matrix> m(new gqsa_matrix);
        const gqsa_status_t st = gqsa::pack_dense(W, N, K, G, bits, keep_per_row, sparsity, hinv_diag, m.get());
        return finish(std::move(m), st, out);
    });
}

// The device image, and the panel image if there is one.
gqsa_status_t upload(gqsa_matrix* m)
{
    if (gqsa_status_t st = gqsa::device_upload(m)) return st;
    if (gqsa_status_t st = gqsa::panels_upload(m)) {
        gqsa::device_release(m);
        return st;
    }
    return GQSA_OK;
}

// Calls with this many activation rows or more go to the matrix-core kernel if the handle has a
// panel image: its time hardly depends on the row count (16 rows' worth of products either way),
// the wavefront kernel's grows with every row, and they cross between 4 and 5 rows on an MI355X
// for K up to 8192 and between 2 and 3 rows beyond (4096x11008, 4096x14336: every workgroup of
// the wavefront kernel stages all of x; group sizes other than 16: between 2 and 3 rows as well,
// since that kernel takes them one row per launch).
constexpr int panel_min_batch(const gqsa_matrix* m) { return m->G == 16 && m->K <= 8192 ? 5 : 3; }

}  // namespace

extern "C" {

gqsa_status_t gqsa_pack(const float* W_host, int64_t N, int64_t K, int G, int bits,
                        double sparsity, gqsa_handle_t* out)
{
    if (out) *out = nullptr;
    if (!W_host || !out) return GQSA_ERR_NULL;
    if (gqsa_status_t st = check_format(N, K, G, bits)) return st;
    if (!(sparsity >= 0.0 && sparsity <= 1.0)) return GQSA_ERR_RANGE;
    return pack_any(W_host, N, K, G, bits, nullptr, sparsity, nullptr, out);
}

gqsa_status_t gqsa_pack_rows(const float* W_host, int64_t N, int64_t K, int G, int bits,
                             const int32_t* keep_per_row, gqsa_handle_t* out)
{
    if (out) *out = nullptr;
    if (!W_host || !out || !keep_per_row) return GQSA_ERR_NULL;
    if (gqsa_status_t st = check_format(N, K, G, bits)) return st;
    return pack_any(W_host, N, K, G, bits, keep_per_row, 0.0, nullptr, out);
}

gqsa_status_t gqsa_pack_hessian(const float* W_host, int64_t N, int64_t K, int G, int bits,
                                double sparsity, const float* hinv_diag, gqsa_handle_t* out)
{
    if (out) *out = nullptr;
    if (!W_host || !out || !hinv_diag) return GQSA_ERR_NULL;
    if (gqsa_status_t st = check_format(N, K, G, bits)) return st;
    if (!(sparsity >= 0.0 && sparsity <= 1.0)) return GQSA_ERR_RANGE;
    return pack_any(W_host, N, K, G, bits, nullptr, sparsity, hinv_diag, out);
}

gqsa_status_t gqsa_pack_device(const float* W_dev, int64_t N, int64_t K, int G, int bits, double sparsity,
                               const int32_t* keep_per_row, const float* hinv_diag_dev, void* hip_stream,
                               gqsa_handle_t* out)
{
    if (out) *out = nullptr;
    if (!W_dev || !out) return GQSA_ERR_NULL;
    if (gqsa_status_t st = check_format(N, K, G, bits)) return st;
    if (!keep_per_row && !(sparsity >= 0.0 && sparsity <= 1.0)) return GQSA_ERR_RANGE;
    if ((reinterpret_cast<uintptr_t>(W_dev) & 3u) != 0 || (reinterpret_cast<uintptr_t>(hinv_diag_dev) & 3u) != 0)
        return GQSA_ERR_ALIGN;
    return guarded([&]() -> gqsa_status_t {
        std::unique_ptr<gqsa_matrix> m(new gqsa_matrix);
        m->N = N; m->K = K; m->G = G; m->bits = bits;
        if (gqsa_status_t st = gqsa::row_pointers(m.get(), keep_per_row, sparsity)) return st;
        if (gqsa_status_t st = gqsa::pack_on_device(W_dev, hinv_diag_dev, m.get(), hip_stream)) {
            gqsa::device_release(m.get());
            return st;
        }
        *out = m.release();
        return GQSA_OK;
    });
}

gqsa_status_t gqsa_import(const int32_t* rowIndex, const int32_t* groups, const uint8_t* values,
                          const uint16_t* scales_f16, const uint16_t* zeros_f16,
                          int64_t N, int64_t K, int G, int bits, gqsa_handle_t* out)
{
    if (out) *out = nullptr;
    if (!rowIndex || !out) return GQSA_ERR_NULL;
    if (gqsa_status_t st = check_format(N, K, G, bits)) return st;
    const int64_t kg = K / G;
    if (rowIndex[0] != 0) return GQSA_ERR_SHAPE;
    for (int64_t n = 0; n < N; ++n) {
        const int64_t cnt = static_cast<int64_t>(rowIndex[n + 1]) - rowIndex[n];
        if (cnt < 0 || cnt > kg) return GQSA_ERR_SHAPE;
    }
    const int64_t nnz = rowIndex[N];
    if (nnz > 0 && (!groups || !values || !scales_f16 || !zeros_f16)) return GQSA_ERR_NULL;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = rowIndex[n]; g < rowIndex[n + 1]; ++g) {
            if (groups[g] < 0 || groups[g] >= kg) return GQSA_ERR_SHAPE;
            if (g > rowIndex[n] && groups[g] <= groups[g - 1]) return GQSA_ERR_SHAPE;
        }
    }
    return guarded([&]() -> gqsa_status_t {
        std::unique_ptr<gqsa_matrix> m(new gqsa_matrix);
        m->N = N; m->K = K; m->G = G; m->bits = bits;
        m->rowIndex.assign(rowIndex, rowIndex + N + 1);
        m->groups.assign(groups, groups + nnz);
        m->values.assign(values, values + nnz * (G * bits / 8));
        m->scales.assign(scales_f16, scales_f16 + nnz);
        m->zeros.assign(zeros_f16, zeros_f16 + nnz);
        return finish(std::move(m), GQSA_OK, out);
    });
}

gqsa_status_t gqsa_default_partition(const int32_t* rowIndex, int64_t N, int64_t K, int G, int bits, int32_t out[6])
{
    if (!rowIndex || !out) return GQSA_ERR_NULL;
    if (gqsa_status_t st = check_format(N, K, G, bits)) return st;
    if (rowIndex[0] != 0) return GQSA_ERR_SHAPE;
    for (int64_t n = 0; n < N; ++n) {
        const int64_t cnt = static_cast<int64_t>(rowIndex[n + 1]) - rowIndex[n];
        if (cnt < 0 || cnt > K / G) return GQSA_ERR_SHAPE;
    }
    return guarded([&]() -> gqsa_status_t {
        gqsa_matrix m;
        m.N = N; m.K = K; m.G = G; m.bits = bits;
        m.rowIndex.assign(rowIndex, rowIndex + N + 1);
        const gqsa::Partition part = gqsa::default_partition(m);
        out[0] = part.n_workgroups; out[1] = part.waves_per_workgroup; out[2] = part.span_tiles;
        out[3] = part.tile_blocks; out[4] = part.tile_lanes; out[5] = part.span_per_worker;
        return GQSA_OK;
    });
}

gqsa_status_t gqsa_set_partition(gqsa_handle_t h, int n_workgroups, int waves_per_workgroup)
{
    if (!h) return GQSA_ERR_NULL;
    if (h->d_image) return GQSA_ERR_UNSUPPORTED;
    if (n_workgroups < 1) return GQSA_ERR_RANGE;
    return guarded([&] {
        gqsa::Partition part;
        part.n_workgroups = n_workgroups;
        part.waves_per_workgroup = waves_per_workgroup;
        return gqsa::build_image(h, part);
    });
}

gqsa_status_t gqsa_set_partition_aligned(gqsa_handle_t h, int span_tiles, int n_workgroups, int waves_per_workgroup)
{
    if (!h) return GQSA_ERR_NULL;
    if (h->d_image) return GQSA_ERR_UNSUPPORTED;
    if (span_tiles < 1) return GQSA_ERR_RANGE;
    return guarded([&] {
        gqsa::Partition part;
        part.n_workgroups = n_workgroups;
        part.waves_per_workgroup = waves_per_workgroup;
        part.span_tiles = span_tiles;
        return gqsa::build_image(h, part);
    });
}

gqsa_status_t gqsa_set_partition_rows(gqsa_handle_t h, int tile_blocks, int tile_lanes, int tiles_per_worker,
                                      int n_workgroups, int waves_per_workgroup)
{
    if (!h) return GQSA_ERR_NULL;
    if (h->d_image) return GQSA_ERR_UNSUPPORTED;
    if (tiles_per_worker < 1 || tile_blocks < 1 || tile_lanes < 1) return GQSA_ERR_RANGE;
    return guarded([&] {
        gqsa::Partition part;
        part.n_workgroups = n_workgroups;
        part.waves_per_workgroup = waves_per_workgroup;
        part.span_tiles = tiles_per_worker;
        part.tile_blocks = tile_blocks;
        part.tile_lanes = tile_lanes;
        part.span_per_worker = 1;
        return gqsa::build_image(h, part);
    });
}

gqsa_status_t gqsa_build_panels(gqsa_handle_t h)
{
    if (!h) return GQSA_ERR_NULL;
    if (h->d_image) return GQSA_ERR_UNSUPPORTED;
    return guarded([&] { return gqsa::build_panels(h); });
}

gqsa_status_t gqsa_upload(gqsa_handle_t h)
{
    if (!h) return GQSA_ERR_NULL;
    if (h->d_image) return GQSA_OK;
    return upload(h);
}

gqsa_status_t gqsa_gemv(gqsa_handle_t h, const void* x_dev, void* y_dev, int batch,
                        void* hip_stream)
{
    if (!h || !x_dev || !y_dev) return GQSA_ERR_NULL;
    if (batch < 1 || batch > gqsa::kMaxBatch) return GQSA_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(x_dev) & 15u) != 0) return GQSA_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(y_dev) & 1u) != 0) return GQSA_ERR_ALIGN;
    if (!h->d_image) {
        if (gqsa::stream_is_capturing(hip_stream)) return GQSA_ERR_UNSUPPORTED;   // an upload cannot be captured
        if (gqsa_status_t st = upload(h)) return st;
    }
    if (h->d_panels && batch >= panel_min_batch(h)) return gqsa::panels_gemm(&h, 1, x_dev, &y_dev, batch, hip_stream);
    return gqsa::device_gemv(&h, 1, x_dev, &y_dev, batch, hip_stream);
}

gqsa_status_t gqsa_gemv_static(gqsa_handle_t h, const void* x_dev, void* y_dev, int batch, void* hip_stream)
{
    if (!h || !x_dev || !y_dev) return GQSA_ERR_NULL;
    if (batch < 1 || batch > gqsa::kMaxBatch) return GQSA_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(x_dev) & 15u) != 0) return GQSA_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(y_dev) & 1u) != 0) return GQSA_ERR_ALIGN;
    if (!h->d_image) return GQSA_ERR_UNSUPPORTED;       // an upload allocates: the caller does it beforehand
    return gqsa::device_gemv_static(h, x_dev, y_dev, batch, hip_stream);
}

gqsa_status_t gqsa_gemv_panels(gqsa_handle_t h, const void* x_dev, void* y_dev, int batch, void* hip_stream)
{
    if (!h || !x_dev || !y_dev) return GQSA_ERR_NULL;
    if (batch < 1 || batch > gqsa::kMaxBatch) return GQSA_ERR_UNSUPPORTED;
    if (h->panel_image.empty()) return GQSA_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(x_dev) & 15u) != 0) return GQSA_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(y_dev) & 1u) != 0) return GQSA_ERR_ALIGN;
    if (!h->d_image) {
        if (gqsa_status_t st = upload(h)) return st;
    }
    return gqsa::panels_gemm(&h, 1, x_dev, &y_dev, batch, hip_stream);
}

gqsa_status_t gqsa_gemv_multi(const gqsa_handle_t* handles, int n_matrices, const void* x_dev,
                              void* const* y_devs, int batch, void* hip_stream)
{
    if (!handles || !x_dev || !y_devs) return GQSA_ERR_NULL;
    if (n_matrices < 1 || n_matrices > gqsa::kMaxMatricesPerLaunch) return GQSA_ERR_UNSUPPORTED;
    if (batch < 1 || batch > gqsa::kMaxBatch) return GQSA_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(x_dev) & 15u) != 0) return GQSA_ERR_ALIGN;
    for (int i = 0; i < n_matrices; ++i) {
        if (!handles[i] || !y_devs[i]) return GQSA_ERR_NULL;
        if ((reinterpret_cast<uintptr_t>(y_devs[i]) & 1u) != 0) return GQSA_ERR_ALIGN;
        const gqsa_matrix* m = handles[i];
        const gqsa_matrix* m0 = handles[0];
        // one launch: same x, same storage format (N and the partitions may differ)
        if (m->K != m0->K || m->G != m0->G || m->bits != m0->bits) return GQSA_ERR_SHAPE;
        for (int j = 0; j < i; ++j)
            if (handles[j] == handles[i]) return GQSA_ERR_SHAPE;   // a handle has one carry workspace
    }
    bool panels = batch >= panel_min_batch(handles[0]);
    for (int i = 0; i < n_matrices; ++i) {
        if (!handles[i]->d_image) {
            if (gqsa_status_t st = upload(handles[i])) return st;
        }
        if (!handles[i]->d_panels) panels = false;
    }
    if (panels) {
        // One launch when the matrices can share a kernel variant (the zero is handled the same
        // way in all of them): a workgroup's panels then come from different matrices and the
        // activations, most of what a compute unit reads, are loaded once for all of them.
        // (Not beyond four panels per compute unit's workgroup: a second round of workgroups
        // would leave most compute units idle.)
        bool alike = true;
        int64_t panels_in_all = 0;
        for (int i = 0; i < n_matrices; ++i) {
            if (handles[i]->panel_integer_zeros != handles[0]->panel_integer_zeros) alike = false;
            panels_in_all += handles[i]->n_panels;
        }
        if (alike && n_matrices > 1 && panels_in_all <= 4 * gqsa::kMaxDefaultWorkgroups)
            return gqsa::panels_gemm(handles, n_matrices, x_dev, y_devs, batch, hip_stream);
        for (int i = 0; i < n_matrices; ++i)
            if (gqsa_status_t st = gqsa::panels_gemm(&handles[i], 1, x_dev, &y_devs[i], batch, hip_stream)) return st;
        return GQSA_OK;
    }
    return gqsa::device_gemv(handles, n_matrices, x_dev, y_devs, batch, hip_stream);
}

gqsa_status_t gqsa_info(gqsa_handle_t h, gqsa_info_t* out)
{
    if (!h || !out) return GQSA_ERR_NULL;
    std::memset(out, 0, sizeof(*out));
    out->N = h->N;
    out->K = h->K;
    out->G = h->G;
    out->bits = h->bits;
    out->nnz_groups = h->nnzg();
    out->values_bytes = h->nnzg() * h->code_bytes();
    out->n_blocks = h->n_blocks;
    out->n_workgroups = h->n_workgroups;
    out->waves_per_workgroup = h->waves_per_workgroup;
    out->needs_fixup = h->needs_fixup;
    out->span_tiles = h->span_tiles;
    out->tile_blocks = h->tile_blocks;
    out->tile_lanes = h->tile_lanes;
    out->span_per_worker = h->span_per_worker;
    out->n_empty_rows = h->n_empty;
    out->device_bytes = static_cast<int64_t>(h->map.total);
    out->algorithmic_bytes = h->nnzg() * (h->code_bytes() + 6) + (h->N + 1) * 4 + (h->K + h->N) * 2;
    out->on_device = h->d_image ? 1 : 0;
    out->panel_bytes = static_cast<int64_t>(h->panel_image.size());
    out->panel_integer_zeros = (!h->panel_image.empty() && h->panel_integer_zeros) ? 1 : 0;
    return GQSA_OK;
}

gqsa_status_t gqsa_export(gqsa_handle_t h, int32_t* rowIndex, int32_t* groups, uint8_t* values,
                          uint16_t* scales_f16, uint16_t* zeros_f16)
{
    if (!h) return GQSA_ERR_NULL;
    if (rowIndex) std::memcpy(rowIndex, h->rowIndex.data(), h->rowIndex.size() * 4);
    if (groups && !h->groups.empty()) std::memcpy(groups, h->groups.data(), h->groups.size() * 4);
    if (values && !h->values.empty()) std::memcpy(values, h->values.data(), h->values.size());
    if (scales_f16 && !h->scales.empty())
        std::memcpy(scales_f16, h->scales.data(), h->scales.size() * 2);
    if (zeros_f16 && !h->zeros.empty())
        std::memcpy(zeros_f16, h->zeros.data(), h->zeros.size() * 2);
    return GQSA_OK;
}

gqsa_status_t gqsa_export_panel_blob(gqsa_handle_t h, void* host_buf, size_t bytes)
{
    if (!h || !host_buf) return GQSA_ERR_NULL;
    if (h->panel_image.empty()) return GQSA_ERR_UNSUPPORTED;
    if (bytes < h->panel_image.size()) return GQSA_ERR_BUFSIZE;
    std::memcpy(host_buf, h->panel_image.data(), h->panel_image.size());
    return GQSA_OK;
}

gqsa_status_t gqsa_export_device_blob(gqsa_handle_t h, void* host_buf, size_t bytes)
{
    if (!h || !host_buf) return GQSA_ERR_NULL;
    if (bytes < h->image.size()) return GQSA_ERR_BUFSIZE;
    std::memcpy(host_buf, h->image.data(), h->image.size());
    return GQSA_OK;
}

namespace {

// File image of a packed matrix: a 48-byte header, then the canonical arrays, little-endian.
struct FileHeader {
    char magic[8];        // "GQSABSR1"
    int64_t N, K;
    int32_t G, bits;
    int64_t nnz_groups;
    int64_t reserved;
};
const char kMagic[8] = {'G', 'Q', 'S', 'A', 'B', 'S', 'R', '1'};

struct FileCloser {
    std::FILE* f;
    ~FileCloser() { if (f) std::fclose(f); }
};

}  // namespace

gqsa_status_t gqsa_save(gqsa_handle_t h, const char* path)
{
    if (!h || !path) return GQSA_ERR_NULL;
    FileCloser file{std::fopen(path, "wb")};
    if (!file.f) return GQSA_ERR_IO;
    FileHeader hd{};
    std::memcpy(hd.magic, kMagic, 8);
    hd.N = h->N; hd.K = h->K; hd.G = h->G; hd.bits = h->bits; hd.nnz_groups = h->nnzg();
    bool ok = std::fwrite(&hd, sizeof(hd), 1, file.f) == 1;
    auto put = [&](const void* p, size_t bytes) {
        if (ok && bytes) ok = std::fwrite(p, 1, bytes, file.f) == bytes;
    };
    put(h->rowIndex.data(), h->rowIndex.size() * 4);
    put(h->groups.data(), h->groups.size() * 4);
    put(h->values.data(), h->values.size());
    put(h->scales.data(), h->scales.size() * 2);
    put(h->zeros.data(), h->zeros.size() * 2);
    if (ok) ok = std::fflush(file.f) == 0;
    return ok ? GQSA_OK : GQSA_ERR_IO;
}

gqsa_status_t gqsa_load(const char* path, gqsa_handle_t* out)
{
    if (out) *out = nullptr;
    if (!path || !out) return GQSA_ERR_NULL;
    FileCloser file{std::fopen(path, "rb")};
    if (!file.f) return GQSA_ERR_IO;
    FileHeader hd{};
    if (std::fread(&hd, sizeof(hd), 1, file.f) != 1) return GQSA_ERR_IO;
    if (std::memcmp(hd.magic, kMagic, 8) != 0) return GQSA_ERR_SHAPE;
    if (gqsa_status_t st = check_format(hd.N, hd.K, hd.G, hd.bits)) return st;
    if (hd.nnz_groups < 0 || hd.nnz_groups > hd.N * (hd.K / hd.G) || hd.nnz_groups > INT32_MAX)
        return GQSA_ERR_SHAPE;
    return guarded([&]() -> gqsa_status_t {
        std::vector<int32_t> rowIndex, groups;
        std::vector<uint8_t> values;
        std::vector<uint16_t> scales, zeros;
        rowIndex.resize(static_cast<size_t>(hd.N) + 1);
        groups.resize(static_cast<size_t>(hd.nnz_groups));
        values.resize(static_cast<size_t>(hd.nnz_groups) * (hd.G * hd.bits / 8));
        scales.resize(static_cast<size_t>(hd.nnz_groups));
        zeros.resize(static_cast<size_t>(hd.nnz_groups));
        bool ok = true;
        auto get = [&](void* p, size_t bytes) {
            if (ok && bytes) ok = std::fread(p, 1, bytes, file.f) == bytes;
        };
        get(rowIndex.data(), rowIndex.size() * 4);
        get(groups.data(), groups.size() * 4);
        get(values.data(), values.size());
        get(scales.data(), scales.size() * 2);
        get(zeros.data(), zeros.size() * 2);
        if (!ok) return GQSA_ERR_IO;                             // truncated
        if (std::fgetc(file.f) != EOF) return GQSA_ERR_SHAPE;     // trailing bytes
        if (rowIndex[static_cast<size_t>(hd.N)] != hd.nnz_groups) return GQSA_ERR_SHAPE;
        // the same consistency checks as for arrays handed in directly
        return gqsa_import(rowIndex.data(), groups.data(), values.data(), scales.data(), zeros.data(), hd.N, hd.K,
                           hd.G, hd.bits, out);
    });
}

void gqsa_free(gqsa_handle_t h)
{
    if (!h) return;
    gqsa::device_release(h);
    gqsa::panels_release(h);
    delete h;
}

const char* gqsa_status_string(gqsa_status_t s)
{
    switch (s) {
        case GQSA_OK: return "ok";
        case GQSA_ERR_NULL: return "null pointer";
        case GQSA_ERR_SHAPE: return "bad shape";
        case GQSA_ERR_UNSUPPORTED: return "unsupported format or batch";
        case GQSA_ERR_RANGE: return "value out of range";
        case GQSA_ERR_ALLOC: return "host allocation failed";
        case GQSA_ERR_HIP: return "HIP runtime error";
        case GQSA_ERR_BUFSIZE: return "buffer too small";
        case GQSA_ERR_ALIGN: return "misaligned device pointer";
        case GQSA_ERR_IO: return "file could not be opened, read or written";
    }
    return "unknown status";
}

}  // extern "C"
