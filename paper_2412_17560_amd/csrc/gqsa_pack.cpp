// Host side of libgqsa: offline pre-processing of a dense matrix into the GQS layer's
// storage (paper Sec. 3.2) and construction of the device image.
//
//   - group pruning: weights are grouped along the row (K) dimension in runs of G, each
//     group gets one saliency, the least salient groups of a row are dropped (Fig. 3); the
//     saliency is the Hessian metric of Eq. 4 when the caller supplies diag(H^-1) (building
//     H needs calibration activations, which is the caller's business), else the group's sum
//     of squares;
//   - quantisation of the kept groups: Eq. 1 (scale, zero-point) and Eq. 2 (codes);
//   - storage: the BSR arrays rowIndex / groups / values of the Sec. 3.2 listing plus
//     one fp16 scale and zero per stored group.
//
// Nothing in this file touches the GPU.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <limits>
#include <numeric>
#include <thread>

#include "gqsa_internal.hpp"

namespace gqsa {
namespace {

inline uint16_t half_bits(float f)
{
    _Float16 h = static_cast<_Float16>(f);  // round-to-nearest-even
    uint16_t b;
    std::memcpy(&b, &h, 2);
    return b;
}

inline float half_value(uint16_t b)
{
    _Float16 h;
    std::memcpy(&h, &b, 2);
    return static_cast<float>(h);
}

// Eq. 1 and Eq. 2 on one kept group of G weights.  The scale is rounded to fp16 first and
// the rounded value is the one the zero-point and the codes are derived from, so that the
// kernel's (q - z) * s uses exactly the parameters the codes were made with.
// False if the group cannot be stored: its range over 2^n - 1 is beyond the largest fp16 number,
// so the scale of Eq. 1 would be infinite and Eq. 3 could not give the weights back.
bool quantise_group(const float* w, int G, int bits, uint8_t* q_out, uint16_t* s_out,
                    uint16_t* z_out)
{
    const float levels = static_cast<float>((1 << bits) - 1);
    const auto mm = std::minmax_element(w, w + G);
    const float lo = *mm.first, hi = *mm.second;
    float s = (hi - lo) / levels;
    uint16_t sb = half_bits(s);
    if ((sb & 0x7FFFu) >= 0x7C00u) return false;
    s = half_value(sb);
    constexpr float kMinScale = 0x1p-14f;  // smallest normal fp16: constant groups, underflow
    if (!(s >= kMinScale)) {
        s = kMinScale;
        sb = half_bits(s);
    }
    float z = std::nearbyint(-lo / s);     // round-half-even; Eq. 1 has no clamp to the code range
    z = std::min(2048.0f, std::max(-2048.0f, z));  // keep it exact in fp16
    *s_out = sb;
    *z_out = half_bits(z);
    for (int j = 0; j < G; ++j) {
        float q = std::nearbyint(w[j] / s) + z;
        q = std::min(levels, std::max(0.0f, q));
        q_out[j] = static_cast<uint8_t>(q);
    }
    return true;
}

// Kept group-columns of one row, ascending.  Order of pruning: ascending saliency, and
// among equal saliencies the lower column goes first.  Saliency of a weight (Sec. 3.1, Eq. 4):
// w^2 / d_k^2 with d = diag(H^-1) of the layer's Hessian, handed in by the caller (nullptr:
// d = 1, the plain sum of squares); a group's saliency is the sum over its members.
bool select_row(const float* wrow, const float* hinv_diag, int64_t kg, int G, int64_t keep,
                std::vector<double>& sal, std::vector<int32_t>& order, std::vector<int32_t>& kept)
{
    bool finite = true;
    for (int64_t c = 0; c < kg; ++c) {
        double acc = 0.0;
        const float* p = wrow + c * G;
        if (hinv_diag) {
            const float* d = hinv_diag + c * G;
            for (int j = 0; j < G; ++j) {
                const double t = static_cast<double>(p[j]) / static_cast<double>(d[j]);
                acc += t * t;
            }
        } else {
            for (int j = 0; j < G; ++j) acc += static_cast<double>(p[j]) * static_cast<double>(p[j]);
        }
        sal[c] = acc;
        finite &= std::isfinite(acc);
    }
    kept.clear();
    if (keep == 0 || !finite) return finite;
    std::iota(order.begin(), order.end(), 0);
    const int64_t drop = kg - keep;
    auto less = [&](int32_t a, int32_t b) {
        return sal[a] < sal[b] || (sal[a] == sal[b] && a < b);
    };
    if (drop > 0) std::nth_element(order.begin(), order.begin() + drop, order.end(), less);
    kept.assign(order.begin() + drop, order.end());
    std::sort(kept.begin(), kept.end());
    return true;
}

}  // namespace

int64_t balanced_keep(int64_t kg, double sparsity)
{
    double drop = std::floor(sparsity * static_cast<double>(kg) + 0.5);
    drop = std::min(static_cast<double>(kg), std::max(0.0, drop));
    return kg - static_cast<int64_t>(drop);
}

// Row pointers from the kept count of every row (keep_per_row, or the same count for every row
// from the sparsity).
gqsa_status_t row_pointers(gqsa_matrix* m, const int32_t* keep_per_row, double sparsity)
{
    const int64_t kg = m->K / m->G;
    m->rowIndex.assign(static_cast<size_t>(m->N) + 1, 0);
    const int64_t uniform_keep = keep_per_row ? -1 : balanced_keep(kg, sparsity);
    int64_t total = 0;
    for (int64_t n = 0; n < m->N; ++n) {
        const int64_t keep = keep_per_row ? keep_per_row[n] : uniform_keep;
        if (keep < 0 || keep > kg) return GQSA_ERR_RANGE;
        total += keep;
        if (total > std::numeric_limits<int32_t>::max()) return GQSA_ERR_SHAPE;
        m->rowIndex[n + 1] = static_cast<int32_t>(total);
    }
    return GQSA_OK;
}

gqsa_status_t pack_dense(const float* W, int64_t N, int64_t K, int G, int bits,
                         const int32_t* keep_per_row, double sparsity, const float* hinv_diag,
                         gqsa_matrix* m)
{
    if (hinv_diag)
        for (int64_t k = 0; k < K; ++k)
            if (!(hinv_diag[k] > 0.0f) || !std::isfinite(hinv_diag[k])) return GQSA_ERR_RANGE;
    const int64_t kg = K / G;
    const int cb = G * bits / 8;
    m->N = N; m->K = K; m->G = G; m->bits = bits;
    try {
        if (gqsa_status_t st = row_pointers(m, keep_per_row, sparsity)) return st;
    } catch (const std::bad_alloc&) { return GQSA_ERR_ALLOC; }
    const int64_t total = m->nnzg();
    try {
        m->groups.assign(total, 0);
        m->values.assign(static_cast<size_t>(total) * cb, 0);
        m->scales.assign(total, 0);
        m->zeros.assign(total, 0);
    } catch (const std::bad_alloc&) { return GQSA_ERR_ALLOC; }

    // rows are independent: split them over host threads
    unsigned nthreads = std::max(1u, std::min(16u, std::thread::hardware_concurrency()));
    if (N * K < (1 << 20)) nthreads = 1;
    std::atomic<int64_t> next_row{0};
    std::atomic<bool> bad{false}, out_of_memory{false};
    // (a worker thread must not let an exception escape: that would end the process)
    auto work = [&]() noexcept {
      try {
        std::vector<double> sal(kg);
        std::vector<int32_t> order(kg), kept;
        std::vector<uint8_t> q(G);
        constexpr int64_t kChunk = 16;
        for (;;) {
            const int64_t r0 = next_row.fetch_add(kChunk);
            if (r0 >= N) break;
            const int64_t r1 = std::min(N, r0 + kChunk);
            for (int64_t n = r0; n < r1; ++n) {
                const float* wrow = W + n * K;
                const int64_t g0 = m->rowIndex[n];
                const int64_t keep = m->rowIndex[n + 1] - g0;
                if (!select_row(wrow, hinv_diag, kg, G, keep, sal, order, kept)) { bad = true; continue; }
                for (int64_t i = 0; i < keep; ++i) {
                    const int64_t g = g0 + i;
                    const int32_t c = kept[i];
                    m->groups[g] = c;
                    if (!quantise_group(wrow + static_cast<int64_t>(c) * G, G, bits, q.data(), &m->scales[g], &m->zeros[g])) {
                        bad = true;
                        continue;
                    }
                    uint8_t* dst = &m->values[static_cast<size_t>(g) * cb];
                    if (bits == 8) {
                        std::memcpy(dst, q.data(), G);
                    } else {
                        for (int j = 0; j < G; j += 2)
                            dst[j / 2] = static_cast<uint8_t>(q[j] | (q[j + 1] << 4));
                    }
                }
            }
        }
      } catch (...) {
        out_of_memory = true;
      }
    };
    if (nthreads == 1) {
        work();
    } else {
        std::vector<std::thread> pool;
        try {
            pool.reserve(nthreads);
            for (unsigned t = 0; t < nthreads; ++t) pool.emplace_back(work);
        } catch (...) {
            // no more threads to be had: the ones that started (or this one) do all the rows
        }
        if (pool.empty()) work();
        for (auto& t : pool) t.join();
    }
    if (out_of_memory) return GQSA_ERR_ALLOC;
    if (bad) return GQSA_ERR_RANGE;
    return GQSA_OK;
}

// Where the rows start in the group stream.  span_groups = 0: one after the other, row n at
// rowIndex[n].  Otherwise the stream is cut into spans of span_groups positions (one per
// workgroup) and a row that fits a span but not what is left of the current one starts at the next
// span; the positions skipped hold null groups (they add nothing to the row before them).  A row
// longer than a span starts where the previous one ended.  Returns the length of the stream (one
// past the last stored group).
int64_t place_rows(const gqsa_matrix& m, int64_t span_groups, std::vector<int64_t>* row_pos)
{
    if (row_pos) row_pos->assign(static_cast<size_t>(m.N), 0);
    int64_t pos = 0;
    for (int64_t n = 0; n < m.N; ++n) {
        const int64_t cnt = m.rowIndex[n + 1] - m.rowIndex[n];
        if (span_groups > 0 && cnt > 0 && cnt <= span_groups && pos % span_groups + cnt > span_groups)
            pos = (pos / span_groups + 1) * span_groups;
        if (row_pos) (*row_pos)[static_cast<size_t>(n)] = pos;
        pos += cnt;
    }
    return pos;
}

namespace {

// Partition by size alone (measured on MI355X).  K up to 4096, or fewer than 2048 tiles: one tile
// per worker -- everything it needs requested at once, one segmented scan to settle it -- up to
// 16384 workers (several rounds of wavefronts per compute unit stream better than a few long
// runs), beyond that the fewest tiles per worker that keep to that count; workgroups of 4
// wavefronts (small workgroups meet sooner after x is staged and fill the compute units more
// evenly), a multiple of 4 of them so that the small-batch kernels can take the same workers 8
// or 16 to a workgroup.  Larger K, where staging x (48 bytes of LDS per 16 elements) is a large
// part of a workgroup's work: 8 wavefronts per workgroup and 256 or 512 workgroups -- one or two
// per compute unit, all alike -- as many as keep the bytes of x staged by all workgroups to
// about a quarter of the matrix's: the multiple of 256 nearest to 448 T / K (beyond K = 8192 the
// one below), at most 512 (a third
// workgroup per compute unit measured slower on every large shape: 23.1 against 22.5 us on
// 28672x8192 at 50 %, 30 against 24 us with the uneven rows of the stress shape of that size).
void partition_by_size(int64_t n_tiles, int64_t K, int64_t* per_worker, int64_t* n_workgroups, int64_t* waves_per_workgroup)
{
    if (K <= 4096 || n_tiles < 2048) {
        *per_worker = std::max<int64_t>(1, (n_tiles + 16383) / 16384);
        const int64_t workers = std::max<int64_t>(1, (n_tiles + *per_worker - 1) / *per_worker);
        *waves_per_workgroup = std::min<int64_t>(4, workers);
        *n_workgroups = (workers + *waves_per_workgroup - 1) / *waves_per_workgroup;
        if (*n_workgroups > 4) *n_workgroups = (*n_workgroups + 3) / 4 * 4;
    } else {
        *per_worker = 0;      // (whatever the deal gives)
        *waves_per_workgroup = 8;
        // round(448 T / K / 256); beyond K = 8192, where a workgroup stages 22 KB of x and more before
        // it can start, rounded down (4096x11008 and 4096x14336 without pruning: 10.1 and 12.3 us with
        // 256 workgroups against 10.9 and 12.9 us with 512)
        const int64_t per_cu = (448 * n_tiles + (K > 8192 ? 0 : 128 * K)) / (256 * K);
        *n_workgroups = kMaxDefaultWorkgroups * std::max<int64_t>(1, std::min<int64_t>(2, per_cu));
    }
}

// Rows kept inside the workers' runs: tiles of U blocks with L of the 64 lanes in use (L * U
// stream positions), t tiles per worker, every worker a span of its own (place_rows) -- a worker
// then holds whole rows only, settles them with its one segmented scan per tile and ends; there
// is no fix-up, no second barrier, nothing for a workgroup to wait for.  (Measured on an MI355X:
// with the rows of 4096x4096 at 30 % sparsity shared between wavefronts a call takes 5.0 us; kept
// apart it takes 4.8 us even in tiles of 4 x 64, where 30 % of the stream is null groups, and
// 4.3 us in tiles of 3 x 60.)  The shape is chosen so that few positions stay empty: 179 groups
// per row fit 3 x 60, two rows of 77 fit 3 x 52, 205 fit 4 x 52, 344 fit 6 x 60, 448 fit 8 x 56.
// Eligible: the shapes the kernel has (tile_shape_supported) that leave at most an eighth of the
// stored groups' count of positions empty with at most 16384 workers -- one tile per worker; for
// K up to 4096, if no shape is eligible (e.g. more than 16384 tiles), 2, 3 or 4 tiles per worker
// of the format's own shape, the fewest that make it eligible.  Of the eligible shapes, those
// within 1/16 of the stored groups of the fewest empty positions; of these
//   K <= 4096: the format's own shape if it is among them (its kernel has nothing to mask), else
//   the fewest blocks per tile (more wavefronts, each done sooner), then the most lanes in use;
//   K > 4096, where every workgroup stages all of x and workgroups are of 8 wavefronts: only with
//   2048 workers or more (a workgroup per compute unit); the fewest workers, then the most lanes
//   in use, then the fewest blocks (4096x11008 at 50 %: 6.2 us in tiles of 6 x 60 against 6.6 us
//   with the rows kept inside the workgroups' spans; 4096x14336 at 70 %: 5.6 against 6.1 us).
bool partition_by_rows(const gqsa_matrix& m, Partition* out)
{
    const bool wide = m.K > 4096;     // x is a large part of what a workgroup reads: fewer, larger workgroups
    const int cb = m.code_bytes();
    const int64_t nnz = m.nnzg();
    if (nnz == 0) return false;
    int64_t longest = 0;
    bool uniform = true;          // every non-empty row as long as the longest: placement in closed form
    for (int64_t n = 0; n < m.N; ++n) longest = std::max<int64_t>(longest, m.rowIndex[n + 1] - m.rowIndex[n]);
    int64_t n_rows = 0;
    for (int64_t n = 0; n < m.N; ++n) {
        const int64_t c = m.rowIndex[n + 1] - m.rowIndex[n];
        if (c > 0) ++n_rows;
        if (c > 0 && c != longest) uniform = false;
    }
    const int wpw = wide ? 8 : 4;
    struct Cand { int u, l, t; int64_t spans, pad; };
    const Cand* best = nullptr;
    std::vector<Cand> cands;
    for (int t = 1; t <= (wide ? 1 : 4) && !best; ++t) {
        cands.clear();
        int64_t least = INT64_MAX;
        for (int u = 1; u <= 8; ++u) {
            for (int l = 32; l <= kLanes; l += 4) {
                if (!tile_shape_supported(cb, m.G, u, l)) continue;
                if (t > 1 && !tile_shape_is_own(cb, u, l)) continue;      // tiles of a chosen shape come one to a worker
                const int64_t span = static_cast<int64_t>(l) * u * t;
                if (longest > span) continue;
                int64_t spans;
                if (uniform) {
                    const int64_t per_span = span / longest;
                    spans = (n_rows + per_span - 1) / per_span;
                } else {
                    const int64_t len = place_rows(m, span, nullptr);
                    spans = (len + span - 1) / span;
                }
                const int64_t pad = spans * span - nnz;
                if (spans > 16384 || pad > nnz / 8) continue;
                if (wide && spans < 8 * kMaxDefaultWorkgroups) continue;      // fewer than a workgroup per compute unit
                cands.push_back(Cand{u, l, t, spans, pad});
                least = std::min(least, pad);
            }
        }
        for (const Cand& c : cands) {
            if (c.pad > least + nnz / 16) continue;
            if (!best) { best = &c; continue; }
            const bool own_c = tile_shape_is_own(cb, c.u, c.l), own_b = tile_shape_is_own(cb, best->u, best->l);
            const bool better = wide ? (c.spans != best->spans ? c.spans < best->spans : c.l != best->l ? c.l > best->l : c.u < best->u)
                                     : (own_c != own_b ? own_c : c.u != best->u ? c.u < best->u : c.l > best->l);
            if (better) best = &c;
        }
    }
    if (!best) return false;
    int64_t wgs = (best->spans + wpw - 1) / wpw;
    if (wgs > 4) wgs = (wgs + 3) / 4 * 4;
    if (wgs > kMaxWorkgroups) return false;
    out->n_workgroups = static_cast<int>(wgs);
    out->waves_per_workgroup = wpw;
    out->span_tiles = best->t;
    out->tile_blocks = best->u;
    out->tile_lanes = best->l;
    out->span_per_worker = 1;
    return true;
}

}  // namespace

// Default partition.  If the rows can be kept inside the workers' runs cheaply, they are
// (partition_by_rows).  Otherwise by size (partition_by_size), with tiles of the format's own
// block count, and then: a row whose groups lie in two workgroups costs both an exchange through
// device memory at the very end of their work (about 0.6 us on an MI355X, whatever the size of
// the matrix); null groups cost their bytes.  So, if the rows can be kept inside the workgroups'
// spans (place_rows) with at most 2 MiB of null groups, they are: spans of 4 t tiles for the
// small shapes (t the tiles per worker by size, or one more if that needs too many null groups
// or more than 16384 workers), the workgroup count again a multiple of 4; for the large ones
// the same 256 or 512 workgroups with the smallest span that holds the rows.
Partition default_partition(const gqsa_matrix& m)
{
    Partition part;
    if (partition_by_rows(m, &part)) return part;
    part.tile_blocks = largest_tile(m.code_bytes());
    part.tile_lanes = kLanes;
    const int64_t tile_groups = static_cast<int64_t>(kLanes) * part.tile_blocks;
    const int64_t nnz = m.nnzg();
    const int64_t n_tiles = (nnz + tile_groups - 1) / tile_groups;
    int64_t t = 1, wgs = 1, wpw = 1;
    partition_by_size(n_tiles, m.K, &t, &wgs, &wpw);
    part.n_workgroups = static_cast<int>(std::min<int64_t>(wgs, kMaxWorkgroups));
    part.waves_per_workgroup = static_cast<int>(wpw);
    if (wpw < 4 || wgs < 2) return part;       // a handful of tiles: nothing to keep apart
    const int64_t max_null_groups = (int64_t{2} << 20) / m.group_bytes();
    int64_t span = 0, a_wgs = 0;
    if (t > 0) {
        bool found = false;
        for (int64_t tt = t; tt <= t + 1 && !found; ++tt) {     // the tiles per worker by size, or one more
            span = wpw * tt;
            const int64_t len = place_rows(m, span * tile_groups, nullptr);
            a_wgs = (len + span * tile_groups - 1) / (span * tile_groups);
            if (a_wgs > 4) a_wgs = (a_wgs + 3) / 4 * 4;
            found = len - nnz <= max_null_groups && a_wgs * wpw <= 16384;
        }
        if (!found) return part;
    } else {
        a_wgs = wgs;
        for (span = (n_tiles + wgs - 1) / wgs;; ++span) {
            const int64_t len = place_rows(m, span * tile_groups, nullptr);
            if (len - nnz > max_null_groups) return part;
            if ((len + span * tile_groups - 1) / (span * tile_groups) <= wgs) break;
        }
    }
    if (a_wgs > kMaxWorkgroups || span > INT32_MAX / 2) return part;
    part.n_workgroups = static_cast<int>(a_wgs);
    part.span_tiles = static_cast<int>(span);
    return part;
}

// Device image.  The stored groups, in canonical order, form a stream that is cut into
// blocks of L groups (part.tile_lanes: the lanes of a wavefront that take a group, 64 by default);
// U blocks make a tile -- part.tile_blocks, by default 4 blocks with up to 16
// code bytes per group, 2 with 32, 1 with 64 (a wavefront's tile stays within about 24
// registers).  The stream is padded with null groups to whole tiles.  With span_tiles > 0 the
// rows are first kept inside spans of that many tiles (place_rows): one span per workgroup and
// T = span_tiles * n_workgroups, or (span_per_worker) one span per wavefront worker and
// T = span_tiles * n_workgroups * waves_per_workgroup; n_workgroups = 0 then stands for as many
// as the rows need.  The T tiles are dealt in contiguous, near-equal runs
// to the W = n_workgroups * waves_per_workgroup workers (wavefronts): worker w gets the tiles
// floor(w T / W) .. floor((w+1) T / W) - 1, so that the workers with one tile more are spread
// evenly over the workgroups (the nnz-balanced version of the paper's task-centric split,
// Sec. 3.5; a row may be shared by neighbouring wavefronts).  The deal does
// not depend on how the workers are grouped into workgroups, so a launch may group them
// differently.  In a tile of U blocks lane l owns U consecutive stream positions, stored one
// per block so that every block is a fully coalesced, lane-interleaved load:
//     stream position (first of the tile) + p  ->  block (p mod U), lane (p div U).
// Block = code planes | L x (scale | zero << 16) | L x (16 * LDS slot | head).  A group of
// G = 16 M elements has G*bits/8 code bytes; plane k holds bytes 16k..16k+15 of every lane's
// code string (a single plane of 8 bytes per lane for 4-bit, G = 16).  The index word is the
// byte offset in LDS of the group's first 16 activations (slot = group-column * M) with the
// row-head flag in bit 0; for G = 8 (half a slot per group; 4 or 8 code bytes) it is 16 times the
// group-column itself, with that flag.  4-bit code words are nibble-permuted so that one AND per pair of
// elements yields a packed fp16 pair: word h of a group holds elements 8h..8h+7, element 8h+2m
// at bits 4m and element 8h+2m+1 at bits 16+4m.
// (fill_blocks = false leaves the blocks empty -- the GPU packer writes them -- and row_pos_out,
// if given, receives the first stream position of every row.)
gqsa_status_t build_image(gqsa_matrix* m, const Partition& part, bool fill_blocks, std::vector<int64_t>* row_pos_out)
{
    int n_workgroups = part.n_workgroups;
    const int waves_per_workgroup = part.waves_per_workgroup, span_tiles = part.span_tiles;
    if (n_workgroups < 0 || n_workgroups > kMaxWorkgroups || span_tiles < 0) return GQSA_ERR_RANGE;
    if (n_workgroups == 0 && span_tiles == 0) return GQSA_ERR_RANGE;
    if (waves_per_workgroup < 1 || waves_per_workgroup > kWavesPerWorkgroup) return GQSA_ERR_RANGE;
    if (part.span_per_worker && span_tiles == 0) return GQSA_ERR_RANGE;
    const int cb = m->code_bytes();
    const int u_max = part.tile_blocks ? part.tile_blocks : largest_tile(cb);
    const int lanes = part.tile_lanes ? part.tile_lanes : kLanes;
    if (!tile_shape_supported(cb, m->G, u_max, lanes)) return GQSA_ERR_UNSUPPORTED;
    // (the kernels for tiles of a chosen shape take one tile per worker)
    if (!tile_shape_is_own(cb, u_max, lanes) && !(part.span_per_worker && span_tiles == 1)) return GQSA_ERR_UNSUPPORTED;
    const int64_t tile_groups = static_cast<int64_t>(lanes) * u_max;
    if (span_tiles > (int64_t{1} << 40) / tile_groups) return GQSA_ERR_RANGE;
    // rows -> stream positions; with spans, one span per workgroup or per worker
    std::vector<int64_t> row_pos;
    const int64_t span_groups = span_tiles * tile_groups;
    const int64_t len = place_rows(*m, span_groups, &row_pos);       // one past the last stored group
    int64_t n_tiles = (len + tile_groups - 1) / tile_groups;
    if (span_tiles > 0) {
        const int64_t n_spans = std::max<int64_t>(1, (len + span_groups - 1) / span_groups);
        const int64_t per_wg = part.span_per_worker ? waves_per_workgroup : 1;      // spans of a workgroup
        const int64_t wgs_needed = (n_spans + per_wg - 1) / per_wg;
        if (n_workgroups == 0) n_workgroups = static_cast<int>(std::min<int64_t>(wgs_needed, kMaxWorkgroups + 1));
        if (wgs_needed > n_workgroups || n_workgroups > kMaxWorkgroups) return GQSA_ERR_RANGE;
        n_tiles = static_cast<int64_t>(span_tiles) * n_workgroups * per_wg;
    }
    const int n_waves = n_workgroups * waves_per_workgroup;
    const int64_t nb = n_tiles * u_max;
    const size_t bb = static_cast<size_t>(m->group_bytes()) * lanes;
    auto align = [](size_t v) { return (v + kAlign - 1) / kAlign * kAlign; };

    std::vector<int32_t> nonempty, empty;
    std::vector<int64_t> head_pos;          // stream positions of the row heads, ascending
    std::vector<uint8_t> head(static_cast<size_t>(len) + 1, 0);
    for (int64_t n = 0; n < m->N; ++n) {
        if (m->rowIndex[n + 1] > m->rowIndex[n]) {
            nonempty.push_back(static_cast<int32_t>(n));
            head_pos.push_back(row_pos[static_cast<size_t>(n)]);
            head[static_cast<size_t>(row_pos[static_cast<size_t>(n)])] = 1;
        } else {
            empty.push_back(static_cast<int32_t>(n));
        }
    }

    ImageMap map;
    map.blocks = 0;
    map.wave_info = align(static_cast<size_t>(nb) * bb);
    map.row_of_rank = align(map.wave_info + static_cast<size_t>(n_waves) * 16);
    map.empty_rows = align(map.row_of_rank + nonempty.size() * 4);
    map.total = std::max(kAlign, align(map.empty_rows + empty.size() * 4));

    std::vector<uint8_t> img;
    try {
        img.assign(map.total, 0);
    } catch (const std::bad_alloc&) { return GQSA_ERR_ALLOC; }

    // A lane's code string: 4-bit codes as nibble-permuted words (word h = elements 8h..8h+7),
    // 8-bit codes as they are.  In the block it is cut into planes of at most 16 bytes per lane.
    const int slots_per_group = m->G >= 16 ? m->G / 16 : 1;    // activation slots a group spans (16 elements each; 8 for G = 8)
    const int plane_bytes = std::min(cb, 16);
    std::vector<uint8_t> code(static_cast<size_t>(cb));
    auto put_group = [&](int64_t g, int64_t pos) {
        const int64_t p = pos % tile_groups;
        const int64_t block = pos / tile_groups * u_max + p % u_max;
        const int lane = static_cast<int>(p / u_max);
        uint8_t* base = img.data() + static_cast<size_t>(block) * bb;
        const uint8_t* v = &m->values[static_cast<size_t>(g) * cb];
        if (m->bits == 4) {
            for (int h = 0; h < cb / 4; ++h) {
                uint32_t word = 0;
                for (int e = 0; e < 8; ++e) {
                    const int j = 8 * h + e;
                    const uint32_t q = (j & 1) ? (v[j >> 1] >> 4) : (v[j >> 1] & 0xF);
                    word |= q << ((e & 1) ? 16 + 4 * (e >> 1) : 4 * (e >> 1));
                }
                std::memcpy(&code[4 * static_cast<size_t>(h)], &word, 4);
            }
        } else {
            std::memcpy(code.data(), v, cb);
        }
        for (int pl = 0; pl * plane_bytes < cb; ++pl)
            std::memcpy(base + static_cast<size_t>(pl) * lanes * plane_bytes + static_cast<size_t>(lane) * plane_bytes,
                        &code[static_cast<size_t>(pl) * plane_bytes], plane_bytes);
        const uint32_t sz = static_cast<uint32_t>(m->scales[g]) |
                            (static_cast<uint32_t>(m->zeros[g]) << 16);
        std::memcpy(base + static_cast<size_t>(lanes) * cb + lane * 4, &sz, 4);
        // byte offset in LDS of the group's first 16 activations, row-head flag in bit 0
        const uint16_t ix = static_cast<uint16_t>(((m->groups[g] * slots_per_group) << 4) | (head[static_cast<size_t>(pos)] ? 1 : 0));
        std::memcpy(base + static_cast<size_t>(lanes) * cb + lanes * 4 + lane * 2, &ix, 2);
    };
    if (fill_blocks)
        for (int64_t n = 0; n < m->N; ++n)
            for (int64_t g = m->rowIndex[n]; g < m->rowIndex[n + 1]; ++g)
                put_group(g, row_pos[static_cast<size_t>(n)] + (g - m->rowIndex[n]));

    // Per worker: {rank_base, tail_closed + 2 * lead_len, lead_first, chain_len}.  (A null group
    // between two rows counts as part of the row before it.)
    //   rank_base   rank (among non-empty rows) of the row that is open when the run starts,
    //               i.e. (row heads before the run) - 1
    //   tail_closed 1 if the row open at the end of the run has no group beyond it
    //   lead_first  worker holding the head of the row that the run's first groups continue,
    //               or -1 if the run starts on a row head or past the last group; a worker
    //               without blocks in the middle of a row has it too (it passes 0 along)
    //   chain_len   for a worker that holds the head of a row continuing past its run: the
    //               number of consecutive workers holding groups of that row, else 0
    //   lead_len    chain_len of worker lead_first (0 without one): tells the worker how the row
    //               it continues is settled without a look at the other worker's record
    auto heads_below = [&](int64_t pos) {
        return static_cast<int64_t>(std::lower_bound(head_pos.begin(), head_pos.end(), pos) -
                                    head_pos.begin());
    };
    // even deal: worker w owns the tiles floor(w T / W) .. floor((w+1) T / W) - 1
    std::vector<int64_t> first_block(static_cast<size_t>(n_waves) + 1, 0);
    for (int w = 0; w <= n_waves; ++w) first_block[w] = (static_cast<int64_t>(w) * n_tiles / n_waves) * u_max;
    auto worker_of = [&](int64_t pos) {   // the worker whose run contains stream position pos
        const int64_t blk = pos / lanes;
        return static_cast<int32_t>(std::upper_bound(first_block.begin(), first_block.end(), blk) -
                                    first_block.begin() - 1);
    };
    int32_t* info = reinterpret_cast<int32_t*>(img.data() + map.wave_info);
    int fix = 0;
    for (int w = 0; w < n_waves; ++w) {
        const int64_t mine = first_block[w + 1] - first_block[w];
        const int64_t first = first_block[w] * lanes;
        const int64_t end = first_block[w + 1] * lanes;
        const int64_t hb = heads_below(std::min(first, len));
        const int64_t he = heads_below(std::min(end, len));
        const int closed = (end >= len || head[static_cast<size_t>(end)]) ? 1 : 0;
        int32_t lead_first = -1, chain_len = 0;
        if (first < len && !head[static_cast<size_t>(first)]) lead_first = worker_of(head_pos[hb - 1]);
        if (mine > 0 && !closed && he > hb) {
            const int64_t row_last = (he < static_cast<int64_t>(head_pos.size()) ? head_pos[he] : len) - 1;
            chain_len = worker_of(row_last) - w + 1;
            fix = 1;
        }
        info[4 * w + 0] = static_cast<int32_t>(hb - 1);
        info[4 * w + 1] = closed;
        info[4 * w + 2] = lead_first;
        info[4 * w + 3] = chain_len;
    }
    for (int w = 0; w < n_waves; ++w)
        if (info[4 * w + 2] >= 0) info[4 * w + 1] += 2 * info[4 * info[4 * w + 2] + 3];
    if (!nonempty.empty())
        std::memcpy(img.data() + map.row_of_rank, nonempty.data(), nonempty.size() * 4);
    if (!empty.empty())
        std::memcpy(img.data() + map.empty_rows, empty.data(), empty.size() * 4);

    if (row_pos_out) row_pos_out->swap(row_pos);
    m->image.swap(img);
    m->map = map;
    m->n_workgroups = n_workgroups;
    m->waves_per_workgroup = waves_per_workgroup;
    m->span_tiles = span_tiles;
    m->span_per_worker = part.span_per_worker ? 1 : 0;
    m->tile_blocks = u_max;
    m->tile_lanes = lanes;
    m->n_waves = n_waves;
    m->n_blocks = nb;
    m->n_tiles = n_tiles;
    m->n_empty = static_cast<int64_t>(empty.size());
    m->needs_fixup = fix;
    return GQSA_OK;
}

}  // namespace gqsa
