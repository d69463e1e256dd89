/*
 * gqsa.h -- C ABI of the MI355X (gfx950) GQSA group-sparse, group-quantised GEMV.
 *
 * The library implements the inference hot path of GQSA ("Group Quantization
 * and Sparsity for Accelerating LLM Inference"): a linear layer y = W x whose
 * weight is stored in the paper's Block-Sparse-Row form (Sec. 3.2) -- only the
 * surviving length-G groups of every output row are kept, as n-bit codes with
 * one scale and one zero-point per group (Sec. 3.1, Eq. 1-2), a group-column
 * index per stored group and row pointers -- multiplied at decode time as a
 * 1xNxK GEMV (Sec. 3.5) with in-register dequantisation (Eq. 3).
 *
 * Conventions
 *   - plain C linkage, plain pointers and sizes; every pointer is marked
 *     [host] or [device] below; nothing is thrown across the boundary.
 *   - every call returns a gqsa_status_t; on failure output handles are NULL
 *     and output buffers are unspecified.
 *   - a handle owns its host arrays, its device image and its device carry
 *     workspace; x and y are borrowed for the duration of the enqueued work.
 *   - pack / import / export / info never touch the GPU and work on a machine
 *     without one; the device image is created by gqsa_upload or by the first
 *     gqsa_gemv on the handle.
 *   - one gqsa_gemv may be in flight per handle at a time (the carry workspace
 *     is shared); calls on one stream are ordered and therefore safe.
 */
#ifndef GQSA_H
#define GQSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gqsa_matrix* gqsa_handle_t;

typedef enum {
    GQSA_OK = 0,
    GQSA_ERR_NULL = 1,         /* a required pointer is NULL */
    GQSA_ERR_SHAPE = 2,        /* N<=0, K<=0, K % G != 0, K > 65536, inconsistent arrays */
    GQSA_ERR_UNSUPPORTED = 3,  /* bits not 4/8, G not 8/16/32/64/128 (8-bit: up to 64), batch outside 1..16 */
    GQSA_ERR_RANGE = 4,        /* sparsity outside [0,1], keep count outside [0,K/G], non-finite W, a kept group whose
                                  range / (2^n - 1) is beyond the largest fp16 number (its scale could not be stored) */
    GQSA_ERR_ALLOC = 5,        /* host allocation failed */
    GQSA_ERR_HIP = 6,          /* a HIP runtime call failed (no device, launch error, ...) */
    GQSA_ERR_BUFSIZE = 7,      /* caller buffer smaller than required */
    GQSA_ERR_ALIGN = 8,        /* device pointer not 16-byte aligned */
    GQSA_ERR_IO = 9            /* file could not be opened, read or written (also: truncated) */
} gqsa_status_t;

typedef struct {
    int64_t N;                  /* output rows */
    int64_t K;                  /* reduction length */
    int32_t G;                  /* group size */
    int32_t bits;               /* code width */
    int64_t nnz_groups;         /* stored groups = rowIndex[N] */
    int64_t values_bytes;       /* bytes of the canonical `values` array */
    int64_t n_blocks;           /* blocks of the device stream (tile_lanes positions each, null groups included) */
    int32_t n_workgroups;       /* workgroups the group stream is dealt to */
    int32_t waves_per_workgroup;/* wavefront workers per workgroup */
    int32_t needs_fixup;        /* 1 if some row is shared by two or more wavefront workers */
    int32_t span_tiles;         /* tiles per workgroup span that rows are kept inside (0: no such spans) */
    int64_t n_empty_rows;       /* rows without any stored group */
    int64_t device_bytes;       /* size of the device image */
    int64_t algorithmic_bytes;  /* compressed bytes one batch-1 call must move (see README of bench) */
    int32_t on_device;          /* 1 once the device image exists */
    int32_t panel_integer_zeros;/* 1 if the second image exists and every stored zero is an integer of magnitude
                                   <= 1024: its kernel then subtracts the zero from the codes (exactly, in fp16)
                                   before the product instead of from the product's sum afterwards */
    int64_t panel_bytes;        /* size of the second image built by gqsa_build_panels, 0 without one */
    int32_t tile_blocks;        /* blocks per tile of the device stream */
    int32_t tile_lanes;         /* stream positions per block: the lanes of a wavefront that take a group (64, or 32..60) */
    int32_t span_per_worker;    /* 1 if a span is one wavefront worker's run (rows never straddle workers), 0 if a workgroup's */
    int32_t reserved0;
} gqsa_info_t;

/*
 * Offline pre-processing (Sec. 3.2; Fig. 3): group the fp32 matrix along K in
 * runs of G, score every group by its sum of squares, prune the least salient
 * groups of every row and quantise the kept ones with Eq. 1-2.
 *   W_host   [host] row-major fp32 [N,K], finite
 *   sparsity fraction of the K/G groups pruned in EVERY row; the pruned count is
 *            floor(sparsity*K/G + 0.5); equal saliencies prune the lower column first
 *   out      [host] receives the handle
 * Scale is stored as fp16 (floored at 2^-14); zero-point = round-half-even(-min/scale)
 * clamped to +-2048 and stored as fp16; codes = clamp(round(w/scale)+zero, 0, 2^bits-1).
 * Group sizes (the axis of the paper's group-size ablation, Sec. 4.5): G = 8, 16, 32, 64 or 128
 * with 4-bit codes, 8, 16, 32 or 64 with 8-bit codes (at most 64 code bytes per group); K a
 * multiple of 16 and of G, K <= 65536 (G = 8: K <= 32768).
 */
gqsa_status_t gqsa_pack(const float* W_host, int64_t N, int64_t K, int G, int bits,
                        double sparsity, gqsa_handle_t* out);

/* Same, with the kept-group count of every row given (imbalanced sparsity; the worked
 * example of Sec. 3.2 keeps 1, 2, 0, 1 groups).  keep_per_row [host] int32[N]. */
gqsa_status_t gqsa_pack_rows(const float* W_host, int64_t N, int64_t K, int G, int bits,
                             const int32_t* keep_per_row, gqsa_handle_t* out);

/*
 * Same as gqsa_pack, with the paper's Hessian metric deciding which groups go (Sec. 3.1, Eq. 4):
 * the saliency of a weight is w^2 / d_k^2, d = diag(H^-1) of the layer's Hessian over its K
 * inputs, and a group's saliency is the sum over its members (Fig. 3 averages, same order).
 *   hinv_diag [host] fp32[K], every entry finite and > 0 (GQSA_ERR_RANGE otherwise)
 * The Hessian itself comes from calibration activations and is the caller's business; d = 1
 * everywhere gives gqsa_pack.  Quantisation of the kept groups does not depend on d.
 */
gqsa_status_t gqsa_pack_hessian(const float* W_host, int64_t N, int64_t K, int G, int bits,
                                double sparsity, const float* hinv_diag, gqsa_handle_t* out);

/*
 * The same offline pre-processing on the GPU (Sec. 3.2, Fig. 3; Eq. 1-2; Eq. 4): saliency of every
 * group, pruning of every row, quantisation of the kept groups and the blocks of the device image
 * are computed by HIP kernels from a matrix that already lies in device memory -- the same
 * arithmetic as gqsa_pack / gqsa_pack_rows / gqsa_pack_hessian operation for operation, hence
 * the same bits in the canonical arrays and in the device image.
 *   W_dev          [device] row-major fp32 [N,K], finite (GQSA_ERR_RANGE otherwise)
 *   sparsity       as in gqsa_pack; ignored when keep_per_row is given
 *   keep_per_row   [host] int32[N] as in gqsa_pack_rows, or NULL
 *   hinv_diag_dev  [device] fp32[K] as in gqsa_pack_hessian (finite, > 0: GQSA_ERR_RANGE
 *                  otherwise), or NULL for the sum-of-squares saliency
 *   hip_stream     the kernels and copies run on it; the call waits for it before it returns
 *   out            [host] receives a handle that is already on the device (the current one);
 *                  its canonical arrays and its host copy of the image have been copied back,
 *                  so export, save and info work as for a host-packed handle
 * Allocates device memory (the image, the workspace, temporaries of about 14 bytes per stored
 * group) and synchronises: not for use under stream capture.  The default partition is chosen
 * as by gqsa_pack; gqsa_set_partition is not possible afterwards (the handle is uploaded).
 */
gqsa_status_t gqsa_pack_device(const float* W_dev, int64_t N, int64_t K, int G, int bits, double sparsity,
                               const int32_t* keep_per_row, const float* hinv_diag_dev, void* hip_stream,
                               gqsa_handle_t* out);

/*
 * Build a handle from existing canonical arrays (the BSR listing of Sec. 3.2 plus the
 * per-group parameters of Eq. 1, which Sec. 3.4 fine-tunes freely -- so scale and zero
 * are arbitrary finite fp16 values here).  All arrays [host]; they are copied.
 *   rowIndex int32[N+1] non-decreasing from 0; groups int32[nnzg] strictly ascending
 *   inside a row, in [0,K/G); values uint8[nnzg*G*bits/8] (4-bit: element 2b in the low
 *   nibble of byte b, 2b+1 in the high nibble); scales_f16/zeros_f16 uint16[nnzg].
 */
gqsa_status_t gqsa_import(const int32_t* rowIndex, const int32_t* groups, const uint8_t* values,
                          const uint16_t* scales_f16, const uint16_t* zeros_f16,
                          int64_t N, int64_t K, int G, int bits, gqsa_handle_t* out);

/* Re-partition the group stream over n_workgroups (1..4096) x waves_per_workgroup (1..16)
 * wavefront workers and rebuild the host copy of the device image.  Only before the handle is
 * uploaded.  The stream is cut into tiles of 4 blocks of 64 groups (2 blocks with 32 code bytes
 * per group, 1 with 64); worker w owns the tiles floor(w T / W) .. floor((w+1) T / W) - 1 of the
 * T tiles, W being the worker count.
 *
 * The default chosen by pack/import/load (Sec. 3.5's task-centric split: a worker's share is a
 * count of stored groups, not of rows):
 *  (1) rows kept inside the workers' runs, if empty positions amounting to at most an eighth of
 *      the stored groups and at most 16384 workers achieve that (gqsa_set_partition_rows below):
 *      of the tile shapes the kernel has (for G = 16: 3, 4, 5 blocks -- 4-bit codes also 6 and
 *      8 -- with 32, 36, .. 64 lanes in use; else the format's own block count with 64 lanes),
 *      one tile per worker (if none is eligible and K <= 4096: 2, 3 or 4 tiles of the format's
 *      own shape, the fewest that are), among those within 1/16 of the stored groups of the
 *      fewest empty positions --
 *      K <= 4096: the format's own shape if it is among them, else the fewest blocks per tile,
 *      then the most lanes in use; workgroups of 4 wavefronts;
 *      K > 4096 (a workgroup stages all of x: fewer, larger workgroups): only with at least
 *      2048 workers; the fewest workers, then the most lanes in use, then the fewest blocks;
 *      workgroups of 8 wavefronts.
 *      The workgroup count is rounded up to a multiple of 4.  Matrices pruned to the same count
 *      in every row take this form.
 *  (2) otherwise by size: for K up to 4096 (or fewer than 2048 tiles) one tile per worker (at
 *      most 16384 workers; more tiles per worker beyond) in workgroups of 4 wavefronts, the
 *      workgroup count rounded up to a multiple of 4; for larger K workgroups of 8 wavefronts,
 *      256 or 512 of them (one or two per compute unit of an MI355X): the multiple of 256
 *      nearest to 448 T / K (beyond K = 8192: the one below), at most 512.  If some row would then lie in two workgroups and 2 MiB of null
 *      groups or less keep every row inside one, the aligned form below with the same wavefronts
 *      per workgroup and: small shapes -- spans of 4 t tiles, t the tiles per worker (or one
 *      more, if that takes too many null groups or more than 16384 workers), the workgroup count
 *      rounded up to a multiple of 4; large shapes -- the same 256 or 512 workgroups and the
 *      smallest span that holds the rows. */
gqsa_status_t gqsa_set_partition(gqsa_handle_t h, int n_workgroups, int waves_per_workgroup);

/* That default, for a matrix known by its row pointers alone (host only, no handle is built):
 * out[6] = {n_workgroups, waves_per_workgroup, span_tiles, tile_blocks, tile_lanes, span_per_worker}
 * (span_tiles as in gqsa_set_partition_aligned / tiles_per_worker of gqsa_set_partition_rows, 0
 * for the plain deal).  rowIndex [host] int32[N+1] as in gqsa_import. */
gqsa_status_t gqsa_default_partition(const int32_t* rowIndex, int64_t N, int64_t K, int G, int bits,
                                     int32_t out[6]);

/*
 * Same, with the rows kept inside the workgroups' shares (a row shared by two workgroups costs
 * both an exchange through device memory at the end of the launch): the stream is cut into spans
 * of span_tiles tiles, one per workgroup; a row that fits a span but not what is left of the
 * current one starts at the next span, the positions skipped hold null groups (read like any
 * other, adding nothing); a longer row starts where the previous one ended.  T = span_tiles *
 * n_workgroups tiles are dealt as above.
 *   span_tiles          >= 1
 *   n_workgroups        1..4096, or 0 for as many as the rows need; GQSA_ERR_RANGE if the rows
 *                       need more spans than that
 *   waves_per_workgroup 1..16
 */
gqsa_status_t gqsa_set_partition_aligned(gqsa_handle_t h, int span_tiles, int n_workgroups,
                                         int waves_per_workgroup);

/*
 * Same, with the rows kept inside the single workers' runs.  A tile has tile_blocks blocks of
 * tile_lanes stream positions (tile_lanes of a wavefront's 64 lanes take a group of every block;
 * a block then has tile_lanes entries in each of its arrays), and every worker is a span of
 * tiles_per_worker tiles of its own (rows placed as above).  A worker whose rows all fit its span
 * shares no row with a neighbour: it writes its rows and ends, and the launch has no fix-up
 * phase (Sec. 3.5's straggler problem does not arise where the rows are of similar length; the
 * positions left empty pay for it).  T = tiles_per_worker * n_workgroups * waves_per_workgroup.
 *   tile_blocks, tile_lanes   a tile shape the kernel is compiled for -- G = 16: 3, 4, 5 blocks
 *                       (4-bit codes: also 6, 8) and 32, 36, .. 64 lanes; any format: its own
 *                       block count (4, 2 or 1, see gqsa_set_partition) with 64 lanes -- else
 *                       GQSA_ERR_UNSUPPORTED
 *   tiles_per_worker    1; of the format's own shape also more
 *   n_workgroups        1..4096, or 0 for as many as the rows need; GQSA_ERR_RANGE if they need more
 *   waves_per_workgroup 1..16
 */
gqsa_status_t gqsa_set_partition_rows(gqsa_handle_t h, int tile_blocks, int tile_lanes, int tiles_per_worker,
                                      int n_workgroups, int waves_per_workgroup);

/*
 * Build a second image of the matrix for calls with several activation rows (the small-batch
 * side of Sec. 3.5's kernel, which may use the matrix cores): the stored groups of 16 consecutive
 * output rows ordered by group-column, so that one group-column of such a panel and the
 * activations under it are a dense 16x16x16 product (absent groups count as zeros).  Codes,
 * scales and zeros are the same bits as in the canonical arrays; the image takes about 12.5
 * bytes per stored 4-bit group of 16 on top of the first one.  Host only; only before the handle
 * is uploaded (GQSA_ERR_UNSUPPORTED after); G >= 16 (GQSA_ERR_UNSUPPORTED for G = 8; a group of
 * 32, 64 or 128 weights takes 2, 4 or 8 products).  Once built, gqsa_upload copies both images and
 * gqsa_gemv / gqsa_gemv_multi use this one for batch >= 5 with G = 16 and K <= 8192 and for
 * batch >= 3 with larger K or larger groups (gqsa_gemv_multi: still one launch, the workgroups' panels taken from all the
 * matrices so that they share the activations they load, if the matrices have at most 1024 panels
 * of 16 rows together and their zeros are either all small integers or not -- else one launch
 * per matrix; same bits either way); results stay within the same bound (fp32
 * accumulation of exact products, one rounding to fp16) but are not bit-identical to those of
 * the other kernel.
 */
gqsa_status_t gqsa_build_panels(gqsa_handle_t h);

/* gqsa_gemv from the second image whatever the batch (1..16): same arguments, same checks;
 * GQSA_ERR_UNSUPPORTED if the handle has no such image. */
gqsa_status_t gqsa_gemv_panels(gqsa_handle_t h, const void* x_dev, void* y_dev, int batch, void* hip_stream);

/* Copy the exact bytes of that second image into host_buf; bytes >= panel_bytes of gqsa_info.
 * GQSA_ERR_UNSUPPORTED if the handle has none. */
gqsa_status_t gqsa_export_panel_blob(gqsa_handle_t h, void* host_buf, size_t bytes);

/* Create the device image and carry workspace on the current HIP device (synchronous). */
gqsa_status_t gqsa_upload(gqsa_handle_t h);

/*
 * The hot path (Sec. 3.5): enqueue y = W^ x on `hip_stream` and return.
 *   x_dev [device] fp16 [batch,K] row-major, 16-byte aligned
 *   y_dev [device] fp16 [batch,N] row-major, fully overwritten; rows without stored
 *         groups receive +0
 *   batch 1..16
 *   hip_stream a hipStream_t (NULL = the default stream)
 * K must not exceed 32768 (x and its group sums are staged in LDS); GQSA_ERR_UNSUPPORTED else.
 * A launch takes 8, 4, 2 or 1 activation rows; 3 go to the kernel for 4 and 7 to the kernel for 8
 * (group sizes other than 16: one row per launch).
 * fp32 accumulation, one round-to-nearest-even to fp16 per output.  Results are
 * bit-identical from run to run.  Does not synchronise.  The current HIP device must be the one
 * the handle was uploaded on (GQSA_ERR_HIP otherwise).  A handle that is not on the device yet is
 * uploaded by its first call (allocations, a synchronous copy): call gqsa_upload before
 * capturing a stream -- a first call on a capturing stream is refused (GQSA_ERR_UNSUPPORTED).
 */
gqsa_status_t gqsa_gemv(gqsa_handle_t h, const void* x_dev, void* y_dev, int batch,
                        void* hip_stream);

/*
 * gqsa_gemv for callers that cannot allocate device memory or let a library do so: code whose
 * launches are being captured into a HIP graph, tight serving loops, harnesses that forbid it.
 * Same arguments, same checks, same kernels (the wavefront kernel, whatever the batch) and the
 * same bits in y as gqsa_gemv gives without a second image -- but nothing is allocated or freed
 * by the call, and the fix-up workspace (carry records, arrival counters and meeting points of
 * rows shared by wavefronts) is not the handle's: it is a fixed array inside the library's device
 * code, 3 211 264 bytes (196 per wavefront worker, 16384 workers), of which every GPU that the
 * library is used on holds one copy until the process ends.
 *   - the handle must already be on the device (gqsa_upload): GQSA_ERR_UNSUPPORTED otherwise;
 *   - a handle whose partition has more than 16384 wavefront workers (n_workgroups x
 *     waves_per_workgroup of gqsa_info; no default partition has) is refused with GQSA_ERR_BUFSIZE
 *     and a message on stderr;
 *   - all calls on one GPU share the array, whatever the handle: calls that may overlap in time
 *     on one GPU (different streams) race on it and give wrong results; calls on one stream are
 *     ordered and safe.  The part of the array a call uses is cleared by a small kernel ahead of
 *     the GEMV (no memset node, so the call can be captured).
 */
gqsa_status_t gqsa_gemv_static(gqsa_handle_t h, const void* x_dev, void* y_dev, int batch,
                               void* hip_stream);

/*
 * Several matrices that share the activation vector -- q/k/v or gate/up of a decoder layer, the
 * way the paper's engine runs seven GEMVs per layer (Sec. 4.4) -- in ONE launch:
 * y_devs[i] = W^_i x for i < n_matrices (1..4).  The workgroups of the launch are dealt to the
 * matrices (each matrix keeps its own partition), so launch and first-byte latency are paid once
 * and the matrices' weights stream side by side.
 *   handles  [host] array of n_matrices distinct handles with equal K, G and bits (N may
 *            differ); GQSA_ERR_SHAPE otherwise
 *   x_dev    [device] fp16 [batch,K], 16-byte aligned
 *   y_devs   [host] array of n_matrices [device] pointers, y_devs[i] fp16 [batch,N_i]
 * Results are bit-identical to n_matrices separate gqsa_gemv calls (which is what happens behind
 * the call when the handles' partitions differ in their wavefronts per workgroup).
 */
gqsa_status_t gqsa_gemv_multi(const gqsa_handle_t* handles, int n_matrices, const void* x_dev,
                              void* const* y_devs, int batch, void* hip_stream);

gqsa_status_t gqsa_info(gqsa_handle_t h, gqsa_info_t* out);

/* Copy the canonical arrays out; any pointer may be NULL to skip it.  Sizes from gqsa_info:
 * rowIndex N+1, groups/scales/zeros nnz_groups, values values_bytes. */
gqsa_status_t gqsa_export(gqsa_handle_t h, int32_t* rowIndex, int32_t* groups, uint8_t* values,
                          uint16_t* scales_f16, uint16_t* zeros_f16);

/* Copy the exact bytes of the device image (host copy) into host_buf; bytes >= device_bytes. */
gqsa_status_t gqsa_export_device_blob(gqsa_handle_t h, void* host_buf, size_t bytes);

/*
 * The canonical arrays (the Sec. 3.2 listing plus scales and zeros) to and from a file: a 48-byte
 * header ("GQSABSR1", N, K, G, bits, nnz_groups, reserved; little-endian) followed by rowIndex,
 * groups, values, scales, zeros.  gqsa_load checks the file like gqsa_import checks its arrays
 * (GQSA_ERR_SHAPE for an inconsistent or foreign file, GQSA_ERR_IO for one it cannot read to
 * the end) and chooses the default partition.  Host only.
 */
gqsa_status_t gqsa_save(gqsa_handle_t h, const char* path);
gqsa_status_t gqsa_load(const char* path, gqsa_handle_t* out);

void gqsa_free(gqsa_handle_t h);

const char* gqsa_status_string(gqsa_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* GQSA_H */
