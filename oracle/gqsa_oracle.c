/*
 * GQSA CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct reference for what the GQSA hot path
 * computes.  Only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the HIP library never does and shares no
 * source, header, table or helper with this file.
 *
 * What it follows (paper: "GQSA: Group Quantization and Sparsity for
 * Accelerating LLM Inference"):
 *   - Sec. 3.1, Eq. 1: uniform asymmetric quantiser parameters
 *         s = (max - min) / (2^n - 1),   z = -round(min / s)
 *   - Sec. 3.1, Eq. 2: codes  q = clamp(round(W / s) + z, 0, 2^n - 1)
 *   - Sec. 3.1, Eq. 3: dequantisation  W^ = (q - z) * s
 *   - Sec. 3.2 and the caption of Fig. 3: weights are grouped along the row
 *     (reduction) dimension in runs of G, a saliency is averaged per group,
 *     the least salient groups are pruned and discarded, the kept groups are
 *     quantised and stored in Block-Sparse-Row form: rowIndex (prefix offsets
 *     in units of stored groups, length rows+1), groups (0-based group-column
 *     of every stored group) and values (the codes, row after row, group after
 *     group).
 *   - Sec. 3.5: the decode step is the GEMV  y[1,N] = x[1,K] . W^T, each
 *     stored group meeting the activation group named by its real group index.
 *
 * The GEMV is exact arithmetic made cheaper (pruned groups are skipped), so
 * the oracle for it is the plain definition: for every row, for every stored
 * group, for every element, accumulate (q - z) * s * x in float64.
 *
 * Readings of points the paper leaves open (all listed in the design notes):
 *   - saliency of a weight (Sec. 3.1, Eq. 4): w^2 / [H^-1]_kk^2 with H the layer's
 *     Hessian over its K inputs -- so the caller hands in d = diag(H^-1), one
 *     positive number per input column (building H needs calibration
 *     activations, which do not exist here); the group's saliency is the sum of
 *     its members' (same ordering as the average of Fig. 3).  Without d the
 *     saliency is the group's sum of squares (d = 1: same ordering as its L2
 *     norm and as the mean of squared magnitudes);
 *   - round() is round-half-to-even;
 *   - the scale is rounded to fp16 first and that stored value is the one the
 *     zero-point and the codes are computed with; a scale below 2^-14 (constant
 *     group or fp16 underflow) is replaced by 2^-14;
 *   - z is an integer, clamped to +-2048 so that fp16 holds it exactly, and is
 *     NOT clamped to the code range (Eq. 1 has no clamp);
 *   - the pruned count of a row is floor(S * K/G + 0.5); among groups of equal
 *     saliency the one with the lower group-column is pruned first;
 *   - 4-bit codes are stored two per byte, even element in the low nibble.
 *
 * Pins: see tests/test_oracle_*.py (brute force in numpy on tiny shapes, a
 * scipy BSR product, closed-form quantiser properties, a lossless
 * construction, the structure of the paper's worked BSR listing).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- fp16 <-> fp32
 * IEEE-754 binary16, written out by hand (gcc 11 has no _Float16 on x86).     */

float gqsa_oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t expo = (uint32_t)(h >> 10) & 0x1Fu;
    uint32_t mant = (uint32_t)h & 0x3FFu;
    double v;
    if (expo == 0x1Fu) {
        v = mant ? NAN : INFINITY;
    } else if (expo == 0) {
        v = ldexp((double)mant, -24);                 /* subnormal: mant * 2^-24 */
    } else {
        v = ldexp((double)(mant + 1024u), (int)expo - 25); /* (1+m/1024)*2^(e-15) */
    }
    return (float)(sign ? -v : v);
}

/* round-to-nearest-even conversion of a float to binary16 bits */
uint16_t gqsa_oracle_f32_to_f16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t absu = u & 0x7FFFFFFFu;
    if (absu > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);   /* NaN */
    if (absu == 0x7F800000u) return (uint16_t)(sign | 0x7C00u);  /* inf */
    double a = fabs((double)f);
    if (a == 0.0) return sign;
    /* value = m * 2^e with the fp16 grid spacing 2^(max(E,-14)-10) */
    int e2;
    (void)frexp(a, &e2);            /* a = frac * 2^e2, frac in [0.5,1) -> E = e2-1 */
    int E = e2 - 1;
    if (E < -14) E = -14;
    double ulp = ldexp(1.0, E - 10);
    double q = a / ulp;             /* exact: power-of-two scaling */
    double r = nearbyint(q);        /* default rounding mode = ties-to-even */
    /* r in [0, 2048]; 2048 means carry into the next binade */
    uint32_t bits;
    if (E == -14 && r < 1024.0) {
        bits = (uint32_t)r;         /* subnormal or zero */
    } else {
        if (r >= 2048.0) { r = 1024.0; E += 1; }
        if (E > 15) return (uint16_t)(sign | 0x7C00u);  /* overflow -> inf */
        bits = ((uint32_t)(E + 15) << 10) | ((uint32_t)r - 1024u);
    }
    return (uint16_t)(sign | bits);
}

/* ---------------------------------------------------------------- pruning   */

/* Number of groups a row keeps under a balanced sparsity S (reading: the pruned
 * count is floor(S * groups_per_row + 0.5), computed in double).             */
int32_t gqsa_oracle_keep_count(int64_t groups_per_row, double sparsity)
{
    double pruned = floor(sparsity * (double)groups_per_row + 0.5);
    if (pruned < 0.0) pruned = 0.0;
    if (pruned > (double)groups_per_row) pruned = (double)groups_per_row;
    return (int32_t)(groups_per_row - (int64_t)pruned);
}

typedef struct { double sal; int32_t col; } sal_entry;

/* ascending saliency; equal saliency -> lower column first (so it is pruned first) */
static int sal_cmp(const void* pa, const void* pb)
{
    const sal_entry* a = (const sal_entry*)pa;
    const sal_entry* b = (const sal_entry*)pb;
    if (a->sal < b->sal) return -1;
    if (a->sal > b->sal) return 1;
    return (a->col > b->col) - (a->col < b->col);
}

/* Fig. 3 / Sec. 3.2 with Eq. 4: per-group saliency of one row -- the sum over the
 * group's G weights of (w / d_k)^2, d = diag(H^-1) of the layer (NULL: d = 1, the
 * sum of squares), accumulated in float64 in index order.                     */
static void row_saliency(const float* wrow, const float* hinv_diag, int64_t kg, int G, sal_entry* out)
{
    for (int64_t c = 0; c < kg; ++c) {
        double acc = 0.0;
        for (int j = 0; j < G; ++j) {
            double w = (double)wrow[c * G + j];
            if (hinv_diag) w = w / (double)hinv_diag[c * G + j];
            acc += w * w;
        }
        out[c].sal = acc;
        out[c].col = (int32_t)c;
    }
}

/* ---------------------------------------------------------------- quantiser */

/* Eq. 1 + Eq. 2 for one kept group.  Writes G codes (one per byte, unpacked),
 * and the fp16 bit patterns of scale and zero.  Returns 0 (and writes nothing)
 * if the scale of Eq. 1 is beyond the fp16 range the parameters are stored in. */
static int quantise_group(const float* w, int G, int bits,
                           uint8_t* codes, uint16_t* scale_h, uint16_t* zero_h)
{
    const float qmax = (float)((1 << bits) - 1);
    float mn = w[0], mx = w[0];
    for (int j = 1; j < G; ++j) {
        if (w[j] < mn) mn = w[j];
        if (w[j] > mx) mx = w[j];
    }
    volatile float range = mx - mn;             /* volatile: one fp32 op each */
    volatile float s32 = range / qmax;
    uint16_t sh = gqsa_oracle_f32_to_f16(s32);
    if ((sh & 0x7FFFu) >= 0x7C00u) return 0;    /* Eq. 1's scale does not fit fp16: Eq. 3 could not undo it */
    float sf = gqsa_oracle_f16_to_f32(sh);
    const float floor_scale = 6.103515625e-05f; /* 2^-14, smallest normal fp16 */
    if (!(sf >= floor_scale)) {
        sf = floor_scale;
        sh = 0x0400u;
    }
    volatile float ratio = -mn / sf;
    float z = nearbyintf(ratio);
    if (z > 2048.0f) z = 2048.0f;
    if (z < -2048.0f) z = -2048.0f;
    *scale_h = sh;
    *zero_h = gqsa_oracle_f32_to_f16(z);
    for (int j = 0; j < G; ++j) {
        volatile float t = w[j] / sf;
        float q = nearbyintf(t) + z;
        if (q < 0.0f) q = 0.0f;
        if (q > qmax) q = qmax;
        codes[j] = (uint8_t)q;
    }
    return 1;
}

/* ---------------------------------------------------------------- pack      */

/* Total stored groups for given per-row keep counts (caller sizes the arrays). */
int64_t gqsa_oracle_count(const int32_t* keep_per_row, int64_t N)
{
    int64_t t = 0;
    for (int64_t n = 0; n < N; ++n) t += keep_per_row[n];
    return t;
}

/*
 * Dense fp32 W[N,K] (row-major) -> canonical BSR arrays (Sec. 3.2 listing):
 *   rowIndex int32[N+1], groups int32[nnzg], values uint8[nnzg*G*bits/8],
 *   scales/zeros uint16[nnzg] (fp16 bit patterns).
 * keep_per_row[n] = number of groups row n keeps (the most salient ones).
 * hinv_diag: K positive finite numbers, diag(H^-1) of Eq. 4, or NULL.
 * Returns 0, or a negative number for an argument the definition excludes.
 */
int gqsa_oracle_pack(const float* W, int64_t N, int64_t K, int G, int bits,
                     const int32_t* keep_per_row, const float* hinv_diag,
                     int32_t* rowIndex, int32_t* groups, uint8_t* values,
                     uint16_t* scales, uint16_t* zeros)
{
    if (!W || !keep_per_row || !rowIndex) return -1;
    if (N <= 0 || K <= 0 || G <= 0 || K % G != 0) return -2;
    if (bits != 4 && bits != 8) return -3;
    if (bits == 4 && (G % 2) != 0) return -3;
    const int64_t kg = K / G;
    if (hinv_diag)
        for (int64_t k = 0; k < K; ++k)
            if (!(hinv_diag[k] > 0.0f) || !isfinite(hinv_diag[k])) return -6;
    sal_entry* ent = (sal_entry*)malloc(sizeof(sal_entry) * (size_t)kg);
    uint8_t* keepmask = (uint8_t*)malloc((size_t)kg);
    uint8_t* codes = (uint8_t*)malloc((size_t)G);
    if (!ent || !keepmask || !codes) { free(ent); free(keepmask); free(codes); return -4; }

    int64_t g = 0;
    rowIndex[0] = 0;
    for (int64_t n = 0; n < N; ++n) {
        const float* wrow = W + n * K;
        int64_t keep = keep_per_row[n];
        if (keep < 0 || keep > kg) { free(ent); free(keepmask); free(codes); return -5; }
        row_saliency(wrow, hinv_diag, kg, G, ent);
        qsort(ent, (size_t)kg, sizeof(sal_entry), sal_cmp);
        /* the first kg-keep entries (least salient) are pruned */
        memset(keepmask, 0, (size_t)kg);
        for (int64_t i = kg - keep; i < kg; ++i) keepmask[ent[i].col] = 1;
        for (int64_t c = 0; c < kg; ++c) {
            if (!keepmask[c]) continue;
            if (!quantise_group(wrow + c * G, G, bits, codes, &scales[g], &zeros[g])) {
                free(ent); free(keepmask); free(codes);
                return -7;
            }
            groups[g] = (int32_t)c;
            if (bits == 8) {
                memcpy(values + g * G, codes, (size_t)G);
            } else {
                for (int j = 0; j < G; j += 2)
                    values[(g * G + j) / 2] = (uint8_t)(codes[j] | (codes[j + 1] << 4));
            }
            ++g;
        }
        rowIndex[n + 1] = (int32_t)g;
    }
    free(ent); free(keepmask); free(codes);
    return 0;
}

/* code of element j of stored group g */
static inline unsigned code_at(const uint8_t* values, int64_t g, int G, int bits, int j)
{
    if (bits == 8) return values[g * G + j];
    uint8_t b = values[(g * G + j) / 2];
    return (j & 1) ? (unsigned)(b >> 4) : (unsigned)(b & 0xFu);
}

/* ---------------------------------------------------------------- densify   */

/* Eq. 3 on every stored group; pruned groups are zero.  Wd is float64 [N,K]. */
int gqsa_oracle_densify(const int32_t* rowIndex, const int32_t* groups,
                        const uint8_t* values, const uint16_t* scales,
                        const uint16_t* zeros, int64_t N, int64_t K, int G, int bits,
                        double* Wd)
{
    if (K % G != 0) return -2;
    memset(Wd, 0, sizeof(double) * (size_t)(N * K));
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = rowIndex[n]; g < rowIndex[n + 1]; ++g) {
            double s = (double)gqsa_oracle_f16_to_f32(scales[g]);
            double z = (double)gqsa_oracle_f16_to_f32(zeros[g]);
            int64_t c = groups[g];
            for (int j = 0; j < G; ++j) {
                double q = (double)code_at(values, g, G, bits, j);
                Wd[n * K + c * G + j] = (q - z) * s;
            }
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- GEMV      */

/*
 * Sec. 3.5 GEMV in its plain definition:
 *   y[b,n] = sum over stored groups g of row n, over j<G, of
 *            (q[g,j] - z[g]) * s[g] * x[b, groups[g]*G + j]        (float64)
 * x is fp16 bit patterns [batch,K]; y is float64 [batch,N].  Rows with no
 * stored group give exactly +0.  Rows are independent, so the loop over rows
 * may run on several threads (the sum inside a row stays in index order).
 */
int gqsa_oracle_gemv(const int32_t* rowIndex, const int32_t* groups,
                     const uint8_t* values, const uint16_t* scales,
                     const uint16_t* zeros, int64_t N, int64_t K, int G, int bits,
                     const uint16_t* x_f16, int batch, double* y, int threads)
{
    if (K % G != 0) return -2;
    double* xd = (double*)malloc(sizeof(double) * (size_t)(batch * K));
    if (!xd) return -4;
    for (int64_t i = 0; i < (int64_t)batch * K; ++i)
        xd[i] = (double)gqsa_oracle_f16_to_f32(x_f16[i]);
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    for (int b = 0; b < batch; ++b) {
        const double* xb = xd + (int64_t)b * K;
#pragma omp parallel for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t g = rowIndex[n]; g < rowIndex[n + 1]; ++g) {
                double s = (double)gqsa_oracle_f16_to_f32(scales[g]);
                double z = (double)gqsa_oracle_f16_to_f32(zeros[g]);
                const double* xg = xb + (int64_t)groups[g] * G;
                for (int j = 0; j < G; ++j) {
                    double q = (double)code_at(values, g, G, bits, j);
                    acc += (q - z) * s * xg[j];
                }
            }
            y[(int64_t)b * N + n] = acc;
        }
    }
    free(xd);
    return 0;
}

int gqsa_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
