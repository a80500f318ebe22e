/*
 * nm_oracle.c -- plain CPU oracle for the N:M-sparse low-bit integer path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the path computes.  It shares no code with the HIP library, is never
 * linked into it, and is called only from the tests, the smoke check and the
 * benchmark's CPU-baseline leg.
 *
 * Convention used everywhere: N = kept entries per group, M = group width
 * (the paper writes the same pattern as "M:N", e.g. its "4:2" is 2:4 here).
 * W is [rows = output neurons][cols = input features], row-major, and groups
 * run along the input (reduction) dimension.
 *
 * What each function follows:
 *   nmo_project        Sec. 3.2, Eq. 3: Euclidean projection onto the N:M set,
 *                      i.e. keep the N largest-magnitude entries of each group.
 *   nmo_row_scale      Sec. 3.3.1 "minimize error on the largest parameter":
 *                      scale = largest magnitude / largest integer code.
 *   nmo_quantize_one   Sec. 3.3, Eq. 5 with offset o = 0 (symmetric).
 *   nmo_compress       Sec. 3.3.1 last paragraph: the two constraints solved in
 *                      sequence, sparsity first; Sec. 4: constraining a trained
 *                      matrix directly (no fine-tuning).
 *   nmo_compress_grouped  the same with one scale per group of rows (Sec. 3.3
 *                      "group-wise quantization", Sec. 4: 32 neurons per scale).
 *   nmo_gemm_sparse    Sec. 5.3: only the kept products are computed, low-bit
 *                      weights widened to the activation type, int32 sums.
 *   nmo_dequant        Sec. 3.3, Eq. 4 with o = 0: x_d = s * x_q.
 *   nmo_admm_project   Sec. 3.1, the Z-update Z = Pi(W + U) (Eq. 3 on W + U), with
 *                      the quantisation constraint solved after the sparsity one
 *                      (Sec. 3.3.1, ADMM-Max: scale = largest magnitude of W + U in
 *                      the scale group / largest code; "group" = a run of output
 *                      neurons, Sec. 4: 32 by default) and the scaled dual update
 *                      U <- U + W - Z of the ADMM decomposition.
 *   nmo_dist_scales    Sec. 3.3.1, the second scale rule ("ADMM-Dist"): the scale that
 *                      minimises the L2 distance between the quantised and the raw
 *                      parameters, searched over a grid of candidates (the paper gives
 *                      no algorithm: the grid is this build's reading, PARITY UNPINNED
 *                      by the paper beyond "the chosen scale has the least error").
 *   nmo_requant        Sec. 5.3 (activations are 8-bit integers) with the scalar
 *                      quantiser of Sec. 3.3, Eq. 5 (o = 0) applied to a layer's
 *                      output, so that the next layer reads int8 again.
 *   nmo_quantize_act   the same quantiser on a floating-point activation tensor (the
 *                      input of the first compressed layer): one scale for the whole
 *                      tensor by the largest-magnitude rule of Sec. 3.3.1, 8 bits.
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - "largest" means largest magnitude; equal magnitudes keep the lower column.
 *   - one scale per output row; an all-zero row gets scale 1.
 *   - fp32 arithmetic for the scale and the quotient: two true IEEE divisions
 *     (amax / qmax, then w / s), round-half-to-even, clamp to [-qmax, +qmax],
 *     qmax = 2^(b-1) - 1.
 *   - packed format: see nmo_packed_sizes.
 *   - the dequantized value is formed in double and rounded once.
 *   - requantised output: the paper does not say where the activation scale
 *     comes from; here the caller supplies it.  The value quantised is the
 *     dequantised output of Eq. 4 exactly as nmo_dequant forms it (double,
 *     rounded once to float), and the quantiser is Eq. 5 as for the weights:
 *     one fp32 division per output, round half to even, clamp to +-127.
 *   - dense matrices (N = M, the "Q4" / "Q8" components of Sec. 5.4): every
 *     entry is kept, no index metadata is stored.
 *   - tiled layout: a byte permutation of the packed rows, see nmo_to_tiled.
 *
 * Build: gcc -O2 -std=c11 -fno-fast-math -ffp-contract=off -fopenmp -shared -fPIC
 *
 * Pins (tests/test_oracle_*.py): brute-force Euclidean projection over all
 * supports, N=1 == argmax, idempotence, max-survives-pruning invariant,
 * quantiser closed forms and half-way cases, an independent numpy decoder of
 * the byte format, numpy int64 matmul on the decompressed matrix, dequant
 * special cases; requantisation against exact rational arithmetic, half-way
 * and saturation cases, and the weight quantiser applied to the dequantised
 * value; the tiled layout against a numpy transposition of the row layout and
 * a hand-placed case.  The tie-break rule and the byte format are this build's own
 * choices (the paper fixes neither): pinned by the written format description
 * and the independent decoder, not by the paper.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum {
    NMO_OK = 0,
    NMO_ERR_NULL = -1,
    NMO_ERR_DIM = -2,
    NMO_ERR_PATTERN = -3,
    NMO_ERR_BITS = -4,
    NMO_ERR_NONFINITE = -5
};

/* Bits of index metadata per kept entry: none for a dense matrix (N = M). */
static int index_bits(int N, int M) { return N >= M ? 0 : (M == 4 ? 2 : 4); }

static int check_pattern(int rows, int cols, int N, int M, int bits)
{
    if (rows <= 0 || cols <= 0) return NMO_ERR_DIM;
    if (M != 4 && M != 8) return NMO_ERR_PATTERN;
    if (N < 1 || N > M) return NMO_ERR_PATTERN;
    if (cols % M != 0) return NMO_ERR_PATTERN;
    if (bits != 4 && bits != 8) return NMO_ERR_BITS;
    return NMO_OK;
}

/*
 * Packed format (the paper does not discuss one; this is the library's own).
 * kc = cols * N / M kept entries per row, numbered e = g*N + j in ascending
 * column order (g = group, j = rank of the kept column inside the group).
 *   values : row-major, row stride ceil(kc*bits/8) bytes.
 *            bits = 8: entry e is byte e (two's complement).
 *            bits = 4: entry e is a two's-complement nibble of byte e/2,
 *                      low nibble when e is even, high nibble when e is odd.
 *   meta   : row-major, row stride ceil(kc*ib/8) bytes, ib = 2 (M=4) or 4 (M=8).
 *            Entry e's column offset inside its group sits in ib bits starting
 *            at bit e*ib of the row, counted LSB-first through the bytes.
 *   scales : one float per row.
 * Unused trailing bits of a row are zero.  A dense matrix (N = M) keeps every
 * entry, so entry e is column e and there is no metadata (meta_bytes = 0).
 */
int nmo_packed_sizes(int rows, int cols, int N, int M, int bits,
                     size_t *vals_bytes, size_t *meta_bytes, size_t *scales_bytes)
{
    int rc = check_pattern(rows, cols, N, M, bits);
    if (rc) return rc;
    size_t kc = (size_t)cols / M * N;
    if (vals_bytes) *vals_bytes = (size_t)rows * ((kc * bits + 7) / 8);
    if (meta_bytes) *meta_bytes = (size_t)rows * ((kc * index_bits(N, M) + 7) / 8);
    if (scales_bytes) *scales_bytes = (size_t)rows * sizeof(float);
    return NMO_OK;
}

/*
 * Eq. 3 for one group: choose the N of M entries that the projection keeps.
 * Entries are ranked by magnitude, larger first; among equal magnitudes the
 * lower column ranks first.  The N best are returned in ascending column order.
 */
static void project_group(const float *w, int N, int M, uint8_t *kept)
{
    int taken[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int pick = 0; pick < N; ++pick) {
        int best = -1;
        for (int c = 0; c < M; ++c) {
            if (taken[c]) continue;
            if (best < 0 || fabsf(w[c]) > fabsf(w[best])) best = c; /* strict: ties stay low */
        }
        taken[best] = 1;
    }
    int j = 0;
    for (int c = 0; c < M; ++c)
        if (taken[c]) kept[j++] = (uint8_t)c;
}

/* Eq. 3 over a matrix: kept[r][g*N + j] = column offset (0..M-1) inside group g. */
int nmo_project(const float *W, int rows, int cols, int ldw, int N, int M, uint8_t *kept)
{
    int rc = check_pattern(rows, cols, N, M, 8);
    if (rc) return rc;
    if (!W || !kept) return NMO_ERR_NULL;
    if (ldw < cols) return NMO_ERR_DIM;
    int groups = cols / M;
    for (int r = 0; r < rows; ++r)
        for (int g = 0; g < groups; ++g) {
            const float *w = W + (size_t)r * ldw + (size_t)g * M;
            for (int c = 0; c < M; ++c)
                if (!isfinite(w[c])) return NMO_ERR_NONFINITE;
            project_group(w, N, M, kept + ((size_t)r * groups + g) * N);
        }
    return NMO_OK;
}

/* Sec. 3.3.1: scale = max |w| over the row / largest code.  All-zero row -> 1. */
float nmo_row_scale(const float *w, int cols, int bits)
{
    float amax = 0.0f;
    for (int c = 0; c < cols; ++c) {
        float a = fabsf(w[c]);
        if (a > amax) amax = a;
    }
    float qmax = (float)((1 << (bits - 1)) - 1);
    volatile float s = amax / qmax; /* one fp32 division, kept in fp32 */
    return amax == 0.0f ? 1.0f : s;
}

/* Eq. 5 with o = 0: divide by the scale, round half to even, clamp. */
int nmo_quantize_one(float w, float s, int bits)
{
    int qmax = (1 << (bits - 1)) - 1;
    volatile float t = w / s;      /* one fp32 division */
    float r = nearbyintf(t);       /* default rounding mode: nearest, ties to even */
    if (r > (float)qmax) r = (float)qmax;
    if (r < (float)-qmax) r = (float)-qmax;
    return (int)r;
}

static int nmo_compress_given(const float *W, int rows, int cols, int ldw, int N, int M, int bits,
                              uint8_t *vals, uint8_t *meta, const float *scales);

static void put_bits(uint8_t *row, size_t bit_offset, int nbits, unsigned value)
{
    for (int b = 0; b < nbits; ++b) {
        size_t pos = bit_offset + (size_t)b;
        if ((value >> b) & 1u) row[pos >> 3] |= (uint8_t)(1u << (pos & 7));
    }
}

static unsigned get_bits(const uint8_t *row, size_t bit_offset, int nbits)
{
    unsigned v = 0;
    for (int b = 0; b < nbits; ++b) {
        size_t pos = bit_offset + (size_t)b;
        v |= (unsigned)((row[pos >> 3] >> (pos & 7)) & 1u) << b;
    }
    return v;
}

/* Column offset inside its group of kept entry e of a packed row (dense: nothing stored, entry j is column j). */
static unsigned kept_offset(const uint8_t *mrow, size_t e, int N, int M)
{
    int ib = index_bits(N, M);
    return ib ? get_bits(mrow, e * ib, ib) : (unsigned)(e % (size_t)N);
}

/*
 * project (Eq. 3), then scale and quantise the kept entries (Eq. 5), then pack.
 * One scale per group of rows_per_scale consecutive rows (Sec. 4: the paper's
 * default is 32 output neurons per scale; the last group may be shorter): the
 * largest magnitude over the group's rows / the largest code, 1 for an all-zero
 * group.  scales[] receives every row's scale.
 */
int nmo_compress_grouped(const float *W, int rows, int cols, int ldw, int N, int M, int bits,
                         int rows_per_scale, uint8_t *vals, uint8_t *meta, float *scales)
{
    int rc = check_pattern(rows, cols, N, M, bits);
    if (rc) return rc;
    if (!W || !vals || (!meta && N < M) || !scales) return NMO_ERR_NULL;
    if (ldw < cols || rows_per_scale < 1) return NMO_ERR_DIM;
    for (int r0 = 0; r0 < rows; r0 += rows_per_scale) {
        int r1 = r0 + rows_per_scale < rows ? r0 + rows_per_scale : rows;
        float s = 0.0f;                      /* the largest of the rows' own scales is the group's: */
        int all_zero = 1;                    /* amax / qmax is monotonic in amax                     */
        for (int r = r0; r < r1; ++r) {
            float sr = nmo_row_scale(W + (size_t)r * ldw, cols, bits);
            int zero_row = 1;
            for (int c = 0; c < cols; ++c)
                if (W[(size_t)r * ldw + c] != 0.0f) zero_row = 0;
            if (!zero_row) {
                all_zero = 0;
                if (sr > s) s = sr;
            }
        }
        for (int r = r0; r < r1; ++r) scales[r] = all_zero ? 1.0f : s;
    }
    return nmo_compress_given(W, rows, cols, ldw, N, M, bits, vals, meta, scales);
}

/* project, quantise and pack with scales the caller supplies, one per row (e.g. those of nmo_dist_scales). */
int nmo_compress_scaled(const float *W, int rows, int cols, int ldw, int N, int M, int bits,
                        const float *scales, uint8_t *vals, uint8_t *meta)
{
    return nmo_compress_given(W, rows, cols, ldw, N, M, bits, vals, meta, scales);
}

/*
 * Sec. 3.3.1, second rule: per scale group (rows_per_scale consecutive rows, the
 * last group may be shorter) the scale that minimises the squared L2 distance
 * between the parameters and their quantised-then-dequantised values.  The paper
 * states the criterion and no algorithm; the reading used here:
 *   - the distance is taken over the entries the N:M projection keeps (the pruned
 *     ones are zero whatever the scale);
 *   - candidates are s_c = (s_max * c) / C for c = C/2 .. C, with C = `candidates`
 *     (even, 2 .. 64) and s_max the max-rule scale of the group (largest magnitude /
 *     largest code, 1 for an all-zero group): the max rule itself (c = C) down to
 *     half of it, which clips the largest entries in exchange for finer steps;
 *     two fp32 operations per candidate, a multiplication and then a division;
 *   - per entry: q = Eq. 5 with s_c (fp32 division, round half to even, clamp),
 *     e = w - s_c * q and e * e in double; the group's error is their plain sum in
 *     double, rows in order, columns in order;
 *   - the least error wins; between equal errors the larger scale.
 * scales[] receives every row's scale; errors, when given, the group errors as
 * [group][C/2 + 1] (index c - C/2).
 */
int nmo_dist_scales(const float *W, int rows, int cols, int ldw, int N, int M, int bits,
                    int rows_per_scale, int candidates, float *scales, double *errors)
{
    int rc = check_pattern(rows, cols, N, M, bits);
    if (rc) return rc;
    if (!W || !scales) return NMO_ERR_NULL;
    if (ldw < cols || rows_per_scale < 1 || candidates < 2 || candidates > 64 || candidates % 2) return NMO_ERR_DIM;
    int groups = cols / M, nc = candidates / 2 + 1;
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < cols; ++c)
            if (!isfinite(W[(size_t)r * ldw + c])) return NMO_ERR_NONFINITE;
    for (int r0 = 0, gi = 0; r0 < rows; r0 += rows_per_scale, ++gi) {
        int r1 = r0 + rows_per_scale < rows ? r0 + rows_per_scale : rows;
        float amax = 0.0f;
        for (int r = r0; r < r1; ++r)
            for (int c = 0; c < cols; ++c)
                if (fabsf(W[(size_t)r * ldw + c]) > amax) amax = fabsf(W[(size_t)r * ldw + c]);
        float qmax = (float)((1 << (bits - 1)) - 1);
        volatile float smax_v = amax / qmax;
        float smax = amax == 0.0f ? 1.0f : smax_v;
        double best_err = 0.0;
        float best_s = smax;
        for (int c = candidates; c >= candidates / 2; --c) {      /* from the largest scale down: a tie keeps the larger */
            volatile float num = smax * (float)c;
            volatile float sc = num / (float)candidates;
            double err = 0.0;
            for (int r = r0; r < r1; ++r)
                for (int g = 0; g < groups; ++g) {
                    const float *w = W + (size_t)r * ldw + (size_t)g * M;
                    uint8_t kept[8];
                    project_group(w, N, M, kept);
                    for (int j = 0; j < N; ++j) {
                        float x = w[kept[j]];
                        double e = (double)x - (double)sc * (double)nmo_quantize_one(x, sc, bits);
                        err += e * e;
                    }
                }
            if (errors) errors[(size_t)gi * nc + (c - candidates / 2)] = err;
            if (c == candidates || err < best_err) {
                best_err = err;
                best_s = sc;
            }
        }
        for (int r = r0; r < r1; ++r) scales[r] = best_s;
    }
    return NMO_OK;
}

/* The same with one scale per row (the library's default granularity). */
int nmo_compress(const float *W, int rows, int cols, int ldw, int N, int M, int bits,
                 uint8_t *vals, uint8_t *meta, float *scales)
{
    return nmo_compress_grouped(W, rows, cols, ldw, N, M, bits, 1, vals, meta, scales);
}

/* Projection, quantisation with the scales given per row, packing. */
static int nmo_compress_given(const float *W, int rows, int cols, int ldw, int N, int M, int bits,
                              uint8_t *vals, uint8_t *meta, const float *scales)
{
    int rc = check_pattern(rows, cols, N, M, bits);
    if (rc) return rc;
    if (!W || !vals || (!meta && N < M) || !scales) return NMO_ERR_NULL;
    if (ldw < cols) return NMO_ERR_DIM;
    int groups = cols / M;
    int ib = index_bits(N, M);
    size_t kc = (size_t)groups * N;
    size_t vstride = (kc * bits + 7) / 8;
    size_t mstride = (kc * ib + 7) / 8;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const float *w = W + (size_t)r * ldw;
        uint8_t *vrow = vals + (size_t)r * vstride;
        uint8_t *mrow = ib ? meta + (size_t)r * mstride : NULL;
        int finite = 1;
        for (int c = 0; c < cols; ++c)
            if (!isfinite(w[c])) finite = 0;
        if (!finite) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        memset(vrow, 0, vstride);
        if (ib) memset(mrow, 0, mstride);
        float s = scales[r];
        for (int g = 0; g < groups; ++g) {
            uint8_t kept[8];
            project_group(w + (size_t)g * M, N, M, kept);
            for (int j = 0; j < N; ++j) {
                size_t e = (size_t)g * N + j;
                int q = nmo_quantize_one(w[(size_t)g * M + kept[j]], s, bits);
                put_bits(vrow, e * bits, bits, (unsigned)q & ((1u << bits) - 1u));
                if (ib) put_bits(mrow, e * ib, ib, kept[j]);
            }
        }
    }
    return bad ? NMO_ERR_NONFINITE : NMO_OK;
}

static int sign_extend(unsigned v, int bits)
{
    int sh = 32 - bits;
    return (int)((int32_t)(v << sh) >> sh);
}

/* Packed -> dense integer matrix Wq[rows][cols] (zeros where nothing was kept). */
int nmo_decompress(const uint8_t *vals, const uint8_t *meta, int rows, int cols,
                   int N, int M, int bits, int8_t *Wq)
{
    int rc = check_pattern(rows, cols, N, M, bits);
    if (rc) return rc;
    if (!vals || (!meta && N < M) || !Wq) return NMO_ERR_NULL;
    int groups = cols / M;
    int ib = index_bits(N, M);
    size_t kc = (size_t)groups * N;
    size_t vstride = (kc * bits + 7) / 8;
    size_t mstride = (kc * ib + 7) / 8;
    memset(Wq, 0, (size_t)rows * cols);
    for (int r = 0; r < rows; ++r)
        for (size_t e = 0; e < kc; ++e) {
            int q = sign_extend(get_bits(vals + (size_t)r * vstride, e * bits, bits), bits);
            unsigned off = kept_offset(ib ? meta + (size_t)r * mstride : NULL, e, N, M);
            size_t col = (e / N) * M + off;
            Wq[(size_t)r * cols + col] = (int8_t)q;
        }
    return NMO_OK;
}

/*
 * Sec. 5.3: acc[t][o] = sum over kept entries e of X[t][col(o,e)] * q[o][e],
 * walking the metadata; nothing is computed for pruned positions.
 */
int nmo_gemm_sparse(const int8_t *X, int tokens, int K, int ldx,
                    const uint8_t *vals, const uint8_t *meta,
                    int O, int N, int M, int bits, int32_t *acc, int ldacc)
{
    int rc = check_pattern(O, K, N, M, bits);
    if (rc) return rc;
    if (!X || !vals || (!meta && N < M) || !acc) return NMO_ERR_NULL;
    if (tokens <= 0 || ldx < K || ldacc < O) return NMO_ERR_DIM;
    int ib = index_bits(N, M);
    size_t kc = (size_t)K / M * N;
    size_t vstride = (kc * bits + 7) / 8;
    size_t mstride = (kc * ib + 7) / 8;
#pragma omp parallel for schedule(static)
    for (int o = 0; o < O; ++o) {
        const uint8_t *vrow = vals + (size_t)o * vstride;
        const uint8_t *mrow = ib ? meta + (size_t)o * mstride : NULL;
        for (int t = 0; t < tokens; ++t) {
            const int8_t *x = X + (size_t)t * ldx;
            int32_t sum = 0;
            for (size_t e = 0; e < kc; ++e) {
                int q = sign_extend(get_bits(vrow, e * bits, bits), bits);
                size_t col = (e / N) * M + kept_offset(mrow, e, N, M);
                sum += (int32_t)x[col] * (int32_t)q;
            }
            acc[(size_t)t * ldacc + o] = sum;
        }
    }
    return NMO_OK;
}

/* The plain definition the sparse product must equal: acc = X * Wq^T, all K terms. */
int nmo_gemm_dense(const int8_t *X, int tokens, int K, int ldx,
                   const int8_t *Wq, int O, int32_t *acc, int ldacc)
{
    if (!X || !Wq || !acc) return NMO_ERR_NULL;
    if (tokens <= 0 || K <= 0 || O <= 0 || ldx < K || ldacc < O) return NMO_ERR_DIM;
#pragma omp parallel for schedule(static)
    for (int o = 0; o < O; ++o)
        for (int t = 0; t < tokens; ++t) {
            int32_t sum = 0;
            for (int k = 0; k < K; ++k)
                sum += (int32_t)X[(size_t)t * ldx + k] * (int32_t)Wq[(size_t)o * K + k];
            acc[(size_t)t * ldacc + o] = sum;
        }
    return NMO_OK;
}

/* float -> bfloat16 bits, round to nearest, ties to even (finite inputs). */
static uint16_t bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/*
 * Eq. 4 with o = 0 applied to the product of two quantised operands:
 * y = acc * s_act * s_w[o] (+ bias[o]), formed in double, rounded once to
 * float; the bfloat16 result is that float rounded to nearest-even.
 * bias, out_f32 and out_bf16 may each be NULL.
 */
int nmo_dequant(const int32_t *acc, int tokens, int O, int ldacc, float act_scale,
                const float *scales, const float *bias,
                float *out_f32, uint16_t *out_bf16, int ldo)
{
    if (!acc || !scales) return NMO_ERR_NULL;
    if (tokens <= 0 || O <= 0 || ldacc < O || ldo < O) return NMO_ERR_DIM;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < tokens; ++t)
        for (int o = 0; o < O; ++o) {
            double y = (double)acc[(size_t)t * ldacc + o] * (double)act_scale * (double)scales[o];
            if (bias) y += (double)bias[o];
            float yf = (float)y;
            if (out_f32) out_f32[(size_t)t * ldo + o] = yf;
            if (out_bf16) out_bf16[(size_t)t * ldo + o] = bf16_rne(yf);
        }
    return NMO_OK;
}

/*
 * A floating-point activation tensor as 8-bit integers (Sec. 5.3: the layers take
 * 8-bit activations; the paper says no more): one scale for the whole tensor,
 * s = max|x| / 127 (Sec. 3.3.1's largest-magnitude rule; 1 for an all-zero tensor),
 * or the caller's when scale_in > 0, then Eq. 5 (o = 0) per element exactly as
 * for the weights.  *scale_out receives the scale used.
 */
int nmo_quantize_act(const float *X, int tokens, int K, int ldx, float scale_in,
                     int8_t *Q, int ldq, float *scale_out)
{
    if (!X || !Q) return NMO_ERR_NULL;
    if (tokens <= 0 || K <= 0 || ldx < K || ldq < K) return NMO_ERR_DIM;
    float amax = 0.0f;
    for (int t = 0; t < tokens; ++t)
        for (int k = 0; k < K; ++k) {
            float x = X[(size_t)t * ldx + k];
            if (!isfinite(x)) return NMO_ERR_NONFINITE;
            if (fabsf(x) > amax) amax = fabsf(x);
        }
    volatile float smax = amax / 127.0f;   /* one fp32 division */
    float s = scale_in > 0.0f ? scale_in : (amax == 0.0f ? 1.0f : smax);
    for (int t = 0; t < tokens; ++t)
        for (int k = 0; k < K; ++k)
            Q[(size_t)t * ldq + k] = (int8_t)nmo_quantize_one(X[(size_t)t * ldx + k], s, 8);
    if (scale_out) *scale_out = s;
    return NMO_OK;
}

/*
 * Layer output as 8-bit activations for the next layer (Sec. 5.3): the
 * dequantised value of Eq. 4 (o = 0), formed as in nmo_dequant (double, rounded
 * once to float), then the quantiser of Eq. 5 (o = 0, 8 bits) with the caller's
 * scale, exactly as it is applied to the weights: one fp32 division, round half
 * to even, clamp to [-127, 127].  absmax, when given, receives max |y| over all
 * outputs, the statistic from which a caller chooses the next out_scale.
 */
int nmo_requant(const int32_t *acc, int tokens, int O, int ldacc, float act_scale,
                const float *scales, const float *bias, float out_scale,
                int8_t *out, int ldo, float *absmax)
{
    if (!acc || !scales || !out) return NMO_ERR_NULL;
    if (tokens <= 0 || O <= 0 || ldacc < O || ldo < O) return NMO_ERR_DIM;
    if (!(out_scale > 0.0f) || !isfinite(out_scale)) return NMO_ERR_NONFINITE;
    float ymax = 0.0f;
    for (int t = 0; t < tokens; ++t)
        for (int o = 0; o < O; ++o) {
            double y = (double)acc[(size_t)t * ldacc + o] * (double)act_scale * (double)scales[o];
            if (bias) y += (double)bias[o];
            float yf = (float)y;
            if (fabsf(yf) > ymax) ymax = fabsf(yf);
            out[(size_t)t * ldo + o] = (int8_t)nmo_quantize_one(yf, out_scale, 8);
        }
    if (absmax) *absmax = ymax;
    return NMO_OK;
}

/*
 * Tiled layout of the packed values and of the index metadata: a permutation of
 * the bytes of the row layout above, chosen so that what one matrix-core
 * fragment consumes (16 rows x 128 input columns) is one contiguous run of
 * memory.  Defined for cols % 128 == 0.
 *   unit    = the packed bytes of one row that cover 32 consecutive input
 *             columns: unit u of row r is bytes [u*UB, (u+1)*UB) of row r in the
 *             row layout, UB = (32/M)*N*bits/8 for values and (32/M)*N*ib/8
 *             for metadata.
 *   block   = the 64 units of 16 consecutive rows (row block rb = r / 16) and
 *             one 128-column slice (s = u / 4); block (rb, s) starts at byte
 *             (rb * (cols/128) + s) * 64 * UB.  Rows are padded with zero bytes
 *             up to a multiple of 16.
 *   in a block, unit number j = (u % 4) * 16 + (r % 16); a unit is cut into
 *             pieces of PB bytes, PB the largest power of two <= 16 dividing UB,
 *             and piece p of unit j lies at byte (p * 64 + j) * PB of the block.
 * nmo_to_tiled converts one array (values or metadata, told apart only by UB);
 * nmo_from_tiled is its inverse.
 */
static size_t tiled_piece_bytes(size_t ub)
{
    size_t pb = 16;
    while (ub % pb) pb >>= 1;
    return pb;
}

static size_t tiled_offset(size_t r, size_t byte_in_row, size_t ub, size_t slices)
{
    size_t u = byte_in_row / ub, i = byte_in_row % ub;
    size_t pb = tiled_piece_bytes(ub);
    size_t block = (r / 16) * slices + u / 4;
    size_t j = (u % 4) * 16 + r % 16;
    return block * 64 * ub + ((i / pb) * 64 + j) * pb + i % pb;
}

size_t nmo_tiled_bytes(int rows, int cols, size_t unit_bytes)
{
    return (size_t)((rows + 15) / 16) * 16 * (size_t)(cols / 32) * unit_bytes;
}

int nmo_to_tiled(const uint8_t *rowmajor, int rows, int cols, size_t unit_bytes, uint8_t *tiled)
{
    if (!rowmajor || !tiled) return NMO_ERR_NULL;
    if (rows <= 0 || cols <= 0 || unit_bytes == 0) return NMO_ERR_DIM;
    if (cols % 128 != 0) return NMO_ERR_PATTERN;
    size_t stride = (size_t)(cols / 32) * unit_bytes;
    memset(tiled, 0, nmo_tiled_bytes(rows, cols, unit_bytes));
    for (int r = 0; r < rows; ++r)
        for (size_t b = 0; b < stride; ++b)
            tiled[tiled_offset((size_t)r, b, unit_bytes, (size_t)cols / 128)] = rowmajor[(size_t)r * stride + b];
    return NMO_OK;
}

int nmo_from_tiled(const uint8_t *tiled, int rows, int cols, size_t unit_bytes, uint8_t *rowmajor)
{
    if (!rowmajor || !tiled) return NMO_ERR_NULL;
    if (rows <= 0 || cols <= 0 || unit_bytes == 0) return NMO_ERR_DIM;
    if (cols % 128 != 0) return NMO_ERR_PATTERN;
    size_t stride = (size_t)(cols / 32) * unit_bytes;
    for (int r = 0; r < rows; ++r)
        for (size_t b = 0; b < stride; ++b)
            rowmajor[(size_t)r * stride + b] = tiled[tiled_offset((size_t)r, b, unit_bytes, (size_t)cols / 128)];
    return NMO_OK;
}

/*
 * The ADMM Z-update and dual update on one weight matrix, in fp32, one operation
 * per step:
 *   V      = W + U                                (U == NULL: V = W)
 *   keep   = Eq. 3 on V (N largest magnitudes of every M, ties to the lower column)
 *   bits 0 : Z = V on kept positions, +0 elsewhere
 *   bits b : scale group = rows_per_scale consecutive rows (the last one may be
 *            shorter); s = (largest |V| in the group) / qmax, 1 for an all-zero
 *            group; q = Eq. 5 (o = 0) of V with s; Z = s * q on kept positions
 *            (one multiplication), +0 elsewhere
 *   U_out  = V - Z                                (when U_out is given)
 * scales, when given (bits > 0), receives the scale of every row (rows of one
 * group hold the same value).
 */
int nmo_admm_project(const float *W, const float *U, int rows, int cols, int ldw,
                     int N, int M, int bits, int rows_per_scale,
                     float *Z, float *U_out, int ldz, float *scales)
{
    int rc = check_pattern(rows, cols, N, M, bits ? bits : 8);
    if (rc) return rc;
    if (!W || !Z) return NMO_ERR_NULL;
    if (ldw < cols || ldz < cols || rows_per_scale < 1) return NMO_ERR_DIM;
    int groups = cols / M;
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < cols; ++c) {
            float w = W[(size_t)r * ldw + c], u = U ? U[(size_t)r * ldw + c] : 0.0f;
            if (!isfinite(w) || !isfinite(u)) return NMO_ERR_NONFINITE;
        }
    for (int r0 = 0; r0 < rows; r0 += rows_per_scale) {
        int r1 = r0 + rows_per_scale < rows ? r0 + rows_per_scale : rows;
        float s = 1.0f;
        if (bits) {
            float amax = 0.0f;
            for (int r = r0; r < r1; ++r)
                for (int c = 0; c < cols; ++c) {
                    volatile float v = U ? W[(size_t)r * ldw + c] + U[(size_t)r * ldw + c] : W[(size_t)r * ldw + c];
                    if (fabsf(v) > amax) amax = fabsf(v);
                }
            float qmax = (float)((1 << (bits - 1)) - 1);
            volatile float t = amax / qmax;
            s = amax == 0.0f ? 1.0f : t;
        }
        for (int r = r0; r < r1; ++r) {
            if (scales && bits) scales[r] = s;
            for (int g = 0; g < groups; ++g) {
                float v[8];
                uint8_t kept[8];
                for (int c = 0; c < M; ++c) {
                    size_t at = (size_t)r * ldw + (size_t)g * M + c;
                    volatile float sum = U ? W[at] + U[at] : W[at];
                    v[c] = sum;
                }
                project_group(v, N, M, kept);
                float z[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
                for (int j = 0; j < N; ++j) {
                    int c = kept[j];
                    if (bits) {
                        volatile float zq = s * (float)nmo_quantize_one(v[c], s, bits);
                        z[c] = zq;
                    } else {
                        z[c] = v[c];
                    }
                }
                for (int c = 0; c < M; ++c) {
                    size_t at = (size_t)r * ldz + (size_t)g * M + c;
                    Z[at] = z[c];
                    if (U_out) {
                        volatile float d = v[c] - z[c];
                        U_out[at] = d;
                    }
                }
            }
        }
    }
    return NMO_OK;
}
