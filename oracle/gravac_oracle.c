/*
 * CPU oracle for the per-worker gradient-compression path of GraVAC
 * (arxiv 2305.12201).  TEST INFRASTRUCTURE ONLY: this file is the plain, slow,
 * single-threaded definition that the GPU library is checked against.  Only the
 * tests, the smoke check and the bench's cpu_baseline leg may call it; the
 * product path never does.  It shares no code with the HIP library.
 *
 * What it computes, with the passage each step follows:
 *   1. error feedback   acc = residual + grad            (Sec. III-B, g_ef; Alg. 1 error-feedback line)
 *   2. Top-k at factor CF: keep the k = ceil(n/CF) entries of largest |acc|,
 *      everything else is dropped from the message       (Sec. II-C: CF definition, Top-k)
 *   3. residual = acc - compressed                       (Alg. 1 "update residual")
 *   4. compression gain ||g_c||^2 / ||g_ef||^2           (Sec. III-B, compression-gain equation;
 *                                                         Alg. 1 gain lines) for every candidate CF
 *   5. the same per tensor ("layerwise", Sec. III-A)     with global indices
 *   6. decompression: rebuild to the dense dimension     (Sec. III-A, t_decompress) and sum the
 *      workers' contributions; the same applied to the parameters as the step -eta * aggregate
 *      (Alg. 1, update of w)
 *
 * The selection is the plain definition: a full sort of all entries by
 * (|acc| descending, index ascending) and a cut after k entries.  No histogram,
 * no threshold search, no blocking.
 *
 * Readings taken where the paper is silent (each also listed in the design notes):
 *   - k = ceil(n / CF), clamped to [1, n]; integral CF uses exact integer arithmetic.
 *   - magnitude order is the order of the IEEE-754 bit pattern with the sign bit
 *     cleared, so +0 and -0 tie, and NaN patterns rank above infinity.
 *   - ties in magnitude go to the lower index.
 *   - the message lists pairs in ascending index order; values keep their sign bits.
 *   - a selected slot's residual is +0.0f (x - x under round-to-nearest).
 *   - the gain is the ratio of squared L2 norms (no mean subtracted), accumulated
 *     in double; if ||acc||^2 == 0 the gain is 1.
 *   - one CF of the list (position `commit`) is the one whose selection is emitted
 *     and removed from the residual; every CF gets its statistics.
 *   - the add of step 1 is one binary32 round-to-nearest-even add (gradients and
 *     residuals are single-precision tensors, Sec. IV-B), no flush to zero.
 *
 * Build: gcc -O2 -ffp-contract=off -fPIC -shared (no -ffast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)
#define ORACLE_CAPACITY (-2)
#define ORACLE_NOMEM (-3)

/* k = ceil(n / cf) clamped to [1, n]  (Sec. II-C: 10 % kept <-> CF 10x, 1 % <-> 100x). */
int64_t oracle_k(int64_t n, double cf)
{
    int64_t k;
    if (n <= 0 || !(cf >= 1.0) || isinf(cf)) return -1;
    if (cf == floor(cf) && cf < 9.0e18) {
        int64_t c = (int64_t)cf;
        k = n / c + (n % c != 0);
    } else {
        k = (int64_t)ceil((double)n / cf);
    }
    if (k < 1) k = 1;
    if (k > n) k = n;
    return k;
}

static uint32_t f32_bits(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    return u;
}

/* One entry of the full sort: magnitude bit pattern and position. */
typedef struct {
    uint32_t mag;
    uint32_t pos;
} entry_t;

/* larger magnitude first; equal magnitudes: lower position first */
static int cmp_entry(const void* a, const void* b)
{
    const entry_t* x = (const entry_t*)a;
    const entry_t* y = (const entry_t*)b;
    if (x->mag != y->mag) return x->mag > y->mag ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}

static int cmp_u32(const void* a, const void* b)
{
    uint32_t x = *(const uint32_t*)a, y = *(const uint32_t*)b;
    return (x > y) - (x < y);
}

/*
 * One tensor (a flat gradient, or one segment of it).  `base` is the offset of
 * this tensor in the flat buffer: emitted indices are base + local position.
 * acc is written into residual first (step 1), then selected slots are zeroed.
 */
static int compress_one(const float* grad, float* residual, int64_t base, int64_t n,
                        const double* cf_list, int n_cf, int commit,
                        int32_t* out_idx, float* out_val, int64_t* n_out, double* stats)
{
    entry_t* order = (entry_t*)malloc((size_t)n * sizeof(entry_t));
    if (!order) return ORACLE_NOMEM;

    /* step 1: acc = residual + grad, one binary32 add per element */
    double ss_dense = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        volatile float a = residual[base + i] + grad[base + i];
        residual[base + i] = a;
        ss_dense += (double)a * (double)a;
        order[i].mag = f32_bits(a) & 0x7FFFFFFFu;
        order[i].pos = (uint32_t)i;
    }

    /* step 2: the full sort that defines "largest by magnitude" */
    qsort(order, (size_t)n, sizeof(entry_t), cmp_entry);

    /* step 4: statistics for every candidate CF from its prefix of the order */
    for (int j = 0; j < n_cf; ++j) {
        int64_t k = oracle_k(n, cf_list[j]);
        double ss_sel = 0.0;
        for (int64_t r = 0; r < k; ++r) {
            double v = (double)residual[base + order[r].pos];
            ss_sel += v * v;
        }
        float last = residual[base + order[k - 1].pos];
        stats[4 * j + 0] = ss_sel;
        stats[4 * j + 1] = ss_dense;
        stats[4 * j + 2] = (ss_dense == 0.0) ? 1.0 : ss_sel / ss_dense;
        stats[4 * j + 3] = fabs((double)last);
    }

    /* steps 2-3 for the committed CF: message in ascending index order, residual update */
    int64_t kc = oracle_k(n, cf_list[commit]);
    uint32_t* chosen = (uint32_t*)malloc((size_t)kc * sizeof(uint32_t));
    if (!chosen) {
        free(order);
        return ORACLE_NOMEM;
    }
    for (int64_t r = 0; r < kc; ++r) chosen[r] = order[r].pos;
    qsort(chosen, (size_t)kc, sizeof(uint32_t), cmp_u32);
    for (int64_t r = 0; r < kc; ++r) {
        int64_t g = base + (int64_t)chosen[r];
        out_idx[r] = (int32_t)g;
        out_val[r] = residual[g]; /* still acc here */
    }
    for (int64_t r = 0; r < kc; ++r) residual[base + (int64_t)chosen[r]] = 0.0f;
    *n_out = kc;

    free(chosen);
    free(order);
    return ORACLE_OK;
}

/*
 * Host pointers throughout.  residual is updated in place.  seg_offsets == NULL
 * (n_seg 0) means one flat tensor; otherwise n_seg + 1 offsets, strictly
 * increasing from 0 to n, and each segment is compressed on its own with
 * k_t = ceil(n_t / CF) (layerwise compression, Sec. III-A); the message is
 * segment-major.  out_stats is [max(n_seg,1)][n_cf][4] doubles:
 * { ||g_c||^2, ||g_ef||^2, gain, |acc| of the smallest selected entry }.
 */
int oracle_compress(const float* grad, float* residual, int64_t n,
                    const double* cf_list, int n_cf, int commit,
                    const int64_t* seg_offsets, int n_seg,
                    int32_t* out_idx, float* out_val, int64_t out_capacity,
                    int64_t* out_count, double* out_stats)
{
    if (!grad || !residual || !cf_list || !out_idx || !out_val || !out_stats) return ORACLE_BAD_ARG;
    if (n <= 0 || n > 2147483647LL || n_cf < 1 || commit < 0 || commit >= n_cf) return ORACLE_BAD_ARG;
    for (int j = 0; j < n_cf; ++j)
        if (!(cf_list[j] >= 1.0) || isinf(cf_list[j])) return ORACLE_BAD_ARG;

    int64_t flat[2] = {0, n};
    const int64_t* off = seg_offsets;
    int ns = n_seg;
    if (!off || ns <= 0) {
        off = flat;
        ns = 1;
    }
    if (off[0] != 0 || off[ns] != n) return ORACLE_BAD_ARG;
    int64_t total = 0;
    for (int t = 0; t < ns; ++t) {
        if (off[t + 1] <= off[t]) return ORACLE_BAD_ARG;
        total += oracle_k(off[t + 1] - off[t], cf_list[commit]);
    }
    if (total > out_capacity) return ORACLE_CAPACITY;

    int64_t written = 0;
    for (int t = 0; t < ns; ++t) {
        int64_t got = 0;
        int rc = compress_one(grad, residual, off[t], off[t + 1] - off[t], cf_list, n_cf, commit,
                              out_idx + written, out_val + written, &got,
                              out_stats + (size_t)t * (size_t)n_cf * 4);
        if (rc != ORACLE_OK) return rc;
        written += got;
    }
    if (out_count) *out_count = written;
    return ORACLE_OK;
}

/*
 * Decompression (Sec. III-A: rebuild the compressed gradient to the original
 * dimension) with aggregation of W workers' messages: worker w's pairs start at
 * sum(counts[0..w)); contributions are added into dense_out in worker order,
 * pairs in stored order, each add one binary32 add.  dense_out is not cleared.
 */
int oracle_decompress_accumulate(const int32_t* idx, const float* val,
                                 const int64_t* counts, int W, int64_t n, float* dense_out)
{
    if (!counts || !dense_out || W < 1 || n <= 0) return ORACLE_BAD_ARG;
    int64_t at = 0;
    for (int w = 0; w < W; ++w) {
        if (counts[w] < 0) return ORACLE_BAD_ARG;
        for (int64_t r = 0; r < counts[w]; ++r) {
            int64_t i = idx[at + r];
            if (i < 0 || i >= n) return ORACLE_BAD_ARG;
            volatile float s = dense_out[i] + val[at + r];
            dense_out[i] = s;
        }
        at += counts[w];
    }
    return ORACLE_OK;
}

/*
 * Parameter update from the W workers' messages without a dense gradient in between (Alg. 1, the update
 * w_{i+1} = w_i - eta * g~ with g~ the aggregate of the compressed gradients; Eq. (1) for the 1/N of the mean):
 * with alpha = -eta / W every pair is one step  w[idx] = w[idx] + alpha * val,  the product rounded to binary32,
 * then the sum rounded to binary32, workers in order, pairs in stored order.  In exact arithmetic this is
 * w - eta * (1/W) * sum of the decompressed messages; alpha = 1 is oracle_decompress_accumulate.
 */
int oracle_decompress_update(const int32_t* idx, const float* val,
                             const int64_t* counts, int W, int64_t n, float alpha, float* w_inout)
{
    if (!counts || !w_inout || W < 1 || n <= 0) return ORACLE_BAD_ARG;
    int64_t at = 0;
    for (int w = 0; w < W; ++w) {
        if (counts[w] < 0) return ORACLE_BAD_ARG;
        for (int64_t r = 0; r < counts[w]; ++r) {
            int64_t i = idx[at + r];
            if (i < 0 || i >= n) return ORACLE_BAD_ARG;
            volatile float step = alpha * val[at + r];
            volatile float s = w_inout[i] + step;
            w_inout[i] = s;
        }
        at += counts[w];
    }
    return ORACLE_OK;
}

/*
 * Commit of a message into the residual (Alg. 1, residual update: residual = g_o - g_c leaves x - x = +0 in
 * the slots that were sent): residual[idx[i]] = +0.0f.  Indices outside [0, n) are skipped.
 */
int oracle_commit(const int32_t* idx, int64_t count, float* residual, int64_t n)
{
    if (!residual || count < 0 || n <= 0 || (count > 0 && !idx)) return ORACLE_BAD_ARG;
    for (int64_t i = 0; i < count; ++i)
        if (idx[i] >= 0 && idx[i] < n) residual[idx[i]] = 0.0f;
    return ORACLE_OK;
}

/*
 * Multi-level compression (Sec. IV-C): given the message X1 = C(theta1, X) as k1 (index, value) pairs in
 * ascending index order, produce X2' = C(theta2', X1) with theta2' = theta2 / theta1: the
 * k2 = ceil(k1 / cf_rel) entries of X1 of largest magnitude, ties to the lower position (= lower index),
 * again in ascending index order.  For Top-k, X2' equals the direct C(theta2, X).
 *
 * Deferred commit: if residual is not NULL it is the residual left by committing X1 (zero in X1's slots);
 * the entries of X1 that are not in X2' go back into it (residual[idx] = value), so that afterwards it is
 * the residual of committing X2' instead (Alg. 1 updates the residual with whichever message is sent).
 *
 * seg_counts (NULL = one tensor): pairs of X1 per tensor, for layerwise messages; each tensor is
 * recompressed on its own with k2_t = ceil(k1_t / cf_rel).  out_stats is [max(n_seg,1)][4]:
 * { ||X2'||^2, ||X1||^2, their ratio (1 if ||X1||^2 == 0), |value| of the smallest selected entry }.
 */
int oracle_recompress(const int32_t* idx1, const float* val1, int64_t k1, double cf_rel,
                      float* residual, int64_t n, const int64_t* seg_counts, int n_seg,
                      int32_t* out_idx, float* out_val, int64_t out_capacity, int64_t* out_count,
                      double* out_stats)
{
    if (!idx1 || !val1 || !out_idx || !out_val || !out_stats || k1 <= 0 || !(cf_rel >= 1.0) || isinf(cf_rel))
        return ORACLE_BAD_ARG;
    int64_t one[1] = {k1};
    const int64_t* cnt = seg_counts;
    int ns = n_seg;
    if (!cnt || ns <= 0) { cnt = one; ns = 1; }
    int64_t sum = 0, total = 0;
    for (int t = 0; t < ns; ++t) {
        if (cnt[t] <= 0) return ORACLE_BAD_ARG;
        sum += cnt[t];
        total += oracle_k(cnt[t], cf_rel);
    }
    if (sum != k1) return ORACLE_BAD_ARG;
    if (total > out_capacity) return ORACLE_CAPACITY;

    int64_t at = 0, written = 0;
    for (int t = 0; t < ns; ++t) {
        const int64_t m = cnt[t], k2 = oracle_k(m, cf_rel);
        entry_t* order = (entry_t*)malloc((size_t)m * sizeof(entry_t));
        uint32_t* chosen = (uint32_t*)malloc((size_t)k2 * sizeof(uint32_t));
        char* keep = (char*)calloc((size_t)m, 1);
        if (!order || !chosen || !keep) { free(order); free(chosen); free(keep); return ORACLE_NOMEM; }
        double ss_all = 0.0, ss_sel = 0.0;
        for (int64_t i = 0; i < m; ++i) {
            order[i].mag = f32_bits(val1[at + i]) & 0x7FFFFFFFu;
            order[i].pos = (uint32_t)i;
            ss_all += (double)val1[at + i] * (double)val1[at + i];
        }
        qsort(order, (size_t)m, sizeof(entry_t), cmp_entry);
        for (int64_t r = 0; r < k2; ++r) {
            chosen[r] = order[r].pos;
            ss_sel += (double)val1[at + order[r].pos] * (double)val1[at + order[r].pos];
        }
        double* st = out_stats + 4 * (size_t)t;
        st[0] = ss_sel;
        st[1] = ss_all;
        st[2] = (ss_all == 0.0) ? 1.0 : ss_sel / ss_all;
        st[3] = fabs((double)val1[at + order[k2 - 1].pos]);
        qsort(chosen, (size_t)k2, sizeof(uint32_t), cmp_u32);
        for (int64_t r = 0; r < k2; ++r) {
            out_idx[written + r] = idx1[at + chosen[r]];
            out_val[written + r] = val1[at + chosen[r]];
            keep[chosen[r]] = 1;
        }
        if (residual) {
            for (int64_t i = 0; i < m; ++i) {
                const int64_t g = idx1[at + i];
                if (g < 0 || g >= n) { free(order); free(chosen); free(keep); return ORACLE_BAD_ARG; }
                if (!keep[i]) residual[g] = val1[at + i];
            }
        }
        free(order); free(chosen); free(keep);
        at += m;
        written += k2;
    }
    if (out_count) *out_count = written;
    return ORACLE_OK;
}


/*
 * Random-k (Sec. II-C: "Random-k does so randomly with negligible compression overhead"): the same
 * error-feedback step, message layout, residual update and gain as Top-k, but the k = ceil(n / CF) entries
 * that are kept are a pseudo-random subset instead of the largest.  Reading taken here (the paper does not
 * say how the subset is drawn): every index i of the flat gradient gets the priority P(seed, i) below, a
 * keyed bijection of the 31-bit integers (so no two indices share a priority), and a tensor keeps its k
 * entries of highest priority.  With one seed the selections for different CFs are nested, and a segment's
 * selection does not depend on how the rest of the gradient is split.  The caller changes the seed from
 * iteration to iteration.
 *
 * P: the seed is first mixed into two 31-bit keys, so that neighbouring seeds give unrelated draws:
 *   z = first output of the SplitMix64 generator started at `seed` (Steele, Lea, Flood 2014):
 *       z = seed + 0x9E3779B97F4A7C15;  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9;
 *       z = (z ^ (z >> 27)) * 0x94D049BB133111EB;  z = z ^ (z >> 31)      (64-bit unsigned arithmetic)
 *   s0 = z mod 2^31,  s1 = (z >> 32) mod 2^31
 * then, with M = 2^31 - 1, on 32-bit unsigned arithmetic:
 *   x = (i + s0) & M
 *   x ^= x >> 16;  x = (x * 0x7FEB352D) & M
 *   x ^= x >> 15;  x = (x * 0x046CA68B) & M
 *   x ^= x >> 16;  x = (x + s1) & M
 *   x ^= x >> 14;  x = (x * 0x2C1B3C6D) & M
 *   x ^= x >> 15;  x = (x * 0x297A2D39) & M
 *   x ^= x >> 15
 * Every step (adding a constant, multiplying by an odd constant, xor with a right shift) is a bijection
 * of [0, 2^31).
 */
uint64_t oracle_splitmix64_first(uint64_t seed)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint32_t oracle_randomk_priority(uint64_t seed, uint32_t i)
{
    const uint32_t M = 0x7FFFFFFFu;
    const uint64_t z = oracle_splitmix64_first(seed);
    const uint32_t s0 = (uint32_t)(z & M), s1 = (uint32_t)((z >> 32) & M);
    uint32_t x = (i + s0) & M;
    x ^= x >> 16; x = (x * 0x7FEB352Du) & M;
    x ^= x >> 15; x = (x * 0x046CA68Bu) & M;
    x ^= x >> 16; x = (x + s1) & M;
    x ^= x >> 14; x = (x * 0x2C1B3C6Du) & M;
    x ^= x >> 15; x = (x * 0x297A2D39u) & M;
    x ^= x >> 15;
    return x;
}

/* One tensor of a Random-k call: as compress_one, ordered by priority instead of magnitude. */
static int randomk_one(const float* grad, float* residual, int64_t base, int64_t n, uint64_t seed,
                       const double* cf_list, int n_cf, int commit,
                       int32_t* out_idx, float* out_val, int64_t* n_out, double* stats)
{
    entry_t* order = (entry_t*)malloc((size_t)n * sizeof(entry_t));
    if (!order) return ORACLE_NOMEM;
    double ss_dense = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        volatile float a = residual[base + i] + grad[base + i];  /* error feedback, one binary32 add */
        residual[base + i] = a;
        ss_dense += (double)a * (double)a;
        order[i].mag = oracle_randomk_priority(seed, (uint32_t)(base + i));
        order[i].pos = (uint32_t)i;
    }
    qsort(order, (size_t)n, sizeof(entry_t), cmp_entry);  /* highest priority first */
    for (int j = 0; j < n_cf; ++j) {
        int64_t k = oracle_k(n, cf_list[j]);
        double ss_sel = 0.0;
        for (int64_t r = 0; r < k; ++r) {
            double v = (double)residual[base + order[r].pos];
            ss_sel += v * v;
        }
        stats[4 * j + 0] = ss_sel;
        stats[4 * j + 1] = ss_dense;
        stats[4 * j + 2] = (ss_dense == 0.0) ? 1.0 : ss_sel / ss_dense;
        stats[4 * j + 3] = (double)order[k - 1].mag;  /* lowest selected priority */
    }
    int64_t kc = oracle_k(n, cf_list[commit]);
    uint32_t* chosen = (uint32_t*)malloc((size_t)kc * sizeof(uint32_t));
    if (!chosen) {
        free(order);
        return ORACLE_NOMEM;
    }
    for (int64_t r = 0; r < kc; ++r) chosen[r] = order[r].pos;
    qsort(chosen, (size_t)kc, sizeof(uint32_t), cmp_u32);
    for (int64_t r = 0; r < kc; ++r) {
        int64_t g = base + (int64_t)chosen[r];
        out_idx[r] = (int32_t)g;
        out_val[r] = residual[g];
    }
    for (int64_t r = 0; r < kc; ++r) residual[base + (int64_t)chosen[r]] = 0.0f;
    *n_out = kc;
    free(chosen);
    free(order);
    return ORACLE_OK;
}

/*
 * Arguments as oracle_compress, plus the seed.  out_stats rows are
 * { ||g_c||^2, ||g_ef||^2, gain, lowest selected priority }.
 */
int oracle_randomk_compress(const float* grad, float* residual, int64_t n,
                            const double* cf_list, int n_cf, int commit, uint64_t seed,
                            const int64_t* seg_offsets, int n_seg,
                            int32_t* out_idx, float* out_val, int64_t out_capacity,
                            int64_t* out_count, double* out_stats)
{
    if (!grad || !residual || !cf_list || !out_idx || !out_val || !out_stats) return ORACLE_BAD_ARG;
    if (n <= 0 || n > 2147483647LL || n_cf < 1 || commit < 0 || commit >= n_cf) return ORACLE_BAD_ARG;
    for (int j = 0; j < n_cf; ++j)
        if (!(cf_list[j] >= 1.0) || isinf(cf_list[j])) return ORACLE_BAD_ARG;
    int64_t flat[2] = {0, n};
    const int64_t* off = seg_offsets;
    int ns = n_seg;
    if (!off || ns <= 0) {
        off = flat;
        ns = 1;
    }
    if (off[0] != 0 || off[ns] != n) return ORACLE_BAD_ARG;
    int64_t total = 0;
    for (int t = 0; t < ns; ++t) {
        if (off[t + 1] <= off[t]) return ORACLE_BAD_ARG;
        total += oracle_k(off[t + 1] - off[t], cf_list[commit]);
    }
    if (total > out_capacity) return ORACLE_CAPACITY;
    int64_t written = 0;
    for (int t = 0; t < ns; ++t) {
        int64_t got = 0;
        int rc = randomk_one(grad, residual, off[t], off[t + 1] - off[t], seed, cf_list, n_cf, commit,
                             out_idx + written, out_val + written, &got,
                             out_stats + (size_t)t * (size_t)n_cf * 4);
        if (rc != ORACLE_OK) return rc;
        written += got;
    }
    if (out_count) *out_count = written;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Threshold sparsifier with error feedback.  Sec. II-C describes DGC's selection rule in one clause:
 * entries below a threshold are discarded; its momentum correction and gradient clipping are named
 * there but not defined, and are not part of this.  Steps:
 *   acc = residual + grad                      (Sec. III-B error feedback, as for every compressor)
 *   keep entry i  <=>  |acc[i]| >= tau         (Sec. II-C, DGC: what lies below the threshold is dropped)
 *   message = the kept (index, acc) pairs in ascending index order; residual = acc with the kept slots
 *   set to +0.0f (Alg. 1 residual update); gain = ||message||^2 / ||acc||^2 (Sec. III-B), 1 if 0 / 0.
 * Readings: "below" is strict, so an entry equal to tau is kept; magnitudes are compared as bit
 * patterns with the sign cleared, as everywhere in this file (a NaN pattern ranks above every finite
 * tau and is kept); tau is a positive, finite binary32 number.  The number of kept entries is data
 * dependent: *out_count always gets it; if it exceeds out_capacity nothing is emitted or removed
 * (the residual holds acc), the statistics are still those of the full selection, and the function
 * returns ORACLE_CAPACITY.  out_stats = { ||g_c||^2, ||g_ef||^2, gain, tau }.
 * ------------------------------------------------------------------------------------------------ */
int oracle_threshold_compress(const float* grad, float* residual, int64_t n, float tau,
                              int32_t* out_idx, float* out_val, int64_t out_capacity,
                              int64_t* out_count, double* out_stats)
{
    if (!grad || !residual || !out_count || !out_stats || n <= 0 || n > 2147483647LL) return ORACLE_BAD_ARG;
    if (!(tau > 0.0f) || isinf(tau)) return ORACLE_BAD_ARG;
    if (out_capacity > 0 && (!out_idx || !out_val)) return ORACLE_BAD_ARG;
    const uint32_t tau_bits = f32_bits(tau);
    double ss_dense = 0.0, ss_sel = 0.0;
    int64_t kept = 0;
    for (int64_t i = 0; i < n; ++i) {
        volatile float a = residual[i] + grad[i];
        residual[i] = a;
        ss_dense += (double)a * (double)a;
        if ((f32_bits(a) & 0x7FFFFFFFu) >= tau_bits) {
            ss_sel += (double)a * (double)a;
            ++kept;
        }
    }
    out_stats[0] = ss_sel;
    out_stats[1] = ss_dense;
    out_stats[2] = (ss_dense == 0.0) ? 1.0 : ss_sel / ss_dense;
    out_stats[3] = (double)tau;
    *out_count = kept;
    if (kept > out_capacity) return ORACLE_CAPACITY;
    int64_t w = 0;
    for (int64_t i = 0; i < n; ++i) {
        if ((f32_bits(residual[i]) & 0x7FFFFFFFu) >= tau_bits) {
            out_idx[w] = (int32_t)i;
            out_val[w] = residual[i];
            residual[i] = 0.0f;
            ++w;
        }
    }
    return ORACLE_OK;
}
