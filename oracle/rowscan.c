/*
 * Row-sampled CPU oracle for sparse graph attention -- TEST INFRASTRUCTURE.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may load
 * this.  It shares no code, header or table with the HIP library.
 *
 * It evaluates masked attention by definition for a *sample of query rows* of
 * problems too large for a dense L x L matrix: for a row i it scans every key
 * j in [0, L), applies the mask predicate of Section II-C, and where the
 * predicate is 0 the score is -inf, which contributes exactly 0 to the softmax
 * sums, so the dot product is skipped.  The row result is the two-pass
 * softmax (max, then exp and sum) of Eq. 1 followed by the weighted sum of V
 * rows, all in double precision from the stored fp32 values (fp16 inputs are
 * widened exactly to fp32 by the caller).
 *
 * Readings of the paper (inclusive window, stride for dilation, caller's
 * scale, empty row -> 0 / -inf, symmetric leading global tokens, block mask
 * with counter-based random key blocks) are the ones listed at the top of
 * oracle/reference.py; this file is pinned against that dense NumPy oracle in
 * tests/test_oracle_rowscan.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t kind;            /* 0 sliding, 1 dilated, 2 global+local, 3 block mask,
                                4 global minus local, 5 2-D dilated blocks */
    int32_t window;
    int32_t stride;
    int32_t n_global;
    int32_t block;
    int32_t window_blocks;
    int32_t n_global_blocks;
    int32_t n_random_blocks;
    int64_t L;
    uint64_t seed;
} orc_mask;

static uint64_t orc_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Membership vector over key blocks for query block b (block mask only).
 * member must hold nb bytes. */
static void orc_block_members(const orc_mask *mk, int64_t b, uint8_t *member)
{
    const int64_t nb = mk->L / mk->block;
    const int64_t G = mk->n_global_blocks;
    if (b < G) {
        memset(member, 1, (size_t)nb);
        return;
    }
    memset(member, 0, (size_t)nb);
    for (int64_t g = 0; g < G && g < nb; ++g) member[g] = 1;
    for (int64_t kb = b - mk->window_blocks; kb <= b + mk->window_blocks; ++kb)
        if (kb >= 0 && kb < nb) member[kb] = 1;
    const uint64_t gold = 0x9E3779B97F4A7C15ULL;
    const uint64_t stream = orc_mix64(mk->seed + gold * (uint64_t)(b + 1));
    int picked = 0;
    uint64_t a = 0;
    while (picked < mk->n_random_blocks) {
        uint64_t cand = orc_mix64(stream + gold * (a + 1)) % (uint64_t)nb;
        ++a;
        if (!member[cand]) {
            member[cand] = 1;
            ++picked;
        }
    }
}

/* A[i][j] for the element-level masks. */
static inline int orc_pred_elem(const orc_mask *mk, int64_t i, int64_t j)
{
    int64_t diff = i - j;
    int64_t ad = diff < 0 ? -diff : diff;
    switch (mk->kind) {
    case 0:
        return ad <= mk->window;
    case 1:
        return ad <= (int64_t)mk->window * mk->stride && (ad % mk->stride) == 0;
    case 2:
        return ad <= mk->window || i < mk->n_global || j < mk->n_global;
    case 4:
        return (i < mk->n_global || j < mk->n_global) && !(ad <= mk->window);
    case 5:
        return i / mk->block == j / mk->block && (i % mk->block) % mk->stride == 0 &&
               (j % mk->block) % mk->stride == 0;
    default:
        return 0;
    }
}

/* Neighbours of row i in increasing key order: scan all j.  Returns the degree;
 * writes at most cap indices into out (out may be NULL to only count). */
int64_t orc_row_neighbors(const orc_mask *mk, int64_t i, int64_t *out, int64_t cap)
{
    int64_t n = 0;
    if (mk->kind == 3) {
        const int64_t B = mk->block;
        const int64_t nb = mk->L / B;
        uint8_t *member = (uint8_t *)malloc((size_t)nb);
        orc_block_members(mk, i / B, member);
        for (int64_t j = 0; j < mk->L; ++j) {
            if (member[j / B]) {
                if (out && n < cap) out[n] = j;
                ++n;
            }
        }
        free(member);
        return n;
    }
    for (int64_t j = 0; j < mk->L; ++j) {
        if (orc_pred_elem(mk, i, j)) {
            if (out && n < cap) out[n] = j;
            ++n;
        }
    }
    return n;
}

/* Degrees of the listed rows (parallel over rows). */
void orc_degrees(const orc_mask *mk, const int64_t *rows, int64_t n_rows, int64_t *deg)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t r = 0; r < n_rows; ++r)
        deg[r] = orc_row_neighbors(mk, rows[r], NULL, 0);
}

/* Total edge count by scanning every (i, j) pair: NNZ of Section II-D. */
int64_t orc_count_edges(const orc_mask *mk)
{
    int64_t total = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : total)
    for (int64_t i = 0; i < mk->L; ++i)
        total += orc_row_neighbors(mk, i, NULL, 0);
    return total;
}

/* Masked attention of one query against an explicit list of n (key, value)
 * rows already gathered: two-pass softmax in double.
 * q [d], Kg/Vg [n][d] float32, out [d] double, lse 1 double. */
void orc_attend_gathered(const float *q, const float *Kg, const float *Vg, int64_t n,
                         int32_t d, double scale, double *out, double *lse)
{
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    if (n == 0) {
        *lse = -INFINITY;
        return;
    }
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    double M = -INFINITY;
    for (int64_t e = 0; e < n; ++e) {
        double acc = 0.0;
        const float *k = Kg + e * d;
        for (int c = 0; c < d; ++c) acc += (double)q[c] * (double)k[c];
        s[e] = scale * acc;
        if (s[e] > M) M = s[e];
    }
    double Z = 0.0;
    for (int64_t e = 0; e < n; ++e) {
        s[e] = exp(s[e] - M);
        Z += s[e];
    }
    for (int64_t e = 0; e < n; ++e) {
        const double p = s[e] / Z;
        const float *v = Vg + e * d;
        for (int c = 0; c < d; ++c) out[c] += p * (double)v[c];
    }
    *lse = M + log(Z);
    free(s);
}

/* Sampled rows of one head with the whole K, V on the host.
 * Q, K, V: [L][d] float32; rows [n_rows]; out [n_rows][d] double; lse [n_rows].
 * Returns the number of edges visited (sum of the sampled rows' degrees). */
int64_t orc_attend_rows(const orc_mask *mk, const float *Q, const float *K, const float *V,
                        int32_t d, double scale, const int64_t *rows, int64_t n_rows,
                        double *out, double *lse)
{
    int64_t edges = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : edges)
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t i = rows[r];
        int64_t deg = orc_row_neighbors(mk, i, NULL, 0);
        int64_t *nb = (int64_t *)malloc(sizeof(int64_t) * (size_t)(deg > 0 ? deg : 1));
        orc_row_neighbors(mk, i, nb, deg);
        float *Kg = (float *)malloc(sizeof(float) * (size_t)(deg > 0 ? deg : 1) * d);
        float *Vg = (float *)malloc(sizeof(float) * (size_t)(deg > 0 ? deg : 1) * d);
        for (int64_t e = 0; e < deg; ++e) {
            memcpy(Kg + e * d, K + nb[e] * d, sizeof(float) * d);
            memcpy(Vg + e * d, V + nb[e] * d, sizeof(float) * d);
        }
        orc_attend_gathered(Q + i * d, Kg, Vg, deg, d, scale, out + r * d, lse + r);
        edges += deg;
        free(nb);
        free(Kg);
        free(Vg);
    }
    return edges;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
