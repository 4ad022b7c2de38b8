/*
 * TEST INFRASTRUCTURE ONLY -- brute-force fp64 definition of knowledge-base
 * retrieval.  Nothing in the product path may link, load or call this file.
 *
 * What is defined here.  The paper's State Selector looks up, in a store of
 * <state, <optimization, score>> entries, the pairs that fit the kernel's state,
 * and the Optimization Selector keeps the top-k of them (Section 3,
 * component list and the paragraph that walks through one task).  The paper
 * gives no numeric form for that step; the numeric model used throughout this
 * repository is: every entry i has a key vector K_i, a query state is a vector
 * Q_r, relevance is the cosine of the two, an optional 64-bit tag filter keeps
 * entry i for query r iff (qmask_r & tag_i) != 0, and the k best survivors are
 * returned ordered by (score descending, index ascending).
 *
 * Fidelity to the paper is therefore unpinned (the paper prints no worked
 * retrieval example); fidelity to the plain definition above is pinned by the
 * CPU tests: a hand-computed cosine example, self-query / permutation /
 * scaling invariants, an independent numpy formulation, an O(N^2) rank count
 * on tiny inputs, and an independent library decode of every bf16 / e4m3 code.
 *
 * Everything is fp64, plain loops, full sort.  No blocking, no partial
 * selection, no shared code with the GPU path.
 *
 * Weighted random selection (second half of this file).  The Optimization
 * Selector picks its top-k at random, with weights given by the predicted
 * performance gains (Section 3, same paragraph).  The
 * paper gives no formula; the model used here: entry i carries a predicted
 * gain g_i > 0, query r draws k entries WITHOUT replacement from its candidate
 * set with probability proportional to w_ri = g_i * exp(score_ri / T), T > 0 a
 * temperature.  By the Gumbel-top-k identity that is the k largest of
 *     key_ri = score_ri / T + ln g_i + G_ri,    G_ri iid standard Gumbel,
 * and G_ri comes from the counter-based generator Philox4x32-10 (Salmon,
 * Moraes, Dror, Shaw, SC'11) keyed by the caller's seed with (entry, query) as
 * the counter, so the draw is a pure function of (seed, r, i).  Pins: the
 * generator's published known-answer vectors, moments of the variates, the
 * closed-form inclusion probabilities for k = 1 and ordered pairs for k = 2,
 * the T -> 0 limit (plain top-k), determinism.  Fidelity of this model to the
 * paper is unpinned for the same reason as above.
 *
 * Row quantisation to E4M3 (end of this file): the storage form of compressed
 * keys and of fp8 queries in the same numeric model: per row, scale = max|x| /
 * 448 and every element goes to the nearest e4m3 value of x / scale (ties to
 * the even code), scale and quotient taken in binary32 because they decide an
 * integer code.  Written as a search over all 127 non-negative finite codes.
 * Pins: an independent library's float32 -> e4m3 conversion on random rows,
 * every midpoint between neighbouring e4m3 values, saturation, zero rows.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_FP8_E4M3 = 2 };

/* bf16 = the upper 16 bits of an IEEE binary32; the value is exact in fp64. */
double oracle_decode_bf16(uint16_t bits)
{
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* OCP 8-bit float E4M3 ("FN" flavour): 1 sign, 4 exponent (bias 7), 3 mantissa
 * bits; exponent field 0 is subnormal m/8 * 2^-6; there is no infinity and the
 * single NaN pattern per sign is S.1111.111; the largest finite value is 448. */
double oracle_decode_e4m3(uint8_t code)
{
    int s = (code >> 7) & 1;
    int e = (code >> 3) & 15;
    int m = code & 7;
    double v;
    if (e == 15 && m == 7)
        return NAN;
    if (e == 0)
        v = ldexp((double)m / 8.0, -6);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

static size_t elem_bytes(int dtype)
{
    return dtype == ORACLE_F32 ? 4 : dtype == ORACLE_BF16 ? 2 : 1;
}

/* Decode row `row` of a row-major [rows, d] array of stored bits into fp64.
 * For e4m3 keys the stored value is row_scale[row] * decode(code). */
static void decode_row(const void *base, int dtype, const float *row_scale, int64_t row, int64_t d, double *out)
{
    const uint8_t *p = (const uint8_t *)base + (size_t)row * (size_t)d * elem_bytes(dtype);
    for (int64_t j = 0; j < d; ++j) {
        if (dtype == ORACLE_F32) {
            float f;
            memcpy(&f, p + 4 * j, 4);
            out[j] = (double)f;
        } else if (dtype == ORACLE_BF16) {
            uint16_t h;
            memcpy(&h, p + 2 * j, 2);
            out[j] = oracle_decode_bf16(h);
        } else {
            double sc = row_scale ? (double)row_scale[row] : 1.0;
            out[j] = sc * oracle_decode_e4m3(p[j]);
        }
    }
}

static double l2norm(const double *v, int64_t d)
{
    double s = 0.0;
    for (int64_t j = 0; j < d; ++j)
        s += v[j] * v[j];
    return sqrt(s);
}

/*
 * scores[r*N + i] = <Q_r, K_i> / (|Q_r| |K_i|), or 0 when either norm is 0.
 * Returns 0 on success, 1 on bad arguments, 2 when out of memory.
 */
int oracle_score_matrix(const void *keys, int key_dtype, const float *row_scale, int64_t N, int64_t d,
                        const void *queries, int q_dtype, int64_t Q, double *scores)
{
    if (!keys || !queries || !scores || N < 0 || Q < 0 || d <= 0)
        return 1;
    /* queries in e4m3 carry no row scale: a positive factor per query row cancels in the cosine */
    if (key_dtype < 0 || key_dtype > 2 || q_dtype < 0 || q_dtype > 2)
        return 1;
    double *qd = (double *)malloc(sizeof(double) * (size_t)(Q > 0 ? Q : 1) * (size_t)d);
    double *qn = (double *)malloc(sizeof(double) * (size_t)(Q > 0 ? Q : 1));
    if (!qd || !qn) {
        free(qd);
        free(qn);
        return 2;
    }
    for (int64_t r = 0; r < Q; ++r) {
        decode_row(queries, q_dtype, NULL, r, d, qd + r * d);
        qn[r] = l2norm(qd + r * d, d);
    }
    int failed = 0;
#pragma omp parallel
    {
        double *kd = (double *)malloc(sizeof(double) * (size_t)d);
        if (!kd) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            if (!kd)
                continue;
            decode_row(keys, key_dtype, row_scale, i, d, kd);
            double kn = l2norm(kd, d);
            for (int64_t r = 0; r < Q; ++r) {
                const double *q = qd + r * d;
                double dot = 0.0;
                for (int64_t j = 0; j < d; ++j)
                    dot += q[j] * kd[j];
                double denom = qn[r] * kn;
                scores[r * N + i] = (qn[r] == 0.0 || kn == 0.0) ? 0.0 : dot / denom;
            }
        }
        free(kd);
    }
    free(qd);
    free(qn);
    return failed ? 2 : 0;
}

typedef struct {
    double score;
    int64_t index;
} pair_t;

/* Strict total order: higher score first, then lower index.  -0.0 == 0.0. */
static int pair_cmp(const void *a, const void *b)
{
    const pair_t *x = (const pair_t *)a, *y = (const pair_t *)b;
    if (x->score > y->score)
        return -1;
    if (x->score < y->score)
        return 1;
    if (x->index < y->index)
        return -1;
    if (x->index > y->index)
        return 1;
    return 0;
}

/*
 * Selection for one query from its N scores: candidate set = all i (tags or
 * qmask absent) or { i : (qmask & tags[i]) != 0 }; the candidates are sorted
 * in full by (score desc, index asc); the first min(k, |C|) are written, the
 * rest of the k slots are padded with index -1 and score -infinity.
 * `use_mask` = 0 means "no filter" (then tags may be NULL and qmask is
 * ignored).  Returns the number of candidates, or -1 on error.
 */
int64_t oracle_select(const double *scores, int64_t N, const uint64_t *tags, int use_mask, uint64_t qmask,
                      int64_t k, int64_t *out_index, double *out_score)
{
    if (!scores || !out_index || !out_score || N < 0 || k < 0 || (use_mask && !tags))
        return -1;
    pair_t *c = (pair_t *)malloc(sizeof(pair_t) * (size_t)(N > 0 ? N : 1));
    if (!c)
        return -1;
    int64_t n = 0;
    for (int64_t i = 0; i < N; ++i) {
        if (use_mask && (qmask & tags[i]) == 0)
            continue;
        if (scores[i] == -INFINITY)     /* only selection keys of zero-gain entries: never candidates */
            continue;
        c[n].score = scores[i];
        c[n].index = i;
        ++n;
    }
    qsort(c, (size_t)n, sizeof(pair_t), pair_cmp);
    for (int64_t p = 0; p < k; ++p) {
        if (p < n) {
            out_index[p] = c[p].index;
            out_score[p] = c[p].score;
        } else {
            out_index[p] = -1;
            out_score[p] = -INFINITY;
        }
    }
    free(c);
    return n;
}

/*
 * The whole query: score matrix, then one selection per query.
 * qmask == NULL means no filtering for any query.  If scores_out is not NULL
 * it receives the full [Q, N] fp64 score matrix (the comparator needs it).
 * Returns 0 on success.
 */
int oracle_query(const void *keys, int key_dtype, const float *row_scale, const uint64_t *tags, int64_t N,
                 int64_t d, const void *queries, int q_dtype, int64_t Q, const uint64_t *qmask, int64_t k,
                 int64_t *out_index, double *out_score, double *scores_out)
{
    if (k < 0 || !out_index || !out_score || (qmask && !tags))
        return 1;
    double *scores = scores_out;
    if (!scores) {
        scores = (double *)malloc(sizeof(double) * (size_t)(Q * N > 0 ? Q * N : 1));
        if (!scores)
            return 2;
    }
    int rc = oracle_score_matrix(keys, key_dtype, row_scale, N, d, queries, q_dtype, Q, scores);
    int bad = 0;
    if (rc == 0) {
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t r = 0; r < Q; ++r) {
            int64_t n = oracle_select(scores + r * N, N, tags, qmask != NULL, qmask ? qmask[r] : 0, k,
                                      out_index + r * k, out_score + r * k);
            if (n < 0) {
#pragma omp atomic write
                bad = 1;
            }
        }
    }
    if (!scores_out)
        free(scores);
    return rc ? rc : (bad ? 2 : 0);
}

/* ------------------------------------------------------------------------
 * Weighted random selection
 * ------------------------------------------------------------------------ */

/* Philox4x32 with 10 rounds: counter 4 x 32 bit, key 2 x 32 bit.  One round
 * multiplies counter words 0 and 2 by two odd constants, keeps both halves of
 * the 64-bit products and mixes in the other two words and the key; the key
 * is bumped by two Weyl constants between rounds. */
void oracle_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4])
{
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0;
        c1 = n1;
        c2 = n2;
        c3 = n3;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

/* The uniform variate of pair (query, entry): generator call with counter
 * (entry / 4, query, 0, 0) and the seed as key; entry % 4 picks one of the
 * four output words; its upper 23 bits b give U = (b + 1/2) / 2^23 = (2b + 1) / 2^24,
 * which is in (0, 1) and exactly representable in binary32 (24-bit significand)
 * and binary64. */
double oracle_uniform(uint64_t seed, uint32_t query, uint64_t entry)
{
    uint32_t ctr[4] = {(uint32_t)(entry >> 2), query, 0u, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    oracle_philox4x32_10(ctr, key, w);
    return ((double)(w[entry & 3] >> 9) + 0.5) / 8388608.0;
}

/* Standard Gumbel variate by inversion: G = -ln(-ln U). */
double oracle_gumbel(uint64_t seed, uint32_t query, uint64_t entry)
{
    return -log(-log(oracle_uniform(seed, query, entry)));
}

/* Selection keys of Q queries (global query numbers first_query, ...) from
 * their [Q, N] score matrix: key = score / T + ln(gain) + Gumbel; an entry
 * with gain <= 0 gets -infinity (it can never be drawn).  Returns 0 on success. */
int oracle_selection_keys(const double *scores, int64_t Q, int64_t N, const float *gain, double temperature,
                          uint64_t seed, int64_t first_query, double *keys_out)
{
    if (!scores || !gain || !keys_out || !(temperature > 0.0) || Q < 0 || N < 0)
        return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < Q; ++r)
        for (int64_t i = 0; i < N; ++i) {
            const double g = (double)gain[i];
            keys_out[r * N + i] = g > 0.0 ? scores[r * N + i] / temperature + log(g) +
                                                oracle_gumbel(seed, (uint32_t)(first_query + r), (uint64_t)i)
                                          : -INFINITY;
        }
    return 0;
}

/* Threads the parallel regions above will use (reported beside timings). */
#ifdef _OPENMP
#include <omp.h>
#endif
/*
 * The e4m3 code nearest to y: the magnitude goes to the closest of the finite non-negative values (codes 0x00
 * .. 0x7E, increasing in value with the code), a tie to the even code, anything above 448 to 448; the sign bit
 * of y is kept (so -0.0 gives 0x80).  y must not be NaN.
 */
uint8_t oracle_encode_e4m3(float y)
{
    const double a = fabs((double)y);
    int best = 0;
    double best_err = a;                       /* code 0 is 0.0 */
    for (int c = 1; c <= 0x7E; ++c) {
        const double err = fabs(oracle_decode_e4m3((uint8_t)c) - a);
        if (err < best_err || (err == best_err && (c & 1) == 0)) {
            best = c;
            best_err = err;
        }
    }
    return (uint8_t)(best | (signbit(y) ? 0x80 : 0));
}

/*
 * rows [n, d] (ORACLE_F32 or ORACLE_BF16 bits) -> codes [n, d], scale [n] (may be NULL):
 *   amax = max_j |x_j|;  scale = amax / 448 in binary32, or 1 when the row is all zeros;
 *   code_j = oracle_encode_e4m3( binary32( x_j / scale ) ).
 * Returns 0, or 1 on bad arguments.
 */
int oracle_quantize_rows(const void *rows, int dtype, int64_t n, int64_t d, uint8_t *codes, float *scale)
{
    if (!rows || !codes || n < 0 || d <= 0 || (dtype != ORACLE_F32 && dtype != ORACLE_BF16))
        return 1;
    double *x = (double *)malloc(sizeof(double) * (size_t)d);
    if (!x)
        return 1;
    for (int64_t i = 0; i < n; ++i) {
        decode_row(rows, dtype, NULL, i, d, x);            /* exact: both types are subsets of binary32 */
        float amax = 0.0f;
        for (int64_t j = 0; j < d; ++j)
            if (fabsf((float)x[j]) > amax)
                amax = fabsf((float)x[j]);
        const float sc = amax > 0.0f ? amax / 448.0f : 1.0f;
        if (scale)
            scale[i] = sc;
        for (int64_t j = 0; j < d; ++j) {
            const float y = (float)x[j] / sc;
            codes[i * d + j] = oracle_encode_e4m3(y);
        }
    }
    free(x);
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
