/*
 * CPU oracle for the SemantiCache compress-then-attend path.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded, fp64.  It shares no
 * code with the HIP library and nothing in the product path may call it; only
 * the tests, the smoke check and the benchmark's cpu_baseline leg do.
 *
 * Every function is the paper's definition written out step by step:
 *   sc_oracle_segment        Sec. 2.2, Eq. 1   (delimiter-bounded chunks)
 *   sc_oracle_cosine         Sec. 2.3, Eq. 2   (cosine similarity of keys)
 *   sc_oracle_gsc_chunk      Sec. 2.3, Alg. 1  (Greedy Seed-Based Clustering)
 *   sc_oracle_compress_head  Sec. 2.4, Eq. 3   (mean-pooled semantic cores,
 *                            concatenated with the untouched delimiter rows)
 *   sc_oracle_decode_head    Sec. 2.4, Eq. 4   (Proportional Attention)
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - strict ">" against the threshold, similarity to the seed's own key;
 *   - a similarity that is not a number (zero-norm key) is "not > tau";
 *   - empty chunks are legal and produce no cluster;
 *   - output rows of a head are ordered by position: for each chunk its cores
 *     in order of seed position, then the delimiter that closes the chunk;
 *   - delimiters and unmerged tokens have size 1; log is the natural log;
 *   - the query attends to every row of the merged cache (no mask).
 *
 * Pins: tests/test_oracle_*.py (brute force, a second token-major formulation,
 * closed-form angle cases, invariants, textbook softmax attention).  Accuracy
 * tables of the paper need its datasets and weights: parity unpinned for those.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/* ---------------------------------------------------------------- Eq. 1 ---
 * mask[0..n): nonzero = delimiter.  The sequence becomes
 * (C_1, d_1, C_2, ..., d_{M-1}, C_M) with M = #delimiters + 1.
 * Encoding: off[0] = 0, off[m+1] = position(d_{m+1}) + 1, off[M] = n + 1, so
 * chunk m (0-based) holds positions [off[m], off[m+1]-1) and its closing
 * delimiter, if any, sits at off[m+1]-1 (< n).
 * offsets must have room for n+2 entries.  Returns M.
 */
int32_t sc_oracle_segment(const uint8_t *mask, int32_t n, int32_t *offsets)
{
    int32_t m = 0;
    offsets[0] = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (mask[i] != 0) {
            m += 1;
            offsets[m] = i + 1;
        }
    }
    m += 1;
    offsets[m] = n + 1;
    return m;
}

/* ---------------------------------------------------------------- Eq. 2 --- */
double sc_oracle_cosine(const double *a, const double *b, int32_t d)
{
    double dot = 0.0, aa = 0.0, bb = 0.0;
    for (int32_t e = 0; e < d; ++e) {
        dot += a[e] * b[e];
        aa += a[e] * a[e];
        bb += b[e] * b[e];
    }
    return dot / (sqrt(aa) * sqrt(bb));
}

/* --------------------------------------------------------------- Alg. 1 ---
 * One chunk of l key rows (row stride ld doubles).  cid[j] receives the index
 * of the cluster token j belongs to; clusters are numbered in the order their
 * seeds are met (ascending seed position).  Returns the number of clusters p.
 * Optional outputs: *min_margin = min |Sim - tau| over every evaluated pair
 * (+inf if none), *n_pairs += number of evaluated pairs.
 */
int32_t sc_oracle_gsc_chunk(const double *K, int64_t ld, int32_t l, int32_t d, double tau,
                            int32_t *cid, double *min_margin, int64_t *n_pairs)
{
    int32_t p = 0;
    double margin = INFINITY;
    int64_t pairs = 0;
    unsigned char *assigned = (unsigned char *)calloc((size_t)(l > 0 ? l : 1), 1);
    for (int32_t i = 0; i < l; ++i) {
        if (!assigned[i]) {
            const double *seed = K + (int64_t)i * ld;
            cid[i] = p;
            assigned[i] = 1;
            for (int32_t j = i + 1; j < l; ++j) {
                if (!assigned[j]) {
                    double s = sc_oracle_cosine(seed, K + (int64_t)j * ld, d);
                    double gap = fabs(s - tau);
                    pairs += 1;
                    if (gap < margin) margin = gap;   /* NaN never lowers the margin */
                    if (s > tau) {
                        cid[j] = p;
                        assigned[j] = 1;
                    }
                }
            }
            p += 1;
        }
    }
    free(assigned);
    if (min_margin) *min_margin = margin;
    if (n_pairs) *n_pairs += pairs;
    return p;
}

/* ---------------------------------------------------------------- Eq. 3 ---
 * One (sequence, KV head): K, V are [n][d] fp64 rows; off[0..M] from
 * sc_oracle_segment.  For every chunk: Alg. 1, then each cluster's mean key
 * and mean value become one output row with counts = |S_t|; the chunk's
 * closing delimiter follows, copied unchanged with count 1.
 * Outputs: Kc, Vc [cap][d], counts [cap], cid [n] (cluster index inside its
 * chunk; -1 for delimiters), chunk_margin [M] (nullable; min |Sim - tau| per
 * chunk), *n_pairs (nullable, accumulated).
 * Returns N' (rows produced); rows beyond cap are counted but not stored.
 */
int64_t sc_oracle_compress_head(const double *K, const double *V, int32_t n, int32_t d,
                                const int32_t *off, int32_t M, double tau,
                                double *Kc, double *Vc, int32_t *counts, int64_t cap,
                                int32_t *cid, double *chunk_margin, int64_t *n_pairs)
{
    int64_t row = 0;
    for (int32_t m = 0; m < M; ++m) {
        int32_t start = off[m];
        int32_t l = off[m + 1] - 1 - start;
        double margin = INFINITY;
        int32_t p = sc_oracle_gsc_chunk(K + (int64_t)start * d, d, l, d, tau, cid + start, &margin, n_pairs);
        if (chunk_margin) chunk_margin[m] = margin;
        for (int32_t t = 0; t < p; ++t) {
            if (row < cap) {
                double *kc = Kc + row * d, *vc = Vc + row * d;
                int32_t size = 0;
                for (int32_t e = 0; e < d; ++e) { kc[e] = 0.0; vc[e] = 0.0; }
                for (int32_t j = 0; j < l; ++j) {
                    if (cid[start + j] == t) {
                        const double *k = K + (int64_t)(start + j) * d;
                        const double *v = V + (int64_t)(start + j) * d;
                        for (int32_t e = 0; e < d; ++e) { kc[e] += k[e]; vc[e] += v[e]; }
                        size += 1;
                    }
                }
                for (int32_t e = 0; e < d; ++e) { kc[e] /= (double)size; vc[e] /= (double)size; }
                counts[row] = size;
            }
            row += 1;
        }
        int32_t delim = off[m + 1] - 1;
        if (delim < n) {
            if (row < cap) {
                for (int32_t e = 0; e < d; ++e) {
                    Kc[row * d + e] = K[(int64_t)delim * d + e];
                    Vc[row * d + e] = V[(int64_t)delim * d + e];
                }
                counts[row] = 1;
            }
            cid[delim] = -1;
            row += 1;
        }
    }
    return row;
}

/* ---------------------------------------------------------------- Eq. 4 ---
 * One query row q[d] against a merged cache of nrows rows:
 *   z_t = q.k_t * scale + ln(s_t);  out = softmax(z) V.
 * nrows == 0 gives out = 0 and lse = -inf.
 */
void sc_oracle_decode_head(const double *q, const double *Kc, const double *Vc, const int32_t *counts,
                           int64_t nrows, int32_t d, double scale, double *out, double *lse)
{
    for (int32_t e = 0; e < d; ++e) out[e] = 0.0;
    if (nrows <= 0) {
        if (lse) *lse = -INFINITY;
        return;
    }
    double *z = (double *)malloc(sizeof(double) * (size_t)nrows);
    double zmax = -INFINITY;
    for (int64_t t = 0; t < nrows; ++t) {
        double dot = 0.0;
        for (int32_t e = 0; e < d; ++e) dot += q[e] * Kc[t * d + e];
        z[t] = dot * scale + log((double)counts[t]);
        if (z[t] > zmax) zmax = z[t];
    }
    double denom = 0.0;
    for (int64_t t = 0; t < nrows; ++t) {
        double w = exp(z[t] - zmax);
        denom += w;
        for (int32_t e = 0; e < d; ++e) out[e] += w * Vc[t * d + e];
    }
    for (int32_t e = 0; e < d; ++e) out[e] /= denom;
    if (lse) *lse = zmax + log(denom);
    free(z);
}
