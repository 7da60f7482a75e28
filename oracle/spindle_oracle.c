/*
 * CPU oracle for the SpindleKV prefill-time KV reduction pass.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, double-precision C written from the
 * paper's equations; it shares no code, tables or helpers with the HIP path
 * and must never be called from the product path.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may load it.
 *
 * All inputs are double arrays holding the exact values of the fp16 / bf16 /
 * fp32 device tensors.  Every function works on ONE independent problem
 * ("unit"): one (batch, kv-head) for the eviction path, one
 * (batch, kv-head, K-or-V) for the codebook path.
 *
 * Readings taken where the paper is silent or garbled are marked READING.
 */
#define _GNU_SOURCE
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Eviction path (Sec. "Attention Weight Based Token Eviction")        */
/* ------------------------------------------------------------------ */

/*
 * Group-averaged accumulated window attention, Eq. (1)-(3).
 *   Q   [hn][lw][d]  window queries of the hn query heads sharing this KV head;
 *                    window row b sits at sequence position l - lw + b
 *   K   [l][d]       cached keys
 *   out [l - lw]     ac'_a for the context tokens a < l_c = l - lw
 * Eq. (1): A = softmax(mask(Q K^T * scale)), causal mask: key a visible to the
 *          query at position p iff a <= p.
 * Eq. (2): ac_{g,a} = (sum over the lw window queries of A[query][a]) / (l - a).
 *          READING: in A_{i,a,b} the index a is the key token and b the query.
 *          norm_mode 1 drops the divisor (plain window sum).
 * Eq. (3): ac'_a = (1/hn) sum_{g=0}^{hn-1} ac_{g,a}
 *          READING: the printed upper limit hn is taken as hn-1 and the printed
 *          divisor (n - a) as (l - a).
 */
int oracle_deep_scores(const double *Q, const double *K, int hn, int lw, int l, int d,
                       double scale, int norm_mode, double *out)
{
    int lc = l - lw;
    if (lc < 0) return -1;
    double *s = (double *)malloc(sizeof(double) * (size_t)(l > 0 ? l : 1));
    double *acc = (double *)malloc(sizeof(double) * (size_t)(lc > 0 ? lc : 1));
    if (!s || !acc) { free(s); free(acc); return -2; }
    for (int a = 0; a < lc; ++a) out[a] = 0.0;
    for (int g = 0; g < hn; ++g) {
        for (int a = 0; a < lc; ++a) acc[a] = 0.0;
        for (int b = 0; b < lw; ++b) {
            const double *q = Q + ((size_t)g * lw + b) * d;
            int p = lc + b;                       /* position of this query */
            double M = -INFINITY;
            for (int a = 0; a <= p; ++a) {
                const double *k = K + (size_t)a * d;
                double dot = 0.0;
                for (int t = 0; t < d; ++t) dot += q[t] * k[t];
                s[a] = dot * scale;
                if (s[a] > M) M = s[a];
            }
            double Z = 0.0;
            for (int a = 0; a <= p; ++a) Z += exp(s[a] - M);
            for (int a = 0; a < lc; ++a) acc[a] += exp(s[a] - M) / Z;
        }
        for (int a = 0; a < lc; ++a) {
            double v = acc[a];
            if (norm_mode == 0) v /= (double)(l - a);
            out[a] += v;
        }
    }
    for (int a = 0; a < lc; ++a) out[a] /= (double)hn;
    free(s); free(acc);
    return 0;
}

/*
 * READING (the paper only says it follows SnapKV): 1-D max pooling of the
 * context scores, odd kernel P, stride 1, same length, neighbours outside
 * [0, n) ignored.  P = 1 is the identity.
 */
void oracle_maxpool(const double *x, int n, int P, double *out)
{
    int r = (P - 1) / 2;
    for (int a = 0; a < n; ++a) {
        double m = x[a];
        for (int j = a - r; j <= a + r; ++j)
            if (j >= 0 && j < n && x[j] > m) m = x[j];
        out[a] = m;
    }
}

static int cmp_desc_then_index(const void *pa, const void *pb, void *key)
{
    const double *p = (const double *)key;
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    if (p[a] > p[b]) return -1;
    if (p[a] < p[b]) return 1;
    return (a > b) - (a < b);
}
static int cmp_int(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/*
 * Eq. (7): eta = argTopK(p, k).  READING: equal scores are taken lowest index
 * first; the selection is returned in ascending position order.
 */
void oracle_topk(const double *p, int n, int k, int32_t *idx_out)
{
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    for (int a = 0; a < n; ++a) order[a] = a;
    qsort_r(order, (size_t)n, sizeof(int32_t), cmp_desc_then_index, (void *)p);
    for (int j = 0; j < k; ++j) idx_out[j] = order[j];
    qsort(idx_out, (size_t)k, sizeof(int32_t), cmp_int);
    free(order);
}

/*
 * Whole eviction step for one unit: scores -> pool -> top-k of the context,
 * then every window token is kept (Sec. "Attention Weight Based Token
 * Eviction": the observation window is reserved in full).
 * READING: `budget` counts the window, so k = budget - lw context tokens;
 * budget >= l keeps everything.
 *   pooled [l - lw]   pooled scores (output)
 *   kept   [min(budget, l)] ascending positions (output)
 * returns the number of kept tokens, or < 0 on error.
 */
int oracle_deep_unit(const double *Q, const double *K, int hn, int lw, int l, int d,
                     double scale, int norm_mode, int P, int budget,
                     double *pooled, int32_t *kept)
{
    int lc = l - lw;
    if (budget < lw || lc < 0) return -1;
    double *ac = (double *)malloc(sizeof(double) * (size_t)(lc > 0 ? lc : 1));
    int rc = oracle_deep_scores(Q, K, hn, lw, l, d, scale, norm_mode, ac);
    if (rc) { free(ac); return rc; }
    oracle_maxpool(ac, lc, P, pooled);
    free(ac);
    int k = budget - lw;
    if (k > lc) k = lc;
    oracle_topk(pooled, lc, k, kept);
    for (int b = 0; b < lw; ++b) kept[k + b] = lc + b;
    return k + lw;
}

/* ------------------------------------------------------------------ */
/* Codebook path (Sec. "Similarity Based Token Replacement", Alg. 1)   */
/* ------------------------------------------------------------------ */

#define WORDS(n) (((n) + 31) / 32)
#define GETBIT(row, b) (((row)[(b) >> 5] >> ((b) & 31)) & 1u)
#define SETBIT(row, b) ((row)[(b) >> 5] |= (1u << ((b) & 31)))

/* Eq. (8): m_a = sqrt(x_a . x_a), summed in index order. */
void oracle_magnitudes(const double *X, int n, int d, double *m)
{
    for (int a = 0; a < n; ++a) {
        const double *x = X + (size_t)a * d;
        double ss = 0.0;
        for (int t = 0; t < d; ++t) ss += x[t] * x[t];
        m[a] = sqrt(ss);
    }
}

/* Eq. (4): cosine similarity of two tokens; READING: 0 if either is the zero vector. */
double oracle_cos(const double *X, const double *m, int d, int a, int b)
{
    const double *x = X + (size_t)a * d, *y = X + (size_t)b * d;
    double dot = 0.0;
    for (int t = 0; t < d; ++t) dot += x[t] * y[t];
    double den = m[a] * m[b];
    return den > 0.0 ? dot / den : 0.0;
}

/*
 * Eq. (9) and (10): G_ab = [S_ab > theta] (strict), bit-packed rows of
 * WORDS(n) 32-bit words, bit b of row a at word b/32, position b%32;
 * deg_a = sum_b G_ab.  READING: the diagonal is 1 (cos(x,x) = 1 > theta) even
 * for a zero vector, so every token is at least its own neighbour.
 */
void oracle_adjacency(const double *X, const double *m, int n, int d, double theta,
                      uint32_t *G, int32_t *deg)
{
    int W = WORDS(n);
    memset(G, 0, sizeof(uint32_t) * (size_t)n * W);
    for (int a = 0; a < n; ++a) {
        SETBIT(G + (size_t)a * W, a);
        for (int b = a + 1; b < n; ++b) {
            if (oracle_cos(X, m, d, a, b) > theta) {
                SETBIT(G + (size_t)a * W, b);
                SETBIT(G + (size_t)b * W, a);
            }
        }
    }
    for (int a = 0; a < n; ++a) {
        int c = 0;
        for (int w = 0; w < W; ++w) c += __builtin_popcount(G[(size_t)a * W + w]);
        deg[a] = c;
    }
}

/* One row of G only (for spot checks at sizes where the full matrix is too slow). */
void oracle_adjacency_row(const double *X, const double *m, int n, int d, double theta,
                          int a, uint32_t *row)
{
    int W = WORDS(n);
    memset(row, 0, sizeof(uint32_t) * (size_t)W);
    for (int b = 0; b < n; ++b)
        if (b == a || oracle_cos(X, m, d, a, b) > theta) SETBIT(row, b);
}

/*
 * The loop of Alg. 1 exactly as the paper states it, on a private copy of G:
 *   repeat until G == 0:
 *     s    = row sums of G                 (Eq. 10; READING: the listing prints
 *                                           the sum over S, which the loop never
 *                                           changes - the degree of G is meant)
 *     iota = argmax s                      (Eq. 11; READING: lowest index on ties)
 *     C   += [token iota]
 *     r[argwhere(G_iota)] = |C| - 1        (Eq. 12)
 *     G   &= outer(not G_iota, not G_iota) (Eq. 13: clears every row and column
 *                                           of iota's neighbourhood)
 * picks[c] = token index of codebook entry c; ref[a] = entry of token a.
 * Returns |C|.  O(|C| n^2 / 32): for small n only.
 */
int oracle_merge_literal(const uint32_t *G_in, int n, int32_t *picks, int32_t *ref)
{
    int W = WORDS(n);
    uint32_t *G = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n * W + 4);
    uint32_t *row = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)W + 4);
    memcpy(G, G_in, sizeof(uint32_t) * (size_t)n * W);
    for (int a = 0; a < n; ++a) ref[a] = -1;
    int nc = 0;
    for (;;) {
        int best = -1, bestdeg = 0;
        for (int a = 0; a < n; ++a) {
            int c = 0;
            for (int w = 0; w < W; ++w) c += __builtin_popcount(G[(size_t)a * W + w]);
            if (c > bestdeg) { bestdeg = c; best = a; }
        }
        if (best < 0) break;                      /* G == 0 */
        memcpy(row, G + (size_t)best * W, sizeof(uint32_t) * (size_t)W);
        picks[nc] = best;
        for (int b = 0; b < n; ++b) if (GETBIT(row, b)) ref[b] = nc;
        ++nc;
        for (int a = 0; a < n; ++a) {
            uint32_t *ga = G + (size_t)a * W;
            if (GETBIT(row, a)) { for (int w = 0; w < W; ++w) ga[w] = 0; }
            else                { for (int w = 0; w < W; ++w) ga[w] &= ~row[w]; }
        }
    }
    free(G); free(row);
    return nc;
}

/*
 * Same result as oracle_merge_literal, without rewriting G: tokens removed by
 * Eq. (13) are tracked in `alive`, and the degrees of the survivors are
 * decremented for every neighbour that was removed.  Used at sizes where the
 * literal form is too slow; the tests require both to agree on small inputs.
 */
int oracle_merge_incremental(const uint32_t *G, int n, int32_t *picks, int32_t *ref)
{
    int W = WORDS(n);
    int32_t *deg = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    uint8_t *alive = (uint8_t *)malloc((size_t)(n + 1));
    int32_t *dying = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    for (int a = 0; a < n; ++a) {
        int c = 0;
        for (int w = 0; w < W; ++w) c += __builtin_popcount(G[(size_t)a * W + w]);
        deg[a] = c; alive[a] = 1; ref[a] = -1;
    }
    int nc = 0, remaining = n;
    while (remaining > 0) {
        int best = -1, bestdeg = 0;
        for (int a = 0; a < n; ++a)
            if (alive[a] && deg[a] > bestdeg) { bestdeg = deg[a]; best = a; }
        const uint32_t *row = G + (size_t)best * W;
        picks[nc] = best;
        int nd = 0;
        for (int b = 0; b < n; ++b)
            if (alive[b] && GETBIT(row, b)) { ref[b] = nc; dying[nd++] = b; }
        ++nc;
        for (int j = 0; j < nd; ++j) alive[dying[j]] = 0;
        remaining -= nd;
        for (int j = 0; j < nd; ++j) {
            const uint32_t *rb = G + (size_t)dying[j] * W;
            for (int w = 0; w < W; ++w) {
                uint32_t bits = rb[w];
                while (bits) {
                    int t = __builtin_ctz(bits); bits &= bits - 1;
                    int v = w * 32 + t;
                    if (alive[v]) deg[v]--;
                }
            }
        }
    }
    free(deg); free(alive); free(dying);
    return nc;
}

/*
 * READING (the paper's codebook size is an outcome of theta; the benchmark
 * configurations bound it): keep the first `cap` entries in pick order; a token
 * whose entry was dropped is re-pointed to the kept entry of highest cosine
 * similarity (Eq. 4), lowest entry index on ties.
 * Returns the number of re-pointed tokens.
 */
int oracle_cap_assign(const double *X, const double *m, int n, int d,
                      const int32_t *picks, int n_codes, int cap, int32_t *ref)
{
    if (n_codes <= cap) return 0;
    int moved = 0;
    for (int a = 0; a < n; ++a) {
        if (ref[a] < cap) continue;
        int best = 0; double bv = -INFINITY;
        for (int j = 0; j < cap; ++j) {
            double c = oracle_cos(X, m, d, a, picks[j]);
            if (c > bv) { bv = c; best = j; }
        }
        ref[a] = best; ++moved;
    }
    return moved;
}

/*
 * Codebook entries (Eq. 11 with the normalisation of Eq. 8): entry c is the
 * picked token's unit vector x / m; no averaging over its members.
 * READING: a zero vector yields a zero entry.
 */
void oracle_codebook(const double *X, const double *m, int d, const int32_t *picks,
                     int n_keep, double *C)
{
    for (int c = 0; c < n_keep; ++c) {
        const double *x = X + (size_t)picks[c] * d;
        double mm = m[picks[c]];
        for (int t = 0; t < d; ++t) C[(size_t)c * d + t] = mm > 0.0 ? x[t] / mm : 0.0;
    }
}

/*
 * Whole codebook step for one unit (Alg. 1 + the cap reading).
 *   mag [n], G [n][WORDS(n)], deg [n], picks [n], ref [n], C [min(cap,n)][d]
 * literal != 0 selects the literal loop.  Returns the uncapped |C|; the number
 * of stored entries is min(|C|, cap).
 */
int oracle_shallow_unit(const double *X, int n, int d, double theta, int cap, int literal,
                        double *mag, uint32_t *G, int32_t *deg, int32_t *picks,
                        int32_t *ref, double *C)
{
    oracle_magnitudes(X, n, d, mag);
    oracle_adjacency(X, mag, n, d, theta, G, deg);
    int nc = literal ? oracle_merge_literal(G, n, picks, ref)
                     : oracle_merge_incremental(G, n, picks, ref);
    oracle_cap_assign(X, mag, n, d, picks, nc, cap, ref);
    oracle_codebook(X, mag, d, picks, nc < cap ? nc : cap, C);
    return nc;
}

/*
 * Decode-time merge (Sec. "Similarity Based Token Replacement", the paragraph after
 * Eq. 14): tokens generated after the prefill first look for a codebook entry to merge
 * with, with theta as the threshold; the tokens that find none get a codebook of their
 * own by the same construction (Alg. 1), appended to the existing one.
 *   X [m][d] new tokens, C_in [nc][d] the stored entries as they are stored (unit
 *   vectors up to the rounding of their storage type).
 * READINGS: an entry c suits token a if cos(x_a, C_c) > theta (strict, as Eq. 9), with the
 * cosine of Eq. 4 taken between the raw token and the stored row, the row's own norm in
 * the denominator; among several suitable entries the one of highest cosine is taken,
 * lowest index on ties.  Alg. 1 runs on the unmatched tokens in their original order; its
 * entries get the indices nc, nc + 1, ... in pick order.  Entries that do not fit into
 * `cap` rows are not stored and their tokens keep ref = -1; the return value (entries
 * needed in total) tells the caller.
 *   mag [m], ref [m], C_new [m][d] (rows actually stored: min(picks, max(cap - nc, 0))),
 *   *n_matched = tokens that merged with an existing entry.
 * Returns nc + number of new picks.
 */
int oracle_decode_merge(const double *X, int m, int d, const double *C_in, int nc, double theta,
                        int cap, int literal, double *mag, int32_t *ref, double *C_new, int32_t *n_matched)
{
    double *cn = (double *)malloc(sizeof(double) * (size_t)(nc + 1));
    oracle_magnitudes(X, m, d, mag);
    oracle_magnitudes(C_in, nc, d, cn);
    int32_t *rest = (int32_t *)malloc(sizeof(int32_t) * (size_t)(m + 1));
    int nr = 0, matched = 0;
    for (int a = 0; a < m; ++a) {
        const double *x = X + (size_t)a * d;
        int best = -1; double bv = -INFINITY;
        for (int c = 0; c < nc; ++c) {
            const double *y = C_in + (size_t)c * d;
            double dot = 0.0;
            for (int t = 0; t < d; ++t) dot += x[t] * y[t];
            double den = mag[a] * cn[c];
            double cs = den > 0.0 ? dot / den : 0.0;
            if (cs > theta && cs > bv) { bv = cs; best = c; }
        }
        ref[a] = best;
        if (best >= 0) ++matched; else rest[nr++] = a;
    }
    *n_matched = matched;
    int picks_n = 0;
    if (nr > 0) {
        int W = WORDS(nr);
        double *XR = (double *)malloc(sizeof(double) * (size_t)nr * d);
        double *mR = (double *)malloc(sizeof(double) * (size_t)nr);
        uint32_t *G = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)nr * W + 4);
        int32_t *deg = (int32_t *)malloc(sizeof(int32_t) * (size_t)nr);
        int32_t *picks = (int32_t *)malloc(sizeof(int32_t) * (size_t)nr);
        int32_t *rr = (int32_t *)malloc(sizeof(int32_t) * (size_t)nr);
        for (int j = 0; j < nr; ++j) memcpy(XR + (size_t)j * d, X + (size_t)rest[j] * d, sizeof(double) * (size_t)d);
        oracle_magnitudes(XR, nr, d, mR);
        oracle_adjacency(XR, mR, nr, d, theta, G, deg);
        picks_n = literal ? oracle_merge_literal(G, nr, picks, rr) : oracle_merge_incremental(G, nr, picks, rr);
        int room = cap - nc; if (room < 0) room = 0;
        for (int j = 0; j < nr; ++j) ref[rest[j]] = rr[j] < room ? nc + rr[j] : -1;
        oracle_codebook(XR, mR, d, picks, picks_n < room ? picks_n : room, C_new);
        free(XR); free(mR); free(G); free(deg); free(picks); free(rr);
    }
    free(cn); free(rest);
    return nc + picks_n;
}

/* Eq. (14): reconstruction  x~_a = C[r_a] * m_a. */
void oracle_reconstruct(const double *C, const int32_t *ref, const double *mag, int n, int d,
                        double *out)
{
    for (int a = 0; a < n; ++a)
        for (int t = 0; t < d; ++t)
            out[(size_t)a * d + t] = C[(size_t)ref[a] * d + t] * mag[a];
}

/*
 * Layer budget allocation, Eq. (5)-(6) and the unnumbered equation before them.
 *   r      total reserve ratio, l sequence length, lw window, m layers, beta
 *   rc_out [m] context retain ratio per layer
 * r_c = (r l - lw) / (l - lw); alpha = (1 + beta)/2.
 * READING: the printed 0.05 is beta; the printed second case of r_c(m-1),
 * "1 - 2 r_c", is negative for r_c > 1/2 and breaks continuity at alpha; the
 * mean-preserving value 2 r_c - 1 is used.  r_c <= beta gives a uniform r_c.
 */
void oracle_layer_ratios(double r, int l, int lw, int m, double beta, double *rc_out)
{
    double lc = (double)(l - lw);
    double rc = (r * l - lw) / lc;
    double alpha = 0.5 * (1.0 + beta);
    double r0, r1;
    if (rc <= beta)       { r0 = rc; r1 = rc; }
    else if (rc <= alpha) { r0 = 2.0 * rc - beta; r1 = beta; }
    else                  { r0 = 1.0; r1 = 2.0 * rc - 1.0; }
    for (int lam = 0; lam < m; ++lam)
        rc_out[lam] = m > 1 ? r0 + (r1 - r0) / (double)(m - 1) * lam : rc;
}

/*
 * Eq. 7: tokens kept in layer lam, k = floor(r_c(lam) * l_c) as printed, plus the window,
 * which is always kept (the budget counts it: r l = r_c l_c + l_w).  budgets_out [m].
 * READING: k is kept within [0, l_c]; Eq. 6 evaluated in doubles can leave r_c(m-1) an ulp
 * below an endpoint that is exactly 0 (beta = 0), whose floor would be -1.
 */
void oracle_layer_budgets(double r, int l, int lw, int m, double beta, int *budgets_out)
{
    double *rc = (double *)malloc(sizeof(double) * (size_t)m);
    oracle_layer_ratios(r, l, lw, m, beta, rc);
    for (int lam = 0; lam < m; ++lam) {
        int k = (int)floor(rc[lam] * (double)(l - lw));
        if (k < 0) k = 0;
        if (k > l - lw) k = l - lw;
        budgets_out[lam] = lw + k;
    }
    free(rc);
}

/*
 * Sec. "Experiments", Eq. 15: reserve ratio of one layer.  r1 = share of the tokens kept by
 * eviction, r2 = codebook entries per kept token, r3 = storage of a replaced token relative
 * to its d_h elements: one index of int_bit bits and one magnitude of mag_bit bits on top,
 * both counted in cache elements of key_bit bits.
 * READING: the printed fraction, int_bit over (key_bit + 1), is garbled; it is read as
 * (d_h + int_bit / key_bit + 1) / d_h, the "+ 1" being a magnitude as wide as a cache
 * element; a magnitude of another width (the text below the equation stores a float)
 * counts mag_bit / key_bit elements.
 * out = {r1, r2, r3, r1 r2 r3}.
 */
void oracle_reserve_ratio(double kept, double total, double entries, int dh, int int_bit, int key_bit,
                          int mag_bit, double *out)
{
    out[0] = kept / total;
    out[1] = entries / kept;
    out[2] = (dh + (double)int_bit / key_bit + (double)mag_bit / key_bit) / dh;
    out[3] = out[0] * out[1] * out[2];
}
