/*
 * CPU oracle for the brute-force Euclidean-distance epsilon self-join.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file; it exists so
 * that the HIP kernels can be checked against a plain, slow, obviously correct evaluation of
 * the definition.  It shares no code, header, table or helper with the HIP path.
 *
 * What it computes (paper Section 2.1, Eq. 1, first line; Section 2.2.1 "Scenario 1"):
 *   dist(p_i, p_j)^2 = sum_{k=1..d} (p_{i,k} - p_{j,k})^2      evaluated in FP64
 *   the self-join returns every pair whose distance is <= epsilon.
 * The inputs are the FP16 bit patterns the GPU path receives; each is decoded exactly to a
 * double, so every difference and every square below is exact in FP64 and only the d-term sum
 * rounds (relative error <= d * 2^-53).  The expansion s_i + s_j - 2 a_ij (Eq. 1, second line;
 * Section 3.1, Steps 1-3) is what the GPU path uses; the oracle deliberately does not.
 *
 * Readings where the paper is silent: "<=" is taken on squared values (D2 <= eps^2 with
 * eps^2 formed in FP64 from the FP32 epsilon); the result lists each unordered pair once
 * (i < j) plus every self pair (i, i) -- the paper's |R| counts self pairs and both orders
 * (Section 4.1.3, S = (|R| - |D|) / |D|), i.e. |R| = 2 * #(i<j) + |D|.
 *
 * Plain loops; OpenMP only spreads the outer loop over cores.  No blocking, no reordering.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE 754 binary16 -> double, written out from the format definition:
 * 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits; exponent 0 = subnormal
 * (value = fraction * 2^-24), exponent 31 = Inf/NaN. */
double orc_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);
    return sign ? -v : v;
}

/* Decode an n x d block (row stride ld elements) into a dense n x d double array.
 * Returns 0, or -1 if any element is Inf or NaN (rejected: the method assumes finite data). */
int orc_decode(const uint16_t *X, int64_t n, int32_t d, int64_t ld, double *P)
{
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < n; ++i)
        for (int32_t k = 0; k < d; ++k) {
            double v = orc_half_to_double(X[i * ld + k]);
            if (!isfinite(v))
                bad |= 1;
            P[i * (int64_t)d + k] = v;
        }
    return bad ? -1 : 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. 1, first line, squared: sum_k (p_ik - p_jk)^2. */
static inline double dist2_rows(const double *a, const double *b, int32_t d)
{
    double acc = 0.0;
    for (int32_t k = 0; k < d; ++k) {
        double t = a[k] - b[k];
        acc += t * t;
    }
    return acc;
}

double orc_dist2(const double *P, int32_t d, int64_t i, int64_t j)
{
    return dist2_rows(P + i * (int64_t)d, P + j * (int64_t)d, d);
}

/* Step 1 of Section 3.1: s_i = sum_k p_ik^2 (FP64 here). */
void orc_norms(const double *P, int64_t n, int32_t d, double *s)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (int32_t k = 0; k < d; ++k)
            acc += P[i * (int64_t)d + k] * P[i * (int64_t)d + k];
        s[i] = acc;
    }
}

/* Dense rows x cols block of squared distances: out[r * cols + c] = D2(i0 + r, j0 + c). */
void orc_dist2_block(const double *P, int32_t d, int64_t i0, int32_t rows, int64_t j0, int32_t cols, double *out)
{
#pragma omp parallel for schedule(static)
    for (int32_t r = 0; r < rows; ++r)
        for (int32_t c = 0; c < cols; ++c)
            out[(int64_t)r * cols + c] = dist2_rows(P + (i0 + r) * (int64_t)d, P + (j0 + c) * (int64_t)d, d);
}

/* All m(m-1)/2 squared distances of a point set, in (i, j>i) order; used to pick epsilon. */
void orc_all_pairs_dist2(const double *P, int64_t m, int32_t d, double *out)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < m; ++i) {
        /* pairs (i, j>i) start after sum_{t<i} (m-1-t) entries */
        int64_t base = i * (m - 1) - i * (i - 1) / 2;
        for (int64_t j = i + 1; j < m; ++j)
            out[base + (j - i - 1)] = dist2_rows(P + i * (int64_t)d, P + j * (int64_t)d, d);
    }
}

/* Neighbour counts: counts[i] = #{ j != i : D2(i,j) <= eps2 }.  Returns #{ i<j : D2 <= eps2 }.
 * Every ordered pair is evaluated on its own (no use of symmetry), so the counts are a
 * direct reading of the definition. */
int64_t orc_selfjoin_count(const double *P, int64_t n, int32_t d, double eps2, uint32_t *counts)
{
    int64_t twice = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : twice)
    for (int64_t i = 0; i < n; ++i) {
        uint32_t c = 0;
        for (int64_t j = 0; j < n; ++j)
            if (j != i && dist2_rows(P + i * (int64_t)d, P + j * (int64_t)d, d) <= eps2)
                ++c;
        if (counts)
            counts[i] = c;
        twice += c;
    }
    return twice / 2;
}

/* Result set: every (i, i) and every (i, j), i < j, with D2 <= eps2, sorted by (i, j).
 * Pass 1 sizes each row, pass 2 fills; returns the number of pairs found (which may exceed
 * `capacity`, in which case only the first `capacity` in sorted order are written).
 * row_start must hold n + 1 entries (scratch / output: CSR offsets by i). */
int64_t orc_selfjoin_pairs(const double *P, int64_t n, int32_t d, double eps2, uint32_t *pairs, double *d2out,
                           int64_t capacity, int64_t *row_start)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; ++i) {
        int64_t c = 1; /* the self pair: D2(i,i) = 0 <= eps2 for every eps */
        for (int64_t j = i + 1; j < n; ++j)
            if (dist2_rows(P + i * (int64_t)d, P + j * (int64_t)d, d) <= eps2)
                ++c;
        row_start[i + 1] = c;
    }
    row_start[0] = 0;
    for (int64_t i = 0; i < n; ++i)
        row_start[i + 1] += row_start[i];
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; ++i) {
        int64_t pos = row_start[i];
        for (int64_t j = i; j < n; ++j) {
            double v = dist2_rows(P + i * (int64_t)d, P + j * (int64_t)d, d);
            if (v <= eps2) {
                if (pos < capacity) {
                    pairs[2 * pos] = (uint32_t)i;
                    pairs[2 * pos + 1] = (uint32_t)j;
                    if (d2out)
                        d2out[pos] = v;
                }
                ++pos;
            }
        }
    }
    return row_start[n];
}

/* Neighbour lists of selected query rows against the whole data set.
 * For query q = rows[r]: every j != q with D2(q, j) <= eps2, ascending j.
 * Call with nbr == NULL to size (fills row_start[0..R]); then again to fill.
 * Also returns, per query row, the D2 of each neighbour when d2out != NULL. */
int64_t orc_rows_join(const double *P, int64_t n, int32_t d, double eps2, const int64_t *rows, int64_t R,
                      int64_t *row_start, uint32_t *nbr, double *d2out)
{
    if (!nbr) {
#pragma omp parallel for schedule(dynamic, 4)
        for (int64_t r = 0; r < R; ++r) {
            int64_t q = rows[r], c = 0;
            for (int64_t j = 0; j < n; ++j)
                if (j != q && dist2_rows(P + q * (int64_t)d, P + j * (int64_t)d, d) <= eps2)
                    ++c;
            row_start[r + 1] = c;
        }
        row_start[0] = 0;
        for (int64_t r = 0; r < R; ++r)
            row_start[r + 1] += row_start[r];
        return row_start[R];
    }
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t r = 0; r < R; ++r) {
        int64_t q = rows[r], pos = row_start[r];
        for (int64_t j = 0; j < n; ++j) {
            if (j == q)
                continue;
            double v = dist2_rows(P + q * (int64_t)d, P + j * (int64_t)d, d);
            if (v <= eps2) {
                nbr[pos] = (uint32_t)j;
                if (d2out)
                    d2out[pos] = v;
                ++pos;
            }
        }
    }
    return row_start[R];
}

/* ------------------------------------------------------------------------------------------------
 * Two-set join: "points" P (np x d) against "query points" Q (nq x d) -- the general form of the
 * distance computation of Section 3.1 (fragments of points and of query points), of which the
 * self-join is the case P = Q.  Result: every (i, j), i < np, j < nq, with D2(p_i, q_j) <= eps2,
 * sorted by (i, j).  No symmetry, no self pairs: P and Q are different sets even when they hold
 * equal points.
 * ------------------------------------------------------------------------------------------------ */

/* counts_p[i] = #{ j : D2(p_i, q_j) <= eps2 }, counts_q[j] likewise (either may be NULL). Returns the total. */
int64_t orc_join_count(const double *P, int64_t np, const double *Q, int64_t nq, int32_t d, double eps2,
                       uint32_t *counts_p, uint32_t *counts_q)
{
    int64_t total = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : total)
    for (int64_t i = 0; i < np; ++i) {
        uint32_t c = 0;
        for (int64_t j = 0; j < nq; ++j)
            if (dist2_rows(P + i * (int64_t)d, Q + j * (int64_t)d, d) <= eps2)
                ++c;
        if (counts_p)
            counts_p[i] = c;
        total += c;
    }
    if (counts_q) {
#pragma omp parallel for schedule(dynamic, 64)
        for (int64_t j = 0; j < nq; ++j) {
            uint32_t c = 0;
            for (int64_t i = 0; i < np; ++i)
                if (dist2_rows(P + i * (int64_t)d, Q + j * (int64_t)d, d) <= eps2)
                    ++c;
            counts_q[j] = c;
        }
    }
    return total;
}

/* Pair list, sorted by (i, j); two passes like orc_selfjoin_pairs. row_start holds np + 1 entries. */
int64_t orc_join_pairs(const double *P, int64_t np, const double *Q, int64_t nq, int32_t d, double eps2,
                       uint32_t *pairs, double *d2out, int64_t capacity, int64_t *row_start)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < np; ++i) {
        int64_t c = 0;
        for (int64_t j = 0; j < nq; ++j)
            if (dist2_rows(P + i * (int64_t)d, Q + j * (int64_t)d, d) <= eps2)
                ++c;
        row_start[i + 1] = c;
    }
    row_start[0] = 0;
    for (int64_t i = 0; i < np; ++i)
        row_start[i + 1] += row_start[i];
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < np; ++i) {
        int64_t pos = row_start[i];
        for (int64_t j = 0; j < nq; ++j) {
            double v = dist2_rows(P + i * (int64_t)d, Q + j * (int64_t)d, d);
            if (v <= eps2) {
                if (pos < capacity) {
                    pairs[2 * pos] = (uint32_t)i;
                    pairs[2 * pos + 1] = (uint32_t)j;
                    if (d2out)
                        d2out[pos] = v;
                }
                ++pos;
            }
        }
    }
    return row_start[np];
}

/* Dense block between the two sets: out[r * cols + c] = D2(p_{i0+r}, q_{j0+c}). */
void orc_dist2_block2(const double *P, const double *Q, int32_t d, int64_t i0, int32_t rows, int64_t j0, int32_t cols,
                      double *out)
{
#pragma omp parallel for schedule(static)
    for (int32_t r = 0; r < rows; ++r)
        for (int32_t c = 0; c < cols; ++c)
            out[(int64_t)r * cols + c] = dist2_rows(P + (i0 + r) * (int64_t)d, Q + (j0 + c) * (int64_t)d, d);
}
