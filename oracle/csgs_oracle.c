/*
 * CPU oracle for one partition's sampled GCN layer step with skewed
 * layer-wise neighbor sampling.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * statement of what the method computes.  Nothing on the product path may
 * call it; it shares no code, header, table or helper with the HIP library.
 * Only the tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * Every function follows the paper's steps in the paper's order:
 *   - neighbor importance weight  ||w_*j||^2 = sum_{i in S_l} w_ij^2   (Section 4.1, text after Eq. 5)
 *   - linear weighted sampling    q_j = ||w_*j||^2 / sum_k ||w_*k||^2  (Eq. 7)
 *   - skewed linear weighted sampling: local weights times s            (Section 4.2, Eq. 10)
 *   - B draws from q, inclusion probability p_j = 1 - (1 - q_j)^B      (Eq. 8)
 *   - unbiased estimator: kept edge w_ij / p_j                          (Eq. 3)
 *   - expected communication = number of sampled remote nodes           (Eq. 4)
 *   - layer:  H = P~ sigma(H_prev) W                                    (Section 3, Eq. 1)
 *
 * Readings the paper leaves open (all listed with their reasons in the design notes):
 *   - B draws are i.i.d. WITH replacement and then deduplicated: that is the one
 *     scheme whose inclusion probability is exactly Eq. 8, which makes Eq. 3 unbiased.
 *   - Weights are held as integers so that sums do not depend on summation order:
 *     wq_ij = max(1, rne(w_ij^2 * 2^shift)), the square formed exactly in double.
 *   - The skew factor is held in 1/16 units (s_fx = round(16 s); remote multiplier 16).
 *   - Candidates are ordered by ascending node id; draw t uses Philox4x32-10 with
 *     key = (seed_lo, seed_hi) and counter = (t, layer, iter_lo, iter_hi); the 64-bit word
 *     r = x0 | x1 << 32 is mapped to u = floor(r * total / 2^64) and the draw is the
 *     first candidate whose inclusive cumulative weight exceeds u.
 *   - sigma is ReLU, applied to the input rows of the aggregation (Eq. 1 puts the
 *     activation on H^(l-1); the bottom layer P X W has none).
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors, brute-force rational
 * arithmetic for q on tiny dense graphs, sum(q) = 1, s = 1 reduces Eq. 10 to Eq. 7,
 * exhaustive enumeration of all draw sequences for E[P~] = P, Monte-Carlo mean of the
 * estimator against the full aggregation, E[#remote] = sum_{j in R} p_j, chi-square
 * of the draw histogram, dense fp64 matmul for aggregation and GEMM.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL -1
#define ORC_ECAP -2
#define ORC_ERANGE -3
#define ORC_EVALUE -4
#define ORC_EEMPTY -5

/* ---------------------------------------------------------------- Philox */

/* Philox4x32 with 10 rounds as published by Salmon, Moraes, Dror and Shaw
 * (SC'11): per round, two 32x32->64 multiplies by fixed constants, a word
 * permutation with the key xored in, then the key is bumped by two Weyl
 * constants. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 64-bit random word of draw t. */
uint64_t orc_draw_word(uint64_t seed, uint64_t iter, uint32_t layer, uint32_t t)
{
    uint32_t ctr[4] = { t, layer, (uint32_t)iter, (uint32_t)(iter >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t x[4];
    orc_philox4x32_10(ctr, key, x);
    return (uint64_t)x[0] | ((uint64_t)x[1] << 32);
}

/* ------------------------------------------------- fixed-point parameters */

static int ceil_log2_u64(uint64_t n) /* smallest e with 2^e >= n, n >= 1 */
{
    int e = 0;
    while (e < 63 && ((uint64_t)1 << e) < n) ++e;
    return e;
}

/* skew in 1/16 units */
int64_t orc_skew_fx(float skew) { return (int64_t)llround((double)skew * 16.0); }

/* Number of fraction bits given to a squared edge weight, chosen so that the
 * skewed total stays below 2^63:  nS * rownorm2_max * 2^shift * s_fx <= 2^61. */
int orc_shift(int32_t nS, float skew, float rownorm2_max)
{
    int e_r = 0;
    while (e_r < 64 && ldexp(1.0, e_r) < (double)rownorm2_max) ++e_r;
    int sh = 61 - ceil_log2_u64((uint64_t)nS) - ceil_log2_u64((uint64_t)orc_skew_fx(skew)) - e_r;
    if (sh > 52) sh = 52;
    return sh;
}

/* -------------------------------------------------------- build_probs */

typedef struct {
    int64_t n_cand, n_local, n_remote, edges_scanned;
    uint64_t w_local, w_remote, total;
    int32_t shift;
    int32_t skew_fx;   /* local multiplier used, in 1/16 units; negative: remote weight was zero */
} orc_stats;

/*
 * Skew by Theorem 1 (Eq. 12): s = D (|N(S_l)| - B) / |R| + 1/2.  Readings: the text wants s > 1,
 * so smaller values are raised to 1 (s = 1 is the unskewed sampler); |R| = 0 leaves nothing to
 * skew against, s = 1; s is cut at the bound the fixed-point format was sized for and rounded
 * to 1/16 (half up).  Returns s in 1/16 units.
 */
int64_t orc_theorem1_skew_fx(int64_t n_cand, int64_t n_remote, int32_t B, double D, int64_t s_fx_max)
{
    double sk = 1.0;
    if (n_remote > 0) sk = D * (double)(n_cand - (int64_t)B) / (double)n_remote + 0.5;
    if (!(sk >= 1.0)) sk = 1.0;
    double fx = floor(sk * 16.0 + 0.5);
    if (fx > (double)s_fx_max) fx = (double)s_fx_max;
    return (int64_t)fx;
}

/*
 * Sampling distribution over N(S_l), the union of the neighbors of the nodes
 * in S (Section 4.1; the layer-wise sampler of Section 5.1 takes all neighbors
 * of the layer-l nodes as candidates).
 * out: cand_id ascending, cand_w = fixed-point ||w_*j||^2 (unskewed),
 *      cdf = inclusive running sum of the skewed weights, q = Eq. 10 as float.
 */
/*
 * mode 0: skew s given (Eq. 10).  mode 1: s from Theorem 1 with constants D, B, the fixed-point
 * format sized for `skew` as the upper bound of s.  mode 2: the "Local" version of Section 5.1,
 * remote candidates get weight zero (they stay in the list and can never be drawn).
 */
int orc_build_probs_ex(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx, const float *val,
                       int32_t local_lo, int32_t local_hi, float rownorm2_max,
                       const int32_t *S, int32_t nS, int mode, float skew, float D, int32_t B,
                       int32_t *cand_id, uint64_t *cand_w, uint64_t *cdf, float *q, int64_t cap,
                       orc_stats *st)
{
    if (mode == 2) skew = 1.0f;
    if (!rowptr || !colidx || !val || !S || !st || nS <= 0 || !(skew >= 1.0f) || skew > 1048576.0f ||
        local_lo > local_hi || !(rownorm2_max > 0.0f) || mode < 0 || mode > 2 ||
        (mode == 1 && (!(D >= 0.0f) || B <= 0)))
        return ORC_EINVAL;
    int shift = orc_shift(nS, skew, rownorm2_max);
    if (shift < 24) return ORC_ERANGE;
    uint64_t s_fx = (uint64_t)orc_skew_fx(skew);
    uint64_t s_remote = 16u;

    uint64_t *acc = (uint64_t *)calloc((size_t)n_nodes, sizeof(uint64_t));
    if (!acc) return ORC_ECAP;
    memset(st, 0, sizeof(*st));
    st->shift = shift;
    int rc = ORC_OK;

    for (int32_t a = 0; a < nS; ++a) {
        int32_t i = S[a];
        if (i < 0 || i >= n_nodes) { rc = ORC_EINVAL; goto done; }
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            double w = (double)val[e];
            if (!isfinite(w)) { rc = ORC_EVALUE; goto done; }
            double sq = w * w;                       /* exact: 24-bit x 24-bit */
            int64_t x = llrint(ldexp(sq, shift));    /* round to nearest even */
            if (x < 1) x = 1;                        /* every candidate stays drawable */
            acc[colidx[e]] += (uint64_t)x;
            st->edges_scanned++;
        }
    }
    if (mode == 1) {   /* the counts |N(S_l)| and |R| of this very candidate set choose s */
        int64_t nc = 0, nr = 0;
        for (int64_t j = 0; j < n_nodes; ++j)
            if (acc[j]) { ++nc; if (!(j >= local_lo && j < local_hi)) ++nr; }
        s_fx = (uint64_t)orc_theorem1_skew_fx(nc, nr, B, (double)D, (int64_t)s_fx);
    }
    if (mode == 2) { s_fx = 16u; s_remote = 0u; }
    st->skew_fx = (int32_t)s_fx * (s_remote ? 1 : -1);
    {
        uint64_t running = 0;
        int64_t n = 0;
        for (int64_t j = 0; j < n_nodes; ++j) {
            if (!acc[j]) continue;
            if (n >= cap) { rc = ORC_ECAP; goto done; }
            int is_local = (j >= local_lo && j < local_hi);
            uint64_t wskew = acc[j] * (is_local ? s_fx : s_remote);   /* Eq. 10 numerator */
            running += wskew;
            cand_id[n] = (int32_t)j;
            cand_w[n] = acc[j];
            cdf[n] = running;
            if (is_local) { st->n_local++; st->w_local += acc[j]; }
            else          { st->n_remote++; st->w_remote += acc[j]; }
            ++n;
        }
        st->n_cand = n;
        st->total = running;
        if (n == 0 || running == 0) { rc = ORC_EEMPTY; goto done; }
        if (q) {
            uint64_t prev = 0;
            for (int64_t k = 0; k < n; ++k) {
                q[k] = (float)((double)(cdf[k] - prev) / (double)running);
                prev = cdf[k];
            }
        }
    }
done:
    free(acc);
    return rc;
}

int orc_build_probs(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx, const float *val,
                    int32_t local_lo, int32_t local_hi, float rownorm2_max,
                    const int32_t *S, int32_t nS, float skew,
                    int32_t *cand_id, uint64_t *cand_w, uint64_t *cdf, float *q, int64_t cap,
                    orc_stats *st)
{
    const int local_only = isinf(skew) && skew > 0;
    return orc_build_probs_ex(n_nodes, rowptr, colidx, val, local_lo, local_hi, rownorm2_max, S, nS,
                              local_only ? 2 : 0, skew, 0.0f, 0, cand_id, cand_w, cdf, q, cap, st);
}

/* -------------------------------------------------------- sample_layer */

static uint64_t mulhi64(uint64_t a, uint64_t b)
{
    return (uint64_t)(((unsigned __int128)a * (unsigned __int128)b) >> 64);
}

/* first k with cdf[k] > u (cdf is non-decreasing, u < cdf[n-1]) */
static int64_t first_greater(const uint64_t *cdf, int64_t n, uint64_t u)
{
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (cdf[mid] > u) hi = mid; else lo = mid + 1;
    }
    return lo;
}

/*
 * B draws with replacement from q (Section 4.1, Eq. 8), the draws given
 * as explicit 64-bit words so that tests can enumerate them; deduplicated to the ascending node
 * set S_next with multiplicities; inclusion probability from Eq. 8 (pd in double, p_incl as float).
 */
int orc_draw_from_words(const int32_t *cand_id, const uint64_t *cdf, int64_t n_cand,
                        const uint64_t *words, int32_t B,
                        int32_t *S_next, int32_t *mult, float *p_incl, double *pd, int32_t *n_next)
{
    if (!cand_id || !cdf || n_cand <= 0 || B <= 0 || !words) return ORC_EINVAL;
    uint64_t total = cdf[n_cand - 1];
    if (total == 0) return ORC_EEMPTY;
    int32_t *cnt = (int32_t *)calloc((size_t)n_cand, sizeof(int32_t));
    if (!cnt) return ORC_ECAP;
    for (int32_t t = 0; t < B; ++t) {
        uint64_t u = mulhi64(words[t], total);
        cnt[first_greater(cdf, n_cand, u)]++;
    }
    int32_t n = 0;
    for (int64_t k = 0; k < n_cand; ++k) {
        if (!cnt[k]) continue;
        uint64_t wk = cdf[k] - (k ? cdf[k - 1] : 0);
        double qk = (double)wk / (double)total;
        double pk = (qk >= 1.0) ? 1.0 : -expm1((double)B * log1p(-qk));   /* Eq. 8 */
        S_next[n] = cand_id[k];
        mult[n] = cnt[k];
        pd[n] = pk;
        p_incl[n] = (float)pk;
        ++n;
    }
    *n_next = n;
    free(cnt);
    return ORC_OK;
}

/*
 * Sampled adjacency of Eq. 3 for an arbitrary row set: rows in the given order, columns =
 * position in S_next ascending, value w_ij / p_j.  With rows = S_l it is the layer operator P~;
 * with rows = S_next it is the sampled subgraph on which a subgraph sampler runs the full
 * convolution (Section 5.1, second sampler).
 */
int orc_sampled_adjacency(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx, const float *val,
                          const int32_t *rows, int32_t n_rows, const int32_t *S_next, int32_t n_next,
                          const double *pd, int32_t *adj_rowptr, int32_t *adj_col, float *adj_val,
                          int64_t adj_cap, int64_t *adj_nnz)
{
    if (!rows || n_rows <= 0 || !S_next || n_next < 0 || !pd) return ORC_EINVAL;
    int32_t *rank = (int32_t *)malloc((size_t)n_nodes * sizeof(int32_t));
    if (!rank) return ORC_ECAP;
    for (int64_t j = 0; j < n_nodes; ++j) rank[j] = -1;
    for (int32_t k = 0; k < n_next; ++k) rank[S_next[k]] = k;
    int rc = ORC_OK;
    int64_t nnz = 0;
    adj_rowptr[0] = 0;
    for (int32_t a = 0; a < n_rows; ++a) {
        int32_t i = rows[a];
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int32_t r = rank[colidx[e]];
            if (r < 0) continue;
            if (nnz >= adj_cap) { rc = ORC_ECAP; goto done; }
            adj_col[nnz] = r;
            adj_val[nnz] = (float)((double)val[e] / pd[r]);                /* Eq. 3 */
            ++nnz;
        }
        adj_rowptr[a + 1] = (int32_t)nnz;
    }
    *adj_nnz = nnz;
done:
    free(rank);
    return rc;
}

int orc_sample_from_words(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx, const float *val,
                          const int32_t *S, int32_t nS,
                          const int32_t *cand_id, const uint64_t *cdf, int64_t n_cand,
                          const uint64_t *words, int32_t B,
                          int32_t *S_next, int32_t *mult, float *p_incl, int32_t *n_next,
                          int32_t *adj_rowptr, int32_t *adj_col, float *adj_val, int64_t adj_cap,
                          int64_t *adj_nnz)
{
    if (B <= 0 || nS <= 0) return ORC_EINVAL;
    double *pd = (double *)malloc((size_t)B * sizeof(double));
    if (!pd) return ORC_ECAP;
    int rc = orc_draw_from_words(cand_id, cdf, n_cand, words, B, S_next, mult, p_incl, pd, n_next);
    if (rc == ORC_OK)
        rc = orc_sampled_adjacency(n_nodes, rowptr, colidx, val, S, nS, S_next, *n_next, pd, adj_rowptr, adj_col,
                                   adj_val, adj_cap, adj_nnz);
    free(pd);
    return rc;
}

/* The draws of csgs: word t from the counter-based generator. */
int orc_draw_nodes(const int32_t *cand_id, const uint64_t *cdf, int64_t n_cand, int32_t B,
                   uint64_t seed, uint64_t iter, uint32_t layer,
                   int32_t *S_next, int32_t *mult, float *p_incl, double *pd, int32_t *n_next)
{
    if (B <= 0) return ORC_EINVAL;
    uint64_t *words = (uint64_t *)malloc((size_t)B * sizeof(uint64_t));
    if (!words) return ORC_ECAP;
    for (int32_t t = 0; t < B; ++t) words[t] = orc_draw_word(seed, iter, layer, (uint32_t)t);
    int rc = orc_draw_from_words(cand_id, cdf, n_cand, words, B, S_next, mult, p_incl, pd, n_next);
    free(words);
    return rc;
}

int orc_sample_layer(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx, const float *val,
                     const int32_t *S, int32_t nS,
                     const int32_t *cand_id, const uint64_t *cdf, int64_t n_cand,
                     int32_t B, uint64_t seed, uint64_t iter, uint32_t layer,
                     int32_t *S_next, int32_t *mult, float *p_incl, int32_t *n_next,
                     int32_t *adj_rowptr, int32_t *adj_col, float *adj_val, int64_t adj_cap,
                     int64_t *adj_nnz)
{
    if (B <= 0) return ORC_EINVAL;
    uint64_t *words = (uint64_t *)malloc((size_t)B * sizeof(uint64_t));
    if (!words) return ORC_ECAP;
    for (int32_t t = 0; t < B; ++t) words[t] = orc_draw_word(seed, iter, layer, (uint32_t)t);
    int rc = orc_sample_from_words(n_nodes, rowptr, colidx, val, S, nS, cand_id, cdf, n_cand, words, B,
                                   S_next, mult, p_incl, n_next, adj_rowptr, adj_col, adj_val, adj_cap,
                                   adj_nnz);
    free(words);
    return rc;
}

/* The candidate positions of the B draws, in draw order (for histogram tests). */
int orc_draw_positions(const uint64_t *cdf, int64_t n_cand, int32_t B,
                       uint64_t seed, uint64_t iter, uint32_t layer, int64_t *pos)
{
    if (!cdf || n_cand <= 0 || B <= 0) return ORC_EINVAL;
    uint64_t total = cdf[n_cand - 1];
    for (int32_t t = 0; t < B; ++t)
        pos[t] = first_greater(cdf, n_cand, mulhi64(orc_draw_word(seed, iter, layer, (uint32_t)t), total));
    return ORC_OK;
}

/* -------------------------------------------------------- remote_count */

/*
 * Communication volume of the step (Eq. 4): sampled nodes outside [lo, hi).
 * Optional per-partition histogram over part_bounds[0..P].  Optional source-row
 * map for the bottom layer's aggregation: local node -> id - lo, remote node ->
 * -1 - (its rank among the sampled remote nodes, ascending id), with the remote
 * ids listed in remote_ids in that order.
 */
int orc_remote_count(const int32_t *S_next, int32_t n_next, int32_t lo, int32_t hi,
                     const int32_t *part_bounds, int32_t P,
                     int64_t *remote_total, int64_t *per_part, int32_t *src_row, int32_t *remote_ids)
{
    if (!S_next || n_next < 0 || lo > hi || !remote_total) return ORC_EINVAL;
    int64_t r = 0;
    if (per_part) for (int32_t p = 0; p < P; ++p) per_part[p] = 0;
    for (int32_t k = 0; k < n_next; ++k) {
        int32_t j = S_next[k];
        int local = (j >= lo && j < hi);
        if (per_part && part_bounds)
            for (int32_t p = 0; p < P; ++p)
                if (j >= part_bounds[p] && j < part_bounds[p + 1]) per_part[p]++;
        if (local) {
            if (src_row) src_row[k] = j - lo;
        } else {
            if (src_row) src_row[k] = -1 - (int32_t)r;
            if (remote_ids) remote_ids[r] = j;
            ++r;
        }
    }
    *remote_total = r;
    return ORC_OK;
}

/* -------------------------------------------------------- aggregate */

static double widen_bf16(uint16_t h)
{
    uint32_t b = (uint32_t)h << 16;
    float f;
    memcpy(&f, &b, sizeof f);
    return (double)f;
}

/*
 * Z = P~ sigma?(X_src)  (Eq. 1 with the sampled operator of Section 3).
 * Column c of P~ reads row src_row[c] of X_local when src_row[c] >= 0, row
 * -1 - src_row[c] of X_remote otherwise; with src_row == NULL column c reads row
 * c of X_local.  dtype 0 = float32, 1 = bfloat16 bit patterns (widened exactly).
 * Accumulation in double, result rounded once to float.
 */
int orc_aggregate(const int32_t *adj_rowptr, const int32_t *adj_col, const float *adj_val, int32_t nS,
                  const void *X_local, int64_t ld_local, const void *X_remote, int64_t ld_remote,
                  const int32_t *src_row, int32_t F, int dtype, int relu_on_input,
                  float *Z, int64_t ldz)
{
    if (!adj_rowptr || !X_local || !Z || nS <= 0 || F <= 0 || (dtype != 0 && dtype != 1)) return ORC_EINVAL;
    double *acc = (double *)malloc((size_t)F * sizeof(double));
    if (!acc) return ORC_ECAP;
    for (int32_t a = 0; a < nS; ++a) {
        for (int32_t f = 0; f < F; ++f) acc[f] = 0.0;
        for (int32_t e = adj_rowptr[a]; e < adj_rowptr[a + 1]; ++e) {
            int32_t c = adj_col[e];
            int64_t sr = src_row ? src_row[c] : c;
            const void *base = X_local; int64_t ld = ld_local;
            if (sr < 0) { base = X_remote; ld = ld_remote; sr = -1 - sr; }
            double w = (double)adj_val[e];
            for (int32_t f = 0; f < F; ++f) {
                double x = dtype == 0 ? (double)((const float *)base)[sr * ld + f]
                                      : widen_bf16(((const uint16_t *)base)[sr * ld + f]);
                if (relu_on_input && x < 0.0) x = 0.0;
                acc[f] += w * x;
            }
        }
        for (int32_t f = 0; f < F; ++f) Z[(int64_t)a * ldz + f] = (float)acc[f];
    }
    free(acc);
    return ORC_OK;
}

/* -------------------------------------------------------- layer_gemm */

/* H = Z W (Eq. 1), row-major, double accumulation, one rounding to float. */
int orc_layer_gemm(const float *Z, int64_t ldz, int32_t M, int32_t K, const float *W, int64_t ldw,
                   int32_t N, float *H, int64_t ldh)
{
    if (!Z || !W || !H || M <= 0 || K <= 0 || N <= 0) return ORC_EINVAL;
    double *acc = (double *)malloc((size_t)N * sizeof(double));
    if (!acc) return ORC_ECAP;
    for (int32_t m = 0; m < M; ++m) {
        for (int32_t n = 0; n < N; ++n) acc[n] = 0.0;
        for (int32_t k = 0; k < K; ++k) {
            double z = (double)Z[(int64_t)m * ldz + k];
            for (int32_t n = 0; n < N; ++n) acc[n] += z * (double)W[(int64_t)k * ldw + n];
        }
        for (int32_t n = 0; n < N; ++n) H[(int64_t)m * ldh + n] = (float)acc[n];
    }
    free(acc);
    return ORC_OK;
}

/* -------------------------------------------------------- gradients of one layer
 *
 * Each GPU obtains a stochastic gradient of the loss through its sampled layers (Section 3,
 * Eq. 1 and Eq. 2).  For one layer H = Z W, Z = P~ sigma(H_prev), with G = dL/dH given, the chain
 * rule is written out as it stands:
 *     dL/dW      = Z^T G
 *     dL/dZ      = G W^T
 *     dL/dH_prev = (P~^T dL/dZ) .* sigma'(H_prev),   sigma = ReLU: sigma'(x) = [x > 0]
 * Double accumulation, one rounding to float.  Pinned by central finite differences of the
 * forward functions in double.
 */

/* dW [K x N] = Z^T [K x M] G [M x N] */
int orc_layer_gemm_grad_w(const float *Z, int64_t ldz, const float *G, int64_t ldg, int32_t M, int32_t K, int32_t N,
                          float *dW, int64_t lddw)
{
    if (!Z || !G || !dW || M < 0 || K <= 0 || N <= 0) return ORC_EINVAL;
    for (int32_t k = 0; k < K; ++k)
        for (int32_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int32_t m = 0; m < M; ++m) acc += (double)Z[(int64_t)m * ldz + k] * (double)G[(int64_t)m * ldg + n];
            dW[(int64_t)k * lddw + n] = (float)acc;
        }
    return ORC_OK;
}

/* dZ [M x K] = G [M x N] W^T [N x K],  W stored [K x N] */
int orc_layer_gemm_grad_z(const float *G, int64_t ldg, int32_t M, int32_t N, const float *W, int64_t ldw, int32_t K,
                          float *dZ, int64_t lddz)
{
    if (!G || !W || !dZ || M < 0 || K <= 0 || N <= 0) return ORC_EINVAL;
    for (int32_t m = 0; m < M; ++m)
        for (int32_t k = 0; k < K; ++k) {
            double acc = 0.0;
            for (int32_t n = 0; n < N; ++n) acc += (double)G[(int64_t)m * ldg + n] * (double)W[(int64_t)k * ldw + n];
            dZ[(int64_t)m * lddz + k] = (float)acc;
        }
    return ORC_OK;
}

/* dH_prev [n_cols x F] = (P~^T dZ) .* [H_prev > 0]   (H_prev NULL: no activation, no mask).
 * P~ is the CSR of the forward step: nS rows, columns < n_cols. */
int orc_aggregate_grad(const int32_t *adj_rowptr, const int32_t *adj_col, const float *adj_val, int32_t nS,
                       int32_t n_cols, const float *dZ, int64_t lddz, int32_t F, const float *H_prev, int64_t ldh,
                       float *dH, int64_t ldd)
{
    if (!adj_rowptr || !dZ || !dH || nS < 0 || n_cols < 0 || F <= 0) return ORC_EINVAL;
    double *acc = (double *)calloc((size_t)(n_cols > 0 ? n_cols : 1) * (size_t)F, sizeof(double));
    if (!acc) return ORC_ECAP;
    for (int32_t r = 0; r < nS; ++r)
        for (int32_t e = adj_rowptr[r]; e < adj_rowptr[r + 1]; ++e) {
            const int32_t c = adj_col[e];
            if (c < 0 || c >= n_cols) { free(acc); return ORC_EINVAL; }
            for (int32_t f = 0; f < F; ++f) acc[(size_t)c * F + f] += (double)adj_val[e] * (double)dZ[(int64_t)r * lddz + f];
        }
    for (int32_t c = 0; c < n_cols; ++c)
        for (int32_t f = 0; f < F; ++f) {
            double v = acc[(size_t)c * F + f];
            if (H_prev && !(H_prev[(int64_t)c * ldh + f] > 0.0f)) v = 0.0;
            dH[(int64_t)c * ldd + f] = (float)v;
        }
    free(acc);
    return ORC_OK;
}
