/*
 * kvm_ref.c -- CPU oracle for the KV-cache merging compression pass.
 *
 * TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  This file is a plain, slow, fp64
 * restatement of what the method computes, written so that it can be checked
 * against the paper by eye.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code with the GPU
 * library and is never used as a fallback.
 *
 * What follows the paper, and where:
 *   - attention map of one head:            Section 2.4, Eq. (1)
 *   - aggregated attention score per key:   Section 4.2, Eq. (7); Algorithm 2, step 2
 *   - cosine similarity of key states:      Section 3.1, Eq. (2)
 *   - merging-set identification:           Section 3.2; Section 4.1, Def. 4.1, Algorithm 1
 *   - conserved states (recent + top-k):    Section 4.1 (last paragraph); Section 5.1
 *   - pivotal state:                        Section 4.2, Eq. (7); Algorithm 2, step 3
 *   - Gaussian-kernel weights and merge:    Section 4.2, Def. 4.2, Eq. (4)-(6); Algorithm 2
 *
 * Readings taken where the paper is silent, garbled or inconsistent (each is
 * marked [reading] at the place it is used):
 *   R-a1  the aggregated score of key j is the column sum of the causal
 *         attention map over all prompt queries (Eq. (7) prints a row index).
 *   R-a3  with several query heads per KV head the per-head scores are summed
 *         (Section 5.2 averages them; a constant factor changes no decision).
 *   R-b1  Algorithm 1 is an adjacent chain: token i-1 joins the set of token i
 *         iff their cosine similarity exceeds the threshold; then i moves down.
 *         The other reading is available as a variant (REF_SETS_ANCHOR): the set of
 *         token i takes the tokens below it, one after the other, as long as their
 *         similarity to k_i itself exceeds the threshold (Section 3.2 groups the states
 *         by their similarity to one given key state); the first token that fails becomes
 *         the next i.  No budget fallback exists for this reading.
 *   R-b3  a zero-norm key has similarity 0 to its neighbours.
 *   R-b4  conserved tokens are singleton sets in their original position and
 *         split the run around them.
 *   R-b5  the recent / top-k proportions of Section 5.1 are fractions of n.
 *   R-b6  budget fallback (an extension, motivated by Section 3.2's remark that
 *         the threshold sets the compression ratio): when the number of sets
 *         exceeds floor(budget*n), the boundaries between two non-conserved
 *         tokens with the largest similarity are removed until it fits.
 *   R-c1  sigma of a set = (sum of Euclidean distances to the pivot) /
 *         (sqrt(2) |S|)  (Eq. (5) defines sigma through g, which itself needs
 *         sigma; Section 5.4 reports a computed sigma near 5, impossible for a mean of
 *         values in (0,1]).  PARITY UNPINNED against the authors' own code.
 *   R-c3  sigma == 0 (all keys of the set equal the pivot) gives g = 1.
 *   R-c4  value weights are the key weights times |S| (Section 4.2), optional.
 *   R-v   (comparison workload only) value-only merging, of which Section 2.3 gives one
 *         sentence: evicted values go to the kept token nearest by position (a tie to the
 *         later one) and the kept value becomes the plain mean.  PARITY UNPINNED against
 *         the scheme's own publication, which is not in the paper.
 *
 * Variants the paper studies (Section 4.2 first experiment, Section 5.4), selectable here:
 *   - average weighted merging: every member of a set gets weight 1/|S|
 *   - pivot = the set's token with the largest index (the choice Section 4.2 makes
 *     for the average-weighted experiment), or a token drawn at random
 *     (Section 5.4, "Choice of Pivotal State").  The random draw is a counter-based
 *     generator (SplitMix64 output function of seed + slice*2^32 + first token of
 *     the set), so that any implementation draws the same pivots.
 *
 * Parity pins live in tests/ (closed forms, brute force, invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { REF_F32 = 0, REF_F16 = 1, REF_BF16 = 2 };
enum { REF_SLICE_OK = 0, REF_SLICE_FALLBACK = 1, REF_SLICE_INFEASIBLE = 2, REF_SLICE_TRUNCATED = 4 };
enum { REF_SIGMA_MEAN_DIST = 0, REF_SIGMA_FIXED = 1 };
enum { REF_WEIGHTS_GAUSSIAN = 0, REF_WEIGHTS_AVERAGE = 1 };
enum { REF_PIVOT_MAX_SCORE = 0, REF_PIVOT_LAST = 1, REF_PIVOT_RANDOM = 2 };
enum { REF_SETS_ADJACENT = 0, REF_SETS_ANCHOR = 1 };

/* ---- exact widening of storage types ------------------------------------ */

static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, m = h & 0x3ff;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(m | 0x400), e - 25);
    return sign ? -v : v;
}

static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static size_t elem_size(int dtype) { return dtype == REF_F32 ? 4 : 2; }

/* copy rows x d elements starting at element offset `off` into fp64 */
static void widen(const void *src, size_t off, size_t count, int dtype, double *dst)
{
    size_t i;
    if (dtype == REF_F32) {
        const float *p = (const float *)src + off;
        for (i = 0; i < count; ++i) dst[i] = (double)p[i];
    } else if (dtype == REF_F16) {
        const uint16_t *p = (const uint16_t *)src + off;
        for (i = 0; i < count; ++i) dst[i] = half_to_double(p[i]);
    } else {
        const uint16_t *p = (const uint16_t *)src + off;
        for (i = 0; i < count; ++i) dst[i] = bf16_to_double(p[i]);
    }
}

static int valid_len(const int32_t *seq_lens, int b, int N)
{
    int n = seq_lens ? seq_lens[b] : N;
    if (n < 0) n = 0;
    if (n > N) n = N;
    return n;
}

/* ========================================================================= */
/* (a) aggregated attention score per key                                     */
/* ========================================================================= */

/* One query head against one key matrix: for every query row t the causal
 * attention row A_t = softmax(q_t K^T / sqrt(d)) over keys 0..t (Eq. (1)); the
 * row is added into a[0..t], so that a[j] ends as the sum over t of A[t][j]
 * ([reading] R-a1). */
static void mass_one_head(const double *q, const double *k, int n, int d, double *a, double *row)
{
    const double scale = 1.0 / sqrt((double)d);
    int t, j, c;
    for (t = 0; t < n; ++t) {
        double mx = -INFINITY, sum = 0.0;
        for (j = 0; j <= t; ++j) {
            double s = 0.0;
            for (c = 0; c < d; ++c) s += q[(size_t)t * d + c] * k[(size_t)j * d + c];
            row[j] = s * scale;
            if (row[j] > mx) mx = row[j];
        }
        for (j = 0; j <= t; ++j) {
            row[j] = exp(row[j] - mx);
            sum += row[j];
        }
        for (j = 0; j <= t; ++j) a[j] += row[j] / sum;
    }
}

/* Q: (B, H*G, N, d), K: (B, H, N, d), mass: (B, H, N) fp64.  Positions >= n_b get 0. */
int kvm_ref_attn_mass(int B, int H, int G, int N, int d, int dtype, const int32_t *seq_lens,
                      const void *Q, const void *K, double *mass)
{
    int bh;
    if (B < 0 || H < 1 || G < 1 || N < 0 || d < 1 || !mass) return 1;
    if (B && N && (!Q || !K)) return 1;
    (void)elem_size;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * H; ++bh) {
        int b = bh / H, h = bh % H, g, j;
        int n = valid_len(seq_lens, b, N);
        double *a = mass + (size_t)bh * N;
        double *kd, *qd, *row;
        for (j = 0; j < N; ++j) a[j] = 0.0;
        if (n == 0) continue;
        kd = (double *)malloc(sizeof(double) * (size_t)n * d);
        qd = (double *)malloc(sizeof(double) * (size_t)n * d);
        row = (double *)malloc(sizeof(double) * (size_t)n);
        widen(K, (size_t)bh * N * d, (size_t)n * d, dtype, kd);
        for (g = 0; g < G; ++g) { /* [reading] R-a3: sum over the query heads of this KV head */
            widen(Q, ((size_t)b * H * G + (size_t)h * G + g) * N * d, (size_t)n * d, dtype, qd);
            mass_one_head(qd, kd, n, d, a, row);
        }
        free(kd);
        free(qd);
        free(row);
    }
    return 0;
}

/* Row statistics of Eq. (1): lse[b, hq, t] = log of the sum over keys j <= t of
 * exp(q_t . k_j / sqrt(d)), i.e. the logarithm of the softmax denominator of query row t
 * (the quantity attention kernels keep per row).  Q: (B, H*G, N, d), K: (B, H, N, d),
 * lse: (B, H*G, N) fp64; rows >= n_b get 0. */
int kvm_ref_row_lse(int B, int H, int G, int N, int d, int dtype, const int32_t *seq_lens,
                    const void *Q, const void *K, double *lse)
{
    int bq;
    if (B < 0 || H < 1 || G < 1 || N < 0 || d < 1 || !lse) return 1;
    if (B && N && (!Q || !K)) return 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (bq = 0; bq < B * H * G; ++bq) {
        const int b = bq / (H * G), h = (bq % (H * G)) / G;
        const int n = valid_len(seq_lens, b, N);
        const double scale = 1.0 / sqrt((double)d);
        double *out = lse + (size_t)bq * N;
        double *kd, *qd, *row;
        int t, j, c;
        for (t = 0; t < N; ++t) out[t] = 0.0;
        if (n == 0) continue;
        kd = (double *)malloc(sizeof(double) * (size_t)n * d);
        qd = (double *)malloc(sizeof(double) * (size_t)n * d);
        row = (double *)malloc(sizeof(double) * (size_t)n);
        widen(K, ((size_t)b * H + h) * N * d, (size_t)n * d, dtype, kd);
        widen(Q, (size_t)bq * N * d, (size_t)n * d, dtype, qd);
        for (t = 0; t < n; ++t) {
            double mx = -INFINITY, sum = 0.0;
            for (j = 0; j <= t; ++j) {
                double sc = 0.0;
                for (c = 0; c < d; ++c) sc += qd[(size_t)t * d + c] * kd[(size_t)j * d + c];
                row[j] = sc * scale;
                if (row[j] > mx) mx = row[j];
            }
            for (j = 0; j <= t; ++j) sum += exp(row[j] - mx);
            out[t] = mx + log(sum);
        }
        free(kd);
        free(qd);
        free(row);
    }
    return 0;
}

/* Decode-time update of the aggregated scores (Eq. (1) for the newest query alone; the column
 * sums of Eq. (7) are sums over query rows, so one more row is one more term per key).  For
 * every batch row with n = n_b >= 1 valid tokens, the newest token sits at position n-1 and its
 * query states are q_new[b, h*G+g, :]:
 *     p_g = softmax over j in [0, n) of q_g . k_j / sqrt(d),
 *     mass[b,h,j] += sum_g p_g[j]  for j < n-1,      mass[b,h,n-1] = sum_g p_g[n-1].
 * Positions >= n are left alone.  q_new: (B, H*G, d), K: (B, H, N, d), mass: (B, H, N) fp64. */
int kvm_ref_attn_mass_append(int B, int H, int G, int N, int d, int dtype, const int32_t *seq_lens,
                             const void *q_new, const void *K, double *mass)
{
    int bh;
    if (B < 0 || H < 1 || G < 1 || N < 0 || d < 1 || !mass) return 1;
    if (B && N && (!q_new || !K)) return 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * H; ++bh) {
        const int b = bh / H, h = bh % H;
        const int n = valid_len(seq_lens, b, N);
        const double scale = 1.0 / sqrt((double)d);
        double *a = mass + (size_t)bh * N;
        double *kd, *qd, *row;
        int g, j, c;
        if (n == 0) continue;
        kd = (double *)malloc(sizeof(double) * (size_t)n * d);
        qd = (double *)malloc(sizeof(double) * (size_t)d);
        row = (double *)malloc(sizeof(double) * (size_t)n);
        widen(K, (size_t)bh * N * d, (size_t)n * d, dtype, kd);
        a[n - 1] = 0.0;
        for (g = 0; g < G; ++g) {
            double mx = -INFINITY, sum = 0.0;
            widen(q_new, ((size_t)b * H * G + (size_t)h * G + g) * d, (size_t)d, dtype, qd);
            for (j = 0; j < n; ++j) {
                double sc = 0.0;
                for (c = 0; c < d; ++c) sc += qd[c] * kd[(size_t)j * d + c];
                row[j] = sc * scale;
                if (row[j] > mx) mx = row[j];
            }
            for (j = 0; j < n; ++j) {
                row[j] = exp(row[j] - mx);
                sum += row[j];
            }
            for (j = 0; j < n; ++j) a[j] += row[j] / sum;
        }
        free(kd);
        free(qd);
        free(row);
    }
    return 0;
}

/* ========================================================================= */
/* (b) merging-set identification                                             */
/* ========================================================================= */

/* Eq. (2); [reading] R-b3 for a zero norm. */
static double cosine(const double *x, const double *y, int d)
{
    double xy = 0.0, xx = 0.0, yy = 0.0;
    int c;
    for (c = 0; c < d; ++c) {
        xy += x[c] * y[c];
        xx += x[c] * x[c];
        yy += y[c] * y[c];
    }
    if (xx == 0.0 || yy == 0.0) return 0.0;
    return xy / (sqrt(xx) * sqrt(yy));
}

/* Output function of SplitMix64 (Steele, Lea, Flood 2014) applied to the counter z. */
static uint64_t splitmix64_at(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Random member of a set of m tokens that starts at token lo of slice bh: the upper 32
 * bits of the draw scaled to [0, m). */
static int random_offset(uint64_t seed, int bh, int lo, int m)
{
    uint64_t r = splitmix64_at(seed + (((uint64_t)(uint32_t)bh << 32) | (uint32_t)lo));
    return (int)(((r >> 32) * (uint64_t)m) >> 32);
}

typedef struct { double v; int idx; } ranked;

static int by_value_desc_index_asc(const void *pa, const void *pb)
{
    const ranked *a = (const ranked *)pa, *b = (const ranked *)pb;
    if (a->v > b->v) return -1;
    if (a->v < b->v) return 1;
    return a->idx < b->idx ? -1 : (a->idx > b->idx ? 1 : 0);
}

static int by_value_desc_index_desc(const void *pa, const void *pb)
{
    const ranked *a = (const ranked *)pa, *b = (const ranked *)pb;
    if (a->v > b->v) return -1;
    if (a->v < b->v) return 1;
    return a->idx > b->idx ? -1 : (a->idx < b->idx ? 1 : 0);
}

/* Algorithm 1, walked from the last token to the first ([reading] R-b1, R-b4).
 * joins[i] != 0 means "token i-1 may join the set that holds token i".
 * Writes first[] = first token of each set, in the order the sets are found
 * (last set first); returns the number of sets. */
static int walk_sets(int n, const unsigned char *joins, int *first)
{
    int m = 0, i = n - 1;
    while (i >= 0) {
        int j = i;                       /* the set starts as {k_i}              */
        while (j >= 1 && joins[j]) --j;  /* neighbour j-1 joins; "i = j"         */
        first[m++] = j;
        i = j - 1;                       /* next set starts below this one       */
    }
    return m;
}

/* Algorithm 1 with the similarity taken to the set's own top token k_i (the anchor):
 * tokens i-1, i-2, ... join while they are not conserved and delta(k_i, k_j) > epsilon;
 * then "i = j" moves on to the first token that did not join.  Same outputs as walk_sets.
 * *margin = smallest |delta - epsilon| over all comparisons made (how close any decision
 * came to the threshold). */
static int walk_sets_anchor(int n, int d, const double *k, const unsigned char *prot, double threshold,
                            int *first, double *margin)
{
    int m = 0, i = n - 1;
    *margin = INFINITY;
    while (i >= 0) {
        int j = i;
        if (!prot[i]) {
            while (j >= 1 && !prot[j - 1]) {
                double c = cosine(k + (size_t)i * d, k + (size_t)(j - 1) * d, d);
                double gap = fabs(c - threshold);
                if (gap < *margin) *margin = gap;
                if (!(c > threshold)) break;
                --j;
            }
        }
        first[m++] = j;
        i = j - 1;
    }
    return m;
}

/*
 * K: (B, H, N, d) storage dtype; mass: (B, H, N) fp64 (the caller widens the
 * fp32 values the GPU path reads, so both sides rank identical numbers).
 * Outputs per slice: set_id[N] (-1 at padding), set_start[cap_rows+1],
 * pivot[cap_rows], n_sets, status, and optionally sim[N], protected_mask[N] and
 * min_removed_sim.
 *
 * set_start[s] = first token of set s for s < M, s <= cap_rows; the remaining
 * entries up to cap_rows hold n (so set_start[M] = n when M <= cap_rows, and a
 * stored set always ends where the next entry says).
 * pivot[s] = -1 for s >= M.  n_sets = M even when M > cap_rows (status then has
 * REF_SLICE_TRUNCATED).
 * min_removed_sim[slice] = smallest similarity among the boundaries the budget
 * fallback removed (+inf if none): the slice's effective threshold lies just
 * below it.
 */
int kvm_ref_identify_sets(int B, int H, int N, int d, int dtype, const int32_t *seq_lens,
                          double budget, double recent_ratio, double heavy_ratio, double threshold,
                          int enforce_budget, int set_rule, int pivot_rule, uint64_t pivot_seed, int cap_rows,
                          const void *K, const double *mass,
                          int32_t *set_id, int32_t *set_start, int32_t *pivot, int32_t *n_sets,
                          int32_t *slice_status, double *sim_out, unsigned char *protected_out,
                          double *min_removed_sim, double *anchor_margin)
{
    int bh;
    if (B < 0 || H < 1 || N < 0 || d < 1 || cap_rows < 0) return 1;
    if (pivot_rule < REF_PIVOT_MAX_SCORE || pivot_rule > REF_PIVOT_RANDOM) return 1;
    if (set_rule != REF_SETS_ADJACENT && set_rule != REF_SETS_ANCHOR) return 1;
    if (!set_id || !set_start || !pivot || !n_sets || !slice_status) return 1;
    if (B && N && (!K || !mass)) return 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * H; ++bh) {
        int b = bh / H;
        int n = valid_len(seq_lens, b, N);
        const double *a = mass + (size_t)bh * N;
        int32_t *sid = set_id + (size_t)bh * N;
        int32_t *sst = set_start + (size_t)bh * (cap_rows + 1);
        int32_t *piv = pivot + (size_t)bh * cap_rows;
        int j, s, M, status = REF_SLICE_OK;
        /* [reading] R-b5: proportions of n, counted by floor */
        int n_recent = (int)floor(recent_ratio * (double)n);
        int n_heavy = (int)floor(heavy_ratio * (double)n);
        int cap = (int)floor(budget * (double)n);
        double *kd = (double *)malloc(sizeof(double) * ((size_t)n * d + 1));
        double *sim = (double *)malloc(sizeof(double) * (size_t)(n + 1));
        unsigned char *prot = (unsigned char *)calloc((size_t)n + 1, 1);
        unsigned char *joins = (unsigned char *)calloc((size_t)n + 1, 1);
        int *first = (int *)malloc(sizeof(int) * (size_t)(n + 1));
        ranked *rk = (ranked *)malloc(sizeof(ranked) * (size_t)(n + 1));
        double min_removed = INFINITY;

        if (n_recent > n) n_recent = n;
        if (n_heavy > n - n_recent) n_heavy = n - n_recent;
        widen(K, (size_t)bh * N * d, (size_t)n * d, dtype, kd);

        /* conserved states: the most recent tokens, and the top-k aggregated scores
         * among the others (ties: lower index first) */
        for (j = n - n_recent; j < n; ++j) prot[j] = 1;
        for (j = 0; j < n - n_recent; ++j) { rk[j].v = a[j]; rk[j].idx = j; }
        qsort(rk, (size_t)(n - n_recent), sizeof(ranked), by_value_desc_index_asc);
        for (j = 0; j < n_heavy; ++j) prot[rk[j].idx] = 1;

        /* similarity of every key to its predecessor, Eq. (2) */
        sim[0] = 0.0;
        for (j = 1; j < n; ++j) sim[j] = cosine(kd + (size_t)(j - 1) * d, kd + (size_t)j * d, d);

        /* Algorithm 1: j-1 joins j iff delta > epsilon (strict) and neither is conserved */
        for (j = 1; j < n; ++j) joins[j] = (!prot[j - 1] && !prot[j] && sim[j] > threshold) ? 1 : 0;
        M = walk_sets(n, joins, first);
        if (set_rule == REF_SETS_ANCHOR) {
            double margin;
            M = walk_sets_anchor(n, d, kd, prot, threshold, first, &margin);
            if (anchor_margin) anchor_margin[bh] = margin;
            if (enforce_budget && M > cap) status |= REF_SLICE_INFEASIBLE; /* no fallback for this reading */
        }

        /* [reading] R-b6: budget fallback */
        if (set_rule == REF_SETS_ADJACENT && enforce_budget && M > cap) {
            int n_nat = 0, r = M - cap;
            for (j = 1; j < n; ++j)
                if (!joins[j] && !prot[j - 1] && !prot[j]) { rk[n_nat].v = sim[j]; rk[n_nat].idx = j; ++n_nat; }
            qsort(rk, (size_t)n_nat, sizeof(ranked), by_value_desc_index_desc);
            if (n_nat < r) { status |= REF_SLICE_INFEASIBLE; r = n_nat; }
            if (r > 0) status |= REF_SLICE_FALLBACK;
            for (j = 0; j < r; ++j) {
                joins[rk[j].idx] = 1;
                if (rk[j].v < min_removed) min_removed = rk[j].v;
            }
            M = walk_sets(n, joins, first);
        }

        /* number the sets in sequence order; pivot = argmax of the score, first on ties
         * (Eq. (7)), or the variant asked for */
        for (j = 0; j < N; ++j) sid[j] = -1;
        for (s = 0; s <= cap_rows; ++s) sst[s] = n;
        for (s = 0; s < cap_rows; ++s) piv[s] = -1;
        for (s = 0; s < M; ++s) {
            int lo = first[M - 1 - s];
            int hi = (s + 1 < M) ? first[M - 2 - s] : n;
            int p = lo;
            for (j = lo; j < hi; ++j) {
                sid[j] = s;
                if (a[j] > a[p]) p = j;
            }
            if (pivot_rule == REF_PIVOT_LAST) p = hi - 1;
            if (pivot_rule == REF_PIVOT_RANDOM) p = lo + random_offset(pivot_seed, bh, lo, hi - lo);
            if (s <= cap_rows) sst[s] = lo;
            if (s < cap_rows) piv[s] = p;
        }
        if (M > cap_rows) status |= REF_SLICE_TRUNCATED;
        n_sets[bh] = M;
        slice_status[bh] = status;
        if (min_removed_sim) min_removed_sim[bh] = min_removed;
        if (sim_out) {
            for (j = 0; j < N; ++j) sim_out[(size_t)bh * N + j] = j < n ? sim[j] : 0.0;
        }
        if (protected_out) {
            for (j = 0; j < N; ++j) protected_out[(size_t)bh * N + j] = j < n ? prot[j] : 0;
        }
        free(kd); free(sim); free(prot); free(joins); free(first); free(rk);
    }
    return 0;
}

/* ========================================================================= */
/* (c) Gaussian-kernel weighted merging                                       */
/* ========================================================================= */

/* Algorithm 2 for one set: keys k[0..m) (rows of d), pivot index p inside the set.
 * Writes the m weights w (they sum to 1). */
static void set_weights(const double *k, int m, int d, int p, int weights_mode, int sigma_mode, double sigma_fixed,
                        double *w)
{
    double dist_sum = 0.0, g_sum = 0.0, sigma;
    int j, c;
    if (weights_mode == REF_WEIGHTS_AVERAGE) { /* average weighted merging, Section 4.2 */
        for (j = 0; j < m; ++j) w[j] = 1.0 / (double)m;
        return;
    }
    for (j = 0; j < m; ++j) { /* w[j] holds ||k_p - k_j|| for now */
        double sq = 0.0;
        for (c = 0; c < d; ++c) {
            double diff = k[(size_t)p * d + c] - k[(size_t)j * d + c];
            sq += diff * diff;
        }
        w[j] = sqrt(sq);
        dist_sum += w[j];
    }
    /* [reading] R-c1 */
    sigma = sigma_mode == REF_SIGMA_FIXED ? sigma_fixed : dist_sum / (sqrt(2.0) * (double)m);
    for (j = 0; j < m; ++j) { /* Eq. (5); [reading] R-c3 */
        w[j] = sigma == 0.0 ? 1.0 : exp(-(w[j] * w[j]) / (2.0 * sigma * sigma));
        g_sum += w[j];
    }
    for (j = 0; j < m; ++j) w[j] /= g_sum; /* Eq. (6) */
}

/*
 * K, V: (B, H, N, d); set_start (B, H, cap_rows+1), pivot (B, H, cap_rows),
 * n_sets (B, H) as written by kvm_ref_identify_sets.  K_out, V_out:
 * (B, H, cap_rows, d) fp64; rows >= min(n_sets, cap_rows) are not written.
 * w_out (optional): (B, H, N) key weight of every token (0 at padding and for
 * tokens of truncated sets).
 */
int kvm_ref_merge(int B, int H, int N, int d, int dtype, const int32_t *seq_lens, int cap_rows,
                  int weights_mode, int sigma_mode, double sigma_fixed, int value_scale_by_set_size,
                  const void *K, const void *V, const int32_t *set_start, const int32_t *pivot,
                  const int32_t *n_sets, double *K_out, double *V_out, double *w_out)
{
    int bh;
    if (B < 0 || H < 1 || N < 0 || d < 1 || cap_rows < 0) return 1;
    if (B && N && (!K || !V || !set_start || !pivot || !n_sets || !K_out || !V_out)) return 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * H; ++bh) {
        int b = bh / H;
        int n = valid_len(seq_lens, b, N);
        const int32_t *sst = set_start + (size_t)bh * (cap_rows + 1);
        const int32_t *piv = pivot + (size_t)bh * cap_rows;
        int M = n_sets[bh] < cap_rows ? n_sets[bh] : cap_rows;
        int s, j, c;
        double *kd = (double *)malloc(sizeof(double) * ((size_t)n * d + 1));
        double *vd = (double *)malloc(sizeof(double) * ((size_t)n * d + 1));
        double *w = (double *)malloc(sizeof(double) * (size_t)(n + 1));
        widen(K, (size_t)bh * N * d, (size_t)n * d, dtype, kd);
        widen(V, (size_t)bh * N * d, (size_t)n * d, dtype, vd);
        if (w_out) for (j = 0; j < N; ++j) w_out[(size_t)bh * N + j] = 0.0;
        for (s = 0; s < M; ++s) {
            int lo = sst[s], hi = sst[s + 1], m = hi - lo;
            double *ko = K_out + ((size_t)bh * cap_rows + s) * d;
            double *vo = V_out + ((size_t)bh * cap_rows + s) * d;
            double vscale = value_scale_by_set_size ? (double)m : 1.0; /* [reading] R-c4 */
            set_weights(kd + (size_t)lo * d, m, d, piv[s] - lo, weights_mode, sigma_mode, sigma_fixed, w);
            for (c = 0; c < d; ++c) { ko[c] = 0.0; vo[c] = 0.0; }
            for (j = 0; j < m; ++j) /* Def. 4.2, Eq. (4) */
                for (c = 0; c < d; ++c) {
                    ko[c] += w[j] * kd[(size_t)(lo + j) * d + c];
                    vo[c] += vscale * w[j] * vd[(size_t)(lo + j) * d + c];
                }
            if (w_out) for (j = 0; j < m; ++j) w_out[(size_t)bh * N + lo + j] = w[j];
        }
        free(kd); free(vd); free(w);
    }
    return 0;
}

/* ========================================================================= */
/* comparison workload: eviction by aggregated attention score                 */
/* ========================================================================= */

/*
 * The selection policy of the heavy-hitter eviction methods the paper compares with
 * (Section 2.3): per slice keep floor(budget n) tokens -- the last floor(recent_ratio n)
 * (cut to the budget if wider) and the largest scores among the others (ties: lower
 * index) -- and drop the rest.  kept: (B, H, cap_rows) ascending positions, -1 beyond
 * n_kept; K_out, V_out: (B, H, cap_rows, d) fp64 copies of the kept rows.
 */
int kvm_ref_evict(int B, int H, int N, int d, int dtype, const int32_t *seq_lens, double budget,
                  double recent_ratio, int cap_rows, const void *K, const void *V, const double *mass,
                  int32_t *kept, int32_t *n_kept, double *K_out, double *V_out)
{
    int bh;
    if (B < 0 || H < 1 || N < 0 || d < 1 || cap_rows < 0 || !n_kept) return 1;
    for (bh = 0; bh < B * H; ++bh) {
        int b = bh / H;
        int n = valid_len(seq_lens, b, N);
        int cap = (int)floor(budget * (double)n);
        int n_recent = (int)floor(recent_ratio * (double)n);
        int pre, k, j, m = 0;
        unsigned char *keep = (unsigned char *)calloc((size_t)n + 1, 1);
        ranked *rk = (ranked *)malloc(sizeof(ranked) * (size_t)(n + 1));
        double *row = (double *)malloc(sizeof(double) * (size_t)d);
        if (cap > cap_rows) cap = cap_rows;
        if (n_recent > cap) n_recent = cap;
        pre = n - n_recent;
        k = cap - n_recent < pre ? cap - n_recent : pre;
        for (j = pre; j < n; ++j) keep[j] = 1;
        for (j = 0; j < pre; ++j) { rk[j].v = mass[(size_t)bh * N + j]; rk[j].idx = j; }
        qsort(rk, (size_t)pre, sizeof(ranked), by_value_desc_index_asc);
        for (j = 0; j < k; ++j) keep[rk[j].idx] = 1;
        for (j = 0; j < n; ++j) {
            if (!keep[j]) continue;
            kept[(size_t)bh * cap_rows + m] = j;
            widen(K, ((size_t)bh * N + j) * d, (size_t)d, dtype, row);
            memcpy(K_out + ((size_t)bh * cap_rows + m) * d, row, sizeof(double) * (size_t)d);
            widen(V, ((size_t)bh * N + j) * d, (size_t)d, dtype, row);
            memcpy(V_out + ((size_t)bh * cap_rows + m) * d, row, sizeof(double) * (size_t)d);
            ++m;
        }
        for (j = m; j < cap_rows; ++j) kept[(size_t)bh * cap_rows + j] = -1;
        n_kept[bh] = m;
        free(keep); free(rk); free(row);
    }
    return 0;
}

/*
 * A second comparison workload: value-only merging.  Section 2.3 says of the value-merging
 * scheme the paper compares with only that it merges the value states about to be evicted into
 * the conserved ones.  Reading built here: the selection is the eviction policy above; the keys
 * of evicted tokens are dropped; every evicted token's value goes to the kept token nearest to
 * it by position (equal distances: the later one), and a kept token's new value is the plain
 * mean of its own value and the values that went to it.  Same outputs as kvm_ref_evict, V_out
 * holding the means; count_opt (B, H, cap_rows), may be NULL: how many values each mean covers.
 */
int kvm_ref_evict_merge_values(int B, int H, int N, int d, int dtype, const int32_t *seq_lens, double budget,
                               double recent_ratio, int cap_rows, const void *K, const void *V, const double *mass,
                               int32_t *kept, int32_t *n_kept, double *K_out, double *V_out, int32_t *count_opt)
{
    int bh, rc;
    rc = kvm_ref_evict(B, H, N, d, dtype, seq_lens, budget, recent_ratio, cap_rows, K, V, mass, kept, n_kept, K_out, V_out);
    if (rc) return rc;
    for (bh = 0; bh < B * H; ++bh) {
        int n = valid_len(seq_lens, bh / H, N);
        int m = n_kept[bh], j, s, e;
        const int32_t *pos = kept + (size_t)bh * cap_rows;
        double *sum = (double *)calloc((size_t)(m > 0 ? m : 1) * (size_t)d, sizeof(double));
        int *cnt = (int *)calloc((size_t)(m > 0 ? m : 1), sizeof(int));
        double *row = (double *)malloc(sizeof(double) * (size_t)d);
        for (j = 0; j < n && m > 0; ++j) {
            int best = 0;
            for (s = 1; s < m; ++s) {                 /* nearest kept position, the later one on a tie */
                int ds = abs(pos[s] - j), db = abs(pos[best] - j);
                if (ds < db || (ds == db && pos[s] > pos[best])) best = s;
            }
            widen(V, ((size_t)bh * N + j) * d, (size_t)d, dtype, row);
            for (e = 0; e < d; ++e) sum[(size_t)best * d + e] += row[e];
            cnt[best] += 1;
        }
        for (s = 0; s < m; ++s) {
            for (e = 0; e < d; ++e) V_out[((size_t)bh * cap_rows + s) * d + e] = sum[(size_t)s * d + e] / (double)cnt[s];
            if (count_opt) count_opt[(size_t)bh * cap_rows + s] = cnt[s];
        }
        if (count_opt) for (s = m; s < cap_rows; ++s) count_opt[(size_t)bh * cap_rows + s] = 0;
        free(sum); free(cnt); free(row);
    }
    return 0;
}

/* Threads the slice loops run on (for the benchmark's report). */
int kvm_ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sets that number (the benchmark also times the oracle on a single thread).  No arithmetic here. */
void kvm_ref_set_num_threads(int k)
{
#ifdef _OPENMP
    if (k >= 1) omp_set_num_threads(k);
#else
    (void)k;
#endif
}

/* The pivot generator, exported for the tests (published test vectors). */
uint64_t kvm_ref_splitmix64_at(uint64_t z) { return splitmix64_at(z); }
int kvm_ref_random_offset(uint64_t seed, int bh, int lo, int m) { return random_offset(seed, bh, lo, m); }

/* Widening helpers exported for the tests (exactness of the fp16 / bf16 readers). */
double kvm_ref_half_to_double(uint16_t h) { return half_to_double(h); }
double kvm_ref_bf16_to_double(uint16_t h) { return bf16_to_double(h); }
