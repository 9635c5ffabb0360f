/*
 * kvm.h -- C ABI of the KV-cache merging compression pass for AMD MI355X (gfx950).
 *
 * The pass runs independently over every (batch, KV-head) slice of a prefilled
 * cache (fold layers into the batch axis) in three calls:
 *
 *   kvm_attn_mass      aggregated attention score of every key
 *   kvm_identify_sets  contiguous merging sets + pivot of each set
 *   kvm_merge          Gaussian-kernel weighted merge into a compacted cache
 * (kvm_evict and kvm_evict_merge_values are comparison workloads: plain eviction by the same
 *  scores, and eviction with the evicted values averaged into the kept ones)
 *
 * Conventions for every call
 *   - Every tensor pointer is a DEVICE pointer to contiguous memory, innermost
 *     axis d; Q is (B, H_kv*G, N, d) with the G query heads of KV head h at
 *     head indices h*G .. h*G+G-1; K and V are (B, H_kv, N, d).
 *   - The caller owns every buffer, including the workspace.  The library
 *     allocates nothing, keeps no state between calls and never synchronises:
 *     work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns.  Outputs are valid after the caller
 *     synchronises the stream.
 *   - Sequences are right-padded: batch row b has valid tokens [0, n_b),
 *     n_b = seq_lens[b] (device array of B int32; values are clamped to
 *     [0, N]) or N when seq_lens is NULL.  Padded positions are never read as
 *     data.
 *   - Errors are return codes; nothing throws or aborts.  Host-detectable
 *     errors (null pointer, unsupported shape, small workspace) return before
 *     any launch and leave outputs untouched; kvm_last_error() then holds a
 *     message.  Data-dependent per-slice conditions are reported on the device
 *     in slice_status and the call still returns KVM_OK.
 *   - v1 limits: d == 128; G >= 1; N >= 0; dtype one of kvm_dtype.
 */
#ifndef KVM_H
#define KVM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { KVM_F32 = 0, KVM_F16 = 1, KVM_BF16 = 2 } kvm_dtype;

typedef enum {
    KVM_OK = 0,
    KVM_ERR_INVALID_ARG = 1,  /* null pointer, negative size, ratio outside [0,1], ...      */
    KVM_ERR_UNSUPPORTED = 2,  /* d != 128, unknown dtype or sigma mode                      */
    KVM_ERR_WORKSPACE = 3,    /* ws == NULL or ws_bytes < kvm_workspace_bytes()             */
    KVM_ERR_LAUNCH = 4        /* the HIP runtime refused a launch; see kvm_last_error()     */
} kvm_status;

/* Bits of slice_status[b,h] written by kvm_identify_sets. */
enum {
    KVM_SLICE_FALLBACK = 1,   /* the budget fallback removed at least one boundary          */
    KVM_SLICE_INFEASIBLE = 2, /* even with every removable boundary gone M > floor(budget n) */
    KVM_SLICE_TRUNCATED = 4   /* M > capacity: only the first `capacity` sets were stored   */
};

typedef enum {
    KVM_SIGMA_MEAN_DIST = 0,  /* sigma = (sum of distances to the pivot) / (sqrt(2) |S|)     */
    KVM_SIGMA_FIXED = 1       /* sigma given by the caller (the fixed-sigma study, Sec. 5.4) */
} kvm_sigma_mode;

/* How the members of a set are weighted (Section 4.2). */
typedef enum {
    KVM_WEIGHTS_GAUSSIAN = 0, /* Gaussian kernel around the pivot, Eq. (5), (6)               */
    KVM_WEIGHTS_AVERAGE = 1   /* every member 1/|S|: the average weighted merging Section 4.2
                                 starts from                                                   */
} kvm_weights;

/* Which member of a set is its pivot. */
typedef enum {
    KVM_PIVOT_MAX_SCORE = 0,  /* largest aggregated attention score, Eq. (7)                  */
    KVM_PIVOT_LAST = 1,       /* largest index (Section 4.2, the average-weighted experiment) */
    KVM_PIVOT_RANDOM = 2      /* drawn at random (Section 5.4, "Choice of Pivotal State")     */
} kvm_pivot_rule;

/* How Algorithm 1 grows a set. */
typedef enum {
    KVM_SETS_ADJACENT = 0,    /* a token joins the set of its successor iff the two are
                                 similar enough (chain of adjacent tokens)                    */
    KVM_SETS_ANCHOR = 1       /* tokens below the set's top token join, one after the other,
                                 as long as they are similar enough to that top token
                                 (Section 3.2: similarity to one given key state)             */
} kvm_set_rule;

typedef struct {
    int32_t B;                /* batch (x layers): every (b, h) slice is independent         */
    int32_t H_kv;             /* KV heads                                                     */
    int32_t G;                /* query heads per KV head (1, or e.g. 4 for grouped queries)   */
    int32_t N;                /* padded sequence length                                       */
    int32_t d;                /* head dimension (128)                                         */
    int32_t dtype;            /* kvm_dtype of Q, K, V and of K_out, V_out                     */
    const int32_t *seq_lens;  /* DEVICE pointer [B], or NULL when every length is N           */
} kvm_shape;

typedef struct {
    double budget;            /* beta: a slice may keep floor(beta n_b) states                */
    double recent_ratio;      /* the last floor(r n_b) tokens are conserved                   */
    double heavy_ratio;       /* the floor(r n_b) largest scores among the others are too     */
    float threshold;          /* epsilon: neighbours merge iff cosine similarity > epsilon    */
    int32_t sigma_mode;       /* kvm_sigma_mode                                               */
    float sigma;              /* used when sigma_mode == KVM_SIGMA_FIXED (must be > 0)        */
    int32_t value_scale_by_set_size; /* 1: value weights are |S| w_i (Sec. 4.2); 0: w_i      */
    int32_t enforce_budget;   /* 1: remove boundaries until M <= floor(beta n_b) (see below)  */
    int32_t weights;          /* kvm_weights                                                  */
    int32_t pivot_rule;       /* kvm_pivot_rule                                               */
    uint64_t pivot_seed;      /* seed of the draws of KVM_PIVOT_RANDOM                        */
    int32_t set_rule;         /* kvm_set_rule                                                 */
    int32_t sim_given;        /* 1: sim_opt already holds the adjacent similarities of every
                                 token below n_b (written by an earlier kvm_identify_sets and
                                 extended by kvm_sim_append); step 2 below is skipped.  Needs
                                 sim_opt and set_rule == KVM_SETS_ADJACENT.  0: computed here   */
} kvm_params;

/*
 * The two scenarios of Section 5.1 ("Implementation details"): budget 0.50 ->
 * recent 0.17, heavy 0.12; budget 0.35 -> recent 0.08, heavy 0.02; threshold
 * 0.75 for both (the proportions are read as fractions of the length).  Other
 * budgets in (0,1] get recent = 0.34 beta, heavy = 0.24 beta (the 0.50 row
 * scaled).  Sets sigma_mode = MEAN_DIST, value_scale_by_set_size = 1,
 * enforce_budget = 1, weights = GAUSSIAN, pivot_rule = MAX_SCORE, pivot_seed = 0,
 * set_rule = ADJACENT, sim_given = 0.
 * Host call.  KVM_ERR_INVALID_ARG if out == NULL or budget
 * is not in (0,1].
 */
kvm_status kvm_params_for_budget(double budget, kvm_params *out);

/*
 * Rows per slice of set_start (+1), pivot, K_out and V_out:
 * floor(budget * N) when enforce_budget is set, else N.  Host call; returns -1
 * on invalid arguments.
 */
int32_t kvm_out_capacity(const kvm_shape *shape, const kvm_params *params);

/*
 * Bytes of device workspace that is enough for any of the three calls on this
 * shape (256-byte aligned pointer expected).  Host call; 0 on invalid
 * arguments.  Contents need no initialisation and are not preserved.
 */
size_t kvm_workspace_bytes(const kvm_shape *shape, const kvm_params *params);

/*
 * Aggregated attention score (Section 2.4 Eq. (1); Section 4.2 Eq. (7);
 * Algorithm 2 step 2):
 *     A_g = causal softmax(Q_g K^T / sqrt(d)) per query head g of the KV head,
 *     mass[b,h,j] = sum over g and over query rows t >= j of A_g[t,j].
 * With G > 1 the per-head maps are summed (the paper averages them for grouped
 * queries, Section 5.2: the same up to the factor G).
 *   Q     in   (B, H_kv*G, N, d) dtype
 *   K     in   (B, H_kv, N, d)   dtype
 *   mass  out  (B, H_kv, N) float32; 0 at positions >= n_b
 * Scores are accumulated in fp32 from the stored inputs; the map is never
 * materialised.  Deterministic (no atomics).
 */
kvm_status kvm_attn_mass(const kvm_shape *shape, const void *Q, const void *K, float *mass,
                         void *ws, size_t ws_bytes, void *stream);

/*
 * kvm_attn_mass and, in the same pass over K, the cosine similarities of adjacent key states
 * (Section 3.1 Eq. (2); the input of Algorithm 1): the kernel that takes the column sums of
 * Eq. (7) holds every key in registers anyway, so the scan of K that kvm_identify_sets starts
 * with is not needed afterwards.
 *   sim   out  (B, H_kv, N) float32: sim[j] = cos(k_{j-1}, k_j); 0 for j = 0, for a key of zero
 *              norm and at positions >= n_b -- what kvm_identify_sets returns in sim_opt, up to
 *              the order of the fp32 additions (a few 1e-7)
 * Pass sim to kvm_identify_sets as sim_opt with params.sim_given = 1 (adjacent rule).  Other
 * arguments, workspace, result and errors as for kvm_attn_mass; mass is bit for bit the same.
 * (fp32 caches: the similarities come from the same streaming scan kvm_identify_sets uses.)
 */
kvm_status kvm_attn_mass_sim(const kvm_shape *shape, const void *Q, const void *K, float *mass, float *sim,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * The same map for a caller that already holds the softmax row statistics of
 * Eq. (1), as prefill attention kernels keep them: only the column sums of
 * Eq. (7) remain, about half of kvm_attn_mass's work.
 *   row_lse  in  (B, H_kv*G, N) float32: natural logarithm of
 *                sum over j <= t of exp(q_t . k_j / sqrt(d)) for query row t;
 *                entries at t >= n_b are not read
 * Other arguments, workspace and result as for kvm_attn_mass.  The result is
 * only as good as row_lse: statistics taken from other scores than the stored
 * Q and K give columns that no longer sum to n_b per query head.
 */
kvm_status kvm_attn_mass_from_lse(const kvm_shape *shape, const void *Q, const void *K,
                                  const float *row_lse, float *mass, void *ws, size_t ws_bytes,
                                  void *stream);

/*
 * Decode-time update of the aggregated attention score: one more query row of
 * Eq. (1) added into the column sums of Eq. (7), so that `mass` stays what
 * kvm_attn_mass would give on the longer sequence without another pass over the
 * prompt.  (The paper runs its method on the prefilled cache and says nothing
 * of decoding; this call only keeps the scores current, the sets and the merge
 * are then refreshed with the two calls below.)
 * Per batch row, n_b = seq_lens[b] counts the newest token, whose key is already
 * stored at K[b, :, n_b - 1]:
 *     p_g = softmax over j < n_b of q_new[b, h*G+g] . K[b,h,j] / sqrt(d),
 *     mass[b,h,j] += sum_g p_g[j] for j < n_b - 1;   mass[b,h,n_b-1] = sum_g p_g[n_b-1].
 *   q_new  in      (B, H_kv*G, d) dtype: query states of the newest token
 *   K      in      (B, H_kv, N, d) dtype
 *   mass   in/out  (B, H_kv, N) float32; entries at j >= n_b are not touched, rows
 *                  with n_b == 0 are skipped
 * Workspace as for kvm_attn_mass.  Deterministic.
 */
kvm_status kvm_attn_mass_append(const kvm_shape *shape, const void *q_new, const void *K,
                                float *mass, void *ws, size_t ws_bytes, void *stream);

/*
 * Decode-time companion of kvm_attn_mass_append for the similarities: only the
 * newest token's similarity to its predecessor (Eq. (2)) is new, so
 *     sim[b,h,n_b-1] = cosine(K[b,h,n_b-2], K[b,h,n_b-1])   (0 if n_b == 1 or a norm is 0)
 * is written, with the bits kvm_identify_sets would write there, and nothing else.
 * A following kvm_identify_sets with params.sim_given = 1 then reads K not at all.
 *   K    in      (B, H_kv, N, d) dtype
 *   sim  in/out  (B, H_kv, N) float32
 */
kvm_status kvm_sim_append(const kvm_shape *shape, const void *K, float *sim, void *stream);

/*
 * Merging-set identification (Section 3.2; Section 4.1 Def. 4.1 and Algorithm 1;
 * conserved states: Section 4.1 last paragraph and Section 5.1; pivot: Eq. (7)).
 * Per slice, with n = n_b:
 *   1. conserved tokens: the last floor(recent_ratio n), plus the
 *      floor(heavy_ratio n) largest `mass` among the others (ties: lower index);
 *   2. sim[j] = cosine similarity of k_{j-1} and k_j (Eq. (2)), 0 if a norm is 0
 *      (norms are accumulated in fp32: a squared norm below 2^-126 counts as 0);
 *   3. token j-1 and j share a set iff sim[j] > threshold and neither is
 *      conserved (Algorithm 1 read as a chain of adjacent tokens); sets are
 *      therefore contiguous, disjoint and cover [0, n); conserved tokens are
 *      singletons;
 *   4. if enforce_budget and the number of sets M > floor(budget n): the
 *      M - floor(budget n) boundaries between two non-conserved tokens with the
 *      largest sim are removed (ties: higher index first), i.e. the slice's
 *      threshold is lowered just enough; if there are not enough of them all are
 *      removed and KVM_SLICE_INFEASIBLE is set;
 *   5. pivot of a set = its token with the largest mass (ties: lowest index);
 *      KVM_PIVOT_LAST: its last token; KVM_PIVOT_RANDOM: first token + floor(u m / 2^32)
 *      for a set of m tokens, u = upper 32 bits of the SplitMix64 output function at the
 *      counter pivot_seed + (slice index b*H_kv+h) * 2^32 + first token (mod 2^64), so the
 *      draws can be reproduced anywhere.
 * With set_rule == KVM_SETS_ANCHOR steps 3 and 4 read: walking down from the last
 * token, the set of token i takes tokens i-1, i-2, ... while they are not conserved and
 * their cosine similarity to k_i exceeds the threshold; the first token that does not
 * join starts the next set.  This reading has no budget fallback: a slice with
 * M > floor(budget n) gets KVM_SLICE_INFEASIBLE (when enforce_budget is set) and is
 * truncated to the capacity.  sim_opt still holds the adjacent similarities.
 *   K            in   (B, H_kv, N, d)
 *   mass         in   (B, H_kv, N) float32 (finite; as written by kvm_attn_mass)
 *   set_id       out  (B, H_kv, N) int32: set of token j, -1 at positions >= n
 *   set_start    out  (B, H_kv, capacity+1) int32: first token of set s for
 *                     s < M (s <= capacity); remaining entries hold n
 *   pivot        out  (B, H_kv, capacity) int32: absolute position; -1 for s >= M
 *   n_sets       out  (B, H_kv) int32: M (may exceed capacity: KVM_SLICE_TRUNCATED)
 *   sim_opt      out  (B, H_kv, N) float32 or NULL; sim[0] and padding are 0
 *                     (in, entries below n_b, and not written, when params->sim_given is set;
 *                     K is then not read and may be NULL)
 *   slice_status out  (B, H_kv) int32: KVM_SLICE_* bits
 * capacity = kvm_out_capacity().  Sets are numbered in sequence order, so the
 * compacted cache stays position-ordered.  Integer outputs are deterministic.
 */
kvm_status kvm_identify_sets(const kvm_shape *shape, const kvm_params *params, const void *K,
                             const float *mass, int32_t *set_id, int32_t *set_start, int32_t *pivot,
                             int32_t *n_sets, float *sim_opt, int32_t *slice_status, void *ws,
                             size_t ws_bytes, void *stream);

/*
 * Gaussian-kernel weighted merging (Section 4.2: Def. 4.2 Eq. (4), Eq. (5), (6);
 * Algorithm 2).  For every stored set S with pivot p:
 *     D_j = ||k_p - k_j||_2,  g_j = exp(-D_j^2 / (2 sigma^2)),  w_j = g_j / sum g,
 *     K_out[s] = sum w_j k_j,   V_out[s] = c sum w_j v_j,  c = |S| or 1.
 * sigma: KVM_SIGMA_MEAN_DIST -> sum_j D_j / (sqrt(2) |S|) (all g = 1 when it is
 * 0, so a singleton is copied bit for bit); KVM_SIGMA_FIXED -> params->sigma.
 * With weights == KVM_WEIGHTS_AVERAGE every g_j is 1 (w_j = 1/|S|; pivot and sigma
 * are not used).
 *   K, V        in   (B, H_kv, N, d)
 *   set_start, pivot, n_sets  in   as written by kvm_identify_sets (entries are
 *               clamped to the slice, so inconsistent maps cannot cause
 *               out-of-range accesses)
 *   K_out,V_out out  (B, H_kv, capacity, d) dtype; row s < min(M, capacity) is
 *               set s; other rows are not written.  fp32 accumulation, one
 *               round-to-nearest-even to dtype.
 *   w_opt       out  (B, H_kv, N) float32 or NULL: key weight of every token
 *               (positions not covered by a stored set are not written)
 *   ws          the work plan (first set of every 64-token tile of a slice, and the
 *               slice's sets of more than 512 tokens, which a whole workgroup merges) is
 *               built there before the merge kernels run
 */
kvm_status kvm_merge(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V,
                     const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets,
                     void *K_out, void *V_out, float *w_opt, void *ws, size_t ws_bytes, void *stream);

/*
 * Decode-time companion of kvm_merge (the paper runs its method on the prefilled cache and says
 * nothing of decoding; this call only avoids redoing work whose result is already known).  After
 * kvm_attn_mass_append, kvm_sim_append and kvm_identify_sets on the grown sequence, most sets of
 * the new maps are sets of the previous maps: same first token, same end, same pivot, hence the
 * same merged state (Def. 4.2 Eq. (4)-(6) depend on nothing else).  Their rows are moved to their
 * new index inside K_out / V_out; only the other sets are merged again.  The result equals what
 * kvm_merge gives on the new maps, bit for bit.
 *   K, V          in      (B, H_kv, N, d): rows of tokens that existed at the previous call unchanged
 *   prev_set_id, prev_set_start, prev_pivot, prev_n_sets
 *                 in      the maps K_out / V_out were merged with (as kvm_identify_sets wrote them;
 *                         buffers different from the new maps)
 *   set_start, pivot, n_sets  in   the new maps
 *   K_out, V_out  in/out  (B, H_kv, capacity, d): the compacted cache of the previous maps on entry,
 *                         of the new maps on return
 *   n_changed_opt out     (B, H_kv) int32 or NULL: sets that were merged again
 *   ws            kvm_workspace_bytes(shape, params) is enough
 * params (weights, sigma, value scaling) must be those of the previous merge.  Not for w_opt.
 */
kvm_status kvm_merge_refresh(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V,
                             const int32_t *prev_set_id, const int32_t *prev_set_start,
                             const int32_t *prev_pivot, const int32_t *prev_n_sets, const int32_t *set_start,
                             const int32_t *pivot, const int32_t *n_sets, void *K_out, void *V_out,
                             int32_t *n_changed_opt, void *ws, size_t ws_bytes, void *stream);

/*
 * kvm_merge for callers that cannot allocate device memory or may not call an allocator
 * where they run: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, kernels and results as kvm_merge, without the workspace: the
 * work plan (per slice one int32 per 64-token tile, one per possible set of more than 512
 * tokens, and three more) is kept in a
 * buffer built into the library, KVM_MERGE_STATIC_MAX_PLAN_ENTRIES int32 (8 MiB) on every
 * GPU the library has run this call on, held until the process ends.  The call allocates
 * nothing and frees nothing.
 *   - B * H_kv * (ceil(N / 64) + floor(N / 513) + 3) > KVM_MERGE_STATIC_MAX_PLAN_ENTRIES returns
 *     KVM_ERR_WORKSPACE before any launch (use kvm_merge with a workspace then).
 *   - The buffer belongs to the device that is current at the call (the device the tensors
 *     live on); its address is looked up on the first call on that device.
 *   - All calls on one GPU share the one buffer: two calls whose kernels may overlap on
 *     that GPU (different streams, different threads) race on it.  Calls on one stream,
 *     one after the other, are safe; the buffer keeps the last call's plan and needs no
 *     clearing, since every entry that is read is written by the same call first.
 */
#define KVM_MERGE_STATIC_MAX_PLAN_ENTRIES (1 << 21)
kvm_status kvm_merge_static(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V,
                            const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets,
                            void *K_out, void *V_out, float *w_opt, void *stream);

/*
 * Comparison workload, not part of the method: eviction by aggregated attention score, the
 * selection policy of the heavy-hitter methods the paper measures itself against (Section 2.3;
 * Section 4.2 compares average weighted merging with it at the same budget).  Per slice it
 * keeps floor(budget n) tokens: the last floor(recent_ratio n) and those with the largest
 * `mass` among the others (ties: lower index), and gathers their rows in sequence order.
 * Nothing is merged.  params is validated as for the other calls; its heavy_ratio, threshold
 * and merge fields are not used.
 *   K, V     in   (B, H_kv, N, d)
 *   mass     in   (B, H_kv, N) float32
 *   kept     out  (B, H_kv, capacity) int32: kept positions, ascending; -1 beyond n_kept
 *   n_kept   out  (B, H_kv) int32
 *   K_out, V_out  out  (B, H_kv, capacity, d): row s = row kept[s] of K / V, bit for bit;
 *            rows >= n_kept are not written
 * capacity = kvm_out_capacity(); ws as for kvm_identify_sets.
 */
kvm_status kvm_evict(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V,
                     const float *mass, int32_t *kept, int32_t *n_kept, void *K_out, void *V_out,
                     void *ws, size_t ws_bytes, void *stream);

/*
 * Second comparison workload, not part of the method: value-only merging.  Section 2.3 says of
 * the value-merging scheme the paper compares with only that the value states about to be
 * evicted are merged into the conserved ones; the reading built here: the selection is
 * kvm_evict's; keys of evicted tokens are dropped; every evicted token's value goes to the kept
 * token nearest to it by position (equal distances: the later one), and a kept token's new
 * value is the plain mean of its own value and those that went to it (fp32 sums, one rounding
 * to the cache type; a kept token that receives nothing keeps its bits).
 * Arguments, layouts, workspace and errors exactly as for kvm_evict; V_out holds the means.
 */
kvm_status kvm_evict_merge_values(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V,
                                  const float *mass, int32_t *kept, int32_t *n_kept, void *K_out, void *V_out,
                                  void *ws, size_t ws_bytes, void *stream);

/*
 * Per-kernel timing for benchmarks (not part of the method; no citation).  While
 * enabled, every kernel the three calls launch is bracketed by two HIP events
 * recorded on the launch stream, so the time is that of the kernel alone on the
 * stream it runs on.  This is the library's only state and the only place where
 * it creates anything (host-side event objects, in kvm_profile_enable):
 *   kvm_profile_enable(max_launches)  creates 2*max_launches events; launches
 *       beyond that are not timed.  Call with no library work in flight.
 *   kvm_profile_collect(out, max)     waits for the recorded events, writes one
 *       record per kernel name (at most max), returns the number of records,
 *       and clears the recording so that it can be filled again.
 *   kvm_profile_disable()             destroys the events.
 * Not thread-safe: enable, launch and collect from one thread.  Launches on a stream that is
 * being captured into a HIP graph are not timed (nothing is recorded into the graph).
 */
typedef struct {
    char name[48];            /* kernel name, e.g. "attn_colsum_kernel"          */
    int32_t launches;         /* timed launches since the last collect          */
    float total_ms;           /* sum of their durations in milliseconds         */
} kvm_kernel_time;

kvm_status kvm_profile_enable(int32_t max_launches);
int32_t kvm_profile_collect(kvm_kernel_time *out, int32_t max_records);
kvm_status kvm_profile_disable(void);

/* Message of the calling thread's last failed call ("" if none).  Static storage. */
const char *kvm_last_error(void);

/* Library version, "major.minor.patch". */
const char *kvm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVM_H */
