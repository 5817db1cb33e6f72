/*
 * csv_decode.h — C ABI of the certified sub-vocabulary LM-head path (CSV-Decode) for AMD MI355X (gfx950).
 *
 * One decode step, per sequence: score a centroid-plus-radius upper bound for every vocabulary cluster,
 * open the clusters that could still reach the top-k or carry more than eps of the softmax mass, score
 * only those clusters' rows of W, certify (exact top-k, eps-softmax), and fall back to all V rows when
 * certification fails within the row budget.
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers owned by the caller; h_* are HOST pointers owned by the
 *     caller.  The library never frees caller memory and keeps no reference to h_* after a call returns.
 *   - W and h are bfloat16 bit patterns (uint16_t); everything else is float32 / int32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  csv_decode_step,
 *     csv_bounds and csv_full_logits only enqueue work: outputs are valid once the caller has
 *     synchronised the stream.  They allocate nothing and never synchronise.
 *   - Every function returns CSV_OK (0) or a negative error code; csv_last_error() returns a
 *     thread-local message for the last failure.  No C++ exception crosses the boundary.
 *   - A csv_workspace serves one call at a time; calls sharing a workspace must be stream-ordered.
 */
#ifndef CSV_DECODE_H
#define CSV_DECODE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CSV_OK       0
#define CSV_EINVAL  (-1)   /* bad argument value */
#define CSV_ENOMEM  (-2)   /* device or host allocation failed */
#define CSV_EHIP    (-3)   /* a HIP runtime call failed */
#define CSV_ESHAPE  (-4)   /* shape outside what the kernels support, or workspace too small */

/* csv_step_out.d_flags bits */
#define CSV_FLAG_TOPK_CERT     1u   /* Definition 1 holds: returned top-k equals the full-vocabulary top-k */
#define CSV_FLAG_SOFTMAX_CERT  2u   /* Theorem 2 holds: total variation of the sub-vocabulary softmax <= eps */
#define CSV_FLAG_FALLBACK      4u   /* all V rows were scored for this sequence */
#define CSV_FLAG_SOFTMAX_RELAXED 16u /* the softmax tail bound holds only at the relaxed tolerance 2*eps (Section IV,
                                       fallback levels); never set together with SOFTMAX_CERT */
#define CSV_FLAG_INVALID_INPUT 8u   /* ||h||^2 is not finite (other outputs of the sequence are cleared) */
#define CSV_FLAG_ABORTED      32u   /* the step could not finish this sequence: a bounded device-side wait ran out (see
                                       csv_workspace_set_spin_limit); its other outputs are undefined.  Set alone. */

#define CSV_SCHEDULE_ROUNDS 0   /* the round-based schedule: tests at round boundaries (see csv_decode_step) */
#define CSV_SCHEDULE_ALG1   1   /* Algorithm 1's own order: one cluster per iteration, the tests after every opening */

#define CSV_COMBINE_ALL 0   /* certified when every enabled certificate holds */
#define CSV_COMBINE_ANY 1   /* certified when any enabled certificate holds (Algorithm 1 stops on either) */

#define CSV_MAX_K        1024   /* largest k */
#define CSV_MAX_CLUSTERS 8192   /* largest C */
#define CSV_MAX_ROUNDS 8         /* most scoring rounds of a sequence on the sub-vocabulary path */
#define CSV_MAX_BATCH    256    /* largest B */
#define CSV_MAX_BIAS_TABLE 8    /* most entries per cluster of the top-m bias table */

typedef struct csv_index csv_index;          /* opaque: permuted W', b', centroids, radii, bias maxima, sizes */
typedef struct csv_workspace csv_workspace;  /* opaque: per-step device scratch */

typedef struct {
    int iters;                   /* Lloyd iterations to run (0 = keep the starting assignment) */
    const int32_t* h_init_labels;/* HOST int32[V] starting cluster of each token, or NULL */
    const int32_t* h_init_rows;  /* HOST int32[C] tokens whose rows are the starting centroids; used when
                                    h_init_labels is NULL.  Both NULL: the seeding rule is C tokens evenly spread over
                                    the vocabulary, token floor(c * V / C) for cluster c */
    float radius_slack;          /* rho >= 0: stored radius = roundup_f32(R_c(1+rho) + rho*||mu_c||) */
    int   centroid_bf16;         /* nonzero: store the centroids rounded to bfloat16 (nearest even) and measure the radii
                                    to the rounded values: the bound stays valid, the bound kernels read half the bytes */
    int   spherical;             /* nonzero: spherical K-means (rows compared by direction: largest cosine) and the angular
                                    bound in place of Eq. "cluster_bound" (Section III, spherical clustering metrics);
                                    see csv_index_set_angular.  Not together with centroid_bf16 or bias_table_m */
    int   bias_table_m;          /* >= 2: build the top-m bias table (Section III, "Advanced Theoretical Improvements", bias
                                    binning; at most CSV_MAX_BIAS_TABLE); 0 or 1: the plain bound */
} csv_build_opts;

/*
 * Offline preprocessing (Section III-A.1, Section IV "Offline Preprocessing").
 * Clusters the rows of W into C clusters by Lloyd's k-means (nearest centroid in squared Euclidean distance,
 * ties to the smaller cluster id; an empty cluster keeps its centroid; the distances are evaluated as
 * ||mu_c||^2 - 2 <W_i,mu_c> with an MFMA product in float32, so two centroids whose distances to a row agree to
 * about 1e-5 of ||mu||^2 may be told apart differently than in exact arithmetic), then forms for every cluster the
 * centroid mu_c = mean of its rows (stored float32), the radius R_c = max_i ||W_i - mu_c||_2 measured to the
 * stored centroid, the bias maximum max_i b_i, and the row permutation that makes every cluster a contiguous
 * range of rows (clusters in id order, tokens inside a cluster by ascending id).  The index keeps its own
 * permuted copy of W and b: the caller may free d_W / d_b afterwards.
 *   d_W  DEVICE bf16[V*d] row-major, original token order.   d_b  DEVICE float32[V] or NULL (no bias).
 *   Requires d % 8 == 0, 1 <= C <= min(V, CSV_MAX_CLUSTERS).
 * Synchronises the stream before returning.  On error *out is NULL.
 */
int csv_build_index(const uint16_t* d_W, const float* d_b, int V, int d, int C,
                    const csv_build_opts* opts, void* stream, csv_index** out);

/*
 * Import an index whose metadata was computed elsewhere (tests, reload of saved metadata; Section IV keeps
 * the metadata in a file).  h_mu float32[C*d], h_R float32[C], h_bmax float32[C], h_n int32[C] rows per
 * cluster (sum V), h_perm int32[V]: permuted row -> original token id, clusters contiguous in id order.
 * Gathers the permuted copy of W and b on the device.  Synchronises the stream before returning.
 */
int csv_index_from_arrays(const uint16_t* d_W, const float* d_b, int V, int d, int C,
                          const float* h_mu, const float* h_R, const float* h_bmax,
                          const int32_t* h_n, const int32_t* h_perm, void* stream, csv_index** out);

/*
 * Switch an imported index to bfloat16 centroids: every value of h_mu must already be a bfloat16 (the radii must have
 * been measured to those rounded centroids); otherwise CSV_EINVAL and the index is unchanged.  Allocates C*d*2 bytes.
 */
int csv_index_use_bf16_centroids(csv_index* idx, void* stream);

/*
 * Top-m bias table (Section III, "Advanced Theoretical Improvements": bias binning).  Per cluster m pairs
 * (rho_j, beta_j): the m-1 tokens with the largest biases (equal biases: smaller token id first) each with their own
 * distance to the centroid and their own bias, and one pair for all other tokens (their largest distance, their
 * largest bias); unused pairs are (0, -inf).  With a table the bound of a cluster is
 *   U_c(h) = <mu_c,h> + max_j (rho_j ||h|| + beta_j)  <=  <mu_c,h> + R_c ||h|| + max_i b_i,
 * still an upper bound of every logit of the cluster, so both certificates hold unchanged.
 * csv_index_set_bias_table installs a table computed elsewhere (h_table HOST float32[C*m*2], m = 0 removes the table);
 * csv_index_get_bias_table returns m and, when h_table is not NULL, the table.  Both synchronise.
 */
int csv_index_set_bias_table(csv_index* idx, int m, const float* h_table, void* stream);
int csv_index_get_bias_table(const csv_index* idx, int* m, float* h_table);

/*
 * Angular index (Section III, "Advanced Theoretical Improvements": spherical clustering metrics).  The centroid array
 * holds unit directions m_c = normalise(sum_i W_i / ||W_i||); per cluster four numbers: cos and sin of the angular radius
 * theta_c = max_i angle(W_i, m_c), the largest and the smallest row norm (all stored with slack on the safe side).
 * For a row w of cluster c the angle to h is at least phi - theta_c, phi = angle(m_c, h), hence with t = <m_c,h>
 *   <w,h> <= rho (t cos(theta_c) + sqrt(||h||^2 - t^2) sin(theta_c))   when phi > theta_c,    <w,h> <= rho_max ||h||   otherwise,
 * rho = rho_max when the bracket is positive, rho_min when it is negative; the cluster bound adds the largest bias.
 * (As printed in the paper the bound, ||h|| (||mu_c|| cos(theta_c) + sin(theta_c)), does not depend on the direction of h and
 * cannot order clusters; it is the form above with cos(phi) and sin(phi) replaced by 1.)
 * csv_index_set_angular installs h_ang HOST float32[C*4] on an index whose centroids are such directions (NULL removes it);
 * csv_index_get_angular reports whether the index is angular and, when h_ang is not NULL, copies the four numbers per cluster.
 */
int csv_index_set_angular(csv_index* idx, const float* h_ang, void* stream);
int csv_index_get_angular(const csv_index* idx, int* present, float* h_ang);

/* Copy the metadata back to HOST buffers of the sizes above (any pointer may be NULL to skip it). Synchronous. */
int csv_index_export(const csv_index* idx, float* h_mu, float* h_R, float* h_bmax, int32_t* h_n, int32_t* h_perm);
int csv_index_dims(const csv_index* idx, int* V, int* d, int* C);
void csv_index_free(csv_index* idx);

/*
 * Scratch for steps of up to B_max sequences in which at most K_cap_rows rows per sequence are scored on
 * the sub-vocabulary path (the budget K_max of Algorithm 1 may not exceed it).  Allocates device memory:
 * about B_max*(8*K_cap_rows + 4*V + 24*C) bytes.
 */
int csv_workspace_create(const csv_index* idx, int B_max, int K_cap_rows, csv_workspace** out);
void csv_workspace_free(csv_workspace* ws);

typedef struct {
    int   k;           /* top-k size, 0..CSV_MAX_K; 0 disables the top-k certificate */
    float eps;         /* softmax tolerance; <= 0 disables the softmax certificate, >= 1 always holds.  The top-p
                          (nucleus) certificate of Section III is this test in delta form: eps = delta / (1 + delta)
                          certifies a coverage of 1 - eps by the scored rows */
    int   K_max_rows;  /* budget K_max of Algorithm 1: a sequence whose planned |S| exceeds it falls back */
    int   combine;     /* CSV_COMBINE_ALL or CSV_COMBINE_ANY */
    /* Fallback levels (Section IV, "Runtime Optimization"); all zero = the two-round schedule with the full
       vocabulary as the only fallback. */
    int   max_rounds;      /* scoring rounds allowed, 2..CSV_MAX_ROUNDS (0 is read as 2): later rounds plan as round 1 does */
    int   delta_clusters;  /* partial expansion S' = S + Delta C: when a planned set exceeds K_max_rows, open the next
                              clusters of the bound order instead (at most this many, not past the planned set, rows
                              within the budget) and test again; 0 = off */
    int   relax;           /* nonzero: when no further expansion is possible, accept a step whose softmax tail bound
                              holds at 2*eps (flag SOFTMAX_RELAXED) before falling back to the full vocabulary */
    float top_p;           /* nucleus mass for d_nucleus, in 0..1 (0 = none); see csv_step_out */
    int   schedule;        /* CSV_SCHEDULE_ROUNDS (0, the fast path) or CSV_SCHEDULE_ALG1: open clusters one at a time in
                              bound order and stop at the first prefix that certifies (Algorithm 1, Section III-C), i.e.
                              with the smallest certifying set of clusters.  A reference mode: one thread block per
                              sequence does all the work of that sequence, so it is slow when many clusters are needed.
                              The budget is tested before a cluster's rows are scored (more than K_max_rows -> fallback).
                              d_rounds reports the clusters opened; d_sel_clusters lists them in bound order; entries of
                              d_ids / d_logits past the rows scored are -1 / -inf (softmax-only certification may stop
                              with fewer than k rows).  No fallback levels.  CSV_ESHAPE when the cluster data (24 bytes
                              per cluster) and h do not fit a compute unit's LDS next to 36 KB of staging. */
} csv_step_params;

typedef struct {
    int32_t*  d_ids;          /* [B*k]  original token ids, by logit descending, equal logits by id ascending */
    float*    d_logits;       /* [B*k]  their logits */
    float*    d_lse;          /* [B]    log-sum-exp over the scored rows (over all V after fallback) */
    uint32_t* d_flags;        /* [B]    CSV_FLAG_* */
    int32_t*  d_n_rows;       /* [B]    rows scored, |S| (V after fallback) */
    int32_t*  d_n_clusters;   /* [B]    clusters opened (C after fallback) */
    int32_t*  d_rounds;       /* [B] or NULL: scoring rounds used on the sub-vocabulary path (0..max_rounds) */
    int32_t*  d_sel_clusters; /* [B*C] or NULL: opened cluster ids (first n_clusters entries): the round-0 clusters
                                 in bound order, then the clusters of each later round by ascending id; untouched
                                 on fallback */
    unsigned long long* d_fallback_count; /* or NULL: incremented once per sequence that falls back */
    /* Certified sub-vocabulary distribution over the returned list, in its order (Section III, top-p certification;
       each may be NULL; k >= 1):
       p~_t = exp(l_t - lse), the probabilities of the softmax restricted to the scored rows S; with SOFTMAX_CERT (or after
       fallback, eps = 0) the full-vocabulary probability of token t lies in [(1 - eps) p~_t, p~_t], because at most eps of
       the mass lies outside S;  the running sums of p~ in list order;  the length of the shortest prefix of the list whose
       running sum reaches params.top_p (0: top_p is 0, or the list ends before that mass): that prefix covers at least
       (1 - eps) top_p of the full-vocabulary mass.  Entries past the scored rows (k > |S|) have p~ = 0. */
    float*    d_probs;        /* [B*k] */
    float*    d_cum;          /* [B*k] */
    int32_t*  d_nucleus;      /* [B]   */
} csv_step_out;

/*
 * One certified decode step for B sequences (Algorithm 1, evaluated as a two-round schedule; Definitions 1-2,
 * Theorems 1-2, Eq. "cluster_bound").  Per sequence, with clusters in descending bound order (equal bounds:
 * smaller id first), P(m) rows in the first m clusters and T(m) the log of the cluster-wise tail bound
 * sum_{j>m} n_j exp(U_j):
 *   round 0: open m0 = min{m : P(m) >= max(k,1)}; theta0 = k-th largest scored logit, Z0 = log-sum-exp;
 *            top-k test: no unopened cluster, or next bound < theta0 (strict); softmax test:
 *            T(m0) - Z0 <= ln(eps/(1-eps)).  Certified -> done.
 *   round 1: a = #{c : U_c >= theta0}; s = min{m >= m0 : T(m) - Z0 <= ln(eps/(1-eps))};
 *            m1 = max(a,s) under ALL, min(a,s) under ANY (a disabled test drops out); open up to m1, test again.
 *   The budget is tested on the planned size before scoring: P(m) > K_max_rows -> fallback; tests failing after
 *   round 1 -> fallback.  Fallback scores all V rows (flags FALLBACK|TOPK_CERT|SOFTMAX_CERT).
 *   With max_rounds > 2, delta_clusters > 0 or relax set, the fallback levels of Section IV apply before the full
 *   vocabulary: every later round plans from the theta and Z of all rows scored so far; a plan over the budget is
 *   replaced by a partial expansion; when neither fits, the relaxed tolerance is tried (see csv_step_params).
 *   d_h  DEVICE bf16[B*d].  1 <= B <= workspace B_max.  Returns CSV_EINVAL when both certificates are disabled,
 *   k > V, or K_max_rows exceeds the workspace capacity.
 */
int csv_decode_step(csv_workspace* ws, const csv_index* idx, const uint16_t* d_h, int B,
                    const csv_step_params* params, const csv_step_out* out, void* stream);

/*
 * Cluster upper bounds only (Eq. "cluster_bound"): d_U[b*C+c] = <mu_c,h_b> + R_c*||h_b||_2 + max_{i in c} b_i
 * (-inf for an empty cluster), d_hnorm[b] = ||h_b||_2.  d_U DEVICE float32[B*C], d_hnorm DEVICE float32[B] or NULL.
 */
int csv_bounds(csv_workspace* ws, const csv_index* idx, const uint16_t* d_h, int B,
               float* d_U, float* d_hnorm, void* stream);

/*
 * csv_bounds for callers that cannot allocate device memory and hold no workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same results as csv_bounds, bit for bit.  Calls no
 * hipMalloc / hipFree and nothing that allocates.  The only scratch the bound kernels use (partial sums of the batched
 * product, more than 4 sequences) lives in an 8 MiB device array inside the library, one copy per GPU, held until the
 * process ends: for more than 4 sequences B * C may be at most about 2^21 / KS, KS <= 32 being the number of K slices
 * chosen for the shape (e.g. up to B = 42 at C = 4096, d = 4608, where KS = 12 beyond 32 sequences; up to B = 64 at C = 1024, d = 4096, where KS = 32); larger requests fail with CSV_ESHAPE and a message,
 * nothing is launched.  The device of the index must be current.  Every call on a GPU shares that GPU's array: calls
 * that overlap on one GPU (different streams, different threads) race on it; stream-ordered calls are safe.  Nothing
 * in the array needs to start at zero (every partial sum is written before it is read).
 */
int csv_bounds_static(const csv_index* idx, const uint16_t* d_h, int B, float* d_U, float* d_hnorm, void* stream);

/*
 * Full-vocabulary logits (Eq. "logit"): d_logits[b*V + i] = <W_i,h_b> + b_i for every ORIGINAL token id i.
 * d_logits DEVICE float32[B*V].
 */
int csv_full_logits(csv_workspace* ws, const csv_index* idx, const uint16_t* d_h, int B,
                    float* d_logits, void* stream);

/*
 * Failure handling of the device-side waits.  The blocks that run round 1 and the fallback as one kernel stay
 * resident, wait for round 0 to be settled when they share its launch, and separate their phases with grid barriers;
 * a block polls such a wait at most `polls` times (default
 * 2^22, about a second), then sets an abort flag that makes every block leave.  Sequences the step had not finished
 * by then carry flag ABORTED; the next csv_decode_step starts from a clean state.  polls = 0 restores the
 * default.  A tiny limit is how the error path is exercised in tests without any kernel failing to exit.
 */
int csv_workspace_set_spin_limit(csv_workspace* ws, int polls);

/*
 * What follows round 0 (further rounds, the full vocabulary for fallback sequences) runs either as one set of blocks
 * that stay resident and leave at once when no sequence needs them (for small batches they ride in the round-0
 * launch, parked until round 0 is settled: two launches per step on the common path of an easy workload; otherwise
 * they are a launch of their own), or as one launch per phase (kernel boundaries instead of grid barriers: faster whenever that work
 * is actually needed).  By default (min_batch = 0) every step follows the recent steps: per-phase launches when at
 * least two of the last eight needed the tail (a device-side bit history mirrored to pinned host memory and read
 * without synchronising, so it may lag a few steps).  min_batch > 0 fixes the choice: batches of at least min_batch
 * sequences use per-phase launches, smaller ones the single kernel (a value above CSV_MAX_BATCH: always the single
 * kernel; 1: always per-phase).  Results do not depend on the choice.
 */
int csv_workspace_set_tail_split(csv_workspace* ws, int min_batch);

/*
 * Measurement support (not part of the method): time the stages of csv_decode_step with HIP events recorded on
 * the step's own stream.  csv_profile_begin allocates events for max_steps steps and switches recording on;
 * each following csv_decode_step on this workspace records CSV_PROFILE_STAGES+1 events (steps beyond max_steps
 * are not recorded).  csv_profile_end synchronises, writes the summed milliseconds of every stage to
 * h_stage_ms[CSV_PROFILE_STAGES] and the number of recorded steps to *h_steps, frees the events and switches
 * recording off.  Stage order: bounds; round 0 (seed selection, gathered GEMV over the seed prefix and its
 * certification; one launch, which for small batches also carries the parked blocks of the tail); the tail (round-1
 * GEMV and certification, full-vocabulary product and top-k for fallback sequences) when it is launched separately.
 * A stage's time runs from the end of the previous stage to its own end, so it includes its launch gap.
 */
#define CSV_PROFILE_STAGES 3
int csv_profile_begin(csv_workspace* ws, int max_steps);
int csv_profile_end(csv_workspace* ws, float* h_stage_ms, int* h_steps);

/*
 * Adaptive row budget (Section IV, "Runtime Optimization": K_max(t+1) = K_max(t) * (1 + alpha * (rho_target -
 * rho_fall(t))), alpha = 0.01, rho_target = 0.02).  Host-side state, no device work.  rho_fall(t) is the fraction of
 * the step's sequences that fell back.  As printed the update lowers the budget when fallbacks exceed the target,
 * which moves the rate away from the target it is meant to hold; literal = 0 uses the sign that gives a negative
 * feedback, K_max * (1 + alpha * (rho_fall - rho_target)), literal = 1 the printed expression.
 * csv_kmax_init: K0 rows to start from; the value handed to a step is floor(K_max) kept inside [K_min, K_cap].
 * csv_kmax_update: feed one step's fallback count (0 <= n_fallback <= n_sequences, n_sequences >= 1); returns the
 * budget in rows for the next step, or a negative CSV_E* code.
 */
typedef struct {
    double K_max;          /* unrounded controller state */
    double alpha, rho_target;
    int    K_min, K_cap;
    int    literal;
} csv_kmax_ctl;
int csv_kmax_init(csv_kmax_ctl* c, int K0, int K_min, int K_cap, double alpha, double rho_target, int literal);
int csv_kmax_update(csv_kmax_ctl* c, int n_fallback, int n_sequences);

const char* csv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CSV_DECODE_H */
