/*
 * pcg_oracle.h -- plain CPU reference ("oracle") for PCG group-level verification.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, double-precision, loop-by-loop
 * statement of what the hot path computes.  It exists so that the HIP library
 * can be checked against something written straight from the paper.  Only the
 * test-suite, the smoke check and the CPU-baseline leg of the benchmark may
 * call it; the product never does.  It shares no code with the HIP path.
 *
 * Everything is double precision, host pointers, no blocking, no fusion:
 *   - row softmax with temperature            (Sec. 2.2 "Complexity and memory";
 *                                              temperature: Sec. 3.1)
 *   - overlap-aware group probabilities       (Eq. 5, equal-split weights Eq. 3)
 *   - group accept test                       (Eq. 7)
 *   - group residual, drawn by inverse CDF    (Eq. 8, Proposition)
 *   - token inside the emitted group          (Eq. 10)
 *   - control flow of one speculative step    (Algorithm 1)
 *   - Philox4x32-10 counter-based generator   (Salmon et al., SC'11)
 *   - residual sampling by thinning           (Eq. 9)
 *   - draft-side proposal coupling            (Eq. 6)
 *   - general per-entry weights               (Eq. 2, Eq. 4)
 *   - similarity-group construction           (Sec. 2.1, Eq. 1)
 *
 * Naming: the paper's body calls the target model q and the draft p, its group
 * distributions Q_c (target) and P_c (draft).  To keep the two apart this file
 * speaks of T[g] (target group probability) and D[g] (draft group
 * probability): accept ratio = T/D, residual = max(0, T - D).
 *
 * Pins: every function here is pinned by the CPU tests (library softmax, sparse
 * mat-vec, textbook token-level speculative sampling as the singleton-group
 * case, exact enumeration of the emitted-group law on tiny vocabularies,
 * chi-square on 10^6 sampled steps, published Philox known-answer vectors).
 * Nothing about audio quality is pinned: that needs the paper's models and data.
 */
#ifndef PCG_ORACLE_H
#define PCG_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { PCG_REF_F32 = 0, PCG_REF_BF16 = 1 };

enum {
  PCG_REF_OK = 0,
  PCG_REF_ERR_ARG = -1,     /* null pointer, bad size, bad dtype, temperature <= 0   */
  PCG_REF_ERR_CSR = -2,     /* row_ptr not monotone, member out of range, bad mult   */
  PCG_REF_ERR_ROW = -3,     /* a logits row has no finite entry or holds NaN / +inf  */
  PCG_REF_ERR_NOMEM = -4
};

/* Width of the band around a decision threshold inside which a uniform draw is
 * reported as a near-tie (on the unit interval). */
#define PCG_REF_NEAR_TIE 1e-6

/* Optional per-call trace; every pointer may be NULL. */
typedef struct {
  double *T_prop;      /* [B*K]  T_i[g] of the proposed group at evaluated positions, NaN elsewhere */
  double *D_prop;      /* [B*K]  D_i[g] likewise                                                     */
  uint8_t *near_acc;   /* [B*K]  1 where |u*D - T| < 1e-6*D at an evaluated position                 */
  uint8_t *near_grp;   /* [B]    1 where u_grp is within 1e-6 of an inner edge of the chosen bin     */
  uint8_t *near_tok;   /* [B]    same for the token draw                                             */
  uint8_t *flags;      /* [B]    bit0: residual total was <= 0, fell back to T                        */
                       /*        bit1: a proposed group had D == 0                                    */
  double *res_S;       /* [B]    un-normalised residual total S on the decision row                   */
  double *res_lo;      /* [B]    normalised lower edge of the chosen group's bin                      */
  double *res_hi;      /* [B]    normalised upper edge                                                */
  double *R_norm;      /* [B*G]  R[g]/S on the decision row (tiny problems only)                      */
} pcg_ref_trace;

/* Philox4x32-10: out = philox(ctr, key). */
void pcg_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Uniforms of position (b, i) under (seed, offset): counter = (offset_lo,
 * offset_hi, b, i), key = (seed_lo, seed_hi); u = (word >> 8) * 2^-24. */
void pcg_ref_uniforms(uint64_t seed, uint64_t offset, uint32_t b, uint32_t i,
                      double *u_acc, double *u_grp, double *u_tok);

/* prob[t] = softmax(logits / temperature)[t], t in [0, V). */
int pcg_ref_softmax_row(const void *logits, int dtype, int64_t V, double temperature, double *prob);

/* mult[v] = number of CSR entries equal to v (0 for uncovered tokens). */
int pcg_ref_count_mult(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                       int32_t *mult);

/* Tokens in no group become their own singleton group, appended in ascending
 * token order after the G given groups.  Call with out_* == NULL to get the
 * sizes (*out_G, *out_nnz) first.  out_row_ptr [*out_G+1], out_members
 * [*out_nnz], out_mult [V]. */
int pcg_ref_canonicalize(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                         int32_t *out_G, int64_t *out_nnz, int32_t *out_row_ptr,
                         int32_t *out_members, int32_t *out_mult);

/* 0 if the CSR is usable on the hot path: row_ptr[0]==0 and non-decreasing,
 * members in [0,V), mult[v] equals the entry count of v and is >= 1. */
int pcg_ref_validate(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                     const int32_t *mult);

/* out[r*G + g] = sum over members t of group g of softmax(row r)[t] / mult[t]   (Eq. 5). */
int pcg_ref_group_probs(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                        const int32_t *mult, const void *logits, int dtype, int64_t rows,
                        int64_t row_stride, double temperature, double *out);

/* One speculative step for B sequences with the uniforms given explicitly:
 * u_acc [B*K], u_grp [B*(K+1)], u_tok [B*(K+1)], indexed by (b, position). */
int pcg_ref_verify_u(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                     const int32_t *mult, const void *target_logits, const void *draft_logits,
                     int dtype, int32_t B, int32_t K, int64_t tgt_batch_stride,
                     int64_t tgt_pos_stride, int64_t dft_batch_stride, int64_t dft_pos_stride,
                     double temperature, const int32_t *prop_tokens, const int32_t *prop_groups,
                     const double *u_acc, const double *u_grp, const double *u_tok,
                     int32_t *accept_len, int32_t *out_tokens, int32_t *out_groups,
                     const pcg_ref_trace *trace, int32_t nthreads);

/* Same, uniforms drawn from Philox(seed, offset).  *threads_used (may be NULL)
 * receives the number of threads that ran. */
int pcg_ref_verify(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                   const int32_t *mult, const void *target_logits, const void *draft_logits,
                   int dtype, int32_t B, int32_t K, int64_t tgt_batch_stride,
                   int64_t tgt_pos_stride, int64_t dft_batch_stride, int64_t dft_pos_stride,
                   double temperature, const int32_t *prop_tokens, const int32_t *prop_groups,
                   uint64_t seed, uint64_t offset, int32_t *accept_len, int32_t *out_tokens,
                   int32_t *out_groups, const pcg_ref_trace *trace, int32_t nthreads,
                   int32_t *threads_used);

/* ------------------------------------------------------------------------- */
/* Residual sampling via thinning (Sec. 2.2 "Residual sampling via thinning", */
/* Eq. 9): the paper's own way to draw from the group residual without        */
/* enumerating the groups.  Same law as the enumerated residual above, a       */
/* different sample path, hence entry points of its own.                       */
/* ------------------------------------------------------------------------- */

/* Reverse index token -> groups holding it (the paper's S(t)): tok_ptr [V+1],
 * tok_groups [nnz]; a token's groups appear in ascending CSR entry position, a
 * group listing the token twice appears twice. */
int pcg_ref_reverse_index(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                          int32_t *tok_ptr, int32_t *tok_groups);

/* Draws of thinning trial `trial` (0, 1, ...) at position (b, i): Philox block
 * with counter (offset_lo, offset_hi, b, i | (trial + 1) << 16); word 0 -> u_y,
 * word 1 >> 8 -> k24 (a 24-bit integer), word 2 -> u_a, word 3 -> u_tok. */
void pcg_ref_trial_uniforms(uint64_t seed, uint64_t offset, uint32_t b, uint32_t i, uint32_t trial,
                            double *u_y, uint32_t *k24, double *u_a, double *u_tok);

typedef struct {
  int32_t y;          /* token drawn from the target distribution                         */
  int32_t group;      /* one of the groups holding y, by the weights w_{k,y}              */
  int32_t accepted;   /* 1 iff u_a < [1 - D[group] / T[group]]_+                          */
  int32_t token;      /* token inside `group` by Eq. (10) (computed whether accepted or not) */
  double T, D;        /* group probabilities of `group`                                   */
  uint8_t near;       /* bit0: u_y near an inner bin edge; bit1: accept draw near its
                         threshold; bit2: u_tok near an inner edge                        */
} pcg_ref_trial;

/* One trial with explicit draws, on given token distributions q (target) and
 * p (draft), both [V].  With p == NULL nothing is subtracted (bonus row):
 * the trial is always accepted. */
int pcg_ref_thin_trial(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                       const int32_t *mult, const int32_t *tok_ptr, const int32_t *tok_groups,
                       const double *q, const double *p, double u_y, uint32_t k24, double u_a,
                       double u_tok, pcg_ref_trial *out);

/* One speculative step for B sequences, reject branch by thinning.  The accept
 * scan and its draws are those of pcg_ref_verify.  On a reject at position i
 * trials 0, 1, ... are run until one is accepted (at most max_trials; then the
 * last candidate is emitted and flags bit1 is set).  On the bonus position the
 * token is drawn from the target row and its group by the weights (Algorithm 1,
 * last step; Eq. 6), using the draws of trial 0.
 *   trials [B]  number of trials run (0 on the bonus position)
 *   flags  [B]  bit0: some decision of the emitted path was within 1e-6 of its
 *               threshold; bit1: max_trials reached
 *   near_acc [B*K] as in pcg_ref_trace (may be NULL) */
int pcg_ref_verify_thinning(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                            const int32_t *mult, const int32_t *tok_ptr,
                            const int32_t *tok_groups, const void *target_logits,
                            const void *draft_logits, int dtype, int32_t B, int32_t K,
                            int64_t tgt_batch_stride, int64_t tgt_pos_stride,
                            int64_t dft_batch_stride, int64_t dft_pos_stride, double temperature,
                            const int32_t *prop_tokens, const int32_t *prop_groups, uint64_t seed,
                            uint64_t offset, int32_t *accept_len, int32_t *out_tokens,
                            int32_t *out_groups, int32_t *trials, uint8_t *flags,
                            uint8_t *near_acc, int32_t max_trials, int32_t nthreads);

/* ------------------------------------------------------------------------- */
/* General weights (Sec. 2.2, Eq. 2 and Eq. 4): any non-negative w_{k,t} with    */
/* sum over the groups holding t equal to 1, one per CSR entry, instead of the  */
/* equal split 1/N(t).  T[k] = sum_j q(t_j) w_j, Eq. (10) becomes q(t) w_{k,t}  */
/* / T[k], and the group label of a token is drawn by its weights.  The _w      */
/* entry points below are the functions above with this extra argument (NULL =  */
/* equal split, which is exactly what the plain names compute).                 */
/* ------------------------------------------------------------------------- */

typedef struct {
  const float *weights;     /* [nnz] w of each CSR entry (fp32, read exactly)          */
  const float *tok_weights; /* [nnz] the same weights in reverse-index order; needed by */
                            /* thinning and proposals only                              */
} pcg_ref_weights;

/* 0 iff every weight is in [0, 1 + tol] and the weights of each token sum to 1 within tol. */
int pcg_ref_validate_weights(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                             const float *weights, double tol);

/* tok_weights [nnz]: weights permuted into the order of pcg_ref_reverse_index. */
int pcg_ref_reverse_weights(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                            const float *weights, float *tok_weights);

int pcg_ref_group_probs_w(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                          const int32_t *mult, const pcg_ref_weights *wt, const void *logits,
                          int dtype, int64_t rows, int64_t row_stride, double temperature,
                          double *out);

int pcg_ref_verify_u_w(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                       const int32_t *mult, const pcg_ref_weights *wt, const void *target_logits,
                       const void *draft_logits, int dtype, int32_t B, int32_t K,
                       int64_t tgt_batch_stride, int64_t tgt_pos_stride, int64_t dft_batch_stride,
                       int64_t dft_pos_stride, double temperature, const int32_t *prop_tokens,
                       const int32_t *prop_groups, const double *u_acc, const double *u_grp,
                       const double *u_tok, int32_t *accept_len, int32_t *out_tokens,
                       int32_t *out_groups, const pcg_ref_trace *trace, int32_t nthreads);

int pcg_ref_verify_w(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                     const int32_t *mult, const pcg_ref_weights *wt, const void *target_logits,
                     const void *draft_logits, int dtype, int32_t B, int32_t K,
                     int64_t tgt_batch_stride, int64_t tgt_pos_stride, int64_t dft_batch_stride,
                     int64_t dft_pos_stride, double temperature, const int32_t *prop_tokens,
                     const int32_t *prop_groups, uint64_t seed, uint64_t offset,
                     int32_t *accept_len, int32_t *out_tokens, int32_t *out_groups,
                     const pcg_ref_trace *trace, int32_t nthreads, int32_t *threads_used);

/* The membership entry of y is drawn by the inverse CDF of y's weights (reverse-index order)
 * at u = k24 / 2^24; near bit0 also covers that draw. */
int pcg_ref_thin_trial_w(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                         const int32_t *mult, const pcg_ref_weights *wt, const int32_t *tok_ptr,
                         const int32_t *tok_groups, const double *q, const double *p, double u_y,
                         uint32_t k24, double u_a, double u_tok, pcg_ref_trial *out);

int pcg_ref_verify_thinning_w(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                              const int32_t *mult, const pcg_ref_weights *wt,
                              const int32_t *tok_ptr, const int32_t *tok_groups,
                              const void *target_logits, const void *draft_logits, int dtype,
                              int32_t B, int32_t K, int64_t tgt_batch_stride,
                              int64_t tgt_pos_stride, int64_t dft_batch_stride,
                              int64_t dft_pos_stride, double temperature,
                              const int32_t *prop_tokens, const int32_t *prop_groups,
                              uint64_t seed, uint64_t offset, int32_t *accept_len,
                              int32_t *out_tokens, int32_t *out_groups, int32_t *trials,
                              uint8_t *flags, uint8_t *near_acc, int32_t max_trials,
                              int32_t nthreads);

/* ------------------------------------------------------------------------- */
/* Draft-side proposal coupling (Sec. 2.2 "Proposal coupling and acceptance",  */
/* Eq. 6; Algorithm 1, the two sampling steps at the top of the loop): a token */
/* x ~ p_i, then a group label among the groups holding x by the weights       */
/* w_{k,x} (equal split: each of the N(x) membership entries equally likely),  */
/* so that Pr(label = k) = D_i[k].                                             */
/* ------------------------------------------------------------------------- */

/* Draws of the proposal at position (b, i): Philox block with counter
 * (offset_lo, offset_hi, b, i | 0xFFFF0000) -- a trial field no thinning trial
 * uses, so the proposal is independent of every draw of the verifier under the
 * same (seed, offset); word 0 -> u_x, word 1 >> 8 -> k24. */
void pcg_ref_propose_uniforms(uint64_t seed, uint64_t offset, uint32_t b, uint32_t i, double *u_x,
                              uint32_t *k24);

/* Proposals for B sequences x K positions from explicit draws u_x [B*K] and
 * k24 [B*K] (24-bit integers): x = inverse CDF of softmax(draft row / temperature)
 * at u_x (ascending token order, first running sum strictly above u_x * total);
 * group = tok_groups[tok_ptr[x] + ((k24 * N(x)) >> 24)].  near [B*K] (may be
 * NULL): u_x within 1e-6 of an inner edge of the chosen token's bin. */
int pcg_ref_propose_u(int32_t V, int32_t G, const int32_t *mult, const int32_t *tok_ptr,
                      const int32_t *tok_groups, const void *draft_logits, int dtype, int32_t B,
                      int32_t K, int64_t dft_batch_stride, int64_t dft_pos_stride,
                      double temperature, const double *u_x, const uint32_t *k24,
                      int32_t *prop_tokens, int32_t *prop_groups, uint8_t *near);

/* Same with the draws of pcg_ref_propose_uniforms at positions pos0 .. pos0+K-1
 * (pos0: position index of the first row, for drafts that call once per token). */
int pcg_ref_propose(int32_t V, int32_t G, const int32_t *mult, const int32_t *tok_ptr,
                    const int32_t *tok_groups, const void *draft_logits, int dtype, int32_t B,
                    int32_t K, int32_t pos0, int64_t dft_batch_stride, int64_t dft_pos_stride,
                    double temperature, uint64_t seed, uint64_t offset, int32_t *prop_tokens,
                    int32_t *prop_groups, uint8_t *near, int32_t nthreads);

/* ------------------------------------------------------------------------- */
/* Acoustic Similarity Groups (Sec. 2.1, Eq. 1): the group of token t is every  */
/* token whose embedding has cosine similarity above theta with t's; the group  */
/* set is the collection of distinct such sets.                                 */
/* ------------------------------------------------------------------------- */

/* Width of the band around theta inside which a pair's similarity is reported as
 * a near-tie of the membership decision. */
#define PCG_REF_ASG_NEAR 1e-5

/* unit[v][k] = emb[v][k] / ||emb[v]||, computed in double and rounded once to
 * bfloat16 (nearest, ties to even); an all-zero row stays zero. */
int pcg_ref_asg_normalize(const float *emb, int32_t V, int32_t d, uint16_t *unit_bf16);

/* cos of tokens a and b: the double-precision dot product of their bf16 unit
 * vectors (the vectors are taken as given: the similarity both sides threshold
 * is that of the stored bf16 values). */
double pcg_ref_asg_similarity(const uint16_t *unit_bf16, int32_t d, int32_t a, int32_t b);

/* Members of G(t), ascending: every v with similarity(t, v) > theta, and t itself
 * (its similarity with itself is 1 up to the bf16 rounding of the unit vector).
 * members_out [V]; *near_pairs (may be NULL) counts the v != t whose similarity
 * is within PCG_REF_ASG_NEAR of theta. */
int pcg_ref_asg_row(const uint16_t *unit_bf16, int32_t V, int32_t d, float theta, int32_t t,
                    int32_t *members_out, int32_t *count, int32_t *near_pairs);

/* All groups: G(t) for t = 0 .. V-1, keeping each distinct set once, in order of
 * first appearance; CSR with members ascending, mult = entry counts.  row_ptr
 * [V+1] (the first *out_G + 1 entries are written), members [members_capacity],
 * mult [V], seed_of [V] (may be NULL): the token whose group each kept row is.
 * near_rows [V] (may be NULL): 1 where some pair of row t is a near-tie.  If
 * *out_nnz exceeds members_capacity the sizes are still returned, nothing else
 * is written and the status is PCG_REF_ERR_NOMEM: call again with more room. */
int pcg_ref_asg_build(const uint16_t *unit_bf16, int32_t V, int32_t d, float theta,
                      int32_t *out_G, int64_t *out_nnz, int32_t *row_ptr, int32_t *members,
                      int64_t members_capacity, int32_t *mult, int32_t *seed_of,
                      uint8_t *near_rows, int32_t nthreads);

/* Eq. (1) as the paper writes it, on the embeddings themselves: the cosine similarity of the
 * float32 rows a and b of emb, every step in double (dot product and both norms summed in
 * ascending k, one square root each, one division).  No rounding of the unit vectors: this is
 * the definition the bf16 routines above approximate.  A zero row has cosine 0 with everything. */
double pcg_ref_asg_cosine(const float *emb, int32_t d, int32_t a, int32_t b);

/* Members of G(t) by Eq. (1), ascending: every v with cosine(t, v) > theta (strict), and t
 * itself (cos(t, t) = 1).  members_out [V].  cos_out (may be NULL) [V] receives every cosine of
 * the row (cos_out[t] = 1), so that a caller can measure how far from theta a pair lies. */
int pcg_ref_asg_row_exact(const float *emb, int32_t V, int32_t d, double theta, int32_t t,
                          int32_t *members_out, int32_t *count, double *cos_out);

/* All groups by Eq. (1) on the embeddings themselves: G(t) from pcg_ref_asg_row_exact for
 * t = 0 .. V-1, the distinct sets once, in order of first appearance; outputs and the
 * members_capacity rule as for pcg_ref_asg_build.  near_rows [V] (may be NULL): 1 where some
 * cosine of row t lies within 1e-12 of theta (a decision that the order of summation could
 * turn). */
int pcg_ref_asg_build_exact(const float *emb, int32_t V, int32_t d, double theta,
                            int32_t *out_G, int64_t *out_nnz, int32_t *row_ptr,
                            int32_t *members, int64_t members_capacity, int32_t *mult,
                            int32_t *seed_of, uint8_t *near_rows, int32_t nthreads);

/* Proposals with general weights: the group label by the inverse CDF of the token's weights
 * at u = k24 / 2^24; near also covers that draw. */
int pcg_ref_propose_u_w(int32_t V, int32_t G, const int32_t *mult, const pcg_ref_weights *wt,
                        const int32_t *tok_ptr, const int32_t *tok_groups,
                        const void *draft_logits, int dtype, int32_t B, int32_t K,
                        int64_t dft_batch_stride, int64_t dft_pos_stride, double temperature,
                        const double *u_x, const uint32_t *k24, int32_t *prop_tokens,
                        int32_t *prop_groups, uint8_t *near);

int pcg_ref_propose_w(int32_t V, int32_t G, const int32_t *mult, const pcg_ref_weights *wt,
                      const int32_t *tok_ptr, const int32_t *tok_groups, const void *draft_logits,
                      int dtype, int32_t B, int32_t K, int32_t pos0, int64_t dft_batch_stride,
                      int64_t dft_pos_stride, double temperature, uint64_t seed, uint64_t offset,
                      int32_t *prop_tokens, int32_t *prop_groups, uint8_t *near, int32_t nthreads);

#ifdef __cplusplus
}
#endif
#endif
