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

#ifdef __cplusplus
}
#endif
#endif
