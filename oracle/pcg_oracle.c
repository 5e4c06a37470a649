/*
 * pcg_oracle.c -- plain CPU reference for PCG group-level verification.
 * TEST INFRASTRUCTURE ONLY; see pcg_oracle.h.  Double precision, plain loops,
 * steps in the order the paper gives them.
 */
#include "pcg_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as   */
/* easy as 1, 2, 3", SC'11).                                                 */
/* ------------------------------------------------------------------------- */

void pcg_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
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

void pcg_ref_uniforms(uint64_t seed, uint64_t offset, uint32_t b, uint32_t i,
                      double *u_acc, double *u_grp, double *u_tok) {
  uint32_t ctr[4] = {(uint32_t)offset, (uint32_t)(offset >> 32), b, i};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  pcg_ref_philox4x32_10(ctr, key, w);
  const double scale = 1.0 / 16777216.0; /* 2^-24: the draw is exact in fp32 and fp64 */
  if (u_acc) *u_acc = (double)(w[0] >> 8) * scale;
  if (u_grp) *u_grp = (double)(w[1] >> 8) * scale;
  if (u_tok) *u_tok = (double)(w[2] >> 8) * scale;
}

/* ------------------------------------------------------------------------- */
/* Row softmax.                                                              */
/* ------------------------------------------------------------------------- */

static double logit_at(const void *base, int dtype, int64_t idx) {
  if (dtype == PCG_REF_F32) return (double)((const float *)base)[idx];
  /* bfloat16: the upper 16 bits of an IEEE binary32 */
  uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

static int softmax_row_at(const void *base, int dtype, int64_t first, int64_t V,
                          double temperature, double *prob) {
  double mx = -INFINITY;
  for (int64_t t = 0; t < V; ++t) {
    double x = logit_at(base, dtype, first + t) / temperature;
    if (isnan(x) || x == INFINITY) return PCG_REF_ERR_ROW;
    prob[t] = x;
    if (x > mx) mx = x;
  }
  if (mx == -INFINITY) return PCG_REF_ERR_ROW;
  double Z = 0.0;
  for (int64_t t = 0; t < V; ++t) {
    prob[t] = exp(prob[t] - mx);
    Z += prob[t];
  }
  for (int64_t t = 0; t < V; ++t) prob[t] /= Z;
  return PCG_REF_OK;
}

int pcg_ref_softmax_row(const void *logits, int dtype, int64_t V, double temperature,
                        double *prob) {
  if (!logits || !prob || V < 1 || !(temperature > 0.0)) return PCG_REF_ERR_ARG;
  if (dtype != PCG_REF_F32 && dtype != PCG_REF_BF16) return PCG_REF_ERR_ARG;
  return softmax_row_at(logits, dtype, 0, V, temperature, prob);
}

/* ------------------------------------------------------------------------- */
/* Group membership.                                                         */
/* ------------------------------------------------------------------------- */

static int csr_shape_ok(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members) {
  if (row_ptr[0] != 0) return 0;
  for (int32_t g = 0; g < G; ++g)
    if (row_ptr[g + 1] < row_ptr[g]) return 0;
  for (int32_t j = 0; j < row_ptr[G]; ++j)
    if (members[j] < 0 || members[j] >= V) return 0;
  return 1;
}

int pcg_ref_count_mult(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                       int32_t *mult) {
  if (V < 1 || G < 0 || !row_ptr || !mult || (G > 0 && row_ptr[G] > 0 && !members))
    return PCG_REF_ERR_ARG;
  if (!csr_shape_ok(V, G, row_ptr, members)) return PCG_REF_ERR_CSR;
  for (int32_t v = 0; v < V; ++v) mult[v] = 0;
  for (int32_t j = 0; j < row_ptr[G]; ++j) mult[members[j]] += 1;
  return PCG_REF_OK;
}

int pcg_ref_canonicalize(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                         int32_t *out_G, int64_t *out_nnz, int32_t *out_row_ptr,
                         int32_t *out_members, int32_t *out_mult) {
  if (V < 1 || G < 0 || !row_ptr || !out_G || !out_nnz) return PCG_REF_ERR_ARG;
  if (G > 0 && row_ptr[G] > 0 && !members) return PCG_REF_ERR_ARG;
  if (!csr_shape_ok(V, G, row_ptr, members)) return PCG_REF_ERR_CSR;
  int32_t *cnt = (int32_t *)calloc((size_t)V, sizeof(int32_t));
  if (!cnt) return PCG_REF_ERR_NOMEM;
  int32_t nnz = row_ptr[G];
  for (int32_t j = 0; j < nnz; ++j) cnt[members[j]] += 1;
  int32_t uncovered = 0;
  for (int32_t v = 0; v < V; ++v)
    if (cnt[v] == 0) ++uncovered;
  *out_G = G + uncovered;
  *out_nnz = (int64_t)nnz + uncovered;
  if (out_row_ptr && out_members && out_mult) {
    for (int32_t g = 0; g <= G; ++g) out_row_ptr[g] = row_ptr[g];
    for (int32_t j = 0; j < nnz; ++j) out_members[j] = members[j];
    int32_t g = G, j = nnz;
    for (int32_t v = 0; v < V; ++v) {
      if (cnt[v] == 0) {        /* a token in no group acts as its own group */
        out_members[j++] = v;
        out_row_ptr[++g] = j;
        out_mult[v] = 1;
      } else {
        out_mult[v] = cnt[v];
      }
    }
  }
  free(cnt);
  return PCG_REF_OK;
}

int pcg_ref_validate(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                     const int32_t *mult) {
  if (V < 1 || G < 1 || !row_ptr || !members || !mult) return PCG_REF_ERR_ARG;
  if (!csr_shape_ok(V, G, row_ptr, members)) return PCG_REF_ERR_CSR;
  int32_t *cnt = (int32_t *)calloc((size_t)V, sizeof(int32_t));
  if (!cnt) return PCG_REF_ERR_NOMEM;
  for (int32_t j = 0; j < row_ptr[G]; ++j) cnt[members[j]] += 1;
  int rc = PCG_REF_OK;
  for (int32_t v = 0; v < V; ++v)
    if (cnt[v] < 1 || cnt[v] != mult[v]) rc = PCG_REF_ERR_CSR;
  free(cnt);
  return rc;
}

/* Eq. (5): the probability a row gives to group g when every token's mass is
 * split equally over the mult[t] groups that hold it. */
/* prob(t) * w_{k,t} for CSR entry j (token t = members[j]): the caller's weight of
 * that entry (Eq. 2) if weights are given, else the equal split prob(t) / N(t) (Eq. 3). */
static double entry_mass(const double *prob, const int32_t *members, const int32_t *mult,
                         const float *weights, int32_t j) {
  int32_t t = members[j];
  return weights ? prob[t] * (double)weights[j] : prob[t] / (double)mult[t];
}

static double group_prob(const double *prob, const int32_t *row_ptr, const int32_t *members,
                         const int32_t *mult, const float *weights, int32_t g) {
  double s = 0.0;
  for (int32_t j = row_ptr[g]; j < row_ptr[g + 1]; ++j)
    s += entry_mass(prob, members, mult, weights, j);
  return s;
}

static const float *entry_weights(const pcg_ref_weights *wt) { return wt ? wt->weights : NULL; }

int pcg_ref_validate_weights(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                             const float *weights, double tol) {
  if (V < 1 || G < 1 || !row_ptr || !members || !weights) return PCG_REF_ERR_ARG;
  if (!csr_shape_ok(V, G, row_ptr, members)) return PCG_REF_ERR_CSR;
  double *sum = (double *)calloc((size_t)V, sizeof(double));
  if (!sum) return PCG_REF_ERR_NOMEM;
  int rc = PCG_REF_OK;
  for (int32_t j = 0; j < row_ptr[G]; ++j) {
    double w = (double)weights[j];
    if (!(w >= 0.0) || w > 1.0 + tol) rc = PCG_REF_ERR_CSR;
    sum[members[j]] += w;
  }
  for (int32_t v = 0; v < V; ++v)
    if (fabs(sum[v] - 1.0) > tol) rc = PCG_REF_ERR_CSR;
  free(sum);
  return rc;
}

int pcg_ref_group_probs(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                        const int32_t *mult, const void *logits, int dtype, int64_t rows,
                        int64_t row_stride, double temperature, double *out) {
  return pcg_ref_group_probs_w(V, G, row_ptr, members, mult, NULL, logits, dtype, rows, row_stride,
                               temperature, out);
}

int pcg_ref_group_probs_w(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                          const int32_t *mult, const pcg_ref_weights *wt, const void *logits,
                          int dtype, int64_t rows, int64_t row_stride, double temperature,
                          double *out) {
  if (!row_ptr || !members || !mult || !logits || !out) return PCG_REF_ERR_ARG;
  if (V < 1 || G < 1 || rows < 0 || !(temperature > 0.0)) return PCG_REF_ERR_ARG;
  if (dtype != PCG_REF_F32 && dtype != PCG_REF_BF16) return PCG_REF_ERR_ARG;
  int rc = pcg_ref_validate(V, G, row_ptr, members, mult);
  if (rc) return rc;
  double *prob = (double *)malloc((size_t)V * sizeof(double));
  if (!prob) return PCG_REF_ERR_NOMEM;
  for (int64_t r = 0; r < rows && rc == PCG_REF_OK; ++r) {
    rc = softmax_row_at(logits, dtype, r * row_stride, V, temperature, prob);
    if (rc) break;
    for (int32_t g = 0; g < G; ++g)
      out[r * (int64_t)G + g] = group_prob(prob, row_ptr, members, mult, entry_weights(wt), g);
  }
  free(prob);
  return rc;
}

/* ------------------------------------------------------------------------- */
/* One speculative step (Algorithm 1) for one sequence.                      */
/* ------------------------------------------------------------------------- */

typedef struct {
  int32_t V, G;
  const int32_t *row_ptr, *members, *mult;
  const float *weights;
  const void *tgt, *dft;
  int dtype;
  int32_t B, K;
  int64_t tbs, tps, dbs, dps;
  double temperature;
  const int32_t *prop_tokens, *prop_groups;
  const double *u_acc, *u_grp, *u_tok;
  int32_t *accept_len, *out_tokens, *out_groups;
  const pcg_ref_trace *trace;
} step_args;

/* scratch: q [V], p [V], Tg [G], Dg [G], R [G] */
static int verify_sequence(const step_args *a, int32_t b, double *q, double *p, double *Tg,
                           double *Dg, double *R) {
  const int32_t K = a->K, G = a->G;
  const pcg_ref_trace *tr = a->trace;
  int32_t *otok = a->out_tokens + (int64_t)b * (K + 1);
  int32_t *ogrp = a->out_groups + (int64_t)b * (K + 1);
  for (int32_t i = 0; i <= K; ++i) otok[i] = ogrp[i] = -1;
  if (tr) {
    for (int32_t i = 0; i < K; ++i) {
      if (tr->T_prop) tr->T_prop[(int64_t)b * K + i] = NAN;
      if (tr->D_prop) tr->D_prop[(int64_t)b * K + i] = NAN;
      if (tr->near_acc) tr->near_acc[(int64_t)b * K + i] = 0;
    }
    if (tr->near_grp) tr->near_grp[b] = 0;
    if (tr->near_tok) tr->near_tok[b] = 0;
    if (tr->flags) tr->flags[b] = 0;
  }

  /* Draft positions in order; stop at the first rejected group. */
  int32_t i = 0;
  int rc;
  while (i < K) {
    rc = softmax_row_at(a->tgt, a->dtype, b * a->tbs + i * a->tps, a->V, a->temperature, q);
    if (rc) return rc;
    rc = softmax_row_at(a->dft, a->dtype, b * a->dbs + i * a->dps, a->V, a->temperature, p);
    if (rc) return rc;
    int32_t g = a->prop_groups[(int64_t)b * K + i];
    if (g < 0 || g >= G) return PCG_REF_ERR_ARG;
    double Tprop = group_prob(q, a->row_ptr, a->members, a->mult, a->weights, g);
    double Dprop = group_prob(p, a->row_ptr, a->members, a->mult, a->weights, g);
    double u = a->u_acc[(int64_t)b * K + i];
    /* Eq. (7): accept iff u < min(1, T/D), written without the division so
     * that D == 0 is defined: T > 0 accepts, T == 0 rejects. */
    int accept = (u * Dprop < Tprop);
    if (tr) {
      if (tr->T_prop) tr->T_prop[(int64_t)b * K + i] = Tprop;
      if (tr->D_prop) tr->D_prop[(int64_t)b * K + i] = Dprop;
      if (tr->near_acc && fabs(u * Dprop - Tprop) < PCG_REF_NEAR_TIE * Dprop)
        tr->near_acc[(int64_t)b * K + i] = 1;
      if (tr->flags && Dprop == 0.0) tr->flags[b] |= 2;
    }
    if (!accept) break;
    otok[i] = a->prop_tokens[(int64_t)b * K + i]; /* the draft token stands for its group */
    ogrp[i] = g;
    ++i;
  }
  a->accept_len[b] = i;

  /* Decision row i: the rejected position, or the bonus position K. */
  if (i == K) {
    rc = softmax_row_at(a->tgt, a->dtype, b * a->tbs + i * a->tps, a->V, a->temperature, q);
    if (rc) return rc;
  }
  for (int32_t g = 0; g < G; ++g) Tg[g] = group_prob(q, a->row_ptr, a->members, a->mult, a->weights, g);
  if (i < K) {
    for (int32_t g = 0; g < G; ++g) Dg[g] = group_prob(p, a->row_ptr, a->members, a->mult, a->weights, g);
    for (int32_t g = 0; g < G; ++g) R[g] = Tg[g] > Dg[g] ? Tg[g] - Dg[g] : 0.0; /* Eq. (8) */
  } else {
    for (int32_t g = 0; g < G; ++g) R[g] = Tg[g]; /* bonus: nothing was proposed here */
  }
  double S = 0.0;
  for (int32_t g = 0; g < G; ++g) S += R[g];
  if (!(S > 0.0)) { /* cannot happen in exact arithmetic; fall back to T */
    S = 0.0;
    for (int32_t g = 0; g < G; ++g) { R[g] = Tg[g]; S += R[g]; }
    if (tr && tr->flags) tr->flags[b] |= 1;
  }

  /* Inverse CDF over groups in ascending id: the first g whose running total
   * strictly exceeds u*S.  Zero-mass groups can never be chosen. */
  double ug = a->u_grp[(int64_t)b * (K + 1) + i];
  double goal = ug * S;
  double cum = 0.0, lo = 0.0, hi = 0.0;
  int32_t gs = -1, last_pos = -1;
  for (int32_t g = 0; g < G; ++g) {
    if (R[g] > 0.0) last_pos = g;
    double nxt = cum + R[g];
    if (gs < 0 && nxt > goal) { gs = g; lo = cum; hi = nxt; }
    cum = nxt;
  }
  if (gs < 0) { /* rounding at the top end: the last group that has mass */
    gs = last_pos < 0 ? 0 : last_pos;
    lo = cum - R[gs];
    hi = cum;
  }
  if (tr) {
    if (tr->res_S) tr->res_S[b] = S;
    if (tr->res_lo) tr->res_lo[b] = lo / S;
    if (tr->res_hi) tr->res_hi[b] = hi / S;
    if (tr->near_grp) {
      int near_lo = lo > 0.0 && (goal - lo) < PCG_REF_NEAR_TIE * S;
      int near_hi = hi < cum && (hi - goal) < PCG_REF_NEAR_TIE * S;
      tr->near_grp[b] = (uint8_t)(near_lo || near_hi);
    }
    if (tr->R_norm)
      for (int32_t g = 0; g < G; ++g) tr->R_norm[(int64_t)b * G + g] = R[g] / S;
  }

  /* Eq. (10): token inside the emitted group, proportional to q(t) w_{g,t}
   * (q(t)/mult[t] under the equal split) over the group's members in CSR order. */
  int32_t beg = a->row_ptr[gs], end = a->row_ptr[gs + 1];
  double C = 0.0;
  for (int32_t j = beg; j < end; ++j) C += entry_mass(q, a->members, a->mult, a->weights, j);
  double ut = a->u_tok[(int64_t)b * (K + 1) + i];
  double tgoal = ut * C;
  double tc = 0.0, tlo = 0.0, thi = 0.0;
  int32_t js = -1, jlast = -1;
  for (int32_t j = beg; j < end; ++j) {
    double c = entry_mass(q, a->members, a->mult, a->weights, j);
    if (c > 0.0) jlast = j;
    double nxt = tc + c;
    if (js < 0 && nxt > tgoal) { js = j; tlo = tc; thi = nxt; }
    tc = nxt;
  }
  if (js < 0) { js = jlast; } /* rounding at the top end: the last member that has mass */
  if (tr && tr->near_tok && C > 0.0 && thi > 0.0) {
    int near_lo = tlo > 0.0 && (tgoal - tlo) < PCG_REF_NEAR_TIE * C;
    int near_hi = thi < tc && (thi - tgoal) < PCG_REF_NEAR_TIE * C;
    tr->near_tok[b] = (uint8_t)(near_lo || near_hi);
  }
  otok[i] = js < 0 ? -1 : a->members[js]; /* -1: the group holds no mass at all (invalid rows only) */
  ogrp[i] = gs;
  return PCG_REF_OK;
}

int pcg_ref_verify_u(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                     const int32_t *mult, const void *target_logits, const void *draft_logits,
                     int dtype, int32_t B, int32_t K, int64_t tgt_batch_stride,
                     int64_t tgt_pos_stride, int64_t dft_batch_stride, int64_t dft_pos_stride,
                     double temperature, const int32_t *prop_tokens, const int32_t *prop_groups,
                     const double *u_acc, const double *u_grp, const double *u_tok,
                     int32_t *accept_len, int32_t *out_tokens, int32_t *out_groups,
                     const pcg_ref_trace *trace, int32_t nthreads) {
  return pcg_ref_verify_u_w(V, G, row_ptr, members, mult, NULL, target_logits, draft_logits, dtype,
                            B, K, tgt_batch_stride, tgt_pos_stride, dft_batch_stride,
                            dft_pos_stride, temperature, prop_tokens, prop_groups, u_acc, u_grp,
                            u_tok, accept_len, out_tokens, out_groups, trace, nthreads);
}

int pcg_ref_verify_u_w(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                       const int32_t *mult, const pcg_ref_weights *wt, const void *target_logits,
                       const void *draft_logits, int dtype, int32_t B, int32_t K,
                       int64_t tgt_batch_stride, int64_t tgt_pos_stride, int64_t dft_batch_stride,
                       int64_t dft_pos_stride, double temperature, const int32_t *prop_tokens,
                       const int32_t *prop_groups, const double *u_acc, const double *u_grp,
                       const double *u_tok, int32_t *accept_len, int32_t *out_tokens,
                       int32_t *out_groups, const pcg_ref_trace *trace, int32_t nthreads) {
  if (!row_ptr || !members || !mult || !target_logits || !draft_logits || !prop_tokens ||
      !prop_groups || !u_acc || !u_grp || !u_tok || !accept_len || !out_tokens || !out_groups)
    return PCG_REF_ERR_ARG;
  if (V < 1 || G < 1 || B < 0 || K < 1 || !(temperature > 0.0)) return PCG_REF_ERR_ARG;
  if (dtype != PCG_REF_F32 && dtype != PCG_REF_BF16) return PCG_REF_ERR_ARG;
  int rc = pcg_ref_validate(V, G, row_ptr, members, mult);
  if (rc) return rc;

  step_args a;
  a.V = V; a.G = G; a.row_ptr = row_ptr; a.members = members; a.mult = mult;
  a.weights = entry_weights(wt);
  a.tgt = target_logits; a.dft = draft_logits; a.dtype = dtype; a.B = B; a.K = K;
  a.tbs = tgt_batch_stride; a.tps = tgt_pos_stride; a.dbs = dft_batch_stride;
  a.dps = dft_pos_stride; a.temperature = temperature;
  a.prop_tokens = prop_tokens; a.prop_groups = prop_groups;
  a.u_acc = u_acc; a.u_grp = u_grp; a.u_tok = u_tok;
  a.accept_len = accept_len; a.out_tokens = out_tokens; a.out_groups = out_groups;
  a.trace = trace;

  if (nthreads < 1) nthreads = 1;
  int status = PCG_REF_OK;
#ifdef _OPENMP
#pragma omp parallel num_threads(nthreads)
#endif
  {
    size_t nd = 2 * (size_t)V + 3 * (size_t)G;
    double *buf = (double *)malloc(nd * sizeof(double));
    if (!buf) {
#ifdef _OPENMP
#pragma omp critical
#endif
      status = PCG_REF_ERR_NOMEM;
    }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
    for (int32_t b = 0; b < B; ++b) {
      if (!buf || status != PCG_REF_OK) continue;
      int r = verify_sequence(&a, b, buf, buf + V, buf + 2 * (size_t)V,
                              buf + 2 * (size_t)V + G, buf + 2 * (size_t)V + 2 * (size_t)G);
      if (r) {
#ifdef _OPENMP
#pragma omp critical
#endif
        status = r;
      }
    }
    free(buf);
  }
  return status;
}

int pcg_ref_verify(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                   const int32_t *mult, const void *target_logits, const void *draft_logits,
                   int dtype, int32_t B, int32_t K, int64_t tgt_batch_stride,
                   int64_t tgt_pos_stride, int64_t dft_batch_stride, int64_t dft_pos_stride,
                   double temperature, const int32_t *prop_tokens, const int32_t *prop_groups,
                   uint64_t seed, uint64_t offset, int32_t *accept_len, int32_t *out_tokens,
                   int32_t *out_groups, const pcg_ref_trace *trace, int32_t nthreads,
                   int32_t *threads_used) {
  return pcg_ref_verify_w(V, G, row_ptr, members, mult, NULL, target_logits, draft_logits, dtype, B,
                          K, tgt_batch_stride, tgt_pos_stride, dft_batch_stride, dft_pos_stride,
                          temperature, prop_tokens, prop_groups, seed, offset, accept_len,
                          out_tokens, out_groups, trace, nthreads, threads_used);
}

int pcg_ref_verify_w(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                     const int32_t *mult, const pcg_ref_weights *wt, const void *target_logits,
                     const void *draft_logits, int dtype, int32_t B, int32_t K,
                     int64_t tgt_batch_stride, int64_t tgt_pos_stride, int64_t dft_batch_stride,
                     int64_t dft_pos_stride, double temperature, const int32_t *prop_tokens,
                     const int32_t *prop_groups, uint64_t seed, uint64_t offset,
                     int32_t *accept_len, int32_t *out_tokens, int32_t *out_groups,
                     const pcg_ref_trace *trace, int32_t nthreads, int32_t *threads_used) {
  if (B < 0 || K < 1) return PCG_REF_ERR_ARG;
  size_t nacc = (size_t)B * (size_t)K, nres = (size_t)B * ((size_t)K + 1);
  double *u = (double *)malloc((nacc + 2 * nres + 1) * sizeof(double));
  if (!u) return PCG_REF_ERR_NOMEM;
  double *u_acc = u, *u_grp = u + nacc, *u_tok = u + nacc + nres;
  for (int32_t b = 0; b < B; ++b) {
    for (int32_t i = 0; i <= K; ++i) {
      double ua, ug, ut;
      pcg_ref_uniforms(seed, offset, (uint32_t)b, (uint32_t)i, &ua, &ug, &ut);
      if (i < K) u_acc[(size_t)b * K + i] = ua;
      u_grp[(size_t)b * (K + 1) + i] = ug;
      u_tok[(size_t)b * (K + 1) + i] = ut;
    }
  }
  if (nthreads < 1) nthreads = 1;
#ifndef _OPENMP
  nthreads = 1;
#endif
  if (threads_used) *threads_used = nthreads;
  int rc = pcg_ref_verify_u_w(V, G, row_ptr, members, mult, wt, target_logits, draft_logits, dtype,
                              B, K, tgt_batch_stride, tgt_pos_stride, dft_batch_stride,
                              dft_pos_stride, temperature, prop_tokens, prop_groups, u_acc, u_grp,
                              u_tok, accept_len, out_tokens, out_groups, trace, nthreads);
  free(u);
  return rc;
}

/* ------------------------------------------------------------------------- */
/* Residual sampling via thinning (Eq. 9).                                   */
/* ------------------------------------------------------------------------- */

int pcg_ref_reverse_index(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                          int32_t *tok_ptr, int32_t *tok_groups) {
  if (V < 1 || G < 1 || !row_ptr || !members || !tok_ptr || !tok_groups) return PCG_REF_ERR_ARG;
  if (!csr_shape_ok(V, G, row_ptr, members)) return PCG_REF_ERR_CSR;
  for (int32_t v = 0; v <= V; ++v) tok_ptr[v] = 0;
  for (int32_t j = 0; j < row_ptr[G]; ++j) tok_ptr[members[j] + 1] += 1;
  for (int32_t v = 0; v < V; ++v) tok_ptr[v + 1] += tok_ptr[v];
  int32_t *fill = (int32_t *)calloc((size_t)V, sizeof(int32_t));
  if (!fill) return PCG_REF_ERR_NOMEM;
  for (int32_t g = 0; g < G; ++g)
    for (int32_t j = row_ptr[g]; j < row_ptr[g + 1]; ++j) {
      int32_t t = members[j];
      tok_groups[tok_ptr[t] + fill[t]++] = g;
    }
  free(fill);
  return PCG_REF_OK;
}

int pcg_ref_reverse_weights(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                            const float *weights, float *tok_weights) {
  if (V < 1 || G < 1 || !row_ptr || !members || !weights || !tok_weights) return PCG_REF_ERR_ARG;
  if (!csr_shape_ok(V, G, row_ptr, members)) return PCG_REF_ERR_CSR;
  int32_t *at = (int32_t *)calloc((size_t)V + 1, sizeof(int32_t));
  if (!at) return PCG_REF_ERR_NOMEM;
  for (int32_t j = 0; j < row_ptr[G]; ++j) at[members[j] + 1] += 1;
  for (int32_t v = 0; v < V; ++v) at[v + 1] += at[v];
  /* same visiting order as pcg_ref_reverse_index: ascending CSR entry position */
  for (int32_t j = 0; j < row_ptr[G]; ++j) tok_weights[at[members[j]]++] = weights[j];
  free(at);
  return PCG_REF_OK;
}

void pcg_ref_trial_uniforms(uint64_t seed, uint64_t offset, uint32_t b, uint32_t i, uint32_t trial,
                            double *u_y, uint32_t *k24, double *u_a, double *u_tok) {
  uint32_t ctr[4] = {(uint32_t)offset, (uint32_t)(offset >> 32), b, i | ((trial + 1u) << 16)};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  pcg_ref_philox4x32_10(ctr, key, w);
  const double scale = 1.0 / 16777216.0;
  *u_y = (double)(w[0] >> 8) * scale;
  *k24 = w[1] >> 8;
  *u_a = (double)(w[2] >> 8) * scale;
  *u_tok = (double)(w[3] >> 8) * scale;
}

/* First index whose running sum strictly exceeds u * total (ascending order);
 * the last index with mass if rounding leaves none; -1 if nothing has mass.
 * *near is set when u * total lies within 1e-6 * total of an inner edge of the
 * chosen bin. */
static int64_t inverse_cdf(const double *w, int64_t n, double u, int *near) {
  double total = 0.0;
  for (int64_t k = 0; k < n; ++k) total += w[k];
  double goal = u * total, cum = 0.0, lo = 0.0, hi = 0.0;
  int64_t pick = -1, last = -1;
  for (int64_t k = 0; k < n; ++k) {
    if (w[k] > 0.0) last = k;
    double nxt = cum + w[k];
    if (pick < 0 && nxt > goal) { pick = k; lo = cum; hi = nxt; }
    cum = nxt;
  }
  if (pick < 0) {
    if (last < 0) { *near = 0; return -1; }
    pick = last; lo = cum - w[last]; hi = cum;
  }
  *near = (lo > 0.0 && goal - lo < PCG_REF_NEAR_TIE * total) ||
          (hi < cum && hi - goal < PCG_REF_NEAR_TIE * total);
  return pick;
}

/* Which of the n = N(x) membership entries of token x the 24-bit draw k24 picks
 * (K ~ w_{k,x} over k in S(x), Eq. 6): under the equal split entry (k24 * n) >> 24;
 * with general weights the inverse CDF of the token's weights (reverse-index
 * order) at u = k24 / 2^24.  Returns the offset inside the token's entries, < 0 on
 * error; *near as for inverse_cdf (always 0 under the equal split). */
static int32_t pick_entry(const int32_t *tok_ptr, const float *tok_weights, int64_t x, uint32_t k24,
                          int *near) {
  int32_t n = tok_ptr[x + 1] - tok_ptr[x];
  *near = 0;
  if (n < 1) return -1;
  if (!tok_weights) return (int32_t)(((uint64_t)k24 * (uint64_t)n) >> 24);
  double *w = (double *)malloc((size_t)n * sizeof(double));
  if (!w) return -1;
  for (int32_t e = 0; e < n; ++e) w[e] = (double)tok_weights[tok_ptr[x] + e];
  int64_t e = inverse_cdf(w, n, (double)k24 / 16777216.0, near);
  free(w);
  return (int32_t)e;
}

int pcg_ref_thin_trial(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                       const int32_t *mult, const int32_t *tok_ptr, const int32_t *tok_groups,
                       const double *q, const double *p, double u_y, uint32_t k24, double u_a,
                       double u_tok, pcg_ref_trial *out) {
  return pcg_ref_thin_trial_w(V, G, row_ptr, members, mult, NULL, tok_ptr, tok_groups, q, p, u_y,
                              k24, u_a, u_tok, out);
}

int pcg_ref_thin_trial_w(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                         const int32_t *mult, const pcg_ref_weights *wt, const int32_t *tok_ptr,
                         const int32_t *tok_groups, const double *q, const double *p, double u_y,
                         uint32_t k24, double u_a, double u_tok, pcg_ref_trial *out) {
  if (!row_ptr || !members || !mult || !tok_ptr || !tok_groups || !q || !out || V < 1 || G < 1)
    return PCG_REF_ERR_ARG;
  if (wt && (wt->weights == NULL) != (wt->tok_weights == NULL)) return PCG_REF_ERR_ARG;
  const float *weights = entry_weights(wt);
  int near = 0;
  out->near = 0;
  /* y ~ q */
  int64_t y = inverse_cdf(q, V, u_y, &near);
  if (y < 0) return PCG_REF_ERR_ROW;
  if (near) out->near |= 1;
  /* K ~ w_{.,y}: one of the N(y) membership entries of y, by the weights */
  int32_t e = pick_entry(tok_ptr, wt ? wt->tok_weights : NULL, y, k24, &near);
  if (e < 0) return PCG_REF_ERR_CSR;
  if (near) out->near |= 1;
  int32_t g = tok_groups[tok_ptr[y] + e];
  double T = group_prob(q, row_ptr, members, mult, weights, g);
  double D = p ? group_prob(p, row_ptr, members, mult, weights, g) : 0.0;
  /* accept with probability [1 - D/T]_+, written without the division */
  int accepted = p ? (u_a * T < T - D) : 1;
  if (p && fabs(u_a * T - (T - D)) < PCG_REF_NEAR_TIE * T) out->near |= 2;
  /* token inside the group, Eq. (10) */
  int32_t beg = row_ptr[g], len = row_ptr[g + 1] - beg;
  double *c = (double *)malloc((size_t)(len > 0 ? len : 1) * sizeof(double));
  if (!c) return PCG_REF_ERR_NOMEM;
  for (int32_t j = 0; j < len; ++j) c[j] = entry_mass(q, members, mult, weights, beg + j);
  int64_t js = inverse_cdf(c, len, u_tok, &near);
  free(c);
  if (near) out->near |= 4;
  out->y = (int32_t)y;
  out->group = g;
  out->accepted = accepted;
  out->token = js < 0 ? -1 : members[beg + js];
  out->T = T;
  out->D = D;
  return PCG_REF_OK;
}

int pcg_ref_verify_thinning(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                            const int32_t *mult, const int32_t *tok_ptr,
                            const int32_t *tok_groups, const void *target_logits,
                            const void *draft_logits, int dtype, int32_t B, int32_t K,
                            int64_t tgt_batch_stride, int64_t tgt_pos_stride,
                            int64_t dft_batch_stride, int64_t dft_pos_stride, double temperature,
                            const int32_t *prop_tokens, const int32_t *prop_groups, uint64_t seed,
                            uint64_t offset, int32_t *accept_len, int32_t *out_tokens,
                            int32_t *out_groups, int32_t *trials, uint8_t *flags,
                            uint8_t *near_acc, int32_t max_trials, int32_t nthreads) {
  return pcg_ref_verify_thinning_w(V, G, row_ptr, members, mult, NULL, tok_ptr, tok_groups,
                                   target_logits, draft_logits, dtype, B, K, tgt_batch_stride,
                                   tgt_pos_stride, dft_batch_stride, dft_pos_stride, temperature,
                                   prop_tokens, prop_groups, seed, offset, accept_len, out_tokens,
                                   out_groups, trials, flags, near_acc, max_trials, nthreads);
}

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
                              int32_t nthreads) {
  const float *weights = entry_weights(wt);
  if (!row_ptr || !members || !mult || !tok_ptr || !tok_groups || !target_logits ||
      !draft_logits || !prop_tokens || !prop_groups || !accept_len || !out_tokens ||
      !out_groups || !trials || !flags)
    return PCG_REF_ERR_ARG;
  if (V < 1 || G < 1 || B < 0 || K < 1 || K > 0xFFFF || max_trials < 1 ||
      !(temperature > 0.0))
    return PCG_REF_ERR_ARG;
  if (dtype != PCG_REF_F32 && dtype != PCG_REF_BF16) return PCG_REF_ERR_ARG;
  int rc = pcg_ref_validate(V, G, row_ptr, members, mult);
  if (rc) return rc;
  if (nthreads < 1) nthreads = 1;
  int status = PCG_REF_OK;
#ifdef _OPENMP
#pragma omp parallel num_threads(nthreads)
#endif
  {
    double *q = (double *)malloc(2 * (size_t)V * sizeof(double));
    double *p = q ? q + V : NULL;
    if (!q) {
#ifdef _OPENMP
#pragma omp critical
#endif
      status = PCG_REF_ERR_NOMEM;
    }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
    for (int32_t b = 0; b < B; ++b) {
      if (!q || status != PCG_REF_OK) continue;
      int32_t *otok = out_tokens + (int64_t)b * (K + 1);
      int32_t *ogrp = out_groups + (int64_t)b * (K + 1);
      for (int32_t i = 0; i <= K; ++i) otok[i] = ogrp[i] = -1;
      flags[b] = 0;
      trials[b] = 0;
      int r = PCG_REF_OK;
      /* the accept scan of Algorithm 1, with the draws of pcg_ref_verify */
      int32_t i = 0;
      while (i < K && r == PCG_REF_OK) {
        r = softmax_row_at(target_logits, dtype, b * tgt_batch_stride + i * tgt_pos_stride, V,
                           temperature, q);
        if (r) break;
        r = softmax_row_at(draft_logits, dtype, b * dft_batch_stride + i * dft_pos_stride, V,
                           temperature, p);
        if (r) break;
        int32_t g = prop_groups[(int64_t)b * K + i];
        if (g < 0 || g >= G) { r = PCG_REF_ERR_ARG; break; }
        double Tp = group_prob(q, row_ptr, members, mult, weights, g);
        double Dp = group_prob(p, row_ptr, members, mult, weights, g);
        double ua;
        pcg_ref_uniforms(seed, offset, (uint32_t)b, (uint32_t)i, &ua, NULL, NULL);
        if (near_acc) near_acc[(int64_t)b * K + i] = fabs(ua * Dp - Tp) < PCG_REF_NEAR_TIE * Dp;
        if (!(ua * Dp < Tp)) break;
        otok[i] = prop_tokens[(int64_t)b * K + i];
        ogrp[i] = g;
        ++i;
      }
      if (near_acc)
        for (int32_t k = i + 1; k < K; ++k) near_acc[(int64_t)b * K + k] = 0;
      if (r == PCG_REF_OK) {
        accept_len[b] = i;
        pcg_ref_trial tr;
        double uy, uacc, ut;
        uint32_t k24;
        if (i == K) { /* bonus: token from the target's last row, its group by the weights */
          r = softmax_row_at(target_logits, dtype, b * tgt_batch_stride + i * tgt_pos_stride, V,
                             temperature, q);
          if (r == PCG_REF_OK) {
            pcg_ref_trial_uniforms(seed, offset, (uint32_t)b, (uint32_t)i, 0, &uy, &k24, &uacc, &ut);
            r = pcg_ref_thin_trial_w(V, G, row_ptr, members, mult, wt, tok_ptr, tok_groups, q, NULL,
                                     uy, k24, uacc, ut, &tr);
            if (r == PCG_REF_OK) {
              otok[i] = tr.y;
              ogrp[i] = tr.group;
              if (tr.near & 1) flags[b] |= 1;
            }
          }
        } else {
          for (int32_t t = 0; r == PCG_REF_OK; ++t) {
            pcg_ref_trial_uniforms(seed, offset, (uint32_t)b, (uint32_t)i, (uint32_t)t, &uy, &k24,
                                   &uacc, &ut);
            r = pcg_ref_thin_trial_w(V, G, row_ptr, members, mult, wt, tok_ptr, tok_groups, q, p,
                                     uy, k24, uacc, ut, &tr);
            if (r) break;
            trials[b] = t + 1;
            if (tr.near & 3) flags[b] |= 1;
            if (tr.accepted || t + 1 >= max_trials) {
              if (tr.near & 4) flags[b] |= 1;
              if (!tr.accepted) flags[b] |= 2;
              otok[i] = tr.token;
              ogrp[i] = tr.group;
              break;
            }
          }
        }
      }
      if (r) {
#ifdef _OPENMP
#pragma omp critical
#endif
        status = r;
      }
    }
    free(q);
  }
  return status;
}

/* ------------------------------------------------------------------------- */
/* Draft-side proposal coupling, Eq. (6)                                       */
/* ------------------------------------------------------------------------- */

void pcg_ref_propose_uniforms(uint64_t seed, uint64_t offset, uint32_t b, uint32_t i, double *u_x,
                              uint32_t *k24) {
  uint32_t ctr[4] = {(uint32_t)offset, (uint32_t)(offset >> 32), b, i | 0xFFFF0000u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  pcg_ref_philox4x32_10(ctr, key, w);
  if (u_x) *u_x = (double)(w[0] >> 8) / 16777216.0;
  if (k24) *k24 = w[1] >> 8;
}

static int propose_one(int32_t V, int32_t G, const int32_t *mult, const float *tok_weights,
                       const int32_t *tok_ptr, const int32_t *tok_groups, const void *draft_logits,
                       int dtype,
                       int64_t first, double temperature, double u_x, uint32_t k24, double *p,
                       int32_t *token, int32_t *group, uint8_t *near) {
  int r = softmax_row_at(draft_logits, dtype, first, V, temperature, p);
  if (r) return r;
  int nr = 0;
  int64_t x = inverse_cdf(p, V, u_x, &nr);          /* x ~ p_i */
  if (x < 0) return PCG_REF_ERR_ROW;
  int32_t n = tok_ptr[x + 1] - tok_ptr[x];          /* N(x) membership entries */
  if (n < 1 || n != mult[x]) return PCG_REF_ERR_CSR;
  int ne = 0;
  int32_t e = pick_entry(tok_ptr, tok_weights, x, k24, &ne);
  if (e < 0) return PCG_REF_ERR_CSR;
  nr |= ne;
  int32_t g = tok_groups[tok_ptr[x] + e];
  if (g < 0 || g >= G) return PCG_REF_ERR_CSR;
  *token = (int32_t)x;
  *group = g;
  if (near) *near = (uint8_t)nr;
  return PCG_REF_OK;
}

static int propose_impl(int32_t V, int32_t G, const int32_t *mult, const float *tok_weights,
                        const int32_t *tok_ptr, const int32_t *tok_groups, const void *draft_logits, int dtype, int32_t B,
                        int32_t K, int32_t pos0, int64_t dft_batch_stride, int64_t dft_pos_stride,
                        double temperature, const double *u_x, const uint32_t *k24, uint64_t seed,
                        uint64_t offset, int32_t *prop_tokens, int32_t *prop_groups, uint8_t *near,
                        int32_t nthreads) {
  if (!mult || !tok_ptr || !tok_groups || !draft_logits || !prop_tokens || !prop_groups)
    return PCG_REF_ERR_ARG;
  if (V < 1 || G < 1 || B < 0 || K < 1 || pos0 < 0 || (int64_t)pos0 + K > 0xFFFF ||
      !(temperature > 0.0))
    return PCG_REF_ERR_ARG;
  if (dtype != PCG_REF_F32 && dtype != PCG_REF_BF16) return PCG_REF_ERR_ARG;
  if (nthreads < 1) nthreads = 1;
  int status = PCG_REF_OK;
#ifdef _OPENMP
#pragma omp parallel num_threads(nthreads)
#endif
  {
    double *p = (double *)malloc((size_t)V * sizeof(double));
    if (!p) {
#ifdef _OPENMP
#pragma omp critical
#endif
      status = PCG_REF_ERR_NOMEM;
    }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
    for (int64_t bi = 0; bi < (int64_t)B * K; ++bi) {
      if (!p || status != PCG_REF_OK) continue;
      int32_t b = (int32_t)(bi / K), i = (int32_t)(bi % K);
      double ux;
      uint32_t kk;
      if (u_x) { ux = u_x[bi]; kk = k24[bi]; }
      else pcg_ref_propose_uniforms(seed, offset, (uint32_t)b, (uint32_t)(pos0 + i), &ux, &kk);
      int r = propose_one(V, G, mult, tok_weights, tok_ptr, tok_groups, draft_logits, dtype,
                          b * dft_batch_stride + i * dft_pos_stride, temperature, ux, kk, p,
                          prop_tokens + bi, prop_groups + bi, near ? near + bi : NULL);
      if (r) {
#ifdef _OPENMP
#pragma omp critical
#endif
        status = r;
      }
    }
    free(p);
  }
  return status;
}

int pcg_ref_propose_u(int32_t V, int32_t G, const int32_t *mult, const int32_t *tok_ptr,
                      const int32_t *tok_groups, const void *draft_logits, int dtype, int32_t B,
                      int32_t K, int64_t dft_batch_stride, int64_t dft_pos_stride,
                      double temperature, const double *u_x, const uint32_t *k24,
                      int32_t *prop_tokens, int32_t *prop_groups, uint8_t *near) {
  return pcg_ref_propose_u_w(V, G, mult, NULL, tok_ptr, tok_groups, draft_logits, dtype, B, K,
                             dft_batch_stride, dft_pos_stride, temperature, u_x, k24, prop_tokens,
                             prop_groups, near);
}

int pcg_ref_propose_u_w(int32_t V, int32_t G, const int32_t *mult, const pcg_ref_weights *wt,
                        const int32_t *tok_ptr, const int32_t *tok_groups,
                        const void *draft_logits, int dtype, int32_t B, int32_t K,
                        int64_t dft_batch_stride, int64_t dft_pos_stride, double temperature,
                        const double *u_x, const uint32_t *k24, int32_t *prop_tokens,
                        int32_t *prop_groups, uint8_t *near) {
  if (!u_x || !k24) return PCG_REF_ERR_ARG;
  return propose_impl(V, G, mult, wt ? wt->tok_weights : NULL, tok_ptr, tok_groups, draft_logits,
                      dtype, B, K, 0,
                      dft_batch_stride, dft_pos_stride, temperature, u_x, k24, 0, 0, prop_tokens,
                      prop_groups, near, 1);
}

int pcg_ref_propose(int32_t V, int32_t G, const int32_t *mult, const int32_t *tok_ptr,
                    const int32_t *tok_groups, const void *draft_logits, int dtype, int32_t B,
                    int32_t K, int32_t pos0, int64_t dft_batch_stride, int64_t dft_pos_stride,
                    double temperature, uint64_t seed, uint64_t offset, int32_t *prop_tokens,
                    int32_t *prop_groups, uint8_t *near, int32_t nthreads) {
  return pcg_ref_propose_w(V, G, mult, NULL, tok_ptr, tok_groups, draft_logits, dtype, B, K, pos0,
                           dft_batch_stride, dft_pos_stride, temperature, seed, offset, prop_tokens,
                           prop_groups, near, nthreads);
}

int pcg_ref_propose_w(int32_t V, int32_t G, const int32_t *mult, const pcg_ref_weights *wt,
                      const int32_t *tok_ptr, const int32_t *tok_groups, const void *draft_logits,
                      int dtype, int32_t B, int32_t K, int32_t pos0, int64_t dft_batch_stride,
                      int64_t dft_pos_stride, double temperature, uint64_t seed, uint64_t offset,
                      int32_t *prop_tokens, int32_t *prop_groups, uint8_t *near,
                      int32_t nthreads) {
  return propose_impl(V, G, mult, wt ? wt->tok_weights : NULL, tok_ptr, tok_groups, draft_logits,
                      dtype, B, K, pos0,
                      dft_batch_stride, dft_pos_stride, temperature, NULL, NULL, seed, offset,
                      prop_tokens, prop_groups, near, nthreads);
}

/* ------------------------------------------------------------------------- */
/* Acoustic Similarity Groups, Eq. (1)                                        */
/* ------------------------------------------------------------------------- */

static double bf16_value(uint16_t h) {
  uint32_t w = (uint32_t)h << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

/* x rounded to bfloat16: nearest, ties to even (|x| well inside the normal range) */
static uint16_t bf16_round(double x) {
  float f = (float)x;                 /* a first guess; its two bf16 neighbours bracket x */
  uint32_t w;
  memcpy(&w, &f, sizeof w);
  uint32_t lo = w & 0xffff0000u;      /* truncation: towards zero */
  uint32_t hi = lo + 0x10000u;        /* next value away from zero */
  float flo, fhi;
  memcpy(&flo, &lo, sizeof flo);
  memcpy(&fhi, &hi, sizeof fhi);
  /* (float)x may have rounded across lo or hi; step until lo and hi bracket x */
  while (fabs((double)flo) > fabs(x)) { hi = lo; lo -= 0x10000u; memcpy(&flo, &lo, 4); memcpy(&fhi, &hi, 4); }
  while (fabs((double)fhi) < fabs(x)) { lo = hi; hi += 0x10000u; memcpy(&flo, &lo, 4); memcpy(&fhi, &hi, 4); }
  double dlo = fabs(x) - fabs((double)flo), dhi = fabs((double)fhi) - fabs(x);
  uint32_t pick = dlo < dhi ? lo : (dhi < dlo ? hi : ((lo >> 16) & 1u ? hi : lo));
  return (uint16_t)(pick >> 16);
}

int pcg_ref_asg_normalize(const float *emb, int32_t V, int32_t d, uint16_t *unit_bf16) {
  if (!emb || !unit_bf16 || V < 1 || d < 1) return PCG_REF_ERR_ARG;
  for (int32_t v = 0; v < V; ++v) {
    const float *e = emb + (int64_t)v * d;
    double ss = 0.0;
    for (int32_t k = 0; k < d; ++k) {
      if (!isfinite(e[k])) return PCG_REF_ERR_ROW;
      ss += (double)e[k] * (double)e[k];
    }
    double norm = sqrt(ss);
    for (int32_t k = 0; k < d; ++k)
      unit_bf16[(int64_t)v * d + k] = norm > 0.0 ? bf16_round((double)e[k] / norm) : 0;
  }
  return PCG_REF_OK;
}

double pcg_ref_asg_similarity(const uint16_t *unit_bf16, int32_t d, int32_t a, int32_t b) {
  const uint16_t *x = unit_bf16 + (int64_t)a * d, *y = unit_bf16 + (int64_t)b * d;
  double s = 0.0;
  for (int32_t k = 0; k < d; ++k) s += bf16_value(x[k]) * bf16_value(y[k]);
  return s;
}

int pcg_ref_asg_row(const uint16_t *unit_bf16, int32_t V, int32_t d, float theta, int32_t t,
                    int32_t *members_out, int32_t *count, int32_t *near_pairs) {
  if (!unit_bf16 || !members_out || !count || V < 1 || d < 1 || t < 0 || t >= V)
    return PCG_REF_ERR_ARG;
  int32_t n = 0, near = 0;
  for (int32_t v = 0; v < V; ++v) {
    if (v == t) { members_out[n++] = v; continue; }
    double s = pcg_ref_asg_similarity(unit_bf16, d, t, v);
    if (s > (double)theta) members_out[n++] = v;              /* Eq. (1) */
    if (fabs(s - (double)theta) < PCG_REF_ASG_NEAR) ++near;
  }
  *count = n;
  if (near_pairs) *near_pairs = near;
  return PCG_REF_OK;
}

double pcg_ref_asg_cosine(const float *emb, int32_t d, int32_t a, int32_t b) {
  const float *x = emb + (int64_t)a * d, *y = emb + (int64_t)b * d;
  double dot = 0.0, xx = 0.0, yy = 0.0;
  for (int32_t k = 0; k < d; ++k) {
    dot += (double)x[k] * (double)y[k];
    xx += (double)x[k] * (double)x[k];
    yy += (double)y[k] * (double)y[k];
  }
  if (!(xx > 0.0) || !(yy > 0.0)) return 0.0;
  return dot / (sqrt(xx) * sqrt(yy));
}

int pcg_ref_asg_row_exact(const float *emb, int32_t V, int32_t d, double theta, int32_t t,
                          int32_t *members_out, int32_t *count, double *cos_out) {
  if (!emb || !members_out || !count || V < 1 || d < 1 || t < 0 || t >= V) return PCG_REF_ERR_ARG;
  int32_t n = 0;
  for (int32_t v = 0; v < V; ++v) {
    double c = v == t ? 1.0 : pcg_ref_asg_cosine(emb, d, t, v);
    if (cos_out) cos_out[v] = c;
    if (v == t || c > theta) members_out[n++] = v;            /* Eq. (1), strict */
  }
  *count = n;
  return PCG_REF_OK;
}

/* Width of the band around theta inside which a pair's exact cosine counts as a near-tie. */
#define PCG_REF_ASG_NEAR_EXACT 1e-12

/* The distinct sets in order of first appearance, from either kind of row: unit_bf16 != NULL
 * thresholds the similarity of the rounded unit vectors, emb != NULL the cosine of Eq. (1). */
static int asg_build_rows(const uint16_t *unit_bf16, const float *emb, int32_t V, int32_t d,
                          double theta, int32_t *out_G, int64_t *out_nnz, int32_t *row_ptr,
                          int32_t *members, int64_t members_capacity, int32_t *mult,
                          int32_t *seed_of, uint8_t *near_rows, int32_t nthreads) {
  if ((!unit_bf16 && !emb) || !out_G || !out_nnz || !row_ptr || !members || !mult || V < 1 ||
      d < 1 || members_capacity < 0)
    return PCG_REF_ERR_ARG;
  if (nthreads < 1) nthreads = 1;
  /* every token's set, then the distinct ones in order of first appearance */
  int32_t **set = (int32_t **)calloc((size_t)V, sizeof(int32_t *));
  int32_t *size = (int32_t *)calloc((size_t)V, sizeof(int32_t));
  uint8_t *kept = (uint8_t *)calloc((size_t)V, 1);
  int status = (set && size && kept) ? PCG_REF_OK : PCG_REF_ERR_NOMEM;
  if (status == PCG_REF_OK) {
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 8)
#endif
    for (int32_t t = 0; t < V; ++t) {
      int32_t *buf = (int32_t *)malloc((size_t)V * sizeof(int32_t));
      double *cosv = emb ? (double *)malloc((size_t)V * sizeof(double)) : NULL;
      int32_t n = 0, near = 0;
      int bad = !buf || (emb && !cosv);
      if (!bad && unit_bf16) bad = pcg_ref_asg_row(unit_bf16, V, d, (float)theta, t, buf, &n, &near);
      if (!bad && emb) {
        bad = pcg_ref_asg_row_exact(emb, V, d, theta, t, buf, &n, cosv);
        for (int32_t v = 0; !bad && v < V; ++v)
          if (v != t && fabs(cosv[v] - theta) < PCG_REF_ASG_NEAR_EXACT) ++near;
      }
      free(cosv);
      if (bad) {
#ifdef _OPENMP
#pragma omp critical
#endif
        status = PCG_REF_ERR_NOMEM;
        free(buf);
        continue;
      }
      set[t] = (int32_t *)realloc(buf, (size_t)n * sizeof(int32_t));
      size[t] = n;
      if (near_rows) near_rows[t] = near > 0;
    }
  }
  int32_t G = 0;
  int64_t nnz = 0;
  if (status == PCG_REF_OK) {
    for (int32_t t = 0; t < V; ++t) {
      int dup = 0;
      for (int32_t s = 0; s < t && !dup; ++s)
        dup = kept[s] && size[s] == size[t] &&
              memcmp(set[s], set[t], (size_t)size[t] * sizeof(int32_t)) == 0;
      kept[t] = !dup;
      if (!dup) { ++G; nnz += size[t]; }
    }
    *out_G = G;
    *out_nnz = nnz;
    if (nnz > members_capacity) {
      status = PCG_REF_ERR_NOMEM;
    } else {
      for (int32_t v = 0; v < V; ++v) mult[v] = 0;
      int32_t g = 0;
      row_ptr[0] = 0;
      for (int32_t t = 0; t < V; ++t) {
        if (!kept[t]) continue;
        memcpy(members + row_ptr[g], set[t], (size_t)size[t] * sizeof(int32_t));
        for (int32_t j = 0; j < size[t]; ++j) mult[set[t][j]] += 1;
        if (seed_of) seed_of[g] = t;
        row_ptr[g + 1] = row_ptr[g] + size[t];
        ++g;
      }
    }
  }
  if (set) for (int32_t t = 0; t < V; ++t) free(set[t]);
  free(set); free(size); free(kept);
  return status;
}

int pcg_ref_asg_build(const uint16_t *unit_bf16, int32_t V, int32_t d, float theta,
                      int32_t *out_G, int64_t *out_nnz, int32_t *row_ptr, int32_t *members,
                      int64_t members_capacity, int32_t *mult, int32_t *seed_of,
                      uint8_t *near_rows, int32_t nthreads) {
  if (!unit_bf16) return PCG_REF_ERR_ARG;
  return asg_build_rows(unit_bf16, NULL, V, d, (double)theta, out_G, out_nnz, row_ptr, members,
                        members_capacity, mult, seed_of, near_rows, nthreads);
}

int pcg_ref_asg_build_exact(const float *emb, int32_t V, int32_t d, double theta,
                            int32_t *out_G, int64_t *out_nnz, int32_t *row_ptr,
                            int32_t *members, int64_t members_capacity, int32_t *mult,
                            int32_t *seed_of, uint8_t *near_rows, int32_t nthreads) {
  if (!emb) return PCG_REF_ERR_ARG;
  return asg_build_rows(NULL, emb, V, d, theta, out_G, out_nnz, row_ptr, members,
                        members_capacity, mult, seed_of, near_rows, nthreads);
}
