/*
 * The C ABI of libpcg used from plain C, with no Python and no PyTorch anywhere: device memory
 * from the HIP runtime, group membership made usable by pcg_groups_canonicalize_host, one
 * pcg_group_probs and one pcg_verify call (Algorithm 1 with Eq. 5, 7, 8, 10).  Inputs come from a
 * small linear congruential generator so that a test can rebuild them and hand them to the CPU
 * oracle; every output is printed as text.
 *
 * Built by __graft_entry__.build() (gcc, C11); run on an MI355X by tests/test_gpu_c_abi.py.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "pcg.h"

#define CK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "HIP error %d at line %d\n", (int) e_, __LINE__); return 2; } } while (0)
#define CK_PCG(x) do { int s_ = (x); if (s_ != PCG_OK) { \
  fprintf(stderr, "libpcg: %s (status %d) at line %d\n", pcg_strerror(s_), s_, __LINE__); return 3; } } while (0)

enum { V = 96, G0 = 20, B = 5, K = 3 };

static uint32_t lcg_state = 12345u;
static uint32_t lcg(void) { lcg_state = lcg_state * 1664525u + 1013904223u; return lcg_state >> 8; }
/* uniform in [-1, 1) on a 2^-23 grid: exact in float */
static float unit(void) { return (float) ((int32_t) (lcg() & 0xffffff) - 0x800000) * (1.0f / 8388608.0f); }

int main(void) {
  /* G0 groups of 2..6 distinct tokens; tokens 90..95 are left uncovered on purpose */
  int32_t row_ptr[G0 + 1], members[G0 * 6];
  row_ptr[0] = 0;
  for (int g = 0; g < G0; ++g) {
    int n = 2 + (int) (lcg() % 5u), k = 0;
    int32_t *m = members + row_ptr[g];
    while (k < n) {
      int32_t t = (int32_t) (lcg() % 90u);
      int dup = 0;
      for (int j = 0; j < k; ++j) dup |= m[j] == t;
      if (!dup) m[k++] = t;
    }
    for (int i = 1; i < n; ++i)          /* ascending members */
      for (int j = i; j > 0 && m[j - 1] > m[j]; --j) { int32_t s = m[j]; m[j] = m[j - 1]; m[j - 1] = s; }
    row_ptr[g + 1] = row_ptr[g] + n;
  }
  int32_t G = 0;
  int64_t nnz = 0;
  CK_PCG(pcg_groups_canonicalize_host(V, G0, row_ptr, members, &G, &nnz, NULL, NULL, NULL));
  int32_t *rp = malloc(sizeof(int32_t) * (size_t) (G + 1)), *mem = malloc(sizeof(int32_t) * (size_t) nnz);
  int32_t *mult = malloc(sizeof(int32_t) * V);
  if (!rp || !mem || !mult) return 1;
  CK_PCG(pcg_groups_canonicalize_host(V, G0, row_ptr, members, &G, &nnz, rp, mem, mult));
  CK_PCG(pcg_groups_validate_host(V, G, rp, mem, mult));

  static float tgt[B][K + 1][V], dft[B][K][V];
  for (int b = 0; b < B; ++b)
    for (int i = 0; i <= K; ++i)
      for (int t = 0; t < V; ++t) tgt[b][i][t] = 3.0f * unit();
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < K; ++i)
      for (int t = 0; t < V; ++t) dft[b][i][t] = tgt[b][i][t] + 0.75f * unit();
  /* any proposal is a legal input: a group, and a token of that group */
  int32_t ptok[B][K], pgrp[B][K];
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < K; ++i) {
      int32_t g = (int32_t) (lcg() % (uint32_t) G);
      pgrp[b][i] = g;
      ptok[b][i] = mem[rp[g] + (int32_t) (lcg() % (uint32_t) (rp[g + 1] - rp[g]))];
    }

  int32_t *d_rp, *d_mem, *d_mult, *d_ptok, *d_pgrp, *d_len, *d_tok, *d_grp;
  float *d_tgt, *d_dft, *d_probs;
  void *d_ws;
  pcg_diag *d_diag;
  CK_HIP(hipMalloc((void **) &d_rp, sizeof(int32_t) * (size_t) (G + 1)));
  CK_HIP(hipMalloc((void **) &d_mem, sizeof(int32_t) * (size_t) nnz));
  CK_HIP(hipMalloc((void **) &d_mult, sizeof(int32_t) * V));
  CK_HIP(hipMalloc((void **) &d_tgt, sizeof tgt));
  CK_HIP(hipMalloc((void **) &d_dft, sizeof dft));
  CK_HIP(hipMalloc((void **) &d_ptok, sizeof ptok));
  CK_HIP(hipMalloc((void **) &d_pgrp, sizeof pgrp));
  CK_HIP(hipMalloc((void **) &d_len, sizeof(int32_t) * B));
  CK_HIP(hipMalloc((void **) &d_tok, sizeof(int32_t) * B * (K + 1)));
  CK_HIP(hipMalloc((void **) &d_grp, sizeof(int32_t) * B * (K + 1)));
  CK_HIP(hipMalloc((void **) &d_probs, sizeof(float) * (size_t) B * (size_t) G));
  CK_HIP(hipMalloc((void **) &d_diag, sizeof(pcg_diag)));
  CK_HIP(hipMemset(d_diag, 0, sizeof(pcg_diag)));
  CK_HIP(hipMemcpy(d_rp, rp, sizeof(int32_t) * (size_t) (G + 1), hipMemcpyHostToDevice));
  CK_HIP(hipMemcpy(d_mem, mem, sizeof(int32_t) * (size_t) nnz, hipMemcpyHostToDevice));
  CK_HIP(hipMemcpy(d_mult, mult, sizeof(int32_t) * V, hipMemcpyHostToDevice));
  CK_HIP(hipMemcpy(d_tgt, tgt, sizeof tgt, hipMemcpyHostToDevice));
  CK_HIP(hipMemcpy(d_dft, dft, sizeof dft, hipMemcpyHostToDevice));
  CK_HIP(hipMemcpy(d_ptok, ptok, sizeof ptok, hipMemcpyHostToDevice));
  CK_HIP(hipMemcpy(d_pgrp, pgrp, sizeof pgrp, hipMemcpyHostToDevice));

  pcg_groups groups = {0};
  groups.V = V; groups.G = G; groups.nnz = nnz;
  groups.row_ptr = d_rp; groups.members = d_mem; groups.mult = d_mult;

  size_t need = pcg_verify_workspace_bytes(V, G, B, K), need2 = pcg_group_probs_workspace_bytes(V, B);
  if (need2 > need) need = need2;
  if (need == 0) return 4;
  CK_HIP(hipMalloc(&d_ws, need));

  /* Eq. (5) for the first target row of every sequence (row stride (K + 1) V) */
  CK_PCG(pcg_group_probs(&groups, d_tgt, PCG_F32, B, (int64_t) (K + 1) * V, 1.0f, d_probs, d_ws, need, NULL));
  CK_PCG(pcg_verify(&groups, d_tgt, d_dft, PCG_F32, B, K, (int64_t) (K + 1) * V, V, (int64_t) K * V, V, 1.0f,
                    &d_ptok[0], &d_pgrp[0], 7u, 3u, d_len, d_tok, d_grp, d_diag, d_ws, need, NULL));
  CK_HIP(hipDeviceSynchronize());

  int32_t len[B], tok[B][K + 1], grp[B][K + 1];
  float *probs = malloc(sizeof(float) * (size_t) B * (size_t) G);
  pcg_diag diag;
  if (!probs) return 1;
  CK_HIP(hipMemcpy(len, d_len, sizeof len, hipMemcpyDeviceToHost));
  CK_HIP(hipMemcpy(tok, d_tok, sizeof tok, hipMemcpyDeviceToHost));
  CK_HIP(hipMemcpy(grp, d_grp, sizeof grp, hipMemcpyDeviceToHost));
  CK_HIP(hipMemcpy(probs, d_probs, sizeof(float) * (size_t) B * (size_t) G, hipMemcpyDeviceToHost));
  CK_HIP(hipMemcpy(&diag, d_diag, sizeof diag, hipMemcpyDeviceToHost));

  printf("version %s\n", pcg_version());
  printf("groups %d %lld\n", (int) G, (long long) nnz);
  for (int b = 0; b < B; ++b) {
    printf("seq %d len %d tokens", b, (int) len[b]);
    for (int i = 0; i <= K; ++i) printf(" %d", (int) tok[b][i]);
    printf(" groups");
    for (int i = 0; i <= K; ++i) printf(" %d", (int) grp[b][i]);
    printf("\n");
  }
  for (int b = 0; b < B; ++b) {
    printf("probs %d", b);
    for (int g = 0; g < G; ++g) printf(" %.9g", (double) probs[(size_t) b * (size_t) G + (size_t) g]);
    printf("\n");
  }
  printf("diag sequences %u accepted %u\n", (unsigned) diag.sequences, (unsigned) diag.accepted_total);
  /* an argument error comes back as a status, nothing is launched */
  int bad = pcg_verify(&groups, d_tgt, d_dft, PCG_F32, B, 0, (int64_t) (K + 1) * V, V, (int64_t) K * V, V, 1.0f,
                       &d_ptok[0], &d_pgrp[0], 7u, 3u, d_len, d_tok, d_grp, NULL, d_ws, need, NULL);
  printf("K=0 status %d %s\n", bad, pcg_strerror(bad));
  hipFree(d_ws); hipFree(d_diag); hipFree(d_probs); hipFree(d_grp); hipFree(d_tok); hipFree(d_len);
  hipFree(d_pgrp); hipFree(d_ptok); hipFree(d_dft); hipFree(d_tgt); hipFree(d_mult); hipFree(d_mem); hipFree(d_rp);
  free(probs); free(mult); free(mem); free(rp);
  return 0;
}
