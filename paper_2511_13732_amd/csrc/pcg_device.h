// Device-side helpers shared by the libpcg kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pcg.h"

namespace pcg {

constexpr int kWave = 64;

// ---------------------------------------------------------------------------------------------
// Logit element access.  bfloat16 is the upper half of an IEEE binary32.
// ---------------------------------------------------------------------------------------------

template <bool BF16>
__device__ __forceinline__ float logit_at(const void *row, int64_t t) {
  if constexpr (BF16) {
    return __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(row)[t] << 16);
  } else {
    return reinterpret_cast<const float *>(row)[t];
  }
}

__device__ __forceinline__ const void *elem_ptr(const void *base, int64_t elems, bool bf16) {
  return reinterpret_cast<const char *>(base) + elems * (bf16 ? 2 : 4);
}

// Where the rows of a call live: set 0 = target rows (b, i), i < npos0; set 1 = draft rows
// (b, i), i < npos1.  Row ids are [0, B*npos0) for set 0 followed by [B*npos0, ...) for set 1.
// pcg_group_probs uses set 0 alone with npos0 = 1 and bs0 = row stride.
struct RowSet {
  const void *base0;
  const void *base1;
  int64_t bs0, ps0, bs1, ps1;   // strides in elements
  int32_t npos0, npos1;
  int64_t nrows0;               // B * npos0
  double inv_npos0, inv_npos1;  // 1 / npos, so that kernels split a row id without dividing
};

// row / npos and row % npos for 0 <= row < 2^40, 1 <= npos <= 65: a multiplication by the
// reciprocal and one correction step instead of a 64-bit integer division.
__device__ __forceinline__ void split_row(int64_t row, int32_t npos, double inv_npos, int64_t &b,
                                          int32_t &i) {
  int64_t q = (int64_t) ((double) row * inv_npos);
  int64_t r = row - q * npos;
  if (r < 0) { --q; r += npos; }
  if (r >= npos) { ++q; r -= npos; }
  b = q;
  i = (int32_t) r;
}

__device__ __forceinline__ const void *row_base(const RowSet &rs, int64_t row, bool bf16) {
  int64_t b;
  int32_t i;
  if (row < rs.nrows0) {
    split_row(row, rs.npos0, rs.inv_npos0, b, i);
    return elem_ptr(rs.base0, b * rs.bs0 + i * rs.ps0, bf16);
  }
  split_row(row - rs.nrows0, rs.npos1, rs.inv_npos1, b, i);
  return elem_ptr(rs.base1, b * rs.bs1 + i * rs.ps1, bf16);
}

// ---------------------------------------------------------------------------------------------
// Cross-lane reductions through DPP (no LDS traffic).
// ---------------------------------------------------------------------------------------------

constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15-i inside each row of 16
constexpr int kDppBcast15 = 0x142;     // lane 15 of a row -> every lane of the next row
constexpr int kDppBcast31 = 0x143;     // lane 31 -> rows 2 and 3

// Value of the DPP source lane; lanes the row mask excludes receive `fallback`.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_get(float v, float fallback) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(fallback), __float_as_int(v),
                                                    CTRL, ROW_MASK, 0xf, false));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_get(double v, double fallback) {
  int2 s = *reinterpret_cast<int2 *>(&v), f = *reinterpret_cast<int2 *>(&fallback), r;
  r.x = __builtin_amdgcn_update_dpp(f.x, s.x, CTRL, ROW_MASK, 0xf, false);
  r.y = __builtin_amdgcn_update_dpp(f.y, s.y, CTRL, ROW_MASK, 0xf, false);
  return *reinterpret_cast<double *>(&r);
}

// Sum over aligned sub-waves of W lanes (W a power of two, 1..64).  The total is valid in the
// LAST lane of each sub-wave (for W <= 16 in all of its lanes).  Fixed tree, so the result does
// not depend on scheduling.
template <int W, typename T>
__device__ __forceinline__ T subwave_sum(T v) {
  if constexpr (W >= 2) v += dpp_get<kDppXor1, 0xf>(v, T(0));
  if constexpr (W >= 4) v += dpp_get<kDppXor2, 0xf>(v, T(0));
  if constexpr (W >= 8) v += dpp_get<kDppHalfMirror, 0xf>(v, T(0));
  if constexpr (W >= 16) v += dpp_get<kDppMirror, 0xf>(v, T(0));
  if constexpr (W >= 32) v += dpp_get<kDppBcast15, 0xa>(v, T(0));
  if constexpr (W >= 64) v += dpp_get<kDppBcast31, 0xc>(v, T(0));
  return v;
}

// Max over the whole wave, returned in every lane.
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_get<kDppXor1, 0xf>(v, v));
  v = fmaxf(v, dpp_get<kDppXor2, 0xf>(v, v));
  v = fmaxf(v, dpp_get<kDppHalfMirror, 0xf>(v, v));
  v = fmaxf(v, dpp_get<kDppMirror, 0xf>(v, v));
  v = fmaxf(v, dpp_get<kDppBcast15, 0xa>(v, v));
  v = fmaxf(v, dpp_get<kDppBcast31, 0xc>(v, v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Sum over the whole wave through DPP, returned in every lane (fixed tree).
__device__ __forceinline__ double wave_sum(double v) {
  v = subwave_sum<64>(v);
  int2 r = *reinterpret_cast<int2 *>(&v);
  r.x = __builtin_amdgcn_readlane(r.x, 63);
  r.y = __builtin_amdgcn_readlane(r.y, 63);
  return *reinterpret_cast<double *>(&r);
}

constexpr int kDppShr1 = 0x111;        // row_shr: lane i <- lane i-k inside each row of 16
constexpr int kDppShr2 = 0x112;
constexpr int kDppShr4 = 0x114;
constexpr int kDppShr8 = 0x118;

// Inclusive prefix sum over the wave through DPP: lane l receives v[0] + ... + v[l] (fixed tree).
__device__ __forceinline__ double wave_scan(double v) {
  v += dpp_get<kDppShr1, 0xf>(v, 0.0);
  v += dpp_get<kDppShr2, 0xf>(v, 0.0);
  v += dpp_get<kDppShr4, 0xf>(v, 0.0);
  v += dpp_get<kDppShr8, 0xf>(v, 0.0);
  v += dpp_get<kDppBcast15, 0xa>(v, 0.0);   // rows 1 and 3 add the total of the row before
  v += dpp_get<kDppBcast31, 0xc>(v, 0.0);   // rows 2 and 3 add the total of rows 0 and 1
  return v;
}

// Value of lane l (the same l in every lane) in every lane.
__device__ __forceinline__ double read_lane(double v, int l) {
  int2 r = *reinterpret_cast<int2 *>(&v);
  r.x = __builtin_amdgcn_readlane(r.x, l);
  r.y = __builtin_amdgcn_readlane(r.y, l);
  return *reinterpret_cast<double *>(&r);
}

__device__ __forceinline__ int32_t read_lane(int32_t v, int l) {
  return __builtin_amdgcn_readlane(v, l);
}

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11), one block per (sequence, position).
// ---------------------------------------------------------------------------------------------

struct Uniforms {
  float acc, grp, tok;   // 24-bit draws in [0, 1): exact in fp32 and fp64
};

__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t m0 = 0xD2511F53u, m1 = 0xCD9E8D57u;
    uint32_t h0 = __umulhi(m0, c0), l0 = m0 * c0;
    uint32_t h1 = __umulhi(m1, c2), l1 = m1 * c2;
    c0 = h1 ^ c1 ^ k0;
    c1 = l1;
    c2 = h0 ^ c3 ^ k1;
    c3 = l0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return make_uint4(c0, c1, c2, c3);
}

// Draws of position (b, i): counter (offset_lo, offset_hi, b, i), key (seed_lo, seed_hi).
__device__ __forceinline__ Uniforms philox_uniforms(uint64_t seed, uint64_t offset, uint32_t b,
                                                    uint32_t i) {
  const uint4 w = philox4x32_10((uint32_t) offset, (uint32_t) (offset >> 32), b, i,
                                (uint32_t) seed, (uint32_t) (seed >> 32));
  const float s = 1.0f / 16777216.0f;
  Uniforms u;
  u.acc = (float) (w.x >> 8) * s;
  u.grp = (float) (w.y >> 8) * s;
  u.tok = (float) (w.z >> 8) * s;
  return u;
}

// Draws of thinning trial `trial` at position (b, i): the block with counter word 3 =
// i | (trial + 1) << 16.  u_y, u_a, u_tok are 24-bit uniforms; k24 is the raw 24-bit integer
// that picks one of a token's membership entries as (k24 * N) >> 24.
struct TrialDraws {
  float u_y, u_a, u_tok;
  uint32_t k24;
};

__device__ __forceinline__ TrialDraws philox_trial(uint64_t seed, uint64_t offset, uint32_t b,
                                                   uint32_t i, uint32_t trial) {
  const uint4 w = philox4x32_10((uint32_t) offset, (uint32_t) (offset >> 32), b,
                                i | ((trial + 1u) << 16), (uint32_t) seed, (uint32_t) (seed >> 32));
  const float s = 1.0f / 16777216.0f;
  TrialDraws d;
  d.u_y = (float) (w.x >> 8) * s;
  d.k24 = w.y >> 8;
  d.u_a = (float) (w.z >> 8) * s;
  d.u_tok = (float) (w.w >> 8) * s;
  return d;
}

// Draws of the draft-side proposal at position (b, i): the block with counter word 3 =
// i | 0xFFFF0000, a trial field no thinning trial reaches.
struct ProposalDraws {
  float u_x;
  uint32_t k24;
};

__device__ __forceinline__ ProposalDraws philox_proposal(uint64_t seed, uint64_t offset, uint32_t b,
                                                         uint32_t i) {
  const uint4 w = philox4x32_10((uint32_t) offset, (uint32_t) (offset >> 32), b, i | 0xFFFF0000u,
                                (uint32_t) seed, (uint32_t) (seed >> 32));
  ProposalDraws d;
  d.u_x = (float) (w.x >> 8) * (1.0f / 16777216.0f);
  d.k24 = w.y >> 8;
  return d;
}

// ---------------------------------------------------------------------------------------------
// Per-row softmax statistics.
// ---------------------------------------------------------------------------------------------

// One wave's share of a row: the exact maximum m of its logits, the log2-domain reference
// t = fl(m * c) and z = sum 2^(x * c - t).
struct StatPart {
  double z;
  float m;
  float t;
};

// A whole row: M = max logit, Z = sum over the row of exp((x - M) / temperature).
struct RowStat {
  double Z;
  float M;
  float pad;
};

// Everything a sequence's finalize step needs (pcg_verify only).
struct FinalizeArgs {
  RowSet rs;
  int32_t K;
  double cd;
  float c, c_lo;           // cd in two fp32 pieces, as the table kernel uses it
  const RowStat *rowstat;
  const int32_t *row_ptr, *members, *mult;
  const float *weights;    // general weights per CSR entry, or NULL for the equal split
  uint64_t seed, offset;
  const int32_t *accept_len;
  float *R;
  int32_t *out_tokens, *out_groups;
  pcg_diag *diag;
};

// Everything a sequence's accept scan needs (pcg_verify, pcg_verify_thinning).
// T_i[g] and D_i[g] of one proposed group (Eq. 5), up to the rows' normalisations: the sums are
// relative to the group's own largest logits, so they can be formed before any row statistic is
// known.  The statistics pass forms them on the side; the accept scan only normalises them.
struct Probe {
  double Tp, Dp;           // sums of 2^((x - ref) c) w over the group's entries, target / draft row
  float Tref, Dref;        // those largest logits
  int32_t bad;             // the proposed group id is out of range
  int32_t pad;
};

struct ProbeArgs {
  const int32_t *row_ptr, *members, *mult, *prop_groups;
  const float *weights;    // general weights per CSR entry, or NULL for the equal split
  int32_t K, G;
  float c_lo;              // low part of log2(e) / temperature (the high part is row_stats' c)
  Probe *out;              // [B * K]; NULL: no probes in this launch
};

struct AcceptArgs {
  RowSet rs;
  int32_t V, G, K, nparts;
  float c;                 // fp32(log2(e) / temperature), as used by row_stats
  double cd;               // log2(e) / temperature
  const StatPart *parts;
  const Probe *probes;     // [B * K], left by the statistics pass
  RowStat *rowstat;
  const int32_t *row_ptr, *members, *mult, *prop_tokens, *prop_groups;
  const float *weights;    // general weights per CSR entry, or NULL for the equal split
  uint64_t seed, offset;
  int32_t *accept_len, *out_tokens, *out_groups;
  pcg_diag *diag;
};

}  // namespace pcg
