// HIP kernels of libpcg for gfx950 (MI355X) and their launchers.
//
// One speculative step (Algorithm 1) runs as four kernels on the caller's stream:
//   row_stats     streams every logits row once: per-wave (max, sum of exponentials)  [HBM-bound];
//                 its leading workgroups also form, for every proposed group, the sums of Eq. (5)
//                 relative to the group's own largest logit (the "probes")
//   accept_delta  per sequence: merges the row statistics, normalises the probes, runs the
//                 accept test of Eq. (7) until the first rejection; then, on the decision row,
//                 the table delta[t] = (q(t) - p(t)) / N(t) (q(t) / N(t) on the bonus row), so
//                 that T[g] - D[g] = sum of delta over G_g
//   gather        the overlap-aware segmented gather-sum of that table over the membership
//                 (Eq. 5, Eq. 8), table tiles staged in LDS.  From the prepared layout, inside
//                 pcg_verify, no sum leaves the kernel: only fp64 totals of max(0, .) per run of
//                 16 consecutive groups and per chunk.  From the CSR (and in pcg_group_probs,
//                 which wants them) every sum is written.
//   finalize      per sequence: the chunk and the run that hold u * total, the run's 16 sums
//                 formed again, the group by inverse CDF, then the token inside it (Eq. 10)
// pcg_group_probs runs row_stats, a weights kernel (q(t) / N(t)) and the same gather;
// pcg_verify_thinning runs row_stats and accept_thin; pcg_propose runs row_stats and propose.
#include "pcg_kernels.h"
#include "pcg_layout.h"

#include <math.h>

#include <algorithm>

namespace pcg {

// =============================================================================================
// row_stats: one wave per 2048-element part of a row.
// =============================================================================================

constexpr int kPartElems = 2048;      // elements per wave: 32 per lane
constexpr int kStatsWaves = 4;        // waves per workgroup

// Row id of a workgroup: grid.y carries the low part, grid.z the rest (grid.y <= 65535).
constexpr int kRowsPerGridY = 32768;

// A 16-byte load, optionally marked as streaming (nontemporal).  Streaming loads reach a higher
// rate on a pass over logits that are larger than the caches, but leave nothing behind for the
// kernels that follow; STREAM is chosen per entry point by how much of the rows those re-read.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <bool STREAM>
__device__ __forceinline__ u32x4 load16(const void *p) {
  if constexpr (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  else return *reinterpret_cast<const u32x4 *>(p);
}

// exp((x - M) / temperature) for one element, argument in two pieces so that its error stays
// relative to the result: (x - M) * (c_hi + c_lo) with c_hi + c_lo = log2(e) / temperature.
__device__ __forceinline__ float exp_rel(float x, float M, float c_hi, float c_lo) {
  const float d = x - M;
  // a -inf logit has no mass; (-inf) * c_lo would turn the sum into inf - inf otherwise
  return d == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(fmaf(d, c_hi, d * c_lo));
}

// The probe of target row `row` = (b, i), i < K, by one wave: T_i[g] and D_i[g] of the proposed
// group g (Eq. 5), each relative to the group's own largest logit.  A chain of four dependent
// loads (proposal -> group -> members -> logits) that needs no row statistic, which is why it
// rides along with the statistics pass instead of waiting for it.
template <bool BF16>
__device__ void probe_row(const RowSet &rs, const ProbeArgs &pa, int64_t row, float c, int lane) {
  int64_t b;
  int32_t i;
  split_row(row, rs.npos0, rs.inv_npos0, b, i);
  const int32_t K = pa.K;
  if (i >= K) return;                                   // the bonus row has no proposal
  const int32_t g = pa.prop_groups[b * K + i];
  const bool ok = g >= 0 && g < pa.G;
  double at = 0.0, ad = 0.0;
  float mt = -INFINITY, md = -INFINITY;
  if (ok) {
    const void *trow = row_base(rs, row, BF16);
    const void *drow = row_base(rs, rs.nrows0 + b * K + i, BF16);
    const int32_t beg = pa.row_ptr[g], end = pa.row_ptr[g + 1];
    // the first 64 members stay in registers; longer groups take a second trip
    const bool has = beg + lane < end;
    const int32_t t0 = has ? pa.members[beg + lane] : 0;
    const float lt0 = has ? logit_at<BF16>(trow, t0) : -INFINITY;
    const float ld0 = has ? logit_at<BF16>(drow, t0) : -INFINITY;
    // the entry's share of its token: 1 / N(t) (Eq. 3), or the caller's weight (Eq. 2)
    const float *wts = pa.weights;
    const float m0 = has && !wts ? (float) pa.mult[t0] : 1.f;
    const float w0 = has && wts ? wts[beg + lane] : 1.f;
    mt = lt0;
    md = ld0;
    for (int32_t j = beg + lane + kWave; j < end; j += kWave) {
      const int32_t t = pa.members[j];
      mt = fmaxf(mt, logit_at<BF16>(trow, t));
      md = fmaxf(md, logit_at<BF16>(drow, t));
    }
    mt = wave_max(mt);
    md = wave_max(md);
    // masses in the kernels' precision: fp32 exponential and division, fp64 sum
    if (lt0 > -INFINITY) at = (double) (exp_rel(lt0, mt, c, pa.c_lo) * w0 / m0);
    if (ld0 > -INFINITY) ad = (double) (exp_rel(ld0, md, c, pa.c_lo) * w0 / m0);
    for (int32_t j = beg + lane + kWave; j < end; j += kWave) {
      const int32_t t = pa.members[j];
      const float m = wts ? 1.f : (float) pa.mult[t];
      const float w = wts ? wts[j] : 1.f;
      const float lt = logit_at<BF16>(trow, t), ld = logit_at<BF16>(drow, t);
      if (lt > -INFINITY) at += (double) (exp_rel(lt, mt, c, pa.c_lo) * w / m);
      if (ld > -INFINITY) ad += (double) (exp_rel(ld, md, c, pa.c_lo) * w / m);
    }
  }
  at = wave_sum(at);
  ad = wave_sum(ad);
  if (lane == 0) {
    Probe p;
    p.Tp = at; p.Dp = ad; p.Tref = mt; p.Dref = md; p.bad = !ok; p.pad = 0;
    pa.out[b * K + i] = p;
  }
}

template <bool BF16, bool VEC, bool STREAM>
__global__ __launch_bounds__(kStatsWaves *kWave) void row_stats_kernel(RowSet rs, int32_t V,
                                                                       int32_t nparts, int64_t nrows,
                                                                       float c, StatPart *parts,
                                                                       ProbeArgs pa, int64_t probe_slots) {
  const int lane = threadIdx.x & (kWave - 1);
  // everything that selects the data is wave-uniform: keep it in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // grid planes (z) continue the count of y: slot runs over the probe slots, then the rows
  const int64_t slot = (int64_t) blockIdx.z * kRowsPerGridY + blockIdx.y;
  if (slot < probe_slots) {
    // The first probe_slots values (launched only with probes) are not rows of logits: each wave
    // of their workgroups forms the probe of one target row.  They are dealt out first, so the
    // chains of dependent loads behind the probes run while the rest of the grid streams.
    const int64_t prow = (slot * gridDim.x + blockIdx.x) * kStatsWaves + wave;
    if (prow < rs.nrows0) probe_row<BF16>(rs, pa, prow, c, lane);
    return;
  }
  const int32_t part = blockIdx.x * kStatsWaves + wave;
  const int64_t row = slot - probe_slots;
  if (part >= nparts || row >= nrows) return;   // whole wave leaves together
  const void *rowp = row_base(rs, row, BF16);
  const int32_t e0 = part * kPartElems;

  float x[32];
  if (VEC && e0 + kPartElems <= V) {
    // interior part of an aligned row: 16-byte loads, all issued before the first use;
    // each load instruction covers 1 KiB of the row
    if constexpr (BF16) {
      const uint4 *src = reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(rowp) + e0);
      u32x4 w[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = load16<STREAM>(src + j * kWave + lane);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t ww[4] = {w[j].x, w[j].y, w[j].z, w[j].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          x[j * 8 + 2 * k] = __uint_as_float(ww[k] << 16);
          x[j * 8 + 2 * k + 1] = __uint_as_float(ww[k] & 0xffff0000u);
        }
      }
    } else {
      const float4 *src = reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(rowp) + e0);
      u32x4 w[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) w[j] = load16<STREAM>(src + j * kWave + lane);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        x[j * 4] = __uint_as_float(w[j].x); x[j * 4 + 1] = __uint_as_float(w[j].y);
        x[j * 4 + 2] = __uint_as_float(w[j].z); x[j * 4 + 3] = __uint_as_float(w[j].w);
      }
    }
  } else {
    // the ragged last part of a row, or rows that are not 16-byte aligned: element loads
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      const int32_t e = e0 + j * kWave + lane;
      x[j] = (e < V) ? logit_at<BF16>(rowp, e) : -INFINITY;
    }
  }

  float m0 = fmaxf(x[0], x[1]), m1 = fmaxf(x[2], x[3]);
#pragma unroll
  for (int j = 4; j < 32; j += 4) {
    m0 = fmaxf(fmaxf(m0, x[j]), x[j + 1]);
    m1 = fmaxf(fmaxf(m1, x[j + 2]), x[j + 3]);
  }
  const float m = wave_max(fmaxf(m0, m1));

  // Exponentials relative to the wave's own maximum, in the log2 domain: t = fl(m * c) is the
  // reference, and each term is 2^(x * c - t) with the product exact inside the fused
  // multiply-add, so terms near the maximum carry no argument error.  Whoever merges the parts
  // rescales by 2^(t - M * c) in double; t is an exact float, so nothing is lost.
  const float t = m * c;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
  for (int j = 0; j < 32; j += 4) {
    s0 += __builtin_amdgcn_exp2f(fmaf(x[j], c, -t));
    s1 += __builtin_amdgcn_exp2f(fmaf(x[j + 1], c, -t));
    s2 += __builtin_amdgcn_exp2f(fmaf(x[j + 2], c, -t));
    s3 += __builtin_amdgcn_exp2f(fmaf(x[j + 3], c, -t));
  }
  double z = (double) ((s0 + s1) + (s2 + s3));
  if (m == -INFINITY) z = 0.0;   // (-inf) - (-inf) is NaN: an all -inf part holds no mass
  z = subwave_sum<64>(z);
  if (lane == kWave - 1) {
    StatPart sp;
    sp.z = z;
    sp.m = m;
    sp.t = t;
    parts[row * nparts + part] = sp;
  }
}

// Merge the parts of one row inside a wave: every lane returns the row's (M, Z).
// c must be the same fp32 factor row_stats used, so that 2^(xc-t) * 2^(t-Mc) = 2^((x-M)c).
__device__ __forceinline__ RowStat merge_row(const StatPart *parts, int64_t row, int32_t nparts,
                                             float c, int lane) {
  const StatPart *rp = parts + row * nparts;
  float M = -INFINITY;
  for (int32_t k = lane; k < nparts; k += kWave) M = fmaxf(M, rp[k].m);
  M = wave_max(M);
  double Z = 0.0;
  for (int32_t k = lane; k < nparts; k += kWave) {
    StatPart sp = rp[k];
    if (sp.z > 0.0) Z += sp.z * exp2((double) sp.t - (double) M * (double) c);
  }
  Z = wave_sum(Z);
  RowStat r;
  r.Z = Z;
  r.M = M;
  r.pad = 0.f;
  return r;
}

// =============================================================================================
// accept: one workgroup per sequence.
// =============================================================================================

constexpr int kTokensPerThread = 8;    // consecutive tokens a thread of the table kernels handles

// Eight consecutive logits of a row as floats; VEC: one (bf16) or two (fp32) 16-byte loads.
template <bool BF16, bool VEC>
__device__ __forceinline__ void load8(const void *row, int32_t t, int32_t V, float *x) {
  if (VEC && t + 8 <= V) {
    if constexpr (BF16) {
      const uint4 w = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(row) + t);
      const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        x[2 * k] = __uint_as_float(ww[k] << 16);
        x[2 * k + 1] = __uint_as_float(ww[k] & 0xffff0000u);
      }
    } else {
      const float4 a = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(row) + t);
      const float4 b = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(row) + t + 4);
      x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
  } else {
#pragma unroll
    for (int k = 0; k < 8; ++k) x[k] = (t + k < V) ? logit_at<BF16>(row, t + k) : -INFINITY;
  }
}

// Divisors of eight consecutive tokens: their multiplicities, or 1 with mult == NULL (general
// weights: the per-entry weight is applied by the gather instead).
template <bool VEC>
__device__ __forceinline__ void load8_mult(const int32_t *mult, int32_t t, int32_t V, float *m) {
  if (!mult) {
#pragma unroll
    for (int k = 0; k < 8; ++k) m[k] = 1.f;
  } else if (VEC && t + 8 <= V) {
    const int4 a = *reinterpret_cast<const int4 *>(mult + t);
    const int4 b = *reinterpret_cast<const int4 *>(mult + t + 4);
    m[0] = (float) a.x; m[1] = (float) a.y; m[2] = (float) a.z; m[3] = (float) a.w;
    m[4] = (float) b.x; m[5] = (float) b.y; m[6] = (float) b.z; m[7] = (float) b.w;
  } else {
#pragma unroll
    for (int k = 0; k < 8; ++k) m[k] = (t + k < V) ? (float) mult[t + k] : 1.f;
  }
}

template <bool VEC>
__device__ __forceinline__ void store8(float *out, int32_t t, int32_t V, const float *v) {
  if (VEC && t + 8 <= V) {
    *reinterpret_cast<float4 *>(out + t) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(out + t + 4) = make_float4(v[4], v[5], v[6], v[7]);
  } else {
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (t + k < V) out[t + k] = v[k];
  }
}

constexpr int kAcceptThreads = 1024;   // 16 waves: one per row to merge / per position to probe
constexpr int kAcceptTokens = kAcceptThreads * kTokensPerThread;   // delta tokens per workgroup

// State of one sequence's accept scan, in LDS.
struct AcceptShared {
  RowStat st_t[PCG_MAX_K + 1];                 // statistics of the target rows 0..K
  RowStat st_d[PCG_MAX_K];                     // ... and of the draft rows 0..K-1
  double Tp[PCG_MAX_K], Dp[PCG_MAX_K];         // probe sums relative to the group's own maxima
  double Tn[PCG_MAX_K], Dn[PCG_MAX_K];         // T_i[g], D_i[g] of the proposed groups
  float Tref[PCG_MAX_K], Dref[PCG_MAX_K];      // those maxima
  float uacc[PCG_MAX_K];                       // accept uniforms
  int bad[PCG_MAX_K], ptok[PCG_MAX_K], pgrp[PCG_MAX_K];
  int istar;                                   // accept_len of the sequence
};

// Statistics of one row from its parts, by the 16 lanes of one DPP row (sub = lane & 15); four
// rows are merged per wave at once.  Every lane of the 16 returns the result.
__device__ __forceinline__ RowStat merge_row16(const StatPart *parts, int64_t row, int32_t nparts,
                                               float c, int sub) {
  const StatPart *rp = parts + row * nparts;
  // a lane's first two parts stay in registers (rows of up to 65 536 logits: all of them), so
  // that the maximum and the sum need one trip to memory, not two
  constexpr int kKeep = 2;
  StatPart keep[kKeep];
  float M = -INFINITY;
#pragma unroll
  for (int j = 0; j < kKeep; ++j) {
    const int32_t k = sub + 16 * j;
    keep[j].z = 0.0; keep[j].m = -INFINITY; keep[j].t = 0.f;
    if (k < nparts) keep[j] = rp[k];
  }
#pragma unroll
  for (int j = 0; j < kKeep; ++j) M = fmaxf(M, keep[j].m);
  for (int32_t k = sub + 16 * kKeep; k < nparts; k += 16) M = fmaxf(M, rp[k].m);
  M = fmaxf(M, dpp_get<kDppXor1, 0xf>(M, M));
  M = fmaxf(M, dpp_get<kDppXor2, 0xf>(M, M));
  M = fmaxf(M, dpp_get<kDppHalfMirror, 0xf>(M, M));
  M = fmaxf(M, dpp_get<kDppMirror, 0xf>(M, M));
  double Z = 0.0;
#pragma unroll
  for (int j = 0; j < kKeep; ++j)
    if (keep[j].z > 0.0) Z += keep[j].z * exp2((double) keep[j].t - (double) M * (double) c);
  for (int32_t k = sub + 16 * kKeep; k < nparts; k += 16) {
    const StatPart sp = rp[k];
    if (sp.z > 0.0) Z += sp.z * exp2((double) sp.t - (double) M * (double) c);
  }
  RowStat r;
  r.Z = subwave_sum<16>(Z);
  r.M = M;
  r.pad = 0.f;
  return r;
}

// The accept scan of sequence b (Algorithm 1 up to the first rejection) by one workgroup of
// kAcceptThreads.  On return sh.istar, sh.st_t and sh.st_d are valid for every thread; with
// `writer` the sequence's outputs, row statistics and counters are written.
template <bool BF16>
__device__ void accept_phase(AcceptShared &sh, const AcceptArgs &a, int b, bool writer) {
  const int K = a.K;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  constexpr int nw = kAcceptThreads / kWave;
  const int64_t B = a.rs.nrows0 / (K + 1);
  // The probes of the proposed groups were formed by the statistics pass; the first wave fetches
  // them (one position per lane), the others merge the row statistics.
  const int nprobe = 1;
  if (wave == 0) {
    for (int i = lane; i < K; i += kWave) {
      const Probe p = a.probes[(int64_t) b * K + i];
      sh.Tp[i] = p.Tp; sh.Dp[i] = p.Dp; sh.Tref[i] = p.Tref; sh.Dref[i] = p.Dref;
      sh.bad[i] = p.bad;
      sh.pgrp[i] = a.prop_groups[(int64_t) b * K + i];
      sh.ptok[i] = a.prop_tokens[(int64_t) b * K + i];
      sh.uacc[i] = philox_uniforms(a.seed, a.offset, (uint32_t) b, (uint32_t) i).acc;
    }
  } else {
    // row statistics of this sequence's 2K+1 rows, four rows per wave at a time
    const int sub = lane & 15;
    for (int r = (wave - nprobe) * 4 + (lane >> 4); r < 2 * K + 1; r += (nw - nprobe) * 4) {
      const bool is_t = r <= K;
      const int64_t row = is_t ? (int64_t) b * (K + 1) + r : B * (K + 1) + (int64_t) b * K + (r - K - 1);
      const RowStat s = merge_row16(a.parts, row, a.nparts, a.c, sub);
      if (sub == 0) {
        if (writer) a.rowstat[row] = s;
        if (is_t) sh.st_t[r] = s; else sh.st_d[r - K - 1] = s;
      }
    }
  }
  __syncthreads();

  // Both chains have met.  One wave, one position per lane (K <= 64): normalise the probe,
  // take the accept test, and find the first rejection with a ballot; the draft token stands
  // for its group on accept.
  if (wave == 0) {
    const int i = lane;
    const bool in = i < K;
    double T = 0.0, D = 0.0, u = 0.0;
    bool bad = false;
    if (in) {
      if (sh.Tp[i] > 0.0) T = sh.Tp[i] * exp2((double) (sh.Tref[i] - sh.st_t[i].M) * a.cd) / sh.st_t[i].Z;
      if (sh.Dp[i] > 0.0) D = sh.Dp[i] * exp2((double) (sh.Dref[i] - sh.st_d[i].M) * a.cd) / sh.st_d[i].Z;
      u = (double) sh.uacc[i];
      bad = sh.bad[i] != 0;
      sh.Tn[i] = T;
      sh.Dn[i] = D;
    }
    const unsigned long long rejects = __ballot(in && !(u * D < T));
    const int istar = rejects ? __ffsll((long long) rejects) - 1 : K;
    const bool evaluated = in && i <= istar;
    const uint32_t near = __popcll(__ballot(evaluated && fabs(u * D - T) < 1e-6 * D));
    const uint32_t zero_d = __popcll(__ballot(evaluated && !bad && D == 0.0));
    const uint32_t nbad = __popcll(__ballot(evaluated && bad));
    if (lane == 0) sh.istar = istar;
    if (writer) {
      int32_t *otok = a.out_tokens + (int64_t) b * (K + 1);
      int32_t *ogrp = a.out_groups + (int64_t) b * (K + 1);
      for (int k = lane; k <= K; k += kWave) {
        otok[k] = k < istar ? sh.ptok[k] : -1;
        ogrp[k] = k < istar ? sh.pgrp[k] : -1;
      }
      if (lane == 0) {
        a.accept_len[b] = istar;
        if (a.diag) {
          if (near) atomicAdd(&a.diag->near_accept, near);
          if (zero_d) atomicAdd(&a.diag->zero_draft_mass, zero_d);
          if (nbad) atomicAdd(&a.diag->bad_proposal, nbad);
          atomicAdd(&a.diag->accepted_total, (uint32_t) istar);
          atomicAdd(&a.diag->sequences, 1u);
        }
      }
    }
  }
  __syncthreads();
}

// accept + delta.  Workgroup (b, s) runs the whole accept scan of sequence b -- every one of
// the sequence's workgroups does, so that none has to wait for another -- and then writes its
// slices of the table the gather sums over, on the decision row i* = accept_len[b]:
//   rejected (i* < K):  delta[t] = (q_{i*}(t) - p_{i*}(t)) / N(t)
//   bonus    (i* = K):  delta[t] =  q_K(t) / N(t)
// Workgroup s = 0 also writes the sequence's outputs, row statistics and counters.
// VEC: rows, mult and the table are 16-byte aligned and V is a multiple of 8.
template <bool BF16, bool VEC>
__global__ __launch_bounds__(kAcceptThreads) void accept_delta_kernel(AcceptArgs a, int32_t nsplit,
                                                                      float c_lo, float *table) {
  __shared__ AcceptShared sh;
  const int b = blockIdx.x / nsplit;
  const int split = blockIdx.x % nsplit;
  const RowSet &rs = a.rs;
  const int32_t V = a.V, K = a.K;
  const float c = a.c;
  const int32_t *mult = a.weights ? nullptr : a.mult;   // with weights delta is q - p as it is
  const int32_t stride = nsplit * kAcceptTokens;
  const int32_t first = split * kAcceptTokens + threadIdx.x * kTokensPerThread;
  // the multiplicities of this thread's first two slices do not depend on the decision row:
  // they are asked for before the accept scan
  float m_a[8], m_b[8];
  if (first < V) load8_mult<VEC>(mult, first, V, m_a);
  if (first + stride < V) load8_mult<VEC>(mult, first + stride, V, m_b);
  accept_phase<BF16>(sh, a, b, split == 0);

  // 4. this workgroup's share of the table on the decision row: slices split, split + nsplit, ...
  const int32_t istar = sh.istar;
  const bool rejected = istar < K;
  const void *trow = row_base(rs, (int64_t) b * (K + 1) + istar, BF16);
  const void *drow = row_base(rs, rs.nrows0 + (int64_t) b * K + (rejected ? istar : 0), BF16);
  const RowStat st = sh.st_t[istar];
  const RowStat sd = sh.st_d[rejected ? istar : 0];
  const double izt = 1.0 / st.Z, izd = rejected ? 1.0 / sd.Z : 0.0;
  auto delta8 = [&](const float *xt, const float *xd, const float *m, float *v) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float et = exp_rel(xt[k], st.M, c, c_lo);
      // two rounded products and a rounded difference (no fused multiply-add), so that
      // identical target and draft rows give exactly zero
      double diff = __dmul_rn((double) et, izt);
      if (rejected) {
        const float ed = exp_rel(xd[k], sd.M, c, c_lo);
        diff = __dsub_rn(diff, __dmul_rn((double) ed, izd));
      }
      v[k] = (float) diff * __builtin_amdgcn_rcpf(m[k]);   // N(t) is a small integer: 1 ulp, a tenth of a division's cost
    }
  };
  float *out = table + (int64_t) b * V;
  // two slices per turn, so that the loads of the second are in flight behind the first
  for (int32_t t = first; t < V; t += 2 * stride) {
    const int32_t t2 = t + stride;
    float xt[8], xd[8], m[8], v[8], xt2[8], xd2[8], m2[8];
    load8<BF16, VEC>(trow, t, V, xt);
    if (rejected) load8<BF16, VEC>(drow, t, V, xd);
    if (t2 < V) {
      load8<BF16, VEC>(trow, t2, V, xt2);
      if (rejected) load8<BF16, VEC>(drow, t2, V, xd2);
    }
    if (t == first) {
#pragma unroll
      for (int k = 0; k < 8; ++k) { m[k] = m_a[k]; m2[k] = m_b[k]; }
    } else {
      load8_mult<VEC>(mult, t, V, m);
      if (t2 < V) load8_mult<VEC>(mult, t2, V, m2);
    }
    delta8(xt, xd, m, v);
    store8<VEC>(out, t, V, v);
    if (t2 < V) {
      delta8(xt2, xd2, m2, v);
      store8<VEC>(out, t2, V, v);
    }
  }
}

// =============================================================================================
// accept + thinning: the reject branch drawn the paper's own way (Sec. 2.2 "Residual sampling
// via thinning", Eq. 9), with no enumeration of the groups: y ~ q, one of the groups holding y
// by the weights, accepted with probability [1 - D/T]_+, repeated until one is.  One workgroup
// per sequence; its 16 waves run 16 trials at a time and the first accepted one (in trial
// order) is emitted, so the result is that of running the trials one after the other.
// =============================================================================================

constexpr int kMaxThinParts = 2048;       // parts of a row the token draw can search (V <= 4 Mi)
constexpr int kThinTrialWaves = 16;       // trials a workgroup runs side by side, one per wave

struct WavePick {
  int32_t index;            // first index whose running sum exceeds u * total; -1: nothing has mass
  double total, goal, lo, hi;
};

// Inverse CDF over f(0..n-1) >= 0 by one wave (ascending order; every lane gets the result).
// `total` < 0: the sum of f is formed here first.
template <typename F>
__device__ WavePick wave_inverse_cdf(int32_t n, F f, double u, int lane, double total = -1.0) {
  if (total < 0.0) {
    total = 0.0;
    for (int32_t j = lane; j < n; j += kWave) {
      const double v = f(j);
      if (v > 0.0) total += v;
    }
    total = wave_sum(total);
  }
  WavePick r;
  r.total = total;
  r.goal = u * total;
  r.index = -1;
  r.lo = r.hi = 0.0;
  double base = 0.0;
  int32_t last = -1;
  double last_v = 0.0;
  for (int32_t j0 = 0; j0 < n; j0 += kWave) {
    const int32_t j = j0 + lane;
    double v = j < n ? f(j) : 0.0;
    if (!(v > 0.0)) v = 0.0;
    const double inc = wave_scan(v);
    const unsigned long long pos = __ballot(v > 0.0);
    if (pos) {
      const int hl = 63 - __clzll((long long) pos);
      last = j0 + hl;
      last_v = read_lane(v, hl);
    }
    const unsigned long long hit = __ballot(v > 0.0 && base + inc > r.goal);
    if (hit) {
      const int l = __ffsll((long long) hit) - 1;
      r.index = j0 + l;
      r.hi = base + read_lane(inc, l);
      r.lo = r.hi - read_lane(v, l);
      return r;
    }
    base += read_lane(inc, kWave - 1);
  }
  if (last >= 0) {   // rounding at the top end: the last index that has mass
    r.index = last;
    r.hi = total;
    r.lo = total - last_v;
  }
  return r;
}

__device__ __forceinline__ bool near_edge(const WavePick &p) {
  return (p.lo > 0.0 && p.goal - p.lo < 1e-6 * p.total) ||
         (p.hi < p.total && p.hi - p.goal < 1e-6 * p.total);
}

// Which of the n membership entries of a token (reverse-index positions e0 .. e0+n-1) the
// 24-bit draw picks, K ~ w_{k,x} over k in S(x) (Eq. 6): entry (k24 n) >> 24 under the equal
// split, else the inverse CDF of the entries' weights at k24 / 2^24, by the whole wave.
// *near: that draw is within 1e-6 of an inner edge of the chosen entry's bin.
__device__ __forceinline__ int32_t pick_entry(const float *tok_weights, int32_t e0, int32_t n,
                                              uint32_t k24, int lane, bool *near) {
  *near = false;
  if (!tok_weights) return (int32_t) (((uint64_t) k24 * (uint64_t) max(n, 1)) >> 24);
  const WavePick pk = wave_inverse_cdf(
      n, [&](int32_t e) { return (double) tok_weights[e0 + e]; }, (double) k24 * (1.0 / 16777216.0), lane);
  if (pk.index < 0) return 0;
  *near = near_edge(pk);
  return pk.index;
}

// Masses of the parts of one row, as the token draw reads them.
struct PartMasses {
  double Zp[kMaxThinParts];     // mass of each part relative to the row maximum, 2^(M c)
  double up[kMaxThinParts];     // 2^(M c - t): from the row's units to the part's own
  float tp[kMaxThinParts];      // log2-domain reference t of each part
};

// Filled by the calling threads (tid of nthreads) from the statistics of row `rp`; a barrier
// must follow.
__device__ __forceinline__ void fill_part_masses(PartMasses &pm, const StatPart *rp, int32_t nparts,
                                                 float M, float c, int tid, int nthreads) {
  for (int32_t p = tid; p < nparts; p += nthreads) {
    const StatPart sp = rp[p];
    const double e = exp2((double) sp.t - (double) M * (double) c);
    const bool has = sp.z > 0.0 && e > 0.0;
    pm.Zp[p] = has ? sp.z * e : 0.0;
    pm.up[p] = has ? 1.0 / e : 0.0;
    pm.tp[p] = sp.t;
  }
}

struct ThinShared {
  PartMasses pm;
  uint32_t redo[kThinTrialWaves][32];     // per wave: one lane's 32 logits, spread over the lanes
  int accepted[kThinTrialWaves], group[kThinTrialWaves];
  int token[kThinTrialWaves], near[kThinTrialWaves];
  int done;
};

// 32 consecutive logits of a row as loaded: bf16 stays packed two per register.
template <bool BF16>
struct Logits32 {
  static constexpr int kWords = BF16 ? 16 : 32;
  uint32_t w[kWords];
  __device__ __forceinline__ float get(int k) const {
    if constexpr (BF16) return __uint_as_float((k & 1) ? (w[k >> 1] & 0xffff0000u) : (w[k >> 1] << 16));
    else return __uint_as_float(w[k]);
  }
};

// Tokens e0 .. e0+31 of a row; tokens at or beyond V read as -inf.
template <bool BF16, bool VEC>
__device__ __forceinline__ void load32(const void *row, int32_t e0, int32_t V, Logits32<BF16> &r) {
  constexpr int nvec = BF16 ? 4 : 8;
  if (VEC && e0 + 32 <= V) {
    const uint4 *src = reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(row) +
                                                       (size_t) e0 * (BF16 ? 2 : 4));
#pragma unroll
    for (int i = 0; i < nvec; ++i) {
      const uint4 q = src[i];
      r.w[4 * i] = q.x; r.w[4 * i + 1] = q.y; r.w[4 * i + 2] = q.z; r.w[4 * i + 3] = q.w;
    }
  } else {
    const uint32_t ninf = BF16 ? 0xff80u : 0xff800000u;
#pragma unroll
    for (int k = 0; k < 32; ++k) {
      uint32_t bits = ninf;
      if (e0 + k < V) {
        if constexpr (BF16) bits = reinterpret_cast<const uint16_t *>(row)[e0 + k];
        else bits = reinterpret_cast<const uint32_t *>(row)[e0 + k];
      }
      if constexpr (BF16) {
        if (k & 1) r.w[k >> 1] |= bits << 16; else r.w[k >> 1] = bits;
      } else {
        r.w[k] = bits;
      }
    }
  }
}

// y ~ q on the row whose part masses are in pm: the part by its mass, then the lane inside the
// part (each lane sums 32 consecutive tokens), then the token among that lane's 32, which are
// handed to 32 lanes through `redo` (32 words of LDS private to the calling wave).
// *near: the draw is within 1e-6 of an inner edge of the token's bin.
template <bool BF16, bool VEC>
__device__ int32_t draw_token(const PartMasses &pm, uint32_t *redo, const void *trow, int32_t V,
                              int32_t nparts, float c, double u, int lane, bool *near) {
  const WavePick pp = wave_inverse_cdf(nparts, [&](int32_t p) { return pm.Zp[p]; }, u, lane);
  if (pp.index < 0) { *near = false; return 0; }
  const int32_t p = pp.index;
  const float t = pm.tp[p];
  const int32_t e0 = p * kPartElems + lane * 32;
  Logits32<BF16> raw;
  load32<BF16, VEC>(trow, e0, V, raw);
  // the same expression row_stats summed
  auto mass = [&](float x) -> float {
    return x > -INFINITY ? __builtin_amdgcn_exp2f(fmaf(x, c, -t)) : 0.f;
  };
  double s = 0.0;
#pragma unroll
  for (int k = 0; k < 32; k += 2) s += (double) mass(raw.get(k)) + (double) mass(raw.get(k + 1));
  const double inc = wave_scan(s);
  // threshold in the part's own units: masses there are relative to 2^t, in Zp to 2^(M c)
  const double scale = pm.up[p];
  const double goal = (pp.goal - pp.lo) * scale;
  const double part_total = read_lane(inc, kWave - 1);
  const unsigned long long hit = __ballot(s > 0.0 && inc > goal);
  const unsigned long long pos = __ballot(s > 0.0);
  if (!pos) { *near = false; return min(p * kPartElems, V - 1); }   // cannot happen: Zp[p] > 0
  const int l = hit ? __ffsll((long long) hit) - 1 : 63 - __clzll((long long) pos);
  // lane l's 32 tokens, one per lane
  if (lane == l) {
#pragma unroll
    for (int k = 0; k < Logits32<BF16>::kWords; ++k) redo[k] = raw.w[k];
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  float x = -INFINITY;
  if (lane < 32) {
    if constexpr (BF16) x = __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(redo)[lane] << 16);
    else x = __uint_as_float(redo[lane]);
  }
  const double v = (double) mass(x);
  const double before = read_lane(inc, l) - read_lane(s, l);
  const double cum = before + wave_scan(v);
  const unsigned long long hit2 = __ballot(v > 0.0 && cum > goal);
  const unsigned long long pos2 = __ballot(v > 0.0);
  const int k = hit2 ? __ffsll((long long) hit2) - 1 : 63 - __clzll((long long) pos2);
  const double hi = read_lane(cum, k), lo = hi - read_lane(v, k);
  const int32_t y = p * kPartElems + l * 32 + k;
  const double tot_units = pp.total * scale;
  const bool first_mass = pp.lo <= 0.0 && lo <= 0.0;            // no bin below
  const bool last_mass = pp.hi >= pp.total && hi >= part_total;  // no bin above
  *near = (!first_mass && goal - lo < 1e-6 * tot_units) || (!last_mass && hi - goal < 1e-6 * tot_units);
  return y;
}

template <bool BF16, bool VEC>
__global__ __launch_bounds__(kAcceptThreads) void accept_thin_kernel(
    AcceptArgs a, const int32_t *tok_ptr, const int32_t *tok_groups, const float *tok_weights,
    int32_t *trials, int32_t max_trials) {
  __shared__ AcceptShared sh;
  __shared__ ThinShared th;
  const int b = blockIdx.x;
  accept_phase<BF16>(sh, a, b, true);
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int32_t K = a.K, V = a.V, istar = sh.istar;
  const bool bonus = istar == K;
  const int64_t trow_id = (int64_t) b * (K + 1) + istar;
  const void *trow = row_base(a.rs, trow_id, BF16);
  const void *drow = row_base(a.rs, a.rs.nrows0 + (int64_t) b * K + (bonus ? 0 : istar), BF16);
  const RowStat st = sh.st_t[istar];
  const RowStat sd = sh.st_d[bonus ? 0 : istar];
  const float c_lo = (float) (a.cd - (double) a.c);

  fill_part_masses(th.pm, a.parts + trow_id * a.nparts, a.nparts, st.M, a.c, threadIdx.x, kAcceptThreads);
  if (threadIdx.x == 0) th.done = 0;
  __syncthreads();

  // q(t) w and p(t) w of CSR entry j holding token t (w = 1 / N(t) under the equal split), up
  // to the rows' normalisations, in the kernels' precision (fp32)
  const float *wts = a.weights;
  auto wq = [&](int32_t j, int32_t t) -> double {
    const float e = exp_rel(logit_at<BF16>(trow, t), st.M, a.c, c_lo);
    return (double) (wts ? e * wts[j] : e / (float) a.mult[t]);
  };
  auto wp = [&](int32_t j, int32_t t) -> double {
    const float e = exp_rel(logit_at<BF16>(drow, t), sd.M, a.c, c_lo);
    return (double) (wts ? e * wts[j] : e / (float) a.mult[t]);
  };

  // Trials run kThinTrialWaves at a time, one per wave; the other waves only keep the barriers.
  for (int32_t round = 0;; ++round) {
    const int32_t trial = round * kThinTrialWaves + wave;
    const bool active = wave < kThinTrialWaves && (bonus ? trial == 0 : trial < max_trials);
    if (active) {   // uniform over the wave
      const TrialDraws d = philox_trial(a.seed, a.offset, (uint32_t) b, (uint32_t) istar,
                                        (uint32_t) trial);
      bool near_y = false;
      const int32_t y = draw_token<BF16, VEC>(th.pm, th.redo[wave], trow, V, a.nparts, a.c,
                                              (double) d.u_y, lane, &near_y);
      const int32_t e0 = tok_ptr[y], n = tok_ptr[y + 1] - e0;
      bool near_e = false;
      const int32_t g = tok_groups[e0 + pick_entry(tok_weights, e0, n, d.k24, lane, &near_e)];
      const int32_t beg = a.row_ptr[g], len = a.row_ptr[g + 1] - beg;
      int accepted = 1, near = near_y || near_e ? 1 : 0;
      int32_t token = y;
      if (!bonus) {
        // the first 64 members stay in registers for the token draw below
        const int32_t t0 = lane < len ? a.members[beg + lane] : -1;
        const double q0 = t0 >= 0 ? wq(beg + lane, t0) : 0.0;
        double at = q0, ad = t0 >= 0 ? wp(beg + lane, t0) : 0.0;
        for (int32_t j = lane + kWave; j < len; j += kWave) {
          const int32_t t = a.members[beg + j];
          at += wq(beg + j, t);
          ad += wp(beg + j, t);
        }
        const double Tn = wave_sum(at), T = Tn / st.Z, D = wave_sum(ad) / sd.Z;
        const double ua = (double) d.u_a;
        accepted = ua * T < T - D;                    // u_a < [1 - D/T]_+
        if (fabs(ua * T - (T - D)) < 1e-6 * T) near |= 1;
        const WavePick pt = wave_inverse_cdf(
            len, [&](int32_t j) { return j < kWave ? q0 : wq(beg + j, a.members[beg + j]); },
            (double) d.u_tok, lane, Tn);
        token = pt.index < 0 ? -1 : (pt.index < kWave ? read_lane(t0, pt.index) : a.members[beg + pt.index]);
        if (pt.index >= 0 && near_edge(pt)) near |= 2;
      }
      if (lane == 0) {
        th.accepted[wave] = accepted; th.group[wave] = g; th.token[wave] = token; th.near[wave] = near;
      }
    } else if (lane == 0 && wave < kThinTrialWaves) {
      th.accepted[wave] = -1;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      uint32_t n_near = 0, n_near_tok = 0;
      int chosen = -1, last_active = -1;
      for (int w = 0; w < kThinTrialWaves && chosen < 0; ++w) {
        if (th.accepted[w] < 0) break;
        last_active = w;
        if (th.near[w] & 1) ++n_near;
        if (th.accepted[w] == 1) chosen = w;
      }
      const bool exhausted = chosen < 0 && (round + 1) * kThinTrialWaves >= max_trials;
      if (exhausted) chosen = last_active;
      if (chosen >= 0) {
        if (th.near[chosen] & 2) ++n_near_tok;
        a.out_groups[(int64_t) b * (K + 1) + istar] = th.group[chosen];
        a.out_tokens[(int64_t) b * (K + 1) + istar] = th.token[chosen];
        trials[b] = bonus ? 0 : round * kThinTrialWaves + chosen + 1;
        th.done = 1;
      }
      if (a.diag) {
        if (n_near) atomicAdd(&a.diag->near_group, n_near);
        if (n_near_tok) atomicAdd(&a.diag->near_token, n_near_tok);
        if (exhausted) atomicAdd(&a.diag->residual_fallback, 1u);
      }
    }
    __syncthreads();
    if (th.done) break;
  }
}

// =============================================================================================
// propose: the draft-side coupling (Sec. 2.2 "Proposal coupling and acceptance", Eq. 6).  One
// wave per draft row: merge the row's part statistics, draw x ~ p through the parts, then one
// of the membership entries of x.
// =============================================================================================

template <bool BF16, bool VEC>
__global__ __launch_bounds__(kWave) void propose_kernel(
    RowSet rs, int32_t V, int32_t K, int32_t pos0, int32_t nparts, float c, const StatPart *parts,
    const int32_t *tok_ptr, const int32_t *tok_groups, const float *tok_weights, uint64_t seed,
    uint64_t offset, int32_t *prop_tokens, int32_t *prop_groups, pcg_diag *diag) {
  __shared__ PartMasses pm;
  __shared__ uint32_t redo[32];
  const int lane = threadIdx.x;
  const int64_t row = blockIdx.x;
  const StatPart *rp = parts + row * nparts;
  float M = -INFINITY;
  for (int32_t p = lane; p < nparts; p += kWave) M = fmaxf(M, rp[p].m);
  M = wave_max(M);
  fill_part_masses(pm, rp, nparts, M, c, lane, kWave);
  __syncthreads();
  int64_t b;
  int32_t i;
  split_row(row, K, rs.inv_npos0, b, i);
  const ProposalDraws d = philox_proposal(seed, offset, (uint32_t) b, (uint32_t) (pos0 + i));
  bool near = false;
  const int32_t x = draw_token<BF16, VEC>(pm, redo, row_base(rs, row, BF16), V, nparts, c,
                                          (double) d.u_x, lane, &near);
  const int32_t e0 = tok_ptr[x], n = tok_ptr[x + 1] - e0;
  bool near_e = false;
  const int32_t e = pick_entry(tok_weights, e0, n, d.k24, lane, &near_e);
  if (lane == 0) {
    prop_tokens[row] = x;
    prop_groups[row] = tok_groups[e0 + e];
    if (diag) {
      if (near || near_e) atomicAdd(&diag->near_token, 1u);
      atomicAdd(&diag->sequences, 1u);
    }
  }
}

// =============================================================================================
// weights: the per-token table of pcg_group_probs.
// =============================================================================================

constexpr int kTableThreads = 256;
constexpr int kTableTokens = kTableThreads * kTokensPerThread;    // tokens per workgroup

// group_probs: w[r][t] = softmax(row r)[t] / N(t) for a batch of rows starting at row0.
template <bool BF16, bool VEC>
__global__ __launch_bounds__(kTableThreads) void weights_kernel(
    RowSet rs, int32_t V, int32_t nparts, int32_t nct, int64_t row0, float c, float c_hi,
    float c_lo, const StatPart *parts, const int32_t *mult, float *table) {
  __shared__ RowStat sh;
  const int32_t local = blockIdx.x / nct;
  const int64_t row = row0 + local;
  if (threadIdx.x < kWave) {
    RowStat s = merge_row(parts, row, nparts, c, threadIdx.x);
    if (threadIdx.x == 0) sh = s;
  }
  __syncthreads();
  const int32_t t = (blockIdx.x % nct) * kTableTokens + threadIdx.x * kTokensPerThread;
  if (t >= V) return;
  const RowStat s = sh;
  const double iz = 1.0 / s.Z;
  const void *rowp = row_base(rs, row, BF16);
  float x[8], m[8], v[8];
  load8<BF16, VEC>(rowp, t, V, x);
  load8_mult<VEC>(mult, t, V, m);
#pragma unroll
  for (int k = 0; k < 8; ++k)
    v[k] = (float) ((double) exp_rel(x[k], s.M, c_hi, c_lo) * iz) * __builtin_amdgcn_rcpf(m[k]);
  store8<VEC>(table + (int64_t) local * V, t, V, v);
}

// =============================================================================================
// gather: out[r][g] = sum over members t of G_g of table[r][t], table row staged in LDS.
// =============================================================================================


// Workgroup id -> (row, chunk).  Workgroups are dealt to the 8 XCDs round-robin by id, so all
// chunks of one row are given ids that are equal mod 8: they then share that XCD's L2 for the
// table row and none other holds it.
template <int W, bool CLAMP>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(
    int32_t V, int32_t G, int32_t nrows, int32_t nchunks, int32_t groups_per_chunk,
    int32_t ntiles, int32_t tile_len, const int32_t *row_ptr, const int32_t *members,
    const float *weights, const float *table, float *out) {
  __shared__ float tab[kTileMax];
  const int xcd = blockIdx.x & 7;
  const int y = blockIdx.x >> 3;
  const int r = xcd + 8 * (y / nchunks);
  const int chunk = y % nchunks;
  if (r >= nrows) return;   // whole workgroup leaves together, before any barrier
  const float *src = table + (int64_t) r * V;
  float *dst = out + (int64_t) r * G;
  const int32_t g_begin = chunk * groups_per_chunk;
  const int32_t g_end = min(G, g_begin + groups_per_chunk);
  constexpr int nsub = kGatherThreads / W;          // groups in flight per workgroup pass
  const int sub = threadIdx.x / W, sl = threadIdx.x % W;

  for (int tile = 0; tile < ntiles; ++tile) {
    const int32_t t0 = tile * tile_len;
    const int32_t tl = min(tile_len, V - t0);
    if (tl <= 0) break;                             // uniform: no tile starts past the row
    if (tile > 0) __syncthreads();                  // everyone is done reading the old tile
    for (int32_t k = threadIdx.x; k < tl; k += kGatherThreads) tab[k] = src[t0 + k];
    __syncthreads();
    // Every lane of a wave runs the same number of passes, so the DPP reduction below is
    // always executed by full waves.  A sub-wave takes kInFlight groups per pass, so that their
    // chains of dependent loads (row_ptr -> members -> table) overlap.
    constexpr int kInFlight = 8;
    for (int32_t gb = g_begin; gb < g_end; gb += nsub * kInFlight) {
      int32_t beg[kInFlight], end[kInFlight], mem[kInFlight];
      float wt[kInFlight], acc[kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {
        const int32_t g = gb + u * nsub + sub;
        const bool valid = g < g_end;
        beg[u] = valid ? row_ptr[g] : 0;
        end[u] = valid ? row_ptr[g + 1] : 0;
      }
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {       // first trip of each group
        const int32_t j = beg[u] + sl;
        const bool has = j < end[u];
        mem[u] = has ? members[j] : -1;
        wt[u] = has && weights ? weights[j] : 1.f;
      }
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {
        const uint32_t t = (uint32_t) (mem[u] - t0);
        acc[u] = 0.f;
        if (mem[u] >= 0 && t < (uint32_t) tl) acc[u] = weights ? tab[t] * wt[u] : tab[t];
      }
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {       // groups longer than the sub-wave
        for (int32_t j = beg[u] + sl + W; j < end[u]; j += W) {
          const uint32_t t = (uint32_t) (members[j] - t0);
          if (t < (uint32_t) tl) acc[u] += weights ? tab[t] * weights[j] : tab[t];
        }
      }
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {
        const int32_t g = gb + u * nsub + sub;
        float a = subwave_sum<W>(acc[u]);
        if (g < g_end && sl == W - 1) {
          if (tile > 0) a += dst[g];                // partial sum of the earlier tiles
          if (CLAMP && tile == ntiles - 1) a = fmaxf(a, 0.f);
          dst[g] = a;
        }
      }
    }
  }
}

// =============================================================================================
// finalize: group from the residual by inverse CDF, then the token inside it (Eq. 10).
// =============================================================================================

constexpr int kFinalThreads = 512;

struct CdfPick {
  int32_t index;    // first index whose running sum exceeds the threshold; -1 if nothing has mass
  double total, lo, hi;   // total mass; running sum before / after the chosen bin
};

// Inverse CDF over f(0..n-1) >= 0 by a whole workgroup of NT threads.  Each thread owns a
// contiguous run, so the running sum is the ascending one up to fp64 rounding.  All threads get
// the result.  The threshold is u * total, or `goal_in` (relative to this range) with have_goal.
template <int NT, int kRegRun = 32, typename F>   // kRegRun: runs up to this length are held in registers
__device__ CdfPick block_inverse_cdf(int32_t n, F f, double u, bool have_goal = false,
                                     double goal_in = 0.0) {
  __shared__ double wave_tot[NT / kWave];
  __shared__ int first_thread, last_pos;
  __shared__ CdfPick res;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int32_t run = (n + NT - 1) / NT;
  const int32_t lo_i = min(n, tid * run), hi_i = min(n, lo_i + run);
  const bool in_regs = run <= kRegRun;           // uniform
  if (tid == 0) { first_thread = INT_MAX; last_pos = -1; }
  double mine = 0.0;
  double vals[kRegRun];
  if (in_regs) {
    // all loads of the run are issued before the first is used
#pragma unroll
    for (int j = 0; j < kRegRun; ++j) vals[j] = (lo_i + j < hi_i) ? f(lo_i + j) : 0.0;
#pragma unroll
    for (int j = 0; j < kRegRun; ++j)
      if (vals[j] > 0.0) mine += vals[j];
  } else {
    for (int32_t k = lo_i; k < hi_i; ++k) {
      const double v = f(k);
      if (v > 0.0) mine += v;
    }
  }
  // inclusive scan inside the wave, then across waves
  const double inc = wave_scan(mine);
  if (lane == kWave - 1) wave_tot[wave] = inc;
  __syncthreads();
  double before = 0.0, total = 0.0;
  for (int w = 0; w < NT / kWave; ++w) {
    if (w < wave) before += wave_tot[w];
    total += wave_tot[w];
  }
  const double excl = before + (inc - mine);
  const double goal = have_goal ? goal_in : u * total;
  // the first thread whose run carries the running sum past the threshold: first lane of each
  // wave by ballot, then one LDS atomic per wave
  const unsigned long long hit = __ballot(mine > 0.0 && excl + mine > goal);
  if (hit != 0 && lane == __ffsll((long long) hit) - 1) atomicMin(&first_thread, tid);
  __syncthreads();
  const int ft = __builtin_amdgcn_readfirstlane(first_thread);   // the same in every lane
  if (kRegRun <= 4 && in_regs) {
    // a run of a few bins: thread ft walks its own registers
    if (ft == tid) {
      double cum = excl, last_v = 0.0;
      int32_t last = lo_i;
      bool done = false;
#pragma unroll
      for (int j = 0; j < kRegRun; ++j) {
        if (!done && vals[j] > 0.0) {
          const double nxt = cum + vals[j];
          if (nxt > goal) { res.index = lo_i + j; res.lo = cum; res.hi = nxt; done = true; }
          else { last = lo_i + j; last_v = vals[j]; cum = nxt; }
        }
      }
      if (!done) { res.index = last; res.lo = cum - last_v; res.hi = cum; }
      res.total = total;
    }
  } else if (in_regs && ft != INT_MAX) {
    // The crossing lies inside thread ft's run: its wave looks at the run's bins side by side, one
    // per lane (a run held in registers is at most 32 long), instead of thread ft walking them
    // one after the other.
    static_assert(kRegRun <= kWave, "one lane per bin of a run");
    if (wave == (ft >> 6)) {                     // uniform over the wave
      const int fl = ft & (kWave - 1);
      const double base = read_lane(excl, fl);
      const int32_t lo = read_lane(lo_i, fl), hi = read_lane(hi_i, fl);
      const int32_t k = lo + lane;
      double v = k < hi ? (double) f(k) : 0.0;
      if (!(v > 0.0)) v = 0.0;
      const double run_inc = wave_scan(v);
      const unsigned long long pos = __ballot(v > 0.0);
      const unsigned long long cross = __ballot(v > 0.0 && base + run_inc > goal);
      // the first bin that carries the sum past the threshold; rounding may leave none (the sum
      // of the run was taken in another order): then the last bin that has mass
      const int l = cross ? __ffsll((long long) cross) - 1 : 63 - __clzll((long long) pos);
      const double top = base + read_lane(run_inc, l), width = read_lane(v, l);
      if (lane == 0) {
        res.index = lo + l; res.hi = top; res.lo = top - width; res.total = total;
      }
    }
  } else if (ft == tid) {
    double cum = excl;
    int32_t last = lo_i;
    bool done = false;
    for (int32_t k = lo_i; k < hi_i && !done; ++k) {
      const double v = f(k);
      if (!(v > 0.0)) continue;
      const double nxt = cum + v;
      if (nxt > goal) { res.index = k; res.lo = cum; res.hi = nxt; done = true; }
      else { last = k; cum = nxt; }
    }
    if (!done) {   // summation order: excl + mine > goal, yet the walk stayed below: last bin
      const double v = (double) f(last);
      res.index = last; res.lo = cum - v; res.hi = cum;
    }
    res.total = total;
  }
  if (ft == INT_MAX) {
    // rounding at the top end (or no mass at all): the last index that has mass
    int32_t my_last = -1;
    for (int32_t k = lo_i; k < hi_i; ++k)
      if (f(k) > 0.0) my_last = k;
    if (my_last >= 0) atomicMax(&last_pos, my_last);
    __syncthreads();
    if (tid == 0) {
      res.index = last_pos; res.total = total; res.lo = total; res.hi = total;
      if (last_pos >= 0) res.lo = total - f(last_pos);
    }
  }
  __syncthreads();
  CdfPick out = res;
  __syncthreads();   // res / first_thread may be reused by the next call
  return out;
}

__device__ __forceinline__ bool near_edge(const CdfPick &p, double u) {
  const double goal = u * p.total;
  const bool near_lo = p.lo > 0.0 && (goal - p.lo) < 1e-6 * p.total;
  const bool near_hi = p.hi < p.total && (p.hi - goal) < 1e-6 * p.total;
  return near_lo || near_hi;
}

// The last step of a sequence, by one whole workgroup of NT threads.  After the CSR gather
// (csum == NULL) R holds the gathered sums T[g] - D[g] (T[g] on a bonus row), clamped here on
// read, and all of it is scanned.  After the prepared gather (csum, runs != NULL) there are no
// sums, only the totals of max(0, .) over chunks of chunk_groups consecutive groups and over runs
// of kRunGroups: the chunk and the run that hold the draw are located from them, and the run's
// sums are formed again here.
template <bool BF16, int NT>
__device__ void finalize_sequence(const FinalizeArgs &fa, int32_t V, int32_t G, int b,
                                  const double *csum, const double *runs, int32_t nchunks,
                                  int32_t chunk_groups) {
  const int32_t K = fa.K;
  const int32_t istar = fa.accept_len[b];
  const int64_t trow_id = (int64_t) b * (K + 1) + istar;
  const void *trow = row_base(fa.rs, trow_id, BF16);
  const RowStat st = fa.rowstat[trow_id];
  const Uniforms u = philox_uniforms(fa.seed, fa.offset, (uint32_t) b, (uint32_t) istar);
  float *Rb = fa.R + (int64_t) b * G;
  const int32_t *row_ptr = fa.row_ptr, *members = fa.members, *mult = fa.mult;
  const float *wts = fa.weights;
  const double cd = fa.cd;

  // q(t) w_{k,t} of CSR entry j on the decision row (q(t) / N(t) under the equal split), in double
  auto weight = [&](int32_t j) -> double {
    const int32_t t = members[j];
    const double e = exp2((double) (logit_at<BF16>(trow, t) - st.M) * cd);
    return wts ? e * (double) wts[j] / st.Z : e / (st.Z * (double) mult[t]);
  };

  CdfPick pg;
  if (csum) {
    // residual total and the chunk that holds u * total, from the per-chunk sums (ascending)
    const double *cs = csum + (int64_t) b * nchunks;
    double S = 0.0;
    for (int32_t c = 0; c < nchunks; ++c) S += cs[c];
    const double goal = (double) u.grp * S;
    double cum = 0.0, base = 0.0;
    int32_t cstar = -1;
    for (int32_t c = 0; c < nchunks; ++c) {
      const double v = cs[c];
      if (!(v > 0.0)) continue;
      cstar = c;
      base = cum;
      if (cum + v > goal) break;
      cum += v;
    }
    pg.index = -1; pg.total = S; pg.lo = pg.hi = 0.0;
    if (S > 0.0 && cstar >= 0) {
      const int32_t g0 = cstar * chunk_groups, ng = min(chunk_groups, G - g0);
      {
        // The gather left no sums, only the totals of runs of kRunGroups groups: find the run
        // that holds the crossing, form its groups' sums again -- 32 lanes per group, the table
        // kernel's arithmetic for every entry (Eq. 8 on the decision row) -- and walk them.
        static_assert(NT == kRunGroups * 32, "one half-wave per group of a run");
        __shared__ float run_r[kRunGroups];
        const int32_t nruns = (ng + kRunGroups - 1) / kRunGroups;
        const double *rp = runs + ((int64_t) b * nchunks + cstar) * (chunk_groups / kRunGroups);
        static_assert(kMaxChunkGroups / kRunGroups <= 2 * NT, "two runs per thread at most");
        const CdfPick pr = block_inverse_cdf<NT, 2>(
            nruns, [&](int32_t k) { return rp[k]; }, 0.0, true, goal - base);
        if (pr.index >= 0) {
          __shared__ int32_t run_n[kRunGroups];
          const bool rejected = istar < K;
          const void *drow = row_base(fa.rs, fa.rs.nrows0 + (int64_t) b * K + (rejected ? istar : 0), BF16);
          const RowStat sd = fa.rowstat[fa.rs.nrows0 + (int64_t) b * K + (rejected ? istar : 0)];
          const double izt = 1.0 / st.Z, izd = rejected ? 1.0 / sd.Z : 0.0;
          const int32_t gr0 = g0 + pr.index * kRunGroups;
          const int k = threadIdx.x >> 5, l = threadIdx.x & 31;
          const int32_t g = gr0 + k;
          float acc = 0.f;
          // the lane's first entry stays in registers: a group of up to 32 entries then has
          // everything the token draw needs in its half-wave
          int32_t n_g = 0, t_first = -1;
          float lt_first = -INFINITY, share_first = 1.f;
          if (g < g0 + ng) {
            const int32_t beg = row_ptr[g], end = row_ptr[g + 1];
            n_g = end - beg;
            for (int32_t j = beg + l; j < end; j += 32) {
              const int32_t t = members[j];
              const float lt = logit_at<BF16>(trow, t);
              const float share = wts ? wts[j] : (float) mult[t];      // w_{k,t}, or N(t)
              if (j == beg + l) { t_first = t; lt_first = lt; share_first = share; }
              const float et = exp_rel(lt, st.M, fa.c, fa.c_lo);
              double diff = __dmul_rn((double) et, izt);
              if (rejected) {
                const float ed = exp_rel(logit_at<BF16>(drow, t), sd.M, fa.c, fa.c_lo);
                diff = __dsub_rn(diff, __dmul_rn((double) ed, izd));
              }
              acc = wts ? fmaf((float) diff, share, acc)
                        : acc + (float) diff * __builtin_amdgcn_rcpf(share);
            }
          }
          acc = subwave_sum<32>(acc);                   // total in the last lane of each 32
          if (l == 31) { run_r[k] = fmaxf(acc, 0.f); run_n[k] = n_g; }
          __syncthreads();
          double cum = base + pr.lo, last_v = 0.0;
          int pick = -1, last = -1;
#pragma unroll
          for (int k2 = 0; k2 < kRunGroups; ++k2) {
            const double v = (double) run_r[k2];
            if (pick < 0 && v > 0.0) {
              if (cum + v > goal) { pick = k2; pg.lo = cum; pg.hi = cum + v; }
              else { last = k2; last_v = v; cum += v; }
            }
          }
          if (pick < 0) {
            // rounding (the run's total was summed in another order): the last group of the run
            // that has mass, or its first group if none has
            pick = last < 0 ? 0 : last;
            pg.hi = cum; pg.lo = cum - last_v;
          }
          pg.index = gr0 + pick;
          if (run_n[pick] <= 32) {                      // uniform over the workgroup
            // The token inside the group (Eq. 10) by the half-wave that formed the group's sum.
            const int wv = __builtin_amdgcn_readfirstlane(pick >> 1);
            if ((int) (threadIdx.x >> 6) == wv) {
              const int lane = threadIdx.x & (kWave - 1);
              double w = 0.0;
              if (k == pick && t_first >= 0) {
                const double e = exp2((double) (lt_first - st.M) * cd);
                w = wts ? e * (double) share_first / st.Z : e / (st.Z * (double) share_first);
                if (!(w > 0.0)) w = 0.0;
              }
              const double total = wave_sum(w);
              const double inc = wave_scan(w);
              const double goal_t = (double) u.tok * total;
              const unsigned long long pos = __ballot(w > 0.0);
              const unsigned long long hit = __ballot(w > 0.0 && inc > goal_t);
              CdfPick pt;
              pt.index = -1; pt.total = total; pt.lo = pt.hi = 0.0;
              int32_t tok = -1;
              if (pos) {
                const int src = hit ? __ffsll((long long) hit) - 1 : 63 - __clzll((long long) pos);
                pt.index = src & 31;
                pt.hi = hit ? read_lane(inc, src) : total;
                pt.lo = pt.hi - read_lane(w, src);
                tok = read_lane(t_first, src);
              }
              if (lane == 0) {
                fa.out_groups[(int64_t) b * (K + 1) + istar] = pg.index;
                fa.out_tokens[(int64_t) b * (K + 1) + istar] = tok;
                if (fa.diag) {
                  if (near_edge(pg, (double) u.grp)) atomicAdd(&fa.diag->near_group, 1u);
                  if (pt.index >= 0 && near_edge(pt, (double) u.tok)) atomicAdd(&fa.diag->near_token, 1u);
                }
              }
            }
            return;                                     // the whole workgroup, together
          }
        }
      }
    }
  } else {
    pg = block_inverse_cdf<NT>(G, [&](int32_t g) { return (double) fmaxf(Rb[g], 0.f); },
                               (double) u.grp);
  }
  bool fallback = false;
  if (!(pg.total > 0.0) || pg.index < 0) {
    // Residual total <= 0 (cannot happen in exact arithmetic): draw from T of this row instead.
    fallback = true;
    for (int32_t g = threadIdx.x; g < G; g += NT) {
      double s = 0.0;
      for (int32_t j = row_ptr[g]; j < row_ptr[g + 1]; ++j) s += weight(j);
      Rb[g] = (float) s;
    }
    __syncthreads();
    pg = block_inverse_cdf<NT>(G, [&](int32_t g) { return (double) Rb[g]; }, (double) u.grp);
  }
  const int32_t gs = pg.index < 0 ? 0 : pg.index;

  const int32_t beg = row_ptr[gs], end = row_ptr[gs + 1];
  CdfPick pt;
  constexpr int kTokRounds = 4;          // entries per lane the one-wave path keeps in registers
  if (end - beg <= kTokRounds * kWave) {
    // The token inside the group (Eq. 10) by the first wave alone: every entry's mass is loaded
    // once, all loads in flight together, and kept in registers for the total and for the scan.
    if (threadIdx.x < kWave) {
      const int lane = threadIdx.x;
      const int32_t n = end - beg;
      double w[kTokRounds];
#pragma unroll
      for (int c = 0; c < kTokRounds; ++c) {
        const int32_t j = c * kWave + lane;
        w[c] = j < n ? weight(beg + j) : 0.0;
        if (!(w[c] > 0.0)) w[c] = 0.0;
      }
      double total = 0.0;
#pragma unroll
      for (int c = 0; c < kTokRounds; ++c) total += wave_sum(w[c]);      // ascending, 64 at a time
      pt.index = -1; pt.total = total; pt.lo = pt.hi = 0.0;
      const double goal = (double) u.tok * total;
      double base = 0.0, last_v = 0.0;
      int32_t last = -1;
      bool done = false;
#pragma unroll
      for (int c = 0; c < kTokRounds; ++c) {
        if (done || c * kWave >= n) continue;                            // uniform
        const double inc = wave_scan(w[c]);
        const unsigned long long pos = __ballot(w[c] > 0.0);
        if (pos) {
          const int hl = 63 - __clzll((long long) pos);
          last = c * kWave + hl;
          last_v = read_lane(w[c], hl);
        }
        const unsigned long long hit = __ballot(w[c] > 0.0 && base + inc > goal);
        if (hit) {
          const int l = __ffsll((long long) hit) - 1;
          pt.index = c * kWave + l;
          pt.hi = base + read_lane(inc, l);
          pt.lo = pt.hi - read_lane(w[c], l);
          done = true;
        } else {
          base += read_lane(inc, kWave - 1);
        }
      }
      if (!done && last >= 0) {          // rounding at the top end: the last entry that has mass
        pt.index = last; pt.hi = total; pt.lo = total - last_v;
      }
    }
  } else {
    pt = block_inverse_cdf<NT>(end - beg, [&](int32_t j) { return weight(beg + j); }, (double) u.tok);
  }
  if (threadIdx.x == 0) {
    fa.out_groups[(int64_t) b * (K + 1) + istar] = gs;
    fa.out_tokens[(int64_t) b * (K + 1) + istar] = pt.index < 0 ? -1 : members[beg + pt.index];
    if (fa.diag) {
      if (pg.index >= 0 && near_edge(pg, (double) u.grp)) atomicAdd(&fa.diag->near_group, 1u);
      if (pt.index >= 0 && near_edge(pt, (double) u.tok)) atomicAdd(&fa.diag->near_token, 1u);
      if (fallback) atomicAdd(&fa.diag->residual_fallback, 1u);
    }
  }
}

// One workgroup per sequence.  csum / nchunks / chunk_groups describe the chunk totals the
// prepared gather wrote (csum == NULL after the CSR gather: the whole range is scanned).
template <bool BF16>
__global__ __launch_bounds__(kFinalThreads) void finalize_kernel(FinalizeArgs fa, int32_t V,
                                                                 int32_t G, const double *csum,
                                                                 const double *runs,
                                                                 int32_t nchunks,
                                                                 int32_t chunk_groups) {
  finalize_sequence<BF16, kFinalThreads>(fa, V, G, blockIdx.x, csum, runs, nchunks, chunk_groups);
}

// ---------------------------------------------------------------------------------------------
// The same sum read from the prepared layout (pcg_prepared): no cross-lane reduction and no
// address arithmetic beyond a shift.  A workgroup owns one chunk of consecutive groups of one
// table row.  Wave w owns the blocks block_of(q, w), q = 0..3, of the chunk and walks them side
// by side; lane l handles each block's 4 groups r*64 + l -- the same 16 groups in every tile
// pass, so their running sums stay in registers.  One 16-byte load per lane brings 2 slots for
// each of a block's 4 groups.  Results are put back into group order through LDS.  Without CSUM
// they leave with coalesced stores; with CSUM (the residual of pcg_verify, Eq. 8) only totals of
// max(0, .) leave, in double and summed in a fixed order: one per run of kRunGroups consecutive
// groups and one for the chunk.
// ---------------------------------------------------------------------------------------------

__device__ __forceinline__ void gather_step(const float *tab, const uint4 w, float *acc) {
  acc[0] += tab[w.x & 0xffffu]; acc[1] += tab[w.y & 0xffffu];
  acc[2] += tab[w.z & 0xffffu]; acc[3] += tab[w.w & 0xffffu];
  acc[0] += tab[w.x >> 16]; acc[1] += tab[w.y >> 16];
  acc[2] += tab[w.z >> 16]; acc[3] += tab[w.w >> 16];
}

// The same with general weights (Eq. 4): every slot comes with its w_{k,t}, 8 floats per lane
// and step next to the 8 slots.
__device__ __forceinline__ void gather_step_w(const float *tab, const uint4 s, const float4 a,
                                              const float4 b, float *acc) {
  acc[0] = fmaf(tab[s.x & 0xffffu], a.x, acc[0]); acc[1] = fmaf(tab[s.y & 0xffffu], a.z, acc[1]);
  acc[2] = fmaf(tab[s.z & 0xffffu], b.x, acc[2]); acc[3] = fmaf(tab[s.w & 0xffffu], b.z, acc[3]);
  acc[0] = fmaf(tab[s.x >> 16], a.y, acc[0]); acc[1] = fmaf(tab[s.y >> 16], a.w, acc[1]);
  acc[2] = fmaf(tab[s.z >> 16], b.y, acc[2]); acc[3] = fmaf(tab[s.w >> 16], b.w, acc[3]);
}

// One step of one block as it comes from memory: 8 slots and, with weights, their 8 weights.
template <bool WEIGHTED>
struct GatherStep;
template <>
struct GatherStep<false> {
  uint4 s;
  __device__ __forceinline__ void load(const uint4 *__restrict__ data, const float4 *, int lane) {
    s = data[lane];
  }
  __device__ __forceinline__ void apply(const float *tab, float *acc) const { gather_step(tab, s, acc); }
};
template <>
struct GatherStep<true> {
  uint4 s;
  float4 w0, w1;
  __device__ __forceinline__ void load(const uint4 *__restrict__ data,
                                       const float4 *__restrict__ wdata, int lane) {
    s = data[lane];
    w0 = wdata[2 * lane];
    w1 = wdata[2 * lane + 1];
  }
  __device__ __forceinline__ void apply(const float *tab, float *acc) const {
    gather_step_w(tab, s, w0, w1, acc);
  }
};

template <bool CSUM, bool WEIGHTED>
__global__ __launch_bounds__(kGatherThreads) void gather_prepared_kernel(
    int32_t V, int32_t G, int32_t nrows, int32_t nchunks, int32_t chunk_groups, int32_t ntiles,
    int32_t tile_len, int32_t bpc, const uint32_t *__restrict__ desc,
    const uint16_t *__restrict__ perm, const uint4 *__restrict__ data,
    const float4 *__restrict__ wdata, const float *__restrict__ table, float *__restrict__ out,
    double *__restrict__ csum, double *__restrict__ runs) {
  __shared__ __attribute__((aligned(16))) float tab[kTileMax];
  __shared__ double wsum[kGatherWaves];
  const int xcd = blockIdx.x & 7;
  const int y = blockIdx.x >> 3;
  const int r = xcd + 8 * (y / nchunks);
  const int chunk = y % nchunks;
  if (r >= nrows) return;   // whole workgroup leaves together, before any barrier
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int32_t g0 = chunk * chunk_groups;
  const int32_t ng = min(chunk_groups, G - g0);
  const float *src = table + (int64_t) r * V;

  float acc[kMaxAcc];
  uint16_t where[kMaxAcc];     // group (inside the chunk) behind each running sum; loaded now,
                               // needed only when the sums are put back into group order
#pragma unroll
  for (int q = 0; q < kMaxBlocksPerWave; ++q) {
    const int bl = block_of(q, wave);
#pragma unroll
    for (int rr = 0; rr < kLaneGroups; ++rr) {
      acc[q * kLaneGroups + rr] = 0.f;
      where[q * kLaneGroups + rr] =
          bl < bpc ? perm[((size_t) chunk * bpc + bl) * kBlockGroups + rr * kWave + lane]
                   : (uint16_t) 0xFFFFu;
    }
  }

  // descriptors (first unit and number of steps) of this wave's blocks in tile h
  auto load_desc = [&](int h, uint32_t (&steps)[kMaxBlocksPerWave], uint32_t (&offs)[kMaxBlocksPerWave]) {
    const uint32_t *dsc = desc + ((size_t) (chunk * ntiles + h) * bpc) * 2;
#pragma unroll
    for (int q = 0; q < kMaxBlocksPerWave; ++q) {
      const int bl = block_of(q, wave);
      steps[q] = 0;
      offs[q] = 0;
      if (bl < bpc && h < ntiles) {                   // uniform over the wave: scalar registers
        steps[q] = __builtin_amdgcn_readfirstlane(dsc[2 * bl + 1]);
        offs[q] = __builtin_amdgcn_readfirstlane(dsc[2 * bl]);
      }
    }
  };
  uint32_t steps[kMaxBlocksPerWave], offs[kMaxBlocksPerWave];
  load_desc(0, steps, offs);

  for (int h = 0; h < ntiles; ++h) {
    const int32_t t0 = h * tile_len;
    const int32_t tl = min(tile_len, V - t0);
    if (h > 0) __syncthreads();                       // everyone is done reading the old tile
    const bool direct = ((V | tl) & 3) == 0;          // rows and tiles are 16-byte aligned
    if (direct) {
      // global memory -> LDS directly, 16 bytes per lane: every load of the tile is in flight at
      // once and none passes through a register (a wave's instruction fills 1 KiB in lane order,
      // which is the table's own order)
      const float4 *s4 = reinterpret_cast<const float4 *>(src + t0);
      const int32_t n4 = tl >> 2;
      for (int32_t k0 = wave * kWave; k0 < n4; k0 += kGatherThreads)
        if (k0 + lane < n4)
          __builtin_amdgcn_global_load_lds(
              (const __attribute__((address_space(1))) void *) (s4 + k0 + lane),
              (__attribute__((address_space(3))) void *) (tab + 4 * k0), 16, 0, 0);
    } else {
      for (int32_t k = threadIdx.x; k < tl; k += kGatherThreads) tab[k] = src[t0 + k];
    }
    if (threadIdx.x < kBanks) tab[tile_len + threadIdx.x] = 0.f;   // the padding slots
    // The wave's blocks of this tile are walked side by side: turn s takes step s of every block
    // that has one (kSide blocks at a time: all four, or two when weights travel along), so one
    // loop with fixed registers serves them all; while a turn is gathered the next one is on its
    // way (a block that has run out re-reads its last step, which keeps every load in bounds and
    // the number of loads in flight the same on every turn).  The first turn and the next tile's
    // descriptors are asked for while the tile is still on its way into LDS.
    constexpr int kSide = WEIGHTED ? 2 : kMaxBlocksPerWave;
    GatherStep<WEIGHTED> bufX[kSide], bufY[kSide];
    uint32_t last[kMaxBlocksPerWave];                 // a block's last step (0 for a block without any)
#pragma unroll
    for (int q = 0; q < kMaxBlocksPerWave; ++q)
      last[q] = __builtin_amdgcn_readfirstlane(steps[q] > 0 ? steps[q] - 1 : 0u);
    auto fetch = [&](GatherStep<WEIGHTED> (&dst)[kSide], int q0, uint32_t turn) {
#pragma unroll
      for (int j = 0; j < kSide; ++j) {
        const uint32_t k = min(turn, last[q0 + j]);                         // scalar
        // a scalar base and the lane as the only vector part: no address arithmetic per load
        dst[j].load(data + ((size_t) offs[q0 + j] + (size_t) k * kWave), wdata + 2 * ((size_t) offs[q0 + j] + (size_t) k * kWave), lane);
      }
    };
    fetch(bufX, 0, 0);
    uint32_t nsteps[kMaxBlocksPerWave], noffs[kMaxBlocksPerWave];
    load_desc(h + 1, nsteps, noffs);
    if (direct) __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wave's part of the tile has landed
    __syncthreads();
#pragma unroll
    for (int q0 = 0; q0 < kMaxBlocksPerWave; q0 += kSide) {
      uint32_t turns = 0;
#pragma unroll
      for (int j = 0; j < kSide; ++j) turns = max(turns, steps[q0 + j]);
      if (q0 > 0) fetch(bufX, q0, 0);
      for (uint32_t t = 0; t < turns; t += 2) {
        fetch(bufY, q0, t + 1);
#pragma unroll
        for (int j = 0; j < kSide; ++j)
          if (t < steps[q0 + j]) bufX[j].apply(tab, acc + (q0 + j) * kLaneGroups);      // uniform
        if (t + 1 >= turns) break;
        fetch(bufX, q0, t + 2);
#pragma unroll
        for (int j = 0; j < kSide; ++j)
          if (t + 1 < steps[q0 + j]) bufY[j].apply(tab, acc + (q0 + j) * kLaneGroups);  // uniform
      }
    }
#pragma unroll
    for (int q = 0; q < kMaxBlocksPerWave; ++q) { steps[q] = nsteps[q]; offs[q] = noffs[q]; }
  }

  // back into group order through LDS, then coalesced stores
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kMaxAcc; ++j)
    if (where[j] != 0xFFFFu) tab[where[j]] = acc[j];
  __syncthreads();
  if constexpr (!CSUM) {
    float *dst = out + (int64_t) r * G + g0;
    if ((((uintptr_t) dst | (uintptr_t) ng) & 15) == 0 && (ng & 3) == 0) {      // 16 bytes at a time
      for (int32_t i = 4 * threadIdx.x; i < ng; i += 4 * kGatherThreads)
        *reinterpret_cast<float4 *>(dst + i) = *reinterpret_cast<const float4 *>(tab + i);
    } else {
      for (int32_t i = threadIdx.x; i < ng; i += kGatherThreads) dst[i] = tab[i];
    }
  } else {
    // The caller draws one group by inverse CDF over max(0, sum).  It does not need the sums
    // themselves for that, only where the running total crosses its threshold: the workgroup
    // leaves the totals of runs of kRunGroups consecutive groups (fp64, fixed order) and the
    // chunk's total; the few sums of the run that holds the crossing are formed again by the
    // caller.  Four neighbouring lanes cover one run, four groups each.
    const float4 *tab4 = reinterpret_cast<const float4 *>(tab);
    double *rp = runs + ((int64_t) r * nchunks + chunk) * (chunk_groups / kRunGroups);
    double part = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxChunkGroups / (4 * kGatherThreads); ++j) {
      const int32_t i4 = threadIdx.x + j * kGatherThreads;
      const int32_t g = 4 * i4;
      double s = 0.0;
      if (g < ng) {
        const float4 v = tab4[i4];
        s = ((double) fmaxf(v.x, 0.f) + (g + 1 < ng ? (double) fmaxf(v.y, 0.f) : 0.0)) +
            ((g + 2 < ng ? (double) fmaxf(v.z, 0.f) : 0.0) + (g + 3 < ng ? (double) fmaxf(v.w, 0.f) : 0.0));
      }
      s = subwave_sum<4>(s);
      if ((lane & 3) == 0 && g < ng) {
        rp[i4 >> 2] = s;
        part += s;
      }
    }
    part = subwave_sum<64>(part);
    if (lane == kWave - 1) wsum[wave] = part;
    __syncthreads();
    if (threadIdx.x == 0) {
      double t = 0.0;
      for (int w = 0; w < kGatherWaves; ++w) t += wsum[w];
      csum[(int64_t) r * nchunks + chunk] = t;
    }
  }
}

// =============================================================================================
// Launchers.
// =============================================================================================

static inline bool rows_vector_aligned(const RowSet &rs, bool bf16) {
  const int64_t per16 = bf16 ? 8 : 4;   // elements in 16 bytes
  auto ok = [&](const void *p, int64_t bs, int64_t ps) {
    return p == nullptr || (((uintptr_t) p & 15) == 0 && bs % per16 == 0 && ps % per16 == 0);
  };
  return ok(rs.base0, rs.bs0, rs.ps0) && ok(rs.base1, rs.bs1, rs.ps1);
}

int32_t stats_nparts(int32_t V) { return (V + kPartElems - 1) / kPartElems; }

hipError_t launch_row_stats(const RowSet &rs, bool bf16, int32_t V, int64_t nrows, float c,
                            bool streaming, StatPart *parts, hipStream_t stream,
                            const ProbeArgs *probes) {
  const int32_t nparts = stats_nparts(V);
  if (nrows == 0) return hipSuccess;
  ProbeArgs pa{};
  if (probes) pa = *probes;
  // With probes, the grid starts with a few rows of workgroups that form them, one target row per
  // wave; the rows of logits follow (the first grid plane holds fewer of them by that much).
  const unsigned gx = (unsigned) ((nparts + kStatsWaves - 1) / kStatsWaves);
  const int64_t probe_y =
      probes ? (rs.nrows0 + (int64_t) gx * kStatsWaves - 1) / ((int64_t) gx * kStatsWaves) : 0;
  const int64_t slots = nrows + probe_y;                    // values of (z, y) the grid must hold
  const unsigned gz = (unsigned) ((slots + kRowsPerGridY - 1) / kRowsPerGridY);
  const dim3 grid(gx, (unsigned) std::min<int64_t>(slots, kRowsPerGridY), gz), block(kStatsWaves * kWave);
  const bool vec = rows_vector_aligned(rs, bf16);
  auto launch = [&](auto kernel) {
    kernel<<<grid, block, 0, stream>>>(rs, V, nparts, nrows, c, parts, pa, probe_y);
  };
  if (bf16) {
    if (!vec) launch(row_stats_kernel<true, false, false>);
    else if (streaming) launch(row_stats_kernel<true, true, true>);
    else launch(row_stats_kernel<true, true, false>);
  } else {
    if (!vec) launch(row_stats_kernel<false, false, false>);
    else if (streaming) launch(row_stats_kernel<false, true, true>);
    else launch(row_stats_kernel<false, true, false>);
  }
  return hipGetLastError();
}

static inline bool table_vector_ok(const RowSet &rs, bool bf16, int32_t V, const int32_t *mult,
                                   const float *table) {
  return rows_vector_aligned(rs, bf16) && V % 8 == 0 && ((uintptr_t) mult & 15) == 0 &&
         ((uintptr_t) table & 15) == 0;
}

// Workgroups per sequence in the accept + delta kernel: enough to give every compute unit one,
// never more than there are slices of the table.
int32_t accept_nsplit(int32_t V, int32_t B) {
  const int32_t slices = (V + kAcceptTokens - 1) / kAcceptTokens;
  return std::max(1, std::min(slices, (256 + B - 1) / B));
}

hipError_t launch_accept_delta(const AcceptArgs &a, bool bf16, int32_t B, float c_lo, float *table,
                               hipStream_t stream) {
  const int32_t nsplit = accept_nsplit(a.V, B);
  const dim3 grid((unsigned) ((int64_t) B * nsplit));
  const bool vec = table_vector_ok(a.rs, bf16, a.V, a.mult, table);
#define PCG_LAUNCH_AD(BF, VE) \
  accept_delta_kernel<BF, VE><<<grid, kAcceptThreads, 0, stream>>>(a, nsplit, c_lo, table)
  if (bf16) { if (vec) PCG_LAUNCH_AD(true, true); else PCG_LAUNCH_AD(true, false); }
  else { if (vec) PCG_LAUNCH_AD(false, true); else PCG_LAUNCH_AD(false, false); }
#undef PCG_LAUNCH_AD
  return hipGetLastError();
}

hipError_t launch_accept_thin(const AcceptArgs &a, bool bf16, int32_t B, const int32_t *tok_ptr,
                              const int32_t *tok_groups, const float *tok_weights, int32_t *trials,
                              int32_t max_trials, hipStream_t stream) {
  const bool vec = rows_vector_aligned(a.rs, bf16) && a.V % 8 == 0;
#define PCG_LAUNCH_AT(BF, VE)                                                                \
  accept_thin_kernel<BF, VE><<<B, kAcceptThreads, 0, stream>>>(a, tok_ptr, tok_groups,        \
                                                               tok_weights, trials, max_trials)
  if (bf16) { if (vec) PCG_LAUNCH_AT(true, true); else PCG_LAUNCH_AT(true, false); }
  else { if (vec) PCG_LAUNCH_AT(false, true); else PCG_LAUNCH_AT(false, false); }
#undef PCG_LAUNCH_AT
  return hipGetLastError();
}

int32_t thin_max_parts() { return kMaxThinParts; }

hipError_t launch_propose(const RowSet &rs, bool bf16, int32_t V, int32_t K, int32_t pos0, float c,
                          const StatPart *parts, const int32_t *tok_ptr, const int32_t *tok_groups,
                          const float *tok_weights, uint64_t seed, uint64_t offset,
                          int32_t *prop_tokens, int32_t *prop_groups, pcg_diag *diag,
                          hipStream_t stream) {
  const bool vec = rows_vector_aligned(rs, bf16) && V % 8 == 0;
  const int32_t nparts = stats_nparts(V);
  const unsigned grid = (unsigned) rs.nrows0;
#define PCG_LAUNCH_PR(BF, VE)                                                                     \
  propose_kernel<BF, VE><<<grid, kWave, 0, stream>>>(rs, V, K, pos0, nparts, c, parts, tok_ptr,   \
                                                     tok_groups, tok_weights, seed, offset,       \
                                                     prop_tokens, prop_groups, diag)
  if (bf16) { if (vec) PCG_LAUNCH_PR(true, true); else PCG_LAUNCH_PR(true, false); }
  else { if (vec) PCG_LAUNCH_PR(false, true); else PCG_LAUNCH_PR(false, false); }
#undef PCG_LAUNCH_PR
  return hipGetLastError();
}

hipError_t launch_weights(const RowSet &rs, bool bf16, const pcg_groups &g, int64_t row0,
                          int32_t nrows, float c, float c_hi, float c_lo, const StatPart *parts,
                          float *table, hipStream_t stream) {
  const int32_t nct = (g.V + kTableTokens - 1) / kTableTokens;
  const dim3 grid((unsigned) ((int64_t) nct * nrows));
  const int32_t nparts = stats_nparts(g.V);
  const bool vec = table_vector_ok(rs, bf16, g.V, g.mult, table);
  // with general weights the table is the plain probability: the gather applies the weights
  const int32_t *mult = g.weights ? nullptr : g.mult;
#define PCG_LAUNCH_WEIGHTS(BF, VE)                                                             \
  weights_kernel<BF, VE><<<grid, kTableThreads, 0, stream>>>(rs, g.V, nparts, nct, row0, c, c_hi, \
                                                             c_lo, parts, mult, table)
  if (bf16) { if (vec) PCG_LAUNCH_WEIGHTS(true, true); else PCG_LAUNCH_WEIGHTS(true, false); }
  else { if (vec) PCG_LAUNCH_WEIGHTS(false, true); else PCG_LAUNCH_WEIGHTS(false, false); }
#undef PCG_LAUNCH_WEIGHTS
  return hipGetLastError();
}

template <int W>
static void gather_dispatch(bool clamp, dim3 grid, hipStream_t stream, int32_t V, int32_t G,
                            int32_t nrows, int32_t nchunks, int32_t gpc, int32_t ntiles,
                            int32_t tile_len, const int32_t *row_ptr, const int32_t *members,
                            const float *weights, const float *table, float *out) {
  if (clamp)
    gather_kernel<W, true><<<grid, kGatherThreads, 0, stream>>>(
        V, G, nrows, nchunks, gpc, ntiles, tile_len, row_ptr, members, weights, table, out);
  else
    gather_kernel<W, false><<<grid, kGatherThreads, 0, stream>>>(
        V, G, nrows, nchunks, gpc, ntiles, tile_len, row_ptr, members, weights, table, out);
}

hipError_t launch_gather(const pcg_groups &g, int32_t nrows, bool clamp, const float *table,
                         float *out, hipStream_t stream) {
  if (nrows == 0) return hipSuccess;
  // lanes per group: the smallest power of two >= the mean group size, within [4, 64]
  const double mean = (double) g.nnz / (double) g.G;
  int W = 4;
  while (W < 64 && W < mean) W *= 2;
  const int nsub = kGatherThreads / W;
  // enough chunks per row to give every CU a workgroup, but no chunk below one pass
  int32_t nchunks = (256 + nrows - 1) / nrows;
  const int32_t max_chunks = (g.G + nsub - 1) / nsub;
  if (nchunks > max_chunks) nchunks = max_chunks;
  if (nchunks < 1) nchunks = 1;
  int32_t gpc = (g.G + nchunks - 1) / nchunks;
  gpc = (gpc + nsub - 1) / nsub * nsub;
  nchunks = (g.G + gpc - 1) / gpc;
  const int32_t ntiles = (g.V + kTileMax - 1) / kTileMax;
  int32_t tile_len = (g.V + ntiles - 1) / ntiles;
  tile_len = (tile_len + 63) / 64 * 64;
  if (tile_len > kTileMax) tile_len = kTileMax;
  const int32_t rows8 = (nrows + 7) / 8;
  const dim3 grid((unsigned) (8 * rows8 * nchunks));
  switch (W) {
    case 4: gather_dispatch<4>(clamp, grid, stream, g.V, g.G, nrows, nchunks, gpc, ntiles, tile_len, g.row_ptr, g.members, g.weights, table, out); break;
    case 8: gather_dispatch<8>(clamp, grid, stream, g.V, g.G, nrows, nchunks, gpc, ntiles, tile_len, g.row_ptr, g.members, g.weights, table, out); break;
    case 16: gather_dispatch<16>(clamp, grid, stream, g.V, g.G, nrows, nchunks, gpc, ntiles, tile_len, g.row_ptr, g.members, g.weights, table, out); break;
    case 32: gather_dispatch<32>(clamp, grid, stream, g.V, g.G, nrows, nchunks, gpc, ntiles, tile_len, g.row_ptr, g.members, g.weights, table, out); break;
    default: gather_dispatch<64>(clamp, grid, stream, g.V, g.G, nrows, nchunks, gpc, ntiles, tile_len, g.row_ptr, g.members, g.weights, table, out); break;
  }
  return hipGetLastError();
}

hipError_t launch_gather_prepared(const pcg_groups &g, int32_t nrows, const float *table, float *out,
                                  double *csum, double *runs, hipStream_t stream) {
  if (nrows == 0) return hipSuccess;
  const pcg_prepared &p = *g.prepared_info;
  const char *blob = reinterpret_cast<const char *>(g.prepared);
  const uint32_t *desc = reinterpret_cast<const uint32_t *>(blob + p.off_desc);
  const uint16_t *perm = reinterpret_cast<const uint16_t *>(blob + p.off_perm);
  const uint4 *data = reinterpret_cast<const uint4 *>(blob + p.off_data);
  const int32_t rows8 = (nrows + 7) / 8;
  const dim3 grid((unsigned) (8 * rows8 * p.nchunks));
  // general weights are read from the blob (the caller's checks made sure it holds them)
  const float4 *wdata =
      g.weights ? reinterpret_cast<const float4 *>(blob + p.off_weights) : nullptr;
  auto launch = [&](auto kernel) {
    kernel<<<grid, kGatherThreads, 0, stream>>>(g.V, g.G, nrows, p.nchunks, p.chunk_groups,
                                                p.ntiles, p.tile_len, p.blocks_per_chunk, desc,
                                                perm, data, wdata, table, out, csum, runs);
  };
  if (wdata) {
    if (csum) launch(gather_prepared_kernel<true, true>);
    else launch(gather_prepared_kernel<false, true>);
  } else {
    if (csum) launch(gather_prepared_kernel<true, false>);
    else launch(gather_prepared_kernel<false, false>);
  }
  return hipGetLastError();
}

hipError_t launch_finalize(const FinalizeArgs &fa, bool bf16, const pcg_groups &g, int32_t B,
                           const double *csum, const double *runs, int32_t nchunks,
                           int32_t chunk_groups, hipStream_t stream) {
  if (bf16)
    finalize_kernel<true><<<B, kFinalThreads, 0, stream>>>(fa, g.V, g.G, csum, runs, nchunks, chunk_groups);
  else
    finalize_kernel<false><<<B, kFinalThreads, 0, stream>>>(fa, g.V, g.G, csum, runs, nchunks, chunk_groups);
  return hipGetLastError();
}

}  // namespace pcg
