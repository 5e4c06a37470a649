// Construction of the Acoustic Similarity Groups (Sec. 2.1, Eq. 1) on gfx950: unit vectors in
// bfloat16, the V x V cosine similarity as a bf16 MFMA contraction with fp32 accumulation that
// is thresholded on the fly (the similarity matrix is never stored), per-token member lists
// sorted ascending, identical sets dropped, and the CSR the verification kernels read.  The
// exact form (pcg_asg_build_exact) uses the same contraction as a filter: pairs whose rounded
// similarity is too close to the threshold to decide are settled by the cosine of the
// embeddings themselves in double, so its groups are those of Eq. (1) as written.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>

#include "pcg_device.h"
#include "pcg_kernels.h"

namespace pcg {

namespace {

constexpr size_t kAsgAlign = 256;
size_t asg_align(size_t n) { return (n + kAsgAlign - 1) / kAsgAlign * kAsgAlign; }

// ---------------------------------------------------------------------------------------------
// Unit vectors: emb[v] / ||emb[v]|| in double, rounded once to bfloat16 (nearest, ties to even).
// ---------------------------------------------------------------------------------------------

__device__ __forceinline__ uint16_t round_to_bf16(double x) {
  // the two bfloat16 values that bracket x, found from the truncation of its fp32 image
  const double ax = fabs(x);
  uint32_t lo = __float_as_uint((float) ax) & 0xffff0000u;
  if ((double) __uint_as_float(lo) > ax) lo -= 0x10000u;       // the fp32 image rounded up past lo
  uint32_t hi = lo + 0x10000u;
  if ((double) __uint_as_float(hi) < ax) { lo = hi; hi += 0x10000u; }
  const double dlo = ax - (double) __uint_as_float(lo), dhi = (double) __uint_as_float(hi) - ax;
  const uint32_t pick = dlo < dhi ? lo : (dhi < dlo ? hi : (((lo >> 16) & 1u) ? hi : lo));
  // the sign travels as it is: a negative zero stays a negative zero, as in IEEE rounding
  return (uint16_t) ((pick >> 16) | (__double_as_longlong(x) < 0 ? 0x8000u : 0u));
}

// norms (may be NULL) receives ||emb[v]|| in double.
__global__ __launch_bounds__(256) void asg_normalize_kernel(const float *emb, int32_t V, int32_t d,
                                                            uint16_t *unit, double *norms) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t v = (int64_t) blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6);
  if (v >= V) return;                       // whole waves leave together
  const float *e = emb + v * d;
  double ss = 0.0;
  for (int32_t k = lane; k < d; k += kWave) ss += (double) e[k] * (double) e[k];
  const double norm = sqrt(wave_sum(ss));
  if (norms && lane == 0) norms[v] = norm;
  for (int32_t k = lane; k < d; k += kWave)
    unit[v * d + k] = norm > 0.0 ? round_to_bf16((double) e[k] / norm) : (uint16_t) 0;
}

// ---------------------------------------------------------------------------------------------
// Similarity + threshold.  A workgroup of four waves owns a 256 x 256 tile of the similarity
// matrix; each wave a 128 x 128 quarter as 4 x 4 MFMA blocks of 32 x 32 (256 accumulators per
// lane; with smaller wave tiles the operand reads alone saturate LDS).  Both operands are rows
// of the same matrix of unit vectors.  They travel global memory -> LDS directly, 32 columns of
// k per stage, four stages resident: while one is used the loads of the next three are in flight,
// and no register is spent on staging.  The matrix is symmetric: only tiles on or above the
// diagonal are computed, and a pair found off the diagonal is recorded for both of its tokens.
// ---------------------------------------------------------------------------------------------

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kSimTile = 256;                 // rows and columns of a workgroup's tile
constexpr int kSimK = 32;                     // k columns per LDS stage: rows of 64 bytes
constexpr int kSimBufs = 4;                   // stages resident in LDS
constexpr int kSimThreads = 256;
constexpr int kSimStageBytes = kSimTile * kSimK * 2;      // one operand of one stage: 16 KiB
constexpr int kSimLoads = 2 * kSimTile / 16 / 4;          // direct-to-LDS loads per wave and stage: 8
constexpr int kSimQueue = 8192;               // pairs a workgroup can hold back in LDS
constexpr int kSimPatchRows = 16, kSimPatchCols = 2;       // tiles that one XCD works on together

// Record v as a member of G(t).
__device__ __forceinline__ void asg_emit(int32_t t, int32_t v, int32_t cap, int32_t *count,
                                         int32_t *cand) {
  const int32_t pos = atomicAdd(&count[t], 1);
  if (pos < cap) cand[(int64_t) t * cap + pos] = v;
}

// A member that the rounded similarity could not decide carries this bit until the exact form
// has settled it (token ids stay below 2^31).
constexpr uint32_t kAsgUnsure = 0x80000000u;

// Appends the pair (t, v) to the workgroup's queue in LDS; pairs beyond its capacity are
// recorded at once.  flag: 0 or kAsgUnsure.
__device__ __forceinline__ void sim_queue_pair(int32_t t, int32_t v, uint32_t flag, int32_t cap,
                                               int32_t *count, int32_t *cand, uint32_t *qn, uint2 *q) {
  const uint32_t k = atomicAdd(qn, 1u);
  if (k < (uint32_t) kSimQueue) {
    q[k] = make_uint2((uint32_t) t, (uint32_t) v | flag);
  } else {
    asg_emit(t, (int32_t) ((uint32_t) v | flag), cap, count, cand);
    if (t != v) asg_emit(v, (int32_t) ((uint32_t) t | flag), cap, count, cand);
  }
}

// Waits until at most N of this wave's vector-memory operations are still in flight.
template <int N>
__device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Meets the other waves of the workgroup without the fence of __syncthreads(), which would wait
// for every load still in flight.  The caller has waited for exactly what it needs.
__device__ __forceinline__ void bare_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// EXACT: pairs above theta are candidates, and those not above theta_hi are marked kAsgUnsure
// for asg_refine_kernel (theta and theta_hi bracket the threshold of Eq. 1 by the rounding band).
template <bool EXACT>
__global__ __launch_bounds__(kSimThreads) void asg_similarity_kernel(
    const uint16_t *__restrict__ unit, int32_t V, int32_t d, float theta, float theta_hi,
    int32_t cap, int32_t *count, int32_t *cand) {
  // Workgroups go to the 8 XCDs round-robin; the 32 that run together on one XCD take a patch of
  // 16 x 2 tiles (measured: 5.0 ms against 5.2 for 8 x 4 and 5.7 for 4 x 8), so that they find each
  // other's rows in their L2.
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  constexpr int kPatch = kSimPatchRows * kSimPatchCols;
  const int patch = (local / kPatch) * 8 + xcd;
  const int within = local % kPatch;
  const int ntl = (V + kSimTile - 1) / kSimTile;
  const int super_cols = (ntl + kSimPatchCols - 1) / kSimPatchCols;
  const int ti = (patch / super_cols) * kSimPatchRows + within / kSimPatchCols;
  const int tj = (patch % super_cols) * kSimPatchCols + within % kSimPatchCols;
  if (ti >= ntl || tj >= ntl || tj < ti) return;      // the whole workgroup leaves
  // [buffer][operand][row][64 bytes].  A 16-byte LDS read is served 16 lanes at a time, free of
  // conflicts when their addresses differ modulo 256 bytes; the four 16-byte chunks of a row are
  // therefore stored at position chunk ^ ((row >> 2) & 3), which spreads the same chunk of 16
  // consecutive rows over all 16 slots.
  __shared__ __attribute__((aligned(1024))) unsigned char lds[kSimBufs * 2 * kSimStageBytes];
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int32_t row0 = ti * kSimTile, col0 = tj * kSimTile;

  // Direct-to-LDS loads: one instruction of a wave fills 1 KiB = 16 rows, lane i the 16 bytes at
  // row i / 4, position i % 4.  Wave w brings rows 64 w .. 64 w + 63 of both operands.
  int32_t src[kSimLoads];
  {
    const int r = lane >> 2, p = lane & 3;
    const int c = p ^ ((r >> 2) & 3);                  // the chunk of the row that belongs there
#pragma unroll
    for (int j = 0; j < kSimLoads / 2; ++j) {
      const int row = wave * 64 + j * 16 + r;
      // rows past the end of the matrix re-read the last row; their results are never recorded
      src[j] = min(row0 + row, V - 1) * d + c * 8;
      src[kSimLoads / 2 + j] = min(col0 + row, V - 1) * d + c * 8;
    }
  }
  const int nstages = d / kSimK;        // even: d is a multiple of 64
  auto load_a = [&](int j, unsigned char *dst, int k0) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void *) (unit + src[j] + k0),
        (__attribute__((address_space(3))) void *) (dst + j * 1024), 16, 0, 0);
  };
  auto load_b = [&](int j, unsigned char *dst, int k0) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void *) (unit + src[kSimLoads / 2 + j] + k0),
        (__attribute__((address_space(3))) void *) (dst + kSimStageBytes + j * 1024), 16, 0, 0);
  };

  floatx16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // operand reads of this lane: row lane % 32 of a block, k half lane / 32 of a 16-column step
  const int fr = lane & 31, fh = lane >> 5;
  const int sw = (fr >> 2) & 3;                        // block rows start at multiples of 32
  const int a_row = (wm * 128 + fr) * 64, b_row = (wn * 128 + fr) * 64;
  const int pos0 = ((0 + fh) ^ sw) * 16, pos1 = ((2 + fh) ^ sw) * 16;

  bf16x8 f0a[4], f0b[4], f1a[4], f1b[4];      // operands of the two 16-column steps of a stage
  // One 16-column step: 16 MFMAs on (ca, cb).  Behind the first eight of them, one at a time,
  // the next step's operands (na, nb) are read from LDS at ta / tb and, with FETCH, the eight
  // loads of a later stage are started.  The LDS and memory queues are short: instructions
  // issued in a burst would hold the MFMAs behind them back, and reads issued late would make
  // the next step wait.  The order is pinned.
  auto step = [&](const bf16x8 (&ca)[4], const bf16x8 (&cb)[4], bf16x8 (&na)[4], bf16x8 (&nb)[4],
                  const unsigned char *ta, const unsigned char *tb, bool with_fetch,
                  unsigned char *dst, int k0) {
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const int i = m >> 2, j = m & 3;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[i], cb[j], acc[i][j], 0, 0, 0);
      if (m < 8) {
        __builtin_amdgcn_sched_barrier(0);
        if (with_fetch) {
          if ((m & 1) == 0) load_a(m >> 1, dst, k0); else load_b(m >> 1, dst, k0);
        }
        if (m < 4) na[m] = *reinterpret_cast<const bf16x8 *>(ta + m * 32 * 64);
        else nb[m - 4] = *reinterpret_cast<const bf16x8 *>(tb + (m - 4) * 32 * 64);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // Loads that would reach past the last stage repeat it instead: nobody reads what they bring,
  // and the number of loads in flight stays the same on every turn, which the waits rely on.
#pragma unroll
  for (int s = 0; s < kSimBufs; ++s) {
    unsigned char *dst = lds + s * 2 * kSimStageBytes + wave * 64 * 64;
    const int k0 = min(s, nstages - 1) * kSimK;
#pragma unroll
    for (int j = 0; j < kSimLoads / 2; ++j) { load_a(j, dst, k0); load_b(j, dst, k0); }
  }
  wait_vm<(kSimBufs - 1) * kSimLoads>();    // stage 0 is in; the ones behind it may be on their way
  bare_barrier();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f0a[i] = *reinterpret_cast<const bf16x8 *>(lds + a_row + pos0 + i * 32 * 64);
    f0b[i] = *reinterpret_cast<const bf16x8 *>(lds + kSimStageBytes + b_row + pos0 + i * 32 * 64);
  }
  for (int s = 0; s < nstages; ++s) {
    unsigned char *cur = lds + (s % kSimBufs) * 2 * kSimStageBytes;
    const unsigned char *nxt = lds + ((s + 1) % kSimBufs) * 2 * kSimStageBytes;
    // first half of the stage; the operands of its second half arrive behind it
    step(f0a, f0b, f1a, f1b, cur + a_row + pos1, cur + kSimStageBytes + b_row + pos1, false, nullptr, 0);
    // This wave's loads of stage s + 1 have landed once only those of the two stages behind it
    // are out; past the barrier everyone's have, and nobody reads buffer `cur` any more (the
    // operands of this stage's second half are in registers).
    wait_vm<(kSimBufs - 2) * kSimLoads>();
    bare_barrier();
    // second half; behind it the loads of stage s + 4 start, into the buffer just freed, and the
    // next stage's first operands are read
    step(f1a, f1b, f0a, f0b, nxt + a_row + pos0, nxt + kSimStageBytes + b_row + pos0, true,
         cur + wave * 64 * 64, min(s + kSimBufs, nstages - 1) * kSimK);
  }

  // Threshold (Eq. 1).  The stage buffers are free once the loads past the end have landed: pairs
  // that pass are collected there, then every thread records its share of them, so that the
  // round trips of the atomics overlap instead of following one another.
  wait_vm<0>();
  __syncthreads();
  uint32_t *qn = reinterpret_cast<uint32_t *>(lds);
  uint2 *q = reinterpret_cast<uint2 *>(lds + 16);
  if (tid == 0) *qn = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // Accumulator r of a lane is row 8 (r / 4) + 4 (lane / 32) + r % 4 and column lane % 32 of
      // the 32 x 32 block.  Most blocks hold nothing above the threshold: one maximum per lane
      // and a ballot settle those.
      const int32_t t0 = row0 + wm * 128 + i * 32, v0 = col0 + wn * 128 + j * 32;
      if (v0 + 31 < t0) continue;                      // wholly below the diagonal
      const floatx16 a = acc[i][j];
      const float m = fmaxf(fmaxf(fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3])),
                                  fmaxf(fmaxf(a[4], a[5]), fmaxf(a[6], a[7]))),
                            fmaxf(fmaxf(fmaxf(a[8], a[9]), fmaxf(a[10], a[11])),
                                  fmaxf(fmaxf(a[12], a[13]), fmaxf(a[14], a[15]))));
      const int32_t v = v0 + (lane & 31), tl = t0 + 4 * (lane >> 5);
      if (__builtin_amdgcn_ballot_w64(m > theta) != 0) {
        uint32_t hits = 0, sure = 0xffffu;
#pragma unroll
        for (int r = 0; r < 16; ++r) hits |= (a[r] > theta ? 1u : 0u) << r;
        if constexpr (EXACT) {
          sure = 0;
#pragma unroll
          for (int r = 0; r < 16; ++r) sure |= (a[r] > theta_hi ? 1u : 0u) << r;
        }
        while (hits) {                                 // only the lanes that hold a pair
          const int r = __builtin_ctz(hits);
          hits &= hits - 1;
          const int32_t t = tl + 8 * (r >> 2) + (r & 3);
          if (t < V && v < V && v > t)
            sim_queue_pair(t, v, ((sure >> r) & 1u) ? 0u : kAsgUnsure, cap, count, cand, qn, q);
        }
      }
      // a token is always a member of its own group, whatever the rounded product says
      if (t0 == v0 && lane < 32 && t0 + lane < V)
        sim_queue_pair(t0 + lane, t0 + lane, 0u, cap, count, cand, qn, q);
    }
  __syncthreads();
  const uint32_t nq = min(*qn, (uint32_t) kSimQueue);
  for (uint32_t k = tid; k < nq; k += kSimThreads) {
    const uint2 pr = q[k];
    const uint32_t flag = pr.y & kAsgUnsure;
    const int32_t t = (int32_t) pr.x, v = (int32_t) (pr.y & ~kAsgUnsure);
    const int32_t p0 = atomicAdd(&count[t], 1);
    const int32_t p1 = t != v ? atomicAdd(&count[v], 1) : cap;
    if (p0 < cap) cand[(int64_t) t * cap + p0] = (int32_t) ((uint32_t) v | flag);
    if (p1 < cap) cand[(int64_t) v * cap + p1] = (int32_t) ((uint32_t) t | flag);
  }
}

// ---------------------------------------------------------------------------------------------
// Exact form: one wave per token settles the members marked kAsgUnsure by Eq. (1) itself -- the
// dot product of the two float32 embeddings and their norms, all in double, strict > theta --
// and closes the gaps in the token's list.  The dot product is summed in the same order for
// (t, v) and (v, t), so both tokens reach the same decision.  A list that did not fit into cap
// stays undecided: its count stays above cap and the call reports PCG_ERR_CAPACITY.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void asg_refine_kernel(const float *__restrict__ emb,
                                                         const double *__restrict__ norms, int32_t V,
                                                         int32_t d, double theta, int32_t cap,
                                                         int32_t *count, int32_t *cand) {
  const int lane = threadIdx.x & (kWave - 1);
  const int32_t t = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6);
  if (t >= V) return;                       // whole waves leave together
  const int32_t found = count[t];
  int32_t *row = cand + (int64_t) t * cap;
  if (found > cap) {
    // undecided, but plain token ids again: the kernels that follow index with them
    for (int32_t k = lane; k < cap; k += kWave) row[k] = (int32_t) ((uint32_t) row[k] & ~kAsgUnsure);
    return;
  }
  const float *et = emb + (int64_t) t * d;
  const double nt = norms[t];
  int32_t kept_total = 0;
  for (int32_t c0 = 0; c0 < found; c0 += kWave) {
    const int32_t k = c0 + lane;
    bool keep = k < found;
    const uint32_t raw = keep ? (uint32_t) row[k] : 0u;
    const int32_t entry = (int32_t) (raw & ~kAsgUnsure);
    unsigned long long unsure = __ballot(keep && (raw & kAsgUnsure) != 0);
    while (unsure) {                                   // uniform over the wave
      const int l = __ffsll((long long) unsure) - 1;
      unsure &= unsure - 1;
      const int32_t v = __builtin_amdgcn_readlane(entry, l);
      const float *ev = emb + (int64_t) v * d;
      double dot = 0.0;
      for (int32_t j = 4 * lane; j < d; j += 4 * kWave) {       // d is a multiple of 64
        const float4 a = *reinterpret_cast<const float4 *>(et + j);
        const float4 b = *reinterpret_cast<const float4 *>(ev + j);
        dot += ((double) a.x * (double) b.x + (double) a.y * (double) b.y) +
               ((double) a.z * (double) b.z + (double) a.w * (double) b.w);
      }
      dot = wave_sum(dot);
      const double nv = norms[v];
      const double cosine = (nt > 0.0 && nv > 0.0) ? dot / (nt * nv) : 0.0;
      if (lane == l && !(cosine > theta)) keep = false;
    }
    const unsigned long long kept = __ballot(keep);
    const int32_t pos = kept_total + __popcll(kept & ((1ull << lane) - 1ull));
    // positions written here lie below c0 + 64, positions read later at or above it
    if (keep) row[pos] = entry;
    kept_total += __popcll(kept);
  }
  if (lane == 0) count[t] = kept_total;
}

// ---------------------------------------------------------------------------------------------
// Per token: members ascending (bitonic sort in LDS), a hash of the set, its size.
// ---------------------------------------------------------------------------------------------

constexpr int kSortThreads = 256;             // four waves, one token each
constexpr int kAsgMaxCap = PCG_ASG_MAX_CAP;

__device__ __forceinline__ uint64_t mix64(uint64_t x) {   // splitmix64 finaliser
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

// Makes a wave's LDS writes visible to its own later reads (no other wave shares the data).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// One wave per token: its members ascending (bitonic sort in the wave's own slice of LDS), an
// order-independent hash of the set, its size.  cap2 = cap rounded up to a power of two; the
// kernel is launched with 4 * cap2 * 4 bytes of dynamic LDS.
__global__ __launch_bounds__(kSortThreads) void asg_sort_kernel(int32_t V, int32_t cap, int32_t cap2,
                                                                const int32_t *count, int32_t *cand,
                                                                int32_t *size, uint64_t *hash,
                                                                int32_t *max_count) {
  extern __shared__ int32_t sort_lds[];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  const int32_t t = blockIdx.x * (kSortThreads / kWave) + wave;
  if (t >= V) return;                       // whole waves leave together; no workgroup barrier below
  int32_t *key = sort_lds + wave * cap2;
  const int32_t found = count[t];
  const int32_t n = min(found, cap);
  // the largest set found so far: read first, since 65 536 atomics on one word take longer
  // than the sort itself
  if (lane == 0 && found > __atomic_load_n(max_count, __ATOMIC_RELAXED)) atomicMax(max_count, found);
  int32_t n2 = 1;
  while (n2 < n) n2 <<= 1;
  int32_t *row = cand + (int64_t) t * cap;
  for (int32_t k = lane; k < n2; k += kWave) key[k] = k < n ? row[k] : INT32_MAX;
  wave_lds_sync();
  for (int32_t len = 2; len <= n2; len <<= 1)
    for (int32_t step = len >> 1; step > 0; step >>= 1) {
      for (int32_t k = lane; k < n2; k += kWave) {
        const int32_t other = k ^ step;
        if (other > k) {
          const bool up = (k & len) == 0;
          const int32_t x = key[k], y = key[other];
          if ((x > y) == up) { key[k] = y; key[other] = x; }
        }
      }
      wave_lds_sync();
    }
  uint64_t h = 0;
  for (int32_t k = lane; k < n; k += kWave) {
    row[k] = key[k];
    h += mix64((uint64_t) key[k]);
  }
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) h += __shfl_xor(h, o, kWave);
  if (lane == 0) {
    hash[t] = h;
    size[t] = n;
  }
}

// keep[t] = 0 iff an earlier token has exactly the same set.  Such a token is a member of G(t)
// (every set holds its own token), so only the members below t are looked at.
__global__ __launch_bounds__(256) void asg_dedup_kernel(int32_t V, int32_t cap, const int32_t *cand,
                                                        const int32_t *size, const uint64_t *hash,
                                                        int32_t *keep) {
  const int lane = threadIdx.x & (kWave - 1);
  const int32_t t = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6);
  if (t >= V) return;
  const int32_t n = size[t];
  const uint64_t h = hash[t];
  const int32_t *mine = cand + (int64_t) t * cap;
  int dup = 0;
  for (int32_t j = 0; j < n && !dup; ++j) {
    const int32_t m = mine[j];                 // uniform over the wave
    if (m >= t) break;
    if (size[m] != n || hash[m] != h) continue;
    const int32_t *theirs = cand + (int64_t) m * cap;
    bool same = true;
    for (int32_t k = lane; k < n; k += kWave) same = same && mine[k] == theirs[k];
    dup = __all(same);
  }
  if (lane == 0) keep[t] = !dup;
}

// Exclusive scans over the tokens by one workgroup, 1024 tokens at a time: gid[t] = kept tokens
// before t, off[t] = members of kept tokens before t; totals[0] = G, totals[1] = nnz.  The
// counts stay below 2^31, so they are exact in the double the wave scan works on.
constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void asg_scan_kernel(int32_t V, const int32_t *keep,
                                                                const int32_t *size, int32_t *gid,
                                                                int64_t *off, int64_t *totals) {
  __shared__ double wg[kScanThreads / kWave], wn[kScanThreads / kWave];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  double base_g = 0.0, base_n = 0.0;
  for (int32_t t0 = 0; t0 < V; t0 += kScanThreads) {
    const int32_t t = t0 + threadIdx.x;
    const bool k = t < V && keep[t] != 0;
    const double g = k ? 1.0 : 0.0, n = k ? (double) size[t] : 0.0;
    const double ig = wave_scan(g), in = wave_scan(n);
    if (lane == kWave - 1) { wg[wave] = ig; wn[wave] = in; }
    __syncthreads();
    double bg = base_g, bn = base_n, tg = 0.0, tn = 0.0;
    for (int w = 0; w < kScanThreads / kWave; ++w) {
      if (w == wave) { bg += tg; bn += tn; }
      tg += wg[w]; tn += wn[w];
    }
    if (t < V) {
      gid[t] = (int32_t) (bg + ig - g);
      off[t] = (int64_t) (bn + in - n);
    }
    base_g += tg;
    base_n += tn;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    totals[0] = (int64_t) base_g;
    totals[1] = (int64_t) base_n;
  }
}

__global__ __launch_bounds__(256) void asg_fill_kernel(int32_t *p, int64_t n, int32_t value) {
  const int64_t i = (int64_t) blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}

__global__ __launch_bounds__(256) void asg_compact_kernel(int32_t V, int32_t cap, const int32_t *cand,
                                                          const int32_t *size, const int32_t *keep,
                                                          const int32_t *gid, const int64_t *off,
                                                          const int64_t *totals, int32_t *row_ptr,
                                                          int32_t *members, int32_t *mult,
                                                          int32_t *seed_of) {
  const int lane = threadIdx.x & (kWave - 1);
  const int32_t t = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6);
  if (t >= V) return;
  if (t == 0 && lane == 0) row_ptr[totals[0]] = (int32_t) totals[1];
  if (!keep[t]) return;
  const int32_t n = size[t], g = gid[t];
  const int64_t o = off[t];
  const int32_t *mine = cand + (int64_t) t * cap;
  for (int32_t k = lane; k < n; k += kWave) {
    const int32_t m = mine[k];
    members[o + k] = m;
    atomicAdd(&mult[m], 1);
  }
  if (lane == 0) {
    row_ptr[g] = (int32_t) o;
    if (seed_of) seed_of[g] = t;
  }
}

}  // namespace

}  // namespace pcg

using namespace pcg;

namespace {

size_t asg_core_workspace_bytes(size_t v, int32_t cap) {
  return asg_align(v * 4) /* count */ + asg_align(v * (size_t) cap * 4) /* cand */ +
         asg_align(v * 4) /* size */ + asg_align(v * 8) /* hash */ + asg_align(v * 4) /* keep */ +
         asg_align(v * 4) /* gid */ + asg_align(v * 8) /* off */ + asg_align(64) /* totals */;
}

// How far the fp32-accumulated dot product of two bf16-rounded unit vectors can lie from the
// cosine of the vectors they were rounded from: every component is off by at most 2^-9 of
// itself, so the products by at most 2^-8 + 2^-18 of themselves, and their absolute values sum
// to at most 1 (Cauchy-Schwarz); the d additions in fp32 add at most d * 2^-23 (a rounding, or a
// truncation, of each partial sum of magnitude at most 1).
float asg_rounding_band(int32_t d) {
  return 0x1p-8f + 0x1p-18f + (float) d * 0x1p-23f;
}

// The groups from the unit vectors; with emb (and norms, workspace of the caller) the exact form.
int asg_build_impl(const float *emb, const double *norms, const uint16_t *unit_bf16, int32_t V,
                   int32_t d, float theta, int32_t cap, int32_t *row_ptr, int32_t *members,
                   int64_t members_capacity, int32_t *mult, int32_t *seed_of, int32_t *out_G,
                   int64_t *out_nnz, int32_t *out_max_size, char *ws, hipStream_t stream) {
  const size_t v = (size_t) V;
  int32_t *count = (int32_t *) ws; ws += asg_align(v * 4);
  int32_t *cand = (int32_t *) ws; ws += asg_align(v * (size_t) cap * 4);
  int32_t *size = (int32_t *) ws; ws += asg_align(v * 4);
  uint64_t *hash = (uint64_t *) ws; ws += asg_align(v * 8);
  int32_t *keep = (int32_t *) ws; ws += asg_align(v * 4);
  int32_t *gid = (int32_t *) ws; ws += asg_align(v * 4);
  int64_t *off = (int64_t *) ws; ws += asg_align(v * 8);
  int64_t *totals = (int64_t *) ws;          // [0] G, [1] nnz, [2] (as int32) largest set found

  auto fail = [](hipError_t e) { return record_hip_error(e); };
  hipError_t e;
  const unsigned vb = (unsigned) ((v + 255) / 256), wb = (unsigned) ((v + 3) / 4);
  asg_fill_kernel<<<vb, 256, 0, stream>>>(count, V, 0);
  asg_fill_kernel<<<vb, 256, 0, stream>>>(mult, V, 0);
  asg_fill_kernel<<<1, 256, 0, stream>>>((int32_t *) totals, 16, 0);
  const int tiles = (V + kSimTile - 1) / kSimTile;
  const int patch_rows = (tiles + kSimPatchRows - 1) / kSimPatchRows;
  const int patch_cols = (tiles + kSimPatchCols - 1) / kSimPatchCols;
  const int patches = (patch_rows * patch_cols + 7) / 8 * 8;      // dealt to the 8 XCDs in turn
  const unsigned sim_grid = (unsigned) (patches * kSimPatchRows * kSimPatchCols);
  if (emb) {
    const float band = asg_rounding_band(d);
    asg_similarity_kernel<true><<<sim_grid, kSimThreads, 0, stream>>>(
        unit_bf16, V, d, theta - band, theta + band, cap, count, cand);
    asg_refine_kernel<<<wb, 256, 0, stream>>>(emb, norms, V, d, (double) theta, cap, count, cand);
  } else {
    asg_similarity_kernel<false><<<sim_grid, kSimThreads, 0, stream>>>(
        unit_bf16, V, d, theta, theta, cap, count, cand);
  }
  if ((e = hipGetLastError()) != hipSuccess) return fail(e);
  int32_t cap2 = 1;
  while (cap2 < cap) cap2 <<= 1;
  asg_sort_kernel<<<wb, kSortThreads, (size_t) (kSortThreads / kWave) * cap2 * sizeof(int32_t), stream>>>(
      V, cap, cap2, count, cand, size, hash, (int32_t *) (totals + 2));
  asg_dedup_kernel<<<wb, 256, 0, stream>>>(V, cap, cand, size, hash, keep);
  asg_scan_kernel<<<1, kScanThreads, 0, stream>>>(V, keep, size, gid, off, totals);
  if ((e = hipGetLastError()) != hipSuccess) return fail(e);
  int64_t host_totals[3] = {0, 0, 0};
  if ((e = hipMemcpyAsync(host_totals, totals, sizeof host_totals, hipMemcpyDeviceToHost, stream)) !=
      hipSuccess)
    return fail(e);
  if ((e = hipStreamSynchronize(stream)) != hipSuccess) return fail(e);
  int32_t largest = 0;
  std::memcpy(&largest, &host_totals[2], sizeof largest);
  *out_G = (int32_t) host_totals[0];
  *out_nnz = host_totals[1];
  *out_max_size = largest;
  if (largest > cap) return PCG_ERR_CAPACITY;          // some set did not fit: nothing is written
  if (host_totals[1] > members_capacity || host_totals[1] > INT32_MAX) return PCG_ERR_CAPACITY;
  asg_compact_kernel<<<wb, 256, 0, stream>>>(V, cap, cand, size, keep, gid, off, totals, row_ptr,
                                             members, mult, seed_of);
  if ((e = hipGetLastError()) != hipSuccess) return fail(e);
  if ((e = hipStreamSynchronize(stream)) != hipSuccess) return fail(e);
  return PCG_OK;
}

int asg_check_outputs(int32_t V, int32_t d, float theta, int32_t cap, const int32_t *row_ptr,
                      const int32_t *members, int64_t members_capacity, const int32_t *mult,
                      const void *workspace) {
  if (V < 1 || d < 64 || d % 64 || cap < 1 || cap > kAsgMaxCap || members_capacity < 1 ||
      (int64_t) V * d > INT32_MAX || !std::isfinite(theta))
    return PCG_ERR_BAD_SHAPE;
  if (((uintptr_t) workspace % kAsgAlign) || ((uintptr_t) row_ptr % 4) || ((uintptr_t) members % 4) ||
      ((uintptr_t) mult % 4))
    return PCG_ERR_MISALIGNED;
  return PCG_OK;
}

}  // namespace

extern "C" {

int pcg_asg_normalize(const float *emb, int32_t V, int32_t d, uint16_t *unit_bf16,
                      void *hip_stream) {
  if (!emb || !unit_bf16) return PCG_ERR_NULL_ARG;
  if (V < 1 || d < 1) return PCG_ERR_BAD_SHAPE;
  if (((uintptr_t) emb % 4) || ((uintptr_t) unit_bf16 % 2)) return PCG_ERR_MISALIGNED;
  hipStream_t stream = (hipStream_t) hip_stream;
  asg_normalize_kernel<<<(unsigned) ((V + 3) / 4), 256, 0, stream>>>(emb, V, d, unit_bf16, nullptr);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? PCG_OK : record_hip_error(e);
}

size_t pcg_asg_build_workspace_bytes(int32_t V, int32_t cap) {
  if (V < 1 || cap < 1 || cap > kAsgMaxCap) return 0;
  return asg_core_workspace_bytes((size_t) V, cap) + kAsgAlign;
}

int pcg_asg_build(const uint16_t *unit_bf16, int32_t V, int32_t d, float theta, int32_t cap,
                  int32_t *row_ptr, int32_t *members, int64_t members_capacity, int32_t *mult,
                  int32_t *seed_of, int32_t *out_G, int64_t *out_nnz, int32_t *out_max_size,
                  void *workspace, size_t workspace_bytes, void *hip_stream) {
  if (!unit_bf16 || !row_ptr || !members || !mult || !out_G || !out_nnz || !out_max_size ||
      !workspace)
    return PCG_ERR_NULL_ARG;
  if (const int rc = asg_check_outputs(V, d, theta, cap, row_ptr, members, members_capacity, mult, workspace))
    return rc;
  if ((uintptr_t) unit_bf16 % 16) return PCG_ERR_MISALIGNED;
  if (workspace_bytes < pcg_asg_build_workspace_bytes(V, cap)) return PCG_ERR_WORKSPACE_TOO_SMALL;
  return asg_build_impl(nullptr, nullptr, unit_bf16, V, d, theta, cap, row_ptr, members,
                        members_capacity, mult, seed_of, out_G, out_nnz, out_max_size,
                        (char *) workspace, (hipStream_t) hip_stream);
}

size_t pcg_asg_build_exact_workspace_bytes(int32_t V, int32_t d, int32_t cap) {
  if (V < 1 || d < 1 || cap < 1 || cap > kAsgMaxCap || (int64_t) V * d > INT32_MAX) return 0;
  const size_t v = (size_t) V;
  return asg_core_workspace_bytes(v, cap) + asg_align(v * (size_t) d * 2) /* unit vectors */ +
         asg_align(v * 8) /* norms */ + kAsgAlign;
}

int pcg_asg_build_exact(const float *emb, int32_t V, int32_t d, float theta, int32_t cap,
                        int32_t *row_ptr, int32_t *members, int64_t members_capacity,
                        int32_t *mult, int32_t *seed_of, int32_t *out_G, int64_t *out_nnz,
                        int32_t *out_max_size, void *workspace, size_t workspace_bytes,
                        void *hip_stream) {
  if (!emb || !row_ptr || !members || !mult || !out_G || !out_nnz || !out_max_size || !workspace)
    return PCG_ERR_NULL_ARG;
  if (const int rc = asg_check_outputs(V, d, theta, cap, row_ptr, members, members_capacity, mult, workspace))
    return rc;
  if ((uintptr_t) emb % 16) return PCG_ERR_MISALIGNED;
  if (workspace_bytes < pcg_asg_build_exact_workspace_bytes(V, d, cap))
    return PCG_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t stream = (hipStream_t) hip_stream;
  const size_t v = (size_t) V;
  char *ws = (char *) workspace;
  uint16_t *unit = (uint16_t *) ws; ws += asg_align(v * (size_t) d * 2);
  double *norms = (double *) ws; ws += asg_align(v * 8);
  asg_normalize_kernel<<<(unsigned) ((V + 3) / 4), 256, 0, stream>>>(emb, V, d, unit, norms);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return record_hip_error(e);
  return asg_build_impl(emb, norms, unit, V, d, theta, cap, row_ptr, members, members_capacity,
                        mult, seed_of, out_G, out_nnz, out_max_size, ws, stream);
}

}  // extern "C"
