// Construction of the Acoustic Similarity Groups (Sec. 2.1, Eq. 1) on gfx950: unit vectors in
// bfloat16, the V x V cosine similarity as a bf16 MFMA contraction with fp32 accumulation that
// is thresholded on the fly (the similarity matrix is never stored), per-token member lists
// sorted ascending, identical sets dropped, and the CSR the verification kernels read.
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
  return (uint16_t) ((pick >> 16) | (x < 0.0 ? 0x8000u : 0u));
}

__global__ __launch_bounds__(256) void asg_normalize_kernel(const float *emb, int32_t V, int32_t d,
                                                            uint16_t *unit) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t v = (int64_t) blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6);
  if (v >= V) return;                       // whole waves leave together
  const float *e = emb + v * d;
  double ss = 0.0;
  for (int32_t k = lane; k < d; k += kWave) ss += (double) e[k] * (double) e[k];
  const double norm = sqrt(wave_sum(ss));
  for (int32_t k = lane; k < d; k += kWave)
    unit[v * d + k] = norm > 0.0 ? round_to_bf16((double) e[k] / norm) : (uint16_t) 0;
}

// ---------------------------------------------------------------------------------------------
// Similarity + threshold.  A workgroup of four waves owns a 128 x 128 tile of the similarity
// matrix; each wave a 64 x 64 quarter as 2 x 2 MFMA blocks of 32 x 32.  Both operands are rows
// of the same matrix of unit vectors, staged through LDS 64 columns of k at a time (double
// buffered; rows padded by 16 bytes so that the 16-byte operand reads of consecutive rows fall
// into different banks).  The matrix is symmetric: only tiles on or above the diagonal are
// computed, and a pair found off the diagonal is recorded for both of its tokens.
// ---------------------------------------------------------------------------------------------

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes on their way to LDS

constexpr int kSimTile = 128;                 // rows and columns of a workgroup's tile
constexpr int kSimK = 64;                     // k columns per LDS stage
constexpr int kSimRowBytes = kSimK * 2 + 16;  // padded LDS row
constexpr int kSimThreads = 256;
constexpr int kSimChunks = kSimTile * (kSimK / 8) / kSimThreads;   // 16-byte chunks per thread and tile

struct SimTiles {
  unsigned char a[2][kSimTile * kSimRowBytes];
  unsigned char b[2][kSimTile * kSimRowBytes];
};

// Record v as a member of G(t).
__device__ __forceinline__ void asg_emit(int32_t t, int32_t v, int32_t cap, int32_t *count,
                                         int32_t *cand) {
  const int32_t pos = atomicAdd(&count[t], 1);
  if (pos < cap) cand[(int64_t) t * cap + pos] = v;
}

// A thread's 16-byte chunks of one stage, from global memory into registers ...
__device__ __forceinline__ void sim_fetch(const uint16_t *__restrict__ unit,
                                          const int32_t (&src_a)[kSimChunks],
                                          const int32_t (&src_b)[kSimChunks], int32_t k0,
                                          u32x4 (&ga)[kSimChunks], u32x4 (&gb)[kSimChunks]) {
#pragma unroll
  for (int c = 0; c < kSimChunks; ++c) {
    ga[c] = *reinterpret_cast<const u32x4 *>(unit + src_a[c] + k0);
    gb[c] = *reinterpret_cast<const u32x4 *>(unit + src_b[c] + k0);
  }
}

// ... and from registers into the LDS tiles.
__device__ __forceinline__ void sim_stage(unsigned char *a, unsigned char *b,
                                          const int32_t (&dst)[kSimChunks],
                                          const u32x4 (&ga)[kSimChunks],
                                          const u32x4 (&gb)[kSimChunks]) {
#pragma unroll
  for (int c = 0; c < kSimChunks; ++c) {
    *reinterpret_cast<u32x4 *>(a + dst[c]) = ga[c];
    *reinterpret_cast<u32x4 *>(b + dst[c]) = gb[c];
  }
}

__global__ __launch_bounds__(kSimThreads) void asg_similarity_kernel(
    const uint16_t *__restrict__ unit, int32_t V, int32_t d, float theta, int32_t cap,
    int32_t *count, int32_t *cand) {
  const int tj = blockIdx.x, ti = blockIdx.y;
  if (tj < ti) return;                         // lower triangle: covered by its mirror tile
  __shared__ __attribute__((aligned(16))) SimTiles lds;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int32_t row0 = ti * kSimTile, col0 = tj * kSimTile;

  // this thread's 16-byte chunks of a stage: tile row and k offset (the same for A and B)
  int32_t src_a[kSimChunks], src_b[kSimChunks], dst[kSimChunks];
#pragma unroll
  for (int c = 0; c < kSimChunks; ++c) {
    const int chunk = tid + c * kSimThreads;
    const int r = chunk >> 3, kc = chunk & 7;
    // rows past the end of the matrix re-read the last row; their results are never recorded
    src_a[c] = min(row0 + r, V - 1) * d + kc * 8;
    src_b[c] = min(col0 + r, V - 1) * d + kc * 8;
    dst[c] = r * kSimRowBytes + kc * 16;
  }
  u32x4 ga[kSimChunks], gb[kSimChunks];

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // operand addresses of this lane: row (lane % 32) of the block, k half (lane / 32)
  const int frag = (lane & 31) * kSimRowBytes + (lane >> 5) * 16;
  const int a_off = (wm * 64) * kSimRowBytes + frag, b_off = (wn * 64) * kSimRowBytes + frag;

  const int nstages = d / kSimK;
  sim_fetch(unit, src_a, src_b, 0, ga, gb);
  sim_stage(lds.a[0], lds.b[0], dst, ga, gb);
  __syncthreads();
  for (int s = 0; s < nstages; ++s) {
    const int buf = s & 1;
    if (s + 1 < nstages) sim_fetch(unit, src_a, src_b, (s + 1) * kSimK, ga, gb);
#pragma unroll
    for (int kk = 0; kk < kSimK / 16; ++kk) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *reinterpret_cast<const bf16x8 *>(lds.a[buf] + a_off + i * 32 * kSimRowBytes + kk * 32);
        fb[i] = *reinterpret_cast<const bf16x8 *>(lds.b[buf] + b_off + i * 32 * kSimRowBytes + kk * 32);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (s + 1 < nstages) sim_stage(lds.a[buf ^ 1], lds.b[buf ^ 1], dst, ga, gb);
    __syncthreads();
  }

  // Threshold (Eq. 1).  Accumulator r of a lane is row 8 (r / 4) + 4 (lane / 32) + r % 4 and
  // column lane % 32 of its 32 x 32 block.
  const bool diagonal = ti == tj;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int32_t t = row0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int32_t v = col0 + wn * 64 + j * 32 + (lane & 31);
        if (t >= V || v >= V) continue;
        if (acc[i][j][r] > theta || t == v) {
          asg_emit(t, v, cap, count, cand);
          if (!diagonal) asg_emit(v, t, cap, count, cand);
        }
      }
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

extern "C" {

int pcg_asg_normalize(const float *emb, int32_t V, int32_t d, uint16_t *unit_bf16,
                      void *hip_stream) {
  if (!emb || !unit_bf16) return PCG_ERR_NULL_ARG;
  if (V < 1 || d < 1) return PCG_ERR_BAD_SHAPE;
  if (((uintptr_t) emb % 4) || ((uintptr_t) unit_bf16 % 2)) return PCG_ERR_MISALIGNED;
  hipStream_t stream = (hipStream_t) hip_stream;
  asg_normalize_kernel<<<(unsigned) ((V + 3) / 4), 256, 0, stream>>>(emb, V, d, unit_bf16);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? PCG_OK : record_hip_error(e);
}

size_t pcg_asg_build_workspace_bytes(int32_t V, int32_t cap) {
  if (V < 1 || cap < 1 || cap > kAsgMaxCap) return 0;
  const size_t v = (size_t) V;
  return asg_align(v * 4) /* count */ + asg_align(v * (size_t) cap * 4) /* cand */ +
         asg_align(v * 4) /* size */ + asg_align(v * 8) /* hash */ + asg_align(v * 4) /* keep */ +
         asg_align(v * 4) /* gid */ + asg_align(v * 8) /* off */ + asg_align(64) /* totals */ +
         kAsgAlign;
}

int pcg_asg_build(const uint16_t *unit_bf16, int32_t V, int32_t d, float theta, int32_t cap,
                  int32_t *row_ptr, int32_t *members, int64_t members_capacity, int32_t *mult,
                  int32_t *seed_of, int32_t *out_G, int64_t *out_nnz, int32_t *out_max_size,
                  void *workspace, size_t workspace_bytes, void *hip_stream) {
  if (!unit_bf16 || !row_ptr || !members || !mult || !out_G || !out_nnz || !out_max_size ||
      !workspace)
    return PCG_ERR_NULL_ARG;
  if (V < 1 || d < kSimK || d % kSimK || cap < 1 || cap > kAsgMaxCap || members_capacity < 1 ||
      (int64_t) V * d > INT32_MAX || !std::isfinite(theta))
    return PCG_ERR_BAD_SHAPE;
  if (((uintptr_t) unit_bf16 % 16) || ((uintptr_t) workspace % kAsgAlign) ||
      ((uintptr_t) row_ptr % 4) || ((uintptr_t) members % 4) || ((uintptr_t) mult % 4))
    return PCG_ERR_MISALIGNED;
  if (workspace_bytes < pcg_asg_build_workspace_bytes(V, cap)) return PCG_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t stream = (hipStream_t) hip_stream;
  const size_t v = (size_t) V;
  char *ws = (char *) workspace;
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
  const unsigned tiles = (unsigned) ((V + kSimTile - 1) / kSimTile);
  asg_similarity_kernel<<<dim3(tiles, tiles), kSimThreads, 0, stream>>>(unit_bf16, V, d, theta, cap,
                                                                        count, cand);
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

}  // extern "C"
