// C ABI of libpcg (see include/pcg.h): argument checks, workspace carving, kernel sequencing.
// No device memory is allocated here and nothing synchronises except pcg_profile_end.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "pcg_kernels.h"
#include "pcg_layout.h"

// The library's own scratch memory (pcg_verify_static): one array per GPU, in that GPU's memory
// from the moment the code object is loaded there until the process ends.  In host code this
// name is only the handle of the symbol, never a device address.
static __device__ __align__(256) unsigned char scratch[PCG_STATIC_SCRATCH_BYTES];

namespace {

using namespace pcg;

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
  g_last_hip_error = (int) e;
  return PCG_ERR_HIP;
}

}  // namespace

namespace pcg {
int record_hip_error(hipError_t e) { return hip_fail(e); }
}  // namespace pcg

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

// ---- per-kernel timing -------------------------------------------------------------------

enum Stage { kStageStats = 0, kStageAccept, kStageTable, kStageGather, kStageFinalize, kStageThin,
             kStagePropose, kStageNull, kNumStages };
static_assert(kNumStages <= PCG_MAX_STAGES, "pcg_profile_end writes PCG_MAX_STAGES floats");
const char *const kStageNames[kNumStages] = {"row_stats", "accept_delta", "weights", "gather", "finalize",
                                             "accept_thin", "propose", "event_overhead"};

struct Profile {
  bool active = false;
  int32_t max_calls = 0, calls = 0;
  // per recorded call: one event before each stage and one after the last
  std::vector<hipEvent_t> ev;
  std::vector<uint8_t> used;   // which stages the call ran
} g_prof;

struct StageTimer {
  hipStream_t stream;
  int slot;          // index of the recorded call, -1 if not recording
  explicit StageTimer(hipStream_t s) : stream(s), slot(-1) {
    // events recorded into a stream that is being captured would become nodes of the caller's
    // graph: a call under capture is never timed
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    const bool capturing =
        g_prof.active && (hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone);
    if (g_prof.active && !capturing && g_prof.calls < g_prof.max_calls) slot = g_prof.calls++;
    // two events with nothing between them: what an event pair costs on this stream, to be
    // taken off the stage times by whoever reads them
    begin(kStageNull);
    end(kStageNull);
  }
  void begin(Stage st) {
    if (slot < 0) return;
    (void) hipEventRecord(g_prof.ev[(size_t) slot * 2 * kNumStages + 2 * st], stream);
    g_prof.used[(size_t) slot * kNumStages + st] = 1;
  }
  void end(Stage st) {
    if (slot < 0) return;
    (void) hipEventRecord(g_prof.ev[(size_t) slot * 2 * kNumStages + 2 * st + 1], stream);
  }
};

bool good_temperature(float t) { return std::isfinite(t) && t > 0.0f; }

int check_groups(const pcg_groups *g) {
  if (!g) return PCG_ERR_NULL_ARG;
  if (!g->row_ptr || !g->mult) return PCG_ERR_NULL_ARG;
  if (g->V < 1 || g->G < 1 || g->nnz < 0 || g->nnz > INT32_MAX) return PCG_ERR_BAD_SHAPE;
  if (g->nnz > 0 && !g->members) return PCG_ERR_NULL_ARG;
  if ((g->prepared == nullptr) != (g->prepared_info == nullptr)) return PCG_ERR_NULL_ARG;
  // with weights the prepared form must have been built with them
  if (g->weights && g->prepared && g->prepared_info->off_weights == 0) return PCG_ERR_BAD_SHAPE;
  if (g->weights && ((uintptr_t) g->weights % 4)) return PCG_ERR_MISALIGNED;
  if (g->prepared) {
    const pcg_prepared &p = *g->prepared_info;
    if (p.V != g->V || p.G != g->G || p.ntiles < 1 || p.tile_len < 1 || p.tile_len > kTileTokensMax ||
        (int64_t) p.ntiles * p.tile_len < g->V || p.chunk_groups < kChunkStep ||
        p.chunk_groups > kMaxChunkGroups || p.chunk_groups % kChunkStep ||
        p.blocks_per_chunk != p.chunk_groups / kBlockGroups ||
        p.nchunks != (g->G + p.chunk_groups - 1) / p.chunk_groups)
      return PCG_ERR_BAD_SHAPE;
    if (p.off_weights != 0 &&
        (p.off_weights % 256 || p.off_weights <= p.off_data || p.off_weights >= p.bytes))
      return PCG_ERR_BAD_SHAPE;
    if ((uintptr_t) g->prepared % 256) return PCG_ERR_MISALIGNED;
  }
  return PCG_OK;
}

bool stride_ok(int64_t s, int32_t V, bool zero_allowed) {
  return s >= V || (zero_allowed && s == 0);
}

struct Factors {
  double cd;          // log2(e) / temperature
  float c, c_lo;      // c = fp32(cd) (also the high piece), c_lo = fp32(cd - c)
};
Factors factors(float temperature) {
  Factors f;
  f.cd = 1.4426950408889634074 / (double) temperature;
  f.c = (float) f.cd;
  f.c_lo = (float) (f.cd - (double) f.c);
  return f;
}

// rows of table staged per gather launch in pcg_group_probs
int64_t group_probs_batch(int32_t V, int64_t rows) {
  int64_t batch = ((int64_t) 64 << 20) / ((int64_t) V * 4);
  if (batch < 8) batch = 8;
  if (batch > 4096) batch = 4096;
  if (batch > rows) batch = rows;
  return batch;
}

}  // namespace

extern "C" {

size_t pcg_group_probs_workspace_bytes(int32_t V, int64_t rows) {
  if (V < 1 || rows < 0) return 0;
  const size_t parts = align_up((size_t) rows * stats_nparts(V) * sizeof(StatPart));
  const size_t table = align_up((size_t) group_probs_batch(V, rows) * V * sizeof(float));
  return parts + table + kAlign;
}

size_t pcg_verify_workspace_bytes(int32_t V, int32_t G, int32_t B, int32_t K) {
  if (V < 1 || G < 1 || B < 0 || K < 1) return 0;
  const size_t rows = (size_t) B * (2 * (size_t) K + 1);
  return align_up(rows * stats_nparts(V) * sizeof(StatPart)) + align_up(rows * sizeof(RowStat)) +
         align_up((size_t) B * K * sizeof(Probe)) +
         align_up((size_t) B * V * sizeof(float)) + align_up((size_t) B * G * sizeof(float)) +
         align_up((size_t) B * ((G + kChunkStep - 1) / kChunkStep) * sizeof(double)) +
         align_up((size_t) B * (((size_t) G + kMaxChunkGroups) / kRunGroups) * sizeof(double)) + kAlign;
}

int pcg_group_probs(const pcg_groups *groups, const void *logits, pcg_dtype dt, int64_t rows,
                    int64_t row_stride, float temperature, float *out, void *workspace,
                    size_t workspace_bytes, void *hip_stream) {
  int rc = check_groups(groups);
  if (rc) return rc;
  if (dt != PCG_F32 && dt != PCG_BF16) return PCG_ERR_BAD_DTYPE;
  if (rows < 0 || rows > ((int64_t) 1 << 40)) return PCG_ERR_BAD_SHAPE;
  if (rows == 0) return PCG_OK;
  if (!logits || !out || !workspace) return PCG_ERR_NULL_ARG;
  if (!stride_ok(row_stride, groups->V, rows == 1)) return PCG_ERR_BAD_STRIDE;
  if (!good_temperature(temperature)) return PCG_ERR_BAD_TEMPERATURE;
  const bool bf16 = dt == PCG_BF16;
  if (((uintptr_t) logits % (bf16 ? 2 : 4)) || ((uintptr_t) workspace % kAlign) ||
      ((uintptr_t) out % 4))
    return PCG_ERR_MISALIGNED;
  if (workspace_bytes < pcg_group_probs_workspace_bytes(groups->V, rows))
    return PCG_ERR_WORKSPACE_TOO_SMALL;
  const int32_t nparts = stats_nparts(groups->V);
  if (rows * nparts / 4 >= INT32_MAX) return PCG_ERR_BAD_SHAPE;

  hipStream_t stream = (hipStream_t) hip_stream;
  char *ws = (char *) workspace;
  StatPart *parts = (StatPart *) ws;
  ws += align_up((size_t) rows * nparts * sizeof(StatPart));
  float *table = (float *) ws;

  RowSet rs;
  std::memset(&rs, 0, sizeof rs);
  rs.base0 = logits;
  rs.bs0 = row_stride;
  rs.npos0 = 1;
  rs.npos1 = 1;
  rs.nrows0 = rows;
  rs.inv_npos0 = rs.inv_npos1 = 1.0;
  const Factors f = factors(temperature);

  StageTimer tm(stream);
  hipError_t e;
  tm.begin(kStageStats);
  if ((e = launch_row_stats(rs, bf16, groups->V, rows, f.c, true, parts, stream)) != hipSuccess)
    return hip_fail(e);
  tm.end(kStageStats);
  const int64_t batch = group_probs_batch(groups->V, rows);
  for (int64_t r0 = 0; r0 < rows; r0 += batch) {
    const int32_t n = (int32_t) std::min(batch, rows - r0);
    if (r0 == 0) tm.begin(kStageTable);
    if ((e = launch_weights(rs, bf16, *groups, r0, n, f.c, f.c, f.c_lo, parts, table, stream)) !=
        hipSuccess)
      return hip_fail(e);
    if (r0 == 0) { tm.end(kStageTable); tm.begin(kStageGather); }
    e = groups->prepared
            ? launch_gather_prepared(*groups, n, table, out + r0 * groups->G, nullptr, nullptr, stream)
            : launch_gather(*groups, n, false, table, out + r0 * groups->G, stream);
    if (e != hipSuccess) return hip_fail(e);
    if (r0 == 0) tm.end(kStageGather);
  }
  return PCG_OK;
}

}  // extern "C"

namespace {

// Host-side checks shared by the two verify entry points; on PCG_OK with B > 0 fills rs.
int check_verify_args(const pcg_groups *groups, const void *target_logits, const void *draft_logits,
                      pcg_dtype dt, int32_t B, int32_t K, int64_t tgt_batch_stride,
                      int64_t tgt_pos_stride, int64_t dft_batch_stride, int64_t dft_pos_stride,
                      float temperature, const int32_t *prop_tokens, const int32_t *prop_groups,
                      const int32_t *accept_len, const int32_t *out_tokens,
                      const int32_t *out_groups, const void *workspace, RowSet &rs) {
  int rc = check_groups(groups);
  if (rc) return rc;
  if (dt != PCG_F32 && dt != PCG_BF16) return PCG_ERR_BAD_DTYPE;
  if (B < 0 || B > (1 << 24) || K < 1 || K > PCG_MAX_K) return PCG_ERR_BAD_SHAPE;
  if (B == 0) return PCG_OK;
  if (!target_logits || !draft_logits || !prop_tokens || !prop_groups || !accept_len ||
      !out_tokens || !out_groups || !workspace)
    return PCG_ERR_NULL_ARG;
  const int32_t V = groups->V;
  if (!stride_ok(tgt_pos_stride, V, false) || !stride_ok(dft_pos_stride, V, K == 1) ||
      !stride_ok(tgt_batch_stride, V, true) || !stride_ok(dft_batch_stride, V, true))
    return PCG_ERR_BAD_STRIDE;
  if (!good_temperature(temperature)) return PCG_ERR_BAD_TEMPERATURE;
  const uintptr_t esz = dt == PCG_BF16 ? 2 : 4;
  if (((uintptr_t) target_logits % esz) || ((uintptr_t) draft_logits % esz) ||
      ((uintptr_t) workspace % kAlign))
    return PCG_ERR_MISALIGNED;
  const int64_t rows = (int64_t) B * (2 * K + 1);
  if (rows * stats_nparts(V) / 4 >= INT32_MAX) return PCG_ERR_BAD_SHAPE;
  if ((int64_t) B * ((V + 2047) / 2048) >= INT32_MAX) return PCG_ERR_BAD_SHAPE;
  rs.base0 = target_logits;
  rs.base1 = draft_logits;
  rs.bs0 = tgt_batch_stride;
  rs.ps0 = tgt_pos_stride;
  rs.bs1 = dft_batch_stride;
  rs.ps1 = dft_pos_stride;
  rs.npos0 = K + 1;
  rs.npos1 = K;
  rs.nrows0 = (int64_t) B * (K + 1);
  rs.inv_npos0 = 1.0 / (K + 1);
  rs.inv_npos1 = 1.0 / K;
  return PCG_OK;
}

ProbeArgs probe_args(const pcg_groups *groups, int32_t K, const Factors &f,
                     const int32_t *prop_groups, Probe *out) {
  ProbeArgs pa;
  pa.row_ptr = groups->row_ptr;
  pa.members = groups->members;
  pa.mult = groups->mult;
  pa.prop_groups = prop_groups;
  pa.weights = groups->weights;
  pa.K = K;
  pa.G = groups->G;
  pa.c_lo = f.c_lo;
  pa.out = out;
  return pa;
}

AcceptArgs accept_args(const pcg_groups *groups, const RowSet &rs, int32_t K, const Factors &f,
                       const StatPart *parts, const Probe *probes, RowStat *rowstat,
                       const int32_t *prop_tokens,
                       const int32_t *prop_groups, uint64_t seed, uint64_t offset,
                       int32_t *accept_len, int32_t *out_tokens, int32_t *out_groups,
                       pcg_diag *diag) {
  AcceptArgs aa;
  aa.rs = rs;
  aa.V = groups->V;
  aa.G = groups->G;
  aa.K = K;
  aa.nparts = stats_nparts(groups->V);
  aa.c = f.c;
  aa.cd = f.cd;
  aa.parts = parts;
  aa.probes = probes;
  aa.rowstat = rowstat;
  aa.row_ptr = groups->row_ptr;
  aa.members = groups->members;
  aa.mult = groups->mult;
  aa.weights = groups->weights;
  aa.prop_tokens = prop_tokens;
  aa.prop_groups = prop_groups;
  aa.seed = seed;
  aa.offset = offset;
  aa.accept_len = accept_len;
  aa.out_tokens = out_tokens;
  aa.out_groups = out_groups;
  aa.diag = diag;
  return aa;
}

// The whole step on `workspace` (device memory, wherever it comes from): shared by pcg_verify,
// whose caller brings the workspace, and pcg_verify_static, which uses the library's own array.
int verify_impl(const pcg_groups *groups, const void *target_logits, const void *draft_logits,
                pcg_dtype dt, int32_t B, int32_t K, int64_t tgt_batch_stride,
                int64_t tgt_pos_stride, int64_t dft_batch_stride, int64_t dft_pos_stride,
                float temperature, const int32_t *prop_tokens, const int32_t *prop_groups,
                uint64_t seed, uint64_t offset, int32_t *accept_len, int32_t *out_tokens,
                int32_t *out_groups, pcg_diag *diag, void *workspace, size_t workspace_bytes,
                void *hip_stream) {
  RowSet rs;
  int rc = check_verify_args(groups, target_logits, draft_logits, dt, B, K, tgt_batch_stride,
                             tgt_pos_stride, dft_batch_stride, dft_pos_stride, temperature,
                             prop_tokens, prop_groups, accept_len, out_tokens, out_groups,
                             workspace, rs);
  if (rc || B == 0) return rc;
  const int32_t V = groups->V;
  const bool bf16 = dt == PCG_BF16;
  if (workspace_bytes < pcg_verify_workspace_bytes(V, groups->G, B, K))
    return PCG_ERR_WORKSPACE_TOO_SMALL;
  const int64_t rows = (int64_t) B * (2 * K + 1);
  const int32_t nparts = stats_nparts(V);

  hipStream_t stream = (hipStream_t) hip_stream;
  char *ws = (char *) workspace;
  StatPart *parts = (StatPart *) ws;
  ws += align_up((size_t) rows * nparts * sizeof(StatPart));
  RowStat *rowstat = (RowStat *) ws;
  ws += align_up((size_t) rows * sizeof(RowStat));
  Probe *probes = (Probe *) ws;
  ws += align_up((size_t) B * K * sizeof(Probe));
  float *table = (float *) ws;
  ws += align_up((size_t) B * V * sizeof(float));
  float *R = (float *) ws;
  ws += align_up((size_t) B * groups->G * sizeof(float));
  double *csum = (double *) ws;
  ws += align_up((size_t) B * ((groups->G + kChunkStep - 1) / kChunkStep) * sizeof(double));
  double *runs = (double *) ws;     // [B][nchunks][chunk_groups / kRunGroups]

  const Factors f = factors(temperature);
  const AcceptArgs aa = accept_args(groups, rs, K, f, parts, probes, rowstat, prop_tokens, prop_groups,
                                    seed, offset, accept_len, out_tokens, out_groups, diag);
  const ProbeArgs pa = probe_args(groups, K, f, prop_groups, probes);
  FinalizeArgs fa;
  fa.rs = rs;
  fa.K = K;
  fa.cd = f.cd;
  fa.c = f.c;
  fa.c_lo = f.c_lo;
  fa.rowstat = rowstat;
  fa.row_ptr = groups->row_ptr;
  fa.members = groups->members;
  fa.mult = groups->mult;
  fa.weights = groups->weights;
  fa.seed = seed;
  fa.offset = offset;
  fa.accept_len = accept_len;
  fa.R = R;
  fa.out_tokens = out_tokens;
  fa.out_groups = out_groups;
  fa.diag = diag;

  StageTimer tm(stream);
  hipError_t e;
  tm.begin(kStageStats);
  // streaming pass: only the rejected position's two rows (2 of 2K+1) are read again
  if ((e = launch_row_stats(rs, bf16, V, rows, f.c, true, parts, stream, &pa)) != hipSuccess) return hip_fail(e);
  tm.end(kStageStats);
  tm.begin(kStageAccept);
  if ((e = launch_accept_delta(aa, bf16, B, f.c_lo, table, stream)) != hipSuccess)
    return hip_fail(e);
  tm.end(kStageAccept);
  tm.begin(kStageGather);
  const bool prepared = groups->prepared != nullptr;
  e = prepared ? launch_gather_prepared(*groups, B, table, R, csum, runs, stream)
               : launch_gather(*groups, B, true, table, R, stream);
  if (e != hipSuccess) return hip_fail(e);
  tm.end(kStageGather);
  tm.begin(kStageFinalize);
  if ((e = launch_finalize(fa, bf16, *groups, B, prepared ? csum : nullptr,
                           prepared ? runs : nullptr,
                           prepared ? groups->prepared_info->nchunks : 1,
                           prepared ? groups->prepared_info->chunk_groups : groups->G, stream)) !=
      hipSuccess)
    return hip_fail(e);
  tm.end(kStageFinalize);
  return PCG_OK;
}

// ---- the library's own scratch memory, for callers that cannot allocate --------------------
//
// `scratch` (top of this file) is only the host-side handle of the symbol: the device address
// is asked for once per device (hipGetSymbolAddress) and kept; every use goes through it.

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device; NULL with *rc set on failure.
void *scratch_address(int *rc) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { *rc = hip_fail(e); return nullptr; }
  if (dev < 0 || dev >= kMaxDevices) { *rc = PCG_ERR_BAD_SHAPE; return nullptr; }
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
  if (p) return p;
  e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !p) { *rc = hip_fail(e == hipSuccess ? hipErrorInvalidSymbol : e); return nullptr; }
  g_scratch_ptr[dev].store(p, std::memory_order_release);
  return p;
}

}  // namespace

extern "C" {

int pcg_verify(const pcg_groups *groups, const void *target_logits, const void *draft_logits,
               pcg_dtype dt, int32_t B, int32_t K, int64_t tgt_batch_stride,
               int64_t tgt_pos_stride, int64_t dft_batch_stride, int64_t dft_pos_stride,
               float temperature, const int32_t *prop_tokens, const int32_t *prop_groups,
               uint64_t seed, uint64_t offset, int32_t *accept_len, int32_t *out_tokens,
               int32_t *out_groups, pcg_diag *diag, void *workspace, size_t workspace_bytes,
               void *hip_stream) {
  return verify_impl(groups, target_logits, draft_logits, dt, B, K, tgt_batch_stride,
                     tgt_pos_stride, dft_batch_stride, dft_pos_stride, temperature, prop_tokens,
                     prop_groups, seed, offset, accept_len, out_tokens, out_groups, diag, workspace,
                     workspace_bytes, hip_stream);
}

size_t pcg_static_scratch_bytes(void) { return PCG_STATIC_SCRATCH_BYTES; }

int pcg_verify_static(const pcg_groups *groups, const void *target_logits,
                      const void *draft_logits, pcg_dtype dt, int32_t B, int32_t K,
                      int64_t tgt_batch_stride, int64_t tgt_pos_stride, int64_t dft_batch_stride,
                      int64_t dft_pos_stride, float temperature, const int32_t *prop_tokens,
                      const int32_t *prop_groups, uint64_t seed, uint64_t offset,
                      int32_t *accept_len, int32_t *out_tokens, int32_t *out_groups,
                      pcg_diag *diag, void *hip_stream) {
  // sizes first: a step that does not fit the array is refused before anything else happens
  if (!groups) return PCG_ERR_NULL_ARG;
  if (groups->V < 1 || groups->G < 1 || B < 0 || K < 1 || K > PCG_MAX_K) return PCG_ERR_BAD_SHAPE;
  if (pcg_verify_workspace_bytes(groups->V, groups->G, B, K) > PCG_STATIC_SCRATCH_BYTES)
    return PCG_ERR_SCRATCH_TOO_SMALL;
  int rc = PCG_OK;
  void *ws = scratch_address(&rc);
  if (!ws) return rc;
  return verify_impl(groups, target_logits, draft_logits, dt, B, K, tgt_batch_stride,
                     tgt_pos_stride, dft_batch_stride, dft_pos_stride, temperature, prop_tokens,
                     prop_groups, seed, offset, accept_len, out_tokens, out_groups, diag, ws,
                     PCG_STATIC_SCRATCH_BYTES, hip_stream);
}

size_t pcg_propose_workspace_bytes(int32_t V, int32_t B, int32_t K) {
  if (V < 1 || B < 0 || K < 1) return 0;
  return align_up((size_t) B * K * stats_nparts(V) * sizeof(StatPart)) + kAlign;
}

int pcg_propose(const pcg_groups *groups, const void *draft_logits, pcg_dtype dt, int32_t B,
                int32_t K, int32_t pos0, int64_t dft_batch_stride, int64_t dft_pos_stride,
                float temperature, uint64_t seed, uint64_t offset, int32_t *prop_tokens,
                int32_t *prop_groups, pcg_diag *diag, void *workspace, size_t workspace_bytes,
                void *hip_stream) {
  int rc = check_groups(groups);
  if (rc) return rc;
  if (dt != PCG_F32 && dt != PCG_BF16) return PCG_ERR_BAD_DTYPE;
  if (B < 0 || K < 1 || pos0 < 0 || (int64_t) pos0 + K > PCG_MAX_K) return PCG_ERR_BAD_SHAPE;
  if (B == 0) return PCG_OK;
  if (!draft_logits || !prop_tokens || !prop_groups || !workspace || !groups->tok_ptr ||
      !groups->tok_groups || (groups->weights && !groups->tok_weights))
    return PCG_ERR_NULL_ARG;
  const int32_t V = groups->V;
  if (!stride_ok(dft_pos_stride, V, K == 1) || !stride_ok(dft_batch_stride, V, true))
    return PCG_ERR_BAD_STRIDE;
  if (!good_temperature(temperature)) return PCG_ERR_BAD_TEMPERATURE;
  const bool bf16 = dt == PCG_BF16;
  if (((uintptr_t) draft_logits % (bf16 ? 2 : 4)) || ((uintptr_t) workspace % kAlign))
    return PCG_ERR_MISALIGNED;
  const int32_t nparts = stats_nparts(V);
  const int64_t rows = (int64_t) B * K;
  if (nparts > thin_max_parts() || rows * nparts / 4 >= INT32_MAX || rows >= INT32_MAX)
    return PCG_ERR_BAD_SHAPE;
  if (workspace_bytes < pcg_propose_workspace_bytes(V, B, K)) return PCG_ERR_WORKSPACE_TOO_SMALL;

  RowSet rs;
  std::memset(&rs, 0, sizeof rs);
  rs.base0 = draft_logits;
  rs.bs0 = dft_batch_stride;
  rs.ps0 = dft_pos_stride;
  rs.npos0 = K;
  rs.npos1 = 1;
  rs.nrows0 = rows;
  rs.inv_npos0 = 1.0 / K;
  rs.inv_npos1 = 1.0;
  const Factors f = factors(temperature);
  hipStream_t stream = (hipStream_t) hip_stream;
  StatPart *parts = (StatPart *) workspace;
  StageTimer tm(stream);
  hipError_t e;
  tm.begin(kStageStats);
  // cached pass: the draw that follows is a chain of small reads into the same rows
  if ((e = launch_row_stats(rs, bf16, V, rows, f.c, false, parts, stream)) != hipSuccess) return hip_fail(e);
  tm.end(kStageStats);
  tm.begin(kStagePropose);
  if ((e = launch_propose(rs, bf16, V, K, pos0, f.c, parts, groups->tok_ptr, groups->tok_groups,
                          groups->weights ? groups->tok_weights : nullptr, seed, offset,
                          prop_tokens, prop_groups, diag, stream)) != hipSuccess)
    return hip_fail(e);
  tm.end(kStagePropose);
  return PCG_OK;
}

size_t pcg_verify_thinning_workspace_bytes(int32_t V, int32_t B, int32_t K) {
  if (V < 1 || B < 0 || K < 1) return 0;
  const size_t rows = (size_t) B * (2 * (size_t) K + 1);
  return align_up(rows * stats_nparts(V) * sizeof(StatPart)) + align_up(rows * sizeof(RowStat)) +
         align_up((size_t) B * K * sizeof(Probe)) + kAlign;
}

int pcg_verify_thinning(const pcg_groups *groups, const void *target_logits,
                        const void *draft_logits, pcg_dtype dt, int32_t B, int32_t K,
                        int64_t tgt_batch_stride, int64_t tgt_pos_stride, int64_t dft_batch_stride,
                        int64_t dft_pos_stride, float temperature, const int32_t *prop_tokens,
                        const int32_t *prop_groups, uint64_t seed, uint64_t offset,
                        int32_t *accept_len, int32_t *out_tokens, int32_t *out_groups,
                        int32_t *trials, pcg_diag *diag, void *workspace, size_t workspace_bytes,
                        void *hip_stream) {
  RowSet rs;
  int rc = check_verify_args(groups, target_logits, draft_logits, dt, B, K, tgt_batch_stride,
                             tgt_pos_stride, dft_batch_stride, dft_pos_stride, temperature,
                             prop_tokens, prop_groups, accept_len, out_tokens, out_groups,
                             workspace, rs);
  if (rc || B == 0) return rc;
  if (!trials || !groups->tok_ptr || !groups->tok_groups) return PCG_ERR_NULL_ARG;
  if (groups->weights && !groups->tok_weights) return PCG_ERR_NULL_ARG;
  const int32_t V = groups->V;
  const int32_t nparts = stats_nparts(V);
  if (nparts > thin_max_parts()) return PCG_ERR_BAD_SHAPE;
  if (workspace_bytes < pcg_verify_thinning_workspace_bytes(V, B, K))
    return PCG_ERR_WORKSPACE_TOO_SMALL;
  const bool bf16 = dt == PCG_BF16;
  const int64_t rows = (int64_t) B * (2 * K + 1);
  hipStream_t stream = (hipStream_t) hip_stream;
  char *ws = (char *) workspace;
  StatPart *parts = (StatPart *) ws;
  ws += align_up((size_t) rows * nparts * sizeof(StatPart));
  RowStat *rowstat = (RowStat *) ws;
  ws += align_up((size_t) rows * sizeof(RowStat));
  Probe *probes = (Probe *) ws;
  const Factors f = factors(temperature);
  const AcceptArgs aa = accept_args(groups, rs, K, f, parts, probes, rowstat, prop_tokens, prop_groups,
                                    seed, offset, accept_len, out_tokens, out_groups, diag);
  const ProbeArgs pa = probe_args(groups, K, f, prop_groups, probes);
  StageTimer tm(stream);
  hipError_t e;
  tm.begin(kStageStats);
  // cached pass: every trial is a chain of small reads into the same rows
  if ((e = launch_row_stats(rs, bf16, V, rows, f.c, false, parts, stream, &pa)) != hipSuccess) return hip_fail(e);
  tm.end(kStageStats);
  tm.begin(kStageThin);
  if ((e = launch_accept_thin(aa, bf16, B, groups->tok_ptr, groups->tok_groups,
                              groups->weights ? groups->tok_weights : nullptr, trials,
                              PCG_THIN_MAX_TRIALS, stream)) != hipSuccess)
    return hip_fail(e);
  tm.end(kStageThin);
  return PCG_OK;
}

// ---- per-kernel timing ---------------------------------------------------------------------

int pcg_profile_begin(int32_t max_calls) {
  if (g_prof.active || max_calls < 1 || max_calls > 100000) return PCG_ERR_BAD_SHAPE;
  g_prof.ev.assign((size_t) max_calls * 2 * kNumStages, nullptr);
  g_prof.used.assign((size_t) max_calls * kNumStages, 0);
  for (auto &ev : g_prof.ev) {
    // timing events need no cache flush of their own
    hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableSystemFence);
    if (e != hipSuccess) {
      for (auto &x : g_prof.ev) if (x) (void) hipEventDestroy(x);
      g_prof.ev.clear();
      return hip_fail(e);
    }
  }
  g_prof.max_calls = max_calls;
  g_prof.calls = 0;
  g_prof.active = true;
  return PCG_OK;
}

int pcg_profile_end(float *stage_ms, int32_t *calls) {
  if (!g_prof.active) return PCG_ERR_BAD_SHAPE;
  if (!stage_ms || !calls) return PCG_ERR_NULL_ARG;
  g_prof.active = false;
  int rc = PCG_OK;
  double sum[kNumStages] = {0};
  int32_t cnt[kNumStages] = {0};
  for (int32_t c = 0; c < g_prof.calls && rc == PCG_OK; ++c) {
    for (int st = 0; st < kNumStages; ++st) {
      if (!g_prof.used[(size_t) c * kNumStages + st]) continue;
      hipEvent_t a = g_prof.ev[(size_t) c * 2 * kNumStages + 2 * st];
      hipEvent_t b = g_prof.ev[(size_t) c * 2 * kNumStages + 2 * st + 1];
      hipError_t e = hipEventSynchronize(b);
      float ms = 0.f;
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
      if (e != hipSuccess) { rc = hip_fail(e); break; }
      sum[st] += ms;
      cnt[st] += 1;
    }
  }
  for (int st = 0; st < PCG_MAX_STAGES; ++st)
    stage_ms[st] = (st < kNumStages && cnt[st]) ? (float) (sum[st] / cnt[st]) : 0.f;
  *calls = g_prof.calls;
  for (auto &x : g_prof.ev) if (x) (void) hipEventDestroy(x);
  g_prof.ev.clear();
  g_prof.used.clear();
  return rc;
}

const char *pcg_stage_name(int32_t stage) {
  return (stage >= 0 && stage < kNumStages) ? kStageNames[stage] : "";
}

// ---- group membership on the host ----------------------------------------------------------

static bool csr_well_formed(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members) {
  if (row_ptr[0] != 0) return false;
  for (int32_t g = 0; g < G; ++g)
    if (row_ptr[g + 1] < row_ptr[g]) return false;
  const int32_t nnz = row_ptr[G];
  for (int32_t j = 0; j < nnz; ++j)
    if ((uint32_t) members[j] >= (uint32_t) V) return false;
  return true;
}

int pcg_groups_validate_host(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                             const int32_t *mult) {
  if (!row_ptr || !members || !mult) return PCG_ERR_NULL_ARG;
  if (V < 1 || G < 1) return PCG_ERR_BAD_SHAPE;
  if (!csr_well_formed(V, G, row_ptr, members)) return PCG_ERR_BAD_CSR;
  std::vector<int32_t> seen((size_t) V, 0);
  for (int32_t j = 0, n = row_ptr[G]; j < n; ++j) ++seen[members[j]];
  for (int32_t v = 0; v < V; ++v)
    if (seen[v] == 0 || seen[v] != mult[v]) return PCG_ERR_BAD_CSR;
  return PCG_OK;
}

int pcg_groups_canonicalize_host(int32_t V, int32_t G, const int32_t *row_ptr,
                                 const int32_t *members, int32_t *out_G, int64_t *out_nnz,
                                 int32_t *out_row_ptr, int32_t *out_members, int32_t *out_mult) {
  if (!row_ptr || !out_G || !out_nnz) return PCG_ERR_NULL_ARG;
  if (V < 1 || G < 0) return PCG_ERR_BAD_SHAPE;
  if (G > 0 && row_ptr[G] > 0 && !members) return PCG_ERR_NULL_ARG;
  if (!csr_well_formed(V, G, row_ptr, members)) return PCG_ERR_BAD_CSR;
  const int32_t nnz = row_ptr[G];
  std::vector<int32_t> seen((size_t) V, 0);
  for (int32_t j = 0; j < nnz; ++j) ++seen[members[j]];
  int32_t lonely = 0;
  for (int32_t v = 0; v < V; ++v) lonely += seen[v] == 0;
  *out_G = G + lonely;
  *out_nnz = (int64_t) nnz + lonely;
  if (!out_row_ptr) return PCG_OK;
  if (!out_members || !out_mult) return PCG_ERR_NULL_ARG;
  std::memcpy(out_row_ptr, row_ptr, sizeof(int32_t) * ((size_t) G + 1));
  if (nnz) std::memcpy(out_members, members, sizeof(int32_t) * (size_t) nnz);
  int32_t next_group = G, next_entry = nnz;
  for (int32_t v = 0; v < V; ++v) {
    out_mult[v] = seen[v] ? seen[v] : 1;
    if (!seen[v]) {
      out_members[next_entry++] = v;
      out_row_ptr[++next_group] = next_entry;
    }
  }
  return PCG_OK;
}

int pcg_groups_reverse_host(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                            int32_t *tok_ptr, int32_t *tok_groups) {
  if (!row_ptr || !members || !tok_ptr || !tok_groups) return PCG_ERR_NULL_ARG;
  if (V < 1 || G < 1) return PCG_ERR_BAD_SHAPE;
  if (!csr_well_formed(V, G, row_ptr, members)) return PCG_ERR_BAD_CSR;
  const int32_t nnz = row_ptr[G];
  std::fill(tok_ptr, tok_ptr + V + 1, 0);
  for (int32_t j = 0; j < nnz; ++j) ++tok_ptr[members[j] + 1];
  for (int32_t v = 0; v < V; ++v) tok_ptr[v + 1] += tok_ptr[v];
  std::vector<int32_t> cursor(tok_ptr, tok_ptr + V);
  for (int32_t g = 0; g < G; ++g)               // ascending entry position within a token's list
    for (int32_t j = row_ptr[g]; j < row_ptr[g + 1]; ++j) tok_groups[cursor[members[j]]++] = g;
  return PCG_OK;
}

int pcg_groups_validate_weights_host(int32_t V, int32_t G, const int32_t *row_ptr,
                                     const int32_t *members, const float *weights, double tol) {
  if (!row_ptr || !members || !weights) return PCG_ERR_NULL_ARG;
  if (V < 1 || G < 1 || !(tol >= 0.0)) return PCG_ERR_BAD_SHAPE;
  if (!csr_well_formed(V, G, row_ptr, members)) return PCG_ERR_BAD_CSR;
  std::vector<double> total((size_t) V, 0.0);
  for (int32_t j = 0; j < row_ptr[G]; ++j) {
    const double w = (double) weights[j];
    if (!(w >= 0.0 && w <= 1.0 + tol)) return PCG_ERR_BAD_CSR;   // also catches NaN
    total[members[j]] += w;
  }
  for (int32_t v = 0; v < V; ++v)
    if (!(std::fabs(total[v] - 1.0) <= tol)) return PCG_ERR_BAD_CSR;
  return PCG_OK;
}

int pcg_groups_reverse_weights_host(int32_t V, int32_t G, const int32_t *row_ptr,
                                    const int32_t *members, const float *weights,
                                    float *tok_weights) {
  if (!row_ptr || !members || !weights || !tok_weights) return PCG_ERR_NULL_ARG;
  if (V < 1 || G < 1) return PCG_ERR_BAD_SHAPE;
  if (!csr_well_formed(V, G, row_ptr, members)) return PCG_ERR_BAD_CSR;
  std::vector<int32_t> cursor((size_t) V + 1, 0);
  for (int32_t j = 0; j < row_ptr[G]; ++j) ++cursor[members[j] + 1];
  for (int32_t v = 0; v < V; ++v) cursor[v + 1] += cursor[v];
  for (int32_t j = 0; j < row_ptr[G]; ++j) tok_weights[cursor[members[j]]++] = weights[j];
  return PCG_OK;
}

// ---- errors ----------------------------------------------------------------------------------

const char *pcg_strerror(int status) {
  switch (status) {
    case PCG_OK: return "ok";
    case PCG_ERR_NULL_ARG: return "a required pointer is NULL";
    case PCG_ERR_BAD_SHAPE: return "a size argument is out of range";
    case PCG_ERR_BAD_DTYPE: return "unknown logits dtype";
    case PCG_ERR_BAD_STRIDE: return "a stride is smaller than V (and not an allowed 0)";
    case PCG_ERR_BAD_TEMPERATURE: return "temperature must be finite and > 0";
    case PCG_ERR_WORKSPACE_TOO_SMALL: return "workspace is smaller than *_workspace_bytes";
    case PCG_ERR_BAD_CSR: return "group membership is not a valid CSR with matching multiplicities";
    case PCG_ERR_HIP: return "a HIP runtime call failed (see pcg_last_hip_error)";
    case PCG_ERR_MISALIGNED: return "a pointer is not aligned as required";
    case PCG_ERR_CAPACITY: return "a similarity group or the member array needs more room";
    case PCG_ERR_SCRATCH_TOO_SMALL:
      return "the step needs more scratch memory than the library's own array holds (use pcg_verify)";
    default: return "unknown status";
  }
}

int pcg_last_hip_error(void) { return g_last_hip_error; }

const char *pcg_version(void) { return "libpcg 0.1 (gfx950)"; }

}  // extern "C"
