// Launchers of the libpcg kernels (defined in pcg_kernels.hip).  Every launcher only enqueues
// on `stream`; shapes have been checked by the C ABI layer before it is called.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pcg.h"
#include "pcg_device.h"

namespace pcg {

int32_t stats_nparts(int32_t V);

// streaming: read the logits with nontemporal loads (faster pass, nothing left in the caches)
// probes: also form the probe of every target row that has a proposal (NULL: none)
hipError_t launch_row_stats(const RowSet &rs, bool bf16, int32_t V, int64_t nrows, float c,
                            bool streaming, StatPart *parts, hipStream_t stream,
                            const ProbeArgs *probes = nullptr);

int32_t accept_nsplit(int32_t V, int32_t B);

hipError_t launch_accept_delta(const AcceptArgs &a, bool bf16, int32_t B, float c_lo, float *table,
                               hipStream_t stream);

hipError_t launch_accept_thin(const AcceptArgs &a, bool bf16, int32_t B, const int32_t *tok_ptr,
                              const int32_t *tok_groups, const float *tok_weights, int32_t *trials,
                              int32_t max_trials, hipStream_t stream);
int32_t thin_max_parts();

hipError_t launch_propose(const RowSet &rs, bool bf16, int32_t V, int32_t K, int32_t pos0, float c,
                          const StatPart *parts, const int32_t *tok_ptr, const int32_t *tok_groups,
                          const float *tok_weights, uint64_t seed, uint64_t offset,
                          int32_t *prop_tokens, int32_t *prop_groups, pcg_diag *diag,
                          hipStream_t stream);

hipError_t launch_weights(const RowSet &rs, bool bf16, const pcg_groups &g, int64_t row0,
                          int32_t nrows, float c, float c_hi, float c_lo, const StatPart *parts,
                          float *table, hipStream_t stream);

hipError_t launch_gather(const pcg_groups &g, int32_t nrows, bool clamp, const float *table,
                         float *out, hipStream_t stream);

hipError_t launch_gather_prepared(const pcg_groups &g, int32_t nrows, const float *table, float *out,
                                  double *csum, double *runs, hipStream_t stream);

hipError_t launch_finalize(const FinalizeArgs &fa, bool bf16, const pcg_groups &g, int32_t B,
                           const double *csum, const double *runs, int32_t nchunks,
                           int32_t chunk_groups, hipStream_t stream);

// Remembers a HIP error for pcg_last_hip_error and returns PCG_ERR_HIP.
int record_hip_error(hipError_t e);

}  // namespace pcg
