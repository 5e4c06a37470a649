/*
 * pcg.h -- C ABI of libpcg: group-level verification for speculative decoding
 * over acoustic tokens ("Principled Coarse-Graining", arXiv 2511.13732) on one
 * AMD MI355X (gfx950).
 *
 * One call to pcg_verify is one speculative step for B sequences
 * (Algorithm 1): softmax of target and draft logits over the vocabulary, the
 * overlap-aware group probabilities of Eq. (5) with equal-split weights
 * (Eq. 3), the group accept test of Eq. (7) on each proposed group until the
 * first rejection, then a group drawn from the normalised residual of Eq. (8)
 * and a token inside it by Eq. (10); when every proposal is accepted the extra
 * ("bonus") position is drawn from the target's last row instead.
 *
 * Naming.  The paper's body writes q for the target model and p for the
 * draft, Q_c / P_c for their group distributions.  This header uses
 *     T[g] = target group probability,   D[g] = draft group probability,
 * so the accept ratio is T/D and the residual is max(0, T - D).
 *
 * Conventions that hold for every entry point unless stated otherwise:
 *   - pointers marked DEVICE point to memory of the current HIP device, are
 *     owned by the caller and must stay valid until the stream has run the
 *     call; pointers marked HOST are ordinary host memory;
 *   - the compute calls allocate no device memory: scratch comes in through
 *     `workspace` (DEVICE, 256-byte aligned, size from the *_workspace_bytes
 *     helpers; its contents need not be initialised and mean nothing after
 *     the call) and may be reused by the next call on the same stream; calls
 *     that may run at the same time need workspaces of their own
 *     (pcg_verify_static, which uses an array of the library, is the one
 *     exception: see there);
 *   - calls only enqueue work on `hip_stream` (a hipStream_t, NULL = default
 *     stream) and return without synchronising (pcg_asg_build and
 *     pcg_profile_end wait: see there);
 *   - the return value is PCG_OK (0) or a negative pcg_status; nothing is
 *     thrown across the boundary;
 *   - arguments are checked on the host before anything is launched, so a
 *     call that returns an argument error (every status but the two below)
 *     has enqueued nothing.  Two statuses can come after some kernels of the
 *     call were enqueued already: PCG_ERR_HIP (a launch failed midway; the
 *     outputs are then undefined) and PCG_ERR_CAPACITY of pcg_asg_build
 *     (reported after its kernels ran);
 *   - state the library keeps between calls, all of it on the host except
 *     the array of pcg_verify_static: the last hipError_t per thread
 *     (pcg_last_hip_error), and, between pcg_profile_begin and
 *     pcg_profile_end only, the HIP events of the recorded calls (created and
 *     destroyed by those two functions, not thread-safe, and never recorded
 *     into a stream that is being captured).  Nothing else: no caches, no
 *     device allocations, no streams of its own.
 */
#ifndef PCG_H
#define PCG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { PCG_F32 = 0, PCG_BF16 = 1 } pcg_dtype;

typedef enum {
  PCG_OK = 0,
  PCG_ERR_NULL_ARG = -1,
  PCG_ERR_BAD_SHAPE = -2,          /* V, G, nnz, B, K, rows out of range                    */
  PCG_ERR_BAD_DTYPE = -3,
  PCG_ERR_BAD_STRIDE = -4,         /* a stride smaller than V (other than 0) or negative    */
  PCG_ERR_BAD_TEMPERATURE = -5,    /* not a finite number > 0                               */
  PCG_ERR_WORKSPACE_TOO_SMALL = -6,
  PCG_ERR_BAD_CSR = -7,            /* host validation of the group membership failed        */
  PCG_ERR_HIP = -8,                /* a HIP runtime call failed                             */
  PCG_ERR_MISALIGNED = -9,         /* workspace not 256-byte aligned, logits not element-aligned */
  PCG_ERR_CAPACITY = -10,          /* pcg_asg_build: a group or the member array did not fit      */
  PCG_ERR_SCRATCH_TOO_SMALL = -11  /* pcg_verify_static: the step needs more than PCG_STATIC_SCRATCH_BYTES */
} pcg_status;

#define PCG_MAX_K 64               /* largest number of draft positions per step           */

/*
 * Group membership (Sec. 2.1, 2.2): the distinct Acoustic Similarity Groups as
 * CSR group -> tokens, plus the per-token multiplicity N(t) of Eq. (3).
 * All three arrays are DEVICE, read-only.  The structure itself is HOST.
 *   row_ptr [G+1]  row_ptr[0] = 0, non-decreasing, row_ptr[G] = nnz
 *   members [nnz]  token ids in [0, V); members of group g are
 *                  members[row_ptr[g] .. row_ptr[g+1])
 *   mult    [V]    mult[v] = number of CSR entries equal to v, >= 1 for all v
 * A token listed twice in one group carries weight 2/mult there.  The arrays
 * must describe a membership that pcg_groups_validate_host accepts; the
 * kernels do not re-check them.
 */
typedef struct pcg_prepared pcg_prepared;

typedef struct {
  int32_t V;
  int32_t G;
  int64_t nnz;
  const int32_t *row_ptr;
  const int32_t *members;
  const int32_t *mult;
  /* Optional fast form of the same membership (see pcg_groups_prepare_host): the blob
   * uploaded to the DEVICE and its HOST descriptor.  Both NULL = use the CSR directly, which
   * gives the same results but re-reads the 4-byte member ids from L2 for every row: at
   * V = G = 65 536 with 32-member groups and 64 sequences a step takes about 0.5 ms from the
   * CSR against about 0.07 ms from the prepared form. */
  const void *prepared;
  const pcg_prepared *prepared_info;
  /* Optional reverse index token -> groups (the paper's S(t); see pcg_groups_reverse_host),
   * DEVICE: tok_ptr [V+1], tok_groups [nnz].  Needed by pcg_verify_thinning and pcg_propose. */
  const int32_t *tok_ptr;
  const int32_t *tok_groups;
  /* Optional general weights w_{k,t} (Sec. 2.2, Eq. 2), DEVICE float [nnz]: weights[j] is the
   * share of token members[j] that group k (the row holding entry j) receives; non-negative,
   * and the weights of one token sum to 1 (see pcg_groups_validate_weights_host).  NULL = the
   * equal split 1 / mult[t] (Eq. 3).  With weights the group probabilities are
   * sum_j prob(members[j]) * weights[j] (Eq. 4), the token inside a group is drawn
   * proportionally to prob(t) * w_{k,t} (Eq. 10) and a token's group label by its weights
   * (Eq. 6).  With weights, `prepared` is either NULL (the CSR is read directly) or a blob that
   * pcg_groups_prepare_weights_host built from these same weights (off_weights != 0).
   * tok_weights: the same weights in reverse-index order (pcg_groups_reverse_weights_host),
   * DEVICE float [nnz]; needed together with weights by pcg_verify_thinning and pcg_propose. */
  const float *weights;
  const float *tok_weights;
} pcg_groups;

/*
 * Prepared membership.  The groups are fixed once the similarity groups have been built
 * (Sec. 2.2 "Complexity and memory": they are built ahead of time and kept), so the gather-sum of Eq. (5) can read them
 * from a layout made for the kernel instead of from the CSR:
 *   - the vocabulary is cut into `ntiles` tiles of `tile_len` tokens, each small enough for
 *     a table of one float per token to sit in a workgroup's LDS;
 *   - the groups are cut into chunks of `chunk_groups` consecutive groups (one workgroup
 *     each); inside a chunk they are sorted by their member counts per tile and dealt 256 at
 *     a time into blocks: lane l of a wave handles the 4 groups at sorted positions
 *     block*256 + r*64 + l, r = 0..3;
 *   - per (chunk, tile, block) the members that fall into the tile are stored as 16-bit
 *     tile-local slots, two per dword, each list padded to the block's longest with slots
 *     tile_len + bank (which read as 0); a lane's 4 dwords of step k (one per group) are
 *     adjacent, so a wave reads step k of a block with one coalesced 16-byte-per-lane load;
 *   - the order of a group's slots is free (a sum), and is chosen per half-wave of 32 lanes
 *     so that the 32 LDS addresses of a step fall into different banks wherever possible.
 * The descriptor is filled by pcg_groups_prepare_host and must be passed back unchanged.
 */
struct pcg_prepared {
  int32_t V, G;
  int32_t ntiles, tile_len;
  int32_t chunk_groups, nchunks;
  int32_t blocks_per_chunk, reserved;
  int64_t off_desc;   /* uint32 [nchunks][ntiles][blocks_per_chunk][2]: data offset (16-byte units), steps */
  int64_t off_perm;   /* uint16 [nchunks][blocks_per_chunk][4][64]: group index inside the chunk, 0xFFFF = none */
  int64_t off_data;   /* uint32 [][64][4]: step k of a block = 64 lanes x 4 dwords, 2 slots per dword */
  int64_t off_weights;/* float [][64][4][2]: the weight w_{k,t} of every slot of off_data, same unit
                         numbering, low slot first; 0 on padding slots.  0 = the blob holds none */
  int64_t bytes;      /* size of the blob */
};

/*
 * Optional counters a call adds to (DEVICE, caller zeroes them; may be NULL).
 * "near" means the uniform draw fell within 1e-6 (on the unit interval) of a
 * threshold that separates two outcomes, as judged in the kernel's own
 * arithmetic.
 */
typedef struct {
  uint32_t near_accept;        /* accept tests with |u*D - T| < 1e-6 * D                    */
  uint32_t near_group;         /* residual group draws near an inner bin edge               */
  uint32_t near_token;         /* in-group token draws near an inner bin edge               */
  uint32_t zero_draft_mass;    /* evaluated proposals with D[g] == 0                        */
  uint32_t residual_fallback;  /* rejected rows whose residual total was <= 0 (drawn from T)*/
  uint32_t bad_proposal;       /* proposed group id outside [0, G): treated as rejected     */
  uint32_t accepted_total;     /* sum of accept_len over the batch                          */
  uint32_t sequences;          /* number of sequences processed                             */
} pcg_diag;

/* ---- group probabilities: Eq. (5) ------------------------------------------------------- */

/*
 * out[r*G + g] = sum over members t of group g of softmax(logits[r,:]/temperature)[t] / mult[t]
 * for r in [0, rows).  No renormalisation is applied (Eq. 2 makes each row sum to 1).
 *   logits            DEVICE [rows, V], element type `dt`, V-axis contiguous,
 *                     row r starts at element r*row_stride (row_stride >= V)
 *   out               DEVICE [rows, G] float32, row-major
 *   workspace         DEVICE, >= pcg_group_probs_workspace_bytes(V, rows)
 * Rows are independent; rows == 0 is a no-op.  Logits must be finite or -inf
 * with at least one finite entry per row, else that row's output is NaN.
 * Accuracy: a group's sum is one float32 running sum over its entries, so next to the 1e-5
 * relative error of the terms themselves it carries up to n 2^-24 of rounding for a group of n
 * entries (measured: within 1e-5 in total for groups of up to a few hundred entries).
 */
int pcg_group_probs(const pcg_groups *groups, const void *logits, pcg_dtype dt, int64_t rows,
                    int64_t row_stride, float temperature, float *out, void *workspace,
                    size_t workspace_bytes, void *hip_stream);

size_t pcg_group_probs_workspace_bytes(int32_t V, int64_t rows);

/* ---- one speculative step: Algorithm 1 with Eq. (5), (7), (8), (10) --------------------- */

/*
 *   target_logits  DEVICE, row (b, i), i in [0, K], starts at element
 *                  b*tgt_batch_stride + i*tgt_pos_stride; V-axis contiguous
 *   draft_logits   DEVICE, row (b, i), i in [0, K), likewise with the dft strides (a
 *                  [B, K+1, V] draft buffer can be passed; its last row is never read)
 *   strides        in elements; each >= V, or 0 for a batch stride (all sequences then
 *                  share the same rows)
 *   prop_tokens    DEVICE int32 [B, K]  the draft's token at each position (only copied out)
 *   prop_groups    DEVICE int32 [B, K]  the group drawn for it by Eq. (6)
 *   seed, offset   Philox4x32-10 key and call counter: position (b, i) uses the block with
 *                  counter (offset_lo, offset_hi, b, i) and key (seed_lo, seed_hi); its
 *                  words 0, 1, 2 give the accept, group and token uniforms as
 *                  (word >> 8) * 2^-24.  A decode loop passes its step index as `offset`.
 *   accept_len     DEVICE int32 [B]     number of accepted proposals, in [0, K]
 *   out_tokens     DEVICE int32 [B, K+1], out_groups likewise: entries [0, accept_len) are
 *                  the accepted (prop_token, prop_group) pairs; entry accept_len is the
 *                  resampled (rejection) or bonus (all accepted) pair; the rest is -1
 *   diag           DEVICE pcg_diag*, may be NULL
 *   workspace      DEVICE, >= pcg_verify_workspace_bytes(V, G, B, K)
 * Accept test (Eq. 7): accept iff u * D[g] < T[g] (so D = 0 < T accepts, T = D = 0
 * rejects).  Inverse-CDF draws take the first index whose running sum strictly exceeds
 * u * total; zero-mass groups and tokens are never chosen.  The accept test never reads
 * prop_tokens, so token-in-group consistency of the proposal is the caller's business.
 * B == 0 is a no-op; 1 <= K <= PCG_MAX_K.
 */
int pcg_verify(const pcg_groups *groups, const void *target_logits, const void *draft_logits,
               pcg_dtype dt, int32_t B, int32_t K, int64_t tgt_batch_stride,
               int64_t tgt_pos_stride, int64_t dft_batch_stride, int64_t dft_pos_stride,
               float temperature, const int32_t *prop_tokens, const int32_t *prop_groups,
               uint64_t seed, uint64_t offset, int32_t *accept_len, int32_t *out_tokens,
               int32_t *out_groups, pcg_diag *diag, void *workspace, size_t workspace_bytes,
               void *hip_stream);

size_t pcg_verify_workspace_bytes(int32_t V, int32_t G, int32_t B, int32_t K);

/* ---- the same step for callers that cannot allocate --------------------------------------- */

#define PCG_STATIC_SCRATCH_BYTES (48u << 20)

/*
 * pcg_verify without a workspace argument, for callers that can neither allocate device memory
 * nor keep a workspace of their own: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as
 * pcg_verify; the scratch memory is an array of PCG_STATIC_SCRATCH_BYTES (48 MiB) that the
 * library itself holds in the memory of every GPU it is loaded on, from load until the process
 * ends.  The call allocates and frees nothing (the first call on a device looks up the
 * array's address there, once).
 *   - a step with pcg_verify_workspace_bytes(V, G, B, K) > PCG_STATIC_SCRATCH_BYTES returns
 *     PCG_ERR_SCRATCH_TOO_SMALL before anything is launched (the headline shape V = G = 65 536,
 *     B = 64, K = 8 needs 37 MB);
 *   - every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (two
 *     streams, two threads) race on it and must be ordered by the caller; nothing in the array
 *     has to survive from one call to the next, and nothing in it is assumed to be zero.
 * pcg_static_scratch_bytes() returns PCG_STATIC_SCRATCH_BYTES.
 */
int pcg_verify_static(const pcg_groups *groups, const void *target_logits,
                      const void *draft_logits, pcg_dtype dt, int32_t B, int32_t K,
                      int64_t tgt_batch_stride, int64_t tgt_pos_stride, int64_t dft_batch_stride,
                      int64_t dft_pos_stride, float temperature, const int32_t *prop_tokens,
                      const int32_t *prop_groups, uint64_t seed, uint64_t offset,
                      int32_t *accept_len, int32_t *out_tokens, int32_t *out_groups,
                      pcg_diag *diag, void *hip_stream);

size_t pcg_static_scratch_bytes(void);

/* ---- the same step with the reject branch drawn by thinning ------------------------------ */

#define PCG_THIN_MAX_TRIALS 65520

/*
 * pcg_verify with the group residual of Eq. (8) drawn the way the paper itself does it
 * (Sec. 2.2 "Residual sampling via thinning", Eq. 9) instead of by enumerating the groups:
 * trial j = 0, 1, ... draws a token y from the target row, one of the mult[y] membership
 * entries of y (hence a group g with probability T[g]), and accepts g with probability
 * [1 - D[g]/T[g]]_+; the first accepted trial emits g and a token inside it by Eq. (10).
 * Same distribution as pcg_verify, a different sample path: the accept scan and its draws are
 * identical, the emitted (token, group) on a rejection is not.  When every proposal is
 * accepted the bonus token is drawn from the target's last row and its group by the weights
 * (Algorithm 1, last step; Eq. 6).
 *   groups        must carry tok_ptr / tok_groups; the prepared form is not used
 *   draws         trial j of position (b, i) uses the Philox block with counter
 *                 (offset_lo, offset_hi, b, i | (j + 1) << 16): word 0 -> token uniform,
 *                 word 1 >> 8 = k24 -> membership entry (k24 * mult[y]) >> 24 (with general
 *                 weights: the inverse CDF of y's tok_weights at k24 / 2^24), word 2 -> accept
 *                 uniform, word 3 -> token-in-group uniform; the bonus position uses trial 0
 *   trials        DEVICE int32 [B]: trials run for the sequence (0 on the bonus position)
 *   diag          near_group counts token / accept draws within 1e-6 of their threshold on the
 *                 emitted path, near_token the token-in-group draw, residual_fallback sequences
 *                 that hit PCG_THIN_MAX_TRIALS (the last candidate is emitted then)
 *   workspace     >= pcg_verify_thinning_workspace_bytes(V, B, K)
 * Other arguments, conventions and limits as for pcg_verify; V must not exceed 4 194 304.
 */
int pcg_verify_thinning(const pcg_groups *groups, const void *target_logits,
                        const void *draft_logits, pcg_dtype dt, int32_t B, int32_t K,
                        int64_t tgt_batch_stride, int64_t tgt_pos_stride, int64_t dft_batch_stride,
                        int64_t dft_pos_stride, float temperature, const int32_t *prop_tokens,
                        const int32_t *prop_groups, uint64_t seed, uint64_t offset,
                        int32_t *accept_len, int32_t *out_tokens, int32_t *out_groups,
                        int32_t *trials, pcg_diag *diag, void *workspace, size_t workspace_bytes,
                        void *hip_stream);

size_t pcg_verify_thinning_workspace_bytes(int32_t V, int32_t B, int32_t K);

/* ---- draft-side proposals ---------------------------------------------------------------- */

/*
 * The two sampling steps at the top of Algorithm 1's loop (Sec. 2.2 "Proposal coupling and
 * acceptance", Eq. 6): for every (b, i) a draft token x ~ softmax(draft row / temperature) by
 * inverse CDF over ascending token ids (first token whose running sum strictly exceeds
 * u * total), then a group label among the groups holding x by the equal-split weights: one
 * of the mult[x] membership entries of x, each equally likely, so that the label is distributed
 * as the draft's group distribution D_i.
 *   groups        must carry tok_ptr / tok_groups; row_ptr / members are not read
 *   draft_logits  DEVICE [B, K, V], V contiguous; strides in elements as for pcg_verify
 *   pos0          position index of row 0 (a draft that samples one token per forward pass
 *                 calls with K = 1 and pos0 = 0, 1, ...); pos0 + K <= PCG_MAX_K
 *   draws         position (b, i) uses the Philox block with counter
 *                 (offset_lo, offset_hi, b, (pos0 + i) | 0xFFFF0000), a block neither
 *                 pcg_verify nor any thinning trial reads: word 0 -> token uniform,
 *                 word 1 >> 8 = k24 -> membership entry (k24 * mult[x]) >> 24 (with general
 *                 weights: the inverse CDF of x's tok_weights at k24 / 2^24)
 *   prop_tokens, prop_groups   DEVICE int32 [B, K], written
 *   diag          optional DEVICE counters: near_token counts token draws within 1e-6 of an
 *                 inner bin edge, sequences the rows processed
 *   workspace     DEVICE, 256-byte aligned, >= pcg_propose_workspace_bytes(V, B, K)
 * A row without any finite logit yields token 0 (the statistics kernel reports nothing: such
 * rows are the caller's error, as for pcg_verify).  V must not exceed 4 194 304.
 */
int pcg_propose(const pcg_groups *groups, const void *draft_logits, pcg_dtype dt, int32_t B,
                int32_t K, int32_t pos0, int64_t dft_batch_stride, int64_t dft_pos_stride,
                float temperature, uint64_t seed, uint64_t offset, int32_t *prop_tokens,
                int32_t *prop_groups, pcg_diag *diag, void *workspace, size_t workspace_bytes,
                void *hip_stream);

size_t pcg_propose_workspace_bytes(int32_t V, int32_t B, int32_t K);

/* ---- construction of the similarity groups ----------------------------------------------- */

/*
 * unit_bf16[v][k] = emb[v][k] / ||emb[v]|| (Sec. 2.1: the cosine of Eq. 1 is the dot product of
 * unit vectors), computed in double and rounded once to bfloat16, nearest with ties to even; a
 * zero row stays zero.  emb DEVICE float [V, d], unit_bf16 DEVICE uint16 [V, d].  Asynchronous
 * on hip_stream.
 */
int pcg_asg_normalize(const float *emb, int32_t V, int32_t d, uint16_t *unit_bf16,
                      void *hip_stream);

#define PCG_ASG_MAX_CAP 4096

/*
 * The Acoustic Similarity Groups of Eq. (1): G(t) = every token v whose unit vector has a dot
 * product with t's above theta (fp32 accumulation of the exact bf16 products), and t itself;
 * the distinct sets, each once, in order of first appearance (ascending t), as the CSR that
 * pcg_groups reads: members ascending inside a group, mult = entry counts.
 *   unit_bf16     DEVICE uint16 [V, d], 16-byte aligned, d a multiple of 64, V * d < 2^31
 *   theta         strict threshold of Eq. (1); values below -1 put everything in one group
 *   cap           room for one group while it is collected, 1 .. PCG_ASG_MAX_CAP
 *   row_ptr       DEVICE int32 [V + 1]: the first *out_G + 1 entries are written
 *   members       DEVICE int32 [members_capacity]
 *   mult          DEVICE int32 [V]
 *   seed_of       DEVICE int32 [V] or NULL: the token whose group each kept row is
 *   out_G, out_nnz, out_max_size   HOST: groups kept, their total size, the largest G(t) found
 *   workspace     DEVICE, 256-byte aligned, >= pcg_asg_build_workspace_bytes(V, cap)
 * Unlike the verification calls this one WAITS for hip_stream: the sizes are returned to the
 * host.  PCG_ERR_CAPACITY if some G(t) has more than cap members or the groups more than
 * members_capacity entries (the out_* sizes are valid then, nothing else is: call again with
 * more room).
 */
int pcg_asg_build(const uint16_t *unit_bf16, int32_t V, int32_t d, float theta, int32_t cap,
                  int32_t *row_ptr, int32_t *members, int64_t members_capacity, int32_t *mult,
                  int32_t *seed_of, int32_t *out_G, int64_t *out_nnz, int32_t *out_max_size,
                  void *workspace, size_t workspace_bytes, void *hip_stream);

size_t pcg_asg_build_workspace_bytes(int32_t V, int32_t cap);

/*
 * The same groups by Eq. (1) exactly as written: G(t) = every v with cos(emb[t], emb[v]) > theta,
 * the cosine of the float32 embeddings themselves in double (dot product and both norms, one
 * division), and t itself.  The bf16 contraction of pcg_asg_build serves as a filter: a pair
 * whose rounded similarity lies within 2^-8 + 2^-18 + d 2^-23 of theta (how far rounding the
 * unit vectors to bfloat16 and summing in fp32 can move it) is decided by the double-precision
 * cosine, every other pair by the rounded one.  Outputs, order of the groups, waiting for the
 * stream and PCG_ERR_CAPACITY as for pcg_asg_build, except that cap must hold every candidate
 * of a group (the pairs above theta minus that band) while it is collected; *out_max_size is
 * the largest G(t) after the decision when everything fitted.
 *   emb           DEVICE float [V, d], 16-byte aligned, d a multiple of 64, V * d < 2^31
 *   workspace     DEVICE, 256-byte aligned, >= pcg_asg_build_exact_workspace_bytes(V, d, cap)
 *                 (it also holds the unit vectors, 2 V d bytes)
 * A zero row has cosine 0 with every other row.
 */
int pcg_asg_build_exact(const float *emb, int32_t V, int32_t d, float theta, int32_t cap,
                        int32_t *row_ptr, int32_t *members, int64_t members_capacity,
                        int32_t *mult, int32_t *seed_of, int32_t *out_G, int64_t *out_nnz,
                        int32_t *out_max_size, void *workspace, size_t workspace_bytes,
                        void *hip_stream);

size_t pcg_asg_build_exact_workspace_bytes(int32_t V, int32_t d, int32_t cap);

/* ---- group membership on the host -------------------------------------------------------- */

/* Every helper below takes the membership as (row_ptr [G + 1], members [row_ptr[G]]): the number of
 * entries is read from row_ptr[G], so the members array (and every per-entry array: weights) must
 * really hold that many -- a C function cannot see an array's length, and a row_ptr[G] beyond it
 * makes the helper read past the end.  Everything else about the arrays is checked and refused
 * with PCG_ERR_BAD_CSR: row_ptr[0] != 0, a decreasing row_ptr, a member outside [0, V). */

/* PCG_OK iff (row_ptr, members, mult), all HOST, form a membership the kernels may use (see
 * pcg_groups above); PCG_ERR_BAD_CSR otherwise. */
int pcg_groups_validate_host(int32_t V, int32_t G, const int32_t *row_ptr,
                             const int32_t *members, const int32_t *mult);

/*
 * Make any CSR usable: a token that is in no group becomes its own singleton group
 * (Eq. 1 puts every token in its own similarity group, so this is what the paper's
 * construction implies).  Singletons are appended after the G given groups in
 * ascending token order; mult is filled with the entry counts.  All pointers HOST.
 * Call with out_row_ptr == NULL to obtain *out_G and *out_nnz, then again with
 * out_row_ptr [*out_G + 1], out_members [*out_nnz], out_mult [V].
 */
int pcg_groups_canonicalize_host(int32_t V, int32_t G, const int32_t *row_ptr,
                                 const int32_t *members, int32_t *out_G, int64_t *out_nnz,
                                 int32_t *out_row_ptr, int32_t *out_members, int32_t *out_mult);

/* PCG_OK iff weights (HOST, [nnz]) are usable for the membership: every weight finite and in
 * [0, 1 + tol], and the weights of each token's entries sum to 1 within tol (Eq. 2);
 * PCG_ERR_BAD_CSR otherwise. */
int pcg_groups_validate_weights_host(int32_t V, int32_t G, const int32_t *row_ptr,
                                     const int32_t *members, const float *weights, double tol);

/* tok_weights [nnz] (HOST): weights permuted into the order of pcg_groups_reverse_host, so that
 * tok_weights[tok_ptr[v] + e] is the weight of the e-th membership entry of token v. */
int pcg_groups_reverse_weights_host(int32_t V, int32_t G, const int32_t *row_ptr,
                                    const int32_t *members, const float *weights,
                                    float *tok_weights);

/* Reverse index of a membership (all pointers HOST): tok_ptr [V+1], tok_groups [nnz]; the
 * groups of a token are listed by ascending CSR entry position (a group that lists the token
 * twice appears twice), so tok_ptr[v+1] - tok_ptr[v] == mult[v]. */
int pcg_groups_reverse_host(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                            int32_t *tok_ptr, int32_t *tok_groups);

/*
 * Build the prepared form of a validated membership (all pointers HOST).  chunk_groups is the
 * number of consecutive groups one workgroup handles: a multiple of 4096 in [4096, 16384], or
 * 0 for the default (16384).  Smaller chunks spread a small batch over more compute units.
 * pcg_groups_prepare_bytes returns the blob size (0 on bad arguments); pcg_groups_prepare_host
 * fills `blob` (blob_bytes >= that size) and `info`.  The caller uploads the blob to the
 * device (256-byte aligned) and points pcg_groups.prepared / prepared_info at it.
 */
size_t pcg_groups_prepare_bytes(int32_t V, int32_t G, const int32_t *row_ptr,
                                const int32_t *members, int32_t chunk_groups);
int pcg_groups_prepare_host(int32_t V, int32_t G, const int32_t *row_ptr, const int32_t *members,
                            int32_t chunk_groups, void *blob, size_t blob_bytes,
                            pcg_prepared *info);

/*
 * The same with general weights (Sec. 2.2, Eq. 2 and 4): weights[j] (HOST float [nnz], as in
 * pcg_groups.weights) travels with entry j into the blob, so that the prepared gather forms
 * sum_j table(members[j]) * weights[j] without touching the CSR.  The blob is the unweighted
 * one followed by the weights (three times the slot data).  The caller passes the same weights
 * on the device in pcg_groups.weights; nothing checks that the two agree.
 */
size_t pcg_groups_prepare_weights_bytes(int32_t V, int32_t G, const int32_t *row_ptr,
                                        const int32_t *members, int32_t chunk_groups);
int pcg_groups_prepare_weights_host(int32_t V, int32_t G, const int32_t *row_ptr,
                                    const int32_t *members, const float *weights,
                                    int32_t chunk_groups, void *blob, size_t blob_bytes,
                                    pcg_prepared *info);

/* ---- per-kernel timing (for the benchmark) ------------------------------------------------ */

#define PCG_MAX_STAGES 8
/*
 * Between pcg_profile_begin and pcg_profile_end every pcg_verify / pcg_group_probs call
 * brackets each of its kernels with HIP events on the call's stream (this costs time; leave
 * it off otherwise).  pcg_profile_end synchronises those events and writes, for each stage,
 * the mean duration in milliseconds over the recorded calls (HOST float [PCG_MAX_STAGES],
 * unused entries 0), the number of calls (HOST) and returns PCG_OK.  At most `max_calls`
 * calls are recorded; later ones run unrecorded.  Stage names: pcg_stage_name(i).  The stage
 * "event_overhead" is an empty event pair recorded at the start of each call: the time an
 * event pair adds, which is included in every other stage's figure.
 * Not thread-safe; one profile at a time.
 */
int pcg_profile_begin(int32_t max_calls);
int pcg_profile_end(float *stage_ms, int32_t *calls);
const char *pcg_stage_name(int32_t stage);

/* ---- errors -------------------------------------------------------------------------------- */

const char *pcg_strerror(int status);
int pcg_last_hip_error(void);
const char *pcg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PCG_H */
