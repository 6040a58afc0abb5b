/*
 * lessdec: per-decode-step attention over an H2O-evicted, slotted KV cache combined with the
 * constant-size low-rank state (H, z) of LESS, for AMD MI355X (gfx950).
 *
 * One "unit" is one (batch row, head) pair, u = b * heads + h.  Units are independent.
 * C = n_heavy + n_recent is the slot capacity of a unit's sparse cache, D the head
 * dimension, R the feature-map rank, R' the feature-map hidden width.
 *
 * Ownership and conventions
 *  - Every pointer in the descriptor and in the call arguments is a DEVICE pointer owned
 *    by the caller (the descriptor itself is a host struct).  The library allocates
 *    nothing, keeps no state between calls and never synchronises: all work is enqueued
 *    on the given HIP stream (`hip_stream` is a hipStream_t; NULL = the default stream).
 *  - All state of the method lives in the descriptor's buffers (k_cache .. pend_psi), so a
 *    checkpoint is a copy of them.  Calls on one descriptor must be stream-ordered; calls on different
 *    descriptors (different buffers) are independent.
 *  - Entry points return 0 on success and a negative LESSDEC_E* code otherwise.  Argument
 *    errors are detected on the host before anything is launched.  No C++ exception
 *    crosses this boundary.
 *  - The per-unit counter n_seen is read and advanced on the device and no call clears
 *    memory with a memset, so a sequence of steps can be recorded into a HIP graph.
 *  - State buffers that were never reset (Algorithm 1's "load" step on arbitrary memory): the
 *    result of a step is then meaningless, but every access stays inside the unit's own arrays.
 *    The kernels read n_seen < 0 as 0, never use more than C slots whatever n_seen says, and
 *    decode any pend_slot word to "nothing pending" or a slot in [0, C]; positions and scores
 *    are only compared, never used as addresses.
 *
 * Arithmetic: everything that decides an eviction (scores, exponentials, the
 * denominator, accumulated probabilities, z, prompt column sums) is computed in fp64;
 * value-side sums (numerator, H, outputs) in fp32; the feature-map MLPs in fp32 with
 * fp16 matrix-core products when dtype is fp16.
 */
#ifndef LESSDEC_H
#define LESSDEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LESSDEC_DTYPE_F32 0 /* q/k/v, cache, weights and out are float   */
#define LESSDEC_DTYPE_F16 1 /* q/k/v, cache, weights and out are IEEE half */

/* flags */
#define LESSDEC_FLAG_SPARSE_DENOM 1u /* H2O accumulates e^s over the sparse-only denominator
                                        instead of the full denominator of Eq. 3            */
#define LESSDEC_FLAG_LAMBDA 2u       /* sparse policy: Lambda-masking instead of H2O (Sec. 4,
                                        "Setup"): the cache keeps the first n_heavy tokens of
                                        the sequence (4 in the paper) and the n_recent most
                                        recent ones, so the oldest token that is not one of
                                        the first leaves.  Scores are still accumulated in
                                        acc but decide nothing                              */

#define LESSDEC_FLAG_PROMPT_STEPWISE 4u /* lessdec_prefill runs the sparse policy from the first
                                        prompt token (the evaluation setting of Sec. 4.1, where
                                        the policy masks query-key pairs throughout the sequence)
                                        instead of pruning once at the end of the prompt     */

#define LESSDEC_OK 0
#define LESSDEC_EINVAL (-1)    /* bad shape, NULL or misaligned pointer, unsupported size */
#define LESSDEC_EWORKSPACE (-2)/* workspace missing or too small                          */
#define LESSDEC_EHIP (-3)      /* a HIP launch or query failed                            */
#define LESSDEC_ESCRATCH (-4)  /* lessdec_step_static: the shape needs more scratch than the
                                  library's built-in LESSDEC_STATIC_SCRATCH_BYTES            */

#define LESSDEC_MAX_RANK 64
#define LESSDEC_MAX_CAPACITY 4094
#define LESSDEC_MAX_HIDDEN 2048
#define LESSDEC_MAX_Q_PER_KV 128
#define LESSDEC_STATIC_SCRATCH_BYTES (4u << 20) /* built-in scratch of lessdec_step_static, per GPU */

typedef struct lessdec_desc {
  int32_t batch, heads, head_dim; /* B, Hh, D; D is 64 or 128                              */
  int32_t n_heavy, n_recent;      /* heavy-hitter and recent slots (Sec. 4: H2O splits its
                                     budget between the two); 1 <= C <= LESSDEC_MAX_CAPACITY */
  int32_t rank, hidden;           /* R <= 64, R' <= 2048 (Eq. 1, Eq. 2)                    */
  int32_t dtype;                  /* LESSDEC_DTYPE_*                                       */
  uint32_t flags;                 /* LESSDEC_FLAG_*                                        */
  int32_t q_per_kv;               /* G: query heads per key/value head (multi-query and
                                     grouped-query attention; Sec. 3.2 extends H2O to the
                                     scores of all query heads).  0 or 1: one.  With G > 1
                                     `heads` counts key/value heads; a unit's G query heads
                                     share its cache and state, each has its own phi, and a
                                     pair's accumulated score grows by its probability under
                                     every one of them.  q, out and Wq1, Wq2 then carry the
                                     extra axis G (see below); C <= 2047                   */
  /* sparse cache K_C, V_C (Sec. 3.1) as slots, replaced in place (Sec. 3.2)               */
  void *k_cache, *v_cache;        /* [B,Hh,C,D] dtype, 16-byte aligned                     */
  double *acc;                    /* [B,Hh,C] accumulated attention probability (H2O)      */
  int32_t *pos;                   /* [B,Hh,C] original token index of the slot, -1 = empty */
  float *psi;                     /* [B,Hh,C,R] psi(k) of the cached key (Eq. 2), kept so
                                     that an eviction needs no MLP evaluation              */
  /* low-rank state (Sec. 2.2, Eq. 4-6)                                                    */
  float *H;                       /* [B,Hh,R,D]                                            */
  double *z;                      /* [B,Hh,R]                                              */
  int32_t *n_seen;                /* [B,Hh] tokens seen so far by each unit                */
  /* write-behind part of the state: lessdec_step leaves the fold of the pair it discarded
     (Eq. 4, Eq. 5) to the head of the next step, where it costs no latency (the psi of the
     discarded slot is only addressable once the eviction is known).  Until then the pair is
     parked here; lessdec_state_sync folds it on request.                                  */
  int32_t *pend_slot;             /* [B,Hh] -1: nothing pending                            */
  void *pend_v;                   /* [B,Hh,D] dtype, value row of the pending pair         */
  float *pend_psi;                /* [B,Hh,R] psi of the last step's key, which is written
                                     into its slot together with the pending fold          */
  /* feature-map weights, per head (Eq. 1, Eq. 2), dtype, stored output-major like a linear
     layer's weight: row i of W?1 holds the D input weights of hidden unit i, i.e. each
     array is the transpose of the matrix of the same name in the equations.  16-byte
     aligned.                                                                              */
  const void *Wq1, *Wq2;          /* phi: [Hh,R',D], [Hh,R,R']; with G > 1 per query head:
                                     [Hh*G,R',D], [Hh*G,R,R'], head h's G in a row          */
  const void *Wk1, *Wk2, *Wk3;    /* psi: [Hh,R',D], [Hh,R,R'], [Hh,R,R]                   */
  void *workspace;                /* >= lessdec_workspace_bytes(), 256-byte aligned.  Scratch,
                                     with one condition: before the first lessdec_step with a
                                     workspace it must either have been handed, in this
                                     descriptor, to lessdec_state_reset or lessdec_prefill, or
                                     be filled with 0xFF bytes (where lessdec_step runs as one
                                     launch, the feature maps reach the attention waves through
                                     an array in it whose unwritten entries must read as empty;
                                     every step leaves it so).  A workspace serves descriptors
                                     of one shape, and calls that share one must be ordered
                                     by a stream                                             */
  size_t workspace_bytes;
} lessdec_desc;

/*
 * Bytes of scratch the calls need.  max_prompt = 0: enough for lessdec_step only;
 * otherwise enough for lessdec_prefill with prompts up to max_prompt tokens as well.
 * Host only.  Returns 0 if the descriptor's shape fields are invalid.
 */
size_t lessdec_workspace_bytes(const lessdec_desc *desc, int32_t max_prompt);

/*
 * Empty state: H_0 = 0, z_0 = 0 (Sec. 2.2), every slot empty (pos = -1, acc = 0, psi = 0),
 * n_seen = 0, nothing pending.  Must be called once before the first step on fresh buffers.
 */
int lessdec_state_reset(const lessdec_desc *desc, void *hip_stream);

/*
 * Folds the pair that the last lessdec_step discarded into H and z (Eq. 4, Eq. 5) and puts
 * the last key's psi into its slot, so that H, z and psi can be read as the state of
 * Algorithm 1 after that step.  Optional: the next lessdec_step does the same fold itself,
 * and its output is the same either way.  Nothing to do after reset or prefill.
 */
int lessdec_state_sync(const lessdec_desc *desc, void *hip_stream);

/*
 * Prompt phase (remark after Eq. 3: with H_0 = z_0 = 0 it is regular attention).
 * Q, K, V: [B,Hh,P,D] dtype, the P prompt tokens of every unit.
 * out:     [B,Hh,P,D] dtype or NULL; causal softmax attention of the prompt.
 * Afterwards each unit's cache holds the n_recent last tokens and the n_heavy tokens with
 * the largest column sums of the causal attention matrix (their H2O scores; ties keep the
 * later token), in ascending token order, with acc = column sum; every other prompt pair
 * is folded into H, z (Eq. 6); n_seen = P.  If P <= C every token is kept.
 * With LESSDEC_FLAG_LAMBDA the first n_heavy tokens are kept in place of the heavy hitters.
 * With q_per_kv = G > 1: Q and out are [B,Hh,G,P,D], and a token's score is the column sum
 * of all G causal attention matrices of its unit.
 * With LESSDEC_FLAG_PROMPT_STEPWISE the call is lessdec_state_reset followed by one
 * lessdec_step per prompt token t with rows Q[.,.,t,.], K[.,.,t,.], V[.,.,t,.] (bit for bit: on
 * the streaming path the steps read and write the rows where they lie in the prompt arrays, one
 * launch per token on large shapes; elsewhere rows are staged and a token takes three launches):
 * out[.,.,t,.] is then Eq. 3's output at token t, and the state afterwards is the state after
 * P steps (a fold may be pending).
 * With LESSDEC_FLAG_LAMBDA as well and P > n_heavy + n_recent the same results (outputs, slot
 * order and state, to rounding) are computed for all prompt tokens at once: under that policy
 * the cache each token meets is known beforehand (Sec. 3.2 builds the same masked matrix for
 * training); nothing is left pending then.
 * Overwrites any previous state of the descriptor (no reset needed before it).
 * P >= 1.  Needs the workspace sized for max_prompt >= P.
 */
int lessdec_prefill(const lessdec_desc *desc, const void *Q, const void *K, const void *V,
                    int32_t P, void *out, void *hip_stream);

/*
 * One generation step (Algorithm 1) for every unit.
 * q, k, v: [B,Hh,D] dtype, this step's query/key/value per unit.
 * out:     [B,Hh,D] dtype, the attention output of Eq. 3 computed with the state from before
 *          this step's eviction.
 * evicted_pos: [B,Hh] or NULL; token index of the pair folded into H, z this step (Eq. 4,
 *          Eq. 5), -1 while the cache is still filling.
 * Per unit: scores the query against the cached keys and k; adds the low-rank terms
 * phi(q) H and phi(q) z^T; adds each pair's probability to its accumulated score (the new
 * pair starts with its own); if the cache is full, discards the pair with the smallest
 * accumulated score among those not within the n_recent most recent tokens (the new one
 * counts as recent; ties discard the older), writes the new pair into its slot and leaves
 * the discarded pair pending (see pend_slot); advances n_seen.  The fold of a pending pair
 * from the previous step into H, z happens first, so Eq. 3 always sees the state Algorithm 1
 * prescribes.  With LESSDEC_FLAG_LAMBDA the discarded pair is instead the oldest one that is
 * neither among the first n_heavy tokens of the sequence nor among the n_recent most recent.
 * With q_per_kv = G > 1: q and out are [B,Hh,G,D] (k, v stay [B,Hh,D]).  Up to 8 query heads
 * with fp16 storage run on a streaming kernel (a block per unit, a wave per query head) that
 * leaves the discarded pair pending like the single-head path; other shapes on a plain kernel
 * that folds the discarded pair at once.
 */
int lessdec_step(const lessdec_desc *desc, const void *q, const void *k, const void *v,
                 void *out, int32_t *evicted_pos, void *hip_stream);

/*
 * The two halves of lessdec_step, for a caller that has q and k before it wants the
 * attention output.  lessdec_step gives exactly the results of the first followed by the
 * second (where lessdec_step_launches gives 1 it runs both in one launch).  Every lessdec_step_features is to be
 * followed by its lessdec_step_attend before the next step on that workspace.
 *  lessdec_step_features: evaluates phi(q) (Eq. 1) and psi(k) (Eq. 2) of the step for every
 *    unit into the workspace.  Touches no state.
 *  lessdec_step_attend: everything else of the step, reading the feature maps that the last
 *    lessdec_step_features on this descriptor left in the workspace; q and k must be the same
 *    arrays.  The workspace must not be used by another call in between.
 */
int lessdec_step_features(const lessdec_desc *desc, const void *q, const void *k, void *hip_stream);
int lessdec_step_attend(const lessdec_desc *desc, const void *q, const void *k, const void *v,
                        void *out, int32_t *evicted_pos, void *hip_stream);

/*
 * Host only: the number of kernel launches one lessdec_step on this descriptor makes (1 where the
 * feature-map jobs run inside the attention launch), 0 if the shape fields are invalid.
 */
int lessdec_step_launches(const lessdec_desc *desc);

/*
 * lessdec_step for callers that cannot bring or allocate scratch memory: code under HIP graph
 * capture, serving loops and harnesses that forbid allocation.  Same arguments, same kernels
 * and bit-identical results; desc->workspace and desc->workspace_bytes are ignored (may be
 * NULL / 0) and the per-step scratch (the feature maps of the step on their way to the
 * attention kernel, the per-block probability sums of the multi-head path) lives in a buffer
 * of LESSDEC_STATIC_SCRATCH_BYTES that is part of the library image on every GPU it runs on.
 * Calls no allocating routine.  A shape whose lessdec_workspace_bytes(desc, 0) exceeds that
 * size is refused with LESSDEC_ESCRATCH before anything is launched (batch 64 x 32 heads at
 * hidden width 512 needs 2.2 MiB).  The first call on a device looks up the buffer's device
 * address (make that call outside a graph capture).  All calls on one GPU share the buffer, in
 * whatever descriptor or stream: calls that overlap in time on one GPU race; calls ordered by
 * a stream do not, and nothing needs clearing between them.
 */
int lessdec_step_static(const lessdec_desc *desc, const void *q, const void *k, const void *v,
                        void *out, int32_t *evicted_pos, void *hip_stream);

/*
 * Measurement aid (Sec. 4.5 times the method; this times the memory it runs on): reads
 * `bytes` of device memory at `buf` (16-byte aligned) once, as `waves` (a multiple of 8)
 * independent contiguous read streams shaped like those of lessdec_step, and discards the data.
 * sink: [waves] device words, left untouched in practice.  Timing it gives the read rate this
 * chip sustains for the access pattern of the decode step, to put beside the published peak.
 */
int lessdec_probe_stream_read(const void *buf, size_t bytes, int32_t waves, uint32_t *sink,
                              void *hip_stream);

/* Static message for a return code. */
const char *lessdec_strerror(int code);

/*
 * Host helper for Table 1: tokens cached at `percent` of `max_len`, rounded down to an
 * even number so that heavy and recent halves are equal.
 */
int32_t lessdec_budget_tokens(double percent, int32_t max_len);

#ifdef __cplusplus
}
#endif
#endif /* LESSDEC_H */
