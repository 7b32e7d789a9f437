/*
 * mla_decode.h -- C ABI of the MI355X (gfx950) MLA decode-attention library.
 *
 * The operation is the per-head attention of the paper's Section 3.1
 * ("Original MLA Computation Mode in Inference"), S = Q K^T, P = softmax(S),
 * O = P V, for one query token per sequence (the decoding setup of Section 4.1:
 * 16 heads, head dimension 576), together with the log-sum-exp L = m + log(l)
 * that Algorithm 1 writes in its last step.  In MLA all heads share ONE latent
 * KV row per token, and V is the first 512 columns of that row.
 *
 * On the device the KV rows of all sequences form one stream of 128-token units
 * that is divided evenly over a persistent grid of workgroups (so ragged batches
 * are balanced, and results are bit-identical from run to run); each workgroup
 * runs the block-wise online-softmax recurrence of Algorithm 1 on its pieces in the transposed orientation of equations (1)-(4)
 * (KV tokens on the matrix-core M axis), and a second kernel merges, by
 * log-sum-exp, the pieces of every sequence that several workgroups shared.  The
 * paper has no split over KV; the merge is the same m / l recurrence applied
 * across workgroups.
 *
 * Conventions for every entry point
 *   - plain C types only; "device" pointers are HIP device pointers, "host"
 *     pointers are ordinary process memory;
 *   - the caller owns every buffer; the library never allocates, frees or
 *     synchronises; mla_decode() is asynchronous on the given stream;
 *   - every host-detectable error is reported BEFORE anything is launched and
 *     leaves the outputs untouched; no exceptions, no global mutable state
 *     visible to the caller; entry points may be called from several threads.
 */
#ifndef MLA_DECODE_H
#define MLA_DECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MLA_OK = 0,
    MLA_ERR_INVALID_ARG = 1,         /* null / misaligned pointer, negative size or stride      */
    MLA_ERR_UNSUPPORTED_SHAPE = 2,   /* anything but 16 heads, d_qk 576, d_v 512, q_len 1 .. 8  */
    MLA_ERR_WORKSPACE_TOO_SMALL = 3, /* workspace_bytes below mla_decode_workspace_size()       */
    MLA_ERR_HIP = 4,                 /* a HIP runtime call or a kernel launch failed            */
    MLA_ERR_STATIC_LIMIT = 5         /* mla_decode_static(): beyond the static workspace        */
} mla_status_t;

/* Fixed problem shape (DeepSeek-R1 share of one GPU, Section 4.1). */
#define MLA_NUM_HEADS 16
#define MLA_MAX_ABS_SCALE 1.0e6f
#define MLA_D_QK 576
#define MLA_D_V 512

/*
 * Workspace size.  Host only, deterministic, touches no device unless
 * num_workgroups == 0 (then the compute-unit count of the current HIP device is
 * queried: the automatic plan is a persistent workgroup on 13 of every 16 compute
 * units, or on every one when the KV stream is short, see
 * mla_decode_planned_workgroups()).
 * The size depends only on (batch, number of workgroups), never on the
 * per-sequence lengths, which live on the device: one partial result (16 x 512 fp32 plus
 * 16 log-sum-exps) for 2 * num_workgroups + batch + MLA_MAX_Q_LEN slots; a workgroup
 * writes one partial result per sequence it touches and per query token it works for,
 * at most two tokens (see mla_decode_typed()).
 *
 *   batch                >= 1 sequences
 *   num_heads            must be MLA_NUM_HEADS
 *   max_seqlen_kv        >= 1, rows allocated per sequence in the KV cache
 *   num_workgroups       workgroups the KV stream is divided over; 0 = automatic
 *   bytes                [out, host] workspace size the call needs
 *   num_workgroups_used  [out, host, may be NULL] num_workgroups, or for 0 the automatic plan
 *                        for one query token per sequence (with more, see mla_decode_typed(),
 *                        the plan is every compute unit, and the size returned for 0 covers it)
 */
mla_status_t mla_decode_workspace_size(int batch, int num_heads, int max_seqlen_kv,
                                       int num_workgroups, size_t *bytes,
                                       int *num_workgroups_used);

/*
 * The same size query for the automatic plan on a device of num_compute_units compute units, without
 * touching any device (for callers that size buffers before a GPU is chosen, and for hosts without
 * one): the bytes mla_decode_workspace_size(batch, num_heads, max_seqlen_kv, 0, ...) returns when the
 * current device has that many compute units, and in *num_workgroups_used (may be NULL) the
 * workgroups the automatic plan launches there for one query token per sequence.
 * num_compute_units outside 1 .. 65536 is MLA_ERR_INVALID_ARG; other errors as above.
 */
mla_status_t mla_decode_workspace_size_for(int batch, int num_heads, int max_seqlen_kv,
                                           int num_compute_units, size_t *bytes,
                                           int *num_workgroups_used);

/*
 * One decode-attention call.
 *
 *   q               device, bf16 [batch][1][16][576], contiguous, 16-byte aligned
 *   kv_cache        device, bf16; sequence b starts at kv_cache + b*kv_batch_stride
 *                   elements; each token is one row of 576 contiguous bf16 (K = the
 *                   whole row, V = its first 512 columns); 16-byte aligned
 *   kv_batch_stride elements between sequences, >= max_seqlen_kv*576, multiple of 8
 *   cache_seqlens   device, int32 [batch]; values are clamped to [0, max_seqlen_kv]
 *                   on the device; rows at or beyond a sequence's length are never
 *                   read into the result
 *   batch, num_heads, max_seqlen_kv   as above
 *   scale           multiplies q.k before the softmax (1/sqrt(192) for DeepSeek-R1); finite and
 *                   |scale| <= MLA_MAX_ABS_SCALE, else MLA_ERR_INVALID_ARG.  The scaled scores are
 *                   held in fp32 and must stay finite there (they do for inputs below 1e14 in
 *                   magnitude); scores that overflow give NaN results
 *   out             device, fp32 [batch][1][16][512], contiguous, 16-byte aligned
 *   lse             device, fp32 [batch][16]: natural log of sum_t exp(scale * q.k_t)
 *   workspace       device, 16-byte aligned, >= mla_decode_workspace_size(.., 0, ..) bytes;
 *                   contents on entry are irrelevant, contents on exit unspecified
 *   stream          hipStream_t (as void*), NULL = the default stream
 *
 * A sequence of length 0 yields out = 0 and lse = -inf.
 * Two calls that share a workspace must be ordered on the same stream.
 */
mla_status_t mla_decode(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                        const int32_t *cache_seqlens, int batch, int num_heads,
                        int max_seqlen_kv, float scale, float *out, float *lse,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Extended call for tuning sweeps, tests of the log-sum-exp merge and per-kernel timing.
 *   num_workgroups  0 = the automatic plan of mla_decode(); otherwise the number of
 *                   workgroups (1 .. 65536) the stream of MLA_UNIT_TOKENS-token units is
 *                   divided over.  The workspace must hold the size
 *                   mla_decode_workspace_size() returns for the same number.
 *   flags           MLA_PHASE_SPLIT launches the split-KV main kernel (every step of
 *                   Algorithm 1 on each workgroup's tiles), MLA_PHASE_COMBINE launches the
 *                   merge of the workgroups' results; at least one of the two must be set and
 *                   mla_decode() is both.  Running the combine phase alone is only meaningful
 *                   after a split phase with the same arguments and workspace.
 *                   MLA_ORIENT_DIRECT, added to the above, makes the split kernel compute in the
 *                   original orientation of Section 3.1 (S = Q K^T and O = P V with heads on the
 *                   matrix-core M axis) instead of the transposed one of equations (1)-(4): the
 *                   same result up to fp32 summation order, kept so that the two orientations can
 *                   be measured against each other.  bf16 and one query token only
 *                   (else MLA_ERR_UNSUPPORTED_SHAPE).
 *                   MLA_UNIT_FINE / MLA_UNIT_COARSE (at most one) force the unit of the stream to
 *                   MLA_UNIT_TOKENS_FINE / MLA_UNIT_TOKENS rows.  Without either the unit is 128
 *                   rows (one 32-row tile for each of a workgroup's four wavefronts) unless
 *                   4 * batch * ceil(max_seqlen_kv / 32) is at most the number of workgroups: so tiny a
 *                   batch is divided by the tile, so that it spreads over more compute units.
 * All other arguments, and all error behaviour, are those of mla_decode().
 */
#define MLA_UNIT_TOKENS 128
#define MLA_UNIT_TOKENS_FINE 32
#define MLA_PHASE_SPLIT 1
#define MLA_PHASE_COMBINE 2
#define MLA_ORIENT_DIRECT 8
#define MLA_UNIT_FINE 16
#define MLA_UNIT_COARSE 32
mla_status_t mla_decode_ex(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                           const int32_t *cache_seqlens, int batch, int num_heads,
                           int max_seqlen_kv, float scale, float *out, float *lse,
                           void *workspace, size_t workspace_bytes, int num_workgroups,
                           int flags, void *stream);

/*
 * The general call: either 16-bit input type, and one or more query tokens per sequence.
 *
 *   dtype  MLA_DTYPE_BF16 or MLA_DTYPE_F16: the element type of q and kv_cache (out and lse
 *          stay fp32); any other value is MLA_ERR_INVALID_ARG.  The paper's own runs are FP16
 *          (Section 4.1); the matrix-core products then take fp16 operands, and the softmax
 *          probabilities enter the second product as ONE fp16 term (11 significant bits)
 *          instead of the two-term bf16 split.
 *   q_len  query tokens per sequence, 1 .. MLA_MAX_Q_LEN (Section 3.1: decoding feeds one or
 *          two tokens per step); other values are MLA_ERR_UNSUPPORTED_SHAPE.  Then
 *            q    is [batch][q_len][16][576],
 *            out  is [batch][q_len][16][512],  lse is [batch][q_len][16],
 *            cache_seqlens[b] counts the KV rows INCLUDING those of the q_len new tokens, which
 *            are the last q_len rows of the sequence, and attention is causal among them: query
 *            token j (0-based) attends to rows [0, cache_seqlens[b] - (q_len - 1 - j)); a token
 *            left with no row yields out = 0 and lse = -inf.
 *          The workspace must have the size mla_decode_workspace_size() returns for
 *          batch * q_len in place of batch.  With q_len >= 2 a workgroup works for two query
 *          tokens (two of its four wavefronts each) on the KV rows it streams, so a row is
 *          fetched once for both; with more than two tokens, ceil(q_len / 2) such workgroups
 *          form a team that takes the same KV rows at the same time, so that a row comes in
 *          from HBM once and the other readers are served by the memory-side cache.  The
 *          automatic plan then uses every compute unit (mla_decode_planned_workgroups()).
 * All other arguments, layouts and error behaviour are those of mla_decode_ex().
 */
#define MLA_DTYPE_BF16 0
#define MLA_DTYPE_F16 1
#define MLA_MAX_Q_LEN 8
mla_status_t mla_decode_typed(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                              const int32_t *cache_seqlens, int batch, int q_len, int num_heads,
                              int max_seqlen_kv, int dtype, float scale, float *out, float *lse,
                              void *workspace, size_t workspace_bytes, int num_workgroups,
                              int flags, void *stream);

/*
 * The number of workgroups the automatic plan (num_workgroups == 0) launches on the current HIP
 * device for `batch` sequences of at most max_seqlen_kv rows and q_len query tokens each: 13 of
 * every 16 compute units for one token and a long KV stream (batch * ceil(max_seqlen_kv / 128)
 * above 8 per compute unit), every compute unit otherwise.  Host only.  q_len outside
 * 1 .. MLA_MAX_Q_LEN is MLA_ERR_UNSUPPORTED_SHAPE; a NULL pointer, batch < 1 or
 * max_seqlen_kv < 1 MLA_ERR_INVALID_ARG.
 */
mla_status_t mla_decode_planned_workgroups(int batch, int q_len, int max_seqlen_kv,
                                           int *num_workgroups);

/*
 * The partition of a batch as the kernels derive it on the device, as a table (tests, diagnosis).
 * Launches one small kernel on `stream` that evaluates the same device functions as the two kernels
 * of mla_decode_typed() called with the same batch, q_len, max_seqlen_kv, num_workgroups and flags
 * (MLA_ORIENT_DIRECT and the MLA_UNIT_ flags matter; phases are ignored), and writes 8 int32 per
 * record into `table` (device, (num_workgroups + batch) * 8 int32 or more; with num_workgroups == 0,
 * size it with mla_decode_planned_workgroups()):
 *   record k < *teams        {total units, active teams, first unit, end unit, first sequence, that
 *                             sequence's first unit, its clamped length, 0} of team k (first unit ..
 *                             the sequence's first unit are -1, the length 0, for an idle team)
 *   record *teams + b        {total units, first unit, units, first team, last team, 0, 0, 0} of
 *                             sequence b (teams -1 for an empty sequence)
 * *teams (host) receives the number of teams (workgroups per query-token pair) the unit stream is
 * divided over and *unit_tokens (host) the rows per unit.  The split over the KV length is not in the
 * paper; see mla_decode_typed().  Errors as for mla_decode_typed(), before anything is launched.
 */
mla_status_t mla_decode_plan_table(const int32_t *cache_seqlens, int batch, int q_len, int max_seqlen_kv,
                                   int num_workgroups, int flags, int32_t *table, int *teams,
                                   int *unit_tokens, void *stream);

/*
 * The call for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  It is mla_decode_typed()
 * with the automatic plan and both phases, and with the partial results kept in a file-scope
 * device array of the library (19.2 MB per GPU, held until the process ends) instead of a caller's
 * workspace.  It calls no allocating routine.  The same kernels run, so the results are bit for bit
 * those of mla_decode_typed(..., num_workgroups = 0, MLA_PHASE_SPLIT | MLA_PHASE_COMBINE).
 *
 * Limits: batch * q_len <= MLA_STATIC_MAX_ROWS and a device of at most MLA_STATIC_MAX_WORKGROUPS
 * compute units; beyond either, MLA_ERR_STATIC_LIMIT is returned before anything is launched.
 * Every call on a GPU shares that GPU's array: calls on one GPU must be ordered (one stream, or
 * events between streams); calls that overlap on one GPU race on the partial results.  The array's
 * contents never need clearing: every slot the merge reads was written by the same call.
 * All other arguments, layouts and error behaviour are those of mla_decode_typed().
 */
#define MLA_STATIC_MAX_ROWS 64
#define MLA_STATIC_MAX_WORKGROUPS 256
mla_status_t mla_decode_static(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                               const int32_t *cache_seqlens, int batch, int q_len, int num_heads,
                               int max_seqlen_kv, int dtype, float scale, float *out, float *lse,
                               void *stream);

/* Static string for a status code (never NULL). */
const char *mla_status_string(mla_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* MLA_DECODE_H */
