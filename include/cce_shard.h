/*
 * libcce, vocabulary-parallel share: what ONE device computes when the LM-head matrix is split
 * by rows (vocabulary) over P devices, each holding W[v_off : v_off + Vs, :], for AMD MI355X
 * (gfx950).
 *
 * The online-softmax state of the Cut Cross-Entropy forward -- a running maximum m and a
 * denominator d = sum exp(z - m) per token (online-softmax definition; its correctness theorem
 * is what allows the state of disjoint vocabulary ranges to be combined in any grouping) --
 * is merged across workgroups inside one device by cce_forward.  Splitting the vocabulary over
 * devices extends the same merge by one level: every device reduces its rows to four numbers
 * per token, the devices exchange them (P x N x 16 bytes; the exchange itself is the caller's:
 * this library opens no connection), and every device folds them, in shard order, into the
 * same loss and log-sum-exp.  In the backward each device forms the gradient tiles of its own
 * rows from the global log-sum-exp: its slice of dW is complete, its dHidden is a partial sum
 * the caller adds over the devices (the paper names multi-device operation as future work and
 * asks that fusion be kept inside the sharding boundary; this is that boundary for the
 * LM-head + loss).
 *
 * With the data split by tokens instead, nothing new is needed: every device runs cce_forward /
 * cce_backward_ex on its rows and passes grad_scale = (its valid rows) / (all valid rows) for
 * a global mean.
 *
 * Conventions are those of cce.h: DEVICE pointers owned by the caller, dense row-major,
 * 16-byte aligned (fp32 vectors: 4-byte); `stream` is a hipStream_t as void*; nothing is
 * allocated, freed or synchronised; CCE_OK or a negative CCE_ERR_* code is returned and
 * nothing is enqueued on an error.  `labels` always index the FULL vocabulary.
 */
#ifndef CCE_SHARD_H_
#define CCE_SHARD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Forward of one shard (Cut Cross-Entropy forward algorithm restricted to the shard's rows).
 *   hidden        in  bf16 [N, D]
 *   weight_shard  in  bf16 [Vs, D]   rows vocab_offset .. vocab_offset + Vs - 1 of the full matrix
 *   labels        in  int32 [N]      full-vocabulary indices; any value is accepted here
 *   stats         out fp32 [N, 4]    per token, for EVERY row (labels are judged by the merge):
 *                   [0] m     max_v z_v over the shard's rows, z = hidden . weight rows, natural units
 *                   [1] d     sum_v exp(z_v - m)
 *                   [2] z_y   the label's logit if vocab_offset <= label < vocab_offset + Vs, else 0
 *                   [3] sum_v z_v if want_sumz != 0 (label smoothing needs the mean logit), else 0
 *   workspace     at least cce_workspace_bytes(N, D, Vs) bytes, 256-byte aligned
 * D must be a multiple of 64; limits as for cce_forward.
 */
int cce_shard_forward(const void* hidden, const void* weight_shard, const int32_t* labels,
                      int64_t N, int64_t D, int64_t Vs, int64_t vocab_offset, int want_sumz,
                      float* stats, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Merge of the P shards' statistics (online-softmax merge; cross-entropy, smoothed
 * cross-entropy and z-loss definitions as in cce_forward_ex).
 *   stats   in  fp32 [P, N, 4]   shard p's cce_shard_forward output at stats + p * N * 4; the
 *                                shards must cover the V_total rows exactly once
 *   loss, lse, mean_loss         as cce_forward_ex writes them (mean_loss may be NULL); folding
 *                                is done in shard order, so every device gets the same bits
 *   status  i/o int32 [1] device, may be NULL: CCE_STATUS_BAD_LABEL is OR-ed in when a label
 *                                is outside [0, V_total) and is not ignore_index (such rows get
 *                                loss = lse = 0, like ignored ones); the caller clears it
 */
int cce_shard_merge(const float* stats, int P, const int32_t* labels, int64_t N, int64_t V_total,
                    int32_t ignore_index, float label_smoothing, float z_loss,
                    float* loss, float* lse, float* mean_loss, int32_t* status, void* stream);

/*
 * Backward of one shard (Cut Cross-Entropy backward theorem restricted to the shard's rows):
 * with G_iv = dloss_i ((1 + 2 z_loss lse_i) exp(z_iv - lse_i) - (1 - eps) [v == y_i] - eps / V_total)
 * for the shard's v only,
 *   dHidden_partial  out bf16 [N, D]   sum over the shard's v of G_iv W_v: the caller adds the
 *                                      P partials (one all-reduce of N x D)
 *   dW_shard         out fp32 [Vs, D]  sum_i G_iv hidden_i, complete; accumulate_dW != 0 adds
 *   lse              in  fp32 [N]      the GLOBAL log-sum-exp (cce_shard_merge's)
 *   dloss, grad_scale, ignore_index, label_smoothing, z_loss   as in cce_backward_ex; a row
 *                    counts as valid when its label lies in [0, V_total) and is not ignore_index
 *   workspace        at least cce_workspace_bytes(N, D, Vs) bytes, 256-byte aligned
 */
int cce_shard_backward(const void* hidden, const void* weight_shard, const int32_t* labels,
                       const float* lse, const float* dloss, float grad_scale,
                       int64_t N, int64_t D, int64_t Vs, int64_t vocab_offset, int64_t V_total,
                       int32_t ignore_index, float label_smoothing, float z_loss,
                       void* dHidden_partial, float* dW_shard, int accumulate_dW,
                       void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CCE_SHARD_H_ */
