/*
 * libcce, row skipping: cce_forward / cce_backward for callers that know (an upper bound on)
 * how many rows take part in the loss, for AMD MI355X (gfx950).
 *
 * A row whose label is ignore_index contributes nothing to the loss or to either gradient (the
 * forward kernel of the paper stores 0 and returns for it), so none of the path's four products
 * needs to see it.  cce_forward / cce_backward process every row because how many rows are valid
 * is only known on the device and the tiling of the work is decided on the host, without a
 * synchronisation.  A training loop usually has the labels on the host as well (the data loader
 * produced them): given the count of valid rows -- or any upper bound -- these entry points
 * number the valid rows, in order (one label scan), and run the same kernels in that compact
 * row space: the operand loaders reach the hidden rows through the row map (nothing is copied),
 * loss / lse / dHidden go to the original rows.  With a fraction f of ignored rows the MFMA work
 * drops by f; the results are those of cce_forward / cce_backward up to fp32 summation order
 * (the tiling differs), and exactly equal for ignored rows (zeros).
 *
 * Conventions are those of cce.h.  A row is valid when its label lies in [0, V) and is not
 * ignore_index.  If there are MORE valid rows than max_valid_rows the surplus rows (the last
 * ones) are dropped: they are treated like ignored rows (loss = lse = 0, a zero dHidden row, no
 * contribution to dW), CCE_STATUS_ROW_BOUND is set in the workspace status word and the results
 * are those of the kept rows only -- check cce_read_status where the bound is not certain.
 * The hidden row of a row that is not valid is never loaded by these calls, so it may hold
 * anything, NaN and Inf included (cce_forward / cce_backward ask for finite values there).  (Where the calls
 * decide not to skip rows, see cce_get_row_skipping, every row is processed and nothing is
 * dropped or flagged.)  max_valid_rows >= N
 * is allowed (nothing is skipped then).
 */
#ifndef CCE_COMPACT_H_
#define CCE_COMPACT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Whether the two calls below skip rows for this shape and bound (1) or process all rows like
 * cce_forward / cce_backward (0): skipping costs a label scan and a few small launches, and the
 * smaller row count may tile the launches worse, so it is used only where a time model rates it
 * faster (few ignored rows do not pay).  Host only. */
int cce_get_row_skipping(int64_t N, int64_t D, int64_t V, int64_t max_valid_rows, int* skipping);
/* The backward tiling cce_backward_compact runs for this shape and bound, in 256-wide tiles per
 * gradient chunk like cce_get_backward_tiling (which it equals where rows are not skipped).
 * Host only. */
int cce_get_compact_tiling(int64_t N, int64_t D, int64_t V, int64_t max_valid_rows,
                           int* row_tiles, int* vocab_tiles);
/* Tuning / testing aid: 1 = never skip, 2 = skip whenever max_valid_rows < N, 0 = automatic. */
int cce_set_row_skipping(int mode);

/* Workspace bytes of the two calls below; within 1 % of the materialised logits of the N rows
 * (never below the 48 MB floor of cce_workspace_bytes).  0 for invalid
 * shapes.  Host only. */
size_t cce_compact_workspace_bytes(int64_t N, int64_t D, int64_t V, int64_t max_valid_rows);

/* cce_forward over the valid rows only.  loss and lse are written for all N rows (0 for rows
 * that are not valid). */
int cce_forward_compact(const void* hidden, const void* weight, const int32_t* labels,
                        int64_t N, int64_t D, int64_t V, int32_t ignore_index, int64_t max_valid_rows,
                        float* loss, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* cce_backward over the valid rows only.  dHidden is written for all N rows (zero rows for rows
 * that are not valid); dloss is required (its entries at rows that are not valid are never read). */
int cce_backward_compact(const void* hidden, const void* weight, const int32_t* labels,
                         const float* lse, const float* dloss,
                         int64_t N, int64_t D, int64_t V, int32_t ignore_index, int64_t max_valid_rows,
                         void* dHidden, float* dW, int accumulate_dW,
                         void* workspace, size_t workspace_bytes, void* stream);

/* The loss variants of cce_forward_ex / cce_backward_ex (label smoothing, z-loss, mean reduction:
 * smoothed cross-entropy definition, z-loss definition and gradient proposition, the division by the
 * number of non-ignored rows in the paper's cross-entropy kernel) over the valid rows only -- the
 * paper's kernel has both in one: it returns early for an ignored row and applies the variants to
 * the others.  Arguments as in cce_forward_ex / cce_backward_ex plus max_valid_rows; results are
 * theirs up to fp32 summation order.  The mean (mean_loss; dloss == NULL in the backward) is taken
 * over the rows that took part: the valid rows, or the kept ones where the bound dropped some
 * (CCE_STATUS_ROW_BOUND).  cce_forward_compact / cce_backward_compact are these calls with
 * label_smoothing = z_loss = 0, no mean_loss, grad_scale = 1. */
int cce_forward_compact_ex(const void* hidden, const void* weight, const int32_t* labels,
                           int64_t N, int64_t D, int64_t V, int32_t ignore_index, int64_t max_valid_rows,
                           float label_smoothing, float z_loss,
                           float* loss, float* lse, float* mean_loss,
                           void* workspace, size_t workspace_bytes, void* stream);

int cce_backward_compact_ex(const void* hidden, const void* weight, const int32_t* labels,
                            const float* lse, const float* dloss, float grad_scale,
                            int64_t N, int64_t D, int64_t V, int32_t ignore_index, int64_t max_valid_rows,
                            float label_smoothing, float z_loss,
                            void* dHidden, float* dW, int accumulate_dW,
                            void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CCE_COMPACT_H_ */
