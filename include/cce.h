/*
 * libcce -- fused language-model-head projection + token-level cross-entropy for
 * AMD MI355X (gfx950), forward and backward, without ever materialising the
 * [tokens x vocab] logit tensor.
 *
 * The operation is the paper's Cut Cross-Entropy (section "Cut Cross-Entropy:
 * Memory-Efficient Loss Computation"):
 *   forward  -- chunked cross-entropy forward algorithm; per-token
 *               loss_i = logsumexp_v(h_i . W_v) - h_i . W_{y_i}
 *               (cross-entropy definition; the running (max, sum-exp) pair is the
 *               online-softmax definition, whose correctness theorem makes the
 *               result independent of how the vocabulary is tiled);
 *   backward -- CCE backward theorem and chunk-level backward algorithm:
 *               G_iv = dloss_i * (exp(h_i . W_v - lse_i) - [v == y_i]),
 *               dH = G W,  dW = G^T H, with the logits recomputed tile by tile.
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library
 *     never allocates, frees or retains device memory and never synchronises the
 *     stream in the compute calls.  Tensors are dense row-major: hidden [N, D],
 *     weight [V, D] (no bias), labels [N], loss/lse/dloss [N], dHidden [N, D],
 *     dW [V, D].  Pointers must be 16-byte aligned.
 *   - bf16 tensors are raw 16-bit patterns (`void*`); fp32 tensors are `float*`.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it, in order.  cce_forward[_ex] and cce_backward[_ex] consist of
 *     kernel launches only (no memset, copy, allocation or synchronisation), so a stream
 *     under HIP graph capture may call them once the library has been used once on the
 *     device outside a capture (the first call raises the kernels' LDS limit).
 *   - D must be a positive multiple of 64 (the K granule of the MFMA main loop);
 *     N, V >= 1 are otherwise arbitrary (ragged tiles are masked).
 *   - A row whose label equals `ignore_index` yields loss = lse = 0, a zero dHidden
 *     row and no contribution to dW; its dloss entry is never used (it may be NaN or
 *     Inf) and its hidden row may hold any FINITE values (as in any dense formulation
 *     of dW = G^T H, a NaN/Inf there would meet the row's zero gradient).  A label
 *     outside [0, V) that is not `ignore_index` is treated the same way and sets
 *     CCE_STATUS_BAD_LABEL in the workspace status word (see cce_read_status).
 *   - Every call returns CCE_OK (0) or a negative error code; nothing throws or
 *     aborts across this boundary.  On CCE_ERR_INVALID / CCE_ERR_UNSUPPORTED nothing was
 *     enqueued.  CCE_ERR_HIP means a launch of THIS call failed (errors left by earlier HIP
 *     calls of the thread are dropped at entry, not reported); launches before the failing
 *     one may have been enqueued and the outputs are then undefined.
 *   - `workspace` is caller-owned device scratch of at least
 *     cce_workspace_bytes(N, D, V) bytes, 256-byte aligned.  Its size is
 *     O(N*D + tile): per-row partial (max, sum-exp, logit-sum) triples, the fp32
 *     dHidden sums of one row block (for large D only their lower halves: the upper
 *     halves then live in dHidden itself until the last vocabulary chunk rounds the
 *     sums to bf16 there) and one bf16 [row block x vocab chunk] gradient chunk; it
 *     never scales with N*V.  Contents are scratch: nothing
 *     needs to survive between forward and backward except what the caller
 *     passes explicitly (lse).
 */
#ifndef CCE_H_
#define CCE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CCE_OK = 0,
    CCE_ERR_INVALID = -1,      /* null pointer, N/D/V <= 0, misaligned pointer, workspace too small */
    CCE_ERR_UNSUPPORTED = -2,  /* D not a multiple of 64, or a size beyond 32-bit tile indexing */
    CCE_ERR_HIP = -3,          /* a HIP call or kernel launch failed (see cce_last_hip_error) */
    CCE_ERR_TOO_LARGE = -4     /* cce_forward_static: the shape needs more than CCE_STATIC_SCRATCH_BYTES */
};

enum {
    CCE_STATUS_BAD_LABEL = 1,  /* some label was outside [0, V) and not ignore_index */
    CCE_STATUS_ROW_BOUND = 2   /* cce_*_compact: more valid rows than max_valid_rows; results are incomplete */
};

/* Library version, "major.minor.patch". Host only. */
const char* cce_version(void);

/* Text for an error code. Host only; the returned string is static. */
const char* cce_strerror(int code);

/* hipError_t (as int) of the last failed HIP call made by this thread, 0 if none. */
int cce_last_hip_error(void);

/* Bytes of device workspace needed by cce_forward / cce_backward for this shape.
 * Pure host function (queries the current device's CU count once); returns 0 for
 * invalid shapes. */
size_t cce_workspace_bytes(int64_t N, int64_t D, int64_t V);

/* Size N*V*4 of the logit tensor that is NOT materialised (the paper's memory
 * equation for the logits: tokens x vocab x 4 bytes), for reporting the workspace
 * as a fraction of it. */
size_t cce_materialised_logit_bytes(int64_t N, int64_t V);

/*
 * Forward (chunked cross-entropy forward algorithm; forward kernel listing).
 *   hidden  in  bf16 [N, D]    device
 *   weight  in  bf16 [V, D]    device
 *   labels  in  int32 [N]      device
 *   loss    out fp32 [N]       device   loss_i = lse_i - h_i . W_{y_i}; 0 for ignored rows
 *   lse     out fp32 [N]       device   log-sum-exp of row i's logits; 0 for ignored rows
 * Logit tiles are accumulated in fp32 and consumed unrounded; the label logit is an
 * fp32 dot product of the bf16 inputs.
 */
int cce_forward(const void* hidden, const void* weight, const int32_t* labels,
                int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                float* loss, float* lse,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * cce_forward without a workspace argument and without any allocation -- for callers that cannot
 * allocate device memory or size a workspace where they call it: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same results (bit for bit)
 * as cce_forward; the scratch the forward needs (status word and the per-vocabulary-split
 * (max, sum-exp) pairs, 12 bytes x N x splits) lives in a static device array of
 * CCE_STATIC_SCRATCH_BYTES inside the library, which every GPU the library runs on holds until
 * the process ends.
 *   hidden, weight, labels, N, D, V, ignore_index, loss, lse, stream   as in cce_forward
 *   status   out int32 [1]  device, may be NULL: the call's status word (bit set of CCE_STATUS_*),
 *            cleared and written by this call's kernels -- read it after the stream work is done
 * Returns CCE_ERR_TOO_LARGE when N x splits does not fit the static array (N = 8192 .. 32768 of
 * the benchmark shapes need 0.8 MB; the limit is reached near N x splits = 1.39 million), the
 * other codes as cce_forward.  Calls no hipMalloc / hipFree or allocating routine; the first call
 * on a device looks the array's address up (hipGetSymbolAddress) and raises the kernels' LDS
 * limit, so make one call outside a graph capture first.  All calls on one GPU share that GPU's
 * array: calls that overlap in time on one GPU (two streams, two threads) race on it and give
 * undefined results -- serialise them.  Nothing in the array needs to survive between calls.
 */
#define CCE_STATIC_SCRATCH_BYTES (16u << 20)
int cce_forward_static(const void* hidden, const void* weight, const int32_t* labels,
                       int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                       float* loss, float* lse, int32_t* status, void* stream);

/*
 * Backward (CCE backward theorem; chunk-level backward algorithm).
 *   hidden, weight, labels, ignore_index, N, D, V   as in cce_forward
 *   lse      in  fp32 [N]     device   as produced by cce_forward for the same inputs
 *   dloss    in  fp32 [N]     device   upstream gradient of each per-token loss
 *                                      (1/N_valid everywhere for a mean loss); entries
 *                                      at ignored rows are never used (may be NaN)
 *   dHidden  out bf16 [N, D]  device   fp32 accumulation, rounded to nearest even (used as
 *                                      scratch for partial sums while the call runs)
 *   dW       out fp32 [V, D]  device   accumulate_dW == 0: overwritten;
 *                                      accumulate_dW != 0: the gradient is added to it
 * The logit gradient tile is rounded to bf16 (nearest even) before the two
 * contractions, which accumulate in fp32.
 */
int cce_backward(const void* hidden, const void* weight, const int32_t* labels,
                 const float* lse, const float* dloss,
                 int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                 void* dHidden, float* dW, int accumulate_dW,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Loss variants in the same kernels (epilogue-only changes): label smoothing and z-loss of the
 * paper's mathematical-foundations section, and the mean reduction of its cross-entropy
 * kernel.  With eps = label_smoothing in [0, 1) and lambda = z_loss >= 0, for non-ignored rows
 *   loss_i = (1 - eps) (lse_i - z_iy) + eps (lse_i - mean_v z_iv) + lambda lse_i^2
 *            (smoothed cross-entropy definition; z-loss definition)
 *   dloss_i/dz_iv = (1 + 2 lambda lse_i) softmax_iv - (1 - eps) [v == y_i] - eps / V
 *            (cross-entropy gradient proposition; z-loss gradient proposition)
 * lse is the plain log-sum-exp in every variant.  eps = lambda = 0 is cce_forward / cce_backward.
 *
 * cce_forward_ex: as cce_forward, plus
 *   mean_loss  out fp32 [1]  device, may be NULL: sum_i loss_i / n_valid over the rows whose label
 *              is neither ignore_index nor out of range (0 when there are none)
 * cce_backward_ex: as cce_backward, plus
 *   dloss      may be NULL = mean reduction: every row's upstream gradient is
 *              grad_scale / n_valid (grad_scale = gradient of the scalar mean loss, normally 1),
 *              n_valid counted on the device; when dloss is given grad_scale is not used
 * Both return CCE_ERR_INVALID for eps outside [0, 1) or a negative / non-finite lambda.
 */
int cce_forward_ex(const void* hidden, const void* weight, const int32_t* labels,
                   int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                   float label_smoothing, float z_loss,
                   float* loss, float* lse, float* mean_loss,
                   void* workspace, size_t workspace_bytes, void* stream);

int cce_backward_ex(const void* hidden, const void* weight, const int32_t* labels,
                    const float* lse, const float* dloss, float grad_scale,
                    int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                    float label_smoothing, float z_loss,
                    void* dHidden, float* dW, int accumulate_dW,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Tuning aid: forces the backward tiling to row blocks of `row_tiles` x 256 tokens and
 * vocabulary chunks of `vocab_tiles` x 256 columns (clamped to the problem size) for all
 * later calls of this process, cce_workspace_bytes included; (0, 0) restores the automatic
 * choice, which stays inside the workspace budget (1 % of the materialised logits, at
 * least 48 MB).  The chunking is a free parameter of the chunk-level backward
 * algorithm: results agree across tilings up to fp32 summation order.  Process-wide host
 * state (an atomic: it may be set from any thread and every call reads it once, so a plan never
 * mixes two settings; size the workspace and compute under the SAME setting).  Returns CCE_ERR_INVALID for negative values or when only one is 0.  A forced
 * tiling whose gradient chunk (rows x columns x 2 bytes) would reach 4 GiB makes the calls that
 * use it fail with CCE_ERR_INVALID (cce_workspace_bytes returns 0).
 */
int cce_set_backward_tiling(int row_tiles, int vocab_tiles);

/* The tiling (in 256-wide tiles) the backward uses for this shape: the forced one, else the
 * automatic choice.  Host only; the two outputs are host ints. */
int cce_get_backward_tiling(int64_t N, int64_t D, int64_t V, int* row_tiles, int* vocab_tiles);

/* Tuning / testing aid like cce_set_backward_tiling: force the output tile of the two gradient
 * contractions to 256 x tile_cols, tile_cols = 128 or 256; 0 restores the automatic choice.
 * Results agree across the two up to fp32 summation order.  Process-wide host state, like the
 * forced tiling. */
int cce_set_backward_gemm_tile(int tile_cols);

/* Tuning / testing aid: how the running sum of dHidden over the vocabulary chunks is kept --
 * 1: fp32 in the workspace; 2: as two 16-bit planes, the upper halves in dHidden itself and
 * the lower halves in the workspace (half the workspace share, exact, slightly slower per
 * launch); 0 restores the automatic choice (2 only where it buys a better tiling, i.e. large D).
 * Results are bit-identical between the two for the same tiling.  Host state only. */
int cce_set_backward_accumulator(int mode);
/* The form (1 or 2) used for this shape.  Host only. */
int cce_get_backward_accumulator(int64_t N, int64_t D, int64_t V, int* mode);

/* Rows x columns of the output tile the two gradient contractions use for this shape (256 x 256
 * or 256 x 128; chosen with the tiling, by the same cost model: the narrow tile when a chunk's
 * outputs would otherwise be too few tiles to fill the GPU, or when D is not a multiple of 256).
 * Host only; the two outputs are host ints. */
int cce_get_backward_gemm_tile(int64_t N, int64_t D, int64_t V, int* tile_rows, int* tile_cols);

/*
 * Measurement aid (not part of the paper's method): per-kernel-family GPU time from HIP
 * events recorded on the caller's stream around every launch of the three MFMA kernel
 * families between cce_profile_begin() and cce_profile_end().  cce_profile_end()
 * synchronises on the recorded events and fills, per family (CCE_KERNEL_*), the summed
 * milliseconds and the number of launches; both arrays are HOST arrays of
 * CCE_KERNEL_FAMILIES entries.  Process-wide host state behind a lock: launches of every thread
 * between the two calls are recorded; begin / end themselves belong to one measuring thread.
 */
enum {
    CCE_KERNEL_LSE_PARTIAL = 0,   /* forward logit tiles + online log-sum-exp            */
    CCE_KERNEL_GRAD_TILE = 1,     /* backward logit-tile recompute + bf16 gradient tile  */
    CCE_KERNEL_GRAD_GEMM = 2,     /* backward dH = G W and dW = G^T H contractions        */
    CCE_KERNEL_FAMILIES = 3
};
int cce_profile_begin(void);
int cce_profile_end(double* ms_out, int64_t* launches_out);

/* Copies the workspace status word (bit set of CCE_STATUS_*) to *status_out (host).
 * Synchronises `stream`.  The word is cleared at the start of every cce_forward; the row-skipping
 * calls (cce_compact.h), forward and backward, set it anew from their label scan. */
int cce_read_status(const void* workspace, void* stream, int32_t* status_out);

#ifdef __cplusplus
}
#endif
#endif /* CCE_H_ */
