/*
 * libcce, auxiliary entry points: the steps immediately around the fused LM-head +
 * cross-entropy path of include/cce.h, for AMD MI355X (gfx950).
 *
 *   in front  -- the final RMSNorm that produces `hidden` (RMSNorm definition of the paper's
 *                mathematical-foundations section; fused RMSNorm forward / backward kernels of
 *                its Triton-kernel section), forward with cached rstd and backward;
 *   behind    -- the fused AdamW step that consumes the fp32 weight gradient, with the
 *                GPU-resident global-norm clipping coefficient (fused AdamW kernel of the
 *                supplementary material; gradient-clipping strategies).
 *
 * All of them are bound by HBM bandwidth, not by MFMA: one pass over their tensors.
 *
 * Conventions are those of cce.h: every tensor pointer is a DEVICE pointer owned by the
 * caller, dense row-major, 16-byte aligned; bf16 tensors are raw 16-bit patterns (void*);
 * `stream` is a hipStream_t passed as void*; nothing is allocated, freed or synchronised;
 * every call returns CCE_OK or a negative CCE_ERR_* code and enqueues nothing on an error.
 */
#ifndef CCE_AUX_H_
#define CCE_AUX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of device workspace cce_rmsnorm_backward needs (per-workgroup partial sums of
 * dgamma); 0 for invalid shapes.  Host only. */
size_t cce_rmsnorm_workspace_bytes(int64_t N, int64_t D);

/*
 * RMSNorm forward (RMSNorm definition; fused RMSNorm forward kernel).
 *   x      in  bf16 [N, D]
 *   gamma  in  bf16 [D]
 *   y      out bf16 [N, D]   y_ij = x_ij * rstd_i * gamma_j, computed in fp32, rounded once
 *   rstd   out fp32 [N]      1 / sqrt(mean_j x_ij^2 + eps), cached for the backward
 * D must be a positive multiple of 64 and at most 8192.
 */
int cce_rmsnorm_forward(const void* x, const void* gamma, int64_t N, int64_t D, float eps,
                        void* y, float* rstd, void* stream);

/*
 * RMSNorm backward: the derivative of the definition above for the upstream gradient dy
 * (the paper's proposition and kernel listing print dx with a stray factor gamma on the
 * second term; this is the derivative itself).
 *   x, gamma  as in the forward;  rstd fp32 [N] as the forward produced it
 *   dy      in  bf16 [N, D]
 *   dx      out bf16 [N, D]   rstd_i * (gamma_j dy_ij - xhat_ij * mean_j(dy_ij gamma_j xhat_ij)),
 *                             xhat = x * rstd; fp32 arithmetic, rounded once
 *   dgamma  out fp32 [D]      sum_i dy_ij xhat_ij; accumulate_dgamma != 0 adds to it.
 *                             Two-stage, fixed-order sum: reproducible run to run
 *   workspace  at least cce_rmsnorm_workspace_bytes(N, D) bytes, 256-byte aligned
 */
int cce_rmsnorm_backward(const void* x, const void* gamma, const float* rstd, const void* dy,
                         int64_t N, int64_t D, void* dx, float* dgamma, int accumulate_dgamma,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * RMSNorm with the residual add that precedes it fused in (fused RMSNorm-with-residual kernel):
 *   h_ij = x_ij + residual_ij   computed in fp32, rounded once to bf16 and stored back into
 *                               `residual` (the residual stream handed to whatever follows)
 *   y, rstd                     cce_rmsnorm_forward of that stored h
 *   x         in  bf16 [N, D]   the last block's output
 *   residual  i/o bf16 [N, D]   in: the residual stream; out: h.  May not overlap x or y.
 * One pass: 2 reads and 2 writes of N x D bf16 instead of the 3 + 2 of an add followed by a norm.
 */
int cce_rmsnorm_residual_forward(const void* x, void* residual, const void* gamma, int64_t N, int64_t D,
                                 float eps, void* y, float* rstd, void* stream);

/*
 * Backward of the fused form.  h is what the forward left in `residual`; x and residual both
 * receive the gradient of h:
 *   dh = [cce_rmsnorm_backward of (h, gamma, rstd, dy)] + d_residual
 *   d_residual  in  bf16 [N, D]  gradient arriving through the residual stream from whatever
 *                                consumed h besides the norm; NULL = none (the final norm)
 * The sum is formed in fp32 and rounded once.  Everything else as cce_rmsnorm_backward.
 */
int cce_rmsnorm_residual_backward(const void* h, const void* gamma, const float* rstd, const void* dy,
                                  const void* d_residual, int64_t N, int64_t D, void* dh, float* dgamma,
                                  int accumulate_dgamma, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of device workspace cce_grad_sumsq needs (a fixed number of partial sums). Host only. */
size_t cce_sumsq_workspace_bytes(void);

/*
 * Sum of squares of an fp32 gradient tensor, the first half of the GPU-resident global-norm
 * clipping (gradient-clipping strategies: the norm is reduced on the GPU, no host sync).
 *   grad   in  fp32 [n]
 *   sumsq  i/o fp64 [1] device   accumulate == 0: set to sum g^2; != 0: sum g^2 is added, so
 *                                that several tensors can share one global norm
 * Two-stage, fixed-order reduction (fp32 per thread, fp64 across threads and workgroups).
 */
int cce_grad_sumsq(const float* grad, int64_t n, double* sumsq, int accumulate,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * clip_coef[0] = min(1, max_norm / (sqrt(sumsq[0]) + eps_norm)), on the device.
 *   sumsq in fp64 [1] device, clip_coef out fp32 [1] device
 */
int cce_clip_coef(const double* sumsq, float max_norm, float eps_norm, float* clip_coef, void* stream);

/*
 * Fused AdamW step, one pass over the tensors (fused AdamW kernel: clip, decoupled weight
 * decay before the update, both moment updates, bias correction, parameter update):
 *   g <- grad * clip;  p <- p (1 - lr wd);  m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2;
 *   p <- p - lr (m / (1 - b1^step)) / (sqrt(v / (1 - b2^step)) + eps)
 *   param       i/o fp32 [n]   master parameters
 *   param_bf16  out bf16 [n]   may be NULL; else the updated parameters rounded to bf16
 *                              (the copy the LM head reads), written in the same pass
 *   grad        in  fp32 [n]   e.g. dW of cce_backward
 *   m, v        i/o fp32 [n]   moments
 *   step        >= 1; the bias corrections are computed on the host
 *   clip_coef   in  fp32 [1] device, may be NULL (= 1)
 * fp32 arithmetic throughout (the paper keeps optimizer arithmetic and state in FP32).
 */
int cce_adamw_step(float* param, void* param_bf16, const float* grad, float* m, float* v, int64_t n,
                   float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                   const float* clip_coef, void* stream);

/*
 * Measurement aid (not part of the paper's method): launches `workgroups` workgroups of 8
 * wavefronts that each issue iters x 8 v_mfma_f32_32x32x16_bf16 on register operands only --
 * workgroups * 8 * iters * 8 * 32768 flop in all.  Timed by the caller (events on `stream`), it
 * gives the MFMA rate the device sustains with nothing else in the way, next to the nominal
 * peak.  `sink` is a device fp32 [1] that is never written in practice.
 */
int cce_mfma_probe(int workgroups, int iters, float* sink, void* stream);

/*
 * Measurement aid: the same register-only loop (same flop count) with every lane's operand
 * fragments loaded once, before the loop, from `operands` -- device, bf16, 512 x 48 values
 * (48 KB), 16-byte aligned, read by every workgroup.  The instruction stream does not depend on
 * the data, so timing it on random values against constants or zeros separates what the
 * device's power management does with operand activity from what the schedule costs.
 */
int cce_mfma_probe_data(int workgroups, int iters, const void* operands, float* sink, void* stream);

/* Compute units and peak shader clock (kHz) of the current device, from the HIP device
 * attributes: compute units x 4096 bf16 flop per clock x clock is the nominal dense MFMA peak.
 * Both outputs are host ints. */
int cce_device_info(int* compute_units, int* clock_khz);

#ifdef __cplusplus
}
#endif
#endif /* CCE_AUX_H_ */
