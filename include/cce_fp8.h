/*
 * libcce, FP8 variant: the logit products of the fused LM-head + cross-entropy path in
 * E4M3 with block scales, for AMD MI355X (gfx950).
 *
 * The paper's FP8 section defines the E4M3 format (1-4-3 bits, bias 7, range +-448) and a
 * block-wise quantiser -- blocks of 128 elements, one scale each, values clamped to +-448 -- and
 * asks for accumulation wider than the operands.  Here the two products that FORM logits (the
 * chunked forward and its recomputation in the backward) run on the block-scaled FP8 matrix
 * instruction of CDNA4, which multiplies 64 K values per instruction at twice the bf16 rate and
 * applies one power-of-two scale per operand row and block by itself, accumulating in fp32.
 * For that the scale is the paper's amax / 448 rounded UP to a power of two and stored as a
 * biased exponent byte (value = code x 2^(byte - 127)); rounding to E4M3 is to nearest, ties to
 * even.  The two gradient contractions (dH = G W, dW = G^T H) keep the bf16 operands: the
 * gradient is taken straight through the quantiser.
 *
 * Layouts: a quantised matrix is `q` uint8 [rows, D] (E4M3 codes, row-major) plus `scales`,
 * cce_fp8_scale_bytes(rows, D) bytes ordered as the matrix instruction consumes them:
 * [D / 128][ceil(rows / 128)][32][4] -- the exponent byte of row r and columns 128 k .. 128 k + 127
 * is scales[((k * ceil(rows / 128) + r / 128) * 32 + r % 32) * 4 + (r % 128) / 32]; entries of
 * rows past the matrix hold 127.  D must be a multiple of 128.
 *
 * Conventions are those of cce.h: DEVICE pointers owned by the caller, 16-byte aligned (scales:
 * 4-byte); `stream` is a hipStream_t as void*; nothing is allocated, freed or synchronised;
 * CCE_OK or a negative CCE_ERR_* code is returned and nothing is enqueued on an error.
 */
#ifndef CCE_FP8_H_
#define CCE_FP8_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of the scale array of a [rows, D] matrix; 0 when D is not a positive multiple of 128.
 * Host only. */
size_t cce_fp8_scale_bytes(int64_t rows, int64_t D);

/*
 * Block-wise E4M3 quantisation (block-wise quantisation algorithm, block size 128, with the
 * power-of-two scale described above).
 *   x       in  bf16 [rows, D]   finite values
 *   q       out uint8 [rows, D]
 *   scales  out uint8 [cce_fp8_scale_bytes(rows, D)]
 * A block of zeros gets exponent byte 127 and codes 0.  One pass: 2 bytes read, 1 written per
 * element.
 */
int cce_quantize_e4m3(const void* x, int64_t rows, int64_t D, void* q, void* scales, void* stream);

/*
 * cce_forward with the logits formed from the quantised operands:
 * z_iv = sum over blocks b of 2^(sh_ib + sw_vb) sum_{k in b} hq_ik wq_vk  (exact products, fp32
 * accumulation), then loss_i = lse_i - z_{i, y_i} exactly as cce_forward.
 *   hidden_q, hidden_scales   quantised hidden [N, D]
 *   weight_q, weight_scales   quantised LM-head weight [V, D]
 *   labels, ignore_index, loss, lse, workspace (cce_workspace_bytes(N, D, V) bytes), status
 *   word: as cce_forward
 */
int cce_fp8_forward(const void* hidden_q, const void* hidden_scales, const void* weight_q, const void* weight_scales,
                    const int32_t* labels, int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                    float* loss, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/*
 * cce_backward with the logit tiles recomputed from the quantised operands (so that, with the
 * lse of cce_fp8_forward, every softmax row sums to one) and the two gradient contractions on
 * the bf16 operands:
 *   G_iv = dloss_i (exp(z_iv - lse_i) - [v == y_i]),  dHidden = G weight,  dW = G^T hidden
 *   hidden, weight            the bf16 tensors the quantised ones were made from
 *   everything else           as cce_backward
 */
int cce_fp8_backward(const void* hidden_q, const void* hidden_scales, const void* weight_q, const void* weight_scales,
                     const void* hidden, const void* weight, const int32_t* labels,
                     const float* lse, const float* dloss,
                     int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                     void* dHidden, float* dW, int accumulate_dW,
                     void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CCE_FP8_H_ */
