// libcce: fused LM-head projection + token-level cross-entropy for gfx950 (MI355X).
// Device kernels and the C ABI declared in include/cce.h.
//
// Forward (chunked cross-entropy forward algorithm of the Cut Cross-Entropy section):
//   lse_partial_kernel   logit tile (MFMA) -> online (max, sum-exp) per token, carried in
//                        registers across the vocabulary tiles of one split (online-softmax
//                        definition); one (m, d) pair per token and split is written out
//   finalize_kernel      merges the pairs of all splits (block form of the same recurrence),
//                        lse = m + ln d, label logit by an fp32 dot product, loss = lse - z_y,
//                        ignore_index rows -> 0
// Backward (CCE backward theorem and chunk-level backward algorithm), for each
// [row block x vocabulary chunk]:
//   grad_tile_kernel     recomputes the logit tile, forms dloss * (exp(z - lse) - onehot),
//                        rounds to bf16 and stores it in a scratch chunk G[rows][chunk]
//   grad_gemm_kernel     dH_block += G * W_chunk   and   dW_chunk (+)= G^T * H_block
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#include <mutex>
#include <vector>

#include "../../include/cce.h"
#include "../../include/cce_shard.h"
#include "../../include/cce_fp8.h"
#include "../../include/cce_compact.h"
#include "gemm_core.h"
#include "host_util.h"
#include "plan.h"
#include "wg_map.h"

namespace cce {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kGRowBytes = 256 * 2 + 16;     // LDS staging row of a G tile (256 bf16 + pad)

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Merge two (max, sum) pairs kept in the log2 domain; safe for empty pairs (m = -inf, d = 0).
__device__ __forceinline__ void md_merge(float& m, float& d, float m2, float d2) {
    const float mn = fmaxf(m, m2);
    const float ms = (mn == -INFINITY) ? 0.f : mn;
    d = d * fast_exp2(m - ms) + d2 * fast_exp2(m2 - ms);
    m = mn;
}

// ------------------------------------------------------------------------------------------
// Forward: per (token tile, vocabulary split) online log-sum-exp.
// Tile orientation: M = vocabulary (A = W, K-major), N = tokens (B = H, K-major), so that in
// the 32x32 accumulator layout a lane owns ONE token column and 16 vocabulary rows of each
// block: the running max / sum of a token is lane-local until the very end.
// partials[token * S + split] = (m, d) with m in the log2 domain (m = max_v z * log2 e).
// ------------------------------------------------------------------------------------------
// SUMZ (label smoothing only): the sum of a token's logits over the vocabulary split is carried
// along as well, partial_sumz[token * S + split]; the smoothed loss needs their mean.
// FP8: H and W are E4M3 bytes (row length D) with one scale-exponent byte per row and 128
// columns in hscale / wscale (grouped layout, see ScaleGroup); the logit tile is then formed by the
// block-scaled FP8 MFMA loop and everything after it is unchanged.
struct Fp8Scales {
    const void* hscale;
    const void* wscale;
    int hgroups, wgroups;       // ceil(rows / 128) of each matrix
};

// Exponent byte of (row, 128-block kb) in the grouped scale layout (see ScaleGroup).
__device__ __forceinline__ int scale_byte(const void* scales, int groups, int row, int kb) {
    const uint8_t* s = (const uint8_t*)scales;
    return s[(((size_t)kb * groups + (row >> 7)) * 32 + (row & 31)) * 4 + ((row >> 5) & 3)];
}

template <bool SUMZ, bool FP8>
__global__ __launch_bounds__(kThreads) void lse_partial_kernel(
        const void* __restrict__ H, const void* __restrict__ W,
        int N, int D, int V, int TT, int VT, int S, float2* __restrict__ partials,
        float* __restrict__ partial_sumz, const Fp8Scales fp8, const int32_t* __restrict__ perm) {
    typedef TileBig Cfg;
    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    CCE_LDS char* smem = (CCE_LDS char*)smem_generic;

    // Work index -> (token tile, vocabulary split).  The 32 workgroups that share an XCD (and
    // its 4 MB L2) take a panel of 4 token tiles x all splits: per K slice they touch 4 H
    // tiles + S W tiles instead of 32 + 1, which is what keeps most operand fetches in L2.
    const int lin = xcd_round_id(blockIdx.x, gridDim.x, 256);
    int tt, s;
    group_map(lin, TT, S, 4, tt, s);
    const int vt0 = (int)((int64_t)s * VT / S), vt1 = (int)((int64_t)(s + 1) * VT / S);
    const int l = threadIdx.x & 63;
    const int wm = wave_m<Cfg>();

    const int ld = FP8 ? D / 2 : D;               // row length in 2-byte units
    OperandTile<true, Cfg::BN> Bop;
    Bop.init(H, ld, tt * Cfg::BN, N, ld, perm);       // perm: token t of the tile space is row perm[t] of H
    ScaleGroup SB;
    const int b_row0 = tt * Cfg::BN + wave_n<Cfg>() * (Cfg::TN * 32);      // this wavefront's first token
    if (FP8) SB.init(fp8.hscale, fp8.hgroups, b_row0 >> 7);

    float run_m[Cfg::TN], run_d[Cfg::TN], run_z[Cfg::TN];
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) { run_m[bn] = -INFINITY; run_d[bn] = 0.f; run_z[bn] = 0.f; }

    for (int vt = vt0; vt < vt1; ++vt) {
        f32x16 acc[Cfg::TM][Cfg::TN];
#pragma unroll
        for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
            for (int bn = 0; bn < Cfg::TN; ++bn)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[bm][bn][r] = 0.f;

        OperandTile<true, Cfg::BM> Aop;
        Aop.init(W, ld, vt * Cfg::BM, V, ld);
        if (FP8) {
            ScaleGroup SA;
            SA.init(fp8.wscale, fp8.wgroups, (vt * Cfg::BM + wm * (Cfg::TM * 32)) >> 7);
            gemm_mainloop_fp8<Cfg>(acc, Aop, Bop, SA, SB, (b_row0 >> 6) & 1, D, smem);
        } else {
            gemm_mainloop<Cfg, true, true>(acc, Aop, Bop, D, smem);
        }

        if ((vt + 1) * Cfg::BM > V) {       // ragged last vocabulary tile: mask rows >= V
#pragma unroll
            for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const bool dead = vt * Cfg::BM + acc_row<Cfg>(bm, r) >= V;
#pragma unroll
                    for (int bn = 0; bn < Cfg::TN; ++bn)
                        acc[bm][bn][r] = dead ? -INFINITY : acc[bm][bn][r];
                }
        }
#pragma unroll
        for (int bn = 0; bn < Cfg::TN; ++bn) {
            float tmax = -INFINITY;
#pragma unroll
            for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
                for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, acc[bm][bn][r]);
            const float mn = fmaxf(run_m[bn], tmax * kLog2e);
            const float ms = (mn == -INFINITY) ? 0.f : mn;
            float sum = 0.f;
#pragma unroll
            for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[bm][bn][r], kLog2e, -ms));
            run_d[bn] = run_d[bn] * fast_exp2(run_m[bn] - ms) + sum;
            run_m[bn] = mn;
            if (SUMZ) {
                float sz = 0.f;
#pragma unroll
                for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sz += (acc[bm][bn][r] == -INFINITY) ? 0.f : acc[bm][bn][r];   // masked tail rows
                run_z[bn] += sz;
            }
        }
    }

    // lanes l and l ^ 32 hold the same token column (different vocabulary rows)
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) {
        const float om = __shfl_xor(run_m[bn], 32), od = __shfl_xor(run_d[bn], 32);
        md_merge(run_m[bn], run_d[bn], om, od);
        if (SUMZ) run_z[bn] += __shfl_xor(run_z[bn], 32);
    }
    // the WM waves stacked along the vocabulary dimension share token columns: merge via LDS
    CCE_LDS f32x2* red = (CCE_LDS f32x2*)smem;        // [WM][BN]
    CCE_LDS float* redz = (CCE_LDS float*)(smem + Cfg::WM * Cfg::BN * 8);   // [WM][BN]
    if (l < 32) {
#pragma unroll
        for (int bn = 0; bn < Cfg::TN; ++bn) {
            red[wm * Cfg::BN + acc_col<Cfg>(bn)] = f32x2{run_m[bn], run_d[bn]};
            if (SUMZ) redz[wm * Cfg::BN + acc_col<Cfg>(bn)] = run_z[bn];
        }
    }
    __syncthreads();
    if (threadIdx.x < Cfg::BN) {
        const int tok = tt * Cfg::BN + threadIdx.x;
        float m = -INFINITY, d = 0.f, z = 0.f;
#pragma unroll
        for (int w = 0; w < Cfg::WM; ++w) {
            const f32x2 p = red[w * Cfg::BN + threadIdx.x];
            md_merge(m, d, p.x, p.y);
            if (SUMZ) z += redz[w * Cfg::BN + threadIdx.x];
        }
        if (tok < N) {
            partials[(size_t)tok * S + s] = make_float2(m, d);
            if (SUMZ) partial_sumz[(size_t)tok * S + s] = z;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Forward finalisation: one wavefront per token.
// ------------------------------------------------------------------------------------------
// With `stats` (vocabulary-parallel share): W holds the rows [v_off, v_off + V) of the full
// matrix; instead of a loss the kernel writes, for EVERY token, the shard's statistics
// stats[tok] = (max logit, sum exp(z - max), label logit or 0 when the label lies in another
// shard, sum of logits or 0) in natural units; labels are not judged here.
__global__ __launch_bounds__(256) void finalize_kernel(
        const uint16_t* __restrict__ H, const uint16_t* __restrict__ W, const int32_t* __restrict__ labels,
        const float2* __restrict__ partials, const float* __restrict__ partial_sumz,
        int N, int D, int V, int S, int32_t ignore_index, float label_smoothing, float z_loss,
        float* __restrict__ loss, float* __restrict__ lse, int32_t* __restrict__ status,
        int v_off, float4* __restrict__ stats, const Fp8Scales fp8, const int32_t* __restrict__ perm) {
    const int l = threadIdx.x & 63;
    const int ctok = blockIdx.x * 4 + (threadIdx.x >> 6);     // token of the (compact) tile space
    if (ctok >= N) return;
    // row skipping: partials are indexed by the compact token, everything else by the original row
    const int tok = perm ? perm[ctok] : ctok;
    if (tok < 0) return;
    const int64_t y_local = (int64_t)labels[tok] - v_off;
    const int32_t y = (y_local >= 0 && y_local < V) ? (int32_t)y_local : -1;     // row of W, or none
    const bool in_range = y >= 0;
    if (!stats && (labels[tok] == ignore_index || !in_range)) {
        if (l == 0) {
            loss[tok] = 0.f;
            lse[tok] = 0.f;
            if (labels[tok] != ignore_index) atomicOr(status, CCE_STATUS_BAD_LABEL);
        }
        return;
    }
    float m = -INFINITY, d = 0.f, sumz = 0.f;
    for (int i = l; i < S; i += 64) {
        const float2 p = partials[(size_t)ctok * S + i];
        md_merge(m, d, p.x, p.y);
        if (partial_sumz) sumz += partial_sumz[(size_t)ctok * S + i];
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float om = __shfl_xor(m, o), od = __shfl_xor(d, o);
        md_merge(m, d, om, od);
        sumz += __shfl_xor(sumz, o);
    }
    // label logit: fp32 dot product of the two bf16 rows
    const uint16_t* h = H + (size_t)tok * D;
    const uint16_t* w = W + (size_t)(in_range ? y : 0) * D;
    float zy = 0.f;
    if (fp8.hscale) {
        // E4M3 rows: four codes per lane and step, decoded by the hardware conversion, the
        // 128-block's two scale exponents applied exactly with ldexp
        const uint8_t* h8 = (const uint8_t*)H + (size_t)tok * D;
        const uint8_t* w8 = (const uint8_t*)W + (size_t)(in_range ? y : 0) * D;
        for (int k = l * 4; in_range && k < D; k += 256) {
            const int hv = *(const int*)(h8 + k), wv = *(const int*)(w8 + k);
            const f32x2 h01 = __builtin_amdgcn_cvt_pk_f32_fp8(hv, false), h23 = __builtin_amdgcn_cvt_pk_f32_fp8(hv, true);
            const f32x2 w01 = __builtin_amdgcn_cvt_pk_f32_fp8(wv, false), w23 = __builtin_amdgcn_cvt_pk_f32_fp8(wv, true);
            const float p = fmaf(h01.x, w01.x, fmaf(h01.y, w01.y, fmaf(h23.x, w23.x, h23.y * w23.y)));
            zy += ldexpf(p, scale_byte(fp8.hscale, fp8.hgroups, tok, k >> 7) + scale_byte(fp8.wscale, fp8.wgroups, y, k >> 7) - 254);
        }
    } else
    for (int k = l * 2; in_range && k < D; k += 128) {
        const uint32_t hv = *(const uint32_t*)(h + k), wv = *(const uint32_t*)(w + k);
        zy = fmaf(__uint_as_float(hv << 16), __uint_as_float(wv << 16), zy);
        zy = fmaf(__uint_as_float(hv & 0xffff0000u), __uint_as_float(wv & 0xffff0000u), zy);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) zy += __shfl_xor(zy, o);
    if (l == 0 && stats) {
        stats[tok] = make_float4(m * kLn2, d, zy, sumz);
    } else if (l == 0) {
        const float out = (m + fast_log2(d)) * kLn2;
        lse[tok] = out;
        // (1 - eps) (lse - z_y) + eps (lse - mean_v z_v) + lambda lse^2   (smoothed cross-entropy
        // and z-loss definitions); eps = lambda = 0 leaves lse - z_y
        float t = out - zy;
        if (label_smoothing != 0.f) t = (1.f - label_smoothing) * t + label_smoothing * (out - sumz / (float)V);
        if (z_loss != 0.f) t = fmaf(z_loss * out, out, t);
        loss[tok] = t;
    }
}

// Vocabulary-parallel merge: one thread per token folds the P shard statistics
// stats[p * N + tok] = (m, d, z_y, sum z) in shard order with the online-softmax merge and
// writes the same loss / lse as finalize_kernel does for the undivided vocabulary.
__global__ __launch_bounds__(256) void shard_merge_kernel(
        const float4* __restrict__ stats, int P, const int32_t* __restrict__ labels, int N, int V,
        int32_t ignore_index, float label_smoothing, float z_loss,
        float* __restrict__ loss, float* __restrict__ lse, int32_t* __restrict__ status) {
    const int tok = blockIdx.x * 256 + threadIdx.x;
    if (tok >= N) return;
    const int32_t y = labels[tok];
    if (y == ignore_index || y < 0 || y >= V) {
        loss[tok] = 0.f;
        lse[tok] = 0.f;
        if (y != ignore_index && status) atomicOr(status, CCE_STATUS_BAD_LABEL);
        return;
    }
    float m = -INFINITY, d = 0.f, zy = 0.f, sumz = 0.f;
    for (int p = 0; p < P; ++p) {
        const float4 st = stats[(size_t)p * N + tok];
        md_merge(m, d, st.x * kLog2e, st.y);
        zy += st.z;
        sumz += st.w;
    }
    const float out = (m + fast_log2(d)) * kLn2;
    lse[tok] = out;
    float t = out - zy;
    if (label_smoothing != 0.f) t = (1.f - label_smoothing) * t + label_smoothing * (out - sumz / (float)V);
    if (z_loss != 0.f) t = fmaf(z_loss * out, out, t);
    loss[tok] = t;
}

__global__ void clear_status_kernel(int32_t* status) { if (threadIdx.x == 0) status[0] = 0; }

// Number of rows that take part in the loss (label in range and not ignore_index), counted by
// one workgroup.  Integer counting: the result does not depend on the order.
__device__ __forceinline__ int count_valid_rows(const int32_t* labels, int N, int V, int32_t ignore_index, int* scratch) {
    int c = 0;
    for (int i = threadIdx.x; i < N; i += blockDim.x) {
        const int32_t y = labels[i];
        c += (y != ignore_index && y >= 0 && y < V) ? 1 : 0;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) c += __shfl_xor(c, o);
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = c;
    __syncthreads();
    int total = 0;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) total += scratch[w];
    __syncthreads();
    return total;
}

// Mean reduction of the backward: every row's upstream gradient is grad_scale / n_valid
// (the materialising cross-entropy kernel of the paper divides the gradient by the number
// of non-ignored rows).  One workgroup of 1024 threads; out is a single float.
__global__ __launch_bounds__(1024) void mean_scale_kernel(const int32_t* __restrict__ labels, int N, int V,
                                                          int32_t ignore_index, float grad_scale, float* __restrict__ out) {
    __shared__ int scratch[16];
    const int n = count_valid_rows(labels, N, V, ignore_index, scratch);
    if (threadIdx.x == 0) out[0] = n > 0 ? grad_scale / (float)n : 0.f;
}

// Mean of the per-token losses over the non-ignored rows (0 when there are none).  One
// workgroup; each thread sums a strided subset in fp32, then a fixed tree: the result is
// reproducible run to run.  `kept` (optional, device): the number of rows that took part, where
// that is not the number of valid labels (row skipping with a bound that dropped rows).
__global__ __launch_bounds__(1024) void mean_loss_kernel(const float* __restrict__ loss, const int32_t* __restrict__ labels,
                                                         int N, int V, int32_t ignore_index, float* __restrict__ out,
                                                         const int32_t* __restrict__ kept) {
    __shared__ int scratch[16];
    __shared__ float fsum[16];
    const int n = kept ? kept[0] : count_valid_rows(labels, N, V, ignore_index, scratch);
    float a = 0.f;
    for (int i = threadIdx.x; i < N; i += blockDim.x) a += loss[i];     // ignored rows hold 0
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) a += __shfl_xor(a, o);
    if ((threadIdx.x & 63) == 0) fsum[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int w = 0; w < 16; ++w) t += fsum[w];
        out[0] = n > 0 ? t / (float)n : 0.f;
    }
}

// ------------------------------------------------------------------------------------------
// Backward, step 1: recompute one logit tile and store the bf16 gradient tile
//   G[i, v] = dloss_i * ((1 + 2 lambda lse_i) exp(z_iv - lse_i) - (1 - eps) [v == y_i] - eps / V),
//   0 where the row is ignored / beyond N or the column is beyond V.  eps = lambda = 0 is the
//   plain softmax - onehot of the CCE backward theorem; eps is the label-smoothing weight
//   (smoothed cross-entropy definition), lambda the z-loss weight (z-loss gradient
//   proposition).  dloss == nullptr selects mean reduction: dloss_i = *mean_scale for all i.
// W may be a vocabulary shard: its V rows are the rows [v_off, v_off + V) of a V_total-row
// matrix, labels index the full one (v_off = 0, V_total = V without sharding).
// Same orientation as the forward (lane owns a token column).  The tile is staged in LDS as
// [token][vocab] and written to the scratch chunk G (row-major [rows_pad][ldg], vocab
// contiguous) with full 512-byte rows.
// Grid: one workgroup per tile of the [row block x chunk]; tile index -> (ti, vi).
// ------------------------------------------------------------------------------------------
template <bool FP8>
__global__ __launch_bounds__(kThreads) void grad_tile_kernel(
        const void* __restrict__ H, const void* __restrict__ W, const int32_t* __restrict__ labels,
        const float* __restrict__ lse, const float* __restrict__ dloss, const float* __restrict__ mean_scale,
        int N, int D, int V, int32_t ignore_index, float label_smoothing, float z_loss,
        int row0, int n_row_tiles, int v0, int n_v_tiles,
        uint16_t* __restrict__ G, int ldg, int v_off, int V_total, const Fp8Scales fp8,
        const int32_t* __restrict__ perm) {
    typedef TileBig Cfg;
    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    CCE_LDS char* smem = (CCE_LDS char*)smem_generic;
    const int l = threadIdx.x & 63;
    const int wm = wave_m<Cfg>();

    const int lin = xcd_round_id(blockIdx.x, gridDim.x, 256);
    int ti, vi;
    group_map(lin, n_row_tiles, n_v_tiles, 4, ti, vi);          // an XCD works on ~4 x 8 tiles
    const int tok0 = row0 + ti * Cfg::BN;        // first token of the tile (global index)
    const int vt0 = v0 + vi * Cfg::BM;           // first vocabulary row of the tile (global index)

    f32x16 acc[Cfg::TM][Cfg::TN];
#pragma unroll
    for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::TN; ++bn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bm][bn][r] = 0.f;

    // Per-token scalars of this lane's columns, and the label of the row this thread will flag:
    // only the raw loads are issued here -- unconditional, from clamped indices, so that there is
    // no branch the compiler would have to wait behind -- and everything derived from them is
    // computed after the main loop, under which their latency hides.
    int32_t raw_y[Cfg::TN], raw_row_y;
    float raw_dl[Cfg::TN], raw_ls[Cfg::TN];
    const float uniform_dl = dloss ? 0.f : mean_scale[0];
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) {
        const int tok = tok0 + acc_col<Cfg>(bn);
        const int t = tok < N ? tok : N - 1;
        raw_y[bn] = labels[t];
        raw_dl[bn] = dloss ? dloss[t] : uniform_dl;
        raw_ls[bn] = lse[t];
    }
    {
        const int tok = tok0 + (int)(threadIdx.x & (Cfg::BN - 1));
        raw_row_y = labels[tok < N ? tok : N - 1];
    }

    OperandTile<true, Cfg::BM> Aop;
    OperandTile<true, Cfg::BN> Bop;
    const int ld = FP8 ? D / 2 : D;               // row length in 2-byte units
    Aop.init(W, ld, vt0, V, ld);
    Bop.init(H, ld, tok0, N, ld, perm);           // perm (row skipping): token t is row perm[t] of H
    if (FP8) {
        ScaleGroup SA, SB;
        const int b_row0 = tok0 + wave_n<Cfg>() * (Cfg::TN * 32);
        SA.init(fp8.wscale, fp8.wgroups, (vt0 + wm * (Cfg::TM * 32)) >> 7);
        SB.init(fp8.hscale, fp8.hgroups, b_row0 >> 7);
        gemm_mainloop_fp8<Cfg>(acc, Aop, Bop, SA, SB, (b_row0 >> 6) & 1, D, smem);
    } else {
        gemm_mainloop<Cfg, true, true>(acc, Aop, Bop, D, smem);
    }

    int32_t col_y[Cfg::TN];
    float col_sp[Cfg::TN], col_ch[Cfg::TN], col_ncs[Cfg::TN], col_nl2[Cfg::TN];
    const float eps_over_v = label_smoothing / (float)V_total;
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) {
        const bool tok_ok = tok0 + acc_col<Cfg>(bn) < N;
        // label as a row of W (W holds the rows [v_off, v_off + V) of a V_total-row matrix)
        const int64_t y_local = tok_ok ? (int64_t)raw_y[bn] - v_off : -1;
        col_y[bn] = (y_local >= 0 && y_local < V) ? (int32_t)y_local : -1;
        const float dl = tok_ok ? raw_dl[bn] : 0.f;
        const float ls = tok_ok ? raw_ls[bn] : 0.f;
        col_sp[bn] = dl * fmaf(2.f * z_loss, ls, 1.f);      // factor of the softmax term
        col_ch[bn] = dl * (1.f - label_smoothing);          // subtracted at the label
        col_ncs[bn] = -dl * eps_over_v;                     // added everywhere
        col_nl2[bn] = -ls * kLog2e;
    }
    const bool row_live = threadIdx.x < Cfg::BN && tok0 + (int)threadIdx.x < N &&
                          raw_row_y != ignore_index && raw_row_y >= 0 && raw_row_y < V_total;

    CCE_LDS unsigned char* live_flags = (CCE_LDS unsigned char*)(smem + 256 * kGRowBytes);
    if (threadIdx.x < Cfg::BN) live_flags[threadIdx.x] = row_live ? 1 : 0;

    // Epilogue: softmax gradient, bf16, staged in LDS as [token][vocab] and stored with
    // full 512-byte rows.  Done in TN phases (the 32 token columns per wavefront of block
    // bn): the global stores of one phase drain while the next phase is computed, and the
    // barriers wait for LDS traffic only.
    const bool ragged = vt0 + Cfg::BM > V;                  // only the last vocabulary tile needs column masking
    const int chunk = threadIdx.x & 31;
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) {
        const int col = acc_col<Cfg>(bn);
        const int32_t y = col_y[bn];
        const float sp = col_sp[bn], ch = col_ch[bn], ncs = col_ncs[bn];
        const float nl2 = col_nl2[bn];
        const int yrel = y - (vt0 + wm * (Cfg::TM * 32));     // label relative to this wave's rows
        const bool hit = (yrel >= 0) && (yrel < Cfg::TM * 32);
#pragma unroll
        for (int bm = 0; bm < Cfg::TM; ++bm) {
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                float g[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) g[e] = fmaf(fast_exp2(fmaf(acc[bm][bn][r4 * 4 + e], kLog2e, nl2)), sp, ncs);
                const int rrel = bm * 32 + 8 * r4 + 4 * (l >> 5);      // first of 4 consecutive rows
                if (hit) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) g[e] -= (rrel + e == yrel) ? ch : 0.f;
                }
                const int vrow = wm * (Cfg::TM * 32) + rrel;            // row inside the tile
                if (ragged) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) g[e] = (vt0 + vrow + e < V) ? g[e] : 0.f;
                }
                union { __bf16 h[4]; u32x2 u; } pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk.h[e] = (__bf16)g[e];
                // (token rows with bit 3 set keep the two 8-byte halves of every 16-byte chunk swapped:
                // with a row pitch that is a multiple of 16 bytes, rows c and c + 8 of the 16 lanes
                // an 8-byte write serves per cycle would otherwise hit the same LDS banks)
                *(CCE_LDS u32x2*)(smem + col * kGRowBytes + ((vrow * 2) ^ (col & 8))) = pk.u;
            }
        }
        barrier_lds_only();
        // rows of this phase: tokens 64 * wn + 32 * bn + (0..31) for the WN wavefront columns;
        // thread -> (row index t / 32 + 16 j, 16-byte chunk t % 32)
#pragma unroll
        for (int j = 0; j < (Cfg::WN * 32) / 16; ++j) {
            const int idx = (threadIdx.x >> 5) + 16 * j;
            const int row = (idx >> 5) * (Cfg::TN * 32) + bn * 32 + (idx & 31);
            const bool live = live_flags[row] != 0;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (live) {
                v = *(const CCE_LDS u32x4*)(smem + row * kGRowBytes + chunk * 16);
                if (row & 8) v = u32x4{v.z, v.w, v.x, v.y};           // undo the half swap of the staging writes
            }
            *(u32x4*)(G + (size_t)(ti * Cfg::BN + row) * ldg + (size_t)vi * Cfg::BM + chunk * 8) = v;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Backward, step 2: the two gradient contractions of one [row block x chunk], in ONE launch
// so that their tiles fill the GPU together.  Both have N = hidden dimension:
//   dH job (A K-major): C[token, d] = sum_v G[token, v] * W[v, d]
//   dW job (A K-slow ): C[vocab, d] = sum_i G[i, vocab] * H[i, d]
// A is the scratch chunk G (zero padded to tile multiples in both directions), B is a slice
// of an input tensor in K-slow layout.  The result is added to / stored in the job's output
// (see GemmJob for its two forms).  Rows >= m_valid and columns >= n_valid are
// dropped.  The host puts the job with the longer reduction first; xcd_two_job_map deals the items
// of both jobs to the workgroup ids so that every XCD starts with its share of the long ones.
// ------------------------------------------------------------------------------------------
// LDS of grad_gemm_kernel: the main loop's stages or the epilogue staging, whichever is larger.
constexpr int gemm_lds_bytes(int main_loop, int bm, int bn) {
    const int one_pass = bm * (bn + 8) * 4;
    const int staging = one_pass <= 150 * 1024 ? one_pass : 64 * (bn + 8) * 4;
    return staging > main_loop ? staging : main_loop;
}
constexpr int kGemmLdsBig = gemm_lds_bytes(TileBig::kLdsBytes, TileBig::BM, TileBig::BN);
constexpr int kGemmLdsNarrow = gemm_lds_bytes(TileNarrow::kLdsBytes, TileNarrow::BM, TileNarrow::BN);
// Row skipping: the LDS table of one row block's row map (kRowTableBytes, plan.h) sits behind these.
static_assert(kGemmLdsNarrow + kRowTableBytes <= 160 * 1024 && kGemmLdsBig + kRowTableBytes <= 160 * 1024, "row table must fit the LDS");

// Output of a job, one of three forms:
//   fp32 (the dW job): out_f32 (+)= C when `beta`.
//   fp32 running sum + bf16 result (the dH job): out_f32 is a workspace accumulator over the
//   vocabulary chunks; on the `final` chunk the sum is rounded to bf16 into out_hi (dHidden).
//   split running sum (the dH job, out_lo given): the fp32 sum is kept as two 16-bit planes --
//   the upper halves of the fp32 words in the bf16 output tensor itself (out_hi, whose final
//   content is written by the last chunk), the lower halves in the workspace (out_lo) -- so
//   that the accumulator costs 2 instead of 4 workspace bytes per element; the split is exact.
//   It costs ~2 us per launch (8-byte instead of 16-byte accesses) and is used only where the
//   smaller accumulator buys a better tiling.
struct GemmJob {
    int a_kmajor;               // 1: A is K-major (the dH job), 0: A is K-slow (the dW job)
    const uint16_t* A; int lda; int a_free_n; int a_k_n;
    const void* B; int ldb; int b_k_n; int k_total;
    int n_tiles; int n_work; int m_valid; int n_valid;
    float* out_f32; int64_t ld_out; int beta;
    uint16_t* out_hi; uint16_t* out_lo; int final;
    const int32_t* row_map;     // row skipping: out_hi row of tile row r is row_map[r] (-1: none); else nullptr
    const char* zero_row;       // row skipping: a row of zeros, read by the dW job for k-rows that map to no row
};

// MODE bit 0: the launch's dH job uses the split running sum; bit 1: its bf16 rows go through
// row_map (row skipping).  Launch-wide constants, compiled as separate kernels so that the plain
// form carries none of their code.
template <class Cfg, bool A_KMAJOR, int MODE>
__device__ __forceinline__ void run_gemm_job(const GemmJob& j, int item, CCE_LDS char* smem) {
    const int mi = item / j.n_tiles, ni = item % j.n_tiles;    // consecutive items share the A band

    f32x16 acc[Cfg::TM][Cfg::TN];
#pragma unroll
    for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::TN; ++bn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bm][bn][r] = 0.f;

    constexpr bool kMappedB = (MODE & 2) != 0 && !A_KMAJOR;        // row skipping, dW job
    OperandTile<A_KMAJOR, Cfg::BM> Aop;
    OperandTile<false, Cfg::BN, kMappedB> Bop;
    Aop.init(j.A, j.lda, mi * Cfg::BM, j.a_free_n, j.a_k_n);
    Bop.init(j.B, j.ldb, ni * Cfg::BN, j.n_valid, j.b_k_n);
    if constexpr ((MODE & 2) != 0 && !A_KMAJOR) {
        // row skipping, dW job: the reduction runs over the compact rows of the block, whose hidden
        // rows are scattered over the original tensor.  The block's row map is copied into LDS
        // (behind everything the kernel otherwise uses) and the operand loader looks each of its
        // k-rows up there.  (The host gives every row-skipping launch its row map.)
        CCE_LDS int32_t* tab = (CCE_LDS int32_t*)(smem + gemm_lds_bytes(Cfg::kLdsBytes, Cfg::BM, Cfg::BN));
        for (int i = threadIdx.x; i < j.b_k_n; i += kThreads) tab[i] = j.row_map[i];
        __syncthreads();
        Bop.kmap = tab;
        Bop.kzero = j.zero_row;
    }
    gemm_mainloop<Cfg, A_KMAJOR, false, true>(acc, Aop, Bop, j.k_total, smem);

    // Epilogue through LDS so that global memory sees 16-byte accesses along full rows:
    // the fp32 tile is staged [rows][BN + 8 floats] (the padding keeps the two 128-byte
    // row segments a wavefront writes per instruction in different halves of the banks),
    // 64 rows at a time when the whole tile does not fit (which also keeps the number of
    // chunks a thread holds per pass, and with it the register pressure, small).
    constexpr int kPasses = (Cfg::BM * (Cfg::BN + 8) * 4 <= 150 * 1024) ? 1 : Cfg::BM / 64;
    constexpr int kRowsPerPass = Cfg::BM / kPasses;
    constexpr int kRowBytes = (Cfg::BN + 8) * 4;
    constexpr int kChunksPerRow = Cfg::BN / 4;                 // 16-byte chunks
    constexpr int kRowsPerIter = kThreads / kChunksPerRow;
    constexpr int kIters = kRowsPerPass / kRowsPerIter;        // chunks per thread and pass
    static_assert(kThreads % kChunksPerRow == 0 && kRowsPerPass % kRowsPerIter == 0, "whole rows per iteration");
    static_assert(kRowsPerPass * kRowBytes <= 160 * 1024, "epilogue staging must fit the LDS");
    static_assert(Cfg::KG == 1 || kPasses == 1, "K-group reduction shares the one-pass staging");
    const int wave_row0 = wave_m<Cfg>() * (Cfg::TM * 32);
    // this thread's chunks of a pass: rows it * kRowsPerIter + threadIdx.x / kChunksPerRow
    const int my_chunk = threadIdx.x % kChunksPerRow, my_row = threadIdx.x / kChunksPerRow;
    const int col = ni * Cfg::BN + my_chunk * 4;
    const bool col_ok = col < j.n_valid;                       // n_valid is a multiple of 8: whole chunks

    // When the tile is added to what the output already holds, those values are fetched
    // as early as possible -- all chunks of a pass at once, right after the main loop /
    // the previous pass -- so that their latency hides under the staging through LDS
    // (whose barriers wait for LDS traffic only).
    // (split form: words 0-1 of old[] hold the upper-half plane, words 2-3 the lower-half plane)
    constexpr bool SPLIT = (MODE & 1) != 0, ROWMAP = (MODE & 2) != 0;
    const bool split = SPLIT && j.out_lo != nullptr;
    // row of out_hi that tile row `row` goes to (-1: a padding row of the compact row space)
    auto hi_row = [&](int row) { return ROWMAP && j.row_map ? j.row_map[row] : row; };
    f32x4 old[kIters];
    auto fetch_old = [&](int pr0) {
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int row = mi * Cfg::BM + pr0 + it * kRowsPerIter + my_row;
            old[it] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (j.beta && col_ok && row < j.m_valid) {
                if (split) {
                    const int orow = hi_row(row);
                    const u32x2 hi = orow >= 0 ? *(const u32x2*)(j.out_hi + (size_t)orow * j.ld_out + col) : u32x2{0u, 0u};
                    const u32x2 lo = *(const u32x2*)(j.out_lo + (size_t)row * j.ld_out + col);
                    old[it] = __builtin_bit_cast(f32x4, u32x4{hi.x, hi.y, lo.x, lo.y});
                } else {
                    old[it] = *(const f32x4*)(j.out_f32 + (size_t)row * j.ld_out + col);
                }
            }
        }
    };
    // the four fp32 values of a chunk from its two planes
    auto join_planes = [](const f32x4 planes) {
        const u32x4 w = __builtin_bit_cast(u32x4, planes);
        const u32x4 bits = {(w.x << 16) | (w.z & 0xffffu), (w.x & 0xffff0000u) | (w.z >> 16),
                            (w.y << 16) | (w.w & 0xffffu), (w.y & 0xffff0000u) | (w.w >> 16)};
        return __builtin_bit_cast(f32x4, bits);
    };
    fetch_old(0);

    if (Cfg::KG == 2) {
        // The two K groups hold partial sums of the same positions.  Each wavefront finalises half
        // of its blocks (K group g the blocks bm with bm / (TM / 2) == g): it hands the other half
        // to its partner through the staging area, at the positions the sums end up in, then adds
        // what the partner left at its own positions and puts the sums there, in place (a lane
        // reads and rewrites its own words only).  All eight wavefronts work in both steps; a + b
        // is the same value whichever group adds.
        static_assert(Cfg::KG == 1 || Cfg::TM % 2 == 0, "blocks split evenly between the K groups");
        const int kg = wave_kg<Cfg>();
#pragma unroll
        for (int bm = 0; bm < Cfg::TM; ++bm) {
            if (bm / (Cfg::TM / 2) == kg) continue;
#pragma unroll
            for (int bn = 0; bn < Cfg::TN; ++bn)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    *(CCE_LDS float*)(smem + acc_row<Cfg>(bm, r) * kRowBytes + acc_col<Cfg>(bn) * 4) = acc[bm][bn][r];
        }
        barrier_lds_only();
#pragma unroll
        for (int bm = 0; bm < Cfg::TM; ++bm) {
            if (bm / (Cfg::TM / 2) != kg) continue;
#pragma unroll
            for (int bn = 0; bn < Cfg::TN; ++bn)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    CCE_LDS float* pos = (CCE_LDS float*)(smem + acc_row<Cfg>(bm, r) * kRowBytes + acc_col<Cfg>(bn) * 4);
                    *pos = acc[bm][bn][r] + *pos;
                }
        }
    }
#pragma unroll
    for (int pass = 0; pass < kPasses; ++pass) {
        const int pr0 = pass * kRowsPerPass;
        if (Cfg::KG == 1) {
#pragma unroll
            for (int bm = 0; bm < Cfg::TM; ++bm) {
                const int brow = wave_row0 + bm * 32;           // the 32-row block lies in one pass
                if (brow < pr0 || brow >= pr0 + kRowsPerPass) continue;
#pragma unroll
                for (int bn = 0; bn < Cfg::TN; ++bn)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        *(CCE_LDS float*)(smem + (acc_row<Cfg>(bm, r) - pr0) * kRowBytes + acc_col<Cfg>(bn) * 4) = acc[bm][bn][r];
            }
        }
        barrier_lds_only();
        f32x4 v[kIters];
#pragma unroll
        for (int it = 0; it < kIters; ++it)
            v[it] = *(const CCE_LDS f32x4*)(smem + (it * kRowsPerIter + my_row) * kRowBytes + my_chunk * 16) +
                    (split ? join_planes(old[it]) : old[it]);
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int row = mi * Cfg::BM + pr0 + it * kRowsPerIter + my_row;
            if (!col_ok || row >= j.m_valid) continue;
            if (j.final) {
                union { __bf16 h[4]; u32x2 u; } cv;
#pragma unroll
                for (int e = 0; e < 4; ++e) cv.h[e] = (__bf16)v[it][e];
                const int orow = hi_row(row);
                if (orow >= 0) *(u32x2*)(j.out_hi + (size_t)orow * j.ld_out + col) = cv.u;
            } else if (!split) {
                *(f32x4*)(j.out_f32 + (size_t)row * j.ld_out + col) = v[it];
            } else {
                const u32x4 b = __builtin_bit_cast(u32x4, v[it]);
                const u32x2 hi = {(b.y & 0xffff0000u) | (b.x >> 16), (b.w & 0xffff0000u) | (b.z >> 16)};
                const u32x2 lo = {(b.y << 16) | (b.x & 0xffffu), (b.w << 16) | (b.z & 0xffffu)};
                const int orow = hi_row(row);
                if (orow >= 0) *(u32x2*)(j.out_hi + (size_t)orow * j.ld_out + col) = hi;
                *(u32x2*)(j.out_lo + (size_t)row * j.ld_out + col) = lo;
            }
        }
        if (pass + 1 < kPasses) {
            fetch_old(pr0 + kRowsPerPass);
            barrier_lds_only();                               // staging is free for the next pass
        }
    }
}

template <class Cfg, int MODE>
__global__ __launch_bounds__(kThreads) void grad_gemm_kernel(const GemmJob first, const GemmJob second) {
    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    CCE_LDS char* smem = (CCE_LDS char*)smem_generic;
    bool in_first;
    int item;
    if (first.n_work >= 8 && second.n_work >= 8) {
        xcd_two_job_map(blockIdx.x, first.n_work, second.n_work, in_first, item);
    } else {
        const int lin = xcd_round_id(blockIdx.x, gridDim.x, 256);
        in_first = lin < first.n_work;
        item = in_first ? lin : lin - first.n_work;
    }
    const GemmJob& j = in_first ? first : second;
    if (j.a_kmajor) run_gemm_job<Cfg, true, MODE>(j, item, smem);
    else run_gemm_job<Cfg, false, (MODE & 2)>(j, item, smem);
}

// ------------------------------------------------------------------------------------------
// Row skipping (label scan of the path's first step: rows whose label is ignore_index take no
// part in any product, so they need not be computed at all).  The valid rows are gathered, in
// order, into a compact row space in which the unchanged kernels run; results are scattered
// back.  perm[r] = original row of compact row r, -1 for the padding behind the last valid one.
// ------------------------------------------------------------------------------------------
// One workgroup of 1024 threads: stable compaction of the valid rows (label in [0, V) and not
// ignore_index).  At most max_rows are kept (more: CCE_STATUS_ROW_BOUND, the rest is dropped).
// loss / lse of the rows that are not valid, and of valid rows that were dropped, are set to zero
// when the pointers are given (a caller that does not poll the status word then sees a zero
// contribution from a dropped row, not stale memory).  zero_row (optional): zero_row_len bf16 zeros
// are written there.  The status word is WRITTEN here (bad label / bound bits or 0): the scan is the
// first launch of a row-skipping call and needs no clearing launch in front of it.
// Each thread owns a contiguous run of rows; counts are scanned inside a wavefront with shuffles,
// the sixteen wavefront totals through LDS: one barrier.
__global__ __launch_bounds__(1024) void row_scan_kernel(
        const int32_t* __restrict__ labels, int N, int V, int32_t ignore_index, int max_rows, int rows_pad,
        int32_t* __restrict__ perm, int32_t* __restrict__ count_out, int32_t* __restrict__ status,
        float* __restrict__ loss, float* __restrict__ lse, uint16_t* __restrict__ zero_row, int zero_row_len) {
    __shared__ int wave_total[16];
    __shared__ int wave_bad[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (N + 1023) / 1024;
    const int i0 = tid * per < N ? tid * per : N, i1 = i0 + per < N ? i0 + per : N;
    int c = 0, bad = 0;
    for (int i = i0; i < i1; ++i) {
        const int32_t y = labels[i];
        const bool in_range = y >= 0 && y < V;
        c += (y != ignore_index && in_range) ? 1 : 0;
        bad |= (y != ignore_index && !in_range) ? 1 : 0;
    }
    int incl = c;                                     // inclusive scan over the lanes of the wavefront
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    const bool wave_has_bad = __ballot(bad != 0) != 0;
    if (lane == 63) wave_total[wave] = incl;
    if (lane == 0) wave_bad[wave] = wave_has_bad ? 1 : 0;
    __syncthreads();
    int before = 0, total = 0, any_bad = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const int t = wave_total[w];
        before += w < wave ? t : 0;
        total += t;
        any_bad |= wave_bad[w];
    }
    int pos = before + incl - c;                      // valid rows in front of this thread's run
    for (int i = i0; i < i1; ++i) {
        const int32_t y = labels[i];
        bool zero = true;
        if (y != ignore_index && y >= 0 && y < V) {
            if (pos < max_rows) { perm[pos] = i; zero = false; }
            ++pos;
        }
        if (zero && loss) {
            loss[i] = 0.f;
            lse[i] = 0.f;
        }
    }
    if (zero_row)
        for (int c = tid; c < zero_row_len; c += 1024) zero_row[c] = 0;
    const int kept = total < max_rows ? total : max_rows;
    for (int r = kept + tid; r < rows_pad; r += 1024) perm[r] = -1;
    if (tid == 0) {
        count_out[0] = kept;
        status[0] = (any_bad ? CCE_STATUS_BAD_LABEL : 0) | (total > max_rows ? CCE_STATUS_ROW_BOUND : 0);
    }
}

// Backward of the row-skipping calls, after the scan, in one launch:
// (a) per-row scalars into the compact row space: labels (ignore_index for padding) and up to two
//     fp32 vectors (0 for padding) -- thread r of the grid handles compact row r;
// (b) zero rows of dHidden for every row that takes no part: label not valid, or a valid row that
//     the compaction dropped because the caller's bound was too small (the compaction is stable, so
//     those are the valid rows behind the last kept one) -- one wavefront per original row.
// Grid: enough workgroups of 256 for both, i.e. max(ceil(rows_pad / 256), ceil(N / 4)).
__global__ __launch_bounds__(256) void compact_prepare_backward_kernel(
        const int32_t* __restrict__ perm, const int32_t* __restrict__ count, int rows_pad,
        const int32_t* __restrict__ labels, int N, int V, int32_t ignore_index, int32_t* __restrict__ labels_c,
        const float* __restrict__ a, float* __restrict__ a_c, const float* __restrict__ b, float* __restrict__ b_c,
        int D, uint16_t* __restrict__ dhidden) {
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r < rows_pad) {
        const int from = perm[r];
        labels_c[r] = from >= 0 ? labels[from] : ignore_index;
        if (a) a_c[r] = from >= 0 ? a[from] : 0.f;
        if (b) b_c[r] = from >= 0 ? b[from] : 0.f;
    }
    const int l = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= N) return;
    const int32_t y = labels[row];
    const int kept = count[0];
    const int last_kept = kept > 0 ? perm[kept - 1] : -1;
    if (y != ignore_index && y >= 0 && y < V && row <= last_kept) return;
    u32x4* dr = (u32x4*)(dhidden + (size_t)row * D);
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int c = l; c < (D >> 3); c += 64) dr[c] = z;
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
thread_local int g_last_hip_error = 0;

// Optional per-kernel-family timing with HIP events (cce_profile_begin / cce_profile_end).
// Off by default; when on, every launch of a timed family is bracketed by two events on the
// caller's stream.  Not thread safe: profile from one host thread at a time.
struct ProfState {
    bool on = false;
    std::vector<hipEvent_t> pool;
    size_t used = 0;
    struct Span { int fam; size_t e0, e1; };
    std::vector<Span> spans;
    size_t take() {
        if (used == pool.size()) {
            hipEvent_t e;
            if (!hip_ok(hipEventCreate(&e))) return (size_t)-1;
            pool.push_back(e);
        }
        return used++;
    }
};
static ProfState g_prof;
static std::mutex g_prof_mu;            // guards g_prof (spans of concurrent callers interleave but stay consistent)
static std::atomic<bool> g_prof_on{false};

struct ProfSpan {
    int fam; hipStream_t s; size_t e0 = (size_t)-1;
    ProfSpan(int fam_, hipStream_t s_) : fam(fam_), s(s_) {
        if (!g_prof_on.load(std::memory_order_relaxed)) return;
        std::lock_guard<std::mutex> lock(g_prof_mu);
        if (!g_prof.on) return;
        e0 = g_prof.take();
        if (e0 != (size_t)-1) (void)hipEventRecord(g_prof.pool[e0], s);
    }
    ~ProfSpan() {
        if (e0 == (size_t)-1) return;
        std::lock_guard<std::mutex> lock(g_prof_mu);
        if (!g_prof.on) return;
        const size_t e1 = g_prof.take();
        if (e1 == (size_t)-1) return;
        (void)hipEventRecord(g_prof.pool[e1], s);
        g_prof.spans.push_back({fam, e0, e1});
    }
};

static int check_common(const void* hidden, const void* weight, const int32_t* labels,
                        int64_t N, int64_t D, int64_t V, void* workspace, size_t workspace_bytes, Plan* plan) {
    if (!hidden || !weight || !labels || !workspace) return CCE_ERR_INVALID;
    if (N <= 0 || D <= 0 || V <= 0) return CCE_ERR_INVALID;
    if (D % 64 != 0) return CCE_ERR_UNSUPPORTED;
    if (N > (1 << 30) || V > (1 << 30) || V * D * 2 >= ((int64_t)1 << 32) || N * D * 2 >= ((int64_t)1 << 32))
        return CCE_ERR_UNSUPPORTED;
    if (((uintptr_t)hidden | (uintptr_t)weight | (uintptr_t)labels) & 15) return CCE_ERR_INVALID;
    if ((uintptr_t)workspace & 255) return CCE_ERR_INVALID;
    if (!make_plan(N, D, V, plan)) return CCE_ERR_INVALID;
    if (workspace_bytes < plan->total) return CCE_ERR_INVALID;
    return CCE_OK;
}

// An error left behind by an earlier, unrelated HIP call of this thread must not be reported as
// this call's: it is dropped before the first launch, so that the check after the last launch
// sees this call's launches only.
static inline void drop_stale_hip_error() { (void)hipGetLastError(); }

template <class K>
static bool allow_big_lds(K kernel, int bytes) {
    return hip_ok(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
}

constexpr int kGradTileLds = (256 * kGRowBytes + 256 > TileBig::kLdsBytes) ? 256 * kGRowBytes + 256 : TileBig::kLdsBytes;

// The MFMA kernels use more dynamic LDS than the default limit: raise it once per device
// (not per call, so that the compute calls consist of kernel launches only).
static bool ensure_kernel_attributes() {
    static std::mutex mu;
    static bool done[64] = {};
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return false;
    if (dev < 0 || dev >= 64) return false;
    std::lock_guard<std::mutex> lock(mu);
    if (done[dev]) return true;
    if (!allow_big_lds(lse_partial_kernel<false, false>, TileBig::kLdsBytes)) return false;
    if (!allow_big_lds(lse_partial_kernel<true, false>, TileBig::kLdsBytes)) return false;
    if (!allow_big_lds(lse_partial_kernel<false, true>, TileBig::kLdsBytes)) return false;
    if (!allow_big_lds(grad_tile_kernel<false>, kGradTileLds)) return false;
    if (!allow_big_lds(grad_tile_kernel<true>, kGradTileLds)) return false;
    if (!allow_big_lds(grad_gemm_kernel<TileBig, 0>, kGemmLdsBig)) return false;
    if (!allow_big_lds(grad_gemm_kernel<TileNarrow, 0>, kGemmLdsNarrow)) return false;
    if (!allow_big_lds(grad_gemm_kernel<TileBig, 1>, kGemmLdsBig)) return false;
    if (!allow_big_lds(grad_gemm_kernel<TileNarrow, 1>, kGemmLdsNarrow)) return false;
    if (!allow_big_lds(grad_gemm_kernel<TileBig, 2>, kGemmLdsBig + kRowTableBytes)) return false;
    if (!allow_big_lds(grad_gemm_kernel<TileNarrow, 2>, kGemmLdsNarrow + kRowTableBytes)) return false;
    if (!allow_big_lds(grad_gemm_kernel<TileBig, 3>, kGemmLdsBig + kRowTableBytes)) return false;
    if (!allow_big_lds(grad_gemm_kernel<TileNarrow, 3>, kGemmLdsNarrow + kRowTableBytes)) return false;
    done[dev] = true;
    return true;
}

}  // namespace cce

using namespace cce;

extern "C" {

const char* cce_version(void) { return "0.1.0"; }

const char* cce_strerror(int code) {
    switch (code) {
        case CCE_OK: return "ok";
        case CCE_ERR_INVALID: return "invalid argument (null or misaligned pointer, non-positive size, workspace too small)";
        case CCE_ERR_UNSUPPORTED: return "unsupported shape (D must be a multiple of 64; tensors must stay below 4 GiB of bf16)";
        case CCE_ERR_HIP: return "HIP runtime error (see cce_last_hip_error)";
        case CCE_ERR_TOO_LARGE: return "problem needs more scratch than the static buffer of cce_forward_static holds (use cce_forward with a workspace)";
        default: return "unknown error code";
    }
}

int cce_last_hip_error(void) { return g_last_hip_error; }

size_t cce_workspace_bytes(int64_t N, int64_t D, int64_t V) {
    Plan p;
    if (N <= 0 || D <= 0 || V <= 0 || D % 64 != 0) return 0;
    if (!make_plan(N, D, V, &p)) return 0;
    return p.total;
}

size_t cce_materialised_logit_bytes(int64_t N, int64_t V) {
    if (N <= 0 || V <= 0) return 0;
    return (size_t)N * (size_t)V * 4u;
}

static bool variant_ok(float label_smoothing, float z_loss) {
    return label_smoothing >= 0.f && label_smoothing < 1.f && z_loss >= 0.f && isfinite(z_loss);
}

// Row skipping: what the two implementation functions need to run in the compact row space.
struct CompactCtx {
    Plan plan;                  // made for the compact rows
    const int32_t* perm;        // device: original row of each compact row, -1 for padding
    const char* zero_row = nullptr;   // device: D bf16 zeros (backward only)
};

// Forward over the V rows of `weight`, which are the rows [v_off, v_off + V) of the full
// matrix.  With `stats` the per-token shard statistics are written instead of loss / lse
// (`smooth` then says whether the logit sums are wanted).
static int forward_impl(const void* hidden, const void* weight, const int32_t* labels,
                        int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                        float label_smoothing, float z_loss,
                        float* loss, float* lse, float* mean_loss,
                        int64_t v_off, float* stats, bool want_sumz, const Fp8Scales* fp8_in,
                        void* workspace, size_t workspace_bytes, void* stream_, const CompactCtx* cc = nullptr,
                        int32_t* status_word = nullptr) {
    Plan p;
    Fp8Scales fp8 = {nullptr, nullptr, 0, 0};
    if (fp8_in) {
        fp8 = *fp8_in;
        if (!fp8.hscale || !fp8.wscale || D % 128 != 0) return fp8.hscale && fp8.wscale ? CCE_ERR_UNSUPPORTED : CCE_ERR_INVALID;
        if (((uintptr_t)fp8.hscale | (uintptr_t)fp8.wscale) & 3) return CCE_ERR_INVALID;
    }
    if (!stats && (!loss || !lse)) return CCE_ERR_INVALID;
    if (((uintptr_t)loss | (uintptr_t)lse | (uintptr_t)mean_loss) & 3) return CCE_ERR_INVALID;
    if ((uintptr_t)stats & 15) return CCE_ERR_INVALID;
    if (!variant_ok(label_smoothing, z_loss)) return CCE_ERR_INVALID;
    if (v_off < 0 || v_off > (1 << 30)) return CCE_ERR_INVALID;
    if (cc) {
        p = cc->plan;           // arguments were checked, the status word written (by the label scan), by the caller
    } else {
        int rc = check_common(hidden, weight, labels, N, D, V, workspace, workspace_bytes, &p);
        if (rc != CCE_OK) return rc;
    }
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)workspace;
    int32_t* status = status_word ? status_word : (int32_t*)(ws + p.off_status);
    float2* partials = (float2*)(ws + p.off_partials);
    const bool smooth = stats ? want_sumz : label_smoothing != 0.f;
    float* sumz = smooth ? (float*)(ws + p.off_sumz) : (float*)nullptr;

    const int32_t* fwd_perm = cc ? cc->perm : (const int32_t*)nullptr;
    if (!ensure_kernel_attributes()) return CCE_ERR_HIP;
    if (!cc) {
        drop_stale_hip_error();
        hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(64), 0, stream, status);
    }
    {
        ProfSpan span(CCE_KERNEL_LSE_PARTIAL, stream);
        if (fp8_in)
            hipLaunchKernelGGL((lse_partial_kernel<false, true>), dim3(p.TT * p.S), dim3(kThreads), TileBig::kLdsBytes, stream,
                               hidden, weight, (int)N, (int)D, (int)V, p.TT, p.VT, p.S, partials, sumz, fp8, fwd_perm);
        else if (smooth)
            hipLaunchKernelGGL((lse_partial_kernel<true, false>), dim3(p.TT * p.S), dim3(kThreads), TileBig::kLdsBytes, stream,
                               hidden, weight, (int)N, (int)D, (int)V, p.TT, p.VT, p.S, partials, sumz, fp8, fwd_perm);
        else
            hipLaunchKernelGGL((lse_partial_kernel<false, false>), dim3(p.TT * p.S), dim3(kThreads), TileBig::kLdsBytes, stream,
                               hidden, weight, (int)N, (int)D, (int)V, p.TT, p.VT, p.S, partials, sumz, fp8, fwd_perm);
    }
    hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, stream,
                       (const uint16_t*)hidden, (const uint16_t*)weight, labels, partials, (const float*)sumz,
                       (int)N, (int)D, (int)V, p.S, ignore_index, label_smoothing, z_loss, loss, lse, status,
                       (int)v_off, (float4*)stats, fp8, fwd_perm);
    if (mean_loss && !stats)
        hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(1024), 0, stream,
                           (const float*)loss, labels, (int)N, (int)V, ignore_index, mean_loss, (const int32_t*)nullptr);
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_forward_ex(const void* hidden, const void* weight, const int32_t* labels,
                   int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                   float label_smoothing, float z_loss,
                   float* loss, float* lse, float* mean_loss,
                   void* workspace, size_t workspace_bytes, void* stream_) {
    return forward_impl(hidden, weight, labels, N, D, V, ignore_index, label_smoothing, z_loss,
                        loss, lse, mean_loss, 0, nullptr, false, nullptr, workspace, workspace_bytes, stream_);
}

int cce_shard_forward(const void* hidden, const void* weight_shard, const int32_t* labels,
                      int64_t N, int64_t D, int64_t Vs, int64_t vocab_offset, int want_sumz,
                      float* stats, void* workspace, size_t workspace_bytes, void* stream_) {
    if (!stats) return CCE_ERR_INVALID;
    return forward_impl(hidden, weight_shard, labels, N, D, Vs, -1, 0.f, 0.f, nullptr, nullptr, nullptr,
                        vocab_offset, stats, want_sumz != 0, nullptr, workspace, workspace_bytes, stream_);
}

int cce_shard_merge(const float* stats, int P, const int32_t* labels, int64_t N, int64_t V_total,
                    int32_t ignore_index, float label_smoothing, float z_loss,
                    float* loss, float* lse, float* mean_loss, int32_t* status, void* stream_) {
    if (!stats || !labels || !loss || !lse) return CCE_ERR_INVALID;
    if (P <= 0 || P > 4096 || N <= 0 || N > (1 << 30) || V_total <= 0 || V_total > (1 << 30)) return CCE_ERR_INVALID;
    if (((uintptr_t)stats & 15) || (((uintptr_t)loss | (uintptr_t)lse | (uintptr_t)mean_loss | (uintptr_t)status | (uintptr_t)labels) & 3))
        return CCE_ERR_INVALID;
    if (!variant_ok(label_smoothing, z_loss)) return CCE_ERR_INVALID;
    hipStream_t stream = (hipStream_t)stream_;
    drop_stale_hip_error();
    hipLaunchKernelGGL(shard_merge_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, stream,
                       (const float4*)stats, P, labels, (int)N, (int)V_total, ignore_index, label_smoothing, z_loss,
                       loss, lse, status);
    if (mean_loss)
        hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(1024), 0, stream,
                           (const float*)loss, labels, (int)N, (int)V_total, ignore_index, mean_loss, (const int32_t*)nullptr);
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_forward(const void* hidden, const void* weight, const int32_t* labels,
                int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                float* loss, float* lse, void* workspace, size_t workspace_bytes, void* stream_) {
    return cce_forward_ex(hidden, weight, labels, N, D, V, ignore_index, 0.f, 0.f, loss, lse, nullptr,
                          workspace, workspace_bytes, stream_);
}

// ------------------------------------------------------------------------------------------
// cce_forward for callers that cannot allocate or bring a workspace: the forward's scratch (status
// word, per-split (max, sum-exp) pairs) lives in a file-scope device array.  In host code the
// array's name is only a handle: its device address is looked up once per device with
// hipGetSymbolAddress and that address, never the name, is what kernels and plans are given.
// ------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[CCE_STATIC_SCRATCH_BYTES];

// Device address of this device's copy of `scratch` (each GPU holds its own), or nullptr.
static void* static_scratch_address() {
    static std::mutex mu;
    static void* address[64] = {};
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev)) || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        void* ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch))) || !ptr) return nullptr;
        address[dev] = ptr;
    }
    return address[dev];
}

int cce_forward_static(const void* hidden, const void* weight, const int32_t* labels,
                       int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                       float* loss, float* lse, int32_t* status, void* stream_) {
    if (!hidden || !weight || !labels || !loss || !lse) return CCE_ERR_INVALID;
    if (N <= 0 || D <= 0 || V <= 0 || ((uintptr_t)status & 3)) return CCE_ERR_INVALID;
    if (D % 64 != 0) return CCE_ERR_UNSUPPORTED;
    Plan p;
    if (!make_plan(N, D, V, &p)) return CCE_ERR_INVALID;
    // the forward touches the workspace up to the end of the partial results only
    if (p.off_dhacc > (size_t)CCE_STATIC_SCRATCH_BYTES) return CCE_ERR_TOO_LARGE;
    void* ws = static_scratch_address();
    if (!ws) return CCE_ERR_HIP;
    // forward_impl checks a workspace against the whole plan (forward + backward); only the part
    // in front of off_dhacc exists here and only that part is addressed by the forward kernels
    return forward_impl(hidden, weight, labels, N, D, V, ignore_index, 0.f, 0.f, loss, lse, nullptr,
                        0, nullptr, false, nullptr, ws, p.total, stream_, nullptr, status);
}

// Backward over the V rows of `weight`, which are the rows [v_off, v_off + V) of a matrix of
// V_total rows that `labels`, label smoothing and the validity of a row refer to.
static int backward_impl(const void* hidden, const void* weight, const int32_t* labels,
                         const float* lse, const float* dloss, float grad_scale,
                         int64_t N, int64_t D, int64_t V, int64_t v_off, int64_t V_total, int32_t ignore_index,
                         float label_smoothing, float z_loss,
                         void* dHidden, float* dW, int accumulate_dW,
                         const void* logit_hidden, const void* logit_weight, const Fp8Scales* fp8_in,
                         void* workspace, size_t workspace_bytes, void* stream_, const CompactCtx* cc = nullptr) {
    Plan p;
    // The logit tiles are recomputed from logit_hidden / logit_weight (the bf16 operands, or
    // their E4M3 copies with fp8_in); the two gradient contractions always use the bf16 ones.
    Fp8Scales fp8 = {nullptr, nullptr, 0, 0};
    if (fp8_in) {
        fp8 = *fp8_in;
        if (!fp8.hscale || !fp8.wscale || !logit_hidden || !logit_weight) return CCE_ERR_INVALID;
        if (D % 128 != 0) return CCE_ERR_UNSUPPORTED;
        if (((uintptr_t)fp8.hscale | (uintptr_t)fp8.wscale) & 3) return CCE_ERR_INVALID;
        if (((uintptr_t)logit_hidden | (uintptr_t)logit_weight) & 15) return CCE_ERR_INVALID;
    }
    if (!lse || !dHidden || !dW) return CCE_ERR_INVALID;
    if (((uintptr_t)dHidden | (uintptr_t)dW) & 15) return CCE_ERR_INVALID;
    if (!variant_ok(label_smoothing, z_loss)) return CCE_ERR_INVALID;
    if (v_off < 0 || V_total > (1 << 30) || v_off + V > V_total) return CCE_ERR_INVALID;
    if (cc) {
        p = cc->plan;
    } else {
        int rc = check_common(hidden, weight, labels, N, D, V, workspace, workspace_bytes, &p);
        if (rc != CCE_OK) return rc;
    }
    if (!ensure_kernel_attributes()) return CCE_ERR_HIP;
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)workspace;
    uint16_t* dh_lo = (uint16_t*)(ws + p.off_dhacc);     // lower halves of the fp32 dH sums (see GemmJob)
    uint16_t* G = (uint16_t*)(ws + p.off_g);
    // mean reduction: the common upstream gradient grad_scale / n_valid lives in the status block
    float* mean_scale = (float*)(ws + p.off_status + 64);
    if (!cc) drop_stale_hip_error();
    if (!dloss)
        hipLaunchKernelGGL(mean_scale_kernel, dim3(1), dim3(1024), 0, stream,
                           labels, (int)N, (int)V_total, ignore_index, grad_scale, mean_scale);
    const int grad_lds = kGradTileLds;

    const GemmTile gt = gemm_tile_of_kind(p.gemm_kind);
    const int d_tiles = (int)((D + gt.bn - 1) / gt.bn);
    const int per256 = 256 / gt.bm;                               // contraction row tiles per 256 rows

    // The [row block x vocabulary chunk] steps in execution order.
    struct Step { int64_t r0, rows, v0, cols; int row_tiles, v_tiles; bool first_chunk, last_chunk; };
    std::vector<Step> steps;
    const int64_t nchunks = (V + p.Vc - 1) / p.Vc;
    for (int64_t r0 = 0; r0 < N; r0 += p.Nb) {
        const int64_t rows = (N - r0 < p.Nb) ? (N - r0) : p.Nb;
        for (int64_t c = 0; c < nchunks; ++c) {
            const int64_t v0 = c * p.Vc;
            const int64_t cols = (V - v0 < p.Vc) ? (V - v0) : p.Vc;
            steps.push_back({r0, rows, v0, cols, (int)((rows + 255) / 256), (int)((cols + 255) / 256), c == 0, c == nchunks - 1});
        }
    }
    const int K = (int)steps.size();

    for (int k = 0; k < K; ++k) {
        const Step& st = steps[k];
        const int ldg = st.v_tiles * 256;                       // the chunk is stored densely padded
        const int n_rows_h = (int)N;
        // 1. gradient tiles of this [row block x chunk]
        {
            ProfSpan span(CCE_KERNEL_GRAD_TILE, stream);
            if (fp8_in)
                hipLaunchKernelGGL(grad_tile_kernel<true>, dim3(st.row_tiles * st.v_tiles), dim3(kThreads), grad_lds, stream,
                                   logit_hidden, logit_weight, labels, lse, dloss, (const float*)mean_scale,
                                   (int)N, (int)D, (int)V, ignore_index, label_smoothing, z_loss,
                                   (int)st.r0, st.row_tiles, (int)st.v0, st.v_tiles, G, ldg, (int)v_off, (int)V_total, fp8,
                                   cc ? cc->perm : (const int32_t*)nullptr);
            else
                hipLaunchKernelGGL(grad_tile_kernel<false>, dim3(st.row_tiles * st.v_tiles), dim3(kThreads), grad_lds, stream,
                                   hidden, weight, labels, lse, dloss, (const float*)mean_scale,
                                   n_rows_h, (int)D, (int)V, ignore_index, label_smoothing, z_loss,
                                   (int)st.r0, st.row_tiles, (int)st.v0, st.v_tiles, G, ldg, (int)v_off, (int)V_total, fp8,
                                   cc ? cc->perm : (const int32_t*)nullptr);
        }
        // 2. both contractions in one launch
        // dH block += G * W_chunk      (M = tokens, K = chunk columns, N = D)
        GemmJob dh;
        dh.a_kmajor = 1;
        dh.A = G; dh.lda = ldg; dh.a_free_n = st.row_tiles * 256; dh.a_k_n = ldg;
        dh.B = (const void*)((const uint16_t*)weight + (size_t)st.v0 * D); dh.ldb = (int)D; dh.b_k_n = (int)st.cols;
        dh.k_total = ldg; dh.n_tiles = d_tiles; dh.n_work = st.row_tiles * per256 * d_tiles;
        dh.m_valid = (int)st.rows; dh.n_valid = (int)D;
        dh.out_f32 = p.split_acc ? (float*)nullptr : (float*)(ws + p.off_dhacc); dh.ld_out = D; dh.beta = st.first_chunk ? 0 : 1;
        dh.out_hi = (uint16_t*)dHidden + (cc ? (size_t)0 : (size_t)st.r0 * D); dh.out_lo = p.split_acc ? dh_lo : (uint16_t*)nullptr;
        dh.final = st.last_chunk ? 1 : 0;
        dh.row_map = cc ? cc->perm + st.r0 : (const int32_t*)nullptr;
        dh.zero_row = nullptr;
        // dW chunk (+)= G^T * H_block   (M = chunk columns, K = rows, N = D)
        GemmJob dw;
        dw.a_kmajor = 0;
        dw.A = G; dw.lda = ldg; dw.a_free_n = ldg; dw.a_k_n = st.row_tiles * 256;
        // (row skipping: hidden is the caller's tensor and the block's rows are reached through the row map)
        dw.B = cc ? hidden : (const void*)((const uint16_t*)hidden + (size_t)st.r0 * D); dw.ldb = (int)D; dw.b_k_n = (int)st.rows;
        dw.k_total = st.row_tiles * 256; dw.n_tiles = d_tiles; dw.n_work = st.v_tiles * per256 * d_tiles;
        dw.m_valid = (int)st.cols; dw.n_valid = (int)D;
        dw.out_f32 = dW + (size_t)st.v0 * D; dw.ld_out = D; dw.beta = (st.r0 > 0 || accumulate_dW) ? 1 : 0;
        dw.out_hi = nullptr; dw.out_lo = nullptr; dw.final = 0;
        dw.row_map = cc ? cc->perm + st.r0 : (const int32_t*)nullptr;
        dw.zero_row = cc ? cc->zero_row : (const char*)nullptr;
        const bool dh_first = dh.k_total >= dw.k_total;          // longer reduction first
        const GemmJob& first = dh_first ? dh : dw;
        const GemmJob& second = dh_first ? dw : dh;
        const int work = dh.n_work + dw.n_work;

        {
            ProfSpan span(CCE_KERNEL_GRAD_GEMM, stream);
            const int mode = (p.split_acc ? 1 : 0) | (cc ? 2 : 0);
#define CCE_LAUNCH_GEMM(CFG, MODE, LDS) \
    hipLaunchKernelGGL((grad_gemm_kernel<CFG, MODE>), dim3(work), dim3(kThreads), (LDS) + ((MODE) >= 2 ? kRowTableBytes : 0), stream, first, second)
            if (gt.kind == 0) {
                if (mode == 0) CCE_LAUNCH_GEMM(TileBig, 0, kGemmLdsBig); else if (mode == 1) CCE_LAUNCH_GEMM(TileBig, 1, kGemmLdsBig);
                else if (mode == 2) CCE_LAUNCH_GEMM(TileBig, 2, kGemmLdsBig); else CCE_LAUNCH_GEMM(TileBig, 3, kGemmLdsBig);
            } else {
                if (mode == 0) CCE_LAUNCH_GEMM(TileNarrow, 0, kGemmLdsNarrow); else if (mode == 1) CCE_LAUNCH_GEMM(TileNarrow, 1, kGemmLdsNarrow);
                else if (mode == 2) CCE_LAUNCH_GEMM(TileNarrow, 2, kGemmLdsNarrow); else CCE_LAUNCH_GEMM(TileNarrow, 3, kGemmLdsNarrow);
            }
#undef CCE_LAUNCH_GEMM
        }
    }
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_backward_ex(const void* hidden, const void* weight, const int32_t* labels,
                    const float* lse, const float* dloss, float grad_scale,
                    int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                    float label_smoothing, float z_loss,
                    void* dHidden, float* dW, int accumulate_dW,
                    void* workspace, size_t workspace_bytes, void* stream_) {
    return backward_impl(hidden, weight, labels, lse, dloss, grad_scale, N, D, V, 0, V, ignore_index,
                         label_smoothing, z_loss, dHidden, dW, accumulate_dW, nullptr, nullptr, nullptr,
                         workspace, workspace_bytes, stream_);
}

// Row skipping pays when enough rows can be skipped: the compact row space costs a label scan and
// a few small launches, and its tiling may fit the launches worse.  The plan for the compact rows is used when the time model rates it
// at least 2 % faster than the plan for all rows (plus ~30 us for the extra small kernels);
// otherwise every row is processed, exactly as cce_forward / cce_backward do.
static bool choose_compact_plan(int64_t N, int64_t D, int64_t V, int64_t max_valid_rows, Plan* p, bool* use_compact) {
    Plan plain, comp;
    int64_t M = max_valid_rows < N ? max_valid_rows : N;
    if (M < 1) M = 1;
    if (!make_plan(N, D, V, &plain)) return false;
    *use_compact = false;
    *p = plain;
    const int force = g_force_row_skipping.load(std::memory_order_relaxed);
    if (M < N && force != 1 && make_plan(M, D, V, &comp, N) &&
        (force == 2 || comp.model_us + 30.0 < 0.98 * plain.model_us)) {
        *use_compact = true;
        *p = comp;
    }
    return true;
}

// Row skipping: shared argument checks and plan.
static int compact_plan(const void* hidden, const void* weight, const int32_t* labels, int64_t N, int64_t D, int64_t V,
                        int64_t max_valid_rows, void* workspace, size_t workspace_bytes, Plan* p, bool* compact_out) {
    if (!hidden || !weight || !labels || !workspace) return CCE_ERR_INVALID;
    if (N <= 0 || D <= 0 || V <= 0 || max_valid_rows < 0) return CCE_ERR_INVALID;
    if (D % 64 != 0) return CCE_ERR_UNSUPPORTED;
    if (N > (1 << 30) || V > (1 << 30) || V * D * 2 >= ((int64_t)1 << 32) || N * D * 2 >= ((int64_t)1 << 32))
        return CCE_ERR_UNSUPPORTED;
    if (((uintptr_t)hidden | (uintptr_t)weight | (uintptr_t)labels) & 15) return CCE_ERR_INVALID;
    if ((uintptr_t)workspace & 255) return CCE_ERR_INVALID;
    bool use_compact = false;
    if (!choose_compact_plan(N, D, V, max_valid_rows, p, &use_compact)) return CCE_ERR_INVALID;
    if (workspace_bytes < p->total) return CCE_ERR_INVALID;
    *compact_out = use_compact;
    return CCE_OK;
}

int cce_set_row_skipping(int mode) {
    if (mode < 0 || mode > 2) return CCE_ERR_INVALID;
    g_force_row_skipping.store(mode, std::memory_order_relaxed);
    return CCE_OK;
}

int cce_get_row_skipping(int64_t N, int64_t D, int64_t V, int64_t max_valid_rows, int* skipping) {
    Plan p;
    bool use_compact = false;
    if (!skipping || N <= 0 || D <= 0 || V <= 0 || max_valid_rows < 0) return CCE_ERR_INVALID;
    if (D % 64 != 0) return CCE_ERR_UNSUPPORTED;
    if (!choose_compact_plan(N, D, V, max_valid_rows, &p, &use_compact)) return CCE_ERR_INVALID;
    *skipping = use_compact ? 1 : 0;
    return CCE_OK;
}

int cce_get_compact_tiling(int64_t N, int64_t D, int64_t V, int64_t max_valid_rows,
                           int* row_tiles, int* vocab_tiles) {
    Plan p;
    bool use_compact = false;
    if (!row_tiles || !vocab_tiles || N <= 0 || D <= 0 || V <= 0 || max_valid_rows < 0) return CCE_ERR_INVALID;
    if (D % 64 != 0) return CCE_ERR_UNSUPPORTED;
    if (!choose_compact_plan(N, D, V, max_valid_rows, &p, &use_compact)) return CCE_ERR_INVALID;
    *row_tiles = (int)(p.Nb / 256);
    *vocab_tiles = (int)(p.Vc / 256);
    return CCE_OK;
}

size_t cce_compact_workspace_bytes(int64_t N, int64_t D, int64_t V, int64_t max_valid_rows) {
    Plan p;
    bool use_compact = false;
    if (N <= 0 || D <= 0 || V <= 0 || D % 64 != 0 || max_valid_rows < 0) return 0;
    if (!choose_compact_plan(N, D, V, max_valid_rows, &p, &use_compact)) return 0;
    return p.total;
}

int cce_forward_compact_ex(const void* hidden, const void* weight, const int32_t* labels,
                           int64_t N, int64_t D, int64_t V, int32_t ignore_index, int64_t max_valid_rows,
                           float label_smoothing, float z_loss,
                           float* loss, float* lse, float* mean_loss,
                           void* workspace, size_t workspace_bytes, void* stream_) {
    CompactCtx cc;
    if (!loss || !lse || (((uintptr_t)loss | (uintptr_t)lse | (uintptr_t)mean_loss) & 3)) return CCE_ERR_INVALID;
    if (!variant_ok(label_smoothing, z_loss)) return CCE_ERR_INVALID;
    bool use_compact = false;
    int rc = compact_plan(hidden, weight, labels, N, D, V, max_valid_rows, workspace, workspace_bytes, &cc.plan, &use_compact);
    if (rc != CCE_OK) return rc;
    if (!use_compact)
        return forward_impl(hidden, weight, labels, N, D, V, ignore_index, label_smoothing, z_loss, loss, lse, mean_loss,
                            0, nullptr, false, nullptr, workspace, workspace_bytes, stream_);
    if (!ensure_kernel_attributes()) return CCE_ERR_HIP;
    const Plan& p = cc.plan;
    const int64_t M = max_valid_rows < 1 ? 1 : (max_valid_rows < N ? max_valid_rows : N);
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)workspace;
    int32_t* status = (int32_t*)(ws + p.off_status);
    int32_t* perm = (int32_t*)(ws + p.off_perm);
    const int rows_pad = (int)p.rows_pad;
    drop_stale_hip_error();
    // (the scan writes the status word: no clearing launch)
    hipLaunchKernelGGL(row_scan_kernel, dim3(1), dim3(1024), 0, stream, labels, (int)N, (int)V, ignore_index,
                       (int)(max_valid_rows < N ? max_valid_rows : N), rows_pad, perm, (int32_t*)(ws + p.off_count), status, loss, lse,
                       (uint16_t*)nullptr, 0);
    // the kernels fetch hidden rows through perm and write loss / lse to the original rows
    cc.perm = perm;
    rc = forward_impl(hidden, weight, labels, M, D, V, ignore_index, label_smoothing, z_loss, loss, lse, nullptr,
                      0, nullptr, false, nullptr, workspace, workspace_bytes, stream_, &cc);
    if (rc != CCE_OK || !mean_loss) return rc;
    // mean over the rows that took part: the rows left out hold loss 0
    hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(1024), 0, stream,
                       (const float*)loss, labels, (int)N, (int)V, ignore_index, mean_loss, (const int32_t*)(ws + p.off_count));
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_forward_compact(const void* hidden, const void* weight, const int32_t* labels,
                        int64_t N, int64_t D, int64_t V, int32_t ignore_index, int64_t max_valid_rows,
                        float* loss, float* lse, void* workspace, size_t workspace_bytes, void* stream_) {
    return cce_forward_compact_ex(hidden, weight, labels, N, D, V, ignore_index, max_valid_rows, 0.f, 0.f,
                                  loss, lse, nullptr, workspace, workspace_bytes, stream_);
}

int cce_backward_compact_ex(const void* hidden, const void* weight, const int32_t* labels,
                            const float* lse, const float* dloss, float grad_scale,
                            int64_t N, int64_t D, int64_t V, int32_t ignore_index, int64_t max_valid_rows,
                            float label_smoothing, float z_loss,
                            void* dHidden, float* dW, int accumulate_dW,
                            void* workspace, size_t workspace_bytes, void* stream_) {
    CompactCtx cc;
    if (!lse || !dHidden || !dW) return CCE_ERR_INVALID;
    if (((uintptr_t)dHidden | (uintptr_t)dW) & 15) return CCE_ERR_INVALID;
    if (!variant_ok(label_smoothing, z_loss)) return CCE_ERR_INVALID;
    bool use_compact = false;
    int rc = compact_plan(hidden, weight, labels, N, D, V, max_valid_rows, workspace, workspace_bytes, &cc.plan, &use_compact);
    if (rc != CCE_OK) return rc;
    if (!use_compact)
        return backward_impl(hidden, weight, labels, lse, dloss, grad_scale, N, D, V, 0, V, ignore_index, label_smoothing, z_loss,
                             dHidden, dW, accumulate_dW, nullptr, nullptr, nullptr, workspace, workspace_bytes, stream_);
    if (!ensure_kernel_attributes()) return CCE_ERR_HIP;
    const Plan& p = cc.plan;
    const int64_t M = max_valid_rows < 1 ? 1 : (max_valid_rows < N ? max_valid_rows : N);
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)workspace;
    int32_t* status = (int32_t*)(ws + p.off_status);
    int32_t* perm = (int32_t*)(ws + p.off_perm);
    int32_t* labels_c = (int32_t*)(ws + p.off_labels_c);
    float* lse_c = (float*)(ws + p.off_fa_c);
    float* dloss_c = (float*)(ws + p.off_fb_c);
    const int rows_pad = (int)p.rows_pad;
    drop_stale_hip_error();
    hipLaunchKernelGGL(row_scan_kernel, dim3(1), dim3(1024), 0, stream, labels, (int)N, (int)V, ignore_index,
                       (int)(max_valid_rows < N ? max_valid_rows : N), rows_pad, perm, (int32_t*)(ws + p.off_count), status,
                       (float*)nullptr, (float*)nullptr, (uint16_t*)(ws + p.off_zero_row), (int)D);
    {
        const unsigned g_gather = (unsigned)((rows_pad + 255) / 256), g_zero = (unsigned)((N + 3) / 4);
        hipLaunchKernelGGL(compact_prepare_backward_kernel, dim3(g_gather > g_zero ? g_gather : g_zero), dim3(256), 0, stream,
                           (const int32_t*)perm, (const int32_t*)(ws + p.off_count), rows_pad,
                           labels, (int)N, (int)V, ignore_index, labels_c, lse, lse_c, dloss, dloss_c,
                           (int)D, (uint16_t*)dHidden);
    }
    cc.perm = perm;
    cc.zero_row = ws + p.off_zero_row;
    // mean reduction (dloss == NULL) counts the compact labels: the rows that take part
    return backward_impl(hidden, weight, labels_c, lse_c, dloss ? dloss_c : (const float*)nullptr, grad_scale, M, D, V, 0, V,
                         ignore_index, label_smoothing, z_loss,
                         dHidden, dW, accumulate_dW, nullptr, nullptr, nullptr, workspace, workspace_bytes, stream_, &cc);
}

int cce_backward_compact(const void* hidden, const void* weight, const int32_t* labels,
                         const float* lse, const float* dloss,
                         int64_t N, int64_t D, int64_t V, int32_t ignore_index, int64_t max_valid_rows,
                         void* dHidden, float* dW, int accumulate_dW,
                         void* workspace, size_t workspace_bytes, void* stream_) {
    if (!dloss) return CCE_ERR_INVALID;
    return cce_backward_compact_ex(hidden, weight, labels, lse, dloss, 1.f, N, D, V, ignore_index, max_valid_rows, 0.f, 0.f,
                                   dHidden, dW, accumulate_dW, workspace, workspace_bytes, stream_);
}

int cce_fp8_forward(const void* hidden_q, const void* hidden_scales, const void* weight_q, const void* weight_scales,
                    const int32_t* labels, int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                    float* loss, float* lse, void* workspace, size_t workspace_bytes, void* stream_) {
    const Fp8Scales fp8 = {hidden_scales, weight_scales, (int)((N + 127) / 128), (int)((V + 127) / 128)};
    return forward_impl(hidden_q, weight_q, labels, N, D, V, ignore_index, 0.f, 0.f, loss, lse, nullptr,
                        0, nullptr, false, &fp8, workspace, workspace_bytes, stream_);
}

int cce_fp8_backward(const void* hidden_q, const void* hidden_scales, const void* weight_q, const void* weight_scales,
                     const void* hidden, const void* weight, const int32_t* labels,
                     const float* lse, const float* dloss,
                     int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                     void* dHidden, float* dW, int accumulate_dW,
                     void* workspace, size_t workspace_bytes, void* stream_) {
    if (!dloss) return CCE_ERR_INVALID;
    const Fp8Scales fp8 = {hidden_scales, weight_scales, (int)((N + 127) / 128), (int)((V + 127) / 128)};
    return backward_impl(hidden, weight, labels, lse, dloss, 1.f, N, D, V, 0, V, ignore_index, 0.f, 0.f,
                         dHidden, dW, accumulate_dW, hidden_q, weight_q, &fp8, workspace, workspace_bytes, stream_);
}

int cce_shard_backward(const void* hidden, const void* weight_shard, const int32_t* labels,
                       const float* lse, const float* dloss, float grad_scale,
                       int64_t N, int64_t D, int64_t Vs, int64_t vocab_offset, int64_t V_total,
                       int32_t ignore_index, float label_smoothing, float z_loss,
                       void* dHidden_partial, float* dW_shard, int accumulate_dW,
                       void* workspace, size_t workspace_bytes, void* stream_) {
    return backward_impl(hidden, weight_shard, labels, lse, dloss, grad_scale, N, D, Vs, vocab_offset, V_total,
                         ignore_index, label_smoothing, z_loss, dHidden_partial, dW_shard, accumulate_dW,
                         nullptr, nullptr, nullptr, workspace, workspace_bytes, stream_);
}

int cce_backward(const void* hidden, const void* weight, const int32_t* labels,
                 const float* lse, const float* dloss,
                 int64_t N, int64_t D, int64_t V, int32_t ignore_index,
                 void* dHidden, float* dW, int accumulate_dW,
                 void* workspace, size_t workspace_bytes, void* stream_) {
    if (!dloss) return CCE_ERR_INVALID;
    return cce_backward_ex(hidden, weight, labels, lse, dloss, 1.f, N, D, V, ignore_index, 0.f, 0.f,
                           dHidden, dW, accumulate_dW, workspace, workspace_bytes, stream_);
}

int cce_set_backward_tiling(int row_tiles, int vocab_tiles) {
    if (row_tiles < 0 || vocab_tiles < 0 || (row_tiles == 0) != (vocab_tiles == 0)) return CCE_ERR_INVALID;
    if (row_tiles > 0x7fff || vocab_tiles > 0xffff) return CCE_ERR_INVALID;
    g_force_tiling.store((row_tiles << 16) | vocab_tiles, std::memory_order_relaxed);
    return CCE_OK;
}

int cce_get_backward_tiling(int64_t N, int64_t D, int64_t V, int* row_tiles, int* vocab_tiles) {
    Plan p;
    if (!row_tiles || !vocab_tiles) return CCE_ERR_INVALID;
    if (N <= 0 || D <= 0 || V <= 0) return CCE_ERR_INVALID;
    if (D % 64 != 0) return CCE_ERR_UNSUPPORTED;
    if (!make_plan(N, D, V, &p)) return CCE_ERR_INVALID;
    *row_tiles = (int)(p.Nb / 256);
    *vocab_tiles = (int)(p.Vc / 256);
    return CCE_OK;
}

int cce_set_backward_gemm_tile(int tile_cols) {
    if (tile_cols != 0 && tile_cols != 128 && tile_cols != 256) return CCE_ERR_INVALID;
    g_force_gemm_cols.store(tile_cols, std::memory_order_relaxed);
    return CCE_OK;
}

int cce_set_backward_accumulator(int mode) {
    if (mode < 0 || mode > 2) return CCE_ERR_INVALID;
    g_force_split_acc.store(mode, std::memory_order_relaxed);
    return CCE_OK;
}

int cce_get_backward_accumulator(int64_t N, int64_t D, int64_t V, int* mode) {
    Plan p;
    if (!mode || N <= 0 || D <= 0 || V <= 0) return CCE_ERR_INVALID;
    if (D % 64 != 0) return CCE_ERR_UNSUPPORTED;
    if (!make_plan(N, D, V, &p)) return CCE_ERR_INVALID;
    *mode = p.split_acc ? 2 : 1;
    return CCE_OK;
}

int cce_get_backward_gemm_tile(int64_t N, int64_t D, int64_t V, int* tile_rows, int* tile_cols) {
    Plan p;
    if (!tile_rows || !tile_cols) return CCE_ERR_INVALID;
    if (N <= 0 || D <= 0 || V <= 0) return CCE_ERR_INVALID;
    if (D % 64 != 0) return CCE_ERR_UNSUPPORTED;
    if (!make_plan(N, D, V, &p)) return CCE_ERR_INVALID;
    const GemmTile gt = gemm_tile_of_kind(p.gemm_kind);
    *tile_rows = gt.bm;
    *tile_cols = gt.bn;
    return CCE_OK;
}

int cce_profile_begin(void) {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    g_prof.on = true;
    g_prof.used = 0;
    g_prof.spans.clear();
    g_prof_on.store(true, std::memory_order_relaxed);
    return CCE_OK;
}

int cce_profile_end(double* ms_out, int64_t* launches_out) {
    if (!ms_out || !launches_out) return CCE_ERR_INVALID;
    std::lock_guard<std::mutex> lock(g_prof_mu);
    g_prof_on.store(false, std::memory_order_relaxed);
    g_prof.on = false;
    for (int i = 0; i < CCE_KERNEL_FAMILIES; ++i) { ms_out[i] = 0.0; launches_out[i] = 0; }
    for (const ProfState::Span& sp : g_prof.spans) {
        float ms = 0.f;
        if (!hip_ok(hipEventSynchronize(g_prof.pool[sp.e1]))) return CCE_ERR_HIP;
        if (!hip_ok(hipEventElapsedTime(&ms, g_prof.pool[sp.e0], g_prof.pool[sp.e1]))) return CCE_ERR_HIP;
        ms_out[sp.fam] += ms;
        launches_out[sp.fam] += 1;
    }
    g_prof.spans.clear();
    g_prof.used = 0;
    return CCE_OK;
}

int cce_read_status(const void* workspace, void* stream_, int32_t* status_out) {
    if (!workspace || !status_out) return CCE_ERR_INVALID;
    hipStream_t stream = (hipStream_t)stream_;
    if (!hip_ok(hipMemcpyAsync(status_out, workspace, sizeof(int32_t), hipMemcpyDeviceToHost, stream))) return CCE_ERR_HIP;
    if (!hip_ok(hipStreamSynchronize(stream))) return CCE_ERR_HIP;
    return CCE_OK;
}

}  // extern "C"
