// libcce, auxiliary kernels: the final RMSNorm in front of the LM head and the fused AdamW
// step (with the clipping coefficient) behind it.  C ABI declared in include/cce_aux.h.
// All of them stream their tensors once: the bound is HBM bandwidth, so the work is 16-byte
// coalesced accesses, wavefront shuffles for the row reductions and no atomics (two-stage
// fixed-order sums keep the results reproducible).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/cce.h"
#include "../../include/cce_aux.h"
#include "../../include/cce_fp8.h"
#include "host_util.h"

namespace cce {

typedef __attribute__((ext_vector_type(4))) unsigned int au32x4;
typedef __attribute__((ext_vector_type(4))) float af32x4;

constexpr int kNormMaxChunks = 16;      // 16-byte chunks per lane and row: D <= 16 * 64 * 8 = 8192
constexpr int kNormBackwardBlocks = 512;        // D <= 1024: four rows in flight per workgroup
constexpr int kNormBackwardBlocksWide = 1024;   // wider rows: two rows or one
constexpr int kSumsqBlocks = 1024;

__device__ __forceinline__ void unpack8(const au32x4& p, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(p[i] << 16);
        f[2 * i + 1] = __uint_as_float(p[i] & 0xffff0000u);
    }
}

__device__ __forceinline__ au32x4 pack8(const float (&f)[8]) {
    au32x4 p;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        union { __bf16 h[2]; unsigned int u; } cv;
        cv.h[0] = (__bf16)f[2 * i];
        cv.h[1] = (__bf16)f[2 * i + 1];
        p[i] = cv.u;
    }
    return p;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// ------------------------------------------------------------------------------------------
// RMSNorm forward (RMSNorm definition; fused forward kernel: one pass, rstd cached).
// One wavefront per row; lane l holds the 16-byte chunks l, l + 64, ... of the row in
// registers between the reduction and the scaling, so x is read once.
// ------------------------------------------------------------------------------------------
template <int CH>      // 16-byte chunks a lane holds per row: D <= CH * 512
__global__ __launch_bounds__(256) void rmsnorm_forward_kernel(
        const uint16_t* __restrict__ x, const uint16_t* __restrict__ gamma, int N, int D, float eps,
        uint16_t* __restrict__ y, float* __restrict__ rstd_out, uint16_t* residual) {
    const int l = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= N) return;
    const int chunks = D >> 3;
    const au32x4* xr = (const au32x4*)(x + (size_t)row * D);
    au32x4* rr = (au32x4*)(residual + (size_t)row * D);
    au32x4 xv[CH];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = l + 64 * i;
        if (c < chunks) {
            xv[i] = xr[c];
            float f[8];
            unpack8(xv[i], f);
            if (residual) {
                // fused residual add (fused RMSNorm-with-residual kernel): h = x + residual in
                // fp32, rounded once to bf16, stored back as the new residual stream, and it is
                // this stored value that is normalised
                float r[8];
                unpack8(rr[c], r);
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] += r[e];
                xv[i] = pack8(f);
                rr[c] = xv[i];
                unpack8(xv[i], f);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) ss = fmaf(f[e], f[e], ss);
        }
    }
    ss = wave_sum(ss);
    const float rstd = 1.0f / sqrtf(ss / (float)D + eps);
    if (l == 0) rstd_out[row] = rstd;
    const au32x4* gr = (const au32x4*)gamma;
    au32x4* yr = (au32x4*)(y + (size_t)row * D);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = l + 64 * i;
        if (c < chunks) {
            float f[8], g[8];
            unpack8(xv[i], f);
            unpack8(gr[c], g);
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = f[e] * rstd * g[e];
            yr[c] = pack8(f);
        }
    }
}

// ------------------------------------------------------------------------------------------
// RMSNorm backward.  Per row
//   c = mean_j(dy_j gamma_j xhat_j),  dx_j = rstd (gamma_j dy_j - xhat_j c),  xhat = x rstd,
// and each lane adds dy_j xhat_j of its columns to a private dgamma partial.
// WPR wavefronts share a row (1 for D <= 1024, 2 up to 2048, 4 beyond): a lane then never
// holds more than CH = 2 (4 for D > 4096) 16-byte chunks of x and of dy per row, twice (the
// next row is loaded while this one is processed), which keeps four wavefronts per SIMD
// resident at every D -- with one wavefront per row, D = 4096 took all 512 registers of a
// lane and left a single wavefront per SIMD to hide the memory latency.  The wavefronts of a
// row exchange one partial sum per row through LDS (one barrier per row, slots alternate).
// The 4 / WPR row groups of a workgroup walk the rows with a grid stride; at the end the
// groups' dgamma partials are added through LDS and the workgroup writes one partial row;
// dgamma_reduce_kernel sums those rows in a fixed order.
// ------------------------------------------------------------------------------------------
template <int CH, int WPR>
__global__ __launch_bounds__(256) void rmsnorm_backward_kernel(
        const uint16_t* __restrict__ x, const uint16_t* __restrict__ gamma, const float* __restrict__ rstd_in,
        const uint16_t* __restrict__ dy, int N, int D, uint16_t* __restrict__ dx, float* __restrict__ partials,
        const uint16_t* __restrict__ dres) {
    constexpr int G = 4 / WPR;                       // rows a workgroup has in flight
    __shared__ float red[4][64 * 8];
    __shared__ float tsum[2][4];
    const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int g = w / WPR, wr = w % WPR;
    const int chunks = D >> 3;
    const au32x4* gr = (const au32x4*)gamma;
    float dg[CH][8];
#pragma unroll
    for (int i = 0; i < CH; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) dg[i][e] = 0.f;
    // chunk i of this lane: the wavefronts of a row interleave in units of 64 chunks (1 KB)
    auto chunk_of = [&](int i) { return l + 64 * (wr + WPR * i); };

    auto load_row = [&](au32x4 (&xv)[CH], au32x4 (&gv)[CH], int row) {
        const au32x4* xr = (const au32x4*)(x + (size_t)row * D);
        const au32x4* dyr = (const au32x4*)(dy + (size_t)row * D);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = chunk_of(i);
            if (c < chunks) { xv[i] = xr[c]; gv[i] = dyr[c]; }
        }
    };
    // `live` is false for the row groups that have run out of rows while another group of the
    // workgroup still has one: they keep taking part in the barrier.
    auto process_row = [&](const au32x4 (&xv)[CH], const au32x4 (&gv)[CH], int row, bool live, int parity) {
        const float rstd = live ? rstd_in[row] : 0.f;
        float t = 0.f;
        if (live) {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int c = chunk_of(i);
                if (c < chunks) {
                    float xf[8], gf[8], ga[8];
                    unpack8(xv[i], xf);
                    unpack8(gv[i], gf);
                    unpack8(gr[c], ga);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float xh = xf[e] * rstd;
                        t = fmaf(gf[e] * ga[e], xh, t);
                        dg[i][e] = fmaf(gf[e], xh, dg[i][e]);
                    }
                }
            }
        }
        t = wave_sum(t);
        if constexpr (WPR > 1) {
            if (l == 0) tsum[parity][w] = t;
            __syncthreads();
            t = 0.f;
#pragma unroll
            for (int j = 0; j < WPR; ++j) t += tsum[parity][g * WPR + j];
        }
        if (!live) return;
        const float cmean = t / (float)D;
        au32x4* dxr = (au32x4*)(dx + (size_t)row * D);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = chunk_of(i);
            if (c < chunks) {
                float xf[8], gf[8], ga[8], o[8];
                unpack8(xv[i], xf);
                unpack8(gv[i], gf);
                unpack8(gr[c], ga);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = rstd * (ga[e] * gf[e] - xf[e] * rstd * cmean);
                if (dres) {         // gradient arriving through the residual stream, added in fp32
                    float u[8];
                    unpack8(((const au32x4*)(dres + (size_t)row * D))[c], u);
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] += u[e];
                }
                dxr[c] = pack8(o);
            }
        }
    };

    // Every wavefront of the workgroup makes the same number of trips (that of row group 0);
    // a row's x and dy are loaded one trip ahead of their use (two register sets, A and B).
    const int stride = gridDim.x * G;
    const int first = blockIdx.x * G;
    const int trips = first < N ? (N - first + stride - 1) / stride : 0;
    const int row0 = first + g;
    au32x4 xa[CH], ga_[CH], xb[CH], gb[CH];
    if (trips > 0 && row0 < N) load_row(xa, ga_, row0);
    for (int k = 0; k < trips; k += 2) {
        const int r1 = row0 + k * stride, r2 = r1 + stride, r3 = r2 + stride;
        if (k + 1 < trips && r2 < N) load_row(xb, gb, r2);
        process_row(xa, ga_, r1, r1 < N, 0);
        if (k + 1 >= trips) break;
        if (k + 2 < trips && r3 < N) load_row(xa, ga_, r3);
        process_row(xb, gb, r2, r2 < N, 1);
    }

    // add the row groups' partials: per chunk index i the workgroup covers 512 * WPR columns
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        if (64 * WPR * i < chunks) {                 // uniform over the workgroup
#pragma unroll
            for (int e = 0; e < 8; ++e) red[w][l * 8 + e] = dg[i][e];
            __syncthreads();
#pragma unroll
            for (int idx = threadIdx.x; idx < 512 * WPR; idx += 256) {
                const int wr2 = idx >> 9, j = idx & 511;
                const int col = 512 * (wr2 + WPR * i) + j;
                if (col < D) {
                    float sum = 0.f;
#pragma unroll
                    for (int gg = 0; gg < G; ++gg) sum += red[gg * WPR + wr2][j];
                    partials[(size_t)blockIdx.x * D + col] = sum;
                }
            }
            __syncthreads();
        }
    }
}

// dgamma[col] = sum over the workgroups' partial rows, in a fixed order: a workgroup owns 64
// columns; its sixteen wavefronts each add every sixteenth row, eight loads in flight at a
// time (the sum is a chain of dependent loads otherwise: a handful of workgroups reading a
// few megabytes is bound by latency, not bandwidth), then the sixteen sums are added.
__global__ __launch_bounds__(1024) void dgamma_reduce_kernel(const float* __restrict__ partials, int blocks, int D,
                                                             float* __restrict__ dgamma, int accumulate) {
    __shared__ float red[16][64];
    const int c = threadIdx.x & 63, r = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + c;
    float s[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] = 0.f;
    if (col < D) {
        int b = r;
        for (; b + 16 * 7 < blocks; b += 16 * 8) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] += partials[(size_t)(b + 16 * e) * D + col];
        }
        for (; b < blocks; b += 16) s[0] += partials[(size_t)b * D + col];
    }
    red[r][c] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
    __syncthreads();
    if (r == 0 && col < D) {
        float t = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) t += red[e][c];
        dgamma[col] = accumulate ? dgamma[col] + t : t;
    }
}

// ------------------------------------------------------------------------------------------
// Global-norm clipping coefficient, resident on the GPU (gradient-clipping strategies).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sumsq_partial_kernel(const float* __restrict__ g, int64_t n, double* __restrict__ partials) {
    __shared__ double red[4];
    const int64_t n4 = n >> 2;
    const af32x4* g4 = (const af32x4*)g;
    float s = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
        const af32x4 v = g4[i];
        s = fmaf(v[0], v[0], s); s = fmaf(v[1], v[1], s); s = fmaf(v[2], v[2], s); s = fmaf(v[3], v[3], s);
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) { const float t = g[(n4 << 2) + threadIdx.x]; s = fmaf(t, t, s); }
    double d = (double)s;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) d += __shfl_xor(d, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = d;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(64) void sumsq_final_kernel(const double* __restrict__ partials, int blocks,
                                                         double* __restrict__ sumsq, int accumulate) {
    double d = 0.0;
    for (int i = threadIdx.x; i < blocks; i += 64) d += partials[i];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) d += __shfl_xor(d, o);
    if (threadIdx.x == 0) sumsq[0] = accumulate ? sumsq[0] + d : d;
}

__global__ void clip_coef_kernel(const double* __restrict__ sumsq, float max_norm, float eps_norm, float* __restrict__ coef) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        const double c = (double)max_norm / (sqrt(sumsq[0]) + (double)eps_norm);
        coef[0] = c < 1.0 ? (float)c : 1.0f;
    }
}

// ------------------------------------------------------------------------------------------
// Fused AdamW (fused AdamW kernel: every tensor is loaded once and stored once).
// ------------------------------------------------------------------------------------------
struct AdamwArgs {
    float lr, beta1, beta2, eps, decay_factor, inv_bc1, inv_bc2;
};

__device__ __forceinline__ void adamw_one(float& p, float g, float& m, float& v, const AdamwArgs& a) {
    p *= a.decay_factor;                                   // decoupled weight decay, before the update
    m = a.beta1 * m + (1.f - a.beta1) * g;
    v = a.beta2 * v + (1.f - a.beta2) * g * g;
    const float m_hat = m * a.inv_bc1, v_hat = v * a.inv_bc2;
    p -= a.lr * (m_hat / (sqrtf(v_hat) + a.eps));
}

__global__ __launch_bounds__(256) void adamw_kernel(float* __restrict__ param, uint16_t* __restrict__ param_bf16,
                                                    const float* __restrict__ grad, float* __restrict__ m,
                                                    float* __restrict__ v, int64_t n, AdamwArgs a,
                                                    const float* __restrict__ clip_coef) {
    const float clip = clip_coef ? clip_coef[0] : 1.f;
    const int64_t n4 = n >> 2;
    af32x4* p4 = (af32x4*)param;
    const af32x4* g4 = (const af32x4*)grad;
    af32x4* m4 = (af32x4*)m;
    af32x4* v4 = (af32x4*)v;
    // every tensor is touched exactly once: streaming (non-temporal) accesses, two independent
    // 16-byte groups per thread and iteration
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x; i0 < n4; i0 += 2 * stride) {
        const int64_t i1 = i0 + stride;
        const bool two = i1 < n4;
        af32x4 p[2], g[2], mm[2], vv[2];
        p[0] = __builtin_nontemporal_load(p4 + i0); g[0] = __builtin_nontemporal_load(g4 + i0);
        mm[0] = __builtin_nontemporal_load(m4 + i0); vv[0] = __builtin_nontemporal_load(v4 + i0);
        if (two) {
            p[1] = __builtin_nontemporal_load(p4 + i1); g[1] = __builtin_nontemporal_load(g4 + i1);
            mm[1] = __builtin_nontemporal_load(m4 + i1); vv[1] = __builtin_nontemporal_load(v4 + i1);
        }
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            if (k == 1 && !two) break;
            const int64_t i = k == 0 ? i0 : i1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float pe = p[k][e], me = mm[k][e], ve = vv[k][e];
                adamw_one(pe, g[k][e] * clip, me, ve, a);
                p[k][e] = pe; mm[k][e] = me; vv[k][e] = ve;
            }
            __builtin_nontemporal_store(p[k], p4 + i);
            __builtin_nontemporal_store(mm[k], m4 + i);
            __builtin_nontemporal_store(vv[k], v4 + i);
            if (param_bf16) {
                union { __bf16 h[4]; unsigned long long u; } cv;
#pragma unroll
                for (int e = 0; e < 4; ++e) cv.h[e] = (__bf16)p[k][e];
                *(unsigned long long*)(param_bf16 + (i << 2)) = cv.u;
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const int64_t i = (n4 << 2) + threadIdx.x;
        float p = param[i], mm = m[i], vv = v[i];
        adamw_one(p, grad[i] * clip, mm, vv, a);
        param[i] = p; m[i] = mm; v[i] = vv;
        if (param_bf16) { union { __bf16 h; uint16_t u; } cv; cv.h = (__bf16)p; param_bf16[i] = cv.u; }
    }
}

// ------------------------------------------------------------------------------------------
// Measurement aid: a register-only MFMA loop (no LDS, no global memory), the rate the matrix
// cores sustain when nothing else is in the way.  Eight wavefronts per workgroup, eight
// independent 32x32 accumulators per wavefront; the operands are lane-dependent constants.
// ------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 abf16x8;
typedef __attribute__((ext_vector_type(16))) float af32x16;

__global__ __launch_bounds__(512) void mfma_probe_kernel(int iters, float seed, float* __restrict__ sink) {
    abf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(seed + 0.001f * (float)((threadIdx.x * 8 + e) % 61));
        b[e] = (__bf16)(seed - 0.002f * (float)((threadIdx.x * 8 + e) % 53));
    }
    af32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) t += acc[i][r];
    if (t == 12345.678f) sink[0] = t;                 // keeps the loop alive; never true in practice
}

// The same register-only loop with operands taken from memory ONCE, before the loop: four A and
// two B fragments per lane (the 128 x 64 wavefront tile of the contraction kernels: 8 MFMAs on 6
// fragments), 96 bytes per thread from operands[threadIdx.x * 48 ...].  What the buffer holds
// (random normal values, constants, zeros) is the caller's choice: the instruction stream is the
// same, so a difference in rate between buffers is the device's response to operand activity
// (clock / power management), not to the schedule.
__global__ __launch_bounds__(512) void mfma_probe_data_kernel(int iters, const uint16_t* __restrict__ operands,
                                                              float* __restrict__ sink) {
    abf16x8 a[4], b[2];
    const au32x4* src = (const au32x4*)operands + (size_t)threadIdx.x * 6;
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(abf16x8, src[i]);
#pragma unroll
    for (int i = 0; i < 2; ++i) b[i] = __builtin_bit_cast(abf16x8, src[4 + i]);
    af32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i >> 1], b[i & 1], acc[i], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) t += acc[i][r];
    if (t == 12345.678f) sink[0] = t;
}

// ------------------------------------------------------------------------------------------
// Block-wise E4M3 quantisation (block-wise quantisation algorithm of the paper's FP8 section:
// blocks of 128 elements, one scale each, clamp to +-448), with the scale rounded up to a
// power of two so that the block-scaled MFMA can apply it: 2^e, e = ceil(log2(amax / 448)).
// 16 lanes own one block (16 bytes of bf16 each); a block is 256 contiguous input bytes
// because the row length is a multiple of 128.  amax = f x 2^p with 1 <= f < 2 gives
// e = p - 8, plus one when f > 1.75 (448 = 1.75 x 2^8): integer work on the fp32 bit pattern.
// ------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) unsigned int q_u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int q_u32x2;

// Scale layout: [D / 128][groups = ceil(rows / 128)][32][4] bytes, byte j of dword i of group g =
// row 128 g + 32 j + i (the order the block-scaled MFMA loop reads them in); entries of rows
// past the matrix in the last group are set to 127.
__global__ __launch_bounds__(256) void quantize_e4m3_kernel(const uint16_t* __restrict__ x, int64_t n_blocks,
                                                            int blocks_per_row, int rows, int groups,
                                                            uint8_t* __restrict__ q, uint8_t* __restrict__ scales) {
    const int64_t gb = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;       // 128-element block
    const int j = threadIdx.x & 15;
    const bool live = gb < n_blocks;
    q_u32x4 v = {0u, 0u, 0u, 0u};
    if (live) v = __builtin_nontemporal_load((const q_u32x4*)(x + gb * 128 + j * 8));
    float f[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(v[i] << 16);
        f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
    }
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(f[i]));
#pragma unroll
    for (int o = 1; o <= 8; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    const uint32_t ab = __float_as_uint(amax);
    int e = (int)(ab >> 23) - 127 - 8 + ((ab & 0x7fffffu) > 0x600000u ? 1 : 0);
    e = ab == 0u ? 0 : e;
    e = e < -127 ? -127 : (e > 127 ? 127 : e);
    int packed[2] = {0, 0};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float a = fminf(fmaxf(ldexpf(f[2 * i], -e), -448.f), 448.f);
        const float b = fminf(fmaxf(ldexpf(f[2 * i + 1], -e), -448.f), 448.f);
        if (i & 1) packed[i >> 1] = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, packed[i >> 1], true);
        else packed[i >> 1] = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, packed[i >> 1], false);
    }
    if (!live) return;
    const q_u32x2 out = {(unsigned)packed[0], (unsigned)packed[1]};
    __builtin_nontemporal_store(out, (q_u32x2*)(q + gb * 128 + j * 8));
    if (j == 0) {
        const int row = (int)(gb / blocks_per_row);
        const int kb = (int)(gb - (int64_t)row * blocks_per_row);
        uint8_t* plane = scales + (size_t)kb * groups * 128;
        plane[((size_t)(row >> 7) * 32 + (row & 31)) * 4 + ((row >> 5) & 3)] = (uint8_t)(e + 127);
        if (row == rows - 1)
            for (int r = rows; r < groups * 128; ++r)
                plane[((size_t)(r >> 7) * 32 + (r & 31)) * 4 + ((r >> 5) & 3)] = 127;
    }
}

static bool norm_shape_ok(int64_t N, int64_t D) {
    return N > 0 && D > 0 && D % 64 == 0 && D <= (int64_t)kNormMaxChunks * 512 && N <= ((int64_t)1 << 30);
}

static int norm_waves_per_row(int64_t D) { return D <= 1024 ? 1 : D <= 2048 ? 2 : 4; }

// Workgroups of the backward: one per 4 / WPR rows until the cap (the partial dgamma rows they
// write are the workspace, and are read once more by the reduction).
static int norm_backward_blocks(int64_t N, int64_t D) {
    const int per = 4 / norm_waves_per_row(D);
    const int64_t want = (N + per - 1) / per;
    const int64_t cap = per == 4 ? kNormBackwardBlocks : kNormBackwardBlocksWide;
    return (int)(want < cap ? want : cap);
}

}  // namespace cce

using namespace cce;

extern "C" {

size_t cce_rmsnorm_workspace_bytes(int64_t N, int64_t D) {
    if (!norm_shape_ok(N, D)) return 0;
    return (size_t)round_up((int64_t)norm_backward_blocks(N, D) * D * 4, 256);
}

static int rmsnorm_forward_impl(const void* x, void* residual, const void* gamma, int64_t N, int64_t D, float eps,
                                void* y, float* rstd, void* stream_) {
    if (!x || !gamma || !y || !rstd) return CCE_ERR_INVALID;
    if (N <= 0 || D <= 0 || !(eps >= 0.f)) return CCE_ERR_INVALID;
    if (!norm_shape_ok(N, D)) return CCE_ERR_UNSUPPORTED;
    if (((uintptr_t)x | (uintptr_t)gamma | (uintptr_t)y) & 15) return CCE_ERR_INVALID;
    if ((uintptr_t)rstd & 3) return CCE_ERR_INVALID;
    const dim3 grid((unsigned)((N + 3) / 4));
    hipStream_t stream = (hipStream_t)stream_;
#define CCE_NORM_FWD(CH) hipLaunchKernelGGL(rmsnorm_forward_kernel<CH>, grid, dim3(256), 0, stream, \
        (const uint16_t*)x, (const uint16_t*)gamma, (int)N, (int)D, eps, (uint16_t*)y, rstd, (uint16_t*)residual)
    if (D <= 1024) CCE_NORM_FWD(2); else if (D <= 2048) CCE_NORM_FWD(4); else if (D <= 4096) CCE_NORM_FWD(8); else CCE_NORM_FWD(16);
#undef CCE_NORM_FWD
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_rmsnorm_forward(const void* x, const void* gamma, int64_t N, int64_t D, float eps,
                        void* y, float* rstd, void* stream_) {
    return rmsnorm_forward_impl(x, nullptr, gamma, N, D, eps, y, rstd, stream_);
}

int cce_rmsnorm_residual_forward(const void* x, void* residual, const void* gamma, int64_t N, int64_t D, float eps,
                                 void* y, float* rstd, void* stream_) {
    if (!residual || ((uintptr_t)residual & 15)) return CCE_ERR_INVALID;
    return rmsnorm_forward_impl(x, residual, gamma, N, D, eps, y, rstd, stream_);
}

static int rmsnorm_backward_impl(const void* x, const void* gamma, const float* rstd, const void* dy, const void* dres,
                                 int64_t N, int64_t D, void* dx, float* dgamma, int accumulate_dgamma,
                                 void* workspace, size_t workspace_bytes, void* stream_) {
    if (!x || !gamma || !rstd || !dy || !dx || !dgamma || !workspace) return CCE_ERR_INVALID;
    if (N <= 0 || D <= 0) return CCE_ERR_INVALID;
    if (!norm_shape_ok(N, D)) return CCE_ERR_UNSUPPORTED;
    if (((uintptr_t)x | (uintptr_t)gamma | (uintptr_t)dy | (uintptr_t)dx) & 15) return CCE_ERR_INVALID;
    if (((uintptr_t)rstd | (uintptr_t)dgamma) & 3) return CCE_ERR_INVALID;
    if (((uintptr_t)workspace & 255) || workspace_bytes < cce_rmsnorm_workspace_bytes(N, D)) return CCE_ERR_INVALID;
    hipStream_t stream = (hipStream_t)stream_;
    const int blocks = norm_backward_blocks(N, D);
    float* partials = (float*)workspace;
#define CCE_NORM_BWD(CH, WPR) hipLaunchKernelGGL((rmsnorm_backward_kernel<CH, WPR>), dim3(blocks), dim3(256), 0, stream, \
        (const uint16_t*)x, (const uint16_t*)gamma, rstd, (const uint16_t*)dy, (int)N, (int)D, (uint16_t*)dx, partials, \
        (const uint16_t*)dres)
    if (D <= 1024) CCE_NORM_BWD(2, 1); else if (D <= 2048) CCE_NORM_BWD(2, 2); else if (D <= 4096) CCE_NORM_BWD(2, 4);
    else CCE_NORM_BWD(4, 4);
#undef CCE_NORM_BWD
    hipLaunchKernelGGL(dgamma_reduce_kernel, dim3((unsigned)((D + 63) / 64)), dim3(1024), 0, stream,
                       (const float*)partials, blocks, (int)D, dgamma, accumulate_dgamma ? 1 : 0);
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_rmsnorm_backward(const void* x, const void* gamma, const float* rstd, const void* dy,
                         int64_t N, int64_t D, void* dx, float* dgamma, int accumulate_dgamma,
                         void* workspace, size_t workspace_bytes, void* stream_) {
    return rmsnorm_backward_impl(x, gamma, rstd, dy, nullptr, N, D, dx, dgamma, accumulate_dgamma,
                                 workspace, workspace_bytes, stream_);
}

int cce_rmsnorm_residual_backward(const void* h, const void* gamma, const float* rstd, const void* dy,
                                  const void* d_residual, int64_t N, int64_t D, void* dh, float* dgamma,
                                  int accumulate_dgamma, void* workspace, size_t workspace_bytes, void* stream_) {
    if ((uintptr_t)d_residual & 15) return CCE_ERR_INVALID;
    return rmsnorm_backward_impl(h, gamma, rstd, dy, d_residual, N, D, dh, dgamma, accumulate_dgamma,
                                 workspace, workspace_bytes, stream_);
}

size_t cce_sumsq_workspace_bytes(void) { return (size_t)kSumsqBlocks * sizeof(double); }

int cce_grad_sumsq(const float* grad, int64_t n, double* sumsq, int accumulate,
                   void* workspace, size_t workspace_bytes, void* stream_) {
    if (!grad || !sumsq || !workspace || n <= 0) return CCE_ERR_INVALID;
    if (((uintptr_t)grad & 15) || ((uintptr_t)sumsq & 7) || ((uintptr_t)workspace & 255)) return CCE_ERR_INVALID;
    if (workspace_bytes < cce_sumsq_workspace_bytes()) return CCE_ERR_INVALID;
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t want = ((n >> 2) + 255) / 256;
    const int blocks = (int)(want < 1 ? 1 : (want < kSumsqBlocks ? want : kSumsqBlocks));
    hipLaunchKernelGGL(sumsq_partial_kernel, dim3(blocks), dim3(256), 0, stream, grad, n, (double*)workspace);
    hipLaunchKernelGGL(sumsq_final_kernel, dim3(1), dim3(64), 0, stream, (const double*)workspace, blocks, sumsq,
                       accumulate ? 1 : 0);
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_clip_coef(const double* sumsq, float max_norm, float eps_norm, float* clip_coef, void* stream_) {
    if (!sumsq || !clip_coef || !(max_norm > 0.f) || !(eps_norm >= 0.f)) return CCE_ERR_INVALID;
    hipLaunchKernelGGL(clip_coef_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream_, sumsq, max_norm, eps_norm, clip_coef);
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

size_t cce_fp8_scale_bytes(int64_t rows, int64_t D) {
    if (rows <= 0 || D <= 0 || D % 128 != 0 || rows > ((int64_t)1 << 30)) return 0;
    return (size_t)(D / 128) * (size_t)((rows + 127) / 128) * 128u;
}

int cce_quantize_e4m3(const void* x, int64_t rows, int64_t D, void* q, void* scales, void* stream_) {
    if (!x || !q || !scales || rows <= 0 || D <= 0) return CCE_ERR_INVALID;
    if (D % 128 != 0 || rows > ((int64_t)1 << 30) || rows * D >= ((int64_t)1 << 40)) return CCE_ERR_UNSUPPORTED;
    if ((((uintptr_t)x | (uintptr_t)q) & 15) || ((uintptr_t)scales & 3)) return CCE_ERR_INVALID;
    const int64_t n_blocks = rows * (D / 128);
    const int64_t grid = (n_blocks * 16 + 255) / 256;
    if (grid > 0x7fffffff) return CCE_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(quantize_e4m3_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream_,
                       (const uint16_t*)x, n_blocks, (int)(D / 128), (int)rows, (int)((rows + 127) / 128),
                       (uint8_t*)q, (uint8_t*)scales);
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_device_info(int* compute_units, int* clock_khz) {
    if (!compute_units || !clock_khz) return CCE_ERR_INVALID;
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return CCE_ERR_HIP;
    if (!hip_ok(hipDeviceGetAttribute(compute_units, hipDeviceAttributeMultiprocessorCount, dev))) return CCE_ERR_HIP;
    if (!hip_ok(hipDeviceGetAttribute(clock_khz, hipDeviceAttributeClockRate, dev))) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_mfma_probe(int workgroups, int iters, float* sink, void* stream_) {
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || !sink) return CCE_ERR_INVALID;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream_, iters, 0.5f, sink);
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_mfma_probe_data(int workgroups, int iters, const void* operands, float* sink, void* stream_) {
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || !sink || !operands) return CCE_ERR_INVALID;
    if ((uintptr_t)operands & 15) return CCE_ERR_INVALID;
    hipLaunchKernelGGL(mfma_probe_data_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream_, iters,
                       (const uint16_t*)operands, sink);
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

int cce_adamw_step(float* param, void* param_bf16, const float* grad, float* m, float* v, int64_t n,
                   float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                   const float* clip_coef, void* stream_) {
    if (!param || !grad || !m || !v || n <= 0 || step < 1) return CCE_ERR_INVALID;
    if (((uintptr_t)param | (uintptr_t)grad | (uintptr_t)m | (uintptr_t)v) & 15) return CCE_ERR_INVALID;
    if ((uintptr_t)param_bf16 & 7) return CCE_ERR_INVALID;
    if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f && eps >= 0.f && lr >= 0.f && weight_decay >= 0.f))
        return CCE_ERR_INVALID;
    AdamwArgs a;
    a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps;
    a.decay_factor = 1.f - lr * weight_decay;
    a.inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
    a.inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
    const int64_t want = ((n >> 2) + 255) / 256;
    const int blocks = (int)(want < 1 ? 1 : (want < 131072 ? want : 131072));
    hipLaunchKernelGGL(adamw_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream_,
                       param, (uint16_t*)param_bf16, grad, m, v, n, a, clip_coef);
    if (!hip_ok(hipGetLastError())) return CCE_ERR_HIP;
    return CCE_OK;
}

}  // extern "C"
