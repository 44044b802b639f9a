// MFMA main loop shared by the four contractions of the fused LM-head + cross-entropy path
// (logit tile of the chunked forward algorithm, its recomputation in the backward
// algorithm, and the two gradient products dH = G W and dW = G^T H).
//
// One workgroup = 512 threads = 8 wavefronts arranged WM x WN, computing a BM x BN fp32 tile
// C[m, n] = sum_k A(m, k) * B(n, k) with v_mfma_f32_32x32x16_bf16.  Each wavefront owns
// TM x TN blocks of 32 x 32 (16 accumulator registers per block and lane).
//
// Operands arrive in one of two global layouts:
//   K-major : element (free f, k) at base[f * ld + k]   (k contiguous)  -- H and W in the
//             logit products, G in dH
//   K-slow  : element (k, free f) at base[k * ld + f]   (f contiguous)  -- W in dH, G and H
//             in dW; fragments are then fetched with the LDS transpose read
//             (ds_read_b64_tr_b16), so no transposed copy of any tensor is ever made.
//
// K is walked in slices of 64.  A slice of both operands is brought straight from global
// memory into LDS (global_load_lds_dwordx4: 16 B per lane, a wavefront fills 1 KB of
// consecutive LDS), double buffered: the loads of slice t+1 are issued before the MFMAs of
// slice t.  Because the LDS side of such a load is fixed (lane * 16 B), the
// bank-conflict-avoiding swizzle is applied on the global side: the lane that fills
// physical 16-byte chunk p of a row fetches logical chunk p ^ f(row).
//   K-major stage: [R rows][128 B]; f(row) = (row >> 1) & 7, so that the 16 lanes served
//                  per LDS cycle by a ds_read_b128 (16 rows, same logical chunk) cover all
//                  64 banks.
//   K-slow  stage: [64 k-rows][2R B]; logical chunk c is stored at c ^ ((k & 3) << 2), so
//                  that the 4 k-rows x 64 B touched per cycle by a transpose read fall in
//                  different quarters of the bank space.
// Rows / columns past the edge of a matrix are clamped to the last valid one (their
// products are discarded or meet zero padding in the other operand), so the loop has a
// single code path for full and ragged tiles.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace cce {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kBK = 64;           // K slice
constexpr int kThreads = 512;     // 8 wavefronts

#define CCE_LDS __attribute__((address_space(3)))
#define CCE_GLOBAL __attribute__((address_space(1)))

// KG_ > 1 splits the k16 steps of every slice between KG_ groups of wavefronts that all work
// on the same output positions (their accumulators are summed once, after the loop): a
// 256 x 128 tile then keeps the 128 x 64 wavefront tile of the 256 x 256 one, i.e. 0.75
// instead of 1 LDS fragment read per MFMA and 8 instead of 4 independent accumulators.
template <int WM_, int WN_, int TM_, int TN_, int STAGES_, int KG_ = 1>
struct TileCfg {
    static_assert(WM_ * WN_ * KG_ == 8, "eight wavefronts per workgroup");
    static_assert(KG_ == 1 || KG_ == 2, "one or two K groups");
    static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_, STAGES = STAGES_, KG = KG_;
    static constexpr int kSteps = 4 / KG_;                      // k16 steps per slice and wavefront
    static constexpr int BM = WM_ * TM_ * 32;
    static constexpr int BN = WN_ * TN_ * 32;
    static constexpr int kAStage = BM * kBK * 2;
    static constexpr int kBStage = BN * kBK * 2;
    static constexpr int kStage = kAStage + kBStage;
    static constexpr int kLdsBytes = STAGES_ * kStage;
    static constexpr int kLoadsPerSlice = BM / 64 + BN / 64;   // 16-byte loads per thread
    static_assert(kLdsBytes <= 160 * 1024, "stages must fit the 160 KB LDS");
};
typedef TileCfg<2, 4, 4, 2, 2> TileBig;      // 256 x 256, wave tile 128 x 64, 2 x 64 KB stages
typedef TileCfg<2, 2, 4, 2, 3, 2> TileNarrow; // 256 x 128, wave tile 128 x 64, 2 K groups, 3 x 48 KB stages

// Wavefront coordinates inside the workgroup: K group, then position along M and N.
template <class Cfg> __device__ __forceinline__ int wave_kg() { return (threadIdx.x >> 6) / (Cfg::WM * Cfg::WN); }
template <class Cfg> __device__ __forceinline__ int wave_m() { return ((threadIdx.x >> 6) % (Cfg::WM * Cfg::WN)) / Cfg::WN; }
template <class Cfg> __device__ __forceinline__ int wave_n() { return ((threadIdx.x >> 6) % (Cfg::WM * Cfg::WN)) % Cfg::WN; }

__device__ __forceinline__ void load16_to_lds(const char* g, CCE_LDS char* lds_wave_base) {
    // global_load_lds_dwordx4: lane i's 16 bytes land at lds_wave_base + 16 * i
    // (lds_wave_base is wave-uniform and travels in M0).
    // Written as inline assembly on purpose: when the compiler sees this load it makes
    // every later LDS read it cannot disambiguate (the transpose reads in particular) wait
    // for ALL outstanding global->LDS loads (s_waitcnt vmcnt(0)), which serialises the
    // prefetch of the next K slice with the current one.  The main loop orders these
    // loads against the LDS reads itself (barrier_pending_loads).
    const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_wave_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(g), "s"(m0) : "memory", "m0");
}

// The same load with the address split as the instruction takes it: a wave-uniform 64-bit base in
// scalar registers plus a 32-bit per-lane byte offset; m0_value is the wave-uniform LDS destination.
// With the base advanced per K slice on the scalar unit and the per-lane offsets constant, a load
// costs no vector-ALU instruction at all (the full-address form above needs an offset add, a
// 64-bit add and, for the LDS destination, an add and a readfirstlane per load).
__device__ __forceinline__ void load16_to_lds_sbase(const char* uniform_base, uint32_t lane_offset, uint32_t m0_value) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(lane_offset), "s"(uniform_base), "s"(m0_value) : "memory", "m0");
}

// One operand (R = 128 or 256 free indices) of one workgroup tile: global -> LDS.
// MAPPED (K-slow only): the k-rows are reached through a row map (kmap, kzero).
template <bool KMAJOR, int R, bool MAPPED = false>
struct OperandTile {
    static_assert(!(KMAJOR && MAPPED), "only a K-slow operand carries a k-row map");
    static constexpr int NL = R / 64;   // 16-byte loads per thread and K slice
    const char* base;       // matrix base address
    uint32_t ld_bytes;      // leading dimension in bytes
    uint32_t off[NL];       // K-major: clamped row offset + swizzled chunk; K-slow: clamped column offset
    int krow[NL];           // K-slow: k-row inside a slice handled by load i
    uint32_t slow_off[NL];  // K-slow: krow[i] * row pitch + off[i] (full slices are loaded from a uniform base)
    int k_last;             // K-slow: last valid k (rows beyond are clamped to it)
    const CCE_LDS int32_t* kmap;   // K-slow, optional: k-row k is matrix row kmap[k]; where it holds -1 the
    const char* kzero;             // row is read from kzero instead: a row of zeros as long as a matrix row

    // free0: first free index of the tile; free_n: number of valid free indices in the matrix
    // (a multiple of 8, at least 8, for a K-slow operand); k_n: valid K extent.
    // row_map (K-major operands only): free index f is fetched from matrix row row_map[f] (row 0
    // where the map holds -1; such rows are padding whose products the caller discards).
    __device__ __forceinline__ void init(const void* p, int64_t ld, int free0, int free_n, int k_n,
                                         const int32_t* row_map = nullptr) {
        base = (const char*)p;
        ld_bytes = (uint32_t)(ld * 2);
        k_last = k_n - 1;
        kmap = nullptr;
        kzero = nullptr;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        if (KMAJOR) {
            const int sw = ((lane >> 4) & 3) | ((wave & 1) << 2);
            const int c = (lane & 7) ^ sw;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                int row = free0 + 64 * i + 8 * wave + (lane >> 3);
                row = row < free_n ? row : free_n - 1;
                if (row_map) {
                    const int mapped = row_map[row];
                    row = mapped < 0 ? 0 : mapped;
                }
                off[i] = (uint32_t)row * ld_bytes + (uint32_t)c * 16u;
                krow[i] = 0;
                slow_off[i] = 0;
            }
        } else {
            constexpr int CR = R / 8;            // 16-byte chunks per k-row
            constexpr int RPL = 512 / R;         // k-rows per wavefront load
            const int sub = lane / CR;           // k-row inside the wavefront load
            const int k3 = (RPL * wave + sub) & 3;
            const int c = (lane % CR) ^ (k3 << 2);
            int col = free0 + c * 8;
            col = col <= free_n - 8 ? col : free_n - 8;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                off[i] = (uint32_t)col * 2u;
                krow[i] = (wave + 8 * i) * RPL + sub;
                slow_off[i] = (uint32_t)krow[i] * ld_bytes + off[i];
            }
        }
    }

    // K slices [0, full_slices()) lie entirely inside the operand's valid K extent (every slice of a
    // K-major operand does: its extent is padded to the slice).
    __device__ __forceinline__ int full_slices() const { return KMAJOR ? 0x7fffffff : (k_last + 1) / kBK; }

    // Issue this thread's loads of the K slice starting at k0 into `stage` (LDS).  FULL (compile time):
    // the caller knows that the slice is one of full_slices().
    template <bool FULL = false>
    __device__ __forceinline__ void issue(CCE_LDS char* stage, int k0) const {
        const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        const uint32_t lds0 = (uint32_t)(uintptr_t)stage + (uint32_t)wave * 1024u;     // wave-uniform
        if (KMAJOR) {
            // uniform base = matrix base + this slice's K offset; lane offsets are those of init()
            const char* sb = base + (size_t)((uint32_t)k0 * 2u);
#pragma unroll
            for (int i = 0; i < NL; ++i) load16_to_lds_sbase(sb, off[i], lds0 + (uint32_t)i * 8192u);
            return;
        }
        if (!MAPPED && (FULL || k0 + 63 <= k_last)) {
            // a full slice of a K-slow operand: uniform base = row k0, lane offset = its k-row inside
            // the slice times the row pitch plus its column offset
            const char* sb = base + (size_t)k0 * ld_bytes;
#pragma unroll
            for (int i = 0; i < NL; ++i) load16_to_lds_sbase(sb, slow_off[i], lds0 + (uint32_t)i * 8192u);
            return;
        }
        if constexpr (MAPPED) {
            // mapped k-rows: lane offset = mapped row times the row pitch plus the
            // column offset, from the matrix base -- unless some lane of the wavefront has a k-row that
            // maps to no row (only behind the last valid row of the whole problem), which takes the
            // per-lane form below
            int m[NL];
            int any = 0;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                int k = k0 + krow[i];
                k = k < k_last ? k : k_last;
                m[i] = kmap[k];
                any |= m[i];
            }
            if (__builtin_amdgcn_ballot_w64(any < 0) == 0) {
#pragma unroll
                for (int i = 0; i < NL; ++i)
                    load16_to_lds_sbase(base, (uint32_t)m[i] * ld_bytes + off[i], lds0 + (uint32_t)i * 8192u);
                return;
            }
        }
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const char* g;
            if (KMAJOR) {
                g = base + (size_t)(off[i] + (uint32_t)k0 * 2u);
            } else {
                int k = k0 + krow[i];
                k = k < k_last ? k : k_last;
                g = base + (size_t)((uint32_t)k * ld_bytes + off[i]);
                if constexpr (MAPPED) {
                    // a k-row that stands for no matrix row must not fetch one: whatever that row
                    // holds (NaN included) would meet the other operand's zero in the MFMA
                    const int mapped = kmap[k];
                    g = mapped < 0 ? kzero + off[i] : base + (size_t)((uint32_t)mapped * ld_bytes + off[i]);
                }
            }
            load16_to_lds(g, stage + (wave + 8 * i) * 1024);
        }
    }
};

// Per-lane LDS byte offsets of the MFMA fragments of one operand, relative to its stage.
// A wavefront of K group kg reads the k16 steps kk = j * KG + kg, j = 0 .. STEPS - 1.
template <bool KMAJOR, int R, int NB, int STEPS, int KG>
struct FragAddr {
    uint32_t a[KMAJOR ? STEPS : NB];   // K-major: one per step j; K-slow: one per 32-wide block

    // tile_off: first row/column of this wave's sub-tile inside the R-wide tile.
    __device__ __forceinline__ void init(int tile_off, int kg) {
        const int l = threadIdx.x & 63;
        if (KMAJOR) {
            const int row = tile_off + (l & 31);
            const int s = ((l & 31) >> 1) & 7;
#pragma unroll
            for (int j = 0; j < STEPS; ++j) {
                const int kk = j * KG + kg;
                a[j] = (uint32_t)(row * 128 + (((2 * kk + (l >> 5)) ^ s) << 4));
            }
        } else {
            const int q = l >> 4, jj = l & 15;
            const int krow = 16 * kg + 8 * (q >> 1) + (jj >> 2);
            const int within = (jj & 1) * 8;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int col = tile_off + b * 32 + 16 * (q & 1) + 4 * (jj & 3);
                const int pc = (col >> 3) ^ ((jj >> 2) << 2);
                a[b] = (uint32_t)(krow * (2 * R) + pc * 16 + within);
            }
        }
    }

    // Fragment of 32-wide block b for this wave's step j of the slice held at `op` (LDS):
    // lane l gets elements (free = block base + l % 32, k = 16 kk + 8 (l / 32) + 0..7).
    __device__ __forceinline__ bf16x8 load(const CCE_LDS char* op, int b, int j) const {
        if (KMAJOR) {
            return *(const CCE_LDS bf16x8*)(op + a[j] + b * (32 * 128));
        } else {
            const CCE_LDS char* p = op + a[b] + j * (KG * 16 * 2 * R);
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CCE_LDS s16x4*)p);
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CCE_LDS s16x4*)(p + 4 * 2 * R));
            s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
        }
    }
};

// Scheduling hint: one MFMA, then PER LDS reads, repeated (compile-time recursion because
// the builtin wants constant arguments).
template <int I, int N_MFMA, int N_READS, int PER>
struct SchedInterleave {
    static __device__ __forceinline__ void run() {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if constexpr (I * PER < N_READS)
            __builtin_amdgcn_sched_group_barrier(0x100, ((I + 1) * PER <= N_READS ? PER : N_READS - I * PER), 0);
        if constexpr (I + 1 < N_MFMA) SchedInterleave<I + 1, N_MFMA, N_READS, PER>::run();
    }
};

// Workgroup barrier that first waits until at most `PENDING` of this thread's global->LDS
// loads are still in flight and all of its LDS reads have returned.  (__syncthreads would
// wait for every outstanding load, which defeats a prefetch distance of more than one
// slice.)  The "memory" clobber keeps the compiler from moving LDS accesses across it.
template <int PENDING>
__device__ __forceinline__ void barrier_pending_loads() {
    static_assert(PENDING >= 0 && PENDING < 64, "vmcnt is a 6-bit counter");
    if constexpr (PENDING == 0) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" :: "n"(PENDING) : "memory");
}

// Workgroup barrier for data exchanged through LDS only: waits for this thread's LDS
// traffic, not for its outstanding global loads (which __syncthreads would also drain).
__device__ __forceinline__ void barrier_lds_only() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// acc[bm][bn] += A-tile * B-tile^T over K slices [0, ceil(k_total / 64)).  The operands
// clamp / meet zero padding so that reads past k_total contribute zero.
// `smem` must hold Cfg::kLdsBytes.  Ends with a workgroup barrier, after which the LDS may
// be reused by the caller.
//
// Software pipeline.  Global -> LDS runs STAGES - 1 K slices ahead (STAGES LDS stages; a
// slice of a 256 x 128 tile lasts only ~0.5 us, less than a trip to L2 / HBM, hence three
// stages there).  LDS -> registers runs one k16 step ahead (two fragment sets): while the
// MFMAs of step kk run, the fragments of step kk + 1 are already being read.  The one
// workgroup barrier per slice sits before the MFMAs of a wavefront's last step: by then every
// wavefront has issued (and waited for) all its LDS reads of the current stage, so after
// the barrier (a) the next slice's data, whose loads each wavefront has waited for, is
// visible to all and its first fragments can be read under those last MFMAs, and (b)
// the current stage may be overwritten by the loads issued at the top of the next
// iteration.
template <class Cfg, bool A_KMAJOR, bool B_KMAJOR, bool PEEL = false, class OpA, class OpB>
__device__ __forceinline__ void gemm_mainloop(f32x16 (&acc)[Cfg::TM][Cfg::TN], const OpA& A, const OpB& B,
                                               int k_total, CCE_LDS char* smem) {
    constexpr int S = Cfg::STAGES;
    constexpr int kAhead = (S - 2) * Cfg::kLoadsPerSlice;    // loads that may stay in flight
    constexpr int SPS = Cfg::kSteps;
    FragAddr<A_KMAJOR, Cfg::BM, Cfg::TM, SPS, Cfg::KG> fa;
    FragAddr<B_KMAJOR, Cfg::BN, Cfg::TN, SPS, Cfg::KG> fb;
    fa.init(wave_m<Cfg>() * (Cfg::TM * 32), wave_kg<Cfg>());
    fb.init(wave_n<Cfg>() * (Cfg::TN * 32), wave_kg<Cfg>());

    const int KT = (k_total + kBK - 1) / kBK;
#pragma unroll
    for (int s = 0; s < S - 1; ++s) {
        if (s < KT) {
            A.issue(smem + s * Cfg::kStage, s * kBK);
            B.issue(smem + s * Cfg::kStage + Cfg::kAStage, s * kBK);
        }
    }
    if (KT >= S - 1) barrier_pending_loads<kAhead>();
    else barrier_pending_loads<0>();

    bf16x8 af[2][Cfg::TM], bfr[2][Cfg::TN];
#pragma unroll
    for (int bm = 0; bm < Cfg::TM; ++bm) af[0][bm] = fa.load(smem, bm, 0);
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) bfr[0][bn] = fb.load(smem + Cfg::kAStage, bn, 0);

    int cur_s = 0;                       // stage holding slice kt
    // One K slice.  more: slice kt + S - 1 exists and is requested during this one (a bool, or a
    // std::true_type / std::false_type where the caller knows it at compile time).
    auto slice = [&](int kt, auto more_tag, auto full_tag) {
        const bool MORE = more_tag;
        constexpr bool FULL = decltype(full_tag)::value;      // the requested slice is a full one of both operands
        CCE_LDS char* cur = smem + cur_s * Cfg::kStage;
        const int nxt_s = (cur_s + 1 == S) ? 0 : cur_s + 1;
        CCE_LDS char* nxt = smem + nxt_s * Cfg::kStage;
        const int ld_s = (cur_s == 0) ? S - 1 : cur_s - 1;       // stage of slice kt - 1, free again
        if (MORE) {
            A.template issue<FULL>(smem + ld_s * Cfg::kStage, (kt + S - 1) * kBK);
            B.template issue<FULL>(smem + ld_s * Cfg::kStage + Cfg::kAStage, (kt + S - 1) * kBK);
        }
#pragma unroll
        for (int kk = 0; kk < SPS; ++kk) {
            const int c = kk & 1, n = c ^ 1;
            if (kk < SPS - 1) {
#pragma unroll
                for (int bm = 0; bm < Cfg::TM; ++bm) af[n][bm] = fa.load(cur, bm, kk + 1);
#pragma unroll
                for (int bn = 0; bn < Cfg::TN; ++bn) bfr[n][bn] = fb.load(cur + Cfg::kAStage, bn, kk + 1);
            } else {
                // slice kt + 1 must have landed; younger slices may still be in flight
                if (MORE) barrier_pending_loads<kAhead>();
                else barrier_pending_loads<0>();
#pragma unroll
                for (int bm = 0; bm < Cfg::TM; ++bm) af[n][bm] = fa.load(nxt, bm, 0);
#pragma unroll
                for (int bn = 0; bn < Cfg::TN; ++bn) bfr[n][bn] = fb.load(nxt + Cfg::kAStage, bn, 0);
            }
#pragma unroll
            for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
                for (int bn = 0; bn < Cfg::TN; ++bn)
                    acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[c][bm], bfr[c][bn], acc[bm][bn], 0, 0, 0);
            // issue order for the scheduler: the LDS reads of the next step are spread
            // one (or two) at a time behind the first MFMAs of this step
            constexpr int kReads = Cfg::TM * (A_KMAJOR ? 1 : 2) + Cfg::TN * (B_KMAJOR ? 1 : 2);
            constexpr int kMfma = Cfg::TM * Cfg::TN;
            constexpr int kPer = (kReads + kMfma - 1) / kMfma;
            SchedInterleave<0, kMfma, kReads, kPer>::run();
        }
        cur_s = nxt_s;
    };
    if constexpr (PEEL) {
        // The last S - 1 slices request nothing: peeled off, so that neither loop body branches on it.
        // Pays in the contraction kernels (2.0 - 2.6 % per launch); the forward and the gradient-tile
        // kernel were 0.5 - 1 % faster with the one loop below.
        // Likewise the slices whose request is a full slice of both operands (all but a ragged last one)
        // run a body whose loads need no clamping of k-rows, hence no branch.
        const int n_more = KT - (S - 1) > 0 ? KT - (S - 1) : 0;
        const int fa_n = A.full_slices(), fb_n = B.full_slices();
        int n_full = (fa_n < fb_n ? fa_n : fb_n) - (S - 1);          // request kt + S - 1 < full slices
        n_full = n_full < 0 ? 0 : (n_full < n_more ? n_full : n_more);
        for (int kt = 0; kt < n_full; ++kt) slice(kt, std::true_type{}, std::true_type{});
        for (int kt = n_full; kt < n_more; ++kt) slice(kt, std::true_type{}, std::false_type{});
        for (int kt = n_more; kt < KT; ++kt) slice(kt, std::false_type{}, std::false_type{});
    } else {
        for (int kt = 0; kt < KT; ++kt) slice(kt, kt + S - 1 < KT, std::false_type{});
    }
    barrier_pending_loads<0>();
}

// ------------------------------------------------------------------------------------------
// FP8 (E4M3) variant of the main loop for two K-major operands with block scales: one
// power-of-two scale (a biased exponent byte, as the block-scaled MFMA takes it) per row and
// 128 consecutive K elements.  v_mfma_scale_f32_32x32x64_f8f6f4 multiplies 64 K values per
// instruction and applies both operands' scales itself, at twice the bf16 rate for the same
// LDS and global traffic per instruction: a 128-byte row of a stage now holds 128 K values,
// so the stage geometry, the global->LDS loads and the swizzle are those of the bf16 loop
// (the operands are handed in as bf16 matrices of half the width), and a K slice is 128.
//
// A lane's 32 operand bytes are the two 16-byte fragments the bf16 loop would read for two
// consecutive k16 steps.  Which K positions the hardware assigns to them does not matter:
// A and B use the same assignment, a dot product does not depend on the order of its terms,
// and all 64 K values of an instruction lie in one 128-block, i.e. share one scale per row.
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

// Block scales of a quantised matrix, in the order the block-scaled MFMA consumes them:
// [D / 128 blocks][ceil(rows / 128) groups][32][4] bytes -- byte j of dword i of a group is the
// exponent byte of row 128 g + 32 j + i.  A wavefront whose 32-row blocks start at a multiple
// of 128 rows then gets the scales of four blocks with ONE dword load per lane and 128-block,
// and picks block j with the instruction's byte selector.
struct ScaleGroup {
    const uint32_t* p;      // this lane's dword of K block 0
    uint32_t step;          // dwords from one K block to the next
    __device__ __forceinline__ void init(const void* scales, int groups, int group) {
        group = group < groups ? group : groups - 1;            // rows past the matrix are masked by the caller
        p = (const uint32_t*)scales + (size_t)group * 32 + (threadIdx.x & 31);
        step = (uint32_t)groups * 32u;
    }
    __device__ __forceinline__ uint32_t load(int kb) const { return p[(size_t)kb * step]; }
};

// One block-scaled FP8 MFMA; OA / OB select the scale byte of each operand (compile time).
template <int OA, int OB>
__device__ __forceinline__ f32x16 mfma_fp8(const i32x8 a, const i32x8 b, const f32x16 c, int sa, int sb) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, OA, sa, OB, sb);
}
__device__ __forceinline__ f32x16 mfma_fp8_sel(int oa, int ob, const i32x8 a, const i32x8 b, const f32x16 c, int sa, int sb) {
    switch (oa * 2 + ob) {          // folded after unrolling
        case 0: return mfma_fp8<0, 0>(a, b, c, sa, sb);
        case 1: return mfma_fp8<0, 1>(a, b, c, sa, sb);
        case 2: return mfma_fp8<1, 0>(a, b, c, sa, sb);
        case 3: return mfma_fp8<1, 1>(a, b, c, sa, sb);
        case 4: return mfma_fp8<2, 0>(a, b, c, sa, sb);
        case 5: return mfma_fp8<2, 1>(a, b, c, sa, sb);
        case 6: return mfma_fp8<3, 0>(a, b, c, sa, sb);
        default: return mfma_fp8<3, 1>(a, b, c, sa, sb);
    }
}

// SA: scale group of the wavefront's TM = 4 A blocks (128 rows); SB: scale group that
// contains its TN = 2 B blocks, b_half = which half of that group (0: rows 0..63).
template <class Cfg>
__device__ __forceinline__ void gemm_mainloop_fp8(f32x16 (&acc)[Cfg::TM][Cfg::TN],
                                                   const OperandTile<true, Cfg::BM>& A,
                                                   const OperandTile<true, Cfg::BN>& B,
                                                   const ScaleGroup& SA, const ScaleGroup& SB, int b_half,
                                                   int k_total, CCE_LDS char* smem) {
    static_assert(Cfg::STAGES == 2 && Cfg::KG == 1 && Cfg::TM == 4 && Cfg::TN == 2, "256 x 256 tile, two stages");
    FragAddr<true, Cfg::BM, Cfg::TM, 4, 1> fa;
    FragAddr<true, Cfg::BN, Cfg::TN, 4, 1> fb;
    fa.init(wave_m<Cfg>() * (Cfg::TM * 32), 0);
    fb.init(wave_n<Cfg>() * (Cfg::TN * 32), 0);
    auto frag = [](const CCE_LDS char* op, uint32_t a, int b) {
        return *(const CCE_LDS i32x4*)(op + a + b * (32 * 128));
    };

    const int KT = (k_total + 127) / 128;
    const int b_shift = 16 * b_half;
    uint32_t sa_next = SA.load(0), sb_next = SB.load(0);

    A.issue(smem, 0);
    B.issue(smem + Cfg::kAStage, 0);
    barrier_pending_loads<0>();

    // A fragments are refreshed in place, block by block, behind the MFMAs that used them; B
    // fragments (needed by every block of a step) are double buffered.
    i32x4 af[Cfg::TM][2], bfr[2][Cfg::TN][2];
#pragma unroll
    for (int bm = 0; bm < Cfg::TM; ++bm) { af[bm][0] = frag(smem, fa.a[0], bm); af[bm][1] = frag(smem, fa.a[1], bm); }
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) {
        bfr[0][bn][0] = frag(smem + Cfg::kAStage, fb.a[0], bn);
        bfr[0][bn][1] = frag(smem + Cfg::kAStage, fb.a[1], bn);
    }

    int cur_s = 0;
    for (int kt = 0; kt < KT; ++kt) {
        CCE_LDS char* cur = smem + cur_s * Cfg::kStage;
        CCE_LDS char* nxt = smem + (cur_s ^ 1) * Cfg::kStage;
        const bool more = kt + 1 < KT;
        // scales of this slice (requested one slice ago, complete since the last barrier) and
        // request of the next slice's, ahead of the operand loads
        const int sa = (int)sa_next, sb = (int)(sb_next >> b_shift);
        // Consume the two scale words HERE, before this iteration's operand loads are issued:
        // the compiler places its wait for them at their first use and cannot see the
        // inline-assembly loads, so a first use after those would make it wait for them too.
        asm volatile("" :: "v"(sa), "v"(sb));
        const int kn = more ? kt + 1 : kt;
        sa_next = SA.load(kn);
        sb_next = SB.load(kn);
        if (more) {
            A.issue(nxt, (kt + 1) * kBK);
            B.issue(nxt + Cfg::kAStage, (kt + 1) * kBK);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int c = t, n = t ^ 1;
            const CCE_LDS char* src = cur;
            int j0 = 2;
            if (t == 1) {
                // slice kt + 1 must have landed before its fragments are read
                barrier_pending_loads<0>();
                src = nxt;
                j0 = 0;
            }
#pragma unroll
            for (int bn = 0; bn < Cfg::TN; ++bn) {
                bfr[n][bn][0] = frag(src + Cfg::kAStage, fb.a[j0], bn);
                bfr[n][bn][1] = frag(src + Cfg::kAStage, fb.a[j0 + 1], bn);
            }
#pragma unroll
            for (int bm = 0; bm < Cfg::TM; ++bm) {
                const i32x8 a8 = __builtin_shufflevector(af[bm][0], af[bm][1], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int bn = 0; bn < Cfg::TN; ++bn) {
                    const i32x8 b8 = __builtin_shufflevector(bfr[c][bn][0], bfr[c][bn][1], 0, 1, 2, 3, 4, 5, 6, 7);
                    acc[bm][bn] = mfma_fp8_sel(bm, bn, a8, b8, acc[bm][bn], sa, sb);
                }
                af[bm][0] = frag(src, fa.a[j0], bm);
                af[bm][1] = frag(src, fa.a[j0 + 1], bm);
            }
            // issue order for the scheduler: the four B reads behind the first two MFMAs, then
            // each A block's two reads behind the MFMA that follows the last use of the block
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0); __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0); __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        cur_s ^= 1;
    }
    barrier_pending_loads<0>();
}

// Tile coordinates of accumulator element acc[bm][bn][r] of the calling lane.
template <class Cfg>
__device__ __forceinline__ int acc_row(int bm, int r) {
    const int l = threadIdx.x & 63;
    return wave_m<Cfg>() * (Cfg::TM * 32) + bm * 32 + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
}
template <class Cfg>
__device__ __forceinline__ int acc_col(int bn) {
    const int l = threadIdx.x & 63;
    return wave_n<Cfg>() * (Cfg::TN * 32) + bn * 32 + (l & 31);
}

}  // namespace cce
