// Host-side planner of libcce: how one call is tiled over the GPU and laid out in the caller's
// workspace -- vocabulary splits of the forward, [row block x vocabulary chunk] of the backward,
// contraction tile, form of the dHidden running sum -- ranked with a small time model whose
// constants were measured on MI355X.  No device code; included by cce_kernels.hip only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <atomic>

#include "gemm_core.h"
#include "host_util.h"

namespace cce {

// Row skipping: a row block's row map lives in an LDS table behind everything else the
// contraction kernel uses, which bounds the block to this many 256-row tiles.
constexpr int kCompactMaxRowTiles = 16;
constexpr int kRowTableBytes = kCompactMaxRowTiles * 256 * 4;

// Compute units of the CURRENT device (looked up once per device ordinal; 256 if the query fails,
// e.g. on a host without a GPU).
static int device_cu_count() {
    static std::atomic<int> cached[64];
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    const int have = cached[dev].load(std::memory_order_relaxed);
    if (have > 0) return have;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    cached[dev].store(n, std::memory_order_relaxed);
    return n;
}


struct Plan {
    int TT, VT, S;              // forward: token tiles, vocabulary tiles, vocabulary splits
    int64_t Nb, Vc;             // backward: rows per row block, vocabulary columns per chunk (multiples of 256)
    int gemm_kind;              // backward: output tile of the contractions, 0 = 256 x 256, 1 = 256 x 128
    int split_acc;              // backward: dH running sum as two 16-bit planes (see GemmJob)
    double model_us;            // modelled time of forward + backward with this plan (ranking only)
    size_t off_status, off_partials, off_sumz, off_dhacc, off_g, total;
    // row skipping only (budget_rows != 0): compact-row bookkeeping
    int64_t rows_pad;           // compact rows rounded up to 256
    size_t off_count, off_perm, off_labels_c, off_fa_c, off_fb_c;
    size_t off_zero_row;        // D zeros (bf16): what the dW contraction reads for a k-row that maps to no row
};

// Workspace budget: 1 % of the materialised fp32 logits, but never below a floor that
// keeps the backward chunks large enough to fill the GPU.
static constexpr size_t kBudgetFloor = 48000000;

// Output tiles of the two gradient contractions: 256 x 256, or 256 x 128 with two K groups.
// The planner picks per shape: the narrow tile costs about 10 % more per flop (more operand
// bytes per MFMA) but gives twice as many tiles, which matters when a chunk's outputs are too
// few to fill the GPU (D = 1024: 124 big tiles per 4096 x 4096 chunk against 248 narrow ones)
// or when D is not a multiple of 256 (D = 896 = 7 x 128).  (A 128 x 224 tile, which would give
// D = 896 exactly 256 equal tiles per chunk, was measured 3 % slower: its 32 x 224 wavefront
// tiles need 1.14 LDS fragment reads per MFMA instead of 0.75.)
struct GemmTile { int kind, bm, bn; double us_per_slice; };
static GemmTile gemm_tile_of_kind(int kind) {
    if (kind == 0) return {0, TileBig::BM, TileBig::BN, 2.0};
    return {1, TileNarrow::BM, TileNarrow::BN, 1.1};
}

// Process-wide tuning / testing knobs (0 = automatic).  Atomics: a knob may be set from any host
// thread; every plan reads each knob once (Knobs::read) and the plan cache is keyed by what it read,
// so a change between two calls can never mix two settings inside one plan.  (A caller that sizes
// its workspace under one setting and computes under another still gets CCE_ERR_INVALID if the
// workspace is too small: the knobs are aids for tests and measurements, not a per-call option.)
static std::atomic<int> g_force_tiling{0};           // cce_set_backward_tiling: (row_tiles << 16) | vocab_tiles
static std::atomic<int> g_force_gemm_cols{0};        // cce_set_backward_gemm_tile: 128 or 256
static std::atomic<int> g_force_split_acc{0};        // cce_set_backward_accumulator: 1 = fp32, 2 = split
static std::atomic<int> g_force_row_skipping{0};     // cce_set_row_skipping: 1 = never, 2 = whenever rows can be skipped
struct Knobs {
    int row_tiles, vocab_tiles, gemm_cols, split_acc;
    static Knobs read() {
        const int t = g_force_tiling.load(std::memory_order_relaxed);
        return {t >> 16, t & 0xffff, g_force_gemm_cols.load(std::memory_order_relaxed),
                g_force_split_acc.load(std::memory_order_relaxed)};
    }
};

// Rough time model of the backward pipeline, in microseconds, used only to rank tilings.
// One compute unit runs one workgroup at a time.  Measured on MI355X with random bf16 data:
// a 256 x 256 x 64 slice of the main loop takes about 2 us, a 256 x 128 x 64 one about 1.1 us;
// a gradient-tile workgroup adds about 9 us (pipeline fill, softmax epilogue, store of the
// tile), a contraction workgroup about 4 us.
struct BackwardModel {
    int cus; int64_t D; GemmTile tile;
    double t_tile() const { return (double)(D / 64) * 2.0 + 9.0; }
    double t_gemm(int k_tiles) const { return (double)(k_tiles * 4) * tile.us_per_slice + 4.0; }
    int d_tiles() const { return (int)((D + tile.bn - 1) / tile.bn); }

    // Completion time of n1 jobs of length c1 followed by n2 jobs of length c2 <= c1, handed in
    // that order to `cus` units, each taking the next job when it becomes free.
    double two_class_makespan(int n1, double c1, int n2, double c2) const {
        const int full = n1 / cus, rem = n1 % cus;
        const double tA = full * c1;                 // units without a long job in the last round
        const double tB = (rem ? full + 1 : full) * c1;
        if (n2 == 0) return tB;
        const int nA = cus - rem, nB = rem;
        // smallest t with nA * floor((t - tA) / c2) + nB * floor((t - tB) / c2) >= n2
        double best = 1e300;
        for (int k = 1; k <= n2; ++k) {             // t = tA + k c2
            const double t = tA + k * c2;
            const double fromB = t > tB ? (double)(int64_t)((t - tB) / c2) : 0.0;
            if ((double)nA * k + (double)nB * fromB >= n2) { best = t; break; }
        }
        if (nB > 0) {
            for (int k = 1; k <= n2; ++k) {         // t = tB + k c2
                const double t = tB + k * c2;
                if (t >= best) break;
                const double fromA = (double)(int64_t)((t - tA) / c2);
                if ((double)nA * fromA + (double)nB * k >= n2) { best = t; break; }
            }
        }
        return best > tB ? best : tB;
    }

    // One step = the gradient tiles, then the contractions, of an [a x b] block of 256 x 256
    // tiles: two launches that follow each other on the caller's stream.
    double step(int a, int b, bool dw_beta) const {
        const int dt = d_tiles(), per256 = 256 / tile.bm;
        const int n_dh = a * per256 * dt, n_dw = b * per256 * dt;
        const double c_dh = t_gemm(b), c_dw = t_gemm(a);
        const double mk = (c_dh >= c_dw) ? two_class_makespan(n_dh, c_dh, n_dw, c_dw)
                                          : two_class_makespan(n_dw, c_dw, n_dh, c_dh);
        // fp32 accumulator traffic of the step at ~3 TB/s
        const double bytes = (double)a * 256 * D * 8.0 + (dw_beta ? (double)b * 256 * D * 8.0 : (double)b * 256 * D * 4.0);
        return ((a * b + cus - 1) / cus) * t_tile() + mk + bytes / 3.0e6 + 4.0;
    }
};

// budget_rows != 0 selects row skipping: the plan is made for N compact rows while the workspace
// budget (1 % of the materialised logits) is that of the budget_rows original rows, and the
// workspace also holds the compact-row bookkeeping (row map and per-row scalars).
static bool make_plan(int64_t N, int64_t D, int64_t V, Plan* p, int64_t budget_rows = 0) {
    if (N <= 0 || D <= 0 || V <= 0) return false;
    const Knobs knobs = Knobs::read();
    const int cus = device_cu_count();
    struct Key { int64_t N, D, V, B; int cus, fa, fb, fc, fs; Plan plan; bool valid; };
    static thread_local Key cache = {0, 0, 0, 0, 0, 0, 0, 0, 0, {}, false};
    if (cache.valid && cache.N == N && cache.D == D && cache.V == V && cache.B == budget_rows && cache.cus == cus &&
        cache.fa == knobs.row_tiles && cache.fb == knobs.vocab_tiles && cache.fc == knobs.gemm_cols &&
        cache.fs == knobs.split_acc) { *p = cache.plan; return true; }
    const bool compact = budget_rows != 0;

    const int64_t Np = round_up(N, 256), Vp = round_up(V, 256);
    p->TT = (int)(Np / 256);
    p->VT = (int)(Vp / 256);
    // Vocabulary splits of the forward: TT x S workgroups run in rounds of `cus`, each walking
    // ceil(VT / S) vocabulary tiles; take the S with the fewest tile-times (the smallest on a tie).
    {
        int best_s = 1;
        int64_t best_cost = INT64_MAX;
        const int s_max = p->VT < 2 * cus ? p->VT : 2 * cus;
        for (int s = 1; s <= s_max; ++s) {
            const int64_t rounds = ((int64_t)p->TT * s + cus - 1) / cus;
            const int64_t cost = rounds * ((p->VT + s - 1) / s);
            if (cost < best_cost) { best_cost = cost; best_s = s; }
        }
        p->S = best_s;
    }
    const int S = p->S;

    // per (token, split): (max, sum-exp) pair + the logit sum that label smoothing needs
    const size_t md_bytes = (size_t)round_up((int64_t)N * S * 8, 256);
    const size_t partial_bytes = md_bytes + (size_t)round_up((int64_t)N * S * 4, 256);
    size_t budget = (size_t)((double)(compact ? budget_rows : N) * (double)V * 4.0 * 0.01);
    if (budget < kBudgetFloor) budget = kBudgetFloor;
    const size_t scalar_bytes = compact ? (size_t)round_up(Np * 4, 256) : 0;      // one per-row int32 / fp32 array
    const size_t zero_row_bytes = compact ? (size_t)round_up(D * 2, 256) : 0;
    const size_t fixed = 256 + partial_bytes + (compact ? 256 + 4 * scalar_bytes + zero_row_bytes : 0);

    // Row block of a tiles, vocabulary chunk of b tiles.
    int acc_bytes = 4;          // per element of the dH running sum: 4 (fp32) or 2 (split planes)
    auto bytes_needed = [&](int64_t a, int64_t b) {
        return (double)fixed + (double)round_up(a * 256 * D * acc_bytes, 256) + (double)(a * 256) * (double)(b * 256) * 2.0;
    };
    // Tiling for a given contraction tile: the (a, b) with the smallest modelled time.
    auto plan_for_kind = [&](int kind, int* a_out, int* b_out) -> double {
        BackwardModel model{cus, D, gemm_tile_of_kind(kind)};
        if (knobs.row_tiles > 0 && knobs.vocab_tiles > 0) {
            *a_out = knobs.row_tiles < p->TT ? knobs.row_tiles : p->TT;
            if (compact && *a_out > kCompactMaxRowTiles) *a_out = kCompactMaxRowTiles;
            *b_out = knobs.vocab_tiles < p->VT ? knobs.vocab_tiles : p->VT;
            return 0.0;
        }
        double best_cost = 1e300;
        // (row skipping: a row block's row map must fit its LDS table)
        const int a_cap = compact ? kCompactMaxRowTiles : 64;
        const int a_max = p->TT < a_cap ? p->TT : a_cap, b_max = p->VT < 128 ? p->VT : 128;
        *a_out = 1; *b_out = 1;
        for (int a = 1; a <= a_max; ++a) {
            for (int b = 1; b <= b_max; ++b) {
                if (bytes_needed(a, b) > (double)budget && !(a == 1 && b == 1)) break;
                const int nblk = (p->TT + a - 1) / a, a_last = p->TT - (nblk - 1) * a;
                const int nch = (p->VT + b - 1) / b, b_last = p->VT - (nch - 1) * b;
                // the first row block overwrites dW, later ones add to it
                auto block_cost = [&](int aa, bool beta) {
                    return (nch - 1) * model.step(aa, b, beta) + model.step(aa, b_last, beta);
                };
                double cost = (nblk == 1) ? block_cost(a_last, false)
                                          : block_cost(a, false) + (nblk - 2) * block_cost(a, true) + block_cost(a_last, true);
                // measured per contraction launch: the split running sum costs 2 us, 9 us when its
                // upper-half plane is also reached through the row map of the compact row space
                if (acc_bytes == 2) cost += (double)nblk * nch * (compact ? 9.0 : 2.0);
                if (cost < best_cost) { best_cost = cost; *a_out = a; *b_out = b; }
            }
        }
        return best_cost;
    };
    // 256 x 256 tiles when D is a multiple of 256 and they fill the rounds of `cus` workgroups
    // of a contraction launch to at least 70 %; else 256 x 128.  (The cost model ranks tilings
    // of one tile shape well but is off by ~15 % between the shapes, so the shape is decided
    // by occupancy: measured, D = 1024 and 2048 gain 17 % with the narrow tile, D = 1536 with
    // 77 % occupancy loses 6 %.)
    auto plan_for_acc = [&](int bytes, int* a_out, int* b_out, int* kind_out) -> double {
        acc_bytes = bytes;
        double cost = 0.0;
        *kind_out = 1;
        if (knobs.gemm_cols != 0) {
            *kind_out = knobs.gemm_cols == 256 ? 0 : 1;
            if (*kind_out == 0) cost = plan_for_kind(0, a_out, b_out);
        } else if (D % 256 == 0) {
            cost = plan_for_kind(0, a_out, b_out);
            const int64_t tiles = (int64_t)(*a_out + *b_out) * (D / 256);
            const int64_t rounds = (tiles + cus - 1) / cus;
            *kind_out = (double)tiles >= 0.7 * (double)(rounds * cus) ? 0 : 1;
        }
        if (*kind_out == 1) cost = plan_for_kind(1, a_out, b_out);
        return cost;
    };
    // The dH running sum: plain fp32 unless the split form (half the workspace, a little slower
    // per launch) buys a tiling that the model rates at least 3 % faster.
    int best_a = 1, best_b = 1, best_kind = 1, sa = 1, sb = 1, skind = 1;
    const double cost_f32 = plan_for_acc(4, &best_a, &best_b, &best_kind);
    const double cost_split = plan_for_acc(2, &sa, &sb, &skind);
    p->split_acc = 0;
    if (knobs.split_acc == 2 || (knobs.split_acc == 0 && cost_split < 0.97 * cost_f32)) {
        best_a = sa; best_b = sb; best_kind = skind; p->split_acc = 1;
    }
    acc_bytes = p->split_acc ? 2 : 4;
    {
        BackwardModel fm{cus, D, gemm_tile_of_kind(0)};
        const int64_t rounds = ((int64_t)p->TT * p->S + cus - 1) / cus;
        p->model_us = (p->split_acc ? cost_split : cost_f32) + (double)(rounds * ((p->VT + p->S - 1) / p->S)) * fm.t_tile();
    }
    p->gemm_kind = best_kind;
    p->Nb = (int64_t)best_a * 256;
    p->Vc = (int64_t)best_b * 256;
    // the gradient chunk is addressed with 32-bit byte offsets (only a forced tiling can get here)
    if (p->Nb * p->Vc * 2 >= ((int64_t)1 << 32)) return false;
    p->off_status = 0;
    p->off_partials = 256;
    p->off_sumz = p->off_partials + md_bytes;
    p->off_dhacc = p->off_partials + partial_bytes;
    p->off_g = p->off_dhacc + (size_t)round_up(p->Nb * D * (p->split_acc ? 2 : 4), 256);
    p->total = p->off_g + (size_t)(p->Nb * p->Vc * 2);
    p->rows_pad = Np;
    p->off_count = p->off_perm = p->off_labels_c = p->off_fa_c = p->off_fb_c = p->off_zero_row = 0;
    if (compact) {
        p->off_count = round_up((int64_t)p->total, 256);
        p->off_perm = p->off_count + 256;
        p->off_labels_c = p->off_perm + scalar_bytes;
        p->off_fa_c = p->off_labels_c + scalar_bytes;
        p->off_fb_c = p->off_fa_c + scalar_bytes;
        p->off_zero_row = p->off_fb_c + scalar_bytes;
        p->total = p->off_zero_row + zero_row_bytes;
    }
    cache = {N, D, V, budget_rows, cus, knobs.row_tiles, knobs.vocab_tiles, knobs.gemm_cols, knobs.split_acc, *p, true};
    return true;
}

}  // namespace cce
