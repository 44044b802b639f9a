// Host-only check of the planner (csrc/plan.h): a seeded sweep of shapes, forced tilings, contraction
// tiles, accumulator forms and row-skipping budgets, built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the HOST side only (tests/test_plan_host.py compiles and runs it; no
// GPU is needed: without a device the planner assumes 256 compute units).  Every plan must lay the
// workspace out without overlap, inside its budget, with aligned offsets and tile-multiple blocks.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

namespace cce { thread_local int g_last_hip_error = 0; }
#include "../../paper_2601_02609_amd/csrc/plan.h"

using namespace cce;

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t next_u64() {            // splitmix64
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static int64_t pick(int64_t lo, int64_t hi) { return lo + (int64_t)(next_u64() % (uint64_t)(hi - lo + 1)); }

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { ++failures; fprintf(stderr, "FAIL %s:%d: %s | ", __FILE__, __LINE__, #cond); \
    fprintf(stderr, __VA_ARGS__); fprintf(stderr, "\n"); } } while (0)

static void check_plan(int64_t N, int64_t D, int64_t V, int64_t budget_rows, bool forced) {
    Plan p;
    const bool ok = make_plan(N, D, V, &p, budget_rows);
    if (!ok) {
        // only a forced tiling whose gradient chunk reaches 4 GiB may be refused
        CHECK(forced, "unforced plan refused N=%lld D=%lld V=%lld B=%lld", (long long)N, (long long)D, (long long)V, (long long)budget_rows);
        return;
    }
    const int64_t Np = round_up(N, 256), Vp = round_up(V, 256);
    CHECK(p.TT == Np / 256 && p.VT == Vp / 256, "tile counts");
    CHECK(p.S >= 1 && p.S <= p.VT, "S=%d VT=%d", p.S, p.VT);
    CHECK(p.Nb > 0 && p.Nb % 256 == 0 && p.Nb <= Np, "Nb=%lld", (long long)p.Nb);
    CHECK(p.Vc > 0 && p.Vc % 256 == 0 && p.Vc <= Vp, "Vc=%lld", (long long)p.Vc);
    CHECK(p.gemm_kind == 0 || p.gemm_kind == 1, "kind");
    CHECK(p.split_acc == 0 || p.split_acc == 1, "split");
    CHECK(p.off_status == 0 && p.off_partials == 256, "head");
    CHECK(p.off_partials % 256 == 0 && p.off_sumz % 256 == 0 && p.off_dhacc % 256 == 0 && p.off_g % 256 == 0, "alignment");
    CHECK(p.off_sumz >= p.off_partials + (size_t)N * p.S * 8, "partials overlap sumz");
    CHECK(p.off_dhacc >= p.off_sumz + (size_t)N * p.S * 4, "sumz overlaps dH sums");
    CHECK(p.off_g >= p.off_dhacc + (size_t)(p.Nb * D * (p.split_acc ? 2 : 4)), "dH sums overlap G");
    const size_t g_end = p.off_g + (size_t)(p.Nb * p.Vc * 2);
    CHECK(p.Nb * p.Vc * 2 < ((int64_t)1 << 32), "chunk beyond 32-bit offsets");
    if (budget_rows == 0) {
        CHECK(p.total == g_end, "total");
    } else {
        CHECK(p.rows_pad == Np, "rows_pad");
        CHECK(p.Nb <= (int64_t)kCompactMaxRowTiles * 256, "row block beyond the LDS row table");
        CHECK(p.off_count >= g_end && p.off_perm >= p.off_count + 4 && p.off_labels_c >= p.off_perm + (size_t)Np * 4 &&
              p.off_fa_c >= p.off_labels_c + (size_t)Np * 4 && p.off_fb_c >= p.off_fa_c + (size_t)Np * 4 &&
              p.off_zero_row >= p.off_fb_c + (size_t)Np * 4 && p.total >= p.off_zero_row + (size_t)D * 2, "row-skipping bookkeeping overlaps");
        CHECK(p.off_count % 256 == 0 && p.off_perm % 256 == 0 && p.off_zero_row % 256 == 0, "bookkeeping alignment");
    }
    if (!forced) {
        double budget = (double)(budget_rows ? budget_rows : N) * (double)V * 4.0 * 0.01;
        if (budget < (double)kBudgetFloor) budget = (double)kBudgetFloor;
        // a 1 x 1 tiling is always allowed (tiny budgets); otherwise the plan stays inside the budget
        if (!(p.Nb == 256 && p.Vc == 256))
            CHECK((double)p.total <= budget + 1.0, "over budget: total=%zu budget=%.0f N=%lld D=%lld V=%lld B=%lld",
                  p.total, budget, (long long)N, (long long)D, (long long)V, (long long)budget_rows);
    }
    CHECK(p.model_us >= 0.0, "model");
}

int main(int argc, char** argv) {
    const int iters = argc > 1 ? atoi(argv[1]) : 3000;
    // the five benchmark shapes first
    const int64_t shapes[5][3] = {{256, 64, 1000}, {8192, 896, 151936}, {16384, 2048, 151936}, {32768, 3584, 151936}, {16384, 4096, 32000}};
    for (auto& s : shapes) {
        check_plan(s[0], s[1], s[2], 0, false);
        check_plan(s[0] - s[0] / 7, s[1], s[2], s[0], false);
    }
    for (int it = 0; it < iters; ++it) {
        const int64_t N = (it % 5 == 0) ? pick(1, 300) : pick(1, 70000);
        const int64_t D = 64 * pick(1, 72);
        const int64_t V = (it % 7 == 0) ? pick(1, 600) : pick(1, 300000);
        if (V * D * 2 >= ((int64_t)1 << 32) || N * D * 2 >= ((int64_t)1 << 32)) continue;
        const bool forced = it % 3 == 0;
        g_force_tiling.store(forced ? (int)((pick(1, 70) << 16) | pick(1, 200)) : 0);
        g_force_gemm_cols.store(it % 4 == 1 ? 128 : (it % 4 == 2 ? 256 : 0));
        g_force_split_acc.store((int)pick(0, 2));
        check_plan(N, D, V, 0, forced);
        const int64_t M = pick(1, N);
        check_plan(M, D, V, N, forced);
        // cached plan must equal a fresh one
        Plan a, b;
        if (make_plan(N, D, V, &a) && make_plan(N, D, V, &b))
            CHECK(a.total == b.total && a.Nb == b.Nb && a.Vc == b.Vc && a.S == b.S, "cache");
    }
    if (failures) { fprintf(stderr, "%d failures\n", failures); return 1; }
    printf("plan_fuzz: %d iterations ok\n", iters);
    return 0;
}
