// Host-only check of the planner (csrc/plan.h): a seeded sweep of shapes, forced tilings, contraction
// tiles, accumulator forms and row-skipping budgets, built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the HOST side only (tests/test_plan_host.py compiles and runs it; no
// GPU is needed: without a device the planner assumes 256 compute units).  Every plan must lay the
// workspace out without overlap, inside its budget, with aligned offsets and tile-multiple blocks.
// The workgroup-id -> work-item mappings of the kernels (csrc/wg_map.h) are walked here as well: for
// every grid size a launch can have, each mapping must hit every item exactly once.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

namespace cce { thread_local int g_last_hip_error = 0; }
#include "../../paper_2601_02609_amd/csrc/plan.h"
#include "../../paper_2601_02609_amd/csrc/wg_map.h"
#include <vector>

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

// Every workgroup id of a grid maps to a distinct item inside the grid (a repeated or out-of-range item
// would be a tile computed twice, one never computed, or a store outside the output).
static void check_maps() {
    std::vector<int> seen;
    for (int nb = 1; nb <= 2600; ++nb) {
        seen.assign(nb, 0);
        for (int b = 0; b < nb; ++b) {
            const int l = xcd_round_id(b, nb, 256);
            CHECK(l >= 0 && l < nb, "xcd_round_id nb=%d b=%d -> %d", nb, b, l);
            if (l >= 0 && l < nb) ++seen[l];
        }
        for (int l = 0; l < nb; ++l) CHECK(seen[l] == 1, "xcd_round_id nb=%d item %d hit %d times", nb, l, seen[l]);
        if (nb <= 256) {
            // one round: the ids of one XCD (equal modulo 8) take consecutive items
            for (int b = 8; b < nb; ++b) CHECK(xcd_linear_id(b, nb) == xcd_linear_id(b - 8, nb) + 1, "xcd_linear_id nb=%d b=%d", nb, b);
        }
    }
    // two jobs in one grid: n1 long items, then n2 short ones, both >= 8
    for (int n1 = 8; n1 <= 420; n1 += (n1 < 80 ? 1 : 7)) {
        for (int n2 = 8; n2 <= 1400; n2 += (n2 < 80 ? 1 : 11)) {
            std::vector<int> s1(n1, 0), s2(n2, 0);
            int long_per_xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int b = 0; b < n1 + n2; ++b) {
                bool in_first = false; int item = -1;
                xcd_two_job_map(b, n1, n2, in_first, item);
                const int n = in_first ? n1 : n2;
                CHECK(item >= 0 && item < n, "two_job n1=%d n2=%d b=%d -> %d/%d", n1, n2, b, (int)in_first, item);
                if (item < 0 || item >= n) continue;
                ++(in_first ? s1 : s2)[item];
                if (in_first) {
                    ++long_per_xcd[b & 7];
                    // an XCD starts its ids in order: its long items come before its short ones
                    CHECK((b >> 3) < (n1 + 7) / 8, "long item late in the queue n1=%d n2=%d b=%d", n1, n2, b);
                }
            }
            for (int i = 0; i < n1; ++i) CHECK(s1[i] == 1, "two_job n1=%d n2=%d long item %d hit %d times", n1, n2, i, s1[i]);
            for (int i = 0; i < n2; ++i) CHECK(s2[i] == 1, "two_job n1=%d n2=%d short item %d hit %d times", n1, n2, i, s2[i]);
            for (int x = 0; x < 8; ++x)
                CHECK(long_per_xcd[x] == n1 / 8 || long_per_xcd[x] == n1 / 8 + 1, "uneven deal n1=%d n2=%d xcd %d: %d", n1, n2, x, long_per_xcd[x]);
        }
    }
    // (i fastest inside groups of `group`) x j: every cell of the n_i x n_j grid exactly once
    for (int n_i = 1; n_i <= 70; ++n_i)
        for (int n_j = 1; n_j <= 40; n_j += (n_j < 12 ? 1 : 9))
            for (int group = 1; group <= 9; group += 3) {
                seen.assign(n_i * n_j, 0);
                for (int lin = 0; lin < n_i * n_j; ++lin) {
                    int i = -1, j = -1;
                    group_map(lin, n_i, n_j, group, i, j);
                    CHECK(i >= 0 && i < n_i && j >= 0 && j < n_j, "group_map %d x %d group %d lin %d -> (%d, %d)", n_i, n_j, group, lin, i, j);
                    if (i >= 0 && i < n_i && j >= 0 && j < n_j) ++seen[i * n_j + j];
                }
                for (int c = 0; c < n_i * n_j; ++c) CHECK(seen[c] == 1, "group_map %d x %d group %d cell %d hit %d times", n_i, n_j, group, c, seen[c]);
            }
}

int main(int argc, char** argv) {
    const int iters = argc > 1 ? atoi(argv[1]) : 3000;
    check_maps();
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
