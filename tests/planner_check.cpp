// Host-side check of the launch planner (csrc/macko_plan.h): for random groups of
// matrices, replay the row assignment the kernels derive from a plan and verify
// that every row is taken exactly once, that no wavefront gets more than 64 rows,
// that the reciprocal multiply the kernels use equals the division, and that a
// resident round has exactly (workgroups per compute unit) x (compute units)
// workgroups.  Built and run by tests/test_library_host.py; prints "ok" on success.
#include "macko_plan.h"

#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

using namespace macko;

static int failures = 0;
#define EXPECT(cond, ...)                      \
  do {                                         \
    if (!(cond)) {                             \
      if (failures < 20) { std::printf("FAIL %s: ", #cond); std::printf(__VA_ARGS__); std::printf("\n"); } \
      ++failures;                              \
    }                                          \
  } while (0)

// the kernels' arithmetic: rows of workgroup `wg`, then of wavefront `wave`
static void replay(const Plan& plan, int n, const PlanInput* in, const char* what) {
  const int nwaves = plan.block / 64;
  EXPECT(plan.block % 64 == 0 && nwaves >= 1 && nwaves <= 16, "%s block %d", what, plan.block);
  const int inv = 65536 / nwaves + 1;
  int64_t wgs = 0;
  for (int i = 0; i < n; ++i) {
    const PlanMat& m = plan.m[i];
    EXPECT(m.nwg >= 1 && (int64_t)m.nwg * m.q + m.r == in[i].rows && m.r >= 0 && m.r < m.nwg,
           "%s matrix %d rows %lld nwg %d q %d r %d", what, i, (long long)in[i].rows, m.nwg, m.q, m.r);
    std::vector<unsigned char> seen((size_t)in[i].rows, 0);
    for (int wg = 0; wg < m.nwg; ++wg) {
      const int row_begin = wg * m.q + std::min(wg, m.r);
      const int wg_rows = m.q + (wg < m.r ? 1 : 0);
      EXPECT(wg_rows <= 1024, "%s wg_rows %d", what, wg_rows);
      const int per_wave = (wg_rows * inv) >> 16;
      EXPECT(per_wave == wg_rows / nwaves, "%s reciprocal: %d / %d gave %d", what, wg_rows, nwaves, per_wave);
      const int extra = wg_rows - per_wave * nwaves;
      for (int wave = 0; wave < nwaves; ++wave) {
        const int b = row_begin + wave * per_wave + std::min(wave, extra);
        const int nb = per_wave + (wave < extra ? 1 : 0);
        EXPECT(nb <= kPlanMaxRowsPerWave, "%s wavefront with %d rows", what, nb);
        for (int r = b; r < b + nb; ++r) {
          EXPECT(r >= 0 && r < in[i].rows, "%s row %d out of range", what, r);
          if (r >= 0 && r < in[i].rows) ++seen[(size_t)r];
        }
      }
    }
    for (int64_t r = 0; r < in[i].rows; ++r)
      if (seen[(size_t)r] != 1) { EXPECT(false, "%s matrix %d row %lld taken %d times", what, i, (long long)r, seen[(size_t)r]); break; }
    wgs += m.nwg;
  }
  EXPECT(wgs == plan.total_wgs, "%s total %lld != %lld", what, (long long)wgs, (long long)plan.total_wgs);
}

int main() {
  std::mt19937_64 rng(20251113061ull);
  auto uni = [&](int64_t lo, int64_t hi) { return lo + (int64_t)(rng() % (uint64_t)(hi - lo + 1)); };
  int resident_plans = 0;
  for (int trial = 0; trial < 3000; ++trial) {
    const int n = (int)uni(1, kMaxGroup);
    PlanInput in[kMaxGroup];
    for (int i = 0; i < n; ++i) {
      const int kind = (int)uni(0, 3);
      in[i].rows = kind == 0 ? uni(1, 300) : kind == 1 ? uni(1000, 12000) : kind == 2 ? uni(20000, 60000) : uni(1, 60000);
      in[i].steps_per_row = uni(1, 60);
      in[i].lds_bytes = 1536 + 16 * uni(8, 9000);
    }
    // many-workgroup regime, any block and rows per workgroup
    {
      const int block = 64 * (int)uni(1, 16);
      int64_t rpw[kMaxGroup];
      for (int i = 0; i < n; ++i) rpw[i] = uni(0, 3) == 0 ? uni(1, 1 << 20) : uni(1, 200);
      Plan plan;
      plan_by_rows_per_wg(plan, n, in, block, rpw);
      EXPECT(plan.block == block, "block");
      replay(plan, n, in, "rows-per-workgroup");
    }
    // resident round, free or forced shape
    for (int cus : {256, 64, 304}) {
      const int forced_block = uni(0, 2) == 0 ? 64 * (int)uni(4, 16) : 0;
      const int forced_k = (int)uni(0, 4);
      Plan plan;
      if (!plan_resident(plan, n, in, cus, forced_block, forced_k)) continue;
      ++resident_plans;
      const int k = forced_k ? forced_k : 2;
      EXPECT(plan.total_wgs == (int64_t)cus * k, "resident round of %lld workgroups on %d units, k %d",
             (long long)plan.total_wgs, cus, k);
      EXPECT(forced_block == 0 || plan.block == forced_block, "forced block");
      int64_t max_lds = 0;
      for (int i = 0; i < n; ++i) max_lds = std::max(max_lds, in[i].lds_bytes);
      EXPECT(k * max_lds <= kPlanLdsPerCu, "LDS of %d workgroups per unit", k);
      EXPECT(k * (plan.block / 64) <= 32, "wavefronts per unit");
      replay(plan, n, in, "resident");
    }
  }
  EXPECT(resident_plans > 500, "only %d resident plans exercised", resident_plans);
  // the dense kernel divides by the wavefront count with a 20-bit reciprocal, rows per workgroup up to 65535
  for (int nw = 1; nw <= 16; ++nw) {
    const int64_t inv = (1 << 20) / nw + 1;
    for (int64_t v = 0; v <= 65535; ++v)
      if (((v * inv) >> 20) != v / nw) { EXPECT(false, "20-bit reciprocal: %lld / %d", (long long)v, nw); break; }
  }
  if (failures) { std::printf("%d failures\n", failures); return 1; }
  std::printf("ok %d resident plans\n", resident_plans);
  return 0;
}
