// Host-side check of the launch planner (csrc/macko_plan.h): for random groups of
// matrices, replay the row assignment the kernels derive from a plan and verify
// that every row is taken exactly once, that no wavefront gets more than 64 rows,
// that the reciprocal multiply the kernels use equals the division, and that a
// resident round has exactly (workgroups per compute unit) x (compute units)
// workgroups.  Chains (several phases in one launch whose workgroups wait for each other): every
// phase deals its rows out exactly once within the one round, and a chain whose round would not
// be resident as a whole is refused.  Built and run by tests/test_library_host.py; prints "ok" on success.
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
  // ---- chains ----------------------------------------------------------------------------
  // residency rule: pessimistic packing of a workgroup's wavefronts over the four SIMDs
  EXPECT(resident_wgs_per_cu(52, 13, 24576 + 16) == 2, "13 wavefronts at 52 registers: 4 + 4 per SIMD fit");
  EXPECT(resident_wgs_per_cu(72, 13, 24576 + 16) == 1, "13 wavefronts at 72 registers: 7 per SIMD hold one workgroup's 4");
  EXPECT(resident_wgs_per_cu(64, 16, 24576) == 2, "16 wavefronts at 64 registers");
  EXPECT(resident_wgs_per_cu(65, 16, 24576) == 1, "16 wavefronts at 65 registers");
  EXPECT(resident_wgs_per_cu(40, 8, 100 * 1024) == 1, "LDS for one workgroup only");
  EXPECT(resident_wgs_per_cu(40, 8, 161 * 1024) == 0, "LDS for none");
  EXPECT(resident_wgs_per_cu(300, 4, 1024) == 1 && resident_wgs_per_cu(600, 4, 1024) == 0, "register limits");
  {
    // the decoder-layer chain: {q,k,v} -> {o} -> {gate,up} -> {down}
    const int sizes[4] = {3, 1, 2, 1};
    PlanInput in[7];
    const int64_t rows[7] = {4096, 4096, 4096, 4096, 11008, 11008, 4096};
    const int64_t cols[7] = {4096, 4096, 4096, 4096, 4096, 4096, 11008};
    for (int i = 0; i < 7; ++i) in[i] = PlanInput{rows[i], (cols[i] / 2 + 511) / 512, 2 * cols[i] + 2560};
    ChainPlan cp;
    int asked = 0;
    const bool ok = plan_chain(cp, 4, sizes, in, 256, [&](int block) { ++asked; return resident_wgs_per_cu(52, block / 64, 24576); });
    EXPECT(ok && asked >= 1 && cp.wgs_per_cu == 2 && cp.total_wgs == 512, "layer chain: ok %d k %d wgs %lld", ok, cp.wgs_per_cu, (long long)cp.total_wgs);
    // the same chain on a device that holds one such workgroup per compute unit: one per compute unit
    const bool ok1 = plan_chain(cp, 4, sizes, in, 256, [&](int) { return 1; });
    EXPECT(ok1 && cp.wgs_per_cu == 1 && cp.total_wgs == 256, "k = 1 plan: ok %d k %d", ok1, cp.wgs_per_cu);
    // and on one that holds none: refused, never launched
    EXPECT(!plan_chain(cp, 4, sizes, in, 256, [&](int) { return 0; }), "a round that is not resident must be refused");
    // too many phases / products, empty phases, matrices without rows
    const int nine[9] = {1, 1, 1, 1, 1, 1, 1, 1, 1};
    EXPECT(!plan_chain(cp, 9, nine, in, 256, [&](int) { return 2; }), "9 phases");
    const int zero[2] = {1, 0};
    EXPECT(!plan_chain(cp, 2, zero, in, 256, [&](int) { return 2; }), "empty phase");
    PlanInput none = in[0];
    none.rows = 0;
    const int one[1] = {1};
    EXPECT(!plan_chain(cp, 1, one, &none, 256, [&](int) { return 2; }), "matrix without rows");
    // x too large for two workgroups' LDS: one per compute unit
    PlanInput wide = PlanInput{8192, 40, 100 * 1024};
    const bool okw = plan_chain(cp, 1, one, &wide, 256, [&](int) { return 4; });
    EXPECT(okw && cp.wgs_per_cu == 1, "wide x: ok %d k %d", okw, cp.wgs_per_cu);
  }
  for (int t = 0; t < 1500; ++t) {
    const int n_phases = 1 + (int)(rng() % kMaxChainPhases);
    int sizes[kMaxChainPhases];
    PlanInput in[kMaxChainMats];
    int total = 0;
    for (int p = 0; p < n_phases; ++p) {
      sizes[p] = 1 + (int)(rng() % 3);
      if (total + sizes[p] > kMaxChainMats) sizes[p] = 1;
      total += sizes[p];
    }
    if (total > kMaxChainMats) continue;
    for (int i = 0; i < total; ++i) {
      const int64_t rows = (rng() % 4 == 0) ? 1 + (int64_t)(rng() % 900) : 1 + (int64_t)(rng() % 60000);
      in[i] = PlanInput{rows, 1 + (int64_t)(rng() % 40), 2048 + (int64_t)(rng() % 60000)};
    }
    const int cus = (rng() % 3 == 0) ? 256 : 1 + (int)(rng() % 300);
    const int cap = (int)(rng() % 4);                       // workgroups the device holds per compute unit
    ChainPlan cp;
    const bool ok = plan_chain(cp, n_phases, sizes, in, cus, [&](int) { return cap; });
    if (!ok) continue;
    EXPECT(cp.wgs_per_cu >= 1 && cp.wgs_per_cu <= cap && cp.wgs_per_cu <= 2, "chain k %d with room for %d", cp.wgs_per_cu, cap);
    EXPECT(cp.total_wgs == (int64_t)cus * cp.wgs_per_cu, "chain round %lld on %d compute units", (long long)cp.total_wgs, cus);
    EXPECT(cp.block % 64 == 0 && cp.block >= 64 && cp.block <= 1024, "chain block %d", cp.block);
    int at = 0;
    for (int p = 0; p < n_phases; ++p) {
      EXPECT(cp.nwaves[p] >= 1 && cp.nwaves[p] * 64 <= cp.block, "phase %d works with %d wavefronts of %d threads", p, cp.nwaves[p], cp.block);
      // replay the phase as a plan of its own at its own wavefront count
      Plan ph;
      ph.block = cp.nwaves[p] * 64;
      ph.total_wgs = 0;
      for (int i = 0; i < sizes[p]; ++i) {
        ph.m[i] = cp.m[at + i];
        ph.total_wgs += ph.m[i].nwg;
      }
      EXPECT(ph.total_wgs <= cp.total_wgs, "phase %d uses %lld of %lld workgroups", p, (long long)ph.total_wgs, (long long)cp.total_wgs);
      replay(ph, sizes[p], in + at, "chain phase");
      at += sizes[p];
    }
  }

  if (failures) { std::printf("%d failures\n", failures); return 1; }
  std::printf("ok %d resident plans\n", resident_plans);
  return 0;
}
