// Launch shapes of the wavefront-per-row kernels (sparse and dense), host side.
//
// A wavefront works on whole rows, a workgroup on a contiguous range of rows,
// and every workgroup keeps its own copy of x in LDS.  Two regimes:
//
//  * plenty of work (large matrices): many more workgroups than the chip holds,
//    about 16 steps of work per wavefront.  The dispatcher hands a new
//    workgroup to whichever compute unit finishes one, so the load balances
//    itself and the size of the last round hardly matters.
//  * little work (the few-microsecond products of one decoder layer): the whole
//    launch is resident at once, so its duration is that of the slowest
//    wavefront.  Rows cannot be split, and with only a handful of rows per
//    wavefront the rounding matters (43 rows per compute unit on 16 wavefronts
//    is 3,3,...,2: 10 % lost; on 22 wavefronts it is 2,2,...,1: 2 % lost).  The
//    planner therefore picks workgroups per compute unit and wavefronts per
//    workgroup such that the largest per-wavefront share, times the number of
//    resident wavefronts that share the memory system, is smallest, and launches
//    exactly a multiple of the compute-unit count.
//
// In both regimes rows are dealt out evenly: q rows per workgroup and one more
// for the first r workgroups; the same again over the wavefronts of a workgroup.
#pragma once

#include <algorithm>
#include <cstdint>

#include "macko_internal.h"

namespace macko {

struct PlanInput {
  int64_t rows;            // > 0
  int64_t steps_per_row;   // wavefront steps an average row takes (>= 1)
  int64_t lds_bytes;       // LDS a workgroup needs for this matrix's x
};

struct PlanMat {
  int nwg;                 // workgroups that work on this matrix
  int q, r;                // rows per workgroup: q, and q + 1 for the first r workgroups
};

struct Plan {
  int block = 0;           // threads per workgroup
  int64_t total_wgs = 0;
  PlanMat m[kMaxGroup] = {};
};

constexpr int64_t kPlanLdsPerCu = 160 * 1024;
constexpr int kPlanMaxRowsPerWave = 64;   // a wavefront keeps its rows' results in one register

inline void plan_split(PlanMat& pm, int64_t rows, int64_t nwg) {
  pm.nwg = (int)nwg;
  pm.q = (int)(rows / nwg);
  pm.r = (int)(rows % nwg);
}

// Oversubscribed regime: `rows_per_wave` rows for every wavefront of a workgroup.
inline void plan_by_rows_per_wg(Plan& plan, int n, const PlanInput* in, int block, const int64_t* rows_per_wg) {
  plan.block = block;
  plan.total_wgs = 0;
  for (int i = 0; i < n; ++i) {
    const int64_t cap = (int64_t)kPlanMaxRowsPerWave * (block / 64);
    const int64_t rpw = std::max<int64_t>(1, std::min(rows_per_wg[i], cap));
    plan_split(plan.m[i], in[i].rows, (in[i].rows + rpw - 1) / rpw);
    plan.total_wgs += plan.m[i].nwg;
  }
}

// Resident regime: try every allowed (workgroups per compute unit, wavefronts
// per workgroup) and keep the one with the smallest modelled duration.  Two
// workgroups per compute unit unless the caller forces another number: measured
// on the decoder-layer shapes, one, three and four are within a few per cent of
// two and none is better across the board.  Returns false when the group has too
// few rows for the model to mean anything.
inline bool plan_resident(Plan& plan, int n, const PlanInput* in, int cus, int forced_block, int forced_k) {
  int64_t total_rows = 0, total_work = 0, max_lds = 0;
  for (int i = 0; i < n; ++i) {
    total_rows += in[i].rows;
    total_work += in[i].rows * in[i].steps_per_row;
    max_lds = std::max(max_lds, in[i].lds_bytes);
  }
  if (total_rows < (int64_t)cus * 4) return false;
  double best_cost = 0;
  int best_k = 0, best_nw = 0;
  PlanMat best_m[kMaxGroup] = {};
  for (int k = 1; k <= 4; ++k) {
    if (k != (forced_k ? forced_k : 2)) continue;
    if (k * max_lds > kPlanLdsPerCu) continue;
    for (int nw = 4; nw <= 16; ++nw) {
      if (forced_block && nw * 64 != forced_block) continue;
      const int waves = k * nw;
      if (waves > 32) continue;
      const int64_t wgs = (int64_t)cus * k;
      if (waves < 12 && total_rows >= (int64_t)cus * 12) continue;  // too few loads in flight
      // deal the workgroups out in proportion to the work, every matrix at least one
      PlanMat pm[kMaxGroup];
      int64_t given = 0;
      int largest = 0;
      bool ok = true;
      for (int i = 0; i < n; ++i) {
        const double share = (double)wgs * (double)(in[i].rows * in[i].steps_per_row) / (double)total_work;
        int64_t g = std::max<int64_t>(1, (int64_t)(share + 0.5));
        g = std::min<int64_t>(g, in[i].rows);
        plan_split(pm[i], in[i].rows, g);
        given += g;
        if (in[i].rows * in[i].steps_per_row > in[largest].rows * in[largest].steps_per_row) largest = i;
      }
      const int64_t fix = pm[largest].nwg + (wgs - given);
      if (fix < 1 || fix > in[largest].rows) continue;
      plan_split(pm[largest], in[largest].rows, fix);
      int64_t worst = 0;
      for (int i = 0; i < n; ++i) {
        const int64_t rows_wg = pm[i].q + (pm[i].r ? 1 : 0);
        const int64_t rows_wave = (rows_wg + nw - 1) / nw;
        if (rows_wave > kPlanMaxRowsPerWave) ok = false;
        worst = std::max(worst, rows_wave * in[i].steps_per_row);
      }
      if (!ok) continue;
      // all resident wavefronts share the memory system: time ~ slowest share x wavefronts;
      // a mild preference for 16..24 wavefronts per compute unit and for fewer, larger workgroups
      double cost = (double)worst * waves;
      cost *= 1.0 + 0.002 * std::abs(waves - 20) + 0.001 * k;
      if (best_k == 0 || cost < best_cost) {
        best_cost = cost;
        best_k = k;
        best_nw = nw;
        std::copy(pm, pm + n, best_m);
      }
    }
  }
  if (best_k == 0) return false;
  plan.block = best_nw * 64;
  plan.total_wgs = (int64_t)cus * best_k;
  std::copy(best_m, best_m + n, plan.m);
  return true;
}

// ---------------------------------------------------------------------------
// A chain: phases of independent products executed in order by ONE launch of
// workgroups that all have to be on the chip at the same time, because a phase
// may only read its inputs once every workgroup has finished the phase before
// (the workgroups wait for each other inside the kernel).  The launch is one
// resident round of k workgroups per compute unit, k the same for every phase;
// a phase uses the first `nwaves` wavefronts of every workgroup, the others idle
// through it.  A plan whose workgroups cannot all be resident is refused: the
// waiting workgroups would hold the compute units that the missing ones need.
// ---------------------------------------------------------------------------
constexpr int kMaxChainPhases = 8;      // MACKO_MAX_CHAIN_PHASES
constexpr int kMaxChainMats = 16;       // MACKO_MAX_CHAIN_PRODUCTS

// Workgroups of `waves` wavefronts that one compute unit certainly holds at the same time, from the
// kernel's vector registers per lane and the LDS one workgroup needs.  Deliberately pessimistic: the
// wavefronts of a workgroup are dealt to the four SIMDs in turn starting anywhere, so each SIMD must
// have room for ceil(waves / 4) of them per workgroup (the runtime's occupancy query packs ideally
// and promised two workgroups of 13 wavefronts at 72 registers, of which only one was resident).
// A SIMD has 512 registers per lane, handed out in blocks of 8, and at most 8 wavefronts.
inline int resident_wgs_per_cu(int vgprs, int waves, int64_t lds_bytes) {
  if (vgprs < 1 || waves < 1 || waves > 16) return 0;
  const int per_wave = (vgprs + 7) / 8 * 8;
  const int waves_per_simd = std::min(8, 512 / per_wave);
  const int by_waves = waves_per_simd / ((waves + 3) / 4);
  const int64_t by_lds = lds_bytes > 0 ? kPlanLdsPerCu / ((lds_bytes + 1023) / 1024 * 1024) : 64;
  return (int)std::min<int64_t>(by_waves, by_lds);
}

struct ChainPlan {
  int wgs_per_cu = 0;       // k
  int64_t total_wgs = 0;    // k x compute units: the whole launch
  int block = 0;            // threads per workgroup: the widest phase
  int nwaves[kMaxChainPhases] = {};        // wavefronts a phase works with
  PlanMat m[kMaxChainMats] = {};           // per product, in phase order
};

// sizes[p] products in phase p; in[] holds them in phase order.  max_wgs_per_cu(block) is
// what the device can hold of the kernel at that workgroup size (the occupancy
// the runtime reports, LDS included).  Returns false when no admissible plan exists.
template <class Occupancy>
inline bool plan_chain(ChainPlan& cp, int n_phases, const int* sizes, const PlanInput* in, int cus,
                       Occupancy max_wgs_per_cu) {
  if (n_phases < 1 || n_phases > kMaxChainPhases || cus < 1) return false;
  int total = 0;
  int64_t max_lds = 0;
  for (int p = 0; p < n_phases; ++p) {
    if (sizes[p] < 1 || sizes[p] > kMaxGroup) return false;
    total += sizes[p];
  }
  if (total > kMaxChainMats) return false;
  for (int i = 0; i < total; ++i) {
    if (in[i].rows < 1) return false;
    max_lds = std::max(max_lds, in[i].lds_bytes);
  }
  for (int k = 2; k >= 1; --k) {
    if (k * max_lds > kPlanLdsPerCu) continue;
    ChainPlan c;
    c.wgs_per_cu = k;
    c.total_wgs = (int64_t)cus * k;
    bool ok = true;
    int at = 0;
    for (int p = 0; p < n_phases && ok; ++p) {
      Plan ph;
      const int n = sizes[p];
      if (!plan_resident(ph, n, in + at, cus, 0, k)) {
        // too few rows for a full round: one wavefront-sized share per workgroup, the matrices
        // side by side, the remaining workgroups idle through this phase
        int64_t given = 0;
        ph.block = 4 * 64;
        for (int i = 0; i < n; ++i) {
          const int64_t want = (in[at + i].rows + 3) / 4;
          const int64_t g = std::max<int64_t>(1, std::min<int64_t>(want, c.total_wgs / n));
          plan_split(ph.m[i], in[at + i].rows, std::min<int64_t>(g, in[at + i].rows));
          given += ph.m[i].nwg;
        }
        if (given > c.total_wgs) ok = false;
        // and few enough rows per wavefront: widen the workgroup if need be
        for (int nw = 4; nw <= 16 && ok; ++nw) {
          bool fits = true;
          for (int i = 0; i < n; ++i) {
            const int64_t rows_wg = ph.m[i].q + (ph.m[i].r ? 1 : 0);
            if ((rows_wg + nw - 1) / nw > kPlanMaxRowsPerWave) fits = false;
          }
          ph.block = nw * 64;
          if (fits) break;
          if (nw == 16) ok = false;
        }
      }
      if (!ok) break;
      c.nwaves[p] = ph.block / 64;
      c.block = std::max(c.block, ph.block);
      for (int i = 0; i < n; ++i) {
        c.m[at + i] = ph.m[i];
        const int64_t rows_wg = ph.m[i].q + (ph.m[i].r ? 1 : 0);
        if ((rows_wg + c.nwaves[p] - 1) / c.nwaves[p] > kPlanMaxRowsPerWave || rows_wg > 1024) ok = false;
      }
      at += n;
    }
    if (!ok) continue;
    if (max_wgs_per_cu(c.block) < k) continue;          // not all resident at once: refused
    cp = c;
    return true;
  }
  return false;
}

}  // namespace macko
