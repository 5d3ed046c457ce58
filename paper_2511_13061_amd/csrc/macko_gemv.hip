// Dense fp16 GEMV y = W x for gfx950: the SplitK scheme of Section 4.3 of the
// paper (lanes of one wavefront split a row's dot product, a cross-lane sum
// finishes it), with 64-lane wavefronts, 16-byte loads per lane, x staged in
// LDS and fp32 accumulation.  This is the baseline the sparse product is
// compared with.
#include "macko_device.h"
#include "macko_internal.h"
#include "macko_plan.h"

#include <climits>

namespace macko {
namespace {

// launches with at most this many wavefront steps per compute unit run as one resident round
constexpr int64_t kResidentStepsPerCu = 256;

// Fast path: cols and ld multiples of 8, W 16-byte aligned.  One wavefront per
// row; per step a lane multiplies 8 consecutive weights with 8 consecutive x.
// A wavefront owns a contiguous share of the workgroup's rows and treats them as
// one stream of (row, step) items: loads run RING items ahead of the arithmetic
// and cross row boundaries, every item issues exactly one load, and the results
// of up to 64 rows are collected in a register and stored with one coalesced
// store.
// One matrix of a grouped launch.  Its rows are dealt out evenly over its
// workgroups: q rows each, one more for the first r of them.
struct GemvMat {
  const uint4* W;
  const uint16_t* x;
  uint16_t* y;
  int64_t ld8;
  int rows, cols, q, r;
  int pad[4];
};
struct GemvGroupArgs {
  GemvMat m[kMaxGroup];
};
// Workgroups [wg_begin[i], wg_begin[i+1]) work on matrix i (wg_begin[0] = 0); unused
// slots hold INT_MAX.  Passed, with inv_nwaves, as separate scalar kernel arguments in
// front of the descriptors so that they can reach a starting wavefront in registers.
struct GemvGroupHeader {
  int wg_begin[kMaxGroup];
  int inv_nwaves;          // floor(2^20 / wavefronts per workgroup) + 1
};

// The work of one workgroup: workgroup number `wg` of the given matrix, whose
// rows are dealt out q (+1 for the first r workgroups) at a time.
template <int RING>
__device__ __forceinline__ void gemv_wave_row_body(const uint4* __restrict__ W, const uint16_t* __restrict__ x,
                                                   uint16_t* __restrict__ y, const int64_t ld8, const int cols,
                                                   const int q, const int r, const int wg,
                                                   const uint32_t waves) {
  extern __shared__ __align__(16) unsigned char lds[];
  // this workgroup's rows, then this wavefront's share of them (both dealt out evenly)
  const int row_begin = wg * q + min(wg, r);
  const int wg_rows = q + (wg < r ? 1 : 0);
  // waves: floor(2^20 / wavefronts per workgroup) + 1 in bits 0..20, wavefronts per workgroup above (an
  // argument that arrives in a register; blockDim would be a load from the dispatch's argument block)
  const int inv_nwaves = (int)(waves & 0x1FFFFFu), nwaves = (int)(waves >> 21);
  const int nthreads = 64 * nwaves;
  const uint4* xs = reinterpret_cast<const uint4*>(lds + kFrontPad);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c8 = cols >> 3;                            // 16-byte chunks per row
  const int nsteps = (c8 + 63) >> 6;
  const bool ragged = (c8 & 63) != 0;                  // last step only partly inside the row
  // wg_rows / nwaves, exact for wg_rows < 2^16 (the host keeps it below)
  const int per_wave = (int)(((uint64_t)(uint32_t)wg_rows * (uint32_t)inv_nwaves) >> 20);
  const int extra = wg_rows - per_wave * nwaves;
  const int wrow_begin = row_begin + wave * per_wave + min(wave, extra);
  const int wrow_end = wrow_begin + per_wave + (wave < extra ? 1 : 0);

  int blk = wrow_begin;
  int nb = max(0, min(64, wrow_end - blk));
  int ld_i = 0, ld_step = 0;                           // load side
  int cp_i = 0, cp_step = 0;                           // compute side
  const uint4* src = W;                                // row the next load reads from
  const uint4* src_next = W;
  int chunk = min(lane, c8 - 1);
  uint4 ring[RING];
  auto issue = [&](int j) {
    src = src_next;
    if (ld_i < nb) {
      chunk = min(ld_step * 64 + lane, c8 - 1);
      if (++ld_step == nsteps) {
        ld_step = 0;
        if (++ld_i < nb) src_next = src + ld8;
      }
    }
    ring[j] = load_stream(src + chunk);                   // padding items re-read the previous address
  };
  auto open_block = [&]() {
    ld_i = ld_step = cp_i = cp_step = 0;
    if (nb > 0) src_next = W + (int64_t)blk * ld8;
#pragma unroll
    for (int j = 0; j < RING; ++j) issue(j);
  };

  // x is requested first, then the first weight loads go out, and only then is
  // x written to LDS: the stream is already in flight behind the barrier
  XStage xst;
  stage_x_begin(xst, x, cols, nthreads);
  open_block();
  stage_x_finish<false>(lds, xst, x, cols, kFrontPad, kBackPad, nthreads);   // ends with a barrier

  while (true) {
    float yv = 0.0f;                                   // lane i: result of row blk + i
    float acc = 0.0f;
    while (cp_i < nb) {
#pragma unroll
      for (int j = 0; j < RING; ++j) {
        uint4 w = ring[j];
        const bool live = cp_i < nb;
        if (!live) cp_step = 0;
        const int idx = cp_step * 64 + lane;
        if (!live || (ragged && cp_step == nsteps - 1)) {
          const bool in = live && idx < c8;
          w.x = in ? w.x : 0u;
          w.y = in ? w.y : 0u;
          w.z = in ? w.z : 0u;
          w.w = in ? w.w : 0u;
        }
        const uint4 xv = xs[idx];                      // chunks past the row end read the zero guard
#define MACKO_LO(u) f16_bits_to_f32((uint16_t)((u) & 0xFFFFu))
#define MACKO_HI(u) f16_bits_to_f32((uint16_t)((u) >> 16))
        acc = fmaf(MACKO_LO(w.x), MACKO_LO(xv.x), acc);
        acc = fmaf(MACKO_HI(w.x), MACKO_HI(xv.x), acc);
        acc = fmaf(MACKO_LO(w.y), MACKO_LO(xv.y), acc);
        acc = fmaf(MACKO_HI(w.y), MACKO_HI(xv.y), acc);
        acc = fmaf(MACKO_LO(w.z), MACKO_LO(xv.z), acc);
        acc = fmaf(MACKO_HI(w.z), MACKO_HI(xv.z), acc);
        acc = fmaf(MACKO_LO(w.w), MACKO_LO(xv.w), acc);
        acc = fmaf(MACKO_HI(w.w), MACKO_HI(xv.w), acc);
#undef MACKO_LO
#undef MACKO_HI
        issue(j);
        if (live && ++cp_step == nsteps) {
          const float total = wave_sum_to_last_lane(acc);
          const int tbits = __builtin_amdgcn_readlane(__builtin_bit_cast(int, total), 63);
          yv = lane == cp_i ? __builtin_bit_cast(float, tbits) : yv;
          acc = 0.0f;
          cp_step = 0;
          ++cp_i;
        }
      }
    }
    if (lane < nb) y[blk + lane] = f32_to_f16_bits(yv);
    blk += 64;
    if (blk >= wrow_end) break;
    nb = min(64, wrow_end - blk);
    open_block();
  }
}

// Grouped launch: the workgroup first finds its matrix.
template <int RING>
__global__ void __launch_bounds__(1024)
gemv_wave_row_kernel(const int wb1, const int wb2, const int wb3, const int wb4, const int wb5, const int wb6,
                     const int wb7, const uint32_t waves, const GemvGroupArgs g) {
  static_assert(kMaxGroup == 8, "one scalar argument per group slot");
  int mi = 0, wg0 = 0;
  const int wbs[kMaxGroup] = {0, wb1, wb2, wb3, wb4, wb5, wb6, wb7};
#pragma unroll
  for (int i = 1; i < kMaxGroup; ++i) {
    const bool in = (int)blockIdx.x >= wbs[i];
    mi = in ? i : mi;
    wg0 = in ? wbs[i] : wg0;
  }
  gemv_wave_row_body<RING>(g.m[mi].W, g.m[mi].x, g.m[mi].y, g.m[mi].ld8, g.m[mi].cols, g.m[mi].q, g.m[mi].r,
                           (int)blockIdx.x - wg0, waves);
}

// One matrix: all scalar arguments, no argument load before the first weights are requested.
template <int RING>
__global__ void __launch_bounds__(1024)
gemv_wave_row_kernel(const uint4* __restrict__ W, const uint16_t* __restrict__ x, uint16_t* __restrict__ y,
                     const int64_t ld8, const int cols, const int q, const int r, const uint32_t waves) {
  gemv_wave_row_body<RING>(W, x, y, ld8, cols, q, r, (int)blockIdx.x, waves);
}

// Any shape / alignment: one wavefront per row, 2-byte loads, x from global.
__global__ void __launch_bounds__(256)
gemv_generic_kernel(const uint16_t* __restrict__ W, const uint16_t* __restrict__ x,
                    uint16_t* __restrict__ y, int rows, int cols, int64_t ld) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  for (int row = blockIdx.x * nwaves + wave; row < rows; row += gridDim.x * nwaves) {
    const uint16_t* wr = W + (int64_t)row * ld;
    float acc = 0.0f;
    for (int c = lane; c < cols; c += 64) acc = fmaf(f16_bits_to_f32(wr[c]), f16_bits_to_f32(x[c]), acc);
    acc = wave_sum_to_last_lane(acc);
    if (lane == 63) y[row] = f32_to_f16_bits(acc);
  }
}

}  // namespace

int launch_gemv_group(int n, const GemvProblem* problems, hipStream_t stream) {
  if (n < 1 || n > kMaxGroup) return MACKO_E_INVALID_ARG;
  const Tuning& t = tuning();
  const int cus = device_cu_count();
  const GemvProblem* wr[kMaxGroup];
  PlanInput in[kMaxGroup];
  int nwr = 0;
  int64_t max_lds = 0, total_steps = 0;
  for (int i = 0; i < n; ++i) {
    const GemvProblem& p = problems[i];
    if (p.rows == 0) continue;
    const int64_t lds_bytes = lds_bytes_for(p.cols);
    const bool fast = p.cols > 0 && (p.cols % 8 == 0) && (p.ld % 8 == 0) &&
                      (reinterpret_cast<uintptr_t>(p.W) & 15) == 0 && lds_bytes <= 160 * 1024 - 64;
    if (!fast) {                                        // any shape / alignment: own launch
      const int64_t grid = std::min<int64_t>((p.rows + 3) / 4, (int64_t)cus * 8);
      hipLaunchKernelGGL(gemv_generic_kernel, dim3((unsigned)std::max<int64_t>(grid, 1)), dim3(256), 0,
                         stream, static_cast<const uint16_t*>(p.W), static_cast<const uint16_t*>(p.x),
                         static_cast<uint16_t*>(p.y), (int)p.rows, (int)p.cols, p.ld);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return hip_fail(e);
      continue;
    }
    wr[nwr] = &p;
    in[nwr].rows = p.rows;
    in[nwr].steps_per_row = (p.cols / 8 + 63) / 64;
    in[nwr].lds_bytes = lds_bytes;
    total_steps += in[nwr].rows * in[nwr].steps_per_row;
    max_lds = std::max(max_lds, lds_bytes);
    ++nwr;
  }
  if (nwr == 0) return MACKO_OK;

  // same two regimes as the sparse product: one resident round of workgroups
  // shaped to the row counts when there is little work, many workgroups otherwise
  Plan plan;
  bool planned = false;
  const bool small = total_steps <= (int64_t)cus * kResidentStepsPerCu;
  // Rows that are a multiple of 4096 bytes apart (4096 or 8192 columns): as for the sparse product, many
  // 256-thread workgroups instead of workgroups that all start at a row start together (measured on the
  // 7B-shaped layer: {gate,up} 31.3 -> 29.6 us, {q,k,v} 18.7 -> 18.0, {o} 7.3 -> 7.1).  The baseline gets
  // every launch-side improvement the sparse kernel gets.
  bool in_step = t.gemv_resident == 0 && t.gemv_block == 0;
  for (int i = 0; i < nwr; ++i) in_step = in_step && wr[i]->ld % 2048 == 0 && wr[i]->cols <= 8192;
  if (!in_step && t.gemv_rows_per_wg == 0 && (t.gemv_resident == 2 || (t.gemv_resident == 0 && small)))
    planned = plan_resident(plan, nwr, in, cus, (int)t.gemv_block, (int)t.gemv_wgs_per_cu);
  if (!planned) {
    const int block = t.gemv_block ? (int)t.gemv_block : (in_step ? 256 : 512);
    const int nwaves = block / 64;
    int64_t rpw[kMaxGroup];
    for (int i = 0; i < nwr; ++i) {
      rpw[i] = t.gemv_rows_per_wg;
      if (rpw[i] == 0) {
        const int64_t target_wgs = (int64_t)cus * 16;
        rpw[i] = std::max<int64_t>((in[i].rows + target_wgs - 1) / target_wgs, nwaves);
      }
      rpw[i] = std::min<int64_t>(rpw[i], 65535);        // the kernel's division by the wavefront count
    }
    plan.block = block;
    plan.total_wgs = 0;
    for (int i = 0; i < nwr; ++i) {
      plan_split(plan.m[i], in[i].rows, (in[i].rows + rpw[i] - 1) / rpw[i]);
      plan.total_wgs += plan.m[i].nwg;
    }
  }
  if (plan.total_wgs >= (int64_t{1} << 31)) return MACKO_E_UNSUPPORTED;

  GemvGroupArgs args{};
  GemvGroupHeader head{};
  head.inv_nwaves = (1 << 20) / (plan.block / 64) + 1;
  int64_t wg_begin = 0;
  for (int i = 0; i < kMaxGroup; ++i) head.wg_begin[i] = INT32_MAX;
  for (int i = 0; i < nwr; ++i) {
    const GemvProblem& p = *wr[i];
    GemvMat& m = args.m[i];
    m.W = static_cast<const uint4*>(p.W);
    m.x = static_cast<const uint16_t*>(p.x);
    m.y = static_cast<uint16_t*>(p.y);
    m.ld8 = p.ld / 8;
    m.rows = (int)p.rows;
    m.cols = (int)p.cols;
    m.q = plan.m[i].q;
    m.r = plan.m[i].r;
    head.wg_begin[i] = (int)wg_begin;
    wg_begin += plan.m[i].nwg;
  }
  const dim3 grid((unsigned)plan.total_wgs), blockdim(plan.block);
  const uint32_t waves = (uint32_t)head.inv_nwaves | ((uint32_t)(plan.block / 64) << 21);
  auto lds_limit = [&](const void* fn) -> int {
    if (max_lds <= 64 * 1024) return MACKO_OK;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_lds);
    return e == hipSuccess ? MACKO_OK : hip_fail(e);
  };
  if (nwr == 1) {
    using K1 = void (*)(const uint4*, const uint16_t*, uint16_t*, int64_t, int, int, int, uint32_t);
    K1 kfn = t.gemv_ring == 2 ? (K1)gemv_wave_row_kernel<2>
             : t.gemv_ring == 8 ? (K1)gemv_wave_row_kernel<8> : (K1)gemv_wave_row_kernel<4>;
    int st = lds_limit(reinterpret_cast<const void*>(kfn));
    if (st != MACKO_OK) return st;
    const GemvMat& m = args.m[0];
    hipLaunchKernelGGL(kfn, grid, blockdim, (size_t)max_lds, stream, m.W, m.x, m.y, m.ld8, m.cols, m.q, m.r, waves);
  } else {
    using KG = void (*)(int, int, int, int, int, int, int, uint32_t, GemvGroupArgs);
    KG kfn = t.gemv_ring == 2 ? (KG)gemv_wave_row_kernel<2>
             : t.gemv_ring == 8 ? (KG)gemv_wave_row_kernel<8> : (KG)gemv_wave_row_kernel<4>;
    int st = lds_limit(reinterpret_cast<const void*>(kfn));
    if (st != MACKO_OK) return st;
    hipLaunchKernelGGL(kfn, grid, blockdim, (size_t)max_lds, stream, head.wg_begin[1], head.wg_begin[2],
                       head.wg_begin[3], head.wg_begin[4], head.wg_begin[5], head.wg_begin[6], head.wg_begin[7],
                       waves, args);
  }
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MACKO_OK : hip_fail(e);
}

}  // namespace macko
