// MACKO sparse matrix-vector product for gfx950 (Section 4.4 of the paper,
// re-designed for 64-lane wavefronts).
//
// Per step a lane owns 8 consecutive stored entries: one 32-bit word of packed
// 4-bit codes and one 128-bit vector of fp16 values, so a wavefront streams
// 256 B of deltas and 1024 B of values per step, fully coalesced.  Column
// positions are rebuilt in registers (per-lane SWAR prefix over the 8 codes,
// then a DPP prefix sum over the lanes), the activation vector is gathered from
// LDS, products are accumulated in fp32 and reduced over the wavefront with DPP.
#include "macko_decode.h"
#include "macko_device.h"
#include "macko_internal.h"
#include "macko_plan.h"

#include <climits>
#include <mutex>

namespace macko {
namespace {

// ---------------------------------------------------------------------------
// Generic kernel: LANES (16, 32 or 64) lanes cooperate on a row, so a wavefront
// works on 64/LANES rows at once.  Every entry is individually masked against
// the row bounds.  Used for short rows and as the fallback
// when x does not fit in LDS (XLDS = false gathers x from global memory).
// ---------------------------------------------------------------------------
// The BD-bit codes of the 8 entries of chunk `chunk`, entry k in bits [BD k, BD (k+1)).
template <int BD>
__device__ __forceinline__ uint64_t load_chunk_codes(const uint32_t* __restrict__ deltas, uint32_t chunk) {
  if (BD == 1) return load_stream(reinterpret_cast<const uint8_t*>(deltas) + chunk);
  if (BD == 2) return load_stream(reinterpret_cast<const uint16_t*>(deltas) + chunk);
  if (BD == 4) return load_stream(deltas + chunk);
  const uint2 v = load_stream(reinterpret_cast<const uint2*>(deltas) + chunk);
  return (uint64_t)v.x | ((uint64_t)v.y << 32);
}

template <int LANES, bool XLDS, int BD>
__global__ void __launch_bounds__(1024)
spmv_subwave_kernel(const uint4* __restrict__ values, const uint32_t* __restrict__ deltas,
                    const uint32_t* __restrict__ row_ptr, const uint16_t* __restrict__ x,
                    uint16_t* __restrict__ y, int rows, int cols, int rows_per_wg) {
  extern __shared__ __align__(16) unsigned char lds[];
  if (XLDS) stage_x_to_lds(lds, x, cols);
  const uint16_t* xs = XLDS ? reinterpret_cast<const uint16_t*>(lds + kFrontPad) : x;

  const int groups = blockDim.x / LANES;
  const int group = threadIdx.x / LANES;
  const int gl = threadIdx.x % LANES;                 // lane within the row's group
  const int row_begin = blockIdx.x * rows_per_wg;
  const int row_end = min(rows, row_begin + rows_per_wg);

  for (int rb = row_begin; rb < row_end; rb += groups) {
    const int row = rb + group;
    const bool active = row < row_end;
    const uint32_t start = active ? row_ptr[row] : 0u;
    const uint32_t end = active ? row_ptr[row + 1] : 0u;
    uint32_t cur = start & ~7u;        // reverse-offset alignment: back up to an 8-entry boundary
    int pos = 0;                       // sum of deltas consumed so far = last column + 1
    float acc = 0.0f;
    while (__any(cur < end)) {
      const uint32_t e0 = cur + 8u * gl;
      uint64_t w = 0;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (e0 < end) {                  // the 8-entry chunk intersects [start, end)
        w = load_chunk_codes<BD>(deltas, e0 >> 3);
        v = load_stream(values + (e0 >> 3));
      }
      const uint32_t vv[4] = {v.x, v.y, v.z, v.w};
      int d[8];
      int local = 0;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const bool valid = (e0 + k >= start) && (e0 + k < end);
        d[k] = valid ? (int)((w >> (BD * k)) & ((1u << BD) - 1u)) + 1 : 0;
        local += d[k];
      }
      int incl = local;                // inclusive prefix over the group (Alg. 1)
#pragma unroll
      for (int off = 1; off < LANES; off <<= 1) {
        const int t = __shfl_up(incl, off, LANES);
        if (gl >= off) incl += t;
      }
      int p = pos + incl - local;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        p += d[k];
        if (d[k] != 0) {
          const uint16_t hv = (uint16_t)(vv[k >> 1] >> (16 * (k & 1)));
          acc = fmaf(f16_bits_to_f32(hv), f16_bits_to_f32(xs[p - 1]), acc);
        }
      }
      pos += __shfl(incl, LANES - 1, LANES);
      cur += 8u * LANES;
    }
#pragma unroll
    for (int off = LANES / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, LANES);
    if (active && gl == 0) y[row] = f32_to_f16_bits(acc);
  }
}

// ---------------------------------------------------------------------------
// Wave-per-row kernel: the fast path for rows of at least a few hundred
// entries.  Row bounds, step counts and the running column base are wavefront
// uniform and live in scalar registers.
//
// Position arithmetic is done in units of bytes of the LDS copy of x, i.e.
// doubled: an entry with code c advances the position by 2c + 2.  Within a lane
// the 8 doubled code prefixes (at most 2*15*8 = 240) fit the bytes of two 32-bit
// words; the constant part 2k of entry k is added bytewise to those words.
//
// A workgroup owns rows [row_begin, row_end); each of its wavefronts owns a
// contiguous share of them, at most 64 rows (the launcher sees to that).
// Lane i fetches row i's pointers once (one coalesced load); the
// scalar row bounds are then picked out of that register with v_readlane, and
// the results are collected in a register (lane i keeps row i's) and stored
// with one coalesced store.  The steady-state loop therefore contains no memory
// instruction other than the two streaming loads per item.
//
// The wavefront's rows form one stream of (row, step) items.  Loads run RING items
// ahead of the arithmetic and cross row boundaries, so the memory pipeline does
// not drain between rows.  Every item issues exactly one deltas load and one
// values load, unconditionally (lanes before the row start re-read the row's first
// chunk, lanes past the row end its last, items past the wavefront's last row re-read
// the last chunk once more), which lets the compiler count outstanding loads exactly.
//
// A row's first step begins at its start rounded down to 8 entries (Section 4.5) or, for
// long rows, to a larger power of two (see kStepAlign).  What a lane holds besides the row:
//  - lanes that lie wholly before the row start (first step, larger alignments only):
//    codes and values cleared; they advance 16 bytes each below x[0];
//  - entries of the previous row in the lane that holds the row start: the base is set
//    so that the row's first entry lands on its own column; the earlier entries then
//    decode to positions <= 0, which read the zero guard in front of x, and their values
//    are cleared as well (y_i depends on row i alone, also when a neighbour holds inf or NaN);
//  - after the row end (last step only): codes and values cleared.
// No load ever leaves [0, alloc_nnz).
// ---------------------------------------------------------------------------
// x element whose plain LDS offset relative to the start of x is q (q may be
// slightly negative or past the end: both land in the zero guards).
__device__ __forceinline__ float gather_x(const unsigned char* xbase, int q) {
  return f16_bits_to_f32(*reinterpret_cast<const uint16_t*>(xbase + q));
}

// One matrix of a grouped launch.  Its rows are dealt out evenly over its
// workgroups: q rows each, one more for the first r of them.
struct SpmvMat {
  const void* values;       // uint4 per chunk (16-bit values) or uint2 (8-bit values)
  const uint32_t* deltas;
  const uint32_t* row_ptr;
  const uint16_t* x;
  uint16_t* y;
  int rows, cols, q, r;
  int amask;                // alignment of a row's first step in entries, minus 1 (7 ... 511)
  int pad;
};
struct SpmvGroupArgs {
  SpmvMat m[kMaxGroup];
};
// Workgroups [wg_begin[i], wg_begin[i+1]) work on matrix i (wg_begin[0] = 0); unused
// slots hold INT_MAX.  These and inv_nwaves (packed with the wavefront count) are separate
// scalar kernel arguments in front of the descriptors: scalar arguments at the start of the
// argument list can be handed to a wavefront in registers when it starts, which saves one
// dependent load on the way to the first row pointer.
struct SpmvGroupHeader {
  int wg_begin[kMaxGroup];
  int inv_nwaves;          // floor(65536 / wavefronts per workgroup) + 1
};

// Rows of at least kAlignMinEntries stored entries begin their first step on a multiple of
// kStepAlign entries instead of where the row begins, so that the 1024 bytes of values and the
// 64 * BD bytes of codes a wavefront requests per step are whole, aligned cache lines that no
// other step touches (otherwise nine lines are touched for eight lines of values, and
// neighbouring steps share lines).  The lanes of the first step that lie wholly before the row
// are cleared and re-read the row's first chunk; the row costs a quarter step more on average.
// Measured on 36864 x 12288: 4-9 % faster from 25 % to 80 % sparsity (rows of 5 steps and
// more), 5-8 % slower at 90 % (3 steps), hence the threshold.  256 entries align the codes of
// 4-bit matrices to their 128-byte lines as well; 512 was no better.
constexpr int kStepAlign = 256;
constexpr int kMaxStepAlign = 512;                     // what the "spmv_step_align" knob may ask for
constexpr int64_t kAlignMinEntries = 1700;
// cleared lanes in front of a row advance 16 bytes each below x[0]: the front guard grows by that
constexpr int kAlignFrontPad = 2 * kMaxStepAlign;
__host__ __device__ constexpr int spmv_front_pad(int b_delta) { return front_pad_for(b_delta) + kAlignFrontPad; }
__host__ __device__ inline int64_t spmv_lds_bytes(int64_t cols, int b_delta) {
  return lds_bytes_for(cols, b_delta) + kAlignFrontPad;
}

// The work of one workgroup: workgroup number `wg` of the matrix given by the
// pointers, whose rows are dealt out q (+1 for the first r workgroups) at a time.
// Gate: what has to happen before x may be read.  The plain kernels have none; a chain's later
// phases wait there for the workgroups that produce x (see spmv_chain_kernel).
struct NoGate {
  static constexpr bool kActive = false;
  __device__ __forceinline__ bool needed() const { return false; }
  __device__ __forceinline__ bool wait() const { return true; }
};

// `nwaves` wavefronts of the workgroup share its rows (all of them in the plain kernels; a chain
// may leave the last ones of a workgroup without rows in some phase: they only help to stage x).
// Returns false when the gate gave up; nothing has been written to y then.
template <int RING, bool SIMPLE, int BD, int VB = 16, class Gate = NoGate>
__device__ __forceinline__ bool spmv_wave_row_body(const void* __restrict__ values,
                                                   const uint32_t* __restrict__ deltas,
                                                   const uint32_t* __restrict__ row_ptr,
                                                   const uint16_t* __restrict__ x, uint16_t* __restrict__ y,
                                                   const int rows, const int cols, const int q, const int r,
                                                   const int wg, const int nwaves, const int inv_nwaves,
                                                   const uint32_t amask, const int block_threads,
                                                   const Gate gate = Gate()) {
  extern __shared__ __align__(16) unsigned char lds[];
  // this workgroup's rows, then this wavefront's share of them (both dealt out evenly)
  const int row_begin = wg * q + min(wg, r);
  const int wg_rows = q + (wg < r ? 1 : 0);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned char* xbase = lds + spmv_front_pad(BD);   // LDS address of x[0]
  const uint32_t lane8 = 8u * lane;
  const int per_wave = (wg_rows * inv_nwaves) >> 16;   // wg_rows / nwaves (exact for wg_rows <= 1024)
  const int extra = wg_rows - per_wave * nwaves;         // wg_rows % nwaves
  const bool has_rows = wave < nwaves;
  const int wrow_begin = row_begin + wave * per_wave + min(wave, extra);
  const int wrow_end = has_rows ? wrow_begin + per_wave + (wave < extra ? 1 : 0) : wrow_begin;

  uint32_t chunk = 0;      // 8-entry chunk index this lane loads next (chunk 0 exists: pad_nnz > 0)
  const int blk = wrow_begin;
  const int nb = wrow_end - wrow_begin;                // at most 64: the host sees to that
  uint32_t rp_lo = 0, rp_hi = 0;
  RowCursor ld, cp;                                    // load side, compute side
  LaneCodes<BD> wq[RING];
  LaneValues<VB> vq[RING];

  auto issue = [&](int j) {
    if (ld.i < nb) {
      const uint32_t e0 = ld.a0 + 512u * ld.step + lane8;
      // lanes before the row (first step) or past it (last step) re-read its first / last chunk
      chunk = min(max(e0, ld.start & ~7u), ld.end - 1u) >> 3;
      if (++ld.step == ld.nsteps) {
        ++ld.i;
        seek_nonempty(ld, nb, rp_lo, rp_hi, amask);
      }
    }                  // else a padding item: every lane re-reads its previous chunk (a line it has just
                       // used; one fixed address would make every wavefront queue at the same L2 channel)
    wq[j].load(deltas, chunk);
    vq[j].load(values, chunk);
  };
  auto fetch_row_ptrs = [&]() {                        // unconditional loads, clamped to the last row
    const int r = min(blk + lane, rows - 1);
    rp_lo = row_ptr[r];
    rp_hi = row_ptr[r + 1];
  };
  auto prime_ring = [&]() {
    ld.i = 0;
    seek_nonempty(ld, nb, rp_lo, rp_hi, amask);
    cp = ld;
#pragma unroll
    for (int j = 0; j < RING; ++j) issue(j);
  };

  // Start-up order: the row pointers and x are requested together; once they
  // are in registers the first streaming loads go out, and only then is x
  // written to LDS, so the stream is already in flight behind the barrier.
  // Behind a gate the matrix streams do not wait (they do not depend on what the gate waits for):
  // pointers and ring first, then the gate, then x.
  // Behind it x is read with device-coherent loads, and y is written through to memory (see Gate).
  constexpr int kXAux = Gate::kActive ? kCoherentLoad : 0;
  XStage xst;
  fetch_row_ptrs();
  // the row pointers are requested before anything that may have to wait for a kernel argument
  // which did not arrive in a register (the scheduler would otherwise put that wait first)
  __builtin_amdgcn_sched_barrier(0);
  const bool gated = Gate::kActive && gate.needed();
  if (!gated) stage_x_begin<0>(xst, x, cols, block_threads);
  prime_ring();
  if (gated) {
    if (!gate.wait()) return false;
    stage_x_begin<kXAux>(xst, x, cols, block_threads);
  }
  stage_x_finish<SIMPLE, kXAux>(lds, xst, x, cols, spmv_front_pad(BD), back_pad_for(BD), block_threads);  // ends with a barrier

  {
    float yv = 0.0f;                                   // lane i: result of row blk + i
    float acc = 0.0f;
    int base2 = 0;                                     // doubled position before this step (uniform)
    while (cp.i < nb) {
#pragma unroll
      for (int j = 0; j < RING; ++j) {
        LaneCodes<BD> w = wq[j];
        LaneValues<VB> v = vq[j];

        const bool live = cp.i < nb;                   // false for the padding items after the last row
        if (!live) base2 = 0;                          // keep the (unused) gathers of padding items in range
        const uint32_t end_eff = live ? cp.end : 0u;
        const uint32_t e0 = cp.a0 + 512u * cp.step + lane8;
        const bool first = live && cp.step == 0;
        const int before = (int)(cp.start - cp.a0);    // entries in front of the row in its first step
        if (!live || cp.step == cp.nsteps - 1 || (first && before >= 8)) {
          // clear what lies past the row end, and the lanes that lie wholly before its start
          uint32_t nv = e0 < end_eff ? end_eff - e0 : 0u;   // valid entries in this lane's chunk
          if (first && (int)lane8 + 8 <= before) nv = 0u;
          w.keep_if(nv != 0);
          v.keep_first(nv);
        }
        w.decode();
        const uint32_t tot = w.total();                // doubled sum of this lane's 8 deltas
        const uint32_t incl = wave_incl_scan_u32(tot);
        if (first) {
          // the row's first entry must land on its own column: the cleared lanes in front of it advance
          // 16 bytes each, and the lane that holds the start counts its entries of the previous row
          base2 = -2 * (before & ~7);
          if (before & 7) {
            base2 -= (int)w.through((before & 7) - 1, before >> 3);
            // the previous row's entries in that lane read the zero guard; their values are cleared all
            // the same, so that an infinity or a NaN among them cannot turn 0 * value into a NaN of this row
            v.clear_first(lane == (before >> 3) ? (uint32_t)(before & 7) : 0u);
          }
        }
        const int lanebase = base2 + (int)(incl - tot);   // byte offset in x of the lane's chunk start
#define MACKO_X(k) gather_x(xbase, lanebase + w.template offset<k>())
        acc = fmaf(v.template get<0>(), MACKO_X(0), acc);
        acc = fmaf(v.template get<1>(), MACKO_X(1), acc);
        acc = fmaf(v.template get<2>(), MACKO_X(2), acc);
        acc = fmaf(v.template get<3>(), MACKO_X(3), acc);
        acc = fmaf(v.template get<4>(), MACKO_X(4), acc);
        acc = fmaf(v.template get<5>(), MACKO_X(5), acc);
        acc = fmaf(v.template get<6>(), MACKO_X(6), acc);
        acc = fmaf(v.template get<7>(), MACKO_X(7), acc);
#undef MACKO_X
        issue(j);                                      // refill the slot just consumed, RING items ahead
        base2 += (int)__builtin_amdgcn_readlane((int)incl, 63);
        if (live && ++cp.step == cp.nsteps) {          // row finished: reduce, keep the result, next row
          const float total = wave_sum_to_last_lane(acc);
          const int tbits = __builtin_amdgcn_readlane(__builtin_bit_cast(int, total), 63);
          yv = lane == cp.i ? __builtin_bit_cast(float, tbits) : yv;
          acc = 0.0f;
          ++cp.i;
          seek_nonempty(cp, nb, rp_lo, rp_hi, amask);
        }
      }
    }
    if (lane < nb) {
      if (Gate::kActive)     // written through to memory: workgroups under other L2 caches read it next
        __hip_atomic_store(y + blk + lane, f32_to_f16_bits(yv), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else
        y[blk + lane] = f32_to_f16_bits(yv);
    }
  }
  return true;
}

// Grouped launch (matrices of one code width): the workgroup first finds its matrix.
template <int RING, bool SIMPLE, int BD, int VB = 16>
__global__ void __launch_bounds__(1024)
spmv_wave_row_kernel(const int wb1, const int wb2, const int wb3, const int wb4, const int wb5, const int wb6,
                     const int wb7, const uint32_t waves, const SpmvGroupArgs g) {
  // waves: floor(65536 / wavefronts per workgroup) + 1 in bits 0..16, wavefronts per workgroup above
  // (blockDim would have to be loaded from the dispatch's argument block)
  const int inv_nwaves = (int)(waves & 0x1FFFFu), nwaves = (int)(waves >> 17);
  static_assert(kMaxGroup == 8, "one scalar argument per group slot");
  int mi = 0, wg0 = 0;
  const int wbs[kMaxGroup] = {0, wb1, wb2, wb3, wb4, wb5, wb6, wb7};
#pragma unroll
  for (int i = 1; i < kMaxGroup; ++i) {
    const bool in = (int)blockIdx.x >= wbs[i];
    mi = in ? i : mi;
    wg0 = in ? wbs[i] : wg0;
  }
  spmv_wave_row_body<RING, SIMPLE, BD, VB>(g.m[mi].values, g.m[mi].deltas, g.m[mi].row_ptr, g.m[mi].x, g.m[mi].y,
                                       g.m[mi].rows, g.m[mi].cols, g.m[mi].q, g.m[mi].r, (int)blockIdx.x - wg0,
                                       nwaves, inv_nwaves, (uint32_t)g.m[mi].amask, 64 * nwaves);
}

// One matrix: the 14 leading arguments, which a starting wavefront finds in registers, hold
// everything it needs to request its row pointers and x at once, without any argument load before:
//   shape    floor(65536 / wavefronts per workgroup) + 1 in bits 0..16, wavefronts per workgroup in
//            bits 17..21, alignment of a row's first step minus 1 in bits 22..30
__host__ __device__ constexpr uint32_t pack_shape(int inv_nwaves, int nwaves, int amask) {
  return (uint32_t)inv_nwaves | ((uint32_t)nwaves << 17) | ((uint32_t)amask << 22);
}
template <int RING, bool SIMPLE, int BD>
__global__ void __launch_bounds__(1024)
spmv_wave_row_kernel(const uint32_t* __restrict__ row_ptr, const uint16_t* __restrict__ x, const int rows,
                     const int q, const int r, const uint32_t shape, const int cols,
                     const uint4* __restrict__ values, const uint32_t* __restrict__ deltas,
                     uint16_t* __restrict__ y) {
  const int nwaves = (int)((shape >> 17) & 31u);
  spmv_wave_row_body<RING, SIMPLE, BD>(values, deltas, row_ptr, x, y, rows, cols, q, r, (int)blockIdx.x, nwaves,
                                       (int)(shape & 0x1FFFFu), shape >> 22, 64 * nwaves);
}

// One matrix with 8-bit values (4-bit codes): 8 bytes of values and 4 bytes of codes per lane and step.
template <bool SIMPLE>
__global__ void __launch_bounds__(1024)
spmv_wave_row_fp8_kernel(const uint32_t* __restrict__ row_ptr, const uint16_t* __restrict__ x, const int rows,
                         const int q, const int r, const uint32_t shape, const int cols,
                         const uint2* __restrict__ values, const uint32_t* __restrict__ deltas,
                         uint16_t* __restrict__ y) {
  const int nwaves = (int)((shape >> 17) & 31u);
  spmv_wave_row_body<2, SIMPLE, 4, 8>(values, deltas, row_ptr, x, y, rows, cols, q, r, (int)blockIdx.x, nwaves,
                                      (int)(shape & 0x1FFFFu), shape >> 22, 64 * nwaves);
}

// ---------------------------------------------------------------------------
// Chain: phases of independent products in ONE launch.  Phase p + 1 may read, as its x,
// what phase p wrote as its y (the products of a decoder layer in the order of Appendix B:
// {q,k,v} -> {o} -> {gate,up} -> {down}); a kernel boundary between dependent products costs
// about 3 us on this hardware, as much as streaming a 4096 x 4096 matrix at 50 % sparsity.
//
// The launch is exactly one resident round (the host has checked that all workgroups fit the
// chip at once).  A workgroup walks the phases in order.  In each it takes its share of the
// phase's rows, fetches their row pointers and starts its load ring -- the matrix arrays do
// not depend on the phase before -- and only then waits until every workgroup has reported the
// previous phase done; then it stages x and runs the ordinary loop.
//
// Scratch memory (32-bit words, all zero before the launch and zero again after it):
//   arrive[g]  g < 8, 64 words apart: workgroups with (number % 8 == g) add 1 after each phase
//              but the last, once their y has reached memory; the gate of phase p waits for
//              the sum to reach p x workgroups
//   abort      set by a workgroup whose wait ran out; every waiting workgroup then gives up too
//   exit1[g], exit2   count the workgroups that are leaving; the last one clears all of the above
//   error      phase (1-based) whose gate gave up; kept until the host reads and clears it
// Visibility without cache maintenance: the compute units sit under eight L2 caches that do not
// snoop each other, and the release / acquire fences that would make ordinary stores and loads
// visible across them write back and invalidate a whole L2 each time (measured: 33 us per phase
// with 512 workgroups doing so).  Instead y is stored write-through (device-scope stores, waited
// for before the workgroup reports) and x is loaded with device-coherent loads, so that no
// stale or dirty line is ever involved; the counters are device-scope atomics.
// The wait is bounded by `wait_ticks` ticks of the 100 MHz wall clock; a workgroup that gives up
// skips the remaining phases and leaves normally, so the launch always ends.
// ---------------------------------------------------------------------------
constexpr int kChainSlot = 64;                         // words between two counters (256 bytes)
constexpr int kChainArrive = 0;                        // 8 slots
constexpr int kChainAbort = 8 * kChainSlot;
constexpr int kChainExit1 = 16 * kChainSlot;           // 8 slots
constexpr int kChainExit2 = 24 * kChainSlot;
constexpr int kChainError = 25 * kChainSlot;
constexpr int kChainScratchWords = 26 * kChainSlot;    // 6656 bytes
static_assert(kChainScratchWords * 4 <= chain_scratch_bytes() && kChainError == chain_error_word(), "scratch layout");

struct ChainArgs {
  SpmvMat m[kMaxChainMats];
  int wg_begin[kMaxChainMats];     // first workgroup of the product within its phase
  int nwg[kMaxChainMats];          // workgroups that work on it
  int first[kMaxChainPhases + 1];  // products first[p] .. first[p + 1] - 1 make up phase p
  int nwaves[kMaxChainPhases];     // wavefronts of a workgroup that take rows in phase p
  int inv_nwaves[kMaxChainPhases];
  int n_phases;
};

struct ChainGate {
  static constexpr bool kActive = true;
  uint32_t* scratch;
  uint32_t target;        // arrivals that complete the previous phase; 0: nothing to wait for
  uint32_t wait_ticks;
  int phase;
  __device__ __forceinline__ bool needed() const { return target != 0u; }   // uniform over the launch
  __device__ __forceinline__ bool wait() const {
    __shared__ int gave_up;
    if (target == 0u) return true;
    if (threadIdx.x < 64) {
      const int lane = threadIdx.x;
      const uint64_t t0 = wall_clock64();
      int fail = 0;
      for (;;) {
        uint32_t v = 0u;                               // lanes 0..7: the arrival counters, lane 8: the abort word
        if (lane < 9) v = __hip_atomic_load(scratch + lane * kChainSlot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t sum = 0u;
#pragma unroll
        for (int g = 0; g < 8; ++g) sum += (uint32_t)__builtin_amdgcn_readlane((int)v, g);
        if (sum >= target) break;
        const uint32_t aborted = (uint32_t)__builtin_amdgcn_readlane((int)v, 8);
        if (aborted != 0u || (uint64_t)(wall_clock64() - t0) >= (uint64_t)wait_ticks) {
          fail = 1;
          break;
        }
        __builtin_amdgcn_s_sleep(2);
      }
      if (fail && lane == 0) {
        __hip_atomic_store(scratch + kChainAbort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_max(scratch + kChainError, (uint32_t)phase + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      if (lane == 0) gave_up = fail;
    }
    __syncthreads();
    return gave_up == 0;
  }
};

template <bool SIMPLE, int BD>
// Register caps: the whole round must be resident, two workgroups of up to 16 wavefronts per compute
// unit, i.e. 8 wavefronts on a SIMD.  That needs at most 64 vector registers and at most 80 scalar
// registers per wavefront (a SIMD has 800; the driver's trap handler takes 16 more per wavefront, so
// a kernel with 82 left room for 7 and only half of the round was resident).
__global__ void __launch_bounds__(1024) __attribute__((amdgpu_num_sgpr(72), amdgpu_num_vgpr(64)))
spmv_chain_kernel(const ChainArgs a, uint32_t* __restrict__ scratch, const uint32_t wait_ticks) {
  const int wg = (int)blockIdx.x;
  const uint32_t total_wgs = gridDim.x;
  bool ok = true;
#pragma unroll 1
  for (int p = 0; p < a.n_phases; ++p) {
    // this workgroup's product in phase p (none: it idles through the phase)
    int mi = -1;
    for (int i = a.first[p]; i < a.first[p + 1]; ++i)
      if (wg >= a.wg_begin[i] && wg < a.wg_begin[i] + a.nwg[i]) mi = i;
    // A workgroup reports phase p only after it has seen phase p - 1 complete, also when it has no
    // rows in phase p: the arrival counters run on from phase to phase, and a workgroup that ran
    // ahead by two phases would be counted twice towards a phase that others are still working on.
    const ChainGate gate{scratch, (uint32_t)p * total_wgs, wait_ticks, p};
    if (mi >= 0) {
      const SpmvMat& m = a.m[mi];
      ok = spmv_wave_row_body<2, SIMPLE, BD, 16, ChainGate>(m.values, m.deltas, m.row_ptr, m.x, m.y, m.rows, m.cols,
                                                           m.q, m.r, wg - a.wg_begin[mi], a.nwaves[p],
                                                           a.inv_nwaves[p], (uint32_t)m.amask, (int)blockDim.x, gate);
    } else {
      ok = gate.wait();
    }
    if (!ok) break;
    // Every wavefront's y has reached memory (the stores are write-through and have been
    // acknowledged) and nobody reads this phase's x in LDS any more; then the workgroup reports.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (p + 1 < a.n_phases && threadIdx.x == 0)
      __hip_atomic_fetch_add(scratch + kChainArrive + (wg & 7) * kChainSlot, 1u, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
  }
  // Leaving: the last workgroup of all clears the counters for the next launch.  A workgroup's own
  // arrivals have been performed (acknowledged) before it is counted as gone.
  __syncthreads();
  if (threadIdx.x == 0) {
    __builtin_amdgcn_s_waitcnt(0);
    const uint32_t g = (uint32_t)wg & 7u;
    const uint32_t in_group = (total_wgs + 7u - g) >> 3;           // workgroups with number % 8 == g
    const uint32_t before = __hip_atomic_fetch_add(scratch + kChainExit1 + g * kChainSlot, 1u, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    if (before + 1u == in_group) {
      const uint32_t groups = total_wgs < 8u ? total_wgs : 8u;
      const uint32_t gone = __hip_atomic_fetch_add(scratch + kChainExit2, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (gone + 1u == groups) {
        for (int i = 0; i < 8; ++i) {
          __hip_atomic_store(scratch + kChainArrive + i * kChainSlot, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(scratch + kChainExit1 + i * kChainSlot, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __hip_atomic_store(scratch + kChainAbort, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(scratch + kChainExit2, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

// y = 0 for a matrix without stored entries
__global__ void __launch_bounds__(256) zero_y_kernel(uint16_t* __restrict__ y, int rows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows) y[i] = 0;
}

template <class K>
int set_lds_limit(K kernel, int64_t bytes) {
  if (bytes > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return hip_fail(e);
  }
  return MACKO_OK;
}

constexpr int64_t kMaxLdsBytes = 160 * 1024 - 64;   // 160 KB per CU minus the static row counter
// launches with at most this many wavefront steps per compute unit run as one resident round
// (the resident round won by 3-7 % up to ~340 steps and lost by 3-10 % from ~500 steps on,
// measured on 31 matrix shapes and the grouped launches of two decoder-layer shapes)
constexpr int64_t kResidentStepsPerCu = 448;
// many-workgroup regime: steps of work per wavefront (whole rows; at least one row)
constexpr int64_t kStepsPerWave = 8;
// rows of at least this many stored entries on average take the wave-per-row kernel (a step
// covers 512 entries; below about 40 % use of a step the sub-wave kernel wins: measured
// crossover between 133 and 247 entries per row on 36864 x 12288 at 98-99 % sparsity)
constexpr int64_t kWaveRowMinEntries = 192;
// x copies of at least this many bytes make a matrix "wide" for the launch planner
constexpr int64_t kWideLdsBytes = 36 * 1024;
// widest x that is staged once per 256-thread workgroup (see the row-length rule in launch_wave_row_group)
constexpr int64_t kInStepMaxCols = 8192;

}  // namespace

namespace {

template <int LANES, int BD>
int launch_subwave_as(const SpmvProblem& p, int block, int64_t grid, int64_t rpw, bool lds_ok, int64_t lds_bytes,
                      hipStream_t stream) {
  const uint4* v4 = reinterpret_cast<const uint4*>(p.values);
  const uint32_t* d4 = reinterpret_cast<const uint32_t*>(p.deltas);
  const uint16_t* xp = static_cast<const uint16_t*>(p.x);
  uint16_t* yp = static_cast<uint16_t*>(p.y);
  if (lds_ok) {
    auto kfn = spmv_subwave_kernel<LANES, true, BD>;
    int st = set_lds_limit(kfn, lds_bytes);
    if (st != MACKO_OK) return st;
    hipLaunchKernelGGL(kfn, dim3((unsigned)grid), dim3(block), (size_t)lds_bytes, stream, v4, d4, p.row_ptr, xp,
                       yp, (int)p.rows, (int)p.cols, (int)rpw);
  } else {
    hipLaunchKernelGGL((spmv_subwave_kernel<LANES, false, BD>), dim3((unsigned)grid), dim3(block), 0, stream, v4,
                       d4, p.row_ptr, xp, yp, (int)p.rows, (int)p.cols, (int)rpw);
  }
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MACKO_OK : hip_fail(e);
}

template <int BD>
int launch_subwave_bd(const SpmvProblem& p, int lanes, int block, int64_t grid, int64_t rpw, bool lds_ok,
                      int64_t lds_bytes, hipStream_t stream) {
  if (lanes == 64) return launch_subwave_as<64, BD>(p, block, grid, rpw, lds_ok, lds_bytes, stream);
  if (lanes == 32) return launch_subwave_as<32, BD>(p, block, grid, rpw, lds_ok, lds_bytes, stream);
  return launch_subwave_as<16, BD>(p, block, grid, rpw, lds_ok, lds_bytes, stream);
}

int launch_subwave(const SpmvProblem& p, int kernel_lanes, hipStream_t stream) {
  const Tuning& t = tuning();
  const int cus = device_cu_count();
  const int64_t lds_bytes = lds_bytes_for(p.cols);    // every entry is masked: the plain guards do
  const bool lds_ok = lds_bytes <= kMaxLdsBytes;
  const int64_t avg = p.rows > 0 ? p.pad_nnz / p.rows : 0;
  int lanes = kernel_lanes;
  if (lanes == 0) lanes = avg >= 256 ? 32 : 16;        // 64 lanes per row measured slower at every length
  // 512 threads: every workgroup stages its own copy of x, and the larger workgroup halves the number
  // of copies (36864 x 12288 at 99 %, 8-bit codes: 9.8 -> 8.4 us)
  const int block = t.spmv_block ? (int)t.spmv_block : 512;
  const int groups = block / lanes;
  int64_t rpw = t.spmv_rows_per_wg;
  if (rpw == 0) {
    const int64_t target_wgs = (int64_t)cus * 4;
    rpw = (p.rows + target_wgs - 1) / target_wgs;
    rpw = (std::max<int64_t>(rpw, groups) + groups - 1) / groups * groups;
  }
  const int64_t grid = (p.rows + rpw - 1) / rpw;
  switch (p.b_delta) {
    case 1: return launch_subwave_bd<1>(p, lanes, block, grid, rpw, lds_ok, lds_bytes, stream);
    case 2: return launch_subwave_bd<2>(p, lanes, block, grid, rpw, lds_ok, lds_bytes, stream);
    case 4: return launch_subwave_bd<4>(p, lanes, block, grid, rpw, lds_ok, lds_bytes, stream);
    case 8: return launch_subwave_bd<8>(p, lanes, block, grid, rpw, lds_ok, lds_bytes, stream);
    default: return MACKO_E_UNSUPPORTED;
  }
}

// The wave-per-row launch of a planned group whose matrices share the code width BD.
template <int BD>
int launch_wave_row_bd(const SpmvGroupArgs& args, const SpmvGroupHeader& head, int nwr, const Plan& plan,
                       int64_t max_lds, bool simple, int ring, hipStream_t stream);

// 8-bit values (4-bit codes, two steps of loads in flight): single-matrix and grouped entry points
int launch_wave_row_fp8(const SpmvGroupArgs& args, const SpmvGroupHeader& head, int nwr, const Plan& plan,
                        int64_t max_lds, bool simple, hipStream_t stream) {
  const dim3 grid((unsigned)plan.total_wgs), blockdim(plan.block);
  if (nwr == 1) {
    auto kfn = simple ? spmv_wave_row_fp8_kernel<true> : spmv_wave_row_fp8_kernel<false>;
    int st = set_lds_limit(kfn, max_lds);
    if (st != MACKO_OK) return st;
    const SpmvMat& m = args.m[0];
    hipLaunchKernelGGL(kfn, grid, blockdim, (size_t)max_lds, stream, m.row_ptr, m.x, m.rows, m.q, m.r,
                       pack_shape(head.inv_nwaves, plan.block / 64, m.amask), m.cols,
                       static_cast<const uint2*>(m.values), m.deltas, m.y);
  } else {
    using KG = void (*)(int, int, int, int, int, int, int, uint32_t, SpmvGroupArgs);
    KG kfn = simple ? (KG)spmv_wave_row_kernel<2, true, 4, 8> : (KG)spmv_wave_row_kernel<2, false, 4, 8>;
    int st = set_lds_limit(kfn, max_lds);
    if (st != MACKO_OK) return st;
    hipLaunchKernelGGL(kfn, grid, blockdim, (size_t)max_lds, stream, head.wg_begin[1], head.wg_begin[2],
                       head.wg_begin[3], head.wg_begin[4], head.wg_begin[5], head.wg_begin[6], head.wg_begin[7],
                       (uint32_t)head.inv_nwaves | ((uint32_t)(plan.block / 64) << 17), args);
  }
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MACKO_OK : hip_fail(e);
}

template <int BD>
int launch_wave_row_bd(const SpmvGroupArgs& args, const SpmvGroupHeader& head, int nwr, const Plan& plan,
                       int64_t max_lds, bool simple, int ring, hipStream_t stream) {
  const dim3 grid((unsigned)plan.total_wgs), blockdim(plan.block);
  if (nwr == 1) {
    using K1 = void (*)(const uint32_t*, const uint16_t*, int, int, int, uint32_t, int, const uint4*, const uint32_t*,
                        uint16_t*);
    K1 kfn = simple ? (K1)spmv_wave_row_kernel<2, true, BD> : (K1)spmv_wave_row_kernel<2, false, BD>;
    if (BD == 4 && ring == 4)
      kfn = simple ? (K1)spmv_wave_row_kernel<4, true, 4> : (K1)spmv_wave_row_kernel<4, false, 4>;
    if (BD == 4 && ring == 3)
      kfn = simple ? (K1)spmv_wave_row_kernel<3, true, 4> : (K1)spmv_wave_row_kernel<3, false, 4>;
    int st = set_lds_limit(kfn, max_lds);
    if (st != MACKO_OK) return st;
    const SpmvMat& m = args.m[0];
    hipLaunchKernelGGL(kfn, grid, blockdim, (size_t)max_lds, stream, m.row_ptr, m.x, m.rows, m.q, m.r,
                       pack_shape(head.inv_nwaves, plan.block / 64, m.amask), m.cols,
                       static_cast<const uint4*>(m.values), m.deltas, m.y);
  } else {
    using KG = void (*)(int, int, int, int, int, int, int, uint32_t, SpmvGroupArgs);
    KG kfn = simple ? (KG)spmv_wave_row_kernel<2, true, BD> : (KG)spmv_wave_row_kernel<2, false, BD>;
    if (BD == 4 && ring == 4)
      kfn = simple ? (KG)spmv_wave_row_kernel<4, true, 4> : (KG)spmv_wave_row_kernel<4, false, 4>;
    if (BD == 4 && ring == 3)
      kfn = simple ? (KG)spmv_wave_row_kernel<3, true, 4> : (KG)spmv_wave_row_kernel<3, false, 4>;
    int st = set_lds_limit(kfn, max_lds);
    if (st != MACKO_OK) return st;
    hipLaunchKernelGGL(kfn, grid, blockdim, (size_t)max_lds, stream, head.wg_begin[1], head.wg_begin[2],
                       head.wg_begin[3], head.wg_begin[4], head.wg_begin[5], head.wg_begin[6], head.wg_begin[7],
                       (uint32_t)head.inv_nwaves | ((uint32_t)(plan.block / 64) << 17), args);
  }
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MACKO_OK : hip_fail(e);
}

// One grouped wave-per-row launch for the matrices wr[0..nwr) (same code width).
int launch_wave_row_group(int nwr, const SpmvProblem* const* wr, int b_delta, int b_val, hipStream_t stream) {
  const Tuning& t = tuning();
  const int cus = device_cu_count();
  PlanInput in[kMaxGroup];
  int64_t max_lds = 0, total_steps = 0;
  for (int i = 0; i < nwr; ++i) {
    const SpmvProblem& p = *wr[i];
    in[i].rows = p.rows;
    in[i].steps_per_row = std::max<int64_t>(1, (p.pad_nnz / p.rows + 511) / 512);
    in[i].lds_bytes = spmv_lds_bytes(p.cols, b_delta);
    total_steps += in[i].rows * in[i].steps_per_row;
    max_lds = std::max(max_lds, in[i].lds_bytes);
  }

  Plan plan;
  bool planned = false;
  // Little work: one resident round of workgroups, shaped to the row counts.
  // Wide matrices (x of more than ~18 K columns, 36 KB in LDS) run as one
  // resident round of a single large workgroup per compute unit whatever their
  // size: every workgroup stages its own copy of x, and the fewer copies are made
  // the better (4-8 % measured on the 18944 .. 49152 column shapes).
  const int64_t resident_steps = t.spmv_resident_steps ? t.spmv_resident_steps : kResidentStepsPerCu;
  const bool small = total_steps <= (int64_t)cus * resident_steps;
  const bool wide = max_lds - kAlignFrontPad >= kWideLdsBytes;
  // Rows of a multiple of 2048 stored entries on average (4096 or 8192 columns at 50 %,
  // 4096 columns dense): every row start is a multiple of 4096 bytes into the values array, and a
  // resident round, which starts all its wavefronts at row starts at the same moment, runs them through
  // the memory system in step.  Such matrices go to many 256-thread workgroups instead, which the
  // dispatcher hands out as compute units become free.  Measured against the resident round (interleaved
  // runs): {gate,up} of a 7B-shaped layer 23.1 -> 21.1 us, {q,k,v} 13.5 -> 13.1, 14336 x 4096 15.7 -> 14.7,
  // 32000 x 4096 30.0 -> 28.3 (dense: 59.6 -> 50.7 against the 512-thread workgroups it used to get),
  // 8192 x 8192 17.8 -> 16.4, 28672 x 8192 49.2 -> 47.8; iid masks with that average gain as much as exact
  // per-row counts (14336 x 4096: 15.7 -> 14.9 and 15.9 -> 14.8).  Other row lengths on the same shapes (30, 70, 80,
  // 90 % sparsity, 3584 columns) are 1-4 % faster in the resident round and stay there; x of more than
  // 8192 columns costs too much to stage once per small workgroup.
  bool in_step = t.spmv_resident == 0 && t.spmv_block == 0;
  for (int i = 0; i < nwr; ++i) {
    const int64_t avg = wr[i]->pad_nnz / wr[i]->rows;
    const int64_t off = (avg + 1024) % 2048 - 1024;            // distance to the nearest multiple of 2048
    in_step = in_step && wr[i]->cols <= kInStepMaxCols && avg >= 2048 - 16 && off >= -16 && off <= 16;
  }
  if (!in_step && t.spmv_rows_per_wg == 0 && (t.spmv_resident == 2 || (t.spmv_resident == 0 && (small || wide)))) {
    const int k = t.spmv_wgs_per_cu ? (int)t.spmv_wgs_per_cu : (wide ? 1 : 0);
    planned = plan_resident(plan, nwr, in, cus, (int)t.spmv_block, k);
  }
  if (!planned) {
    // Plenty of work: many workgroups, about 8 steps per wavefront (short rows:
    // several rows per wavefront), but never so few workgroups that the launch
    // has under ~16 wavefronts per compute unit.  Workgroups go to the eight XCDs in
    // turn whatever their load, and what a compute unit is still working on when the
    // others have finished is lost: 16 steps per wavefront measured 3-9 % slower on
    // launches of 30-70 us, fewer than 6 slower again on short rows.  Every workgroup holds its own
    // copy of x in LDS; when that copy is large (more than ~24 K columns) only
    // one to three fit a compute unit, so each brings 16 wavefronts instead of 8.
    const int block = t.spmv_block ? (int)t.spmv_block : (in_step ? 256 : (max_lds - kAlignFrontPad > 48 * 1024 ? 1024 : 512));
    const int nwaves = block / 64;
    int64_t group_rows = 0;
    for (int i = 0; i < nwr; ++i) group_rows += in[i].rows;
    int64_t rpw[kMaxGroup];
    for (int i = 0; i < nwr; ++i) {
      rpw[i] = t.spmv_rows_per_wg;
      if (rpw[i] == 0) {
        const int64_t target = t.spmv_steps_per_wave ? t.spmv_steps_per_wave : kStepsPerWave;
        const int64_t want = std::max<int64_t>(1, (2 * target + in[i].steps_per_row) / (2 * in[i].steps_per_row));  // nearest
        const int64_t cap = std::max<int64_t>(1, group_rows / ((int64_t)cus * 16));
        rpw[i] = std::min(want, cap) * nwaves;
      }
    }
    plan_by_rows_per_wg(plan, nwr, in, block, rpw);
  }
  if (plan.total_wgs >= (int64_t{1} << 31)) return MACKO_E_UNSUPPORTED;

  SpmvGroupArgs args{};
  SpmvGroupHeader head{};
  const int nwaves = plan.block / 64;
  head.inv_nwaves = 65536 / nwaves + 1;
  int64_t wg_begin = 0;
  bool simple = true;
  for (int i = 0; i < kMaxGroup; ++i) head.wg_begin[i] = INT32_MAX;
  for (int i = 0; i < nwr; ++i) {
    const SpmvProblem& p = *wr[i];
    SpmvMat& m = args.m[i];
    m.values = p.values;
    m.deltas = reinterpret_cast<const uint32_t*>(p.deltas);
    m.row_ptr = p.row_ptr;
    m.x = static_cast<const uint16_t*>(p.x);
    m.y = static_cast<uint16_t*>(p.y);
    m.rows = (int)p.rows;
    m.cols = (int)p.cols;
    m.q = plan.m[i].q;
    m.r = plan.m[i].r;
    const int64_t align_knob = t.spmv_step_align;      // 0: by row length
    const int align = align_knob ? (int)align_knob : (p.pad_nnz / p.rows >= kAlignMinEntries ? kStepAlign : 8);
    m.amask = std::min(std::max(align, 8), kMaxStepAlign) - 1;
    m.pad = 0;
    head.wg_begin[i] = (int)wg_begin;
    wg_begin += plan.m[i].nwg;
    // the lean start-up path needs an aligned x whose length is a multiple of 8 and fits the staging registers
    simple = simple && stage_x_is_simple(m.x, m.cols, plan.block);
  }
  // Two steps of loads in flight per wavefront are enough at 16+ wavefronts per
  // compute unit, and the smaller loop body matters when a wavefront runs it only
  // a few times.
  // Ring depth: two steps in flight per wavefront, except in a resident round of at most 16
  // wavefronts per compute unit working on long rows (4096 x 11008: one row of 11 steps per
  // wavefront), where two steps leave the memory system short of requests: four there (6 %).
  // Not for the wide matrices (one 16-wavefront workgroup per compute unit, rows of 20-48
  // steps): measured 3-7 % slower with four on the seven shapes of 18944 columns and more.
  int ring = (int)t.spmv_ring;
  if (ring == 0 && planned && !wide && plan.total_wgs * nwaves <= (int64_t)cus * 16) {
    int64_t min_steps = in[0].steps_per_row;
    for (int i = 1; i < nwr; ++i) min_steps = std::min(min_steps, in[i].steps_per_row);
    if (min_steps >= 8) ring = 4;
  }
  if (b_val == 8) return launch_wave_row_fp8(args, head, nwr, plan, max_lds, simple, stream);
  switch (b_delta) {
    case 1: return launch_wave_row_bd<1>(args, head, nwr, plan, max_lds, simple, ring, stream);
    case 2: return launch_wave_row_bd<2>(args, head, nwr, plan, max_lds, simple, ring, stream);
    case 4: return launch_wave_row_bd<4>(args, head, nwr, plan, max_lds, simple, ring, stream);
    case 8: return launch_wave_row_bd<8>(args, head, nwr, plan, max_lds, simple, ring, stream);
    default: return MACKO_E_UNSUPPORTED;
  }
}

}  // namespace

namespace {

// Scratch memory of macko_spmv_chain_static: one copy per device, part of the loaded code object, zero when
// the library is loaded and left zero by every chain.  Host code never uses this name as an address (on the
// host it is a stand-in for the symbol): chain_static_scratch() asks the runtime for the device address once per device.
static __device__ __align__(256) unsigned char g_chain_scratch[chain_scratch_bytes()];

struct OccupancyKey {
  const void* kernel;
  int block;
  int64_t lds;
  int dev;
  int result;
};
std::mutex g_occ_mutex;
constexpr int kOccSlots = 64;           // a fixed table: nothing on the launch path allocates
OccupancyKey g_occ[kOccSlots];
int g_occ_n = 0;

// Workgroups of `kernel` that one compute unit holds at a time: the smaller of what the runtime
// reports (registers, LDS and wavefront slots) and the pessimistic count from the kernel's own
// register use; asked once per (kernel, shape, device) and remembered.
int occupancy_of(const void* kernel, int block, int64_t lds) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  std::lock_guard<std::mutex> lock(g_occ_mutex);
  for (int i = 0; i < g_occ_n; ++i) {
    const OccupancyKey& k = g_occ[i];
    if (k.kernel == kernel && k.block == block && k.lds == lds && k.dev == dev) return k.result;
  }
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, block, (size_t)lds) != hipSuccess) {
    (void)hipGetLastError();
    n = 0;
  }
  // and never more than the pessimistic count from the kernel's own resource use
  hipFuncAttributes attr{};
  if (hipFuncGetAttributes(&attr, kernel) != hipSuccess) {
    (void)hipGetLastError();
    n = 0;
  } else {
    n = std::min(n, resident_wgs_per_cu(attr.numRegs, block / 64, lds + (int64_t)attr.sharedSizeBytes));
  }
  if (g_occ_n < kOccSlots) g_occ[g_occ_n++] = OccupancyKey{kernel, block, lds, dev, n};
  return n;
}

}  // namespace

int chain_static_scratch(uint32_t** out) {
  static std::mutex mutex;
  static uint32_t* address[64] = {};
  int dev = 0;
  MACKO_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return MACKO_E_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mutex);
  if (!address[dev]) {
    void* p = nullptr;
    MACKO_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(g_chain_scratch)));
    if (!p) return MACKO_E_HIP;
    address[dev] = static_cast<uint32_t*>(p);
  }
  *out = address[dev];
  return MACKO_OK;
}

int launch_spmv_chain(int n_phases, const int* sizes, const SpmvProblem* problems, uint32_t* scratch,
                      uint32_t wait_ticks, hipStream_t stream) {
  if (n_phases < 1 || n_phases > kMaxChainPhases || !sizes || !problems || !scratch) return MACKO_E_INVALID_ARG;
  const Tuning& t = tuning();
  const int cus = device_cu_count();
  int total = 0;
  for (int p = 0; p < n_phases; ++p) {
    if (sizes[p] < 1 || sizes[p] > kMaxGroup) return MACKO_E_INVALID_ARG;
    total += sizes[p];
  }
  if (total > kMaxChainMats) return MACKO_E_UNSUPPORTED;
  // one kernel for the whole chain: every product must be one the wave-per-row kernel serves,
  // with the same code width and 16-bit values
  const int bd = problems[0].b_delta;
  if (bd != 4 && bd != 2) return MACKO_E_UNSUPPORTED;
  PlanInput in[kMaxChainMats];
  int64_t max_lds = 0;
  bool simple_x = true;
  for (int i = 0; i < total; ++i) {
    const SpmvProblem& q = problems[i];
    if (q.rows < 1 || q.pad_nnz < 1 || q.b_delta != bd || q.b_val != 16) return MACKO_E_UNSUPPORTED;
    if (q.pad_nnz > (int64_t{1} << 32) - 4096) return MACKO_E_UNSUPPORTED;
    in[i].rows = q.rows;
    in[i].steps_per_row = std::max<int64_t>(1, (q.pad_nnz / q.rows + 511) / 512);
    in[i].lds_bytes = spmv_lds_bytes(q.cols, bd);
    if (in[i].lds_bytes > kMaxLdsBytes) return MACKO_E_UNSUPPORTED;
    max_lds = std::max(max_lds, in[i].lds_bytes);
  }
  using KC = void (*)(ChainArgs, uint32_t*, uint32_t);
  auto kernel_for = [&](bool simple) -> KC {
    if (bd == 2) return simple ? (KC)spmv_chain_kernel<true, 2> : (KC)spmv_chain_kernel<false, 2>;
    return simple ? (KC)spmv_chain_kernel<true, 4> : (KC)spmv_chain_kernel<false, 4>;
  };
  // the general x staging needs no more resources than the lean one: plan with it, choose afterwards
  {
    int st = set_lds_limit(kernel_for(false), max_lds);
    if (st != MACKO_OK) return st;
    st = set_lds_limit(kernel_for(true), max_lds);
    if (st != MACKO_OK) return st;
  }
  ChainPlan plan;
  const bool planned = plan_chain(plan, n_phases, sizes, in, cus, [&](int block) {
    return std::min(occupancy_of(reinterpret_cast<const void*>(kernel_for(false)), block, max_lds),
                    occupancy_of(reinterpret_cast<const void*>(kernel_for(true)), block, max_lds));
  });
  if (!planned) return MACKO_E_UNSUPPORTED;             // some workgroup would not be resident

  ChainArgs args{};
  args.n_phases = n_phases;
  int at = 0;
  for (int p = 0; p < n_phases; ++p) {
    args.first[p] = at;
    args.nwaves[p] = plan.nwaves[p];
    args.inv_nwaves[p] = 65536 / plan.nwaves[p] + 1;
    int wg_begin = 0;
    for (int i = 0; i < sizes[p]; ++i, ++at) {
      const SpmvProblem& q = problems[at];
      SpmvMat& m = args.m[at];
      m.values = q.values;
      m.deltas = reinterpret_cast<const uint32_t*>(q.deltas);
      m.row_ptr = q.row_ptr;
      m.x = static_cast<const uint16_t*>(q.x);
      m.y = static_cast<uint16_t*>(q.y);
      m.rows = (int)q.rows;
      m.cols = (int)q.cols;
      m.q = plan.m[at].q;
      m.r = plan.m[at].r;
      const int64_t align_knob = t.spmv_step_align;
      const int align = align_knob ? (int)align_knob : (q.pad_nnz / q.rows >= kAlignMinEntries ? kStepAlign : 8);
      m.amask = std::min(std::max(align, 8), kMaxStepAlign) - 1;
      args.wg_begin[at] = wg_begin;
      args.nwg[at] = plan.m[at].nwg;
      wg_begin += plan.m[at].nwg;
      simple_x = simple_x && stage_x_is_simple(m.x, m.cols, plan.block);
    }
  }
  args.first[n_phases] = at;
  hipLaunchKernelGGL(kernel_for(simple_x), dim3((unsigned)plan.total_wgs), dim3(plan.block), (size_t)max_lds, stream,
                     args, scratch, wait_ticks);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MACKO_OK : hip_fail(e);
}

int launch_spmv_group(int n, const SpmvProblem* problems, hipStream_t stream) {
  if (n < 1 || n > kMaxGroup) return MACKO_E_INVALID_ARG;
  const Tuning& t = tuning();
  auto wants_wave_row = [&](const SpmvProblem& p) {
    if (p.rows == 0 || p.pad_nnz == 0) return false;
    if (spmv_lds_bytes(p.cols, p.b_delta) > kMaxLdsBytes) return false;
    if (t.spmv_kernel != 0) return t.spmv_kernel == 2;
    return p.pad_nnz / p.rows >= kWaveRowMinEntries;
  };
  // matrices that do not go into a grouped wave-per-row launch
  for (int i = 0; i < n; ++i) {
    const SpmvProblem& p = problems[i];
    if (p.rows == 0) continue;
    // the kernels index entries with 32 bits and look up to two steps past a row's end
    if (p.pad_nnz > (int64_t{1} << 32) - 4096) return MACKO_E_UNSUPPORTED;
    if (p.pad_nnz == 0) {                               // nothing stored: y = 0
      hipLaunchKernelGGL(zero_y_kernel, dim3((unsigned)((p.rows + 255) / 256)), dim3(256), 0, stream,
                         static_cast<uint16_t*>(p.y), (int)p.rows);
      hipError_t e0 = hipGetLastError();
      if (e0 != hipSuccess) return hip_fail(e0);
    } else if (p.b_val == 8) {                          // 8-bit values: 4-bit codes, wave-per-row kernel only
      if (p.b_delta != 4 || spmv_lds_bytes(p.cols, 4) > kMaxLdsBytes) return MACKO_E_UNSUPPORTED;
    } else if (!wants_wave_row(p)) {                    // short rows or x larger than LDS: own launch
      int st = launch_subwave(p, (int)t.spmv_lanes, stream);
      if (st != MACKO_OK) return st;
    }
  }
  // one grouped launch per code width
  for (int bd : {4, 2, 8, 1}) {
    const SpmvProblem* wr[kMaxGroup];
    int nwr = 0;
    for (int i = 0; i < n; ++i)
      if (problems[i].b_delta == bd && problems[i].b_val == 16 && wants_wave_row(problems[i])) wr[nwr++] = &problems[i];
    if (nwr == 0) continue;
    int st = launch_wave_row_group(nwr, wr, bd, 16, stream);
    if (st != MACKO_OK) return st;
  }
  // and one for the matrices with 8-bit values
  {
    const SpmvProblem* wr[kMaxGroup];
    int nwr = 0;
    for (int i = 0; i < n; ++i)
      if (problems[i].b_val == 8 && problems[i].rows > 0 && problems[i].pad_nnz > 0) wr[nwr++] = &problems[i];
    if (nwr > 0) {
      int st = launch_wave_row_group(nwr, wr, 4, 8, stream);
      if (st != MACKO_OK) return st;
    }
  }
  return MACKO_OK;
}

}  // namespace macko
