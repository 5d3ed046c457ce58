// Device-side helpers shared by the gfx950 kernels: wave64 cross-lane
// primitives on DPP, and staging of the activation vector into LDS.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace macko {

constexpr int kWave = 64;

// The activation vector x sits in LDS between two zero-filled guard regions:
//   [0, front) zeros | x[0 .. C) | zeros up to the end of the allocation.
// Entries that a lane loads but that belong to a neighbouring row decode to
// positions just before column 0 or after the row's last column; the guards
// make those reads return +0 so that they contribute nothing.
// Front guard: a row's first chunk holds at most 7 entries of the previous row,
// each at most 2^b_delta columns wide (224 bytes before x[0] for 4-bit codes,
// 3584 for 8-bit ones).  Back guard: in a row's last step the lanes past the row
// end advance by one column per entry, plus at most 7 real deltas in the lane
// that straddles the end (at most 504 + 7 * 2^b_delta columns); the dense kernel
// reads at most 62 16-byte chunks past the end.
constexpr int kFrontPad = 256;   // bytes, codes of up to 4 bits (and the dense kernel)
constexpr int kBackPad = 1280;   // bytes

__host__ __device__ constexpr int front_pad_for(int b_delta) { return b_delta <= 4 ? kFrontPad : 3584; }
__host__ __device__ constexpr int back_pad_for(int b_delta) { return b_delta <= 4 ? kBackPad : 4608; }

__host__ __device__ inline int64_t lds_bytes_for(int64_t cols, int b_delta = 4) {
  return front_pad_for(b_delta) + 16 * ((cols + 7) / 8) + back_pad_for(b_delta);
}

// ---- loads of data that is read once ------------------------------------------
// The format arrays (and the dense matrix of the baseline) are streamed through once per
// product; marking their loads non-temporal keeps them from displacing x, the row pointers
// and each other's neighbours in the caches.  Measured on seven shapes: 3-5 % per product.
typedef uint32_t macko_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t macko_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
  const macko_u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const macko_u32x4*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint2 load_stream(const uint2* p) {
  const macko_u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const macko_u32x2*>(p));
  return make_uint2(t.x, t.y);
}
__device__ __forceinline__ uint32_t load_stream(const uint32_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint16_t load_stream(const uint16_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint8_t load_stream(const uint8_t* p) { return __builtin_nontemporal_load(p); }

// ---- DPP cross-lane primitives (wave64, GCN DPP controls) --------------------
// row_shr:n shifts within a row of 16 lanes; row_bcast:15 / row_bcast:31 carry a
// row's (half-wave's) last lane into the following rows.  Lanes without a source
// keep `old` (= the additive identity).

// One DPP step "v += lanes shifted by ctrl", emitted as a single VALU
// instruction.  The leading s_nop covers the two wait states a DPP read needs
// after a VALU write of the same register.  bound_ctrl:0 makes lanes without a
// source read 0; rows excluded by row_mask keep their value (dst is tied to v).
#define MACKO_DPP_ADD(op, v, ctrl, rmask)                                                     \
  asm volatile("s_nop 1\n\t" op " %0, %0, %0 " ctrl " row_mask:" rmask " bank_mask:0xf bound_ctrl:0" \
               : "+v"(v))

// Inclusive prefix sum over the 64 lanes (Alg. 1 of the paper computes the same
// quantity with five shuffle levels on 32 lanes; a wavefront needs six).
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
  MACKO_DPP_ADD("v_add_u32_dpp", v, "row_shr:1", "0xf");
  MACKO_DPP_ADD("v_add_u32_dpp", v, "row_shr:2", "0xf");
  MACKO_DPP_ADD("v_add_u32_dpp", v, "row_shr:4", "0xf");
  MACKO_DPP_ADD("v_add_u32_dpp", v, "row_shr:8", "0xf");
  MACKO_DPP_ADD("v_add_u32_dpp", v, "row_bcast:15", "0xa");
  MACKO_DPP_ADD("v_add_u32_dpp", v, "row_bcast:31", "0xc");
  return v;
}

// Inclusive running maximum over the 64 lanes (unsigned; lanes without a source read 0).
__device__ __forceinline__ uint32_t wave_incl_scan_max_u32(uint32_t v) {
  MACKO_DPP_ADD("v_max_u32_dpp", v, "row_shr:1", "0xf");
  MACKO_DPP_ADD("v_max_u32_dpp", v, "row_shr:2", "0xf");
  MACKO_DPP_ADD("v_max_u32_dpp", v, "row_shr:4", "0xf");
  MACKO_DPP_ADD("v_max_u32_dpp", v, "row_shr:8", "0xf");
  MACKO_DPP_ADD("v_max_u32_dpp", v, "row_bcast:15", "0xa");
  MACKO_DPP_ADD("v_max_u32_dpp", v, "row_bcast:31", "0xc");
  return v;
}

// Sum over the 64 lanes; the total ends up in lane 63 (other lanes hold prefixes).
__device__ __forceinline__ float wave_sum_to_last_lane(float v) {
  MACKO_DPP_ADD("v_add_f32_dpp", v, "row_shr:1", "0xf");
  MACKO_DPP_ADD("v_add_f32_dpp", v, "row_shr:2", "0xf");
  MACKO_DPP_ADD("v_add_f32_dpp", v, "row_shr:4", "0xf");
  MACKO_DPP_ADD("v_add_f32_dpp", v, "row_shr:8", "0xf");
  MACKO_DPP_ADD("v_add_f32_dpp", v, "row_bcast:15", "0xa");
  MACKO_DPP_ADD("v_add_f32_dpp", v, "row_bcast:31", "0xc");
  return v;
}

// The same for N registers at once (N = 2, 4 or 8).  A DPP read needs two wait states after a VALU
// write of its register, and the hazard is not seen inside inline assembly, so the s_nop has to sit in
// the same asm statement as the instruction it protects (a separate statement could be scheduled away
// from it).  First level: every instruction carries its own s_nop (the producer of a[b] is ordinary
// code).  Later levels, N >= 4: the producer is the previous level's instruction for the same register,
// and the level's other N - 1 instructions, which volatile asm keeps in order, cover the wait states.
#define MACKO_DPP_ADD_NOWAIT(op, v, ctrl, rmask) \
  asm volatile(op " %0, %0, %0 " ctrl " row_mask:" rmask " bank_mask:0xf bound_ctrl:0" : "+v"(v))
template <int N>
__device__ __forceinline__ void wave_sum_to_last_lane_n(float (&a)[N]) {
  static_assert(N == 2 || N == 4 || N == 8, "batch piece sizes");
#define MACKO_LEVEL(ctrl, rmask, first)                                      \
  {                                                                          \
    _Pragma("unroll") for (int b = 0; b < N; ++b) {                          \
      if (first || N < 4) MACKO_DPP_ADD("v_add_f32_dpp", a[b], ctrl, rmask); \
      else MACKO_DPP_ADD_NOWAIT("v_add_f32_dpp", a[b], ctrl, rmask);         \
    }                                                                        \
  }
  MACKO_LEVEL("row_shr:1", "0xf", true)
  MACKO_LEVEL("row_shr:2", "0xf", false)
  MACKO_LEVEL("row_shr:4", "0xf", false)
  MACKO_LEVEL("row_shr:8", "0xf", false)
  MACKO_LEVEL("row_bcast:15", "0xa", false)
  MACKO_LEVEL("row_bcast:31", "0xc", false)
#undef MACKO_LEVEL
}

// (a << sh) + b in one full-rate VALU instruction.  Written as asm so that the
// compiler does not fuse chains of these into a quarter-rate 32-bit multiply.
template <int SH>
__device__ __forceinline__ uint32_t lshl_add(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "n"(SH), "v"(b));
  return r;
}

// fp32 -> fp16 bits, round to nearest even (v_cvt_f16_f32 under the default mode)
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
  _Float16 h = (_Float16)f;
  return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) {
  return (float)__builtin_bit_cast(_Float16, b);
}

// ---- row cursor of the wavefront-per-row kernels ------------------------------
// A wavefront keeps the pointers of its (at most 64) rows in two registers, lane i
// holding row i's; the scalar bounds of the current row are read out of them.
struct RowCursor {
  int i;               // row index within the block (== nb when exhausted)
  uint32_t start, end; // its entry range
  uint32_t a0;         // start rounded down to ALIGN entries: where the row's first step begins
  int nsteps, step;
};

// Move the cursor to the first non-empty row at or after cur.i.  Only lanes
// below nb hold pointers of the wavefront's rows; others are never selected.
// amask + 1 is the alignment of the row's first step in entries: 8 is the reverse-offset
// alignment of the paper (a lane's 16-byte chunk never straddles the row start); larger powers
// of two up to 512 make every step of the row begin on a multiple of that many entries.
__device__ __forceinline__ void seek_nonempty(RowCursor& cur, int nb, uint32_t rp_lo, uint32_t rp_hi,
                                              uint32_t amask = 7u) {
  cur.start = cur.end = 0;
  while (cur.i < nb) {
    cur.start = (uint32_t)__builtin_amdgcn_readlane((int)rp_lo, cur.i);
    cur.end = (uint32_t)__builtin_amdgcn_readlane((int)rp_hi, cur.i);
    if (cur.end > cur.start) break;
    ++cur.i;
  }
  cur.a0 = cur.start & ~amask;
  cur.nsteps = (int)((cur.end - cur.a0 + 511u) >> 9);
  cur.step = 0;
}

// Staging of x (fp16[cols], global) into the LDS layout described above, split
// in two so that a kernel can put its own first loads between the halves:
// stage_x_begin only issues global loads into registers (up to XR 16-byte chunks
// per thread, fast path for a 16-byte aligned x); stage_x_finish writes them to
// LDS, copies whatever did not fit (or everything, for an unaligned x), zeroes
// the guards and ends with a barrier.  Both must be called by every thread.
constexpr int kXStageRegs = 4;

struct XStage {
  uint4 r[kXStageRegs];
};

// The loads go through a raw buffer descriptor that covers exactly the whole
// chunks of x: threads whose chunk lies beyond it (and every thread, when x is
// not 16-byte aligned and the descriptor is made empty) get zeros back without
// touching memory.  The loads are therefore unconditional, which keeps the
// compiler's count of outstanding loads exact.
// AUX: cache policy bits of the loads (0: ordinary; kCoherentLoad: coherent over the whole device,
// for an x that workgroups on other parts of the chip have just written, see spmv_chain_kernel).
constexpr int kCoherentLoad = 16;     // sc1: the load does not hit lines that another L2 may have made stale
// nt: threads of the workgroup (a kernel that has it in an argument register passes that: reading
// blockDim is a scalar load from the dispatch's argument block, one memory round trip at start-up)
template <int AUX = 0>
__device__ __forceinline__ void stage_x_begin(XStage& st, const uint16_t* __restrict__ x, int cols, int nt) {
  const bool aligned = (reinterpret_cast<uintptr_t>(x) & 15) == 0;
  const int bytes = aligned ? (cols >> 3) * 16 : 0;   // whole 16-byte chunks of x
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(x), 0, bytes, 0x00020000);
#pragma unroll
  for (int k = 0; k < kXStageRegs; ++k) {
    const int i = (int)threadIdx.x + k * nt;
    const auto v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, i * 16, 0, AUX);
    st.r[k] = make_uint4(v[0], v[1], v[2], v[3]);
  }
}

// one element / one aligned 16-byte chunk of x, device-coherent when AUX asks for it
template <int AUX>
__device__ __forceinline__ uint16_t load_x_elem(const uint16_t* x) {
  if (AUX == 0) return *x;
  return __hip_atomic_load(x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <int AUX>
__device__ __forceinline__ uint4 load_x_chunk(const uint4* x) {
  if (AUX == 0) return *x;
  const unsigned long long* q = reinterpret_cast<const unsigned long long*>(x);
  const unsigned long long lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned long long hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
}

// SIMPLE promises: x is 16-byte aligned, cols is a multiple of 8 and x fits the
// staging registers (cols <= 8 * kXStageRegs * blockDim.x).  The general version
// also copies what did not fit, the ragged tail, or all of an unaligned x.
template <bool SIMPLE, int AUX = 0>
__device__ __forceinline__ void stage_x_finish(unsigned char* lds, const XStage& st,
                                               const uint16_t* __restrict__ x, int cols,
                                               int front_pad, int back_pad, int nt) {
  const int tid = threadIdx.x;
  const uint4 zero = make_uint4(0, 0, 0, 0);
  uint4* lds16 = reinterpret_cast<uint4*>(lds);
  const int chunks = cols >> 3;
  const int tail_chunks = (cols + 7) >> 3;            // chunks touched by x
  // guards: front_pad/16 chunks in front, back_pad/16 behind
  const int guard_chunks = (front_pad + back_pad) / 16;
  for (int i = tid; i < guard_chunks; i += nt)
    lds16[i < front_pad / 16 ? i : i + tail_chunks] = zero;
  uint16_t* xs = reinterpret_cast<uint16_t*>(lds + front_pad);
  uint4* xd = reinterpret_cast<uint4*>(xs);
  if (SIMPLE || (reinterpret_cast<uintptr_t>(x) & 15) == 0) {
#pragma unroll
    for (int k = 0; k < kXStageRegs; ++k) {
      const int i = tid + k * nt;
      if (i < chunks) xd[i] = st.r[k];
    }
    if (!SIMPLE) {
      const uint4* xg = reinterpret_cast<const uint4*>(x);
      for (int i = tid + kXStageRegs * nt; i < chunks; i += nt) xd[i] = load_x_chunk<AUX>(xg + i);
      for (int i = chunks * 8 + tid; i < tail_chunks * 8; i += nt)
        xs[i] = i < cols ? load_x_elem<AUX>(x + i) : (uint16_t)0;
    }
  } else {
    for (int i = tid; i < tail_chunks * 8; i += nt) xs[i] = i < cols ? load_x_elem<AUX>(x + i) : (uint16_t)0;
  }
  __syncthreads();
}

__host__ __device__ inline bool stage_x_is_simple(const void* x, int64_t cols, int block) {
  return (reinterpret_cast<uintptr_t>(x) & 15) == 0 && cols % 8 == 0 &&
         cols <= (int64_t)8 * kXStageRegs * block;
}

__device__ __forceinline__ void stage_x_to_lds(unsigned char* lds, const uint16_t* __restrict__ x, int cols) {
  XStage st;
  stage_x_begin(st, x, cols, (int)blockDim.x);
  stage_x_finish<false>(lds, st, x, cols, kFrontPad, kBackPad, (int)blockDim.x);
}

}  // namespace macko
