// Expanding the format on the device: the column index of every stored entry
// (Section 4.4: a column is the running sum of the row's deltas; the sums are
// formed as in Algorithm 1, per lane and then across the wavefront) and, from
// those, the dense matrix back (the format is lossless, Section 5.2).
//
// Both use the in-register decode and the cross-lane prefix sum of the product
// kernels, so the column indices they write are the ones the product gathers x
// with; the tests compare them entry by entry with the CPU oracle.
//
// One wavefront per row and 512 entries per step, as in the product.  Expanding
// a matrix is a conversion, not a per-token operation.  Roofline: HBM; the dense
// expansion reads 2.5 n bytes and writes 2 R C bytes once (rows are assembled in
// LDS); rows too long for LDS are cleared in HBM first and then scattered into.
#include "macko_decode.h"
#include "macko_device.h"
#include "macko_internal.h"

namespace macko {
namespace {

constexpr int kExpandBlock = 256;

template <int BD, bool DENSE>
__global__ void __launch_bounds__(kExpandBlock)
expand_kernel(const uint4* __restrict__ values, const uint32_t* __restrict__ deltas,
              const uint32_t* __restrict__ row_ptr, const int rows, const int cols,
              int32_t* __restrict__ cols_out, uint16_t* __restrict__ dense, const int64_t ld) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (kExpandBlock / 64) + (threadIdx.x >> 6)));
  const int nwaves = (int)gridDim.x * (kExpandBlock / 64);
  for (int row = wave; row < rows; row += nwaves) {          // wavefront-uniform
    const uint32_t start = (uint32_t)__builtin_amdgcn_readfirstlane((int)row_ptr[row]);
    const uint32_t end = (uint32_t)__builtin_amdgcn_readfirstlane((int)row_ptr[row + 1]);
    if (end <= start) continue;
    const uint32_t a0 = start & ~7u;                         // the lanes' chunks are aligned to 8 entries
    const int nsteps = (int)((end - a0 + 511u) >> 9);
    int base2 = 0;                                           // doubled position before this step
    for (int step = 0; step < nsteps; ++step) {
      const uint32_t e0 = a0 + 512u * (uint32_t)step + 8u * (uint32_t)lane;
      const uint32_t chunk = min(e0, end - 1u) >> 3;         // lanes past the row end re-read its last chunk
      LaneCodes<BD> w;
      w.load(deltas, chunk);
      uint4 v = make_uint4(0, 0, 0, 0);
      if (DENSE) v = load_stream(values + chunk);
      w.keep_if(e0 < end);
      w.decode();
      const uint32_t tot = w.total();
      const uint32_t incl = wave_incl_scan_u32(tot);
      if (step == 0) {
        const int before = (int)(start - a0);                // entries of the previous row in lane 0's chunk
        if (before > 0) base2 = -(int)w.through(before - 1);
      }
      const int lanebase = base2 + (int)(incl - tot);
      const uint32_t vv[4] = {v.x, v.y, v.z, v.w};
#define MACKO_ENTRY(k)                                                                  \
  {                                                                                     \
    const uint32_t e = e0 + k;                                                          \
    if (e >= start && e < end) {                                                        \
      const int col = (lanebase + w.template offset<k>()) >> 1;                         \
      if (DENSE) {                                                                      \
        if (col < cols) dense[(int64_t)row * ld + col] = (uint16_t)(vv[k >> 1] >> (16 * (k & 1))); \
      } else {                                                                          \
        cols_out[e] = col;                                                              \
      }                                                                                 \
    }                                                                                   \
  }
      MACKO_ENTRY(0) MACKO_ENTRY(1) MACKO_ENTRY(2) MACKO_ENTRY(3)
      MACKO_ENTRY(4) MACKO_ENTRY(5) MACKO_ENTRY(6) MACKO_ENTRY(7)
#undef MACKO_ENTRY
      base2 += (int)__builtin_amdgcn_readlane((int)incl, 63);
    }
  }
}

// What the product kernels take on trust about an encoding, checked row by row:
// row_ptr starts at 0, never decreases and ends at pad_nnz, and no entry decodes
// to a column at or beyond cols.  The smallest offending row number is left in
// *first_bad (which the caller sets to `rows` beforehand).  A row whose pointers
// are out of order or out of range is reported without being decoded, so the
// check itself reads nothing outside [0, pad_nnz).
template <int BD>
__global__ void __launch_bounds__(kExpandBlock)
check_kernel(const uint32_t* __restrict__ deltas, const uint32_t* __restrict__ row_ptr, const int rows,
             const int cols, const uint32_t pad_nnz, unsigned int* __restrict__ first_bad) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (kExpandBlock / 64) + (threadIdx.x >> 6)));
  const int nwaves = (int)gridDim.x * (kExpandBlock / 64);
  for (int row = wave; row < rows; row += nwaves) {          // wavefront-uniform
    const uint32_t start = (uint32_t)__builtin_amdgcn_readfirstlane((int)row_ptr[row]);
    const uint32_t end = (uint32_t)__builtin_amdgcn_readfirstlane((int)row_ptr[row + 1]);
    bool bad = end < start || end > pad_nnz || (row == 0 && start != 0u) || (row == rows - 1 && end != pad_nnz);
    if (!bad && end > start) {
      const uint32_t a0 = start & ~7u;
      const int nsteps = (int)((end - a0 + 511u) >> 9);
      int base2 = 0;
      bool lane_bad = false;
      for (int step = 0; step < nsteps; ++step) {
        const uint32_t e0 = a0 + 512u * (uint32_t)step + 8u * (uint32_t)lane;
        const uint32_t chunk = min(e0, end - 1u) >> 3;
        LaneCodes<BD> w;
        w.load(deltas, chunk);
        w.keep_if(e0 < end);
        w.decode();
        const uint32_t tot = w.total();
        const uint32_t incl = wave_incl_scan_u32(tot);
        if (step == 0) {
          const int before = (int)(start - a0);
          if (before > 0) base2 = -(int)w.through(before - 1);
        }
        const int lanebase = base2 + (int)(incl - tot);
#define MACKO_ENTRY(k)                                                                    \
  {                                                                                       \
    const uint32_t e = e0 + k;                                                            \
    if (e >= start && e < end && ((lanebase + w.template offset<k>()) >> 1) >= cols) lane_bad = true; \
  }
        MACKO_ENTRY(0) MACKO_ENTRY(1) MACKO_ENTRY(2) MACKO_ENTRY(3)
        MACKO_ENTRY(4) MACKO_ENTRY(5) MACKO_ENTRY(6) MACKO_ENTRY(7)
#undef MACKO_ENTRY
        base2 += (int)__builtin_amdgcn_readlane((int)incl, 63);
        // a row that runs past the last column keeps running: stop before the positions overflow
        if (__any(lane_bad)) break;
      }
      bad = __any(lane_bad);
    }
    if (bad && lane == 0) atomicMin(first_bad, (unsigned int)row);
  }
}

// dense[r][0 .. cols) = +0 for every row (cells between cols and ld are left alone)
template <bool VEC>
__global__ void __launch_bounds__(256) zero_rows_kernel(uint16_t* __restrict__ dense, const int rows, const int cols,
                                                         const int64_t ld) {
  const int per_row = VEC ? cols / 8 : cols;                 // stores per row
  const int64_t total = (int64_t)rows * per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / per_row;
    const int c = (int)(i - r * per_row);
    if (VEC) reinterpret_cast<uint4*>(dense + r * ld)[c] = make_uint4(0, 0, 0, 0);
    else dense[r * ld + c] = 0;
  }
}

// The dense matrix back, one pass: a wavefront builds its row in LDS (zeros, then the stored
// values at their columns) and writes it out with full-width stores, so every byte of the dense
// matrix is written exactly once and nothing of it is read.  Every wavefront of the workgroup has
// a row buffer of cols values rounded up to 16 bytes.  VB: bits per value (16: fp16, 8: E4M3
// bytes).  VEC: 16-byte stores (dense and ld aligned to 16 bytes, a row a multiple of 16 bytes).
template <int BD, int VB, bool VEC>
__global__ void __launch_bounds__(512)
decode_rows_kernel(const void* __restrict__ values, const uint32_t* __restrict__ deltas,
                   const uint32_t* __restrict__ row_ptr, const int rows, const int cols,
                   void* __restrict__ dense, const int64_t ld) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int EB = VB / 8;                                  // bytes per value
  const int lane = threadIdx.x & 63;
  const int wave_in_wg = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int waves_per_wg = (int)blockDim.x >> 6;
  const int wave = (int)blockIdx.x * waves_per_wg + wave_in_wg;
  const int nwaves = (int)gridDim.x * waves_per_wg;
  const int chunks = (cols * EB + 15) >> 4;                   // 16-byte chunks of the row buffer
  unsigned char* rowbuf = lds + (size_t)wave_in_wg * chunks * 16;
  uint4* rowbuf4 = reinterpret_cast<uint4*>(rowbuf);
  for (int row = wave; row < rows; row += nwaves) {          // wavefront-uniform
    const uint32_t start = (uint32_t)__builtin_amdgcn_readfirstlane((int)row_ptr[row]);
    const uint32_t end = (uint32_t)__builtin_amdgcn_readfirstlane((int)row_ptr[row + 1]);
    for (int c = lane; c < chunks; c += 64) rowbuf4[c] = make_uint4(0, 0, 0, 0);
    if (end > start) {
      const uint32_t a0 = start & ~7u;
      const int nsteps = (int)((end - a0 + 511u) >> 9);
      int base2 = 0;
      LaneCodes<BD> wn;                                      // the next step's loads, one step ahead
      LaneValues<VB> vn;
      {
        const uint32_t chunk = min(a0 + 8u * (uint32_t)lane, end - 1u) >> 3;
        wn.load(deltas, chunk);
        vn.load(values, chunk);
      }
      for (int step = 0; step < nsteps; ++step) {
        const uint32_t e0 = a0 + 512u * (uint32_t)step + 8u * (uint32_t)lane;
        LaneCodes<BD> w = wn;
        const LaneValues<VB> v = vn;
        {                                                    // lanes past the row end re-read its last chunk
          const uint32_t chunk = min(e0 + 512u, end - 1u) >> 3;
          wn.load(deltas, chunk);
          vn.load(values, chunk);
        }
        w.keep_if(e0 < end);
        w.decode();
        const uint32_t tot = w.total();
        const uint32_t incl = wave_incl_scan_u32(tot);
        if (step == 0) {
          const int before = (int)(start - a0);
          if (before > 0) base2 = -(int)w.through(before - 1);
        }
        const int lanebase = base2 + (int)(incl - tot);
#define MACKO_ENTRY(k)                                                                  \
  {                                                                                     \
    const uint32_t e = e0 + k;                                                          \
    const int col = (lanebase + w.template offset<k>()) >> 1;                           \
    if (e >= start && e < end && col < cols) {                                          \
      if (VB == 16) reinterpret_cast<uint16_t*>(rowbuf)[col] = (uint16_t)v.template bits<k>(); \
      else rowbuf[col] = (unsigned char)v.template bits<k>();                           \
    }                                                                                   \
  }
        MACKO_ENTRY(0) MACKO_ENTRY(1) MACKO_ENTRY(2) MACKO_ENTRY(3)
        MACKO_ENTRY(4) MACKO_ENTRY(5) MACKO_ENTRY(6) MACKO_ENTRY(7)
#undef MACKO_ENTRY
        base2 += (int)__builtin_amdgcn_readlane((int)incl, 63);
      }
    }
    // the row buffer is private to the wavefront, whose LDS operations complete in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    unsigned char* out = static_cast<unsigned char*>(dense) + (int64_t)row * ld * EB;
    if (VEC) {
      typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
      for (int c = lane; c < chunks; c += 64) {
        const uint4 t = rowbuf4[c];
        u32x4 q = {t.x, t.y, t.z, t.w};
        __builtin_nontemporal_store(q, reinterpret_cast<u32x4*>(out) + c);
      }
    } else if (VB == 16) {
      for (int c = lane; c < cols; c += 64)
        reinterpret_cast<uint16_t*>(out)[c] = reinterpret_cast<const uint16_t*>(rowbuf)[c];
    } else {
      for (int c = lane; c < cols; c += 64) out[c] = rowbuf[c];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();                         // the buffer is cleared again only after it was read
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

template <int BD, int VB>
int launch_decode_rows_bd(const SpmvProblem& p, void* dense, int64_t ld, bool vec, int waves_per_wg,
                          int64_t lds_bytes, hipStream_t stream) {
  const int block = 64 * waves_per_wg;
  const int64_t waves_wanted = std::min<int64_t>(p.rows, (int64_t)device_cu_count() * 32);
  const dim3 grid((unsigned)((waves_wanted + waves_per_wg - 1) / waves_per_wg));
  const uint32_t* deltas = reinterpret_cast<const uint32_t*>(p.deltas);
  auto kfn = vec ? decode_rows_kernel<BD, VB, true> : decode_rows_kernel<BD, VB, false>;
  if (lds_bytes > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds_bytes);
    if (e != hipSuccess) return hip_fail(e);
  }
  hipLaunchKernelGGL(kfn, grid, dim3(block), (size_t)lds_bytes, stream, static_cast<const void*>(p.values), deltas,
                     p.row_ptr, (int)p.rows, (int)p.cols, dense, ld);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MACKO_OK : hip_fail(e);
}

template <bool DENSE>
int launch_expand(const SpmvProblem& p, int32_t* cols_out, uint16_t* dense, int64_t ld, hipStream_t stream) {
  const int64_t waves_wanted = std::min<int64_t>(p.rows, (int64_t)device_cu_count() * 64);
  const dim3 grid((unsigned)((waves_wanted + kExpandBlock / 64 - 1) / (kExpandBlock / 64))), block(kExpandBlock);
  const uint4* values = reinterpret_cast<const uint4*>(p.values);
  const uint32_t* deltas = reinterpret_cast<const uint32_t*>(p.deltas);
  switch (p.b_delta) {
    case 1:
      hipLaunchKernelGGL((expand_kernel<1, DENSE>), grid, block, 0, stream, values, deltas, p.row_ptr, (int)p.rows,
                         (int)p.cols, cols_out, dense, ld);
      break;
    case 2:
      hipLaunchKernelGGL((expand_kernel<2, DENSE>), grid, block, 0, stream, values, deltas, p.row_ptr, (int)p.rows,
                         (int)p.cols, cols_out, dense, ld);
      break;
    case 4:
      hipLaunchKernelGGL((expand_kernel<4, DENSE>), grid, block, 0, stream, values, deltas, p.row_ptr, (int)p.rows,
                         (int)p.cols, cols_out, dense, ld);
      break;
    case 8:
      hipLaunchKernelGGL((expand_kernel<8, DENSE>), grid, block, 0, stream, values, deltas, p.row_ptr, (int)p.rows,
                         (int)p.cols, cols_out, dense, ld);
      break;
    default:
      return MACKO_E_UNSUPPORTED;
  }
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MACKO_OK : hip_fail(e);
}

}  // namespace

int launch_check(const SpmvProblem& p, unsigned int* first_bad, hipStream_t stream) {
  const int64_t waves_wanted = std::min<int64_t>(p.rows, (int64_t)device_cu_count() * 64);
  const dim3 grid((unsigned)((waves_wanted + kExpandBlock / 64 - 1) / (kExpandBlock / 64))), block(kExpandBlock);
  const uint32_t* deltas = reinterpret_cast<const uint32_t*>(p.deltas);
  switch (p.b_delta) {
    case 1:
      hipLaunchKernelGGL(check_kernel<1>, grid, block, 0, stream, deltas, p.row_ptr, (int)p.rows, (int)p.cols,
                         (uint32_t)p.pad_nnz, first_bad);
      break;
    case 2:
      hipLaunchKernelGGL(check_kernel<2>, grid, block, 0, stream, deltas, p.row_ptr, (int)p.rows, (int)p.cols,
                         (uint32_t)p.pad_nnz, first_bad);
      break;
    case 4:
      hipLaunchKernelGGL(check_kernel<4>, grid, block, 0, stream, deltas, p.row_ptr, (int)p.rows, (int)p.cols,
                         (uint32_t)p.pad_nnz, first_bad);
      break;
    case 8:
      hipLaunchKernelGGL(check_kernel<8>, grid, block, 0, stream, deltas, p.row_ptr, (int)p.rows, (int)p.cols,
                         (uint32_t)p.pad_nnz, first_bad);
      break;
    default:
      return MACKO_E_UNSUPPORTED;
  }
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MACKO_OK : hip_fail(e);
}

int launch_columns(const SpmvProblem& p, int32_t* cols_out, hipStream_t stream) {
  if (p.rows == 0 || p.pad_nnz == 0) return MACKO_OK;
  return launch_expand<false>(p, cols_out, nullptr, 0, stream);
}

int launch_decode(const SpmvProblem& p, void* dense_any, int64_t ld, hipStream_t stream) {
  if (p.rows == 0 || p.cols == 0) return MACKO_OK;
  const int eb = p.b_val / 8;                                // bytes per value
  const bool vec = (p.cols * eb) % 16 == 0 && (ld * eb) % 16 == 0 && (reinterpret_cast<uintptr_t>(dense_any) & 15) == 0;
  // one pass through a row buffer in LDS per wavefront
  const int64_t row_bytes = 16 * ((p.cols * eb + 15) / 16);
  constexpr int64_t kLdsLimit = 160 * 1024;
  if (row_bytes <= kLdsLimit) {
    // row buffers per compute unit: workgroups of 4 wavefronts while 8 or more fit, else one workgroup of 1..7
    const int per_cu = (int)(kLdsLimit / row_bytes);
    const int waves_per_wg = per_cu >= 8 ? 4 : per_cu;
    const int64_t lds_bytes = row_bytes * waves_per_wg;
    if (p.b_val == 8) {                                      // 8-bit values come with 4-bit codes
      if (p.b_delta != 4) return MACKO_E_UNSUPPORTED;
      return launch_decode_rows_bd<4, 8>(p, dense_any, ld, vec, waves_per_wg, lds_bytes, stream);
    }
    switch (p.b_delta) {
      case 1: return launch_decode_rows_bd<1, 16>(p, dense_any, ld, vec, waves_per_wg, lds_bytes, stream);
      case 2: return launch_decode_rows_bd<2, 16>(p, dense_any, ld, vec, waves_per_wg, lds_bytes, stream);
      case 4: return launch_decode_rows_bd<4, 16>(p, dense_any, ld, vec, waves_per_wg, lds_bytes, stream);
      case 8: return launch_decode_rows_bd<8, 16>(p, dense_any, ld, vec, waves_per_wg, lds_bytes, stream);
      default: return MACKO_E_UNSUPPORTED;
    }
  }
  if (p.b_val != 16) return MACKO_E_UNSUPPORTED;             // 8-bit rows of more than 163840 columns
  uint16_t* dense = static_cast<uint16_t*>(dense_any);
  // rows too long for LDS: clear the matrix, then scatter the stored values (two kernels in stream order)
  const int64_t stores = p.rows * (vec ? p.cols / 8 : p.cols);
  const int64_t wgs = std::min<int64_t>((stores + 255) / 256, (int64_t)device_cu_count() * 32);
  if (vec)
    hipLaunchKernelGGL(zero_rows_kernel<true>, dim3((unsigned)wgs), dim3(256), 0, stream, dense, (int)p.rows,
                       (int)p.cols, ld);
  else
    hipLaunchKernelGGL(zero_rows_kernel<false>, dim3((unsigned)wgs), dim3(256), 0, stream, dense, (int)p.rows,
                       (int)p.cols, ld);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e);
  if (p.pad_nnz == 0) return MACKO_OK;
  return launch_expand<true>(p, nullptr, dense, ld, stream);
}

}  // namespace macko
