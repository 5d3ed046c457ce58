// Expanding the format on the device: the column index of every stored entry
// (Section 4.4: a column is the running sum of the row's deltas; the sums are
// formed as in Algorithm 1, per lane and then across the wavefront) and, from
// those, the dense matrix back (the format is lossless, Section 5.2).
//
// Both use the in-register decode and the cross-lane prefix sum of the product
// kernels, so the column indices they write are the ones the product gathers x
// with; the tests compare them entry by entry with the CPU oracle.
//
// One wavefront per row and 512 entries per step, as in the product.  Nothing
// here is tuned beyond coalesced loads: expanding a matrix is a conversion, not
// a per-token operation.  Roofline: HBM; the dense expansion writes 2 R C bytes
// of zeros, reads 2.5 n bytes and writes 2 nnz bytes again.
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

int launch_decode(const SpmvProblem& p, uint16_t* dense, int64_t ld, hipStream_t stream) {
  if (p.rows == 0 || p.cols == 0) return MACKO_OK;
  const bool vec = p.cols % 8 == 0 && ld % 8 == 0 && (reinterpret_cast<uintptr_t>(dense) & 15) == 0;
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
