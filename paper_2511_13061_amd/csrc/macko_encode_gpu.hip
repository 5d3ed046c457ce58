// Dense fp16 -> MACKO conversion on the GPU (format of Section 4.1, tail
// padding of Section 4.5).  Three passes: count the stored entries of every
// row, prefix-sum the counts into row_ptr, then write values and codes.  The
// output is bit-identical to the host encoder's.
//
// One wavefront works on one row; per step a lane looks at 8 consecutive
// columns.  The column of the previous stored entry is carried across lanes
// with a max-scan and across steps in a register, so each lane can price its own
// non-zeros: a non-zero at distance g from the previously stored column costs
// (g-1)/16 padding entries plus itself.
#include "macko_device.h"
#include "macko_internal.h"

namespace macko {
namespace {

struct EncodeStats {
  unsigned long long nnz;
  unsigned long long pad_nnz;
  unsigned int empty_rows;
  unsigned int max_row_entries;
};

struct Chunk {
  uint16_t h[8];
  unsigned mask;   // bit k set iff h[k] is neither +0 nor -0
};

__device__ __forceinline__ Chunk load_chunk(const uint16_t* __restrict__ row, int col0, int cols,
                                            bool vec_ok) {
  Chunk c;
  if (vec_ok && col0 + 8 <= cols) {
    const uint4 q = *reinterpret_cast<const uint4*>(row + col0);
    const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int k = 0; k < 8; ++k) c.h[k] = (uint16_t)(u[k >> 1] >> (16 * (k & 1)));
  } else {
#pragma unroll
    for (int k = 0; k < 8; ++k) c.h[k] = (col0 + k < cols) ? row[col0 + k] : (uint16_t)0;
  }
  c.mask = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) c.mask |= ((c.h[k] & 0x7FFFu) != 0 ? 1u : 0u) << k;
  return c;
}

// column of the last stored entry before this lane's chunk
__device__ __forceinline__ int prev_stored_column(unsigned mask, int col0, int lane, int* carry) {
  const int last_in = mask ? col0 + (31 - __clz((int)mask)) : -1;
  int incl = last_in;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(incl, off);
    if (lane >= off) incl = max(incl, t);
  }
  int prev = __shfl_up(incl, 1);
  if (lane == 0) prev = -1;
  prev = max(prev, *carry);
  *carry = max(*carry, __shfl(incl, 63));
  return prev;
}

__global__ void __launch_bounds__(256)
encode_count_kernel(const uint16_t* __restrict__ dense, int rows, int cols, int64_t ld, bool vec_ok,
                    uint32_t* __restrict__ row_entries, EncodeStats* __restrict__ stats) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  for (int row = blockIdx.x * nwaves + wave; row < rows; row += gridDim.x * nwaves) {
    const uint16_t* src = dense + (int64_t)row * ld;
    int carry = -1;
    unsigned entries = 0, nnz = 0;
    for (int base = 0; base < cols; base += 512) {
      const int col0 = base + lane * 8;
      const Chunk c = load_chunk(src, col0, cols, vec_ok);
      int p = prev_stored_column(c.mask, col0, lane, &carry);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if ((c.mask >> k) & 1u) {
          const int col = col0 + k;
          entries += 1u + (unsigned)((col - p - 1) >> kDeltaBits);
          ++nnz;
          p = col;
        }
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      entries += __shfl_xor(entries, off);
      nnz += __shfl_xor(nnz, off);
    }
    if (lane == 0) {
      row_entries[row] = entries;
      atomicAdd(&stats->nnz, (unsigned long long)nnz);
      if (entries == 0) atomicAdd(&stats->empty_rows, 1u);
      atomicMax(&stats->max_row_entries, entries);
    }
  }
}

// row_ptr[r] = sum of row_entries[0..r); one workgroup.  The total goes to
// stats->pad_nnz as a 64-bit number so that the host can detect overflow of the
// 32-bit row pointers before anything is written through them.
__global__ void __launch_bounds__(1024)
encode_scan_kernel(const uint32_t* __restrict__ row_entries, int rows, uint32_t* __restrict__ row_ptr,
                   EncodeStats* __restrict__ stats) {
  __shared__ unsigned long long part[1024];
  const int t = threadIdx.x;
  const int seg = (rows + 1023) / 1024;
  const int lo = min(rows, t * seg), hi = min(rows, lo + seg);
  unsigned long long s = 0;
  for (int r = lo; r < hi; ++r) s += row_entries[r];
  part[t] = s;
  __syncthreads();
  if (t == 0) {
    unsigned long long run = 0;
    for (int i = 0; i < 1024; ++i) {
      const unsigned long long v = part[i];
      part[i] = run;
      run += v;
    }
    stats->pad_nnz = run;
    row_ptr[rows] = (uint32_t)run;
  }
  __syncthreads();
  unsigned long long run = part[t];
  for (int r = lo; r < hi; ++r) {
    row_ptr[r] = (uint32_t)run;
    run += row_entries[r];
  }
}

__global__ void __launch_bounds__(256)
encode_fill_kernel(const uint16_t* __restrict__ dense, int rows, int cols, int64_t ld, bool vec_ok,
                   const uint32_t* __restrict__ row_ptr, uint16_t* __restrict__ values,
                   uint8_t* __restrict__ codes8) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  for (int row = blockIdx.x * nwaves + wave; row < rows; row += gridDim.x * nwaves) {
    const uint16_t* src = dense + (int64_t)row * ld;
    int carry = -1;
    uint32_t cursor = row_ptr[row];              // first entry of this step
    for (int base = 0; base < cols; base += 512) {
      const int col0 = base + lane * 8;
      const Chunk c = load_chunk(src, col0, cols, vec_ok);
      const int prev = prev_stored_column(c.mask, col0, lane, &carry);
      unsigned mine = 0;
      int p = prev;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if ((c.mask >> k) & 1u) {
          mine += 1u + (unsigned)((col0 + k - p - 1) >> kDeltaBits);
          p = col0 + k;
        }
      }
      unsigned incl = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const unsigned t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
      size_t o = (size_t)cursor + (incl - mine);
      p = prev;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if ((c.mask >> k) & 1u) {
          const int g1 = col0 + k - p - 1;       // gap - 1
          for (int pads = g1 >> kDeltaBits; pads > 0; --pads) {
            values[o] = 0;
            codes8[o] = kMaxDelta - 1;
            ++o;
          }
          values[o] = c.h[k];
          codes8[o] = (uint8_t)(g1 & (kMaxDelta - 1));
          ++o;
          p = col0 + k;
        }
      }
      cursor += __shfl(incl, 63);
    }
  }
}

// deltas word i packs the codes of entries 8i .. 8i+7, entry k in bits 4(k&7)..
__global__ void __launch_bounds__(256)
encode_pack_kernel(const uint8_t* __restrict__ codes8, int64_t words, uint32_t* __restrict__ deltas) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words;
       i += (int64_t)gridDim.x * blockDim.x) {
    const uint2 c = *reinterpret_cast<const uint2*>(codes8 + 8 * i);
    uint32_t w = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      w |= ((c.x >> (8 * k)) & 15u) << (4 * k);
      w |= ((c.y >> (8 * k)) & 15u) << (4 * k + 16);
    }
    deltas[i] = w;
  }
}

struct DeviceBuf {
  void* p = nullptr;
  ~DeviceBuf() {
    if (p) (void)hipFree(p);
  }
  hipError_t alloc(size_t n) { return hipMalloc(&p, n ? n : 16); }
  void* release() {
    void* q = p;
    p = nullptr;
    return q;
  }
};

}  // namespace

int encode_on_device(const uint16_t* dense, int64_t rows, int64_t cols, int64_t ld, hipStream_t stream,
                     uint16_t** values, uint8_t** deltas, uint32_t** row_ptr, int64_t* nnz,
                     int64_t* pad_nnz, int64_t* alloc_nnz, int64_t* empty_rows,
                     int64_t* max_row_entries) {
  const int cus = device_cu_count();
  const bool vec_ok = (ld % 8 == 0) && (reinterpret_cast<uintptr_t>(dense) & 15) == 0;
  DeviceBuf counts, stats_d, rp, vals, dels, codes;
  if (counts.alloc(4 * (size_t)rows) != hipSuccess || stats_d.alloc(sizeof(EncodeStats)) != hipSuccess ||
      rp.alloc(4 * (size_t)(rows + 1)) != hipSuccess) {
    (void)hipGetLastError();
    return MACKO_E_OUT_OF_MEMORY;
  }
  MACKO_HIP_TRY(hipMemsetAsync(stats_d.p, 0, sizeof(EncodeStats), stream));
  const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((rows + 3) / 4, (int64_t)cus * 16));
  if (rows > 0) {
    hipLaunchKernelGGL(encode_count_kernel, dim3(grid), dim3(256), 0, stream, dense, (int)rows,
                       (int)cols, ld, vec_ok, static_cast<uint32_t*>(counts.p),
                       static_cast<EncodeStats*>(stats_d.p));
  }
  hipLaunchKernelGGL(encode_scan_kernel, dim3(1), dim3(1024), 0, stream,
                     static_cast<const uint32_t*>(counts.p), (int)rows, static_cast<uint32_t*>(rp.p),
                     static_cast<EncodeStats*>(stats_d.p));
  MACKO_HIP_TRY(hipGetLastError());
  EncodeStats st{};
  MACKO_HIP_TRY(hipMemcpyAsync(&st, stats_d.p, sizeof(st), hipMemcpyDeviceToHost, stream));
  MACKO_HIP_TRY(hipStreamSynchronize(stream));
  if (st.pad_nnz >= (1ull << 32)) return MACKO_E_OVERFLOW;
  const int64_t pad = (int64_t)st.pad_nnz;
  const int64_t alloc = (pad + kAllocGranule - 1) / kAllocGranule * kAllocGranule;
  if (alloc >= (int64_t{1} << 32)) return MACKO_E_OVERFLOW;
  if (vals.alloc((size_t)alloc * 2) != hipSuccess || dels.alloc((size_t)alloc / 2) != hipSuccess ||
      codes.alloc((size_t)alloc) != hipSuccess) {
    (void)hipGetLastError();
    return MACKO_E_OUT_OF_MEMORY;
  }
  if (alloc > pad) {  // zero tail of both arrays
    MACKO_HIP_TRY(hipMemsetAsync(static_cast<uint16_t*>(vals.p) + pad, 0, (size_t)(alloc - pad) * 2, stream));
    MACKO_HIP_TRY(hipMemsetAsync(static_cast<uint8_t*>(codes.p) + pad, 0, (size_t)(alloc - pad), stream));
  }
  if (rows > 0 && pad > 0) {
    hipLaunchKernelGGL(encode_fill_kernel, dim3(grid), dim3(256), 0, stream, dense, (int)rows, (int)cols,
                       ld, vec_ok, static_cast<const uint32_t*>(rp.p), static_cast<uint16_t*>(vals.p),
                       static_cast<uint8_t*>(codes.p));
  }
  if (alloc > 0) {
    const int64_t words = alloc / 8;
    const unsigned pgrid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((words + 255) / 256, (int64_t)cus * 16));
    hipLaunchKernelGGL(encode_pack_kernel, dim3(pgrid), dim3(256), 0, stream,
                       static_cast<const uint8_t*>(codes.p), words, static_cast<uint32_t*>(dels.p));
  }
  MACKO_HIP_TRY(hipGetLastError());
  MACKO_HIP_TRY(hipStreamSynchronize(stream));
  *values = static_cast<uint16_t*>(vals.release());
  *deltas = static_cast<uint8_t*>(dels.release());
  *row_ptr = static_cast<uint32_t*>(rp.release());
  *nnz = (int64_t)st.nnz;
  *pad_nnz = pad;
  *alloc_nnz = alloc;
  *empty_rows = st.empty_rows;
  *max_row_entries = st.max_row_entries;
  return MACKO_OK;
}

}  // namespace macko
