// Dense fp16 -> MACKO conversion on the GPU (format of Section 4.1, tail
// padding of Section 4.5).  Three passes: count the stored entries of every
// row, prefix-sum the counts into row_ptr, then write values and codes.  The
// output is bit-identical to the host encoder's.
//
// One wavefront works on one row; per step a lane looks at 8 consecutive
// columns (one 16-byte load, issued one step ahead).  The position of the
// previous stored entry is carried across lanes with a DPP max-scan and across
// steps in a register, so each lane can price its own non-zeros: a non-zero at
// distance g from the previously stored column costs (g-1) / 2^b_delta padding
// entries plus itself.  Per-row counts go to arrays that the scan kernel totals (no atomics).
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

// 8 consecutive columns as loaded (4 x 2 fp16), and the same with the non-zero mask.
struct RawChunk {
  uint32_t u[4];
};
struct Chunk {
  uint16_t h[8];
  unsigned mask;   // bit k set iff h[k] is neither +0 nor -0
};

// Loads only; columns at or beyond `cols` read as +0.  The caller decodes the
// result one loop iteration later, so the load is in flight behind the work on
// the current chunk.
__device__ __forceinline__ RawChunk load_raw(const uint16_t* __restrict__ row, int col0, int cols,
                                             bool vec_ok) {
  RawChunk r;
  if (vec_ok && col0 + 8 <= cols) {
    const uint4 q = *reinterpret_cast<const uint4*>(row + col0);
    r.u[0] = q.x; r.u[1] = q.y; r.u[2] = q.z; r.u[3] = q.w;
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t lo = (col0 + 2 * k < cols) ? row[col0 + 2 * k] : 0u;
      const uint32_t hi = (col0 + 2 * k + 1 < cols) ? row[col0 + 2 * k + 1] : 0u;
      r.u[k] = lo | (hi << 16);
    }
  }
  return r;
}

__device__ __forceinline__ Chunk decode_chunk(const RawChunk& r) {
  Chunk c;
  c.mask = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    c.h[k] = (uint16_t)(r.u[k >> 1] >> (16 * (k & 1)));
    c.mask |= ((c.h[k] & 0x7FFFu) != 0 ? 1u : 0u) << k;
  }
  return c;
}

// What a lane needs to know about its 8 columns.  Two non-zeros inside one
// chunk are at most 7 columns apart, so with deltas of up to 8 or more only the
// first non-zero of a chunk can need padding entries in front of it; for 1- and
// 2-bit codes the gaps inside the chunk are priced one by one.
struct LaneView {
  unsigned entries;   // stored entries this chunk contributes (non-zeros + padding)
  unsigned nnz;       // non-zeros in the chunk
  int lead;           // (gap - 1) of the chunk's first non-zero: column - previous stored column - 1
};

// `carry` is the position (column + 1, 0 = none) of the last stored entry of the
// steps already consumed; it is advanced over this step.
__device__ __forceinline__ LaneView view_chunk(unsigned mask, int col0, int lane, int b_delta, uint32_t* carry) {
  const uint32_t lastpos = mask ? (uint32_t)(col0 + 32 - __clz((int)mask)) : 0u;
  const uint32_t incl = wave_incl_scan_max_u32(lastpos);
  uint32_t prevpos = (uint32_t)__shfl_up((int)incl, 1);
  if (lane == 0) prevpos = 0;
  prevpos = max(prevpos, *carry);
  *carry = max(*carry, (uint32_t)__builtin_amdgcn_readlane((int)incl, 63));
  LaneView v;
  v.nnz = (unsigned)__popc(mask);
  v.lead = mask ? col0 + (__ffs((int)mask) - 1) - (int)prevpos : 0;
  v.entries = mask ? v.nnz + (unsigned)(v.lead >> b_delta) : 0u;
  if (b_delta < 3) {               // deltas of at most 2 or 4: gaps inside the chunk can need padding too
    unsigned m = mask & (mask - 1);                      // every non-zero but the first
    int prevk = mask ? __ffs((int)mask) - 1 : 0;
    while (m) {
      const int k = __ffs((int)m) - 1;
      m &= m - 1;
      v.entries += (unsigned)((k - prevk - 1) >> b_delta);
      prevk = k;
    }
  }
  return v;
}

__global__ void __launch_bounds__(256)
encode_count_kernel(const uint16_t* __restrict__ dense, int rows, int cols, int64_t ld, bool vec_ok, int b_delta,
                    uint32_t* __restrict__ row_entries, uint32_t* __restrict__ row_nnz) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  for (int row = blockIdx.x * nwaves + wave; row < rows; row += gridDim.x * nwaves) {
    const uint16_t* src = dense + (int64_t)row * ld;
    uint32_t carry = 0;
    unsigned entries = 0, nnz = 0;
    RawChunk nxt = load_raw(src, lane * 8, cols, vec_ok);
    for (int base = 0; base < cols; base += 512) {
      const int col0 = base + lane * 8;
      const Chunk c = decode_chunk(nxt);
      nxt = load_raw(src, col0 + 512, cols, vec_ok);                 // next step's columns, in flight
      const LaneView v = view_chunk(c.mask, col0, lane, b_delta, &carry);
      entries += v.entries;
      nnz += v.nnz;
    }
    entries = wave_incl_scan_u32(entries);
    nnz = wave_incl_scan_u32(nnz);
    if (lane == 63) {
      row_entries[row] = entries;
      row_nnz[row] = nnz;
    }
  }
}

// row_ptr[r] = sum of row_entries[0..r); one workgroup.  Also totals the
// statistics of the storage report.  The entry total is kept as a 64-bit number
// so that the host can detect overflow of the 32-bit row pointers before
// anything is written through them.
__global__ void __launch_bounds__(1024)
encode_scan_kernel(const uint32_t* __restrict__ row_entries, const uint32_t* __restrict__ row_nnz,
                   int rows, uint32_t* __restrict__ row_ptr, EncodeStats* __restrict__ stats) {
  __shared__ unsigned long long wave_sum[16];
  __shared__ unsigned long long wave_nnz[16];
  __shared__ unsigned int wave_empty[16];
  __shared__ unsigned int wave_max[16];
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int seg = (rows + 1023) / 1024;
  const int lo = min(rows, t * seg), hi = min(rows, lo + seg);
  unsigned long long s = 0, n = 0;
  unsigned int empty = 0, longest = 0;
  for (int r = lo; r < hi; ++r) {
    const uint32_t e = row_entries[r];
    s += e;
    n += row_nnz[r];
    empty += e == 0;
    longest = max(longest, e);
  }
  // inclusive scan of the segment sums over the wavefront, totals of the rest
  unsigned long long incl = s;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned long long up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    n += __shfl_xor(n, off);
    empty += __shfl_xor(empty, off);
    longest = max(longest, __shfl_xor(longest, off));
  }
  if (lane == 63) {
    wave_sum[wave] = incl;
    wave_nnz[wave] = n;
    wave_empty[wave] = empty;
    wave_max[wave] = longest;
  }
  __syncthreads();
  unsigned long long before = 0;                       // entries of the wavefronts in front of this one
  for (int i = 0; i < wave; ++i) before += wave_sum[i];
  if (t == 1023) {
    unsigned long long nn = 0;
    unsigned int em = 0, mx = 0;
    for (int i = 0; i < 16; ++i) {
      nn += wave_nnz[i];
      em += wave_empty[i];
      mx = max(mx, wave_max[i]);
    }
    const unsigned long long total = before + incl;
    stats->pad_nnz = total;
    stats->nnz = nn;
    stats->empty_rows = em;
    stats->max_row_entries = mx;
    row_ptr[rows] = (uint32_t)total;
  }
  unsigned long long run = before + incl - s;
  for (int r = lo; r < hi; ++r) {
    row_ptr[r] = (uint32_t)run;
    run += row_entries[r];
  }
}

__global__ void __launch_bounds__(256)
encode_fill_kernel(const uint16_t* __restrict__ dense, int rows, int cols, int64_t ld, bool vec_ok, int b_delta,
                   const uint32_t* __restrict__ row_ptr, uint16_t* __restrict__ values,
                   uint8_t* __restrict__ codes8) {
  const int full = (1 << b_delta) - 1;             // code of the largest delta
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  for (int row = blockIdx.x * nwaves + wave; row < rows; row += gridDim.x * nwaves) {
    const uint16_t* src = dense + (int64_t)row * ld;
    uint32_t carry = 0;
    uint32_t cursor = row_ptr[row];              // first entry of this step
    RawChunk nxt = load_raw(src, lane * 8, cols, vec_ok);
    for (int base = 0; base < cols; base += 512) {
      const int col0 = base + lane * 8;
      const Chunk c = decode_chunk(nxt);
      nxt = load_raw(src, col0 + 512, cols, vec_ok);                 // next step's columns, in flight
      const LaneView v = view_chunk(c.mask, col0, lane, b_delta, &carry);
      const uint32_t incl = wave_incl_scan_u32(v.entries);
      size_t o = (size_t)cursor + (incl - v.entries);
      if (c.mask) {
        unsigned m = c.mask;
        int g1 = v.lead;                         // (gap - 1) in front of the next stored non-zero
        int prevk = -1;
        while (m) {
          const int k = __ffs((int)m) - 1;
          m &= m - 1;
          if (prevk >= 0) g1 = k - prevk - 1;
          for (int pads = g1 >> b_delta; pads > 0; --pads) {        // padding entries, greedy
            values[o] = 0;
            codes8[o] = (uint8_t)full;
            ++o;
          }
          values[o] = c.h[k];
          codes8[o] = (uint8_t)(g1 & full);
          ++o;
          prevk = k;
        }
      }
      cursor += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    }
  }
}

// Packed word i holds the codes of entries (32 / b_delta) i ..., entry k in bits
// b_delta (k mod (32 / b_delta)) upwards; one code byte per entry comes in.
__global__ void __launch_bounds__(256)
encode_pack_kernel(const uint8_t* __restrict__ codes8, int64_t words, int b_delta, uint32_t* __restrict__ deltas) {
  const int per_word = 32 / b_delta;                 // 32, 16, 8 or 4 entries: a multiple of 4 bytes of input
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words;
       i += (int64_t)gridDim.x * blockDim.x) {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(codes8 + (int64_t)per_word * i);
    uint32_t w = 0;
    for (int q = 0; q < per_word / 4; ++q) {
      const uint32_t c = src[q];
#pragma unroll
      for (int k = 0; k < 4; ++k) w |= ((c >> (8 * k)) & 0xFFu) << (b_delta * (4 * q + k));
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

int encode_on_device(const uint16_t* dense, int64_t rows, int64_t cols, int64_t ld, int b_delta,
                     hipStream_t stream,
                     uint16_t** values, uint8_t** deltas, uint32_t** row_ptr, int64_t* nnz,
                     int64_t* pad_nnz, int64_t* alloc_nnz, int64_t* empty_rows,
                     int64_t* max_row_entries) {
  const int cus = device_cu_count();
  const bool vec_ok = (ld % 8 == 0) && (reinterpret_cast<uintptr_t>(dense) & 15) == 0;
  DeviceBuf counts, nnzs, stats_d, rp, vals, dels, codes;
  if (counts.alloc(4 * (size_t)rows) != hipSuccess || nnzs.alloc(4 * (size_t)rows) != hipSuccess || stats_d.alloc(sizeof(EncodeStats)) != hipSuccess ||
      rp.alloc(4 * (size_t)(rows + 1)) != hipSuccess) {
    (void)hipGetLastError();
    return MACKO_E_OUT_OF_MEMORY;
  }
  const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((rows + 3) / 4, (int64_t)cus * 16));
  if (rows > 0) {
    hipLaunchKernelGGL(encode_count_kernel, dim3(grid), dim3(256), 0, stream, dense, (int)rows,
                       (int)cols, ld, vec_ok, b_delta, static_cast<uint32_t*>(counts.p),
                       static_cast<uint32_t*>(nnzs.p));
  }
  hipLaunchKernelGGL(encode_scan_kernel, dim3(1), dim3(1024), 0, stream,
                     static_cast<const uint32_t*>(counts.p), static_cast<const uint32_t*>(nnzs.p),
                     (int)rows, static_cast<uint32_t*>(rp.p),
                     static_cast<EncodeStats*>(stats_d.p));
  MACKO_HIP_TRY(hipGetLastError());
  EncodeStats st{};
  MACKO_HIP_TRY(hipMemcpyAsync(&st, stats_d.p, sizeof(st), hipMemcpyDeviceToHost, stream));
  MACKO_HIP_TRY(hipStreamSynchronize(stream));
  if (st.pad_nnz >= (1ull << 32)) return MACKO_E_OVERFLOW;
  const int64_t pad = (int64_t)st.pad_nnz;
  const int64_t granule = alloc_granule(b_delta);
  const int64_t alloc = (pad + granule - 1) / granule * granule;
  if (alloc >= (int64_t{1} << 32)) return MACKO_E_OVERFLOW;
  if (vals.alloc((size_t)alloc * 2) != hipSuccess || dels.alloc((size_t)alloc * b_delta / 8) != hipSuccess ||
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
                       ld, vec_ok, b_delta, static_cast<const uint32_t*>(rp.p), static_cast<uint16_t*>(vals.p),
                       static_cast<uint8_t*>(codes.p));
  }
  if (alloc > 0) {
    const int64_t words = alloc * b_delta / 32;
    const unsigned pgrid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((words + 255) / 256, (int64_t)cus * 16));
    hipLaunchKernelGGL(encode_pack_kernel, dim3(pgrid), dim3(256), 0, stream,
                       static_cast<const uint8_t*>(codes.p), words, b_delta, static_cast<uint32_t*>(dels.p));
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
