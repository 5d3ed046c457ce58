// Dense fp16 -> MACKO conversion on the GPU (format of Section 4.1, tail
// padding of Section 4.5).  Passes: count the stored entries of every row,
// prefix-sum the counts into row_ptr, write values and one code byte per entry,
// pack the code bytes.  The output is bit-identical to the host encoder's.
//
// One wavefront works on one row; per step a lane looks at 8 consecutive
// columns (one 16-byte load, issued one step ahead).  The position of the
// previous stored entry is carried across lanes with a DPP max-scan and across
// steps in a register, so each lane can price its own non-zeros: a non-zero at
// distance g from the previously stored column costs (g-1) / 2^b_delta padding
// entries plus itself.  Per-row counts go to arrays that the scan kernel totals (no atomics).
#include "macko_device.h"
#include "macko_internal.h"

#include <mutex>

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
//
// 8-bit values (IN8) are widened on the way in, sign to bit 15 and the other seven bits in
// place, so that "neither +0 nor -0" is the same test for both widths; the fill pass then
// writes 16-bit values to scratch and a last pass narrows them again.
__device__ __forceinline__ uint32_t widen8(uint32_t b) { return (b & 0x7Fu) | ((b & 0x80u) << 8); }

template <bool IN8>
__device__ __forceinline__ RawChunk load_raw(const void* __restrict__ row_v, int col0, int cols, bool vec_ok) {
  RawChunk r;
  if (IN8) {
    const uint8_t* row = static_cast<const uint8_t*>(row_v);
    uint32_t b[8];
    if (vec_ok && col0 + 8 <= cols) {
      const uint2 q = *reinterpret_cast<const uint2*>(row + col0);
#pragma unroll
      for (int k = 0; k < 8; ++k) b[k] = ((k < 4 ? q.x : q.y) >> (8 * (k & 3))) & 0xFFu;
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) b[k] = (col0 + k < cols) ? row[col0 + k] : 0u;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) r.u[k] = widen8(b[2 * k]) | (widen8(b[2 * k + 1]) << 16);
    return r;
  }
  const uint16_t* row = static_cast<const uint16_t*>(row_v);
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

template <bool IN8>
__global__ void __launch_bounds__(256)
encode_count_kernel(const void* __restrict__ dense, int rows, int cols, int64_t ld, bool vec_ok, int b_delta,
                    uint32_t* __restrict__ row_entries, uint32_t* __restrict__ row_nnz) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  for (int row = blockIdx.x * nwaves + wave; row < rows; row += gridDim.x * nwaves) {
    const void* src = static_cast<const unsigned char*>(dense) + (int64_t)row * ld * (IN8 ? 1 : 2);
    uint32_t carry = 0;
    unsigned entries = 0, nnz = 0;
    RawChunk nxt = load_raw<IN8>(src, lane * 8, cols, vec_ok);
    for (int base = 0; base < cols; base += 512) {
      const int col0 = base + lane * 8;
      const Chunk c = decode_chunk(nxt);
      nxt = load_raw<IN8>(src, col0 + 512, cols, vec_ok);            // next step's columns, in flight
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

// Row pointers from the per-row counts in three small launches: every block of
// 1024 rows totals its counts, one workgroup turns the block totals into block
// offsets (and totals the statistics of the storage report), every block then
// prefix-sums its own rows.  The entry total is kept as a 64-bit number so that
// the host can detect overflow of the 32-bit row pointers before anything is
// written through them.
struct BlockSums {
  unsigned long long entries;
  unsigned long long nnz;
  unsigned int empty;
  unsigned int longest;
};

__device__ __forceinline__ unsigned long long wave_incl_scan_u64(unsigned long long v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned long long up = __shfl_up(v, off);
    if (lane >= off) v += up;
  }
  return v;
}

__global__ void __launch_bounds__(1024)
encode_block_sums_kernel(const uint32_t* __restrict__ row_entries, const uint32_t* __restrict__ row_nnz, int rows,
                         BlockSums* __restrict__ sums) {
  __shared__ BlockSums part[16];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int r = blockIdx.x * 1024 + t;
  const uint32_t e = r < rows ? row_entries[r] : 0u;
  unsigned long long se = e, sn = r < rows ? row_nnz[r] : 0u;
  unsigned int empty = (r < rows && e == 0) ? 1u : 0u, longest = e;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    se += __shfl_xor(se, off);
    sn += __shfl_xor(sn, off);
    empty += __shfl_xor(empty, off);
    longest = max(longest, __shfl_xor(longest, off));
  }
  if (lane == 0) part[wave] = BlockSums{se, sn, empty, longest};
  __syncthreads();
  if (t == 0) {
    BlockSums b = part[0];
    for (int i = 1; i < 16; ++i) {
      b.entries += part[i].entries;
      b.nnz += part[i].nnz;
      b.empty += part[i].empty;
      b.longest = max(b.longest, part[i].longest);
    }
    sums[blockIdx.x] = b;
  }
}

// one workgroup: block_off[b] = entries of the blocks in front of b; totals to *stats
__global__ void __launch_bounds__(1024)
encode_block_offsets_kernel(const BlockSums* __restrict__ sums, int nblocks, unsigned long long* __restrict__ block_off,
                            uint32_t* __restrict__ row_ptr_last, EncodeStats* __restrict__ stats) {
  __shared__ unsigned long long wave_tot[16];
  __shared__ unsigned long long carry_s;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  unsigned long long nnz = 0;
  unsigned int empty = 0, longest = 0;
  if (t == 0) carry_s = 0;
  __syncthreads();
  for (int base = 0; base < nblocks; base += 1024) {
    const int b = base + t;
    const BlockSums v = b < nblocks ? sums[b] : BlockSums{0, 0, 0, 0};
    nnz += v.nnz;
    empty += v.empty;
    longest = max(longest, v.longest);
    const unsigned long long incl = wave_incl_scan_u64(v.entries, lane);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    unsigned long long before = carry_s;
    for (int i = 0; i < wave; ++i) before += wave_tot[i];
    if (b < nblocks) block_off[b] = before + incl - v.entries;
    __syncthreads();
    if (t == 1023) carry_s = before + incl;
    __syncthreads();
  }
  // totals of the statistics over the workgroup
  __shared__ unsigned long long s_nnz[16];
  __shared__ unsigned int s_empty[16], s_long[16];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    nnz += __shfl_xor(nnz, off);
    empty += __shfl_xor(empty, off);
    longest = max(longest, __shfl_xor(longest, off));
  }
  if (lane == 0) {
    s_nnz[wave] = nnz;
    s_empty[wave] = empty;
    s_long[wave] = longest;
  }
  __syncthreads();
  if (t == 0) {
    unsigned long long nn = 0;
    unsigned int em = 0, mx = 0;
    for (int i = 0; i < 16; ++i) {
      nn += s_nnz[i];
      em += s_empty[i];
      mx = max(mx, s_long[i]);
    }
    stats->pad_nnz = carry_s;
    stats->nnz = nn;
    stats->empty_rows = em;
    stats->max_row_entries = mx;
    *row_ptr_last = (uint32_t)carry_s;
  }
}

__global__ void __launch_bounds__(1024)
encode_row_ptr_kernel(const uint32_t* __restrict__ row_entries, int rows, const unsigned long long* __restrict__ block_off,
                      uint32_t* __restrict__ row_ptr, uint32_t total) {
  __shared__ unsigned long long wave_tot[16];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int r = blockIdx.x * 1024 + t;
  const unsigned long long e = r < rows ? row_entries[r] : 0u;
  const unsigned long long incl = wave_incl_scan_u64(e, lane);
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  unsigned long long before = block_off[blockIdx.x];
  for (int i = 0; i < wave; ++i) before += wave_tot[i];
  if (r < rows) row_ptr[r] = (uint32_t)(before + incl - e);
  if (r == rows - 1) row_ptr[rows] = total;
}

// Second pass: values and one code byte per entry.  A wavefront's entries of one step are
// contiguous in the output (from `cursor` on), but every lane holds a different number of them;
// they are first put in order in LDS (index = position in the output modulo 16, so that aligned
// 16-byte pieces of LDS are aligned 16-byte pieces of the arrays) and then written out with
// 16-byte stores, the ragged first and last piece element by element.  A step with more than
// kStage entries (long runs of padding) writes straight to memory instead.
constexpr int kStage = 1024;
constexpr int kFillWaves = 4;

template <bool IN8>
__global__ void __launch_bounds__(64 * kFillWaves)
encode_fill_kernel(const void* __restrict__ dense, int rows, int cols, int64_t ld, bool vec_ok, int b_delta,
                   const uint32_t* __restrict__ row_ptr, uint16_t* __restrict__ values,
                   uint8_t* __restrict__ codes8, uint32_t pad_nnz, uint32_t alloc_nnz) {
  // the zero tail of both arrays (fewer than 128 entries): the first workgroup writes it
  if (blockIdx.x == 0)
    for (uint32_t k = pad_nnz + threadIdx.x; k < alloc_nnz; k += blockDim.x) {
      values[k] = 0;
      codes8[k] = 0;
    }
  __shared__ __align__(16) uint16_t stage_v[kFillWaves][kStage + 16];
  __shared__ __align__(16) uint8_t stage_c[kFillWaves][kStage + 16];
  const int full = (1 << b_delta) - 1;             // code of the largest delta
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  uint16_t* sv = stage_v[wave];
  uint8_t* sc = stage_c[wave];
  for (int row = blockIdx.x * nwaves + wave; row < rows; row += gridDim.x * nwaves) {
    const void* src = static_cast<const unsigned char*>(dense) + (int64_t)row * ld * (IN8 ? 1 : 2);
    uint32_t carry = 0;
    uint32_t cursor = row_ptr[row];              // first entry of this step
    RawChunk nxt = load_raw<IN8>(src, lane * 8, cols, vec_ok);
    for (int base = 0; base < cols; base += 512) {
      const int col0 = base + lane * 8;
      const Chunk c = decode_chunk(nxt);
      nxt = load_raw<IN8>(src, col0 + 512, cols, vec_ok);            // next step's columns, in flight
      const LaneView v = view_chunk(c.mask, col0, lane, b_delta, &carry);
      const uint32_t incl = wave_incl_scan_u32(v.entries);
      const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
      const bool staged = total <= (uint32_t)kStage;                 // wavefront-uniform
      const uint32_t align = cursor & 15u;
      // where this lane's first entry goes: LDS index (staged) or output index (direct)
      size_t o = staged ? (size_t)(align + (incl - v.entries)) : (size_t)cursor + (incl - v.entries);
      if (c.mask && staged && b_delta >= 3) {
        // Common case.  Only the chunk's first non-zero can have padding in front of it; the
        // eight columns are then visited in a fixed order, so that no register is picked with a
        // run-time index and every lane runs the same eight predicated stores.
        for (int pads = v.lead >> b_delta; pads > 0; --pads) {       // padding entries, greedy
          sv[o] = 0;
          sc[o] = (uint8_t)full;
          ++o;
        }
        int g1 = v.lead & full;                  // code of the next stored non-zero
        bool seen = false;                       // zeros in front of the first non-zero are part of v.lead
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          if ((c.mask >> k) & 1u) {
            sv[o] = c.h[k];
            sc[o] = (uint8_t)g1;
            ++o;
            g1 = 0;                              // the next non-zero is g1 + 1 columns further
            seen = true;
          } else if (seen) {
            ++g1;
          }
        }
      } else if (c.mask) {
        unsigned m = c.mask;
        int g1 = v.lead;                         // (gap - 1) in front of the next stored non-zero
        int prevk = -1;
        while (m) {
          const int k = __ffs((int)m) - 1;
          m &= m - 1;
          if (prevk >= 0) g1 = k - prevk - 1;
          for (int pads = g1 >> b_delta; pads > 0; --pads) {        // padding entries, greedy
            if (staged) {
              sv[o] = 0;
              sc[o] = (uint8_t)full;
            } else {
              values[o] = 0;
              codes8[o] = (uint8_t)full;
            }
            ++o;
          }
          if (staged) {
            sv[o] = c.h[k];
            sc[o] = (uint8_t)(g1 & full);
          } else {
            values[o] = c.h[k];
            codes8[o] = (uint8_t)(g1 & full);
          }
          ++o;
          prevk = k;
        }
      }
      if (staged && total > 0) {
        __builtin_amdgcn_wave_barrier();
        const uint32_t first = align, last = align + total;         // staged entries [first, last)
        const size_t out0 = (size_t)cursor - align;                  // output index of staged index 0 (multiple of 16)
        // values: pieces of 8 entries
        for (uint32_t p = lane; 8u * p < last; p += 64) {
          const uint32_t lo = 8u * p, hi = lo + 8u;
          if (hi <= first) continue;
          if (lo >= first && hi <= last) {
            *reinterpret_cast<uint4*>(values + out0 + lo) = *reinterpret_cast<const uint4*>(sv + lo);
          } else {
            for (uint32_t k = max(lo, first); k < min(hi, last); ++k) values[out0 + k] = sv[k];
          }
        }
        // code bytes: pieces of 16 entries
        for (uint32_t p = lane; 16u * p < last; p += 64) {
          const uint32_t lo = 16u * p, hi = lo + 16u;
          if (hi <= first) continue;
          if (lo >= first && hi <= last) {
            *reinterpret_cast<uint4*>(codes8 + out0 + lo) = *reinterpret_cast<const uint4*>(sc + lo);
          } else {
            for (uint32_t k = max(lo, first); k < min(hi, last); ++k) codes8[out0 + k] = sc[k];
          }
        }
        __builtin_amdgcn_wave_barrier();
      }
      cursor += total;
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

// 8-bit values: the widened 16-bit values of the fill pass back to bytes (4 entries per thread and step)
__global__ void __launch_bounds__(256)
encode_narrow_kernel(const uint16_t* __restrict__ wide, int64_t quads, uint32_t* __restrict__ values8) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < quads; i += (int64_t)gridDim.x * blockDim.x) {
    const uint2 q = reinterpret_cast<const uint2*>(wide)[i];
    const uint32_t h[4] = {q.x & 0xFFFFu, q.x >> 16, q.y & 0xFFFFu, q.y >> 16};
    uint32_t w = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) w |= ((h[k] & 0x7Fu) | ((h[k] >> 8) & 0x80u)) << (8 * k);
    values8[i] = w;
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

// Scratch memory of the encoder (per-row counts, block sums, the code bytes), kept per
// device and reused from call to call; it only grows.  One encoder call at a time uses it.
struct Workspace {
  void* p = nullptr;
  size_t cap = 0;
  EncodeStats* pinned_stats = nullptr;   // host, pinned: the counting pass reports through it
};
std::mutex g_ws_mutex;
Workspace g_ws[64];
constexpr size_t kKeepScratchBytes = size_t{64} << 20;

hipError_t workspace_reserve(Workspace& ws, size_t bytes) {
  if (bytes <= ws.cap) return hipSuccess;
  if (ws.p) (void)hipFree(ws.p);
  ws.p = nullptr;
  ws.cap = 0;
  const size_t want = bytes + bytes / 4;             // some slack so that similar sizes do not reallocate
  hipError_t e = hipMalloc(&ws.p, want);
  if (e == hipSuccess) ws.cap = want;
  return e;
}

constexpr size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

// The handle's three arrays live in ONE allocation (*block, to be released with hipFree):
// values first, then deltas, then row_ptr, each at a multiple of 256 bytes.
int encode_on_device(const void* dense, int64_t rows, int64_t cols, int64_t ld, int b_delta, int b_val,
                     hipStream_t stream, void** block,
                     void** values, uint8_t** deltas, uint32_t** row_ptr, int64_t* nnz,
                     int64_t* pad_nnz, int64_t* alloc_nnz, int64_t* empty_rows,
                     int64_t* max_row_entries) {
  const int cus = device_cu_count();
  const bool in8 = b_val == 8;
  // 8 columns per load: 16 bytes of fp16, 8 bytes of 8-bit values
  const bool vec_ok = (ld % 8 == 0) && (reinterpret_cast<uintptr_t>(dense) & (in8 ? 7 : 15)) == 0;
  int dev = 0;
  MACKO_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return MACKO_E_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  Workspace& ws = g_ws[dev];
  if (!ws.pinned_stats) {
    void* h = nullptr;
    if (hipHostMalloc(&h, sizeof(EncodeStats), hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return MACKO_E_OUT_OF_MEMORY;
    }
    ws.pinned_stats = static_cast<EncodeStats*>(h);
  }
  // scratch layout of the counting pass
  const int64_t nblocks = (rows + 1023) / 1024;
  const size_t o_counts = 0;
  const size_t o_nnz = align_up(o_counts + 4 * (size_t)rows, 256);
  const size_t o_rowptr = align_up(o_nnz + 4 * (size_t)rows, 256);
  const size_t o_sums = align_up(o_rowptr + 256, 256);
  const size_t o_boff = align_up(o_sums + sizeof(BlockSums) * (size_t)std::max<int64_t>(nblocks, 1), 256);
  const size_t o_stats = align_up(o_boff + 8 * (size_t)std::max<int64_t>(nblocks, 1), 256);
  const size_t o_codes = align_up(o_stats + sizeof(EncodeStats), 256);
  // room for the code bytes is reserved for the expected case right away (half the cells), so
  // that the common call does not have to grow the scratch after the counting pass
  if (workspace_reserve(ws, o_codes + (size_t)rows * (size_t)cols / 2 + 4096) != hipSuccess) {
    (void)hipGetLastError();
    return MACKO_E_OUT_OF_MEMORY;
  }
  auto at = [&](size_t off) { return static_cast<unsigned char*>(ws.p) + off; };
  uint32_t* counts = reinterpret_cast<uint32_t*>(at(o_counts));
  uint32_t* nnzs = reinterpret_cast<uint32_t*>(at(o_nnz));
  uint32_t* rp_last = reinterpret_cast<uint32_t*>(at(o_rowptr));   // scratch word for the 32-bit total
  BlockSums* sums = reinterpret_cast<BlockSums*>(at(o_sums));
  unsigned long long* boff = reinterpret_cast<unsigned long long*>(at(o_boff));
  EncodeStats* stats_d = reinterpret_cast<EncodeStats*>(at(o_stats));

  const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((rows + 3) / 4, (int64_t)cus * 16));
  if (rows > 0) {
    if (in8)
      hipLaunchKernelGGL(encode_count_kernel<true>, dim3(grid), dim3(256), 0, stream, dense, (int)rows,
                         (int)cols, ld, vec_ok, b_delta, counts, nnzs);
    else
      hipLaunchKernelGGL(encode_count_kernel<false>, dim3(grid), dim3(256), 0, stream, dense, (int)rows,
                         (int)cols, ld, vec_ok, b_delta, counts, nnzs);
    hipLaunchKernelGGL(encode_block_sums_kernel, dim3((unsigned)nblocks), dim3(1024), 0, stream, counts, nnzs,
                       (int)rows, sums);
  }
  hipLaunchKernelGGL(encode_block_offsets_kernel, dim3(1), dim3(1024), 0, stream, sums, (int)nblocks, boff,
                     rp_last, stats_d);
  MACKO_HIP_TRY(hipGetLastError());
  MACKO_HIP_TRY(hipMemcpyAsync(ws.pinned_stats, stats_d, sizeof(EncodeStats), hipMemcpyDeviceToHost, stream));
  MACKO_HIP_TRY(hipStreamSynchronize(stream));
  const EncodeStats st = *ws.pinned_stats;
  if (st.pad_nnz >= (1ull << 32)) return MACKO_E_OVERFLOW;
  const int64_t pad = (int64_t)st.pad_nnz;
  const int64_t granule = alloc_granule(b_delta);
  const int64_t alloc = (pad + granule - 1) / granule * granule;
  if (alloc >= (int64_t{1} << 32)) return MACKO_E_OVERFLOW;

  // the output block; the code bytes get more scratch if the guess above was too small
  // (nothing in the old scratch but the per-row counts is needed any more, so they are
  // turned into row pointers before the scratch moves)
  const size_t b_values = 0;
  const size_t b_deltas = align_up(b_values + (size_t)alloc * (in8 ? 1 : 2), 256);
  const size_t b_rowptr = align_up(b_deltas + (size_t)alloc * b_delta / 8, 256);
  const size_t b_total = b_rowptr + 4 * (size_t)(rows + 1);
  DeviceBuf out;
  if (out.alloc(b_total) != hipSuccess) {
    (void)hipGetLastError();
    return MACKO_E_OUT_OF_MEMORY;
  }
  unsigned char* ob = static_cast<unsigned char*>(out.p);
  void* vals = ob + b_values;
  uint32_t* dels = reinterpret_cast<uint32_t*>(ob + b_deltas);
  uint32_t* rp = reinterpret_cast<uint32_t*>(ob + b_rowptr);
  if (rows > 0)
    hipLaunchKernelGGL(encode_row_ptr_kernel, dim3((unsigned)nblocks), dim3(1024), 0, stream, counts, (int)rows,
                       boff, rp, (uint32_t)pad);
  else
    MACKO_HIP_TRY(hipMemsetAsync(rp, 0, 4, stream));
  // scratch after the counts: one code byte per entry, and for 8-bit values the widened values
  const size_t o_wide = align_up(o_codes + (size_t)alloc + 256, 256);
  const size_t scratch_needed = in8 ? o_wide + 2 * (size_t)alloc + 256 : o_codes + (size_t)alloc + 256;
  if (scratch_needed > ws.cap) {
    MACKO_HIP_TRY(hipStreamSynchronize(stream));       // the launch above reads the old scratch
    if (workspace_reserve(ws, scratch_needed) != hipSuccess) {
      (void)hipGetLastError();
      return MACKO_E_OUT_OF_MEMORY;
    }
  }
  uint8_t* codes = static_cast<unsigned char*>(ws.p) + o_codes;

  if (rows > 0 && alloc > 0) {
    if (in8) {
      uint16_t* wide = reinterpret_cast<uint16_t*>(static_cast<unsigned char*>(ws.p) + o_wide);
      hipLaunchKernelGGL(encode_fill_kernel<true>, dim3(grid), dim3(64 * kFillWaves), 0, stream, dense, (int)rows,
                         (int)cols, ld, vec_ok, b_delta, static_cast<const uint32_t*>(rp), wide, codes,
                         (uint32_t)pad, (uint32_t)alloc);
      const int64_t quads = alloc / 4;                   // alloc is a multiple of 16
      const unsigned ngrid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((quads + 255) / 256, (int64_t)cus * 16));
      hipLaunchKernelGGL(encode_narrow_kernel, dim3(ngrid), dim3(256), 0, stream, static_cast<const uint16_t*>(wide),
                         quads, static_cast<uint32_t*>(vals));
    } else {
      hipLaunchKernelGGL(encode_fill_kernel<false>, dim3(grid), dim3(64 * kFillWaves), 0, stream, dense, (int)rows,
                         (int)cols, ld, vec_ok, b_delta, static_cast<const uint32_t*>(rp),
                         static_cast<uint16_t*>(vals), codes, (uint32_t)pad, (uint32_t)alloc);
    }
    const int64_t words = alloc * b_delta / 32;
    const unsigned pgrid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((words + 255) / 256, (int64_t)cus * 16));
    hipLaunchKernelGGL(encode_pack_kernel, dim3(pgrid), dim3(256), 0, stream, static_cast<const uint8_t*>(codes),
                       words, b_delta, dels);
  }
  MACKO_HIP_TRY(hipGetLastError());
  MACKO_HIP_TRY(hipStreamSynchronize(stream));
  // a large scratch buffer is not kept: after a 36864 x 12288 matrix it would hold 280 MB until the process ends
  if (ws.cap > kKeepScratchBytes) {
    (void)hipFree(ws.p);
    ws.p = nullptr;
    ws.cap = 0;
  }
  *block = out.release();
  *values = vals;
  *deltas = reinterpret_cast<uint8_t*>(dels);
  *row_ptr = rp;
  *nnz = (int64_t)st.nnz;
  *pad_nnz = pad;
  *alloc_nnz = alloc;
  *empty_rows = st.empty_rows;
  *max_row_entries = st.max_row_entries;
  return MACKO_OK;
}

}  // namespace macko
