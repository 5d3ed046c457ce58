// Small-batch product Y = W X^T for the MACKO format on gfx950: the same
// wavefront-per-row streaming kernel as the matrix-vector product (Section 4.4
// of the paper), with the decode done once per stored entry and reused for
// BT = 2, 4 or 8 activation vectors, for every code width and for 16- and 8-bit values.  The paper leaves matrix-matrix products
// with small batch dimensions as future work (Section 7); this is the natural
// extension: the streamed bytes per entry stay 2.5, the arithmetic per byte
// grows with the batch.
//
// LDS holds the activations interleaved by column: the BT values of column c
// are adjacent (2*BT bytes), so one gather address per entry fetches all of
// them with a single ds_read_b32 / b64 / b128.  Guards of zeros in front of and
// behind the columns play the same role as in the matrix-vector kernel.
#include "macko_decode.h"
#include "macko_device.h"
#include "macko_internal.h"
#include "macko_plan.h"

namespace macko {
namespace {

template <int BT> struct XVec;
template <> struct XVec<2> { using type = uint32_t; };
template <> struct XVec<4> { using type = uint2; };
template <> struct XVec<8> { using type = uint4; };

template <int BT>
__device__ __forceinline__ void unpack_x(const typename XVec<BT>::type& v, float* out);
template <>
__device__ __forceinline__ void unpack_x<2>(const uint32_t& v, float* out) {
  out[0] = f16_bits_to_f32((uint16_t)(v & 0xFFFFu));
  out[1] = f16_bits_to_f32((uint16_t)(v >> 16));
}
template <>
__device__ __forceinline__ void unpack_x<4>(const uint2& v, float* out) {
  unpack_x<2>(v.x, out);
  unpack_x<2>(v.y, out + 2);
}
template <>
__device__ __forceinline__ void unpack_x<8>(const uint4& v, float* out) {
  unpack_x<2>(v.x, out);
  unpack_x<2>(v.y, out + 2);
  unpack_x<2>(v.z, out + 4);
  unpack_x<2>(v.w, out + 6);
}

// Copy X (batch vectors of `cols` fp16, vector b at X + b*ldx) into LDS, interleaved
// by column, between zero guards of front_pad*BT and back_pad*BT bytes.  Vectors
// b >= batch are filled with zeros.  In two parts, so that the kernel can send its
// first streaming loads between them: begin() only issues the global loads of the
// thread's first 8 columns into registers; finish() writes them to LDS, copies the
// rest, clears the guards and ends with a barrier.  Both are called by every thread.
template <int BT>
struct XStageBatch {
  uint32_t u[BT][4];      // vector b, the thread's first 8 columns, two per word

  // 16-byte loads, all issued together (a vector past the batch re-reads vector 0 and is cleared)
  static __device__ __forceinline__ void load_fast(uint32_t (&u)[BT][4], const uint16_t* __restrict__ X, int64_t ldx,
                                                   int batch, int t) {
#pragma unroll
    for (int b = 0; b < BT; ++b) {
      const uint4 q = *reinterpret_cast<const uint4*>(X + (int64_t)(b < batch ? b : 0) * ldx + 8 * t);
      u[b][0] = q.x; u[b][1] = q.y; u[b][2] = q.z; u[b][3] = q.w;
    }
#pragma unroll
    for (int b = 0; b < BT; ++b)
      if (b >= batch) u[b][0] = u[b][1] = u[b][2] = u[b][3] = 0u;
  }
  static __device__ __forceinline__ void load_slow(uint32_t (&u)[BT][4], const uint16_t* __restrict__ X, int64_t ldx,
                                                   int batch, int cols, int t) {
#pragma unroll
    for (int b = 0; b < BT; ++b) {
      const uint16_t* src = X + (int64_t)b * ldx + 8 * t;
#pragma unroll
      for (int k = 0; k < 8; k += 2) {
        const uint32_t lo = (b < batch && 8 * t + k < cols) ? src[k] : 0u;
        const uint32_t hi = (b < batch && 8 * t + k + 1 < cols) ? src[k + 1] : 0u;
        u[b][k >> 1] = lo | (hi << 16);
      }
    }
  }
  // column 8t+k of vectors b, b+1 -> one word; the BT values of a column are adjacent in LDS
  static __device__ __forceinline__ void store(const uint32_t (&u)[BT][4], uint16_t* xs, int t) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      uint32_t out[BT / 2];
#pragma unroll
      for (int b = 0; b < BT; b += 2) {
        const uint32_t lo = u[b][k >> 1], hi = u[b + 1][k >> 1];
        out[b >> 1] = (k & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
      }
      unsigned char* dst = reinterpret_cast<unsigned char*>(xs + (size_t)(8 * t + k) * BT);
      if (BT == 8) *reinterpret_cast<uint4*>(dst) = make_uint4(out[0], out[1], out[2 % (BT / 2)], out[3 % (BT / 2)]);
      else if (BT == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(out[0], out[1 % (BT / 2)]);
      else *reinterpret_cast<uint32_t*>(dst) = out[0];
    }
  }

  __device__ __forceinline__ void begin(const uint16_t* __restrict__ X, int64_t ldx, int batch, int cols) {
    const int t = threadIdx.x;
    const bool vec_ok = (reinterpret_cast<uintptr_t>(X) & 15) == 0 && (ldx & 7) == 0;
    if (vec_ok && 8 * t + 8 <= cols) load_fast(u, X, ldx, batch, t);
  }

  __device__ __forceinline__ void finish(unsigned char* lds, const uint16_t* __restrict__ X, int64_t ldx, int batch,
                                         int cols, int front_pad, int back_pad) {
    const int tid = threadIdx.x, nt = blockDim.x;
    const int chunks = (cols + 7) >> 3;
    const bool vec_ok = (reinterpret_cast<uintptr_t>(X) & 15) == 0 && (ldx & 7) == 0;
    uint4* lds16 = reinterpret_cast<uint4*>(lds);
    const uint4 zero = make_uint4(0, 0, 0, 0);
    const int front16 = front_pad * BT / 16, back16 = back_pad * BT / 16, body16 = chunks * BT;   // 16-byte units
    for (int i = tid; i < front16 + back16; i += nt) lds16[i < front16 ? i : i + body16] = zero;
    uint16_t* xs = reinterpret_cast<uint16_t*>(lds + front_pad * BT);
    if (tid < chunks) {
      if (!(vec_ok && 8 * tid + 8 <= cols)) load_slow(u, X, ldx, batch, cols, tid);   // else begin() loaded it
      store(u, xs, tid);
    }
    for (int t = tid + nt; t < chunks; t += nt) {
      uint32_t v[BT][4];
      if (vec_ok && 8 * t + 8 <= cols) load_fast(v, X, ldx, batch, t);
      else load_slow(v, X, ldx, batch, cols, t);
      store(v, xs, t);
    }
    __syncthreads();
  }
};

// VB: bits per stored value (16: fp16; 8: E4M3, 4-bit codes only).
template <int BT, int BD, int VB>
__global__ void __launch_bounds__(1024)
spmm_wave_row_kernel(const void* __restrict__ values, const uint32_t* __restrict__ deltas,
                     const uint32_t* __restrict__ row_ptr, const uint16_t* __restrict__ X, int64_t ldx,
                     uint16_t* __restrict__ Y, int64_t ldy, int batch, int rows, int cols, int q, int r_extra,
                     int inv_nwaves) {
  constexpr int RING = 2;
  using XV = typename XVec<BT>::type;
  extern __shared__ __align__(16) unsigned char lds[];
  // rows dealt out evenly: q per workgroup, one more for the first r_extra; the same over the wavefronts
  const int wg = (int)blockIdx.x;
  const int row_begin = wg * q + min(wg, r_extra);
  const int wg_rows = q + (wg < r_extra ? 1 : 0);
  const int nwaves = blockDim.x >> 6;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned char* xbase = lds + front_pad_for(BD) * BT;   // LDS address of column 0
  const uint32_t lane8 = 8u * lane;
  const int per_wave = (wg_rows * inv_nwaves) >> 16;     // wg_rows / nwaves (exact for wg_rows <= 1024)
  const int extra = wg_rows - per_wave * nwaves;
  const int blk = row_begin + wave * per_wave + min(wave, extra);
  const int nb = per_wave + (wave < extra ? 1 : 0);      // at most 64: the host sees to that

  uint32_t chunk = 0;
  RowCursor ld, cp;
  LaneCodes<BD> wq[RING];
  LaneValues<VB> vq[RING];
  const int r = min(blk + lane, rows - 1);             // unconditional loads, clamped to the last row
  const uint32_t rp_lo = row_ptr[r];
  const uint32_t rp_hi = row_ptr[r + 1];
  // start-up order as in the matrix-vector kernel: row pointers and activations are requested
  // together, the first streaming loads follow, and only then are the activations written to LDS
  XStageBatch<BT> xst;
  xst.begin(X, ldx, batch, cols);

  auto issue = [&](int j) {
    if (ld.i < nb) {
      const uint32_t e0 = ld.a0 + 512u * ld.step + lane8;
      chunk = min(e0, ld.end - 1u) >> 3;
      if (++ld.step == ld.nsteps) {
        ++ld.i;
        seek_nonempty(ld, nb, rp_lo, rp_hi);
      }
    } else {
      chunk = 0;
    }
    wq[j].load(deltas, chunk);
    vq[j].load(values, chunk);
  };
  ld.i = 0;
  seek_nonempty(ld, nb, rp_lo, rp_hi);
  cp = ld;
#pragma unroll
  for (int j = 0; j < RING; ++j) issue(j);
  xst.finish(lds, X, ldx, batch, cols, front_pad_for(BD), back_pad_for(BD));    // ends with a barrier

  float yv[BT], acc[BT];
#pragma unroll
  for (int b = 0; b < BT; ++b) yv[b] = acc[b] = 0.0f;
  int base2 = 0;
  while (cp.i < nb) {
#pragma unroll
    for (int j = 0; j < RING; ++j) {
      LaneCodes<BD> w = wq[j];
      LaneValues<VB> v = vq[j];
      const bool live = cp.i < nb;
      if (!live) base2 = 0;
      const uint32_t end_eff = live ? cp.end : 0u;
      const uint32_t e0 = cp.a0 + 512u * cp.step + lane8;
      if (!live || cp.step == cp.nsteps - 1) {
        const uint32_t nv = e0 < end_eff ? end_eff - e0 : 0u;
        w.keep_if(nv != 0);
        v.keep_first(nv);
      }
      w.decode();
      const uint32_t tot = w.total();
      const uint32_t incl = wave_incl_scan_u32(tot);
      if (live && cp.step == 0) {
        base2 = 0;
        const int before = (int)(cp.start - cp.a0);
        if (before > 0) {
          base2 = -(int)w.through(before - 1);
          // lane 0 also holds the previous row's last entries: they read the zero guard, and their values
          // are cleared so that an infinity or a NaN among them cannot become a NaN of this row
          v.clear_first(lane == 0 ? (uint32_t)before : 0u);
        }
      }
      const int lanebase = base2 + (int)(incl - tot);
      // entry K: one gather address fetches the BT activations of its column
#define MACKO_ENTRY(K)                                                                       \
      {                                                                                      \
        const int q = lanebase + w.template offset<K>();     /* byte offset for one vector */ \
        const XV xraw = *reinterpret_cast<const XV*>(xbase + q * BT);                          \
        float xf[BT];                                                                        \
        unpack_x<BT>(xraw, xf);                                                              \
        const float wk = v.template get<K>();                                                \
        _Pragma("unroll") for (int b = 0; b < BT; ++b) acc[b] = fmaf(wk, xf[b], acc[b]);     \
      }
      MACKO_ENTRY(0) MACKO_ENTRY(1) MACKO_ENTRY(2) MACKO_ENTRY(3)
      MACKO_ENTRY(4) MACKO_ENTRY(5) MACKO_ENTRY(6) MACKO_ENTRY(7)
#undef MACKO_ENTRY
      issue(j);
      base2 += (int)__builtin_amdgcn_readlane((int)incl, 63);
      if (live && ++cp.step == cp.nsteps) {
        wave_sum_to_last_lane_n<BT>(acc);                // the BT sums side by side
#pragma unroll
        for (int b = 0; b < BT; ++b) {
          const int tbits = __builtin_amdgcn_readlane(__builtin_bit_cast(int, acc[b]), 63);
          yv[b] = lane == cp.i ? __builtin_bit_cast(float, tbits) : yv[b];
          acc[b] = 0.0f;
        }
        ++cp.i;
        seek_nonempty(cp, nb, rp_lo, rp_hi);
      }
    }
  }
  if (lane < nb) {
#pragma unroll
    for (int b = 0; b < BT; ++b)
      if (b < batch) Y[(int64_t)b * ldy + blk + lane] = f32_to_f16_bits(yv[b]);
  }
}

__global__ void __launch_bounds__(256) zero_Y_kernel(uint16_t* __restrict__ Y, int64_t ldy, int batch, int rows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows)
    for (int b = 0; b < batch; ++b) Y[(int64_t)b * ldy + i] = 0;
}

template <int BT, int BD, int VB = 16>
int launch_bt_bd(const SpmvProblem& p, const uint16_t* X, int64_t ldx, uint16_t* Y, int64_t ldy, int batch,
                 hipStream_t stream) {
  const int cus = device_cu_count();
  const int64_t lds = (int64_t)BT * lds_bytes_for(p.cols, BD);
  const int64_t avg = p.pad_nnz / p.rows;
  PlanInput in{p.rows, std::max<int64_t>(1, (avg + 511) / 512), lds};
  // The interleaved copy of X is BT times the size of x, so a workgroup is expensive to start:
  // one resident round (a single 16-wavefront workgroup per compute unit once the copy passes
  // 36 KB) unless the matrix is large, as for the matrix-vector kernel.
  Plan plan;
  bool planned = false;
  if (in.rows * in.steps_per_row <= (int64_t)cus * 800 || lds >= 36 * 1024)
    planned = plan_resident(plan, 1, &in, cus, 0, lds >= 36 * 1024 ? 1 : 0);
  if (!planned) {
    const int block = lds > 48 * 1024 ? 1024 : 512;
    const int64_t want = (16 + in.steps_per_row - 1) / in.steps_per_row;
    const int64_t cap = std::max<int64_t>(1, p.rows / ((int64_t)cus * 16));
    const int64_t rpw = std::min(want, cap) * (block / 64);
    plan_by_rows_per_wg(plan, 1, &in, block, &rpw);
  }
  const int block = plan.block;
  const int64_t grid = plan.total_wgs;
  if (grid >= (int64_t{1} << 31)) return MACKO_E_UNSUPPORTED;
  auto kfn = spmm_wave_row_kernel<BT, BD, VB>;
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e);
  }
  hipLaunchKernelGGL(kfn, dim3((unsigned)grid), dim3(block), (size_t)lds, stream,
                     static_cast<const void*>(p.values), reinterpret_cast<const uint32_t*>(p.deltas),
                     p.row_ptr, X, ldx, Y, ldy, batch, (int)p.rows, (int)p.cols, plan.m[0].q, plan.m[0].r,
                     65536 / (block / 64) + 1);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MACKO_OK : hip_fail(e);
}

template <int BT>
int launch_bt(const SpmvProblem& p, const uint16_t* X, int64_t ldx, uint16_t* Y, int64_t ldy, int batch,
              hipStream_t stream) {
  if (p.b_val == 8) return p.b_delta == 4 ? launch_bt_bd<BT, 4, 8>(p, X, ldx, Y, ldy, batch, stream) : MACKO_E_UNSUPPORTED;
  switch (p.b_delta) {
    case 1: return launch_bt_bd<BT, 1>(p, X, ldx, Y, ldy, batch, stream);
    case 2: return launch_bt_bd<BT, 2>(p, X, ldx, Y, ldy, batch, stream);
    case 4: return launch_bt_bd<BT, 4>(p, X, ldx, Y, ldy, batch, stream);
    case 8: return launch_bt_bd<BT, 8>(p, X, ldx, Y, ldy, batch, stream);
    default: return MACKO_E_UNSUPPORTED;
  }
}

}  // namespace

// Y[b][r] = sum over row r of W * X[b][column], b < batch.  The batch is cut into
// pieces of 8, 4, 2 or 1 vectors, each the largest that fits LDS; single vectors
// (and matrices with short rows) go through the matrix-vector path.
int launch_spmm(const SpmvProblem& p, const void* X, int64_t ldx, void* Y, int64_t ldy, int batch,
                hipStream_t stream) {
  if (p.pad_nnz > (int64_t{1} << 32) - 4096) return MACKO_E_UNSUPPORTED;   // 32-bit entry indices in the kernel
  const uint16_t* Xp = static_cast<const uint16_t*>(X);
  uint16_t* Yp = static_cast<uint16_t*>(Y);
  if (p.rows == 0 || batch == 0) return MACKO_OK;
  if (p.pad_nnz == 0) {
    hipLaunchKernelGGL(zero_Y_kernel, dim3((unsigned)((p.rows + 255) / 256)), dim3(256), 0, stream, Yp, ldy,
                       batch, (int)p.rows);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? MACKO_OK : hip_fail(e);
  }
  const int64_t one = lds_bytes_for(p.cols, p.b_delta);
  const int64_t limit = 160 * 1024 - 64;
  const bool long_rows = p.pad_nnz / p.rows >= 384;
  int done = 0;
  while (done < batch) {
    const int left = batch - done;
    const uint16_t* Xb = Xp + (int64_t)done * ldx;
    uint16_t* Yb = Yp + (int64_t)done * ldy;
    int st;
    int take;
    if (long_rows && left >= 5 && 8 * one <= limit) {
      take = std::min(left, 8);
      st = launch_bt<8>(p, Xb, ldx, Yb, ldy, take, stream);
    } else if (long_rows && left >= 3 && 4 * one <= limit) {
      take = std::min(left, 4);
      st = launch_bt<4>(p, Xb, ldx, Yb, ldy, take, stream);
    } else if (long_rows && left >= 2 && 2 * one <= limit) {
      take = 2;
      st = launch_bt<2>(p, Xb, ldx, Yb, ldy, take, stream);
    } else {
      take = long_rows ? 1 : std::min(left, kMaxGroup);
      SpmvProblem q[kMaxGroup];
      for (int i = 0; i < take; ++i) {
        q[i] = p;
        q[i].x = Xb + (int64_t)i * ldx;
        q[i].y = Yb + (int64_t)i * ldy;
      }
      st = launch_spmv_group(take, q, stream);
    }
    if (st != MACKO_OK) return st;
    done += take;
  }
  return MACKO_OK;
}

}  // namespace macko
