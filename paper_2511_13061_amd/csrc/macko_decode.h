// In-register decode of the packed column codes, shared by the matrix-vector
// and the small-batch kernels.
#pragma once

#include "macko_device.h"

namespace macko {

// ---------------------------------------------------------------------------
// Codes of a lane's 8 consecutive entries and the positions they decode to, for
// code widths of 1, 2, 4 and 8 bits (the product kernels use 2, 4 and 8).  All positions are doubled (bytes of the LDS
// copy of x) and include the +1 per entry, i.e. entry k advances by 2 code + 2.
//   load(deltas, chunk)  the 2 / 4 / 8 bytes of chunk `chunk` (8 entries)
//   clear()              all codes 0 (every entry one column after the other)
//   decode()             prefix sums inside the lane
//   total()              doubled sum of the lane's 8 deltas
//   offset<K>()          doubled position of entry K relative to the lane's start, minus 2
//                        (= byte offset of its column in x when the lane starts at column 0)
//   through(k, l)        lane l's doubled position after its entry k (k and l wavefront-uniform)
// ---------------------------------------------------------------------------
template <int BD>
struct LaneCodes;

// 2- and 4-bit codes: the eight doubled prefixes are at most 2*15*8 = 240 and fit
// the bytes of two words; the constant part 2K of entry K is added bytewise.
template <int BD>
struct LaneCodesBytes {
  uint32_t w;           // packed codes as loaded
  uint32_t P, E;        // byte m: doubled code prefix through entry 2m+1 / 2m
  uint32_t P2, E2;      // the same plus the constant part: doubled position of the entry, minus 2
  __device__ __forceinline__ void clear() { w = 0u; }
  __device__ __forceinline__ void keep_if(bool c) { w = c ? w : 0u; }
  __device__ __forceinline__ void decode() {
    uint32_t lo2, hi2;                                 // doubled codes of even / odd entries, one per byte
    if (BD == 4) {
      lo2 = (w << 1) & 0x1E1E1E1Eu;
      hi2 = (w >> 3) & 0x1E1E1E1Eu;
    } else {                                           // 2-bit codes: one nibble per pair of entries
      uint32_t t = w & 0xFFFFu;
      t = (t | (t << 8)) & 0x00FF00FFu;
      t = (t | (t << 4)) & 0x0F0F0F0Fu;                // byte m: codes of entries 2m (bits 0-1) and 2m+1 (bits 2-3)
      lo2 = (t << 1) & 0x06060606u;
      hi2 = (t >> 1) & 0x06060606u;
    }
    P = lo2 + hi2;                                     // pair sums
    P = lshl_add<8>(P, P);
    P = lshl_add<16>(P, P);
    E = lshl_add<8>(P, lo2);
    E2 = E + 0x0C080400u;                              // the largest byte, 240 + 14, still fits
    P2 = P + 0x0E0A0602u;
  }
  __device__ __forceinline__ uint32_t total() const { return (P >> 24) + 16u; }
  template <int K>
  __device__ __forceinline__ int offset() const {
    return (int)((((K & 1) ? P2 : E2) >> (8 * (K >> 1))) & 0xFFu);
  }
  __device__ __forceinline__ uint32_t through(int k, int l = 0) const {
    const uint32_t src = (uint32_t)__builtin_amdgcn_readlane((int)((k & 1) ? P : E), l);
    return ((src >> (8 * (k >> 1))) & 0xFFu) + 2u * (uint32_t)(k + 1);
  }
};
template <>
struct LaneCodes<4> : LaneCodesBytes<4> {
  __device__ __forceinline__ void load(const uint32_t* __restrict__ deltas, uint32_t chunk) { w = load_stream(deltas + chunk); }
};
template <>
struct LaneCodes<2> : LaneCodesBytes<2> {
  __device__ __forceinline__ void load(const uint32_t* __restrict__ deltas, uint32_t chunk) {
    w = load_stream(reinterpret_cast<const uint16_t*>(deltas) + chunk);
  }
};

// 1-bit codes: a prefix is a population count of the low bits.
template <>
struct LaneCodes<1> {
  uint32_t w;           // the 8 codes, entry k in bit k
  __device__ __forceinline__ void load(const uint32_t* __restrict__ deltas, uint32_t chunk) {
    w = load_stream(reinterpret_cast<const uint8_t*>(deltas) + chunk);
  }
  __device__ __forceinline__ void clear() { w = 0u; }
  __device__ __forceinline__ void keep_if(bool c) { w = c ? w : 0u; }
  __device__ __forceinline__ void decode() {}
  __device__ __forceinline__ uint32_t total() const { return 2u * (uint32_t)__builtin_popcount(w) + 16u; }
  template <int K>
  __device__ __forceinline__ int offset() const {
    return 2 * __builtin_popcount(w & ((2u << K) - 1u)) + 2 * K;
  }
  __device__ __forceinline__ uint32_t through(int k, int l = 0) const {
    const uint32_t s = (uint32_t)__builtin_amdgcn_readlane((int)w, l);
    return 2u * (uint32_t)__builtin_popcount(s & ((2u << k) - 1u)) + 2u * (uint32_t)(k + 1);
  }
};

// 8-bit codes: prefixes reach 8 * 512 = 4096 and are kept as 16-bit halves of four words.
template <>
struct LaneCodes<8> {
  uint32_t w0, w1;      // codes of entries 0..3 and 4..7, one per byte
  // halves of Xi: doubled position after entry 2i and after entry 2i+1 (four named
  // registers: an array indexed by a run-time value would be put in scratch memory)
  uint32_t X0, X1, X2, X3;
  uint32_t tot;
  __device__ __forceinline__ void load(const uint32_t* __restrict__ deltas, uint32_t chunk) {
    const uint2 v = load_stream(reinterpret_cast<const uint2*>(deltas) + chunk);
    w0 = v.x;
    w1 = v.y;
  }
  __device__ __forceinline__ void clear() { w0 = w1 = 0u; }
  __device__ __forceinline__ void keep_if(bool c) {
    w0 = c ? w0 : 0u;
    w1 = c ? w1 : 0u;
  }
  // bytes (c_a, c_b) of w -> halves holding 2c + 2, then low half: the first entry alone, high half: the pair
  static __device__ __forceinline__ uint32_t pair(uint32_t w, uint32_t sel) {
    const uint32_t y = (__builtin_amdgcn_perm(0u, w, sel) << 1) + 0x00020002u;
    return lshl_add<16>(y, y);
  }
  __device__ __forceinline__ void decode() {
    const uint32_t Y0 = pair(w0, 0x0C010C00u), Y1 = pair(w0, 0x0C030C02u);
    const uint32_t Y2 = pair(w1, 0x0C010C00u), Y3 = pair(w1, 0x0C030C02u);
    const uint32_t r1 = Y0 >> 16;
    const uint32_t r2 = r1 + (Y1 >> 16);
    const uint32_t r3 = r2 + (Y2 >> 16);
    tot = r3 + (Y3 >> 16);
    X0 = Y0;
    X1 = Y1 + (r1 | (r1 << 16));
    X2 = Y2 + (r2 | (r2 << 16));
    X3 = Y3 + (r3 | (r3 << 16));
  }
  __device__ __forceinline__ uint32_t total() const { return tot; }
  template <int K>
  __device__ __forceinline__ int offset() const {
    const uint32_t x = (K >> 1) == 0 ? X0 : ((K >> 1) == 1 ? X1 : ((K >> 1) == 2 ? X2 : X3));
    return (int)((K & 1) ? (x >> 16) : (x & 0xFFFFu)) - 2;
  }
  __device__ __forceinline__ uint32_t through(int k, int l = 0) const {
    // lane l's four words as scalars, then a scalar choice
    const uint32_t s0 = (uint32_t)__builtin_amdgcn_readlane((int)X0, l), s1 = (uint32_t)__builtin_amdgcn_readlane((int)X1, l);
    const uint32_t s2 = (uint32_t)__builtin_amdgcn_readlane((int)X2, l), s3 = (uint32_t)__builtin_amdgcn_readlane((int)X3, l);
    const int i = k >> 1;
    const uint32_t src = i == 0 ? s0 : (i == 1 ? s1 : (i == 2 ? s2 : s3));
    return (k & 1) ? (src >> 16) : (src & 0xFFFFu);
  }
};

// The 8 values of a lane's chunk, 16 or 8 bits each.  16-bit values are fp16 and feed
// v_fma_mix_f32 directly; 8-bit values are OCP E4M3 numbers, converted two at a time
// with the hardware conversion (v_cvt_pk_f32_fp8).
template <int VB>
struct LaneValues;
template <>
struct LaneValues<16> {
  uint4 v;
  __device__ __forceinline__ void load(const void* __restrict__ values, uint32_t chunk) {
    v = load_stream(static_cast<const uint4*>(values) + chunk);
  }
  __device__ __forceinline__ void keep_first(uint32_t nv) {       // clear the values of entries nv, nv+1, ...
    v.x &= nv >= 2 ? 0xFFFFFFFFu : (nv == 1 ? 0xFFFFu : 0u);
    v.y &= nv >= 4 ? 0xFFFFFFFFu : (nv == 3 ? 0xFFFFu : 0u);
    v.z &= nv >= 6 ? 0xFFFFFFFFu : (nv == 5 ? 0xFFFFu : 0u);
    v.w &= nv >= 8 ? 0xFFFFFFFFu : (nv == 7 ? 0xFFFFu : 0u);
  }
  __device__ __forceinline__ void clear_first(uint32_t n) {       // clear the values of entries 0 .. n-1 (n <= 7)
    v.x &= n >= 2 ? 0u : (n == 1 ? 0xFFFF0000u : 0xFFFFFFFFu);
    v.y &= n >= 4 ? 0u : (n == 3 ? 0xFFFF0000u : 0xFFFFFFFFu);
    v.z &= n >= 6 ? 0u : (n == 5 ? 0xFFFF0000u : 0xFFFFFFFFu);
    v.w &= n == 7 ? 0xFFFF0000u : 0xFFFFFFFFu;
  }
  template <int K>
  __device__ __forceinline__ uint32_t bits() const {              // the stored bit pattern of entry K
    const uint32_t w = (K >> 1) == 0 ? v.x : ((K >> 1) == 1 ? v.y : ((K >> 1) == 2 ? v.z : v.w));
    return (K & 1) ? (w >> 16) : (w & 0xFFFFu);
  }
  template <int K>
  __device__ __forceinline__ float get() const {
    return f16_bits_to_f32((uint16_t)bits<K>());
  }
};
template <>
struct LaneValues<8> {
  uint2 v;
  __device__ __forceinline__ void load(const void* __restrict__ values, uint32_t chunk) {
    v = load_stream(static_cast<const uint2*>(values) + chunk);
  }
  __device__ __forceinline__ void keep_first(uint32_t nv) {
    const uint32_t lo = nv >= 4 ? 4u : nv, hi = nv >= 8 ? 4u : (nv > 4 ? nv - 4u : 0u);
    v.x &= lo == 4 ? 0xFFFFFFFFu : ((1u << (8u * lo)) - 1u);
    v.y &= hi == 4 ? 0xFFFFFFFFu : ((1u << (8u * hi)) - 1u);
  }
  __device__ __forceinline__ void clear_first(uint32_t n) {       // n <= 7
    const uint32_t lo = n >= 4 ? 4u : n, hi = n > 4 ? n - 4u : 0u;
    v.x &= lo == 4 ? 0u : ~((1u << (8u * lo)) - 1u);
    v.y &= ~((1u << (8u * hi)) - 1u);
  }
  template <int K>
  __device__ __forceinline__ uint32_t bits() const {
    return ((K < 4 ? v.x : v.y) >> (8 * (K & 3))) & 0xFFu;
  }
  template <int K>
  __device__ __forceinline__ float get() const {
    typedef float float2v __attribute__((ext_vector_type(2)));
    const float2v p = __builtin_amdgcn_cvt_pk_f32_fp8((int)(K < 4 ? v.x : v.y), (K & 2) != 0);
    return (K & 1) ? p.y : p.x;
  }
};


}  // namespace macko
