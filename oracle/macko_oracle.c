/*
 * CPU ORACLE for the MACKO sparse format and its matrix-vector product.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or
 * call this file; it shares no code with the GPU library.  It is written to be
 * read against the paper, not to be fast: one straight loop per definition,
 * fp64 arithmetic, no blocking or reordering.
 *
 * What it follows:
 *   - the storage format of Section 4.1 (values / deltas / row_pointers,
 *     delta coding with zero padding so that every delta lies in
 *     [1, 2^b_delta], deltas packed 8/b_delta per byte),
 *   - the array tail padding to multiples of 16 bytes of Section 4.5,
 *   - the product Y = M V of Appendix A, computed from the format buffers
 *     (walk of Section 4.4: column = running sum of deltas) and, separately,
 *     from the dense matrix by the plain definition.
 *
 * Readings taken where the paper leaves a choice (all also listed in the
 * design document):
 *   - a delta in [1, 2^b] is stored as the b-bit code delta-1;
 *   - entry k sits in byte (k*b)>>3 at bit (k*b)&7 (little-endian fields);
 *   - the delta of the first entry of a row is measured from column -1
 *     (0-based), i.e. equals its 1-based column, as in the worked example of
 *     Section 4.1 (first value in 1-based column 2 has delta 2);
 *   - padding entries are placed greedily at the farthest reachable column
 *     (the worked example pads column 9 = 5 + 4 with 2-bit deltas), hold the
 *     value +0 and therefore the code 2^b - 1;
 *   - an element whose fp16 bit pattern is +0 or -0 is a zero; everything else
 *     (subnormals, infinities, NaNs) is kept;
 *   - nothing is stored after the last non-zero of a row;
 *   - row_pointers are 32-bit entry indices, R+1 of them;
 *   - both arrays are zero-filled up to alloc_nnz = pad_nnz rounded up to a
 *     multiple of 128/b_delta entries (16 bytes of deltas; values then are a
 *     multiple of 16 bytes too).
 *
 * Parity pins (tests/test_oracle_*.py): the worked example of Section 4.1,
 * eqs. 8-10, exact round trip, brute force over all masks of a short row,
 * numpy's fp16 conversion and fp64 matmul.  The 8-bit-value functions at the
 * end are pinned by tests/test_oracle_fp8.py (the 256 values against their
 * closed form and a library conversion, the coordinates against the pinned
 * 16-bit encoder, round trip, numpy fp64 matmul).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_API __attribute__((visibility("default")))

/* ---- fp16 <-> fp64 by bit manipulation (exact / round-to-nearest-even) --- */

static double oracle_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int exp = (h >> 10) & 0x1F;
  int frac = h & 0x3FF;
  double v;
  if (exp == 0)        v = ldexp((double)frac, -24);               /* zero / subnormal */
  else if (exp == 31)  v = frac ? NAN : INFINITY;
  else                 v = ldexp((double)(frac + 1024), exp - 25); /* 1.frac * 2^(exp-15) */
  return sign ? -v : v;
}

static uint16_t oracle_double_to_half(double v) {
  uint16_t sign = signbit(v) ? 0x8000u : 0;
  double a = fabs(v);
  if (isnan(v)) return (uint16_t)(sign | 0x7E00u);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u);  /* >= max + half ulp rounds to inf */
  if (a < ldexp(1.0, -14)) {
    /* subnormal range: multiples of 2^-24; nearbyint rounds to nearest even */
    double q = nearbyint(ldexp(a, 24));
    return (uint16_t)(sign | (uint16_t)q);              /* q == 1024 is the smallest normal */
  }
  int e;
  double m = frexp(a, &e);                              /* a = m * 2^e, m in [0.5,1) */
  double q = nearbyint(ldexp(m, 11));                   /* 11-bit significand, in [1024, 2048] */
  if (q == 2048.0) { q = 1024.0; e += 1; }
  int he = e - 1 + 15;
  if (he >= 31) return (uint16_t)(sign | 0x7C00u);
  return (uint16_t)(sign | (he << 10) | ((int)q - 1024));
}

ORACLE_API void oracle_half_to_double_array(const uint16_t* in, double* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = oracle_half_to_double(in[i]);
}

ORACLE_API void oracle_double_to_half_array(const double* in, uint16_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = oracle_double_to_half(in[i]);
}

/* ---- packed b-bit codes --------------------------------------------------- */

static inline unsigned oracle_get_code(const uint8_t* deltas, int64_t k, int b) {
  int64_t bit = k * b;
  return (deltas[bit >> 3] >> (bit & 7)) & ((1u << b) - 1u);
}

static inline void oracle_put_code(uint8_t* deltas, int64_t k, int b, unsigned code) {
  int64_t bit = k * b;
  deltas[bit >> 3] |= (uint8_t)(code << (bit & 7));
}

static int oracle_valid_b(int b) { return b == 1 || b == 2 || b == 4 || b == 8; }

/* entries per 16 bytes of deltas */
ORACLE_API int64_t oracle_alloc_granule(int b_delta) { return 128 / b_delta; }

/* ---- encoder (Section 4.1) ----------------------------------------------- */

/*
 * Number of stored entries (non-zeros plus padding) of the whole matrix;
 * *nnz_out receives the number of non-zeros.  Returns -1 on bad arguments.
 */
ORACLE_API int64_t oracle_count_entries(const uint16_t* dense, int64_t R, int64_t C, int64_t ld,
                                        int b_delta, int64_t* nnz_out) {
  if (!oracle_valid_b(b_delta) || R < 0 || C < 0 || ld < C) return -1;
  const int64_t D = (int64_t)1 << b_delta;
  int64_t e = 0, nnz = 0;
  for (int64_t r = 0; r < R; ++r) {
    int64_t prev = -1;
    for (int64_t c = 0; c < C; ++c) {
      if ((dense[r * ld + c] & 0x7FFFu) == 0) continue;
      int64_t gap = c - prev;
      while (gap > D) { ++e; prev += D; gap -= D; }
      ++e; ++nnz; prev = c;
    }
  }
  if (nnz_out) *nnz_out = nnz;
  return e;
}

/*
 * Encode.  values must hold alloc_nnz fp16 slots, deltas alloc_nnz*b_delta/8
 * bytes, row_ptr R+1 slots, where alloc_nnz = pad_nnz rounded up to a multiple
 * of oracle_alloc_granule(b_delta) and pad_nnz = oracle_count_entries(...).
 * Returns pad_nnz, or -1 on bad arguments, or -2 if an index exceeds 32 bits.
 */
ORACLE_API int64_t oracle_encode(const uint16_t* dense, int64_t R, int64_t C, int64_t ld,
                                 int b_delta, uint16_t* values, uint8_t* deltas,
                                 uint32_t* row_ptr, int64_t alloc_nnz) {
  if (!oracle_valid_b(b_delta) || R < 0 || C < 0 || ld < C) return -1;
  if (alloc_nnz >= ((int64_t)1 << 32)) return -2;
  const int64_t D = (int64_t)1 << b_delta;
  memset(values, 0, (size_t)alloc_nnz * 2);
  memset(deltas, 0, (size_t)(alloc_nnz * b_delta / 8));
  int64_t e = 0;
  row_ptr[0] = 0;
  for (int64_t r = 0; r < R; ++r) {
    int64_t prev = -1;                       /* column of the previous stored entry */
    for (int64_t c = 0; c < C; ++c) {
      uint16_t w = dense[r * ld + c];
      if ((w & 0x7FFFu) == 0) continue;      /* +0 and -0 are zeros */
      int64_t gap = c - prev;
      while (gap > D) {                      /* padding entry at column prev + D */
        if (e >= alloc_nnz) return -1;
        values[e] = 0;
        oracle_put_code(deltas, e, b_delta, (unsigned)(D - 1));
        ++e; prev += D; gap -= D;
      }
      if (e >= alloc_nnz) return -1;
      values[e] = w;
      oracle_put_code(deltas, e, b_delta, (unsigned)(gap - 1));
      ++e; prev = c;
    }
    row_ptr[r + 1] = (uint32_t)e;
  }
  return e;
}

/* ---- decoder: format -> dense (lossless, Section 5.2) --------------------- */

/* Returns 0, or -(r+1) if row r decodes to a column >= C. */
ORACLE_API int64_t oracle_decode(const uint16_t* values, const uint8_t* deltas,
                                 const uint32_t* row_ptr, int64_t R, int64_t C, int b_delta,
                                 uint16_t* dense, int64_t ld) {
  for (int64_t r = 0; r < R; ++r) memset(dense + r * ld, 0, (size_t)C * 2);
  for (int64_t r = 0; r < R; ++r) {
    int64_t col = -1;
    for (int64_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
      col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;
      if (col >= C) return -(r + 1);
      dense[r * ld + col] = values[k];
    }
  }
  return 0;
}

/* Unpacked view of the coordinates: delta[k] = code+1 and absolute column. */
ORACLE_API void oracle_unpack(const uint8_t* deltas, const uint32_t* row_ptr, int64_t R,
                              int b_delta, int32_t* delta_out, int32_t* col_out) {
  for (int64_t r = 0; r < R; ++r) {
    int64_t col = -1;
    for (int64_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
      int d = (int)oracle_get_code(deltas, k, b_delta) + 1;
      col += d;
      if (delta_out) delta_out[k] = d;
      if (col_out) col_out[k] = (int32_t)col;
    }
  }
}

/*
 * Structural invariants of a well-formed encoding.  Returns 0 when all hold,
 * otherwise a positive code naming the first violated one:
 *  1 row_ptr[0] != 0            2 row_ptr not non-decreasing
 *  3 row_ptr[R] > alloc_nnz     4 a row decodes to a column >= C
 *  5 a zero-valued entry whose code is not 2^b-1 (padding must use the full step)
 *  6 a zero-valued entry that is the last of its row
 *  7 non-zero bytes in the tail [pad_nnz, alloc_nnz)
 *  8 alloc_nnz is not pad_nnz rounded up to the granule
 */
ORACLE_API int oracle_check(const uint16_t* values, const uint8_t* deltas, const uint32_t* row_ptr,
                            int64_t R, int64_t C, int b_delta, int64_t alloc_nnz) {
  const unsigned full = (1u << b_delta) - 1u;
  if (row_ptr[0] != 0) return 1;
  for (int64_t r = 0; r < R; ++r) if (row_ptr[r + 1] < row_ptr[r]) return 2;
  int64_t pad_nnz = row_ptr[R];
  if (pad_nnz > alloc_nnz) return 3;
  int64_t g = oracle_alloc_granule(b_delta);
  if (alloc_nnz != (pad_nnz + g - 1) / g * g) return 8;
  for (int64_t r = 0; r < R; ++r) {
    int64_t col = -1;
    for (int64_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
      unsigned code = oracle_get_code(deltas, k, b_delta);
      col += (int64_t)code + 1;
      if (col >= C) return 4;
      if ((values[k] & 0x7FFFu) == 0) {
        if (values[k] != 0 || code != full) return 5;
        if (k + 1 == row_ptr[r + 1]) return 6;
      }
    }
  }
  for (int64_t k = pad_nnz; k < alloc_nnz; ++k) {
    if (values[k] != 0 || oracle_get_code(deltas, k, b_delta) != 0) return 7;
  }
  return 0;
}

/* ---- the product, from the format (Section 4.4 walk, fp64) ---------------- */

/*
 * y64[r] = sum over the row's entries, in storage order, of value * x[column].
 * abs64[r] (optional) = sum of |value * x[column]|, the scale of the
 * acceptance tolerance.  Padding entries contribute 0 * x[column].
 */
ORACLE_API void oracle_spmv(const uint16_t* values, const uint8_t* deltas, const uint32_t* row_ptr,
                            int64_t R, int64_t C, int b_delta, const uint16_t* x,
                            double* y64, double* abs64) {
  (void)C;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t r = 0; r < R; ++r) {
    double acc = 0.0, mag = 0.0;
    int64_t col = -1;
    for (int64_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
      col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;
      double p = oracle_half_to_double(values[k]) * oracle_half_to_double(x[col]);
      acc += p;
      mag += fabs(p);
    }
    y64[r] = acc;
    if (abs64) abs64[r] = mag;
  }
}

/* ---- the product, by definition from the dense matrix (Appendix A) -------- */

ORACLE_API void oracle_dense_matvec(const uint16_t* dense, int64_t R, int64_t C, int64_t ld,
                                    const uint16_t* x, double* y64, double* abs64) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    double acc = 0.0, mag = 0.0;
    for (int64_t c = 0; c < C; ++c) {
      double p = oracle_half_to_double(dense[r * ld + c]) * oracle_half_to_double(x[c]);
      acc += p;
      mag += fabs(p);
    }
    y64[r] = acc;
    if (abs64) abs64[r] = mag;
  }
}

/* ==========================================================================
 * 8-bit values.  The paper names b_val = 8 as a setting the format covers and
 * leaves its kernel to future work (Section 6, "Limitations"; Section 7); it
 * does not say what an 8-bit value is.  Reading taken here and in the library:
 * the OCP 8-bit floating point format E4M3 (1 sign, 4 exponent bits with bias
 * 7, 3 fraction bits; exponent 0 holds zero and the subnormals f * 2^-9; there
 * are no infinities, and exponent 15 with fraction 7 is the only NaN, so the
 * largest finite value is 1.75 * 2^8 = 448).  The format itself does not
 * change: values holds one byte per stored entry, a padding entry holds +0
 * (0x00), an element is a zero when its bits other than the sign are 0, and
 * the coordinates, the row pointers and the tail padding (alloc_nnz = pad_nnz
 * rounded up to 128 / b_delta entries) are exactly those of the 16-bit case.
 * x and y stay fp16 and the product is still sum_j w_ij * x_j.
 * ========================================================================== */

static double oracle_fp8_to_double(uint8_t b) {
  int sign = (b >> 7) & 1;
  int exp = (b >> 3) & 0xF;
  int frac = b & 7;
  double v;
  if (exp == 0)                      v = ldexp((double)frac, -9);            /* zero / subnormal */
  else if (exp == 15 && frac == 7)   v = NAN;
  else                               v = ldexp((double)(frac + 8), exp - 10); /* 1.frac * 2^(exp-7) */
  return sign ? -v : v;
}

ORACLE_API void oracle_fp8_to_double_array(const uint8_t* in, double* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = oracle_fp8_to_double(in[i]);
}

ORACLE_API int64_t oracle_count_entries8(const uint8_t* dense, int64_t R, int64_t C, int64_t ld,
                                         int b_delta, int64_t* nnz_out) {
  if (!oracle_valid_b(b_delta) || R < 0 || C < 0 || ld < C) return -1;
  const int64_t D = (int64_t)1 << b_delta;
  int64_t e = 0, nnz = 0;
  for (int64_t r = 0; r < R; ++r) {
    int64_t prev = -1;
    for (int64_t c = 0; c < C; ++c) {
      if ((dense[r * ld + c] & 0x7Fu) == 0) continue;
      int64_t gap = c - prev;
      while (gap > D) { ++e; prev += D; gap -= D; }
      ++e; ++nnz; prev = c;
    }
  }
  if (nnz_out) *nnz_out = nnz;
  return e;
}

/* As oracle_encode, with one byte per value. */
ORACLE_API int64_t oracle_encode8(const uint8_t* dense, int64_t R, int64_t C, int64_t ld,
                                  int b_delta, uint8_t* values, uint8_t* deltas,
                                  uint32_t* row_ptr, int64_t alloc_nnz) {
  if (!oracle_valid_b(b_delta) || R < 0 || C < 0 || ld < C) return -1;
  if (alloc_nnz >= ((int64_t)1 << 32)) return -2;
  const int64_t D = (int64_t)1 << b_delta;
  memset(values, 0, (size_t)alloc_nnz);
  memset(deltas, 0, (size_t)(alloc_nnz * b_delta / 8));
  int64_t e = 0;
  row_ptr[0] = 0;
  for (int64_t r = 0; r < R; ++r) {
    int64_t prev = -1;
    for (int64_t c = 0; c < C; ++c) {
      uint8_t w = dense[r * ld + c];
      if ((w & 0x7Fu) == 0) continue;          /* +0 and -0 are zeros */
      int64_t gap = c - prev;
      while (gap > D) {                        /* padding entry at column prev + D */
        if (e >= alloc_nnz) return -1;
        values[e] = 0;
        oracle_put_code(deltas, e, b_delta, (unsigned)(D - 1));
        ++e; prev += D; gap -= D;
      }
      if (e >= alloc_nnz) return -1;
      values[e] = w;
      oracle_put_code(deltas, e, b_delta, (unsigned)(gap - 1));
      ++e; prev = c;
    }
    row_ptr[r + 1] = (uint32_t)e;
  }
  return e;
}

ORACLE_API int64_t oracle_decode8(const uint8_t* values, const uint8_t* deltas,
                                  const uint32_t* row_ptr, int64_t R, int64_t C, int b_delta,
                                  uint8_t* dense, int64_t ld) {
  for (int64_t r = 0; r < R; ++r) memset(dense + r * ld, 0, (size_t)C);
  for (int64_t r = 0; r < R; ++r) {
    int64_t col = -1;
    for (int64_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
      col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;
      if (col >= C) return -(r + 1);
      dense[r * ld + col] = values[k];
    }
  }
  return 0;
}

ORACLE_API void oracle_spmv8(const uint8_t* values, const uint8_t* deltas, const uint32_t* row_ptr,
                             int64_t R, int64_t C, int b_delta, const uint16_t* x,
                             double* y64, double* abs64) {
  (void)C;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t r = 0; r < R; ++r) {
    double acc = 0.0, mag = 0.0;
    int64_t col = -1;
    for (int64_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
      col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;
      double p = oracle_fp8_to_double(values[k]) * oracle_half_to_double(x[col]);
      acc += p;
      mag += fabs(p);
    }
    y64[r] = acc;
    if (abs64) abs64[r] = mag;
  }
}

ORACLE_API void oracle_dense_matvec8(const uint8_t* dense, int64_t R, int64_t C, int64_t ld,
                                     const uint16_t* x, double* y64, double* abs64) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    double acc = 0.0, mag = 0.0;
    for (int64_t c = 0; c < C; ++c) {
      double p = oracle_fp8_to_double(dense[r * ld + c]) * oracle_half_to_double(x[c]);
      acc += p;
      mag += fabs(p);
    }
    y64[r] = acc;
    if (abs64) abs64[r] = mag;
  }
}

ORACLE_API int oracle_max_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}

ORACLE_API void oracle_set_threads(int n) {
#ifdef _OPENMP
  extern void omp_set_num_threads(int);
  omp_set_num_threads(n);
#else
  (void)n;
#endif
}
