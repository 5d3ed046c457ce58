/*
 * Seeded synthetic input generators (weights, masks, activation vectors).
 *
 * This file holds no arithmetic of the sparse format or of the matrix-vector
 * product: it only draws numbers.  Both the CPU oracle's tests and the GPU
 * library's tests feed on what it writes, so the two sides see identical bits.
 *
 * Randomness is counter based: every draw is a pure function of
 * (seed, stream, row, counter), so results do not depend on the thread count
 * or on the order in which rows are produced.
 *
 * All matrices are fp16 bit patterns (uint16_t), row-major.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#define WL_API __attribute__((visibility("default")))

/* ---- counter-based generator ------------------------------------------- */

static inline uint64_t wl_mix(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static inline uint64_t wl_row_key(uint64_t seed, uint64_t stream, uint64_t row) {
  return wl_mix(wl_mix(wl_mix(seed) ^ (stream * 0xD6E8FEB86659FD93ull)) + row);
}

/* uniform in [0,1) with 53 random bits */
static inline double wl_uniform(uint64_t key, uint64_t ctr) {
  return (double)(wl_mix(key + ctr * 0x2545F4914F6CDD1Dull) >> 11) * (1.0 / 9007199254740992.0);
}

/* standard normal by Box-Muller from two uniforms (counters 2c and 2c+1) */
static inline double wl_normal(uint64_t key, uint64_t c) {
  double u1 = 1.0 - wl_uniform(key, 2 * c);     /* (0,1] */
  double u2 = wl_uniform(key, 2 * c + 1);
  return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

/* ---- double -> fp16 bits, round to nearest even ------------------------- */

static uint16_t wl_to_half(double v) {
  uint64_t b;
  memcpy(&b, &v, 8);
  uint16_t sign = (uint16_t)((b >> 48) & 0x8000u);
  int64_t e = (int64_t)((b >> 52) & 0x7FF) - 1023;
  uint64_t frac = b & 0xFFFFFFFFFFFFFull;
  if (((b >> 52) & 0x7FF) == 0x7FF) return (uint16_t)(sign | 0x7C00u | (frac ? 0x200u : 0));
  if (((b >> 52) & 0x7FF) == 0) return sign;               /* double subnormal -> 0 */
  uint64_t sig = frac | (1ull << 52);                      /* 1.frac, 53 bits */
  int shift;                                               /* bits to drop      */
  int64_t he;                                              /* biased half exp   */
  if (e >= -14) { he = e + 15; shift = 42; }
  else          { he = 0;      shift = (int)(42 + (-14 - e)); }
  if (shift > 63) return sign;
  uint64_t kept = sig >> shift;
  uint64_t rem = sig & ((1ull << shift) - 1);
  uint64_t half = 1ull << (shift - 1);
  if (rem > half || (rem == half && (kept & 1))) kept++;
  uint64_t out;
  if (he > 0) out = ((uint64_t)(he - 1) << 10) + kept;     /* kept carries the hidden 1 */
  else        out = kept;                                  /* subnormal (may carry into normal) */
  if (out >= 0x7C00u) out = 0x7C00u;                       /* overflow -> inf */
  return (uint16_t)(sign | (uint16_t)out);
}

/* a normal(0, sigma) value rounded to fp16, redrawn until it is not +-0 */
static inline uint16_t wl_nonzero_half(uint64_t key, uint64_t slot, double sigma) {
  for (uint64_t attempt = 0; attempt < 64; ++attempt) {
    uint16_t h = wl_to_half(sigma * wl_normal(key, slot * 64 + attempt));
    if (h & 0x7FFFu) return h;
  }
  return 0x0001u; /* unreachable in practice */
}

/* ---- exported generators ------------------------------------------------ */

/* n values ~ N(0, sigma) rounded to fp16 (zeros allowed when nonzero == 0). */
WL_API void wl_normal_f16(uint16_t* out, int64_t n, double sigma, uint64_t seed, uint64_t stream,
                          int nonzero) {
  const int64_t block = 4096;
  const int64_t nblocks = (n + block - 1) / block;
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < nblocks; ++b) {
    uint64_t key = wl_row_key(seed, stream, (uint64_t)b);
    int64_t lo = b * block, hi = lo + block < n ? lo + block : n;
    for (int64_t i = lo; i < hi; ++i) {
      uint64_t slot = (uint64_t)(i - lo);
      out[i] = nonzero ? wl_nonzero_half(key, slot, sigma)
                       : wl_to_half(sigma * wl_normal(key, slot * 64));
    }
  }
}

/*
 * Matrix whose row r keeps exactly keep[r] positions, chosen uniformly among
 * all subsets of that size (sequential selection sampling), values
 * N(0, sigma) rounded to fp16 and never +-0; every other cell is +0.
 * row0 is the global index of the first row written (so that a matrix can be
 * produced in slabs with identical content).
 */
WL_API void wl_rows_exact(uint16_t* out, int64_t rows, int64_t cols, int64_t ld,
                          const int64_t* keep, double sigma, uint64_t seed, uint64_t stream,
                          int64_t row0) {
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t r = 0; r < rows; ++r) {
    uint64_t kmask = wl_row_key(seed, stream * 2 + 0, (uint64_t)(row0 + r));
    uint64_t kval = wl_row_key(seed, stream * 2 + 1, (uint64_t)(row0 + r));
    uint16_t* dst = out + r * ld;
    int64_t need = keep[r] < 0 ? 0 : (keep[r] > cols ? cols : keep[r]);
    for (int64_t c = 0; c < cols; ++c) {
      int64_t left = cols - c;
      int take = need > 0 && wl_uniform(kmask, (uint64_t)c) * (double)left < (double)need;
      if (take) { dst[c] = wl_nonzero_half(kval, (uint64_t)c, sigma); --need; }
      else dst[c] = 0;
    }
  }
}

/* Matrix with every cell kept independently with probability density. */
WL_API void wl_bernoulli(uint16_t* out, int64_t rows, int64_t cols, int64_t ld, double density,
                         double sigma, uint64_t seed, uint64_t stream, int64_t row0) {
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t r = 0; r < rows; ++r) {
    uint64_t kmask = wl_row_key(seed, stream * 2 + 0, (uint64_t)(row0 + r));
    uint64_t kval = wl_row_key(seed, stream * 2 + 1, (uint64_t)(row0 + r));
    uint16_t* dst = out + r * ld;
    for (int64_t c = 0; c < cols; ++c) {
      int take = density >= 1.0 || wl_uniform(kmask, (uint64_t)c) < density;
      dst[c] = take ? wl_nonzero_half(kval, (uint64_t)c, sigma) : 0;
    }
  }
}

/* n uniforms in [0,1) (used for per-row sparsity draws). */
WL_API void wl_uniforms(double* out, int64_t n, uint64_t seed, uint64_t stream) {
  uint64_t key = wl_row_key(seed, stream, 0);
  for (int64_t i = 0; i < n; ++i) out[i] = wl_uniform(key, (uint64_t)i);
}
