// Host code of libmacko under AddressSanitizer and UndefinedBehaviorSanitizer: the encoders for
// every code width and both value widths, the decoders, the storage report and the argument
// checks, on random, ragged, strided, empty and degenerate shapes, and the overflow of the 32-bit
// row pointers (Section 4.1: 32 bits per row pointer).  The encodings are checked here only for
// self-consistency (round trip, pointer arithmetic, byte counts); bit-exactness against the oracle
// is the job of tests/test_library_host.py.  Built and run by that file; prints "ok" on success.
#include <sys/mman.h>

#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>
#include <vector>

#include "macko.h"

static int failures = 0;
#define EXPECT(cond, ...)                                                                     \
  do {                                                                                        \
    if (!(cond)) {                                                                            \
      if (failures < 20) { std::printf("FAIL %s: ", #cond); std::printf(__VA_ARGS__); std::printf("\n"); } \
      ++failures;                                                                             \
    }                                                                                         \
  } while (0)

template <class T>
static std::vector<T> random_matrix(int64_t rows, int64_t cols, int64_t ld, double density, std::mt19937_64& rng, T fill) {
  std::vector<T> W((size_t)(rows * ld), fill);                 // cells between cols and ld hold `fill`: they must be ignored
  std::uniform_real_distribution<double> u(0.0, 1.0);
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      T v = 0;
      if (u(rng) < density) {
        v = (T)(rng() & (sizeof(T) == 2 ? 0xFFFFu : 0xFFu));
        if ((v & (T)(sizeof(T) == 2 ? 0x7FFF : 0x7F)) == 0) v = 1;
      } else if (rng() % 16 == 0) {
        v = (T)(sizeof(T) == 2 ? 0x8000 : 0x80);               // -0 is a zero
      }
      W[(size_t)(r * ld + c)] = v;
    }
  return W;
}

static void check16(int64_t rows, int64_t cols, int64_t ld, double density, int b_delta, std::mt19937_64& rng) {
  std::vector<uint16_t> W = random_matrix<uint16_t>(rows, cols, ld, density, rng, (uint16_t)0x3C00);
  if (rows > 2) for (int64_t c = 0; c < cols; ++c) W[(size_t)(1 * ld + c)] = 0;      // an empty row
  macko_handle_t h = nullptr;
  macko_report_t rep;
  const int st = macko_encode_ex(W.data(), rows, cols, ld, b_delta, &h, &rep);
  EXPECT(st == MACKO_OK && h, "encode %lldx%lld b %d: %d", (long long)rows, (long long)cols, b_delta, st);
  if (st != MACKO_OK) return;
  const uint16_t* v;
  const uint8_t* d;
  const uint32_t* rp;
  EXPECT(macko_host_buffers(h, &v, &d, &rp) == MACKO_OK, "host buffers");
  EXPECT(rp[0] == 0 && (int64_t)rp[rows] == rep.pad_nnz, "row pointers");
  const int64_t granule = 128 / b_delta;
  EXPECT(rep.alloc_nnz % granule == 0 && rep.alloc_nnz >= rep.pad_nnz && rep.alloc_nnz - rep.pad_nnz < granule, "alloc");
  EXPECT(rep.values_bytes == 2 * rep.alloc_nnz && rep.deltas_bytes == rep.alloc_nnz * b_delta / 8 &&
             rep.rowptr_bytes == 4 * (rows + 1) && rep.total_bytes == rep.values_bytes + rep.deltas_bytes + rep.rowptr_bytes,
         "byte counts");
  // walk the whole arrays (every byte of values and deltas is read), rebuild the matrix by hand
  std::vector<uint16_t> back((size_t)(rows * cols), 0);
  int64_t nnz = 0;
  for (int64_t r = 0; r < rows; ++r) {
    int64_t col = -1;
    for (int64_t k = rp[r]; k < rp[r + 1]; ++k) {
      const unsigned code = (d[(k * b_delta) >> 3] >> ((k * b_delta) & 7)) & ((1u << b_delta) - 1u);
      col += code + 1;
      EXPECT(col < cols, "column %lld of %lld", (long long)col, (long long)cols);
      if (col < cols) back[(size_t)(r * cols + col)] = v[k];
      nnz += (v[k] & 0x7FFF) != 0;
    }
  }
  for (int64_t k = rep.pad_nnz; k < rep.alloc_nnz; ++k) EXPECT(v[k] == 0, "tail value");
  EXPECT(nnz == rep.nnz, "nnz %lld != %lld", (long long)nnz, (long long)rep.nnz);
  std::vector<uint16_t> dec((size_t)(rows * (cols + 3)), 0xABCD);
  EXPECT(macko_decode(h, dec.data(), cols + 3) == MACKO_OK, "decode");
  bool same = true, kept = true;
  for (int64_t r = 0; r < rows; ++r) {
    for (int64_t c = 0; c < cols; ++c) {
      const uint16_t in = W[(size_t)(r * ld + c)];
      const uint16_t want = (in & 0x7FFF) ? in : 0;
      same = same && dec[(size_t)(r * (cols + 3) + c)] == want && back[(size_t)(r * cols + c)] == want;
    }
    for (int64_t c = cols; c < cols + 3; ++c) kept = kept && dec[(size_t)(r * (cols + 3) + c)] == 0xABCD;
  }
  EXPECT(same, "round trip %lldx%lld ld %lld b %d", (long long)rows, (long long)cols, (long long)ld, b_delta);
  EXPECT(kept, "decode wrote between cols and ld");
  int64_t by_width[4];
  int best = -1;
  EXPECT(macko_storage_by_code_width(W.data(), rows, cols, ld, by_width, &best) == MACKO_OK, "storage by width");
  const int idx = b_delta == 1 ? 0 : b_delta == 2 ? 1 : b_delta == 4 ? 2 : 3;
  EXPECT(by_width[idx] == rep.total_bytes, "storage_by_code_width[%d] %lld != %lld", idx, (long long)by_width[idx], (long long)rep.total_bytes);
  macko_report_t rep2;
  EXPECT(macko_get_report(h, &rep2) == MACKO_OK && std::memcmp(&rep, &rep2, sizeof(rep)) == 0, "report copy");
  // device operations on a handle without device buffers are refused before anything is launched
  EXPECT(macko_spmv(h, W.data(), W.data(), nullptr) == (rows == 0 ? MACKO_E_NOT_BOUND : MACKO_E_NOT_BOUND), "unbound spmv");
  macko_destroy(h);
}

static void check8(int64_t rows, int64_t cols, int64_t ld, double density, std::mt19937_64& rng) {
  std::vector<uint8_t> W = random_matrix<uint8_t>(rows, cols, ld, density, rng, (uint8_t)0x38);
  macko_handle_t h = nullptr;
  macko_report_t rep;
  EXPECT(macko_encode_fp8(W.data(), rows, cols, ld, &h, &rep) == MACKO_OK && h, "encode fp8");
  if (!h) return;
  EXPECT(rep.b_val == 8 && rep.values_bytes == rep.alloc_nnz, "8-bit report");
  const uint8_t* v8 = nullptr;
  EXPECT(macko_host_values_fp8(h, &v8) == MACKO_OK && (v8 || rep.alloc_nnz == 0), "host values");
  const uint16_t* v16 = nullptr;
  EXPECT(macko_host_buffers(h, &v16, nullptr, nullptr) == MACKO_E_UNSUPPORTED, "16-bit view of 8-bit values");
  std::vector<uint8_t> dec((size_t)(rows * cols), 0xEE);
  EXPECT(macko_decode_fp8(h, dec.data(), cols) == MACKO_OK, "decode fp8");
  std::vector<uint16_t> d16((size_t)(rows * cols));
  EXPECT(macko_decode(h, d16.data(), cols) == MACKO_E_UNSUPPORTED, "fp16 decode of 8-bit values");
  bool same = true;
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      const uint8_t in = W[(size_t)(r * ld + c)];
      same = same && dec[(size_t)(r * cols + c)] == ((in & 0x7F) ? in : 0);
    }
  EXPECT(same, "fp8 round trip %lldx%lld", (long long)rows, (long long)cols);
  macko_destroy(h);
}

int main() {
  std::mt19937_64 rng(2511013061ull);
  const int64_t shapes[][3] = {{1, 1, 1}, {7, 13, 13}, {33, 257, 300}, {5, 4000, 4000}, {130, 777, 1024},
                               {64, 64, 64}, {3, 100000, 100000}, {257, 31, 32}};
  for (auto& s : shapes)
    for (int b : {1, 2, 4, 8})
      for (double d : {0.0, 0.02, 0.5, 1.0}) check16(s[0], s[1], s[2], d, b, rng);
  for (auto& s : shapes)
    for (double d : {0.03, 0.6}) check8(s[0], s[1], s[2], d, rng);
  // empty shapes are valid; bad arguments are refused and leave no handle behind
  macko_handle_t h = reinterpret_cast<macko_handle_t>(0x1);
  uint16_t one = 0x3C00;
  EXPECT(macko_encode(&one, 0, 5, 5, &h, nullptr) == MACKO_OK && h, "0 rows");
  macko_destroy(h);
  EXPECT(macko_encode(&one, 5, 0, 0, &h, nullptr) == MACKO_OK && h, "0 cols");
  {
    std::vector<uint16_t> dec(1);
    EXPECT(macko_decode(h, dec.data(), 0) == MACKO_OK, "decode of 5 x 0");
  }
  macko_destroy(h);
  h = reinterpret_cast<macko_handle_t>(0x1);
  EXPECT(macko_encode(&one, 1, 2, 1, &h, nullptr) == MACKO_E_INVALID_ARG && h == nullptr, "ld < cols");
  EXPECT(macko_encode(nullptr, 1, 1, 1, &h, nullptr) == MACKO_E_INVALID_ARG, "null matrix");
  EXPECT(macko_encode(&one, -1, 1, 1, &h, nullptr) == MACKO_E_INVALID_ARG, "negative rows");
  EXPECT(macko_encode_ex(&one, 1, 1, 1, 3, &h, nullptr) == MACKO_E_INVALID_ARG, "code width 3");
  EXPECT(macko_encode(&one, 1, 1, 1, nullptr, nullptr) == MACKO_E_INVALID_ARG, "null out");
  macko_destroy(nullptr);
  int64_t value = -1;
  EXPECT(macko_set_tuning("no_such_knob", 1) == MACKO_E_INVALID_ARG && macko_get_tuning("spmv_ring", &value) == MACKO_OK &&
             value == 0, "tuning");
  EXPECT(std::strcmp(macko_status_string(MACKO_E_OVERFLOW), macko_status_string(12345)) != 0, "status strings");
  // More stored entries than 32-bit row pointers can address: with 1-bit codes a gap of 2^21 columns is
  // bridged by 2^20 padding entries, so 4100 rows with one non-zero in their last column hold 4.3e9 entries.
  // The matrix is 17 GB of untouched zero pages of an anonymous mapping plus one non-zero per row; the
  // encoder must refuse after its counting pass, before it allocates or writes anything.
  {
    const int64_t rows = 4100, cols = (int64_t{1} << 21) + 1;
    const size_t bytes = (size_t)(rows * cols) * 2;
    void* p = mmap(nullptr, bytes, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0);
    if (p == MAP_FAILED) {
      std::printf("note: no address space for the overflow case, skipped\n");
    } else {
      uint16_t* W = static_cast<uint16_t*>(p);
      for (int64_t r = 0; r < rows; ++r) W[(size_t)(r * cols + cols - 1)] = 0x3C00;
      h = reinterpret_cast<macko_handle_t>(0x1);
      const int st = macko_encode_ex(W, rows, cols, cols, 1, &h, nullptr);
      EXPECT(st == MACKO_E_OVERFLOW && h == nullptr, "4.3e9 entries with 1-bit codes: status %d", st);
      munmap(p, bytes);
    }
  }
  if (failures) { std::printf("%d failures\n", failures); return 1; }
  std::printf("ok\n");
  return 0;
}
