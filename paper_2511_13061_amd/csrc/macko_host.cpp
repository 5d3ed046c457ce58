// Host side of libmacko: the C ABI, the handle, the host encoder / decoder and
// the storage report.  The format is that of Section 4.1 with b_val = 16 and
// b_delta = 4 by default (1, 2 and 8 through the _ex entry points); see
// include/macko.h for the byte layout.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <mutex>
#include <new>
#include <string>
#include <thread>

#include "macko_internal.h"

namespace macko {

static thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  (void)hipGetLastError();  // clear the sticky error so later calls report their own
  return MACKO_E_HIP;
}

Tuning& tuning() {
  static Tuning t;
  return t;
}

int device_cu_count() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

// Storage report: eq. 2 for the measured effective density, eqs. 8-10 for the
// best / worst / expected cases at the measured density.
void fill_report(macko_report_t* rep, int64_t rows, int64_t cols, int64_t nnz, int64_t pad_nnz,
                 int64_t alloc_nnz, int64_t empty_rows, int64_t max_row_entries, int b_delta, int b_val) {
  const double max_delta = static_cast<double>(1 << b_delta);
  std::memset(rep, 0, sizeof(*rep));
  rep->rows = rows;
  rep->cols = cols;
  rep->nnz = nnz;
  rep->pad_nnz = pad_nnz;
  rep->alloc_nnz = alloc_nnz;
  rep->padding_entries = nnz >= 0 ? pad_nnz - nnz : -1;
  rep->empty_rows = empty_rows;
  rep->max_row_entries = max_row_entries;
  rep->values_bytes = alloc_nnz * b_val / 8;
  rep->deltas_bytes = alloc_nnz * b_delta / 8;
  rep->rowptr_bytes = 4 * (rows + 1);
  rep->total_bytes = rep->values_bytes + rep->deltas_bytes + rep->rowptr_bytes;
  rep->dense_bytes = rows * cols * b_val / 8;
  rep->b_val = b_val;
  rep->b_delta = b_delta;
  const double cells = static_cast<double>(rows) * static_cast<double>(cols);
  const double nan = std::numeric_limits<double>::quiet_NaN();
  rep->effd = cells > 0 ? static_cast<double>(rep->total_bytes) / (cells * b_val / 8.0) : 0.0;
  if (nnz < 0 || cells <= 0) {
    rep->density = rep->effd_best = rep->effd_expected = rep->effd_worst = cells > 0 ? nan : 0.0;
    return;
  }
  const double d = static_cast<double>(nnz) / cells;
  const double per_entry = static_cast<double>(b_val + b_delta) / b_val;
  rep->density = d;
  rep->effd_best = d * per_entry;
  rep->effd_worst = (d + (1.0 - d) / max_delta) * per_entry;
  const double z = std::pow(1.0 - d, max_delta);
  rep->effd_expected = (d > 0.0 && d < 1.0) ? d * (1.0 + z / (1.0 - z)) * per_entry : d * per_entry;
}

namespace {

inline bool is_nonzero(uint16_t bits) { return (bits & 0x7FFFu) != 0; }
inline bool is_nonzero(uint8_t bits) { return (bits & 0x7Fu) != 0; }    // 8-bit values: everything but the sign

template <class F>
void parallel_blocks(int64_t n, F&& body) {
  unsigned hw = std::thread::hardware_concurrency();
  int64_t nthreads = std::max<int64_t>(1, std::min<int64_t>(hw ? hw : 1, 32));
  nthreads = std::min<int64_t>(nthreads, std::max<int64_t>(1, n / 64));
  if (nthreads <= 1) {
    body(0, n);
    return;
  }
  std::vector<std::thread> pool;
  int64_t chunk = (n + nthreads - 1) / nthreads;
  for (int64_t t = 0; t < nthreads; ++t) {
    int64_t lo = t * chunk, hi = std::min(n, lo + chunk);
    if (lo >= hi) break;
    pool.emplace_back([=, &body] { body(lo, hi); });
  }
  for (auto& th : pool) th.join();
}

template <class T> std::vector<T>& values_of(macko_matrix* m);
template <> inline std::vector<uint16_t>& values_of<uint16_t>(macko_matrix* m) { return m->h_values; }
template <> inline std::vector<uint8_t>& values_of<uint8_t>(macko_matrix* m) { return m->h_values8; }

// Stored entries of one row: a non-zero whose distance to the previously
// stored column is g costs (g-1) / 2^b_delta padding entries plus itself.
template <class T>
inline void count_row(const T* row, int64_t cols, int b_delta, int64_t* entries, int64_t* nnz) {
  int64_t prev = -1, e = 0, n = 0;
  for (int64_t c = 0; c < cols; ++c) {
    if (!is_nonzero(row[c])) continue;
    e += 1 + ((c - prev - 1) >> b_delta);
    ++n;
    prev = c;
  }
  *entries = e;
  *nnz = n;
}

// Write one row's entries; codes go to a byte-per-entry scratch array that is
// packed afterwards (two rows may share a byte of the packed array).
template <class T>
inline void fill_row(const T* row, int64_t cols, int b_delta, T* values, uint8_t* codes) {
  const int64_t full = (int64_t{1} << b_delta) - 1;   // code of the largest delta
  int64_t prev = -1, k = 0;
  for (int64_t c = 0; c < cols; ++c) {
    const T w = row[c];
    if (!is_nonzero(w)) continue;
    const int64_t g1 = c - prev - 1;          // gap - 1
    for (int64_t p = g1 >> b_delta; p > 0; --p) {
      values[k] = 0;
      codes[k] = static_cast<uint8_t>(full);
      ++k;
    }
    values[k] = w;
    codes[k] = static_cast<uint8_t>(g1 & full);
    ++k;
    prev = c;
  }
}

template <class T>
int encode_host(const T* dense, int64_t rows, int64_t cols, int64_t ld, int b_delta, macko_matrix* m) {
  constexpr int b_val = 8 * (int)sizeof(T);
  std::vector<T>& h_values = values_of<T>(m);
  std::vector<int64_t> entries(rows), nnzs(rows);
  parallel_blocks(rows, [&](int64_t lo, int64_t hi) {
    for (int64_t r = lo; r < hi; ++r) count_row(dense + r * ld, cols, b_delta, &entries[r], &nnzs[r]);
  });
  int64_t pad_nnz = 0, nnz = 0, empty = 0, longest = 0;
  m->h_row_ptr.assign(rows + 1, 0);
  for (int64_t r = 0; r < rows; ++r) {
    pad_nnz += entries[r];
    nnz += nnzs[r];
    empty += entries[r] == 0;
    longest = std::max(longest, entries[r]);
    if (pad_nnz >= (int64_t{1} << 32)) return MACKO_E_OVERFLOW;
    m->h_row_ptr[r + 1] = static_cast<uint32_t>(pad_nnz);
  }
  const int64_t granule = alloc_granule(b_delta);
  const int64_t alloc = (pad_nnz + granule - 1) / granule * granule;
  if (alloc >= (int64_t{1} << 32)) return MACKO_E_OVERFLOW;
  h_values.assign(alloc, 0);
  m->h_deltas.assign(alloc * b_delta / 8, 0);
  std::vector<uint8_t> codes(alloc, 0);
  parallel_blocks(rows, [&](int64_t lo, int64_t hi) {
    for (int64_t r = lo; r < hi; ++r) {
      const int64_t at = m->h_row_ptr[r];
      fill_row(dense + r * ld, cols, b_delta, h_values.data() + at, codes.data() + at);
    }
  });
  // entry k occupies bits [k * b_delta, (k + 1) * b_delta) of the packed array (low bits first)
  const int per_byte = 8 / b_delta;
  parallel_blocks(alloc / per_byte, [&](int64_t lo, int64_t hi) {
    for (int64_t b = lo; b < hi; ++b) {
      unsigned byte = 0;
      for (int j = 0; j < per_byte; ++j) byte |= static_cast<unsigned>(codes[per_byte * b + j]) << (b_delta * j);
      m->h_deltas[b] = static_cast<uint8_t>(byte);
    }
  });
  m->rows = rows;
  m->cols = cols;
  m->pad_nnz = pad_nnz;
  m->alloc_nnz = alloc;
  m->b_delta = b_delta;
  m->b_val = b_val;
  m->has_host = true;
  fill_report(&m->report, rows, cols, nnz, pad_nnz, alloc, empty, longest, b_delta, b_val);
  return MACKO_OK;
}

}  // namespace
}  // namespace macko

using macko::tuning;

extern "C" {

static bool valid_b_delta(int b) { return b == 1 || b == 2 || b == 4 || b == 8; }

int macko_encode(const uint16_t* dense_host, int64_t rows, int64_t cols, int64_t ld,
                 macko_handle_t* out, macko_report_t* report) {
  return macko_encode_ex(dense_host, rows, cols, ld, macko::kDeltaBits, out, report);
}

int macko_encode_ex(const uint16_t* dense_host, int64_t rows, int64_t cols, int64_t ld, int b_delta,
                    macko_handle_t* out, macko_report_t* report) {
  if (out) *out = nullptr;
  if (!out || rows < 0 || cols < 0 || ld < cols || !valid_b_delta(b_delta)) return MACKO_E_INVALID_ARG;
  if (!dense_host && rows > 0 && cols > 0) return MACKO_E_INVALID_ARG;
  if (cols >= (int64_t{1} << 31) || rows >= (int64_t{1} << 31)) return MACKO_E_UNSUPPORTED;
  macko_matrix* m = nullptr;
  try {
    m = new macko_matrix();
    int st = macko::encode_host(dense_host, rows, cols, ld, b_delta, m);
    if (st != MACKO_OK) {
      delete m;
      return st;
    }
  } catch (const std::bad_alloc&) {
    delete m;
    return MACKO_E_OUT_OF_MEMORY;
  } catch (...) {
    delete m;
    return MACKO_E_INVALID_ARG;
  }
  if (report) *report = m->report;
  *out = m;
  return MACKO_OK;
}

int macko_storage_by_code_width(const uint16_t* dense_host, int64_t rows, int64_t cols, int64_t ld,
                                int64_t total_bytes[4], int* best_b_delta) {
  if (!total_bytes || rows < 0 || cols < 0 || ld < cols) return MACKO_E_INVALID_ARG;
  if (!dense_host && rows > 0 && cols > 0) return MACKO_E_INVALID_ARG;
  if (cols >= (int64_t{1} << 31) || rows >= (int64_t{1} << 31)) return MACKO_E_UNSUPPORTED;
  static const int widths[4] = {1, 2, 4, 8};
  try {
    std::vector<int64_t> entries(rows), nnzs(rows);
    for (int i = 0; i < 4; ++i) {
      const int b = widths[i];
      macko::parallel_blocks(rows, [&](int64_t lo, int64_t hi) {
        for (int64_t r = lo; r < hi; ++r) macko::count_row(dense_host + r * ld, cols, b, &entries[r], &nnzs[r]);
      });
      int64_t pad_nnz = 0;
      for (int64_t r = 0; r < rows; ++r) pad_nnz += entries[r];
      const int64_t granule = macko::alloc_granule(b);
      const int64_t alloc = (pad_nnz + granule - 1) / granule * granule;
      total_bytes[i] = alloc >= (int64_t{1} << 32) ? -1 : alloc * 2 + alloc * b / 8 + 4 * (rows + 1);
    }
  } catch (const std::bad_alloc&) {
    return MACKO_E_OUT_OF_MEMORY;
  }
  if (best_b_delta) {
    int best = -1;
    for (int i : {2, 0, 1, 3}) {                       // ties: 4 bits first, then the narrower width
      if (total_bytes[i] < 0) continue;
      if (best < 0 || total_bytes[i] < total_bytes[best]) best = i;
    }
    *best_b_delta = best < 0 ? 0 : widths[best];
  }
  return MACKO_OK;
}

int macko_encode_fp8(const uint8_t* dense_host, int64_t rows, int64_t cols, int64_t ld,
                     macko_handle_t* out, macko_report_t* report) {
  if (out) *out = nullptr;
  if (!out || rows < 0 || cols < 0 || ld < cols) return MACKO_E_INVALID_ARG;
  if (!dense_host && rows > 0 && cols > 0) return MACKO_E_INVALID_ARG;
  if (cols >= (int64_t{1} << 31) || rows >= (int64_t{1} << 31)) return MACKO_E_UNSUPPORTED;
  macko_matrix* m = nullptr;
  try {
    m = new macko_matrix();
    int st = macko::encode_host(dense_host, rows, cols, ld, macko::kDeltaBits, m);
    if (st != MACKO_OK) {
      delete m;
      return st;
    }
  } catch (const std::bad_alloc&) {
    delete m;
    return MACKO_E_OUT_OF_MEMORY;
  } catch (...) {
    delete m;
    return MACKO_E_INVALID_ARG;
  }
  if (report) *report = m->report;
  *out = m;
  return MACKO_OK;
}

int macko_encode_device(const void* dense_dev, int64_t rows, int64_t cols, int64_t ld, void* stream,
                        macko_handle_t* out, macko_report_t* report) {
  return macko_encode_device_ex(dense_dev, rows, cols, ld, macko::kDeltaBits, stream, out, report);
}

static int encode_device_any(const void* dense_dev, int64_t rows, int64_t cols, int64_t ld, int b_delta, int b_val,
                             void* stream, macko_handle_t* out, macko_report_t* report);

int macko_encode_device_ex(const void* dense_dev, int64_t rows, int64_t cols, int64_t ld, int b_delta,
                           void* stream, macko_handle_t* out, macko_report_t* report) {
  return encode_device_any(dense_dev, rows, cols, ld, b_delta, 16, stream, out, report);
}

int macko_encode_device_fp8(const void* dense_dev, int64_t rows, int64_t cols, int64_t ld, void* stream,
                            macko_handle_t* out, macko_report_t* report) {
  return encode_device_any(dense_dev, rows, cols, ld, macko::kDeltaBits, 8, stream, out, report);
}

static int encode_device_any(const void* dense_dev, int64_t rows, int64_t cols, int64_t ld, int b_delta, int b_val,
                             void* stream, macko_handle_t* out, macko_report_t* report) {
  if (out) *out = nullptr;
  if (!out || rows < 0 || cols < 0 || ld < cols || !valid_b_delta(b_delta)) return MACKO_E_INVALID_ARG;
  if (!dense_dev && rows > 0 && cols > 0) return MACKO_E_INVALID_ARG;
  if (cols >= (int64_t{1} << 31) || rows >= (int64_t{1} << 31)) return MACKO_E_UNSUPPORTED;
  macko_matrix* m = new (std::nothrow) macko_matrix();
  if (!m) return MACKO_E_OUT_OF_MEMORY;
  void* v = nullptr;
  uint8_t* d = nullptr;
  uint32_t* rp = nullptr;
  int64_t nnz = 0, pad = 0, alloc = 0, empty = 0, longest = 0;
  void* block = nullptr;
  int st = macko::encode_on_device(dense_dev, rows, cols, ld, b_delta, b_val,
                                   static_cast<hipStream_t>(stream), &block, &v, &d, &rp, &nnz, &pad, &alloc,
                                   &empty, &longest);
  if (st != MACKO_OK) {
    delete m;
    return st;
  }
  m->rows = rows;
  m->cols = cols;
  m->pad_nnz = pad;
  m->alloc_nnz = alloc;
  m->d_values = static_cast<const uint16_t*>(v);
  m->d_deltas = d;
  m->d_row_ptr = rp;
  m->b_delta = b_delta;
  m->b_val = b_val;
  m->bound = true;
  m->owns_device = true;
  m->d_block = block;
  macko::fill_report(&m->report, rows, cols, nnz, pad, alloc, empty, longest, b_delta, b_val);
  if (report) *report = m->report;
  *out = m;
  return MACKO_OK;
}

int macko_wrap_device(int64_t rows, int64_t cols, int64_t pad_nnz, const void* values_dev,
                      const void* deltas_dev, const void* rowptr_dev, macko_handle_t* out) {
  return macko_wrap_device_ex(rows, cols, pad_nnz, macko::kDeltaBits, values_dev, deltas_dev, rowptr_dev, out);
}

int macko_wrap_device_ex(int64_t rows, int64_t cols, int64_t pad_nnz, int b_delta, const void* values_dev,
                         const void* deltas_dev, const void* rowptr_dev, macko_handle_t* out) {
  if (out) *out = nullptr;
  if (!out || rows < 0 || cols < 0 || pad_nnz < 0 || !rowptr_dev || !valid_b_delta(b_delta))
    return MACKO_E_INVALID_ARG;
  if (pad_nnz > 0 && (!values_dev || !deltas_dev)) return MACKO_E_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(values_dev) & 15) || (reinterpret_cast<uintptr_t>(deltas_dev) & 15) ||
      (reinterpret_cast<uintptr_t>(rowptr_dev) & 3))
    return MACKO_E_INVALID_ARG;
  const int64_t granule = macko::alloc_granule(b_delta);
  const int64_t alloc = (pad_nnz + granule - 1) / granule * granule;
  if (alloc >= (int64_t{1} << 32)) return MACKO_E_OVERFLOW;
  if (cols >= (int64_t{1} << 31) || rows >= (int64_t{1} << 31)) return MACKO_E_UNSUPPORTED;
  macko_matrix* m = new (std::nothrow) macko_matrix();
  if (!m) return MACKO_E_OUT_OF_MEMORY;
  m->rows = rows;
  m->cols = cols;
  m->pad_nnz = pad_nnz;
  m->alloc_nnz = alloc;
  m->d_values = static_cast<const uint16_t*>(values_dev);
  m->d_deltas = static_cast<const uint8_t*>(deltas_dev);
  m->d_row_ptr = static_cast<const uint32_t*>(rowptr_dev);
  m->b_delta = b_delta;
  m->bound = true;
  macko::fill_report(&m->report, rows, cols, -1, pad_nnz, alloc, -1, -1, b_delta);
  *out = m;
  return MACKO_OK;
}

int macko_wrap_device_fp8(int64_t rows, int64_t cols, int64_t pad_nnz, const void* values_dev,
                          const void* deltas_dev, const void* rowptr_dev, macko_handle_t* out) {
  int st = macko_wrap_device_ex(rows, cols, pad_nnz, macko::kDeltaBits, values_dev, deltas_dev, rowptr_dev, out);
  if (st != MACKO_OK) return st;
  (*out)->b_val = 8;
  macko::fill_report(&(*out)->report, rows, cols, -1, pad_nnz, (*out)->alloc_nnz, -1, -1, macko::kDeltaBits, 8);
  return MACKO_OK;
}

int macko_get_report(macko_handle_t h, macko_report_t* report) {
  if (!h || !report) return MACKO_E_INVALID_ARG;
  *report = h->report;
  return MACKO_OK;
}

int macko_device_bytes(macko_handle_t h, int64_t* values_bytes, int64_t* deltas_bytes,
                       int64_t* rowptr_bytes) {
  if (!h) return MACKO_E_INVALID_ARG;
  if (values_bytes) *values_bytes = h->alloc_nnz * h->b_val / 8;
  if (deltas_bytes) *deltas_bytes = h->alloc_nnz * h->b_delta / 8;
  if (rowptr_bytes) *rowptr_bytes = 4 * (h->rows + 1);
  return MACKO_OK;
}

int macko_bind_device(macko_handle_t h, void* values_dev, void* deltas_dev, void* rowptr_dev,
                      void* stream) {
  if (!h || !rowptr_dev) return MACKO_E_INVALID_ARG;
  if (!h->has_host) return MACKO_E_UNSUPPORTED;
  if (h->alloc_nnz > 0 && (!values_dev || !deltas_dev)) return MACKO_E_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(values_dev) & 15) || (reinterpret_cast<uintptr_t>(deltas_dev) & 15) ||
      (reinterpret_cast<uintptr_t>(rowptr_dev) & 3))
    return MACKO_E_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (h->alloc_nnz > 0) {
    const void* hv = h->b_val == 8 ? static_cast<const void*>(h->h_values8.data()) : static_cast<const void*>(h->h_values.data());
    MACKO_HIP_TRY(hipMemcpyAsync(values_dev, hv, h->alloc_nnz * h->b_val / 8, hipMemcpyHostToDevice, s));
    MACKO_HIP_TRY(hipMemcpyAsync(deltas_dev, h->h_deltas.data(), h->alloc_nnz * h->b_delta / 8, hipMemcpyHostToDevice, s));
  }
  MACKO_HIP_TRY(hipMemcpyAsync(rowptr_dev, h->h_row_ptr.data(), 4 * (h->rows + 1), hipMemcpyHostToDevice, s));
  // the host vectors are pageable: make sure the copies have left them before returning
  MACKO_HIP_TRY(hipStreamSynchronize(s));
  h->d_values = static_cast<const uint16_t*>(values_dev);
  h->d_deltas = static_cast<const uint8_t*>(deltas_dev);
  h->d_row_ptr = static_cast<const uint32_t*>(rowptr_dev);
  h->bound = true;
  h->owns_device = false;
  return MACKO_OK;
}

int macko_host_buffers(macko_handle_t h, const uint16_t** values, const uint8_t** deltas,
                       const uint32_t** row_ptr) {
  if (!h) return MACKO_E_INVALID_ARG;
  if (!h->has_host) return MACKO_E_UNSUPPORTED;
  if (values && h->b_val != 16) return MACKO_E_UNSUPPORTED;     // 8-bit values: macko_host_values_fp8
  if (values) *values = h->h_values.data();
  if (deltas) *deltas = h->h_deltas.data();
  if (row_ptr) *row_ptr = h->h_row_ptr.data();
  return MACKO_OK;
}

int macko_fetch_device(macko_handle_t h, uint16_t* values_host, uint8_t* deltas_host,
                       uint32_t* rowptr_host) {
  if (!h || !rowptr_host) return MACKO_E_INVALID_ARG;
  if (!h->bound) return MACKO_E_NOT_BOUND;
  if (h->alloc_nnz > 0) {
    if (!values_host || !deltas_host) return MACKO_E_INVALID_ARG;
    MACKO_HIP_TRY(hipMemcpy(values_host, h->d_values, h->alloc_nnz * h->b_val / 8, hipMemcpyDeviceToHost));
    MACKO_HIP_TRY(hipMemcpy(deltas_host, h->d_deltas, h->alloc_nnz * h->b_delta / 8, hipMemcpyDeviceToHost));
  }
  MACKO_HIP_TRY(hipMemcpy(rowptr_host, h->d_row_ptr, 4 * (h->rows + 1), hipMemcpyDeviceToHost));
  return MACKO_OK;
}

int macko_decode(macko_handle_t h, uint16_t* dense_host_out, int64_t ld) {
  if (!h || ld < h->cols) return MACKO_E_INVALID_ARG;
  if (!h->has_host || h->b_val != 16) return MACKO_E_UNSUPPORTED;
  if (!dense_host_out && h->rows > 0 && h->cols > 0) return MACKO_E_INVALID_ARG;
  for (int64_t r = 0; r < h->rows; ++r) {
    uint16_t* row = dense_host_out + r * ld;
    std::fill(row, row + h->cols, uint16_t{0});
    int64_t pos = 0;  // column + 1 of the last decoded entry
    const int b = h->b_delta;
    for (int64_t k = h->h_row_ptr[r]; k < h->h_row_ptr[r + 1]; ++k) {
      const int64_t bit = k * b;
      pos += ((h->h_deltas[bit >> 3] >> (bit & 7)) & ((1u << b) - 1u)) + 1;
      if (pos > h->cols) return MACKO_E_INVALID_ARG;
      row[pos - 1] = h->h_values[k];
    }
  }
  return MACKO_OK;
}

int macko_host_values_fp8(macko_handle_t h, const uint8_t** values) {
  if (!h || !values) return MACKO_E_INVALID_ARG;
  if (!h->has_host || h->b_val != 8) return MACKO_E_UNSUPPORTED;
  *values = h->h_values8.data();
  return MACKO_OK;
}

int macko_decode_fp8(macko_handle_t h, uint8_t* dense_host_out, int64_t ld) {
  if (!h || ld < h->cols) return MACKO_E_INVALID_ARG;
  if (!h->has_host || h->b_val != 8) return MACKO_E_UNSUPPORTED;
  if (!dense_host_out && h->rows > 0 && h->cols > 0) return MACKO_E_INVALID_ARG;
  for (int64_t r = 0; r < h->rows; ++r) {
    uint8_t* row = dense_host_out + r * ld;
    std::fill(row, row + h->cols, uint8_t{0});
    int64_t pos = 0;  // column + 1 of the last decoded entry
    const int b = h->b_delta;
    for (int64_t k = h->h_row_ptr[r]; k < h->h_row_ptr[r + 1]; ++k) {
      const int64_t bit = k * b;
      pos += ((h->h_deltas[bit >> 3] >> (bit & 7)) & ((1u << b) - 1u)) + 1;
      if (pos > h->cols) return MACKO_E_INVALID_ARG;
      row[pos - 1] = h->h_values8[k];
    }
  }
  return MACKO_OK;
}

static int check_vec_ptrs(const void* x_dev, const void* y_dev, int64_t cols) {
  if (!y_dev || (!x_dev && cols > 0)) return MACKO_E_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(x_dev) & 1) || (reinterpret_cast<uintptr_t>(y_dev) & 1))
    return MACKO_E_INVALID_ARG;
  return MACKO_OK;
}

int macko_check_device(macko_handle_t h, void* stream, int64_t* first_bad_row) {
  if (!h) return MACKO_E_INVALID_ARG;
  if (!h->bound) return MACKO_E_NOT_BOUND;
  if (first_bad_row) *first_bad_row = -1;
  if (h->rows == 0) return h->pad_nnz == 0 ? MACKO_OK : MACKO_E_CORRUPT;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned int* d_first = nullptr;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&d_first), sizeof(unsigned int));
  if (e != hipSuccess) return e == hipErrorOutOfMemory ? MACKO_E_OUT_OF_MEMORY : macko::hip_fail(e);
  unsigned int first = (unsigned int)h->rows;
  int st = MACKO_OK;
  e = hipMemcpyAsync(d_first, &first, sizeof(first), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) {
    const macko::SpmvProblem p{h->d_values, h->d_deltas, h->d_row_ptr, h->rows, h->cols, h->pad_nnz,
                               nullptr, nullptr, h->b_delta};
    st = macko::launch_check(p, d_first, s);
    if (st == MACKO_OK) e = hipMemcpyAsync(&first, d_first, sizeof(first), hipMemcpyDeviceToHost, s);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);     // also on a failed launch: nothing may still use d_first
  else (void)hipStreamSynchronize(s);
  (void)hipFree(d_first);
  if (st != MACKO_OK) return st;
  if (e != hipSuccess) return macko::hip_fail(e);
  if (first < (unsigned int)h->rows) {
    if (first_bad_row) *first_bad_row = (int64_t)first;
    return MACKO_E_CORRUPT;
  }
  return MACKO_OK;
}

int macko_columns_device(macko_handle_t h, int32_t* cols_dev, void* stream) {
  if (!h) return MACKO_E_INVALID_ARG;
  if (!h->bound) return MACKO_E_NOT_BOUND;
  if (h->rows == 0 || h->pad_nnz == 0) return MACKO_OK;
  if (!cols_dev || (reinterpret_cast<uintptr_t>(cols_dev) & 3)) return MACKO_E_INVALID_ARG;
  const macko::SpmvProblem p{h->d_values, h->d_deltas, h->d_row_ptr, h->rows, h->cols, h->pad_nnz,
                             nullptr, nullptr, h->b_delta};
  return macko::launch_columns(p, cols_dev, static_cast<hipStream_t>(stream));
}

int macko_decode_device(macko_handle_t h, void* dense_dev, int64_t ld, void* stream) {
  if (!h) return MACKO_E_INVALID_ARG;
  if (!h->bound) return MACKO_E_NOT_BOUND;
  if (h->rows == 0 || h->cols == 0) return MACKO_OK;
  if (!dense_dev || ld < h->cols) return MACKO_E_INVALID_ARG;
  if (h->b_val == 16 && (reinterpret_cast<uintptr_t>(dense_dev) & 1)) return MACKO_E_INVALID_ARG;
  const macko::SpmvProblem p{h->d_values, h->d_deltas, h->d_row_ptr, h->rows, h->cols, h->pad_nnz,
                             nullptr, nullptr, h->b_delta, h->b_val};
  return macko::launch_decode(p, dense_dev, ld, static_cast<hipStream_t>(stream));
}

int macko_spmv(macko_handle_t h, const void* x_dev, void* y_dev, void* stream) {
  return macko_spmv_group(1, &h, &x_dev, &y_dev, stream);
}

int macko_spmv_group(int n, const macko_handle_t* handles, const void* const* x_dev, void* const* y_dev,
                     void* stream) {
  if (n < 1 || n > MACKO_MAX_GROUP || !handles || !x_dev || !y_dev) return MACKO_E_INVALID_ARG;
  macko::SpmvProblem p[MACKO_MAX_GROUP];
  int m = 0;
  for (int i = 0; i < n; ++i) {
    macko_handle_t h = handles[i];
    if (!h) return MACKO_E_INVALID_ARG;
    if (!h->bound) return MACKO_E_NOT_BOUND;
    if (h->rows == 0) continue;
    int st = check_vec_ptrs(x_dev[i], y_dev[i], h->cols);
    if (st != MACKO_OK) return st;
    p[m++] = macko::SpmvProblem{h->d_values, h->d_deltas, h->d_row_ptr, h->rows, h->cols, h->pad_nnz,
                                x_dev[i], y_dev[i], h->b_delta, h->b_val};
  }
  if (m == 0) return MACKO_OK;
  return macko::launch_spmv_group(m, p, static_cast<hipStream_t>(stream));
}

namespace {

// Side streams of macko_spmv_many, one set per device, created on first use and kept until the
// process ends (default priority).  The mutex covers creation and every call's enqueue phase:
// the fork / join events are shared.
constexpr int kManyStreams = 3;
struct ManyStreams {
  bool ready = false;
  hipStream_t side[kManyStreams] = {};
  hipEvent_t fork = nullptr;
  hipEvent_t join[kManyStreams] = {};
};
std::mutex g_many_mutex;
ManyStreams g_many[64];

int many_streams_for(int dev, ManyStreams** out) {
  if (dev < 0 || dev >= 64) return MACKO_E_UNSUPPORTED;
  ManyStreams& ms = g_many[dev];
  if (!ms.ready) {
    MACKO_HIP_TRY(hipEventCreateWithFlags(&ms.fork, hipEventDisableTiming));
    for (int i = 0; i < kManyStreams; ++i) {
      MACKO_HIP_TRY(hipStreamCreateWithFlags(&ms.side[i], hipStreamNonBlocking));
      MACKO_HIP_TRY(hipEventCreateWithFlags(&ms.join[i], hipEventDisableTiming));
    }
    ms.ready = true;
  }
  *out = &ms;
  return MACKO_OK;
}

}  // namespace

int macko_spmv_many(int64_t n, const macko_handle_t* handles, const void* const* x_dev, void* const* y_dev,
                    void* stream) {
  if (n < 0 || (n > 0 && (!handles || !x_dev || !y_dev))) return MACKO_E_INVALID_ARG;
  for (int64_t i = 0; i < n; ++i) {                      // everything is checked before anything is enqueued
    macko_handle_t h = handles[i];
    if (!h) return MACKO_E_INVALID_ARG;
    if (!h->bound) return MACKO_E_NOT_BOUND;
    if (h->rows == 0) continue;
    int st = check_vec_ptrs(x_dev[i], y_dev[i], h->cols);
    if (st != MACKO_OK) return st;
  }
  if (n <= MACKO_MAX_GROUP) return n == 0 ? MACKO_OK : macko_spmv_group((int)n, handles, x_dev, y_dev, stream);
  int dev = 0;
  MACKO_HIP_TRY(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(g_many_mutex);
  ManyStreams* ms = nullptr;
  int st = many_streams_for(dev, &ms);
  if (st != MACKO_OK) return st;
  hipStream_t main = static_cast<hipStream_t>(stream);
  // fork: the side streams start after everything already enqueued on the caller's stream
  MACKO_HIP_TRY(hipEventRecord(ms->fork, main));
  for (int i = 0; i < kManyStreams; ++i) MACKO_HIP_TRY(hipStreamWaitEvent(ms->side[i], ms->fork, 0));
  int result = MACKO_OK;
  int turn = 0;
  for (int64_t at = 0; at < n && result == MACKO_OK; at += MACKO_MAX_GROUP, ++turn) {
    const int count = (int)std::min<int64_t>(MACKO_MAX_GROUP, n - at);
    result = macko_spmv_group(count, handles + at, x_dev + at, y_dev + at, ms->side[turn % kManyStreams]);
  }
  // join, also after a failed launch: the caller's stream continues once every side stream is done
  for (int i = 0; i < kManyStreams; ++i) {
    hipError_t e = hipEventRecord(ms->join[i], ms->side[i]);
    if (e == hipSuccess) e = hipStreamWaitEvent(main, ms->join[i], 0);
    if (e != hipSuccess && result == MACKO_OK) result = macko::hip_fail(e);
  }
  return result;
}

namespace {

// argument checks and problem list shared by the two chain entry points
int chain_problems(int n_phases, const int* phase_sizes, const macko_handle_t* handles, const void* const* x_dev,
                   void* const* y_dev, macko::SpmvProblem* p, int* total_out) {
  if (n_phases < 1 || !phase_sizes || !handles || !x_dev || !y_dev) return MACKO_E_INVALID_ARG;
  if (n_phases > MACKO_MAX_CHAIN_PHASES) return MACKO_E_UNSUPPORTED;
  int total = 0;
  for (int ph = 0; ph < n_phases; ++ph) {
    if (phase_sizes[ph] < 1 || phase_sizes[ph] > MACKO_MAX_GROUP) return MACKO_E_INVALID_ARG;
    total += phase_sizes[ph];
    if (total > MACKO_MAX_CHAIN_PRODUCTS) return MACKO_E_UNSUPPORTED;
  }
  for (int i = 0; i < total; ++i) {
    macko_handle_t h = handles[i];
    if (!h) return MACKO_E_INVALID_ARG;
    if (!h->bound) return MACKO_E_NOT_BOUND;
    int st = check_vec_ptrs(x_dev[i], y_dev[i], h->cols);
    if (st != MACKO_OK) return st;
    p[i] = macko::SpmvProblem{h->d_values, h->d_deltas, h->d_row_ptr, h->rows, h->cols, h->pad_nnz,
                              x_dev[i], y_dev[i], h->b_delta, h->b_val};
  }
  *total_out = total;
  return MACKO_OK;
}

uint32_t chain_wait_ticks() {
  const macko::Tuning& t = macko::tuning();
  if (t.chain_no_wait) return 0u;
  const int64_t us = t.chain_wait_us ? t.chain_wait_us : 1000000;      // default: one second
  return (uint32_t)(us * 100);                                          // the wall clock ticks at 100 MHz
}

int chain_status_of(uint32_t* scratch, hipStream_t s, int* failed_phase) {
  if (failed_phase) *failed_phase = -1;
  uint32_t* word = scratch + macko::chain_error_word();
  uint32_t err = 0;
  MACKO_HIP_TRY(hipStreamSynchronize(s));
  MACKO_HIP_TRY(hipMemcpy(&err, word, sizeof(err), hipMemcpyDeviceToHost));
  if (err == 0) return MACKO_OK;
  MACKO_HIP_TRY(hipMemset(word, 0, sizeof(err)));
  if (failed_phase) *failed_phase = (int)err - 1;
  return MACKO_E_WAIT_EXPIRED;
}

}  // namespace

int macko_spmv_chain(int n_phases, const int* phase_sizes, const macko_handle_t* handles, const void* const* x_dev,
                     void* const* y_dev, void* workspace_dev, int64_t workspace_bytes, void* stream) {
  macko::SpmvProblem p[MACKO_MAX_CHAIN_PRODUCTS];
  int total = 0;
  int st = chain_problems(n_phases, phase_sizes, handles, x_dev, y_dev, p, &total);
  if (st != MACKO_OK) return st;
  if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) || workspace_bytes < MACKO_CHAIN_WORKSPACE_BYTES)
    return MACKO_E_INVALID_ARG;
  return macko::launch_spmv_chain(n_phases, phase_sizes, p, static_cast<uint32_t*>(workspace_dev), chain_wait_ticks(),
                                  static_cast<hipStream_t>(stream));
}

int macko_spmv_chain_static(int n_phases, const int* phase_sizes, const macko_handle_t* handles,
                            const void* const* x_dev, void* const* y_dev, void* stream) {
  macko::SpmvProblem p[MACKO_MAX_CHAIN_PRODUCTS];
  int total = 0;
  int st = chain_problems(n_phases, phase_sizes, handles, x_dev, y_dev, p, &total);
  if (st != MACKO_OK) return st;
  uint32_t* scratch = nullptr;
  st = macko::chain_static_scratch(&scratch);
  if (st != MACKO_OK) return st;
  return macko::launch_spmv_chain(n_phases, phase_sizes, p, scratch, chain_wait_ticks(), static_cast<hipStream_t>(stream));
}

int macko_chain_status(void* workspace_dev, void* stream, int* failed_phase) {
  uint32_t* scratch = static_cast<uint32_t*>(workspace_dev);
  if (!scratch) {                                      // the library's own scratch
    int st = macko::chain_static_scratch(&scratch);
    if (st != MACKO_OK) return st;
  }
  return chain_status_of(scratch, static_cast<hipStream_t>(stream), failed_phase);
}

int macko_spmm(macko_handle_t h, int batch, const void* X_dev, int64_t ldx, void* Y_dev, int64_t ldy,
               void* stream) {
  if (!h || batch < 0 || batch > MACKO_MAX_BATCH) return MACKO_E_INVALID_ARG;
  if (!h->bound) return MACKO_E_NOT_BOUND;
  if (h->rows == 0 || batch == 0) return MACKO_OK;
  if (ldx < h->cols || ldy < h->rows) return MACKO_E_INVALID_ARG;
  int st = check_vec_ptrs(X_dev, Y_dev, h->cols);
  if (st != MACKO_OK) return st;
  macko::SpmvProblem p{h->d_values, h->d_deltas, h->d_row_ptr, h->rows, h->cols, h->pad_nnz, nullptr, nullptr,
                       h->b_delta, h->b_val};
  return macko::launch_spmm(p, X_dev, ldx, Y_dev, ldy, batch, static_cast<hipStream_t>(stream));
}

int macko_dense_gemv(const void* W_dev, int64_t rows, int64_t cols, int64_t ld, const void* x_dev,
                     void* y_dev, void* stream) {
  return macko_dense_gemv_group(1, &W_dev, &rows, &cols, &ld, &x_dev, &y_dev, stream);
}

int macko_dense_gemv_group(int n, const void* const* W_dev, const int64_t* rows, const int64_t* cols,
                           const int64_t* ld, const void* const* x_dev, void* const* y_dev, void* stream) {
  if (n < 1 || n > MACKO_MAX_GROUP || !W_dev || !rows || !cols || !ld || !x_dev || !y_dev)
    return MACKO_E_INVALID_ARG;
  macko::GemvProblem p[MACKO_MAX_GROUP];
  int m = 0;
  for (int i = 0; i < n; ++i) {
    if (rows[i] < 0 || cols[i] < 0 || ld[i] < cols[i]) return MACKO_E_INVALID_ARG;
    if (rows[i] == 0) continue;
    int st = check_vec_ptrs(x_dev[i], y_dev[i], cols[i]);
    if (st != MACKO_OK) return st;
    if (cols[i] > 0 && (!W_dev[i] || (reinterpret_cast<uintptr_t>(W_dev[i]) & 1))) return MACKO_E_INVALID_ARG;
    if (cols[i] >= (int64_t{1} << 31) || rows[i] >= (int64_t{1} << 31)) return MACKO_E_UNSUPPORTED;
    p[m++] = macko::GemvProblem{W_dev[i], rows[i], cols[i], ld[i], x_dev[i], y_dev[i]};
  }
  if (m == 0) return MACKO_OK;
  return macko::launch_gemv_group(m, p, static_cast<hipStream_t>(stream));
}

void macko_destroy(macko_handle_t h) {
  if (!h) return;
  if (h->owns_device && h->d_block) (void)hipFree(h->d_block);   // the three arrays are parts of it
  delete h;
}

const char* macko_status_string(int status) {
  switch (status) {
    case MACKO_OK: return "ok";
    case MACKO_E_INVALID_ARG: return "invalid argument";
    case MACKO_E_OVERFLOW: return "entry count does not fit 32-bit row pointers";
    case MACKO_E_UNSUPPORTED: return "unsupported";
    case MACKO_E_OUT_OF_MEMORY: return "out of memory";
    case MACKO_E_NOT_BOUND: return "handle has no device buffers";
    case MACKO_E_HIP: return "HIP error";
    case MACKO_E_CORRUPT: return "the device arrays are not a valid encoding";
    case MACKO_E_WAIT_EXPIRED: return "a chain's workgroups gave up waiting for each other; its results are incomplete";
    default: return "unknown status";
  }
}

int macko_last_hip_error(void) { return macko::g_last_hip_error; }

static int64_t* tuning_slot(const char* name) {
  if (!name) return nullptr;
  macko::Tuning& t = tuning();
  const std::string n(name);
  if (n == "spmv_kernel") return &t.spmv_kernel;
  if (n == "spmv_lanes") return &t.spmv_lanes;
  if (n == "spmv_block") return &t.spmv_block;
  if (n == "spmv_rows_per_wg") return &t.spmv_rows_per_wg;
  if (n == "spmv_ring") return &t.spmv_ring;
  if (n == "spmv_resident") return &t.spmv_resident;
  if (n == "spmv_wgs_per_cu") return &t.spmv_wgs_per_cu;
  if (n == "spmv_steps_per_wave") return &t.spmv_steps_per_wave;
  if (n == "spmv_resident_steps") return &t.spmv_resident_steps;
  if (n == "spmv_step_align") return &t.spmv_step_align;
  if (n == "chain_wait_us") return &t.chain_wait_us;
  if (n == "chain_no_wait") return &t.chain_no_wait;
  if (n == "gemv_resident") return &t.gemv_resident;
  if (n == "gemv_wgs_per_cu") return &t.gemv_wgs_per_cu;
  if (n == "gemv_block") return &t.gemv_block;
  if (n == "gemv_rows_per_wg") return &t.gemv_rows_per_wg;
  if (n == "gemv_ring") return &t.gemv_ring;
  return nullptr;
}

int macko_set_tuning(const char* name, int64_t value) {
  int64_t* slot = tuning_slot(name);
  if (!slot || value < 0) return MACKO_E_INVALID_ARG;
  const std::string n(name);
  if (n == "spmv_kernel" && value > 2) return MACKO_E_INVALID_ARG;
  if (n == "gemv_ring" && value != 0 && value != 2 && value != 4 && value != 8) return MACKO_E_INVALID_ARG;
  if (n == "spmv_ring" && value != 0 && (value < 2 || value > 4)) return MACKO_E_INVALID_ARG;
  if ((n == "spmv_resident" || n == "gemv_resident") && value > 2) return MACKO_E_INVALID_ARG;
  if ((n == "spmv_wgs_per_cu" || n == "gemv_wgs_per_cu") && value > 4) return MACKO_E_INVALID_ARG;
  if (n == "spmv_steps_per_wave" && value > 4096) return MACKO_E_INVALID_ARG;
  if (n == "spmv_resident_steps" && value > (int64_t{1} << 30)) return MACKO_E_INVALID_ARG;
  if (n == "spmv_step_align" && value != 0 && (value < 8 || value > 512 || (value & (value - 1)) != 0))
    return MACKO_E_INVALID_ARG;
  if (n == "chain_wait_us" && value > 40000000) return MACKO_E_INVALID_ARG;   // the tick count is 32 bits wide
  if (n == "chain_no_wait" && value > 1) return MACKO_E_INVALID_ARG;
  if (n == "spmv_lanes" && value != 0 && value != 16 && value != 32 && value != 64) return MACKO_E_INVALID_ARG;
  if ((n == "spmv_block" || n == "gemv_block") && value != 0 && (value % 64 != 0 || value > 1024))
    return MACKO_E_INVALID_ARG;
  if ((n == "spmv_rows_per_wg" || n == "gemv_rows_per_wg") && value > (int64_t{1} << 30))
    return MACKO_E_INVALID_ARG;
  *slot = value;
  return MACKO_OK;
}

int macko_get_tuning(const char* name, int64_t* value) {
  int64_t* slot = tuning_slot(name);
  if (!slot || !value) return MACKO_E_INVALID_ARG;
  *value = *slot;
  return MACKO_OK;
}

}  // extern "C"
