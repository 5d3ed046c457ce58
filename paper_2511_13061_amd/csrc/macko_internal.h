// Internal declarations shared by the translation units of libmacko.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "macko.h"

namespace macko {

constexpr int kDeltaBits = 4;           // default b_delta
// entries per 16 bytes of packed codes: both arrays are padded to a multiple of this
constexpr int64_t alloc_granule(int b_delta) { return 128 / b_delta; }

struct Tuning {
  int64_t spmv_kernel = 0;
  int64_t spmv_lanes = 0;
  int64_t spmv_block = 0;
  int64_t spmv_rows_per_wg = 0;
  int64_t spmv_ring = 0;
  int64_t spmv_resident = 0;      // 0 auto, 1 never, 2 always one resident round of workgroups
  int64_t spmv_wgs_per_cu = 0;    // resident round: workgroups per compute unit (0 = planner's choice)
  int64_t spmv_steps_per_wave = 0; // many-workgroup regime: steps of work per wavefront (0 = default)
  int64_t spmv_step_align = 0;     // entries a row's first step is aligned to (8 ... 512, power of two; 0 = by row length)
  int64_t spmv_resident_steps = 0; // largest work (steps per compute unit) launched as one resident round (0 = default)
  int64_t chain_wait_us = 0;       // longest wait of a chain's workgroups for each other (0 = default, -1 = none)
  int64_t chain_no_wait = 0;       // 1: such a wait gives up at once when the phase before is unfinished
  int64_t gemv_block = 0;
  int64_t gemv_rows_per_wg = 0;
  int64_t gemv_ring = 0;
  int64_t gemv_resident = 0;
  int64_t gemv_wgs_per_cu = 0;
};
Tuning& tuning();

// record a failing HIP call for macko_last_hip_error()
int hip_fail(hipError_t e);
#define MACKO_HIP_TRY(expr)                                   \
  do {                                                        \
    hipError_t e__ = (expr);                                  \
    if (e__ != hipSuccess) return ::macko::hip_fail(e__);     \
  } while (0)

int device_cu_count();

// launchers implemented in the .hip files; all return a macko_status
constexpr int kMaxGroup = 8;            // MACKO_MAX_GROUP

struct SpmvProblem {
  const uint16_t* values;
  const uint8_t* deltas;
  const uint32_t* row_ptr;
  int64_t rows, cols, pad_nnz;
  const void* x;
  void* y;
  int b_delta = kDeltaBits;
  int b_val = 16;           // bits per value: 16 (fp16) or 8 (E4M3)
};
struct GemvProblem {
  const void* W;
  int64_t rows, cols, ld;
  const void* x;
  void* y;
};
// n independent products, as few kernel launches as the shapes allow (1 <= n <= kMaxGroup)
int launch_spmv_group(int n, const SpmvProblem* problems, hipStream_t stream);
int launch_gemv_group(int n, const GemvProblem* problems, hipStream_t stream);
// phases of products in one launch, phase p + 1 after phase p: sizes[p] products in phase p, listed in
// phase order; `scratch` is chain_scratch_bytes() of zeroed device memory that the launch leaves zeroed
int launch_spmv_chain(int n_phases, const int* sizes, const SpmvProblem* problems, uint32_t* scratch,
                      uint32_t wait_ticks, hipStream_t stream);
constexpr int64_t chain_scratch_bytes() { return 8192; }
// device address, on the current device, of the library's own chain scratch (a static device array)
int chain_static_scratch(uint32_t** out);
constexpr int chain_error_word() { return 25 * 64; }
// batch products with one matrix: Y[b] = W X[b], vectors ldx / ldy elements apart (p.x, p.y unused)
int launch_spmm(const SpmvProblem& p, const void* X, int64_t ldx, void* Y, int64_t ldy, int batch,
                hipStream_t stream);
// device-side expansion: column index of every stored entry; the dense matrix back
int launch_columns(const SpmvProblem& p, int32_t* cols_out, hipStream_t stream);
// structural check of bound device arrays; *first_bad (device) must hold `rows` beforehand
int launch_check(const SpmvProblem& p, unsigned int* first_bad, hipStream_t stream);
int launch_decode(const SpmvProblem& p, void* dense, int64_t ld, hipStream_t stream);
// GPU encoder: counting pass + fill pass.  The three arrays are parts of one hipMalloc'd *block.
int encode_on_device(const void* dense, int64_t rows, int64_t cols, int64_t ld, int b_delta, int b_val,
                     hipStream_t stream, void** block,
                     void** values, uint8_t** deltas, uint32_t** row_ptr, int64_t* nnz,
                     int64_t* pad_nnz, int64_t* alloc_nnz, int64_t* empty_rows,
                     int64_t* max_row_entries);

void fill_report(macko_report_t* rep, int64_t rows, int64_t cols, int64_t nnz, int64_t pad_nnz,
                 int64_t alloc_nnz, int64_t empty_rows, int64_t max_row_entries, int b_delta, int b_val = 16);

}  // namespace macko

struct macko_matrix {
  int64_t rows = 0, cols = 0;
  int64_t pad_nnz = 0, alloc_nnz = 0;
  int b_delta = macko::kDeltaBits;
  int b_val = 16;            // 16: fp16 values; 8: OCP E4M3 values (h_values8 holds the host copy)
  macko_report_t report{};
  // host copy (empty for device-encoded and wrapped handles)
  bool has_host = false;
  std::vector<uint16_t> h_values;
  std::vector<uint8_t> h_values8;
  std::vector<uint8_t> h_deltas;
  std::vector<uint32_t> h_row_ptr;
  // device binding
  const uint16_t* d_values = nullptr;
  const uint8_t* d_deltas = nullptr;
  const uint32_t* d_row_ptr = nullptr;
  bool bound = false;
  bool owns_device = false;
  void* d_block = nullptr;   // owns_device: the one allocation that holds the three arrays
};
