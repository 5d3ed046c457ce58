/*
 * libmacko -- MACKO sparse matrix-vector product for AMD Instinct MI355X (gfx950).
 *
 * C ABI.  Implements the storage format of Section 4.1 of "MACKO: Sparse
 * Matrix-Vector Multiplication for Low Sparsity" (arXiv 2511.13061) for
 * b_val = 16 (fp16 values) and b_delta = 4 (4-bit delta-coded column
 * coordinates; 1, 2 and 8 bits through the _ex entry points, Appendix C), and
 * the product Y = M V of its Appendix A / Section 4.4, plus the dense fp16 GEMV
 * of Section 4.3 that the paper measures speedups against.  The _fp8 entry
 * points hold the same format with b_val = 8 (one byte per stored value).
 *
 * Conventions
 *   - Every function returns MACKO_OK (0) or a negative macko_status code; no
 *     C++ exception crosses this boundary.  On failure output handles are set
 *     to NULL and nothing is leaked.
 *   - "host" pointers are ordinary CPU memory, "dev" pointers are HIP device
 *     memory on the current device; `stream` is a hipStream_t passed as void*
 *     (NULL = the default stream).
 *   - fp16 data is passed as raw IEEE binary16 bit patterns (uint16_t).
 *   - Matrices are row-major; `ld` is the distance between rows in elements.
 *   - The kernels only enqueue work on `stream` and never synchronise, unless
 *     a function's comment says otherwise.
 *
 * Format layout (identical on host and device)
 *   values   uint16_t[alloc_nnz]   fp16 bits; +0 at padding entries and in the tail
 *                                  (uint8_t[alloc_nnz], E4M3 bits, with 8-bit values)
 *   deltas   uint8_t [alloc_nnz/2] entry k is the 4-bit code (delta-1) in byte k>>1,
 *                                  bits 4*(k&1) .. 4*(k&1)+3
 *   row_ptr  uint32_t[rows+1]      index of each row's first entry
 *   The delta of a row's first entry is its column + 1; a gap larger than 16 is
 *   bridged by zero-valued entries with delta 16 placed greedily.  An element
 *   is a zero iff its bits are +0 or -0.  alloc_nnz = pad_nnz rounded up to 32
 *   (both arrays are multiples of 16 bytes, Section 4.5).
 *   With b_delta bits per code (1, 2, 4 or 8): entry k is the code (delta-1) in
 *   bits [k*b_delta, (k+1)*b_delta) of the deltas array, low bits first (the
 *   "bit shifting" packing of Section 4.1); the largest delta is 2^b_delta; the
 *   array is alloc_nnz*b_delta/8 bytes and alloc_nnz = pad_nnz rounded up to
 *   128/b_delta entries (16 bytes of codes).
 */
#ifndef MACKO_H_
#define MACKO_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MACKO_API __attribute__((visibility("default")))

typedef enum macko_status {
  MACKO_OK = 0,
  MACKO_E_INVALID_ARG = -1,   /* NULL pointer, negative size, ld < cols, misaligned buffer */
  MACKO_E_OVERFLOW = -2,      /* alloc_nnz >= 2^32: does not fit the 32-bit row pointers    */
  MACKO_E_UNSUPPORTED = -3,   /* shape or option this build has no kernel for               */
  MACKO_E_OUT_OF_MEMORY = -4, /* host or device allocation failed                           */
  MACKO_E_NOT_BOUND = -5,     /* device operation on a handle that has no device buffers    */
  MACKO_E_HIP = -6,           /* a HIP call failed; see macko_last_hip_error()              */
  MACKO_E_CORRUPT = -7,       /* macko_check_device: the bound arrays are not a valid encoding */
  MACKO_E_WAIT_EXPIRED = -8   /* macko_chain_status: a chain's workgroups gave up waiting for each other */
} macko_status;

/* Opaque encoded matrix.  Created by the encode / wrap calls, released by
 * macko_destroy.  Immutable once bound, so concurrent macko_spmv calls on
 * different streams are allowed. */
typedef struct macko_matrix* macko_handle_t;

/* Storage / padding report (Section 3.1 eq. 2, Section 4.2 eqs. 8-10). */
typedef struct macko_report {
  int64_t rows, cols;
  int64_t nnz;              /* non-zero elements of the dense input                    */
  int64_t pad_nnz;          /* stored entries = nnz + padding_entries                  */
  int64_t alloc_nnz;        /* pad_nnz rounded up to 32 (array tail padding)           */
  int64_t padding_entries;  /* zero entries inserted to keep every delta <= 16         */
  int64_t empty_rows;
  int64_t max_row_entries;  /* longest row, in stored entries                          */
  int64_t values_bytes, deltas_bytes, rowptr_bytes, total_bytes, dense_bytes;
  double density;           /* d = nnz / (rows*cols)                                   */
  double effd;              /* total_bytes / dense_bytes (eq. 2, row pointers included) */
  double effd_best;         /* eq. 8  at this d                                        */
  double effd_expected;     /* eq. 10 at this d                                        */
  double effd_worst;        /* eq. 9  at this d                                        */
  int32_t b_val, b_delta;   /* 16 (8 for the _fp8 calls); 4 unless an _ex call chose 1, 2 or 8 */
} macko_report_t;

/* ---- encoding (Section 4.1) ---------------------------------------------- */

/* Encode a dense fp16 matrix held in host memory.  The new handle owns host
 * copies of the three arrays; it has no device buffers until macko_bind_device.
 * `report` may be NULL.  rows == 0 or cols == 0 is valid. */
MACKO_API int macko_encode(const uint16_t* dense_host, int64_t rows, int64_t cols, int64_t ld,
                           macko_handle_t* out, macko_report_t* report);

/* Encode a dense fp16 matrix held in device memory, on the GPU.  The library
 * allocates the device arrays (one hipMalloc) and the handle owns them; the handle
 * is bound on return and keeps no host copy.  Synchronises `stream` (the sizes
 * of the outputs are only known after a counting pass).  The result is
 * bit-identical to macko_encode on the same input.  The encoder keeps one scratch
 * buffer per device between calls as long as it is at most 64 MiB (matrices of up
 * to about 100 M cells then encode without any allocation but the output's); a
 * larger one is released before the call returns.  One call at a time per process. */
MACKO_API int macko_encode_device(const void* dense_dev, int64_t rows, int64_t cols, int64_t ld,
                                  void* stream, macko_handle_t* out, macko_report_t* report);

/* Adopt device buffers that already hold an encoding (a copy made by the
 * caller, a loaded checkpoint).  The caller keeps ownership of the buffers and
 * must keep them alive while the handle is used.  values_dev and deltas_dev
 * must be 16-byte aligned, rowptr_dev 4-byte aligned; pad_nnz must equal
 * row_ptr[rows].  The contents are trusted, not validated. */
MACKO_API int macko_wrap_device(int64_t rows, int64_t cols, int64_t pad_nnz, const void* values_dev,
                                const void* deltas_dev, const void* rowptr_dev, macko_handle_t* out);

/* The same three calls for another code width b_delta in {1, 2, 4, 8} (Section
 * 4.1 allows exactly these; Appendix C: 2 bits store less below ~45 % sparsity,
 * 8 bits above ~95 %).  Everything else -- handles, binding, decode, the report,
 * macko_spmv, macko_spmv_group and macko_spmm -- works for every width.  Any
 * other b_delta is MACKO_E_INVALID_ARG. */
MACKO_API int macko_encode_ex(const uint16_t* dense_host, int64_t rows, int64_t cols, int64_t ld,
                              int b_delta, macko_handle_t* out, macko_report_t* report);

/* Storage of the matrix for every code width without encoding it (Section 4.2,
 * eq. 8 with the padding counted exactly instead of estimated; Appendix C):
 * total_bytes[i] = values + codes + row pointers for b_delta = 1, 2, 4, 8
 * (i = 0..3), as macko_report.total_bytes would give it, or -1 for a width
 * whose entry count does not fit 32-bit row pointers.  *best_b_delta (may be
 * NULL) is the width with the fewest bytes, the paper's 4 bits on a tie with
 * it, else the narrower one; 0 if no width fits.  dense_host as for
 * macko_encode; one pass over the matrix per width. */
MACKO_API int macko_storage_by_code_width(const uint16_t* dense_host, int64_t rows, int64_t cols, int64_t ld,
                                          int64_t total_bytes[4], int* best_b_delta);
MACKO_API int macko_encode_device_ex(const void* dense_dev, int64_t rows, int64_t cols, int64_t ld,
                                     int b_delta, void* stream, macko_handle_t* out,
                                     macko_report_t* report);
MACKO_API int macko_wrap_device_ex(int64_t rows, int64_t cols, int64_t pad_nnz, int b_delta,
                                   const void* values_dev, const void* deltas_dev,
                                   const void* rowptr_dev, macko_handle_t* out);

/* Copy of the report computed at encode time (for wrapped handles only the
 * size fields are known; nnz-derived fields are -1 / NaN). */
MACKO_API int macko_get_report(macko_handle_t h, macko_report_t* report);

/* Bytes the caller must provide to macko_bind_device for each array. */
MACKO_API int macko_device_bytes(macko_handle_t h, int64_t* values_bytes, int64_t* deltas_bytes,
                                 int64_t* rowptr_bytes);

/* Attach caller-owned device buffers (each at least as large as reported by
 * macko_device_bytes; values_dev and deltas_dev 16-byte aligned) and copy the
 * encoding into them: the three host-to-device copies are enqueued on `stream`
 * and the call then SYNCHRONISES `stream` (the host arrays are ordinary pageable
 * memory, so the copies are staged by the runtime; on return the device arrays
 * are complete and the handle is bound).  A one-time set-up call, not part of
 * the product path.  The buffers must outlive the handle's use. */
MACKO_API int macko_bind_device(macko_handle_t h, void* values_dev, void* deltas_dev,
                                void* rowptr_dev, void* stream);

/* ---- 8-bit values ---------------------------------------------------------- */

/* The format with b_val = 8: one byte per stored value instead of two (Section
 * 4.1 defines the format for any b_val; Section 6 names 8-bit values as a
 * setting whose kernel is left to future work, and does not say what an 8-bit
 * value is).  Reading taken: a value is a number of the OCP 8-bit floating
 * point format E4M3 (1 sign, 4 exponent, 3 fraction bits, bias 7, no
 * infinities, S.1111.111 = NaN, largest finite value 448); scaling, if any, is
 * the caller's (y can be scaled per row afterwards).  An element is a zero when
 * its bits other than the sign are 0; padding entries hold 0x00.  Coordinates
 * (4-bit codes), row pointers and tail padding are those of the 16-bit format.
 *
 * dense_host: uint8 [rows x ld] E4M3 bit patterns, row-major.  The handle
 * behaves like any other: macko_device_bytes (values: alloc_nnz bytes),
 * macko_bind_device, macko_fetch_device (values_host then receives bytes),
 * macko_get_report (b_val = 8; effd and dense_bytes relative to a dense 8-bit
 * matrix), macko_spmv / macko_spmv_group (x and y stay fp16, fp32
 * accumulation; the wave-per-row kernel serves every row length; x must fit
 * LDS, about 78 K columns, otherwise MACKO_E_UNSUPPORTED), macko_columns_device,
 * macko_check_device, macko_decode_device (the dense matrix as bytes),
 * macko_spmm (the same batch kernel as for 16-bit values: the matrix is read and
 * decoded once per piece of up to 8 vectors).
 * macko_decode and macko_host_buffers' `values` are MACKO_E_UNSUPPORTED for
 * such a handle (macko_decode_fp8, macko_host_values_fp8 instead). */
MACKO_API int macko_encode_fp8(const uint8_t* dense_host, int64_t rows, int64_t cols, int64_t ld,
                               macko_handle_t* out, macko_report_t* report);
/* macko_encode_device for a dense matrix of 8-bit values in device memory (uint8 [rows x ld]);
 * same contract, bit-identical to macko_encode_fp8; the encoder's scratch holds 3 bytes per
 * stored entry for such a call. */
MACKO_API int macko_encode_device_fp8(const void* dense_dev, int64_t rows, int64_t cols, int64_t ld, void* stream,
                                      macko_handle_t* out, macko_report_t* report);
/* macko_wrap_device for arrays that hold 8-bit values (values_dev: alloc_nnz bytes,
 * 16-byte aligned; 4-bit codes).  Same rules: trusted, not validated, caller owned. */
MACKO_API int macko_wrap_device_fp8(int64_t rows, int64_t cols, int64_t pad_nnz, const void* values_dev,
                                    const void* deltas_dev, const void* rowptr_dev, macko_handle_t* out);
/* Host copy of the values of a macko_encode_fp8 handle (borrowed, alloc_nnz bytes). */
MACKO_API int macko_host_values_fp8(macko_handle_t h, const uint8_t** values);
/* Decode the host copy back to a dense rows x cols matrix of 8-bit values. */
MACKO_API int macko_decode_fp8(macko_handle_t h, uint8_t* dense_host_out, int64_t ld);

/* Borrowed pointers to the host arrays (valid until macko_destroy); any output
 * pointer may be NULL.  MACKO_E_UNSUPPORTED for handles without host copies. */
MACKO_API int macko_host_buffers(macko_handle_t h, const uint16_t** values, const uint8_t** deltas,
                                 const uint32_t** row_ptr);

/* Copy the bound device arrays back into caller-provided host memory of the
 * sizes reported by macko_device_bytes.  Synchronous. */
MACKO_API int macko_fetch_device(macko_handle_t h, uint16_t* values_host, uint8_t* deltas_host,
                                 uint32_t* rowptr_host);

/* Decode the host copy back to a dense rows x cols fp16 matrix (the format is
 * lossless; -0 inputs come back as +0). */
MACKO_API int macko_decode(macko_handle_t h, uint16_t* dense_host_out, int64_t ld);

/* Check, on the device, what the kernels take on trust about bound arrays
 * (meant for macko_wrap_device: a loaded checkpoint, a copy made elsewhere):
 * row_ptr[0] == 0, row_ptr never decreases, row_ptr[rows] == pad_nnz, and no
 * entry decodes to a column >= cols (Section 4.1: a column is the sum of the
 * row's deltas).  Returns MACKO_OK, or MACKO_E_CORRUPT with the smallest
 * offending row in *first_bad_row (may be NULL).  Rows with bad pointers are
 * reported without being decoded, so the check reads nothing outside the
 * arrays' pad_nnz entries and rows + 1 pointers.  Synchronises `stream`;
 * allocates and frees 4 bytes of device memory. */
MACKO_API int macko_check_device(macko_handle_t h, void* stream, int64_t* first_bad_row);

/* ---- expanding the format on the device ----------------------------------- */

/* Column index of every stored entry, computed on the device as the product
 * computes it (Section 4.4: the running sum of a row's deltas, formed per lane
 * and across the wavefront as in Algorithm 1).  Together with the values
 * array and the row pointers this is the matrix in CSR form, padding entries
 * included as explicit zeros at the column where they sit.
 * cols_dev: int32[alloc_nnz] on the device, 4-byte aligned, caller owned;
 * entries [0, pad_nnz) are written, the tail is left untouched.  The handle
 * must be bound.  Only enqueues on `stream`. */
MACKO_API int macko_columns_device(macko_handle_t h, int32_t* cols_dev, void* stream);

/* The dense rows x cols matrix back from the bound device arrays (the format
 * is lossless, Section 5.2; -0 inputs come back as +0).
 * dense_dev: fp16 [rows x ld] on the device (uint8 [rows x ld] for a matrix
 * with 8-bit values, at most 163840 columns), ld >= cols elements, aligned to
 * its element size (16-byte aligned with rows of a multiple of 16 bytes for
 * full-width stores), caller owned, must not overlap the format arrays.  Cells [r][0, cols)
 * are overwritten, cells between cols and ld are left untouched.  Enqueues one
 * kernel on `stream` (two for rows of more than 81920 columns) and does not
 * synchronise. */
MACKO_API int macko_decode_device(macko_handle_t h, void* dense_dev, int64_t ld, void* stream);

/* ---- the product (Section 4.4; Y = M V of Appendix A) --------------------- */

/* y[r] = sum_k values[k] * x[column(k)] over row r's entries, fp32
 * accumulation, result rounded to fp16 (round to nearest even).
 * x_dev: fp16[cols], y_dev: fp16[rows], both on the device, 2-byte aligned
 * (16-byte aligned x takes the fast staging path); they must not alias each
 * other or the format arrays.  y is overwritten.  Enqueues one kernel. */
MACKO_API int macko_spmv(macko_handle_t h, const void* x_dev, void* y_dev, void* stream);

/* Dense fp16 GEMV y = W x with fp32 accumulation (SplitK over lanes of a
 * wavefront, Section 4.3): the baseline the sparse product is compared with.
 * W_dev: fp16, rows x cols, row-major with leading dimension ld. */
MACKO_API int macko_dense_gemv(const void* W_dev, int64_t rows, int64_t cols, int64_t ld,
                               const void* x_dev, void* y_dev, void* stream);

/* Small-batch product with one matrix (the matrix is streamed and decoded once per piece of
 * up to 8 vectors, for every code width and both value widths; rows shorter than 384
 * stored entries on average, and batches whose interleaved vectors do not fit LDS, run
 * as independent matrix-vector products instead).  From batch 8 on the kernel is bound
 * by vector arithmetic, not by memory: on the Llama2-7B shapes at 50 % sparsity the
 * vendor library's dense fp16 GEMM on the decoded matrix (macko_decode_device) is as
 * fast at batch 8 and faster beyond; this call is meant for batch 2 to 8.
 * Y[b][r] = sum_k values[k] * X[b][column(k)] for b < batch, 0 <= batch <= MACKO_MAX_BATCH.
 * X_dev: fp16, batch vectors of `cols` elements, vector b at X_dev + b*ldx
 * (ldx >= cols); Y_dev: fp16, vector b at Y_dev + b*ldy (ldy >= rows).  fp32
 * accumulation, fp16 results.  The paper names small-batch products as future
 * work (Section 7); the format and the accuracy contract are those of macko_spmv. */
#define MACKO_MAX_BATCH 64
MACKO_API int macko_spmm(macko_handle_t h, int batch, const void* X_dev, int64_t ldx, void* Y_dev,
                         int64_t ldy, void* stream);

/* Grouped forms: n independent products (1 <= n <= MACKO_MAX_GROUP) enqueued
 * with as few kernel launches as possible -- one, when every matrix takes the
 * wavefront-per-row kernel.  Intended for products that share an input or have
 * no dependence on each other (q/k/v, gate/up of a decoder layer): a dependent
 * kernel launch costs about 3 us on this hardware, as much as streaming a
 * 4096 x 4096 matrix at 50 % sparsity.  No ordering is guaranteed among the n
 * products; the y vectors must not alias each other or any x.  Argument
 * meaning per product is that of the single-product call. */
#define MACKO_MAX_GROUP 8
MACKO_API int macko_spmv_group(int n, const macko_handle_t* handles, const void* const* x_dev,
                               void* const* y_dev, void* stream);

/* Any number of independent products (the linear layers of a whole stack, one
 * x and one y each): grouped launches of up to MACKO_MAX_GROUP consecutive
 * products, dealt in turn to three side streams that the library keeps per
 * device, so that the end of one launch overlaps the start of the next (a
 * launch costs about 3 us whatever its size; on one stream 128 launches of a
 * 13B-shaped stack take 2.54 ms, dealt out like this 2.1 ms).  The side
 * streams start after the work already enqueued on `stream`, and `stream`
 * continues after all of them (event fork / join, no host synchronisation, so
 * the call can be captured into a graph).  No ordering among the products; the
 * y vectors must not alias each other or any x.  n <= MACKO_MAX_GROUP is
 * macko_spmv_group.  Calls are serialised by a mutex while they enqueue. */
MACKO_API int macko_spmv_many(int64_t n, const macko_handle_t* handles, const void* const* x_dev,
                              void* const* y_dev, void* stream);
/* A chain of dependent products in ONE kernel launch (the linear layers of a decoder
 * layer in the order a decoding step needs them, Appendix B and Section 5.2:
 * {q,k,v} -> {o} -> {gate,up} -> {down}).  n_phases phases; phase p holds
 * phase_sizes[p] independent products (1 .. MACKO_MAX_GROUP); handles, x_dev and
 * y_dev list the products phase by phase.  Every product of phase p is complete,
 * and its y visible, before any product of phase p + 1 reads its x: the x of a
 * later phase may be the y of an earlier one.  Within a phase the rules of
 * macko_spmv_group apply.  Per product the arithmetic is that of macko_spmv.
 *
 * How: a single resident round of workgroups that walk the phases together.  The
 * matrix arrays of the next phase are requested before a workgroup waits for the
 * others, so only x is on the dependent path; a kernel boundary between two
 * dependent products costs about 3 us otherwise.
 *
 * Limits (MACKO_E_UNSUPPORTED otherwise): at most MACKO_MAX_CHAIN_PHASES phases
 * and MACKO_MAX_CHAIN_PRODUCTS products; fp16 values; 2- or 4-bit codes, the same
 * for all; no empty matrix; x of every product fits LDS next to another
 * workgroup's; at most 64 rows per wavefront of the round (about 1.6 M rows per
 * phase on 256 compute units); the device can hold the whole round at once.
 *
 * workspace_dev: MACKO_CHAIN_WORKSPACE_BYTES of device memory, 256-byte aligned,
 * caller owned, zero before the first call; every call leaves it zero again
 * (except the error word, see macko_chain_status).  Calls that share a workspace
 * must not overlap in time.  While a chain runs on a device, kernels on other
 * streams that occupy compute units for long delay it: its workgroups wait for
 * each other at most "chain_wait_us" microseconds (macko_set_tuning; default one
 * second), then the remaining phases are skipped, the kernel ends normally, and
 * macko_chain_status reports it.  Two chains must never run at the same time on one
 * device: each could hold the compute units the other is waiting for.
 * Only enqueues on `stream`; allocates nothing. */
#define MACKO_MAX_CHAIN_PHASES 8
#define MACKO_MAX_CHAIN_PRODUCTS 16
#define MACKO_CHAIN_WORKSPACE_BYTES 8192
MACKO_API int macko_spmv_chain(int n_phases, const int* phase_sizes, const macko_handle_t* handles,
                               const void* const* x_dev, void* const* y_dev, void* workspace_dev,
                               int64_t workspace_bytes, void* stream);

/* macko_spmv_chain for callers that can neither allocate nor hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and limits without workspace_dev: the 8 KB of scratch
 * memory (MACKO_CHAIN_WORKSPACE_BYTES) are a static array in the library's device
 * code, one copy per GPU, held until the process ends, zero when the library is
 * loaded and left zero by every call.  The call allocates nothing on the host or the
 * device (the first call on a device looks the array's address up and asks the
 * runtime for the kernel's resource use: make that call outside a graph capture;
 * later calls can be captured, the launch records one kernel node and no memset).  More than
 * MACKO_MAX_CHAIN_PHASES phases or MACKO_MAX_CHAIN_PRODUCTS products do not fit the
 * scratch layout and the kernel's argument block: MACKO_E_UNSUPPORTED.  Every call on
 * a GPU shares that GPU's array: calls that overlap in time on one GPU race (the
 * bounded wait of the chain then ends them with MACKO_E_WAIT_EXPIRED at best, wrong
 * results at worst); calls in stream order on one stream, or otherwise ordered, are
 * fine.  macko_chain_status(NULL, ...) reports on this scratch. */
MACKO_API int macko_spmv_chain_static(int n_phases, const int* phase_sizes, const macko_handle_t* handles,
                                      const void* const* x_dev, void* const* y_dev, void* stream);

/* Whether any chain that used workspace_dev (NULL: the library's own scratch of
 * macko_spmv_chain_static on the current device) since the last call of this function
 * gave up waiting: MACKO_OK, or MACKO_E_WAIT_EXPIRED with the phase (0-based) whose
 * inputs were not ready in *failed_phase (may be NULL); the results of that chain are
 * incomplete.  Synchronises `stream` and clears the record. */
MACKO_API int macko_chain_status(void* workspace_dev, void* stream, int* failed_phase);
MACKO_API int macko_dense_gemv_group(int n, const void* const* W_dev, const int64_t* rows,
                                     const int64_t* cols, const int64_t* ld, const void* const* x_dev,
                                     void* const* y_dev, void* stream);

/* ---- housekeeping ---------------------------------------------------------- */

MACKO_API void macko_destroy(macko_handle_t h);

MACKO_API const char* macko_status_string(int status);

/* hipError_t of the most recent failing HIP call on this thread (0 if none). */
MACKO_API int macko_last_hip_error(void);

/* Launch-shape knobs for experiments; every value has a safe default and out
 * of range values are rejected with MACKO_E_INVALID_ARG.
 *   "spmv_kernel"       0 auto, 1 generic sub-wave kernel, 2 wave-per-row kernel
 *   "spmv_lanes"        0 auto, else lanes per row for the generic kernel (16/32/64)
 *   "spmv_block"        threads per workgroup for spmv (multiple of 64, <= 1024), 0 auto
 *   "spmv_rows_per_wg"  rows handled by one workgroup, 0 auto
 *   "spmv_ring"         steps of loads kept in flight per wavefront (2 or 4), 0 auto
 *   "spmv_resident"     0 auto, 1 never, 2 always: launch exactly one resident round of
 *                       workgroups (a multiple of the compute-unit count) shaped to the row counts
 *   "spmv_wgs_per_cu"   workgroups per compute unit of such a round (1..4), 0 auto
 *   "spmv_resident_steps"  largest launch, in wavefront steps (512 entries) per compute unit,
 *                       that "spmv_resident" = 0 runs as one resident round, 0 default
 *   "spmv_steps_per_wave"  larger launches: steps of work per wavefront, 0 default
 *   "spmv_step_align"   stored entries that the first step of every row is aligned to in the
 *                       wave-per-row kernel (power of two, 8..512), 0 auto (by row length)
 *   "chain_wait_us"     longest wait of a chain's workgroups for each other, in microseconds
 *                       (at most 40,000,000), 0 default (one second)
 *   "chain_no_wait"     1: such a wait gives up at once when the phase before is unfinished (for
 *                       tests of the give-up path; the chain then reports MACKO_E_WAIT_EXPIRED)
 *   "gemv_block", "gemv_rows_per_wg", "gemv_ring" (2, 4 or 8), "gemv_resident",
 *   "gemv_wgs_per_cu"   the same for the dense GEMV
 * Settings are process wide and not thread safe: macko_set_tuning must not run
 * at the same time as any call that launches a kernel (macko_spmv, macko_spmv_group,
 * macko_spmv_many, macko_spmv_chain*, macko_spmm, macko_dense_gemv*) on another host
 * thread; those calls read the settings without locking.  With all knobs at 0, which
 * is the state of a process that never calls macko_set_tuning, the launching calls
 * may run concurrently on any number of host threads (macko_spmv_many and
 * macko_encode_device serialise themselves). */
MACKO_API int macko_set_tuning(const char* name, int64_t value);
MACKO_API int macko_get_tuning(const char* name, int64_t* value);

#ifdef __cplusplus
}
#endif
#endif /* MACKO_H_ */
