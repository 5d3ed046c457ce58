// Stand-ins for the GPU launchers of libmacko, so that its host translation unit (encoders,
// decoders, storage report, argument checks) can be linked into a CPU-only program and run under
// AddressSanitizer / UndefinedBehaviorSanitizer (tests/host_sanitizer_check.cpp).  None of them
// may be reached by that program: each aborts.
#include <cstdio>
#include <cstdlib>

#include "macko_internal.h"

namespace macko {
[[noreturn]] static void unreachable(const char* what) {
  std::fprintf(stderr, "host sanitizer check reached the GPU launcher %s\n", what);
  std::abort();
}
int launch_spmv_group(int, const SpmvProblem*, hipStream_t) { unreachable("launch_spmv_group"); }
int launch_gemv_group(int, const GemvProblem*, hipStream_t) { unreachable("launch_gemv_group"); }
int launch_spmv_chain(int, const int*, const SpmvProblem*, uint32_t*, uint32_t, hipStream_t) {
  unreachable("launch_spmv_chain");
}
int chain_static_scratch(uint32_t**) { unreachable("chain_static_scratch"); }
int launch_spmm(const SpmvProblem&, const void*, int64_t, void*, int64_t, int, hipStream_t) { unreachable("launch_spmm"); }
int launch_columns(const SpmvProblem&, int32_t*, hipStream_t) { unreachable("launch_columns"); }
int launch_check(const SpmvProblem&, unsigned int*, hipStream_t) { unreachable("launch_check"); }
int launch_decode(const SpmvProblem&, void*, int64_t, hipStream_t) { unreachable("launch_decode"); }
int encode_on_device(const void*, int64_t, int64_t, int64_t, int, int, hipStream_t, void**, void**, uint8_t**,
                     uint32_t**, int64_t*, int64_t*, int64_t*, int64_t*, int64_t*) {
  unreachable("encode_on_device");
}
}  // namespace macko
