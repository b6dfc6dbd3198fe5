// Stand-ins for the device side of the library (kernels.hip) in the sanitizer build of the host
// side: host-only plans never launch anything, so every entry here reports "not available".
#include "../../paper_2212_10432_amd/csrc/internal.h"

namespace spmv {

int launch_part(const Part &, spmv_dtype_t, int64_t, int64_t, const void *, void *, void *, void *, void *) { return 1; }
int launch_part_multi(const Part &, spmv_dtype_t, int64_t, int64_t, const void *, int64_t, void *, int64_t, int, void *) { return 1; }
int launch_jit(const Part &, spmv_dtype_t, int64_t, int64_t, const void *, void *, void *, void *, void *) { return 1; }
int prepare_device() { return 1; }
int static_scratch(void **) { return 1; }
int stream_ceiling(size_t, int, void *, double *, double *) { return 1; }
int flush_read(void *, size_t, void *) { return 1; }
const char *hip_error_text(int) { return "no device code in the sanitizer build"; }

}  // namespace spmv
