// Dense-training forward and backward (paper Sec. 3.2 "Dense Training", Eq. 3).
#include "gemm_core.h"

namespace dsmoe {

size_t dense_saved_bytes(const dsmoe_ctx* c, int T) { (void)c; (void)T; return 0; }
size_t dense_bwd_scratch_bytes(const dsmoe_ctx* c, int T) { (void)c; (void)T; return 0; }

hipError_t launch_dense_fwd(const dsmoe_ctx*, const void*, const void*, const void*, const void*, const void*,
                            const void*, int, void*, float*, void*, hipStream_t) {
  return hipErrorNotSupported;
}
hipError_t launch_dense_bwd(const dsmoe_ctx*, const void*, const void*, const void*, const void*, const void*,
                            const void*, const void*, int, void*, void*, float*, float*, float*, float*, float*,
                            hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace dsmoe
