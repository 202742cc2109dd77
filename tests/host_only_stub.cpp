// Stand-ins for the entry points that launch kernels, for a build of the host logic alone
// (composer, planner, plan checker, graph and layout passes) with the host compiler under
// AddressSanitizer / UndefinedBehaviorSanitizer.  Every one of them reports AMAP_E_HIP, as the
// real ones do on a machine without a GPU.  Test infrastructure: not part of libamap.so.
#include "amap.h"

extern "C" {
amap_status amap_execute(const void *const *, void *, const amap_t *, void *) { return AMAP_E_HIP; }
amap_status amap_execute_kernel(const void *const *, void *, const amap_t *, void *, int) { return AMAP_E_HIP; }
amap_status amap_execute_multi(const void *const *, void *const *, const amap_t *const *, int, void *) { return AMAP_E_HIP; }
amap_status amap_gemm_fused(const void *, const amap_t *, const void *, int64_t, void *, void *) { return AMAP_E_HIP; }
amap_status amap_gemm_fused_store(const void *, const amap_t *, const void *, int64_t, const amap_t *, void *, void *) { return AMAP_E_HIP; }
amap_status amap_gemm_mapped(const void *, const amap_t *, const void *, const amap_t *, const amap_t *, void *, void *) { return AMAP_E_HIP; }
amap_status amap_gemm_gather(const void *const *, const amap_t *, const void *, const amap_t *, int64_t, const amap_t *, void *, void *) { return AMAP_E_HIP; }
amap_status amap_gemm_selfcheck(const amap_t *, const amap_t *, int64_t, const amap_t *, int, int64_t *) { return AMAP_E_HIP; }
}
