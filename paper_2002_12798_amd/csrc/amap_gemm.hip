// placeholder until the fused GEMM lands
#include "amap_map.hpp"
extern "C" amap_status amap_gemm_fused(const void *, const amap_t *, const void *, int64_t, void *, void *) {
    return AMAP_E_UNSUPPORTED;
}
