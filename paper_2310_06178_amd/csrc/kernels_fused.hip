// placeholder until the fused LDS kernels land
#include "msgemm_internal.h"
namespace msgemm {
int fused_choose_shape(Plan&) { return MSGEMM_ERR_UNSUPPORTED; }
int launch_repack(const Plan&, hipStream_t) { return MSGEMM_ERR_UNSUPPORTED; }
int launch_fused(const Plan&, const void*, int64_t, void*, int64_t, hipStream_t) { return MSGEMM_ERR_UNSUPPORTED; }
}
