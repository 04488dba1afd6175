// placeholder until the dequant + MFMA comparison kernel lands
#include "msgemm_internal.h"
namespace msgemm {
int launch_dequant_mfma(const Plan&, const void*, int64_t, void*, int64_t, hipStream_t) { return MSGEMM_ERR_UNSUPPORTED; }
}
