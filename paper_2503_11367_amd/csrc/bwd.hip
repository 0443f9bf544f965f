// placeholder until the backward kernels land
#include "attn_common.h"
namespace mm {
size_t bwd_workspace(int64_t, int64_t, int32_t, int32_t, int32_t) { return 256; }
int launch_bwd(const AttnArgs&, const void*, const float*, const void*, void*, void*, void*, void*,
               hipStream_t) { return MMATTN_ERR_UNSUPPORTED; }
}
