#include "common.h"
namespace sepattn {
size_t backward_bf16_workspace(const sepattn_params &) { return 256; }
int launch_backward_bf16(const sepattn_params &, const void *, const void *, const void *, const void *,
                         const float *, const void *, const int32_t *, const int32_t *, const int32_t *,
                         void *, void *, void *, void *, hipStream_t) { return SEPATTN_ERR_DTYPE; }
}
