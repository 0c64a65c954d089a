#include "tq_common.h"
tq_status tqi_forward_bf16(const TqLayout& L, const TqWorkspace& W, int flags, const uint8_t* blob,
                           const uint16_t* x, int32_t T, uint16_t* y, uint8_t* ws, hipStream_t stream,
                           const float* topk_w)
{
    return TQ_ERR_UNSUPPORTED;
}
