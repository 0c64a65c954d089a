// Host side of the C ABI: argument checks, workspace carve-up and the kernel sequence of
// tq_moe_forward.  Nothing here allocates, frees or synchronises.
#include "tq_common.h"

extern "C" const char* tq_status_str(tq_status s)
{
    switch (s) {
        case TQ_OK: return "ok";
        case TQ_ERR_NULL: return "null pointer";
        case TQ_ERR_SHAPE: return "bad shape";
        case TQ_ERR_ALIGN: return "misaligned pointer";
        case TQ_ERR_RANGE: return "value out of range";
        case TQ_ERR_WORKSPACE: return "buffer too small";
        case TQ_ERR_UNSUPPORTED: return "unsupported";
        case TQ_ERR_HIP: return "HIP error";
        case TQ_ERR_BLOB: return "packed blob does not match descriptor";
    }
    return "unknown status";
}

namespace {
hipEvent_t g_stage_events[TQ_N_STAGE_EVENTS];
int g_n_stage_events = 0;
}  // namespace

void tqi_record_stage(int stage, hipStream_t stream)
{
    if (stage < g_n_stage_events && g_stage_events[stage]) (void)hipEventRecord(g_stage_events[stage], stream);
}

extern "C" tq_status tq_set_profile_events(void* const* events, int32_t n)
{
    if (n < 0 || n > TQ_N_STAGE_EVENTS) return TQ_ERR_SHAPE;
    if (n > 0 && !events) return TQ_ERR_NULL;
    for (int i = 0; i < n; ++i) g_stage_events[i] = (hipEvent_t)events[i];
    g_n_stage_events = n;
    return TQ_OK;
}

extern "C" size_t tq_moe_workspace_size(const tq_layer_desc* desc, int32_t T)
{
    TqLayout L;
    if (!tq_make_layout(desc, &L) || T < 0) return 0;
    if ((int64_t)T * (L.k + L.S) > 0x3FFFFFFF) return 0;
    TqWorkspace W;
    tq_make_workspace(L, desc->act_dtype, T, &W);
    return W.total;
}

extern "C" tq_status tq_moe_forward(const tq_layer_desc* desc, const void* packed, const void* x,
                                    const int32_t* topk_idx, const float* topk_w, int32_t T, void* y,
                                    void* workspace, size_t workspace_bytes, void* stream)
{
    if (!desc || !packed || !x || !topk_idx || !topk_w || !y || !workspace) return TQ_ERR_NULL;
    TqLayout L;
    if (!tq_make_layout(desc, &L) || T < 0) return TQ_ERR_SHAPE;
    if ((int64_t)T * (L.k + L.S) > 0x3FFFFFFF) return TQ_ERR_SHAPE;
    if (((uintptr_t)packed | (uintptr_t)workspace) & 255) return TQ_ERR_ALIGN;
    if (((uintptr_t)x | (uintptr_t)y | (uintptr_t)topk_idx | (uintptr_t)topk_w) & 15) return TQ_ERR_ALIGN;
    TqWorkspace W;
    tq_make_workspace(L, desc->act_dtype, T, &W);
    if (workspace_bytes < W.total) return TQ_ERR_WORKSPACE;
    if (T == 0) return TQ_OK;
    hipStream_t st = (hipStream_t)stream;
    uint8_t* ws = (uint8_t*)workspace;
    int32_t* ctrl = (int32_t*)(ws + W.ctrl);
    tqi_record_stage(0, st);
    tq_status rc = tqi_launch_permute(topk_idx, topk_w, T, L.E, L.S, L.k, (int32_t*)(ws + W.offsets),
                                      (int32_t*)(ws + W.slot_of), L.k + L.S, nullptr,
                                      (int32_t*)(ws + W.row_token), (float*)(ws + W.row_w),
                                      (int32_t*)(ws + W.tile_e), (int32_t*)(ws + W.tile_row0), W.rt_max, ctrl,
                                      ctrl, (int32_t*)(ws + W.hist), W.nblk, packed, &L, st);
    if (rc != TQ_OK) return rc;
    tqi_record_stage(1, st);
    if (desc->act_dtype == TQ_ACT_FP32)
        return tqi_forward_f32(L, W, (const uint8_t*)packed, (const float*)x, T, (float*)y, ws, st, topk_w);
    return tqi_forward_bf16(L, W, desc->flags, (const uint8_t*)packed, (const uint16_t*)x, T, (uint16_t*)y, ws, st,
                            topk_w);
}
