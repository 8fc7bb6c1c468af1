// vmoba_workspace_bytes: sizes of the caller-provided workspaces.
#include "common.h"

size_t vmoba_select_workspace_bytes(int B, int Hh, int64_t S, int nb);
size_t vmoba_attn_fwd_workspace_bytes(int B, int Hh, int64_t S, int D, int64_t cap, int dtype);
size_t vmoba_attn_bwd_workspace_bytes(int B, int Hh, int64_t S, int D, int64_t cap, int dtype);

extern "C" size_t vmoba_workspace_bytes(int op, int B, int Hh, int64_t S, int D, int32_t n_blocks,
                                        int64_t nnz_capacity, int dtype) {
    if (B <= 0 || Hh <= 0 || S <= 0 || n_blocks <= 0 || D <= 0 || nnz_capacity < 0) return 0;
    switch (op) {
        case VMOBA_OP_SELECT: return vmoba_select_workspace_bytes(B, Hh, S, n_blocks);
        case VMOBA_OP_ATTN_FWD: return vmoba_attn_fwd_workspace_bytes(B, Hh, S, D, nnz_capacity, dtype);
        case VMOBA_OP_ATTN_BWD: return vmoba_attn_bwd_workspace_bytes(B, Hh, S, D, nnz_capacity, dtype);
        default: return 0;
    }
}

ProfileSlot g_profile[4] = {};

extern "C" int vmoba_profile_events(int slot, void* start_event, void* stop_event) {
    if (slot < 0 || slot >= 4) return VMOBA_ERR_INVALID_ARG;
    g_profile[slot].start = (hipEvent_t)start_event;
    g_profile[slot].stop = (hipEvent_t)stop_event;
    return VMOBA_OK;
}
