// Schedules (placeholder).
#include "rov_internal.h"
extern "C" int rov_layer_step(int, const rov_gemm_desc*, int, const rov_attn_desc*, uint64_t,
                              uint64_t, uint64_t*, void*, void*) {
    return ROV_ERR_UNSUPPORTED;
}
extern "C" size_t rov_block_workspace_bytes(const rov_block_cfg*, int, int, int) { return 0; }
extern "C" int rov_block_forward(const rov_block_weights*, const void*, void*, int, int,
                                 const rov_block_cfg*, int, uint64_t, uint64_t, int, uint64_t*,
                                 uint64_t*, void*, size_t, void*, void*) {
    return ROV_ERR_UNSUPPORTED;
}
