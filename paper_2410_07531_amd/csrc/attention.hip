// Attention (placeholder until the kernel lands): reports ROV_ERR_UNSUPPORTED.
#include "rov_internal.h"
namespace rov {
int launch_attention(const void*, const void*, const void*, void*, int, int, int, int, int,
                     const int64_t*, int, int, float, const uint64_t*, uint64_t, uint64_t,
                     hipStream_t) {
    return ROV_ERR_UNSUPPORTED;
}
}  // namespace rov
extern "C" int rov_attention_fwd_dropout(const void* Q, const void* K, const void* V, void* O, int B,
                                         int H, int Hkv, int S, int d, const int64_t strides[12],
                                         int dtype, int causal, float p, const uint64_t* mask,
                                         uint64_t seed, uint64_t offset, void* stream) {
    return rov::launch_attention(Q, K, V, O, B, H, Hkv, S, d, strides, dtype, causal, p, mask, seed,
                                 offset, (hipStream_t)stream);
}
