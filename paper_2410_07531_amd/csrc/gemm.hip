// GEMM (placeholder until the MFMA kernel lands): reports ROV_ERR_UNSUPPORTED.
#include "rov_internal.h"
namespace rov {
int launch_gemm(const void*, const void*, void*, int, int, int, int, int, float, float, hipStream_t) {
    return ROV_ERR_UNSUPPORTED;
}
}  // namespace rov
extern "C" int rov_gemm(const void* A, const void* Bm, void* C, int M, int N, int K, int dtype,
                        int transB, float scaleA, float scaleB, void* stream) {
    return rov::launch_gemm(A, Bm, C, M, N, K, dtype, transB, scaleA, scaleB, (hipStream_t)stream);
}
