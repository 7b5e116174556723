// FP4 (E2M1) activation variant on the scaled FP4 matrix instruction.
#include "common.h"

int bl_launch_gemm_fp4(const void* q, const uint8_t* scale, int64_t M, int64_t K, const void* Wp,
                       const float* alpha, int64_t N, void* Y, bl_dtype ydt, hipStream_t s) {
  (void)q; (void)scale; (void)M; (void)K; (void)Wp; (void)alpha; (void)N; (void)Y; (void)ydt; (void)s;
  return BL_EUNSUPPORTED;
}
