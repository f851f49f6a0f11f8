#include "kernels.hpp"
namespace msd {
int launch_dequant_gemm_w8(const uint16_t*, int64_t, int64_t, int64_t, const int8_t*, const float*, int64_t,
                           void*, int, int64_t, hipStream_t) { return MSD_ERR_UNSUPPORTED; }
int launch_dequant_gemm_w4(const uint16_t*, int64_t, int64_t, int64_t, const uint8_t*, const uint8_t*, int64_t,
                           void*, int, int64_t, hipStream_t) { return MSD_ERR_UNSUPPORTED; }
}  // namespace msd
