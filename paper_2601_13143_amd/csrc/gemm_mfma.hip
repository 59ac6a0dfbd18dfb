#include "common.hpp"
namespace fastav {
bool mfma_linear_supported(int64_t, int, int, int, int) { return false; }
fastav_status_t launch_linear_mfma(const void*, const void* const*, const int*, int, const void*, void*, int64_t, int64_t, int, int, int, hipStream_t) { return fail(FASTAV_EUNSUPPORTED, "mfma gemm not built"); }
}
