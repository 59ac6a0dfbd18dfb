#include "common.hpp"
namespace fastav {
bool mfma_attention_supported(int, int, int64_t, int64_t, int64_t) { return false; }
fastav_status_t launch_attention_mfma(const void*, int64_t, const void*, const void*, int64_t, void*, int64_t, const int32_t*, int, int64_t, int, int, int, int, float*, float*, hipStream_t) { return fail(FASTAV_EUNSUPPORTED, "mfma attention not built"); }
}
