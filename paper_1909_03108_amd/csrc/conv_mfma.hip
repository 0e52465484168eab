// placeholder until the MFMA kernels land
#include "common.h"
namespace sp3d {
bool conv_mfma_supported(const Geo &, int, int, sp_dtype_t) { return false; }
size_t conv_mfma_ws_bytes(const Geo &, int, int) { return 0; }
int launch_conv_mfma(const void *, const void *, const float *, void *, const Geo &, int, int, bool,
                     bool, void *, hipStream_t) { return SP_EUNSUPPORTED; }
bool wgrad_mfma_supported(const Geo &, int, int, sp_dtype_t) { return false; }
size_t wgrad_mfma_ws_bytes(const Geo &, int, int) { return 0; }
int launch_wgrad_mfma(const void *, const void *, float *, float *, const Geo &, int, int, void *,
                      hipStream_t) { return SP_EUNSUPPORTED; }
}
