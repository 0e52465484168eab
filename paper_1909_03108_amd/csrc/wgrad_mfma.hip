// placeholder until the MFMA weight-gradient kernel lands
#include "common.h"
namespace sp3d {
bool wgrad_mfma_supported(const Geo &, int, int, sp_dtype_t) { return false; }
size_t wgrad_mfma_ws_bytes(const Geo &, int, int) { return 0; }
int launch_wgrad_mfma(const void *, const void *, float *, float *, const Geo &, int, int, void *,
                      hipStream_t) { return SP_EUNSUPPORTED; }
}
