// Placeholder until the MFMA kernels land: reports the MFMA path as unavailable so every
// model runs on the shape-generic kernels.
#include "sl_common.h"
bool sl_mfma_supported(const sl_config*) { return false; }
size_t sl_mfma_packed_bytes(const sl_config*) { return 0; }
int sl_mfma_pack_all(sl_ctx*, hipStream_t, void*) { return SL_EINVAL; }
int sl_mfma_layer(sl_ctx*, hipStream_t, int, void*, void*, void*, void*, void*, float*, const int32_t*, const int32_t*,
                  int, const void*) { return SL_EINVAL; }
int sl_mfma_lm_head(sl_ctx*, hipStream_t, const void*, const int32_t*, const int32_t*, int, void*) { return SL_EINVAL; }
