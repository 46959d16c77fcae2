// MFMA (bf16) path -- placeholder until the kernels land: reports "unsupported" so every
// model runs on the any-shape path.
#include "la_internal.h"

namespace la {
int mfma_supported(const la_model_desc *) { return 0; }
int mfma_create(la_model *) { set_error("MFMA path not built"); return LA_EINVAL; }
void mfma_destroy(la_model *) {}
int mfma_set_layer(la_model *, int, const la_layer_weights *, hipStream_t) { return LA_EINVAL; }
int mfma_set_head(la_model *, const void *, hipStream_t) { return LA_EINVAL; }
int mfma_forward(la_model *, int, int, float *, int, const int32_t *, const uint64_t *, la_kv *, hipStream_t) { return LA_EINVAL; }
int mfma_unembed_argmax(la_model *, const float *, int, int32_t *, float *, hipStream_t) { return LA_EINVAL; }
}  // namespace la
