// MLP passes (placeholder until they land).
#include "common.h"

extern "C" {
int mlp_create(tgemm_ctx*, tgemm_mlp**, int32_t, const int64_t*, void* const*, int32_t, int32_t, size_t) { return tg::fail(TGEMM_EARG, "mlp: not implemented yet"); }
int mlp_destroy(tgemm_mlp*) { return TGEMM_OK; }
int mlp_forward(tgemm_mlp*, const void*, int64_t, float*) { return tg::fail(TGEMM_EARG, "mlp: not implemented yet"); }
int mlp_backward(tgemm_mlp*, const int32_t*, void* const*, float*) { return tg::fail(TGEMM_EARG, "mlp: not implemented yet"); }
int mlp_step(tgemm_mlp*, const void*, const int32_t*, int64_t, float, float*) { return tg::fail(TGEMM_EARG, "mlp: not implemented yet"); }
int mlp_read(tgemm_mlp*, int32_t, int32_t, void*, size_t) { return tg::fail(TGEMM_EARG, "mlp: not implemented yet"); }
}
