// Out-of-core tile engine (placeholder until the engine lands).
#include "common.h"

namespace tg {

int run_out_of_core(tgemm_ctx*, const void*, const void*, float*, int64_t, int64_t, int64_t, int32_t, int32_t, size_t)
{
    return fail(TGEMM_EARG, "out-of-core runs are not implemented yet");
}

void destroy_engine(tgemm_ctx*) {}

}  // namespace tg
