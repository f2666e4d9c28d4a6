// Shared internals of the tgemm library: error reporting and the context object.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>

#include <vector>

#include "../../include/tgemm.h"

struct tgemm_ctx;

namespace tg {

// Records the message for tgemm_last_error() on this thread and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

#define TG_HIP(call)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            return tg::fail(TGEMM_EHIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), \
                            __FILE__, __LINE__);                                             \
    } while (0)

enum PtrKind { PTR_DEVICE = 0, PTR_PINNED = 1, PTR_PAGEABLE = 2 };
PtrKind classify_pointer(const void* p, int device);

class Engine;   // out-of-core tile engine (engine.cpp)
struct SkWorkspace;   // plan and workspace of the balanced in-core fp32 product (gemm_f32.hip)
// With TGEMM_LOG=1 in the environment: one line on stderr with the call's statistics.
void log_call(const char* what, const tgemm_ctx* ctx, int rc);

// The balanced schedule's plan for a product, without a device (gemm_f32.hip); fills *out (applies = 0 where
// tgemm_run would take one launch) and copies up to cap segments.  May throw std::bad_alloc.
int sk_inspect(int64_t M, int64_t N, int64_t K, int32_t T, bool bf16, int n_cus, bool forced, tgemm_balance* out,
               tgemm_segment* segments, int64_t cap);

// Address of the current device's copy of the static scratch array of mlp_forward_static (mlp.hip);
// looked up once per device.  `device` must be current.  out may be NULL.
int static_scratch_resolve(int device, void** out);

}  // namespace tg

struct tgemm_ctx {
    int device = 0;
    hipStream_t streams[4] = {nullptr, nullptr, nullptr, nullptr};
    tgemm_opts opts{};
    tgemm_stats stats{};
    hipEvent_t ev_start = nullptr, ev_stop = nullptr;
    bool kernel_timing_pending = false;
    std::vector<tgemm_trace_rec> trace;
    tg::Engine* engine = nullptr;
    // in-core fp32 tgemm_run: the balanced schedule's state, the device's compute units, fork / join events
    tg::SkWorkspace* sk = nullptr;
    int n_cus = 0;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
};

namespace tg {
// Device-side staging + scheduling of one out-of-core product (engine.cpp).
int run_out_of_core(tgemm_ctx* ctx, const void* A, const void* B, float* C, int64_t M, int64_t N,
                    int64_t K, int32_t T, int32_t dtype, size_t hbm_budget);
void destroy_engine(tgemm_ctx* ctx);
// Drops the cached tiles of every matrix that starts at host_base; returns how many there were.
int64_t invalidate_tiles(tgemm_ctx* ctx, const void* host_base);
}  // namespace tg
