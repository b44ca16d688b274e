// Internal helpers shared by the host state machine and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <cstdarg>
#include <cstdio>
#include "ld.h"
#include "ld_kernels.h"

namespace ld {

void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
void clear_error();

inline ld_status fail(ld_status s, const char *what) {
    set_error("%s", what);
    return s;
}

#define LD_HIP_TRY(expr)                                                                  \
    do {                                                                                  \
        hipError_t e_ = (expr);                                                           \
        if (e_ != hipSuccess) {                                                           \
            ld::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return LD_E_HIP;                                                              \
        }                                                                                 \
    } while (0)

// Per-kernel timing: while a pass is being profiled, every kernel launch of this thread asks the
// timer for an event pair that the runtime attaches to the dispatch itself (start and end of the
// kernel, not of the gap around it).  Null when profiling is off.
struct LaunchTimer {
    virtual void next(hipEvent_t *start, hipEvent_t *stop) = 0;
    virtual ~LaunchTimer() {}
};
extern thread_local LaunchTimer *g_launch_timer;

ld_status paged_attention_split(const float *q, int q_stride, const void *pool_layer, int dtype, const int32_t *table,
                                int table_stride, const int32_t *seq_slot, const int32_t *ctx_len, int max_ctx, int T,
                                int H, int Hkv, int hd, int window, uint16_t *xs_out, void *scratch,
                                size_t scratch_bytes, hipStream_t stream, int image_rows = 0);

// ldk_linear for the rows of an engine pass: f16_flag and W_f16 as in launch_gemm (nullptr: ldk_linear itself).
ld_status linear_pass(const void *W, int32_t dtype, const float *x, const float *g, float eps, int32_t T, int32_t N,
                      int32_t K, int32_t epilogue, float *y, void *scratch, size_t scratch_bytes, void *stream,
                      int *f16_flag, const void *W_f16 = nullptr);
// Integer value of an environment variable (a tuning knob), dflt when unset.
int env_flag(const char *name, int dflt);

}  // namespace ld

// Every kernel of the library is launched through this macro.
#define LD_LAUNCH(kernel, grid, block, shmem, stream, ...)                                        \
    do {                                                                                          \
        hipEvent_t ev_s_ = nullptr, ev_e_ = nullptr;                                              \
        if (ld::g_launch_timer) ld::g_launch_timer->next(&ev_s_, &ev_e_);                         \
        hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, ev_s_, ev_e_, 0, __VA_ARGS__);  \
    } while (0)

namespace ld {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace ld
