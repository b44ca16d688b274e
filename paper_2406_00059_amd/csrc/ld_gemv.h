// Batch-1 matrix-vector kernels (bf16 matrices): launcher interface.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ld {

enum { GEMV_STORE = 0, GEMV_ADD = 1, GEMV_SWIGLU = 2, GEMV_ROPE_KV = 3 };

// Arguments of the fused "rotate q,k and append k,v to the paged cache" epilogue (one input row).
struct RopeKvArgs {
    const float2 *cos_sin;      // [hd/2] (cos, sin) of the row's position
    const int32_t *pos;         // [1]
    const int32_t *seq_slot;    // [1]
    const int32_t *table;       // block table [*, table_stride]
    int32_t table_stride;
    uint16_t *pool;             // one layer's slice [block][2][Hkv][16][hd], bf16
    int32_t H, Hkv, hd;
};

// True if the slab kernel handles this shape (bf16, one input row).
bool gemv1_supported(int N, int K, int epi);

// y = epilogue(W x) for one input row x [K]; W bf16 [N, K] ([2N, K] for GEMV_SWIGLU).
// With g != nullptr, x is RMS-normalised on the fly (gain g, epsilon eps).
// GEMV_ROPE_KV: N = (H + 2 Hkv) hd; y receives the rotated q heads ([H hd] floats); k, v go to the pool.
void launch_gemv1(const uint16_t *W, const float *x, const float *g, float eps, int N, int K, int epi, float *y,
                  const RopeKvArgs *rk, hipStream_t s);

}  // namespace ld
