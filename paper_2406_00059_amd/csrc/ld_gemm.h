// Multi-row linear layers on the matrix cores (bf16 matrices): launcher interface.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>
#include "ld_gemv.h"

namespace ld {

enum { GEMM_STORE = 0, GEMM_ADD = 1, GEMM_SWIGLU = 2 };

// True if the MFMA kernel handles this shape (K a multiple of 128).
bool gemm_supported(int T, int N, int K);

// Bytes of scratch for the bf16 (high, low) images of a [T, K] activation matrix, and for a whole
// launch_norm_split + launch_gemm pair (split image followed by the split-K partial sums).
size_t gemm_split_bytes(int T, int K);
size_t gemm_scratch_bytes(int T, int N, int K, int epi);

// xs <- split(x * rsqrt(mean x^2 + eps) * g)  (g == nullptr: plain split), row by row:
// hi = bf16(v), lo = bf16(v - hi), stored as two [T, K] bf16 matrices (hi first).
void launch_norm_split(const float *x, const float *g, float eps, int T, int K, uint16_t *xs, hipStream_t s);

// y = epilogue(X W^T) with X given by its split image at the start of the scratch area xs
// (gemm_scratch_bytes bytes); W bf16 [N, K] ([2N, K] for GEMM_SWIGLU).
// next != nullptr with GEMM_ADD (N a multiple of 4): y is the residual stream and the next GEMM takes its
// RMS-normalised rows; next->xs (gemm_split_bytes(T, N) bytes, not inside this call's scratch area) receives
// split(y * rsqrt(mean y^2 + eps) * g) from the kernel that finishes y, with the values launch_norm_split
// would write.  With GEMM_SWIGLU (g unused): the result goes to next->xs as split(result) and y is not written.
// With GEMM_STORE and rope != nullptr (the q-k-v projection; cos_sin, pos and seq_slot indexed by row): the kernel
// that finishes y rotates the q heads in y and writes the rotated k heads and the v heads into the paged pool,
// with the values the separate rotate-and-append pass would write (k and v are not stored to y).
//
// f16_flag != nullptr: the caller allows the rows of this pass to enter the product rounded to fp16 (11 significant
// bits instead of the 16 of the two-term split) where that pays: more than 64 rows in the big-tile kernel
// (gemm_f16_rows), i.e. the rows of prefill chunks; the rows of the split image that take this form are overwritten
// with their fp16 values.  The caller has made sure that the matrix holds nothing beyond the fp16 range
// (launch_weight_range_check); *f16_flag (device memory) is set to 1 when an activation does not fit, and the
// results of the pass are then to be thrown away and the pass repeated without the flag.  W16 != nullptr: W's fp16
// image (launch_weight_to_f16), read in W's place by the rows that take the fp16 form, which otherwise turn every
// weight fragment into fp16 on its way to the matrix cores; same values either way, bit-equal results.
struct GemmNext { const float *g; float eps; uint16_t *xs; const RopeKvArgs *rope = nullptr; };
void launch_gemm(const uint16_t *W, uint16_t *xs, int T, int N, int K, int epi, float *y, hipStream_t s,
                 const GemmNext *next = nullptr, int *f16_flag = nullptr, const uint16_t *W16 = nullptr);
bool gemm_f16_rows(int T, int N, int K, int epi);
// *flag (device memory) = 1 if the bf16 matrix W (n elements, a multiple of 8) holds a value beyond +-65504 or not a number.
void launch_weight_range_check(const uint16_t *W, int64_t n, int *flag, hipStream_t s);
// The same check, and out[n] = W as fp16 (exact where the flag stays clear, values below 2^-14 in magnitude aside).
void launch_weight_to_f16(const uint16_t *W, int64_t n, uint16_t *out, int *flag, hipStream_t s);

// Skinny product alone (T <= 32 rows, K a multiple of 128): partial[z][t][row] for the skinny_slabs(K)
// 512-wide K slabs z; the caller adds the slabs in order.
int skinny_slabs(int K);
void launch_gemm_skinny(const uint16_t *W, const uint16_t *xhi, const uint16_t *xlo, int T, int n_rows, int K,
                        float *partial, hipStream_t s);

}  // namespace ld
