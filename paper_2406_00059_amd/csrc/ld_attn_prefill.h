// Chunk-prefill attention on the matrix cores: launcher interface.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ld {

// Supported: bf16 pool, head_dim 128.
bool prefill_attention_supported(int dtype_is_bf16, int hd);

// tiles: DEVICE int32[n_tiles][4] = (first row, rows <= 128, position of the first row, block-table row).
// q rows at q + row * q_stride (+ head * 128); out dense [rows, H, 128].
// window > 0: a row at position p sees positions max(0, p - window + 1) .. p; 0: positions 0 .. p.
// max_pos (HOST): largest position of any row, sizes the KV split.  scratch (may be null: no split): up to
// prefill_attention_scratch_bytes() bytes for the partial results of split tiles.
// xs_hi / xs_lo non-null: the rows go out as the (hi, lo) bf16 operand images of the output projection
// ([rows of the pass][H * 128] each, indexed like out) instead of floats.
// f16_flag non-null (DEVICE): queries and probabilities enter the products as one fp16 term, keys and values widened
// to fp16; *f16_flag is set to 1 when a query, key or value lies beyond the fp16 range (results then to be discarded).
size_t prefill_attention_scratch_bytes();
void launch_prefill_attention(const float *q, int q_stride, const uint16_t *pool, int Hkv, const int32_t *table,
                              int table_stride, const int32_t *tiles, int n_tiles, int H, int window, int max_pos,
                              float *out, void *scratch, size_t scratch_bytes, hipStream_t s,
                              uint16_t *xs_hi = nullptr, uint16_t *xs_lo = nullptr, int *f16_flag = nullptr);

}  // namespace ld
