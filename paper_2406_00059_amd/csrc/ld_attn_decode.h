// Grouped-head paged decode attention on the matrix cores: launcher interface.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ld {

// Supported: bf16 pool, head_dim 128, 2 .. 16 query heads per KV head.
bool grouped_decode_supported(int dtype_is_bf16, int hd, int H, int Hkv);

// Partial attention of T single-token rows: for row t, KV head j and chunk c (cb blocks of the visible
// context, cb a multiple of 8) the unnormalised output, maximum and sum of every query head of the group,
// in the layout the merge kernel of the scalar path reads:
//   part_o [((t * H + h) * max_chunks + c)][128], part_ml [((t * H + h) * max_chunks + c)][2].
void launch_grouped_decode_partial(const float *q, int q_stride, const uint16_t *pool, int Hkv, const int32_t *table,
                                   int table_stride, const int32_t *seq_slot, const int32_t *ctx_len, int T, int H,
                                   int window, int max_chunks, int cb, float *part_o, float *part_ml, hipStream_t s);

}  // namespace ld
