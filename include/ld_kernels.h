/*
 * libld, kernel-level entry points: each step of the decode / prefill pass as a call of its
 * own, so that tests and micro-benchmarks can drive one kernel at a time.  ld_prefill /
 * ld_decode_step / ld_step_mixed are compositions of exactly these launches.
 *
 * All data pointers are DEVICE pointers owned by the caller unless marked HOST.  `stream`
 * is a hipStream_t as void*.  Calls only enqueue work; they return LD_E_INVAL for
 * unsupported shapes (before launching anything) and LD_E_HIP if the launch failed.
 * Activations are float32 throughout; `dtype` (LD_F32 | LD_BF16) is the element type of
 * matrices and of the KV pool.
 */
#ifndef LD_KERNELS_H
#define LD_KERNELS_H

#include "ld.h"

#ifdef __cplusplus
extern "C" {
#endif

enum { LDK_STORE = 0, LDK_ADD = 1, LDK_SWIGLU = 2 };

/* x[t, :] = embed[tok[t], :] widened to float32.  tok values must be < vocab (checked by the
 * caller of the step functions on the host). */
ld_status ldk_embed(const void *embed, int32_t dtype, const int32_t *tok, int32_t T, int32_t d, float *x,
                    void *stream);

/* out[r, i] = x[row, i] / sqrt(mean_j x[row, j]^2 + eps) * g[i], row = row_idx ? row_idx[r] : r. */
ld_status ldk_rmsnorm(const float *x, const float *g, const int32_t *row_idx, int32_t R, int32_t d, float eps,
                      float *out, void *stream);

/* Scratch bytes ldk_linear (ldk_qkv_rope: epilogue LDK_STORE, N = (H + 2 Hkv) hd) can use for T rows
 * (0 for T < 2): the two-part bf16 image of the input plus split-K partial sums. */
size_t ldk_linear_scratch_bytes(int32_t T, int32_t N, int32_t K, int32_t epilogue);

/* Linear layer on T rows: acc[t, n] = sum_k W[n, k] x[t, k], float32 accumulation.
 *   LDK_STORE : y[t, n]  = acc[t, n]                          W [N, K]
 *   LDK_ADD   : y[t, n] += acc[t, n]   (residual)             W [N, K]
 *   LDK_SWIGLU: y[t, n]  = silu(acc[t, n]) * acc[t, N + n]    W [2N, K]  (gate rows, then up rows)
 * If g != NULL the input is RMS-normalised on the fly: x[t, k] is replaced by
 * x[t, k] * rsqrt(mean_k x[t, k]^2 + eps) * g[k].
 * x [T, K], y [T, N] dense row-major.  K must be a multiple of 8.
 * Kernel choice: one bf16 row -> bandwidth-bound matrix-vector kernel; several bf16 rows with
 * K a multiple of 128 and scratch of ldk_linear_scratch_bytes(...) bytes -> matrix cores
 * (activations split into two bf16 parts, float32 accumulation); otherwise (float32 matrices, no
 * scratch) a plain vector-ALU kernel.  scratch may be NULL. */
ld_status ldk_linear(const void *W, int32_t dtype, const float *x, const float *g, float eps, int32_t T,
                     int32_t N, int32_t K, int32_t epilogue, float *y, void *scratch, size_t scratch_bytes,
                     void *stream);

/* ldk_linear on a bf16 matrix in the form the engine uses for the rows of long prefill chunks (rows that reach
 * later tokens only through cached keys and values; the paper's section 4.1 fixes no precision): where more than 64
 * rows run on the big-tile matrix-core kernel, the activations enter the product rounded to fp16 (11 significant
 * bits) in one term instead of the two bf16 terms (16 bits), and the bf16 matrix entries are widened to fp16 on the
 * way to the matrix cores, which is exact for 2^-14 <= |w| <= 65504.  Other row counts and shapes: exactly
 * ldk_linear.  overflow (device memory, 4 bytes, the caller clears it) is set to 1 when the matrix or an
 * activation holds a value beyond +-65504 or not a number; y is then not to be used (the engine repeats such a
 * pass with ldk_linear's arithmetic).  scratch: ldk_linear_scratch_bytes(...) bytes.
 * W_f16 (device memory, may be NULL): the matrix as fp16, same layout as W, written by ldk_weights_to_f16 with its
 * overflow flag left clear.  The rows that take the fp16 form then read it in W's place and widen nothing on the
 * way (the other rows, e.g. those past a multiple of 256, still read W); the matrix is not looked at again.  The
 * products are those of the values W holds either way: y is bit-equal with and without the image. */
ld_status ldk_linear_f16(const void *W, const void *W_f16, const float *x, const float *g, float eps, int32_t T,
                         int32_t N, int32_t K, int32_t epilogue, float *y, void *scratch, size_t scratch_bytes,
                         int32_t *overflow, void *stream);

/* out[i] = W[i] as fp16 for the n entries of a bf16 matrix (n a multiple of 8; both device memory, out n * 2
 * bytes, not overlapping W): exact for 2^-14 <= |w| <= 65504, smaller magnitudes lose their low bits (truncated
 * toward zero).  overflow (device memory, 4 bytes, the caller clears it) is set to 1 when an entry lies beyond
 * +-65504 or is not a number; the image is then not to be used.  The engine keeps such an image of every layer
 * matrix from its first pass of 512 rows or more on (see ld.h, Arithmetic). */
ld_status ldk_weights_to_f16(const void *W, int64_t n, void *out, int32_t *overflow, void *stream);

/* cos_sin[t, i] = (cos, sin)(pos[t] * rope_base^(-2i/hd)) for i < hd/2, as float32 pairs; the
 * angle is formed in float64 so that large positions lose no accuracy.  hd is 64 or 128. */
ld_status ldk_rope_table(const int32_t *pos, int32_t T, int32_t hd, float rope_base, float *cos_sin, void *stream);

/* Rotary embedding + cache append for T rows of a fused projection qkv [T, (H + 2 Hkv) hd]:
 * rotates every q head and k head of row t in place by the angles in cos_sin[t] (pair i =
 * elements (i, i + hd/2) of a head), then stores k and v, rounded to `dtype` (nearest even), into
 * block b = table[seq_slot[t] * table_stride + pos[t] / 16], slot s = pos[t] % 16 of pool_layer:
 *   pool_layer[b][0][kv_head][s][:] = k,     pool_layer[b][1][kv_head][:][s] = v   (values transposed).
 * pool_layer is one layer's slice of the pool: keys [block][0][Hkv][16][hd], values [block][1][Hkv][hd][16].
 * Rows of one call must address distinct (sequence, position) pairs. */
ld_status ldk_rope_kv_write(float *qkv, const float *cos_sin, const int32_t *pos, const int32_t *seq_slot,
                            const int32_t *table, int32_t table_stride, void *pool_layer, int32_t dtype, int32_t T,
                            int32_t H, int32_t Hkv, int32_t hd, void *stream);

/* Fused projection + rotary embedding + cache append: qkv[t, :] = W rmsnorm(x[t, :]; g, eps) with
 * W [(H + 2 Hkv) hd, K] (g == NULL: no normalisation), then exactly what ldk_rope_kv_write does.
 * On return the q part of qkv (first H hd floats of each row) is rotated; the k and v parts of qkv
 * are unspecified (their values are in the pool).  x [T, K], qkv [T, (H + 2 Hkv) hd]. */
ld_status ldk_qkv_rope(const void *W, int32_t dtype, const float *x, const float *g, float eps, float *qkv,
                       const float *cos_sin, const int32_t *pos, const int32_t *seq_slot, const int32_t *table,
                       int32_t table_stride, void *pool_layer, int32_t T, int32_t K, int32_t H, int32_t Hkv, int32_t hd,
                       void *scratch, size_t scratch_bytes, void *stream);

/* Scratch bytes ldk_paged_attention needs for T rows with contexts up to max_ctx (same H, Hkv, window
 * as the call). */
size_t ldk_attention_scratch_bytes(int32_t T, int32_t H, int32_t Hkv, int32_t hd, int32_t max_ctx, int32_t window);

/* Paged attention of T single-token queries (section 2.1): row t, head h attends to cached
 * positions 0 .. ctx_len[t]-1 of the sequence whose block-table row is seq_slot[t]:
 *   s_j = q.k_j / sqrt(hd),  p = softmax(s),  out = sum_j p_j v_j.
 * q row t, head h starts at q + t * q_stride + h * hd; out is dense [T, H, hd].
 * Query head h reads KV head h / (H / Hkv); the H / Hkv query heads of a KV head are served by one
 * workgroup (keys and values loaded once) when that ratio is 2, 4 or 8.
 * window > 0: banded attention, the row (at position ctx_len[t]-1) sees only positions
 * max(0, ctx_len[t] - window) .. ctx_len[t]-1; window == 0: every cached position.
 * ctx_len[t] >= 1.  max_ctx >= max_t ctx_len[t] sizes the launch (HOST value). */
ld_status ldk_paged_attention(const float *q, int32_t q_stride, const void *pool_layer, int32_t dtype,
                              const int32_t *table, int32_t table_stride, const int32_t *seq_slot,
                              const int32_t *ctx_len, int32_t max_ctx, int32_t T, int32_t H, int32_t Hkv,
                              int32_t hd, int32_t window, float *out, void *scratch, size_t scratch_bytes,
                              void *stream);

/* ldk_paged_attention for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation): same arguments, same kernels and the same results,
 * without the scratch pair.  The chunk partials go to a device array built into the library, of
 * LDK_STATIC_SCRATCH_BYTES bytes, which every GPU the library is used on holds from the first call on that GPU
 * until the process ends; its address is looked up once per device.  The call allocates and frees nothing.
 * A launch whose partials (T * H * chunks * (hd + 2) floats; chunks as the launch itself is cut, at most
 * ceil(max_ctx / 64)) would not fit is refused with LD_E_RANGE before anything is launched: 64 MiB serves
 * e.g. 64 rows x 40 heads at contexts up to 16384 (42 MB).  Nothing in the array has to start at zero (every partial
 * a merge reads was written by the same call), but all calls on one GPU share it: calls that overlap on one
 * GPU (different streams, or different threads) race; calls on one stream do not. */
#define LDK_STATIC_SCRATCH_BYTES (64u << 20)
size_t ldk_static_scratch_bytes(void);
ld_status ldk_paged_attention_static(const float *q, int32_t q_stride, const void *pool_layer, int32_t dtype,
                                     const int32_t *table, int32_t table_stride, const int32_t *seq_slot,
                                     const int32_t *ctx_len, int32_t max_ctx, int32_t T, int32_t H, int32_t Hkv,
                                     int32_t hd, int32_t window, float *out, void *stream);

/* Attention for prefill segments (section 2.1: all tokens of a prompt go through the model in one
 * iteration): a segment is a run of rows of one sequence at consecutive positions whose keys
 * and values are already in the pool; row r at position p attends to cached positions 0 .. p
 * (window > 0: positions max(0, p - window + 1) .. p).
 * tiles: DEVICE int32[n_tiles][4] = (first row, number of rows (1..128), position of the first row,
 * block-table row of the sequence); a segment longer than 128 rows is given as several tiles.
 * q and out as in ldk_paged_attention.  Supported: dtype LD_BF16 with hd = 128 (LD_E_INVAL otherwise;
 * such shapes run their prefill rows through ldk_paged_attention with ctx_len = position + 1).
 * max_pos (HOST value) >= the position of every row.  When few tiles face a long context the KV range of
 * a tile is split over several workgroups whose partial results go through scratch (DEVICE, up to
 * ldk_prefill_attention_scratch_bytes() bytes are used) and are merged in split order; scratch == NULL or a
 * smaller buffer only limits the split, never the result. */
size_t ldk_prefill_attention_scratch_bytes(void);
ld_status ldk_prefill_attention(const float *q, int32_t q_stride, const void *pool_layer, int32_t dtype,
                                const int32_t *table, int32_t table_stride, const int32_t *tiles, int32_t n_tiles,
                                int32_t H, int32_t Hkv, int32_t hd, int32_t window, int32_t max_pos, float *out,
                                void *scratch, size_t scratch_bytes, void *stream);

/* ldk_prefill_attention in the form the engine uses in passes of 512 rows or more (see ldk_linear_f16): with
 * overflow != NULL the queries and the probabilities enter the matrix-core products as one fp16 term (11 significant
 * bits; two bf16 terms otherwise) and the cached keys and values are widened from bf16 to fp16, which is exact within
 * +-65504.  *overflow (DEVICE, 4 bytes, cleared by the caller) is set to 1 when a scaled query, a key or a value of a
 * position the walk touches lies beyond that range or is not a number; out is then not to be used.  overflow == NULL:
 * exactly ldk_prefill_attention. */
ld_status ldk_prefill_attention_f16(const float *q, int32_t q_stride, const void *pool_layer, int32_t dtype,
                                    const int32_t *table, int32_t table_stride, const int32_t *tiles,
                                    int32_t n_tiles, int32_t H, int32_t Hkv, int32_t hd, int32_t window,
                                    int32_t max_pos, float *out, void *scratch, size_t scratch_bytes,
                                    int32_t *overflow, void *stream);

/* out[r] = smallest index of the maximum of logits[r, 0..V). */
ld_status ldk_argmax(const float *logits, int32_t R, int32_t V, int32_t *out, void *stream);

/* Token choice with temperature (section 4.1 decodes at temperature 0 = ldk_argmax; this is the same
 * decision with noise): out[r] = smallest index of the maximum of logits[r, i] / temperature[r] + g(r, i),
 * g = -log(-log(u)) standard Gumbel noise, which draws i with probability softmax(logits[r] / temperature[r]).
 * u = (k + 1/2) / 2^23 with k the top 23 bits of the SplitMix64 output function applied to
 * seed[r] + (pos[r] * V + i + 1) * 0x9E3779B97F4A7C15: a pure function of (seed, pos, i).  Rows with
 * temperature[r] == 0 are the plain argmax.  temperature, seed, pos: DEVICE arrays of R entries. */
ld_status ldk_sample(const float *logits, int32_t R, int32_t V, const float *temperature, const uint64_t *seed,
                     const int32_t *pos, int32_t *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LD_KERNELS_H */
