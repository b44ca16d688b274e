// Decoder layer for a decode batch (2..32 rows, one token per sequence) on bf16 weights: the four
// skinny MFMA projections with their reductions fused into the producers of the next operand.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ld {

struct BatchLayerArgs {
    // weights of the layer (bf16) and gains (float32)
    const uint16_t *wqkv, *wo, *wgate_up, *wdown;
    const float *attn_norm;       // gain of this layer's attention norm (already applied to xs on entry)
    const float *ffn_norm;        // gain of this layer's FFN norm
    const float *next_norm;       // gain of the next layer's attention norm, or nullptr after the last layer
    // shapes
    int T, d, H, Hkv, hd, ffn;
    float eps;
    // activations / scratch (device)
    float *x;                     // residual stream [T, d], updated in place
    float *q;                     // rotated queries, row stride q_stride
    int q_stride;
    uint16_t *xs;                 // split operand image (hi then lo), capacity 2 * T * max(d, H hd, ffn)
    float *partial;               // split-K partial sums, capacity ks_max * T * max(nqkv, d, 2 ffn)
    float *ss_part;               // [2][T][d / 1024] partial sums of squares (attention norm, FFN norm)
    // cache
    const float *cos_sin;         // [T, hd/2, 2]
    const int32_t *pos, *seq_slot, *table;
    int table_stride;
    uint16_t *pool;               // this layer's slice
};

// True if the fused batch layer handles this shape.
bool batch_layer_supported(int T, int d, int H, int Hkv, int hd, int ffn);
size_t batch_layer_xs_bytes(int T, int d, int H, int hd, int ffn);
size_t batch_layer_partial_bytes(int T, int d, int H, int Hkv, int hd, int ffn);
size_t batch_layer_ss_bytes(int T, int d);

// Before the first layer: xs = split(x * g), ss_part[0] = partial sums of squares of x.
void launch_batch_prepare(const float *x, const float *g, int T, int d, uint16_t *xs, float *ss_part, hipStream_t s);

// Part 1: q/k/v projection, RoPE, cache append (q ready for attention).
void launch_batch_qkv(const BatchLayerArgs &a, hipStream_t s);
// After attention wrote its split output into a.xs: output projection + residual; gate/up + SwiGLU;
// down projection + residual (each leaves the next product's operand in a.xs).
void launch_batch_wo(const BatchLayerArgs &a, hipStream_t s);
void launch_batch_gate_up(const BatchLayerArgs &a, hipStream_t s);
void launch_batch_down(const BatchLayerArgs &a, hipStream_t s);

}  // namespace ld
