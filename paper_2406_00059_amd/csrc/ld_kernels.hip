// HIP kernels of the decode / chunked-prefill pass for gfx950 (wave64) and their launchers.
//
// Numerical scheme: activations, accumulators, softmax statistics and logits are float32;
// matrices and the KV pool are float32 or bf16.  bf16 -> float32 widening is exact.
#include "ld_internal.h"
#include "ld_device.h"
#include "ld_gemv.h"
#include "ld_gemm.h"
#include "ld_attn_prefill.h"
#include "ld_attn_decode.h"
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <mutex>

using namespace ldd;

namespace {

// ---------------------------------------------------------------- embedding gather

template <typename WT>
__global__ void k_embed(const WT *__restrict__ E, const int32_t *__restrict__ tok, int d, float *__restrict__ x) {
    const int t = blockIdx.x;
    const WT *row = E + (int64_t)tok[t] * d;
    for (int i = threadIdx.x * 8; i < d; i += blockDim.x * 8) {
        float v[8];
        load8(row + i, v);
#pragma unroll
        for (int e = 0; e < 8; e++) x[(int64_t)t * d + i + e] = v[e];
    }
}

// ---------------------------------------------------------------- RMSNorm (stand-alone, with row gather)

__global__ __launch_bounds__(256) void k_rmsnorm(const float *__restrict__ x, const float *__restrict__ g,
                                                 const int32_t *__restrict__ row_idx, int d, float eps,
                                                 float *__restrict__ out) {
    __shared__ float red[4];
    const int r = blockIdx.x;
    const float *row = x + (int64_t)(row_idx ? row_idx[r] : r) * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) ss += row[i] * row[i];
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float rstd = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / d + eps);
    for (int i = threadIdx.x; i < d; i += 256) out[(int64_t)r * d + i] = row[i] * rstd * g[i];
}

// ---------------------------------------------------------------- linear layer, vector-ALU version
//
// One wave owns R output rows (2R matrix rows for the SwiGLU epilogue) for a tile of TT input
// rows and streams those matrix rows once, 16 bytes per lane per load, lanes striding over K.
// With NORM the RMS statistics of the input rows are accumulated from the same x loads and the
// scale 1/rms is applied to the finished dot products (the gain is applied to x on the fly).

template <typename WT, int TT, int R, int EPI, bool NORM>
__global__ __launch_bounds__(256) void k_linear_valu(const WT *__restrict__ W, const float *__restrict__ x,
                                                     const float *__restrict__ g, float eps, int T, int N, int K,
                                                     float *__restrict__ y) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = (blockIdx.x * 4 + wave) * R;
    const int t0 = blockIdx.y * TT;
    if (n0 >= N) return;
    constexpr int NW = (EPI == LDK_SWIGLU) ? 2 * R : R;
    const WT *wrow[NW];
#pragma unroll
    for (int r = 0; r < R; r++) {
        const int n = min(n0 + r, N - 1);  // clamped rows are computed and dropped
        wrow[r] = W + (int64_t)n * K;
        if constexpr (EPI == LDK_SWIGLU) wrow[R + r] = W + (int64_t)(N + n) * K;
    }
    float acc[NW][TT];
    float ss[TT];
#pragma unroll
    for (int t = 0; t < TT; t++) {
        ss[t] = 0.f;
#pragma unroll
        for (int r = 0; r < NW; r++) acc[r][t] = 0.f;
    }
    for (int k = lane * 8; k < K; k += WAVE * 8) {
        float wv[NW][8];
#pragma unroll
        for (int r = 0; r < NW; r++) load8(wrow[r] + k, wv[r]);
        float gv[8];
        if (NORM) load8(g + k, gv);
#pragma unroll
        for (int t = 0; t < TT; t++) {
            float xv[8];
            if (t0 + t < T) {
                load8(x + (int64_t)(t0 + t) * K + k, xv);
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++) xv[e] = 0.f;
            }
            if (NORM) {
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    ss[t] = fmaf(xv[e], xv[e], ss[t]);
                    xv[e] *= gv[e];
                }
            }
#pragma unroll
            for (int r = 0; r < NW; r++)
#pragma unroll
                for (int e = 0; e < 8; e++) acc[r][t] = fmaf(wv[r][e], xv[e], acc[r][t]);
        }
    }
#pragma unroll
    for (int t = 0; t < TT; t++) {
        float rstd = 1.f;
        if (NORM) rstd = 1.0f / sqrtf(wave_sum(ss[t]) / K + eps);
#pragma unroll
        for (int r = 0; r < NW; r++) acc[r][t] = wave_sum(acc[r][t]) * rstd;
    }
    if (lane == 0) {
#pragma unroll
        for (int t = 0; t < TT; t++) {
            if (t0 + t >= T) continue;
#pragma unroll
            for (int r = 0; r < R; r++) {
                if (n0 + r >= N) continue;
                float *dst = y + (int64_t)(t0 + t) * N + n0 + r;
                if constexpr (EPI == LDK_STORE) *dst = acc[r][t];
                else if constexpr (EPI == LDK_ADD) *dst += acc[r][t];
                else {
                    const float gate = acc[r][t], up = acc[R + r][t];
                    *dst = gate / (1.0f + __expf(-gate)) * up;
                }
            }
        }
    }
}

// ---------------------------------------------------------------- rotary tables, RoPE + cache append

// cs[t][i] = (cos, sin)(pos[t] * base^(-2i/hd)), angle formed in float64.
__global__ void k_rope_table(const int32_t *__restrict__ pos, int hd, double base, float2 *__restrict__ cs) {
    const int t = blockIdx.x, i = threadIdx.x, half = hd / 2;
    if (i >= half) return;
    const double theta = pow(base, -2.0 * (double)i / (double)hd);
    double s, c;
    sincos((double)pos[t] * theta, &s, &c);
    cs[(int64_t)t * half + i] = make_float2((float)c, (float)s);
}

template <typename KVT>
__global__ void k_rope_kv_write(float *__restrict__ qkv, const float2 *__restrict__ cs,
                                const int32_t *__restrict__ pos, const int32_t *__restrict__ seq_slot,
                                const int32_t *__restrict__ table, int table_stride, KVT *__restrict__ pool,
                                int H, int Hkv, int hd) {
    const int t = blockIdx.y, hh = blockIdx.x, i = threadIdx.x, half = hd / 2;
    if (i >= half) return;
    const int nqkv = (H + 2 * Hkv) * hd;
    const float2 c = cs[(int64_t)t * half + i];
    float *row = qkv + (int64_t)t * nqkv;
    if (hh < H) {
        float *u = row + hh * hd;
        const float2 r = rope_rotate(u[i], u[i + half], c);
        u[i] = r.x;
        u[i + half] = r.y;
        return;
    }
    const int j = hh - H;
    const float *ku = row + (H + j) * hd;
    const float *vu = row + (H + Hkv + j) * hd;
    const float a = ku[i], b = ku[i + half];
    const int p = pos[t];
    const int64_t phys = table[(int64_t)seq_slot[t] * table_stride + (p >> 4)];
    KVT *blk = pool + phys * kv_block_elems(Hkv, hd);
    const int slot = p & 15;
    const float2 r = rope_rotate(a, b, c);
    store_elem(blk + kv_k_offset(hd, j, slot, i), r.x);
    store_elem(blk + kv_k_offset(hd, j, slot, i + half), r.y);
    store_elem(blk + kv_v_offset(Hkv, hd, j, slot, i), vu[i]);
    store_elem(blk + kv_v_offset(Hkv, hd, j, slot, i + half), vu[i + half]);
}

// ---------------------------------------------------------------- paged decode attention
//
// Work item = (row t, head group, chunk c).  A head group is the G query heads that share one KV head
// (G = 1 for ungrouped attention): the keys and values of a block are loaded once and used for all G
// queries.  Chunk c covers CB consecutive KV blocks (CB*16 tokens) of the VISIBLE part of the row's
// context: with an attention band of W positions the row (at position ctx-1) sees positions
// max(0, ctx - W) .. ctx-1 and the walk starts at the block that holds the first of them.  A workgroup
// of 4 waves takes one work item, wave w the blocks w, w+4, ... of the chunk.  Inside a wave, a lane
// group of HD/8 adjacent lanes covers one key row with 16-byte loads (8 elements each) and owns a fixed
// run of a block's 16 positions (4 of them for head_dim 128); scores are reduced across the group with
// xor shuffles.  The values of a block are stored transposed ([dim][position]), so the same group reads,
// for each of its dimensions, exactly its own positions in one small load, and one load instruction of
// the wave still covers a contiguous run of memory.  Each lane group keeps its own online-softmax state
// (m, l, acc) per query in the log2 domain, merged across groups, waves and finally chunks.

// KV blocks per chunk: a multiple of 4 (one per wave), chosen per launch by attn_chunk_blocks().

// first visible position and first visible block of a row
__device__ __forceinline__ int band_first(int ctx, int window) { return (window > 0 && ctx > window) ? ctx - window : 0; }

template <int HD, typename KVT, int G>
__global__ __launch_bounds__(256) void k_attn_partial(const float *__restrict__ q, int q_stride,
                                                      const KVT *__restrict__ pool, int Hkv,
                                                      const int32_t *__restrict__ table, int table_stride,
                                                      const int32_t *__restrict__ seq_slot,
                                                      const int32_t *__restrict__ ctx_len, int H, int window,
                                                      float scale_log2e, int max_chunks, int cb,
                                                      float *__restrict__ part_o, float *__restrict__ part_ml) {
    constexpr int LPT = HD / 8;      // lanes per key row = lanes of a lane group
    constexpr int NG = WAVE / LPT;   // lane groups per wave
    constexpr int NI = 16 / NG;      // positions of a block per lane group: group g owns slots NI*g .. NI*g+NI-1
    constexpr int NV = HD / LPT;     // value dimensions per lane (= 8): dims sub, sub + LPT, ...
    const int c = blockIdx.x, t = blockIdx.z;
    // G > 1: blockIdx.y is the KV head and the queries are heads kvh*G .. kvh*G+G-1; G == 1: blockIdx.y is the head
    const int h0 = blockIdx.y * G;
    const int kvh = (G > 1) ? blockIdx.y : blockIdx.y / (H / Hkv);
    const int ctx = ctx_len[t];
    const int first = band_first(ctx, window);
    const int nblk = (ctx + 15) >> 4;
    const int b_begin = (first >> 4) + c * cb;
    if (b_begin >= nblk) return;
    const int b_end = min(b_begin + cb, nblk);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int group = lane / LPT, sub = lane % LPT;
    const int64_t block_stride = kv_block_elems(Hkv, HD);
    const int32_t *trow = table + (int64_t)seq_slot[t] * table_stride;

    float qv[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        const float *qp = q + (int64_t)t * q_stride + (h0 + g) * HD + sub * 8;
#pragma unroll
        for (int e = 0; e < 8; e++) qv[g][e] = qp[e] * scale_log2e;
    }
    // Online softmax in the log2 domain, one state per lane group and query: the group's LPT lanes split a
    // key row for the scores and the value dimensions for the weighted sum, always over the group's own
    // NI positions of a block, so that no probability ever crosses a lane group.
    float m[G], l[G], acc[G][NV];
#pragma unroll
    for (int g = 0; g < G; g++) {
        m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
        for (int v = 0; v < NV; v++) acc[g][v] = 0.f;
    }

    // The physical ids of this wave's blocks (b_begin + wave + 4 i; at most 16 of a chunk) are fetched at once,
    // one per lane: a lookup inside the walk would put a dependent memory round trip in front of every block's loads.
    const int n_it = (b_end - b_begin - wave + 3) >> 2;
    const int my_blk = lane < n_it ? trow[b_begin + wave + 4 * lane] : 0;
    for (int it = 0; it < n_it; it++) {
        const int b = b_begin + wave + 4 * it;
        const KVT *blk = pool + (int64_t)__builtin_amdgcn_readlane(my_blk, it) * block_stride;
        // keys: row of slot NI*group + i, elements sub*8 .. +8; a load instruction reads NG rows of 16*LPT bytes
        const KVT *kb = blk + kv_k_offset(HD, kvh, NI * group, sub * 8);
        // values (transposed): dimension sub + LPT*v, slots NI*group .. +NI; a load instruction reads
        // LPT dimensions x 16 slots = one contiguous run
        const KVT *vb = blk + kv_v_offset(Hkv, HD, kvh, NI * group, sub);
        float kf[NI][8], vf[NV][NI];
#pragma unroll
        for (int i = 0; i < NI; i++) load8_stream(kb + i * HD, kf[i]);
#pragma unroll
        for (int v = 0; v < NV; v++) loadn_stream<NI>(vb + v * LPT * 16, vf[v]);
        bool valid[NI];
#pragma unroll
        for (int i = 0; i < NI; i++) {
            const int pos = b * 16 + NI * group + i;
            valid[i] = pos >= first && pos < ctx;
            if (!valid[i]) {        // an unwritten slot may hold anything
#pragma unroll
                for (int v = 0; v < NV; v++) vf[v][i] = 0.f;
            }
        }
#pragma unroll
        for (int g = 0; g < G; g++) {
            float s[NI];
            float mb = -INFINITY;
#pragma unroll
            for (int i = 0; i < NI; i++) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; e++) d = fmaf(qv[g][e], kf[i][e], d);
#pragma unroll
                for (int off = 1; off < LPT; off <<= 1) d += __shfl_xor(d, off, WAVE);
                s[i] = valid[i] ? d : -INFINITY;
                mb = fmaxf(mb, s[i]);
            }
            const float m_new = fmaxf(m[g], mb);
            if (m_new > -INFINITY) {
                const float sc = fast_exp2(m[g] - m_new);
                l[g] *= sc;
#pragma unroll
                for (int v = 0; v < NV; v++) acc[g][v] *= sc;
#pragma unroll
                for (int i = 0; i < NI; i++) {
                    const float p = fast_exp2(s[i] - m_new);
                    l[g] += p;
#pragma unroll
                    for (int v = 0; v < NV; v++) acc[g][v] = fmaf(p, vf[v][i], acc[g][v]);
                }
                m[g] = m_new;
            }
        }
    }
    // merge the lane groups of this wave
#pragma unroll
    for (int g = 0; g < G; g++) {
#pragma unroll
        for (int off = LPT; off < WAVE; off <<= 1) {
            const float m_o = __shfl_xor(m[g], off, WAVE), l_o = __shfl_xor(l[g], off, WAVE);
            const float m_n = fmaxf(m[g], m_o);
            const float a = (m_n > -INFINITY) ? fast_exp2(m[g] - m_n) : 0.f;
            const float bsc = (m_n > -INFINITY) ? fast_exp2(m_o - m_n) : 0.f;
            l[g] = l[g] * a + l_o * bsc;
#pragma unroll
            for (int v = 0; v < NV; v++) acc[g][v] = acc[g][v] * a + __shfl_xor(acc[g][v], off, WAVE) * bsc;
            m[g] = m_n;
        }
    }
    __shared__ float sm_m[4][G], sm_l[4][G], sm_acc[4][G][HD];
    if (lane < LPT) {
#pragma unroll
        for (int g = 0; g < G; g++) {
#pragma unroll
            for (int v = 0; v < NV; v++) sm_acc[wave][g][sub + LPT * v] = acc[g][v];
            if (lane == 0) { sm_m[wave][g] = m[g]; sm_l[wave][g] = l[g]; }
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * HD; idx += 256) {
        const int g = idx / HD, d = idx % HD;
        // a wave that saw no visible position keeps m = -inf and weight 0; wave 0 always sees one
        const float M = fmaxf(fmaxf(sm_m[0][g], sm_m[1][g]), fmaxf(sm_m[2][g], sm_m[3][g]));
        float o = 0.f, L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; w++) {
            const float a = fast_exp2(sm_m[w][g] - M);
            o += a * sm_acc[w][g][d];
            L += a * sm_l[w][g];
        }
        const int64_t item = ((int64_t)t * H + h0 + g) * max_chunks + c;
        part_o[item * HD + d] = o;
        if (d == 0) { part_ml[item * 2] = M; part_ml[item * 2 + 1] = L; }
    }
}

// Merges the chunk partials of one (row, head): 256 threads = 256/HD thread groups, group g takes the
// chunks g, g + 256/HD, ...; the chunk maxima and sums go through LDS first so that the loop over the
// partial outputs has no dependent loads.
template <int HD>
__global__ __launch_bounds__(256) void k_attn_merge(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                                    const int32_t *__restrict__ ctx_len, int H, int window,
                                                    int max_chunks, int cb, float *__restrict__ out,
                                                    bf16_t *__restrict__ xs_out, int T) {
    constexpr int NGRP = 256 / HD, MAXC = 512;   // MAXC: chunks whose statistics fit the LDS cache
    __shared__ float sm_m[MAXC], sm_l[MAXC], sm_o[NGRP][HD], sm_L[NGRP], sm_red[4];
    const int h = blockIdx.x, t = blockIdx.y, d = threadIdx.x % HD, grp = threadIdx.x / HD;
    const int ctx = ctx_len[t];
    const int nch = ((ctx + 15) / 16 - (band_first(ctx, window) >> 4) + cb - 1) / cb;
    const int64_t base = ((int64_t)t * H + h) * max_chunks;
    float mx = -INFINITY;
    for (int c = threadIdx.x; c < nch; c += 256) {
        const float2 ml = *reinterpret_cast<const float2 *>(part_ml + (base + c) * 2);
        if (c < MAXC) { sm_m[c] = ml.x; sm_l[c] = ml.y; }
        mx = fmaxf(mx, ml.x);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, WAVE));
    if ((threadIdx.x & 63) == 0) sm_red[threadIdx.x >> 6] = mx;
    __syncthreads();
    const float M = fmaxf(fmaxf(sm_red[0], sm_red[1]), fmaxf(sm_red[2], sm_red[3]));
    float o = 0.f, L = 0.f;
#pragma unroll 4
    for (int c = grp; c < nch; c += NGRP) {
        const float mc = c < MAXC ? sm_m[c] : part_ml[(base + c) * 2];
        const float lc = c < MAXC ? sm_l[c] : part_ml[(base + c) * 2 + 1];
        const float a = fast_exp2(mc - M);
        o += a * part_o[(base + c) * HD + d];
        L += a * lc;
    }
    sm_o[grp][d] = o;
    if (d == 0) sm_L[grp] = L;
    __syncthreads();
    if (grp != 0) return;
    o = 0.f; L = 0.f;
#pragma unroll
    for (int g = 0; g < NGRP; g++) { o += sm_o[g][d]; L += sm_L[g]; }   // fixed order
    const float r = o / L;
    if (xs_out) {   // operand of the output projection: split (hi, lo) image [2][T][H * HD]
        const bf16_t hi = f32_to_bf16(r);
        xs_out[((int64_t)t * H + h) * HD + d] = hi;
        xs_out[((int64_t)(T + t) * H + h) * HD + d] = f32_to_bf16(r - bf16_to_f32(hi));
    } else {
        out[((int64_t)t * H + h) * HD + d] = r;
    }
}

// ---------------------------------------------------------------- greedy argmax (lowest index on ties)

__global__ __launch_bounds__(1024) void k_argmax(const float *__restrict__ logits, int V, int32_t *__restrict__ out) {
    __shared__ float sv[16];
    __shared__ int si[16];
    const int r = blockIdx.x;
    const float *row = logits + (int64_t)r * V;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    // eight loads in flight per thread, compared in ascending index order (a strict "greater" keeps the lowest
    // index among equal values)
    int i = threadIdx.x;
    for (; i + 7 * 1024 < V; i += 8 * 1024) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = row[i + u * 1024];
#pragma unroll
        for (int u = 0; u < 8; u++)
            if (v[u] > bv || bi == 0x7fffffff) { bv = v[u]; bi = i + u * 1024; }
    }
    for (; i < V; i += 1024) {
        const float v = row[i];
        if (v > bv || bi == 0x7fffffff) { bv = v; bi = i; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(bv, off, WAVE);
        const int oi = __shfl_xor(bi, off, WAVE);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; w++)
            if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
        out[r] = bi;
    }
}

// ---------------------------------------------------------------- token choice with temperature
//
// argmax_i (logit_i / T + g_i), g_i = -log(-log(u_i)) standard Gumbel noise: a draw from softmax(logits / T).
// u_i = (k + 1/2) / 2^23, k = top 23 bits of the SplitMix64 output function applied to
// seed + (counter + 1) * 0x9E3779B97F4A7C15, counter = pos * V + i: a pure function of (seed, pos, i), exact in
// float32.  Rows with temperature 0 are the plain argmax.  Lowest index on ties.

__device__ __forceinline__ float gumbel_noise(uint64_t seed, uint64_t counter) {
    uint64_t z = seed + (counter + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    const float u = ((float)(uint32_t)(z >> 41) + 0.5f) * (1.0f / 8388608.0f);
    return -logf(-logf(u));
}

__global__ __launch_bounds__(1024) void k_sample(const float *__restrict__ logits, int V,
                                                 const float *__restrict__ temperature,
                                                 const uint64_t *__restrict__ seed, const int32_t *__restrict__ pos,
                                                 int32_t *__restrict__ out) {
    __shared__ float sv[16];
    __shared__ int si[16];
    const int r = blockIdx.x;
    const float *row = logits + (int64_t)r * V;
    const float temp = temperature[r];
    const float inv_t = temp > 0.f ? 1.0f / temp : 1.0f;
    const uint64_t sd = seed[r], c0 = (uint64_t)pos[r] * (uint64_t)V;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < V; i += 1024) {
        float v = row[i];
        if (temp > 0.f) v = v * inv_t + gumbel_noise(sd, c0 + i);
        if (v > bv || bi == 0x7fffffff) { bv = v; bi = i; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(bv, off, WAVE);
        const int oi = __shfl_xor(bi, off, WAVE);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; w++)
            if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
        out[r] = bi;
    }
}

// ---------------------------------------------------------------- launch helpers

inline ld_status launched(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        ld::set_error("launch of %s failed: %s", what, hipGetErrorString(e));
        return LD_E_HIP;
    }
    return LD_OK;
}

template <typename WT, int TT, int R, bool NORM>
void launch_linear_epi(const WT *W, const float *x, const float *g, float eps, int T, int N, int K, int epi,
                       float *y, hipStream_t s) {
    dim3 grid((N + 4 * R - 1) / (4 * R), (T + TT - 1) / TT), block(256);
    if (epi == LDK_STORE)
        LD_LAUNCH((k_linear_valu<WT, TT, R, LDK_STORE, NORM>), grid, block, 0, s, W, x, g, eps, T, N, K, y);
    else if (epi == LDK_ADD)
        LD_LAUNCH((k_linear_valu<WT, TT, R, LDK_ADD, NORM>), grid, block, 0, s, W, x, g, eps, T, N, K, y);
    else
        LD_LAUNCH((k_linear_valu<WT, TT, R, LDK_SWIGLU, NORM>), grid, block, 0, s, W, x, g, eps, T, N, K, y);
}

template <typename WT, bool NORM>
void launch_linear(const WT *W, const float *x, const float *g, float eps, int T, int N, int K, int epi, float *y,
                   hipStream_t s) {
    // rows per wave: keep at least ~2048 waves in the grid when N allows it
    const bool wide = (int64_t)N >= 8192 && epi != LDK_SWIGLU;
    if (T == 1) {
        if (wide) launch_linear_epi<WT, 1, 4, NORM>(W, x, g, eps, T, N, K, epi, y, s);
        else launch_linear_epi<WT, 1, 2, NORM>(W, x, g, eps, T, N, K, epi, y, s);
    } else if (T == 2) {
        launch_linear_epi<WT, 2, 2, NORM>(W, x, g, eps, T, N, K, epi, y, s);
    } else if (T <= 4) {
        launch_linear_epi<WT, 4, 2, NORM>(W, x, g, eps, T, N, K, epi, y, s);
    } else {
        launch_linear_epi<WT, 8, 2, NORM>(W, x, g, eps, T, N, K, epi, y, s);
    }
}

}  // namespace

// ---------------------------------------------------------------- C ABI (kernel level)

extern "C" {

ld_status ldk_embed(const void *embed, int32_t dtype, const int32_t *tok, int32_t T, int32_t d, float *x,
                    void *stream) {
    if (!embed || !tok || !x || T < 0 || d <= 0 || d % 8) return ld::fail(LD_E_INVAL, "ldk_embed: bad argument");
    if (T == 0) return LD_OK;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == LD_BF16) LD_LAUNCH(k_embed<bf16_t>, dim3(T), dim3(128), 0, s, (const bf16_t *)embed, tok, d, x);
    else if (dtype == LD_F32) LD_LAUNCH(k_embed<float>, dim3(T), dim3(128), 0, s, (const float *)embed, tok, d, x);
    else return ld::fail(LD_E_INVAL, "ldk_embed: bad dtype");
    return launched("k_embed");
}

ld_status ldk_rmsnorm(const float *x, const float *g, const int32_t *row_idx, int32_t R, int32_t d, float eps,
                      float *out, void *stream) {
    if (!x || !g || !out || R < 0 || d <= 0) return ld::fail(LD_E_INVAL, "ldk_rmsnorm: bad argument");
    if (R == 0) return LD_OK;
    LD_LAUNCH(k_rmsnorm, dim3(R), dim3(256), 0, (hipStream_t)stream, x, g, row_idx, d, eps, out);
    return launched("k_rmsnorm");
}

size_t ldk_linear_scratch_bytes(int32_t T, int32_t N, int32_t K, int32_t epilogue) {
    return (T >= 2 && N > 0 && K >= 128) ? ld::gemm_scratch_bytes(T, N, K, epilogue) : 0;
}

ld_status ldk_linear(const void *W, int32_t dtype, const float *x, const float *g, float eps, int32_t T, int32_t N,
                     int32_t K, int32_t epilogue, float *y, void *scratch, size_t scratch_bytes, void *stream) {
    return ld::linear_pass(W, dtype, x, g, eps, T, N, K, epilogue, y, scratch, scratch_bytes, stream, nullptr);
}

ld_status ldk_linear_f16(const void *W, const void *W_f16, const float *x, const float *g, float eps, int32_t T,
                         int32_t N, int32_t K, int32_t epilogue, float *y, void *scratch, size_t scratch_bytes,
                         int32_t *overflow, void *stream) {
    if (!overflow) return ld::fail(LD_E_INVAL, "ldk_linear_f16: null overflow flag");
    if (!W_f16 && T > 0 && W && N > 0 && K > 0 && K % 8 == 0)   // an image was checked when it was made
        ld::launch_weight_range_check((const uint16_t *)W, (int64_t)N * (epilogue == LDK_SWIGLU ? 2 : 1) * K, overflow,
                                      (hipStream_t)stream);
    return ld::linear_pass(W, LD_BF16, x, g, eps, T, N, K, epilogue, y, scratch, scratch_bytes, stream, overflow, W_f16);
}

ld_status ldk_weights_to_f16(const void *W, int64_t n, void *out, int32_t *overflow, void *stream) {
    if (!W || !out || !overflow || n < 0 || n % 8) return ld::fail(LD_E_INVAL, "ldk_weights_to_f16: bad argument (n must be a multiple of 8)");
    if (n == 0) return LD_OK;
    ld::launch_weight_to_f16((const uint16_t *)W, n, (uint16_t *)out, overflow, (hipStream_t)stream);
    return launched("k_weight_to_f16");
}

}  // extern "C"

int ld::env_flag(const char *name, int dflt) {
    const char *v = getenv(name);
    return v ? atoi(v) : dflt;
}

ld_status ld::linear_pass(const void *W, int32_t dtype, const float *x, const float *g, float eps, int32_t T, int32_t N,
                          int32_t K, int32_t epilogue, float *y, void *scratch, size_t scratch_bytes, void *stream,
                          int *f16_flag, const void *W_f16) {
    if (T == 0) return LD_OK;   // nothing to do: pointers of empty buffers may be null
    if (!W || !x || !y || T < 0 || N <= 0 || K <= 0 || K % 8 || epilogue < 0 || epilogue > 2)
        return ld::fail(LD_E_INVAL, "ldk_linear: bad argument (K must be a multiple of 8)");
    hipStream_t s = (hipStream_t)stream;
    if (dtype == LD_BF16 && T == 1 && ld::gemv1_supported(N, K, epilogue)) {
        ld::launch_gemv1((const bf16_t *)W, x, g, eps, N, K, epilogue, y, nullptr, s);
        return launched("k_gemv1");
    }
    if (dtype == LD_BF16 && scratch && ld::gemm_supported(T, N, K) && scratch_bytes >= ld::gemm_scratch_bytes(T, N, K, epilogue)) {
        ld::launch_norm_split(x, g, eps, T, K, (uint16_t *)scratch, s);
        ld::launch_gemm((const bf16_t *)W, (uint16_t *)scratch, T, N, K, epilogue, y, s, nullptr, f16_flag, (const uint16_t *)W_f16);
        return launched("k_gemm_mfma");
    }
    if (dtype == LD_BF16) {
        if (g) launch_linear<bf16_t, true>((const bf16_t *)W, x, g, eps, T, N, K, epilogue, y, s);
        else launch_linear<bf16_t, false>((const bf16_t *)W, x, g, eps, T, N, K, epilogue, y, s);
    } else if (dtype == LD_F32) {
        if (g) launch_linear<float, true>((const float *)W, x, g, eps, T, N, K, epilogue, y, s);
        else launch_linear<float, false>((const float *)W, x, g, eps, T, N, K, epilogue, y, s);
    } else {
        return ld::fail(LD_E_INVAL, "ldk_linear: bad dtype");
    }
    return launched("k_linear");
}

extern "C" {

ld_status ldk_rope_table(const int32_t *pos, int32_t T, int32_t hd, float rope_base, float *cos_sin, void *stream) {
    if (!pos || !cos_sin || T < 0 || (hd != 64 && hd != 128)) return ld::fail(LD_E_INVAL, "ldk_rope_table: bad argument");
    if (T == 0) return LD_OK;
    LD_LAUNCH(k_rope_table, dim3(T), dim3(64), 0, (hipStream_t)stream, pos, hd, (double)rope_base,
                       (float2 *)cos_sin);
    return launched("k_rope_table");
}

ld_status ldk_rope_kv_write(float *qkv, const float *cos_sin, const int32_t *pos, const int32_t *seq_slot,
                            const int32_t *table, int32_t table_stride, void *pool_layer, int32_t dtype, int32_t T,
                            int32_t H, int32_t Hkv, int32_t hd, void *stream) {
    if (!qkv || !cos_sin || !pos || !seq_slot || !table || !pool_layer || T < 0 || H <= 0 || Hkv <= 0 || H % Hkv ||
        (hd != 64 && hd != 128))
        return ld::fail(LD_E_INVAL, "ldk_rope_kv_write: bad argument");
    if (T == 0) return LD_OK;
    dim3 grid(H + Hkv, T), block(64);
    hipStream_t s = (hipStream_t)stream;
    if (dtype == LD_BF16)
        LD_LAUNCH(k_rope_kv_write<bf16_t>, grid, block, 0, s, qkv, (const float2 *)cos_sin, pos, seq_slot,
                           table, table_stride, (bf16_t *)pool_layer, H, Hkv, hd);
    else if (dtype == LD_F32)
        LD_LAUNCH(k_rope_kv_write<float>, grid, block, 0, s, qkv, (const float2 *)cos_sin, pos, seq_slot,
                           table, table_stride, (float *)pool_layer, H, Hkv, hd);
    else return ld::fail(LD_E_INVAL, "ldk_rope_kv_write: bad dtype");
    return launched("k_rope_kv_write");
}

ld_status ldk_qkv_rope(const void *W, int32_t dtype, const float *x, const float *g, float eps, float *qkv,
                       const float *cos_sin, const int32_t *pos, const int32_t *seq_slot, const int32_t *table,
                       int32_t table_stride, void *pool_layer, int32_t T, int32_t K, int32_t H, int32_t Hkv, int32_t hd,
                       void *scratch, size_t scratch_bytes, void *stream) {
    if (!W || !x || !qkv || !cos_sin || !pos || !seq_slot || !table || !pool_layer || T < 0 || H <= 0 || Hkv <= 0 ||
        H % Hkv || (hd != 64 && hd != 128) || K <= 0 || K % 8)
        return ld::fail(LD_E_INVAL, "ldk_qkv_rope: bad argument");
    if (T == 0) return LD_OK;
    const int N = (H + 2 * Hkv) * hd;
    if (dtype == LD_BF16 && T == 1 && ld::gemv1_supported(N, K, ld::GEMV_ROPE_KV)) {
        ld::RopeKvArgs rk{(const float2 *)cos_sin, pos, seq_slot, table, table_stride, (bf16_t *)pool_layer, H, Hkv, hd};
        ld::launch_gemv1((const bf16_t *)W, x, g, eps, N, K, ld::GEMV_ROPE_KV, qkv, &rk, (hipStream_t)stream);
        return launched("k_gemv1 (rope + cache append)");
    }
    ld_status rc = ldk_linear(W, dtype, x, g, eps, T, N, K, LDK_STORE, qkv, scratch, scratch_bytes, stream);
    if (rc != LD_OK) return rc;
    return ldk_rope_kv_write(qkv, cos_sin, pos, seq_slot, table, table_stride, pool_layer, dtype, T, H, Hkv, hd, stream);
}

// Most KV blocks a row can see: all of its context, or with a band of W positions the blocks that W
// consecutive positions can touch.
static int visible_blocks(int max_ctx, int window) {
    const int all = (max_ctx + 15) / 16;
    return window > 0 ? std::min(all, (window + 14) / 16 + 1) : all;
}
// Query heads that one workgroup serves.  mfma: the matrix-core kernel takes the whole group of a KV head
// (2 .. 16 heads); otherwise the scalar kernel takes it when the group size is 2, 4 or 8.
static int head_group(int H, int Hkv, bool mfma) {
    const int r = H / Hkv;
    if (mfma) return r;
    return (r == 2 || r == 4 || r == 8) ? r : 1;
}
// Chunk size in KV blocks: small chunks when few (row, head group) pairs exist, so that the launch still
// has about two workgroups per CU (measured: a workgroup's fixed cost, table lookup, first loads, merge,
// makes finer chunks slower); a multiple of 4 (one block per wave and round), of 8 for the matrix-core kernel
// (two blocks per wave and round).  At most 32 blocks (512 tokens) per chunk in the scalar kernel and 64 in the
// matrix-core kernel: contexts in a batch differ, so the longest chunks set the tail of the launch, and with 64
// the scalar kernel measured 12 % slower at batch 32 (contexts 512 .. 8192) and 36 % slower at batch 16
// (contexts 256 .. 4096), where all workgroups fit the chip at once; 16 and 32 measure alike.
static int attn_chunk_cap(bool mfma) { return mfma ? 64 : 32; }
static int attn_chunk_blocks(int T, int H, int Hkv, int max_ctx, int window, bool mfma) {
    const int64_t blocks = (int64_t)T * (H / head_group(H, Hkv, mfma)) * visible_blocks(max_ctx, window);
    const int q = mfma ? 8 : 4;
    int64_t cb = (blocks + 511) / 512;
    cb = (cb + q - 1) / q * q;
    return (int)std::min<int64_t>(std::max<int64_t>(cb, q), attn_chunk_cap(mfma));
}
static int attn_max_chunks(int T, int H, int Hkv, int max_ctx, int window, bool mfma) {
    const int cb = attn_chunk_blocks(T, H, Hkv, max_ctx, window, mfma);
    return (visible_blocks(max_ctx, window) + cb - 1) / cb;
}

// Most chunks any launch with contexts up to max_ctx can use.  The chunk size follows the launch's own
// longest context, so the chunk count is not monotonic in it: bound it over all shorter contexts.  With nb
// visible blocks, cb >= T * units * nb / 512 gives nb / cb <= 512 / (T * units) unless cb hit its cap,
// where the count is nb / cap; and cb >= q gives nb / q.
static int attn_chunk_bound(int T, int H, int Hkv, int max_ctx, int window, bool mfma) {
    const int q = mfma ? 8 : 4, cap = attn_chunk_cap(mfma);
    const int64_t units = (int64_t)T * (H / head_group(H, Hkv, mfma));
    const int64_t nb = visible_blocks(max_ctx, window);
    const int64_t by_target = std::max<int64_t>(512 / units + 1, (nb + cap - 1) / cap), by_min = (nb + q - 1) / q;
    return (int)std::max<int64_t>(1, std::min(by_target, by_min));
}

size_t ldk_attention_scratch_bytes(int32_t T, int32_t H, int32_t Hkv, int32_t hd, int32_t max_ctx, int32_t window) {
    if (T <= 0 || H <= 0 || Hkv <= 0 || H % Hkv || hd <= 0 || max_ctx <= 0 || window < 0) return 0;
    int mc = attn_chunk_bound(T, H, Hkv, max_ctx, window, false);     // enough for either kernel
    if (ld::grouped_decode_supported(1, hd, H, Hkv)) mc = std::max(mc, attn_chunk_bound(T, H, Hkv, max_ctx, window, true));
    return (size_t)T * H * mc * (hd + 2) * sizeof(float);
}

static ld_status paged_attention_impl(const float *q, int32_t q_stride, const void *pool_layer, int32_t dtype,
                                      const int32_t *table, int32_t table_stride, const int32_t *seq_slot,
                                      const int32_t *ctx_len, int32_t max_ctx, int32_t T, int32_t H, int32_t Hkv,
                                      int32_t hd, int32_t window, float *out, uint16_t *xs_out, void *scratch,
                                      size_t scratch_bytes, void *stream, int image_rows = 0) {
    if (T == 0) return LD_OK;
    if (!q || !pool_layer || !table || !seq_slot || !ctx_len || (!out && !xs_out) || !scratch || T < 0 || H <= 0 ||
        Hkv <= 0 || H % Hkv || (hd != 64 && hd != 128) || max_ctx <= 0 || window < 0)
        return ld::fail(LD_E_INVAL, "ldk_paged_attention: bad argument");
    const bool mfma = ld::grouped_decode_supported(dtype == LD_BF16, hd, H, Hkv);
    const int mc = attn_max_chunks(T, H, Hkv, max_ctx, window, mfma);
    if (scratch_bytes < (size_t)T * H * mc * (hd + 2) * sizeof(float))
        return ld::fail(LD_E_INVAL, "ldk_paged_attention: scratch too small");
    const int cb = attn_chunk_blocks(T, H, Hkv, max_ctx, window, mfma);
    const int G = head_group(H, Hkv, mfma);
    float *part_o = (float *)scratch;
    float *part_ml = part_o + (size_t)T * H * mc * hd;
    const float sl2 = (float)(1.4426950408889634 / std::sqrt((double)hd));
    dim3 grid(mc, H / G, T), block(256);
    hipStream_t s = (hipStream_t)stream;
    const int img = image_rows > 0 ? image_rows : T;     // rows of the split image the low parts sit behind
    if (mfma) {
        ld::launch_grouped_decode_partial(q, q_stride, (const uint16_t *)pool_layer, Hkv, table, table_stride, seq_slot,
                                          ctx_len, T, H, window, mc, cb, part_o, part_ml, s);
        LD_LAUNCH((k_attn_merge<128>), dim3(H, T), dim3(256), 0, s, part_o, part_ml, ctx_len, H, window, mc, cb, out,
                  xs_out, img);
        return launched("k_attn (grouped)");
    }
#define LD_ATT_G(HD_, KVT_, G_)                                                                                    \
    LD_LAUNCH((k_attn_partial<HD_, KVT_, G_>), grid, block, 0, s, q, q_stride, (const KVT_ *)pool_layer, Hkv,     \
              table, table_stride, seq_slot, ctx_len, H, window, sl2, mc, cb, part_o, part_ml)
#define LD_ATT(HD_, KVT_)                                                                                          \
    do {                                                                                                           \
        if (G == 8) LD_ATT_G(HD_, KVT_, 8);                                                                       \
        else if (G == 4) LD_ATT_G(HD_, KVT_, 4);                                                                  \
        else if (G == 2) LD_ATT_G(HD_, KVT_, 2);                                                                  \
        else LD_ATT_G(HD_, KVT_, 1);                                                                              \
        LD_LAUNCH((k_attn_merge<HD_>), dim3(H, T), dim3(256), 0, s, part_o, part_ml, ctx_len, H, window, mc, cb,  \
                  out, xs_out, img);                                                                               \
    } while (0)
    if (dtype == LD_BF16 && hd == 128) LD_ATT(128, bf16_t);
    else if (dtype == LD_BF16 && hd == 64) LD_ATT(64, bf16_t);
    else if (dtype == LD_F32 && hd == 128) LD_ATT(128, float);
    else if (dtype == LD_F32 && hd == 64) LD_ATT(64, float);
    else return ld::fail(LD_E_INVAL, "ldk_paged_attention: bad dtype");
#undef LD_ATT
#undef LD_ATT_G
    return launched("k_attn");
}

ld_status ldk_paged_attention(const float *q, int32_t q_stride, const void *pool_layer, int32_t dtype,
                              const int32_t *table, int32_t table_stride, const int32_t *seq_slot,
                              const int32_t *ctx_len, int32_t max_ctx, int32_t T, int32_t H, int32_t Hkv, int32_t hd,
                              int32_t window, float *out, void *scratch, size_t scratch_bytes, void *stream) {
    return paged_attention_impl(q, q_stride, pool_layer, dtype, table, table_stride, seq_slot, ctx_len, max_ctx, T, H, Hkv,
                                hd, window, out, nullptr, scratch, scratch_bytes, stream);
}

// ---- the same attention for callers that cannot allocate: the chunk partials live in a file-scope device
// array instead of a caller's buffer.  In host code the array's name is only a handle for the runtime's
// symbol lookup; the address each device holds its copy at comes from hipGetSymbolAddress, asked once per
// device with that device current, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char ld_static_scratch[LDK_STATIC_SCRATCH_BYTES];

static ld_status static_scratch_ptr(void **out) {
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static void *ptr[MAX_DEV] = {nullptr};
    int dev = -1;
    LD_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEV) return ld::fail(LD_E_RANGE, "ldk_paged_attention_static: device ordinal beyond 63");
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        LD_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(ld_static_scratch)));
        if (!p || ((uintptr_t)p & 255)) return ld::fail(LD_E_HIP, "ldk_paged_attention_static: bad address of the device array");
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return LD_OK;
}

size_t ldk_static_scratch_bytes(void) { return LDK_STATIC_SCRATCH_BYTES; }

ld_status ldk_paged_attention_static(const float *q, int32_t q_stride, const void *pool_layer, int32_t dtype,
                                     const int32_t *table, int32_t table_stride, const int32_t *seq_slot,
                                     const int32_t *ctx_len, int32_t max_ctx, int32_t T, int32_t H, int32_t Hkv,
                                     int32_t hd, int32_t window, float *out, void *stream) {
    if (T == 0) return LD_OK;
    if (T < 0 || H <= 0 || Hkv <= 0 || H % Hkv || (hd != 64 && hd != 128) || max_ctx <= 0 || window < 0)
        return ld::fail(LD_E_INVAL, "ldk_paged_attention_static: bad argument");
    // what this launch itself needs (not the bound over all shorter contexts a reusable buffer is sized by)
    const bool mfma = ld::grouped_decode_supported(dtype == LD_BF16, hd, H, Hkv);
    const size_t need = (size_t)T * H * attn_max_chunks(T, H, Hkv, max_ctx, window, mfma) * (hd + 2) * sizeof(float);
    if (need > LDK_STATIC_SCRATCH_BYTES) {
        ld::set_error("ldk_paged_attention_static: %zu bytes of chunk partials exceed the built-in %zu; use "
                      "ldk_paged_attention with a buffer of the caller's", need, (size_t)LDK_STATIC_SCRATCH_BYTES);
        return LD_E_RANGE;
    }
    void *dev_scratch = nullptr;
    ld_status rc = static_scratch_ptr(&dev_scratch);
    if (rc != LD_OK) return rc;
    return paged_attention_impl(q, q_stride, pool_layer, dtype, table, table_stride, seq_slot, ctx_len, max_ctx, T, H, Hkv,
                                hd, window, out, nullptr, dev_scratch, LDK_STATIC_SCRATCH_BYTES, stream);
}

size_t ldk_prefill_attention_scratch_bytes(void) { return ld::prefill_attention_scratch_bytes(); }

ld_status ldk_prefill_attention(const float *q, int32_t q_stride, const void *pool_layer, int32_t dtype,
                                const int32_t *table, int32_t table_stride, const int32_t *tiles, int32_t n_tiles,
                                int32_t H, int32_t Hkv, int32_t hd, int32_t window, int32_t max_pos, float *out,
                                void *scratch, size_t scratch_bytes, void *stream) {
    return ldk_prefill_attention_f16(q, q_stride, pool_layer, dtype, table, table_stride, tiles, n_tiles, H, Hkv, hd, window,
                                     max_pos, out, scratch, scratch_bytes, nullptr, stream);
}

ld_status ldk_prefill_attention_f16(const float *q, int32_t q_stride, const void *pool_layer, int32_t dtype,
                                    const int32_t *table, int32_t table_stride, const int32_t *tiles, int32_t n_tiles,
                                    int32_t H, int32_t Hkv, int32_t hd, int32_t window, int32_t max_pos, float *out,
                                    void *scratch, size_t scratch_bytes, int32_t *overflow, void *stream) {
    if (!q || !pool_layer || !table || !tiles || !out || n_tiles < 0 || H <= 0 || Hkv <= 0 || H % Hkv || q_stride % 4 ||
        window < 0 || max_pos < 0)
        return ld::fail(LD_E_INVAL, "ldk_prefill_attention: bad argument");
    if (!ld::prefill_attention_supported(dtype == LD_BF16, hd))
        return ld::fail(LD_E_INVAL, "ldk_prefill_attention: needs a bf16 pool and head_dim 128");
    if (n_tiles == 0) return LD_OK;
    ld::launch_prefill_attention(q, q_stride, (const uint16_t *)pool_layer, Hkv, table, table_stride, tiles, n_tiles, H,
                                 window, max_pos, out, scratch, scratch_bytes, (hipStream_t)stream, nullptr, nullptr, overflow);
    return launched("k_attn_prefill");
}

ld_status ldk_argmax(const float *logits, int32_t R, int32_t V, int32_t *out, void *stream) {
    if (R == 0) return LD_OK;
    if (!logits || !out || R < 0 || V <= 0) return ld::fail(LD_E_INVAL, "ldk_argmax: bad argument");
    LD_LAUNCH(k_argmax, dim3(R), dim3(1024), 0, (hipStream_t)stream, logits, V, out);
    return launched("k_argmax");
}

ld_status ldk_sample(const float *logits, int32_t R, int32_t V, const float *temperature, const uint64_t *seed,
                     const int32_t *pos, int32_t *out, void *stream) {
    if (R == 0) return LD_OK;
    if (!logits || !temperature || !seed || !pos || !out || R < 0 || V <= 0)
        return ld::fail(LD_E_INVAL, "ldk_sample: bad argument");
    LD_LAUNCH(k_sample, dim3(R), dim3(1024), 0, (hipStream_t)stream, logits, V, temperature, seed, pos, out);
    return launched("k_sample");
}

}  // extern "C"

namespace ld {

// Single-query paged attention whose output is written as the split (hi, lo) bf16 operand of the
// output projection: xs_out [2][image_rows][H * hd], of which these T rows are the first (image_rows 0: T).
ld_status paged_attention_split(const float *q, int q_stride, const void *pool_layer, int dtype, const int32_t *table,
                                int table_stride, const int32_t *seq_slot, const int32_t *ctx_len, int max_ctx, int T,
                                int H, int Hkv, int hd, int window, uint16_t *xs_out, void *scratch,
                                size_t scratch_bytes, hipStream_t stream, int image_rows) {
    return paged_attention_impl(q, q_stride, pool_layer, dtype, table, table_stride, seq_slot, ctx_len, max_ctx, T, H, Hkv,
                                hd, window, nullptr, xs_out, scratch, scratch_bytes, (void *)stream, image_rows);
}

}  // namespace ld
