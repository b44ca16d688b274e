// Decoder layer for a decode batch of 2..32 rows (bf16 weights, head_dim 128).
//
// Each projection is the skinny MFMA product (ld_gemm.hip), which leaves per-slab partial sums.  Instead
// of a generic reduce kernel followed by a separate normalise/split kernel, the slab sums are added by
// the kernel that produces the NEXT operand, so a layer is 4 products + 4 small element-wise kernels
// (+ attention):
//   k_red_rope         : q/k/v sums -> 1/rms scale -> RoPE -> q (float32) and k, v into the paged pool
//   (attention)        : writes its output directly as a split (hi, lo) bf16 operand
//   k_red_add_split    : residual += sums; operand for the next product = split(residual * gain);
//                        per-workgroup partial sums of squares of the new residual
//   k_red_swiglu_split : silu(gate) * up from the gate/up sums -> split operand of the down projection
// RMSNorm: the gain is applied to the operand, the scalar 1/rms is applied to the finished sums by the
// consumer, which adds the few partial sums of squares in fixed order (deterministic).
#include "ld_batch.h"
#include "ld_gemm.h"
#include "ld_device.h"
#include "ld_internal.h"
#include <algorithm>

using namespace ldd;

namespace {

constexpr int RB = 1024;   // columns of one row handled by a workgroup of k_red_add_split (256 threads x 4)

__device__ __forceinline__ void split4(const float (&v)[4], uint2 &hi, uint2 &lo) {
    hi.x = split2_bf16(v[0], v[1], lo.x);
    hi.y = split2_bf16(v[2], v[3], lo.y);
}

__device__ __forceinline__ float row_rstd(const float *ss_part, int t, int nssp, int d, float eps) {
    float s = 0.f;
    for (int j = 0; j < nssp; j++) s += ss_part[t * nssp + j];
    return 1.0f / sqrtf(s / d + eps);
}

// x[t, :] += sum_z partial[z][t][:]  (ks may be 0: no sums to add);  if g: xs = split(x * g) and
// ss_part[t][blockIdx.x] = sum over this workgroup's columns of x^2.   grid (d / RB, T), 256 threads.
__global__ __launch_bounds__(256) void k_red_add_split(const float *__restrict__ partial, int ks, float *__restrict__ x,
                                                       const float *__restrict__ g, int T, int d,
                                                       bf16_t *__restrict__ xs, float *__restrict__ ss_part) {
    __shared__ float red[4];
    const int t = blockIdx.y, n = blockIdx.x * RB + threadIdx.x * 4;
    float4 v = *reinterpret_cast<const float4 *>(x + (int64_t)t * d + n);
    if (ks) v = slab_sum(reinterpret_cast<const float4 *>(partial + (int64_t)t * d + n), (int64_t)T * d / 4, ks, v);
    if (ks) *reinterpret_cast<float4 *>(x + (int64_t)t * d + n) = v;
    if (!g) return;
    const float4 gv = *reinterpret_cast<const float4 *>(g + n);
    const float f[4] = {v.x * gv.x, v.y * gv.y, v.z * gv.z, v.w * gv.w};
    uint2 hi, lo;
    split4(f, hi, lo);
    *reinterpret_cast<uint2 *>(xs + (int64_t)t * d + n) = hi;
    *reinterpret_cast<uint2 *>(xs + (int64_t)(T + t) * d + n) = lo;
    float ss = wave_sum(v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) ss_part[t * gridDim.x + blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

// One thread per (row t, head hh of H + 2 Hkv, pair i < 64).
__global__ __launch_bounds__(256) void k_red_rope(const float *__restrict__ partial, int ks, const float *__restrict__ ss_part,
                                                  int nssp, float eps, int d, int T, int H, int Hkv,
                                                  const float2 *__restrict__ cs, const int32_t *__restrict__ pos,
                                                  const int32_t *__restrict__ seq_slot, const int32_t *__restrict__ table,
                                                  int table_stride, float *__restrict__ q, int q_stride,
                                                  bf16_t *__restrict__ pool) {
    constexpr int HD = 128, HALF = 64;
    const int heads = H + 2 * Hkv, nqkv = heads * HD;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= T * heads * HALF) return;
    const int i = idx % HALF, hh = (idx / HALF) % heads, t = idx / (HALF * heads);
    const float *p0 = partial + (int64_t)t * nqkv + hh * HD + i;
    float a = slab_sum(p0, (int64_t)T * nqkv, ks, 0.f), b = slab_sum(p0 + HALF, (int64_t)T * nqkv, ks, 0.f);
    const float rstd = row_rstd(ss_part, t, nssp, d, eps);
    a *= rstd;
    b *= rstd;
    if (hh < H + Hkv) {
        const float2 c = cs[t * HALF + i];
        const float ra = a * c.x - b * c.y, rb = a * c.y + b * c.x;
        a = ra;
        b = rb;
    }
    if (hh < H) {
        float *dst = q + (int64_t)t * q_stride + hh * HD;
        dst[i] = a;
        dst[i + HALF] = b;
    } else {
        const int which = hh < H + Hkv ? 0 : 1, j = hh - H - which * Hkv, p = pos[t];
        const int64_t phys = table[(int64_t)seq_slot[t] * table_stride + (p >> 4)];
        bf16_t *blk = pool + phys * kv_block_elems(Hkv, HD);
        const int slot = p & 15;
        if (which == 0) {
            blk[kv_k_offset(HD, j, slot, i)] = f32_to_bf16(a);
            blk[kv_k_offset(HD, j, slot, i + HALF)] = f32_to_bf16(b);
        } else {
            blk[kv_v_offset(Hkv, HD, j, slot, i)] = f32_to_bf16(a);
            blk[kv_v_offset(Hkv, HD, j, slot, i + HALF)] = f32_to_bf16(b);
        }
    }
}

// One thread per (row t, 4 outputs): act = silu(rstd * gate) * (rstd * up) -> split operand [T, F].
__global__ __launch_bounds__(256) void k_red_swiglu_split(const float *__restrict__ partial, int ks,
                                                          const float *__restrict__ ss_part, int nssp, float eps, int d,
                                                          int T, int F, bf16_t *__restrict__ xs) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)T * (F / 4)) return;
    const int t = (int)(idx / (F / 4)), n = (int)(idx % (F / 4)) * 4;
    const float4 *p0 = reinterpret_cast<const float4 *>(partial + (int64_t)t * (2 * F) + n);
    const float4 gs = slab_sum(p0, (int64_t)T * (2 * F) / 4, ks, make_float4(0, 0, 0, 0));
    const float4 us = slab_sum(p0 + F / 4, (int64_t)T * (2 * F) / 4, ks, make_float4(0, 0, 0, 0));
    const float rstd = row_rstd(ss_part, t, nssp, d, eps);
    const float gg[4] = {gs.x * rstd, gs.y * rstd, gs.z * rstd, gs.w * rstd};
    const float uu[4] = {us.x * rstd, us.y * rstd, us.z * rstd, us.w * rstd};
    float act[4];
#pragma unroll
    for (int e = 0; e < 4; e++) act[e] = gg[e] / (1.0f + __expf(-gg[e])) * uu[e];
    uint2 hi, lo;
    split4(act, hi, lo);
    *reinterpret_cast<uint2 *>(xs + (int64_t)t * F + n) = hi;
    *reinterpret_cast<uint2 *>(xs + (int64_t)(T + t) * F + n) = lo;
}

}  // namespace

namespace ld {

bool batch_layer_supported(int T, int d, int H, int Hkv, int hd, int ffn) {
    return T >= 2 && T <= 32 && hd == 128 && d % RB == 0 && (H * hd) % 128 == 0 && ffn % 128 == 0 && H % Hkv == 0;
}
size_t batch_layer_xs_bytes(int T, int d, int H, int hd, int ffn) {
    return (size_t)2 * T * std::max(std::max(d, H * hd), ffn) * sizeof(bf16_t);
}
size_t batch_layer_partial_bytes(int T, int d, int H, int Hkv, int hd, int ffn) {
    const size_t nqkv = (size_t)(H + 2 * Hkv) * hd, nq = (size_t)H * hd;
    size_t m = skinny_slabs(d) * nqkv;                       // q/k/v: K = d
    m = std::max(m, (size_t)skinny_slabs((int)nq) * d);      // wo: K = nq
    m = std::max(m, (size_t)skinny_slabs(d) * 2 * ffn);      // gate/up: K = d
    m = std::max(m, (size_t)skinny_slabs(ffn) * d);          // down: K = ffn
    return m * T * sizeof(float);
}
size_t batch_layer_ss_bytes(int T, int d) { return (size_t)2 * T * (d / RB) * sizeof(float); }

void launch_batch_prepare(const float *x, const float *g, int T, int d, uint16_t *xs, float *ss_part, hipStream_t s) {
    LD_LAUNCH(k_red_add_split, dim3(d / RB, T), dim3(256), 0, s, nullptr, 0, const_cast<float *>(x), g, T, d, xs,
                       ss_part);
}

void launch_batch_qkv(const BatchLayerArgs &a, hipStream_t s) {
    const int nqkv = (a.H + 2 * a.Hkv) * a.hd, nssp = a.d / RB;
    launch_gemm_skinny(a.wqkv, a.xs, a.xs + (size_t)a.T * a.d, a.T, nqkv, a.d, a.partial, s);
    const int n = a.T * (a.H + 2 * a.Hkv) * 64;
    LD_LAUNCH(k_red_rope, dim3((n + 255) / 256), dim3(256), 0, s, a.partial, skinny_slabs(a.d), a.ss_part, nssp,
                       a.eps, a.d, a.T, a.H, a.Hkv, (const float2 *)a.cos_sin, a.pos, a.seq_slot, a.table, a.table_stride,
                       a.q, a.q_stride, a.pool);
}

void launch_batch_wo(const BatchLayerArgs &a, hipStream_t s) {
    // output projection; residual; operand + statistics of the FFN norm
    const int nq = a.H * a.hd, nssp = a.d / RB;
    launch_gemm_skinny(a.wo, a.xs, a.xs + (size_t)a.T * nq, a.T, a.d, nq, a.partial, s);
    LD_LAUNCH(k_red_add_split, dim3(nssp, a.T), dim3(256), 0, s, a.partial, skinny_slabs(nq), a.x, a.ffn_norm, a.T,
                       a.d, a.xs, a.ss_part + (size_t)a.T * nssp);
}

void launch_batch_gate_up(const BatchLayerArgs &a, hipStream_t s) {
    // gate/up; SwiGLU; operand of the down projection
    const int nssp = a.d / RB;
    launch_gemm_skinny(a.wgate_up, a.xs, a.xs + (size_t)a.T * a.d, a.T, 2 * a.ffn, a.d, a.partial, s);
    const int64_t n = (int64_t)a.T * (a.ffn / 4);
    LD_LAUNCH(k_red_swiglu_split, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a.partial, skinny_slabs(a.d),
                       a.ss_part + (size_t)a.T * nssp, nssp, a.eps, a.d, a.T, a.ffn, a.xs);
}

void launch_batch_down(const BatchLayerArgs &a, hipStream_t s) {
    // down; residual; operand + statistics of the next layer's attention norm
    const int nssp = a.d / RB;
    launch_gemm_skinny(a.wdown, a.xs, a.xs + (size_t)a.T * a.ffn, a.T, a.d, a.ffn, a.partial, s);
    LD_LAUNCH(k_red_add_split, dim3(nssp, a.T), dim3(256), 0, s, a.partial, skinny_slabs(a.ffn), a.x, a.next_norm,
                       a.T, a.d, a.xs, a.ss_part);
}

}  // namespace ld
