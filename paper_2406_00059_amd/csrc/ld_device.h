// Device-side helpers shared by the kernel files: element conversion, 16-byte loads, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ldd {

constexpr int WAVE = 64;
typedef uint16_t bf16_t;

// ---------------------------------------------------------------- element helpers

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// float32 -> bf16, round to nearest even (the hardware conversion, v_cvt_pk_bf16_f32).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

// Two conversions in one instruction: low half = bf16(a), high half = bf16(b).
__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){a, b}, bf16x2_t));
}

// x = hi + lo with both parts bf16: returns the packed high parts of (a, b), stores the packed low parts.
__device__ __forceinline__ uint32_t split2_bf16(float a, float b, uint32_t &lo) {
    const uint32_t hi = pack2_bf16(a, b);
    lo = pack2_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
    return hi;
}

// Writes v as a GEMM operand: high and low bf16 parts at the same index of the two images.
__device__ __forceinline__ void store_split(bf16_t *__restrict__ hi, bf16_t *__restrict__ lo, int64_t idx, float v) {
    uint32_t l;
    const uint32_t h = split2_bf16(v, 0.f, l);
    hi[idx] = (bf16_t)h;
    lo[idx] = (bf16_t)l;
}
// Rotation of the pair (a, b) by the angle whose (cos, sin) is c, every product rounded: the kernels that rotate
// a row's q and k heads must agree bit for bit.
__device__ __forceinline__ float2 rope_rotate(float a, float b, float2 c) {
#pragma clang fp contract(off)
    return make_float2(a * c.x - b * c.y, a * c.y + b * c.x);
}
// a * b rounded to float, never fused into a following addition or subtraction.
__device__ __forceinline__ float mul_rounded(float a, float b) {
#pragma clang fp contract(off)
    return a * b;
}

// Load 8 consecutive elements (16-byte aligned for bf16, 32-byte for float) as floats.
__device__ __forceinline__ void load8(const bf16_t *p, float (&v)[8]) {
    const uint4 u = *reinterpret_cast<const uint4 *>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void load8(const float *p, float (&v)[8]) {
    const float4 a = reinterpret_cast<const float4 *>(p)[0];
    const float4 b = reinterpret_cast<const float4 *>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

__device__ __forceinline__ void store_elem(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(bf16_t *p, float v) { *p = f32_to_bf16(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// 16-byte load of data that is read exactly once (weights, cached keys/values): the non-temporal hint
// keeps the stream from displacing reusable lines in the caches.
__device__ __forceinline__ u32x4_t load_stream16(const void *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
}

// load8 with the streaming hint (bf16: one 16-byte load; float: two).
__device__ __forceinline__ void load8_stream(const bf16_t *p, float (&v)[8]) {
    const u32x4_t u = load_stream16(p);
#pragma unroll
    for (int i = 0; i < 4; i++) {
        v[2 * i] = __uint_as_float(u[i] << 16);
        v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void load8_stream(const float *p, float (&v)[8]) {
    const u32x4_t a = load_stream16(p), b = load_stream16(p + 4);
#pragma unroll
    for (int i = 0; i < 4; i++) {
        v[i] = __uint_as_float(a[i]);
        v[4 + i] = __uint_as_float(b[i]);
    }
}

// N = 2 or 4 consecutive elements with the streaming hint, as floats (aligned to N elements).
template <int N>
__device__ __forceinline__ void loadn_stream(const bf16_t *p, float (&v)[N]) {
    typedef uint32_t uN __attribute__((ext_vector_type(N / 2)));
    static_assert(N == 4, "bf16: four elements (8 bytes)");
    const uN u = __builtin_nontemporal_load(reinterpret_cast<const uN *>(p));
#pragma unroll
    for (int i = 0; i < N / 2; i++) {
        v[2 * i] = __uint_as_float(u[i] << 16);
        v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
}
template <>
__device__ __forceinline__ void loadn_stream<2>(const bf16_t *p, float (&v)[2]) {
    const uint32_t u = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p));
    v[0] = __uint_as_float(u << 16);
    v[1] = __uint_as_float(u & 0xffff0000u);
}
template <int N>
__device__ __forceinline__ void loadn_stream(const float *p, float (&v)[N]) {
    typedef float fN __attribute__((ext_vector_type(N)));
    const fN u = __builtin_nontemporal_load(reinterpret_cast<const fN *>(p));
#pragma unroll
    for (int i = 0; i < N; i++) v[i] = u[i];
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also carries a memory fence, which
// on this target waits for every outstanding global load (vmcnt(0)) and so drains loads that were
// issued ahead on purpose; this one waits for the LDS/scalar counter only and leaves them in flight.
// Use it only where the data exchanged between waves goes through LDS.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---------------------------------------------------------------- layout of one KV block
// A block holds 16 positions of every KV head: the keys position-major, [kv_head][slot][hd], then the
// values TRANSPOSED, [kv_head][hd][slot].  A key row (one position, hd elements) is contiguous, which is
// the operand shape of q.k; a value row of the transposed part holds the 16 positions of one dimension,
// contiguous, which is the operand shape of the probability-weighted sum on the matrix cores (the
// contraction runs over positions) and costs the scalar kernels nothing.  Offsets in elements:
__device__ __forceinline__ int64_t kv_block_elems(int Hkv, int hd) { return (int64_t)2 * Hkv * 16 * hd; }
__device__ __forceinline__ int64_t kv_k_offset(int hd, int kvh, int slot, int dim) {
    return ((int64_t)kvh * 16 + slot) * hd + dim;
}
__device__ __forceinline__ int64_t kv_v_offset(int Hkv, int hd, int kvh, int slot, int dim) {
    return (int64_t)Hkv * 16 * hd + ((int64_t)kvh * hd + dim) * 16 + slot;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// acc + p[0] + p[stride] + ... + p[(ks - 1) stride], added in that order (split-K slabs: the order is part of
// the result).  The loads of eight (then four) slabs are issued together; a plain loop would pay one memory
// latency per slab.
template <typename V>
__device__ __forceinline__ V slab_sum(const V *p, int64_t stride, int ks, V acc) {
    int z = 0;
    for (; z + 8 <= ks; z += 8) {
        V v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = p[(z + u) * stride];
#pragma unroll
        for (int u = 0; u < 8; u++) acc += v[u];
    }
    if (z + 4 <= ks) {
        V v[4];
#pragma unroll
        for (int u = 0; u < 4; u++) v[u] = p[(z + u) * stride];
#pragma unroll
        for (int u = 0; u < 4; u++) acc += v[u];
        z += 4;
    }
    for (; z < ks; z++) acc += p[z * stride];
    return acc;
}


}  // namespace ldd
