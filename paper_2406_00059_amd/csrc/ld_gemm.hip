// Linear layers on T >= 2 rows with the matrix cores: Y[T, N] = X[T, K] W[N, K]^T, W bf16.
//
// Precision: the float32 activations are split into two bf16 numbers, x = hi + lo (|lo| <= 2^-9 |hi|),
// and both parts are multiplied with the (exact) bf16 weights and accumulated in float32, so the
// product carries ~16 significant bits of the activation instead of 8.  In the decode regime the
// kernel is bound by the weight stream from HBM, where the second MFMA pass is free.
//
// Three kernels by row count, all with the token index on the MFMA row side (an accumulator register
// then holds 32 consecutive output columns of one token and stores are 128-byte contiguous), all fed
// by the (hi, lo) bf16 images of the activations, which k_norm_split writes in a pass of its own or a
// producer writes directly (k_reduce_add_norm_split and the SwiGLU epilogues here, the attention kernels,
// the fused reducers of ld_batch.hip):
//  - k_gemm_skinny (2..48 rows): weight-stream bound; slab-resident, see its comment.
//  - k_gemm_mfma (49..64 rows): W streamed from global memory straight into B-operand registers
//    (lane (n = lane % 32, h = lane / 32) loads 16 bytes of row n; the contraction order over k is
//    permuted so that the four loads of a 64-wide k-group give a row 128 contiguous bytes), X staged
//    through padded LDS, loads issued one chunk ahead.
//  - k_gemm_big (> 64 rows): MFMA-bound; both operands through LDS, see its comment.
// Workgroups that share a W panel (same columns, different token tiles) are mapped to the same XCD so
// that the panel is fetched into one L2 only.  Split-K partial sums are added in fixed slab order.
#include "ld_gemm.h"
#include "ld_device.h"
#include "ld_internal.h"
#include <algorithm>
#include <cstdlib>

using namespace ldd;

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) __fp16 fp16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // native 16-byte vector (keeps arrays of it in registers)

constexpr float F16_LIMIT = 65504.f;   // largest finite fp16

// Eight bf16 numbers as fp16: exact where fp16 can hold the value (8 significant bits fit into 11; truncation
// only below 2^-14, where a bf16 weight is lost in the sums anyway).
__device__ __forceinline__ f16x8 bf16x8_to_f16x8(const __attribute__((ext_vector_type(4))) uint32_t &w) {
    uint32_t h[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
        h[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w[i] << 16), __uint_as_float(w[i] & 0xffff0000u)));
    return __builtin_bit_cast(f16x8, (__attribute__((ext_vector_type(4))) uint32_t){h[0], h[1], h[2], h[3]});
}

constexpr int KC = 128;          // K granularity the launcher requires (largest chunk any variant stages)
constexpr int XPAD = 8;          // bf16 elements of row padding in LDS
constexpr int NW = 4;            // waves per workgroup

// SwiGLU of one (gate, up) pair with the last product rounded to float, as a store to memory would: where the
// value goes straight into the bf16 split, a product fused into the split's subtraction would change the low part.
__device__ __forceinline__ float swiglu(float gate, float up) {
#pragma clang fp contract(off)
    return gate / (1.0f + __expf(-gate)) * up;
}

// Sum of squares in a fixed order of fused multiply-adds: the kernels that normalise a row must agree bit for bit.
__device__ __forceinline__ float add_squares(float ss, const float4 &v) {
    ss = fmaf(v.x, v.x, ss);
    ss = fmaf(v.y, v.y, ss);
    ss = fmaf(v.z, v.z, ss);
    return fmaf(v.w, v.w, ss);
}

// v * rstd * g with both products rounded: the split that follows subtracts the rounded value's high part, and a
// product fused into that subtraction would give a different low part in one kernel than in another.
__device__ __forceinline__ float4 scale4(const float4 &v, float rstd, const float4 &g) {
#pragma clang fp contract(off)
    return make_float4(v.x * rstd * g.x, v.y * rstd * g.y, v.z * rstd * g.z, v.w * rstd * g.w);
}

__global__ __launch_bounds__(256) void k_norm_split(const float *__restrict__ x, const float *__restrict__ g,
                                                    float eps, int K, bf16_t *__restrict__ hi,
                                                    bf16_t *__restrict__ lo) {
    __shared__ float red[4];
    const int t = blockIdx.x;
    const float *row = x + (int64_t)t * K;
    float rstd = 1.f;
    if (g) {
        float ss = 0.f;
        for (int i = threadIdx.x * 4; i < K; i += 1024) {
            const float4 v = *reinterpret_cast<const float4 *>(row + i);
            ss = add_squares(ss, v);
        }
        ss = wave_sum(ss);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
        __syncthreads();
        rstd = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / K + eps);
    }
    for (int i = threadIdx.x * 4; i < K; i += 1024) {
        float4 v = *reinterpret_cast<const float4 *>(row + i);
        if (g) {
            const float4 gv = *reinterpret_cast<const float4 *>(g + i);
            v = scale4(v, rstd, gv);
        }
        uint32_t l0, l1;
        const uint32_t h0 = split2_bf16(v.x, v.y, l0), h1 = split2_bf16(v.z, v.w, l1);
        *reinterpret_cast<uint2 *>(hi + (int64_t)t * K + i) = make_uint2(h0, h1);
        *reinterpret_cast<uint2 *>(lo + (int64_t)t * K + i) = make_uint2(l0, l1);
    }
}

// TT: token tiles of 32 rows per workgroup.  WC: 32-column tiles per wave.  KCH: K chunk staged in LDS.
// A wave multiplies TT x WF accumulator tiles per k-step, WF = WC (x 2 for SwiGLU: gate and up rows).
// The (hi, lo) images of n8 * 8 activations become one fp16 image in place of the high one (hi + lo is exact in
// float32; one rounding to fp16).  *flag is set when a value does not fit into fp16.
__global__ __launch_bounds__(256) void k_split_to_f16(bf16_t *__restrict__ hi, const bf16_t *__restrict__ lo, int64_t n8,
                                                      int *__restrict__ flag) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const u32x4 h = *reinterpret_cast<const u32x4 *>(hi + i * 8), l = *reinterpret_cast<const u32x4 *>(lo + i * 8);
    uint32_t o[4];
    bool big = false;
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const float a = __uint_as_float(h[e] << 16) + __uint_as_float(l[e] << 16);
        const float b = __uint_as_float(h[e] & 0xffff0000u) + __uint_as_float(l[e] & 0xffff0000u);
        big = big || !(fabsf(a) <= F16_LIMIT) || !(fabsf(b) <= F16_LIMIT);
        const _Float16 ha = (_Float16)a, hb = (_Float16)b;
        o[e] = (uint32_t)__builtin_bit_cast(uint16_t, ha) | ((uint32_t)__builtin_bit_cast(uint16_t, hb) << 16);
    }
    *reinterpret_cast<u32x4 *>(hi + i * 8) = (u32x4){o[0], o[1], o[2], o[3]};
    if (big) *flag = 1;
}

// *flag is set when a bf16 matrix holds a value that fp16 cannot (beyond +-65504, or not a number).
__global__ __launch_bounds__(256) void k_weight_range(const bf16_t *__restrict__ w, int64_t n8, int *__restrict__ flag) {
    bool big = false;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(w + i * 8));
#pragma unroll
        for (int e = 0; e < 4; e++)
            big = big || !(fabsf(__uint_as_float(v[e] << 16)) <= F16_LIMIT) || !(fabsf(__uint_as_float(v[e] & 0xffff0000u)) <= F16_LIMIT);
    }
    if (big) *flag = 1;
}

// The same look at a matrix, and its fp16 image written beside it (exact wherever *flag stays clear, up to values
// below 2^-14 in magnitude).
__global__ __launch_bounds__(256) void k_weight_to_f16(const bf16_t *__restrict__ w, int64_t n8, uint16_t *__restrict__ out,
                                                       int *__restrict__ flag) {
    bool big = false;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(w + i * 8));
#pragma unroll
        for (int e = 0; e < 4; e++)
            big = big || !(fabsf(__uint_as_float(v[e] << 16)) <= F16_LIMIT) || !(fabsf(__uint_as_float(v[e] & 0xffff0000u)) <= F16_LIMIT);
        *reinterpret_cast<f16x8 *>(out + i * 8) = bf16x8_to_f16x8(v);
    }
    if (big) *flag = 1;
}

template <int TT, int WC, int KCH, int EPI>
__global__ __launch_bounds__(256) void k_gemm_mfma(const bf16_t *__restrict__ W, const bf16_t *__restrict__ xhi,
                                                   const bf16_t *__restrict__ xlo, int T, int N, int K,
                                                   float *__restrict__ y, int n_ttiles, int ks,
                                                   float *__restrict__ partial, bf16_t *__restrict__ hi_out,
                                                   bf16_t *__restrict__ lo_out) {
    constexpr int WR = (EPI == ld::GEMM_SWIGLU) ? 2 : 1;
    constexpr int WF = WC * WR;                          // W fragments per wave per k-step
    constexpr int TROWS = TT * 32;
    constexpr int NT = 32 * WC * NW;                     // output columns per workgroup
    constexpr int XLD = KCH + XPAD;                      // LDS row stride in elements
    constexpr int XV = TROWS * (KCH / 8) * 2 / 256;      // 16-byte pieces per thread to stage one chunk (hi + lo)
    constexpr int KG = KCH / 64;                         // 64-wide k-groups per chunk
    __shared__ __attribute__((aligned(16))) bf16_t xs[2][TROWS][XLD];

    // XCD-aware decode of the linear block id: blocks b, b+8, b+16, ... run on the same XCD
    const int b = blockIdx.x, xcd = b & 7, s = b >> 3;
    const int kz = s % ks, tt_idx = (s / ks) % n_ttiles, nb = (s / (ks * n_ttiles)) * 8 + xcd;
    const int n_nblocks = (N + NT - 1) / NT;
    if (nb >= n_nblocks) return;
    const int t0 = tt_idx * TROWS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int n0 = nb * NT + wave * (32 * WC);

    // W rows of this lane (clamped in range; out-of-range columns are never stored); fragment f = c * WR + r
    const bf16_t *wrow[WF];
#pragma unroll
    for (int c = 0; c < WC; c++)
#pragma unroll
        for (int r = 0; r < WR; r++) {
            const int n = min(n0 + c * 32 + l32, N - 1);
            wrow[c * WR + r] = W + ((int64_t)r * N + n) * K + half * 32;
        }
    // staging assignment: piece v -> (part, row, col16)
    int st_row[XV], st_c16[XV], st_part[XV];
    const bf16_t *st_src[XV];
#pragma unroll
    for (int v = 0; v < XV; v++) {
        const int idx = threadIdx.x + 256 * v;
        st_part[v] = idx / (TROWS * (KCH / 8));
        const int rem = idx % (TROWS * (KCH / 8));
        st_row[v] = rem / (KCH / 8);
        st_c16[v] = rem % (KCH / 8);
        const int t = min(t0 + st_row[v], T - 1);        // rows past T are staged from row T-1 and never stored
        st_src[v] = (st_part[v] ? xlo : xhi) + (int64_t)t * K + st_c16[v] * 8;
    }

    f32x16 acc[WF][TT];
#pragma unroll
    for (int f = 0; f < WF; f++)
#pragma unroll
        for (int tt = 0; tt < TT; tt++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[f][tt][i] = 0.f;

    u32x4 wA[WF][KG * 4], wB[WF][KG * 4], xr[XV];
    auto load_w = [&](u32x4 (&w)[WF][KG * 4], int kc) {
#pragma unroll
        for (int f = 0; f < WF; f++)
#pragma unroll
            for (int kg = 0; kg < KG; kg++)
#pragma unroll
                for (int j = 0; j < 4; j++)
                    w[f][kg * 4 + j] = *reinterpret_cast<const u32x4 *>(wrow[f] + kc * KCH + kg * 64 + j * 8);
    };
    auto load_x = [&](u32x4 (&xv)[XV], int kc) {
#pragma unroll
        for (int v = 0; v < XV; v++) xv[v] = *reinterpret_cast<const u32x4 *>(st_src[v] + kc * KCH);
    };
    auto compute = [&](u32x4 (&w)[WF][KG * 4]) {
#pragma unroll
        for (int kg = 0; kg < KG; kg++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int k = kg * 64 + half * 32 + j * 8;
                bf16x8 ah[TT], al[TT];
#pragma unroll
                for (int tt = 0; tt < TT; tt++) {
                    ah[tt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&xs[0][tt * 32 + l32][k]));
                    al[tt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&xs[1][tt * 32 + l32][k]));
                }
                // all high parts, then all low parts: consecutive MFMAs never share an accumulator
#pragma unroll
                for (int f = 0; f < WF; f++) {
                    const bf16x8 bw = __builtin_bit_cast(bf16x8, w[f][kg * 4 + j]);
#pragma unroll
                    for (int tt = 0; tt < TT; tt++)
                        acc[f][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[tt], bw, acc[f][tt], 0, 0, 0);
                }
#pragma unroll
                for (int f = 0; f < WF; f++) {
                    const bf16x8 bw = __builtin_bit_cast(bf16x8, w[f][kg * 4 + j]);
#pragma unroll
                    for (int tt = 0; tt < TT; tt++)
                        acc[f][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[tt], bw, acc[f][tt], 0, 0, 0);
                }
            }
    };
    auto stage = [&](const u32x4 (&xv)[XV]) {
#pragma unroll
        for (int v = 0; v < XV; v++)
            *reinterpret_cast<u32x4 *>(&xs[st_part[v]][st_row[v]][st_c16[v] * 8]) = xv[v];
    };

    // this workgroup's K slab: chunks [c_begin, n_chunks) of K / KCH, split evenly over ks workgroups
    const int c_begin = (int)((int64_t)kz * (K / KCH) / ks), n_chunks = (int)((int64_t)(kz + 1) * (K / KCH) / ks);
    load_x(xr, c_begin);
    load_w(wA, c_begin);
    for (int kc = c_begin; kc < n_chunks; kc += 2) {
        lds_barrier();                 // everyone finished reading the previous chunk from LDS
        stage(xr);
        lds_barrier();
        if (kc + 1 < n_chunks) { load_x(xr, kc + 1); load_w(wB, kc + 1); }
        compute(wA);
        if (kc + 1 < n_chunks) {
            lds_barrier();
            stage(xr);
            lds_barrier();
            if (kc + 2 < n_chunks) { load_x(xr, kc + 2); load_w(wA, kc + 2); }
            compute(wB);
        }
    }

    // accumulator element i of lane (l32, half): token t0 + tt*32 + 8*(i/4) + 4*half + i%4, column n0 + 32c + l32
#pragma unroll
    for (int c = 0; c < WC; c++) {
        const int n = n0 + c * 32 + l32;
        if (n >= N) continue;
#pragma unroll
        for (int tt = 0; tt < TT; tt++)
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int t = t0 + tt * 32 + 8 * (i / 4) + 4 * half + (i % 4);
                if (t >= T) continue;
                if (ks > 1) {
                    // split-K: raw partial sums, [kz][t][r * N + n]; a second kernel adds the slabs in fixed order
#pragma unroll
                    for (int r = 0; r < WR; r++)
                        partial[((int64_t)kz * T + t) * (WR * N) + r * N + n] = acc[c * WR + r][tt][i];
                } else {
                    float *dst = y + (int64_t)t * N + n;
                    if constexpr (EPI == ld::GEMM_STORE) *dst = acc[c][tt][i];
                    else if constexpr (EPI == ld::GEMM_ADD) *dst += acc[c][tt][i];
                    else {
                        const float a = swiglu(acc[c * WR][tt][i], acc[c * WR + 1][tt][i]);
                        if (hi_out) store_split(hi_out, lo_out, (int64_t)t * N + n, a);
                        else *dst = a;
                    }
                }
            }
    }
}

// Up to 32 rows (decode batches; up to 48 in two groups of rows): the weight stream is everything, so a workgroup
// takes 128 rows of W and a 512-wide K slab, requests its whole W slab at once (32 independent 16-byte loads per
// lane), stages the matching X slab (hi and lo) in LDS meanwhile, and multiplies as the loads land: one memory
// round trip per workgroup, no barrier inside the product loop.  Every (slab, row) partial sum goes to scratch and
// a reduction kernel adds the slabs in fixed order (for SwiGLU the gate and up rows are plain rows here and are
// paired by the reduce kernel).
//
// W is fetched in the layout the memory system likes, not in the one the matrix cores want: a load instruction
// covers 8 rows x 128 contiguous bytes (8 lanes per row), so every 128-byte line is touched by one instruction
// (with lane = row, the B-operand layout, an instruction touches 32 lines and each line takes part in eight
// instructions: 37.6 against 30.9 us for the loads alone of the 7B gate/up matrix).  Each 64-wide k-group then
// passes through 4 KB of LDS private to the wave (written as fetched, read back with lane = row).
// LDS: X slab [part][row][64 pieces of 16 bytes], piece c of row r in slot c ^ (r & 15) (rows are 1 KB apart, so
// the 16 rows that a fragment read touches at one c land in 16 different bank groups without padding); per wave
// 32 rows x 128 bytes for the W k-group, piece p of row r in slot p ^ ((r >> 1) & 7).  80 KB: two workgroups per CU.
constexpr int SL = 512;   // K slab per workgroup

// FULL: K is a multiple of the slab width, every slab is whole and every load unconditional.
template <bool FULL>
__global__ __launch_bounds__(256, 2) void k_gemm_skinny(const bf16_t *__restrict__ W, const bf16_t *__restrict__ xhi,
                                                        const bf16_t *__restrict__ xlo, int T, int n_rows, int K,
                                                        int ks, float *__restrict__ partial) {
    __shared__ __attribute__((aligned(16))) char xs[2 * 32 * SL * 2];
    __shared__ __attribute__((aligned(16))) char tp[NW][32 * 128];
    const int b = blockIdx.x;
    const int kz = b % ks, nb = b / ks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int r8 = lane >> 3, p8 = lane & 7;
    const int k0 = kz * SL;
    const int slab = FULL ? SL : min(SL, K - k0);          // multiple of 128
    const int n_kg = FULL ? 8 : slab / 64;
    const int n = nb * 128 + wave * 32 + l32;

    // X slab of a group of 32 rows: 64 rows of 1 KB (2 parts x 32), 16 per wave, one load instruction per row; lane
    // l fills slot l of the row, so it fetches piece l ^ (row & 15).  Requested before W and staged while W is in flight.
    u32x4 xv[16];
    auto x_request = [&](int t0) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const int prow = wave * 16 + v, part = prow >> 5, row = prow & 31;
            int c = lane ^ (row & 15);
            if (!FULL && c * 8 >= slab) c = 0;      // slots beyond a short slab are never read
            const int t = min(t0 + row, T - 1);
            xv[v] = *reinterpret_cast<const u32x4 *>((part ? xlo : xhi) + (int64_t)t * K + k0 + c * 8);
        }
    };
    auto x_stage = [&]() {
#pragma unroll
        for (int v = 0; v < 16; v++) *reinterpret_cast<u32x4 *>(xs + (wave * 16 + v) * 1024 + lane * 16) = xv[v];
    };
    x_request(0);
    __builtin_amdgcn_sched_barrier(0);     // X first: its waits then leave the W loads in flight
    u32x4 w[32];
#pragma unroll
    for (int kg = 0; kg < 8; kg++) {
        if (FULL || kg < n_kg) {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int row = min(nb * 128 + wave * 32 + i * 8 + r8, n_rows - 1);
                w[kg * 4 + i] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(W + (int64_t)row * K + k0 + kg * 64 + p8 * 8));
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // LDS addresses: what depends on the lane sits in a few registers, the rest are immediates
    const char *xf[2][4];       // X fragment of piece (k1 * 8 + half * 4 + j) of row l32; + (kg >> 1) * 256, + 32 KB for the low part
#pragma unroll
    for (int k1 = 0; k1 < 2; k1++)
#pragma unroll
        for (int j = 0; j < 4; j++) xf[k1][j] = xs + (l32 * 64 + ((k1 * 8 + half * 4 + j) ^ (l32 & 15))) * 16;
    char *tw = tp[wave];
    char *tw_st[2];             // where this lane's piece of row i * 8 + r8 goes: + (i >> 1) * 2048 for the row pair
#pragma unroll
    for (int i1 = 0; i1 < 2; i1++) tw_st[i1] = tw + (i1 * 8 + r8) * 128 + ((p8 ^ (((i1 * 8 + r8) >> 1) & 7)) * 16);
    const char *tw_ld[4];
#pragma unroll
    for (int j = 0; j < 4; j++) tw_ld[j] = tw + l32 * 128 + (((half * 4 + j) ^ ((l32 >> 1) & 7)) * 16);

    // Rows are taken 32 at a time against the same weight registers (one group for a decode batch, two for
    // up to 64 rows): the X slab of a group is staged, multiplied and its partial sums written before the next
    // group's slab replaces it in LDS.  The first group is spelled out ahead of the loop: there the W loads are
    // still in flight and each k-group waits for its own four only.
    auto group = [&](int t0) {
        f32x16 acc_h, acc_l;
#pragma unroll
        for (int i = 0; i < 16; i++) acc_h[i] = acc_l[i] = 0.f;
#pragma unroll
        for (int kg = 0; kg < 8; kg++) {
            if (FULL || kg < n_kg) {
                // the k-group through the wave's own LDS rows (a wave's LDS operations execute in order)
#pragma unroll
                for (int i = 0; i < 4; i++) *reinterpret_cast<u32x4 *>(tw_st[i & 1] + (i >> 1) * 2048) = w[kg * 4 + i];
                __builtin_amdgcn_wave_barrier();
                u32x4 bw[4];
#pragma unroll
                for (int j = 0; j < 4; j++) bw[j] = *reinterpret_cast<const u32x4 *>(tw_ld[j]);
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int j = 0; j < 4; j++) {      // k = kg * 64 + half * 32 + j * 8
                    const char *xa = xf[kg & 1][j] + (kg >> 1) * 256;
                    const bf16x8 ah = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(xa));
                    const bf16x8 al = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(xa + 32 * 1024));
                    acc_h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, __builtin_bit_cast(bf16x8, bw[j]), acc_h, 0, 0, 0);
                    acc_l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, __builtin_bit_cast(bf16x8, bw[j]), acc_l, 0, 0, 0);
                }
            }
        }
        if (n < n_rows) {
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int t = t0 + 8 * (i / 4) + 4 * half + (i % 4);
                if (t < T) partial[((int64_t)kz * T + t) * n_rows + n] = acc_h[i] + acc_l[i];
            }
        }
    };
    x_stage();
    lds_barrier();
    group(0);
    for (int t0 = 32; t0 < T; t0 += 32) {
        lds_barrier();      // every wave has finished reading the previous group's slab
        x_request(t0);
        x_stage();
        lds_barrier();
        group(t0);
    }
}

// More than 64 rows (prefill chunks, mixed steps): MFMA-bound.  64*WM tokens x BN weight rows per
// workgroup, 2*WM waves as WM (tokens) x 2 (columns), both operands through LDS.  What limits this kernel is
// the operand traffic from L2 per flop (the split doubles the X side), so the tile is as large as the
// accumulators allow: 256 x 256 with eight waves from 512 rows on, 128 x 256 (or x 128) below.  K advances
// in chunks of 32; the global loads of a chunk are issued D chunks before their data is written to LDS, in
// a ring of register sets; LDS is double buffered, one barrier per chunk.  LDS holds 16-byte pieces
// segment-major ([k-segment][row], segment stride padded by 64 bytes): the operand reads of 16 consecutive
// lanes are 256 contiguous bytes and the staging writes of a 16-lane group (4 rows x 4 segments) cover all
// 64 banks once.
template <int WM, int BN, int D, int EPI>
__global__ __launch_bounds__(128 * WM) void k_gemm_big(const bf16_t *__restrict__ W, const bf16_t *__restrict__ xhi,
                                                       const bf16_t *__restrict__ xlo, int T, int N, int K,
                                                       float *__restrict__ y, int n_ttiles, int ks,
                                                       float *__restrict__ partial, int col0, int col1,
                                                       bf16_t *__restrict__ hi_out, bf16_t *__restrict__ lo_out) {
    constexpr bool SWI = (EPI == ld::GEMM_SWIGLU);
    constexpr int NT = 128 * WM;                  // threads
    constexpr int BM = 64 * WM, BK = 32, SEGS = BK / 8;
    constexpr int WCT = BN / 2 / 32;              // 32-column accumulator tiles per wave
    constexpr int NOUT = SWI ? BN / 2 : BN;       // output columns per workgroup
    constexpr int XSEG = BM * 16 + 64, WSEG = BN * 16 + 64;   // bytes per k-segment of a stage
    constexpr int NVX = 2 * BM * SEGS / NT, NVW = BN * SEGS / NT;   // 16-byte pieces per thread per chunk
    __shared__ __attribute__((aligned(16))) char xs[2][2][SEGS][XSEG];
    __shared__ __attribute__((aligned(16))) char ws[2][SEGS][WSEG];

    const int b = blockIdx.x, xcd = b & 7, s = b >> 3;
    const int kz = s % ks, tt_idx = (s / ks) % n_ttiles, nb = (s / (ks * n_ttiles)) * 8 + xcd;
    const int n_nblocks = (col1 - col0 + NOUT - 1) / NOUT;   // this launch covers output columns [col0, col1)
    if (nb >= n_nblocks) return;
    const int t0 = tt_idx * BM, n0 = col0 + nb * NOUT;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    // global source of every piece this thread stages (rows clamped; clamped rows are never stored)
    const bf16_t *xsrc[NVX], *wsrc[NVW];
    int xdst[NVX], wdst[NVW];
#pragma unroll
    for (int v = 0; v < NVX; v++) {
        const int p = threadIdx.x + NT * v, part = p / (BM * SEGS), r = (p % (BM * SEGS)) >> 2, seg = p & 3;
        xsrc[v] = (part ? xlo : xhi) + (int64_t)min(t0 + r, T - 1) * K + seg * 8;
        xdst[v] = (part * SEGS + seg) * XSEG + r * 16;
    }
#pragma unroll
    for (int v = 0; v < NVW; v++) {
        const int p = threadIdx.x + NT * v, wr = p >> 2, seg = p & 3;
        int grow;
        if (SWI) {   // local rows of a wave column: gate tiles, then the up tiles of the same columns
            const int wcol = wr / (BN / 2), within = wr % (BN / 2);
            const int col = n0 + wcol * (BN / 4) + (within % (BN / 4));
            grow = min(col, N - 1) + (within >= BN / 4 ? N : 0);
        } else {
            grow = min(n0 + wr, N - 1);
        }
        wsrc[v] = W + (int64_t)grow * K + seg * 8;
        wdst[v] = seg * WSEG + wr * 16;
    }

    f32x16 acc[2][WCT];
#pragma unroll
    for (int tt = 0; tt < 2; tt++)
#pragma unroll
        for (int wc = 0; wc < WCT; wc++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[tt][wc][i] = 0.f;

    u32x4 ring[D][NVX + NVW];
    auto issue = [&](u32x4 (&r)[NVX + NVW], int kc) {
#pragma unroll
        for (int v = 0; v < NVX; v++) r[v] = *reinterpret_cast<const u32x4 *>(xsrc[v] + kc * BK);
#pragma unroll
        for (int v = 0; v < NVW; v++) r[NVX + v] = *reinterpret_cast<const u32x4 *>(wsrc[v] + kc * BK);
    };
    auto stage = [&](const u32x4 (&r)[NVX + NVW], int st) {
#pragma unroll
        for (int v = 0; v < NVX; v++) *reinterpret_cast<u32x4 *>(&xs[st][0][0][0] + xdst[v]) = r[v];
#pragma unroll
        for (int v = 0; v < NVW; v++) *reinterpret_cast<u32x4 *>(&ws[st][0][0] + wdst[v]) = r[NVX + v];
    };
    auto compute = [&](int st) {
#pragma unroll
        for (int kstep = 0; kstep < BK / 16; kstep++) {
            const int seg = kstep * 2 + half;
            bf16x8 a[2][2], bw[WCT];
#pragma unroll
            for (int part = 0; part < 2; part++)
#pragma unroll
                for (int tt = 0; tt < 2; tt++)
                    a[part][tt] = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const u32x4 *>(&xs[st][part][seg][(wm * 64 + tt * 32 + l32) * 16]));
#pragma unroll
            for (int wc = 0; wc < WCT; wc++)
                bw[wc] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const u32x4 *>(&ws[st][seg][(wn * (BN / 2) + wc * 32 + l32) * 16]));
#pragma unroll
            for (int part = 0; part < 2; part++)
#pragma unroll
                for (int tt = 0; tt < 2; tt++)
#pragma unroll
                    for (int wc = 0; wc < WCT; wc++)
                        acc[tt][wc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[part][tt], bw[wc], acc[tt][wc], 0, 0, 0);
        }
    };

    const int c_begin = (int)((int64_t)kz * (K / BK) / ks), c_end = (int)((int64_t)(kz + 1) * (K / BK) / ks);
#pragma unroll
    for (int d = 0; d < D; d++)
        if (c_begin + d < c_end) issue(ring[d], c_begin + d);
    for (int c = c_begin; c < c_end; c += D) {
#pragma unroll
        for (int d = 0; d < D; d++) {
            const int cc = c + d;
            if (cc < c_end) {
                const int st = (D % 2 == 0) ? (d & 1) : ((cc - c_begin) & 1);   // LDS stage alternates per chunk
                stage(ring[d], st);
                lds_barrier();
                if (cc + D < c_end) issue(ring[d], cc + D);
                compute(st);
            }
        }
    }

    // accumulator element i of lane (l32, half): token t0 + wm*64 + tt*32 + 8*(i/4) + 4*half + i%4
    constexpr int WOUT = SWI ? WCT / 2 : WCT;     // output column tiles per wave
    const int ncols = SWI ? 2 * N : N;            // row length of the partial-sum buffer
#pragma unroll
    for (int wc = 0; wc < WOUT; wc++) {
        const int n = n0 + wn * (NOUT / 2) + wc * 32 + l32;
        if (n >= col1) continue;
#pragma unroll
        for (int tt = 0; tt < 2; tt++)
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int t = t0 + wm * 64 + tt * 32 + 8 * (i / 4) + 4 * half + (i % 4);
                if (t >= T) continue;
                if (ks > 1) {
                    float *dst = partial + ((int64_t)kz * T + t) * ncols + n;
                    dst[0] = acc[tt][wc][i];
                    if constexpr (SWI) dst[N] = acc[tt][wc + WCT / 2][i];
                } else {
                    float *dst = y + (int64_t)t * N + n;
                    if constexpr (EPI == ld::GEMM_STORE) *dst = acc[tt][wc][i];
                    else if constexpr (EPI == ld::GEMM_ADD) *dst += acc[tt][wc][i];
                    else {
                        const float a = swiglu(acc[tt][wc][i], acc[tt][wc + WCT / 2][i]);
                        if (hi_out) store_split(hi_out, lo_out, (int64_t)t * N + n, a);
                        else *dst = a;
                    }
                }
            }
    }
}

// The same tile scheme with the operands copied from global memory straight into LDS
// (global_load_lds_dwordx4: lane l of a wave writes its 16 bytes at the wave's LDS base + 16 l), so that no
// operand byte passes through registers on its way to LDS and the registers of the prefetch ring are free.
// A stage holds the tile's rows row-major, 64 bytes (one K chunk of 32) per row: X hi rows, X lo rows, W
// rows.  One copy instruction of a wave covers 16 rows x 4 sixteen-byte pieces (1 KB of LDS, 64 contiguous
// bytes of 16 rows in memory).  Piece `seg` of row r sits in slot seg ^ ((r >> 2) & 3) of the row, which
// makes the operand reads of 16 consecutive rows hit 16 different bank groups; the swizzle costs nothing
// because a lane may fetch any global piece into its fixed slot.  S stages; the copies of chunk c + S - 1
// are issued right after the barrier of chunk c, when every wave has finished reading the stage they
// overwrite; before the barrier of chunk c a wave waits until its own copies of chunk c have landed
// (s_waitcnt vmcnt with the number of younger copies still allowed in flight).
// WM x WN waves; a wave owns 64 rows x BN / WN columns of the tile.  Both shapes in use run eight waves, two
// per SIMD, so that one wave's operand reads and barrier waits sit under the other's MFMAs: 256 x 256 as
// 4 x 2 waves of 64 x 128, 128 x 256 as 2 x 4 waves of 64 x 64 (measured against four waves of 64 x 128 on
// the same tile: layer GEMMs at 128 - 512 rows 4 - 7 % faster, the full-grid rate 410 -> 440 TFLOP/s; sixteen
// waves of 64 x 64 on the 256 x 256 tile fit in 109 registers and change nothing).
//
// F16 != 0 (rows that nobody reads at full precision, see launch_gemm): one operand image instead of two, the
// activations rounded to fp16 (11 significant bits; xhi then points at a [T, K] fp16 matrix): half the matrix-core
// work and two thirds of the operand traffic of the two-term form.  F16 == 1: W is the bf16 matrix and every wave
// turns the fragments it reads from LDS into fp16 on their way to the matrix cores (exact for 2^-14 <= |w| < 65520,
// which the launcher has checked on the whole matrix).  F16 == 2: W is the matrix's fp16 image (k_weight_to_f16),
// used as it is; same values, same sums.
template <int WM, int BN, int S, int EPI, int WN, int F16>
__global__ __launch_bounds__(64 * WM * WN) void k_gemm_dma(const bf16_t *__restrict__ W, const bf16_t *__restrict__ xhi,
                                                       const bf16_t *__restrict__ xlo, int T, int N, int K,
                                                       float *__restrict__ y, int n_ttiles, int ks,
                                                       float *__restrict__ partial, int col0, int col1,
                                                       bf16_t *__restrict__ hi_out, bf16_t *__restrict__ lo_out) {
    constexpr bool SWI = (EPI == ld::GEMM_SWIGLU);
    constexpr int NW = WM * WN;                   // waves: WM along the rows (64 each) x WN along the columns
    constexpr int BM = 64 * WM, BK = 32;
    constexpr int WCOLS = BN / WN;                // W rows of the tile that one wave column multiplies
    constexpr int WCT = WCOLS / 32;               // 32-column accumulator tiles per wave
    constexpr int NOUT = SWI ? BN / 2 : BN;       // output columns per workgroup
    constexpr int TERMS = F16 ? 1 : 2;
    constexpr int XR = TERMS * BM;                // X rows of a stage: hi and lo images (one fp16 image)
    constexpr int ROWS = XR + BN;                 // rows of a stage: X hi, X lo, W
    constexpr int STAGE = ROWS * 64;              // bytes
    constexpr int P = ROWS / 16 / NW;             // copy instructions per wave per chunk
    static_assert(ROWS % (16 * NW) == 0, "rows must split evenly over the waves");
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int b = blockIdx.x, xcd = b & 7, s = b >> 3;
    const int kz = s % ks, tt_idx = (s / ks) % n_ttiles, nb = (s / (ks * n_ttiles)) * 8 + xcd;
    const int n_nblocks = (col1 - col0 + NOUT - 1) / NOUT;   // this launch covers output columns [col0, col1)
    if (nb >= n_nblocks) return;
    const int t0 = tt_idx * BM, n0 = col0 + nb * NOUT;
    // the wave index as a scalar: what depends on it alone (which rows a copy covers, its LDS address) stays in SGPRs
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;

    // Global source of the piece this lane fetches in copy j of a chunk: a base pointer that is the same for the
    // whole wave (the 16 rows of a copy lie in one of the three matrices) plus a 32-bit byte offset per lane, the
    // form in which the copy instruction takes a scalar base and advancing along K is scalar arithmetic (the
    // launcher keeps matrices of 4 GB or more away).  Rows are clamped; clamped rows are never stored.
    const char *cbase[P];
    uint32_t coff[P];
#pragma unroll
    for (int j = 0; j < P; j++) {
        const int vr0 = (wave * P + j) * 16;                       // first row of the copy (scalar)
        const int vr = vr0 + (lane >> 2);                          // row of the stage
        const int slot = lane & 3;
        const int seg = slot ^ ((vr >> 2) & 3);
        if (vr0 < XR) {
            const int r = vr % BM;
            cbase[j] = reinterpret_cast<const char *>(vr0 < BM ? xhi : xlo);
            coff[j] = ((uint32_t)min(t0 + r, T - 1) * (uint32_t)K + seg * 8) * 2u;
        } else {
            const int wr = vr - XR;
            int grow;
            if (SWI) {   // local rows of a wave column: gate tiles, then the up tiles of the same columns
                const int wcol = wr / WCOLS, within = wr % WCOLS;
                const int col = n0 + wcol * (WCOLS / 2) + (within % (WCOLS / 2));
                grow = min(col, N - 1) + (within >= WCOLS / 2 ? N : 0);
            } else {
                grow = min(n0 + wr, N - 1);
            }
            cbase[j] = reinterpret_cast<const char *>(W);
            coff[j] = ((uint32_t)grow * (uint32_t)K + seg * 8) * 2u;
        }
    }
    auto copy_chunk = [&](int kc, int st) {
#pragma unroll
        for (int j = 0; j < P; j++)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(cbase[j] + (size_t)kc * (BK * 2) + (size_t)coff[j]),
                (__attribute__((address_space(3))) void *)(lds + st * STAGE + (wave * P + j) * 1024), 16, 0, 0);
    };

    f32x16 acc[2][WCT];
#pragma unroll
    for (int tt = 0; tt < 2; tt++)
#pragma unroll
        for (int wc = 0; wc < WCT; wc++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[tt][wc][i] = 0.f;

    struct Frags { u32x4 a[TERMS][2], bw[WCT]; };
    auto load_frags = [&](Frags &f, int st, int kstep) {
        const char *base = lds + st * STAGE;
        const int seg = kstep * 2 + half;
#pragma unroll
        for (int part = 0; part < TERMS; part++)
#pragma unroll
            for (int tt = 0; tt < 2; tt++) {
                const int r = wm * 64 + tt * 32 + l32;       // BM is a multiple of 16: (r >> 2) & 3 is the stage row's
                f.a[part][tt] = *reinterpret_cast<const u32x4 *>(base + (part * BM + r) * 64 + ((seg ^ ((r >> 2) & 3)) * 16));
            }
#pragma unroll
        for (int wc = 0; wc < WCT; wc++) {
            const int r = wn * WCOLS + wc * 32 + l32;
            f.bw[wc] = *reinterpret_cast<const u32x4 *>(base + (XR + r) * 64 + ((seg ^ ((r >> 2) & 3)) * 16));
        }
    };
    auto mfmas = [&](const Frags &f) {
        if constexpr (F16) {
            f16x8 wv[WCT];
#pragma unroll
            for (int wc = 0; wc < WCT; wc++)
                wv[wc] = F16 == 2 ? __builtin_bit_cast(f16x8, f.bw[wc]) : bf16x8_to_f16x8(f.bw[wc]);
#pragma unroll
            for (int tt = 0; tt < 2; tt++)
#pragma unroll
                for (int wc = 0; wc < WCT; wc++)
                    acc[tt][wc] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, f.a[0][tt]), wv[wc],
                                                                        acc[tt][wc], 0, 0, 0);
        } else {
#pragma unroll
            for (int part = 0; part < TERMS; part++)
#pragma unroll
                for (int tt = 0; tt < 2; tt++)
#pragma unroll
                    for (int wc = 0; wc < WCT; wc++)
                        acc[tt][wc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[part][tt]),
                                                                             __builtin_bit_cast(bf16x8, f.bw[wc]),
                                                                             acc[tt][wc], 0, 0, 0);
        }
    };
    // Wait until this wave's copies of the oldest outstanding chunk have landed; `younger` later chunks
    // (P copies each) may stay in flight.  The count is an immediate, so only the steady-state values are
    // spelled out; near the end of a slab waiting for everything is exact enough.
    auto wait_copies = [&](int younger) {
        if (younger >= S - 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * P) : "memory");
        else if (S >= 4 && younger == S - 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S >= 4 ? S - 3 : 0) * P) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };

    // Software pipeline.  The operand registers of a K step are read from LDS while the MFMAs of the step
    // before run; the barrier that makes chunk c + 1 visible sits in the middle of chunk c's arithmetic.
    // After that barrier every wave has finished reading chunk c - 1, whose stage the copies of chunk
    // c + S - 1 then overwrite (S stages hold chunks c - 1 .. c + S - 2 until then).
    const int c_begin = (int)((int64_t)kz * (K / BK) / ks), c_end = (int)((int64_t)(kz + 1) * (K / BK) / ks);
    const int n_chunks = c_end - c_begin;
#pragma unroll
    for (int d = 0; d < S - 1; d++)
        if (d < n_chunks) copy_chunk(c_begin + d, d);
    wait_copies(min(n_chunks, S - 1) - 1);
    asm volatile("s_barrier" ::: "memory");
    Frags f0, f1;
    load_frags(f0, 0, 0);
    int st = 0;
    // issue order inside a half step: one operand read after every second MFMA, so that the reads are in
    // flight under the arithmetic of the half step before the one that needs them
    auto interleave = [&]() {
#pragma unroll
        for (int k = 0; k < 2 * TERMS + WCT; k++) {
            __builtin_amdgcn_sched_group_barrier(0x008, TERMS, 0);   // MFMAs (2 * TERMS * WCT per half step)
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);       // 1 LDS read (2 * TERMS + WCT per half step)
        }
    };
    // the half step that also requests a chunk: its P copies one by one between the MFMAs rather than in a row
    // behind the barrier (1 - 3 % on the layer shapes)
    auto interleave_copies = [&]() {
        constexpr int NM = 2 * TERMS * WCT, NR = 2 * TERMS + WCT, CSTEP = NM / P > 0 ? NM / P : 1;
#pragma unroll
        for (int k = 0; k < NM; k++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (k % TERMS == TERMS - 1 && k / TERMS < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (k % CSTEP == CSTEP - 1 && k / CSTEP < P) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
    };
    // every chunk but the last (the next one always exists): first the steady state, in which a chunk S - 1 ahead
    // is still to be requested (no condition around the copies, so that their issue can sit between the MFMAs),
    // then the last S - 2 of them
    int i = 0;
    for (; i + S - 1 < n_chunks; i++) {
        load_frags(f1, st, 1);
        mfmas(f0);
        interleave();
        const int st1 = st + 1 == S ? 0 : st + 1;
        wait_copies(S - 3);                        // outstanding: chunks i+1 .. i+S-2
        asm volatile("s_barrier" ::: "memory");
        copy_chunk(c_begin + i + S - 1, st == 0 ? S - 1 : st - 1);
        load_frags(f0, st1, 0);
        mfmas(f1);
        interleave_copies();
        st = st1;
    }
    for (; i + 1 < n_chunks; i++) {
        load_frags(f1, st, 1);
        mfmas(f0);
        interleave();
        const int st1 = st + 1 == S ? 0 : st + 1;
        wait_copies(n_chunks - 1 - (i + 1));       // outstanding: chunks i+1 .. n-1
        asm volatile("s_barrier" ::: "memory");
        load_frags(f0, st1, 0);
        mfmas(f1);
        interleave();
        st = st1;
    }
    load_frags(f1, st, 1);
    mfmas(f0);
    mfmas(f1);

    // accumulator element i of lane (l32, half): token t0 + wm*64 + tt*32 + 8*(i/4) + 4*half + i%4
    constexpr int WOUT = SWI ? WCT / 2 : WCT;     // output column tiles per wave
    const int ncols = SWI ? 2 * N : N;            // row length of the partial-sum buffer
#pragma unroll
    for (int wc = 0; wc < WOUT; wc++) {
        const int n = n0 + wn * (NOUT / WN) + wc * 32 + l32;
        if (n >= col1) continue;
#pragma unroll
        for (int tt = 0; tt < 2; tt++)
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int t = t0 + wm * 64 + tt * 32 + 8 * (i / 4) + 4 * half + (i % 4);
                if (t >= T) continue;
                if (ks > 1) {
                    float *dst = partial + ((int64_t)kz * T + t) * ncols + n;
                    dst[0] = acc[tt][wc][i];
                    if constexpr (SWI) dst[N] = acc[tt][wc + WCT / 2][i];
                } else {
                    float *dst = y + (int64_t)t * N + n;
                    if constexpr (EPI == ld::GEMM_STORE) *dst = acc[tt][wc][i];
                    else if constexpr (EPI == ld::GEMM_ADD) *dst += acc[tt][wc][i];
                    else {
                        const float a = swiglu(acc[tt][wc][i], acc[tt][wc + WCT / 2][i]);
                        if (hi_out) store_split(hi_out, lo_out, (int64_t)t * N + n, a);
                        else *dst = a;
                    }
                }
            }
    }
}

// Adds the ks K-slab partial sums in slab order and applies the epilogue.  One thread per output.
template <int EPI>
__global__ __launch_bounds__(256) void k_splitk_reduce(const float *__restrict__ partial, int T, int N, int ks,
                                                       float *__restrict__ y, int col0, int col1,
                                                       bf16_t *__restrict__ hi_out, bf16_t *__restrict__ lo_out) {
    constexpr int WR = (EPI == ld::GEMM_SWIGLU) ? 2 : 1;
    const int nc = col1 - col0;                    // output columns [col0, col1) of N
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)T * nc) return;
    const int t = (int)(idx / nc), n = col0 + (int)(idx % nc);
    const float *p0 = partial + (int64_t)t * (WR * N) + n;
    const float a = slab_sum(p0, (int64_t)T * (WR * N), ks, 0.f);
    const float b = WR == 2 ? slab_sum(p0 + N, (int64_t)T * (WR * N), ks, 0.f) : 0.f;
    float *dst = y + (int64_t)t * N + n;
    if constexpr (EPI == ld::GEMM_STORE) *dst = a;
    else if constexpr (EPI == ld::GEMM_ADD) *dst += a;
    else {
        const float v = swiglu(a, b);
        if (hi_out) store_split(hi_out, lo_out, (int64_t)t * N + n, v);
        else *dst = v;
    }
}

// Residual rows that feed the next normalised GEMM: finishes y (adds the ks K-slab partial sums of the
// output columns [col0, col1) in slab order, as k_splitk_reduce<GEMM_ADD> does; the other columns were
// already added by the product kernel's epilogue) and writes the next operand split(y * rsqrt(mean y^2 + eps) * g)
// in the same pass over the row, with k_norm_split's arithmetic in k_norm_split's order: the results are those
// of the two separate kernels, bit for bit.  One workgroup per row; N a multiple of 4.
__global__ __launch_bounds__(256) void k_reduce_add_norm_split(const float *__restrict__ partial, int T, int N, int ks,
                                                               int col0, int col1, float *__restrict__ y,
                                                               const float *__restrict__ g, float eps,
                                                               bf16_t *__restrict__ hi, bf16_t *__restrict__ lo) {
    __shared__ float red[4];
    const int t = blockIdx.x;
    float *row = y + (int64_t)t * N;
    const float *prow = partial + (int64_t)t * N;
    const int64_t slab = (int64_t)T * N;
    float ss = 0.f;
    for (int i = threadIdx.x * 4; i < N; i += 1024) {
        float4 v = *reinterpret_cast<const float4 *>(row + i);
        if (i >= col0 && i + 3 < col1) {      // all four columns still miss their slab sums
            const float4 a = slab_sum(reinterpret_cast<const float4 *>(prow + i), slab / 4, ks, make_float4(0.f, 0.f, 0.f, 0.f));
            v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
            *reinterpret_cast<float4 *>(row + i) = v;
        } else if (i + 3 >= col0 && i < col1) {      // some of them do
            if (i >= col0 && i < col1) v.x += slab_sum(prow + i, slab, ks, 0.f);
            if (i + 1 >= col0 && i + 1 < col1) v.y += slab_sum(prow + i + 1, slab, ks, 0.f);
            if (i + 2 >= col0 && i + 2 < col1) v.z += slab_sum(prow + i + 2, slab, ks, 0.f);
            if (i + 3 >= col0 && i + 3 < col1) v.w += slab_sum(prow + i + 3, slab, ks, 0.f);
            *reinterpret_cast<float4 *>(row + i) = v;
        }
        ss = add_squares(ss, v);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float rstd = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / N + eps);
    for (int i = threadIdx.x * 4; i < N; i += 1024) {
        float4 v = *reinterpret_cast<const float4 *>(row + i);     // this thread's own stores of the first pass
        const float4 gv = *reinterpret_cast<const float4 *>(g + i);
        v = scale4(v, rstd, gv);
        uint32_t l0, l1;
        const uint32_t h0 = split2_bf16(v.x, v.y, l0), h1 = split2_bf16(v.z, v.w, l1);
        *reinterpret_cast<uint2 *>(hi + (int64_t)t * N + i) = make_uint2(h0, h1);
        *reinterpret_cast<uint2 *>(lo + (int64_t)t * N + i) = make_uint2(l0, l1);
    }
}

// Rows of the q-k-v projection: finishes them (split-K slab sums of the columns [col0, col1) in slab order; the
// other columns are already in y) and does what the rotate-and-append pass does, one wave per (head, row): q heads
// rotated into y, rotated k heads and v heads into the paged pool.  Row t of this launch is row row0 + t of the pass.
__global__ __launch_bounds__(64) void k_reduce_rope_kv(const float *__restrict__ partial, int T, int N, int ks, int col0,
                                                       int col1, float *__restrict__ y, ld::RopeKvArgs rk, int row0) {
    const int t = blockIdx.y, hh = blockIdx.x, i = threadIdx.x, half = rk.hd / 2, hd = rk.hd;
    if (i >= half) return;
    const float *prow = partial + (int64_t)t * N;
    float *row = y + (int64_t)t * N;
    const int64_t slab = (int64_t)T * N;
    auto val = [&](int col) { return col >= col0 && col < col1 ? slab_sum(prow + col, slab, ks, 0.f) : row[col]; };
    const float2 c = rk.cos_sin[(int64_t)(row0 + t) * half + i];
    if (hh < rk.H) {
        const float2 r = rope_rotate(val(hh * hd + i), val(hh * hd + i + half), c);
        row[hh * hd + i] = r.x;
        row[hh * hd + i + half] = r.y;
        return;
    }
    const int j = hh - rk.H, kc = (rk.H + j) * hd, vc = (rk.H + rk.Hkv + j) * hd;
    const float2 r = rope_rotate(val(kc + i), val(kc + i + half), c);
    const float va = val(vc + i), vb = val(vc + i + half);
    const int p = rk.pos[row0 + t];
    const int64_t phys = rk.table[(int64_t)rk.seq_slot[row0 + t] * rk.table_stride + (p >> 4)];
    bf16_t *blk = rk.pool + phys * kv_block_elems(rk.Hkv, hd);
    const int slot = p & 15;
    blk[kv_k_offset(hd, j, slot, i)] = f32_to_bf16(r.x);
    blk[kv_k_offset(hd, j, slot, i + half)] = f32_to_bf16(r.y);
    blk[kv_v_offset(rk.Hkv, hd, j, slot, i)] = f32_to_bf16(va);
    blk[kv_v_offset(rk.Hkv, hd, j, slot, i + half)] = f32_to_bf16(vb);
}

// Kernel by row count: up to 48 rows -> k_gemm_skinny; 49..64 rows -> k_gemm_mfma with 64 x 128 tiles and
// 128-wide K chunks; more -> k_gemm_big.
struct Shape { int tt, wc, kch; };

int env_int(const char *name, int dflt) {
    const char *v = getenv(name);
    return v ? atoi(v) : dflt;
}
// Tile, workgroup count and split-K factor of the big-tile kernel for a row count: the candidate with the
// smallest estimated time.  A candidate runs ceil(workgroups / 256) rounds of one workgroup per CU (two for
// the 128 x 128 tile, at half the rate each); the per-CU rates are the measured full-grid rates of the three
// tiles; split-K adds the write and the ordered re-read of its partial sums.
struct BigPlan { int wm, bn, n_ttiles, n_nblocks, ks; double est_us; int nb_a, ks_b; };   // nb_a > 0: two phases
// f16: the single-term fp16 form.  Its three constants (0.69 of the two-term time per workgroup, split-K partial
// sums at a third of the two-term form's cost per byte, the last-round factor below) are fitted to the measured
// times of the 7B, grouped-KV and 13B layer shapes at 1056, 2048 and 2111 rows.
BigPlan plan_big(int T, int N, int K, int epi, bool f16 = false) {
    const bool swi = epi == ld::GEMM_SWIGLU;
    struct Tile { int wm, bn; double tflops; };           // nominal (unsplit) TFLOP/s of a full grid
    static const Tile tiles[3] = {{4, 256, 520.0}, {2, 256, 440.0}, {2, 128, 300.0}};
    BigPlan best{};
    double best_t = 1e30;
    const char *forced = getenv("LD_GEMM_BIG");            // tuning knob: "wm,bn,ks"
    int f_wm = 0, f_bn = 0, f_ks = 0;
    if (forced && sscanf(forced, "%d,%d,%d", &f_wm, &f_bn, &f_ks) != 3) f_wm = 0;
    for (const Tile &tl : tiles) {
        if (f_wm && (tl.wm != f_wm || tl.bn != f_bn)) continue;
        if (f16 && tl.bn != 256) continue;      // the fp16 form exists for the 256-wide weight tiles only
        const int bm = 64 * tl.wm, nout = swi ? tl.bn / 2 : tl.bn;
        const int n_tt = (T + bm - 1) / bm, n_nb = (N + nout - 1) / nout;
        const int max_ks = std::max(1, std::min(8, K / 32 / 8));   // at least eight chunks per slab
        for (int ks = 1; ks <= max_ks; ks++) {
            if (f_wm && ks != std::min(f_ks, max_ks)) continue;
            const int64_t wgs = (int64_t)n_tt * n_nb * ks;
            const int64_t rounds = (wgs + 255) / 256;
            const double wg_us = (f16 ? 0.69 : 1.0) * 2.0 * bm * tl.bn * (double)(K / ks) / (tl.tflops * 1e6 / 256.0);
            double t = rounds * wg_us;
            // fp16 form: a last round that leaves CUs idle runs its workgroups faster than a full one (measured on
            // the 13B down projection: 180 workgroups in 0.74 of a full round's time)
            if (f16 && wgs % 256) t = (double)(wgs / 256) * wg_us + std::max((double)(wgs % 256) / 256.0, 0.74) * wg_us;
            if (ks > 1) t += 3.0 + (double)T * N * (swi ? 2 : 1) * 4.0 * (2.0 * ks + 1.0) / (f16 ? 9.0e6 : 3.0e6);
            if (t < best_t) { best_t = t; best = {tl.wm, tl.bn, n_tt, n_nb, ks, t, 0, 0}; }
        }
        // Two phases: the column blocks that fill a whole round run unsplit; the remaining blocks, which would
        // leave most CUs idle for a second round, run with a split K (their partial sums only).  Only between one
        // and two rounds of the 256 x 256 tile: with more rounds the workgroups stagger and the last round
        // costs less than the model's whole round (measured: no gain, or a loss with the smaller tiles).
        static const int two_phase = env_int("LD_GEMM_TWO_PHASE", 1);   // tuning knob
        const int64_t n_all = (int64_t)n_tt * n_nb;
        if (two_phase && !f_wm && tl.wm == 4 && n_all > 256 && n_all < 512) {
            const int nb_a = (int)(n_all / 256 * 256 / n_tt), nb_b = n_nb - nb_a;
            const double wg_us = (f16 ? 0.69 : 1.0) * 2.0 * bm * tl.bn * (double)K / (tl.tflops * 1e6 / 256.0);
            const double t_a = (double)(((int64_t)nb_a * n_tt + 255) / 256) * wg_us;
            for (int ks = 2; ks <= max_ks && nb_a > 0 && nb_b > 0; ks++) {
                const int64_t rounds_b = ((int64_t)nb_b * n_tt * ks + 255) / 256;
                const double cols_b = (double)std::min(N - nb_a * nout, nb_b * nout);
                const double t = t_a + rounds_b * wg_us / ks + 6.0 + (double)T * cols_b * (swi ? 2 : 1) * 4.0 * (2.0 * ks + 1.0) / 3.0e6;
                if (t < best_t) { best_t = t; best = {tl.wm, tl.bn, n_tt, n_nb, 1, t, nb_a, ks}; }
            }
        }
    }
    return best;
}
Shape pick_shape(int T, int epi) {
    (void)T; (void)epi;
    return {2, 1, 128};   // up to 64 rows: 64 x 128 tiles, 128-wide K chunks
}

// Most rows the skinny kernel takes (measured on the 7B and 13B layer shapes: two groups of rows beat the
// 64-row kernel up to 48 rows by 7 %, are level with it at 64 rows on the former and 0.5 % behind on the
// latter).  LD_GEMM_SKINNY_MAX: tuning knob, 32 .. 64.
int skinny_max_rows() {
    static const int v = env_int("LD_GEMM_SKINNY_MAX", 48);
    return std::min(std::max(v, 32), 64);
}

int split_factor(int T, int N, int K, int epi, bool f16 = false) {
    if (T <= skinny_max_rows()) return (K + SL - 1) / SL;   // skinny kernel: one 512-wide slab per workgroup
    if (T > 64) { const BigPlan p = plan_big(T, N, K, epi, f16); return std::max(p.ks, p.ks_b); }
    const Shape sh = pick_shape(T, epi);
    const int n_ttiles = (T + sh.tt * 32 - 1) / (sh.tt * 32), n_nblocks = (N + 128 * sh.wc - 1) / (128 * sh.wc);
    const int wgs = n_ttiles * n_nblocks;
    int ks = (768 + wgs - 1) / wgs;               // aim at ~3 workgroups per CU
    ks = std::min(ks, K / sh.kch / 2);            // at least two chunks per slab
    ks = std::min(ks, K / (8 * T));               // partial sums: at most a quarter of the matrix bytes
    ks = std::min(ks, 32);
    static const int forced = env_int("LD_GEMM_KS", 0);   // tuning knob
    if (forced > 0) ks = std::min(forced, K / sh.kch);
    return std::max(ks, 1);
}

template <int TT, int WC, int KCH>
void launch_shape(const bf16_t *W, const bf16_t *hi, const bf16_t *lo, int T, int N, int K, int epi, float *y,
                  float *partial, hipStream_t s, bool reduce = true, bf16_t *hi_out = nullptr, bf16_t *lo_out = nullptr) {
    const int n_ttiles = (T + TT * 32 - 1) / (TT * 32);
    const int n_nblocks = (N + 128 * WC - 1) / (128 * WC);
    const int ks = split_factor(T, N, K, epi);
    const int grid = ((n_nblocks + 7) / 8) * 8 * n_ttiles * ks;
    const int rgrid = (int)(((int64_t)T * N + 255) / 256);
#define LD_GEMM(EPI_)                                                                                                  \
    do {                                                                                                               \
        LD_LAUNCH((k_gemm_mfma<TT, WC, KCH, EPI_>), dim3(grid), dim3(256), 0, s, W, hi, lo, T, N, K, y, n_ttiles, \
                           ks, partial, hi_out, lo_out);                                                               \
        if (ks > 1 && reduce)                                                                                          \
            LD_LAUNCH((k_splitk_reduce<EPI_>), dim3(rgrid), dim3(256), 0, s, partial, T, N, ks, y, 0, N, hi_out, lo_out); \
    } while (0)
    if (epi == ld::GEMM_STORE) LD_GEMM(ld::GEMM_STORE);
    else if (epi == ld::GEMM_ADD) LD_GEMM(ld::GEMM_ADD);
    else if constexpr (WC == 1) LD_GEMM(ld::GEMM_SWIGLU);   // SwiGLU always runs with one column tile per wave
#undef LD_GEMM
}

}  // namespace

namespace ld {

bool gemm_supported(int T, int N, int K) { return T >= 2 && N > 0 && K > 0 && K % KC == 0; }

size_t gemm_split_bytes(int T, int K) { return (((size_t)2 * T * K * sizeof(bf16_t)) + 255) / 256 * 256; }

// Rows that would only start one more, nearly empty 256-row tile (a mixed step's 4 x 257 + 28 rows, a 2048-row
// chunk beside 63 decode rows) are cut off and go through the small-batch kernels: the weights are streamed
// once more, which costs less than a tile of padding.  Returns the number of such tail rows (0: no cut),
// decided by the same cost model that picks the tile.
int tail_rows(int T, int N, int K, int epi, bool f16) {
    const int r = T % 256;
    static const int enabled = env_int("LD_GEMM_TAIL", 1);   // tuning knob: 0 keeps every row in the tiled kernel
    if (!enabled || T <= 256 || r == 0 || r > 64 || getenv("LD_GEMM_BIG")) return 0;
    const double whole = plan_big(T, N, K, epi, f16).est_us, main_part = plan_big(T - r, N, K, epi, f16).est_us;
    const double tail = (double)N * (epi == GEMM_SWIGLU ? 2 : 1) * K * 2.0 / 4.0e6 + 12.0;   // ~4 TB/s + two launches
    return main_part + tail < whole ? r : 0;
}

static size_t partial_bytes(int T, int N, int K, int epi, bool f16 = false) {
    const int ks = split_factor(T, N, K, epi, f16);
    return (ks > 1 || T <= skinny_max_rows()) ? (size_t)ks * T * N * (epi == GEMM_SWIGLU ? 2 : 1) * sizeof(float) : 0;
}

size_t gemm_scratch_bytes(int T, int N, int K, int epi) {
    const int r = tail_rows(T, N, K, epi, false);
    size_t part = r ? std::max(partial_bytes(T - r, N, K, epi), partial_bytes(r, N, K, epi)) : partial_bytes(T, N, K, epi);
    if (T > 64) {      // the same pass in the fp16 form may split K differently
        const int rf = tail_rows(T, N, K, epi, true);
        part = std::max(part, partial_bytes(T - rf, N, K, epi, true));
        if (rf) part = std::max(part, partial_bytes(rf, N, K, epi));
    }
    return gemm_split_bytes(T, K) + part;
}

void launch_norm_split(const float *x, const float *g, float eps, int T, int K, uint16_t *xs, hipStream_t s) {
    LD_LAUNCH(k_norm_split, dim3(T), dim3(256), 0, s, x, g, eps, K, xs, xs + (size_t)T * K);
}

int skinny_slabs(int K) { return (K + SL - 1) / SL; }

// K a multiple of the slab width: every workgroup's slab is whole and its loads are unconditional (the compiler
// can then count how many loads may stay in flight at each use)
static void skinny_launch(const uint16_t *W, const uint16_t *xhi, const uint16_t *xlo, int T, int n_rows, int K, int ks,
                          float *partial, hipStream_t s) {
    const dim3 grid(((n_rows + 127) / 128) * ks);
    if (K % SL == 0) LD_LAUNCH(k_gemm_skinny<true>, grid, dim3(256), 0, s, W, xhi, xlo, T, n_rows, K, ks, partial);
    else LD_LAUNCH(k_gemm_skinny<false>, grid, dim3(256), 0, s, W, xhi, xlo, T, n_rows, K, ks, partial);
}

void launch_gemm_skinny(const uint16_t *W, const uint16_t *xhi, const uint16_t *xlo, int T, int n_rows, int K,
                        float *partial, hipStream_t s) {
    const int ks = skinny_slabs(K);
    skinny_launch(W, xhi, xlo, T, n_rows, K, ks, partial, s);
}

// The direct-to-LDS kernel addresses its operands with 32-bit byte offsets from the start of each matrix.
static bool dma_offsets_fit(int T, int N, int K, int epi) {
    const int64_t lim = (int64_t)1 << 32;
    return (int64_t)T * K * 2 < lim && (int64_t)N * (epi == GEMM_SWIGLU ? 2 : 1) * K * 2 < lim;
}

// One launch of the big-tile kernel over output columns [col0, col1) with split factor ks (+ its reduction).
static void launch_big_cols(const uint16_t *W, const bf16_t *hi, const bf16_t *lo, int T, int N, int K, int epi, float *y,
                            float *partial, int wm, int bn, int n_ttiles, int ks, int col0, int col1, hipStream_t s,
                            bool reduce, bf16_t *hi_out, bf16_t *lo_out, int f16) {
    const int nout = epi == GEMM_SWIGLU ? bn / 2 : bn;
    const int n_nblocks = (col1 - col0 + nout - 1) / nout;
    const int grid = ((n_nblocks + 7) / 8) * 8 * n_ttiles * ks;
    const int rgrid = (int)(((int64_t)T * (col1 - col0) + 255) / 256);
#define LD_BIG(WM_, BN_, D_, EPI_)                                                                                     \
    do {                                                                                                               \
        LD_LAUNCH((k_gemm_big<WM_, BN_, D_, EPI_>), dim3(grid), dim3(128 * WM_), 0, s, W, hi, lo, T, N, K, y,           \
                  n_ttiles, ks, partial, col0, col1, hi_out, lo_out);                                                  \
        if (ks > 1 && reduce)                                                                                          \
            LD_LAUNCH((k_splitk_reduce<EPI_>), dim3(rgrid), dim3(256), 0, s, partial, T, N, ks, y, col0, col1, hi_out, lo_out); \
    } while (0)
#define LD_DMA_M(WM_, BN_, S_, EPI_, WN_, F16_)                                                                        \
    do {                                                                                                               \
        constexpr int lds_bytes = ((F16_ ? 1 : 2) * 64 * WM_ + BN_) * 64 * S_;                                         \
        static bool attr_set = false;                                                                                  \
        if (!attr_set) {                                                                                               \
            (void)hipFuncSetAttribute((const void *)k_gemm_dma<WM_, BN_, S_, EPI_, WN_, F16_>,                         \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);                          \
            attr_set = true;                                                                                           \
        }                                                                                                              \
        LD_LAUNCH((k_gemm_dma<WM_, BN_, S_, EPI_, WN_, F16_>), dim3(grid), dim3(64 * WM_ * WN_), lds_bytes, s, W, hi,   \
                  lo, T, N, K, y, n_ttiles, ks, partial, col0, col1, hi_out, lo_out);                                  \
    } while (0)
    // The fp16 form has one operand image to stage, so the 256 x 256 tile fits a fourth stage into the CU's 160 KB
    // (128 KB): with the weight image, 5 - 9 % on the layer shapes at 2048 rows, level at 1056; a fifth changes nothing.
#define LD_DMA(WM_, BN_, S_, EPI_, WN_)                                                                                \
    do {                                                                                                               \
        if (f16 == 2) LD_DMA_M(WM_, BN_, (WM_ == 4 ? 4 : S_), EPI_, WN_, 2);                                           \
        else if (f16) LD_DMA_M(WM_, BN_, (WM_ == 4 ? 4 : S_), EPI_, WN_, 1);                                           \
        else LD_DMA_M(WM_, BN_, S_, EPI_, WN_, 0);                                                                     \
        if (ks > 1 && reduce)                                                                                          \
            LD_LAUNCH((k_splitk_reduce<EPI_>), dim3(rgrid), dim3(256), 0, s, partial, T, N, ks, y, col0, col1, hi_out, lo_out); \
    } while (0)
    // 256-row weight tiles: operands copied straight into LDS (the slab needs a few chunks to fill the stages)
    if (bn == 256 && (K / 32) / ks >= 4 && dma_offsets_fit(T, N, K, epi)) {
        if (wm == 4) {          // 256 x 256: eight waves, 64 x 128 each
            if (epi == GEMM_STORE) LD_DMA(4, 256, 3, GEMM_STORE, 2);
            else if (epi == GEMM_ADD) LD_DMA(4, 256, 3, GEMM_ADD, 2);
            else LD_DMA(4, 256, 3, GEMM_SWIGLU, 2);
        } else {                // 128 x 256: eight waves, 64 x 64 each
            if (epi == GEMM_STORE) LD_DMA(2, 256, 4, GEMM_STORE, 4);
            else if (epi == GEMM_ADD) LD_DMA(2, 256, 4, GEMM_ADD, 4);
            else LD_DMA(2, 256, 4, GEMM_SWIGLU, 4);
        }
        return;
    }
    if (wm == 4) {
        if (epi == GEMM_STORE) LD_BIG(4, 256, 3, GEMM_STORE);
        else if (epi == GEMM_ADD) LD_BIG(4, 256, 3, GEMM_ADD);
        else LD_BIG(4, 256, 3, GEMM_SWIGLU);
    } else if (bn == 256) {
        if (epi == GEMM_STORE) LD_BIG(2, 256, 4, GEMM_STORE);
        else if (epi == GEMM_ADD) LD_BIG(2, 256, 4, GEMM_ADD);
        else LD_BIG(2, 256, 4, GEMM_SWIGLU);
    } else {
        if (epi == GEMM_STORE) LD_BIG(2, 128, 4, GEMM_STORE);
        else if (epi == GEMM_ADD) LD_BIG(2, 128, 4, GEMM_ADD);
        else LD_BIG(2, 128, 4, GEMM_SWIGLU);
    }
#undef LD_BIG
#undef LD_DMA
#undef LD_DMA_M
}

// Where the rows of a residual GEMM go next: the operand image of the normalised GEMM that follows.
struct RowsNext { const float *g; float eps; bf16_t *hi, *lo; const RopeKvArgs *rope; int row0; };

// nx != nullptr with GEMM_ADD: y's rows are finished and turned into the next operand by one fused kernel in
// place of the split-K reduction.  With GEMM_SWIGLU: the epilogue (or the split-K reduction) writes its result
// as the next operand instead of floats.
// Whether the fp16 form serves a product of T rows: the direct-to-LDS kernel with 256-wide weight tiles must be the
// plan's choice in every phase.
static bool f16_plan_ok(const BigPlan &p, int K) {
    return p.bn == 256 && (K / 32) / std::max(p.ks, 1) >= 4 && (p.nb_a == 0 || (K / 32) / std::max(p.ks_b, 1) >= 4);
}
bool gemm_f16_rows(int T, int N, int K, int epi) {
    return T > 64 && dma_offsets_fit(T, N, K, epi) && f16_plan_ok(plan_big(T, N, K, epi, true), K);
}

// f16_flag != nullptr (more than 64 rows, gemm_f16_rows): the rows' images are turned into one fp16 image in place
// and multiplied in the single-term form; *f16_flag is set if an activation does not fit.  W16: the matrix's fp16
// image where the caller keeps one (the kernel then reads it in W's place and converts nothing), else nullptr.
static void gemm_rows(const uint16_t *W, bf16_t *hi, const bf16_t *lo, int T, int N, int K, int epi, float *y,
                      float *partial, hipStream_t s, const RowsNext *nx = nullptr, int *f16_flag = nullptr,
                      const uint16_t *W16 = nullptr) {
    const bool chain_rope = nx && epi == GEMM_STORE && nx->rope;
    const bool chain_add = (nx && epi == GEMM_ADD) || chain_rope;      // a finishing kernel replaces the split-K reduction
    bf16_t *ho = nx && epi == GEMM_SWIGLU ? nx->hi : nullptr, *lo_o = nx && epi == GEMM_SWIGLU ? nx->lo : nullptr;
    // slabs and output columns whose partial sums the finishing kernel still has to add (none: ks 1)
    auto finish = [&](int ks, int col0, int col1, bool always_partial = false) {
        if (ks <= 1 && !always_partial) col0 = col1 = 0;
        if (chain_rope)
            LD_LAUNCH(k_reduce_rope_kv, dim3(nx->rope->H + nx->rope->Hkv, T), dim3(64), 0, s, partial, T, N, ks, col0, col1, y,
                      *nx->rope, nx->row0);
        else
            LD_LAUNCH(k_reduce_add_norm_split, dim3(T), dim3(256), 0, s, partial, T, N, ks, col0, col1, y, nx->g, nx->eps,
                      nx->hi, nx->lo);
    };
    if (T <= skinny_max_rows()) {
        const int ks = split_factor(T, N, K, epi), n_rows = N * (epi == GEMM_SWIGLU ? 2 : 1);
        skinny_launch(W, hi, lo, T, n_rows, K, ks, partial, s);
        const int rgrid = (int)(((int64_t)T * N + 255) / 256);
        bf16_t *none = nullptr;
        if (chain_add) finish(ks, 0, N, true);     // the skinny kernel writes partial sums even for one slab
        else if (epi == GEMM_STORE) LD_LAUNCH((k_splitk_reduce<GEMM_STORE>), dim3(rgrid), dim3(256), 0, s, partial, T, N, ks, y, 0, N, none, none);
        else if (epi == GEMM_ADD) LD_LAUNCH((k_splitk_reduce<GEMM_ADD>), dim3(rgrid), dim3(256), 0, s, partial, T, N, ks, y, 0, N, none, none);
        else LD_LAUNCH((k_splitk_reduce<GEMM_SWIGLU>), dim3(rgrid), dim3(256), 0, s, partial, T, N, ks, y, 0, N, ho, lo_o);
        return;
    }
    if (T > 64) {
        const int f16 = f16_flag ? (W16 ? 2 : 1) : 0;
        const BigPlan p = plan_big(T, N, K, epi, f16 != 0);
        if (f16 == 2) W = W16;
        if (f16) {
            const int64_t n8 = (int64_t)T * K / 8;
            LD_LAUNCH(k_split_to_f16, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s, hi, lo, n8, f16_flag);
        }
        if (p.nb_a > 0) {
            // two phases: whole rounds of unsplit tiles, then the remaining column blocks with a split K
            const int nout = (epi == GEMM_SWIGLU ? p.bn / 2 : p.bn), mid = p.nb_a * nout;
            launch_big_cols(W, hi, lo, T, N, K, epi, y, partial, p.wm, p.bn, p.n_ttiles, 1, 0, mid, s, true, ho, lo_o, f16);
            launch_big_cols(W, hi, lo, T, N, K, epi, y, partial, p.wm, p.bn, p.n_ttiles, p.ks_b, mid, N, s, !chain_add, ho, lo_o, f16);
            if (chain_add) finish(p.ks_b, mid, N);
        } else {
            launch_big_cols(W, hi, lo, T, N, K, epi, y, partial, p.wm, p.bn, p.n_ttiles, p.ks, 0, N, s, !chain_add, ho, lo_o, f16);
            if (chain_add) finish(p.ks, 0, N);
        }
        return;
    }
    launch_shape<2, 1, 128>(W, hi, lo, T, N, K, epi, y, partial, s, !chain_add, ho, lo_o);   // 49..64 rows
    if (chain_add) finish(split_factor(T, N, K, epi), 0, N);
}

void launch_gemm(const uint16_t *W, uint16_t *xs, int T, int N, int K, int epi, float *y, hipStream_t s,
                 const GemmNext *next, int *f16_flag, const uint16_t *W16) {
    float *partial = (float *)((char *)xs + gemm_split_bytes(T, K));
    bf16_t *hi = xs, *lo = xs + (size_t)T * K;
    // the rows beyond a multiple of 256 that the cost model sends through the small-batch kernels keep both terms
    int r = tail_rows(T, N, K, epi, f16_flag != nullptr);
    if (f16_flag && !gemm_f16_rows(T - r, N, K, epi)) {
        f16_flag = nullptr;
        r = tail_rows(T, N, K, epi, false);
    }
    // the next operand is a [2][T][N] image: rows of the main part first, the tail's rows behind them
    RowsNext a{}, b{};
    if (next) {
        a = {next->g, next->eps, next->xs, next->xs ? next->xs + (size_t)T * N : nullptr, next->rope, 0};
        b = {next->g, next->eps, next->xs ? a.hi + (size_t)(T - r) * N : nullptr, next->xs ? a.lo + (size_t)(T - r) * N : nullptr,
             next->rope, T - r};
    }
    gemm_rows(W, hi, lo, T - r, N, K, epi, y, partial, s, next ? &a : nullptr, f16_flag, W16);
    // the tail reuses the partial-sum scratch: the stream orders it behind the main part's reduction
    if (r) gemm_rows(W, hi + (size_t)(T - r) * K, lo + (size_t)(T - r) * K, r, N, K, epi, y + (size_t)(T - r) * N, partial, s,
                     next ? &b : nullptr);
}

void launch_weight_range_check(const uint16_t *W, int64_t n, int *flag, hipStream_t s) {
    LD_LAUNCH(k_weight_range, dim3(1024), dim3(256), 0, s, W, n / 8, flag);
}

void launch_weight_to_f16(const uint16_t *W, int64_t n, uint16_t *out, int *flag, hipStream_t s) {
    LD_LAUNCH(k_weight_to_f16, dim3(1024), dim3(256), 0, s, W, n / 8, out, flag);
}

}  // namespace ld
