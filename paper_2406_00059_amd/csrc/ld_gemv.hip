// Batch-1 matrix-vector product for bf16 matrices, organised by column slabs.
//
// HBM-bound: every matrix element is read exactly once, so the design goal is to keep as many
// 16-byte loads in flight per CU as possible, with as few vector-ALU instructions per loaded byte
// as possible, and with the same amount of work on every CU.
//
//  - The grid is a small multiple of the CU count; workgroup i owns the contiguous output range
//    [i N / G, (i+1) N / G), so all workgroups stream the same number of bytes (+-1 row).
//  - Inside a workgroup the K dimension is split over the waves: wave w owns the column slab
//    [w * 512 * CPW, (w+1) * 512 * CPW).  Its slice of the input vector (already multiplied by the
//    RMSNorm gain) lives in 8*CPW registers per lane for the whole kernel; the input is read once
//    per wave instead of once per output row.
//  - Matrix rows are processed in groups of GL loads per lane.  All loads of a group are issued
//    back to back (they are independent), and the next group's loads are issued before the
//    current group is reduced (double buffering in registers).
//  - A group's per-lane partial sums are reduced across the 64 lanes with a transposing butterfly
//    (GL - 1 + log2(64 / GL) shuffles for GL rows instead of 6 per row), then across the waves
//    through LDS, one barrier per group.
//  - The RMSNorm scale 1 / rms(x) is a scalar, so it is applied to the finished dot products; its
//    sum of squares is accumulated from the same input slice and shares the first barrier.
//  - Epilogues: store, residual add, SwiGLU (gate row r with up row N + r), and "RoPE + cache
//    append" for the fused q/k/v projection (row i of a head with row i + hd/2, then rotate by
//    the position's angle and write k, v straight into the paged pool).
#include "ld_gemv.h"
#include "ld_device.h"
#include "ld_internal.h"
#include <cstdlib>

using namespace ldd;

namespace {

constexpr int MAX_WAVES = 16;
constexpr int MAX_GL = 16;

// Transposing butterfly: on entry every lane holds G partial sums a[0..G); on exit lane L holds in
// a[0] the sum over all 64 lanes of row row_of_lane<G>(L).
template <int G>
__device__ __forceinline__ float transpose_reduce(float (&a)[G], int lane) {
    int off = 32;
#pragma unroll
    for (int n = G; n > 1; n >>= 1) {
        const int half = n >> 1;
        const bool upper = (lane & off) != 0;
#pragma unroll
        for (int j = 0; j < half; j++) {
            const float send = upper ? a[j] : a[j + half];
            const float keep = upper ? a[j + half] : a[j];
            a[j] = keep + __shfl_xor(send, off, WAVE);
        }
        off >>= 1;
    }
    for (; off > 0; off >>= 1) a[0] += __shfl_xor(a[0], off, WAVE);
    return a[0];
}
template <int G>
__device__ __forceinline__ int row_of_lane(int lane) {
    int row = 0, bit = 5;
#pragma unroll
    for (int n = G; n > 1; n >>= 1) {
        row = (row << 1) | ((lane >> bit) & 1);
        bit--;
    }
    return row;
}
template <int G>
__device__ __forceinline__ bool lane_writes(int lane) {
    // one lane per row: the lanes whose bits below the row bits are zero
    int used = 0;
    for (int n = G; n > 1; n >>= 1) used++;
    return (lane & ((1 << (6 - used)) - 1)) == 0;
}

__device__ __forceinline__ float dot8(const u32x4_t &w, const float (&x)[8]) {
    float s = 0.f;
    s = fmaf(__uint_as_float(w.x << 16), x[0], s);
    s = fmaf(__uint_as_float(w.x & 0xffff0000u), x[1], s);
    s = fmaf(__uint_as_float(w.y << 16), x[2], s);
    s = fmaf(__uint_as_float(w.y & 0xffff0000u), x[3], s);
    s = fmaf(__uint_as_float(w.z << 16), x[4], s);
    s = fmaf(__uint_as_float(w.z & 0xffff0000u), x[5], s);
    s = fmaf(__uint_as_float(w.w << 16), x[6], s);
    s = fmaf(__uint_as_float(w.w & 0xffff0000u), x[7], s);
    return s;
}

// Matrix row of unit u, member m (m = 0: first row of the unit; m = 1: its partner row).
template <int EPI>
__device__ __forceinline__ int unit_row(int u, int m, int N, int half_hd) {
    if constexpr (EPI == ld::GEMV_SWIGLU) return u + m * N;
    else if constexpr (EPI == ld::GEMV_ROPE_KV) return (u / half_hd) * (2 * half_hd) + (u % half_hd) + m * half_hd;
    else return u;
}

// GL = 16-byte loads issued per lane per group: 8 keeps the kernel under 128 VGPRs (up to 16 waves
// per workgroup, 4 waves per SIMD) with two groups in flight.
template <int CPW, int GL, int EPI, bool NORM>
__global__ __launch_bounds__(1024) void k_gemv1(const bf16_t *__restrict__ W, const float *__restrict__ x,
                                                const float *__restrict__ g, float eps, int N, int K,
                                                float *__restrict__ y, ld::RopeKvArgs rk) {
    constexpr bool PAIRED = (EPI == ld::GEMV_SWIGLU || EPI == ld::GEMV_ROPE_KV);
    constexpr int G = GL / CPW;                // matrix rows per group
    constexpr int UG = PAIRED ? G / 2 : G;     // output units per group
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int half_hd = (EPI == ld::GEMV_ROPE_KV) ? rk.hd / 2 : 1;
    const int n_units = (EPI == ld::GEMV_ROPE_KV) ? N / 2 : N;
    const int u_begin = (int)((int64_t)blockIdx.x * n_units / gridDim.x);
    const int u_end = (int)((int64_t)(blockIdx.x + 1) * n_units / gridDim.x);
    const int n_groups = (u_end - u_begin + UG - 1) / UG;
    __shared__ float part[2][MAX_WAVES][MAX_GL];
    __shared__ float part_ss[MAX_WAVES];

    // column offsets of this lane inside a row; a lane past the end of the row contributes zeros
    int kofs[CPW];
    bool kval[CPW];
#pragma unroll
    for (int c = 0; c < CPW; c++) {
        kofs[c] = (wave * CPW + c) * (WAVE * 8) + lane * 8;
        kval[c] = kofs[c] < K;
        if (!kval[c]) kofs[c] = 0;
    }

    u32x4_t bufA[G][CPW], bufB[G][CPW];
    auto issue = [&](u32x4_t (&buf)[G][CPW], int gi) {
        const int u0 = u_begin + gi * UG;
#pragma unroll
        for (int r = 0; r < G; r++) {
            const int u = u0 + (PAIRED ? r % UG : r);
            if (u < u_end) {   // uniform over the workgroup: units past the range are not fetched
                const int row = unit_row<EPI>(u, PAIRED ? r / UG : 0, N, half_hd);
                const bf16_t *p = W + (int64_t)row * K;
#pragma unroll
                for (int c = 0; c < CPW; c++) buf[r][c] = load_stream16(p + kofs[c]);
            } else {
#pragma unroll
                for (int c = 0; c < CPW; c++) buf[r][c] = (u32x4_t){0u, 0u, 0u, 0u};
            }
        }
    };
    if (n_groups > 0) issue(bufA, 0);

    // cache append: position and physical block are looked up once, right after the first weight loads are
    // on their way, so that the chain of dependent loads (position -> block table) overlaps the weight
    // stream instead of ending every output group
    int kv_pos = 0;
    int64_t kv_phys = 0;
    if constexpr (EPI == ld::GEMV_ROPE_KV) {
        kv_pos = rk.pos[0];
        kv_phys = rk.table[(int64_t)rk.seq_slot[0] * rk.table_stride + (kv_pos >> 4)];
    }

    // this wave's slice of the input (gain applied), and its share of the sum of squares
    float xs[CPW][8];
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < CPW; c++) {
        if (kval[c]) {
            load8(x + kofs[c], xs[c]);
            if (NORM) {
                float gv[8];
                load8(g + kofs[c], gv);
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    ss = fmaf(xs[c][e], xs[c][e], ss);
                    xs[c][e] *= gv[e];
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; e++) xs[c][e] = 0.f;
        }
    }
    if (NORM) {
        ss = wave_sum(ss);
        if (lane == 0) part_ss[wave] = ss;
    }
    float rstd = 1.f;

    auto consume = [&](u32x4_t (&buf)[G][CPW], int gi) {
        // the old value for the residual add is requested before the arithmetic, not after the barrier
        const int u = u_begin + gi * UG + (int)threadIdx.x;
        const bool mine = threadIdx.x < UG && u < u_end;
        float pre0 = 0.f;
        if constexpr (EPI == ld::GEMV_ADD) {
            if (mine) pre0 = y[u];
        }
        float acc[G];
#pragma unroll
        for (int r = 0; r < G; r++) {
            acc[r] = 0.f;
#pragma unroll
            for (int c = 0; c < CPW; c++) acc[r] += dot8(buf[r][c], xs[c]);
        }
        const float tot = transpose_reduce<G>(acc, lane);
        if (lane_writes<G>(lane)) part[gi & 1][wave][row_of_lane<G>(lane)] = tot;
        lds_barrier();
        if (NORM && gi == 0) {
            float s2 = 0.f;
            for (int w = 0; w < nwaves; w++) s2 += part_ss[w];
            rstd = 1.0f / sqrtf(s2 / K + eps);
        }
        if (mine) {
            float a = 0.f, b = 0.f;
            for (int w = 0; w < nwaves; w++) {
                a += part[gi & 1][w][threadIdx.x];
                if (PAIRED) b += part[gi & 1][w][threadIdx.x + UG];
            }
            a *= rstd;
            b *= rstd;
            if constexpr (EPI == ld::GEMV_STORE) {
                y[u] = a;
            } else if constexpr (EPI == ld::GEMV_ADD) {
                y[u] = pre0 + a;
            } else if constexpr (EPI == ld::GEMV_SWIGLU) {
                y[u] = a / (1.0f + __expf(-a)) * b;
            } else {
                const int hh = u / half_hd, i = u % half_hd, hd = 2 * half_hd;
                if (hh < rk.H + rk.Hkv) {   // q or k head: rotate the pair
                    const float2 cs = rk.cos_sin[i];
                    const float ra = a * cs.x - b * cs.y, rb = a * cs.y + b * cs.x;
                    a = ra;
                    b = rb;
                }
                if (hh < rk.H) {
                    y[hh * hd + i] = a;
                    y[hh * hd + i + half_hd] = b;
                } else {
                    const int which = hh < rk.H + rk.Hkv ? 0 : 1;
                    const int j = hh - rk.H - which * rk.Hkv;
                    bf16_t *blk = rk.pool + kv_phys * kv_block_elems(rk.Hkv, hd);
                    const int slot = kv_pos & 15;
                    if (which == 0) {
                        blk[kv_k_offset(hd, j, slot, i)] = f32_to_bf16(a);
                        blk[kv_k_offset(hd, j, slot, i + half_hd)] = f32_to_bf16(b);
                    } else {
                        blk[kv_v_offset(rk.Hkv, hd, j, slot, i)] = f32_to_bf16(a);
                        blk[kv_v_offset(rk.Hkv, hd, j, slot, i + half_hd)] = f32_to_bf16(b);
                    }
                }
            }
        }
    };

    for (int gi = 0; gi < n_groups; gi += 2) {
        if (gi + 1 < n_groups) issue(bufB, gi + 1);
        consume(bufA, gi);
        if (gi + 1 < n_groups) {
            if (gi + 2 < n_groups) issue(bufA, gi + 2);
            consume(bufB, gi + 1);
        }
    }
}

template <int CPW, int GL, bool NORM>
void launch_cpw(const bf16_t *W, const float *x, const float *g, float eps, int N, int K, int epi, float *y,
                const ld::RopeKvArgs &rk, int grid, int threads, hipStream_t s) {
#define LD_GEMV1(EPI_) LD_LAUNCH((k_gemv1<CPW, GL, EPI_, NORM>), dim3(grid), dim3(threads), 0, s, W, x, g, eps, N, K, y, rk)
    switch (epi) {
        case ld::GEMV_STORE: LD_GEMV1(ld::GEMV_STORE); break;
        case ld::GEMV_ADD: LD_GEMV1(ld::GEMV_ADD); break;
        case ld::GEMV_SWIGLU: LD_GEMV1(ld::GEMV_SWIGLU); break;
        default: LD_GEMV1(ld::GEMV_ROPE_KV); break;
    }
#undef LD_GEMV1
}

int env_int(const char *name, int dflt) {
    const char *v = getenv(name);
    return v ? atoi(v) : dflt;
}

}  // namespace

namespace ld {

bool gemv1_supported(int N, int K, int epi) {
    if (K % 8 || K <= 0 || N <= 0) return false;
    const int chunks = (K + 511) / 512;
    if (chunks > 2 * MAX_WAVES) return false;
    if (epi == GEMV_ROPE_KV && N % 2) return false;
    return true;
}

void launch_gemv1(const uint16_t *W, const float *x, const float *g, float eps, int N, int K, int epi, float *y,
                  const RopeKvArgs *rk, hipStream_t s) {
    static int n_cu = 0;
    if (!n_cu) {
        hipDeviceProp_t p;
        int dev = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess) n_cu = p.multiProcessorCount;
        if (n_cu <= 0) n_cu = 256;
    }
    const int chunks = (K + 511) / 512;
    const int cpw = chunks <= MAX_WAVES ? 1 : 2;
    const int waves = (chunks + cpw - 1) / cpw;
    const int n_units = epi == GEMV_ROPE_KV ? N / 2 : N;
    // Workgroups per CU (measured on the 7B shapes): long rows (two slabs per wave) like one resident
    // workgroup, matrices with many outputs like six, the rest two.
    static const int forced = env_int("LD_GEMV_WGS_PER_CU", 0);   // tuning knob
    const int grid_per_cu = forced > 0 ? forced : (cpw == 2 ? 1 : (n_units >= 10000 ? 6 : 2));
    int grid = n_cu * grid_per_cu;
    if (grid > n_units) grid = n_units;
    RopeKvArgs none{};
    const RopeKvArgs &r = rk ? *rk : none;
    if (cpw == 1) {
        if (g) launch_cpw<1, 8, true>(W, x, g, eps, N, K, epi, y, r, grid, waves * 64, s);
        else launch_cpw<1, 8, false>(W, x, g, eps, N, K, epi, y, r, grid, waves * 64, s);
    } else {
        if (g) launch_cpw<2, 8, true>(W, x, g, eps, N, K, epi, y, r, grid, waves * 64, s);
        else launch_cpw<2, 8, false>(W, x, g, eps, N, K, epi, y, r, grid, waves * 64, s);
    }
}

}  // namespace ld
