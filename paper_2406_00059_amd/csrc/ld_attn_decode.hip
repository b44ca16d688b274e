// Paged decode attention for grouped KV heads on the matrix cores (bf16 pool, head_dim 128,
// 2 .. 16 query heads per KV head).
//
// When several query heads share one KV head, the scalar kernel's arithmetic per cached byte grows with
// the group size and it stops keeping up with HBM.  Here the G queries of a group are the columns of
// 16x16x32 MFMA tiles (columns G .. 15 are zero), so the arithmetic per cached byte is the same for any
// G <= 16 and small next to the load time.
//
// Work item = (row t, KV head, chunk c) as in the scalar kernel; a workgroup of 4 waves takes one item,
// wave w the 32-position steps w, w+4, ... of the chunk.  Nothing goes through LDS but the final merge
// of the four waves: keys and (transposed) values are loaded straight into MFMA operand registers, in two
// register sets of one step (16 KB per wave) each, refilled as soon as a step has been multiplied; two
// workgroups share a CU.
//
//   S^T[pos, q]  = K[pos, :] . Q[q, :]       one 16 x 16 tile per block: A = key rows (lane l: slot l % 16,
//                                            dims 32 j + 8 (l / 16) .. +8 in k-step j), B = Q (hi + lo)
//   O^T[d, q]   += V^T[d, pos] P^T[pos, q]   contraction over the 32 positions of a step: A = V^T
//                                            (lane l: dim 16 nt + l % 16; slots 4 (l/16) .. +4 of the
//                                            step's first block, then of its second block), B = P^T =
//                                            the score registers: in the 16 x 16 accumulator layout lane
//                                            l holds, for query l % 16, rows 4 (l/16) .. +4 of each tile.
// Scores are kept in the log2 domain; m, l and O are float32; P is split into bf16 hi + lo like Q.
#include "ld_attn_decode.h"
#include "ld_device.h"
#include "ld_internal.h"

using namespace ldd;

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int HD = 128;

__device__ __forceinline__ int band_first(int ctx, int window) { return (window > 0 && ctx > window) ? ctx - window : 0; }

__global__ __launch_bounds__(256, 2) void k_attn_decode_grouped(const float *__restrict__ q, int q_stride,
                                                                const bf16_t *__restrict__ pool, int Hkv,
                                                                const int32_t *__restrict__ table, int table_stride,
                                                                const int32_t *__restrict__ seq_slot,
                                                                const int32_t *__restrict__ ctx_len, int H, int G,
                                                                int window, float scale_log2e, int max_chunks, int cb,
                                                                float *__restrict__ part_o,
                                                                float *__restrict__ part_ml) {
    const int c = blockIdx.x, kvh = blockIdx.y, t = blockIdx.z;
    const int h0 = kvh * G;
    const int ctx = ctx_len[t];
    const int first = band_first(ctx, window);
    const int nblk = (ctx + 15) >> 4;
    const int b_begin = (first >> 4) + c * cb;       // cb is a multiple of 8: four steps of two blocks
    if (b_begin >= nblk) return;
    const int b_end = min(b_begin + cb, nblk);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, rg = lane >> 4;        // column / row-in-tile, and the lane's group of 4 rows or 8 k
    const int64_t block_stride = kv_block_elems(Hkv, HD);
    const int32_t *trow = table + (int64_t)seq_slot[t] * table_stride;

    // Q operand of k-step j: dims 32 j + 8 rg .. +8 of query l16 (zero for l16 >= G), hi and lo parts
    bf16x8 qh[4], ql[4];
    {
        const bool real = l16 < G;
        const float *qp = q + (int64_t)t * q_stride + (h0 + (real ? l16 : 0)) * HD + 8 * rg;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            float v[8];
            load8(qp + 32 * j, v);
            uint32_t hw[4], lw[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const float a = real ? v[2 * e] * scale_log2e : 0.f, b = real ? v[2 * e + 1] * scale_log2e : 0.f;
                hw[e] = split2_bf16(a, b, lw[e]);
            }
            qh[j] = __builtin_bit_cast(bf16x8, (u32x4){hw[0], hw[1], hw[2], hw[3]});
            ql[j] = __builtin_bit_cast(bf16x8, (u32x4){lw[0], lw[1], lw[2], lw[3]});
        }
    }

    f32x4 o[8];      // O^T: dims 16 nt + 4 rg + i of query l16
#pragma unroll
    for (int nt = 0; nt < 8; nt++) o[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    // One step = blocks (b, b+1).  kf[blk][j]: key operand of k-step j; vf[nt][blk]: 4 positions of a dimension.
    struct Step { u32x4 kf[2][4]; u32x2 vf[8][2]; };
    // The physical ids of all blocks this wave will walk (steps n = 0, 1, ...: blocks b_begin + 2 wave + 8 n and the
    // one after it; at most 16 of a 64-block chunk) are fetched at once, lane 2 n + blk holding one: a table lookup
    // inside the walk would be a load younger than the keys and values already requested for the step ahead, and
    // waiting for it (loads return in order) would wait for all of those first.  A second block past the chunk
    // is read again from the chunk's last one and masked out in compute().
    const int my_blk = lane < 16 ? trow[min(b_begin + 2 * wave + 8 * (lane >> 1) + (lane & 1), b_end - 1)] : 0;
    auto block_of = [&](int b, int blk) {
        return (int64_t)__builtin_amdgcn_readlane(my_blk, ((b - b_begin - 2 * wave) >> 2) + blk);
    };
    // Keys are fetched as they lie in memory (a block's 16 key rows of this KV head are 4 KB in a row: load j of a
    // block covers slots 4 j .. 4 j + 3, lane l the 16 bytes at 1024 j + 16 l, so that every 128-byte line belongs to
    // one instruction) and take the A-operand layout (lane = slot) through 4 KB of LDS private to the wave in
    // compute(): piece p (8 dims) of slot s sits in slot (p ^ s) of its 256-byte row.
    __shared__ __attribute__((aligned(16))) char sm_k[4][4096];
    char *tk = sm_k[wave];
    char *tk_st[4];
    const char *tk_ld[4];
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const int sl = 4 * j + rg;
        tk_st[j] = tk + sl * 256 + ((l16 ^ sl) & 15) * 16;
        tk_ld[j] = tk + l16 * 256 + (((4 * j + rg) ^ l16) & 15) * 16;
    }
    auto load_k = [&](Step &s, int b) {
#pragma unroll
        for (int blk = 0; blk < 2; blk++) {
            const bf16_t *kp = pool + block_of(b, blk) * block_stride + kv_k_offset(HD, kvh, 0, 0) + 8 * lane;
#pragma unroll
            for (int j = 0; j < 4; j++) s.kf[blk][j] = load_stream16(kp + 512 * j);
        }
    };
    auto load_v = [&](Step &s, int b) {
#pragma unroll
        for (int blk = 0; blk < 2; blk++) {
            const bf16_t *vp = pool + block_of(b, blk) * block_stride + kv_v_offset(Hkv, HD, kvh, 4 * rg, l16);
#pragma unroll
            for (int nt = 0; nt < 8; nt++)
                s.vf[nt][blk] = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(vp + nt * 16 * 16));
        }
    };

    auto compute = [&](Step &s, int b) {
        // positions of this lane's 4 rows in each tile, and whether the query sees them
        bool ok[2][4];
        bool all_ok = true;
#pragma unroll
        for (int blk = 0; blk < 2; blk++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int pos = (b + blk) * 16 + 4 * rg + i;
                ok[blk][i] = (b + blk) < b_end && pos >= first && pos < ctx;
                all_ok = all_ok && ok[blk][i];
            }
        // ---- scores
        f32x4 st[2];
#pragma unroll
        for (int blk = 0; blk < 2; blk++) {
            st[blk] = (f32x4){0.f, 0.f, 0.f, 0.f};
            // the block's keys through the wave's LDS rows (a wave's LDS operations execute in order)
#pragma unroll
            for (int j = 0; j < 4; j++) *reinterpret_cast<u32x4 *>(tk_st[j]) = s.kf[blk][j];
            __builtin_amdgcn_wave_barrier();
            u32x4 kt[4];
#pragma unroll
            for (int j = 0; j < 4; j++) kt[j] = *reinterpret_cast<const u32x4 *>(tk_ld[j]);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const bf16x8 ka = __builtin_bit_cast(bf16x8, kt[j]);
                st[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qh[j], st[blk], 0, 0, 0);
                st[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, ql[j], st[blk], 0, 0, 0);
            }
        }
        // ---- online softmax of column l16 (rows spread over the four lanes l16, l16+16, l16+32, l16+48)
        float mb = -INFINITY;
#pragma unroll
        for (int blk = 0; blk < 2; blk++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                st[blk][i] = ok[blk][i] ? st[blk][i] : -INFINITY;
                mb = fmaxf(mb, st[blk][i]);
            }
        mb = fmaxf(mb, __shfl_xor(mb, 16, WAVE));
        mb = fmaxf(mb, __shfl_xor(mb, 32, WAVE));
        const float m_new = fmaxf(m, mb);       // finite: every step walked holds a visible position
        const float sc = fast_exp2(m - m_new);
        m = m_new;
        float p[8];
        float psum = 0.f;
#pragma unroll
        for (int blk = 0; blk < 2; blk++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                p[4 * blk + i] = fast_exp2(st[blk][i] - m_new);
                psum += p[4 * blk + i];
            }
        l = l * sc + psum;
        uint32_t ph[4], pl[4];
#pragma unroll
        for (int e = 0; e < 4; e++) ph[e] = split2_bf16(p[2 * e], p[2 * e + 1], pl[e]);
        const bf16x8 pbh = __builtin_bit_cast(bf16x8, (u32x4){ph[0], ph[1], ph[2], ph[3]});
        const bf16x8 pbl = __builtin_bit_cast(bf16x8, (u32x4){pl[0], pl[1], pl[2], pl[3]});
        if (!__all(all_ok)) {      // a partly visible step: unwritten slots may hold anything, also NaN
#pragma unroll
            for (int blk = 0; blk < 2; blk++)
#pragma unroll
                for (int nt = 0; nt < 8; nt++) {
                    u32x2 v = s.vf[nt][blk];
                    v[0] = (ok[blk][0] ? v[0] & 0x0000ffffu : 0u) | (ok[blk][1] ? v[0] & 0xffff0000u : 0u);
                    v[1] = (ok[blk][2] ? v[1] & 0x0000ffffu : 0u) | (ok[blk][3] ? v[1] & 0xffff0000u : 0u);
                    s.vf[nt][blk] = v;
                }
        }
        // ---- O^T = O^T * sc + V^T P^T
        const bool rescale = __any(sc != 1.f);
#pragma unroll
        for (int nt = 0; nt < 8; nt++) {
            if (rescale) {
#pragma unroll
                for (int i = 0; i < 4; i++) o[nt][i] *= sc;
            }
            const bf16x8 va = __builtin_bit_cast(
                bf16x8, (u32x4){s.vf[nt][0][0], s.vf[nt][0][1], s.vf[nt][1][0], s.vf[nt][1][1]});
            o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pbh, o[nt], 0, 0, 0);
            o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pbl, o[nt], 0, 0, 0);
        }
    };

    // steps of this wave: blocks b_begin + 2 (wave + 4 n).  Two register sets: the loads of the step after
    // next are issued before the next step is multiplied, so 16 .. 32 KB per wave are in flight all the time.
    // The steady state requests unconditionally (a request under a condition makes the wait before a product
    // cover every load in flight, the step ahead included); the last one or two steps are peeled off.
    {
        Step sa, sb;
        int b = b_begin + 2 * wave;
        if (b < b_end) {
            load_k(sa, b); load_v(sa, b);
            while (b + 16 < b_end) {
                load_k(sb, b + 8); load_v(sb, b + 8);
                compute(sa, b);
                load_k(sa, b + 16); load_v(sa, b + 16);
                compute(sb, b + 8);
                b += 16;
            }
            if (b + 8 < b_end) {
                load_k(sb, b + 8); load_v(sb, b + 8);
                compute(sa, b);
                compute(sb, b + 8);
            } else {
                compute(sa, b);
            }
        }
    }

    // column statistics: l was summed per lane over its own rows
    l += __shfl_xor(l, 16, WAVE);
    l += __shfl_xor(l, 32, WAVE);
    __shared__ float sm_m[4][16], sm_l[4][16], sm_acc[4][16][HD + 4];
    if (l16 < G) {
#pragma unroll
        for (int nt = 0; nt < 8; nt++)
            *reinterpret_cast<float4 *>(&sm_acc[wave][l16][16 * nt + 4 * rg]) =
                make_float4(o[nt][0], o[nt][1], o[nt][2], o[nt][3]);
        if (rg == 0) { sm_m[wave][l16] = m; sm_l[wave][l16] = l; }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * HD; idx += 256) {
        const int g = idx / HD, d = idx % HD;
        // a wave that walked no step keeps m = -inf and weight 0; wave 0 always walks one
        const float M = fmaxf(fmaxf(sm_m[0][g], sm_m[1][g]), fmaxf(sm_m[2][g], sm_m[3][g]));
        float acc = 0.f, L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; w++) {
            const float a = fast_exp2(sm_m[w][g] - M);
            acc += a * sm_acc[w][g][d];
            L += a * sm_l[w][g];
        }
        const int64_t item = ((int64_t)t * H + h0 + g) * max_chunks + c;
        part_o[item * HD + d] = acc;
        if (d == 0) { part_ml[item * 2] = M; part_ml[item * 2 + 1] = L; }
    }
}

}  // namespace

namespace ld {

bool grouped_decode_supported(int dtype_is_bf16, int hd, int H, int Hkv) {
    const int G = H / Hkv;
    return dtype_is_bf16 && hd == HD && G >= 2 && G <= 16;
}

void launch_grouped_decode_partial(const float *q, int q_stride, const uint16_t *pool, int Hkv, const int32_t *table,
                                   int table_stride, const int32_t *seq_slot, const int32_t *ctx_len, int T, int H,
                                   int window, int max_chunks, int cb, float *part_o, float *part_ml, hipStream_t s) {
    const float sl2 = 1.4426950408889634f / sqrtf((float)HD);
    LD_LAUNCH(k_attn_decode_grouped, dim3(max_chunks, Hkv, T), dim3(256), 0, s, q, q_stride, pool, Hkv, table,
              table_stride, seq_slot, ctx_len, H, H / Hkv, window, sl2, max_chunks, cb, part_o, part_ml);
}

}  // namespace ld
