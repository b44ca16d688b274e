// Chunk-prefill attention over the paged KV pool on the matrix cores (bf16 pool, head_dim 128).
//
// A prefill segment is a run of consecutive rows of one sequence at consecutive positions; row r
// (position p_r) attends to every cached position j <= p_r: the earlier context plus, causally, the
// rows of its own chunk, whose keys/values were appended to the pool just before.  With an attention
// band of W positions it attends to max(0, p_r - W + 1) <= j <= p_r only: the walk over the KV positions
// starts at the first position the tile's first row sees, and a wave skips the steps that lie wholly
// before the band of its own first row.
//
// Work split: a workgroup (4 waves) takes 128 consecutive rows of a segment and one head; wave w
// owns rows [32w, 32w+32).  All four waves walk the same KV positions in steps of 32 tokens; the key
// rows and the (transposed) value tile of a step are copied into LDS once, in 16-byte pieces that were
// loaded into registers one step earlier, and shared by the four waves.  LDS is double buffered: one
// barrier per step.  Two workgroups fit a CU, so that one wave's softmax overlaps another's MFMAs.
//
// Both products are computed transposed, so that the query index is the MFMA column (= lane % 32)
// everywhere and the online-softmax statistics of a query live in the lanes that hold its scores:
//   S^T[kv, q] = K[kv, :] . Q[q, :]      A = K rows   (LDS),
//                                        B = Q        (registers, split into bf16 hi + lo)
//   O^T[d, q] += V^T[d, kv] P^T[kv, q]   A = V^T      (LDS; the pool stores the values of a block
//                                                      transposed, [dim][16 positions]),
//                                        B = P^T      (the score registers themselves: in the 32x32
//                                                      accumulator layout a lane already holds, for
//                                                      its query, exactly the 8 kv slots of an operand)
// Row r of a score tile is NOT position kv0 + r: within each 16 rows, bits 2 and 3 of the row index are
// swapped (row r <-> position 16 (r/16) + tau(r%16), tau(r) = (r & 3) | (r & 4) << 1 | (r & 8) >> 1), so
// that the 8 accumulator registers a lane feeds into one value MFMA are 8 CONSECUTIVE positions, i.e. one
// 16-byte piece of the transposed value tile.
// Scores are kept in the log2 domain (q is pre-multiplied by log2(e)/sqrt(hd)); m, l and O are float32.
//
// Few tiles with long contexts (an observation appended to one long sequence) would leave most CUs idle
// and make every workgroup walk the whole context, so the KV range of a tile can be split over gridDim.z
// workgroups; each then writes its unnormalised output with its maximum and sum, and a merge kernel
// combines the splits in fixed order.
#include "ld_attn_prefill.h"
#include "ld_device.h"
#include "ld_internal.h"

using namespace ldd;

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) uint16_t u16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int HD = 128;
constexpr int KVB = 32;          // kv positions per step
constexpr int KLD = HD + 8;      // LDS row stride of the key tile (elements): 272 bytes, conflict-free 16-byte reads
constexpr int VLD = KVB + 8;     // LDS row stride of the transposed value tile (elements): 80 bytes

__device__ __forceinline__ int tau(int r) { return (r & 19) | ((r & 4) << 1) | ((r & 8) >> 1); }

// Two floats as packed fp16, rounded to nearest.
__device__ __forceinline__ uint32_t pack2_f16(float a, float b) {
    return __builtin_bit_cast(uint32_t, (f16x2){(_Float16)a, (_Float16)b});
}
// Eight bf16 numbers as fp16: exact where fp16 can hold the value (truncation below 2^-14, the largest finite
// fp16 beyond +-65504: the caller looks for such values with `mag`, the running maximum of the magnitudes).
__device__ __forceinline__ u32x4 bf16x8_to_f16x8(const u32x4 &w, u16x2 &mag) {
    u32x4 h;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        h[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w[i] << 16), __uint_as_float(w[i] & 0xffff0000u)));
        mag = __builtin_elementwise_max(mag, __builtin_bit_cast(u16x2, w[i] & 0x7fff7fffu));
    }
    return h;
}

// F16 (the long passes whose rows the engine lets enter the products rounded to fp16): queries and probabilities as
// one fp16 term instead of two bf16 terms, keys and values widened from bf16 to fp16 when they are staged in LDS
// (once per workgroup, exact within the fp16 range): half the matrix-core work.  *f16_flag is set when a query, a
// key or a value lies beyond +-65504 (the pass is then repeated with two terms).
template <bool F16>
__global__ __launch_bounds__(256, 2) void k_attn_prefill(const float *__restrict__ q, int q_stride,
                                                         const bf16_t *__restrict__ pool, int Hkv,
                                                         const int32_t *__restrict__ table, int table_stride,
                                                         const int4 *__restrict__ tiles, int H, int window,
                                                         float scale_log2e, float *__restrict__ out,
                                                         float *__restrict__ part_o, float *__restrict__ part_ml,
                                                         bf16_t *__restrict__ xs_hi, bf16_t *__restrict__ xs_lo,
                                                         int *__restrict__ f16_flag) {
    __shared__ __attribute__((aligned(16))) bf16_t ks[2][KVB][KLD];
    __shared__ __attribute__((aligned(16))) bf16_t vt[2][HD][VLD];
    const int4 tile = tiles[blockIdx.x];      // x: first row, y: rows (<= 128), z: position of first row, w: seq slot
    const int h = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int kvh = h / (H / Hkv);
    const int64_t block_stride = kv_block_elems(Hkv, HD);
    const int32_t *trow = table + (int64_t)tile.w * table_stride;

    // this lane's query: row index inside the tile, validity, absolute position
    const int qi = wave * 32 + l32;
    const bool q_valid = qi < tile.y;
    const int q_pos = tile.z + min(qi, tile.y - 1);
    const int wg_last_pos = tile.z + tile.y - 1;                       // last position any wave needs
    const int wave_last_pos = tile.z + min(wave * 32 + 31, tile.y - 1);
    const bool wave_active = wave * 32 < tile.y;
    // band: lowest position visible to this lane's query, to the wave's first query, to the tile's first query
    const int q_low = window > 0 ? max(q_pos - window + 1, 0) : 0;
    const int wave_low = window > 0 ? max(tile.z + wave * 32 - window + 1, 0) : 0;
    const int wave_first_pos = tile.z + wave * 32;                      // position of the wave's first query
    const int wave_low_hi = window > 0 ? max(wave_last_pos - window + 1, 0) : 0;   // lowest position its last query sees
    const int kv_start = window > 0 ? (max(tile.z - window + 1, 0) & ~(KVB - 1)) : 0;
    // first position of the lowest block any row of the tile sees: block-table entries below it may belong
    // to blocks the sequence has given up (ld_kv_trim) and are never dereferenced
    const int first_held_pos = window > 0 ? (max(tile.z - window + 1, 0) & ~15) : 0;

    // Q operand: for k-step j the lane supplies dims half*64 + j*8 .. +8 of its query (hi and lo parts; F16: one
    // fp16 term in qh)
    u32x4 qh[8], ql[F16 ? 1 : 8];
    bool out_of_range = false;      // F16: a value beyond the fp16 range was seen by this lane
    u16x2 mag = {0, 0};             // F16: largest bf16 magnitude (bit pattern) among the keys and values this lane staged
    {
        const float *qp = q + (int64_t)(tile.x + min(qi, tile.y - 1)) * q_stride + h * HD + half * 64;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            float v[8];
            load8(qp + j * 8, v);
            uint32_t hw[4], lw[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const float a = v[2 * e] * scale_log2e, b = v[2 * e + 1] * scale_log2e;
                if constexpr (F16) {
                    out_of_range = out_of_range || !(fabsf(a) <= 65504.f) || !(fabsf(b) <= 65504.f);
                    hw[e] = pack2_f16(a, b);
                } else {
                    hw[e] = split2_bf16(a, b, lw[e]);
                }
            }
            qh[j] = (u32x4){hw[0], hw[1], hw[2], hw[3]};
            if constexpr (!F16) ql[j] = (u32x4){lw[0], lw[1], lw[2], lw[3]};
        }
    }

    f32x16 o[4];   // O^T: dims 32*nt + 8*(i/4) + 4*half + i%4 of this lane's query
#pragma unroll
    for (int nt = 0; nt < 4; nt++)
#pragma unroll
        for (int i = 0; i < 16; i++) o[nt][i] = 0.f;
    float m = -INFINITY, l = 0.f;

    // The pieces this thread copies per step: key rows (position kr, 16-byte piece kc of the row) and
    // value pieces (dimension vd, positions 8*vh .. +8 of block v of the step).
    const int kr = threadIdx.x >> 4, kc = (threadIdx.x & 15) * 8;       // + 16 rows for the second piece
    const int vd = threadIdx.x >> 1, vh = (threadIdx.x & 1) * 8;
    // Global loads run PF steps ahead of the arithmetic, in PF register sets: with one or two workgroups on
    // a CU the arithmetic of a single step is much shorter than the memory latency it would have to cover.
    constexpr int PF = 3;
    u32x4 kreg[PF][2], vreg[PF][2];
    auto load_step = [&](int set, int kv0) {
#pragma unroll
        for (int v = 0; v < 2; v++) {
            // a block past the last needed position is read again from the last needed block, one below
            // the first visible block from that block; never used
            const int pos = max(min(kv0 + 16 * v, wg_last_pos), first_held_pos);
            const bf16_t *blk = pool + (int64_t)trow[pos >> 4] * block_stride;
            kreg[set][v] = *reinterpret_cast<const u32x4 *>(blk + kv_k_offset(HD, kvh, kr, kc));
            vreg[set][v] = *reinterpret_cast<const u32x4 *>(blk + kv_v_offset(Hkv, HD, kvh, vh, vd));
        }
    };
    // Values of positions past the tile's last row were never written (the rest of the last block, or the
    // second block of a step that ends the walk): they may hold anything, also NaN, and a probability of zero
    // does not neutralise a NaN, so they are staged as zeros.  (Keys need nothing: their scores are replaced,
    // not multiplied.)
    auto stage = [&](int st, int set, int kv0) {
#pragma unroll
        for (int v = 0; v < 2; v++) {
            if constexpr (F16) {
                // a key row past the tile's last position was never written (its scores are masked): whatever it
                // holds does not count as out of range
                u16x2 seen = mag;
                *reinterpret_cast<u32x4 *>(&ks[st][16 * v + kr][kc]) = bf16x8_to_f16x8(kreg[set][v], seen);
                if (kv0 + 16 * v + kr <= wg_last_pos) mag = seen;
            } else {
                *reinterpret_cast<u32x4 *>(&ks[st][16 * v + kr][kc]) = kreg[set][v];
            }
            u32x4 vv = vreg[set][v];
            const int p0 = kv0 + 16 * v + vh;      // position of this piece's first element
            if (p0 + 7 > wg_last_pos) {
#pragma unroll
                for (int e = 0; e < 4; e++)
                    vv[e] = (p0 + 2 * e <= wg_last_pos ? vv[e] & 0x0000ffffu : 0u) |
                            (p0 + 2 * e + 1 <= wg_last_pos ? vv[e] & 0xffff0000u : 0u);
            }
            if constexpr (F16) vv = bf16x8_to_f16x8(vv, mag);
            *reinterpret_cast<u32x4 *>(&vt[st][vd][16 * v + vh]) = vv;
        }
    };
    // this workgroup's share of the tile's steps (all of them when the grid has one split)
    const int n_splits = gridDim.z, split = blockIdx.z;
    const int n_steps = (wg_last_pos - kv_start) / KVB + 1, per = (n_steps + n_splits - 1) / n_splits;
    const int kv_begin = kv_start + split * per * KVB;
    const int kv_end = min(kv_begin + per * KVB, wg_last_pos + 1);      // exclusive; may be <= kv_begin (empty share)
#pragma unroll
    for (int pf = 0; pf < PF; pf++)
        if (kv_begin + pf * KVB < kv_end) load_step(pf, kv_begin + pf * KVB);

    auto compute = [&](int kv0, int st) {

        // ---- S^T = K Q^T for 32 kv positions x 32 queries; tile row l32 is position kv0 + tau(l32)
        f32x16 sc_t;
#pragma unroll
        for (int i = 0; i < 16; i++) sc_t[i] = 0.f;
        const bf16_t *krow = &ks[st][tau(l32)][half * 64];
        // The matrix-core phases run at a raised wave priority: the other workgroup's wave on this SIMD then
        // fills the issue slots between the MFMAs with its softmax arithmetic instead of competing for them.
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const u32x4 ka = *reinterpret_cast<const u32x4 *>(krow + j * 8);
            if constexpr (F16) {
                sc_t = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, ka), __builtin_bit_cast(f16x8, qh[j]), sc_t, 0, 0, 0);
            } else {
                sc_t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka), __builtin_bit_cast(bf16x8, qh[j]), sc_t, 0, 0, 0);
                sc_t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka), __builtin_bit_cast(bf16x8, ql[j]), sc_t, 0, 0, 0);
            }
        }
        __builtin_amdgcn_s_setprio(0);
        // ---- online softmax; accumulator element i is row 8*(i/4) + 4*half + i%4 of the tile, which holds
        // position kv0 + 16*(i/8) + 8*half + i%8
        float mb = -INFINITY;
        if (kv0 + KVB - 1 <= wave_first_pos && kv0 >= wave_low_hi) {
            // every position of the step is visible to every query of the wave (the common case away from
            // the diagonal and the band edge): no masks; rows past the tile compute on a copy of the last row
#pragma unroll
            for (int i = 0; i < 16; i++) mb = fmaxf(mb, sc_t[i]);
        } else {
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int kv_pos = kv0 + 16 * (i / 8) + 8 * half + (i % 8);
                const bool ok = q_valid && kv_pos <= q_pos && kv_pos >= q_low;
                sc_t[i] = ok ? sc_t[i] : -INFINITY;
                mb = fmaxf(mb, sc_t[i]);
            }
        }
        mb = fmaxf(mb, __shfl_xor(mb, 32, WAVE));
        // m is the reference the exponents are taken against, not necessarily the running maximum: it moves up
        // only when the maximum has outgrown it by more than 2^8, so p stays below 256 and the accumulators
        // are rescaled on few steps instead of most.  o, l and m stay consistent, which is all the final
        // division and the split merge need.
        const float m_new = mb > m + 8.f ? mb : m;
        float sc = 1.f;
        uint32_t ph[8], pl[8];
        if (m_new > -INFINITY) {
            sc = fast_exp2(m - m_new);
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const float p0 = fast_exp2(sc_t[i] - m_new), p1 = fast_exp2(sc_t[i + 1] - m_new);
                psum += p0 + p1;
                if constexpr (F16) ph[i / 2] = pack2_f16(p0, p1);      // p < 2^8: well inside fp16
                else ph[i / 2] = split2_bf16(p0, p1, pl[i / 2]);
            }
            l = l * sc + psum;
            m = m_new;
        } else {
#pragma unroll
            for (int e = 0; e < 8; e++) ph[e] = pl[e] = 0u;
        }
        // ---- O^T = O^T * sc + V^T P^T; the rescale is skipped when no query of the wave raised its maximum
        const bool rescale = __any(sc != 1.f);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int nt = 0; nt < 4; nt++) {
            if (rescale) {
#pragma unroll
                for (int i = 0; i < 16; i++) o[nt][i] *= sc;
            }
#pragma unroll
            for (int mm = 0; mm < 2; mm++) {
                // slot e of this lane <-> position kv0 + 16*mm + 8*half + e
                const u32x4 va = *reinterpret_cast<const u32x4 *>(&vt[st][nt * 32 + l32][16 * mm + 8 * half]);
                const u32x4 pbh = (u32x4){ph[4 * mm], ph[4 * mm + 1], ph[4 * mm + 2], ph[4 * mm + 3]};
                if constexpr (F16) {
                    o[nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, va), __builtin_bit_cast(f16x8, pbh), o[nt], 0, 0, 0);
                } else {
                    const u32x4 pbl = (u32x4){pl[4 * mm], pl[4 * mm + 1], pl[4 * mm + 2], pl[4 * mm + 3]};
                    o[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va), __builtin_bit_cast(bf16x8, pbh), o[nt], 0, 0, 0);
                    o[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va), __builtin_bit_cast(bf16x8, pbl), o[nt], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
    };

    int st = 0;
    for (int base = kv_begin; base < kv_end; base += PF * KVB) {
#pragma unroll
        for (int u = 0; u < PF; u++) {
            const int kv0 = base + u * KVB;
            if (kv0 < kv_end) {      // uniform over the workgroup
                // Stage this step, then fetch the step PF ahead into the set just emptied.  One barrier per
                // step: a wave that writes buffer st for step n has passed the barrier of step n-1, which
                // every wave reaches only after it has finished reading buffer st for step n-2.
                stage(st, u, kv0);
                lds_barrier();
                if (kv0 + PF * KVB < kv_end) load_step(u, kv0 + PF * KVB);
                if (wave_active && kv0 <= wave_last_pos && kv0 + KVB > wave_low) compute(kv0, st);   // else nothing visible to this wave
                st ^= 1;
            }
        }
    }
    if constexpr (F16) {      // 0x4780 is 65536 as bf16: the first magnitude that fp16 cannot hold (also infinities and NaNs)
        if (out_of_range || mag[0] >= 0x4780 || mag[1] >= 0x4780) *f16_flag = 1;
    }
    // the two halves of a query's scores were summed separately
    l += __shfl_xor(l, 32, WAVE);
    if (n_splits > 1) {      // unnormalised share: [tile][row in tile][head][split][HD] and (m, l)
        if (q_valid) {
            const int64_t item = (((int64_t)blockIdx.x * 128 + qi) * H + h) * n_splits + split;
            float *op = part_o + item * HD;
#pragma unroll
            for (int nt = 0; nt < 4; nt++)
#pragma unroll
                for (int a = 0; a < 4; a++)
                    *reinterpret_cast<float4 *>(op + nt * 32 + 8 * a + 4 * half) =
                        make_float4(o[nt][4 * a], o[nt][4 * a + 1], o[nt][4 * a + 2], o[nt][4 * a + 3]);
            if (half == 0) { part_ml[item * 2] = m; part_ml[item * 2 + 1] = l; }
        }
        return;
    }
    if (q_valid) {
        const float inv = 1.0f / l;
        const int64_t at = (int64_t)(tile.x + qi) * (H * HD) + h * HD;
#pragma unroll
        for (int nt = 0; nt < 4; nt++)
#pragma unroll
            for (int a = 0; a < 4; a++) {
                // products rounded to float: what a store would hold, also where they go straight into the split
                const float4 v = make_float4(mul_rounded(o[nt][4 * a], inv), mul_rounded(o[nt][4 * a + 1], inv),
                                             mul_rounded(o[nt][4 * a + 2], inv), mul_rounded(o[nt][4 * a + 3], inv));
                const int64_t e = at + nt * 32 + 8 * a + 4 * half;
                if (xs_hi) {      // the output projection's (hi, lo) operand instead of floats
                    uint32_t l0, l1;
                    const uint32_t h0 = split2_bf16(v.x, v.y, l0), h1 = split2_bf16(v.z, v.w, l1);
                    *reinterpret_cast<uint2 *>(xs_hi + e) = make_uint2(h0, h1);
                    *reinterpret_cast<uint2 *>(xs_lo + e) = make_uint2(l0, l1);
                } else {
                    *reinterpret_cast<float4 *>(out + e) = v;
                }
            }
    }
}

// One workgroup per (tile row slot, head): adds the splits of a row in split order.  A split that saw no
// visible position of the row has m = -inf and weight 0; split 0 or a later one always saw one.
__global__ __launch_bounds__(128) void k_attn_prefill_merge(const int4 *__restrict__ tiles, int H, int n_splits,
                                                            const float *__restrict__ part_o,
                                                            const float *__restrict__ part_ml,
                                                            float *__restrict__ out, bf16_t *__restrict__ xs_hi,
                                                            bf16_t *__restrict__ xs_lo) {
    const int4 tile = tiles[blockIdx.y >> 7];
    const int r = blockIdx.y & 127, h = blockIdx.x, d = threadIdx.x;
    if (r >= tile.y) return;
    const int64_t base = ((int64_t)blockIdx.y * H + h) * n_splits;
    float M = -INFINITY;
    for (int z = 0; z < n_splits; z++) M = fmaxf(M, part_ml[(base + z) * 2]);
    float o = 0.f, L = 0.f;
    for (int z = 0; z < n_splits; z++) {
        const float a = fast_exp2(part_ml[(base + z) * 2] - M);
        o += a * part_o[(base + z) * HD + d];
        L += a * part_ml[(base + z) * 2 + 1];
    }
    const int64_t e = ((int64_t)(tile.x + r) * H + h) * HD + d;
    if (xs_hi) store_split(xs_hi, xs_lo, e, o / L);
    else out[e] = o / L;
}

}  // namespace

namespace ld {

bool prefill_attention_supported(int dtype_is_bf16, int hd) { return dtype_is_bf16 && hd == HD; }

// Splits of the KV range per tile: enough to give the launch about two workgroups per CU, at least 8 steps
// (256 positions) each, at most 8, and only as many as the scratch holds.
int prefill_attention_splits(int n_tiles, int H, int max_pos, int window, size_t scratch_bytes) {
    const int span = window > 0 ? std::min(max_pos + 1, window + 128) : max_pos + 1;   // positions a tile walks
    int s = 512 / std::max(1, n_tiles * H);
    s = std::min(s, (span / KVB) / 8);
    s = std::min(s, 8);
    const size_t per_split = (size_t)n_tiles * 128 * H * (HD + 2) * sizeof(float);
    if (per_split) s = (int)std::min<size_t>(s, scratch_bytes / per_split);
    if (n_tiles * 128 > 65535) s = 1;       // the merge launch has one grid row per tile row slot
    return std::max(s, 1);
}

size_t prefill_attention_scratch_bytes() {
    // splits > 1 only while n_tiles * H * splits <= 512; 128 rows per tile
    return (size_t)512 * 128 * (HD + 2) * sizeof(float);
}

void launch_prefill_attention(const float *q, int q_stride, const uint16_t *pool, int Hkv, const int32_t *table,
                              int table_stride, const int32_t *tiles, int n_tiles, int H, int window, int max_pos,
                              float *out, void *scratch, size_t scratch_bytes, hipStream_t s, uint16_t *xs_hi,
                              uint16_t *xs_lo, int *f16_flag) {
    const float sl2 = 1.4426950408889634f / sqrtf((float)HD);
    const int ns = scratch ? prefill_attention_splits(n_tiles, H, max_pos, window, scratch_bytes) : 1;
    float *part_o = (float *)scratch;
    float *part_ml = part_o ? part_o + (size_t)n_tiles * 128 * H * ns * HD : nullptr;
    if (f16_flag)
        LD_LAUNCH(k_attn_prefill<true>, dim3(n_tiles, H, ns), dim3(256), 0, s, q, q_stride, pool, Hkv, table, table_stride,
                  (const int4 *)tiles, H, window, sl2, out, part_o, part_ml, xs_hi, xs_lo, f16_flag);
    else
        LD_LAUNCH(k_attn_prefill<false>, dim3(n_tiles, H, ns), dim3(256), 0, s, q, q_stride, pool, Hkv, table, table_stride,
                  (const int4 *)tiles, H, window, sl2, out, part_o, part_ml, xs_hi, xs_lo, f16_flag);
    if (ns > 1)
        LD_LAUNCH(k_attn_prefill_merge, dim3(H, n_tiles * 128), dim3(128), 0, s, (const int4 *)tiles, H, ns, part_o,
                  part_ml, out, xs_hi, xs_lo);
}

}  // namespace ld
