// Host side of libld: model registry, paged-KV block allocator, sequence state machine,
// step planner (which rows go through one pass), launch sequence, token hand-off to the callback.
#include "ld_internal.h"
#include "ld_batch.h"
#include "ld_gemm.h"
#include "ld_attn_prefill.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

namespace ld {

static thread_local std::string g_err;

void set_error(const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
}
void clear_error() { g_err.clear(); }

thread_local LaunchTimer *g_launch_timer = nullptr;

}  // namespace ld

using ld::fail;

struct ld_model {
    ld_model_config c;
    int f16_weights = -1;     // layer matrices within the fp16 range: -1 not looked at yet, 0 no, 1 yes
    const void *embed, *lm_head;
    const float *final_norm;
    std::vector<const float *> attn_norm, ffn_norm;
    std::vector<const void *> wqkv, wo, wgate_up, wdown;
    std::vector<const uint16_t *> h_qkv, h_wo, h_gate_up, h_down;   // fp16 images in the caller's buffer (ld_model_attach_f16_image), or empty
    size_t layer_matrix_elems() const { return ((size_t)nqkv() + nq()) * c.d_model + (size_t)3 * c.d_ffn * c.d_model; }
    int nq() const { return c.n_heads * c.head_dim; }
    int nkv() const { return c.n_kv_heads * c.head_dim; }
    int nqkv() const { return nq() + 2 * nkv(); }
    size_t elem() const { return c.dtype == LD_BF16 ? 2 : 4; }
    size_t block_elems() const { return (size_t)2 * c.n_kv_heads * c.kv_block * c.head_dim; }
};

namespace {

struct Seq {
    bool active = false, stopped = false, has_pending = false;
    bool swapped = false;          // keys/values live in a caller's host buffer; no block is held
    float temperature = 0.f;       // 0: greedy
    uint64_t seed = 0;
    int32_t pending = -1;
    int64_t n_cached = 0;
    int32_t n_mapped = 0;          // logical blocks 0..n_mapped-1 may be mapped (holes possible via ld_kv_map)
    int32_t first_block = 0;       // logical blocks below it were released by ld_kv_trim (attention band)
    int32_t dirty_lo = 0, dirty_hi = 0;  // table entries [lo, hi) not yet copied to the device
};

// Layout of the workspace: every region 256-byte aligned.
struct Workspace {
    int32_t *table, *meta, *out_tok;
    int32_t *flags;      // [0]: a value of this pass did not fit the fp16 form of the multi-row products
    float *x, *qkv, *attn, *act, *hn, *logits, *cos_sin;
    void *att_scratch, *lin_scratch, *lin_scratch2;   // lin_scratch2: second GEMM scratch area (bf16 models), same size
    size_t att_scratch_bytes, lin_scratch_bytes;
    uint16_t *b_xs;      // decode-batch layer: split operand image, split-K partial sums, norm statistics
    float *b_partial, *b_ss;
    size_t total;
};

Workspace plan_workspace(const ld_model &m, char *base, int max_tokens, int max_seqs, int max_blocks) {
    const ld_model_config &c = m.c;
    Workspace w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += ld::align_up(bytes, 256);
        return p;
    };
    const size_t T = max_tokens;
    w.table = (int32_t *)take((size_t)max_seqs * max_blocks * 4);
    // tok | pos | seq_slot | ctx_len | emit_row | prefill tiles (4 ints each) | sampling (seed 2, temperature, pos per emitting row)
    w.meta = (int32_t *)take((T * 9 + 2 + (size_t)max_seqs * 4) * 4);
    w.out_tok = (int32_t *)take((size_t)max_seqs * 4);
    w.flags = (int32_t *)take(64);
    w.x = (float *)take(T * c.d_model * 4);
    w.qkv = (float *)take(T * m.nqkv() * 4);
    w.attn = (float *)take(T * m.nq() * 4);
    w.act = (float *)take(T * c.d_ffn * 4);
    w.hn = (float *)take((size_t)max_seqs * c.d_model * 4);
    w.logits = (float *)take((size_t)max_seqs * c.vocab * 4);
    w.cos_sin = (float *)take(T * c.head_dim * 4);
    w.att_scratch_bytes = 0;   // the chunking depends on the row count: size for the worst one
    for (int t = 1; t <= max_tokens; t++)
        w.att_scratch_bytes = std::max(w.att_scratch_bytes,
                                       ldk_attention_scratch_bytes(t, c.n_heads, c.n_kv_heads, c.head_dim,
                                                                   max_blocks * c.kv_block, c.window));
    if (c.dtype == LD_BF16 && c.head_dim == 128 && max_tokens > 1)   // split partials of chunk-prefill attention
        w.att_scratch_bytes = std::max(w.att_scratch_bytes, ldk_prefill_attention_scratch_bytes());
    w.att_scratch = take(w.att_scratch_bytes);
    w.lin_scratch_bytes = 0;   // the split-K factor depends on the row count: size for the worst one
    for (int t = 2; t <= max_tokens; t++) {
        size_t b = ldk_linear_scratch_bytes(t, m.nqkv(), c.d_model, LDK_STORE);
        b = std::max(b, ldk_linear_scratch_bytes(t, c.d_model, m.nq(), LDK_ADD));
        b = std::max(b, ldk_linear_scratch_bytes(t, c.d_ffn, c.d_model, LDK_SWIGLU));
        b = std::max(b, ldk_linear_scratch_bytes(t, c.d_model, c.d_ffn, LDK_ADD));
        if (t <= max_seqs) b = std::max(b, ldk_linear_scratch_bytes(t, c.vocab, c.d_model, LDK_STORE));
        w.lin_scratch_bytes = std::max(w.lin_scratch_bytes, b);
    }
    w.lin_scratch = take(w.lin_scratch_bytes);
    w.lin_scratch2 = c.dtype == LD_BF16 && max_tokens >= 2 ? take(w.lin_scratch_bytes) : nullptr;
    {
        const int tb = std::min(max_tokens, 32);
        w.b_xs = (uint16_t *)take(ld::batch_layer_xs_bytes(tb, c.d_model, c.n_heads, c.head_dim, c.d_ffn));
        w.b_partial = (float *)take(ld::batch_layer_partial_bytes(tb, c.d_model, c.n_heads, c.n_kv_heads, c.head_dim, c.d_ffn));
        w.b_ss = (float *)take(ld::batch_layer_ss_bytes(tb, std::max(c.d_model, 1024)));
    }
    w.total = off;
    return w;
}

// One row of a pass: which token is fed for which sequence at which position.
struct Row { int32_t tok, pos, seq; };

}  // namespace

struct ld_kv {
    ld_model *m;
    char *pool;
    int64_t n_blocks;
    int32_t max_tokens, max_seqs, max_blocks;
    Workspace ws;
    std::vector<int32_t> free_stack;
    std::vector<int32_t> refs;   // sequences holding each block (prefix sharing); 0 = on the free stack
    std::vector<Seq> seqs;
    std::vector<int32_t> table;  // host copy [max_seqs][max_blocks], -1 = unmapped
    // pinned staging, created by the first pass.  Metadata and emitted tokens are double-buffered (two
    // slots) so that a step can be prepared while the previous one is still in flight; step_ev[slot] marks
    // the end of the pass that used the slot.
    int32_t *pin_meta = nullptr, *pin_out = nullptr, *pin_table = nullptr;
    hipEvent_t step_ev[2] = {nullptr, nullptr};
    size_t meta_ints() const { return (size_t)max_tokens * 9 + 2 + (size_t)max_seqs * 4; }
    // optional per-kernel timing
    bool prof_on = false;
    ld_profile prof{};
    struct Timer : ld::LaunchTimer {
        std::vector<hipEvent_t> ev;        // pairs (start, stop), reused from pass to pass
        std::vector<int> cat;              // category of pair i in the current pass
        int current = LD_PROF_OTHER;
        bool failed = false;
        void next(hipEvent_t *start, hipEvent_t *stop) override {
            const size_t i = cat.size();
            while (ev.size() < 2 * (i + 1)) {
                hipEvent_t e;
                if (hipEventCreate(&e) != hipSuccess) { failed = true; return; }
                ev.push_back(e);
            }
            *start = ev[2 * i];
            *stop = ev[2 * i + 1];
            cat.push_back(current);
        }
    } timer;
    // Set when a HIP call failed after a pass was planned (blocks reserved, copies or kernels possibly enqueued):
    // the cache's contents and the allocator no longer describe each other, every later step is refused.
    bool broken = false;
    int32_t *trow(int s) { return table.data() + (size_t)s * max_blocks; }
    const int32_t *trow(int s) const { return table.data() + (size_t)s * max_blocks; }
};

namespace {

// A failed HIP call leaves the cache unusable (see ld_kv::broken); validation errors leave it untouched.
ld_status seal(ld_kv *kv, ld_status rc) {
    if (rc == LD_E_HIP) kv->broken = true;
    return rc;
}
#define LD_REFUSE_BROKEN(kv, who)                                                                              \
    do {                                                                                                       \
        if ((kv)->broken) return fail(LD_E_STATE, who ": the cache is unusable after a failed HIP call; destroy it"); \
    } while (0)

Seq *get_seq(ld_kv *kv, ld_seq s) {
    if (!kv || s < 0 || s >= kv->max_seqs || !kv->seqs[s].active) return nullptr;
    return &kv->seqs[s];
}

int64_t blocks_for(const ld_kv *kv, int64_t tokens) {
    const int b = kv->m->c.kv_block;
    return (tokens + b - 1) / b;
}

int64_t count_missing(const ld_kv *kv, int s, int64_t need) {
    int64_t miss = 0;
    const int32_t *t = kv->trow(s);
    for (int64_t i = kv->seqs[s].first_block; i < need; i++) miss += t[i] < 0;
    return miss;
}

// Maps logical blocks first_block..need-1 (pops from the free stack).  The caller has checked availability.
void map_blocks(ld_kv *kv, int s, int64_t need) {
    int32_t *t = kv->trow(s);
    Seq &q = kv->seqs[s];
    for (int64_t i = q.first_block; i < need; i++) {
        if (t[i] >= 0) continue;
        t[i] = kv->free_stack.back();
        kv->free_stack.pop_back();
        kv->refs[t[i]] = 1;
        if (q.dirty_lo == q.dirty_hi) { q.dirty_lo = (int32_t)i; q.dirty_hi = (int32_t)i + 1; }
        else { q.dirty_lo = std::min<int32_t>(q.dirty_lo, i); q.dirty_hi = std::max<int32_t>(q.dirty_hi, i + 1); }
    }
    q.n_mapped = std::max<int32_t>(q.n_mapped, (int32_t)need);
}

// Drops every block a sequence holds, last logical block first; a block returns to the free stack when its
// last holder drops it.
void release_blocks(ld_kv *kv, int s) {
    int32_t *t = kv->trow(s);
    for (int i = kv->max_blocks - 1; i >= 0; i--)
        if (t[i] >= 0) {
            if (--kv->refs[t[i]] == 0) kv->free_stack.push_back(t[i]);
            t[i] = -1;
        }
    kv->seqs[s].n_mapped = 0;
    kv->seqs[s].dirty_lo = kv->seqs[s].dirty_hi = 0;
}

ld_status ensure_pinned(ld_kv *kv) {
    if (kv->pin_meta) return LD_OK;
    LD_HIP_TRY(hipHostMalloc((void **)&kv->pin_out, ((size_t)2 * kv->max_seqs + 2) * 4, hipHostMallocDefault));   // + one flag per slot
    LD_HIP_TRY(hipHostMalloc((void **)&kv->pin_table, (size_t)kv->max_seqs * kv->max_blocks * 4, hipHostMallocDefault));
    for (hipEvent_t &e : kv->step_ev) LD_HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    LD_HIP_TRY(hipHostMalloc((void **)&kv->pin_meta, 2 * kv->meta_ints() * 4, hipHostMallocDefault));
    return LD_OK;
}

// Enqueues one pass over `rows` (all rows' blocks are mapped) without waiting for it.  emit[i] = index of
// the row whose logits / greedy token are wanted, in callback order; once step_ev[slot] has passed,
// pin_out[slot * max_seqs + i] holds the tokens.  The last n_single rows are one-row segments (decode rows);
// the rows before them form multi-row prefill segments, each a run of consecutive rows of one sequence at
// consecutive positions.  (The one-row segments come last because the rows past the last full 256-row tile of a
// pass are the ones that the small-batch kernels take with both bf16 terms also when the rest of a long pass
// goes with one fp16 term: with whole chunks in front these are the decode rows, which emit.)  tok_from_prev: row t's input token is the token that the previous pass on this stream
// emitted for its row t (read on the device), not rows[t].tok.
ld_status enqueue_pass(ld_kv *kv, const std::vector<Row> &rows, int n_single, const std::vector<int32_t> &emit,
                       hipStream_t st, float *logits_out, int slot, bool tok_from_prev, int *ops, bool allow_f16 = false) {
    const ld_model &m = *kv->m;
    const ld_model_config &c = m.c;
    const int T = (int)rows.size(), R = (int)emit.size();
    ld_status rc = ensure_pinned(kv);
    if (rc) return rc;
    const Workspace &w = kv->ws;

    // metadata: tok | pos | seq_slot | ctx_len | emit_row, each T (emit: R) entries at stride T
    int32_t *pm = kv->pin_meta + (size_t)slot * kv->meta_ints();
    int max_ctx = 1;
    for (int t = 0; t < T; t++) {
        pm[t] = rows[t].tok;
        pm[T + t] = rows[t].pos;
        pm[2 * T + t] = rows[t].seq;
        pm[3 * T + t] = rows[t].pos + 1;
        max_ctx = std::max(max_ctx, rows[t].pos + 1);
    }
    for (int r = 0; r < R; r++) pm[4 * T + r] = emit[r];
    // prefill tiles: (first row, rows <= 128, first position, sequence) for the rows after the decode rows
    const bool mfma_attn = c.dtype == LD_BF16 && c.head_dim == 128;
    int n_tiles = 0;
    int32_t *pt = pm + 5 * T;
    if (mfma_attn) {
        for (int t = 0; t < T - n_single;) {
            int e = t + 1;
            while (e < T - n_single && e - t < 128 && rows[e].seq == rows[t].seq) e++;
            pt[4 * n_tiles] = t; pt[4 * n_tiles + 1] = e - t; pt[4 * n_tiles + 2] = rows[t].pos; pt[4 * n_tiles + 3] = rows[t].seq;
            n_tiles++;
            t = e;
        }
    }
    const int n_dec_rows = mfma_attn ? n_single : T;   // rows that go through the single-query kernel: [dec0, T)
    const int dec0 = T - n_dec_rows;
    int max_ctx_dec = 1;
    for (int t = dec0; t < T; t++) max_ctx_dec = std::max(max_ctx_dec, rows[t].pos + 1);
    // sampling parameters of the emitting rows, only when some sequence samples: seeds (8-byte aligned),
    // temperatures, position the emitted token will take
    bool sampling = false;
    for (int r = 0; r < R; r++) sampling = sampling || kv->seqs[rows[emit[r]].seq].temperature > 0.f;
    const int samp_off = (5 * T + 4 * n_tiles + 1) & ~1;
    int meta_ints = 5 * T + 4 * n_tiles;
    if (sampling) {
        uint64_t *ps = reinterpret_cast<uint64_t *>(pm + samp_off);
        float *ptemp = reinterpret_cast<float *>(pm + samp_off + 2 * R);
        int32_t *ppos = pm + samp_off + 3 * R;
        for (int r = 0; r < R; r++) {
            const Seq &sq = kv->seqs[rows[emit[r]].seq];
            ps[r] = sq.seed; ptemp[r] = sq.temperature; ppos[r] = rows[emit[r]].pos + 1;
        }
        meta_ints = samp_off + 4 * R;
    }
    LD_HIP_TRY(hipMemcpyAsync(w.meta, pm, (size_t)meta_ints * 4, hipMemcpyHostToDevice, st));
    // allow_f16: the multi-row products may take their rows rounded to fp16 (launch_gemm); flags[0] tells afterwards
    // whether a value did not fit, pin_out[2 * max_seqs + slot] carries it to the host
    int *f16_flag = allow_f16 ? w.flags : nullptr;
    if (f16_flag) LD_HIP_TRY(hipMemsetAsync(w.flags, 0, 4, st));
    const int32_t *d_tok = tok_from_prev ? w.out_tok : w.meta, *d_pos = w.meta + T, *d_slot = w.meta + 2 * T, *d_ctx = w.meta + 3 * T,
                  *d_emit = w.meta + 4 * T, *d_tiles = w.meta + 5 * T;

    // block-table rows that changed since the last pass
    for (int t = 0; t < T; t++) {
        Seq &q = kv->seqs[rows[t].seq];
        if (q.dirty_lo == q.dirty_hi) continue;
        const size_t o = (size_t)rows[t].seq * kv->max_blocks + q.dirty_lo;
        const size_t n = q.dirty_hi - q.dirty_lo;
        memcpy(kv->pin_table + o, kv->table.data() + o, n * 4);
        LD_HIP_TRY(hipMemcpyAsync(w.table + o, kv->pin_table + o, n * 4, hipMemcpyHostToDevice, st));
        q.dirty_lo = q.dirty_hi = 0;
    }

#define LD_TRY(call) do { ld_status s_ = (call); if (s_ != LD_OK) return s_; } while (0)
    // With profiling on, every kernel launched inside `call` gets an event pair attached to its dispatch.
    kv->timer.cat.clear();
    struct TimerScope {
        explicit TimerScope(ld::LaunchTimer *t) { ld::g_launch_timer = t; }
        ~TimerScope() { ld::g_launch_timer = nullptr; }
    } timer_scope(kv->prof_on ? &kv->timer : nullptr);
#define LD_TIMED(cat_, call)          \
    do {                              \
        kv->timer.current = cat_;     \
        ops[cat_]++;                  \
        LD_TRY(call);                 \
    } while (0)
    const int d = c.d_model, nq = m.nq(), nqkv = m.nqkv(), H = c.n_heads, Hkv = c.n_kv_heads, hd = c.head_dim;
    const size_t layer_bytes = (size_t)kv->n_blocks * m.block_elems() * m.elem();
    LD_TIMED(LD_PROF_OTHER, ldk_embed(m.embed, c.dtype, d_tok, T, d, w.x, st));
    LD_TIMED(LD_PROF_OTHER, ldk_rope_table(d_pos, T, hd, c.rope_base, w.cos_sin, st));
    // Decode batches of 2..32 rows on bf16 weights take the fused batch layer; everything else the
    // general per-step composition below.
    const bool batch_path = c.dtype == LD_BF16 && n_tiles == 0 && c.n_layers > 0 &&
                            ld::batch_layer_supported(T, d, H, Hkv, hd, c.d_ffn);
    auto timed_void = [](auto &&fn) { fn(); return LD_OK; };
    // Multi-row passes of bf16 models whose four layer matrices all run on the matrix-core GEMMs chain the
    // normalisations into the kernels that finish the residual GEMMs (LD_FUSE_NORM=0: tuning knob, separate passes).
    const char *fuse_env = getenv("LD_FUSE_NORM");
    const bool chained = !batch_path && c.dtype == LD_BF16 && T >= 2 && c.n_layers > 0 && w.lin_scratch2 &&
                         !(fuse_env && fuse_env[0] == '0') && d % 4 == 0 && ld::gemm_supported(T, nqkv, d) &&
                         ld::gemm_supported(T, d, nq) && ld::gemm_supported(T, c.d_ffn, d) && ld::gemm_supported(T, d, c.d_ffn);
    if (batch_path) {
        ld::BatchLayerArgs a{};
        a.T = T; a.d = d; a.H = H; a.Hkv = Hkv; a.hd = hd; a.ffn = c.d_ffn; a.eps = c.rms_eps;
        a.x = w.x; a.q = w.qkv; a.q_stride = nqkv; a.xs = w.b_xs; a.partial = w.b_partial; a.ss_part = w.b_ss;
        a.cos_sin = w.cos_sin; a.pos = d_pos; a.seq_slot = d_slot; a.table = w.table; a.table_stride = kv->max_blocks;
        LD_TIMED(LD_PROF_OTHER, timed_void([&] { ld::launch_batch_prepare(w.x, m.attn_norm[0], T, d, w.b_xs, w.b_ss, st); }));
        for (int l = 0; l < c.n_layers; l++) {
            void *pool_l = kv->pool + (size_t)l * layer_bytes;
            a.wqkv = (const uint16_t *)m.wqkv[l]; a.wo = (const uint16_t *)m.wo[l];
            a.wgate_up = (const uint16_t *)m.wgate_up[l]; a.wdown = (const uint16_t *)m.wdown[l];
            a.attn_norm = m.attn_norm[l]; a.ffn_norm = m.ffn_norm[l];
            a.next_norm = l + 1 < c.n_layers ? m.attn_norm[l + 1] : nullptr;
            a.pool = (uint16_t *)pool_l;
            LD_TIMED(LD_PROF_QKV, timed_void([&] { ld::launch_batch_qkv(a, st); }));
            LD_TIMED(LD_PROF_ATTENTION, ld::paged_attention_split(w.qkv, nqkv, pool_l, c.dtype, w.table, kv->max_blocks, d_slot,
                                                                  d_ctx, max_ctx_dec, T, H, Hkv, hd, c.window, w.b_xs,
                                                                  w.att_scratch, w.att_scratch_bytes, st));
            LD_TIMED(LD_PROF_WO, timed_void([&] { ld::launch_batch_wo(a, st); }));
            LD_TIMED(LD_PROF_GATE_UP, timed_void([&] { ld::launch_batch_gate_up(a, st); }));
            LD_TIMED(LD_PROF_DOWN, timed_void([&] { ld::launch_batch_down(a, st); }));
        }
        LD_HIP_TRY(hipGetLastError());
    } else if (chained) {
        // Two GEMM scratch areas: A holds the operands (and partial sums) of the output and down projections,
        // B those of the q-k-v and gate/up projections.  The kernel that finishes a residual GEMM (in A) writes
        // the normalised operand of the GEMM after it (into B), so no separate norm/split pass runs between them.
        uint16_t *A = (uint16_t *)w.lin_scratch, *B = (uint16_t *)w.lin_scratch2;
        auto mat = [](const void *p) { return (const uint16_t *)p; };
        auto img = [&](const std::vector<const uint16_t *> &v, int l) { return f16_flag && !v.empty() ? v[l] : nullptr; };
        for (int l = 0; l < c.n_layers; l++) {
            void *pool_l = kv->pool + (size_t)l * layer_bytes;
            // the kernel that finishes the q-k-v rows also rotates them and appends k, v to the cache
            const ld::RopeKvArgs rk{(const float2 *)w.cos_sin, d_pos, d_slot, w.table, kv->max_blocks, (uint16_t *)pool_l, H, Hkv, hd};
            const ld::GemmNext to_cache{nullptr, 0.f, nullptr, &rk};
            LD_TIMED(LD_PROF_QKV, timed_void([&] {
                if (l == 0) ld::launch_norm_split(w.x, m.attn_norm[0], c.rms_eps, T, d, B, st);
                ld::launch_gemm(mat(m.wqkv[l]), B, T, nqkv, d, ld::GEMM_STORE, w.qkv, st, &to_cache, f16_flag, img(m.h_qkv, l));
            }));
            // attention writes the output projection's operand (A) directly: the single-query rows, then the tiles' rows
            if (n_dec_rows)
                LD_TIMED(LD_PROF_ATTENTION, ld::paged_attention_split(w.qkv + (size_t)dec0 * nqkv, nqkv, pool_l, c.dtype, w.table,
                                                                      kv->max_blocks, d_slot + dec0, d_ctx + dec0, max_ctx_dec,
                                                                      n_dec_rows, H, Hkv, hd, c.window, A + (size_t)dec0 * nq,
                                                                      w.att_scratch, w.att_scratch_bytes, st, T));
            if (n_tiles)
                LD_TIMED(LD_PROF_ATTENTION, timed_void([&] {
                    ld::launch_prefill_attention(w.qkv, nqkv, (const uint16_t *)pool_l, Hkv, w.table, kv->max_blocks, d_tiles,
                                                 n_tiles, H, c.window, max_ctx - 1, w.attn, w.att_scratch,
                                                 w.att_scratch_bytes, st, A, A + (size_t)T * nq, f16_flag);
                }));
            const ld::GemmNext to_ffn{m.ffn_norm[l], c.rms_eps, B};
            const ld::GemmNext to_next{l + 1 < c.n_layers ? m.attn_norm[l + 1] : nullptr, c.rms_eps, B};
            LD_TIMED(LD_PROF_WO, timed_void([&] { ld::launch_gemm(mat(m.wo[l]), A, T, d, nq, ld::GEMM_ADD, w.x, st, &to_ffn, f16_flag, img(m.h_wo, l)); }));
            const ld::GemmNext to_down{nullptr, 0.f, A};      // the gated activation goes straight into the down projection's operand
            LD_TIMED(LD_PROF_GATE_UP, timed_void([&] { ld::launch_gemm(mat(m.wgate_up[l]), B, T, c.d_ffn, d, ld::GEMM_SWIGLU, w.act, st, &to_down, f16_flag, img(m.h_gate_up, l)); }));
            LD_TIMED(LD_PROF_DOWN, timed_void([&] {
                ld::launch_gemm(mat(m.wdown[l]), A, T, d, c.d_ffn, ld::GEMM_ADD, w.x, st, to_next.g ? &to_next : nullptr, f16_flag, img(m.h_down, l));
            }));
        }
        LD_HIP_TRY(hipGetLastError());
    } else
    for (int l = 0; l < c.n_layers; l++) {
        void *pool_l = kv->pool + (size_t)l * layer_bytes;
        auto img = [&](const std::vector<const uint16_t *> &v) { return f16_flag && !v.empty() ? v[l] : nullptr; };
        if (T == 1 || !f16_flag)
            LD_TIMED(LD_PROF_QKV, ldk_qkv_rope(m.wqkv[l], c.dtype, w.x, m.attn_norm[l], c.rms_eps, w.qkv, w.cos_sin, d_pos,
                                               d_slot, w.table, kv->max_blocks, pool_l, T, d, H, Hkv, hd, w.lin_scratch, w.lin_scratch_bytes, st));
        else {
            LD_TIMED(LD_PROF_QKV, ld::linear_pass(m.wqkv[l], c.dtype, w.x, m.attn_norm[l], c.rms_eps, T, nqkv, d, LDK_STORE, w.qkv,
                                                  w.lin_scratch, w.lin_scratch_bytes, st, f16_flag, img(m.h_qkv)));
            LD_TIMED(LD_PROF_QKV, ldk_rope_kv_write(w.qkv, w.cos_sin, d_pos, d_slot, w.table, kv->max_blocks, pool_l, c.dtype, T, H, Hkv, hd, st));
        }
        if (n_dec_rows)
            LD_TIMED(LD_PROF_ATTENTION, ldk_paged_attention(w.qkv + (size_t)dec0 * nqkv, nqkv, pool_l, c.dtype, w.table, kv->max_blocks,
                                                            d_slot + dec0, d_ctx + dec0, max_ctx_dec, n_dec_rows, H, Hkv, hd, c.window,
                                                            w.attn + (size_t)dec0 * nq, w.att_scratch, w.att_scratch_bytes, st));
        if (n_tiles)
            LD_TIMED(LD_PROF_ATTENTION, ldk_prefill_attention_f16(w.qkv, nqkv, pool_l, c.dtype, w.table, kv->max_blocks, d_tiles,
                                                                  n_tiles, H, Hkv, hd, c.window, max_ctx - 1, w.attn,
                                                                  w.att_scratch, w.att_scratch_bytes, f16_flag, st));
        LD_TIMED(LD_PROF_WO, ld::linear_pass(m.wo[l], c.dtype, w.attn, nullptr, 0.f, T, d, nq, LDK_ADD, w.x, w.lin_scratch, w.lin_scratch_bytes, st, f16_flag, img(m.h_wo)));
        LD_TIMED(LD_PROF_GATE_UP, ld::linear_pass(m.wgate_up[l], c.dtype, w.x, m.ffn_norm[l], c.rms_eps, T, c.d_ffn, d, LDK_SWIGLU, w.act, w.lin_scratch,
                                                    w.lin_scratch_bytes, st, f16_flag, img(m.h_gate_up)));
        LD_TIMED(LD_PROF_DOWN, ld::linear_pass(m.wdown[l], c.dtype, w.act, nullptr, 0.f, T, d, c.d_ffn, LDK_ADD, w.x, w.lin_scratch, w.lin_scratch_bytes, st, f16_flag, img(m.h_down)));
    }
    if (T == 1 && R == 1) {
        // one row, and it emits: the final norm rides in the LM head's own pass over x (as in every layer)
        LD_TIMED(LD_PROF_LM_HEAD, ldk_linear(m.lm_head, c.dtype, w.x, m.final_norm, c.rms_eps, 1, c.vocab, d, LDK_STORE, w.logits,
                                             w.lin_scratch, w.lin_scratch_bytes, st));
    } else {
        LD_TIMED(LD_PROF_OTHER, ldk_rmsnorm(w.x, m.final_norm, d_emit, R, d, c.rms_eps, w.hn, st));
        LD_TIMED(LD_PROF_LM_HEAD, ldk_linear(m.lm_head, c.dtype, w.hn, nullptr, 0.f, R, c.vocab, d, LDK_STORE, w.logits,
                                             w.lin_scratch, w.lin_scratch_bytes, st));
    }
    if (sampling)
        LD_TIMED(LD_PROF_OTHER, ldk_sample(w.logits, R, c.vocab, reinterpret_cast<const float *>(w.meta + samp_off + 2 * R),
                                           reinterpret_cast<const uint64_t *>(w.meta + samp_off), w.meta + samp_off + 3 * R,
                                           w.out_tok, st));
    else
        LD_TIMED(LD_PROF_OTHER, ldk_argmax(w.logits, R, c.vocab, w.out_tok, st));
#undef LD_TIMED
#undef LD_TRY
    if (R)
        LD_HIP_TRY(hipMemcpyAsync(kv->pin_out + (size_t)slot * kv->max_seqs, w.out_tok, (size_t)R * 4, hipMemcpyDeviceToHost, st));
    if (logits_out && R)
        LD_HIP_TRY(hipMemcpyAsync(logits_out, w.logits, (size_t)R * c.vocab * 4, hipMemcpyDeviceToHost, st));
    if (f16_flag)
        LD_HIP_TRY(hipMemcpyAsync(kv->pin_out + (size_t)2 * kv->max_seqs + slot, w.flags, 4, hipMemcpyDeviceToHost, st));
    LD_HIP_TRY(hipEventRecord(kv->step_ev[slot], st));
    return LD_OK;
}

// One pass, waited for: on return pin_out[i] holds the tokens.
// Rows of prefill chunks reach later tokens only through the cached keys and values, which are rounded to bf16
// anyway: in passes of at least LD_GEMM_F16_MIN_ROWS rows (512; LD_GEMM_F16=0 switches it off) the big-tile products
// take them rounded to fp16.  The first such pass looks once at the model's layer matrices (all within +-65504?);
// a pass in which an activation did not fit is repeated in the two-term form (the pass is a function of its
// inputs and of the cache before it; cache writes of the first attempt are overwritten).
static ld_status f16_weights_ok(ld_kv *kv, hipStream_t st, bool *ok) {
    ld_model &m = *kv->m;
    if (m.f16_weights < 0) {
        const ld_model_config &c = m.c;
        LD_HIP_TRY(hipMemsetAsync(kv->ws.flags + 1, 0, 4, st));
        for (int l = 0; l < c.n_layers; l++) {
            ld::launch_weight_range_check((const uint16_t *)m.wqkv[l], (int64_t)m.nqkv() * c.d_model, kv->ws.flags + 1, st);
            ld::launch_weight_range_check((const uint16_t *)m.wo[l], (int64_t)c.d_model * m.nq(), kv->ws.flags + 1, st);
            ld::launch_weight_range_check((const uint16_t *)m.wgate_up[l], (int64_t)2 * c.d_ffn * c.d_model, kv->ws.flags + 1, st);
            ld::launch_weight_range_check((const uint16_t *)m.wdown[l], (int64_t)c.d_model * c.d_ffn, kv->ws.flags + 1, st);
        }
        int32_t bad = 1;
        LD_HIP_TRY(hipMemcpyAsync(&bad, kv->ws.flags + 1, 4, hipMemcpyDeviceToHost, st));
        LD_HIP_TRY(hipStreamSynchronize(st));
        m.f16_weights = bad ? 0 : 1;
    }
    *ok = m.f16_weights == 1;
    return LD_OK;
}

ld_status run_pass(ld_kv *kv, const std::vector<Row> &rows, int n_single, const std::vector<int32_t> &emit,
                   hipStream_t st, float *logits_out) {
    int ops[LD_PROF_N] = {0};
    const int f16_on = ld::env_flag("LD_GEMM_F16", 1), f16_min_rows = ld::env_flag("LD_GEMM_F16_MIN_ROWS", 512);   // read per pass
    const ld_model_config &mc = kv->m->c;
    bool f16 = f16_on && mc.dtype == LD_BF16 && mc.n_layers > 0 && (int)rows.size() >= f16_min_rows && mc.d_model % 8 == 0 && mc.d_ffn % 8 == 0;
    if (f16) {
        ld_status rc0 = f16_weights_ok(kv, st, &f16);
        if (rc0) return rc0;
    }
    ld_status rc = enqueue_pass(kv, rows, n_single, emit, st, logits_out, 0, false, ops, f16);
    if (rc) return rc;
    LD_HIP_TRY(hipStreamSynchronize(st));
    if (f16 && kv->pin_out[(size_t)2 * kv->max_seqs]) {      // a value beyond the fp16 range: once more, both terms
        rc = enqueue_pass(kv, rows, n_single, emit, st, logits_out, 0, false, ops, false);
        if (rc) return rc;
        LD_HIP_TRY(hipStreamSynchronize(st));
    }
    if (kv->prof_on) {
        if (kv->timer.failed) return fail(LD_E_HIP, "profiling: hipEventCreate failed");
        for (size_t i = 0; i < kv->timer.cat.size(); i++) {
            float ms = 0.f;
            LD_HIP_TRY(hipEventElapsedTime(&ms, kv->timer.ev[2 * i], kv->timer.ev[2 * i + 1]));
            kv->prof.ms[kv->timer.cat[i]] += ms;
        }
        for (int k = 0; k < LD_PROF_N; k++) kv->prof.launches[k] += ops[k];
    }
    return LD_OK;
}

// One planned step: for each listed sequence a run of tokens to feed (pending first); every
// sequence emits one token from its last row.  Validates, reserves blocks, runs, commits state.
struct Feed { ld_seq seq; const int32_t *tokens; int32_t n; };

ld_status run_step(ld_kv *kv, const std::vector<Feed> &feeds, void *stream, ld_token_cb cb, void *user,
                   float *logits_out, const char *who) {
    const ld_model_config &c = kv->m->c;
    // --- validate, no state change
    if (kv->broken) { ld::set_error("%s: the cache is unusable after a failed HIP call; destroy it", who); return LD_E_STATE; }
    std::vector<char> seen(kv->max_seqs, 0);
    int64_t total_rows = 0, total_missing = 0;
    for (const Feed &f : feeds) {
        Seq *q = get_seq(kv, f.seq);
        if (!q) { ld::set_error("%s: bad sequence handle %d", who, f.seq); return LD_E_INVAL; }
        if (seen[f.seq]) { ld::set_error("%s: sequence %d listed twice", who, f.seq); return LD_E_INVAL; }
        seen[f.seq] = 1;
        if (q->stopped) { ld::set_error("%s: sequence %d was stopped by its callback", who, f.seq); return LD_E_STATE; }
        if (q->swapped) { ld::set_error("%s: sequence %d is swapped out", who, f.seq); return LD_E_STATE; }
        if (f.n < 0 || (f.n > 0 && !f.tokens)) { ld::set_error("%s: bad token array", who); return LD_E_INVAL; }
        const int64_t rows = f.n + (q->has_pending ? 1 : 0);
        if (rows == 0) { ld::set_error("%s: sequence %d has nothing to feed (no pending token)", who, f.seq); return LD_E_STATE; }
        for (int i = 0; i < f.n; i++)
            if (f.tokens[i] < 0 || f.tokens[i] >= c.vocab) { ld::set_error("%s: token id %d out of range", who, f.tokens[i]); return LD_E_RANGE; }
        const int64_t need = blocks_for(kv, q->n_cached + rows);
        if (need > kv->max_blocks) { ld::set_error("%s: sequence %d would exceed max_blocks_per_seq", who, f.seq); return LD_E_RANGE; }
        total_missing += count_missing(kv, f.seq, need);
        total_rows += rows;
    }
    if (total_rows > kv->max_tokens) { ld::set_error("%s: %lld rows exceed the workspace's max_tokens %d", who, (long long)total_rows, kv->max_tokens); return LD_E_RANGE; }
    if ((int64_t)feeds.size() > kv->max_seqs) return fail(LD_E_RANGE, "too many sequences in one step");
    if (total_missing > (int64_t)kv->free_stack.size()) { ld::set_error("%s: out of KV blocks (%lld needed, %zu free)", who, (long long)total_missing, kv->free_stack.size()); return LD_E_NOMEM; }

    // --- reserve blocks (in argument order, logical order within a sequence) and build rows:
    //     the multi-row prefill segments first, then the one-row feeds (decode rows)
    std::vector<Row> rows;
    std::vector<int32_t> emit(feeds.size());
    rows.reserve(total_rows);
    for (const Feed &f : feeds) {
        Seq &q = kv->seqs[f.seq];
        map_blocks(kv, f.seq, blocks_for(kv, q.n_cached + f.n + (q.has_pending ? 1 : 0)));
    }
    // A prefill feed whose row count is one more than a multiple of the 128-row attention tile (a
    // 256-token observation behind a pending token) sends its first row through the single-query
    // path, so that the rest fills whole tiles.
    auto peel_first = [&](int64_t n_rows) { return n_rows > 1 && n_rows % 128 == 1; };
    int n_single = 0;
    for (int pass = 1; pass >= 0; pass--)
        for (size_t i = 0; i < feeds.size(); i++) {
            const Feed &f = feeds[i];
            Seq &q = kv->seqs[f.seq];
            const int64_t n_rows = f.n + (q.has_pending ? 1 : 0);
            const int32_t pos0 = (int32_t)q.n_cached;
            auto tok_at = [&](int64_t r) { return q.has_pending ? (r == 0 ? q.pending : f.tokens[r - 1]) : f.tokens[r]; };
            if (pass == 0) {
                if (n_rows == 1 || peel_first(n_rows)) {
                    rows.push_back({tok_at(0), pos0, f.seq});
                    n_single++;
                    if (n_rows == 1) emit[i] = (int32_t)rows.size() - 1;
                }
            } else if (n_rows > 1) {
                for (int64_t r = peel_first(n_rows) ? 1 : 0; r < n_rows; r++) rows.push_back({tok_at(r), pos0 + (int32_t)r, f.seq});
                emit[i] = (int32_t)rows.size() - 1;
            }
        }
    ld_status rc = run_pass(kv, rows, n_single, emit, (hipStream_t)stream, logits_out);
    if (rc) return seal(kv, rc);

    // --- commit state, then hand the tokens over
    for (size_t i = 0; i < feeds.size(); i++) {
        Seq &q = kv->seqs[feeds[i].seq];
        q.n_cached += feeds[i].n + (q.has_pending ? 1 : 0);
        q.pending = kv->pin_out[i];
        q.has_pending = true;
    }
    if (cb)
        for (size_t i = 0; i < feeds.size(); i++) {
            Seq &q = kv->seqs[feeds[i].seq];
            const int r = cb(user, feeds[i].seq, q.pending, (int32_t)q.n_cached);
            if (r != LD_CB_CONTINUE && r != LD_CB_PAUSE) q.stopped = true;
        }
    return LD_OK;
}

}  // namespace

extern "C" {

const char *ld_last_error(void) { return ld::g_err.c_str(); }

ld_status ld_model_create(const ld_model_config *cfg, const ld_weights *w, ld_model **out) {
    if (!cfg || !w || !out) return fail(LD_E_INVAL, "ld_model_create: null argument");
    const ld_model_config &c = *cfg;
    if (c.n_layers < 0 || c.d_model <= 0 || c.n_heads <= 0 || c.n_kv_heads <= 0 || c.d_ffn <= 0 || c.vocab <= 0 ||
        c.max_chunk <= 0)
        return fail(LD_E_INVAL, "ld_model_create: non-positive dimension");
    if (c.head_dim != 64 && c.head_dim != 128) return fail(LD_E_INVAL, "ld_model_create: head_dim must be 64 or 128");
    if (c.kv_block != 16) return fail(LD_E_INVAL, "ld_model_create: kv_block must be 16");
    if (c.n_heads % c.n_kv_heads) return fail(LD_E_INVAL, "ld_model_create: n_heads must be a multiple of n_kv_heads");
    if (c.d_model % 8 || c.d_ffn % 8) return fail(LD_E_INVAL, "ld_model_create: d_model and d_ffn must be multiples of 8");
    if (c.dtype != LD_F32 && c.dtype != LD_BF16) return fail(LD_E_INVAL, "ld_model_create: bad dtype");
    if (!(c.rms_eps > 0.f) || !(c.rope_base > 1.f)) return fail(LD_E_INVAL, "ld_model_create: bad rms_eps / rope_base");
    if (c.window < 0) return fail(LD_E_INVAL, "ld_model_create: negative attention window");
    if (!w->embed || !w->lm_head || !w->final_norm) return fail(LD_E_INVAL, "ld_model_create: null weight pointer");
    if (c.n_layers > 0 && (!w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm || !w->wgate_up || !w->wdown))
        return fail(LD_E_INVAL, "ld_model_create: null per-layer table");
    for (int l = 0; l < c.n_layers; l++)
        if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->wgate_up[l] || !w->wdown[l])
            return fail(LD_E_INVAL, "ld_model_create: null per-layer weight pointer");
    ld_model *m = new ld_model();
    m->c = c;
    m->embed = w->embed; m->lm_head = w->lm_head; m->final_norm = w->final_norm;
    for (int l = 0; l < c.n_layers; l++) {
        m->attn_norm.push_back(w->attn_norm[l]); m->ffn_norm.push_back(w->ffn_norm[l]);
        m->wqkv.push_back(w->wqkv[l]); m->wo.push_back(w->wo[l]);
        m->wgate_up.push_back(w->wgate_up[l]); m->wdown.push_back(w->wdown[l]);
    }
    *out = m;
    return LD_OK;
}

void ld_model_destroy(ld_model *m) { delete m; }

size_t ld_model_f16_image_bytes(const ld_model *m) {
    if (!m || m->c.dtype != LD_BF16) return 0;
    return (size_t)m->c.n_layers * m->layer_matrix_elems() * 2;
}

ld_status ld_model_attach_f16_image(ld_model *m, void *buf, size_t bytes, void *stream, int32_t *in_range) {
    if (!m) return fail(LD_E_INVAL, "ld_model_attach_f16_image: null model");
    m->h_qkv.clear(); m->h_wo.clear(); m->h_gate_up.clear(); m->h_down.clear();
    if (in_range) *in_range = 0;
    if (!buf) return LD_OK;                                     // detached
    const ld_model_config &c = m->c;
    const size_t need = ld_model_f16_image_bytes(m);
    if (need == 0) return fail(LD_E_INVAL, "ld_model_attach_f16_image: the model has no bf16 layer matrices");
    if (bytes < need + 256 || ((uintptr_t)buf & 15)) {
        ld::set_error("ld_model_attach_f16_image: %zu bytes given, %zu + 256 needed, 16-byte aligned", bytes, need);
        return LD_E_INVAL;
    }
    // the flag lives in the buffer's last 256 bytes, so that no workspace is needed here
    hipStream_t st = (hipStream_t)stream;
    uint16_t *p = (uint16_t *)buf;
    int *flag = (int *)((char *)buf + need);
    LD_HIP_TRY(hipMemsetAsync(flag, 0, 4, st));
    std::vector<const uint16_t *> q, o, g, dn;
    auto conv = [&](const void *W, size_t n, std::vector<const uint16_t *> &v) {
        ld::launch_weight_to_f16((const uint16_t *)W, (int64_t)n, p, flag, st);
        v.push_back(p);
        p += n;
    };
    for (int l = 0; l < c.n_layers; l++) {
        conv(m->wqkv[l], (size_t)m->nqkv() * c.d_model, q);
        conv(m->wo[l], (size_t)c.d_model * m->nq(), o);
        conv(m->wgate_up[l], (size_t)2 * c.d_ffn * c.d_model, g);
        conv(m->wdown[l], (size_t)c.d_model * c.d_ffn, dn);
    }
    LD_HIP_TRY(hipGetLastError());
    int32_t bad = 1;
    LD_HIP_TRY(hipMemcpyAsync(&bad, flag, 4, hipMemcpyDeviceToHost, st));
    LD_HIP_TRY(hipStreamSynchronize(st));
    m->f16_weights = bad ? 0 : 1;
    if (!bad) { m->h_qkv = q; m->h_wo = o; m->h_gate_up = g; m->h_down = dn; }
    if (in_range) *in_range = bad ? 0 : 1;
    return LD_OK;
}

size_t ld_kv_bytes(const ld_model *m, int64_t n_blocks) {
    if (!m || n_blocks <= 0) return 0;
    return (size_t)m->c.n_layers * n_blocks * m->block_elems() * m->elem();
}

size_t ld_workspace_bytes(const ld_model *m, int32_t max_tokens, int32_t max_seqs, int32_t max_blocks_per_seq) {
    if (!m || max_tokens <= 0 || max_seqs <= 0 || max_blocks_per_seq <= 0) return 0;
    return plan_workspace(*m, nullptr, max_tokens, max_seqs, max_blocks_per_seq).total;
}

ld_status ld_kv_create(ld_model *m, void *pool, int64_t n_blocks, void *ws, size_t ws_bytes, int32_t max_tokens,
                       int32_t max_seqs, int32_t max_blocks_per_seq, ld_kv **out) {
    if (!m || !out || n_blocks <= 0 || max_tokens <= 0 || max_seqs <= 0 || max_blocks_per_seq <= 0)
        return fail(LD_E_INVAL, "ld_kv_create: bad argument");
    if (!pool || !ws) return fail(LD_E_INVAL, "ld_kv_create: null pool or workspace");
    if (n_blocks > INT32_MAX) return fail(LD_E_RANGE, "ld_kv_create: too many blocks");
    if (((uintptr_t)pool | (uintptr_t)ws) & 255) return fail(LD_E_INVAL, "ld_kv_create: pool and workspace must be 256-byte aligned");
    const size_t need = ld_workspace_bytes(m, max_tokens, max_seqs, max_blocks_per_seq);
    if (ws_bytes < need) { ld::set_error("ld_kv_create: workspace of %zu bytes, %zu needed", ws_bytes, need); return LD_E_INVAL; }
    ld_kv *kv = new ld_kv();
    kv->m = m; kv->pool = (char *)pool; kv->n_blocks = n_blocks;
    kv->max_tokens = max_tokens; kv->max_seqs = max_seqs; kv->max_blocks = max_blocks_per_seq;
    kv->ws = plan_workspace(*m, (char *)ws, max_tokens, max_seqs, max_blocks_per_seq);
    kv->free_stack.resize(n_blocks);
    kv->refs.assign(n_blocks, 0);
    for (int64_t i = 0; i < n_blocks; i++) kv->free_stack[i] = (int32_t)(n_blocks - 1 - i);
    kv->seqs.resize(max_seqs);
    kv->table.assign((size_t)max_seqs * max_blocks_per_seq, -1);
    *out = kv;
    return LD_OK;
}

void ld_kv_destroy(ld_kv *kv) {
    if (!kv) return;
    if (kv->pin_meta) (void)hipHostFree(kv->pin_meta);
    if (kv->pin_out) (void)hipHostFree(kv->pin_out);
    if (kv->pin_table) (void)hipHostFree(kv->pin_table);
    for (hipEvent_t e : kv->step_ev)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : kv->timer.ev) (void)hipEventDestroy(e);
    delete kv;
}

ld_status ld_kv_alloc(ld_kv *kv, int64_t reserve_tokens, ld_seq *out) {
    if (!kv || !out || reserve_tokens < 0) return fail(LD_E_INVAL, "ld_kv_alloc: bad argument");
    int s = 0;
    while (s < kv->max_seqs && kv->seqs[s].active) s++;
    if (s == kv->max_seqs) return fail(LD_E_NOMEM, "ld_kv_alloc: no free sequence handle");
    const int64_t need = blocks_for(kv, reserve_tokens);
    if (need > kv->max_blocks) return fail(LD_E_RANGE, "ld_kv_alloc: reservation exceeds max_blocks_per_seq");
    if (need > (int64_t)kv->free_stack.size()) return fail(LD_E_NOMEM, "ld_kv_alloc: out of KV blocks");
    kv->seqs[s] = Seq();
    kv->seqs[s].active = true;
    map_blocks(kv, s, need);
    *out = s;
    return LD_OK;
}

ld_status ld_kv_map(ld_kv *kv, ld_seq seq, int32_t logical, int32_t physical) {
    Seq *q = get_seq(kv, seq);
    if (!q || logical < 0 || logical >= kv->max_blocks) return fail(LD_E_INVAL, "ld_kv_map: bad argument");
    if (q->swapped) return fail(LD_E_STATE, "ld_kv_map: sequence is swapped out");
    int32_t *t = kv->trow(seq);
    if (t[logical] >= 0) return fail(LD_E_STATE, "ld_kv_map: logical block already mapped");
    auto it = std::find(kv->free_stack.begin(), kv->free_stack.end(), physical);
    if (it == kv->free_stack.end()) return fail(LD_E_NOMEM, "ld_kv_map: physical block is not free");
    kv->free_stack.erase(it);
    kv->refs[physical] = 1;
    t[logical] = physical;
    if (q->dirty_lo == q->dirty_hi) { q->dirty_lo = logical; q->dirty_hi = logical + 1; }
    else { q->dirty_lo = std::min(q->dirty_lo, logical); q->dirty_hi = std::max(q->dirty_hi, logical + 1); }
    q->n_mapped = std::max(q->n_mapped, logical + 1);
    return LD_OK;
}

ld_status ld_kv_free(ld_kv *kv, ld_seq seq) {
    Seq *q = get_seq(kv, seq);
    if (!q) return fail(LD_E_INVAL, "ld_kv_free: bad sequence handle");
    release_blocks(kv, seq);
    *q = Seq();
    return LD_OK;
}

ld_status ld_kv_block_table(const ld_kv *kv, ld_seq seq, int32_t *out, int32_t cap, int32_t *n) {
    const Seq *q = get_seq(const_cast<ld_kv *>(kv), seq);
    if (!q || !out || !n) return fail(LD_E_INVAL, "ld_kv_block_table: bad argument");
    if (cap < q->n_mapped) return fail(LD_E_RANGE, "ld_kv_block_table: output too small");
    memcpy(out, kv->trow(seq), (size_t)q->n_mapped * 4);
    *n = q->n_mapped;
    return LD_OK;
}

int64_t ld_kv_len(const ld_kv *kv, ld_seq seq) {
    const Seq *q = get_seq(const_cast<ld_kv *>(kv), seq);
    return q ? q->n_cached : -1;
}

int64_t ld_kv_free_blocks(const ld_kv *kv) { return kv ? (int64_t)kv->free_stack.size() : -1; }

// Bytes of one block over all layers is n_layers pieces of block_bytes, one per layer slice of the pool.
static size_t block_bytes(const ld_kv *kv) {
    const ld_model_config &c = kv->m->c;
    return (size_t)2 * c.n_kv_heads * c.kv_block * c.head_dim * (c.dtype == LD_BF16 ? 2 : 4);
}

size_t ld_kv_swap_bytes(const ld_kv *kv, ld_seq seq) {
    const Seq *q = get_seq(const_cast<ld_kv *>(kv), seq);
    if (!q) return 0;
    return (size_t)blocks_for(kv, q->n_cached) * kv->m->c.n_layers * block_bytes(kv);
}

ld_status ld_kv_swap_out(ld_kv *kv, ld_seq seq, void *host_buf, size_t bytes, void *stream) {
    Seq *q = get_seq(kv, seq);
    if (!q || (!host_buf && q->n_cached > 0)) return fail(LD_E_INVAL, "ld_kv_swap_out: bad argument");
    LD_REFUSE_BROKEN(kv, "ld_kv_swap_out");
    if (q->swapped) return fail(LD_E_STATE, "ld_kv_swap_out: sequence is already swapped out");
    if (bytes < ld_kv_swap_bytes(kv, seq)) return fail(LD_E_RANGE, "ld_kv_swap_out: host buffer too small");
    const size_t bb = block_bytes(kv);
    const int L = kv->m->c.n_layers;
    const int64_t nb = blocks_for(kv, q->n_cached);
    int32_t *t = kv->trow(seq);
    // one strided copy per logical block: its n_layers pieces lie one layer slice apart in the pool
    for (int64_t j = q->first_block; j < nb; j++)      // released blocks: their part of the buffer is not written
        if (hipMemcpy2DAsync((char *)host_buf + (size_t)j * L * bb, bb, kv->pool + (size_t)t[j] * bb,
                             (size_t)kv->n_blocks * bb, bb, L, hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess) {
            kv->broken = true;      // some blocks' copies may be on their way: the sequence is neither in nor out
            return fail(LD_E_HIP, "ld_kv_swap_out: hipMemcpy2DAsync failed");
        }
    release_blocks(kv, seq);
    q->swapped = true;
    return LD_OK;
}

ld_status ld_kv_swap_in(ld_kv *kv, ld_seq seq, const void *host_buf, size_t bytes, void *stream) {
    Seq *q = get_seq(kv, seq);
    if (!q || (!host_buf && q->n_cached > 0)) return fail(LD_E_INVAL, "ld_kv_swap_in: bad argument");
    LD_REFUSE_BROKEN(kv, "ld_kv_swap_in");
    if (!q->swapped) return fail(LD_E_STATE, "ld_kv_swap_in: sequence is not swapped out");
    if (bytes < ld_kv_swap_bytes(kv, seq)) return fail(LD_E_RANGE, "ld_kv_swap_in: host buffer too small");
    const int64_t nb = blocks_for(kv, q->n_cached);
    if (count_missing(kv, seq, nb) > (int64_t)kv->free_stack.size()) return fail(LD_E_NOMEM, "ld_kv_swap_in: out of KV blocks");
    map_blocks(kv, seq, nb);
    const size_t bb = block_bytes(kv);
    const int L = kv->m->c.n_layers;
    const int32_t *t = kv->trow(seq);
    for (int64_t j = q->first_block; j < nb; j++)
        if (hipMemcpy2DAsync(kv->pool + (size_t)t[j] * bb, (size_t)kv->n_blocks * bb,
                             (const char *)host_buf + (size_t)j * L * bb, bb, bb, L, hipMemcpyHostToDevice,
                             (hipStream_t)stream) != hipSuccess) {
            kv->broken = true;      // blocks are taken and partly filled
            return fail(LD_E_HIP, "ld_kv_swap_in: hipMemcpy2DAsync failed");
        }
    q->swapped = false;
    return LD_OK;
}

ld_status ld_kv_trim(ld_kv *kv, ld_seq seq, int32_t *released) {
    Seq *q = get_seq(kv, seq);
    if (!q || !released) return fail(LD_E_INVAL, "ld_kv_trim: bad argument");
    if (q->swapped) return fail(LD_E_STATE, "ld_kv_trim: sequence is swapped out");
    *released = 0;
    const ld_model_config &c = kv->m->c;
    const int64_t low = q->n_cached - c.window + 1;      // lowest position the next query (at n_cached) sees
    if (c.window <= 0 || low <= 0) return LD_OK;
    const int64_t keep_from = low / c.kv_block;
    int32_t *t = kv->trow(seq);
    for (int64_t i = q->first_block; i < keep_from; i++)
        if (t[i] >= 0) {
            if (--kv->refs[t[i]] == 0) kv->free_stack.push_back(t[i]);
            t[i] = -1;
            ++*released;
        }
    if (keep_from > q->first_block) q->first_block = (int32_t)keep_from;
    return LD_OK;
}

ld_status ld_kv_set_sampling(ld_kv *kv, ld_seq seq, float temperature, uint64_t seed) {
    Seq *q = get_seq(kv, seq);
    if (!q || !(temperature >= 0.f)) return fail(LD_E_INVAL, "ld_kv_set_sampling: bad argument");
    q->temperature = temperature;
    q->seed = seed;
    return LD_OK;
}

ld_status ld_kv_fork(ld_kv *kv, ld_seq parent, int64_t n_tokens, void *stream, ld_seq *out) {
    Seq *p = get_seq(kv, parent);
    if (!p || !out || n_tokens < 0 || n_tokens > p->n_cached) return fail(LD_E_INVAL, "ld_kv_fork: bad argument");
    LD_REFUSE_BROKEN(kv, "ld_kv_fork");
    if (p->swapped) return fail(LD_E_STATE, "ld_kv_fork: parent is swapped out");
    int s = 0;
    while (s < kv->max_seqs && kv->seqs[s].active) s++;
    if (s == kv->max_seqs) return fail(LD_E_NOMEM, "ld_kv_fork: no free sequence handle");
    const int bs = kv->m->c.kv_block;
    const int64_t full = n_tokens / bs, tail = n_tokens % bs;
    if (p->first_block > 0) {   // the child's next query must not need a block the parent has released
        const int64_t low = std::max<int64_t>(n_tokens - kv->m->c.window + 1, 0);
        if (low / bs < p->first_block) return fail(LD_E_STATE, "ld_kv_fork: the prefix reaches below the blocks the parent still holds");
    }
    if (tail && kv->free_stack.empty()) return fail(LD_E_NOMEM, "ld_kv_fork: no block for the copied tail");
    const int32_t *pt = kv->trow(parent);
    int32_t *t = kv->trow(s);
    Seq &q = kv->seqs[s];
    q = Seq();
    q.active = true;
    q.n_cached = n_tokens;
    const int32_t fb = p->first_block;
    q.first_block = fb;
    for (int64_t j = fb; j < full; j++) { t[j] = pt[j]; kv->refs[pt[j]]++; }
    q.n_mapped = (int32_t)full;
    if (full > fb) { q.dirty_lo = fb; q.dirty_hi = (int32_t)full; }
    if (tail) {
        map_blocks(kv, s, full + 1);    // pops one block for logical block `full`
        const size_t bb = block_bytes(kv);
        if (hipMemcpy2DAsync(kv->pool + (size_t)t[full] * bb, (size_t)kv->n_blocks * bb,
                             kv->pool + (size_t)pt[full] * bb, (size_t)kv->n_blocks * bb, bb, kv->m->c.n_layers,
                             hipMemcpyDeviceToDevice, (hipStream_t)stream) != hipSuccess) {
            kv->broken = true;      // the child exists and holds blocks, its copied tail does not
            return fail(LD_E_HIP, "ld_kv_fork: hipMemcpy2DAsync failed");
        }
    }
    *out = s;
    return LD_OK;
}

ld_status ld_kv_assume(ld_kv *kv, ld_seq seq, int64_t n_tokens, int32_t pending) {
    Seq *q = get_seq(kv, seq);
    if (!q || n_tokens < 0) return fail(LD_E_INVAL, "ld_kv_assume: bad argument");
    if (q->swapped) return fail(LD_E_STATE, "ld_kv_assume: sequence is swapped out");
    if (pending >= kv->m->c.vocab) return fail(LD_E_RANGE, "ld_kv_assume: pending token out of range");
    const int64_t need = blocks_for(kv, q->n_cached + n_tokens);
    if (need > kv->max_blocks) return fail(LD_E_RANGE, "ld_kv_assume: exceeds max_blocks_per_seq");
    if (count_missing(kv, seq, need) > (int64_t)kv->free_stack.size()) return fail(LD_E_NOMEM, "ld_kv_assume: out of KV blocks");
    map_blocks(kv, seq, need);
    q->n_cached += n_tokens;
    if (pending >= 0) { q->pending = pending; q->has_pending = true; }
    return LD_OK;
}

ld_status ld_kv_profile(ld_kv *kv, int32_t enable) {
    if (!kv) return fail(LD_E_INVAL, "ld_kv_profile: null kv");
    kv->prof_on = enable != 0;
    if (enable) kv->prof = ld_profile{};
    return LD_OK;
}

ld_status ld_kv_profile_read(const ld_kv *kv, ld_profile *out) {
    if (!kv || !out) return fail(LD_E_INVAL, "ld_kv_profile_read: null argument");
    *out = kv->prof;
    return LD_OK;
}

ld_status ld_prefill(ld_kv *kv, ld_seq seq, const int32_t *tokens, int32_t n, void *stream, ld_token_cb cb,
                     void *user, float *logits_out) {
    if (!kv) return fail(LD_E_INVAL, "ld_prefill: null kv");
    LD_REFUSE_BROKEN(kv, "ld_prefill");
    Seq *q = get_seq(kv, seq);
    if (!q) return fail(LD_E_INVAL, "ld_prefill: bad sequence handle");
    if (q->stopped) return fail(LD_E_STATE, "ld_prefill: sequence was stopped by its callback");
    if (q->swapped) return fail(LD_E_STATE, "ld_prefill: sequence is swapped out");
    if (n < 0 || (n > 0 && !tokens)) return fail(LD_E_INVAL, "ld_prefill: bad token array");
    const ld_model_config &c = kv->m->c;
    const int chunk = std::min(c.max_chunk, kv->max_tokens);
    const int64_t total = (int64_t)n + (q->has_pending ? 1 : 0);
    if (total == 0) return fail(LD_E_INVAL, "ld_prefill: nothing to feed");
    for (int i = 0; i < n; i++)
        if (tokens[i] < 0 || tokens[i] >= c.vocab) return fail(LD_E_RANGE, "ld_prefill: token id out of range");
    // reserve every block of the whole call first, so that a shortage leaves the state untouched
    const int64_t need = blocks_for(kv, q->n_cached + total);
    if (need > kv->max_blocks) return fail(LD_E_RANGE, "ld_prefill: sequence would exceed max_blocks_per_seq");
    if (count_missing(kv, seq, need) > (int64_t)kv->free_stack.size()) return fail(LD_E_NOMEM, "ld_prefill: out of KV blocks");
    map_blocks(kv, seq, need);

    // all chunks but the last: rows only, nothing emitted
    std::vector<Row> rows;
    int64_t fed = 0;      // rows fed so far (of `total`)
    int32_t consumed = 0; // entries of tokens[] consumed
    while (total - fed > chunk) {
        rows.clear();
        int32_t pos = (int32_t)q->n_cached;
        if (q->has_pending) rows.push_back({q->pending, pos++, seq});
        while ((int)rows.size() < chunk) rows.push_back({tokens[consumed++], pos++, seq});
        std::vector<int32_t> emit;  // none
        ld_status rc = run_pass(kv, rows, 0, emit, (hipStream_t)stream, nullptr);
        if (rc) return seal(kv, rc);
        q->n_cached += rows.size();
        q->has_pending = false; q->pending = -1;
        fed += rows.size();
    }
    std::vector<Feed> last{{seq, tokens + consumed, n - consumed}};
    return run_step(kv, last, stream, cb, user, logits_out, "ld_prefill");
}

ld_status ld_decode_step(ld_kv *kv, const ld_seq *seqs, int32_t n_seqs, void *stream, ld_token_cb cb, void *user,
                         float *logits_out) {
    if (!kv || !seqs || n_seqs <= 0) return fail(LD_E_INVAL, "ld_decode_step: bad argument");
    std::vector<Feed> feeds;
    for (int i = 0; i < n_seqs; i++) {
        Seq *q = get_seq(kv, seqs[i]);
        if (q && !q->has_pending) { ld::set_error("ld_decode_step: sequence %d has no pending token", seqs[i]); return LD_E_STATE; }
        feeds.push_back({seqs[i], nullptr, 0});
    }
    return run_step(kv, feeds, stream, cb, user, logits_out, "ld_decode_step");
}

ld_status ld_decode_run(ld_kv *kv, const ld_seq *seqs, int32_t n_seqs, int32_t max_steps, void *stream, ld_token_cb cb,
                        void *user, int32_t *steps_done) {
    if (steps_done) *steps_done = 0;
    if (!kv || !seqs || n_seqs <= 0 || max_steps < 0) return fail(LD_E_INVAL, "ld_decode_run: bad argument");
    LD_REFUSE_BROKEN(kv, "ld_decode_run");
    if (n_seqs > kv->max_seqs || n_seqs > kv->max_tokens) return fail(LD_E_RANGE, "ld_decode_run: too many sequences in one step");
    std::vector<char> seen(kv->max_seqs, 0);
    for (int i = 0; i < n_seqs; i++) {
        Seq *q = get_seq(kv, seqs[i]);
        if (!q) { ld::set_error("ld_decode_run: bad sequence handle %d", seqs[i]); return LD_E_INVAL; }
        if (seen[seqs[i]]) { ld::set_error("ld_decode_run: sequence %d listed twice", seqs[i]); return LD_E_INVAL; }
        seen[seqs[i]] = 1;
        if (q->stopped || q->swapped || !q->has_pending) {
            ld::set_error("ld_decode_run: sequence %d is stopped, swapped out or has no pending token", seqs[i]);
            return LD_E_STATE;
        }
    }
    if (max_steps == 0) return LD_OK;
    hipStream_t st = (hipStream_t)stream;
    ld_status rc = LD_OK;

    // Step k is prepared while step k-1 runs: its rows sit one position further, its blocks are reserved
    // now, and its input tokens are read on the device from what step k-1 emits.  Every reservation is
    // recorded so that a step that turns out to be unwanted can be taken back exactly.
    struct Undo { int32_t seq, logical, n_mapped_before; };
    std::vector<Undo> undo[2];
    std::vector<Row> rows(n_seqs);
    std::vector<int32_t> emit(n_seqs);
    for (int i = 0; i < n_seqs; i++) emit[i] = i;
    int enq = 0, done = 0;
    bool end = false;            // a callback ended the run, or the next step cannot be prepared
    int ops[LD_PROF_N] = {0};
    auto prepare = [&](int k) -> ld_status {
        const int ahead = k - done;
        int64_t missing = 0;
        for (int i = 0; i < n_seqs; i++) {
            const Seq &q = kv->seqs[seqs[i]];
            const int64_t need = blocks_for(kv, q.n_cached + ahead + 1);
            if (need > kv->max_blocks) { ld::set_error("ld_decode_run: sequence %d would exceed max_blocks_per_seq", seqs[i]); return LD_E_RANGE; }
            missing += count_missing(kv, seqs[i], need);
        }
        if (missing > (int64_t)kv->free_stack.size()) {
            ld::set_error("ld_decode_run: out of KV blocks (%lld needed, %zu free)", (long long)missing, kv->free_stack.size());
            return LD_E_NOMEM;
        }
        std::vector<Undo> &u = undo[k & 1];
        u.clear();
        for (int i = 0; i < n_seqs; i++) {
            Seq &q = kv->seqs[seqs[i]];
            const int64_t need = blocks_for(kv, q.n_cached + ahead + 1);
            const int32_t *t = kv->trow(seqs[i]);
            for (int64_t j = q.first_block; j < need; j++)
                if (t[j] < 0) u.push_back({seqs[i], (int32_t)j, q.n_mapped});
            map_blocks(kv, seqs[i], need);
            rows[i] = {q.pending, (int32_t)(q.n_cached + ahead), seqs[i]};
        }
        return enqueue_pass(kv, rows, n_seqs, emit, st, nullptr, k & 1, ahead > 0, ops);
    };
    // With per-kernel timing on, the events of a pass are read after it: no step is prepared ahead.
    const int depth = kv->prof_on ? 1 : 2;
    rc = prepare(0);
    if (rc) return seal(kv, rc);
    enq = 1;
    for (;;) {
        if (!end && enq < max_steps && enq - done < depth) {
            rc = prepare(enq);
            if (rc == LD_OK) enq++;
            else if (rc == LD_E_NOMEM || rc == LD_E_RANGE) end = true;   // the steps in flight are still delivered
            else { (void)hipStreamSynchronize(st); return seal(kv, rc); }
        }
        if (done == enq) break;
        if (hipEventSynchronize(kv->step_ev[done & 1]) != hipSuccess) {
            kv->broken = true;
            return fail(LD_E_HIP, "ld_decode_run: waiting for a step failed");
        }
        if (kv->prof_on) {
            if (kv->timer.failed) return fail(LD_E_HIP, "profiling: hipEventCreate failed");
            for (size_t i = 0; i < kv->timer.cat.size(); i++) {
                float ms = 0.f;
                LD_HIP_TRY(hipEventElapsedTime(&ms, kv->timer.ev[2 * i], kv->timer.ev[2 * i + 1]));
                kv->prof.ms[kv->timer.cat[i]] += ms;
            }
            for (int k = 0; k < LD_PROF_N; k++) { kv->prof.launches[k] += ops[k]; ops[k] = 0; }
        }
        const int32_t *out = kv->pin_out + (size_t)(done & 1) * kv->max_seqs;
        for (int i = 0; i < n_seqs; i++) {
            Seq &q = kv->seqs[seqs[i]];
            q.n_cached += 1;
            q.pending = out[i];
        }
        done++;
        if (steps_done) *steps_done = done;
        if (cb)
            for (int i = 0; i < n_seqs; i++) {
                Seq &q = kv->seqs[seqs[i]];
                const int r = cb(user, seqs[i], q.pending, (int32_t)q.n_cached);
                if (r == LD_CB_CONTINUE) continue;
                end = true;
                if (r != LD_CB_PAUSE) q.stopped = true;
            }
        if (end && enq > done) {
            // The step prepared ahead is not wanted: return its blocks, last taken first, so that the allocator
            // is where `done` single steps would have left it.  The step still executes; what it writes lands in
            // the slot the pending token will take anyway, or in a block that is free again, so it has to finish
            // before anyone can be given that block.
            std::vector<Undo> &u = undo[done & 1];
            for (auto it = u.rbegin(); it != u.rend(); ++it) {
                int32_t *t = kv->trow(it->seq);
                const int32_t b = t[it->logical];
                t[it->logical] = -1;
                kv->refs[b] = 0;
                kv->free_stack.push_back(b);
                kv->seqs[it->seq].n_mapped = it->n_mapped_before;
            }
            enq = done;
            LD_HIP_TRY(hipStreamSynchronize(st));
        }
    }
    return LD_OK;
}

ld_status ld_step_mixed(ld_kv *kv, const ld_seq *dec, int32_t n_dec, const ld_seq *pf, const int32_t *const *pf_tokens,
                        const int32_t *pf_n, int32_t n_pf, void *stream, ld_token_cb cb, void *user, float *logits_out) {
    if (!kv || n_dec < 0 || n_pf < 0 || n_dec + n_pf == 0 || (n_dec && !dec) || (n_pf && (!pf || !pf_tokens || !pf_n)))
        return fail(LD_E_INVAL, "ld_step_mixed: bad argument");
    std::vector<Feed> feeds;
    for (int i = 0; i < n_dec; i++) {
        Seq *q = get_seq(kv, dec[i]);
        if (q && !q->has_pending) { ld::set_error("ld_step_mixed: decoding sequence %d has no pending token", dec[i]); return LD_E_STATE; }
        feeds.push_back({dec[i], nullptr, 0});
    }
    for (int i = 0; i < n_pf; i++) feeds.push_back({pf[i], pf_tokens[i], pf_n[i]});
    return run_step(kv, feeds, stream, cb, user, logits_out, "ld_step_mixed");
}

}  // extern "C"
