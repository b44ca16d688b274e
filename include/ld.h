/*
 * libld: single-GPU decode / chunked-prefill engine over a paged KV cache (gfx950).
 *
 * The serving system this library sits under invokes the LLM once per scheduling
 * iteration, hands every generated token to a streaming parser during decoding, and
 * later feeds collected tool observations back for prefilling (paper section 3.3,
 * workflow steps (2), (3), (8); section 2.2 step (g); section 2.1 for the attention /
 * KV-cache / prefill / decode definitions; section 4.1: temperature 0 = greedy).
 *
 * Conventions
 *  - Every call returns an ld_status; nothing throws or aborts, and ld_last_error()
 *    returns a thread-local description.  Argument, state and capacity errors
 *    (LD_E_INVAL, LD_E_STATE, LD_E_RANGE, LD_E_NOMEM) are found before anything is
 *    changed: the out parameters and all sequence / allocator state are as before the
 *    call.  LD_E_HIP (a HIP runtime call failed while a pass was being enqueued or
 *    waited for) is different: blocks may be reserved, a prompt may be partly fed, copies
 *    may be on their way.  The cache is then marked unusable, every later step, swap or
 *    fork on it returns LD_E_STATE, and the caller destroys it (ld_kv_free and
 *    ld_kv_destroy still work).
 *  - "DEVICE" pointers are HIP device memory owned by the caller (allocate it with
 *    any allocator, e.g. a torch tensor's data_ptr()); it must stay valid until the
 *    object that received it is destroyed.  "HOST" pointers are borrowed for the
 *    duration of the call only.  The library owns only host structures and a small
 *    pinned host staging area.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A step
 *    call enqueues all of its kernels on that stream, waits for the emitted tokens
 *    to reach the host, then runs the callbacks on the calling thread.
 *  - Matrices are row-major with the output index first ([n_out, n_in]), element type
 *    cfg.dtype.  RMSNorm gains are always float32.
 *  - Arithmetic (bf16 models; the paper's section 4.1 fixes none): float32 between kernels and in every
 *    accumulation; cached keys and values rounded to bf16.  The matrix products of a pass take the rows'
 *    activations as two bf16 terms (16 significant bits), except in passes of 512 rows or more (long prefill
 *    chunks, steps that mix decode rows with chunks), whose big-tile products take them rounded to fp16 (11
 *    bits) as long as every value of the pass and of the layer matrices lies within the fp16 range (+-65504);
 *    a pass that meets a larger value is repeated with two terms.  LD_GEMM_F16=0 in the environment keeps two
 *    terms everywhere.  ld_model_attach_f16_image trades memory for time in those passes, with equal results.
 *  - Sequence state: n_cached tokens have keys/values in the pool; `pending` is a token
 *    that was emitted but not fed yet (none right after ld_kv_alloc).
 */
#ifndef LD_H
#define LD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ld_model ld_model; /* opaque, library-owned */
typedef struct ld_kv ld_kv;       /* opaque, library-owned */
typedef int32_t ld_seq;           /* sequence handle inside one ld_kv */

typedef enum {
    LD_OK = 0,
    LD_E_INVAL = -1, /* bad argument (null pointer, bad handle, bad shape) */
    LD_E_NOMEM = -2, /* out of KV blocks or sequence slots */
    LD_E_STATE = -3, /* call not allowed in the sequence's state (no pending token, stopped, ...) */
    LD_E_HIP = -4,   /* a HIP runtime call failed */
    LD_E_RANGE = -5  /* token id >= vocab, context beyond max_blocks_per_seq, step larger than workspace */
} ld_status;

enum { LD_F32 = 0, LD_BF16 = 1 };

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps;     /* added to the mean square inside the root */
    float rope_base;   /* rotary angle of pair i at position p: p * rope_base^(-2i/head_dim) */
    int32_t dtype;     /* LD_F32 | LD_BF16: element type of matrices AND of the KV pool */
    int32_t kv_block;  /* tokens per KV block; must be 16 */
    int32_t max_chunk; /* ld_prefill splits longer inputs into chunks of this many rows */
    int32_t window;    /* attention band: > 0, a token at position p attends to positions
                          max(0, p - window + 1) .. p (the model family of section 4.1); 0: to all of 0 .. p.
                          The cache keeps every position either way. */
} ld_model_config;

/* DEVICE pointers.  Per-layer members are HOST arrays of n_layers DEVICE pointers
 * (the arrays themselves are copied by ld_model_create).
 *   embed, lm_head  [vocab, d_model]
 *   wqkv            [(n_heads + 2 n_kv_heads) * head_dim, d_model]   q rows, then k rows, then v rows
 *   wo              [d_model, n_heads * head_dim]
 *   wgate_up        [2 * d_ffn, d_model]                             gate rows, then up rows
 *   wdown           [d_model, d_ffn]
 *   attn_norm, ffn_norm, final_norm  [d_model] float32 */
typedef struct {
    const void *embed, *lm_head;
    const float *final_norm;
    const float *const *attn_norm;
    const void *const *wqkv;
    const void *const *wo;
    const float *const *ffn_norm;
    const void *const *wgate_up;
    const void *const *wdown;
} ld_weights;

/* Called once per emitted token, on the calling thread, in ascending order of the
 * sequence's index in the step's argument list.  `pos` is the absolute position the
 * token will occupy once fed.  Return LD_CB_CONTINUE to go on.  LD_CB_PAUSE ends a multi-step
 * run (ld_decode_run) after the current step and leaves the sequence as it is (a tool call is
 * complete and its observation comes next); in single-step calls it means the same as
 * LD_CB_CONTINUE.  Any other value marks the sequence stopped (early abort, section 4.3 case #2):
 * stepping it again returns LD_E_STATE until it is freed.  The callback must not call into the
 * library for the same cache. */
enum { LD_CB_CONTINUE = 0, LD_CB_ABORT = 1, LD_CB_PAUSE = 2 };
typedef int (*ld_token_cb)(void *user, ld_seq seq, int32_t token, int32_t pos);

/* Registers a model (section 3.3 step (a)).  Validates shapes, copies the configuration
 * and the pointer tables; touches no device memory.  Supported: head_dim 64 or 128,
 * kv_block 16, d_model and d_ffn multiples of 8, n_heads a multiple of n_kv_heads. */
ld_status ld_model_create(const ld_model_config *cfg, const ld_weights *w, ld_model **out);
void ld_model_destroy(ld_model *m);

/* Optional, bf16 models: an fp16 copy of the layer matrices for the passes that take the fp16 form (see Arithmetic
 * above).  Without it those passes widen every bf16 weight fragment to fp16 on its way to the matrix cores, in every
 * wave that reads it; with it they read fp16 directly.  Same products either way: tokens and logits are bit-equal.
 * The price is device memory: ld_model_f16_image_bytes(m) = 2 bytes per layer-matrix entry (0 for float32 models),
 * i.e. the layers' own size once more.
 * buf (device memory, 16-byte aligned, at least ld_model_f16_image_bytes(m) + 256 bytes) stays the caller's and must
 * live until the model is destroyed or the image is detached (buf NULL: detach; bytes ignored).  The call fills it
 * on `stream` from the weights as they are now, waits for the stream, and sets *in_range (may be NULL) to 1 when
 * every entry lies within +-65504.  Otherwise (*in_range 0) the buffer is not used, nor is the fp16 form: this model
 * then keeps two bf16 terms in every pass.  Weights changed later need a new call.  Not to be called while a pass of
 * this model is in flight. */
size_t ld_model_f16_image_bytes(const ld_model *m);
ld_status ld_model_attach_f16_image(ld_model *m, void *buf, size_t bytes, void *stream, int32_t *in_range);

/* Bytes of the KV pool for n_blocks blocks.  Pool layout (element type cfg.dtype):
 *   keys    [layer][block][0][kv_head][slot 0..15][head_dim]
 *   values  [layer][block][1][kv_head][head_dim][slot 0..15]     (transposed inside the block)
 * Token j of a sequence lives in physical block table[j / 16], slot j % 16.  A key row is
 * contiguous over head_dim; the 16 positions of one value dimension are contiguous, which is the
 * operand order of the probability-weighted sum over positions. */
size_t ld_kv_bytes(const ld_model *m, int64_t n_blocks);

/* Bytes of scratch a step of up to max_tokens rows (decode rows + prefill-chunk rows)
 * over at most max_seqs sequences of at most max_blocks_per_seq blocks needs. */
size_t ld_workspace_bytes(const ld_model *m, int32_t max_tokens, int32_t max_seqs, int32_t max_blocks_per_seq);

/* Creates the paged cache over caller-owned DEVICE memory: `pool` of ld_kv_bytes(m, n_blocks)
 * bytes and `ws` of at least ld_workspace_bytes(...) bytes, both 256-byte aligned.  The pool's
 * contents are not touched and need not be initialised: a slot is read only after a step has written
 * it (what an unwritten slot holds, NaN patterns included, never reaches a result).  No device call is made here (pinned staging is created lazily by
 * the first step).  The free list is a LIFO stack whose first pops return blocks 0, 1, 2, ... */
ld_status ld_kv_create(ld_model *m, void *pool, int64_t n_blocks, void *ws, size_t ws_bytes,
                       int32_t max_tokens, int32_t max_seqs, int32_t max_blocks_per_seq, ld_kv **out);
void ld_kv_destroy(ld_kv *kv);

/* New sequence (lowest free handle), with ceil(reserve_tokens / 16) blocks mapped up front.
 * LD_E_NOMEM if no handle or not enough free blocks. */
ld_status ld_kv_alloc(ld_kv *kv, int64_t reserve_tokens, ld_seq *out);
/* Test hook: map a sequence's logical block to a chosen free physical block (permuted tables).
 * LD_E_STATE if the logical block is already mapped, LD_E_NOMEM if the physical block is not free. */
ld_status ld_kv_map(ld_kv *kv, ld_seq seq, int32_t logical_block, int32_t physical_block);
/* Ends a sequence (finished or aborted early): pushes its blocks back in reverse logical order. */
ld_status ld_kv_free(ld_kv *kv, ld_seq seq);
/* Copies the sequence's block table (physical ids of logical blocks 0..n-1) to HOST out[cap]. */
ld_status ld_kv_block_table(const ld_kv *kv, ld_seq seq, int32_t *out, int32_t cap, int32_t *n);
/* Number of cached tokens of a sequence (-1 for a bad handle); number of free blocks. */
int64_t ld_kv_len(const ld_kv *kv, ld_seq seq);
int64_t ld_kv_free_blocks(const ld_kv *kv);
/* KV retention across a tool call (section 2.2: a request that waits for a tool can keep its cache
 * on the GPU, swap it to host memory, or discard it and prefill again).  Discarding is ld_kv_free
 * followed by a prefill of the token history; swapping is this pair.
 * ld_kv_swap_out copies the keys and values of the sequence's cached positions to HOST memory
 * (ld_kv_swap_bytes(kv, seq) bytes, layout [logical block][layer][block bytes]; pinned memory makes the
 * copy asynchronous) and returns every block the sequence holds to the free list in the order
 * ld_kv_free uses.  The handle, the token count and the pending token stay; until ld_kv_swap_in the
 * sequence cannot be stepped, mapped or extended (LD_E_STATE).  ld_kv_swap_in takes blocks for the
 * cached length as a reservation would (LD_E_NOMEM, nothing changed, if there are too few) and copies
 * the contents back.  Both calls only enqueue copies on `stream`: the host buffer holds the data once
 * the stream has passed them, must stay untouched until the swap-in's copies are done, and freed
 * blocks must not be written by work on OTHER streams before the swap-out's copies are done. */
size_t ld_kv_swap_bytes(const ld_kv *kv, ld_seq seq);
ld_status ld_kv_swap_out(ld_kv *kv, ld_seq seq, void *host_buf, size_t bytes, void *stream);
ld_status ld_kv_swap_in(ld_kv *kv, ld_seq seq, const void *host_buf, size_t bytes, void *stream);

/* Prefix sharing (section 2.1: many requests are served at once; section 4.1: every prompt carries the
 * same tool descriptions): a new sequence (lowest free handle) that starts with the first n_tokens cached
 * positions of `parent` (0 <= n_tokens <= its length).  Blocks the prefix fills completely are shared: both
 * sequences' tables name the same physical block, which returns to the free list when its last holder
 * frees or swaps it out; nothing ever writes a full block again.  A partly filled last block is copied
 * (all layers, device to device, enqueued on `stream`) into a block of the child's own, taken from the
 * free list (LD_E_NOMEM, nothing changed, if there is none).  The child has no pending token: continue it
 * with ld_prefill. */
ld_status ld_kv_fork(ld_kv *kv, ld_seq parent, int64_t n_tokens, void *stream, ld_seq *out);

/* Sliding-window memory (models with an attention band, cfg.window > 0): gives up the blocks of `seq` whose
 * 16 positions all lie below n_cached - window + 1, the lowest position the sequence's next query can see
 * (later queries see less), lowest logical block first; a block shared with other sequences (ld_kv_fork)
 * returns to the free stack when its last holder gives it up.  Their block-table entries read -1 afterwards
 * and no kernel dereferences them.  *released = blocks given up by this call (0 without a band).
 * A trimmed sequence swaps out and in as before (only the blocks it still holds travel; the buffer layout
 * and ld_kv_swap_bytes are unchanged); ld_kv_fork from it returns LD_E_STATE when the child's first query
 * would need a released block.  LD_E_STATE while swapped out.  released: HOST. */
ld_status ld_kv_trim(ld_kv *kv, ld_seq seq, int32_t *released);

/* Token choice of a sequence: temperature 0 (the default, and what section 4.1 uses) emits the greedy
 * token; temperature > 0 draws from softmax(logits / temperature) as ldk_sample does, with the position
 * the emitted token will take as the counter, so a run is reproducible from (seed, tokens fed). */
ld_status ld_kv_set_sampling(ld_kv *kv, ld_seq seq, float temperature, uint64_t seed);

/* Test / benchmark hook: declare that the next n_tokens positions of a sequence are already
 * cached (their blocks are mapped; the caller has written, or will write, their keys and values
 * straight into the pool using the layout above), and set the pending token (none if < 0). */
ld_status ld_kv_assume(ld_kv *kv, ld_seq seq, int64_t n_tokens, int32_t pending);

/* Prefill (prompt, or a tool observation appended to a live sequence): feeds
 * [pending?] ++ tokens[0..n) at positions n_cached.., in chunks of at most cfg.max_chunk
 * rows; emits argmax(logits of the last row) through cb (may be NULL) and keeps it as
 * the new pending token.  tokens: HOST.  logits_out: HOST float[vocab] or NULL. */
ld_status ld_prefill(ld_kv *kv, ld_seq seq, const int32_t *tokens, int32_t n, void *stream,
                     ld_token_cb cb, void *user, float *logits_out);

/* One decode iteration for n_seqs distinct sequences (each must have a pending token):
 * feeds the pending token, emits the next one per sequence.  seqs: HOST.
 * logits_out: HOST float[n_seqs, vocab] or NULL. */
ld_status ld_decode_step(ld_kv *kv, const ld_seq *seqs, int32_t n_seqs, void *stream,
                         ld_token_cb cb, void *user, float *logits_out);

/* Up to max_steps decode iterations for the same n_seqs sequences, with the callback one step behind the
 * GPU (section 3.3: every decoding iteration hands its tokens to the parser while the model goes on
 * decoding): step k+1 is enqueued before the tokens of step k are handed over, its input tokens read on the
 * device from what step k emitted, so parsing, the callback and the launch work of the next step overlap
 * the current step instead of leaving the GPU idle between steps.  Tokens, callback order and the state of
 * every sequence after the call are exactly those of *steps_done successive ld_decode_step calls.
 * The run ends after max_steps steps, after the first step in which a callback returns non-zero
 * (LD_CB_PAUSE: the sequence stays live; other values: it is stopped), or before a step whose blocks cannot
 * be reserved (then *steps_done < max_steps and no callback asked for the end; with no step done at all the
 * error itself is returned).  When a callback ends the run, the one step already enqueued beyond it is
 * discarded: its block reservations are returned and the call waits for it to drain, which costs one step
 * of GPU time; give max_steps the exact count when it is known.  steps_done: HOST, may be NULL. */
ld_status ld_decode_run(ld_kv *kv, const ld_seq *seqs, int32_t n_seqs, int32_t max_steps, void *stream,
                        ld_token_cb cb, void *user, int32_t *steps_done);

/* One mixed iteration of continuous batching: n_dec decoding sequences plus n_pf sequences that
 * each get [pending?] ++ pf_tokens[i][0..pf_n[i]) prefilled in the same pass (one chunk each,
 * total rows <= workspace max_tokens).  Every listed sequence emits one token; callbacks run for
 * dec[0..n_dec) first, then pf[0..n_pf).  All sequences distinct.  All arrays HOST.
 * logits_out: HOST float[n_dec + n_pf, vocab] or NULL. */
ld_status ld_step_mixed(ld_kv *kv, const ld_seq *dec, int32_t n_dec, const ld_seq *pf,
                        const int32_t *const *pf_tokens, const int32_t *pf_n, int32_t n_pf, void *stream,
                        ld_token_cb cb, void *user, float *logits_out);

/* Per-kernel timing for benchmarks (off by default).  While enabled, every kernel of a pass is launched
 * with a pair of HIP events attached to its dispatch (on the step's stream), which record the start and
 * the end of that kernel; after the pass has finished the kernel durations are added to the category of
 * the step they belong to.  ms[] is therefore pure kernel time (no launch gaps); launches[] counts steps
 * of the pass (one per layer for the per-layer categories), each of which may be several kernels.
 * Enabling clears the counters. */
enum { LD_PROF_QKV = 0, LD_PROF_ROPE_KV = 1, LD_PROF_ATTENTION = 2, LD_PROF_WO = 3, LD_PROF_GATE_UP = 4,
       LD_PROF_DOWN = 5, LD_PROF_LM_HEAD = 6, LD_PROF_OTHER = 7, LD_PROF_N = 8 };
typedef struct {
    double ms[LD_PROF_N];        /* summed device time per category, milliseconds */
    int64_t launches[LD_PROF_N]; /* timed steps per category */
} ld_profile;
ld_status ld_kv_profile(ld_kv *kv, int32_t enable);
ld_status ld_kv_profile_read(const ld_kv *kv, ld_profile *out); /* out: HOST */

/* Text of the last error on this thread ("" if none). */
const char *ld_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LD_H */
