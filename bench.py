#!/usr/bin/env python3
"""Decode throughput of the 7B-shaped bf16 decoder on one MI355X, tool-call pattern.

Workload (batch 1): prompt of 1024 random token ids, then rounds of "greedily emit 256 tokens, append a
128..512-token random observation through chunked prefill (chunk 256)".  A *step* is one decode iteration:
the whole decode pass (32 layers + LM head + argmax), the token hand-off to the host and the callback.  The
steps of a round run inside one ld_decode_run call, which enqueues step k+1 before it hands over the token
of step k (the callback still sees every token, one step behind the GPU).  `value` is decode tokens/s over
exactly --steps timed steps; prompt and observation prefills run between the rounds and are reported
beside it.  Inputs (weights, tokens) are seeded and
synthetic and are resident in HBM before timing starts.

Prints ONE JSON line.  `roofline` describes the kernel with the largest share of the step
(HIP events attached to every kernel dispatch during a profiled tail of the same run); `cpu_baseline` is the CPU oracle
timed on this machine's host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # bytes/s, MI355X HBM3E
# HBM bytes per launch of the dominant kernel from rocprofv3 FETCH_SIZE + WRITE_SIZE counters, scaled by a
# 256 MiB copy (profiles/gate_up_gemv_hbm_traffic.md); valid only for the kernel source it was taken on.
TRAFFIC_BYTES = 180_870_000
TRAFFIC_KERNEL_MD5 = "0468ef4efdc5"
ATTN_TRAFFIC_RATIO = 1.007
ATTN_TRAFFIC_MD5 = "ef39af836308"
ROUND_TOKENS = 256         # tokens emitted per round (1 by the preceding prefill + 255 decode steps)
CHUNK = 256


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3 * (ROUND_TOKENS - 1))
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--profile-steps", type=int, default=32, help="extra steps run with per-kernel events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-batch32", action="store_true", help="skip the batch-32 continuous-batching leg")
    ap.add_argument("--no-attention-microbench", action="store_true", help="skip the decode-attention micro-benchmark leg")
    ap.add_argument("--no-gqa", action="store_true", help="skip the batch-32 leg on the grouped-KV 7B shape")
    ap.add_argument("--no-f16-image", action="store_true",
                    help="do not give the models the fp16 copy of their layer matrices (passes of 512+ rows then widen "
                         "the bf16 weights in the kernel)")
    ap.add_argument("--no-13b", action="store_true", help="skip the 13B-shaped batch-64 leg (200 GB KV pool)")
    ap.add_argument("--steps-13b", type=int, default=16, help="timed steps of the 13B leg (the workload has 64)")
    ap.add_argument("--only-batch32", action="store_true", help="debug: run only the batch-32 leg (prints its dict)")
    ap.add_argument("--only-gqa", action="store_true",
                    help="run only the batch-32 leg on the grouped-KV 7B shape (8 KV heads, attention band 4096); "
                         "prints its dict")
    ap.add_argument("--only-13b", action="store_true",
                    help="run only the 13B-shaped batch-64 workload (~200 GB KV pool, 64 steps of 63 decode rows + one "
                         "2048-token prefill chunk); prints its dict instead of the benchmark line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 256 MiB device-to-device copy (a plain copy kernel of known size, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--kernel-probe", action="store_true",
                    help="run only the dominant kernel (gate/up projection, 7B shape, batch 1) 16 times on 4 rotating "
                         "matrices, plus the calibration copy: the short program the rocprofv3 --pmc runs use")
    ap.add_argument("--attention-probe", action="store_true",
                    help="launch only the batch-32 decode attention (+ 256 MiB copies), for the HBM-traffic counter runs")
    ap.add_argument("--skinny-probe", action="store_true",
                    help="launch only the 32-row gate/up projection (small-batch matrix-core kernel + its reduction) and "
                         "256 MiB copies, for the HBM-traffic counter runs")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="launch only the prefill-side matrix-core kernels (layer GEMMs at 1056 and 2048 rows, chunk-prefill "
                         "attention of a mixed step), for the MFMA counter runs")
    ap.add_argument("--layers", type=int, default=0, help="debug: fewer layers (result is NOT the benchmark)")
    return ap.parse_args()


MFMA_PEAK = 2.5e15         # flop/s, bf16 dense


def ld_gemm_terms(rows):
    """Matrix-core terms per float32 activation in a pass of `rows` rows: two bf16 terms (high + low part); one
    fp16 term in passes of at least LD_GEMM_F16_MIN_ROWS (512) rows unless LD_GEMM_F16=0 (the few rows past the
    last full 256-row tile, which keep both terms, are not counted apart)."""
    on = os.environ.get("LD_GEMM_F16", "1") != "0"
    return 1 if on and rows >= int(os.environ.get("LD_GEMM_F16_MIN_ROWS", "512")) else 2


def _source_md5(name):
    import hashlib
    try:
        return hashlib.md5(open(os.path.join(ROOT, "paper_2406_00059_amd", "csrc", name), "rb").read()).hexdigest()
    except OSError:
        return ""


def attention_traffic_ratio():
    """FETCH_SIZE + WRITE_SIZE over algorithmic bytes of the batch-32 decode attention launch
    (profiles/decode_attention_b32_hbm_traffic.md), or None once the kernel's source has changed since."""
    return ATTN_TRAFFIC_RATIO if _source_md5("ld_kernels.hip").startswith(ATTN_TRAFFIC_MD5) else None


def kernel_traffic():
    """Measured HBM bytes per launch of the dominant kernel, or None if its source changed since."""
    import hashlib
    src = os.path.join(ROOT, "paper_2406_00059_amd", "csrc", "ld_gemv.hip")
    try:
        h = hashlib.md5(open(src, "rb").read()).hexdigest()
    except OSError:
        return None
    return TRAFFIC_BYTES if h.startswith(TRAFFIC_KERNEL_MD5) else None


def noop_cb(seq, tok, pos):
    return 0


def cpu_baseline(shape, weights, ctx, steps, seed):
    """The oracle, as it stands, on the host cores: `steps` decode steps at context `ctx` over an injected
    synthetic KV history (values do not change the work done)."""
    import numpy as np
    import oracle
    from workloads import gen
    om = oracle.Model(shape, weights)
    nblk = (ctx + steps + 16) // 16 + 1
    okv = oracle.KV(om, nblk, 1, nblk)
    rc, s = okv.alloc(0)
    hist = gen.normal(seed, 900, (ctx, shape.n_layers, 2, shape.n_kv_heads, shape.head_dim)).bfloat16().double().numpy()
    assert okv.inject(s, hist, pending=1) == 0
    del hist
    okv.decode(s, want_logits=False)          # one untimed step: page in the weights
    t0 = time.perf_counter()
    for _ in range(steps):
        rc, tok, _ = okv.decode(s, want_logits=False)
        assert rc == 0
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": steps / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"{steps} decode steps of the same 7B bf16 decoder at context {ctx} (injected KV history), "
                      f"batch 1; {dt:.1f} s of CPU work"}


def run_batch1(args, ld, torch, shape, weights, model):
    import numpy as np
    from workloads import gen, SEED_BASE
    seed = SEED_BASE + 2
    K, W = args.steps, args.warmup
    # decode steps per round: 255 in the workload; a short run (--steps below three rounds) keeps the round
    # structure by shortening the rounds, so that observation prefills happen inside it
    per_round = max(1, min(ROUND_TOKENS - 1, K // 3))
    rounds = max(1, -(-K // per_round))
    max_ctx = 1024 + rounds * (ROUND_TOKENS + 513) + args.profile_steps + 64
    nblk_seq = -(-max_ctx // 16)
    kv = ld.KV(model, nblk_seq + 16, CHUNK, 2, nblk_seq)
    stream = torch.cuda.current_stream()

    # warm-up on a throw-away sequence
    ws = ld.ld_kv_alloc(kv.h, 0)
    ld.ld_prefill(kv.h, ws, gen.randint(seed, 90, 0, shape.vocab - 1, 64).numpy().astype(np.int32), stream, noop_cb)
    ld.ld_decode_run(kv.h, [ws], W, stream, noop_cb)
    ld.ld_kv_free(kv.h, ws)

    s = ld.ld_kv_alloc(kv.h, 0)
    prompt = gen.randint(seed, 100, 0, shape.vocab - 1, 1024).numpy().astype(np.int32)
    obs_len = gen.randint(seed, 101, 128, 512, rounds).tolist()
    torch.cuda.synchronize()
    pf_tokens, pf_time = 0, 0.0
    t0 = time.perf_counter()
    ld.ld_prefill(kv.h, s, prompt, stream, noop_cb)
    pf_time += time.perf_counter() - t0; pf_tokens += prompt.size

    step_ms, step_bytes = [], []
    Wb, kappa = shape.weight_bytes_per_step, shape.kv_bytes_per_token
    done = 0
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    obs_ms, obs_rows = [], []
    for r in range(rounds):
        n = min(per_round, K - done)
        ctx = ld.ld_kv_len(kv.h, s) + 1
        stamps = [time.perf_counter()]
        rc, got = ld.ld_decode_run(kv.h, [s], n, stream, lambda q, tok, pos: stamps.append(time.perf_counter()) and 0)
        stamps[-1] = time.perf_counter()                     # the call returns right after the last callback
        assert got == n
        step_ms += [(b - a) * 1e3 for a, b in zip(stamps, stamps[1:])]
        step_bytes += [Wb + (ctx + i) * kappa for i in range(n)]
        done += n
        if done >= K and r == rounds - 1 and n < per_round:
            break
        obs = gen.randint(seed, 200 + r, 0, shape.vocab - 1, obs_len[r]).numpy().astype(np.int32)
        t0 = time.perf_counter()
        ld.ld_prefill(kv.h, s, obs, stream, noop_cb)
        dt = time.perf_counter() - t0
        pf_time += dt; pf_tokens += obs.size + 1
        obs_ms.append(dt * 1e3); obs_rows.append(obs.size + 1)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_begin
    assert len(step_ms) == K
    dec_s = sum(step_ms) / 1e3

    # per-kernel durations: a profiled tail of the same run
    ld.ld_kv_profile(kv.h, True)
    ctx_prof = ld.ld_kv_len(kv.h, s) + 1
    for _ in range(args.profile_steps):
        ld.ld_decode_step(kv.h, [s], stream, noop_cb)
    prof = ld.ld_kv_profile_read(kv.h)
    ld.ld_kv_profile(kv.h, False)
    e = 2
    d, f, V = shape.d_model, shape.d_ffn, shape.vocab
    nqkv = (shape.n_heads + 2 * shape.n_kv_heads) * shape.head_dim
    alg_bytes = {   # algorithmic bytes per launch: the matrix once, input row(s), gain, output row(s)
        "qkv": nqkv * d * e + d * 4 * 2 + nqkv * 4,
        "wo": d * d * e + d * 4 * 3,
        "gate_up": 2 * f * d * e + d * 4 * 2 + f * 4,
        "down": d * f * e + f * 4 + d * 4 * 2,
        "lm_head": V * d * e + d * 4 + V * 4,
        "attention": (ctx_prof + args.profile_steps // 2) * 2 * shape.n_kv_heads * shape.head_dim * e,
    }
    kernels = {}
    for name, (ms, n) in prof.items():
        if n:
            avg = ms / n
            kernels[name] = {"avg_us": round(avg * 1e3, 2), "launches_per_step": n // args.profile_steps}
            if name in alg_bytes:
                kernels[name]["GBps"] = round(alg_bytes[name] / (avg * 1e-3) / 1e9, 1)
    per_step_ms = {k: v[0] / args.profile_steps for k, v in prof.items()}
    dominant = max((k for k in per_step_ms if k in alg_bytes), key=lambda k: per_step_ms[k])
    # Duration of the dominant kernel (the gate/up projection with fused RMSNorm + SwiGLU): HIP events
    # attached to its dispatches on the step's stream during the profiled steps above (kernel start to
    # kernel end, like a kernel trace).  Beside it: the same launch on every layer's weights in turn between
    # ONE pair of events, which adds the launch gap between consecutive kernels.
    assert dominant == "gate_up", (dominant, {k: round(v["avg_us"], 1) for k, v in kernels.items()})
    avg_s = prof[dominant][0] / prof[dominant][1] * 1e-3
    xin = torch.randn(1, d, device="cuda"); yout = torch.empty(1, f, device="cuda")
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    L = shape.n_layers
    for l in range(L):
        ld.ldk_linear(weights["wgate_up"][l], xin, yout, ld.LDK_SWIGLU, g=weights["ffn_norm"][l], eps=shape.rms_eps)
    reps = 8
    ev0.record(stream)
    for _ in range(reps):
        for l in range(L):
            ld.ldk_linear(weights["wgate_up"][l], xin, yout, ld.LDK_SWIGLU, g=weights["ffn_norm"][l], eps=shape.rms_eps)
    ev1.record(stream)
    torch.cuda.synchronize()
    b2b_s = ev0.elapsed_time(ev1) * 1e-3 / (reps * L)
    roofline = {"bound": "hbm", "kernel": "k_gemv1<1, 8, 2, true> (gate/up projection, fused RMSNorm + SwiGLU)",
                "achieved": round(alg_bytes[dominant] / avg_s / 1e9, 1),
                "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": round(alg_bytes[dominant] / avg_s / HBM_PEAK, 4),
                "traffic": kernel_traffic(), "avg_launch_us": round(avg_s * 1e6, 2),
                "bytes_per_launch": alg_bytes[dominant], "launches_timed": prof[dominant][1],
                "back_to_back_us_incl_launch_gap": round(b2b_s * 1e6, 2),
                "share_of_step_kernel_time": round(per_step_ms[dominant] / sum(per_step_ms.values()), 3)}
    out = {
        "value": K / dec_s, "ms_per_step": statistics.mean(step_ms),
        "ms_per_step_median": statistics.median(step_ms),
        "ms_per_step_std": statistics.pstdev(step_ms),
        "step_hbm_GBps": round(sum(step_bytes) / dec_s / 1e9, 1),
        "step_hbm_frac": round(sum(step_bytes) / dec_s / HBM_PEAK, 4),
        "prefill_tokens_per_s": round(pf_tokens / pf_time, 1), "prefill_tokens": pf_tokens,
        "decode_steps_per_round": per_round, "observations": len(obs_ms),
        "observation_rows": obs_rows, "observation_prefill_ms": [round(t, 3) for t in obs_ms],
        "observation_ms_per_256_rows": round(256.0 * sum(obs_ms) / max(sum(obs_rows), 1), 3) if obs_ms else None,
        "scenario_s": round(t_total, 3), "final_context": int(ld.ld_kv_len(kv.h, s)),
        "kernel_sum_ms_per_step": round(sum(per_step_ms.values()), 4),
        "kernels": kernels, "roofline": roofline,
    }
    kv.close()
    return out


def run_batch32(args, ld, torch, shape, model):
    """Continuous batching at batch 32: contexts uniform in [512, 8192] (synthetic KV history written
    straight into the pool), 128 steps; every 16th step 4 random sequences get a 256-token observation
    chunk prefilled in the same pass."""
    import numpy as np
    from workloads import gen, SEED_BASE
    seed = SEED_BASE + 3
    B, steps = 32, 128
    lens = gen.randint(seed, 1, 512, 8192, B).tolist()
    max_ctx = max(lens) + steps + 8 * 257 + 16
    nblk_seq = -(-max_ctx // 16)
    total_blocks = sum(-(-(n + steps + 8 * 257) // 16) for n in lens) + 64
    T_max = (B - 4) + 4 * 257
    pdt = torch.bfloat16
    pool = torch.empty((shape.n_layers, total_blocks, 2, shape.n_kv_heads, 16, shape.head_dim), dtype=pdt, device="cuda")
    for l in range(shape.n_layers):       # N(0,1) history, one layer at a time
        pool[l] = gen.normal(seed, 1000 + l, tuple(pool[l].shape), device="cuda").to(pdt)
    kv = ld.KV(model, total_blocks, T_max, B, nblk_seq, pool=pool)
    stream = torch.cuda.current_stream()
    f16_image = (not args.no_f16_image) and ld_gemm_terms(T_max) == 1 and model.attach_f16_image(stream)
    seqs = []
    for b in range(B):
        s = ld.ld_kv_alloc(kv.h, 0)
        ld.ld_kv_assume(kv.h, s, lens[b], pending=int(gen.randint(seed, 2, 0, shape.vocab - 1, B)[b]))
        seqs.append(s)
    for _ in range(3):                    # warm-up steps (they advance every context by one token)
        ld.ld_decode_step(kv.h, seqs, stream, noop_cb)
    torch.cuda.synchronize()
    pure_ms, mixed_ms, pure_bytes = [], [], []
    Wb, kappa = shape.weight_bytes_per_step, shape.kv_bytes_per_token
    visible = (lambda n: min(n, shape.window)) if shape.window else (lambda n: n)   # positions a decode row reads
    t_begin = time.perf_counter()
    step = 1
    while step <= steps:
        if step % 16 == 0:
            pick = gen.permutation(seed, 3000 + step, B)[:4].tolist()
            pf = [seqs[i] for i in pick]
            dec = [s for s in seqs if s not in pf]
            obs = [gen.randint(seed, 4000 + step * 8 + i, 0, shape.vocab - 1, 256).numpy().astype(np.int32) for i in range(4)]
            t0 = time.perf_counter()
            ld.ld_step_mixed(kv.h, dec, pf, obs, stream, noop_cb)
            mixed_ms.append((time.perf_counter() - t0) * 1e3)
            step += 1
        else:
            n = min(16 - step % 16, steps - step + 1)        # the pure decode steps up to the next mixed one
            lens_now = [ld.ld_kv_len(kv.h, s) + 1 for s in seqs]
            t0 = time.perf_counter()
            rc, got = ld.ld_decode_run(kv.h, seqs, n, stream, noop_cb)
            dt = (time.perf_counter() - t0) * 1e3
            assert got == n
            pure_ms += [dt / n] * n
            pure_bytes += [Wb + sum(visible(c + i) for c in lens_now) * kappa for i in range(n)]
            step += n
    torch.cuda.synchronize()
    total = time.perf_counter() - t_begin
    ld.ld_kv_profile(kv.h, True)
    for _ in range(4):
        ld.ld_decode_step(kv.h, seqs, stream, noop_cb)
    prof = ld.ld_kv_profile_read(kv.h)
    ld.ld_kv_profile(kv.h, False)
    sum_ctx = sum(visible(ld.ld_kv_len(kv.h, s)) for s in seqs)
    # one more mixed step with per-kernel timing (the four shortest sequences take the observation): the GEMM
    # categories against the MFMA peak, nominal flops 2 * rows * weight elements and twice that on the matrix
    # cores (the fp32 activations go in as two bf16 parts)
    short = sorted(range(B), key=lambda i: ld.ld_kv_len(kv.h, seqs[i]))[:4]
    pf = [seqs[i] for i in short]
    obs = [gen.randint(seed, 9000 + i, 0, shape.vocab - 1, 256).numpy().astype(np.int32) for i in range(4)]
    ld.ld_kv_profile(kv.h, True)
    ld.ld_step_mixed(kv.h, [s for s in seqs if s not in pf], pf, obs, stream, noop_cb)
    prof_mixed = ld.ld_kv_profile_read(kv.h)
    ld.ld_kv_profile(kv.h, False)
    rows_mixed = (B - 4) + 4 * 257
    layer_elems = shape.n_layers * ((shape.n_heads + 2 * shape.n_kv_heads) * shape.head_dim * shape.d_model +
                                    shape.n_heads * shape.head_dim * shape.d_model + 3 * shape.d_model * shape.d_ffn)
    gemm_ms_mixed = sum(prof_mixed[c][0] for c in ("qkv", "wo", "gate_up", "down"))
    gemm_nominal = 2.0 * rows_mixed * layer_elems
    att_bytes = sum_ctx * 2 * shape.n_kv_heads * shape.head_dim * 2
    att_avg = prof["attention"][0] / max(prof["attention"][1], 1) * 1e-3
    out = {
        "workload": f"{shape.name}-shaped bf16 decoder ({shape.n_heads} heads on {shape.n_kv_heads} KV heads, "
                    f"attention band {shape.window or 'none'}), continuous batching at batch 32, contexts U[512,8192], "
                    "128 steps, 4 sequences get a 256-token observation chunk every 16th step",
        "decode_tokens_per_s": round(B * len(pure_ms) / (sum(pure_ms) / 1e3), 1),
        "ms_per_pure_decode_step": round(statistics.mean(pure_ms), 3),
        "ms_per_mixed_step": round(statistics.mean(mixed_ms), 3),
        "rows_per_mixed_step": (B - 4) + 4 * 257,
        "all_tokens_per_s": round((B * steps + 8 * 4 * 256) / total, 1),
        "step_hbm_frac": round(sum(pure_bytes) / (sum(pure_ms) / 1e3) / HBM_PEAK, 4),
        "attention_avg_us": round(att_avg * 1e6, 1),
        "attention_GBps": round(att_bytes / att_avg / 1e9, 1),
        "attention_hbm_frac": round(att_bytes / att_avg / HBM_PEAK, 4),
        "kernel_ms_per_step": {k: round(v[0] / 4, 4) for k, v in prof.items()},
        "sum_visible_context": int(sum_ctx),
        "kernel_ms_mixed_step": {k: round(v[0], 3) for k, v in prof_mixed.items()},
        # MFMA fractions: first on the method's flops (2 * rows * weight elements), then on what the matrix cores
        # execute (twice that when the float32 activations go in as two bf16 terms, once in the fp16 form)
        "mixed_step_gemm_terms": ld_gemm_terms(rows_mixed),
        "f16_weight_image_GB": round(ld.ld_model_f16_image_bytes(model.h) / 1e9, 2) if f16_image else 0,
        "mixed_step_gemm_TFLOPs": round(gemm_nominal / (gemm_ms_mixed * 1e-3) / 1e12, 1),
        "mixed_step_gemm_mfma_frac": round(gemm_nominal / (gemm_ms_mixed * 1e-3) / MFMA_PEAK, 4),
        "mixed_step_gemm_mfma_frac_executed": round(ld_gemm_terms(rows_mixed) * gemm_nominal / (gemm_ms_mixed * 1e-3) / MFMA_PEAK, 4),
        "decode_gemm_weight_GBps": round(Wb / (sum(prof[c][0] for c in ("qkv", "wo", "gate_up", "down", "lm_head")) / 4 * 1e-3) / 1e9, 1),
        "roofline": {"bound": "hbm", "kernel": "decode attention (k_attn_partial / k_attn_decode_grouped + k_attn_merge), one layer, 32 rows",
                     "achieved": round(att_bytes / att_avg / 1e9, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                     "frac": round(att_bytes / att_avg / HBM_PEAK, 4), "avg_launch_us": round(att_avg * 1e6, 1),
                     "bytes_per_launch": int(att_bytes), "launches_timed": int(prof["attention"][1]),
                     "share_of_step_kernel_time": round(prof["attention"][0] / sum(v[0] for v in prof.values()), 3),
                     "traffic_over_algorithmic": attention_traffic_ratio() if not shape.window and shape.n_kv_heads == shape.n_heads else None},
    }
    kv.close()
    if f16_image:
        model.detach_f16_image()
    return out


def run_attention_microbench(args, ld, torch):
    """Decode-attention micro-benchmark: batch 16, 32 heads x 128, bf16 paged cache with block size 16 and a
    randomly permuted block table, contexts uniform in [256, 4096], keys / values / queries N(0,1), one query
    per sequence.  Timed: the split-KV attention kernel plus its merge (one ldk_paged_attention call), HIP
    events around the loop.  Cold: four pools (4 x 0.57 GB) in rotation, so that a pool's lines have left the
    256 MB memory-side cache when its turn comes again; warm: the same pool every time."""
    from workloads import gen, SEED_BASE
    seed = SEED_BASE + 1
    B, H, hd, reps, n_pools = 16, 32, 128, 200, 4
    lens = gen.randint(seed, 1, 256, 4096, B).tolist()
    nb = [-(-n // 16) for n in lens]
    total = sum(nb)
    perm = gen.permutation(seed, 1, total).tolist()
    table = torch.zeros((B, max(nb)), dtype=torch.int32)
    it = iter(perm)
    for b in range(B):
        for j in range(nb[b]):
            table[b, j] = next(it)
    table = table.cuda()
    pools = [gen.normal(seed, 10 + i, (total, 2, H, 16, hd), device="cuda", dtype=torch.bfloat16) for i in range(n_pools)]
    q = gen.normal(seed, 3, (B, H * hd), device="cuda")
    out = torch.empty(B, H * hd, device="cuda")
    ctx = torch.tensor(lens, dtype=torch.int32, device="cuda")
    slot = torch.arange(B, dtype=torch.int32, device="cuda")
    scratch = torch.empty(ld.ldk_attention_scratch_bytes(B, H, H, hd, max(lens)), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    call = lambda pool: ld.ldk_paged_attention(q, H * hd, pool, table, slot, ctx, max(lens), H, H, hd, out, scratch, stream=stream)
    alg = sum(lens) * 2 * H * hd * 2 + 2 * B * H * hd * 4 + total * 4
    res = {}
    for name, seq in (("cold", lambda i: pools[i % n_pools]), ("warm", lambda i: pools[0])):
        for i in range(8):
            call(seq(i))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(reps):
            call(seq(i))
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        res[name] = {"us_per_call": round(us, 2), "GBps": round(alg / us / 1e3, 1), "hbm_frac": round(alg / (us * 1e-6) / HBM_PEAK, 4)}
    return {"workload": "decode attention, bf16, batch 16, 32 heads x 128, block 16, permuted block table, contexts "
                        f"U[256,4096] (sum {sum(lens)}), one query per sequence; attention kernel + merge per call",
            "reps": reps, "pools_in_rotation": n_pools, "algorithmic_bytes_per_call": alg,
            "cold": res["cold"], "warm": res["warm"], "target_GBps": 5600.0}


def run_13b(args, ld, torch):
    """13B-shaped decoder, batch 64, paged pool of ~200 GB: contexts drawn uniform in [1024, 16384] and
    scaled by a common factor so that they fit the pool; every step one sequence is a finished request that
    is replaced (its blocks freed, the first 2048-token chunk of a new request prefilled) while the other
    63 decode one token."""
    import numpy as np
    from workloads import LLAMA13B, SEED_BASE, gen, make_weights
    shape = LLAMA13B if not args.layers else LLAMA13B.with_layers(args.layers)
    seed = SEED_BASE + 4
    B, steps, chunk = 64, max(1, args.steps_13b), 2048
    weights = make_weights(shape, seed, device="cuda")
    model = ld.Model(shape, weights, max_chunk=chunk)
    n_blocks = int(200e9 // (shape.kv_bytes_per_token * 16)) if not args.layers else 15258
    drawn = gen.randint(seed, 1, 1024, 16384, B).tolist()
    budget = n_blocks * 16 - B * (steps + 16) - (chunk + 16) - B * 16
    scale = min(1.0, budget / sum(drawn))
    lens = [max(16, int(n * scale)) for n in drawn]
    nblk_seq = (max(max(lens), chunk) + steps + 32) // 16 + 1
    pool = torch.empty((shape.n_layers, n_blocks, 2, shape.n_kv_heads, 16, shape.head_dim), dtype=torch.bfloat16,
                       device="cuda")
    for l in range(shape.n_layers):
        pool[l].normal_(0.0, 1.0)
    kv = ld.KV(model, n_blocks, B + chunk, B, nblk_seq, pool=pool)
    stream = torch.cuda.current_stream()
    f16_image = (not args.no_f16_image) and ld_gemm_terms(B - 1 + chunk) == 1 and model.attach_f16_image(stream)
    pend = gen.randint(seed, 2, 0, shape.vocab - 1, B).tolist()
    seqs = []
    for b in range(B):
        s = ld.ld_kv_alloc(kv.h, 0)
        ld.ld_kv_assume(kv.h, s, lens[b], pending=pend[b])
        seqs.append(s)
    for _ in range(2):
        ld.ld_decode_step(kv.h, seqs, stream, noop_cb)
    torch.cuda.synchronize()
    ms, kv_bytes = [], []
    t_begin = time.perf_counter()
    for step in range(steps):
        k = step % B
        ld.ld_kv_free(kv.h, seqs[k])
        seqs[k] = ld.ld_kv_alloc(kv.h, 0)
        new_tokens = gen.randint(seed, 5000 + step, 0, shape.vocab - 1, chunk).numpy().astype(np.int32)
        dec = [s for i, s in enumerate(seqs) if i != k]
        sum_ctx = sum(ld.ld_kv_len(kv.h, s) + 1 for s in dec)
        t0 = time.perf_counter()
        ld.ld_step_mixed(kv.h, dec, [seqs[k]], [new_tokens], stream, noop_cb)
        ms.append((time.perf_counter() - t0) * 1e3)
        kv_bytes.append(sum_ctx * shape.kv_bytes_per_token)
    torch.cuda.synchronize()
    total = time.perf_counter() - t_begin
    ld.ld_kv_profile(kv.h, True)
    k = steps % B
    ld.ld_kv_free(kv.h, seqs[k]); seqs[k] = ld.ld_kv_alloc(kv.h, 0)
    ld.ld_step_mixed(kv.h, [s for i, s in enumerate(seqs) if i != k], [seqs[k]],
                     [gen.randint(seed, 9999, 0, shape.vocab - 1, chunk).numpy().astype(np.int32)], stream, noop_cb)
    prof = ld.ld_kv_profile_read(kv.h)
    ld.ld_kv_profile(kv.h, False)
    gemm_flops = (B - 1 + chunk) * 2 * (shape.weight_bytes_per_step / 2)
    gemm_ms = sum(prof[c][0] for c in ("qkv", "wo", "gate_up", "down", "lm_head"))
    out = {
        "workload": "13B-shaped bf16 decoder, batch 64, KV pool of %d blocks (%.1f GB), contexts %d..%d after scaling "
                    "by %.3f, steps of 63 decode rows + one 2048-token prefill chunk" %
                    (n_blocks, n_blocks * 16 * shape.kv_bytes_per_token / 1e9, min(lens), max(lens), scale),
        "ms_per_step": round(statistics.mean(ms), 2), "tokens_per_s": round((B - 1 + chunk) * steps / total, 1),
        "decode_tokens_per_s": round((B - 1) * steps / total, 1),
        "kv_GB_per_step": round(statistics.mean(kv_bytes) / 1e9, 1),
        "kernel_ms_one_step": {c: round(v[0], 3) for c, v in prof.items()},
        "attention_GBps_if_all_attention_time_were_decode": round(statistics.mean(kv_bytes) / (prof["attention"][0] * 1e-3) / 1e9, 1),
        "gemm_TFLOPs": round(gemm_flops / (gemm_ms * 1e-3) / 1e12, 1),
        "gemm_mfma_frac": round(gemm_flops / (gemm_ms * 1e-3) / MFMA_PEAK, 4),
        "gemm_terms": ld_gemm_terms(B - 1 + chunk),
        "f16_weight_image_GB": round(ld.ld_model_f16_image_bytes(model.h) / 1e9, 2) if f16_image else 0,
        "gemm_mfma_frac_executed": round(ld_gemm_terms(B - 1 + chunk) * gemm_flops / (gemm_ms * 1e-3) / MFMA_PEAK, 4),
        "attention_ms_one_step": round(prof["attention"][0], 3),
        "steps_timed": steps, "n_layers": shape.n_layers,
    }
    del pool
    kv.close()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2406_00059_amd as ld
    from workloads import LLAMA7B, MISTRAL7B, SEED_BASE, make_weights
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    ld.lib()
    torch.cuda.set_device(0)
    if args.only_13b:
        print(json.dumps(run_13b(args, ld, torch)))
        return
    if args.only_gqa:
        shape = MISTRAL7B if not args.layers else MISTRAL7B.with_layers(args.layers)
        weights = make_weights(shape, SEED_BASE + 5, device="cuda")
        print(json.dumps(run_batch32(args, ld, torch, shape, ld.Model(shape, weights, max_chunk=CHUNK))))
        return
    shape = LLAMA7B if not args.layers else LLAMA7B.with_layers(args.layers)
    if args.kernel_probe:
        d, f = shape.d_model, shape.d_ffn
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        b = torch.empty_like(a)
        ws = [torch.empty(2 * f, d, device="cuda").normal_(0, 0.02).bfloat16() for _ in range(4)]
        g = torch.ones(d, device="cuda"); x = torch.randn(1, d, device="cuda"); y = torch.empty(1, f, device="cuda")
        for i in range(16):
            ld.ldk_linear(ws[i % 4], x, y, ld.LDK_SWIGLU, g=g, eps=shape.rms_eps)
            if i % 4 == 0:
                b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"probe": "k_gemv1 gate/up 7B batch 1", "launches": 16,
                          "algorithmic_bytes_per_launch": 2 * f * d * 2 + d * 8 + f * 4,
                          "copy_bytes_each_way": 256 << 20, "copies": 4}))
        return
    if args.skinny_probe:
        d, f = shape.d_model, shape.d_ffn
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        b = torch.empty_like(a)
        ws = [torch.empty(2 * f, d, device="cuda").normal_(0, 0.02).bfloat16() for _ in range(4)]
        g = torch.ones(d, device="cuda"); x = torch.randn(32, d, device="cuda"); y = torch.empty(32, f, device="cuda")
        scratch = torch.empty(ld.ldk_linear_scratch_bytes(32, f, d, ld.LDK_SWIGLU), dtype=torch.uint8, device="cuda")
        for i in range(16):
            ld.ldk_linear(ws[i % 4], x, y, ld.LDK_SWIGLU, g=g, eps=shape.rms_eps, scratch=scratch)
            if i % 4 == 0:
                b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"probe": "gate/up projection, 7B shape, 32 rows (k_norm_split + k_gemm_skinny + k_splitk_reduce)",
                          "launches": 16, "weight_bytes_per_launch": 2 * f * d * 2,
                          "algorithmic_bytes_per_launch": 2 * f * d * 2 + 32 * d * 4 + 32 * f * 4,
                          "partial_sum_bytes_written_per_launch": (d // 512) * 32 * 2 * f * 4,
                          "copy_bytes_each_way": 256 << 20, "copies": 4}))
        return
    if args.mfma_probe:
        d, f, H, hd = shape.d_model, shape.d_ffn, shape.n_heads, shape.head_dim
        out = {"probe": "prefill-side matrix-core kernels, 7B layer shapes", "launches_per_case": 3, "gemm": [], "attention": None}
        mats = [("qkv", 3 * d, d, ld.LDK_STORE), ("wo", d, d, ld.LDK_ADD), ("gate_up", f, d, ld.LDK_SWIGLU), ("down", d, f, ld.LDK_ADD)]
        for T in (1056, 2048):
            for name, N, K, epi in mats:
                rows = N * (2 if epi == ld.LDK_SWIGLU else 1)
                W = torch.empty(rows, K, device="cuda").normal_(0, 0.02).bfloat16()
                x = torch.randn(T, K, device="cuda"); y = torch.zeros(T, N, device="cuda")
                scratch = torch.empty(ld.ldk_linear_scratch_bytes(T, N, K, epi), dtype=torch.uint8, device="cuda")
                for _ in range(3):
                    ld.ldk_linear(W, x, y, epi, scratch=scratch)
                torch.cuda.synchronize()
                # the form the engine's passes of 512 rows or more take: one fp16 term
                flag = torch.zeros(1, dtype=torch.int32, device="cuda")
                for _ in range(3):
                    ld.ldk_linear_f16(W, x, y, flag, epi, scratch=scratch)
                torch.cuda.synchronize()
                assert int(flag.item()) == 0
                # the same with the matrix's fp16 image (nothing widened inside the kernel)
                Wh = torch.empty(rows, K, dtype=torch.float16, device="cuda")
                ld.ldk_weights_to_f16(W, Wh, flag)
                for _ in range(3):
                    ld.ldk_linear_f16(W, x, y, flag, epi, scratch=scratch, W_f16=Wh)
                torch.cuda.synchronize()
                assert int(flag.item()) == 0
                del Wh
                out["gemm"].append({"rows": T, "matrix": name, "weight_rows": rows, "K": K,
                                    "nominal_flops": 2 * T * rows * K, "mfma_flops_with_split": 4 * T * rows * K,
                                    "mfma_flops_fp16_rows": 2 * T * rows * K})
        # chunk-prefill attention of a mixed step: four 256-row observations behind long contexts
        segs = [(3001, 256), (5001, 256), (7501, 256), (1201, 256)]
        lens = [p0 + n for p0, n in segs]
        nblk = [-(-n // 16) for n in lens]
        pool = torch.empty(sum(nblk), 2, shape.n_kv_heads, 16, hd, device="cuda").normal_(0, 1).bfloat16()
        table = torch.full((len(segs), max(nblk)), -1, dtype=torch.int32)
        o = 0
        for b in range(len(segs)):
            table[b, :nblk[b]] = torch.arange(o, o + nblk[b], dtype=torch.int32); o += nblk[b]
        table = table.cuda()
        Tq = sum(n for _, n in segs)
        q = torch.randn(Tq, H * hd, device="cuda"); ao = torch.empty(Tq, H * hd, device="cuda")
        tiles, r = [], 0
        for sidx, (p0, n) in enumerate(segs):
            for off in range(0, n, 128):
                tiles.append([r + off, min(128, n - off), p0 + off, sidx])
            r += n
        tiles = torch.tensor(tiles, dtype=torch.int32, device="cuda")
        scratch = torch.empty(ld.ldk_prefill_attention_scratch_bytes(), dtype=torch.uint8, device="cuda")
        for _ in range(3):
            ld.ldk_prefill_attention(q, H * hd, pool, table, tiles, H, shape.n_kv_heads, hd, ao, max(lens) - 1, scratch=scratch)
        torch.cuda.synchronize()
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        for _ in range(3):      # the form of passes of 512 rows or more: q and p as one fp16 term
            ld.ldk_prefill_attention_f16(q, H * hd, pool, table, tiles, H, shape.n_kv_heads, hd, ao, max(lens) - 1, flag, scratch=scratch)
        torch.cuda.synchronize()
        assert int(flag.item()) == 0
        nominal = sum(sum(range(p0 + 1, p0 + n + 1)) for p0, n in segs) * H * hd * 4
        out["attention"] = {"tiles": len(tiles), "rows": Tq, "nominal_flops": nominal, "mfma_flops_with_split": 2 * nominal}
        print(json.dumps(out))
        return
    if args.attention_probe:
        from workloads import gen
        B, H, Hkv, hd = 32, shape.n_heads, shape.n_kv_heads, shape.head_dim
        lens = gen.randint(SEED_BASE + 3, 1, 512, 8192, B).tolist()       # the batch-32 leg's contexts
        nblk = [-(-n // 16) for n in lens]
        pool = torch.empty(sum(nblk), 2, Hkv, 16, hd, device="cuda").normal_(0, 1).bfloat16()
        table = torch.full((B, max(nblk)), -1, dtype=torch.int32)
        o = 0
        for b in range(B):
            table[b, :nblk[b]] = torch.arange(o, o + nblk[b], dtype=torch.int32); o += nblk[b]
        table = table.cuda()
        slot = torch.arange(B, dtype=torch.int32, device="cuda")
        ctx = torch.tensor(lens, dtype=torch.int32, device="cuda")
        q = torch.randn(B, H * hd, device="cuda"); out = torch.empty(B, H * hd, device="cuda")
        scratch = torch.empty(ld.ldk_attention_scratch_bytes(B, H, Hkv, hd, max(lens)), dtype=torch.uint8, device="cuda")
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        b2 = torch.empty_like(a)
        for i in range(8):
            ld.ldk_paged_attention(q, H * hd, pool, table, slot, ctx, max(lens), H, Hkv, hd, out, scratch)
            if i % 2 == 0:
                b2.copy_(a)                  # also evicts the pool from the last-level cache between launches
        torch.cuda.synchronize()
        print(json.dumps({"probe": "decode attention, 7B shape, batch 32, contexts U[512,8192]", "launches": 8,
                          "algorithmic_bytes_per_launch": sum(lens) * 2 * Hkv * hd * 2 + 2 * B * H * hd * 4,
                          "sum_context": sum(lens), "copy_bytes_each_way": 256 << 20, "copies": 4}))
        return
    weights = make_weights(shape, SEED_BASE + 2, device="cuda")
    model = ld.Model(shape, weights, max_chunk=CHUNK)

    if args.calibrate_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        b = torch.empty_like(a)
        for _ in range(4):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    if args.only_batch32:
        print(json.dumps(run_batch32(args, ld, torch, shape, model)))
        return
    res = run_batch1(args, ld, torch, shape, weights, model)
    b32 = None if args.no_batch32 else run_batch32(args, ld, torch, shape, model)
    amb = None if args.no_attention_microbench else run_attention_microbench(args, ld, torch)
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(shape, weights, ctx=1024, steps=160, seed=SEED_BASE + 2)
    # the remaining legs need the memory: drop the 7B decoder first
    import gc
    model.close(); del model, weights
    gc.collect(); torch.cuda.empty_cache()
    gqa = None
    if not args.no_gqa:
        gshape = MISTRAL7B if not args.layers else MISTRAL7B.with_layers(args.layers)
        gweights = make_weights(gshape, SEED_BASE + 5, device="cuda")
        gmodel = ld.Model(gshape, gweights, max_chunk=CHUNK)
        gqa = run_batch32(args, ld, torch, gshape, gmodel)
        gmodel.close(); del gmodel, gweights
        gc.collect(); torch.cuda.empty_cache()
    b13 = None
    if not args.no_13b:
        b13 = run_13b(args, ld, torch)
        gc.collect(); torch.cuda.empty_cache()

    line = {
        "metric": "decode tokens/sec + % peak HBM BW, 7B-shape bf16 at batch 1 and 32, 1 MI355X",
        "value": round(res.pop("value"), 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(res.pop("ms_per_step"), 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "7B-shaped bf16 decoder (32 layers, d 4096, 32x128 heads, FFN 11008, vocab 32000), "
                               "batch 1, tool-call pattern: prompt 1024, rounds of 256 greedy tokens + 128-512-token "
                               "observation via chunked prefill (chunk 256); value = decode steps only",
                   "n_layers": shape.n_layers, "kv_block": 16, "chunk": CHUNK},
        "roofline": res.pop("roofline"),
        "cpu_baseline": cpu,
        "batch1": res,
        "batch32": b32,
        "attention_microbench": amb,
        "gqa_batch32": gqa,
        "13b_batch64": b13,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
