"""Writes tests/golden/tiny_fp32_tokens.json: the greedy tokens of workload 0 (2-layer fp32 decoder, prompt of
32 seeded token ids, 64 decoded tokens, KV block 16) as computed by the CPU oracle.  Calls only oracle/ and the
seeded input generators.  Run from the repository root:  python tests/golden/make_tiny_tokens.py"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from workloads import TINY, SEED_BASE, make_weights, gen  # noqa: E402


def compute():
    m = oracle.Model(TINY, make_weights(TINY, SEED_BASE + 0))
    kv = oracle.KV(m, 8, 1, 8)
    rc, s = kv.alloc(0)
    prompt = gen.randint(SEED_BASE, 100, 0, TINY.vocab - 1, 32).numpy().astype(np.int32)
    rc, t, lg = kv.prefill(s, prompt)
    toks, top = [t], [float(lg.max())]
    for _ in range(63):
        rc, t, lg = kv.decode(s)
        toks.append(t); top.append(float(lg.max()))
    return {"source": "oracle/ld_oracle.c via tests/golden/make_tiny_tokens.py; workload 0 of the benchmark definition",
            "seed": SEED_BASE, "prompt": prompt.tolist(), "tokens": toks,
            "max_logit_first_last": [top[0], top[-1]], "block_table": kv.block_table(s)[1].tolist()}


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_fp32_tokens.json")
    with open(out, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", out)
