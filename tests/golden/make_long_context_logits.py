"""Writes tests/golden/long_context_logits.npz: the oracle's stair logits at the longest context the library
accepts (max_seq = 60000), which the oracle needs minutes for and the GPU test therefore does not compute live.

Calls only the oracle and the seeded input generators.  The prompt is ingested through the oracle's own cached
forward in pieces of 512 rows (a causal forward over a cache is the same function of the sequence however the
rows are grouped; this only bounds the size of the score matrix), then one stair batch of 32 rows with fixed,
seeded draft tokens is scored (Sec. 3.2: the k+1 stair prefixes as one causal forward).

    python tests/golden/make_long_context_logits.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth_inputs as si                       # noqa: E402
from oracle import stairs_oracle as so          # noqa: E402

MAX_SEQ = 60000
K = 31
P = MAX_SEQ - (K + 1) - 8                       # a few positions short of the end: the batch ends inside the cache


def workload():
    return si.scaled_workload("cfg2_125m", target=dict(n_layers=2, d_model=256, n_heads=2, d_ffn=256, vocab=512),
                              draft=dict(kind="prefix", n_layers=1), P=P, G=1)


def draft_tokens(w):
    rng = np.random.default_rng([w["seed"], 777])
    return rng.integers(0, w["target"]["vocab"], size=K).astype(np.int32)


def main():
    w = workload()
    target, _ = si.make_pair(w)
    prompt = si.make_prompt(w)
    T = so.OracleModel(target, np.float64)
    cache = so.KVCache.empty(T, MAX_SEQ)
    t0 = time.time()
    for a in range(0, P - 1, 512):
        b = min(P - 1, a + 512)
        so.forward_cached(T, cache, prompt[a:b], a)
        if (a // 512) % 16 == 0:
            print(f"rows {a}..{b} ({time.time() - t0:.0f} s)", flush=True)
    d = draft_tokens(w)
    rows = [int(prompt[-1])] + [int(x) for x in d]
    logits = so.forward_cached(T, cache, rows, P - 1)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "long_context_logits.npz")
    np.savez_compressed(out, logits=logits.astype(np.float32), draft=d, P=np.int32(P), max_seq=np.int32(MAX_SEQ))
    print("wrote", out, logits.shape, f"{time.time() - t0:.0f} s")


if __name__ == "__main__":
    main()
