"""Writes tests/golden/cfg5_stair_logits.npz: the oracle's stair logits of the long-context workload (7B-class
target, 8192-token prompt, k = 4) at its real context length, which the oracle needs tens of minutes for and the
GPU test therefore does not compute live.

Calls only the oracle and the seeded input generators.  The prompt is ingested through the oracle's own cached
forward in pieces of 512 rows (a causal forward over a cache is the same function of the sequence however the
rows are grouped; this only bounds the size of the score matrix), then one stair batch of k + 1 = 5 rows with
fixed, seeded draft tokens is scored (Sec. 3.3: the k+1 stair prefixes, here as one causal forward over the
cache).  The oracle runs in float32 and decodes each layer's matrices when it uses them (memory).

    python tests/golden/make_cfg5_logits.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth_inputs as si                       # noqa: E402
from oracle import stairs_oracle as so          # noqa: E402

NAME = "cfg5_7b_longctx_indep_draft"
K = 4
PIECE = 512


def draft_tokens(w):
    rng = np.random.default_rng([w["seed"], 778])
    return rng.integers(0, w["target"]["vocab"], size=K).astype(np.int32)


def main():
    w = si.WORKLOADS[NAME]
    t0 = time.time()
    t = w["target"]
    # the target alone: same tensors as the workload's pair (its draft is an independent model, not needed here)
    target = si.make_model(w["seed"], t["n_layers"], t["d_model"], t["n_heads"], t["d_ffn"], t["vocab"], w["dtype"],
                           deep_from=w["target_deep_from"], deep_scale=w["deep_scale"], threads=8)
    print(f"weights drawn ({time.time() - t0:.0f} s)", flush=True)
    prompt = si.make_prompt(w)
    P = len(prompt)
    T = so.OracleModel(target, np.float32, keep=False)
    cache = so.KVCache.empty(T, P + K + 1)
    for a in range(0, P - 1, PIECE):
        b = min(P - 1, a + PIECE)
        so.forward_cached(T, cache, prompt[a:b], a)
        print(f"rows {a}..{b} ({time.time() - t0:.0f} s)", flush=True)
    d = draft_tokens(w)
    rows = [int(prompt[-1])] + [int(x) for x in d]
    logits = so.forward_cached(T, cache, rows, P - 1)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg5_stair_logits.npz")
    np.savez_compressed(out, logits=logits.astype(np.float32), draft=d, P=np.int32(P))
    print("wrote", out, logits.shape, f"{time.time() - t0:.0f} s")


if __name__ == "__main__":
    main()
