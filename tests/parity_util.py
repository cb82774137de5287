"""Shared driver of the GPU parity tests: runs the HIP library step by step through its C ABI
and the CPU oracle side by side on the same seeded inputs, the oracle teacher-forced onto the
GPU's prefix so that one near-tie does not void the rest of the comparison."""
import numpy as np

import paper_2407_19947_amd as pkg
from oracle import stairs_oracle as so

LOGIT_TOL_BF16 = 2e-2      # spec tolerance: bf16 GPU vs fp32 oracle, absolute, per stair logit
MARGIN_TOL = 2e-2          # a token may differ from the oracle's only where its top-2 margin is below this


def eps_greedy_ok(oracle_row, tok, tol=MARGIN_TOL):
    """tok is an acceptable greedy choice under the oracle's logits."""
    return oracle_row[tok] >= np.max(oracle_row) - tol


def run_side_by_side(target, draft, prompt, G, k, oracle_dtype, logit_tol, check_draft=True, max_iters=None,
                     oracle_keep=True, log=None):
    """Returns dict(max_logit_err, tokens, iterations, n_accepted list, token_mismatches)."""
    T = so.OracleModel(target, oracle_dtype, keep=oracle_keep)
    D = so.OracleModel(draft, oracle_dtype, keep=oracle_keep) if k > 0 else None
    cap = len(prompt) + G + k + 2
    orc = so.CachedStairs(T, D, prompt, cap)
    with pkg.Stairs(target, draft if k > 0 else None, k_max=k, max_seq=cap) as gpu:
        gpu.prefill(prompt)
        return compare_generation(orc, gpu, len(prompt), G, k, logit_tol, check_draft, max_iters, log)


def run_encdec_side_by_side(target, draft, src, G, k, logit_tol, check_draft=True, max_iters=None, log=None,
                            max_src=None):
    """The same comparison with an encoder-decoder pair: the oracle's models are bound to the source sequence, the
    decoder sequence starts with the start token."""
    import synth_inputs as si
    from oracle import encdec_oracle as eo
    T = eo.BoundDecoder(eo.EncDecOracleModel(target), src)
    D = eo.BoundDecoder(eo.EncDecOracleModel(draft), src) if k > 0 else None
    cap = 1 + G + k + 2
    orc = so.CachedStairs(T, D, [si.DECODER_START], cap)
    with pkg.StairsEncDec(target, draft if k > 0 else None, k_max=k, max_src=max_src or len(src), max_seq=cap,
                          start_token=si.DECODER_START) as gpu:
        gpu.encode(src)
        return compare_generation(orc, gpu, 1, G, k, logit_tol, check_draft, max_iters, log)


def compare_generation(orc, gpu, P, G, k, logit_tol, check_draft=True, max_iters=None, log=None):
    """orc: the oracle's CachedStairs after its prompt; gpu: the library's context after prefill / encode."""
    res = dict(max_logit_err=0.0, max_draft_logit_err=None, n_accepted=[], token_mismatches=0, draft_mismatches=0)
    if True:
        iters = 0
        while len(orc.seq) - P < G and (max_iters is None or iters < max_iters):
            L = len(orc.seq)
            d_gpu = [int(x) for x in gpu.propose(k)] if k > 0 else []
            if k > 0 and check_draft:
                dl = []
                orc.propose(k, forced=d_gpu, logits_out=dl)
                for j in range(k):
                    if int(np.argmax(dl[j])) != d_gpu[j]:
                        res["draft_mismatches"] += 1
                    assert eps_greedy_ok(dl[j], d_gpu[j]), \
                        f"draft token {j} at L={L}: gpu {d_gpu[j]} is not within {MARGIN_TOL} of the oracle's best"
            tgt, n, logits = gpu.verify(k, logits=True)
            it = orc.verify(d_gpu)                       # oracle scores the same stair batch
            err = float(np.max(np.abs(logits.astype(np.float64) - it.logits.astype(np.float64))))
            res["max_logit_err"] = max(res["max_logit_err"], err)
            assert err <= logit_tol, f"stair logits differ by {err} > {logit_tol} at L={L}"
            # every emitted token must be an (eps-)greedy choice under the oracle's logits
            for i in range(n + 1):
                if int(tgt[i]) != it.predicted[i]:
                    res["token_mismatches"] += 1
                assert eps_greedy_ok(it.logits[i], int(tgt[i])), \
                    f"target token row {i} at L={L}: gpu {tgt[i]} vs oracle {it.predicted[i]}, margin {so.top2_margin(it.logits[i])}"
            # the acceptance walk itself is integer work: exact given the GPU's own t and d
            assert n == so.count_accepted(d_gpu, [int(x) for x in tgt])
            orc.adopt(L, [int(x) for x in tgt[:n + 1]])   # teacher forcing
            res["n_accepted"].append(n)
            iters += 1
            if log:
                log(f"iter {iters} L={L} n={n} err={err:.3g}")
        seq = gpu.tokens()
        assert list(seq) == orc.seq
    res["tokens"] = orc.seq[P:P + G]
    res["iterations"] = iters
    return res
