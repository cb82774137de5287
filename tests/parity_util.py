"""Shared driver of the GPU parity tests: runs the HIP library step by step through its C ABI
and the CPU oracle side by side on the same seeded inputs, the oracle teacher-forced onto the
GPU's prefix so that one near-tie does not void the rest of the comparison."""
import numpy as np

import paper_2407_19947_amd as pkg
from oracle import sampling_oracle as sa
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


# ----------------------------------------------------------------------------------------------------------------
# sampling variant: floating point decides integers (argmax of perturbed scores, u < p/q), so the oracle is
# teacher-forced onto the GPU's choices and every choice must be the oracle's own unless the oracle's margin is within
# what the logit differences measured in that iteration allow
# ----------------------------------------------------------------------------------------------------------------
def _draw_ok(scores, pos, stream, key, tok, tol):
    """tok maximises scores + Gumbel noise of (pos, stream) up to tol (tol may be per token)."""
    s = np.asarray(scores, dtype=np.float64) + sa.gumbel(pos, stream, len(scores), key)
    tol = np.broadcast_to(np.asarray(tol, dtype=np.float64), s.shape)
    best = int(np.argmax(s))
    return s[tok] + tol[tok] >= s[best] - tol[best], (tok, best, float(s[tok]), float(s[best]))


def compare_sampled(orc, gpu, P, G, k, temp, seed, logit_tol):
    key = orc.key
    res = dict(n=[], draft_differs=0, decision_differs=0, final_differs=0, max_err=0.0)
    while len(orc.seq) - P < G:
        L = len(orc.seq)
        if k > 0:
            d_gpu, dl_gpu = gpu.propose_sampled(k, temp, seed)
            d_gpu = [int(x) for x in d_gpu]
            d_orc, dl = orc.propose_sampled(k, forced=d_gpu)
            e_d = float(np.max(np.abs(dl_gpu.astype(np.float64) - dl)))
            assert e_d <= logit_tol, f"assistant logits differ by {e_d} at L={L}"
            for j in range(k):
                ok, info = _draw_ok(dl[j] / temp, L + j, sa.STREAM_DRAFT, key, d_gpu[j], 2 * e_d / temp + 1e-9)
                assert ok, f"assistant draw {j} at L={L}: {info}"
                res["draft_differs"] += d_gpu[j] != d_orc[j]
        else:
            d_gpu, dl, e_d = [], np.zeros((0, orc.target.V)), 0.0
        emitted, n, tl_gpu = gpu.verify_sampled(k, temp, seed)
        emitted = [int(x) for x in emitted]
        it = orc.verify_sampled(d_gpu, dl)
        e_t = float(np.max(np.abs(tl_gpu.astype(np.float64) - it.target_logits)))
        assert e_t <= logit_tol, f"stair logits differ by {e_t} at L={L}"
        res["max_err"] = max(res["max_err"], e_t, e_d)
        band = 2 * (e_t + e_d) / temp + 1e-6                 # what log(p/q) can differ by
        assert emitted[:n] == d_gpu[:n] and len(emitted) == n + 1
        if n != it.n_accepted:                               # the first decision that differs must be a near-tie
            i = min(n, it.n_accepted)
            assert abs(np.log(it.uniforms[i]) - np.log(it.ratios[i])) <= band, \
                f"keep/replace decision {i} at L={L}: u={it.uniforms[i]} ratio={it.ratios[i]} band={band}"
            res["decision_differs"] += 1
        for i in range(min(n, it.n_accepted)):               # decisions both made the same way
            assert it.uniforms[i] < it.ratios[i] * np.exp(band)
        # the last emitted token under the oracle's distributions at the GPU's n
        pos = L + n
        if n < k:
            logp = sa.log_softmax(it.target_logits[n] / temp)
            logq = sa.log_softmax(dl[n] / temp)
            p, q = np.exp(logp), np.exp(logq)
            diff = p - q
            slack = p * (2 * e_t / temp) + q * (2 * e_d / temp) + 1e-12      # what p - q can differ by
            scores = np.where(diff > 0, np.log(np.maximum(diff, 1e-300)), -np.inf)
            # a token whose difference is inside the slack may have any score up to log(slack)
            tol = np.where(diff > slack, np.log1p(slack / np.maximum(diff - slack, 1e-300)) + slack / np.maximum(diff, 1e-300), np.inf)
            t = emitted[n]
            if not np.isfinite(tol[t]):
                assert abs(diff[t]) <= 4 * slack[t], f"replacement token {t} at L={L} has no positive mass"
            else:
                ok, info = _draw_ok(scores, pos, sa.STREAM_TARGET, key, t, np.where(np.isfinite(tol), tol, 0.0))
                assert ok, f"replacement draw at L={L}: {info}"
        else:
            ok, info = _draw_ok(it.target_logits[k] / temp, pos, sa.STREAM_TARGET, key, emitted[n], 2 * e_t / temp + 1e-9)
            assert ok, f"extra-token draw at L={L}: {info}"
        if n == it.n_accepted:
            res["final_differs"] += emitted[n] != it.emitted[n]
        orc.adopt(L, emitted)                                # teacher forcing
        res["n"].append(n)
    assert list(gpu.tokens()) == orc.seq
    return res
