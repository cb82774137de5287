"""GPU parity of the sampling variant: draws, keep / replace decisions and emitted tokens of the HIP library against
the CPU oracle on the same seeded inputs and the same counter-based random numbers.  Floating point decides integers
here (argmax of perturbed scores, u < p/q), so the oracle is teacher-forced onto the GPU's choices and every choice
must be the oracle's own unless the oracle's margin is within what the measured logit differences allow."""
import numpy as np
import pytest

import paper_2407_19947_amd as pkg
import synth_inputs as si
from oracle import sampling_oracle as sa
from oracle import stairs_oracle as so
from parity_util import LOGIT_TOL_BF16

pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)


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


def _run(workload, k, temp, seed, G, oracle_dtype=np.float64, logit_tol=LOGIT_TOL_BF16):
    target, draft = si.make_pair(workload)
    prompt = si.make_prompt(workload)
    T = so.OracleModel(target, oracle_dtype)
    D = so.OracleModel(draft, oracle_dtype) if k > 0 else None
    cap = len(prompt) + G + k + 2
    orc = sa.SampledStairs(T, D, prompt, cap, temp, seed)
    with pkg.Stairs(target, draft if k > 0 else None, k_max=k, max_seq=cap) as gpu:
        gpu.prefill(prompt)
        res = compare_sampled(orc, gpu, len(prompt), G, k, temp, seed, logit_tol)
    _log(f"  k={k} T={temp}: kept {res['n']}, max logit err {res['max_err']:.3g}, differing draws "
         f"{res['draft_differs']}/{res['final_differs']}, near-tie decisions {res['decision_differs']}")
    return res


@pytest.mark.parametrize("k,temp", [(0, 0.05), (1, 0.05), (4, 0.05), (4, 0.02), (7, 0.1), (4, 1.0)])
def test_fp32_pair_sampled(k, temp):
    w = si.scaled_workload("cfg1_tiny_fp32", G=48)
    res = _run(w, k, temp, 17, 48, logit_tol=2e-4)
    assert res["draft_differs"] == 0 and res["final_differs"] == 0 and res["decision_differs"] == 0
    if k == 4 and temp == 0.05:
        assert 0 < sum(res["n"]) < 4 * len(res["n"])        # both outcomes of the walk occur


@pytest.mark.parametrize("k,temp", [(0, 0.1), (3, 0.1), (5, 0.03)])
def test_bf16_pair_sampled(k, temp):
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=3, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=40, G=40)
    res = _run(w, k, temp, 5, 40)
    assert res["max_err"] < 5e-3
    assert res["draft_differs"] + res["final_differs"] + res["decision_differs"] <= 2


def test_sampled_generation_properties(monkeypatch):
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=3, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=40, G=64)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    with pkg.Stairs(target, draft, k_max=6, max_seq=160) as s:
        greedy, _ = s.generate(prompt, 64, 3)
        cold, st = s.generate_sampled(prompt, 64, 3, 1e-4, 1)      # temperature -> 0: the greedy output
        assert np.array_equal(cold, greedy)
        a, sta = s.generate_sampled(prompt, 64, 3, 0.1, 1)
        b, _ = s.generate_sampled(prompt, 64, 3, 0.1, 1)
        assert np.array_equal(a, b)                                  # same seed, same run
        c, _ = s.generate_sampled(prompt, 64, 3, 0.1, 2)
        assert not np.array_equal(a, c)
        assert not np.array_equal(a, greedy)
        assert sta.iterations < 64 and sum(sta.accept_hist[1:4]) > 0
        # the draft equal to the target keeps everything
    with pkg.Stairs(target, target, k_max=4, max_seq=160) as s:
        toks, st = s.generate_sampled(prompt, 60, 4, 0.1, 3)
        assert st.accept_hist[4] == st.iterations
        plain, _ = s.generate_sampled(prompt, 60, 0, 0.1, 3)
        assert len(plain) == 60
    monkeypatch.setenv("STAIRS_NO_GRAPH", "1")
    with pkg.Stairs(target, draft, k_max=6, max_seq=160) as s:
        eager, _ = s.generate_sampled(prompt, 64, 3, 0.1, 1)
    assert np.array_equal(eager, a)                                  # graph replay == one-by-one launches


def test_sampled_errors_and_encoder_decoder_context():
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=20, G=16)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    with pkg.Stairs(target, draft, k_max=3, max_seq=64) as s:
        with pytest.raises(pkg.StairsError) as e:
            s.generate_sampled(prompt, 16, 2, 0.0, 1)
        assert e.value.code == -1
        s.prefill(prompt)
        s.propose(2)                                                 # a greedy proposal is pending
        with pytest.raises(pkg.StairsError) as e:
            s.verify_sampled(2, 0.5, 1, logits=False)
        assert e.value.code == -3
    we = si.scaled_encdec_workload("t5_tiny")
    t, d = si.make_encdec_pair(we)
    src = si.make_source(we)
    with pkg.StairsEncDec(t, d, k_max=4, max_src=64, max_seq=64) as s:
        s.encode(src)
        greedy, _ = s.decode(32, 3)
        s.encode(src)
        cold, _ = s.decode_sampled(32, 3, 1e-5, 9)
        assert np.array_equal(cold, greedy)
        s.encode(src)
        warm, st = s.decode_sampled(32, 3, 0.2, 9)
        s.encode(src)
        again, _ = s.decode_sampled(32, 3, 0.2, 9)
        assert np.array_equal(warm, again) and not np.array_equal(warm, greedy)
