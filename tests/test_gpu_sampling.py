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
from parity_util import LOGIT_TOL_BF16, compare_sampled

pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)


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


def test_widest_sampled_stair_batch():
    """k = 31: 32 stair rows, 31 assistant logits rows, 63 log-sum-exps."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=24, G=66)
    res = _run(w, 31, 0.05, 9, 66)
    assert res["max_err"] < 5e-3 and max(res["n"]) > 0


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
    with pkg.Stairs(target, draft, k_max=3, max_seq=64) as s:
        s.reserve_batch(2)                                           # sampling takes one sequence per context
        with pytest.raises(pkg.StairsError) as e:
            s.generate_sampled(prompt, 8, 2, 0.5, 1)
        assert e.value.code == -1
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
