"""GPU tests of the end-token stop of the generation loops (Sec. 3.2, last sentence: the cycle runs until the answer
is complete): against the oracle's loops with the same end token, and against the library's own unlimited output."""
import numpy as np
import pytest

import paper_2407_19947_amd as pkg
import synth_inputs as si
from oracle import stairs_oracle as so

pytestmark = pytest.mark.gpu


def _cut(full, eos):
    full = [int(x) for x in full]
    return full[:full.index(eos) + 1] if eos in full else full


def test_fp32_pair_stops_where_the_oracle_stops():
    """fp32 pair (the GPU's tokens equal the oracle's exactly): for end tokens that fall on the first emitted token
    of an iteration, on an accepted assistant token and on the last prediction, every k gives the oracle's answer."""
    w = si.WORKLOADS["cfg1_tiny_fp32"]
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    T, D = so.OracleModel(target, np.float64), so.OracleModel(draft, np.float64)
    G = 40
    full = so.greedy_bruteforce(T, prompt, G)
    with pkg.Stairs(target, draft, k_max=8, max_seq=len(prompt) + G + 16) as s:
        base, _ = s.generate(prompt, G, 0)
        assert [int(x) for x in base] == full
        for j in (0, 1, 7, 18, 39):
            eos = full[j]
            want = so.greedy_bruteforce(T, prompt, G, eos=eos)
            s.set_eos(eos)
            for k in (0, 1, 3, 8):
                toks, st = s.generate(prompt, G, k)
                oracle = so.stairs_cached(T, D if k else None, prompt, G, k, eos=eos)
                assert oracle.tokens == want
                assert st.tokens == len(want), (j, k)
                assert [int(x) for x in toks[:st.tokens]] == want, (j, k)
                assert all(int(x) == eos for x in toks[st.tokens:])            # the rest is filled with the end token
                assert st.iterations == len(oracle.iterations), (j, k)
                assert [int(x) for x in s.tokens()] == [int(x) for x in prompt] + want   # nothing kept after it
            s.set_eos(-1)
            toks, st = s.generate(prompt, G, 3)
            assert st.tokens == G and [int(x) for x in toks] == full


def test_bf16_stop_is_the_unlimited_output_cut_and_generation_can_go_on():
    """bf16 pair: the stopped output is the library's own unlimited output cut after the end token (graph replay
    and one-by-one launches), and after the stop the context continues as the unlimited run did: the rollback left
    exactly the sequence up to the end token in both caches."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=4, d_model=256, n_heads=4, d_ffn=768, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=70, G=48)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    G = w["G"]
    with pkg.Stairs(target, draft, k_max=6, max_seq=256) as s:
        full, _ = s.generate(prompt, G, 0)
        full = [int(x) for x in full]
        for j in (3, 20, 33):
            eos = full[j]
            want = _cut(full, eos)
            for k in (2, 5):
                s.set_eos(eos)
                toks, st = s.generate(prompt, G, k)
                assert st.tokens == len(want) and [int(x) for x in toks[:st.tokens]] == want, (j, k)
                s.set_eos(-1)
                more, st2 = s.decode(G - len(want), k)
                assert [int(x) for x in more] == full[len(want):], (j, k)
        # adaptive draft length and the sampled loop at T -> 0 stop at the same place
        eos = full[11]
        want = _cut(full, eos)
        s.set_eos(eos)
        s.prefill(prompt)
        toks, st = s.decode_adaptive(G, 2)
        assert [int(x) for x in toks[:st.tokens]] == want
        with pytest.raises(pkg.StairsError):
            s.set_eos(2048)
        with pytest.raises(pkg.StairsError):
            s.set_eos(-2)


def test_batch_sequences_stop_one_by_one():
    """Several sequences per forward: each stops at its own end token (or at G), the others go on unchanged."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=3, d_model=256, n_heads=4, d_ffn=768, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=40, G=32)
    target, draft = si.make_pair(w)
    rng = np.random.default_rng([w["seed"], 91])
    prompts = [rng.integers(0, 2048, n).astype(np.int32) for n in (40, 7, 65, 33)]
    G, k = 32, 3
    with pkg.Stairs(target, draft, k_max=4, max_seq=160) as s:
        s.reserve_batch(4)
        full, st0 = s.generate_batch(prompts, G, k)
        assert st0.tokens == 4 * G
        # an end token that sequence 0 emits early, sequence 2 late, the others possibly never
        eos = int(full[0][5])
        s.set_eos(eos)
        toks, st = s.generate_batch(prompts, G, k)
        total = 0
        for b in range(4):
            want = _cut(full[b], eos)
            total += len(want)
            assert [int(x) for x in toks[b][:len(want)]] == want, b
            assert all(int(x) == eos for x in toks[b][len(want):]), b
        assert st.tokens == total and total < 4 * G
        s.set_eos(-1)
        again, _ = s.generate_batch(prompts, G, k)
        assert np.array_equal(again, full)


def test_encoder_decoder_context_stops_at_the_end_token():
    """The paper's model family ends its answers with an end-of-sequence id; the encoder-decoder loop is the same
    loop and stops the same way: the unlimited output cut after the end token, for every draft length."""
    w = si.scaled_encdec_workload("t5_tiny")
    t, d = si.make_encdec_pair(w)
    src = si.make_source(w)
    G = 40
    with pkg.StairsEncDec(t, d, k_max=5, max_src=len(src), max_seq=G + 16, start_token=si.DECODER_START) as s:
        full, _ = s.generate(src, G, 0)
        full = [int(x) for x in full]
        for j in (2, 17):
            eos = full[j]
            want = _cut(full, eos)
            s.set_eos(eos)
            for k in (0, 2, 5):
                toks, st = s.generate(src, G, k)
                assert st.tokens == len(want) and [int(x) for x in toks[:st.tokens]] == want, (j, k)
        s.set_eos(-1)
        toks, st = s.generate(src, G, 5)
        assert st.tokens == G and [int(x) for x in toks] == full
