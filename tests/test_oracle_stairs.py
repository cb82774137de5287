"""Pins for the oracle's generation loops (CPU only): the paper's invariant that stairs-assisted
greedy generation returns what the main model alone would generate (abstract, Sec. 1), the
validation walk of Sec. 3.3 on hand-derived cases, and closed forms for the acceptance counts."""
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import synth_inputs as si
from oracle import stairs_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "stairs_validation_cases.txt")


def _cases():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = [[] if p.strip() == "-" else [int(x) for x in p.split()] for p in line.split("|")]
        out.append(tuple(parts))
    return out


@pytest.mark.parametrize("prefix,draft,pred,truth", _cases())
def test_validation_golden(prefix, draft, pred, truth):
    rows = [prefix + draft[:i] for i in range(len(draft) + 1)]
    assert so.stairs_validate(rows, pred) == truth
    n = so.count_accepted(draft, pred)
    assert prefix + pred[:n + 1] == truth          # the token-level form agrees with the vector walk
    assert 1 <= len(truth) - len(prefix) <= len(draft) + 1


@given(st.lists(st.integers(0, 3), min_size=0, max_size=6), st.data())
@settings(max_examples=200, deadline=None)
def test_validation_bruteforce(draft, data):
    pred = data.draw(st.lists(st.integers(0, 3), min_size=len(draft) + 1, max_size=len(draft) + 1))
    prefix = [1, 2]
    rows = [prefix + draft[:i] for i in range(len(draft) + 1)]
    truth = so.stairs_validate(rows, pred)
    # brute force: the longest n such that d_1..d_n equal t_0..t_{n-1}
    n = max(j for j in range(len(draft) + 1) if draft[:j] == pred[:j])
    assert truth == prefix + pred[:n + 1]


def _pair(seed, deep_scale, L=4, Ld=2, d=32, H=2, f=64, V=50):
    t = si.make_model(seed, L, d, H, f, V, "fp32", deep_from=Ld, deep_scale=deep_scale)
    return t, si.prefix_draft(t, Ld)


@pytest.mark.parametrize("seed,deep_scale", [(7, 0.05), (7, 0.5), (8, 1.0), (9, 0.5)])
@pytest.mark.parametrize("k", [0, 1, 2, 4, 7])
def test_literal_stairs_equals_plain_greedy(seed, deep_scale, k):
    t, d = _pair(seed, deep_scale)
    T, D = so.OracleModel(t, np.float64), so.OracleModel(d, np.float64)
    prompt = [3, 1, 4, 1, 5]
    G = 14
    want = so.greedy_bruteforce(T, prompt, G)
    gen = so.stairs_literal(T, D, prompt, G, k)
    assert gen.tokens == want
    assert len(gen.tokens) == G
    for it in gen.iterations:
        assert 0 <= it.n_accepted <= k
    assert sum(it.n_accepted + 1 for it in gen.iterations) >= G


@given(seed=st.integers(0, 10_000), k=st.integers(0, 5), P=st.integers(1, 6), G=st.integers(1, 10),
       scale=st.sampled_from([0.05, 0.5, 1.0]))
@settings(max_examples=25, deadline=None)
def test_cached_equals_literal_equals_greedy(seed, k, P, G, scale):
    t, d = _pair(seed, scale, L=3, Ld=1, d=16, H=2, f=32, V=24)
    T, D = so.OracleModel(t, np.float64), so.OracleModel(d, np.float64)
    prompt = [int(x) for x in np.random.default_rng(seed).integers(0, 24, P)]
    lit = so.stairs_literal(T, D, prompt, G, k, keep_logits=True)
    ca = so.stairs_cached(T, D if k else None, prompt, G, k, keep_logits=True)
    assert ca.tokens == lit.tokens == so.greedy_bruteforce(T, prompt, G)
    assert len(ca.iterations) == len(lit.iterations)
    for a, b in zip(ca.iterations, lit.iterations):
        assert (a.L, a.draft, a.predicted, a.n_accepted) == (b.L, b.draft, b.predicted, b.n_accepted)
        assert np.allclose(a.logits, b.logits, atol=1e-12)


def test_batch_of_prompts_is_each_prompt_on_its_own():
    """Pin of stairs_batch: for prompts of different lengths every sequence equals brute-force greedy decoding of
    the target on that prompt alone (nothing leaks between sequences)."""
    t, d = _pair(11, 0.05, L=3, Ld=1, d=16, H=2, f=32, V=24)
    T, D = so.OracleModel(t, np.float64), so.OracleModel(d, np.float64)
    prompts = [[3], [5, 1, 7, 2], [23, 0]]
    gens = so.stairs_batch(T, D, prompts, 9, 2)
    assert len(gens) == 3
    for p, g in zip(prompts, gens):
        assert g.tokens == so.greedy_bruteforce(T, p, 9)


def test_adaptive_draft_length_rule_and_invariance():
    """Pins of the adaptive loop: the rule on hand-worked cases; the output is brute-force greedy decoding whatever
    the lengths were; every iteration's length follows from the one before; with a draft identical to the target all
    tokens are kept, so the lengths climb 1, 2, 3, ... to k_max."""
    assert [so.next_draft_length(k, n, 5) for k, n in [(1, 1), (4, 4), (5, 5), (4, 0), (4, 2), (3, 2), (1, 0)]] == \
        [2, 5, 5, 1, 3, 3, 1]
    t, d = _pair(21, 0.05, L=3, Ld=1, d=16, H=2, f=32, V=24)
    T, D = so.OracleModel(t, np.float64), so.OracleModel(d, np.float64)
    prompt = [4, 9, 2]
    gen = so.stairs_adaptive(T, D, prompt, 17, 2, 4)
    assert gen.tokens == so.greedy_bruteforce(T, prompt, 17)
    ks = [len(it.draft) for it in gen.iterations]
    assert ks[0] == 2
    for a, it, b in zip(ks, gen.iterations, ks[1:]):
        assert b == so.next_draft_length(a, it.n_accepted, 4)
    same = so.stairs_adaptive(T, T, prompt, 20, 1, 4)
    assert [len(it.draft) for it in same.iterations][:5] == [1, 2, 3, 4, 4]
    assert all(it.n_accepted == len(it.draft) for it in same.iterations)
    assert same.tokens == so.greedy_bruteforce(T, prompt, 20)


def test_independent_draft_also_returns_plain_greedy():
    t = si.make_model(31, 3, 32, 2, 64, 50, "fp32")
    d = si.make_model(32, 2, 16, 2, 32, 50, "fp32")           # different width, unrelated weights
    T, D = so.OracleModel(t, np.float64), so.OracleModel(d, np.float64)
    prompt = [9, 8, 7]
    want = so.greedy_bruteforce(T, prompt, 12)
    assert so.stairs_literal(T, D, prompt, 12, 3).tokens == want
    assert so.stairs_cached(T, D, prompt, 12, 3).tokens == want


@pytest.mark.parametrize("k,G", [(1, 9), (3, 12), (3, 13), (4, 5)])
def test_draft_identical_to_target_accepts_everything(k, G):
    """Assistant == main model: every iteration keeps k assistant tokens, so the number of
    main-model iterations is ceil(G / (k+1))."""
    t, _ = _pair(13, 1.0)
    T = so.OracleModel(t, np.float64)
    for fn in (so.stairs_literal, so.stairs_cached):
        gen = fn(T, T, [2, 7, 1], G, k)
        assert all(it.n_accepted == k for it in gen.iterations)
        assert len(gen.iterations) == -(-G // (k + 1))
        assert gen.tokens == so.greedy_bruteforce(T, [2, 7, 1], G)


def test_adversarial_draft_accepts_nothing():
    """Assistant tokens forced to differ from the main model's prediction: n = 0 every time, so
    the number of iterations equals G and the output is still plain greedy."""
    t, d = _pair(14, 0.5)
    T, D = so.OracleModel(t, np.float64), so.OracleModel(d, np.float64)
    prompt, G, k = [5, 6], 7, 3
    want = so.greedy_bruteforce(T, prompt, G)
    st_ = so.CachedStairs(T, D, prompt, 32)
    iters = 0
    while len(st_.seq) - st_.P < G:
        nxt = want[len(st_.seq) - st_.P]
        bad = [(nxt + 1) % 50] + [0] * (k - 1)
        it = st_.verify(bad)
        assert it.n_accepted == 0 and it.predicted[0] == nxt
        iters += 1
    assert iters == G and st_.seq[st_.P:] == want


def test_generation_is_truncated_to_G():
    t, _ = _pair(15, 1.0)
    T = so.OracleModel(t, np.float64)
    gen = so.stairs_cached(T, T, [1, 2, 3], 5, 3)             # 2 iterations produce 8, keep 5
    assert len(gen.tokens) == 5 and len(gen.iterations) == 2


def test_top2_margin():
    assert so.top2_margin(np.array([0.1, 3.0, 2.5, -1.0])) == pytest.approx(0.5)
    assert so.greedy_token(np.array([1.0, 7.0, 7.0])) == 1     # ties -> lowest index


# ----------------------------------------------------------------------------------------------------------------
# the teacher-forcing hooks the GPU parity tests lean on: CachedStairs.propose(forced=) and .adopt
# ----------------------------------------------------------------------------------------------------------------
def _hook_models():
    w = si.scaled_workload("cfg1_tiny_fp32", target=dict(n_layers=3, d_model=64, n_heads=2, d_ffn=128, vocab=96),
                           draft=dict(kind="prefix", n_layers=1), deep_scale=0.3, P=7, G=20)
    target, draft = si.make_pair(w)
    return so.OracleModel(target, np.float64), so.OracleModel(draft, np.float64), [int(x) for x in si.make_prompt(w)]


def test_forcing_the_oracles_own_choices_changes_nothing():
    T, D, prompt = _hook_models()
    k, G = 3, 18
    free = so.CachedStairs(T, D, prompt, len(prompt) + G + k + 2).run(G, k, keep_logits=True)
    st = so.CachedStairs(T, D, prompt, len(prompt) + G + k + 2)
    for it in free.iterations:
        L = len(st.seq)
        assert L == it.L
        d = st.propose(k, forced=it.draft)
        assert d == it.draft
        got = st.verify(d)
        assert got.predicted == it.predicted and got.n_accepted == it.n_accepted
        assert np.array_equal(got.logits, it.logits)
        st.adopt(L, it.predicted[:it.n_accepted + 1])          # adopting its own result again is the identity
    assert st.seq[len(prompt):len(prompt) + G] == free.tokens


def test_forced_tokens_are_what_the_assistant_is_fed():
    """With forced tokens f_1..f_k the j-th logits row is the assistant's distribution after seq + f_1..f_{j-1}
    (a plain full forward), whatever the oracle itself would have chosen."""
    T, D, prompt = _hook_models()
    k = 4
    st = so.CachedStairs(T, D, prompt, len(prompt) + 3 * (k + 1) + 2)
    rng = np.random.default_rng(0)
    seq = list(prompt)
    for _ in range(2):
        L = len(st.seq)
        forced = [int(x) for x in rng.integers(0, T.V, k)]
        rows = []
        own = st.propose(k, forced=forced, logits_out=rows)
        assert len(rows) == k
        for j in range(k):
            want = so.forward_full(D, st.seq + forced[:j])[-1]
            assert np.allclose(rows[j], want, atol=1e-10)
            assert own[j] == int(np.argmax(want))
        # the main model scores the forced tokens; the test adopts a SHORTER stair path than the oracle's own walk
        it = st.verify(forced)
        want = so.forward_full(T, st.seq[:L] + forced)[L - 1:]
        assert np.allclose(it.logits, want, atol=1e-10)
        st.adopt(L, it.predicted[:1])
        seq = seq + it.predicted[:1]
        assert st.seq == seq
        assert st.tc.length == L and st.dc.length <= L


def test_adopting_another_path_keeps_the_caches_consistent():
    """After adopt() onto tokens another implementation accepted (here: fewer than the oracle's own walk kept), the next
    stair batch's logits are those of a full forward over the adopted sequence: the cache rows beyond it are dead."""
    T, D, prompt = _hook_models()
    k = 3
    st = so.CachedStairs(T, T, prompt, len(prompt) + 40)           # assistant == main model: everything is accepted
    seq = list(prompt)
    for cut in (0, 2, 1, 3):
        L = len(st.seq)
        d = st.propose(k)
        it = st.verify(d)
        assert it.n_accepted == k
        st.adopt(L, it.predicted[:cut + 1])                         # keep only `cut` assistant tokens
        seq = seq + it.predicted[:cut + 1]
        assert st.seq == seq
        d2 = st.propose(k)
        full = so.forward_full(T, seq + d2)
        assert d2 == [int(np.argmax(full[len(seq) - 1 + j])) for j in range(k)]   # the assistant's cache is consistent too
        it2 = st.verify(d2)
        assert np.allclose(it2.logits, full[len(seq) - 1:], atol=1e-10)
        seq = st.seq


# ---- end token (Sec. 3.2, last sentence: the cycle runs until the answer is complete) -------------------------
def test_cut_after_end_token_hand_cases():
    assert so.cut_after_end_token([5, 6, 7], None) == ([5, 6, 7], False)
    assert so.cut_after_end_token([5, 6, 7], 9) == ([5, 6, 7], False)
    assert so.cut_after_end_token([5, 6, 7], 5) == ([5], True)
    assert so.cut_after_end_token([5, 6, 7], 6) == ([5, 6], True)
    assert so.cut_after_end_token([5, 6, 6], 6) == ([5, 6], True)          # the first one ends the answer
    assert so.cut_after_end_token([7], 7) == ([7], True)


def _first_index(tokens, tok):
    return list(tokens).index(tok)


@pytest.mark.parametrize("seed,deep_scale", [(7, 0.05), (8, 1.0)])
def test_greedy_with_an_end_token_is_the_plain_output_cut_after_it(seed, deep_scale):
    t, _ = _pair(seed, deep_scale)
    T = so.OracleModel(t, np.float64)
    prompt = [3, 1, 4, 1, 5]
    full = so.greedy_bruteforce(T, prompt, 16)
    for j in (0, 5, 15):
        eos = full[j]
        cut = _first_index(full, eos) + 1                                  # the token may occur earlier than j
        assert so.greedy_bruteforce(T, prompt, 16, eos=eos) == full[:cut]
    absent = next(v for v in range(50) if v not in full)
    assert so.greedy_bruteforce(T, prompt, 16, eos=absent) == full


@pytest.mark.parametrize("k", [0, 1, 3, 6])
@pytest.mark.parametrize("seed,deep_scale", [(7, 0.05), (7, 0.5), (9, 1.0)])
def test_stairs_with_an_end_token_equals_greedy_with_it(seed, deep_scale, k):
    """Literal and cached loops stop where stand-alone greedy decoding stops, wherever the end token falls inside an
    iteration (first emitted token, an accepted assistant token, the last prediction) and when G comes first."""
    t, d = _pair(seed, deep_scale)
    T, D = so.OracleModel(t, np.float64), so.OracleModel(d, np.float64)
    prompt = [2, 7, 1, 8]
    G = 13
    full = so.greedy_bruteforce(T, prompt, G)
    for j in range(0, G, 2):
        eos = full[j]
        want = so.greedy_bruteforce(T, prompt, G, eos=eos)
        assert want[-1] == eos and eos not in want[:-1]
        lit = so.stairs_literal(T, D, prompt, G, k, eos=eos)
        assert lit.tokens == want
        st_ = so.CachedStairs(T, D if k else None, prompt, len(prompt) + G + k + 2)
        gen = st_.run(G, k, eos=eos)
        assert gen.tokens == want
        assert st_.seq == prompt + want                                    # nothing after the end token is kept
        assert st_.tc.length <= len(st_.seq) - 1                           # and the cache holds no row of it
        assert len(gen.iterations) == len(lit.iterations)
    # an end token that comes after G: the length limit wins
    late = so.greedy_bruteforce(T, prompt, G + 6)
    cand = [x for x in late[G:] if x not in late[:G]]
    if cand:
        assert so.stairs_cached(T, D if k else None, prompt, G, k, eos=cand[0]).tokens == full


def test_continuing_after_an_end_token_continues_the_plain_sequence():
    """The stop only cuts; the state left behind is the sequence up to the end token, from which the loop goes on as
    plain greedy decoding would (the check the GPU library's rollback is held to)."""
    t, d = _pair(7, 0.5)
    T, D = so.OracleModel(t, np.float64), so.OracleModel(d, np.float64)
    prompt = [3, 1, 4, 1, 5]
    full = so.greedy_bruteforce(T, prompt, 20)
    eos = full[6]
    cut = _first_index(full, eos) + 1
    st_ = so.CachedStairs(T, D, prompt, 64)
    assert st_.run(20, 4, eos=eos).tokens == full[:cut]
    st_.P = len(st_.seq)
    assert st_.run(20 - cut, 4).tokens == full[cut:]


def test_batch_with_an_end_token_is_each_prompt_on_its_own():
    t, d = _pair(8, 0.5)
    T, D = so.OracleModel(t, np.float64), so.OracleModel(d, np.float64)
    prompts = [[3, 1, 4], [1, 5, 9, 2], [6, 5]]
    eos = so.greedy_bruteforce(T, prompts[0], 10)[4]
    gens = so.stairs_batch(T, D, prompts, 10, 2, eos=eos)
    for p, g in zip(prompts, gens):
        assert g.tokens == so.greedy_bruteforce(T, p, 10, eos=eos)
