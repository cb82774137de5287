"""Pins of the sampling oracle (CPU only): the counter-based generator's statistics, Gumbel-max draws against the
softmax, the keep/replace rule against the distribution it must reproduce and its closed-form keep probability, and the
special cases that reduce to the greedy method."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import sampling_oracle as sa
from oracle import stairs_oracle as so

KEY = sa.key_from_seed(11)


def _chi2_ok(counts, probs, n, sigmas=5.0):
    """Pearson statistic within `sigmas` standard deviations of its mean (dof = cells - 1)."""
    exp = probs * n
    keep = exp > 5
    stat = float(np.sum((counts[keep] - exp[keep]) ** 2 / exp[keep]))
    dof = int(keep.sum()) - 1
    return abs(stat - dof) < sigmas * np.sqrt(2 * dof), (stat, dof)


def test_generator_is_deterministic_uniform_and_streams_differ():
    a = sa.squares32(sa.counters(3, 1, 1000), KEY)
    assert np.array_equal(a, sa.squares32(sa.counters(3, 1, 1000), KEY))
    assert a.max() < 2 ** 32
    for other in (sa.counters(3, 2, 1000), sa.counters(4, 1, 1000)):
        assert np.mean(sa.squares32(other, KEY) == a) < 0.01
    assert np.mean(sa.squares32(sa.counters(3, 1, 1000), sa.key_from_seed(12)) == a) < 0.01
    u = sa.uniform(9, 0, 400000, KEY)
    assert 0.0 < u.min() and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 5 * np.sqrt(1 / 12 / len(u))
    assert abs(u.var() - 1 / 12) < 1e-3
    ok, info = _chi2_ok(np.bincount((u * 64).astype(int), minlength=64), np.full(64, 1 / 64), len(u))
    assert ok, info
    # neighbouring counters are uncorrelated, and so are the same index of neighbouring positions
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.01
    v = np.array([sa.uniform(p, 0, 1, KEY)[0] for p in range(4000)])
    assert abs(np.corrcoef(v[:-1], v[1:])[0, 1]) < 0.06 and abs(v.mean() - 0.5) < 0.03
    # every bit of the output is set about half of the time
    r = sa.squares32(sa.counters(1, 0, 100000), KEY)
    for b in range(32):
        assert abs(np.mean((r >> np.uint64(b)) & np.uint64(1)) - 0.5) < 0.01


def test_generator_arithmetic_in_unbounded_integers():
    """The four squaring rounds redone with Python's unbounded integers reduced mod 2^64 by hand (no fixed-width
    wrap-around to rely on), for counters of every stream and large positions, and the key derivation likewise."""
    M = 1 << 64

    def rot32(x):
        return ((x >> 32) | (x << 32)) % M

    def squares(ctr, key):
        x = (ctr * key) % M
        y = x
        z = (y + key) % M
        x = rot32((x * x + y) % M)
        x = rot32((x * x + z) % M)
        x = rot32((x * x + y) % M)
        return ((x * x + z) % M) >> 32

    for seed in (0, 1, 11, 2 ** 40 + 7):
        z = (seed + 0x9E3779B97F4A7C15) % M
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) % M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) % M
        key = (z ^ (z >> 31)) | 1
        assert sa.key_from_seed(seed) == key
        for pos, stream in ((0, 0), (5, 1), (59999, 2), (123456, 0)):
            ctrs = sa.counters(pos, stream, 50)
            got = sa.squares32(ctrs, key)
            for v in (0, 1, 17, 49):
                ctr = (pos << 34) | (stream << 32) | v
                assert int(ctrs[v]) == ctr
                assert int(got[v]) == squares(ctr, key)


def test_gumbel_max_draws_follow_the_softmax():
    rng = np.random.default_rng(0)
    z = rng.standard_normal(12) * 1.5
    p = np.exp(sa.log_softmax(z))
    n = 60000
    counts = np.bincount([sa.draw(z, pos, sa.STREAM_TARGET, KEY) for pos in range(n)], minlength=12)
    ok, info = _chi2_ok(counts, p, n)
    assert ok, info
    assert np.isclose(np.exp(sa.log_softmax(z)).sum(), 1.0)


def test_residual_scores_are_the_positive_part():
    logp = np.log(np.array([0.5, 0.3, 0.2, 0.0 + 1e-300]))
    logq = np.log(np.array([0.2, 0.3, 0.4, 0.1]))
    r = sa.residual_scores(logp, logq)
    assert np.isclose(np.exp(r[0]), 0.3) and np.all(np.isinf(r[1:])) and np.all(r[1:] < 0)


@pytest.mark.parametrize("k", [1, 3])
def test_emitted_tokens_follow_the_main_model(k):
    """Fixed distributions p_i (main model) and q_j (assistant) over 6 tokens, independent of the prefix: whatever the
    assistant proposes, the first emitted token must be distributed as p_0, and the first proposal must be kept with
    probability sum_v min(p_0(v), q_1(v))."""
    rng = np.random.default_rng(k)
    V, T = 6, 0.7
    tl = rng.standard_normal((k + 1, V)) * 1.2
    dl = rng.standard_normal((k, V)) * 1.2
    p0 = np.exp(sa.log_softmax(tl[0] / T))
    q1 = np.exp(sa.log_softmax(dl[0] / T))
    n_iter = 40000
    first = np.zeros(V, int)
    kept_first = 0
    total_kept = 0
    for it in range(n_iter):
        L = 10 + it * (k + 2)                      # fresh positions = fresh random numbers
        d = [sa.draw(dl[j] / T, L + j, sa.STREAM_DRAFT, KEY) for j in range(k)]
        n, emitted, us, ratios = sa.validate_sampled(L, d, tl, dl, T, KEY)
        assert len(emitted) == n + 1 and emitted[:n] == d[:n] and len(us) == min(n + 1, k)
        first[emitted[0]] += 1
        kept_first += n >= 1
        total_kept += n
    ok, info = _chi2_ok(first, p0, n_iter)
    assert ok, info
    want = float(np.minimum(p0, q1).sum())
    assert abs(kept_first / n_iter - want) < 5 * np.sqrt(want * (1 - want) / n_iter)
    if k == 3:                                     # expected number kept: sum over j of prod_{i<=j} a_i
        a = [float(np.minimum(np.exp(sa.log_softmax(tl[j] / T)), np.exp(sa.log_softmax(dl[j] / T))).sum()) for j in range(k)]
        want_n = a[0] + a[0] * a[1] + a[0] * a[1] * a[2]
        assert abs(total_kept / n_iter - want_n) < 0.03


def _models(G=20):
    w = si.scaled_workload("cfg1_tiny_fp32", G=G)
    t, d = si.make_pair(w)
    return so.OracleModel(t, np.float64), so.OracleModel(d, np.float64), si.make_prompt(w)


def test_identical_assistant_keeps_everything():
    T, D, prompt = _models()
    toks, its = sa.stairs_sampled(T, T, prompt, 20, 4, 0.3, 5)
    assert all(it.n_accepted == 4 for it in its)
    assert all(abs(r - 1.0) < 1e-9 for it in its for r in it.ratios)


def test_cold_sampling_is_the_greedy_method():
    T, D, prompt = _models()
    want = so.greedy_bruteforce(T, prompt, 20)
    for k in (0, 2, 5):
        toks, its = sa.stairs_sampled(T, D, prompt, 20, k, 1e-5, 5)
        assert toks == want
    greedy = so.stairs_cached(T, D, prompt, 20, 5)
    assert [it.n_accepted for it in its] == [it.n_accepted for it in greedy.iterations]


def test_draft_length_zero_is_plain_sampling_and_seeds_matter():
    T, D, prompt = _models()
    temp = 0.05
    toks, its = sa.stairs_sampled(T, None, prompt, 12, 0, temp, 5)
    seq = list(prompt)
    key = sa.key_from_seed(5)
    for _ in range(12):
        z = so.forward_full(T, seq)[-1]
        seq.append(sa.draw(z / temp, len(seq), sa.STREAM_TARGET, key))
    assert toks == seq[len(prompt):]
    other, _ = sa.stairs_sampled(T, None, prompt, 12, 0, temp, 6)
    assert other != toks
    # with an assistant the iterations mix kept and replaced tokens at this temperature
    toks4, its4 = sa.stairs_sampled(T, D, prompt, 40, 4, temp, 5)
    acc = [it.n_accepted for it in its4]
    assert 0 < sum(acc) < 4 * len(acc), acc


def test_fallback_when_nothing_is_left_of_p_minus_q(monkeypatch):
    """A token that is not kept while p - q has no positive entry.  In exact arithmetic this has probability zero (not
    kept means p(d) < q(d), and two distributions cannot differ downwards only); the scheme the paper points to (Sec. 2.2,
    Sec. 5) therefore says nothing about it, and in float64 no honest input reaches it (p == q gives a ratio of
    exactly 1 > u).  The reading: the replacement is drawn from p itself, which is the right distribution when p == q.
    The walk is driven there by substituting a keep/replace uniform of 1."""
    rng = np.random.default_rng(4)
    V, k, L, temp, key = 50, 3, 11, 0.7, sa.key_from_seed(9)
    logits = rng.standard_normal((k + 1, V))
    d = [int(x) for x in rng.integers(0, V, k)]
    real_uniform = sa.uniform

    def fake_uniform(pos, stream, n, key_):
        if stream == sa.STREAM_ACCEPT and pos == L + 1:      # the second proposal is refused whatever its ratio is
            return np.ones(n)
        return real_uniform(pos, stream, n, key_)

    monkeypatch.setattr(sa, "uniform", fake_uniform)
    n, emitted, us, ratios = sa.validate_sampled(L, d, logits, logits[:k], temp, key)     # assistant == main model
    assert n == 1 and emitted[:1] == d[:1] and len(emitted) == 2
    assert ratios == [1.0, 1.0] and us[1] == 1.0
    logp = sa.log_softmax(logits[1] / temp)
    assert not np.any(np.isfinite(sa.residual_scores(logp, logp)))
    assert emitted[1] == sa.draw(logp, L + 1, sa.STREAM_TARGET, key)                    # a draw from p at that position
    # and such draws follow p: over many positions the emitted token's frequencies match (chi-square, 30 cells)
    p = np.exp(sa.log_softmax(logits[0][:30] / temp))
    counts = np.zeros(30)
    N = 6000
    for pos in range(N):
        monkeypatch.setattr(sa, "uniform", lambda ps, st, n_, k_: np.ones(n_) if st == sa.STREAM_ACCEPT else real_uniform(ps, st, n_, k_))
        _, em, _, _ = sa.validate_sampled(pos, [d[0] % 30], logits[:2, :30], logits[:1, :30], temp, key)
        counts[em[0]] += 1
    chi2 = float(np.sum((counts - N * p) ** 2 / (N * p)))
    assert chi2 < 70.0, chi2                                                              # 29 degrees of freedom
