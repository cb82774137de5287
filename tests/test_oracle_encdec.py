"""Pins of the encoder-decoder oracle (CPU only): the relative-position bucket rule against hand-computed values
and exact integer arithmetic, attention against PyTorch's library routine, structural invariants of the model, and
the stairs == greedy invariant with an encoder-decoder target."""
import os

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import encdec_oracle as eo
from oracle import stairs_oracle as so

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "relative_position_buckets.txt")


def _tiny(**over):
    w = si.scaled_encdec_workload("t5_tiny", **over)
    t, d = si.make_encdec_pair(w)
    return w, t, d, si.make_source(w)


def _clone(t):
    """Copy of a model's inputs whose per-layer dicts and tables can be replaced without touching the original."""
    import copy
    c = copy.copy(t)
    c.enc_layers = [dict(l) for l in t.enc_layers]
    c.dec_layers = [dict(l) for l in t.dec_layers]
    return c


def test_hand_computed_buckets():
    n = 0
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if not line:
            continue
        mode, rel, want = line[0], int(line[1]), int(line[2])
        got = int(eo.relative_position_bucket(np.array([rel]), mode == "two", 32, 128)[0])
        assert got == want, (mode, rel, got, want)
        n += 1
    assert n >= 25


@pytest.mark.parametrize("buckets,maxd", [(32, 128), (16, 64), (64, 256)])
def test_bucket_rule_in_exact_integer_arithmetic(buckets, maxd):
    """floor(log(n/E)/log(D/E)*Q) = j  <=>  (D/E)^j <= (n/E)^Q < (D/E)^(j+1), checked with big integers."""
    for bidir in (True, False):
        side = buckets // 2 if bidir else buckets
        E, Q = side // 2, side - side // 2
        n = np.arange(0, 4 * maxd)
        got = eo.relative_position_bucket(-n, bidir, buckets, maxd)
        for ni, b in zip(n.tolist(), got.tolist()):
            if ni < E:
                assert b == ni
                continue
            j = 0
            while (ni ** Q) * (E ** (j + 1)) >= (maxd ** (j + 1)) * (E ** Q):   # (n/E)^Q >= (D/E)^(j+1)
                j += 1
            assert b == min(E + j, side - 1), (bidir, ni, b, j)
        # keys after the query: upper half (two-sided) or distance 0 (one-sided)
        after = eo.relative_position_bucket(n, bidir, buckets, maxd)
        if bidir:
            assert np.array_equal(after[1:], got[1:] + side) and after[0] == 0
        else:
            assert np.all(after == 0)
        # every bucket is used, except the two-sided rule's first upper one (distance 0 is never 'after')
        assert len(set(got.tolist()) | set(after.tolist())) == buckets - (1 if bidir else 0)
        assert np.all(np.diff(got) >= 0)


def test_attention_against_library_routine():
    rng = np.random.default_rng(5)
    M, T, H, hd = 5, 11, 3, 8
    q, k, v = (rng.standard_normal((n, H, hd)) for n in (M, T, T))
    bias = rng.standard_normal((H, M, T))
    hidden = np.arange(T)[None, :] > (T - M + np.arange(M))[:, None]
    got = eo.biased_attention(q, k, v, bias, hidden)
    mask = torch.from_numpy(np.where(hidden[None], -np.inf, bias))
    tq, tk, tv = (torch.from_numpy(np.transpose(a, (1, 0, 2))) for a in (q, k, v))
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=1.0)
    assert np.allclose(got, np.transpose(want.numpy(), (1, 0, 2)), atol=1e-12)
    # no bias, no mask
    got = eo.biased_attention(q, k, v, None, None)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=1.0)
    assert np.allclose(got, np.transpose(want.numpy(), (1, 0, 2)), atol=1e-12)


def test_position_bias_layout():
    table = np.arange(32 * 2, dtype=np.float64).reshape(32, 2)
    b = eo.position_bias(table, np.array([3, 4]), np.arange(6), False, 128)
    assert b.shape == (2, 2, 6)
    assert b[1, 0, 1] == table[2, 1]          # query 3, key 1: distance 2
    assert b[0, 1, 5] == table[0, 0]          # key after the query
    b = eo.position_bias(table, np.arange(4), np.arange(4), True, 128)
    assert b[1, 0, 3] == table[16 + 3, 1] and b[1, 3, 0] == table[3, 1]


def test_feed_forward_against_library_routine():
    w, t, d, src = _tiny()
    m = eo.EncDecOracleModel(t)
    x = np.random.default_rng(1).standard_normal((4, t.d_model))
    got = m.ffn("dec", 1, x)
    tx = torch.from_numpy(x)
    g = torch.from_numpy(m.w("dec", 1, "ffn_norm"))
    h = tx * torch.rsqrt(tx.pow(2).mean(-1, keepdim=True) + t.rms_eps) * g
    want = tx + torch.nn.functional.linear(torch.relu(torch.nn.functional.linear(h, torch.from_numpy(m.w("dec", 1, "w_in")))),
                                           torch.from_numpy(m.w("dec", 1, "w_out")))
    assert np.allclose(got, want.numpy(), atol=1e-12)


def test_source_order_only_matters_through_the_bias():
    """Without position bias the encoder is permutation-equivariant and cross-attention permutation-invariant: a
    shuffled source gives the same decoder logits.  With the bias it must not."""
    w, t, d, src = _tiny()
    perm = np.random.default_rng(2).permutation(len(src))
    ids = [0, 5, 9, 11]
    for zero in (True, False):
        tt = _clone(t)
        if zero:
            tt.enc_rel_bias = np.zeros_like(tt.enc_rel_bias)
        m = eo.EncDecOracleModel(tt)
        a = so.forward_full(eo.BoundDecoder(m, src), ids)
        b = so.forward_full(eo.BoundDecoder(m, src[perm]), ids)
        if zero:
            assert np.allclose(a, b, atol=1e-10)
        else:
            assert np.max(np.abs(a - b)) > 1e-4


def test_single_source_token_makes_cross_queries_irrelevant():
    """One source position: every cross-attention row is that position's value vector whatever the query is."""
    w, t, d, src = _tiny()
    ids = [0, 7, 3]
    a = so.forward_full(eo.BoundDecoder(eo.EncDecOracleModel(t), src[:1]), ids)
    t2 = _clone(t)
    for l in range(t2.n_dec_layers):
        t2.dec_layers[l]["cq"] = t2.dec_layers[l]["wq"]
    b = so.forward_full(eo.BoundDecoder(eo.EncDecOracleModel(t2), src[:1]), ids)
    assert np.allclose(a, b, atol=1e-12)
    c = so.forward_full(eo.BoundDecoder(eo.EncDecOracleModel(t), src[:2]), ids)
    assert np.max(np.abs(a - c)) > 1e-6


def test_decoder_is_causal_and_cache_equals_no_cache():
    w, t, d, src = _tiny()
    T = eo.BoundDecoder(eo.EncDecOracleModel(t), src)
    ids = [0] + list(np.random.default_rng(3).integers(1, t.vocab, 20))
    full = so.forward_full(T, ids)
    other = ids[:12] + [1, 2, 3, 4, 5, 6, 7, 8, 9]
    assert np.allclose(full[:12], so.forward_full(T, other)[:12], atol=1e-12)      # later tokens do not reach back
    assert np.max(np.abs(full[12:] - so.forward_full(T, other)[12:])) > 1e-6
    cache = so.KVCache.empty(T, 32)
    parts = [so.forward_cached(T, cache, ids[a:b], a) for a, b in ((0, 1), (1, 8), (8, 9), (9, 21))]
    assert np.allclose(np.concatenate(parts), full, atol=1e-10)


def test_decoder_bias_reaches_the_scores():
    w, t, d, src = _tiny()
    ids = [0, 4, 8, 15, 16, 23, 42]
    a = so.forward_full(eo.BoundDecoder(eo.EncDecOracleModel(t), src), ids)
    t2 = _clone(t)
    t2.dec_rel_bias = np.zeros_like(t2.dec_rel_bias)
    b = so.forward_full(eo.BoundDecoder(eo.EncDecOracleModel(t2), src), ids)
    assert np.allclose(a[0], b[0], atol=1e-12)            # a single key: the bias cancels in the softmax
    assert np.max(np.abs(a[1:] - b[1:])) > 1e-5


@pytest.mark.parametrize("k", [1, 3, 6])
def test_stairs_equals_greedy_with_an_encoder_decoder_target(k):
    w, t, d, src = _tiny()
    T = eo.BoundDecoder(eo.EncDecOracleModel(t), src)
    D = eo.BoundDecoder(eo.EncDecOracleModel(d), src)
    G = 24
    want = so.greedy_bruteforce(T, [si.DECODER_START], G)
    cached = so.stairs_cached(T, D, [si.DECODER_START], G, k)
    assert cached.tokens == want
    assert so.stairs_literal(T, D, [si.DECODER_START], G, k).tokens == want
    acc = [it.n_accepted for it in cached.iterations]
    assert len(set(want)) > G // 3 and 0 < sum(acc) < k * len(acc)       # neither degenerate nor trivial


def test_independent_draft_and_wide_attention():
    """Draft with its own weights and shape; attention width n_heads * head_dim != d_model in the target."""
    w = si.scaled_encdec_workload("t5_tiny", target=dict(n_enc_layers=2, n_dec_layers=2, d_model=256, n_heads=4, head_dim=128),
                                  draft=dict(kind="independent", seed=77, n_enc_layers=1, n_dec_layers=1, d_model=256,
                                             n_heads=2, head_dim=64, d_ffn=256))
    t, d = si.make_encdec_pair(w)
    assert t.d_attn == 512 and d.d_attn == 128
    src = si.make_source(w)
    T = eo.BoundDecoder(eo.EncDecOracleModel(t), src)
    D = eo.BoundDecoder(eo.EncDecOracleModel(d), src)
    assert so.stairs_cached(T, D, [0], 12, 3).tokens == so.greedy_bruteforce(T, [0], 12)
