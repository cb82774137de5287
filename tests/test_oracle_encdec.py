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


# ----------------------------------------------------------------------------------------------------------------
# the composition of the blocks (which norm feeds which projection, where the residuals are added, the encoder's final
# norm in front of the cross-attention keys and values): the whole model again out of PyTorch library routines, with a
# different gain vector on every norm so that a misplaced or missing one changes the result
# ----------------------------------------------------------------------------------------------------------------
def _with_distinct_gains(t, seed=11):
    rng = np.random.default_rng(seed)
    c = _clone(t)
    gain = lambda: (1.0 + 0.5 * rng.standard_normal(t.d_model)).astype(np.float32)     # noqa: E731
    for l in c.enc_layers:
        l["attn_norm"], l["ffn_norm"] = gain(), gain()
    for l in c.dec_layers:
        l["attn_norm"], l["cross_norm"], l["ffn_norm"] = gain(), gain(), gain()
    c.enc_final_norm, c.dec_final_norm = gain(), gain()
    return c


def _torch_encdec_logits(t, src, ids):
    """Encoder-decoder forward of the original T5 layout out of torch.nn.functional routines (float64)."""
    F = torch.nn.functional
    f64 = lambda a: torch.from_numpy(so._decode(np.asarray(a), np.float64).copy())     # noqa: E731
    H, hd, d = t.n_heads, t.head_dim, t.d_model

    def norm(x, g):
        return F.rms_norm(x, (d,), weight=f64(g), eps=t.rms_eps)

    def heads(x):                                   # [T, H*hd] -> [H, T, hd]
        return x.reshape(x.shape[0], H, hd).transpose(0, 1)

    def attn(xq, xkv, lw, names, mask):
        q, k, v = (heads(F.linear(x, f64(lw[n]))) for x, n in zip((xq, xkv, xkv), names[:3]))
        a = F.scaled_dot_product_attention(q, k, v, attn_mask=mask, scale=1.0)
        return F.linear(a.transpose(0, 1).reshape(xq.shape[0], H * hd), f64(lw[names[3]]))

    def ffn(x, lw):
        return F.linear(F.relu(F.linear(norm(x, lw["ffn_norm"]), f64(lw["w_in"]))), f64(lw["w_out"]))

    S, M = len(src), len(ids)
    emb = f64(t.tok_emb)
    pos_s, pos_m = np.arange(S), np.arange(M)
    enc_mask = torch.from_numpy(eo.position_bias(t.enc_rel_bias.astype(np.float64), pos_s, pos_s, True, t.rel_max_distance))
    x = emb[torch.as_tensor(np.asarray(src, dtype=np.int64))]
    for lw in t.enc_layers:
        h = norm(x, lw["attn_norm"])
        x = x + attn(h, h, lw, ("wq", "wk", "wv", "wo"), enc_mask)
        x = x + ffn(x, lw)
    memory = norm(x, t.enc_final_norm)
    dec_bias = eo.position_bias(t.dec_rel_bias.astype(np.float64), pos_m, pos_m, False, t.rel_max_distance)
    causal = np.where(pos_m[None, :] > pos_m[:, None], -np.inf, 0.0)
    dec_mask = torch.from_numpy(dec_bias + causal[None])
    y = emb[torch.as_tensor(np.asarray(ids, dtype=np.int64))]
    for lw in t.dec_layers:
        h = norm(y, lw["attn_norm"])
        y = y + attn(h, h, lw, ("wq", "wk", "wv", "wo"), dec_mask)
        y = y + attn(norm(y, lw["cross_norm"]), memory, lw, ("cq", "ck", "cv", "co"), None)
        y = y + ffn(y, lw)
    return F.linear(norm(y, t.dec_final_norm), f64(t.lm_head)).numpy()


def test_whole_model_against_a_library_composition_with_distinct_gains():
    w, t, d, src = _tiny()
    tt = _with_distinct_gains(t)
    ids = [0] + list(np.random.default_rng(8).integers(1, t.vocab, 9))
    got = so.forward_full(eo.BoundDecoder(eo.EncDecOracleModel(tt), src), ids)
    want = _torch_encdec_logits(tt, src, ids)
    assert np.allclose(got, want, atol=1e-9), float(np.max(np.abs(got - want)))
    # the check has teeth: every one of the gain vectors moves the logits
    for stack, name in (("enc", "attn_norm"), ("enc", "ffn_norm"), ("dec", "attn_norm"), ("dec", "cross_norm"),
                        ("dec", "ffn_norm"), (None, "enc_final_norm"), (None, "dec_final_norm")):
        t2 = _clone(tt)
        if stack is None:
            setattr(t2, name, np.ones(t.d_model, np.float32))
        else:
            (t2.enc_layers if stack == "enc" else t2.dec_layers)[0][name] = np.ones(t.d_model, np.float32)
        other = so.forward_full(eo.BoundDecoder(eo.EncDecOracleModel(t2), src), ids)
        assert np.max(np.abs(other - want)) > 1e-6, (stack, name)


def test_cross_attention_block_written_out_with_loops():
    """One decoder layer, one head, decoder matrices that switch self-attention and feed-forward off (zero output
    projections): logits = unembedding of norm(x + W_co sum_s softmax_s(q . k_s) v_s) with q from the cross norm of the
    embedding and k_s, v_s from the encoder output, written out element by element."""
    w = si.scaled_encdec_workload("t5_tiny", target=dict(n_enc_layers=1, n_dec_layers=1, d_model=256, n_heads=1, head_dim=64,
                                                       d_ffn=256, vocab=64))
    t, _ = si.make_encdec_pair(w)
    tt = _with_distinct_gains(t, seed=3)
    lw = tt.dec_layers[0]
    lw["wo"] = np.zeros_like(lw["wo"])
    lw["w_out"] = np.zeros_like(lw["w_out"])
    src = si.make_source(w)[:5]
    m = eo.EncDecOracleModel(tt)
    ids = [0, 9]
    got = so.forward_full(eo.BoundDecoder(m, src), ids)
    enc = m.encode(src)                                   # [S, d]; the encoder stack is pinned by the test above
    dec = lambda a: so._decode(np.asarray(a), np.float64)  # noqa: E731
    emb, cq, ck, cv, co, head = (dec(a) for a in (tt.tok_emb, lw["cq"], lw["ck"], lw["cv"], lw["co"], tt.lm_head))
    d_model, hd = t.d_model, t.head_dim
    for row, tok in enumerate(ids):
        x = emb[tok]
        ms = sum(float(v) ** 2 for v in x) / d_model
        h = [float(x[i]) / np.sqrt(ms + tt.rms_eps) * float(lw["cross_norm"][i]) for i in range(d_model)]
        q = [sum(cq[e, i] * h[i] for i in range(d_model)) for e in range(hd)]
        scores, vals = [], []
        for s in range(len(src)):
            k_s = [sum(ck[e, i] * enc[s, i] for i in range(d_model)) for e in range(hd)]
            vals.append([sum(cv[e, i] * enc[s, i] for i in range(d_model)) for e in range(hd)])
            scores.append(sum(q[e] * k_s[e] for e in range(hd)))
        mx = max(scores)
        wts = [np.exp(s - mx) for s in scores]
        a = [sum(wts[s] * vals[s][e] for s in range(len(src))) / sum(wts) for e in range(hd)]
        y = [float(x[i]) + sum(co[i, e] * a[e] for e in range(hd)) for i in range(d_model)]
        ms = sum(v * v for v in y) / d_model
        z = [y[i] / np.sqrt(ms + tt.rms_eps) * float(tt.dec_final_norm[i]) for i in range(d_model)]
        want = [sum(head[v, i] * z[i] for i in range(d_model)) for v in range(t.vocab)]
        assert np.allclose(got[row], want, atol=1e-9)
