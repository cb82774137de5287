"""Pins for the oracle's forward pass (CPU only).

Each component is checked against a PyTorch CPU library routine or a textbook identity, and
the assembled forward against closed forms of degenerate models, so that a dropped term, a
wrong sign or index, or a transposed operand in oracle/stairs_oracle.py fails at least one test.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import stairs_oracle as so

RNG = np.random.default_rng(1234)


def test_bf16_round_matches_torch():
    x = RNG.standard_normal(100000).astype(np.float32) * np.float32(3.0)
    x[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]      # exact ties: to even
    ours = si.bf16_round(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    back = so._decode(ours, np.float32)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_rmsnorm_vs_torch_and_unit_rms():
    x = RNG.standard_normal((5, 48))
    g = RNG.standard_normal(48)
    ours = so.rmsnorm(x, g, 1e-5)
    ref = F.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), 1e-5).numpy()
    assert np.allclose(ours, ref, rtol=0, atol=1e-12)
    unit = so.rmsnorm(x * 100, np.ones(48), 0.0)
    assert np.allclose(np.sqrt(np.mean(unit ** 2, -1)), 1.0, atol=1e-12)


def test_softmax_and_silu_vs_torch():
    s = RNG.standard_normal((4, 9)) * 5
    assert np.allclose(so.softmax_rows(s), torch.softmax(torch.from_numpy(s), -1).numpy(), atol=1e-14)
    assert np.allclose(so.softmax_rows(s + 1000.0), so.softmax_rows(s), atol=1e-12)   # shift invariance
    assert np.allclose(so.silu(s), F.silu(torch.from_numpy(s)).numpy(), atol=1e-14)


@pytest.mark.parametrize("pos0,M,T", [(0, 6, 6), (5, 3, 8), (7, 1, 8)])
def test_attention_vs_torch_sdpa(pos0, M, T):
    H, hd = 3, 16
    q = RNG.standard_normal((M, H, hd))
    k = RNG.standard_normal((T, H, hd))
    v = RNG.standard_normal((T, H, hd))
    ours = so.attention(q, k, v, pos0)
    allowed = torch.arange(T)[None, :] <= (pos0 + torch.arange(M))[:, None]
    ref = F.scaled_dot_product_attention(torch.from_numpy(q).permute(1, 0, 2)[None],
                                         torch.from_numpy(k).permute(1, 0, 2)[None],
                                         torch.from_numpy(v).permute(1, 0, 2)[None],
                                         attn_mask=allowed)[0].permute(1, 0, 2).numpy()
    assert np.allclose(ours, ref, atol=1e-12)


def test_rope_textbook_properties():
    hd, H, T = 16, 2, 12
    theta = 10000.0
    x = RNG.standard_normal((T, H, hd))
    pos = np.arange(T) + 3
    cos, sin = so.rope_cos_sin(pos, hd, theta, np.float64)
    y = so.apply_rope(x, cos, sin)
    # (a) complex form: (x_i + j x_{i+hd/2}) * exp(j * p * theta^(-2i/hd))
    z = x[..., :hd // 2] + 1j * x[..., hd // 2:]
    freq = theta ** (-2.0 * np.arange(hd // 2) / hd)
    zr = z * np.exp(1j * pos[:, None, None] * freq[None, None, :])
    assert np.allclose(y[..., :hd // 2], zr.real, atol=1e-12)
    assert np.allclose(y[..., hd // 2:], zr.imag, atol=1e-12)
    # (b) rotation keeps the norm; position 0 is the identity
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)
    c0, s0 = so.rope_cos_sin(np.array([0]), hd, theta, np.float64)
    assert np.array_equal(so.apply_rope(x[:1], c0, s0), x[:1])
    # (c) the score depends only on the position difference
    q = RNG.standard_normal((1, 1, hd))
    kk = RNG.standard_normal((1, 1, hd))

    def score(m, n):
        cm, sm = so.rope_cos_sin(np.array([m]), hd, theta, np.float64)
        cn, sn = so.rope_cos_sin(np.array([n]), hd, theta, np.float64)
        return float(np.sum(so.apply_rope(q, cm, sm) * so.apply_rope(kk, cn, sn)))
    assert abs(score(9, 4) - score(105, 100)) < 1e-10
    assert abs(score(9, 4) - score(4, 9)) > 1e-6          # not symmetric: the sign of the angle matters


def _tiny(seed=3, L=2, d=32, H=2, f=48, V=40):
    return si.make_model(seed, L, d, H, f, V, "fp32")


def test_forward_zero_residual_writers_closed_form():
    """W_o = W_down = 0: the layers add nothing, logits = lm_head . rmsnorm(emb[token])."""
    m = _tiny()
    for lyr in m.layers:
        lyr["wo"] = np.zeros_like(lyr["wo"])
        lyr["w_down"] = np.zeros_like(lyr["w_down"])
    m.final_norm = (1.0 + 0.1 * RNG.standard_normal(m.d_model)).astype(np.float32)
    M = so.OracleModel(m, np.float64)
    ids = [5, 0, 39, 5]
    lg = so.forward_full(M, ids)
    emb = m.tok_emb.astype(np.float64)[ids]
    h = emb / np.sqrt((emb ** 2).mean(-1, keepdims=True) + m.rms_eps) * m.final_norm.astype(np.float64)
    for t in range(len(ids)):
        for v in (0, 7, 39):
            want = sum(m.lm_head[v, c].astype(np.float64) * h[t, c] for c in range(m.d_model))
            assert abs(lg[t, v] - want) < 1e-12


def test_forward_one_layer_uniform_attention_closed_form():
    """One layer, W_q = 0 (all scores 0 -> uniform attention over the visible keys, RoPE cannot
    matter), W_gate = 0 (silu(0) = 0 -> the feed-forward adds nothing):
    x1[t] = emb[t] + W_o . mean_{s<=t}(W_v . rmsnorm(emb[s])), written with explicit loops."""
    m = _tiny(seed=11, L=1, d=16, H=2, f=24, V=30)
    lyr = m.layers[0]
    lyr["wq"] = np.zeros_like(lyr["wq"])
    lyr["w_gate"] = np.zeros_like(lyr["w_gate"])
    lyr["attn_norm"] = (1.0 + 0.1 * RNG.standard_normal(16)).astype(np.float32)
    M = so.OracleModel(m, np.float64)
    ids = [4, 29, 4, 17, 2]
    lg = so.forward_full(M, ids)
    d = 16
    emb = m.tok_emb.astype(np.float64)
    wv, wo, head = (lyr["wv"].astype(np.float64), lyr["wo"].astype(np.float64), m.lm_head.astype(np.float64))
    g = lyr["attn_norm"].astype(np.float64)
    vals = []
    for tok in ids:
        e = emb[tok]
        hn = e / np.sqrt(np.mean(e * e) + m.rms_eps) * g
        vals.append(np.array([sum(wv[o, i] * hn[i] for i in range(d)) for o in range(d)]))
    for t, tok in enumerate(ids):
        mean_v = sum(vals[:t + 1]) / (t + 1)
        x1 = emb[tok] + np.array([sum(wo[o, i] * mean_v[i] for i in range(d)) for o in range(d)])
        hn = x1 / np.sqrt(np.mean(x1 * x1) + m.rms_eps)
        want = np.array([sum(head[v, i] * hn[i] for i in range(d)) for v in range(30)])
        assert np.allclose(lg[t], want, atol=1e-12)


def test_forward_ffn_only_closed_form():
    """One layer, W_o = 0: x1 = emb + W_down . (silu(W_gate h) * (W_up h)), explicit loops; the
    rectangular shapes (f != d) make a transposed operand fail."""
    m = _tiny(seed=12, L=1, d=16, H=2, f=24, V=30)
    lyr = m.layers[0]
    lyr["wo"] = np.zeros_like(lyr["wo"])
    M = so.OracleModel(m, np.float64)
    ids = [9, 1]
    lg = so.forward_full(M, ids)
    d, f = 16, 24
    emb = m.tok_emb.astype(np.float64)
    wg, wu, wd = (lyr[n].astype(np.float64) for n in ("w_gate", "w_up", "w_down"))
    head = m.lm_head.astype(np.float64)
    for t, tok in enumerate(ids):
        e = emb[tok]
        hn = e / np.sqrt(np.mean(e * e) + m.rms_eps)
        gate = np.array([sum(wg[j, i] * hn[i] for i in range(d)) for j in range(f)])
        up = np.array([sum(wu[j, i] * hn[i] for i in range(d)) for j in range(f)])
        act = gate / (1 + np.exp(-gate)) * up
        x1 = e + np.array([sum(wd[o, j] * act[j] for j in range(f)) for o in range(d)])
        hn = x1 / np.sqrt(np.mean(x1 * x1) + m.rms_eps)
        want = np.array([sum(head[v, i] * hn[i] for i in range(d)) for v in range(30)])
        assert np.allclose(lg[t], want, atol=1e-12)


def _torch_forward(m, ids):
    """The same architecture composed from PyTorch CPU library routines (float64)."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    T, H, hd = len(ids), m.n_heads, m.head_dim
    x = t(m.tok_emb)[torch.tensor(ids)]
    inv = m.rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)                       # e^{j angle}

    def rope(u):                                                        # u [T, H, hd]
        z = torch.complex(u[..., :hd // 2], u[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], -1)
    for lyr in m.layers:
        h = F.rms_norm(x, (m.d_model,), t(lyr["attn_norm"]), m.rms_eps)
        q = rope(F.linear(h, t(lyr["wq"])).view(T, H, hd))
        k = rope(F.linear(h, t(lyr["wk"])).view(T, H, hd))
        v = F.linear(h, t(lyr["wv"])).view(T, H, hd)
        a = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True)[0]
        x = x + F.linear(a.transpose(0, 1).reshape(T, m.d_model), t(lyr["wo"]))
        h = F.rms_norm(x, (m.d_model,), t(lyr["ffn_norm"]), m.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, t(lyr["w_gate"]))) * F.linear(h, t(lyr["w_up"])), t(lyr["w_down"]))
    return F.linear(F.rms_norm(x, (m.d_model,), t(m.final_norm), m.rms_eps), t(m.lm_head)).numpy()


@pytest.mark.parametrize("seed", [1, 2])
def test_forward_vs_torch_library_composition(seed):
    m = si.make_model(seed, 3, 32, 4, 80, 64, "fp32")
    for lyr in m.layers:       # non-trivial gains so that a misplaced norm shows
        lyr["attn_norm"] = (1 + 0.2 * RNG.standard_normal(32)).astype(np.float32)
        lyr["ffn_norm"] = (1 + 0.2 * RNG.standard_normal(32)).astype(np.float32)
    ids = list(RNG.integers(0, 64, 11))
    ours = so.forward_full(so.OracleModel(m, np.float64), ids)
    assert np.allclose(ours, _torch_forward(m, ids), atol=1e-11)


def test_forward_is_causal():
    m = _tiny(seed=5, L=2)
    M = so.OracleModel(m, np.float64)
    a = [1, 2, 3, 4, 5, 6]
    b = [1, 2, 3, 9, 5, 6]
    la, lb = so.forward_full(M, a), so.forward_full(M, b)
    assert np.array_equal(la[:3], lb[:3])
    assert not np.allclose(la[3:], lb[3:])


def test_cached_forward_equals_full_forward():
    """Stair batch == one causal forward: last-position logits of each stair row equal the rows
    of a single forward over prefix + draft, with or without the cache."""
    m = _tiny(seed=6, L=3, d=32, H=4)
    M = so.OracleModel(m, np.float64)
    seq = [int(t) for t in RNG.integers(0, 40, 9)]
    full = so.forward_full(M, seq)
    for i in range(5, 10):                        # stair rows seq[:i]
        assert np.allclose(so.forward_full(M, seq[:i])[-1], full[i - 1], atol=1e-13)
    cache = so.KVCache.empty(M, 16)
    so.forward_cached(M, cache, seq[:4], 0)
    got = so.forward_cached(M, cache, seq[4:], 4)
    assert np.allclose(got, full[4:], atol=1e-13)
    # stale entries beyond the rows just written are never read (rollback = length reset)
    cache.k[0][9:] = 1e9
    got2 = so.forward_cached(M, cache, seq[4:7], 4)
    assert np.allclose(got2, full[4:7], atol=1e-13)


def test_fp32_oracle_close_to_fp64():
    m = si.make_model(21, 4, 256, 4, 1024, 1024, "fp32", deep_from=2, deep_scale=0.05)
    ids = list(RNG.integers(0, 1024, 40))
    l32 = so.forward_full(so.OracleModel(m, np.float32), ids)
    l64 = so.forward_full(so.OracleModel(m, np.float64), ids)
    assert l32.dtype == np.float32
    assert np.max(np.abs(l32 - l64)) < 2e-5
