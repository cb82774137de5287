"""GPU parity of the encoder-decoder path: the HIP library through its C ABI against the CPU oracle, stair logits
element by element and tokens one by one (teacher-forced onto the GPU's prefix), plus the invariants that hold at
any size (stairs == plain greedy on the same kernels, graph replay == one-by-one launches)."""
import numpy as np
import pytest

import paper_2407_19947_amd as pkg
import synth_inputs as si
from parity_util import LOGIT_TOL_BF16, run_encdec_side_by_side

pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)


def _pair(name="t5_tiny", **over):
    w = si.scaled_encdec_workload(name, **over)
    t, d = si.make_encdec_pair(w)
    return w, t, d, si.make_source(w)


@pytest.mark.parametrize("k", [0, 1, 4, 7])
def test_tiny_pair_against_the_oracle(k):
    w, t, d, src = _pair()
    _log(f"encdec tiny: k={k} S={len(src)}")
    res = run_encdec_side_by_side(t, d, src, w["G"], k, LOGIT_TOL_BF16)
    _log(f"  max logit err {res['max_logit_err']:.3g}, accepted {res['n_accepted']}")
    assert res["max_logit_err"] < 5e-3
    if k > 0:
        assert 0 < sum(res["n_accepted"]) < k * len(res["n_accepted"])


@pytest.mark.parametrize("S", [1, 2, 31, 33, 127, 128, 129, 300])
def test_source_lengths(S):
    """Source ends before / on / after a 32-row encoder block and a 128-key attention chunk; max_src == S."""
    w, t, d, src = _pair(S=300)
    _log(f"encdec source length S={S}")
    res = run_encdec_side_by_side(t, d, src[:S], 12, 3, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 5e-3


def test_long_source_takes_the_stand_alone_merge():
    """3300 source positions = 26 attention chunks: above the limit of the fused chunk merge, so the encoder's
    attention (bias, fixed key set) and the cross-attention run the merge as a kernel of its own."""
    w, t, d, src = _pair(S=3300)
    _log("encdec long source S=3300")
    res = run_encdec_side_by_side(t, d, src, 10, 3, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 5e-3


def test_long_decoder_sequence_reaches_the_last_bucket():
    """200 decoder positions: key distances pass 128, where the one-sided rule stays in its last bucket, and the
    decoder's self-attention crosses a 128-key chunk boundary (two chunks, fused merge with bias)."""
    w, t, d, src = _pair()
    res = run_encdec_side_by_side(t, d, src, 200, 4, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 5e-3


def test_wide_attention_and_independent_draft():
    """n_heads * head_dim != d_model (head_dim 128) in the target; a draft with its own weights and shape."""
    w, t, d, src = _pair(target=dict(n_enc_layers=2, n_dec_layers=2, d_model=256, n_heads=4, head_dim=128),
                         draft=dict(kind="independent", seed=77, n_enc_layers=1, n_dec_layers=1, d_model=256, n_heads=4,
                                    head_dim=64, d_ffn=256))
    assert t.d_attn == 512
    res = run_encdec_side_by_side(t, d, src, 16, 3, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 5e-3


def test_widest_stair_batch():
    w, t, d, src = _pair()
    res = run_encdec_side_by_side(t, d, src, 70, 31, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 5e-3


def test_generate_equals_plain_greedy_and_graph_replay(monkeypatch):
    w, t, d, src = _pair(S=200)
    G = 64
    with pkg.StairsEncDec(t, d, k_max=8, max_src=256, max_seq=G + 16) as s:
        base, st0 = s.generate(src, G, 0)
        assert st0.iterations == G
        for k in (1, 3, 8):
            toks, st = s.generate(src, G, k)
            assert np.array_equal(toks, base), k
            assert st.iterations < G
        # another source of the same length (captured iterations are reused), checked against a fresh context
        src2 = src[::-1].copy()
        same_len, _ = s.generate(src2, G, 3)
        with pkg.StairsEncDec(t, d, k_max=8, max_src=256, max_seq=G + 16) as s3:
            fresh2, _ = s3.generate(src2, G, 3)
        assert np.array_equal(same_len, fresh2) and not np.array_equal(same_len, base)
        # another source of another length on the same context, then the first one again
        other, _ = s.generate(src[:77], G, 3)
        again, _ = s.generate(src, G, 3)
        assert np.array_equal(again, base)
        assert not np.array_equal(other, base)
        with pkg.StairsEncDec(t, d, k_max=8, max_src=256, max_seq=G + 16) as s2:
            fresh, _ = s2.generate(src[:77], G, 3)
        assert np.array_equal(other, fresh)
        adaptive_ctx_tokens = None
        s.encode(src)
        adaptive_ctx_tokens, _ = s.decode_adaptive(G, 2)
        assert np.array_equal(adaptive_ctx_tokens, base)
    monkeypatch.setenv("STAIRS_NO_GRAPH", "1")
    with pkg.StairsEncDec(t, d, k_max=8, max_src=256, max_seq=G + 16) as s:
        eager, _ = s.generate(src, G, 3)
    assert np.array_equal(eager, base)


def test_error_paths():
    w, t, d, src = _pair()
    with pkg.StairsEncDec(t, d, k_max=4, max_src=32, max_seq=40) as s:
        with pytest.raises(pkg.StairsError) as e:
            s.prefill([1, 2, 3])
        assert e.value.code == -1
        with pytest.raises(pkg.StairsError) as e:
            s.propose(2)                                   # nothing encoded yet
        assert e.value.code == -3
        with pytest.raises(pkg.StairsError) as e:
            s.encode(src[:33])                             # max_src is 32
        assert e.value.code == -2
        with pytest.raises(pkg.StairsError) as e:
            s.encode([t.vocab])
        assert e.value.code == -1
        with pytest.raises(pkg.StairsError) as e:
            s.reserve_batch(2)
        assert e.value.code == -1
        with pytest.raises(pkg.StairsError) as e:
            s.generate(src[:32], 40, 4)                    # 1 + 40 + 4 + 1 > 40
        assert e.value.code == -2
        toks, _ = s.generate(src[:32], 34, 4)              # exactly fits
        base, _ = s.generate(src[:32], 34, 0)
        assert np.array_equal(toks, base)
    tt = si.make_encdec_model(1, 1, 1, 128, 2, 64, 256, 512)      # d_model not a multiple of 256
    with pytest.raises(pkg.StairsError):
        pkg.StairsEncDec(tt, None, k_max=0, max_src=8, max_seq=8)
    pt, pd = si.make_pair(si.scaled_workload("cfg2_125m", target=dict(n_layers=1, d_model=256, n_heads=4, d_ffn=256, vocab=512),
                                             draft=dict(kind="prefix", n_layers=1)))
    with pkg.Stairs(pt, pd, k_max=2, max_seq=16) as plain:
        with pytest.raises(pkg.StairsError) as e:
            pkg.stairs_encode(plain.ctx, [1])                  # a decoder-only context has no encoder
        assert e.value.code == -1


def test_large_shape_pair_against_the_oracle():
    """The shape of the paper's large checkpoint (24 + 24 layers, d 1024, 16 heads of 64, ffn 4096, vocabulary 32128)
    with its 6 + 6 layer prefix draft; the oracle runs in float32 here (float64 would need 6 GB for the matrices)."""
    w, t, d, src = _pair("t5_large_shape")
    _log("encdec large shape: oracle + gpu, G=24 k=4")
    from parity_util import compare_generation
    from oracle import encdec_oracle as eo, stairs_oracle as so
    T = eo.BoundDecoder(eo.EncDecOracleModel(t, np.float32), src)
    D = eo.BoundDecoder(eo.EncDecOracleModel(d, np.float32), src)
    orc = so.CachedStairs(T, D, [si.DECODER_START], 64)
    with pkg.StairsEncDec(t, d, k_max=4, max_src=len(src), max_seq=64) as gpu:
        gpu.encode(src)
        res = compare_generation(orc, gpu, 1, 24, 4, LOGIT_TOL_BF16, log=_log)
    _log(f"  max logit err {res['max_logit_err']:.3g}, accepted {res['n_accepted']}")


@pytest.mark.parametrize("case", range(8))
def test_encdec_shape_sweep_against_the_oracle(case):
    """Seeded sweep over the documented limits: model widths with an odd number of 256-wide weight units, attention
    widths that differ from d_model, both head sizes, feed-forward widths that are not multiples of 512, source lengths
    from 1 to a few hundred, draft lengths on every GEMM / attention path."""
    rng = np.random.default_rng([2025, case])
    d = int(rng.choice([256, 512, 768]))
    hd = int(rng.choice([64, 128]))
    a = int(rng.choice([256, 512, 768]))
    f = int(rng.choice([256, 768, 1280]))
    V = int(rng.choice([272, 1008, 2048]))
    k = [0, 1, 3, 4, 6, 9, 16, 31][case]
    S = int(rng.integers(1, 400))
    w = si.scaled_encdec_workload("t5_tiny", seed=7000 + case,
                                  target=dict(n_enc_layers=2, n_dec_layers=2, d_model=d, n_heads=a // hd, head_dim=hd,
                                              d_ffn=f, vocab=V), S=400)
    _log(f"encdec shape sweep {case}: d={d} a={a} hd={hd} f={f} V={V} S={S} k={k}")
    t, dr = si.make_encdec_pair(w)
    res = run_encdec_side_by_side(t, dr, si.make_source(w, S), 2 * (k + 1) + 6, k, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 5e-3
