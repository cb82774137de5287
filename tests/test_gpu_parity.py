"""GPU parity proper: the HIP path through its C ABI against the CPU oracle, element by
element on per-stair logits and token by token on the generated sequence."""
import numpy as np
import pytest

import paper_2407_19947_amd as pkg
import synth_inputs as si
from oracle import stairs_oracle as so
from parity_util import LOGIT_TOL_BF16, MARGIN_TOL, eps_greedy_ok as eps_ok, run_side_by_side

pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)


def test_cfg1_tiny_fp32_full():
    """Workload 1 at full size: fp32 pair, P=32, G=64, k=4; oracle in float64."""
    w = si.WORKLOADS["cfg1_tiny_fp32"]
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    res = run_side_by_side(target, draft, prompt, w["G"], 4, np.float64, 2e-4, log=_log)
    assert res["token_mismatches"] == 0
    T = so.OracleModel(target, np.float64)
    assert res["tokens"] == so.greedy_bruteforce(T, prompt, w["G"])
    _log(f"cfg1: iterations={res['iterations']} max_logit_err={res['max_logit_err']:.3g} n={res['n_accepted']}")


@pytest.mark.parametrize("k", [0, 1, 2, 7, 16])
def test_cfg1_other_k(k):
    w = si.WORKLOADS["cfg1_tiny_fp32"]
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    res = run_side_by_side(target, draft, prompt, 40, k, np.float64, 2e-4)
    assert res["token_mismatches"] == 0


@pytest.mark.parametrize("P", [1, 2, 3, 33, 130])
def test_fp32_prompt_lengths(P):
    """Shortest prompts (nothing to prefill, the draft's two-row step starts before position 0)
    and prompts that cross prefill-chunk and attention-chunk boundaries."""
    w = si.scaled_workload("cfg1_tiny_fp32", P=max(P, 1))
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    res = run_side_by_side(target, draft, prompt, 12, 3, np.float64, 2e-4)
    assert res["token_mismatches"] == 0


def test_bf16_small_pair():
    """bf16 path on a reduced 125M-style pair (d=256, 4 heads of 64, vocab 2048): several GEMM
    tiles, ragged k slices (d_ffn = 768 -> 3 units), a sequence that crosses an attention chunk."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=4, d_model=256, n_heads=4, d_ffn=768, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=120, G=40)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    for k in (0, 3, 8):
        res = run_side_by_side(target, draft, prompt, w["G"], k, np.float64, LOGIT_TOL_BF16, log=_log)
        _log(f"bf16 small k={k}: err={res['max_logit_err']:.3g} mism={res['token_mismatches']} n={res['n_accepted']}")


def test_bf16_head_dim_128_and_independent_draft():
    w = dict(seed=77, dtype="bf16", target=dict(n_layers=3, d_model=512, n_heads=4, d_ffn=1024, vocab=4096),
             draft=dict(kind="independent", seed=78, n_layers=2, d_model=256, n_heads=4, d_ffn=512),
             deep_scale=1.0, P=70, G=24, ks=[4])
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    res = run_side_by_side(target, draft, prompt, w["G"], 4, np.float64, LOGIT_TOL_BF16, log=_log)
    _log(f"hd128: err={res['max_logit_err']:.3g} n={res['n_accepted']}")


@pytest.mark.parametrize("k", [2, 4, 8])
def test_cfg2_125m_full_shape(k):
    """Workload 2 at its full model shape and prompt; G shortened to 48 tokens so that the
    float32 oracle finishes in seconds (the full G runs in the self-consistency test below)."""
    w = si.WORKLOADS["cfg2_125m"]
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    res = run_side_by_side(target, draft, prompt, 48, k, np.float32, LOGIT_TOL_BF16, log=_log)
    _log(f"cfg2 k={k}: err={res['max_logit_err']:.3g} mism={res['token_mismatches']} n={res['n_accepted']}")


def test_generate_equals_plain_greedy_on_gpu():
    """The paper's invariant on the device itself: stairs generation with any k returns the
    tokens of k = 0 (the target alone), bit for bit; workload 2 at full size."""
    w = si.WORKLOADS["cfg2_125m"]
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    cap = w["P"] + w["G"] + 20
    with pkg.Stairs(target, draft, k_max=16, max_seq=cap) as s:
        base, st0 = s.generate(prompt, w["G"], 0)
        assert st0.iterations == w["G"]
        for k in (1, 2, 4, 8, 16):
            toks, st = s.generate(prompt, w["G"], k)
            _log(f"k={k}: iterations={st.iterations} accepted={st.accepted} decode_ms={st.ms_decode:.1f}")
            assert np.array_equal(toks, base), f"k={k} differs from plain greedy"
            assert st.iterations + st.accepted >= w["G"]
            assert sum(st.accept_hist) == st.iterations
        again, _ = s.generate(prompt, w["G"], 4)
        assert np.array_equal(again, base)


def test_forced_accept_and_reject_counts():
    """Closed forms: draft == target keeps every assistant token (iterations = ceil(G/(k+1)));
    assistant tokens forced to differ keep none (iterations = G)."""
    w = si.scaled_workload("cfg1_tiny_fp32")
    target, _ = si.make_pair(w)
    prompt = si.make_prompt(w)
    G, k = 30, 4
    with pkg.Stairs(target, target, k_max=k, max_seq=128) as s:
        toks, st = s.generate(prompt, G, k)
        assert st.iterations == -(-G // (k + 1)) and st.accept_hist[k] == st.iterations
        base, _ = s.generate(prompt, G, 0)
        assert np.array_equal(toks, base)
        s.prefill(prompt)
        for i in range(G):
            bad = [(int(base[i]) + 1) % w["target"]["vocab"]] + [0] * (k - 1)
            tgt, n, _ = s.verify_tokens(bad)
            assert n == 0 and tgt[0] == base[i]
        assert list(s.tokens()[len(prompt):]) == list(base)


def test_error_paths_on_device():
    w = si.scaled_workload("cfg1_tiny_fp32")
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    with pkg.Stairs(target, draft, k_max=4, max_seq=64) as s:
        with pytest.raises(pkg.StairsError) as e:
            s.verify(0)
        assert e.value.code == -3                              # verify before prefill
        with pytest.raises(pkg.StairsError) as e:
            s.prefill(list(prompt) * 2)                        # 64 + k_max + 1 > max_seq
        assert e.value.code == -2
        with pytest.raises(pkg.StairsError) as e:
            s.prefill([5, 99999])
        assert e.value.code == -1
        s.prefill(prompt)
        with pytest.raises(pkg.StairsError) as e:
            s.verify(3)                                        # no pending proposal
        assert e.value.code == -3
        with pytest.raises(pkg.StairsError) as e:
            s.propose(5)                                       # k > k_max
        assert e.value.code == -1
        s.propose(2)
        with pytest.raises(pkg.StairsError) as e:
            s.propose(2)                                       # already pending
        assert e.value.code == -3
        with pytest.raises(pkg.StairsError) as e:
            s.verify(3)                                        # pending k differs
        assert e.value.code == -3
        s.verify(2)
        with pytest.raises(pkg.StairsError) as e:
            s.generate(prompt, 40, 4)                          # P + G + k + 1 > max_seq
        assert e.value.code == -2


def test_graph_replay_matches_eager_launches(monkeypatch):
    """stairs_decode replays one captured HIP graph per iteration; every replay must give what the same
    launches give when issued one by one (STAIRS_NO_GRAPH=1), across prefills, draft lengths and
    interleaved step-by-step (eager) calls."""
    w = si.WORKLOADS["cfg2_125m"]
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    cap = w["P"] + w["G"] + 20
    monkeypatch.setenv("STAIRS_NO_GRAPH", "1")
    with pkg.Stairs(target, draft, k_max=8, max_seq=cap) as eager:
        ref = {k: eager.generate(prompt, w["G"], k) for k in (0, 3, 8)}
    monkeypatch.delenv("STAIRS_NO_GRAPH")
    with pkg.Stairs(target, draft, k_max=8, max_seq=cap) as s:
        for rep in range(2):
            for k in (3, 0, 8):
                toks, st = s.generate(prompt, w["G"], k)
                assert np.array_equal(toks, ref[k][0]), f"graph replay differs from eager launches (k={k})"
                assert st.iterations == ref[k][1].iterations and st.accepted == ref[k][1].accepted
                assert list(st.accept_hist) == list(ref[k][1].accept_hist)
            # eager work between replays: a step-by-step iteration, then a decode that continues from it
            s.prefill(prompt)
            d = s.propose(3)
            tgt, n, _ = s.verify(3)
            assert list(tgt[:n + 1]) == list(ref[3][0][:n + 1])
            rest, _ = s.decode(20, 3)
            assert list(rest) == list(ref[3][0][n + 1:n + 21])


def test_graph_replay_at_the_end_of_the_cache(monkeypatch):
    """The replayed attention grid is padded to a multiple of 4 chunks but must never reach past the
    partial-result buffers (sized for max_seq): sequence that ends in the last chunk the cache has."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=4, d_model=256, n_heads=4, d_ffn=768, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=120, G=200)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    k = 3
    cap = w["P"] + w["G"] + k + 2                      # 325 positions = 3 chunks of 128
    monkeypatch.setenv("STAIRS_NO_GRAPH", "1")
    with pkg.Stairs(target, draft, k_max=k, max_seq=cap) as eager:
        ref_t, ref_s = eager.generate(prompt, w["G"], k)
    monkeypatch.delenv("STAIRS_NO_GRAPH")
    with pkg.Stairs(target, draft, k_max=k, max_seq=cap) as s:
        for rep in range(6):
            toks, st = s.generate(prompt, w["G"], k)
            assert np.array_equal(toks, ref_t)
            assert list(st.accept_hist) == list(ref_s.accept_hist)


@pytest.mark.parametrize("P", [127, 128, 129, 256, 257])
def test_bf16_prompt_lengths_around_chunk_boundaries(P):
    """Prompt ends just before / on / after an attention chunk boundary (128 keys) and a prefill chunk
    boundary (32 rows); the first stair batch then straddles it."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=3, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=P, G=8)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    res = run_side_by_side(target, draft, prompt, 8, 5, np.float64, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 2e-3


@pytest.mark.parametrize("P,heads,k", [(2700, 2, 5), (5000, 4, 16), (5300, 2, 3), (6300, 4, 8)])
def test_attention_chunk_counts_of_every_merge_form(P, heads, k):
    """Contexts of 11, 20, 21 and 25 attention chunks of 256 keys: the chunk merge with all loads in front of its
    table for up to 10 and up to 20 chunks (the shorter prompts of the other tests cover the first), the grouped merge
    inside the attention kernel (21..24 chunks) and the merge kernel of its own (from 25 on); head_dim 128 and 64;
    stair batches of 4 to 17 rows (two query tiles, several passes of the merging work-group)."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=2, d_model=256, n_heads=heads, d_ffn=256, vocab=512),
                           draft=dict(kind="prefix", n_layers=1), P=P, G=6)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    _log(f"attention merge forms: P={P}, head_dim {256 // heads}, k={k}")
    res = run_side_by_side(target, draft, prompt, 6, k, np.float64, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 5e-3


def test_widest_stair_batch_and_exact_capacity():
    """k = k_max = 31 (32 rows, the most one forward takes) with max_seq sized to the last position used."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=40, G=70)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    k = 31
    res = run_side_by_side(target, draft, prompt, 70, k, np.float64, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 2e-3
    cap = w["P"] + w["G"] + k + 1                            # the documented requirement of stairs_generate
    with pkg.Stairs(target, draft, k_max=k, max_seq=cap) as s:
        toks, st = s.generate(prompt, w["G"], k)
        base, _ = s.generate(prompt, w["G"], 0)
        assert np.array_equal(toks, base)
        with pytest.raises(pkg.StairsError) as e:
            s.generate(prompt, w["G"] + 1, k)                # one position too many
        assert e.value.code == -2


def test_degenerate_requests():
    """G = 0, a target without any draft model (only k = 0 is legal), generation continued by stairs_decode."""
    w = si.scaled_workload("cfg1_tiny_fp32")
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    with pkg.Stairs(target, None, k_max=0, max_seq=128) as s:
        toks, st = s.generate(prompt, 0, 0)
        assert len(toks) == 0 and st.iterations == 0
        plain, _ = s.generate(prompt, 20, 0)
        with pytest.raises(pkg.StairsError) as e:
            s.generate(prompt, 4, 1)                          # k > k_max
        assert e.value.code == -1
    with pkg.Stairs(target, draft, k_max=4, max_seq=128) as s:
        a, _ = s.generate(prompt, 7, 4)
        b, _ = s.decode(13, 2)                                # continue the same sequence with another k
        assert list(a) + list(b) == list(plain)
        assert list(s.tokens()) == list(prompt) + list(plain)


# ---- several sequences in one context (stairs_generate_batch) ---------------------------------------------

def _batch_pair():
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=3, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=40, G=48)
    target, draft = si.make_pair(w)
    return w, target, draft


def _prompts(w, lengths):
    rng = np.random.default_rng([w["seed"], 77])
    return [rng.integers(0, w["target"]["vocab"], n).astype(np.int32) for n in lengths]


@pytest.mark.parametrize("k", [0, 1, 3, 7])
def test_batch_of_sequences_equals_each_sequence_alone(k):
    """Every sequence of a batch gets, bit for bit, the tokens the same context generates for it alone (each stair
    row's arithmetic does not depend on what else is in the forward), with prompts of different lengths, some
    ending on a chunk boundary, and sequences that finish at different iterations."""
    w, target, draft = _batch_pair()
    lengths = [40, 1, 129, 128][: max(1, min(4, 32 // (k + 1)))]
    prompts = _prompts(w, lengths)
    G = 48
    with pkg.Stairs(target, draft, k_max=7, max_seq=256) as s:
        alone = [s.generate(p, G, k)[0].copy() for p in prompts]
        s.reserve_batch(4)
        toks, st = s.generate_batch(prompts, G, k)
        assert toks.shape == (len(prompts), G)
        for b in range(len(prompts)):
            assert np.array_equal(toks[b], alone[b]), (b, k)
        assert st.tokens == len(prompts) * G
        # the single-sequence calls still work afterwards (on slot 0 of the enlarged context)
        again, _ = s.generate(prompts[0], G, k)
        assert np.array_equal(again, alone[0])
        # and graph replay against one-by-one launches
    import os
    os.environ["STAIRS_NO_GRAPH"] = "1"
    try:
        with pkg.Stairs(target, draft, k_max=7, max_seq=256) as s:
            s.reserve_batch(4)
            toks2, _ = s.generate_batch(prompts, G, k)
    finally:
        del os.environ["STAIRS_NO_GRAPH"]
    assert np.array_equal(toks2, toks)


def test_batch_against_the_oracle():
    """The oracle's definition of a batch is the oracle run once per sequence."""
    w, target, draft = _batch_pair()
    prompts = _prompts(w, [33, 64, 20])
    G, k = 24, 3
    T = so.OracleModel(target, np.float64)
    with pkg.Stairs(target, draft, k_max=k, max_seq=128) as s:
        s.reserve_batch(3)
        toks, st = s.generate_batch(prompts, G, k)
    for b, p in enumerate(prompts):
        # every generated token must be an eps-greedy choice under the oracle's logits for the GPU's own prefix
        seq = np.concatenate([p, toks[b]])
        logits = so.forward_full(T, seq[:-1])
        for j in range(G):
            row = logits[len(p) - 1 + j]
            assert row[toks[b][j]] >= row.max() - MARGIN_TOL, (b, j)
    assert st.iterations >= G // (k + 1)


def test_wide_batches_on_the_block_kernels():
    """Forwards of more than 32 rows (many sequences) run on the block kernels of the prompt ingestion.  Every token
    must be an eps-greedy choice under the oracle's logits for the sequence's own prefix; a sequence's tokens do not
    depend on which other sequences share the forward (20 sequences x 3 rows against 12 x 3 rows); graph replay equals
    one-by-one launches; k = 0 (a batch of plain greedy decodes) and the limits."""
    import os
    w, target, draft = _batch_pair()
    lengths = [5, 70, 33, 64, 20, 1, 129, 17, 90, 40, 65, 8, 100, 31, 32, 2, 77, 50, 128, 11]
    prompts = _prompts(w, lengths)
    G, k = 20, 2
    T = so.OracleModel(target, np.float64)
    with pkg.Stairs(target, draft, k_max=3, max_seq=256) as s:
        s.reserve_batch(40)
        toks, st = s.generate_batch(prompts, G, k)                    # 60 rows per verification, 40 / 20 per draft step
        assert toks.shape == (len(prompts), G) and st.tokens == len(prompts) * G
        part, _ = s.generate_batch(prompts[:12], G, k)                # 36 rows
        assert np.array_equal(part, toks[:12])
        plain, _ = s.generate_batch(prompts + prompts, G, 0)          # 40 sequences, k = 0: 40 rows
        assert np.array_equal(plain[:20], plain[20:])
        with pytest.raises(pkg.StairsError) as e:
            s.generate_batch(prompts + prompts, 4, 7)                 # 40 x 8 rows do not fit
        assert e.value.code == -1
        small, _ = s.generate_batch(prompts[:4], G, k)                # 12 rows: the decode kernels, bit-exact path
        alone, _ = s.generate(prompts[1], G, k)
        assert np.array_equal(small[1], alone)
    mism = 0
    for out in (toks, plain[:20]):
        for b, p in enumerate(prompts):
            seq = np.concatenate([p, out[b]])
            logits = so.forward_full(T, seq[:-1])
            for j in range(G):
                row = logits[len(p) - 1 + j]
                assert row[out[b][j]] >= row.max() - MARGIN_TOL, (b, j)
                mism += int(np.argmax(row)) != int(out[b][j])
    _log(f"wide batch: {st.iterations} iterations, {mism} tokens differ from the oracle's argmax (near-ties)")
    os.environ["STAIRS_NO_GRAPH"] = "1"
    try:
        with pkg.Stairs(target, draft, k_max=3, max_seq=256) as s:
            s.reserve_batch(20)
            toks2, _ = s.generate_batch(prompts, G, k)
    finally:
        del os.environ["STAIRS_NO_GRAPH"]
    assert np.array_equal(toks2, toks)


@pytest.mark.parametrize("B,k", [(12, 2), (16, 2), (13, 3), (16, 3), (9, 6), (7, 8)])
def test_batches_of_33_to_64_rows_equal_each_sequence_alone(B, k):
    """36, 48, 52, 64, 63 and 63 rows per verification (three and four column tiles of the hand-off-free GEMM, the
    second fragment block, draft steps of 2 B rows): still the weight-streaming kernels with one order of additions
    per row, so every sequence is bit for bit the sequence generated alone, and so is graph replay vs plain launches."""
    w, target, draft = _batch_pair()
    lengths = [40, 1, 129, 128, 5, 77, 64, 33, 2, 100, 17, 90, 31, 65, 8, 127][:B]
    prompts = _prompts(w, lengths)
    G = 24
    with pkg.Stairs(target, draft, k_max=8, max_seq=256) as s:
        alone = [s.generate(p, G, k)[0].copy() for p in prompts]
        s.reserve_batch(16)
        toks, st = s.generate_batch(prompts, G, k)
        for b in range(B):
            assert np.array_equal(toks[b], alone[b]), (b, k)
        assert st.tokens == B * G
    import os
    os.environ["STAIRS_NO_GRAPH"] = "1"
    try:
        with pkg.Stairs(target, draft, k_max=8, max_seq=256) as s:
            s.reserve_batch(16)
            toks2, _ = s.generate_batch(prompts, G, k)
    finally:
        del os.environ["STAIRS_NO_GRAPH"]
    assert np.array_equal(toks2, toks)


def test_wide_streaming_batch_against_the_oracle():
    """48 rows per forward (16 sequences, k = 2) against the oracle: every sequence's tokens are an eps-greedy path of
    the oracle's logits (the batch holds the same bits as the sequence alone, which the single-sequence tests compare
    logit by logit; this closes the loop through the batched call itself on a model with several weight tiles per
    wave: d_model 512, d_ffn 1536)."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=3, d_model=512, n_heads=8, d_ffn=1536, vocab=4096),
                           draft=dict(kind="prefix", n_layers=1), P=40, G=16)
    target, draft = si.make_pair(w)
    rng = np.random.default_rng([w["seed"], 78])
    prompts = [rng.integers(0, 4096, n).astype(np.int32) for n in [40, 3, 129, 70, 9, 33, 64, 1, 100, 17, 90, 31, 65, 8, 127, 50]]
    T = so.OracleModel(target, np.float64)
    G, k = 16, 2
    with pkg.Stairs(target, draft, k_max=2, max_seq=256) as s:
        s.reserve_batch(16)
        toks, _ = s.generate_batch(prompts, G, k)
    for b, p in enumerate(prompts):
        seq = [int(x) for x in p]
        for i in range(G):
            lg = so.forward_full(T, seq)[-1]
            assert eps_ok(lg, int(toks[b][i])), (b, i)
            seq.append(int(toks[b][i]))


def test_batch_limits_and_errors():
    w, target, draft = _batch_pair()
    prompts = _prompts(w, [8, 9])
    with pkg.Stairs(target, draft, k_max=15, max_seq=128) as s:
        with pytest.raises(pkg.StairsError) as e:
            s.generate_batch(prompts, 4, 1)                   # nothing reserved beyond one sequence
        assert e.value.code == -1
        s.reserve_batch(16)
        toks, _ = s.generate_batch(_prompts(w, [5] * 16), 6, 1)   # 16 sequences x 2 rows = the widest forward
        assert toks.shape == (16, 6)
        toks, _ = s.generate_batch(_prompts(w, [5] * 16), 6, 3)   # 16 x 4 rows: the widest the streaming kernels take
        assert toks.shape == (16, 6)
        with pytest.raises(pkg.StairsError) as e:
            s.generate_batch(_prompts(w, [5] * 16), 6, 4)     # 16 x 5 rows do not fit
        assert e.value.code == -1
        with pytest.raises(pkg.StairsError) as e:
            s.generate_batch(prompts, 120, 3)                 # capacity
        assert e.value.code == -2
        empty, st = s.generate_batch(prompts, 0, 3)
        assert empty.shape == (2, 0) and st.iterations == 0
        with pytest.raises(pkg.StairsError):
            s.reserve_batch(129)                              # beyond STAIRS_MAX_BATCH
    fp32 = si.scaled_workload("cfg1_tiny_fp32")
    t32, d32 = si.make_pair(fp32)
    with pkg.Stairs(t32, d32, k_max=2, max_seq=64) as s:
        with pytest.raises(pkg.StairsError) as e:
            s.reserve_batch(2)                                # fp32 models keep float caches: one sequence only
        assert e.value.code == -1


def test_block_prefill_against_row_prefill_and_oracle(monkeypatch):
    """Prompts of 64 rows and more are ingested in blocks on the block GEMM; the first stair batch after either
    kind of prefill must agree with the oracle, and the two kinds with each other far inside the tolerance."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=3, d_model=256, n_heads=4, d_ffn=768, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=600, G=8)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)                 # 599 rows: one full block of 512 and a ragged one
    d_tokens = [3, 1, 4]
    T = so.OracleModel(target, np.float64)
    ref = so.forward_full(T, np.concatenate([prompt, d_tokens]))[len(prompt) - 1:]
    got = {}
    for mode in ("block", "rows"):
        if mode == "rows":
            monkeypatch.setenv("STAIRS_NO_BLOCK_PREFILL", "1")
        with pkg.Stairs(target, draft, k_max=3, max_seq=640) as s:
            s.prefill(prompt)
            _, _, logits = s.verify_tokens(d_tokens, logits=True)
            got[mode] = logits.copy()
        assert np.max(np.abs(got[mode] - ref)) < LOGIT_TOL_BF16, mode
    assert np.max(np.abs(got["block"] - got["rows"])) < 2e-3


@pytest.mark.parametrize("P", [64, 65, 66, 97, 129, 513, 514, 545, 577])
def test_block_prefill_row_counts(P, monkeypatch):
    """Block ingestion at the row counts where its pieces change: the smallest block (P - 1 = 64 rows; one row fewer goes through the decode kernels), whole
    32-row groups with and without a ragged group, one row past a 512-row block; against the row prefill."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=P, G=8)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    got = {}
    for mode in ("block", "rows"):
        if mode == "rows":
            monkeypatch.setenv("STAIRS_NO_BLOCK_PREFILL", "1")
        with pkg.Stairs(target, draft, k_max=2, max_seq=P + 16) as s:
            s.prefill(prompt)
            _, _, logits = s.verify_tokens([5, 6], logits=True)
            got[mode] = logits.copy()
    assert np.max(np.abs(got["block"] - got["rows"])) < 2e-3, np.max(np.abs(got["block"] - got["rows"]))


def test_adaptive_draft_length_on_gpu():
    """stairs_decode_adaptive: same tokens as plain greedy decoding on the GPU bit for bit, and on the fp32 pair the
    same iterations and acceptance counts as the oracle's adaptive loop (both follow the rule stated in the header)."""
    w = si.scaled_workload("cfg1_tiny_fp32")
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    G, k_first, k_max = 60, 2, 6
    T, D = so.OracleModel(target, np.float64), so.OracleModel(draft, np.float64)
    want = so.stairs_adaptive(T, D, prompt, G, k_first, k_max)
    with pkg.Stairs(target, draft, k_max=k_max, max_seq=160) as s:
        plain, _ = s.generate(prompt, G, 0)
        s.prefill(prompt)
        toks, st = s.decode_adaptive(G, k_first)
        assert np.array_equal(toks, plain)
        assert list(toks) == want.tokens
        assert st.iterations == len(want.iterations)
        assert st.accepted == sum(it.n_accepted for it in want.iterations)
        with pytest.raises(pkg.StairsError) as e:
            s.decode_adaptive(4, 0)
        assert e.value.code == -1
    w2 = si.scaled_workload("cfg2_125m", target=dict(n_layers=3, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                            draft=dict(kind="prefix", n_layers=1), P=70, G=40)
    t2, d2 = si.make_pair(w2)
    p2 = si.make_prompt(w2)
    with pkg.Stairs(t2, d2, k_max=8, max_seq=160) as s:
        plain, _ = s.generate(p2, 40, 0)
        s.prefill(p2)
        toks, st = s.decode_adaptive(40, 3)
        assert np.array_equal(toks, plain) and st.tokens == 40


def test_longest_context_stair_batches(monkeypatch):
    """max_seq = 60000 (the most the library takes: 469 attention chunks, the stand-alone chunk merge with its
    largest table).  The 32-row stair batch is compared with the oracle's logits stored by
    tests/golden/make_long_context_logits.py; batches of 8 rows and 1 row from the same state must give the
    same bits for the rows they share (a row's result does not depend on how many rows ride along)."""
    import os
    g = np.load(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "long_context_logits.npz"))
    P, max_seq, d, want = int(g["P"]), int(g["max_seq"]), g["draft"], g["logits"]
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=2, d_model=256, n_heads=2, d_ffn=256, vocab=512),
                           draft=dict(kind="prefix", n_layers=1), P=P, G=1)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    got = {}
    for kk in (31, 7, 0):
        _log(f"longest context: block prefill P={P}, stair batch of {kk + 1} rows")
        with pkg.Stairs(target, draft, k_max=31, max_seq=max_seq) as s:
            s.prefill(prompt)
            tgt, n, lg = s.verify_tokens(d[:kk], logits=True)
            got[kk] = (tgt.copy(), lg.copy())
    err = float(np.max(np.abs(got[31][1].astype(np.float64) - want)))
    _log(f"longest context: max logit error {err:.3g}")
    assert err <= LOGIT_TOL_BF16
    for i in range(32):
        assert eps_ok(want[i], int(got[31][0][i]))
    assert np.array_equal(got[7][1], got[31][1][:8])
    assert np.array_equal(got[0][1], got[31][1][:1])
    # the prompt ingested 32 rows at a time through the decoding kernels instead of by blocks
    monkeypatch.setenv("STAIRS_NO_BLOCK_PREFILL", "1")
    _log("longest context: row prefill")
    with pkg.Stairs(target, draft, k_max=31, max_seq=max_seq) as s:
        s.prefill(prompt)
        tgt, n, lg = s.verify_tokens(d, logits=True)
    err = float(np.max(np.abs(lg.astype(np.float64) - want)))
    _log(f"longest context, row prefill: max logit error {err:.3g}")
    assert err <= LOGIT_TOL_BF16


def test_five_to_eight_rows_on_wide_projections():
    """Stair batches of 5..8 rows on a model whose projections are wide and long enough for the LDS-resident GEMM in
    its one-work-group-per-CU form (d_model 2048: k = 2048, QKV 384 tiles, gate/up 256, unembedding 512; the down
    projection with k = 2048 too): logits against the oracle for every such row count, the rows of a shorter batch
    bit-identical to the same rows of the longest one, and the tokens of every k equal to plain greedy decoding."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=2, d_model=2048, n_heads=16, d_ffn=2048, vocab=8192),
                           draft=dict(kind="prefix", n_layers=1), P=70, G=12)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    T = so.OracleModel(target, np.float64)
    rng = np.random.default_rng([w["seed"], 5])
    d = [int(x) for x in rng.integers(0, 8192, 8)]
    want = so.forward_full(T, [int(x) for x in prompt] + d)[len(prompt) - 1:]        # rows of the stair batch
    with pkg.Stairs(target, draft, k_max=8, max_seq=128) as s:
        logits = {}
        for kk in (8, 7, 6, 5, 4, 3, 0):
            s.prefill(prompt)
            tgt, n, lg = s.verify_tokens(d[:kk], logits=True)
            err = float(np.max(np.abs(lg.astype(np.float64) - want[:kk + 1])))
            _log(f"{kk + 1} rows: max logit error {err:.3g}")
            assert err <= LOGIT_TOL_BF16
            logits[kk] = lg.copy()
        for kk in (7, 6, 5, 4, 3, 0):
            assert np.array_equal(logits[kk], logits[8][:kk + 1]), kk
        base, _ = s.generate(prompt, w["G"], 0)
        for kk in (4, 5, 6, 7, 8):
            toks, _ = s.generate(prompt, w["G"], kk)
            assert np.array_equal(toks, base), kk


@pytest.mark.parametrize("case", range(14))
def test_shape_sweep_against_the_oracle(case):
    """Seeded sweep over the documented shape limits: widths with an odd number of 256-wide weight units (768, 1280),
    feed-forward widths that are not multiples of 512, vocabularies that are multiples of 16 but not of 64, both head
    sizes, prompt lengths from 1 to a few hundred, draft lengths on every GEMM / attention path (<= 4 rows, 5..8,
    9..16, 17..32 rows)."""
    rng = np.random.default_rng([2024, case])
    d = int(rng.choice([256, 512, 768, 1280]))
    hd = int(rng.choice([64, 128]))
    f = int(rng.choice([256, 768, 1024, 2816]))
    V = int(rng.choice([272, 1008, 2048, 4112]))
    k = int([0, 1, 2, 3, 4, 5, 7, 8, 9, 12, 15, 16, 23, 31][case])
    P = int(rng.integers(1, 300))
    G = 2 * (k + 1) + 6
    w = si.scaled_workload("cfg2_125m", seed=5000 + case,
                           target=dict(n_layers=2, d_model=d, n_heads=d // hd, d_ffn=f, vocab=V),
                           draft=dict(kind="prefix", n_layers=1), P=P, G=G)
    _log(f"shape sweep {case}: d={d} hd={hd} f={f} V={V} P={P} k={k}")
    target, draft = si.make_pair(w)
    res = run_side_by_side(target, draft, si.make_prompt(w), G, k, np.float64, LOGIT_TOL_BF16)
    assert res["max_logit_err"] < 5e-3


def test_long_generation_and_two_contexts_interleaved():
    """700 tokens after a 300-token prompt (the attention grid grows from 3 to 8 chunks, so several captured
    iterations are made and replayed) on two contexts used in turns: every result equals plain greedy decoding and
    does not depend on what the other context did in between."""
    w = si.scaled_workload("cfg2_125m", target=dict(n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=2048),
                           draft=dict(kind="prefix", n_layers=1), P=300, G=700)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    other = si.make_prompt(w)[::-1].copy()
    with pkg.Stairs(target, draft, k_max=5, max_seq=1100) as a, pkg.Stairs(target, draft, k_max=5, max_seq=1100) as b:
        base, st0 = a.generate(prompt, 700, 0)
        base_other, _ = b.generate(other, 700, 0)
        assert st0.iterations == 700 and not np.array_equal(base, base_other)
        # turn by turn: a decodes 350 tokens, b runs a whole generation, a continues
        a.prefill(prompt)
        first, _ = a.decode(350, 3)
        got_other, _ = b.generate(other, 700, 5)
        second, st = a.decode(350, 3)
        assert np.array_equal(np.concatenate([first, second]), base)
        assert np.array_equal(got_other, base_other)
        assert st.iterations < 350
