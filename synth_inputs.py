"""Seeded synthetic inputs (model weights and prompts) for stairs-assisted greedy generation.

This module only *draws* inputs; it holds none of the method's arithmetic (no forward pass,
no argmax, no acceptance rule).  Both the CPU oracle and the HIP library are fed from it so
that they see bit-identical weights and prompts.  It imports neither of them.

The workloads stand in for the paper's trained T5 checkpoints and its single translation
prompt (Sec. 2.3, Sec. 4.2), which cannot be obtained here: the benchmark workloads are
decoder-only pre-RMSNorm transformers (RoPE, SwiGLU, untied embedding / unembedding) with
N(0, 0.02) weights, and every prompt is uniform over the vocabulary.  The second half of the
file draws encoder-decoder models in the shape of the paper's own model family.

Tensor layout: every matrix is ``[out_features, in_features]`` row-major.  A model whose
dtype is ``"bf16"`` stores its matrices as ``uint16`` arrays holding bfloat16 bit patterns
(fp32 draws rounded to nearest-even); ``"fp32"`` models store ``float32``.  Norm gains are
always ``float32`` ones.
"""
from __future__ import annotations

import copy
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

WEIGHT_STD = 0.02
ROPE_THETA = 10000.0
RMS_EPS = 1e-5

# tensor ids inside one layer (the seed of a tensor is [model_seed, layer * 16 + id])
_T_WQ, _T_WK, _T_WV, _T_WO, _T_GATE, _T_UP, _T_DOWN = range(7)
_T_TOK_EMB = 1_000_000
_T_LM_HEAD = 1_000_001
_T_PROMPT = 0xFFFF


@dataclass
class ModelInputs:
    """Weights of one decoder-only model plus its shape parameters."""
    n_layers: int
    d_model: int
    n_heads: int
    d_ffn: int
    vocab: int
    dtype: str                      # "fp32" | "bf16"
    rope_theta: float = ROPE_THETA
    rms_eps: float = RMS_EPS
    tok_emb: Optional[np.ndarray] = None        # [V, d]
    lm_head: Optional[np.ndarray] = None        # [V, d]
    final_norm: Optional[np.ndarray] = None     # [d] fp32
    layers: List[Dict[str, np.ndarray]] = field(default_factory=list)

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads

    def n_params(self) -> int:
        d, f = self.d_model, self.d_ffn
        return self.n_layers * (4 * d * d + 3 * d * f) + self.vocab * d

    def weight_bytes_streamed(self) -> int:
        """Bytes of matrices one forward pass has to read (all layers + unembedding)."""
        return self.n_params() * (2 if self.dtype == "bf16" else 4)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def _draw(seed: int, tensor_id: int, shape, scale: float, dtype: str) -> np.ndarray:
    rng = np.random.default_rng([seed, tensor_id])
    w = rng.standard_normal(shape, dtype=np.float32)
    w *= np.float32(WEIGHT_STD * scale)
    return bf16_round(w) if dtype == "bf16" else w


def make_model(seed: int, n_layers: int, d_model: int, n_heads: int, d_ffn: int, vocab: int,
               dtype: str, deep_from: Optional[int] = None, deep_scale: float = 1.0,
               threads: int = 8) -> ModelInputs:
    """Draw one model.  Layers with index >= ``deep_from`` have both matrices that write into
    the residual stream (attention output projection and FFN down projection) scaled by
    ``deep_scale`` before rounding."""
    assert d_model % n_heads == 0
    m = ModelInputs(n_layers, d_model, n_heads, d_ffn, vocab, dtype)
    d, f = d_model, d_ffn
    jobs = [("tok_emb", None, _T_TOK_EMB, (vocab, d), 1.0),
            ("lm_head", None, _T_LM_HEAD, (vocab, d), 1.0)]
    for l in range(n_layers):
        s = deep_scale if (deep_from is not None and l >= deep_from) else 1.0
        jobs += [("wq", l, l * 16 + _T_WQ, (d, d), 1.0), ("wk", l, l * 16 + _T_WK, (d, d), 1.0),
                 ("wv", l, l * 16 + _T_WV, (d, d), 1.0), ("wo", l, l * 16 + _T_WO, (d, d), s),
                 ("w_gate", l, l * 16 + _T_GATE, (f, d), 1.0), ("w_up", l, l * 16 + _T_UP, (f, d), 1.0),
                 ("w_down", l, l * 16 + _T_DOWN, (d, f), s)]
    m.layers = [dict(attn_norm=np.ones(d, np.float32), ffn_norm=np.ones(d, np.float32))
                for _ in range(n_layers)]
    m.final_norm = np.ones(d, np.float32)

    def run(job):
        name, l, tid, shape, s = job
        return name, l, _draw(seed, tid, shape, s, dtype)

    with ThreadPoolExecutor(max(1, threads)) as ex:
        for name, l, arr in ex.map(run, jobs):
            if l is None:
                setattr(m, name, arr)
            else:
                m.layers[l][name] = arr
    return m


def prefix_draft(target: ModelInputs, n_layers: int) -> ModelInputs:
    """Draft model made of the target's first ``n_layers`` layers with the target's final norm
    and unembedding; every tensor is the *same array object* as the target's."""
    assert 1 <= n_layers <= target.n_layers
    dr = copy.copy(target)
    dr.n_layers = n_layers
    dr.layers = target.layers[:n_layers]
    return dr


# ----------------------------------------------------------------------------------------
# The five benchmark workloads.  P = prompt length, G = tokens to generate, ks = draft lengths.
# ----------------------------------------------------------------------------------------
WORKLOADS = {
    "cfg1_tiny_fp32": dict(seed=101, dtype="fp32",
                           target=dict(n_layers=4, d_model=256, n_heads=4, d_ffn=1024, vocab=1024),
                           draft=dict(kind="prefix", n_layers=2), deep_scale=0.05,
                           P=32, G=64, ks=[4]),
    "cfg2_125m": dict(seed=102, dtype="bf16",
                      target=dict(n_layers=12, d_model=768, n_heads=12, d_ffn=3072, vocab=32000),
                      draft=dict(kind="prefix", n_layers=3), deep_scale=0.1,
                      P=128, G=256, ks=[2, 4, 8]),
    "cfg3_1b": dict(seed=103, dtype="bf16",
                    target=dict(n_layers=16, d_model=2048, n_heads=16, d_ffn=8192, vocab=32000),
                    draft=dict(kind="prefix", n_layers=4), deep_scale=0.1,
                    P=512, G=512, ks=[4, 8]),
    "cfg4_7b": dict(seed=104, dtype="bf16",
                    target=dict(n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000),
                    draft=dict(kind="prefix", n_layers=4), deep_scale=0.1,
                    P=2048, G=256, ks=list(range(1, 17))),
    # same target tensors as cfg4 (same seed), independent random draft
    "cfg5_7b_longctx_indep_draft": dict(seed=104, dtype="bf16",
                                        target=dict(n_layers=32, d_model=4096, n_heads=32, d_ffn=11008,
                                                    vocab=32000),
                                        target_deep_from=4,
                                        draft=dict(kind="independent", seed=105, n_layers=6, d_model=1024,
                                                   n_heads=16, d_ffn=4096),
                                        deep_scale=0.1, P=8192, G=256, ks=[4]),
}


def scaled_workload(name: str, **over) -> dict:
    """A copy of a workload with some entries replaced (used by tests that need the same
    structure at a size the oracle finishes quickly)."""
    w = copy.deepcopy(WORKLOADS[name])
    for key, val in over.items():
        if isinstance(val, dict) and isinstance(w.get(key), dict):
            w[key].update(val)
        else:
            w[key] = val
    return w


def make_pair(workload, threads: int = 8):
    """-> (target, draft) ModelInputs for a workload name or dict."""
    w = WORKLOADS[workload] if isinstance(workload, str) else workload
    t, dr = w["target"], w["draft"]
    if dr["kind"] == "prefix":
        deep_from = w.get("target_deep_from", dr["n_layers"])
    else:
        deep_from = w.get("target_deep_from", None)
    target = make_model(w["seed"], dtype=w["dtype"], deep_from=deep_from,
                        deep_scale=w.get("deep_scale", 1.0), threads=threads, **t)
    if dr["kind"] == "prefix":
        draft = prefix_draft(target, dr["n_layers"])
    else:
        draft = make_model(dr["seed"], dr["n_layers"], dr["d_model"], dr["n_heads"], dr["d_ffn"],
                           t["vocab"], w["dtype"], threads=threads)
    return target, draft


def make_prompt(workload, P: Optional[int] = None) -> np.ndarray:
    """Uniform-random prompt token ids (int32) for a workload."""
    w = WORKLOADS[workload] if isinstance(workload, str) else workload
    rng = np.random.default_rng([w["seed"], _T_PROMPT])
    full = rng.integers(0, w["target"]["vocab"], size=w["P"], dtype=np.int64).astype(np.int32)
    return full if P is None else full[:P].copy()


# ----------------------------------------------------------------------------------------
# Encoder-decoder models (the model family of the paper's experiments, Sec. 2.3, Sec. 4.3, Sec. 4.4: T5)
# ----------------------------------------------------------------------------------------
REL_BUCKETS = 32
REL_MAX_DISTANCE = 128
REL_BIAS_STD = 0.5
T5_EPS = 1e-6
DECODER_START = 0          # the decoder sequence begins with this token id
# embeddings are drawn 10 x wider than the matrices: with the ReLU feed-forward's one-sided output a narrower
# embedding lets a token-independent direction dominate the residual stream and every model emits one token forever
EMB_SCALE_ENCDEC = 10.0

# tensor ids inside one encoder-decoder layer
(_E_WQ, _E_WK, _E_WV, _E_WO, _E_WIN, _E_WOUT, _E_CQ, _E_CK, _E_CV, _E_CO) = range(10)
_T_ENC_BIAS = 1_000_002
_T_DEC_BIAS = 1_000_003
_DEC_LAYER0 = 10_000       # decoder layer l draws from tensor ids (_DEC_LAYER0 + l) * 16 + id


@dataclass
class EncDecInputs:
    """Weights of one encoder-decoder model in the shape of the original T5: RMS layer norm before every block,
    attention without 1/sqrt(head_dim) and with a learned bias per (bucket of relative position, head) shared by the
    layers of a stack, ReLU feed-forward without gate, no biases elsewhere, untied unembedding.  The attention width
    n_heads * head_dim need not equal d_model.  Matrices [out, in]; bf16 bit patterns (uint16); gains and bias
    tables float32."""
    n_enc_layers: int
    n_dec_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"
    rel_buckets: int = REL_BUCKETS
    rel_max_distance: int = REL_MAX_DISTANCE
    rms_eps: float = T5_EPS
    tok_emb: Optional[np.ndarray] = None        # [V, d] shared by encoder and decoder
    lm_head: Optional[np.ndarray] = None        # [V, d]
    enc_rel_bias: Optional[np.ndarray] = None   # [buckets, H] float32
    dec_rel_bias: Optional[np.ndarray] = None   # [buckets, H] float32
    enc_final_norm: Optional[np.ndarray] = None
    dec_final_norm: Optional[np.ndarray] = None
    enc_layers: List[Dict[str, np.ndarray]] = field(default_factory=list)   # attn_norm wq wk wv wo ffn_norm w_in w_out
    dec_layers: List[Dict[str, np.ndarray]] = field(default_factory=list)   # + cross_norm cq ck cv co

    @property
    def d_attn(self) -> int:
        return self.n_heads * self.head_dim

    def decoder_bytes_streamed(self) -> int:
        """Bytes of matrices one decoder forward reads (all decoder layers + unembedding)."""
        d, a, f = self.d_model, self.d_attn, self.d_ffn
        return (self.n_dec_layers * (8 * d * a + 2 * d * f) + self.vocab * d) * 2


def make_encdec_model(seed: int, n_enc_layers: int, n_dec_layers: int, d_model: int, n_heads: int, head_dim: int,
                      d_ffn: int, vocab: int, deep_from: Optional[int] = None, deep_scale: float = 1.0,
                      threads: int = 8) -> EncDecInputs:
    """Draw one encoder-decoder model; ``deep_from`` / ``deep_scale`` as in make_model, applied to the matrices
    that write into the residual stream (wo, co, w_out) of encoder and decoder layers with index >= deep_from."""
    m = EncDecInputs(n_enc_layers, n_dec_layers, d_model, n_heads, head_dim, d_ffn, vocab)
    d, a, f = d_model, n_heads * head_dim, d_ffn
    jobs = [("tok_emb", None, None, _T_TOK_EMB, (vocab, d), EMB_SCALE_ENCDEC),
            ("lm_head", None, None, _T_LM_HEAD, (vocab, d), 1.0)]
    for stack, n, base in (("enc", n_enc_layers, 0), ("dec", n_dec_layers, _DEC_LAYER0)):
        for l in range(n):
            s = deep_scale if (deep_from is not None and l >= deep_from) else 1.0
            t = (base + l) * 16
            jobs += [("wq", stack, l, t + _E_WQ, (a, d), 1.0), ("wk", stack, l, t + _E_WK, (a, d), 1.0),
                     ("wv", stack, l, t + _E_WV, (a, d), 1.0), ("wo", stack, l, t + _E_WO, (d, a), s),
                     ("w_in", stack, l, t + _E_WIN, (f, d), 1.0), ("w_out", stack, l, t + _E_WOUT, (d, f), s)]
            if stack == "dec":
                jobs += [("cq", stack, l, t + _E_CQ, (a, d), 1.0), ("ck", stack, l, t + _E_CK, (a, d), 1.0),
                         ("cv", stack, l, t + _E_CV, (a, d), 1.0), ("co", stack, l, t + _E_CO, (d, a), s)]
    ones = lambda: np.ones(d, np.float32)                                   # noqa: E731
    m.enc_layers = [dict(attn_norm=ones(), ffn_norm=ones()) for _ in range(n_enc_layers)]
    m.dec_layers = [dict(attn_norm=ones(), cross_norm=ones(), ffn_norm=ones()) for _ in range(n_dec_layers)]
    m.enc_final_norm, m.dec_final_norm = ones(), ones()
    for name, tid in (("enc_rel_bias", _T_ENC_BIAS), ("dec_rel_bias", _T_DEC_BIAS)):
        rng = np.random.default_rng([seed, tid])
        setattr(m, name, (rng.standard_normal((m.rel_buckets, n_heads), dtype=np.float32)
                          * np.float32(REL_BIAS_STD)).astype(np.float32))

    def run(job):
        name, stack, l, tid, shape, s = job
        return name, stack, l, _draw(seed, tid, shape, s, "bf16")

    with ThreadPoolExecutor(max(1, threads)) as ex:
        for name, stack, l, arr in ex.map(run, jobs):
            if stack is None:
                setattr(m, name, arr)
            else:
                (m.enc_layers if stack == "enc" else m.dec_layers)[l][name] = arr
    return m


def encdec_prefix_draft(target: EncDecInputs, n_enc_layers: int, n_dec_layers: int) -> EncDecInputs:
    """Draft made of the target's first encoder and decoder layers with the target's final norms, bias tables and
    unembedding; every tensor is the same array object as the target's."""
    assert 1 <= n_enc_layers <= target.n_enc_layers and 1 <= n_dec_layers <= target.n_dec_layers
    dr = copy.copy(target)
    dr.n_enc_layers, dr.n_dec_layers = n_enc_layers, n_dec_layers
    dr.enc_layers = target.enc_layers[:n_enc_layers]
    dr.dec_layers = target.dec_layers[:n_dec_layers]
    return dr


# S = source (encoder) length, G = tokens to generate.  Shapes of the checkpoints the paper names (Sec. 2.3):
# "t5_large" 24+24 layers, d 1024, 16 heads of 64, ffn 4096; "t5_3b" 24+24 layers, d 1024, 32 heads of 128, ffn 16384;
# vocabulary 32128.  The draft is the target's first 6+6 layers (the depth of the small checkpoint): an independently
# drawn random draft would never agree with the target.  deep_scale sets how much the layers the draft lacks change
# the residual stream, i.e. how often the draft is right (0.03: about 3 tokens per iteration at k = 4 on the large
# shape; at 0.05 these random models fall into a short cycle that the draft always predicts).
ENCDEC_WORKLOADS = {
    "t5_tiny": dict(seed=201, target=dict(n_enc_layers=3, n_dec_layers=3, d_model=256, n_heads=4, head_dim=64,
                                          d_ffn=512, vocab=2048),
                    draft=dict(kind="prefix", n_enc_layers=1, n_dec_layers=1), deep_scale=0.1, S=48, G=48, ks=[4]),
    "t5_large_shape": dict(seed=202, target=dict(n_enc_layers=24, n_dec_layers=24, d_model=1024, n_heads=16,
                                                 head_dim=64, d_ffn=4096, vocab=32128),
                           draft=dict(kind="prefix", n_enc_layers=6, n_dec_layers=6), deep_scale=0.03,
                           S=128, G=256, ks=[1, 2, 3, 4, 6, 8]),
    "t5_3b_shape": dict(seed=203, target=dict(n_enc_layers=24, n_dec_layers=24, d_model=1024, n_heads=32,
                                              head_dim=128, d_ffn=16384, vocab=32128),
                        draft=dict(kind="prefix", n_enc_layers=6, n_dec_layers=6), deep_scale=0.03,
                        S=128, G=256, ks=[1, 2, 3, 4, 6, 8]),
}


def scaled_encdec_workload(name: str, **over) -> dict:
    w = copy.deepcopy(ENCDEC_WORKLOADS[name])
    for key, val in over.items():
        if isinstance(val, dict) and isinstance(w.get(key), dict):
            w[key].update(val)
        else:
            w[key] = val
    return w


def make_encdec_pair(workload, threads: int = 8):
    """-> (target, draft) EncDecInputs for a workload name or dict."""
    w = ENCDEC_WORKLOADS[workload] if isinstance(workload, str) else workload
    t, dr = w["target"], w["draft"]
    if dr["kind"] == "prefix":
        target = make_encdec_model(w["seed"], deep_from=min(dr["n_enc_layers"], dr["n_dec_layers"]),
                                   deep_scale=w.get("deep_scale", 1.0), threads=threads, **t)
        return target, encdec_prefix_draft(target, dr["n_enc_layers"], dr["n_dec_layers"])
    target = make_encdec_model(w["seed"], threads=threads, **t)
    draft = make_encdec_model(dr["seed"], dr["n_enc_layers"], dr["n_dec_layers"], dr["d_model"], dr["n_heads"],
                              dr["head_dim"], dr["d_ffn"], t["vocab"], threads=threads)
    return target, draft


def make_source(workload, S: Optional[int] = None) -> np.ndarray:
    """Uniform-random source (encoder) token ids (int32) for an encoder-decoder workload."""
    w = ENCDEC_WORKLOADS[workload] if isinstance(workload, str) else workload
    rng = np.random.default_rng([w["seed"], _T_PROMPT])
    full = rng.integers(1, w["target"]["vocab"], size=w["S"], dtype=np.int64).astype(np.int32)
    return full if S is None else full[:S].copy()
