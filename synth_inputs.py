"""Seeded synthetic inputs (model weights and prompts) for stairs-assisted greedy generation.

This module only *draws* inputs; it holds none of the method's arithmetic (no forward pass,
no argmax, no acceptance rule).  Both the CPU oracle and the HIP library are fed from it so
that they see bit-identical weights and prompts.  It imports neither of them.

The workloads stand in for the paper's trained T5 checkpoints and its single translation
prompt (Sec. 2.3, Sec. 4.2), which cannot be obtained here: every model is a decoder-only
pre-RMSNorm transformer (RoPE, SwiGLU, untied embedding / unembedding) with N(0, 0.02)
weights, and every prompt is uniform over the vocabulary.

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
