"""CPU oracle for "stairs" assisted greedy generation.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this file.
It shares no code with the HIP library and never imports it; the library never imports it.

What it computes
----------------
* The *definition* of the result: stand-alone greedy decoding of the target model
  (Sec. 3.1: feed the tokens, take the vocabulary entry with the highest probability, append,
  repeat).  The paper's claim (abstract, Sec. 1) is that the stairs method returns this same
  output, only with fewer target-model iterations.
* The method itself, step by step in the paper's order (Sec. 3.3): the assistant model
  generates k tokens greedily; the sequence is broken into the k+1 "stair" subsequences
  (prefix, prefix+1 token, ..., prefix+k tokens), stacked as a batch; the main model predicts
  one more token for each row; "stairs" validation walks the rows, keeping a ground-truth
  vector, and stops at the first row that does not equal it.
* A KV-cached variant of the same loop (the paper is silent on caching; this is the
  realisation the GPU library uses: one causal forward over [last token, d_1..d_k] yields the
  k+1 last-position logits of the stair batch).  It is checked against the literal one.

Model family (not in the paper, fixed by the benchmark workloads): decoder-only, pre-RMSNorm,
multi-head causal attention with rotary position embedding in the rotate-half pairing
(i, i + hd/2), theta = 10000, SwiGLU feed-forward, no biases, untied embedding/unembedding,
attention scale 1/sqrt(hd), argmax ties broken towards the lowest vocabulary index.

Parity pins (tests/test_oracle_*.py): library routines of PyTorch CPU for every forward
component, closed forms for degenerate models, the greedy-equivalence invariant, acceptance
count closed forms, hand-derived validation cases under tests/golden/.  Nothing in the paper
prints a numeric value for this path (its figures carry the only worked example and are not
part of the text), so no value here is pinned to a number printed by the paper.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np


# ----------------------------------------------------------------------------------------
# model container
# ----------------------------------------------------------------------------------------
def _decode(t: np.ndarray, dtype) -> np.ndarray:
    """Weights arrive as float32 or as uint16 bfloat16 bit patterns; return real numbers."""
    if t.dtype == np.uint16:
        return (t.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(dtype, copy=False)
    return t.astype(dtype, copy=False)


class OracleModel:
    """Real-valued view of one set of model inputs.

    ``keep=True`` decodes every matrix once and keeps it (fast repeated forwards, memory =
    n_params * itemsize); ``keep=False`` decodes a layer each time it is used.
    """

    def __init__(self, inputs, dtype=np.float32, keep: bool = True):
        self.inp = inputs
        self.dtype = np.dtype(dtype)
        self.n_layers = inputs.n_layers
        self.d = inputs.d_model
        self.H = inputs.n_heads
        self.hd = inputs.d_model // inputs.n_heads
        self.f = inputs.d_ffn
        self.V = inputs.vocab
        self.theta = float(inputs.rope_theta)
        self.eps = float(inputs.rms_eps)
        self.keep = keep
        self._cache = {}

    def _get(self, key, arr):
        if not self.keep:
            return _decode(arr, self.dtype)
        got = self._cache.get(key)
        if got is None:
            got = self._cache[key] = _decode(arr, self.dtype)
        return got

    def tok_emb(self):
        return self._get("tok_emb", self.inp.tok_emb)

    def lm_head(self):
        return self._get("lm_head", self.inp.lm_head)

    def final_norm(self):
        return self._get("final_norm", self.inp.final_norm)

    def layer(self, l: int, name: str):
        return self._get((l, name), self.inp.layers[l][name])


# ----------------------------------------------------------------------------------------
# forward components
# ----------------------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * g   along the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope_cos_sin(positions: np.ndarray, hd: int, theta: float, dtype) -> Tuple[np.ndarray, np.ndarray]:
    """cos/sin of position * theta^(-2i/hd), i = 0..hd/2-1.  Angles are formed in float64 so
    that position 8000+ does not lose the low bits of the angle; the result is cast."""
    i = np.arange(hd // 2, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / hd)
    ang = positions.astype(np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang).astype(dtype), np.sin(ang).astype(dtype)


def apply_rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """x: [T, H, hd]; cos, sin: [T, hd/2].  Pair (i, i+hd/2) is rotated by the angle of i."""
    half = x.shape[-1] // 2
    a, b = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    s = s - np.max(s, axis=-1, keepdims=True)
    e = np.exp(s)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos0: int) -> np.ndarray:
    """Causal multi-head attention.  q: [M, H, hd] at absolute positions q_pos0..q_pos0+M-1;
    k, v: [T, H, hd] at positions 0..T-1.  Query at position p attends to keys 0..p."""
    M, H, hd = q.shape
    T = k.shape[0]
    scale = 1.0 / np.sqrt(hd)
    out = np.empty_like(q)
    key_pos = np.arange(T)[None, :]
    q_pos = (q_pos0 + np.arange(M))[:, None]
    hidden = key_pos > q_pos                               # [M, T]
    for h in range(H):
        s = (q[:, h, :] @ k[:, h, :].T) * scale            # [M, T]
        s = np.where(hidden, -np.inf, s)
        out[:, h, :] = softmax_rows(s) @ v[:, h, :]
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


@dataclass
class KVCache:
    """Per-layer key/value history [capacity, H, hd] and the number of valid positions."""
    k: List[np.ndarray]
    v: List[np.ndarray]
    length: int = 0

    @staticmethod
    def empty(model: OracleModel, capacity: int) -> "KVCache":
        shape = (capacity, model.H, model.hd)
        return KVCache([np.zeros(shape, model.dtype) for _ in range(model.n_layers)],
                       [np.zeros(shape, model.dtype) for _ in range(model.n_layers)], 0)


def _forward(model: OracleModel, ids: np.ndarray, pos0: int, cache: Optional[KVCache],
             kv_round=None) -> np.ndarray:
    """Rows ``ids`` sit at positions pos0..pos0+M-1.  Without a cache pos0 must be 0 and the rows
    are the whole sequence; with a cache, positions < pos0 come from it and the new keys/values
    are written at pos0.. (cache.length is NOT changed here: the caller decides what stays).
    ``kv_round``: optional function applied to keys and values before they are used/stored (the
    GPU keeps its cache in bfloat16; the parity tests can ask the oracle for the same storage
    rounding to separate that effect from arithmetic error; default: none)."""
    if hasattr(model, "decoder_forward"):      # the decoder of an encoder-decoder model bound to its source
        return model.decoder_forward(ids, pos0, cache, kv_round)
    dt = model.dtype
    ids = np.asarray(ids, dtype=np.int64)
    M = ids.shape[0]
    x = model.tok_emb()[ids].astype(dt)                                    # [M, d]
    pos = pos0 + np.arange(M)
    cos, sin = rope_cos_sin(pos, model.hd, model.theta, dt)
    for l in range(model.n_layers):
        h = rmsnorm(x, model.layer(l, "attn_norm"), model.eps)
        q = (h @ model.layer(l, "wq").T).reshape(M, model.H, model.hd)
        k = (h @ model.layer(l, "wk").T).reshape(M, model.H, model.hd)
        v = (h @ model.layer(l, "wv").T).reshape(M, model.H, model.hd)
        q = apply_rope(q, cos, sin)
        k = apply_rope(k, cos, sin)
        if kv_round is not None:
            k, v = kv_round(k), kv_round(v)
        if cache is None:
            assert pos0 == 0
            k_all, v_all = k, v
        else:
            cache.k[l][pos0:pos0 + M] = k
            cache.v[l][pos0:pos0 + M] = v
            k_all, v_all = cache.k[l][:pos0 + M], cache.v[l][:pos0 + M]
        a = attention(q, k_all, v_all, pos0).reshape(M, model.d)
        x = x + a @ model.layer(l, "wo").T
        h = rmsnorm(x, model.layer(l, "ffn_norm"), model.eps)
        gate = h @ model.layer(l, "w_gate").T
        up = h @ model.layer(l, "w_up").T
        x = x + (silu(gate) * up) @ model.layer(l, "w_down").T
    h = rmsnorm(x, model.final_norm(), model.eps)
    return h @ model.lm_head().T                                           # [M, V]


def forward_full(model: OracleModel, ids: Sequence[int]) -> np.ndarray:
    """Plain causal forward of a whole sequence, no cache: logits [T, V]."""
    return _forward(model, np.asarray(ids), 0, None)


def forward_cached(model: OracleModel, cache: KVCache, ids: Sequence[int], pos0: int,
                   kv_round=None) -> np.ndarray:
    return _forward(model, np.asarray(ids), pos0, cache, kv_round)


def greedy_token(logits_row: np.ndarray) -> int:
    """Highest-probability vocabulary entry (Sec. 3.1); ties -> lowest index."""
    return int(np.argmax(logits_row))


# ----------------------------------------------------------------------------------------
# the definition: stand-alone greedy generation of the main model (Sec. 3.1)
# ----------------------------------------------------------------------------------------
def greedy_bruteforce(model: OracleModel, prompt: Sequence[int], G: int, eos: Optional[int] = None) -> List[int]:
    """eos: the main model's end token; the answer is complete once it has been emitted (Sec. 3.2, last sentence:
    the cycle runs until the prompt is fully answered; reading: for a model with an end token that is the moment it
    is predicted), at the latest after G tokens."""
    seq = [int(t) for t in prompt]
    for _ in range(G):
        seq.append(greedy_token(forward_full(model, seq)[-1]))
        if eos is not None and seq[-1] == eos:
            break
    return seq[len(prompt):]


def cut_after_end_token(new_tokens: Sequence[int], eos: Optional[int]) -> Tuple[List[int], bool]:
    """What an iteration may append when the answer ends at the first end token: the tokens up to and including it
    (the walk of Sec. 3.3 returned more, but nothing follows the end of the answer), and whether it was there."""
    out = [int(x) for x in new_tokens]
    if eos is not None and eos in out:
        return out[:out.index(eos) + 1], True
    return out, False


# ----------------------------------------------------------------------------------------
# "stairs" batch validation (Sec. 3.3, second and third paragraphs)
# ----------------------------------------------------------------------------------------
def stairs_validate(rows: List[List[int]], predicted: Sequence[int]) -> List[int]:
    """rows[i] is the i-th stair (prefix plus the first i assistant tokens); predicted[i] is the
    token the main model appended to rows[i].  The first row with its prediction is the ground
    truth.  Each following row is compared, as a whole vector, with the ground truth (i.e. the
    row's output sequence without its own new last token); on a match the ground truth becomes
    that row plus its prediction; the first mismatch ends the walk.  Returns the ground truth."""
    ground_truth = list(rows[0]) + [int(predicted[0])]
    for i in range(1, len(rows)):
        if list(rows[i]) != ground_truth:
            break
        ground_truth = list(rows[i]) + [int(predicted[i])]
    return ground_truth


def count_accepted(draft: Sequence[int], predicted: Sequence[int]) -> int:
    """The same walk expressed on the new tokens only: n = number of leading assistant tokens
    d_1..d_n with d_i == predicted[i-1]."""
    n = 0
    while n < len(draft) and int(draft[n]) == int(predicted[n]):
        n += 1
    return n


# ----------------------------------------------------------------------------------------
# the method, literally (no cache, every stair row forwarded on its own)
# ----------------------------------------------------------------------------------------
@dataclass
class Iteration:
    L: int                    # sequence length before the iteration
    draft: List[int]          # d_1..d_k
    predicted: List[int]      # t_0..t_k
    n_accepted: int           # assistant tokens kept
    logits: Optional[np.ndarray] = None   # [k+1, V] main-model last-position logits per stair


@dataclass
class Generation:
    tokens: List[int]                                  # the generated tokens: G, fewer when an end token closed the answer
    iterations: List[Iteration] = field(default_factory=list)

    def mean_tokens_per_iteration(self) -> float:
        return sum(it.n_accepted + 1 for it in self.iterations) / max(1, len(self.iterations))


def stairs_literal(target: OracleModel, draft: OracleModel, prompt: Sequence[int], G: int, k: int,
                   keep_logits: bool = False, eos: Optional[int] = None) -> Generation:
    seq = [int(t) for t in prompt]
    P = len(seq)
    gen = Generation(tokens=[])
    ended = False
    while len(seq) - P < G and not ended:
        # assistant model generates k tokens in advance, greedily
        ext = list(seq)
        for _ in range(k):
            ext.append(greedy_token(forward_full(draft, ext)[-1]))
        d = ext[len(seq):]
        # stair batch: the prefix, then progressively one more assistant token per row
        rows = [seq + d[:i] for i in range(k + 1)]
        # the main model predicts one additional token for each row
        row_logits = [forward_full(target, r)[-1] for r in rows]
        t = [greedy_token(lg) for lg in row_logits]
        # stairs validation
        truth = stairs_validate(rows, t)
        n = len(truth) - len(seq) - 1
        gen.iterations.append(Iteration(len(seq), d, t, n,
                                        np.stack(row_logits) if keep_logits else None))
        new, ended = cut_after_end_token(truth[len(seq):], eos)
        seq = seq + new
    gen.tokens = seq[P:P + G]
    return gen


# ----------------------------------------------------------------------------------------
# the method with KV caches (one causal forward per stair batch)
# ----------------------------------------------------------------------------------------
class CachedStairs:
    """State of a cached stairs generation; usable step by step (so that a test can force the
    oracle along a prefix produced elsewhere) or through ``run``."""

    def __init__(self, target: OracleModel, draft: Optional[OracleModel], prompt: Sequence[int],
                 capacity: int, kv_round=None):
        self.target, self.draft = target, draft
        self.seq = [int(t) for t in prompt]
        self.P = len(self.seq)
        self.kv_round = kv_round
        self.tc = KVCache.empty(target, capacity)
        self.dc = KVCache.empty(draft, capacity) if draft is not None else None
        # both models ingest all but the last prompt token
        if self.P > 1:
            forward_cached(target, self.tc, self.seq[:-1], 0, kv_round)
            self.tc.length = self.P - 1
            if draft is not None:
                forward_cached(draft, self.dc, self.seq[:-1], 0, kv_round)
                self.dc.length = self.P - 1

    def propose(self, k: int, forced: Optional[Sequence[int]] = None,
                logits_out: Optional[list] = None) -> List[int]:
        """k greedy assistant tokens after self.seq.  ``forced`` (teacher forcing, used by the
        parity tests): the tokens another implementation chose; they are fed back instead of
        this oracle's own choices, so that its logits can be compared step by step even after a
        near-tie was resolved differently.  ``logits_out`` collects each step's logits row."""
        L = len(self.seq)
        d: List[int] = []
        if k == 0:
            return d
        # catch up on everything the assistant has not ingested yet, then decode one by one
        pend = self.seq[self.dc.length:]
        lg = forward_cached(self.draft, self.dc, pend, self.dc.length, self.kv_round)
        self.dc.length = L
        for j in range(k):
            if j > 0:
                lg = forward_cached(self.draft, self.dc, [fed], L - 1 + j, self.kv_round)
                self.dc.length = L + j
            if logits_out is not None:
                logits_out.append(lg[-1])
            d.append(greedy_token(lg[-1]))
            fed = d[-1] if forced is None else int(forced[j])
        return d

    def verify(self, d: Sequence[int]) -> Iteration:
        """Score the stair batch for assistant tokens d, validate, roll the caches back."""
        L = len(self.seq)
        k = len(d)
        rows_new = [self.seq[-1]] + [int(x) for x in d]
        logits = forward_cached(self.target, self.tc, rows_new, L - 1, self.kv_round)   # [k+1, V]
        t = [greedy_token(logits[i]) for i in range(k + 1)]
        n = count_accepted(d, t)
        it = Iteration(L, [int(x) for x in d], t, n, logits)
        self.adopt(L, t[:n + 1])
        return it

    def adopt(self, L: int, new_tokens: Sequence[int]):
        """Make ``seq[:L] + new_tokens`` the sequence after an iteration that started at length
        L.  verify() calls it with its own result; a parity test calls it again with the tokens
        another implementation accepted (teacher forcing).  new_tokens must be a stair path of
        the batch just scored (accepted assistant tokens plus one prediction), so the cache rows
        written for it are the right ones: positions L-1 .. L-2+len(new_tokens) stay valid."""
        self.seq = self.seq[:L] + [int(x) for x in new_tokens]
        n = len(new_tokens) - 1
        self.tc.length = L + n
        if self.dc is not None:
            self.dc.length = min(self.dc.length, L + n)

    def run(self, G: int, k: int, keep_logits: bool = False, eos: Optional[int] = None) -> Generation:
        gen = Generation(tokens=[])
        ended = False
        while len(self.seq) - self.P < G and not ended:
            it = self.verify(self.propose(k))
            if not keep_logits:
                it.logits = None
            gen.iterations.append(it)
            new, ended = cut_after_end_token(self.seq[it.L:], eos)
            if ended:
                self.adopt(it.L, new)
        gen.tokens = self.seq[self.P:self.P + G]
        return gen


def next_draft_length(k: int, n: int, k_max: int) -> int:
    """Draft length after an iteration that proposed k tokens and kept n: everything kept -> one more (at most k_max),
    otherwise one more than was kept (at least 1).  The paper fixes one length per model pair by a sweep (Sec. 4.3);
    any rule gives the same output (Sec. 3.1), so this one is a choice of this build, stated in the C header too."""
    return min(k + 1, k_max) if n == k else max(1, n + 1)


def stairs_adaptive(target: OracleModel, draft: OracleModel, prompt: Sequence[int], G: int, k_first: int,
                    k_max: int) -> Generation:
    """The cached stairs loop with the draft length following next_draft_length."""
    st = CachedStairs(target, draft, prompt, len(prompt) + G + k_max + 2)
    gen = Generation(tokens=[])
    k = k_first
    while len(st.seq) - st.P < G:
        it = st.verify(st.propose(k))
        it.logits = None
        gen.iterations.append(it)
        k = next_draft_length(k, it.n_accepted, k_max)
    gen.tokens = st.seq[st.P:st.P + G]
    return gen


def stairs_cached(target: OracleModel, draft: Optional[OracleModel], prompt: Sequence[int], G: int,
                  k: int, keep_logits: bool = False, kv_round=None, eos: Optional[int] = None) -> Generation:
    st = CachedStairs(target, draft, prompt, len(prompt) + G + k + 2, kv_round)
    return st.run(G, k, keep_logits, eos)


def stairs_batch(target: OracleModel, draft: Optional[OracleModel], prompts: Sequence[Sequence[int]], G: int,
                 k: int, eos: Optional[int] = None) -> list:
    """Several prompts at once.  Sec. 3.3 treats one sentence; sequences do not interact (Sec. 3.1: the model maps
    one token sequence to one distribution), so the result for a set of prompts is the result of the method for each
    of them on its own: a list with one Generation per prompt."""
    return [stairs_cached(target, draft, p, G, k, eos=eos) for p in prompts]


def top2_margin(logits_row: np.ndarray) -> float:
    """Difference between the largest and second-largest logit of one row."""
    part = np.partition(logits_row, -2)
    return float(part[-1] - part[-2])
