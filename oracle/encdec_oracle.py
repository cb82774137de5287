"""CPU oracle for stairs-assisted greedy generation with an encoder-decoder model.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this file.  It shares no code with
the HIP library and never imports it; the library never imports it.

The paper's experiments run encoder-decoder checkpoints (Sec. 2.3, Sec. 4.3, Sec. 4.4): the source text goes through the
encoder once, and the stair batch of Sec. 3.3 is made of prefixes of the DECODER sequence; every stair row reads the
same encoder output.  The paper gives no model arithmetic; the model here follows the published description of the
original T5 (Raffel et al., 2020, Sec. 2.1) in this oracle's own code:
  * RMS layer norm (no mean subtraction, no bias) before every block, residual connection after it;
  * attention: scores = q k^T + bias[bucket(key position - query position), head], no 1/sqrt(head_dim); the bias
    table is shared by the layers of a stack; the encoder uses the two-sided bucket rule, the decoder's
    self-attention the one-sided rule with the causal mask, cross-attention no bias and no mask;
  * feed-forward: W_out relu(W_in x); no biases; untied unembedding; no scaling of embeddings or logits.
  * bucket rule for a distance n >= 0 with B buckets per side: n itself while n < B/2, beyond that
    B/2 + floor(log(n / (B/2)) / log(max_distance / (B/2)) * (B/2)) capped at B - 1.  Two-sided: B = buckets/2 and
    keys after the query take the upper half (+B); one-sided: B = buckets and keys after the query use n = 0.
    The logarithms are taken in float64 (a distance that sits exactly on a bucket edge does not occur for the
    (32, 128) tables used here other than at the cap).

A model bound to a source sequence (``BoundDecoder``) offers the cached forward the decoder-only oracle's stairs
drivers call, so stair construction, validation and cache rollback are the very functions of stairs_oracle.py.

Parity pins (tests/test_oracle_encdec.py): hand-computed buckets, bucket structure (exact / logarithmic / capped
ranges, symmetry), softmax attention against PyTorch's library routine with an additive mask, source-permutation
invariance with zero bias tables, cached decoder forward == uncached, stairs == brute-force greedy.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from oracle import stairs_oracle as so


def relative_position_bucket(rel: np.ndarray, bidirectional: bool, num_buckets: int, max_distance: int) -> np.ndarray:
    """rel = key position - query position (integers, any shape) -> bucket index."""
    rel = np.asarray(rel, dtype=np.int64)
    if bidirectional:
        side = num_buckets // 2
        offset = np.where(rel > 0, side, 0)
        n = np.abs(rel)
    else:
        side = num_buckets
        offset = np.zeros_like(rel)
        n = np.maximum(-rel, 0)
    exact = side // 2
    nn = np.maximum(n, 1).astype(np.float64)
    far = exact + np.floor(np.log(nn / exact) / np.log(max_distance / exact) * (side - exact)).astype(np.int64)
    far = np.minimum(far, side - 1)
    return offset + np.where(n < exact, n, far)


def position_bias(table: np.ndarray, q_pos: np.ndarray, k_pos: np.ndarray, bidirectional: bool,
                  max_distance: int) -> np.ndarray:
    """table [buckets, H] -> bias [H, M, T] for queries at q_pos and keys at k_pos."""
    rel = k_pos[None, :] - q_pos[:, None]
    b = relative_position_bucket(rel, bidirectional, table.shape[0], max_distance)     # [M, T]
    return np.transpose(table[b], (2, 0, 1))


def biased_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, bias: Optional[np.ndarray],
                     hidden: Optional[np.ndarray]) -> np.ndarray:
    """q [M, H, hd], k, v [T, H, hd]; bias [H, M, T] or None; hidden [M, T] True where a key is masked."""
    M, H, hd = q.shape
    out = np.empty_like(q)
    for h in range(H):
        s = q[:, h, :] @ k[:, h, :].T
        if bias is not None:
            s = s + bias[h]
        if hidden is not None:
            s = np.where(hidden, -np.inf, s)
        out[:, h, :] = so.softmax_rows(s) @ v[:, h, :]
    return out


class EncDecOracleModel:
    """Real-valued view of EncDecInputs."""

    def __init__(self, inputs, dtype=np.float64):
        self.inp = inputs
        self.dtype = np.dtype(dtype)
        self.d, self.H, self.hd = inputs.d_model, inputs.n_heads, inputs.head_dim
        self.V = inputs.vocab
        self.eps = float(inputs.rms_eps)
        self.max_distance = int(inputs.rel_max_distance)
        self._cache = {}

    def w(self, stack: str, l: Optional[int], name: str) -> np.ndarray:
        key = (stack, l, name)
        got = self._cache.get(key)
        if got is None:
            src = getattr(self.inp, name) if l is None else \
                (self.inp.enc_layers if stack == "enc" else self.inp.dec_layers)[l][name]
            got = self._cache[key] = so._decode(src, self.dtype)
        return got

    def heads(self, x: np.ndarray) -> np.ndarray:
        return x.reshape(x.shape[0], self.H, self.hd)

    def ffn(self, stack: str, l: int, x: np.ndarray) -> np.ndarray:
        h = so.rmsnorm(x, self.w(stack, l, "ffn_norm"), self.eps)
        return x + np.maximum(h @ self.w(stack, l, "w_in").T, 0) @ self.w(stack, l, "w_out").T

    def encode(self, src: Sequence[int]) -> np.ndarray:
        """Encoder output [S, d] (after the encoder's final norm)."""
        ids = np.asarray(src, dtype=np.int64)
        S = ids.shape[0]
        pos = np.arange(S)
        x = self.w(None, None, "tok_emb")[ids].astype(self.dtype)
        bias = position_bias(self.w(None, None, "enc_rel_bias"), pos, pos, True, self.max_distance)
        for l in range(self.inp.n_enc_layers):
            h = so.rmsnorm(x, self.w("enc", l, "attn_norm"), self.eps)
            q, k, v = (self.heads(h @ self.w("enc", l, n).T) for n in ("wq", "wk", "wv"))
            a = biased_attention(q, k, v, bias, None).reshape(S, -1)
            x = x + a @ self.w("enc", l, "wo").T
            x = self.ffn("enc", l, x)
        return so.rmsnorm(x, self.w(None, None, "enc_final_norm"), self.eps)


class BoundDecoder:
    """The decoder of an encoder-decoder model together with one encoded source: behaves like a decoder-only model
    for the stairs drivers of stairs_oracle.py (they call ``decoder_forward`` through their cached/full forward)."""

    def __init__(self, model: EncDecOracleModel, src: Sequence[int], kv_round=None):
        self.m = model
        self.dtype = model.dtype
        self.n_layers = model.inp.n_dec_layers
        self.H, self.hd, self.V = model.H, model.hd, model.V
        enc = model.encode(src)
        self.cross_k: List[np.ndarray] = []
        self.cross_v: List[np.ndarray] = []
        for l in range(self.n_layers):
            k, v = model.heads(enc @ model.w("dec", l, "ck").T), model.heads(enc @ model.w("dec", l, "cv").T)
            if kv_round is not None:
                k, v = kv_round(k), kv_round(v)
            self.cross_k.append(k)
            self.cross_v.append(v)

    def decoder_forward(self, ids: np.ndarray, pos0: int, cache, kv_round=None) -> np.ndarray:
        """Rows ids at decoder positions pos0.. -> logits [M, V]; cache as in stairs_oracle._forward."""
        m = self.m
        ids = np.asarray(ids, dtype=np.int64)
        M = ids.shape[0]
        x = m.w(None, None, "tok_emb")[ids].astype(m.dtype)
        q_pos = pos0 + np.arange(M)
        k_pos = np.arange(pos0 + M)
        bias = position_bias(m.w(None, None, "dec_rel_bias"), q_pos, k_pos, False, m.max_distance)
        hidden = k_pos[None, :] > q_pos[:, None]
        for l in range(self.n_layers):
            h = so.rmsnorm(x, m.w("dec", l, "attn_norm"), m.eps)
            q, k, v = (m.heads(h @ m.w("dec", l, n).T) for n in ("wq", "wk", "wv"))
            if kv_round is not None:
                k, v = kv_round(k), kv_round(v)
            if cache is None:
                assert pos0 == 0
                k_all, v_all = k, v
            else:
                cache.k[l][pos0:pos0 + M] = k
                cache.v[l][pos0:pos0 + M] = v
                k_all, v_all = cache.k[l][:pos0 + M], cache.v[l][:pos0 + M]
            a = biased_attention(q, k_all, v_all, bias, hidden).reshape(M, -1)
            x = x + a @ m.w("dec", l, "wo").T
            h = so.rmsnorm(x, m.w("dec", l, "cross_norm"), m.eps)
            q = m.heads(h @ m.w("dec", l, "cq").T)
            a = biased_attention(q, self.cross_k[l], self.cross_v[l], None, None).reshape(M, -1)
            x = x + a @ m.w("dec", l, "co").T
            x = m.ffn("dec", l, x)
        h = so.rmsnorm(x, m.w(None, None, "dec_final_norm"), m.eps)
        return h @ m.w(None, None, "lm_head").T
