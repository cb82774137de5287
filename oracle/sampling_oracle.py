"""CPU oracle for the sampling variant of stairs-assisted generation.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this file.  It shares no code with
the HIP library and never imports it; the library never imports it.

The paper leaves sampling to future work (Sec. 5: greedy generation replaced with sampling for the assistant and the
main model, which brings in the temperature) and describes the rejection-sampling schemes of the related work only in
words (Sec. 2.2).  What is computed here is that published scheme (Leviathan et al. 2023; Chen et al. 2023), written
out in the order the stairs method runs:
  1. the assistant SAMPLES k tokens d_1..d_k, one after the other, from q_j = softmax(assistant logits / T);
  2. the main model scores the k+1 stair rows in one batch: p_i = softmax(main logits of row i / T), i = 0..k;
  3. validation walks the rows: d_i is kept with probability min(1, p_{i-1}(d_i) / q_i(d_i)); at the first token that
     is not kept, one token is drawn from the normalised positive part of p_{i-1} - q_i and the walk stops; if all k
     are kept, one more token is drawn from p_k.
Every iteration emits n + 1 tokens (n kept), and the emitted tokens are distributed as if the main model had sampled
them itself.

Random numbers: both this oracle and the HIP library implement the counter-based generator "squares" (Widynski 2020,
four rounds of squaring on a 64-bit counter * key): r(ctr, key) in [0, 2^32).  The counter of a draw is
(position of the token being decided << 34) | (stream << 32) | vocabulary index, with streams 0 = assistant's draw,
1 = the keep/reject uniform, 2 = the main model's draw (replacement or extra token).  A categorical draw is
argmax_v(score_v + g_v) with g_v = -log(-log(u_v)), u_v = (r + 0.5) / 2^32 (Gumbel-max), so that the decision is an
argmax like the greedy one and can be compared across implementations with the same margin rule.

Parity pins (tests/test_oracle_sampling.py): uniformity and stream independence of the generator, Gumbel-max draws
against the softmax (chi-square), emitted-token distribution == main model's distribution and the closed form
sum_v min(p_v, q_v) of the keep probability (Monte Carlo over positions), identical assistant => everything kept,
temperature -> 0 => the greedy stairs output, k = 0 => plain sampling.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

from oracle import stairs_oracle as so

MASK64 = (1 << 64) - 1
STREAM_DRAFT, STREAM_ACCEPT, STREAM_TARGET = 0, 1, 2


def key_from_seed(seed: int) -> int:
    """64-bit odd key from a small seed (one splitmix64 step)."""
    z = (seed + 0x9E3779B97F4A7C15) & MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return (z ^ (z >> 31)) | 1


def squares32(ctr: np.ndarray, key: int) -> np.ndarray:
    """Widynski's squares generator, 32-bit output, vectorised over uint64 counters."""
    ctr = np.asarray(ctr, dtype=np.uint64)
    k = np.uint64(key)
    with np.errstate(over="ignore"):
        x = ctr * k
        y = x
        z = y + k
        x = x * x + y
        x = (x >> np.uint64(32)) | (x << np.uint64(32))
        x = x * x + z
        x = (x >> np.uint64(32)) | (x << np.uint64(32))
        x = x * x + y
        x = (x >> np.uint64(32)) | (x << np.uint64(32))
        return ((x * x + z) >> np.uint64(32)).astype(np.uint64)


def counters(pos: int, stream: int, n: int) -> np.ndarray:
    return (np.uint64(pos) << np.uint64(34)) | (np.uint64(stream) << np.uint64(32)) | np.arange(n, dtype=np.uint64)


def uniform(pos: int, stream: int, n: int, key: int) -> np.ndarray:
    """n uniforms in (0, 1) for (position, stream)."""
    return (squares32(counters(pos, stream, n), key).astype(np.float64) + 0.5) / 4294967296.0


def gumbel(pos: int, stream: int, n: int, key: int) -> np.ndarray:
    return -np.log(-np.log(uniform(pos, stream, n, key)))


def log_softmax(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    m = np.max(z)
    return z - (m + np.log(np.sum(np.exp(z - m))))


def draw(scores: np.ndarray, pos: int, stream: int, key: int) -> int:
    """Categorical draw proportional to exp(scores): Gumbel-max, ties -> lowest index."""
    return int(np.argmax(np.asarray(scores, dtype=np.float64) + gumbel(pos, stream, len(scores), key)))


def residual_scores(logp: np.ndarray, logq: np.ndarray) -> np.ndarray:
    """log of the positive part of p - q (-inf where p <= q)."""
    diff = np.exp(logp) - np.exp(logq)
    with np.errstate(divide="ignore"):
        return np.where(diff > 0, np.log(np.maximum(diff, 1e-300)), -np.inf)


@dataclass
class SampledIteration:
    L: int
    draft: List[int]
    n_accepted: int
    emitted: List[int]
    target_logits: Optional[np.ndarray] = None      # [k+1, V]
    draft_logits: Optional[np.ndarray] = None       # [k, V]
    uniforms: List[float] = field(default_factory=list)
    ratios: List[float] = field(default_factory=list)   # p(d_i) / q(d_i) for the rows the walk looked at


def validate_sampled(L: int, d: Sequence[int], target_logits: np.ndarray, draft_logits: np.ndarray, temperature: float,
                     key: int):
    """Step 3 above for the stair batch that starts at sequence length L.  target_logits [k+1, V] (row i predicts the
    token at position L + i), draft_logits [k, V] (row j-1 is the distribution d_j was drawn from).
    -> (n kept, emitted tokens (n + 1 of them), uniforms used, ratios seen)."""
    k = len(d)
    us, ratios = [], []
    for i in range(1, k + 1):
        pos = L + i - 1
        logp = log_softmax(target_logits[i - 1] / temperature)
        logq = log_softmax(draft_logits[i - 1] / temperature)
        u = float(uniform(pos, STREAM_ACCEPT, 1, key)[0])
        ratio = float(np.exp(logp[d[i - 1]] - logq[d[i - 1]]))
        us.append(u)
        ratios.append(ratio)
        if not u < ratio:
            rs = residual_scores(logp, logq)
            if not np.any(np.isfinite(rs)):     # p == q to the last bit yet not kept (rounding only): p itself
                rs = logp
            t = draw(rs, pos, STREAM_TARGET, key)
            return i - 1, [int(x) for x in d[:i - 1]] + [t], us, ratios
    t = draw(target_logits[k] / temperature, L + k, STREAM_TARGET, key)
    return k, [int(x) for x in d] + [t], us, ratios


class SampledStairs(so.CachedStairs):
    """Cached stairs generation with sampling; step-wise like its greedy parent so that a test can force it along
    another implementation's choices."""

    def __init__(self, target, draft, prompt, capacity, temperature: float, seed: int, kv_round=None):
        super().__init__(target, draft, prompt, capacity, kv_round)
        self.temperature = float(temperature)
        self.key = key_from_seed(seed)

    def propose_sampled(self, k: int, forced: Optional[Sequence[int]] = None):
        """k assistant tokens drawn one by one -> (tokens, logits [k, V]); ``forced`` as in CachedStairs.propose."""
        L = len(self.seq)
        d: List[int] = []
        rows = []
        if k == 0:
            return d, np.zeros((0, self.target.V))
        pend = self.seq[self.dc.length:]
        lg = so.forward_cached(self.draft, self.dc, pend, self.dc.length, self.kv_round)
        self.dc.length = L
        for j in range(k):
            if j > 0:
                lg = so.forward_cached(self.draft, self.dc, [fed], L - 1 + j, self.kv_round)
                self.dc.length = L + j
            rows.append(np.asarray(lg[-1], dtype=np.float64))
            d.append(draw(rows[-1] / self.temperature, L + j, STREAM_DRAFT, self.key))
            fed = d[-1] if forced is None else int(forced[j])
        return d, np.stack(rows)

    def verify_sampled(self, d: Sequence[int], draft_logits: np.ndarray) -> SampledIteration:
        L = len(self.seq)
        rows_new = [self.seq[-1]] + [int(x) for x in d]
        logits = np.asarray(so.forward_cached(self.target, self.tc, rows_new, L - 1, self.kv_round), dtype=np.float64)
        n, emitted, us, ratios = validate_sampled(L, d, logits, draft_logits, self.temperature, self.key)
        it = SampledIteration(L, [int(x) for x in d], n, emitted, logits, draft_logits, us, ratios)
        self.adopt(L, emitted)
        return it

    def run_sampled(self, G: int, k: int) -> List[SampledIteration]:
        its = []
        while len(self.seq) - self.P < G:
            d, dl = self.propose_sampled(k)
            its.append(self.verify_sampled(d, dl))
        return its


def stairs_sampled(target, draft, prompt: Sequence[int], G: int, k: int, temperature: float, seed: int):
    """-> (G tokens, iterations)."""
    s = SampledStairs(target, draft if k > 0 else None, prompt, len(prompt) + G + k + 2, temperature, seed)
    its = s.run_sampled(G, k)
    return s.seq[len(prompt):len(prompt) + G], its
