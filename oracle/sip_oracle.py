"""Slow CPU oracle for the batched token-sampling stage.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the HIP library is compared against.  It is imported by
``tests/``, by ``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of
``bench.py`` and by nothing else; it shares no code with the GPU path and is never a
fallback for it.

What it computes (paper Sec. 2.1 step 3 "Sampling", display equation
``p = Filter(softmax(ApplyPenalty(z, y_<s) / tau); k, p)`` followed by
``y_s ~ Categorical(p)``; restated step by step in Sec. 5.1): per row of a ``[B, V]``
logits matrix, penalties from the row's token history, temperature, softmax, top-k,
top-p and min-p filters, one seeded categorical draw, and log-probabilities.

Everything the paper leaves open (penalty forms and order, tie handling, min-p, the
random number generator, the order of the CDF, what a logprob is) follows the readings
documented next to each step below.  The route is deliberately the plain one: widen to
fp32, fp32 penalty/temperature arithmetic, then fp64 ``exp``, a full stable sort,
explicit cumulative sums, an explicit CDF.  No blocking, no fusion, no selection
algorithms.

Pinned (tests/test_oracle_*.py, all run without a GPU): Philox known answers; brute-force
O(V^2) set definitions on tiny inputs; closed forms (uniform and geometric logits);
``scipy.special.log_softmax`` and ``numpy.partition`` special cases; hand-computed penalty
micro cases; the invariants of the benchmark spec (probabilities sum to one, k=1 and
tau=0 reduce to lowest-index argmax, p=1 with k=0 is a no-op, unseen tokens untouched);
chi-square of draw frequencies.  The conventions themselves (tie handling, filter order,
index-order CDF, pre-filter logprobs) are not fixed by the paper and are therefore
"parity unpinned" with respect to it: they are pinned only to their own definitions.

The persistent decode state at the end of the file (history appended and token frequencies
updated incrementally from one iteration to the next, Sec. 5.1) is pinned in
tests/test_oracle_state.py: a hand-worked greedy sequence, the from-scratch route on a
history the test records by itself and counts with numpy, and the invariants of slots.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

# ----------------------------------------------------------------------------------
# Random numbers: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).  The paper only
# says "Categorical" (Sec. 2.1 step 3); the generator and its keying are this build's
# reading: counter = (row_id lo, row_id hi, step lo, step hi), key = (seed lo, seed hi),
# uniform = top 24 bits of output word 0 scaled by 2^-24.
# ----------------------------------------------------------------------------------
_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = 0xFFFFFFFF


def philox4x32_10(counter: Sequence[int], key: Sequence[int]):
    """Ten rounds of Philox-4x32 on a 128-bit counter with a 64-bit key; returns 4 words."""
    c0, c1, c2, c3 = (int(x) & _MASK32 for x in counter)
    k0, k1 = (int(x) & _MASK32 for x in key)
    for _ in range(10):
        prod0 = _PHILOX_M0 * c0
        prod1 = _PHILOX_M1 * c2
        hi0, lo0 = prod0 >> 32, prod0 & _MASK32
        hi1, lo1 = prod1 >> 32, prod1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0 = (k0 + _PHILOX_W0) & _MASK32
        k1 = (k1 + _PHILOX_W1) & _MASK32
    return c0, c1, c2, c3


def row_uniform(seed: int, row_id: int, step: int) -> float:
    """The one uniform in [0, 1) a row consumes; exactly representable in fp32."""
    seed, row_id, step = int(seed), int(row_id), int(step)
    x0 = philox4x32_10((row_id & _MASK32, (row_id >> 32) & _MASK32,
                        step & _MASK32, (step >> 32) & _MASK32),
                       (seed & _MASK32, (seed >> 32) & _MASK32))[0]
    return float(x0 >> 8) * (2.0 ** -24)


# ----------------------------------------------------------------------------------
# Row-level steps
# ----------------------------------------------------------------------------------
def widen(row: np.ndarray) -> np.ndarray:
    """fp32 view of a logits row; uint16 input is taken as bf16 bit patterns (exact)."""
    if row.dtype == np.uint16:
        return (row.astype(np.uint32) << np.uint32(16)).view(np.float32).copy()
    return np.array(row, dtype=np.float32, copy=True)


def history_counts(history: np.ndarray, V: int) -> np.ndarray:
    """c_v = occurrences of token v among the previously generated tokens y_<s of the row
    (Sec. 2.1 step 3; Sec. 5.1 CalcPenalty).  Ids outside [0, V) are padding and skipped."""
    c = np.zeros(V, dtype=np.int64)
    if history is None:
        return c
    h = np.asarray(history).astype(np.int64).ravel()
    for t in h[(h >= 0) & (h < V)]:
        c[t] += 1
    return c


def apply_penalties(z: np.ndarray, c: np.ndarray, theta: float, phi: float, psi: float,
                    c_prompt: Optional[np.ndarray] = None) -> np.ndarray:
    """ApplyPenalty of Sec. 2.1 (1) / Sec. 5.1, in IEEE fp32, one rounding per operation,
    only where c_v > 0, in the order repetition -> frequency -> presence.

    ``c_prompt`` (optional): occurrences in the sequence's prompt, handed in separately from the
    generated tokens.  Sec. 2.1 defines y_<s as the *generated* tokens while a sequence is prompt
    plus output; the reading taken for a separate prompt is the usual one of serving engines: the
    repetition penalty looks at prompt and output together, frequency and presence at the output
    only.  Without ``c_prompt`` one history serves all three.

    The paper writes all three as ``Z - alpha * f``.  Frequency and presence are taken
    that way (f = count, resp. f = 1 for seen tokens).  Repetition is taken in the
    multiplicative form of the work the paper cites for it (divide positive logits by
    theta, multiply the others), the form under which theta = 1 is "off"."""
    f32 = np.float32
    out = z.astype(np.float32, copy=True)
    th, ph, ps = f32(theta), f32(phi), f32(psi)
    if c_prompt is not None and th != f32(1.0):
        # repetition over prompt and output; the tokens of the output alone go on below
        rep = np.flatnonzero((c > 0) | (np.asarray(c_prompt) > 0))
        y = out[rep]
        out[rep] = np.where(y > f32(0.0), y / th, y * th).astype(np.float32)
        th = f32(1.0)
    seen = np.flatnonzero(c > 0)
    if seen.size == 0:
        return out
    x = out[seen]
    if th != f32(1.0):
        x = np.where(x > f32(0.0), x / th, x * th).astype(np.float32)
    if ph != f32(0.0):
        x = (x - (ph * c[seen].astype(np.float32)).astype(np.float32)).astype(np.float32)
    if ps != f32(0.0):
        x = (x - ps).astype(np.float32)
    out[seen] = x
    return out


@dataclass
class RowResult:
    token: int
    logprob: float                         # log-softmax of the sampled token (fp64)
    top_ids: np.ndarray                    # n best tokens by logprob, ties lowest index first
    top_logprobs: np.ndarray               # their logprobs (fp64)
    greedy: bool
    kept: Optional[np.ndarray] = None      # boolean mask of the final candidate set K3
    u: float = 0.0
    draw_margin: float = math.inf          # min distance of u from a normalised CDF boundary
    topp_margin: float = math.inf          # distance of the top-p cut from the nearest group edge
    m: float = 0.0
    logZ: float = 0.0                      # L = ln sum_v exp(s_v - m)
    S1: float = 0.0
    S3: float = 0.0
    s: Optional[np.ndarray] = field(default=None, repr=False)
    # Near-boundary accounting.  ``topp_matters``: moving the top-p cut by the one value group
    # that lies within the margin changes the final kept set (it does not when min-p removes
    # that group anyway).  ``alt_tokens``: what the draw returns under each such neighbouring
    # decision -- the cut one group earlier or later, the CDF entry before or after the one
    # chosen -- i.e. the only other ids a correct implementation in lower precision may return
    # for a near-boundary row.  Filled in when a margin is below 1e-5.
    topp_matters: bool = True
    alt_tokens: tuple = ()

    def flagged(self, eps: float = 1e-6) -> bool:
        """Near-boundary row: the fp64 decision is closer than eps (relative mass) to
        flipping, so an fp32 implementation may legitimately pick the neighbour."""
        return (self.draw_margin < eps) or (self.topp_margin < eps and self.topp_matters)


def sample_row(row: np.ndarray, *, temperature: float = 1.0, top_k: int = 0, top_p: float = 1.0,
               min_p: float = 0.0, repetition_penalty: float = 1.0, frequency_penalty: float = 0.0,
               presence_penalty: float = 0.0, history: Optional[np.ndarray] = None,
               seed: int = 0, step: int = 0, row_id: int = 0, n_logprobs: int = 0,
               u_override: Optional[float] = None, keep_arrays: bool = False,
               counts: Optional[np.ndarray] = None, prompt: Optional[np.ndarray] = None) -> RowResult:
    f32 = np.float32
    V = int(row.shape[0])
    idx = np.arange(V)

    # (0) widen, (1) counts, (2) penalties -- fp32
    # ``counts`` (instead of ``history``) hands in a frequency vector kept up to date across
    # iterations, the incremental construction of Sec. 5.1 (see DecodeState below).
    z = widen(row)
    c = history_counts(history, V) if counts is None else np.asarray(counts, dtype=np.int64)
    z = apply_penalties(z, c, repetition_penalty, frequency_penalty, presence_penalty,
                        None if prompt is None else history_counts(prompt, V))

    tau = f32(temperature)
    k = int(top_k)
    greedy = (tau == f32(0.0)) or (k == 1)

    # (3)/(4) temperature: s = z / tau in fp32 (Sec. 2.1 (2), Sec. 5.1 Z'' = Z'/tau, tau > 0).
    # tau = 0 is the greedy flag; greedy rows report logprobs at tau = 1.
    s = z if greedy else (z / tau).astype(np.float32)

    # (5) softmax statistics in fp64 (Sec. 5.1 row-wise softmax)
    m = f32(np.max(s))
    d = s.astype(np.float64) - np.float64(m)
    e = np.exp(d)
    Z = float(np.sum(e))
    logZ = math.log(Z)
    logprob = d - logZ                                   # over the full vocabulary, before filters

    # ordering used by every sorted step: value descending, index ascending on ties
    order = np.argsort(-s, kind="stable")

    n = max(0, min(int(n_logprobs), V))
    top_ids = order[:n].astype(np.int64)
    top_lp = logprob[top_ids]

    if greedy:
        tok = int(order[0])                              # = lowest-index arg max
        return RowResult(tok, float(logprob[tok]), top_ids, top_lp, True, None, 0.0,
                         math.inf, math.inf, float(m), logZ, Z, Z,
                         s if keep_arrays else None)

    s_sorted = s[order]
    e_sorted = e[order]

    # (6) top-k (Sec. 2.1 (2)): keep every token whose value is >= the k-th largest value,
    # i.e. { v : #{w : s_w > s_v} < k }.  Equal values stand or fall together.
    if 2 <= k < V:
        t_k = s_sorted[k - 1]
        in_k1_sorted = s_sorted >= t_k
    else:
        in_k1_sorted = np.ones(V, dtype=bool)
    n1 = int(np.count_nonzero(in_k1_sorted))             # K1 is a prefix of the sorted order
    cum = np.cumsum(e_sorted[:n1])                       # explicit running mass, fp64
    S1 = float(cum[-1])

    # (7) top-p (Sec. 2.1 (2)): smallest value-closed prefix of the descending order whose
    # mass reaches p, measured against the mass left after top-k:
    # keep v iff (mass of K1 tokens with strictly larger value) < p * S1.
    p = f32(top_p)
    topp_margin = math.inf
    n2 = n1
    if f32(0.0) < p < f32(1.0):
        excl = np.concatenate(([0.0], cum[:-1]))         # mass of sorted predecessors
        vals = s_sorted[:n1]
        # first position of each element's value group (vals is non-increasing)
        first = np.searchsorted(-vals, -vals, side="left")
        mass_gt = excl[first]
        target_p = float(np.float64(p)) * S1
        target = target_p
        keep2 = mass_gt < target
        n2 = int(np.count_nonzero(keep2))                # again a prefix
        # how close the cut came to landing one group earlier or later
        last_kept = mass_gt[n2 - 1]
        topp_margin = abs(last_kept - target) / S1
        if n2 < n1:
            topp_margin = min(topp_margin, abs(mass_gt[n2] - target) / S1)

    # (8) min-p (only named in Sec. 7.1 "Workload"): keep p_v >= min_p * p_max, decided as
    # the exact fp32 comparison (s_v - m) >= float32(ln(min_p)).
    keep_sorted = np.zeros(V, dtype=bool)
    keep_sorted[:n2] = True
    mp = f32(min_p)
    if mp > f32(0.0):
        t = f32(math.log(float(np.float64(mp))))
        keep_sorted &= (s_sorted - m).astype(np.float32) >= t

    minp_sorted = np.ones(V, dtype=bool)
    if mp > f32(0.0):
        minp_sorted = (s_sorted - m).astype(np.float32) >= t

    kept = np.zeros(V, dtype=bool)
    kept[order[keep_sorted]] = True

    # (9) draw (Sec. 2.1 (3)): explicit CDF over the kept set in ascending vocabulary index
    u = row_uniform(seed, row_id, step) if u_override is None else float(u_override)

    def draw(kept_mask):
        k_idx = idx[kept_mask]
        c = np.cumsum(e[k_idx])
        tgt = u * float(c[-1])
        h = np.flatnonzero(c > tgt)
        ps = int(h[0]) if h.size else k_idx.size - 1
        return k_idx, c, ps

    kept_idx, cdf, pos = draw(kept)
    S3 = float(cdf[-1])
    tok = int(kept_idx[pos])
    draw_margin = float(np.min(np.abs(cdf / S3 - u)))

    # neighbouring decisions of a near-boundary row (see RowResult.alt_tokens)
    near = 1e-5
    alts = set()
    topp_matters = True
    if draw_margin < near:
        for q in (pos - 1, pos + 1):
            if 0 <= q < kept_idx.size:
                alts.add(int(kept_idx[q]))
    if topp_margin < near:
        topp_matters = False
        variants = []
        if abs(mass_gt[n2 - 1] - target_p) / S1 < near and first[n2 - 1] > 0:
            variants.append(int(first[n2 - 1]))                       # the last kept group dropped
        if n2 < n1 and abs(mass_gt[n2] - target_p) / S1 < near:
            variants.append(int(np.searchsorted(-vals, -vals[n2], side="right")))   # the next group kept too
        for n2v in variants:
            ks = np.zeros(V, dtype=bool)
            ks[:n2v] = True
            ks &= minp_sorted
            kv = np.zeros(V, dtype=bool)
            kv[order[ks]] = True
            if kv.any() and not np.array_equal(kv, kept):
                topp_matters = True
                k_idx, c, ps = draw(kv)
                alts.add(int(k_idx[ps]))
                for q in (ps - 1, ps + 1):                            # and its own neighbours
                    if 0 <= q < k_idx.size and float(np.min(np.abs(c / float(c[-1]) - u))) < near:
                        alts.add(int(k_idx[q]))
    alts.discard(tok)

    return RowResult(tok, float(logprob[tok]), top_ids, top_lp, False,
                     kept if keep_arrays else None, u, draw_margin, topp_margin,
                     float(m), logZ, S1, S3, s if keep_arrays else None,
                     topp_matters, tuple(sorted(alts)))


# ----------------------------------------------------------------------------------
# Batch front end (same argument vocabulary as the C boundary, host arrays)
# ----------------------------------------------------------------------------------
_DEFAULTS = dict(temperature=1.0, top_k=0, top_p=1.0, min_p=0.0,
                 repetition_penalty=1.0, frequency_penalty=0.0, presence_penalty=0.0)


def sample_batch(logits: np.ndarray, params: dict, hist_indptr: Optional[np.ndarray],
                 hist_tokens: Optional[np.ndarray], seed: int, step: int, n_logprobs: int,
                 row_ids: Optional[np.ndarray] = None, rows: Optional[Sequence[int]] = None,
                 keep_arrays: bool = False, prompt_indptr: Optional[np.ndarray] = None,
                 prompt_tokens: Optional[np.ndarray] = None):
    """Run ``sample_row`` on the chosen rows (default all) and return the RowResults.

    ``params`` maps the names of ``_DEFAULTS`` to per-row arrays or None (feature off)."""
    B = logits.shape[0]
    rows = range(B) if rows is None else rows
    out = []
    for b in rows:
        kw = {}
        for name, dflt in _DEFAULTS.items():
            arr = params.get(name)
            kw[name] = dflt if arr is None else arr[b]
        hist = None
        if hist_indptr is not None and hist_tokens is not None:
            hist = hist_tokens[int(hist_indptr[b]):int(hist_indptr[b + 1])]
        prompt = None
        if prompt_indptr is not None and prompt_tokens is not None:
            prompt = prompt_tokens[int(prompt_indptr[b]):int(prompt_indptr[b + 1])]
        rid = b if row_ids is None else int(row_ids[b])
        out.append(sample_row(logits[b], history=hist, seed=seed, step=step, row_id=rid,
                              n_logprobs=n_logprobs, keep_arrays=keep_arrays, prompt=prompt, **kw))
    return out


# ----------------------------------------------------------------------------------
# State that persists across decode iterations (Sec. 5.1, "memory reuse" and "incremental
# penalty construction").  The paper preallocates the output matrix Y (L_max x B) and
# appends each iteration's ids to it, and keeps a frequency table f (V x B) per penalty
# type that it updates only at the B newly generated tokens instead of rebuilding it from
# Y.  Here a *slot* is one column of those tables: a sequence keeps its slot for its whole
# life, a batch names the slot of each of its rows, and a finished sequence's slot is
# handed to a new one by ``assign``.  Microbatches in flight at once (the paper's p
# replicas of the state) are disjoint sets of slots of one state.
#
# Readings (the paper does not say): a full slot (L_max tokens) takes no further tokens,
# its history stays as it is and ``overflow`` counts the dropped ids; a prompt longer
# than L_max keeps its first L_max tokens and counts once; the random stream of call
# number t on a state (t = 0 for the first call after ``__init__``) uses Philox step
# ``step + t``, so that a caller who replays one recorded call still gets fresh numbers.

class DecodeState:
    def __init__(self, slots: int, L_max: int, V: int):
        self.slots, self.L_max, self.V = int(slots), int(L_max), int(V)
        self.Y = np.full((self.slots, self.L_max), -1, dtype=np.int32)   # token history per slot
        self.length = np.zeros(self.slots, dtype=np.int64)
        self.f = np.zeros((self.slots, self.V), dtype=np.int32)          # occurrences of v in the slot's history
        self.tick = 0                                                     # sampling calls made so far
        self.overflow = 0

    def _push(self, s: int, t: int) -> bool:
        if self.length[s] >= self.L_max:
            return False
        self.Y[s, self.length[s]] = t
        self.length[s] += 1
        if 0 <= t < self.V:                 # ids outside the vocabulary are padding: stored, never counted
            self.f[s, t] += 1
        return True

    def assign(self, slot: int, tokens: Sequence[int]) -> None:
        """Hand ``slot`` to a new sequence whose history so far (its prompt) is ``tokens``."""
        s = int(slot)
        self.Y[s, :] = -1
        self.length[s] = 0
        self.f[s, :] = 0
        dropped = False
        for t in tokens:
            if not self._push(s, int(t)):
                dropped = True
        self.overflow += int(dropped)

    def history(self, slot: int) -> np.ndarray:
        return self.Y[int(slot), :int(self.length[int(slot)])].copy()


def sample_state(logits: np.ndarray, params: dict, state: DecodeState, slot_of_row: Sequence[int],
                 seed: int, step: int, n_logprobs: int, row_ids: Optional[np.ndarray] = None):
    """One decode iteration on persistent state: every row is sampled with the frequency
    vector of its slot as it stands *before* this call, then the B new ids are appended
    (Y) and counted (f).  A row whose slot is outside [0, slots) has no history and leaves
    no trace.  The slots named by one call must be distinct."""
    B = logits.shape[0]
    out = []
    for b in range(B):
        kw = {}
        for name, dflt in _DEFAULTS.items():
            arr = params.get(name)
            kw[name] = dflt if arr is None else arr[b]
        s = int(slot_of_row[b])
        counts = state.f[s] if 0 <= s < state.slots else np.zeros(state.V, dtype=np.int32)
        rid = b if row_ids is None else int(row_ids[b])
        out.append(sample_row(logits[b], counts=counts, seed=seed, step=step + state.tick, row_id=rid,
                              n_logprobs=n_logprobs, **kw))
    for b in range(B):
        s = int(slot_of_row[b])
        if 0 <= s < state.slots and not state._push(s, int(out[b].token)):
            state.overflow += 1
    state.tick += 1
    return out


# ----------------------------------------------------------------------------------
# Vocabulary-sharded logits (Sec. 5.1 (3), "pipelined integration"): with tensor parallelism of
# degree t each worker of the last stage emits a B x V/t piece of the logits, and the sampler
# sees them side by side.  Definition: piece i holds the vocabulary ids [i * V/t, (i+1) * V/t),
# and sampling the pieces is sampling the matrix they form when put side by side in that order.

def join_shards(shards: Sequence[np.ndarray]) -> np.ndarray:
    return np.concatenate([np.asarray(x) for x in shards], axis=1)


def sample_sharded(shards: Sequence[np.ndarray], params: dict, hist_indptr, hist_tokens, seed: int, step: int,
                   n_logprobs: int, row_ids: Optional[np.ndarray] = None, rows: Optional[Sequence[int]] = None):
    return sample_batch(join_shards(shards), params, hist_indptr, hist_tokens, seed, step, n_logprobs,
                        row_ids=row_ids, rows=rows)
