"""Closed forms, library special cases, hand-computed cases and invariants that pin the
oracle (no GPU).  Each test names the mistake it is there to catch."""
import math

import numpy as np
import pytest
from scipy import special, stats

import workloads
from oracle import sip_oracle as O

f32 = np.float32


# ------------------------------------------------------------------ penalties
def test_penalty_micro_cases_by_hand():
    # +2 -> /2 = 1 -> -0.5*3 = -0.5 -> -0.3 = -0.8 ; -2 -> *2 = -4 -> -5.5 -> -5.8
    z = np.array([2.0, -2.0, 7.0, 0.0], dtype=np.float32)
    hist = np.array([0, 1, 0, 1, 0, 1, 3, 99, -1], dtype=np.int32)    # 99 and -1 are padding
    c = O.history_counts(hist, 4)
    assert c.tolist() == [3, 3, 0, 1]
    out = O.apply_penalties(z, c, 2.0, 0.5, 0.3)
    exp0 = f32(f32(f32(2.0) / f32(2.0)) - f32(f32(0.5) * f32(3.0))) - f32(0.3)
    exp1 = f32(f32(f32(-2.0) * f32(2.0)) - f32(1.5)) - f32(0.3)
    assert out[0] == f32(exp0) and abs(float(out[0]) + 0.8) < 1e-6
    assert out[1] == f32(exp1) and abs(float(out[1]) + 5.8) < 1e-6
    assert out[2] == f32(7.0)                                  # unseen: untouched
    assert out[3] == f32(f32(f32(0.0) * f32(2.0)) - f32(0.5)) - f32(0.3)   # zero counts as "not positive"


def test_repetition_applies_once_per_distinct_token_and_frequency_per_occurrence():
    z = np.array([4.0, 4.0], dtype=np.float32)
    one = O.apply_penalties(z, O.history_counts(np.array([0]), 2), 2.0, 0.0, 0.0)
    five = O.apply_penalties(z, O.history_counts(np.array([0] * 5), 2), 2.0, 0.0, 0.0)
    assert one[0] == five[0] == f32(2.0)
    fr = O.apply_penalties(z, O.history_counts(np.array([0] * 5), 2), 1.0, 0.25, 0.0)
    assert fr[0] == f32(4.0 - 1.25) and fr[1] == f32(4.0)
    pr = O.apply_penalties(z, O.history_counts(np.array([0] * 5), 2), 1.0, 0.0, 0.25)
    assert pr[0] == f32(3.75)                                  # presence ignores the count


def test_penalties_leave_unseen_tokens_bit_identical():
    rng = np.random.default_rng(0)
    V = 500
    z = (rng.standard_normal(V) * 3).astype(np.float32)
    hist = rng.integers(0, V, 60)
    out = O.apply_penalties(z, O.history_counts(hist, V), 1.3, 0.7, -0.2)
    unseen = np.setdiff1d(np.arange(V), hist)
    assert np.array_equal(out[unseen].view(np.uint32), z[unseen].view(np.uint32))
    assert np.all(out[np.unique(hist)] != z[np.unique(hist)])
    # neutral parameters are an exact no-op even on seen tokens
    same = O.apply_penalties(z, O.history_counts(hist, V), 1.0, 0.0, 0.0)
    assert np.array_equal(same.view(np.uint32), z.view(np.uint32))


def test_penalty_changes_the_sampled_distribution_as_expected():
    # two tokens, equal logits; token 0 seen twice with frequency 0.5 -> one nat lower
    z = np.zeros(2, dtype=np.float32)
    r = O.sample_row(z, history=np.array([0, 0]), frequency_penalty=0.5, n_logprobs=2)
    assert r.top_ids.tolist() == [1, 0]
    assert math.isclose(r.top_logprobs[0] - r.top_logprobs[1], 1.0, rel_tol=1e-12)


# ------------------------------------------------------------------ softmax / logprobs
@pytest.mark.parametrize("tau", [0.3, 1.0, 1.7])
def test_logprobs_equal_library_log_softmax(tau):
    rng = np.random.default_rng(3)
    V = 3000
    z = (rng.standard_normal(V) * 4).astype(np.float32)
    r = O.sample_row(z, temperature=tau, top_k=40, top_p=0.9, n_logprobs=V, keep_arrays=True)
    s = (z / f32(tau)).astype(np.float32)
    ref = special.log_softmax(s.astype(np.float64))
    # logprobs are over the whole vocabulary and ignore the filters
    assert np.allclose(r.top_logprobs, np.sort(ref)[::-1], rtol=0, atol=1e-12)
    assert np.allclose(ref[r.top_ids], r.top_logprobs, rtol=0, atol=1e-12)
    assert abs(np.exp(r.top_logprobs).sum() - 1.0) < 1e-12       # probabilities sum to one
    assert math.isclose(r.logprob, ref[r.token], abs_tol=1e-12)


def test_kept_probabilities_sum_to_one():
    rng = np.random.default_rng(4)
    z = (rng.standard_normal(2000) * 2).astype(np.float32)
    r = O.sample_row(z, temperature=0.8, top_k=100, top_p=0.8, min_p=0.01, keep_arrays=True)
    e = np.exp(r.s.astype(np.float64) - r.m)
    assert math.isclose(e[r.kept].sum() / r.S3, 1.0, rel_tol=1e-13)


def test_top_logprob_order_breaks_ties_by_lowest_index():
    z = np.array([1.0, 3.0, 3.0, 0.0, 3.0, 1.0], dtype=np.float32)
    r = O.sample_row(z, n_logprobs=6)
    assert r.top_ids.tolist() == [1, 2, 4, 0, 5, 3]


# ------------------------------------------------------------------ top-k vs library selection
@pytest.mark.parametrize("k", [2, 7, 50, 999])
def test_topk_threshold_equals_partition_kth_value(k):
    rng = np.random.default_rng(k)
    V = 1000
    z = np.round(rng.standard_normal(V) * 3, 1).astype(np.float32)      # rounded -> ties exist
    r = O.sample_row(z, temperature=1.3, top_k=k, keep_arrays=True)
    s = (z / f32(1.3)).astype(np.float32)
    kth = np.partition(s, V - k)[V - k]
    assert np.array_equal(r.kept, s >= kth)
    assert r.kept.sum() >= k


# ------------------------------------------------------------------ closed forms
def test_uniform_logits_closed_form():
    V = 96
    z = np.full(V, 1.25, dtype=np.float32)
    for j in range(64):
        u = j / 64.0
        r = O.sample_row(z, temperature=0.7, top_p=0.5, top_k=10, min_p=0.5, u_override=u,
                         n_logprobs=3, keep_arrays=True)
        assert r.kept.all()                       # one tie group: every filter keeps all of it
        assert r.token == math.floor(u * V)
        assert math.isclose(r.logprob, -math.log(V), rel_tol=1e-13)
        assert r.top_ids.tolist() == [0, 1, 2]


@pytest.mark.parametrize("tau,base", [(1.0, 2.0), (0.5, 4.0)])
def test_geometric_logits_closed_form(tau, base):
    V = 40
    z = (-np.arange(V) * math.log(2.0)).astype(np.float32)     # p_v ~ base^-v
    r = O.sample_row(z, temperature=tau, n_logprobs=V)
    norm = (1 - base ** -V) / (1 - 1 / base)
    expect = np.array([base ** -v / norm for v in range(V)])
    assert np.allclose(np.exp(r.top_logprobs), expect, rtol=2e-6)
    assert r.top_ids.tolist() == list(range(V))
    for p in [0.5, 0.7, 0.9, 0.99, 0.999]:
        rr = O.sample_row(z, temperature=tau, top_p=p, keep_arrays=True)
        size = math.ceil(math.log(1.0 / (1.0 - p)) / math.log(base) - 1e-9)
        assert np.flatnonzero(rr.kept).tolist() == list(range(size)), p
    for mp in [0.3, 0.05, 0.001]:
        rr = O.sample_row(z, temperature=tau, min_p=mp, keep_arrays=True)
        last = math.floor(math.log(1.0 / mp) / math.log(base) + 1e-9)
        assert np.flatnonzero(rr.kept).tolist() == list(range(last + 1)), mp
    for k in [2, 5, 17]:
        rr = O.sample_row(z, temperature=tau, top_k=k, keep_arrays=True)
        assert np.flatnonzero(rr.kept).tolist() == list(range(k))
    # top-p is measured on the mass left by top-k: with k=2 the two survivors hold
    # base/(base+1) and 1/(base+1); p just below the first share keeps one token only
    share = base / (base + 1)
    assert O.sample_row(z, temperature=tau, top_k=2, top_p=share - 0.01, keep_arrays=True).kept.sum() == 1
    assert O.sample_row(z, temperature=tau, top_k=2, top_p=share + 0.01, keep_arrays=True).kept.sum() == 2
    # min-p is applied after top-p (not order-free): p=0.5 keeps token 0 only, whatever min_p says
    assert O.sample_row(z, temperature=tau, top_p=0.4, min_p=0.001, keep_arrays=True).kept.sum() == 1


def test_dominant_spike_is_always_sampled():
    rng = np.random.default_rng(8)
    z = rng.standard_normal(5000).astype(np.float32)
    z[4321] = 60.0
    for step in range(50):
        r = O.sample_row(z, temperature=1.0, top_p=0.9, seed=1, step=step)
        assert r.token == 4321
        r = O.sample_row(z, temperature=1.4, seed=1, step=step)
        assert r.token == 4321


# ------------------------------------------------------------------ invariants of the benchmark spec
def test_greedy_is_lowest_index_argmax_with_ties():
    z = np.array([0.5, 9.0, -1.0, 9.0, 9.0, 2.0], dtype=np.float32)
    for kw in (dict(temperature=0.0), dict(temperature=0.0, top_k=50, top_p=0.1),
               dict(temperature=0.6, top_k=1), dict(temperature=1.0, top_k=1, min_p=0.9)):
        for step in range(5):
            r = O.sample_row(z, step=step, **kw)
            assert r.greedy and r.token == 1
    # greedy rows report logprobs at temperature 1
    r = O.sample_row(z, temperature=0.0, n_logprobs=2)
    ref = special.log_softmax(z.astype(np.float64))
    assert math.isclose(r.logprob, ref[1], abs_tol=1e-12)
    # a tiny positive temperature is a stochastic row that lands on one of the tied maxima
    toks = {O.sample_row(z, temperature=1e-3, step=s).token for s in range(64)}
    assert toks <= {1, 3, 4} and len(toks) > 1


def test_filters_off_is_an_exact_noop():
    rng = np.random.default_rng(9)
    V = 4000
    z = (rng.standard_normal(V) * 2).astype(np.float32)
    for step in range(20):
        a = O.sample_row(z, temperature=0.9, seed=5, step=step, keep_arrays=True)
        b = O.sample_row(z, temperature=0.9, top_k=0, top_p=1.0, min_p=0.0, seed=5, step=step,
                         keep_arrays=True)
        c = O.sample_row(z, temperature=0.9, top_k=V, top_p=1.0, seed=5, step=step, keep_arrays=True)
        assert a.kept.all() and b.kept.all() and c.kept.all()
        assert a.token == b.token == c.token
        assert a.S3 == b.S3 == c.S3


def test_monotonicity_of_each_filter():
    rng = np.random.default_rng(10)
    V = 800
    z = (rng.standard_normal(V) * 2.5).astype(np.float32)
    def size(**kw):
        return int(O.sample_row(z, temperature=0.8, keep_arrays=True, **kw).kept.sum())
    ks = [size(top_k=k) for k in (2, 5, 20, 100, 500, 799)]
    ps = [size(top_p=p) for p in (0.1, 0.3, 0.6, 0.9, 0.99)]
    ms = [size(min_p=q) for q in (0.9, 0.5, 0.1, 0.01, 0.0001)]
    assert ks == sorted(ks) and ps == sorted(ps) and ms == sorted(ms)
    assert ks[0] == 2 and ps[0] >= 1


def test_kept_set_is_permutation_equivariant():
    rng = np.random.default_rng(12)
    V = 600
    z = np.round(rng.standard_normal(V) * 2, 2).astype(np.float32)
    perm = rng.permutation(V)
    a = O.sample_row(z, temperature=0.7, top_k=80, top_p=0.85, min_p=0.02, keep_arrays=True)
    b = O.sample_row(z[perm], temperature=0.7, top_k=80, top_p=0.85, min_p=0.02, keep_arrays=True)
    assert np.array_equal(a.kept[perm], b.kept)


def test_row_result_does_not_depend_on_batch_composition():
    w = workloads.make(2, B=6, V=3000, H=64)
    full = O.sample_batch(w.logits, w.params, w.hist_indptr, w.hist_tokens, 0, 3, 5)
    for b in (0, 3, 5):
        alone = O.sample_batch(w.logits, w.params, w.hist_indptr, w.hist_tokens, 0, 3, 5, rows=[b])[0]
        assert alone.token == full[b].token and alone.logprob == full[b].logprob
        assert np.array_equal(alone.top_ids, full[b].top_ids)
    # a caller-supplied row id replaces the batch position in the random stream
    moved = O.sample_batch(w.logits[3:4], {k: (None if v is None else v[3:4]) for k, v in w.params.items()},
                           np.array([0, 64]), w.history(3), 0, 3, 5, row_ids=np.array([3]))[0]
    assert moved.token == full[3].token


def test_bf16_rows_are_widened_exactly():
    x = np.array([1.0, -2.5, 3.140625, 1e-3], dtype=np.float32)
    bits = workloads.f32_to_bf16_bits(x)
    wide = O.widen(bits)
    assert np.array_equal(wide, workloads.bf16_bits_to_f32(bits))
    assert wide[0] == 1.0 and wide[1] == -2.5 and wide[2] == f32(3.140625)
    # round to nearest even at the 8th mantissa bit: 1 + 2^-8 ties to 1, 1 + 3*2^-8 ties up to 1 + 2^-6
    assert workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(np.array([1 + 2 ** -8], dtype=np.float32)))[0] == 1.0
    assert workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(np.array([1 + 3 * 2 ** -8], dtype=np.float32)))[0] == f32(1 + 2 ** -6)


# ------------------------------------------------------------------ draw statistics
def test_draw_frequencies_follow_the_filtered_distribution():
    z = np.array([2.0, 0.5, 1.0, -1.0, 1.5, 0.0, 2.0, -3.0], dtype=np.float32)
    tau, k = 0.9, 4                        # top-4 keeps values >= 1.0 -> tokens 0, 2, 4, 6
    s = (z / f32(tau)).astype(np.float64)
    keep = np.array([0, 2, 4, 6])
    pr = special.softmax(s[keep])
    N = 20000
    cnt = np.zeros(8)
    for step in range(N):
        cnt[O.sample_row(z, temperature=tau, top_k=k, seed=42, step=step, row_id=7).token] += 1
    assert cnt[[1, 3, 5, 7]].sum() == 0
    chi = ((cnt[keep] - N * pr) ** 2 / (N * pr)).sum()
    assert stats.chi2.sf(chi, len(keep) - 1) > 1e-4


# ------------------------------------------------------------------ near-boundary bookkeeping
def test_margins_flag_the_rows_that_can_flip():
    z = np.zeros(4, dtype=np.float32)                         # CDF boundaries at 0.25, 0.5, 0.75, 1
    assert O.sample_row(z, u_override=0.5 + 1e-8).flagged()
    assert not O.sample_row(z, u_override=0.6).flagged()
    # top-p cut: two tokens with masses 2/3, 1/3 and p = 2/3 lands on the group edge
    zz = np.array([math.log(2.0), 0.0], dtype=np.float32)
    r = O.sample_row(zz, top_p=2.0 / 3.0, u_override=0.1)
    assert r.topp_margin < 1e-6 and r.flagged()
    assert not O.sample_row(zz, top_p=0.5, u_override=0.1).flagged()


# ---------------------------------------------------------------- near-boundary accounting
def test_alternatives_of_a_draw_next_to_a_cdf_edge_are_the_neighbouring_tokens():
    # four equal logits: CDF edges at 1/4, 1/2, 3/4; a uniform just below 1/2 picks token 1 and is
    # within 1e-6 of the edge, so a lower-precision CDF may land on token 2 (or, the other way, 0)
    row = np.zeros(4, dtype=np.float32)
    r = O.sample_row(row, temperature=1.0, u_override=0.5 - 1e-9)
    assert r.token == 1 and r.flagged() and r.draw_margin < 1e-8
    assert set(r.alt_tokens) == {0, 2}
    far = O.sample_row(row, temperature=1.0, u_override=0.4)
    assert far.token == 1 and not far.flagged() and far.alt_tokens == ()


def test_alternatives_of_a_nucleus_cut_on_a_group_edge():
    # probabilities 1/2, 1/4, 1/8, 1/8 and p = 3/4: the mass above the tied pair {2, 3} equals the
    # target up to rounding, so the pair is kept or dropped on the last bit; u = 0.9 then draws
    # token 3 (pair kept) or token 1 (pair dropped) -- one is the result, the other the alternative
    row = np.log(np.array([0.5, 0.25, 0.125, 0.125])).astype(np.float32)
    r = O.sample_row(row, temperature=1.0, top_p=0.75, u_override=0.9)
    assert r.topp_margin < 1e-9 and r.topp_matters and r.flagged()
    assert {r.token} | set(r.alt_tokens) == {1, 3}
    # with min-p 0.3 the pair (1/8 < 0.3 * 1/2) is removed wherever the nucleus ends: the same
    # razor-edge cut no longer decides anything, and the row is not near-boundary
    q = O.sample_row(row, temperature=1.0, top_p=0.75, min_p=0.3, u_override=0.9)
    assert q.topp_margin < 1e-9 and not q.topp_matters and not q.flagged()
    assert q.token == 1 and q.alt_tokens == ()


# ---------------------------------------------------------------- separate prompt tokens
def test_a_separate_prompt_feeds_the_repetition_penalty_only():
    # z = +2 / -2, theta = 2, phi = 0.5, psi = 0.3.  Token 0: in the output 3 times -> all three
    # penalties (+2 -> 1 -> -0.5 -> -0.8).  Token 1: in the prompt only -> repetition only (-2 -> -4).
    # Token 2: in both (output once) -> 2 -> 1 -> 0.5 -> 0.2.  Token 3: in neither -> untouched.
    z = np.array([2.0, -2.0, 2.0, -2.0], dtype=np.float32)
    c_out = np.array([3, 0, 1, 0])
    c_prompt = np.array([0, 5, 2, 0])
    got = O.apply_penalties(z, c_out, 2.0, 0.5, 0.3, c_prompt)
    f = np.float32
    want = np.array([f(-0.5) - f(0.3), -4.0, f(0.5) - f(0.3), -2.0], dtype=np.float32)     # one fp32 rounding per step
    assert np.array_equal(got, want) and abs(float(got[0]) + 0.8) < 1e-6 and abs(float(got[2]) - 0.2) < 1e-6
    # a prompt that is handed in as part of the one history counts for everything instead
    merged = O.apply_penalties(z, c_out + c_prompt, 2.0, 0.5, 0.3)
    assert np.array_equal(merged, np.array([np.float32(1.0) - np.float32(1.5) - np.float32(0.3),
                                            np.float32(-4.0) - np.float32(2.5) - np.float32(0.3),
                                            np.float32(1.0) - np.float32(1.5) - np.float32(0.3), -2.0], dtype=np.float32))
    # no prompt given, or an empty one, or theta = 1: the separate prompt changes nothing
    assert np.array_equal(O.apply_penalties(z, c_out, 2.0, 0.5, 0.3, np.zeros(4, int)), O.apply_penalties(z, c_out, 2.0, 0.5, 0.3))
    assert np.array_equal(O.apply_penalties(z, c_out, 1.0, 0.5, 0.3, c_prompt), O.apply_penalties(z, c_out, 1.0, 0.5, 0.3))
    # and through the row front end
    r = O.sample_row(z, temperature=0.0, repetition_penalty=2.0, frequency_penalty=0.5, presence_penalty=0.3,
                     history=np.array([0, 0, 0, 2]), prompt=np.array([1, 1, 2]), n_logprobs=4, keep_arrays=True)
    assert np.array_equal(r.s, want) and r.token == 2
