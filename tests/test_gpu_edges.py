"""GPU edge cases: ties, -inf, degenerate sizes, histories with padding and empty rows,
filters at their limits.  Compared with the oracle under the rules of tests/sip_harness.py."""
import numpy as np
import pytest

import workloads
from tests import sip_harness as H

pytestmark = pytest.mark.gpu


def _check(w, steps=(0, 1, 2), seed=1, k=None):
    d = H.to_device(w)
    st = H.ParityStats()
    for step in steps:
        st.merge(H.compare(w, H.run_gpu(d, seed, step, k_logprobs=k), seed, step, k_logprobs=k))
    return st


def test_ties_everywhere():
    rng = np.random.default_rng(0)
    grid = np.array([-2.0, -1.0, 0.0, 0.5, 1.0, 3.0], dtype=np.float32)
    z = rng.choice(grid, size=(24, 4099)).astype(np.float32)
    B = z.shape[0]
    params = dict(temperature=rng.choice([0.0, 0.5, 1.0, 1.3], B), top_k=rng.choice([0, 1, 2, 7, 100, 5000], B),
                  top_p=rng.choice([1.0, 0.9, 0.5, 0.1], B), min_p=rng.choice([0.0, 0.05, 0.5, 1.0], B))
    _check(H.custom("ties", z, params, k_logprobs=9))


def test_all_equal_rows_and_greedy_tie_break():
    z = np.full((6, 1000), 0.75, dtype=np.float32)
    params = dict(temperature=[0.0, 1.0, 0.6, 1.0, 1.0, 1.0], top_k=[0, 0, 1, 5, 0, 0],
                  top_p=[1.0, 1.0, 1.0, 0.3, 0.5, 1.0], min_p=[0.0, 0.0, 0.0, 0.0, 0.2, 1.0])
    st = _check(H.custom("equal", z, params, k_logprobs=4), steps=range(6))
    assert st.greedy_rows == 12


def test_minus_infinity_logits_are_never_sampled():
    rng = np.random.default_rng(1)
    z = (rng.standard_normal((8, 3001)) * 2).astype(np.float32)
    z[:, ::3] = -np.inf
    z[3, 1:] = -np.inf                 # only token 0... which is -inf as well, so keep one finite
    z[3, 7] = 0.25
    params = dict(temperature=[0.0, 1.0, 0.7, 1.0, 1.2, 1.0, 0.9, 1.0], top_k=[0, 0, 40, 0, 0, 3000, 2, 0],
                  top_p=[1.0, 1.0, 0.9, 0.9, 1.0, 0.99, 1.0, 0.2])
    w = H.custom("neginf", z, params, k_logprobs=3)
    d = H.to_device(w)
    for step in range(4):
        out = H.run_gpu(d, 2, step)
        H.compare(w, out, 2, step)
        assert np.isfinite(z[np.arange(8), out[0]]).all()
        assert out[0][3] == 7


@pytest.mark.parametrize("V", [1, 2, 3, 4, 5, 63, 64, 65, 255, 257, 1023, 4097])
def test_tiny_and_ragged_vocabularies(V):
    rng = np.random.default_rng(V)
    z = (rng.standard_normal((5, V)) * 2).astype(np.float32)
    params = dict(temperature=[0.0, 1.0, 0.8, 1.1, 0.9], top_k=[0, 0, 3, 0, 2],
                  top_p=[1.0, 1.0, 1.0, 0.7, 0.6], min_p=[0.0, 0.0, 0.0, 0.1, 0.0],
                  repetition_penalty=1.2, frequency_penalty=0.1, presence_penalty=0.2)
    hist = [rng.integers(0, V, 7).tolist() for _ in range(5)]
    _check(H.custom(f"tinyV{V}", z, params, hist, k_logprobs=6))           # k_logprobs > V for small V
    zb = workloads.f32_to_bf16_bits(z)
    _check(H.custom(f"tinyV{V}bf16", zb, params, hist, k_logprobs=2))


def test_filters_at_their_limits():
    rng = np.random.default_rng(5)
    V = 7001
    z = (rng.standard_normal((10, V)) * 3).astype(np.float32)
    z[6, 1234] = 40.0                                # single-token nucleus
    params = dict(temperature=[1.0, 1.0, 1.0, 0.5, 1.0, 1e-3, 1.0, 2.5, 1.0, 1.0],
                  top_k=[V, V + 7, V - 1, 2, 0, 0, 0, 0, -3, 6999],
                  top_p=[1.0, 1.0, 1.0, 1.0, 1e-6, 1.0, 0.5, 0.999999, 1.5, 0.97],
                  min_p=[0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 1e-30, 0.0, 1e-6])
    st = _check(H.custom("limits", z, params, k_logprobs=64), steps=range(4))
    assert st.rows == 40


def test_history_padding_empty_rows_and_duplicates():
    rng = np.random.default_rng(6)
    V = 6007
    z = (rng.standard_normal((6, V)) * 2).astype(np.float32)
    z[2, 17] = 9.0                                   # the repeated favourite gets pushed down
    hist = [[], [5, 5, 5, -1, V, V + 100, 2 ** 31 - 1, -7], [17] * 40 + [3, 4], list(range(0, V, 2)),
            rng.integers(0, V, 3000).tolist(), [V - 1, 0, V - 1]]
    params = dict(temperature=[1.0, 0.0, 0.7, 1.0, 0.9, 0.0], top_k=[0, 0, 50, 0, 100, 0],
                  top_p=[0.9, 1.0, 1.0, 0.95, 0.9, 1.0],
                  repetition_penalty=[1.3, 1.3, 1.0, 0.8, 1.1, 2.0],
                  frequency_penalty=[0.5, 0.5, 0.25, 0.0, -0.1, 0.0],
                  presence_penalty=[0.2, 0.2, 0.0, 0.3, 0.1, 0.0])
    _check(H.custom("hist", z, params, hist, k_logprobs=5), steps=range(3))
    zb = workloads.f32_to_bf16_bits(z)
    _check(H.custom("hist_bf16", zb, params, hist, k_logprobs=5), steps=range(3))


def test_k_logprobs_variants_and_no_logprobs():
    rng = np.random.default_rng(7)
    z = (rng.standard_normal((4, 2050)) * 2).astype(np.float32)
    w = H.custom("klp", z, dict(temperature=0.9, top_p=0.9), k_logprobs=0)
    d = H.to_device(w)
    base = H.run_gpu(d, 3, 0, k_logprobs=0)
    for k in (-1, 1, 20, 64):
        out = H.run_gpu(d, 3, 0, k_logprobs=k)
        assert np.array_equal(out[0], base[0])                 # the draw does not depend on k_logprobs
        if k < 0:
            assert out[1] is None and out[2] is None
        else:
            H.compare(w, out, 3, 0, k_logprobs=k)
