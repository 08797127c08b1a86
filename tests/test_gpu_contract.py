"""GPU tests of what include/sip.h promises beyond plain parity: bad data in device memory
affects its own row only and never memory safety; what a row returns does not depend on the
batch it sits in; rows that are almost entirely masked, and near-zero temperatures, still come
out right.  Compared with the oracle under the rules of tests/sip_harness.py."""
import numpy as np
import pytest
import torch

import paper_2506_22033_amd as sip
import workloads
from tests import sip_harness as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("V,dtype", [(40000, "f32"), (40000, "bf16"), (3000, "f32")])
def test_bad_rows_leave_good_rows_alone(V, dtype):
    """NaN / +inf logits, a negative temperature, top_p <= 0 and a history that names no valid
    token, mixed into a batch: the good rows equal the oracle's, the bad rows' ids are ids."""
    rng = np.random.default_rng(V)
    B = 16
    z = (rng.standard_normal((B, V)) * 2.5).astype(np.float32)
    params = dict(temperature=rng.uniform(0.4, 1.4, B), top_k=rng.choice([0, 30, 800], B),
                  top_p=rng.uniform(0.8, 1.0, B), min_p=rng.choice([0.0, 0.05], B),
                  frequency_penalty=0.4, presence_penalty=0.2, repetition_penalty=1.1)
    params = {k: np.asarray(np.broadcast_to(v, (B,))).copy() for k, v in params.items()}
    hist = [rng.integers(0, V, 200).tolist() for _ in range(B)]
    bad = [1, 4, 6, 9, 12, 14]
    z[1, 17] = np.nan                                   # one NaN
    z[4, :] = np.nan                                    # all NaN
    z[6, 100] = np.inf                                  # +inf
    params["temperature"][9] = -0.7                     # negative temperature
    params["top_p"][12] = 0.0                           # top_p <= 0
    params["top_p"][14] = -1.0
    hist[3] = [-5, V, V + 9, 2 ** 31 - 1] * 20          # only padding: legal, the row stays a good row
    logits = workloads.f32_to_bf16_bits(z) if dtype == "bf16" else z
    w = H.custom("bad_rows", logits, params, hist, k_logprobs=5)
    good = [b for b in range(B) if b not in bad]
    d = H.to_device(w)
    for step in (0, 1):
        out = H.run_gpu(d, 5, step)
        st = H.compare(w, out, 5, step, rows=good)
        assert st.rows == len(good)
        ids = out[0]
        assert ((ids[bad] >= 0) & (ids[bad] < V)).all(), ids[bad]


def test_a_row_returns_the_same_whatever_batch_it_sits_in():
    """One sequence alone (B = 1: its row is cut into 16 chunks) and inside B = 256 (4 chunks),
    under the same row id: the same token and best-n ids, unless the oracle calls the row
    near-boundary; log-probabilities within the library's tolerance of each other (partial sums
    are formed per chunk, so their last bits may differ)."""
    w = workloads.make(2)                               # B = 256, V = 152064
    d = H.to_device(w)
    full = H.run_gpu(d, 7, 3)
    ref = {r_b: r for r_b, r in zip(range(0, 256, 37), H.oracle_rows(w, 7, 3, w.k_logprobs, range(0, 256, 37)))}
    for b, r in ref.items():
        one = workloads.make(2)
        one.B = 1
        one.logits = w.logits[b:b + 1].copy()
        one.params = {k: (None if v is None else v[b:b + 1].copy()) for k, v in w.params.items()}
        h = w.history(b)
        one.hist_indptr = np.array([0, len(h)], dtype=np.int64)
        one.hist_tokens = np.asarray(h, dtype=np.int32)
        d1 = H.to_device(one)
        rid = torch.tensor([b], dtype=torch.int64, device=H.DEV)
        alone = H.run_gpu(d1, 7, 3, row_ids=rid)
        if not r.flagged():
            assert alone[0][0] == full[0][b] == r.token
        else:
            assert int(alone[0][0]) in (r.token,) + r.alt_tokens and int(full[0][b]) in (r.token,) + r.alt_tokens
        assert np.array_equal(alone[1][0, 1:], full[1][b, 1:])
        err = np.abs(alone[2][0, 1:].astype(np.float64) - full[2][b, 1:].astype(np.float64))
        assert (err <= 2 * (H.LP_ABS + H.LP_REL * np.abs(full[2][b, 1:]))).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rows_that_are_almost_entirely_masked(dtype):
    """Grammar-style masks: 99 % of the vocabulary at -inf (the threshold estimate of the
    streaming pass then falls into the masked part), a single finite token, and a normal row."""
    rng = np.random.default_rng(12)
    V, B = 50000, 6
    z = (rng.standard_normal((B, V)) * 2.0).astype(np.float32)
    for b in range(4):
        keep = rng.choice(V, 500 if b < 3 else 1, replace=False)
        m = np.full(V, -np.inf, dtype=np.float32)
        m[keep] = z[b, keep]
        z[b] = m
    params = dict(temperature=[1.0, 0.7, 0.0, 1.0, 0.9, 1.0], top_k=[0, 20, 0, 0, 0, 50],
                  top_p=[0.9, 1.0, 1.0, 0.95, 0.9, 1.0], min_p=[0.0, 0.05, 0.0, 0.0, 0.02, 0.0],
                  presence_penalty=0.3)
    hist = [rng.integers(0, V, 100).tolist() for _ in range(B)]
    logits = workloads.f32_to_bf16_bits(np.nan_to_num(z, neginf=-1e30)) if dtype == "bf16" else z
    w = H.custom("masked", logits, params, hist, k_logprobs=4)
    d = H.to_device(w)
    for step in (0, 1, 2):
        out = H.run_gpu(d, 9, step)
        st = H.compare(w, out, 9, step)
        assert st.rows == B
    print(f"[masked {dtype}] row paths {H.last_row_path.tolist()}", flush=True)
    if dtype == "f32":
        # the rows with 500 finite tokens are settled from their list (the threshold steps down to
        # the lowest finite sample value); the normal rows anyway
        assert (H.last_row_path[[0, 1, 2, 4, 5]] == 1).all(), H.last_row_path


def test_tiny_temperatures_are_ordinary_stochastic_rows():
    rng = np.random.default_rng(13)
    V, B = 30000, 6
    z = (rng.standard_normal((B, V)) * 2.0).astype(np.float32)
    z[1, 5] = z[1, 9] = z[1].max() + 0.5                # tied maxima: tau -> 0 keeps both
    params = dict(temperature=[1e-6, 1e-6, 1e-4, 3e-2, 1e-6, 1e-3], top_k=[0, 0, 5, 0, 0, 0],
                  top_p=[1.0, 0.9, 1.0, 0.5, 1.0, 1.0], min_p=[0.0, 0.0, 0.0, 0.0, 0.1, 0.0])
    w = H.custom("tiny_tau", z, params, k_logprobs=3)
    d = H.to_device(w)
    for step in range(4):
        st = H.compare(w, H.run_gpu(d, 4, step), 4, step)
        assert st.rows == B
