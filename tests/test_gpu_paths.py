"""GPU parity on inputs built to drive every code path of the library at a vocabulary large
enough for the single-pass kernels: the path taken is read back from the workspace
(include/sip.h: 1 single pass, 15 second attempt, 16 finished over the whole row, other = exact
path and why) and the result is
compared with the oracle under the rules of tests/sip_harness.py whichever path ran."""
import numpy as np
import pytest

import workloads
from tests import sip_harness as H

pytestmark = pytest.mark.gpu


def _check(w, steps=(0, 1), seed=2, k=None):
    d = H.to_device(w)
    st = H.ParityStats()
    paths = []
    for step in steps:
        out = H.run_gpu(d, seed, step, k_logprobs=k)
        paths.append(H.last_row_path.copy())
        st.merge(H.compare(w, out, seed, step, k_logprobs=k))
    return st, np.stack(paths)


def test_every_kind_of_row_on_the_single_pass_path():
    rng = np.random.default_rng(0)
    V, B = 40000, 24
    z = (rng.standard_normal((B, V)) * 2.5).astype(np.float32)
    z[:, ::7] = -np.inf                                    # masked vocabulary entries
    z[5, 123] = 30.0                                       # dominant token
    z[6, :] = np.round(z[6, :], 1)                         # many exact ties
    params = dict(temperature=rng.choice([0.0, 0.4, 0.8, 1.0, 1.4], B),
                  top_k=rng.choice([0, 1, 2, 40, 1000, 3000], B),
                  top_p=rng.choice([1.0, 0.95, 0.7, 0.2], B),
                  min_p=rng.choice([0.0, 0.02, 0.1], B),
                  repetition_penalty=rng.choice([1.0, 1.2], B),
                  frequency_penalty=rng.choice([0.0, 0.3], B),
                  presence_penalty=rng.choice([0.0, 0.4, -0.2], B))
    hist = [rng.integers(0, V, int(rng.integers(0, 900))).tolist() for _ in range(B)]
    hist[3] = np.argsort(-z[3])[:300].tolist() * 2          # the whole top of the row carries a penalty
    st, paths = _check(H.custom("mix", z, params, hist, k_logprobs=20), steps=(0, 1, 2))
    assert (paths == 1).mean() > 0.5, paths
    zb = workloads.f32_to_bf16_bits(np.nan_to_num(z, neginf=-60.0))
    st, paths = _check(H.custom("mix_bf16", zb, params, hist, k_logprobs=20), steps=(0, 1))
    assert (paths == 1).mean() > 0.5, paths


def test_second_attempt_with_a_lower_threshold():
    rng = np.random.default_rng(1)
    V, B = 33000, 12
    z = (rng.standard_normal((B, V)) * 2.0).astype(np.float32)
    # rows 0-5: a nucleus of several thousand tokens with nothing else to bound it;
    # rows 6-11: min-p, but the whole top of the row carries a heavy penalty, so the maximum
    # (and with it the min-p cut) ends up far below what the first candidate list covers
    params = dict(temperature=[1.0] * 6 + [0.8] * 6, top_p=[0.9] * 6 + [1.0] * 6, min_p=[0.0] * 6 + [0.05] * 6,
                  presence_penalty=[0.0] * 6 + [6.0] * 6)
    hist = [[] for _ in range(6)] + [np.argsort(-z[b])[:400].tolist() for b in range(6, 12)]
    st, paths = _check(H.custom("retry", z, params, hist, k_logprobs=5), steps=(0, 1, 2))
    assert (paths == 15).any(), paths                      # at least one row needed the retry ...
    assert st.rows == 36                                   # ... and every row matched the oracle


def test_batches_of_more_rows_than_compute_units_queue_their_hard_rows():
    """Up to one row per compute unit a workgroup takes its row through the heavier logic itself;
    beyond that the rows that need it are queued for a kernel of their own.  The same twelve hard
    rows as above, 25 times over (300 rows), must match the oracle on that route as well."""
    rng = np.random.default_rng(1)
    V, B0, rep = 33000, 12, 25
    z0 = (rng.standard_normal((B0, V)) * 2.0).astype(np.float32)
    hist0 = [[] for _ in range(6)] + [np.argsort(-z0[b])[:400].tolist() for b in range(6, 12)]
    params = dict(temperature=([1.0] * 6 + [0.8] * 6) * rep, top_p=([0.9] * 3 + [1.0] * 9) * rep,
                  min_p=([0.0] * 6 + [0.05] * 6) * rep, presence_penalty=([0.0] * 6 + [6.0] * 6) * rep)
    st, paths = _check(H.custom("queued", np.tile(z0, (rep, 1)), params, hist0 * rep, k_logprobs=5), steps=(1,))
    assert st.rows == B0 * rep
    assert (paths == 15).any() and (paths == 16).any(), np.unique(paths, return_counts=True)


def test_large_batch_with_top_k_in_the_thousands():
    """Beyond 512 rows a row is cut into as few as two chunks, whose queues bound the longest list a
    row may have: rows with top_k from 1000 to 7000 (with and without history) must come out
    right whether the list holds them, overflows, or is never made."""
    rng = np.random.default_rng(5)
    V, B = 40000, 1024
    z = (rng.standard_normal((B, V)) * 2.0).astype(np.float32)
    ks = rng.choice([1000, 3000, 4500, 5500, 7000], B)
    params = dict(temperature=rng.uniform(0.6, 1.2, B), top_k=ks, top_p=rng.choice([1.0, 0.95], B),
                  frequency_penalty=rng.choice([0.0, 0.3], B))
    hist = [rng.integers(0, V, int(n)).tolist() for n in rng.choice([0, 200, 1500], B)]
    st, paths = _check(H.custom("big_k", z, params, hist, k_logprobs=2), steps=(0,))
    assert st.rows == B
    assert (paths[0][ks == 1000] == 1).all(), np.unique(paths[0][ks == 1000], return_counts=True)
    why = H.last_row_why
    print("[big_k] (path, reason of the finishing kernel) by k:",
          {int(k): sorted(set(zip(paths[0][ks == k].tolist(), why[ks == k].tolist()))) for k in np.unique(ks)}, flush=True)
    assert (why[ks == 1000] == 1).all()                    # settled by the finishing kernel itself
    assert (why[ks == 7000] != 1).all()                    # beyond what two chunks hand over, or what it sorts


@pytest.mark.parametrize("bf16", [False, True])
def test_nucleus_that_reaches_far_below_the_candidate_list(bf16):
    """top-p alone on flat and on hot distributions keeps tens of thousands of tokens: the cut is
    settled by a radix descent over the whole row and the token drawn there, still on the
    single-pass path.  With and without penalties, with a min-p that does not bound the set."""
    rng = np.random.default_rng(11)
    V, B = 70001, 8
    z = (rng.standard_normal((B, V)) * np.array([0.05, 0.5, 1.0, 2.0, 2.5, 2.5, 1.0, 0.3])[:, None]).astype(np.float32)
    params = dict(temperature=[1.0, 1.0, 1.3, 1.5, 1.5, 2.0, 0.9, 1.0], top_p=[0.9, 0.5, 0.95, 0.9, 0.99, 0.8, 0.7, 0.999],
                  min_p=[0.0, 0.0, 0.0, 0.0, 1e-6, 0.0, 1e-4, 0.0], frequency_penalty=[0.0, 0.7, 0.0, 0.4, 0.0, 0.0, 0.3, 0.0],
                  repetition_penalty=[1.0, 1.2, 1.0, 1.0, 1.1, 1.0, 1.0, 1.0])
    hist = [[] if b % 2 == 0 else rng.integers(0, V, 700).tolist() for b in range(B)]
    logits = workloads.f32_to_bf16_bits(z) if bf16 else z
    st, paths = _check(H.custom("wide_nucleus", logits, params, hist, k_logprobs=5), steps=(0, 1, 2))
    assert st.rows == 3 * B
    assert np.isin(paths, (1, 15, 16)).mean() >= 0.75, paths   # bf16 ties by the hundred may still need the exact path
    assert (paths == 16).any(), paths


def test_rows_that_must_take_the_exact_path():
    rng = np.random.default_rng(2)
    V, B = 50000, 6
    z = (rng.standard_normal((B, V)) * 2.0).astype(np.float32)
    params = dict(temperature=[1.0, 0.9, 1.0, 0.7, 1.0, 0.7], top_k=[0, 20000, 0, 0, 50, 0],
                  top_p=[1.0, 1.0, 0.999, 1.0, 1.0, 1.0], min_p=[0.0, 0.0, 0.0, 0.1, 0.0, 0.1])
    long_hist = rng.integers(0, V, 9000).tolist()                  # > 4096 distinct history tokens
    hist = [[], [], [], long_hist, [], long_hist]
    params.update(repetition_penalty=[1.0, 1.0, 1.0, 1.3, 1.0, 1.3],
                  frequency_penalty=[0.0, 0.0, 0.0, 0.2, 0.0, 0.0])
    st, paths = _check(H.custom("exact", z, params, hist, k_logprobs=3), steps=(0, 1))
    assert (paths[:, 0] == 16).all()                       # plain temperature sampling: single pass + whole-row draw
    assert (paths[:, 1] == 2).all()                        # k far beyond the candidate list
    assert (paths[:, 3] == 4).all()                        # more distinct history tokens than any table of multiplicities holds
    assert (paths[:, 4] == 1).all()
    assert (paths[:, 5] == 1).all()                        # the same history without a frequency penalty needs no multiplicities


@pytest.mark.parametrize("B", [1, 3, 5, 9])
def test_grid_sizes_that_are_not_a_multiple_of_eight(B):
    w = workloads.make(2, B=B, V=70001, H=200)
    st, paths = _check(w, steps=(0,))
    assert st.rows == B


@pytest.mark.parametrize("B,V,dtype_index", [(8, 152064, 2), (2, 262144, 2), (16, 129280, 3)])
def test_small_batches_cut_rows_into_the_largest_number_of_chunks(B, V, dtype_index):
    """Few rows of a large vocabulary: the launch plan uses as many chunks per row as the
    finishing kernel's segment table holds (fp32 and bf16)."""
    w = workloads.make(dtype_index, B=B, V=V, H=300)
    st, paths = _check(w, steps=(0,))
    assert st.rows == B
    assert np.isin(paths, (1, 15)).all()


def test_vocabulary_beyond_the_single_pass_kernels():
    w = workloads.make(4, B=2, V=300000, H=64)
    st, paths = _check(w, steps=(0,))
    assert (paths == 14).all()


def test_plain_temperature_sampling_draws_over_the_whole_row():
    rng = np.random.default_rng(7)
    V, B = 50001, 10
    z = (rng.standard_normal((B, V)) * 2.0).astype(np.float32)
    z[2, 100:40000] = -np.inf
    params = dict(temperature=[1.0, 0.6, 1.7, 0.9, 1.0, 1.3, 0.5, 1.0, 2.0, 0.8],
                  repetition_penalty=[1.0, 1.3, 1.0, 1.0, 1.1, 1.0, 1.0, 1.2, 1.0, 1.0],
                  frequency_penalty=[0.0, 0.2, 0.0, 0.0, 0.0, 0.4, 0.0, 0.0, 0.0, 0.0])
    hist = [rng.integers(0, V, 700).tolist() for _ in range(B)]
    st, paths = _check(H.custom("plain", z, params, hist, k_logprobs=8), steps=(0, 1, 2, 3))
    assert (paths == 16).all(), paths
    zb = workloads.f32_to_bf16_bits(np.nan_to_num(z, neginf=-80.0))
    st, paths = _check(H.custom("plain_bf16", zb, params, hist, k_logprobs=8), steps=(0, 1))
    assert (paths == 16).all(), paths
