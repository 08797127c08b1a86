"""The CPU sampler in the paper's column-wise layout (baselines/columnwise, a baseline for bench.py)
against the oracle: same tokens except on rows the oracle flags as near-boundary, same best-n,
logprobs within the library's tolerance -- over several decode iterations, so that its
incrementally kept frequency table is what the penalties come from.  No GPU."""
import numpy as np
import pytest

import workloads
from oracle import sip_oracle as O
from baselines.columnwise import ColumnwiseSampler

LP_ABS, LP_REL = 1e-5, 2.0 ** -22


def _params(rng, B, V):
    p = {
        "temperature": np.where(rng.random(B) < 0.15, 0.0, rng.uniform(0.3, 1.8, B)).astype(np.float32),
        "top_k": rng.choice([0, 0, 1, 2, 7, 50, 400, V, V + 3], B).astype(np.int32),
        "top_p": np.where(rng.random(B) < 0.35, 1.0, rng.uniform(0.1, 0.999, B)).astype(np.float32),
        "min_p": np.where(rng.random(B) < 0.5, 0.0, rng.uniform(0.001, 0.4, B)).astype(np.float32),
        "repetition_penalty": np.where(rng.random(B) < 0.4, 1.0, rng.uniform(0.8, 1.5, B)).astype(np.float32),
        "frequency_penalty": np.where(rng.random(B) < 0.4, 0.0, rng.uniform(-0.4, 1.2, B)).astype(np.float32),
        "presence_penalty": np.where(rng.random(B) < 0.4, 0.0, rng.uniform(-0.4, 0.9, B)).astype(np.float32),
    }
    return p


def _check(ref, got, n, ctx):
    ids, lp_ids, lp = got
    flagged = 0
    for b, r in enumerate(ref):
        if r.greedy or not r.flagged():
            assert ids[b] == r.token, f"{ctx} row {b}: {ids[b]} != {r.token}"
        else:
            flagged += 1
        assert lp_ids[b, 0] == ids[b]
        if ids[b] == r.token:
            assert abs(lp[b, 0] - r.logprob) <= LP_ABS + LP_REL * abs(r.logprob), ctx
        k = len(r.top_ids)
        assert np.array_equal(lp_ids[b, 1:1 + k], r.top_ids), f"{ctx} row {b}: best-n ids"
        assert (np.abs(lp[b, 1:1 + k] - r.top_logprobs) <= LP_ABS + LP_REL * np.abs(r.top_logprobs)).all(), ctx
        assert (lp_ids[b, 1 + k:] == -1).all()
    return flagged


@pytest.mark.parametrize("seed,kind,bf16", [(0, "gauss", False), (1, "quantised", False), (2, "heavy", True),
                                            (3, "flat", False), (4, "peaked", True)])
def test_decode_iterations_match_the_oracle(seed, kind, bf16):
    rng = np.random.default_rng(300 + seed)
    B, V, T, n = int(rng.choice([5, 16, 37])), int(rng.choice([900, 3001, 7000])), 4, 4
    cw = ColumnwiseSampler(B, V, threads=4)
    ost = O.DecodeState(B, 64, V)
    for b in range(B):
        prompt = rng.integers(0, V, int(rng.choice([0, 3, 40]))).tolist()
        if prompt and b % 3 == 0:
            prompt[0] = -1
        ost.assign(b, prompt)
        cw.set_history(b, prompt)
    row_ids = np.arange(70, 70 + B, dtype=np.int64)
    flagged = 0
    for t in range(T):
        if kind == "gauss":
            z = rng.normal(0, 2.0, (B, V))
        elif kind == "quantised":
            z = np.round(rng.normal(0, 2.0, (B, V)) * 4) / 4
        elif kind == "heavy":
            z = rng.standard_t(3, (B, V)) * 1.5
        elif kind == "flat":
            z = rng.normal(0, 0.05, (B, V))
        else:
            z = rng.normal(-5, 1, (B, V)); z[np.arange(B), rng.integers(0, V, B)] = 12.0
        z = z.astype(np.float32)
        for b in range(B):
            h = ost.history(b); h = h[(h >= 0) & (h < V)]
            z[b, h[-5:]] += 5.0
        logits = workloads.f32_to_bf16_bits(z) if bf16 else z
        p = _params(rng, B, V)
        ref = O.sample_state(logits, p, ost, list(range(B)), 11, 0, n, row_ids=row_ids)
        half = V // 2                                        # the logits arrive as two vocabulary pieces
        cw.load_logits(np.ascontiguousarray(logits[:, :half]), 0)
        cw.load_logits(np.ascontiguousarray(logits[:, half:]), half)
        got = cw.sample(p, 11, t, n, row_ids=row_ids)        # the oracle's state counts its calls itself
        flagged += _check(ref, got, n, f"{kind} iteration {t}")
        # both continue from the oracle's token (a flagged row may have taken the neighbour)
        cw.push_tokens(np.array([r.token for r in ref], dtype=np.int32))
    cw.close()
    assert flagged <= B
