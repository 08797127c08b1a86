"""GPU parity on seeded random configurations: vocabulary size, batch, dtype, the shape of the
logit distribution and every sampling parameter are drawn per case (and per row), so that the
single-pass kernels meet list lengths, ties, history sizes and threshold positions that the
five named workloads do not.  Whatever path a row takes, the result must match the oracle
under the rules of tests/sip_harness.py."""
import numpy as np
import pytest

import workloads
from tests import sip_harness as H

pytestmark = pytest.mark.gpu


def _logits(rng, B, V, kind):
    if kind == "gauss":
        z = rng.normal(0.0, rng.uniform(0.5, 4.0), (B, V))
    elif kind == "heavy":                      # Student-t: a few far outliers per row
        z = rng.standard_t(3, (B, V)) * rng.uniform(0.5, 2.0)
    elif kind == "flat":                       # nearly uniform probabilities
        z = rng.normal(0.0, 0.05, (B, V))
    elif kind == "quantised":                  # few distinct values: ties by the thousand
        z = np.round(rng.normal(0.0, 2.0, (B, V)) * 4.0) / 4.0
    elif kind == "peaked":                     # one dominant token per row on a quiet floor
        z = rng.normal(-5.0, 1.0, (B, V))
        z[np.arange(B), rng.integers(0, V, B)] = 12.0
    else:                                      # sorted: the maximum and all candidates sit in one chunk
        z = np.sort(rng.normal(0.0, 2.0, (B, V)), axis=1)
        if rng.random() < 0.5:
            z = z[:, ::-1]
    return np.ascontiguousarray(z, dtype=np.float32)


def _params(rng, B, V):
    p = {}
    p["temperature"] = np.where(rng.random(B) < 0.15, 0.0, rng.uniform(0.2, 2.0, B)).astype(np.float32)
    k_choices = np.array([0, 1, 2, 7, 50, 300, 1000, 3000, min(9000, V - 1), V, V + 5])
    p["top_k"] = k_choices[rng.integers(0, len(k_choices), B)].astype(np.int32)
    p["top_p"] = np.where(rng.random(B) < 0.3, 1.0, rng.uniform(0.05, 0.999, B)).astype(np.float32)
    p["min_p"] = np.where(rng.random(B) < 0.5, 0.0, rng.uniform(0.001, 0.5, B)).astype(np.float32)
    p["repetition_penalty"] = np.where(rng.random(B) < 0.5, 1.0, rng.uniform(0.8, 1.5, B)).astype(np.float32)
    p["frequency_penalty"] = np.where(rng.random(B) < 0.5, 0.0, rng.uniform(-0.5, 1.5, B)).astype(np.float32)
    p["presence_penalty"] = np.where(rng.random(B) < 0.5, 0.0, rng.uniform(-0.5, 1.0, B)).astype(np.float32)
    # some cases leave a parameter out altogether (NULL array at the C boundary)
    for k in list(p):
        if k != "temperature" and rng.random() < 0.15:
            del p[k]
    return p


def _histories(rng, B, V, logits):
    hs = []
    for b in range(B):
        n = int(rng.choice([0, 1, 17, 300, 1100, 2500]))
        if n == 0:
            hs.append([])
            continue
        h = rng.integers(0, V, n)
        # half of the history repeats a few of the row's largest tokens, so that penalties move
        # the head of the distribution and not only its bulk
        top = np.argsort(logits[b])[-8:]
        mask = rng.random(n) < 0.5
        h[mask] = top[rng.integers(0, 8, int(mask.sum()))]
        if rng.random() < 0.3:
            h[rng.integers(0, n)] = -1                                  # padding id
        hs.append(h.tolist())
    return hs


CASES = [(s, kind) for s, kind in enumerate(["gauss", "heavy", "flat", "quantised", "peaked", "sorted",
                                              "gauss", "heavy", "quantised", "gauss"])]


# (seed, kind, batch): the last ones are batches of more rows than the device has compute units,
# which are finished by the lean kernel, two workgroups per compute unit, with the rows it cannot
# settle queued for the rescue kernel, and streamed in two or three chunks per row
CASES = [(s, kind, 0) for s, kind in CASES] + [(20, "gauss", 300), (21, "heavy", 700), (22, "quantised", 1100),
                                              (23, "sorted", 520)]


@pytest.mark.parametrize("seed,kind,batch", CASES)
def test_random_configuration(seed, kind, batch):
    rng = np.random.default_rng(1000 + seed)
    V = int(rng.choice([16384, 20011, 33333, 50257, 70001]))
    B = int(rng.choice([3, 8, 13]))
    if batch:
        B, V = batch, int(rng.choice([16384, 20011, 33333]))
    z = _logits(rng, B, V, kind)
    bf16 = seed % 3 == 1
    logits = workloads.f32_to_bf16_bits(z) if bf16 else z
    k_lp = int(rng.choice([-1, 0, 5, 20])) if seed != 0 else 20
    w = H.custom(f"random[{seed},{kind},{'bf16' if bf16 else 'f32'}] B={B} V={V}", logits, _params(rng, B, V),
                 _histories(rng, B, V, z), k_logprobs=max(k_lp, 0))
    d = H.to_device(w)
    st = H.ParityStats()
    for step in ((0, 1) if not batch else (0,)):
        out = H.run_gpu(d, 7 + seed, step, k_logprobs=k_lp)
        st.merge(H.compare(w, out, 7 + seed, step, k_logprobs=k_lp))
    codes, cnt = np.unique(H.last_row_path, return_counts=True)
    print(f"[random] {w.name}: row paths {dict(zip(codes.tolist(), cnt.tolist()))} flagged={st.flagged} "
          f"mismatch={st.flagged_mismatch} max|dlogprob|={st.max_lp_err:.2e}")
    assert st.rows == (2 if not batch else 1) * B
