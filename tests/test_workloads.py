"""The seeded input generators: shapes, determinism and the stated distributions (no GPU)."""
import numpy as np
import pytest

import workloads


@pytest.mark.parametrize("i", range(5))
def test_small_variants_are_deterministic_and_well_formed(i):
    a = workloads.make(i, B=8, V=4096, H=32)
    b = workloads.make(i, B=8, V=4096, H=32)
    assert a.name == workloads.NAMES[i] and a.B == 8 and a.V == 4096
    assert np.array_equal(a.logits, b.logits)
    assert a.logits.shape == (8, 4096)
    assert a.logits.dtype == (np.float32 if a.dtype == "f32" else np.uint16)
    for k, v in a.params.items():
        if v is not None:
            assert v.shape == (8,) and np.array_equal(v, b.params[k])
    if a.hist_indptr is not None:
        assert a.hist_indptr.dtype == np.int64 and a.hist_tokens.dtype == np.int32
        assert a.hist_indptr[0] == 0 and a.hist_indptr[-1] == a.hist_tokens.size == 8 * 32
        assert a.hist_tokens.min() >= 0 and a.hist_tokens.max() < 4096
        assert np.array_equal(a.hist_tokens, b.hist_tokens)
    assert np.isfinite(a.logits_f32()).all()


def test_c1_full_shape_and_row_kinds():
    w = workloads.make(0)
    assert (w.B, w.V, w.dtype, w.k_logprobs) == (4, 32000, "f32", 5)
    assert w.params["temperature"].tolist() == pytest.approx([0.0, 0.8, 1.0, 0.7])
    assert w.params["top_k"].tolist() == [0, 50, 0, 0]
    assert w.params["top_p"].tolist() == pytest.approx([1.0, 1.0, 0.9, 1.0])
    assert w.params["min_p"].tolist() == pytest.approx([0.0, 0.0, 0.0, 0.05])
    assert abs(float(w.logits.std()) - 2.0) < 0.02 and w.hist_indptr is None


def test_c3_parameter_ranges_and_zipf_history():
    w = workloads.make(2, B=64, V=20000, H=1024)
    t = w.params["temperature"]
    assert t.min() >= 0.3 and t.max() <= 1.5
    assert set(np.unique(w.params["top_k"]).tolist()) <= {0, 20, 50, 1000}
    assert w.params["top_p"].min() >= 0.8 and w.params["top_p"].max() <= 1.0
    # Zipf: heavy duplication, and the most frequent token is shared by all rows
    tops = [np.bincount(w.history(b), minlength=w.V).argmax() for b in range(w.B)]
    assert len(set(tops)) == 1
    assert np.unique(w.history(0)).size < 0.7 * 1024


def test_c2_spikes_and_bf16_grid():
    w = workloads.make(1, B=4, V=8192, H=16)
    z = w.logits_f32()
    assert np.array_equal(workloads.f32_to_bf16_bits(z), w.logits)       # already on the bf16 grid
    assert (z > 3 * 3.0 + 2).sum(axis=1).min() >= 1                        # spikes stick out
