"""sip_sample_noalloc (for callers that cannot allocate: the workspace is an array inside the
library's device code) against sip_sample on the same inputs: two calls in a row, the second on a
smaller input, every output bit equal; and its host-side rejections."""
import numpy as np
import pytest
import torch

import paper_2506_22033_amd as sip
import workloads
from tests import sip_harness as H

pytestmark = pytest.mark.gpu


def _both(w, seed, step):
    d = H.to_device(w)
    k = w.k_logprobs
    want = H.run_gpu(d, seed, step)
    ids = torch.full((w.B,), -7, dtype=torch.int32, device=H.DEV)
    lp_ids = torch.full((w.B, 1 + k), -7, dtype=torch.int32, device=H.DEV)
    lp = torch.full((w.B, 1 + k), float("nan"), dtype=torch.float32, device=H.DEV)
    sip.sip_sample_noalloc(d.logits, d.params, d.indptr, d.tokens, seed, step, k, out_ids=ids, out_lp_ids=lp_ids,
                           out_lp=lp, V=d.V)
    torch.cuda.synchronize()
    got = (ids.cpu().numpy(), lp_ids.cpu().numpy(), lp.cpu().numpy())
    for name, g, x in zip(("ids", "logprob ids", "logprobs"), got, want):
        assert np.array_equal(g.view(np.int32), x.view(np.int32)), f"{w.name} B={w.B} V={w.V}: {name} differ"
    return want


def test_noalloc_equals_sip_sample_twice_second_call_smaller():
    sip.sip_init()
    big = workloads.make(2, B=24, V=50021, H=300)           # penalties, every filter, best-20
    small = workloads.make(1, B=5, V=20480, H=64)           # bf16, repetition penalty, smaller in every way
    assert sip.sip_workspace_bytes(big.B, big.V, sip.SIP_F32, int(big.hist_tokens.size), big.k_logprobs) \
        <= sip.sip_noalloc_scratch_bytes()
    out_big = _both(big, 3, 0)
    out_small = _both(small, 3, 1)
    # and against the oracle, under the usual rules
    H.compare(big, out_big, 3, 0)
    H.compare(small, out_small, 3, 1)


def test_noalloc_rejects_what_does_not_fit_before_enqueuing():
    lib = sip.load()
    need = sip.sip_workspace_bytes(2048, 256000, sip.SIP_F32, 0, 0)
    assert need > sip.sip_noalloc_scratch_bytes()
    assert sip.sip_workspace_bytes(256, 152064, sip.SIP_F32, 256 * 1024, 20) <= sip.sip_noalloc_scratch_bytes()
    st = lib.sip_sample_noalloc(0x10000, 2048, 256000, 256000, sip.SIP_F32, None, None, None, 0, 0, 0,
                                0x20000, None, None, -1, None)
    assert st == sip.binding.SIP_ERR_SCRATCH
    assert "scratch" in sip.sip_status_string(st)
