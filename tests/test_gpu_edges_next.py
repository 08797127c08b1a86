"""Corner cases of the device-resident state, the sharded logits and the hand-off: smallest and
largest shapes, rows without history, piece counts that do not divide the sample's blocks, no
logprobs asked for, more ids than one publishing pass of 256 threads holds."""
import numpy as np
import pytest
import torch

import paper_2506_22033_amd as sip
import workloads
from oracle import sip_oracle as O
from tests import sip_harness as H
from tests.test_gpu_random import _histories, _logits, _params
from tests.test_gpu_sharded import _run_sharded
from tests.test_gpu_state import _decode

pytestmark = pytest.mark.gpu
DEV = H.DEV


def test_one_slot_of_one_token():
    st = _decode("state 1x1", 16384, 1, 1, 1, [0], {}, T=3, seed=1)
    assert st.rows == 3


def test_no_row_has_a_slot():
    _decode("state no slots", 20011, 4, 2, 8, [-1, 5, -3, 2**30], {0: [1, 2, 3]}, T=2, seed=2)


def test_state_at_the_largest_single_pass_vocabulary_bf16():
    rng = np.random.default_rng(7)
    prompts = {0: rng.integers(0, 262144, 300).tolist(), 1: rng.integers(0, 262144, 5).tolist()}
    _decode("state V=262144 bf16", 262144, 2, 3, 512, [1, 0], prompts, T=2, seed=3, bf16=True)


@pytest.mark.parametrize("t,V_shard,bf16,k_lp", [(8, 32768, False, 5), (7, 8200, True, 0), (6, 9000, False, -1)])
def test_sharded_corner_shapes(t, V_shard, bf16, k_lp):
    rng = np.random.default_rng(t + V_shard)
    B, V = 3, t * V_shard
    z = _logits(rng, B, V, "gauss")
    logits = workloads.f32_to_bf16_bits(z) if bf16 else z
    w = H.custom(f"sharded corner t={t} V_shard={V_shard}", logits, _params(rng, B, V), _histories(rng, B, V, z),
                 max(k_lp, 0))
    out, path = _run_sharded(w, t, 4, 0, k_lp)
    H.compare(w, out, 4, 0, k_logprobs=k_lp)
    assert (path != 14).all()                              # served by the single-pass kernels


def test_hand_off_of_more_ids_than_one_pass_of_the_publishing_workgroup():
    B = 2048 + 77
    ids = torch.randint(0, 1 << 30, (B,), dtype=torch.int32, device=DEV)
    host = torch.zeros(B, dtype=torch.int32).pin_memory()
    flag = torch.zeros(1, dtype=torch.int64).pin_memory()
    sip.sip_publish_ids(ids, host, flag, 41)
    assert sip.sip_wait_ids(flag, 41, 10_000_000_000)
    got = host.numpy().copy()
    torch.cuda.synchronize()
    assert np.array_equal(got, ids.cpu().numpy())
    assert not sip.sip_wait_ids(flag, 42, 1_000_000)        # a ticket nobody publishes: time-out, no hang
