"""The ids reach a host thread through pinned memory and a polled ticket (sip_publish_ids /
sip_wait_ids), without any stream synchronisation, and are the ids the oracle gives."""
import numpy as np
import pytest
import torch

import paper_2506_22033_amd as sip
import workloads
from tests import sip_harness as H

pytestmark = pytest.mark.gpu
DEV = H.DEV
TEN_SECONDS = 10_000_000_000


def test_ids_arrive_on_the_host_with_their_ticket():
    w = workloads.make(0)                                   # C1: 4 rows, V = 32000
    d = H.to_device(w)
    host_ids = torch.full((w.B,), -7, dtype=torch.int32).pin_memory()
    flag = torch.zeros(1, dtype=torch.int64).pin_memory()
    for step, ticket in ((0, 1), (1, 2), (5, 9)):
        ids, lpi, lp = sip.sip_sample(d.logits, d.params, d.indptr, d.tokens, 42, step, w.k_logprobs, V=w.V)
        sip.sip_publish_ids(ids, host_ids, flag, ticket)
        assert sip.sip_wait_ids(flag, ticket, TEN_SECONDS)                      # no torch / HIP synchronisation before this
        got = host_ids.numpy().copy()
        assert int(flag[0]) == ticket
        torch.cuda.synchronize()
        assert np.array_equal(got, ids.cpu().numpy())
        H.compare(w, (got, lpi.cpu().numpy(), lp.cpu().numpy()), 42, step)


def test_ring_of_slots_keeps_several_batches_in_flight():
    """Six decode iterations on a device-resident state are enqueued back to back, each publishing
    into slot i % 3 of a ring; the host then collects them in order.  What arrives is what the
    state recorded."""
    V, B, slots, L_max, T, R = 20011, 6, 6, 16, 6, 3
    rng = np.random.default_rng(2)
    z = rng.normal(0, 2, (B, V)).astype(np.float32)
    dl = H.logits_to_device(z)
    params = {"temperature": torch.full((B,), 0.9, device=DEV), "top_k": torch.full((B,), 50, dtype=torch.int32, device=DEV),
              "frequency_penalty": torch.full((B,), 0.8, device=DEV)}
    state = torch.empty(sip.sip_state_bytes(slots, L_max), dtype=torch.uint8, device=DEV)
    sip.sip_state_init(state, slots, L_max)
    slot_of_row = torch.arange(B, dtype=torch.int32, device=DEV)
    ring_ids = [torch.full((B,), -1, dtype=torch.int32).pin_memory() for _ in range(R)]
    ring_flag = [torch.zeros(1, dtype=torch.int64).pin_memory() for _ in range(R)]
    outs = [torch.empty(B, dtype=torch.int32, device=DEV) for _ in range(R)]
    ws = torch.empty(sip.sip_workspace_bytes(B, V, sip.SIP_F32, B * L_max, -1), dtype=torch.uint8, device=DEV)
    seen = []
    for i in range(T):
        if i >= R:                                           # the slot is reused: its previous batch must have been read
            j = i - R
            assert sip.sip_wait_ids(ring_flag[j % R], j + 1, TEN_SECONDS)
            seen.append(ring_ids[j % R].numpy().copy())
        sip.sip_sample_state(dl, params, state, slots, L_max, slot_of_row, 7, 0, -1, out_ids=outs[i % R],
                             workspace=ws, V=V)
        sip.sip_publish_ids(outs[i % R], ring_ids[i % R], ring_flag[i % R], i + 1)
    for j in range(T - R, T):
        assert sip.sip_wait_ids(ring_flag[j % R], j + 1, TEN_SECONDS)
        seen.append(ring_ids[j % R].numpy().copy())
    torch.cuda.synchronize()
    _, _, length, tokens = sip.state_views(state, slots, L_max)
    assert (length.cpu().numpy() == T).all()
    assert np.array_equal(tokens.cpu().numpy()[:, :T], np.stack(seen, axis=1))
