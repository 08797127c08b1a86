"""GPU parity of the device-resident sampler state (sip_state_init / sip_state_assign /
sip_sample_state, through the C boundary) against the oracle's DecodeState: several decode
iterations in a row, the history never leaving the device, compared after every iteration
under the rules of tests/sip_harness.py, and the state's tables compared entry by entry at
the end."""
import numpy as np
import pytest
import torch

import paper_2506_22033_amd as sip
from oracle import sip_oracle as O
from tests import sip_harness as H

pytestmark = pytest.mark.gpu
DEV = H.DEV


def _params(rng, B, V):
    return {
        "temperature": np.where(rng.random(B) < 0.2, 0.0, rng.uniform(0.3, 1.6, B)).astype(np.float32),
        "top_k": rng.choice([0, 1, 5, 40, 400], B).astype(np.int32),
        "top_p": np.where(rng.random(B) < 0.4, 1.0, rng.uniform(0.3, 0.98, B)).astype(np.float32),
        "min_p": np.where(rng.random(B) < 0.6, 0.0, rng.uniform(0.005, 0.2, B)).astype(np.float32),
        "repetition_penalty": rng.uniform(0.9, 1.4, B).astype(np.float32),
        "frequency_penalty": rng.uniform(0.0, 1.0, B).astype(np.float32),
        "presence_penalty": rng.uniform(0.0, 0.8, B).astype(np.float32),
    }


class DeviceState:
    def __init__(self, slots, L_max):
        self.slots, self.L_max = slots, L_max
        self.buf = torch.empty(sip.sip_state_bytes(slots, L_max), dtype=torch.uint8, device=DEV)
        self.buf.fill_(0xA5)                       # whatever was there before must not matter
        sip.sip_state_init(self.buf, slots, L_max)

    def assign(self, slot_ids, prompts):
        indptr = np.concatenate(([0], np.cumsum([len(p) for p in prompts]))).astype(np.int64)
        toks = np.array([t for p in prompts for t in p], dtype=np.int32)
        sip.sip_state_assign(self.buf, self.slots, self.L_max,
                             torch.tensor(slot_ids, dtype=torch.int32, device=DEV),
                             torch.from_numpy(indptr).to(DEV) if len(toks) else None,
                             torch.from_numpy(toks).to(DEV) if len(toks) else None)

    def read(self):
        torch.cuda.synchronize()
        tick, ovf, length, tokens = sip.state_views(self.buf, self.slots, self.L_max)
        return int(tick.item()), int(ovf.item()), length.cpu().numpy(), tokens.cpu().numpy()


def _follow(st: O.DecodeState, slot: int, gpu_id: int):
    """A near-boundary row may legitimately land on the neighbouring token: the oracle's state
    then continues from the id the device appended, so that later iterations stay comparable."""
    n = int(st.length[slot])
    old = int(st.Y[slot, n - 1])
    st.f[slot, old] -= 1
    st.Y[slot, n - 1] = gpu_id
    st.f[slot, gpu_id] += 1


def _decode(name, V, B, slots, L_max, slot_of_row, prompts, T, seed, bf16=False, k_lp=4, reassign=None, tweak=None):
    import workloads
    rng = np.random.default_rng(seed)
    ost = O.DecodeState(slots, L_max, V)
    dst = DeviceState(slots, L_max)
    live = [s for s in prompts]
    for s in live:
        ost.assign(s, prompts[s])
    dst.assign(live, [prompts[s] for s in live])
    slot_dev = torch.tensor(slot_of_row, dtype=torch.int32, device=DEV)
    row_ids = np.arange(500, 500 + B, dtype=np.int64)
    stats = H.ParityStats()
    paths = {}
    for t in range(T):
        if reassign and t in reassign:
            s, prompt = reassign[t]
            ost.assign(s, prompt)
            dst.assign([s], [prompt])
        z = rng.normal(0.0, 2.5, (B, V)).astype(np.float32)
        for b, s in enumerate(slot_of_row):                         # make the history matter: its tokens lead
            if 0 <= s < slots and ost.length[s] > 0:
                h = ost.history(s)
                h = h[(h >= 0) & (h < V)]
                z[b, h[-6:]] += 6.0
        logits = workloads.f32_to_bf16_bits(z) if bf16 else z
        p = _params(rng, B, V)
        if tweak:
            tweak(p)
        dparams = {k: torch.from_numpy(v).to(DEV) for k, v in p.items()}
        dparams["row_id"] = torch.from_numpy(row_ids).to(DEV)
        dl = H.logits_to_device(logits)
        need = sip.sip_workspace_bytes(B, V, sip.binding.dtype_code(dl), B * L_max, k_lp)
        ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        before = ost.length.copy()
        ids, lp_ids, lp = sip.sip_sample_state(dl, dparams, dst.buf, slots, L_max, slot_dev, 77, 1000, k_lp,
                                               V=V, workspace=ws)
        torch.cuda.synchronize()
        for c in ws[:4 * B].view(torch.int32).cpu().tolist():
            paths[c] = paths.get(c, 0) + 1
        out = (ids.cpu().numpy(), lp_ids.cpu().numpy(), lp.cpu().numpy())
        ref = O.sample_state(logits, p, ost, slot_of_row, 77, 1000, k_lp, row_ids=row_ids)
        stats.merge(H.check_rows(f"{name} iteration {t}", range(B), ref, out, k_lp))
        for b, s in enumerate(slot_of_row):
            if 0 <= s < slots and ost.length[s] > before[s] and out[0][b] != ref[b].token:
                _follow(ost, s, int(out[0][b]))
    tick, ovf, length, tokens = dst.read()
    assert tick == ost.tick == T and ovf == ost.overflow
    assert np.array_equal(length, ost.length)
    for s in range(slots):
        assert np.array_equal(tokens[s, :length[s]], ost.history(s)), f"{name}: slot {s}"
    # each slot's table of multiplicities, kept up to date at the one new token per call, against
    # the oracle's frequency vector f (Sec. 5.1: f is updated at the newly generated tokens only)
    distinct, keys, counts = sip.state_table_views(dst.buf, slots, L_max)
    distinct, keys, counts = distinct.cpu().numpy(), keys.cpu().numpy(), counts.cpu().numpy()
    for s in range(slots):
        h = ost.history(s)
        h = h[h >= 0]
        want = dict(zip(*[x.tolist() for x in np.unique(h, return_counts=True)]))
        if distinct[s] == -1:
            assert len(want) > 3072, f"{name}: slot {s} gave its table up at {len(want)} distinct tokens"
            continue
        used = keys[s] != -1
        got = dict(zip(keys[s][used].tolist(), counts[s][used].tolist()))
        assert distinct[s] == len(want) and got == want, f"{name}: slot {s} table"
        in_v = {t: c for t, c in want.items() if t < V}
        assert all(ost.f[s, t] == c for t, c in in_v.items()) and int(ost.f[s].sum()) == sum(in_v.values())
    print(f"[state] {name}: {stats.rows} rows, paths {paths}, flagged={stats.flagged} "
          f"mismatch={stats.flagged_mismatch} overflow={ovf} max|dlogprob|={stats.max_lp_err:.2e}")
    return stats


@pytest.mark.parametrize("V,bf16", [(20011, False), (33333, True), (1000, False)])
def test_decode_iterations_on_device_state_match_the_oracle(V, bf16):
    rng = np.random.default_rng(V)
    B, slots, L_max = 7, 12, 96
    slot_of_row = [9, 0, -1, 4, 11, 2, 40]                     # -1 and 40: rows without a slot
    prompts = {9: rng.integers(0, V, 30).tolist(), 0: [], 4: rng.integers(0, V, 80).tolist(),
               11: [5, 5, 5, -1, V + 3, 7], 2: rng.integers(0, V, 3).tolist(), 6: [1, 2, 3]}
    st = _decode(f"state V={V} {'bf16' if bf16 else 'f32'}", V, B, slots, L_max, slot_of_row, prompts, T=6,
                 seed=V, bf16=bf16)
    assert st.rows == 6 * B


def test_first_row_of_the_batch_leaves_the_streaming_kernel_early():
    """Row 0 asks for a top_k that no candidate list holds, so the first workgroup of the streaming
    kernel -- the one that also takes the call's number from the state and resets the queue of
    hard rows -- returns before it streams anything.  The call counter, the appended ids and the
    other rows must not notice."""
    rng = np.random.default_rng(3)
    V, B, slots, L_max = 20011, 6, 6, 64
    prompts = {s: rng.integers(0, V, 10 + 5 * s).tolist() for s in range(slots)}

    def tweak(p):
        p["top_k"][0] = 15000
        p["temperature"][0] = 0.9
    st = _decode("state row 0 exact", V, B, slots, L_max, list(range(B)), prompts, T=4, seed=8, tweak=tweak)
    assert st.rows == 4 * B


def test_long_histories_use_the_tables_the_state_keeps():
    """Histories of a few thousand tokens: the finishing kernel copies the slot's table of
    multiplicities instead of counting the history.  Slot 2 has more distinct tokens than a table
    takes: its table is given up and the row is counted, and finished, the long way."""
    rng = np.random.default_rng(21)
    V, B, slots, L_max = 40009, 4, 4, 4200
    zipf = lambda n: (rng.zipf(1.2, n) % V).tolist()
    prompts = {0: zipf(2500), 1: zipf(3900), 2: rng.permutation(V)[:3500].tolist(), 3: zipf(2100)}
    _decode("state long", V, B, slots, L_max, [0, 1, 2, 3], prompts, T=4, seed=10)


def test_full_slots_stay_as_they_are_and_long_prompts_are_cut():
    V, B, slots, L_max = 16384, 4, 4, 8
    rng = np.random.default_rng(3)
    prompts = {0: rng.integers(0, V, 6).tolist(), 1: rng.integers(0, V, 8).tolist(),
               2: rng.integers(0, V, 13).tolist(), 3: []}
    _decode("state overflow", V, B, slots, L_max, [0, 1, 2, 3], prompts, T=5, seed=8)


def test_a_slot_handed_to_a_new_sequence_forgets_the_old_one():
    V, B, slots, L_max = 20011, 3, 5, 40
    rng = np.random.default_rng(4)
    prompts = {1: rng.integers(0, V, 20).tolist(), 2: rng.integers(0, V, 10).tolist(), 3: [9] * 12}
    reassign = {2: (2, [4, 4, 4]), 4: (3, [])}
    _decode("state reuse", V, B, slots, L_max, [1, 2, 3], prompts, T=6, seed=9, reassign=reassign)


def test_state_call_equals_csr_call_at_the_benchmark_shape():
    """B=256, V=152064 fp32 in the launch configuration that bench.py times: the same histories
    once as a CSR and once in a state give the same output bits; afterwards every slot holds its
    history plus the sampled id."""
    import workloads
    w = workloads.make(2)
    d = H.to_device(w)
    B, V = w.B, w.V
    L_max = 4096
    lens = np.diff(w.hist_indptr)
    assert lens.max() < L_max
    slots = B + 5
    slot_of_row = (np.arange(B)[::-1] + 3).astype(np.int32)            # not the identity
    dst = DeviceState(slots, L_max)
    sip.sip_state_assign(dst.buf, slots, L_max, torch.from_numpy(slot_of_row).to(DEV), d.indptr, d.tokens)
    k = w.k_logprobs
    ids0, lpi0, lp0 = sip.sip_sample(d.logits, d.params, d.indptr, d.tokens, 5, 9, k, V=V)
    ids1, lpi1, lp1 = sip.sip_sample_state(d.logits, d.params, dst.buf, slots, L_max,
                                           torch.from_numpy(slot_of_row).to(DEV), 5, 9, k, V=V)
    torch.cuda.synchronize()
    assert torch.equal(ids0, ids1) and torch.equal(lpi0, lpi1) and torch.equal(lp0.view(torch.int32), lp1.view(torch.int32))
    tick, ovf, length, tokens = dst.read()
    assert tick == 1 and ovf == 0
    ids = ids1.cpu().numpy()
    for b in (0, 1, 100, 255):
        s = slot_of_row[b]
        want = np.concatenate((w.hist_tokens[w.hist_indptr[b]:w.hist_indptr[b + 1]], ids[b:b + 1]))
        assert length[s] == len(want) and np.array_equal(tokens[s, :length[s]], want)
    assert (length[:3] == 0).all() and (length[B + 3:] == 0).all()
    # second call: tick = 1, so step 8 here is step 9 there, on the histories grown by one
    ids2, _, _ = sip.sip_sample_state(d.logits, d.params, dst.buf, slots, L_max,
                                      torch.from_numpy(slot_of_row).to(DEV), 5, 8, k, V=V)
    torch.cuda.synchronize()
    _, _, length2, tokens2 = dst.read()
    indptr2 = np.concatenate(([0], np.cumsum(lens + 1))).astype(np.int64)
    toks2 = np.concatenate([tokens2[slot_of_row[b], :length2[slot_of_row[b]] - 1] for b in range(B)]).astype(np.int32)
    ids3, _, _ = sip.sip_sample(d.logits, d.params, torch.from_numpy(indptr2).to(DEV), torch.from_numpy(toks2).to(DEV),
                                5, 9, k, V=V)
    torch.cuda.synchronize()
    assert torch.equal(ids2, ids3)


def test_recorded_decode_step_replays_with_fresh_numbers_each_time():
    """One sip_sample_state call recorded into a graph and replayed: every replay reads the state
    the previous one left (history one longer, tick one higher) and matches the oracle."""
    V, B, slots, L_max, k = 20011, 5, 5, 32, 3
    rng = np.random.default_rng(21)
    slot_of_row = list(range(B))
    p = _params(rng, B, V)
    p["temperature"][:] = np.maximum(p["temperature"], 0.5)             # all rows stochastic
    p["top_k"][:] = 0
    dparams = {kk: torch.from_numpy(v).to(DEV) for kk, v in p.items()}
    dl = torch.zeros(B, (V + 7) // 8 * 8, dtype=torch.float32, device=DEV)      # 16-byte rows
    slot_dev = torch.tensor(slot_of_row, dtype=torch.int32, device=DEV)
    ids = torch.empty(B, dtype=torch.int32, device=DEV)
    lpi = torch.empty(B, 1 + k, dtype=torch.int32, device=DEV)
    lp = torch.empty(B, 1 + k, dtype=torch.float32, device=DEV)
    ws = torch.empty(sip.sip_workspace_bytes(B, V, sip.SIP_F32, B * L_max, k), dtype=torch.uint8, device=DEV)
    dst = DeviceState(slots, L_max)
    z0 = rng.normal(0, 2, (B, V)).astype(np.float32)
    dl[:, :V].copy_(torch.from_numpy(z0))
    # eager call first (one-time kernel attributes are set outside the recording), then start over
    sip.sip_sample_state(dl, dparams, dst.buf, slots, L_max, slot_dev, 3, 0, k, out_ids=ids, out_lp_ids=lpi,
                         out_lp=lp, workspace=ws, V=V)
    sip.sip_state_init(dst.buf, slots, L_max)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sip.sip_sample_state(dl, dparams, dst.buf, slots, L_max, slot_dev, 3, 0, k, out_ids=ids, out_lp_ids=lpi,
                             out_lp=lp, workspace=ws, V=V)
    torch.cuda.synchronize()
    sip.sip_state_init(dst.buf, slots, L_max)                           # recording does not run anything; be sure
    ost = O.DecodeState(slots, L_max, V)
    stats = H.ParityStats()
    seen = []
    for t in range(4):
        z = rng.normal(0, 2, (B, V)).astype(np.float32)
        dl[:, :V].copy_(torch.from_numpy(z))                                # the program's own eager work between replays
        g.replay()
        torch.cuda.synchronize()
        out = (ids.cpu().numpy().copy(), lpi.cpu().numpy().copy(), lp.cpu().numpy().copy())
        ref = O.sample_state(z, p, ost, slot_of_row, 3, 0, k)
        stats.merge(H.check_rows(f"graph replay {t}", range(B), ref, out, k))
        for b in range(B):
            if out[0][b] != ref[b].token:
                _follow(ost, b, int(out[0][b]))
        seen.append(out[0])
    tick, ovf, length, tokens = dst.read()
    assert tick == 4 and ovf == 0 and (length == 4).all()
    assert np.array_equal(tokens[:, :4], np.stack(seen, axis=1))


def test_two_batches_in_flight_on_disjoint_slots_of_one_state():
    """The microbatches of a pipeline share one state and run on their own streams with their own
    workspaces: neither sees the other's slots, every call gets a call-counter value of its own,
    and each batch's ids equal the oracle's for the counter value it drew."""
    import workloads
    rng = np.random.default_rng(31)
    V, Bh, slots, L_max, T = 30011, 6, 12, 64, 3
    dst = DeviceState(slots, L_max)
    prompts = {s: rng.integers(0, V, int(rng.integers(0, 30))).tolist() for s in range(slots)}
    dst.assign(list(range(slots)), [prompts[s] for s in range(slots)])
    ost = O.DecodeState(slots, L_max, V)
    for s in range(slots):
        ost.assign(s, prompts[s])
    halves = [list(range(0, 6)), list(range(6, 12))]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for t in range(T):
        work = []
        for hidx, (rows_slots, st) in enumerate(zip(halves, streams)):
            z = rng.normal(0.0, 2.5, (Bh, V)).astype(np.float32)
            p = _params(rng, Bh, V)
            p["temperature"][:] = np.maximum(p["temperature"], 0.3)        # stochastic rows: the counter matters
            p["top_k"][:] = np.where(p["top_k"] == 1, 5, p["top_k"])
            dparams = {k: torch.from_numpy(v).to(DEV) for k, v in p.items()}
            rid = np.arange(100 * hidx, 100 * hidx + Bh, dtype=np.int64)
            dparams["row_id"] = torch.from_numpy(rid).to(DEV)
            dl = H.logits_to_device(z)
            ws = torch.empty(sip.sip_workspace_bytes(Bh, V, sip.SIP_F32, Bh * L_max, 2), dtype=torch.uint8, device=DEV)
            slot_dev = torch.tensor(rows_slots, dtype=torch.int32, device=DEV)
            work.append((z, p, rid, dl, dparams, ws, slot_dev, rows_slots))
        torch.cuda.synchronize()
        outs = []
        for (z, p, rid, dl, dparams, ws, slot_dev, rows_slots), st in zip(work, streams):      # both enqueued, no wait between
            with torch.cuda.stream(st):
                outs.append(sip.sip_sample_state(dl, dparams, dst.buf, slots, L_max, slot_dev, 5, 40, 2, V=V,
                                                 workspace=ws, stream=st))
        torch.cuda.synchronize()
        # which call drew which counter value is decided on the device: either order must explain both
        base = ost.tick
        ok = False
        for order in ((0, 1), (1, 0)):
            trial = [None, None]
            good = True
            for tick_off, hidx in enumerate(order):
                z, p, rid, dl, dparams, ws, slot_dev, rows_slots = work[hidx]
                ref = [O.sample_row(z[b], counts=ost.f[rows_slots[b]], seed=5, step=40 + base + tick_off, row_id=int(rid[b]),
                                    n_logprobs=2, **{k: v[b] for k, v in p.items()}) for b in range(Bh)]
                ids = outs[hidx][0].cpu().numpy()
                good &= all(ids[b] == r.token or (r.flagged() and int(ids[b]) in r.alt_tokens) for b, r in enumerate(ref))
                trial[hidx] = ids
            if good:
                ok = True
                break
        assert ok, f"iteration {t}: no order of the two calls explains their ids"
        for hidx in (0, 1):
            for b, s in enumerate(halves[hidx]):
                ost._push(s, int(trial[hidx][b]))
        ost.tick += 2
    tick, ovf, length, tokens = dst.read()
    assert tick == 2 * T and ovf == 0
    for s in range(slots):
        assert np.array_equal(tokens[s, :length[s]], ost.history(s)), f"slot {s}"
