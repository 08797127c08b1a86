"""sip_sample_call: the combinations that no other entry point offers -- logits as vocabulary
pieces AND histories in a device-resident state AND the ids handed to the host behind the call --
against the oracle's decode state on the pieces put side by side; and the plain combinations
against the entry points they come from, bit for bit."""
import numpy as np
import pytest
import torch

import paper_2506_22033_amd as sip
import workloads
from oracle import sip_oracle as O
from tests import sip_harness as H
from tests.test_gpu_state import DeviceState, _follow, _params

pytestmark = pytest.mark.gpu
DEV = H.DEV


@pytest.mark.parametrize("t,V_shard,bf16", [(4, 20000, False), (2, 16384, True), (3, 1000, False)])
def test_decode_on_pieces_with_state_and_hand_off(t, V_shard, bf16):
    rng = np.random.default_rng(t * 7 + V_shard)
    V, B, slots, L_max, T, k = t * V_shard, 5, 8, 48, 5, 3
    slot_of_row = [3, 0, 7, -1, 5]
    ost, dst = O.DecodeState(slots, L_max, V), DeviceState(slots, L_max)
    prompts = {3: rng.integers(0, V, 20).tolist(), 0: [], 7: rng.integers(0, V, 40).tolist(), 5: [1, 1, 2]}
    for s, p in prompts.items():
        ost.assign(s, p)
    dst.assign(list(prompts), [prompts[s] for s in prompts])
    slot_dev = torch.tensor(slot_of_row, dtype=torch.int32, device=DEV)
    host_ids = torch.full((B,), -1, dtype=torch.int32).pin_memory()
    flag = torch.zeros(1, dtype=torch.int64).pin_memory()
    stats = H.ParityStats()
    for it in range(T):
        z = rng.normal(0, 2.5, (B, V)).astype(np.float32)
        for b, s in enumerate(slot_of_row):
            if 0 <= s < slots and ost.length[s]:
                z[b, ost.history(s)[-5:]] += 6.0
        logits = workloads.f32_to_bf16_bits(z) if bf16 else z
        pieces = [np.ascontiguousarray(logits[:, i * V_shard:(i + 1) * V_shard]) for i in range(t)]
        dpieces = [H.logits_to_device(x) for x in pieces]
        p = _params(rng, B, V)
        dparams = {kk: torch.from_numpy(v).to(DEV) for kk, v in p.items()}
        before = ost.length.copy()
        ids, lpi, lp = sip.sip_sample_call(shards=dpieces, V=V_shard, params=dparams, state=dst.buf, slots=slots,
                                           L_max=L_max, slot_of_row=slot_dev, seed=5, step=100, k_logprobs=k,
                                           host_ids=host_ids, host_flag=flag, ticket=it + 1)
        assert sip.sip_wait_ids(flag, it + 1, 10_000_000_000)
        got = host_ids.numpy().copy()                                       # before any synchronisation
        torch.cuda.synchronize()
        assert np.array_equal(got, ids.cpu().numpy())
        ref = O.sample_state(O.join_shards(pieces), p, ost, slot_of_row, 5, 100, k)
        stats.merge(H.check_rows(f"call t={t} iteration {it}", range(B), ref, (got, lpi.cpu().numpy(), lp.cpu().numpy()), k))
        for b, s in enumerate(slot_of_row):
            if 0 <= s < slots and ost.length[s] > before[s] and got[b] != ref[b].token:
                _follow(ost, s, int(got[b]))
    tick, ovf, length, tokens = dst.read()
    assert tick == T and ovf == 0 and np.array_equal(length, ost.length)
    for s in range(slots):
        assert np.array_equal(tokens[s, :length[s]], ost.history(s))
    print(f"[call] t={t} V_shard={V_shard}: {stats.rows} rows flagged={stats.flagged} max|dlogprob|={stats.max_lp_err:.2e}")


def test_plain_combinations_equal_the_entry_points_they_come_from():
    w = workloads.make(2, B=16, V=40000, H=200)
    d = H.to_device(w)
    k = w.k_logprobs
    a = sip.sip_sample(d.logits, d.params, d.indptr, d.tokens, 3, 4, k, V=w.V)
    b = sip.sip_sample_call(logits=d.logits, V=w.V, params=d.params, hist_indptr=d.indptr, hist_tokens=d.tokens,
                            seed=3, step=4, k_logprobs=k)
    Vs = w.V // 2
    pieces = [d.logits[:, :Vs].contiguous(), d.logits[:, Vs:w.V].contiguous()]
    c = sip.sip_sample_sharded(pieces, d.params, d.indptr, d.tokens, 3, 4, k, V_shard=Vs)
    e = sip.sip_sample_call(shards=pieces, V=Vs, params=d.params, hist_indptr=d.indptr, hist_tokens=d.tokens,
                            seed=3, step=4, k_logprobs=k)
    torch.cuda.synchronize()
    for x, y in ((a, b), (c, e)):
        assert torch.equal(x[0], y[0]) and torch.equal(x[1], y[1]) and torch.equal(x[2].view(torch.int32), y[2].view(torch.int32))


def test_many_rows_many_paths_on_pieces_with_state():
    """48 rows with the whole range of parameters (greedy, huge top-k, nucleus below the list, plain
    temperature sampling: every way a row can leave the single-pass path, each of which gathers the
    row from its pieces first) decoding on a state for three iterations."""
    from tests.test_gpu_random import _params as wide_params
    rng = np.random.default_rng(77)
    t, V_shard, B, slots, L_max, T, k = 4, 20000, 48, 64, 40, 3, 5
    V = t * V_shard
    slot_of_row = rng.permutation(slots)[:B].tolist()
    ost, dst = O.DecodeState(slots, L_max, V), DeviceState(slots, L_max)
    prompts = {s: rng.integers(0, V, int(rng.choice([0, 5, 30]))).tolist() for s in slot_of_row}
    for s, p in prompts.items():
        ost.assign(s, p)
    dst.assign(list(prompts), [prompts[s] for s in prompts])
    slot_dev = torch.tensor(slot_of_row, dtype=torch.int32, device=DEV)
    stats, paths = H.ParityStats(), {}
    for it in range(T):
        z = rng.normal(0, 2.0, (B, V)).astype(np.float32)
        pieces = [np.ascontiguousarray(z[:, i * V_shard:(i + 1) * V_shard]) for i in range(t)]
        p = wide_params(rng, B, V)
        full = {kk: p.get(kk) for kk in ("temperature", "top_k", "top_p", "min_p", "repetition_penalty",
                                        "frequency_penalty", "presence_penalty")}
        dparams = {kk: torch.from_numpy(v).to(DEV) for kk, v in full.items() if v is not None}
        before = ost.length.copy()
        ws = torch.empty(sip.sip_workspace_bytes_sharded(B, V_shard, t, sip.SIP_F32, B * L_max, k), dtype=torch.uint8, device=DEV)
        ids, lpi, lp = sip.sip_sample_call(shards=[H.logits_to_device(x) for x in pieces], V=V_shard, params=dparams,
                                           state=dst.buf, slots=slots, L_max=L_max, slot_of_row=slot_dev, seed=1,
                                           step=0, k_logprobs=k, workspace=ws)
        torch.cuda.synchronize()
        for c in ws[:4 * B].view(torch.int32).cpu().tolist():
            paths[c] = paths.get(c, 0) + 1
        out = (ids.cpu().numpy(), lpi.cpu().numpy(), lp.cpu().numpy())
        ref = O.sample_state(z, full, ost, slot_of_row, 1, 0, k)
        stats.merge(H.check_rows(f"call many paths iteration {it}", range(B), ref, out, k))
        for b, s in enumerate(slot_of_row):
            if ost.length[s] > before[s] and out[0][b] != ref[b].token:
                _follow(ost, s, int(out[0][b]))
    tick, ovf, length, tokens = dst.read()
    assert tick == T and np.array_equal(length, ost.length)
    for s in range(slots):
        assert np.array_equal(tokens[s, :length[s]], ost.history(s))
    print(f"[call] many paths: {stats.rows} rows, paths {paths}, flagged={stats.flagged} mismatch={stats.flagged_mismatch}")
    assert len(set(paths) - {1}) >= 2, "the parameters were meant to send rows down several paths"


@pytest.mark.parametrize("V,bf16", [(40000, False), (40000, True), (1000, False)])
def test_separate_prompt_tokens_feed_the_repetition_penalty_only(V, bf16):
    """sip_sample_call with the prompt handed in as a CSR of its own: repetition over prompt and
    history, frequency and presence over the history alone; on the single-pass kernels and on the
    exact path, with rows that have no history, no prompt, or a repetition penalty of 1."""
    import workloads
    from oracle import sip_oracle as O
    rng = np.random.default_rng(V + bf16)
    B = 12
    z = (rng.standard_normal((B, V)) * 2.5).astype(np.float32)
    hist = [rng.integers(0, V, int(n)).tolist() for n in rng.choice([0, 0, 40, 300], B)]
    prompts = [rng.integers(0, V, int(n)).tolist() for n in rng.choice([0, 25, 500], B)]
    for b in range(B):                                        # make prompt and history matter: their tokens lead the row
        for t in (hist[b][-3:] + prompts[b][:3]):
            z[b, t] += 7.0
        if hist[b] and prompts[b]:
            prompts[b][0] = hist[b][0]                        # a token in both
    params = dict(temperature=rng.choice([0.0, 0.7, 1.0], B), top_k=rng.choice([0, 30], B),
                  top_p=rng.choice([1.0, 0.9], B), min_p=rng.choice([0.0, 0.05], B),
                  repetition_penalty=rng.choice([1.0, 1.3, 0.8], B), frequency_penalty=rng.choice([0.0, 0.4], B),
                  presence_penalty=rng.choice([0.0, 0.5], B))
    logits = workloads.f32_to_bf16_bits(z) if bf16 else z
    w = H.custom("prompt", logits, params, hist, k_logprobs=4)
    d = H.to_device(w)
    p_indptr = np.concatenate(([0], np.cumsum([len(p) for p in prompts]))).astype(np.int64)
    p_tokens = np.array([t for p in prompts for t in p], dtype=np.int32)
    for step in (0, 1):
        ids, lp_ids, lp = sip.sip_sample_call(logits=d.logits, V=V, params=d.params, hist_indptr=d.indptr,
                                              hist_tokens=d.tokens, seed=3, step=step, k_logprobs=4,
                                              prompt_indptr=torch.from_numpy(p_indptr).to(H.DEV),
                                              prompt_tokens=torch.from_numpy(p_tokens).to(H.DEV))
        torch.cuda.synchronize()
        ref = O.sample_batch(w.logits, w.params, w.hist_indptr, w.hist_tokens, 3, step, 4,
                             prompt_indptr=p_indptr, prompt_tokens=p_tokens)
        st = H.check_rows(f"prompt V={V} step {step}", range(B), ref, (ids.cpu().numpy(), lp_ids.cpu().numpy(), lp.cpu().numpy()), 4)
        assert st.rows == B
    # and the prompt does change the result: without it some row differs
    ref0 = O.sample_batch(w.logits, w.params, w.hist_indptr, w.hist_tokens, 3, 0, 4)
    ref1 = O.sample_batch(w.logits, w.params, w.hist_indptr, w.hist_tokens, 3, 0, 4, prompt_indptr=p_indptr, prompt_tokens=p_tokens)
    assert any(abs(a.logprob - c.logprob) > 1e-3 for a, c in zip(ref0, ref1))
