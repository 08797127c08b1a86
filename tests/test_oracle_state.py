"""Pins of the oracle's persistent decode state (oracle.sip_oracle.DecodeState / sample_state;
Sec. 5.1 "memory reuse" and "incremental penalty construction") against things other than
itself: a hand-worked greedy sequence, the from-scratch route (explicit CSR of a history the
test keeps on its own, counted by numpy), and the invariants the construction must have
(slot reuse, batch order, disjoint microbatches, a full slot).  No GPU."""
import numpy as np

from oracle import sip_oracle as O


def _params(rng, B):
    return {
        "temperature": np.where(rng.random(B) < 0.25, 0.0, rng.uniform(0.3, 1.5, B)).astype(np.float32),
        "top_k": rng.choice([0, 1, 3, 20], B).astype(np.int32),
        "top_p": np.where(rng.random(B) < 0.4, 1.0, rng.uniform(0.2, 0.95, B)).astype(np.float32),
        "min_p": np.where(rng.random(B) < 0.6, 0.0, rng.uniform(0.01, 0.2, B)).astype(np.float32),
        "repetition_penalty": rng.uniform(0.8, 1.4, B).astype(np.float32),
        "frequency_penalty": rng.uniform(-0.3, 1.0, B).astype(np.float32),
        "presence_penalty": rng.uniform(-0.3, 0.8, B).astype(np.float32),
    }


def test_hand_worked_greedy_sequence_under_a_frequency_penalty():
    # z = (1.0, 0.9, 0.8), phi = 0.15, greedy.  By hand:
    #   s=0: (1.00, 0.90, 0.80) -> 0      s=1: (0.85, 0.90, 0.80) -> 1
    #   s=2: (0.85, 0.75, 0.80) -> 0      s=3: (0.70, 0.75, 0.80) -> 2
    #   s=4: (0.70, 0.75, 0.65) -> 1      s=5: (0.70, 0.60, 0.65) -> 0
    z = np.array([[1.0, 0.9, 0.8]], dtype=np.float32)
    p = {"temperature": np.zeros(1, np.float32), "frequency_penalty": np.full(1, 0.15, np.float32)}
    st = O.DecodeState(slots=2, L_max=16, V=3)
    got = [O.sample_state(z, p, st, [1], seed=0, step=0, n_logprobs=0)[0].token for _ in range(6)]
    assert got == [0, 1, 0, 2, 1, 0]
    assert st.history(1).tolist() == got and st.length[0] == 0 and st.tick == 6
    assert st.f[1].tolist() == [3, 2, 1]


def test_incremental_state_equals_the_from_scratch_route_step_by_step():
    rng = np.random.default_rng(5)
    V, B, slots, L_max, T = 101, 5, 9, 40, 12
    st = O.DecodeState(slots, L_max, V)
    slot_of_row = [7, 2, 8, 0, 4]
    mine = {s: [] for s in range(slots)}                 # the test's own record of every slot
    for s in (7, 2, 0):
        prompt = rng.integers(0, V, rng.integers(1, 9)).tolist()
        if s == 2:
            prompt[0] = -1                               # padding id: stored, never counted
        st.assign(s, prompt)
        mine[s] = list(prompt)
    row_ids = np.array([100, 101, 102, 103, 104], dtype=np.int64)
    for t in range(T):
        z = rng.normal(0, 2, (B, V)).astype(np.float32)
        p = _params(rng, B)
        # from scratch: CSR of the test's record, counted anew, explicit step
        indptr = np.concatenate(([0], np.cumsum([len(mine[s]) for s in slot_of_row]))).astype(np.int64)
        toks = np.array([x for s in slot_of_row for x in mine[s]], dtype=np.int32)
        want = O.sample_batch(z, p, indptr, toks, seed=9, step=30 + t, n_logprobs=3, row_ids=row_ids)
        got = O.sample_state(z, p, st, slot_of_row, seed=9, step=30, n_logprobs=3, row_ids=row_ids)
        for b, s in enumerate(slot_of_row):
            assert got[b].token == want[b].token, (t, b)
            assert got[b].logprob == want[b].logprob
            assert np.array_equal(got[b].top_ids, want[b].top_ids)
            mine[s].append(int(want[b].token))
        for s in range(slots):
            assert st.history(s).tolist() == mine[s]
            h = np.array([x for x in mine[s] if 0 <= x < V], dtype=np.int64)
            assert np.array_equal(st.f[s], np.bincount(h, minlength=V))
    assert st.tick == T and st.overflow == 0


def test_a_full_slot_takes_no_more_tokens_and_is_counted():
    z = np.array([[0.0, 3.0, 1.0, 2.0]], dtype=np.float32)
    p = {"temperature": np.zeros(1, np.float32), "presence_penalty": np.full(1, 1.5, np.float32)}
    st = O.DecodeState(slots=1, L_max=3, V=4)
    st.assign(0, [0, 0])
    toks = [O.sample_state(z, p, st, [0], 0, 0, 0)[0].token for _ in range(4)]
    # s=0 history (0,0): (-1.5, 3, 1, 2) -> 1, appended.  Afterwards the history stays (0,0,1):
    # (-1.5, 1.5, 1, 2) -> 3 every time, never appended.
    assert toks == [1, 3, 3, 3]
    assert st.history(0).tolist() == [0, 0, 1] and st.overflow == 3
    st2 = O.DecodeState(slots=1, L_max=3, V=4)
    st2.assign(0, [2, 2, 1, 3, 3])
    assert st2.history(0).tolist() == [2, 2, 1] and st2.overflow == 1 and st2.f[0].tolist() == [0, 1, 2, 0]


def test_reused_slot_behaves_like_a_fresh_one_and_rows_without_a_slot_leave_no_trace():
    rng = np.random.default_rng(11)
    V, B = 64, 3
    zs = [rng.normal(0, 2, (B, V)).astype(np.float32) for _ in range(5)]
    p = _params(rng, B)
    used = O.DecodeState(4, 20, V)
    for s in range(4):
        used.assign(s, rng.integers(0, V, 10).tolist())
    for z in zs[:2]:
        O.sample_state(z, p, used, [0, 1, 2], 3, 0, 0)
    fresh = O.DecodeState(4, 20, V)
    for st in (used, fresh):
        st.assign(1, [5, 5, 9])
        st.assign(2, [])
    a = [[r.token for r in O.sample_state(z, p, used, [1, -1, 2], 3, 10 - used.tick, 0)] for z in zs[2:]]
    b = [[r.token for r in O.sample_state(z, p, fresh, [1, 99, 2], 3, 10 - fresh.tick, 0)] for z in zs[2:]]
    assert a == b
    assert used.history(1).tolist() == [5, 5, 9] + [x[0] for x in a]
    assert used.history(2).tolist() == [x[2] for x in a]
    # the slot-less middle row: same draw as a row with an empty history, nothing stored
    want = O.sample_batch(zs[2], p, None, None, 3, 10, 0)
    assert a[0][1] == want[1].token
    assert used.length[3] == 10 and fresh.length[3] == 0


def test_batch_order_does_not_matter_when_row_ids_travel_with_the_sequences():
    rng = np.random.default_rng(13)
    V, B, T = 80, 4, 6
    p = _params(rng, B)
    zs = [rng.normal(0, 1.5, (B, V)).astype(np.float32) for _ in range(T)]
    ids = np.array([40, 41, 42, 43], dtype=np.int64)
    a, b = O.DecodeState(B, 16, V), O.DecodeState(B, 16, V)
    for t, z in enumerate(zs):
        perm = rng.permutation(B)
        O.sample_state(z, p, a, [0, 1, 2, 3], 1, 0, 0, row_ids=ids)
        O.sample_state(z[perm], {k: v[perm] for k, v in p.items()}, b, perm.tolist(), 1, 0, 0, row_ids=ids[perm])
    for s in range(B):
        assert a.history(s).tolist() == b.history(s).tolist() and len(a.history(s)) == T


def test_microbatches_on_disjoint_slots_of_one_state_do_not_see_each_other():
    # two microbatches alternate on one state (the paper's replicas of the sampler state for
    # batches in flight, Sec. 5.1) -- same tokens as two states of their own, the call counter
    # made up for by the step argument
    rng = np.random.default_rng(17)
    V, B, T = 50, 3, 5
    p = _params(rng, B)
    z = {m: [rng.normal(0, 2, (B, V)).astype(np.float32) for _ in range(T)] for m in (0, 1)}
    both = O.DecodeState(2 * B, 8, V)
    own = {m: O.DecodeState(B, 8, V) for m in (0, 1)}
    for t in range(T):
        for m in (0, 1):
            slots = [m * B + i for i in range(B)]
            x = O.sample_state(z[m][t], p, both, slots, 4, 0, 0, row_ids=np.array(slots))
            y = O.sample_state(z[m][t], p, own[m], [0, 1, 2], 4, both.tick - 1 - own[m].tick, 0, row_ids=np.array(slots))
            assert [r.token for r in x] == [r.token for r in y]
    for m in (0, 1):
        for i in range(B):
            assert both.history(m * B + i).tolist() == own[m].history(i).tolist()


def test_shards_are_vocabulary_ranges_in_rank_order():
    # two pieces of two ids each: the largest logit sits in piece 1, column 0 -> vocabulary id 2;
    # a history token 3 is column 1 of piece 1
    pieces = [np.array([[0.0, 5.0]], np.float32), np.array([[9.0, 8.5]], np.float32)]
    greedy = {"temperature": np.zeros(1, np.float32)}
    assert O.sample_sharded(pieces, greedy, None, None, 0, 0, 0)[0].token == 2
    pen = dict(greedy, presence_penalty=np.full(1, 1.0, np.float32))
    r = O.sample_sharded(pieces, pen, np.array([0, 1]), np.array([2], np.int32), 0, 0, 3)[0]
    assert r.token == 3 and r.top_ids.tolist() == [3, 2, 1]          # 9 - 1 = 8 < 8.5
    whole = O.sample_batch(np.array([[0.0, 5.0, 9.0, 8.5]], np.float32), pen, np.array([0, 1]),
                           np.array([2], np.int32), 0, 0, 3)[0]
    assert whole.token == r.token and whole.logprob == r.logprob
