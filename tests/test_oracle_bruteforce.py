"""Brute-force pins for the oracle's filtered distribution and its u -> token map (no GPU).

The oracle sorts and accumulates; the checker here never sorts and never forms a running
sum: it evaluates the set definitions of the three filters element by element in
O(V^2) and the draw by enumerating prefix masses with ``math.fsum``.  Inputs are tiny and
drawn from a small value grid so that ties at every cut are common."""
import itertools
import math

import numpy as np
import pytest

from oracle import sip_oracle as O

f32 = np.float32


def brute_sets(s, e, k, p, min_p):
    """K1, K2, K3 from the definitions: top-k keeps v iff fewer than k tokens are strictly
    larger; top-p keeps v iff the K1-mass of strictly larger tokens is < p * mass(K1);
    min-p keeps v iff fp32(s_v - max) >= fp32(ln min_p)."""
    V = len(s)
    allv = list(range(V))
    if 2 <= k < V:
        K1 = [v for v in allv if sum(1 for w in allv if s[w] > s[v]) < k]
    else:
        K1 = allv
    S1 = math.fsum(e[v] for v in K1)
    if 0.0 < p < 1.0:
        K2 = [v for v in K1 if math.fsum(e[w] for w in K1 if s[w] > s[v]) < float(p) * S1]
    else:
        K2 = K1
    if min_p > 0.0:
        m = max(s)
        t = f32(math.log(float(min_p)))
        K3 = [v for v in K2 if f32(s[v] - m) >= t]
    else:
        K3 = K2
    return K1, K2, K3, S1


def brute_draw(e, K3, u):
    S3 = math.fsum(e[v] for v in K3)
    for v in sorted(K3):
        if math.fsum(e[w] for w in K3 if w <= v) > u * S3:
            return v
    return max(K3)


def scaled(z, tau):
    s = (z / f32(tau)).astype(np.float32)
    m = float(np.max(s))
    e = [math.exp(float(x) - m) for x in s]
    return s, e


GRID = np.array([-3.0, -1.5, -0.5, 0.0, 0.5, 1.0, 1.5, 2.5], dtype=np.float32)


@pytest.mark.parametrize("V", [5, 17, 48])
def test_filter_sets_and_draw_match_brute_force(V):
    rng = np.random.default_rng(1000 + V)
    checked = 0
    for trial in range(40):
        if trial % 2 == 0:
            z = rng.choice(GRID, size=V).astype(np.float32)            # many ties
        else:
            z = (rng.standard_normal(V) * 2).astype(np.float32)
        tau = float(rng.choice([0.25, 0.7, 1.0, 1.9]))
        ks = [0, 2, 3, V // 2, V - 1, V, V + 5]
        ps = [1.0, 0.97, 0.6, 0.3, 0.05]
        mps = [0.0, 0.02, 0.3, 1.0]
        for k, p, mp in itertools.product(ks, ps, mps):
            s, e = scaled(z, tau)
            K1, K2, K3, S1 = brute_sets(s, e, k, f32(p), f32(mp))
            r = O.sample_row(z, temperature=tau, top_k=k, top_p=p, min_p=mp,
                             seed=3, step=trial, row_id=V, keep_arrays=True)
            if r.topp_margin < 1e-12:
                continue                      # a genuine coin flip between two summation orders
            assert sorted(np.flatnonzero(r.kept).tolist()) == sorted(K3), (z, tau, k, p, mp)
            assert math.isclose(r.S1, S1, rel_tol=1e-13)
            if r.draw_margin > 1e-12:
                assert r.token == brute_draw(e, K3, r.u)
            checked += 1
    assert checked > 1000


def test_u_to_token_map_on_a_fine_grid():
    rng = np.random.default_rng(5)
    V = 23
    z = rng.choice(GRID, size=V).astype(np.float32)
    tau, k, p, mp = 0.8, 9, 0.9, 0.05
    s, e = scaled(z, tau)
    _, _, K3, _ = brute_sets(s, e, k, f32(p), f32(mp))
    seen = set()
    for j in range(0, 4096):
        u = j / 4096.0
        r = O.sample_row(z, temperature=tau, top_k=k, top_p=p, min_p=mp, u_override=u)
        if r.draw_margin < 1e-12:
            continue
        assert r.token == brute_draw(e, K3, u)
        seen.add(r.token)
    assert seen == set(K3)                   # every kept token owns an interval of u
    # the map is monotone: larger u never selects a smaller index
    toks = [O.sample_row(z, temperature=tau, top_k=k, top_p=p, min_p=mp, u_override=j / 512.0).token
            for j in range(512)]
    assert toks == sorted(toks)


def test_argmax_is_always_kept_and_sets_are_nested():
    rng = np.random.default_rng(11)
    for _ in range(50):
        V = int(rng.integers(3, 40))
        z = rng.choice(GRID, size=V).astype(np.float32)
        k = int(rng.integers(0, V + 2))
        p = float(rng.uniform(0.01, 1.0))
        mp = float(rng.choice([0.0, 0.1, 0.9, 1.0]))
        r = O.sample_row(z, temperature=0.9, top_k=k, top_p=p, min_p=mp, keep_arrays=True)
        if r.greedy:
            continue
        assert r.kept[int(np.argmax(z))]
        assert r.kept[r.token]
        # value-closed: no dropped token has a value >= a kept token's value
        assert r.s[~r.kept].max(initial=-np.inf) < r.s[r.kept].min()
