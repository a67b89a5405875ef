"""Pins for the CPU oracle: each test checks oracle/s2o_oracle.py against something that
is not the oracle itself -- a closed form, a textbook routine, brute force in pure Python
on tiny inputs, an invariant of the mathematics, or a number the paper prints."""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import s2o_oracle as orc

RNG = np.random.default_rng(1234)


def rand_qkv(Z, H, Hkv, L, D, rng=RNG, scale=1.0):
    return (rng.standard_normal((Z, H, L, D)) * scale,
            rng.standard_normal((Z, Hkv, L, D)) * scale,
            rng.standard_normal((Z, Hkv, L, D)))


# ---------------------------------------------------------------- pure-Python literal model
def py_dense(q, k, v, scale):
    """Triple-loop causal softmax attention on lists (one head)."""
    L, D = len(q), len(q[0])
    out = []
    for i in range(L):
        w = [math.exp(scale * sum(q[i][d] * k[j][d] for d in range(D))) for j in range(i + 1)]
        tot = sum(w)
        out.append([sum(w[j] * v[j][d] for j in range(i + 1)) / tot for d in range(D)])
    return out


def py_s2o(q, k, v, S, BM, BN, tau, stop_mode, scale):
    """Literal model of the two steps on an explicit L x L weight matrix, one head,
    pure Python: ranking by pooled scores with (score desc, index asc) order, then per
    permuted query tile a walk over the ranked prefix in tiles of BN keys where the tile
    is dropped / kept-then-stop when every row's (tile weight / weight so far) < tau."""
    L, D = len(q), len(q[0])
    N = L // S
    dot = lambda a, b: sum(x * y for x, y in zip(a, b))
    W = [[math.exp(scale * dot(q[i], k[j])) if j <= i else 0.0 for j in range(L)] for i in range(L)]
    kguide = [sum(k[s][d] for s in range(S)) / S for d in range(D)]
    out = [None] * L
    counts = []
    maps = []
    for n in range(N):
        qmean = [sum(q[n * S + s][d] for s in range(S)) / S for d in range(D)]
        sq = [dot(q[n * S + s], kguide) for s in range(S)]
        qperm = sorted(range(S), key=lambda s: (-sq[s], s))
        sk = [dot(qmean, k[t]) for t in range(n * S)]
        kvperm = sorted(range(n * S), key=lambda t: (-sk[t], t))
        maps.append((qperm, kvperm))
        for j in range(S // BM):
            rows = [n * S + qperm[j * BM + i] for i in range(BM)]
            visited = {i: list(range(n * S, i + 1)) for i in rows}
            nK = n * S // BN
            issued = folded = 0
            for kt in range(nK):
                T = kvperm[kt * BN:(kt + 1) * BN]
                gains = [sum(W[i][t] for t in T) / sum(W[i][t] for t in visited[i]) for i in rows]
                stop = max(gains) < tau
                issued += 1
                if stop and stop_mode == 0:
                    break
                for i in rows:
                    visited[i] = visited[i] + T
                folded += 1
                if stop:
                    break
            counts.append((folded, nK - issued))
            for i in rows:
                tot = sum(W[i][t] for t in visited[i])
                out[i] = [sum(W[i][t] * v[t][d] for t in visited[i]) / tot for d in range(D)]
    return out, counts, maps


# ---------------------------------------------------------------- dense reference pins
def test_dense_matches_scipy_softmax_and_python_loops():
    Q, K, V = rand_qkv(1, 2, 1, 24, 4)
    O = orc.dense_attention(Q, K, V)
    scale = 1 / math.sqrt(4)
    for h in range(2):
        x = scale * Q[0, h] @ K[0, 0].T
        x[np.triu_indices(24, 1)] = -np.inf
        np.testing.assert_allclose(O[0, h], scipy_softmax(x, axis=1) @ V[0, 0], atol=1e-13)
        ref = py_dense(Q[0, h].tolist(), K[0, 0].tolist(), V[0, 0].tolist(), scale)
        np.testing.assert_allclose(O[0, h], np.array(ref), atol=1e-13)


def test_dense_closed_forms():
    # all-zero queries: uniform weights -> O[i] = prefix mean of V
    Q, K, V = rand_qkv(1, 1, 1, 16, 3)
    O = orc.dense_attention(np.zeros_like(Q), K, V)
    pm = np.cumsum(V[0, 0], axis=0) / np.arange(1, 17)[:, None]
    np.testing.assert_allclose(O[0, 0], pm, atol=1e-14)
    # first row attends only to itself
    O = orc.dense_attention(Q, K, V)
    np.testing.assert_allclose(O[0, 0, 0], V[0, 0, 0], atol=1e-14)
    # GQA: head h reads KV head h // G
    Q, K, V = rand_qkv(1, 4, 2, 8, 2)
    O = orc.dense_attention(Q, K, V)
    O3 = orc.dense_attention(Q[:, 3:4], K[:, 1:2], V[:, 1:2])
    np.testing.assert_allclose(O[0, 3], O3[0, 0], atol=1e-14)
    # row subset
    np.testing.assert_allclose(orc.dense_attention(Q, K, V, rows=[5, 2])[0, 1], O[0, 1, [5, 2]], atol=1e-14)


# ---------------------------------------------------------------- plan pins (Alg. 1)
def test_plan_against_python_loops_and_gqa():
    Z, H, Hkv, L, D, S = 1, 4, 2, 32, 3, 8
    Q, K, V = rand_qkv(Z, H, Hkv, L, D)
    p = orc.plan(Q, K, S)
    for h in range(H):
        g = h // 2
        _, _, maps = py_s2o(Q[0, h].tolist(), K[0, g].tolist(), V[0, g].tolist(), S, 4, 4, 0.0, 0, 1.0)
        for n in range(L // S):
            assert p["q_perm"][0, h, n].tolist() == maps[n][0]
            o = orc.kv_row_offset(n, S)
            assert p["kv_perm"][0, h, o:o + n * S].tolist() == maps[n][1]
    # explicit values of the pooled quantities
    np.testing.assert_allclose(p["k_guide"][0, 1], K[0, 1, :S].sum(0) / S, atol=1e-14)
    np.testing.assert_allclose(p["q_mean"][0, 3, 2], Q[0, 3, 16:24].sum(0) / S, atol=1e-14)
    np.testing.assert_allclose(p["s_q"][0, 3, 2, 5], Q[0, 3, 21] @ p["k_guide"][0, 1], atol=1e-13)
    o = orc.kv_row_offset(3, S)
    np.testing.assert_allclose(p["s_k"][0, 2, o + 7], p["q_mean"][0, 2, 3] @ K[0, 1, 7], atol=1e-13)


def test_plan_maps_are_sorted_permutations_with_stable_ties():
    Z, H, Hkv, L, D, S = 1, 2, 1, 64, 2, 16
    # small integer alphabet -> many exact ties
    Q = RNG.integers(-1, 2, size=(Z, H, L, D)).astype(float)
    K = RNG.integers(-1, 2, size=(Z, Hkv, L, D)).astype(float)
    p = orc.plan(Q, K, S)
    for h in range(H):
        for n in range(L // S):
            qp = p["q_perm"][0, h, n]
            assert sorted(qp.tolist()) == list(range(S))
            s = p["s_q"][0, h, n]
            assert qp.tolist() == sorted(range(S), key=lambda i: (-s[i], i))
            o = orc.kv_row_offset(n, S)
            kp = p["kv_perm"][0, h, o:o + n * S]
            sk = p["s_k"][0, h, o:o + n * S]
            assert sorted(kp.tolist()) == list(range(n * S))
            assert np.all(np.diff(sk[kp]) <= 0)
            assert kp.tolist() == np.lexsort((np.arange(n * S), -sk)).tolist()
    # -0.0 and +0.0 tie
    assert orc.stable_argsort_desc(np.array([0.0, -0.0, 1.0, -0.0])).tolist() == [2, 0, 1, 3]


def test_packed_row_offsets():
    S = 8
    off = 0
    for n in range(1, 9):
        assert orc.kv_row_offset(n, S) == off
        off += n * S
    assert orc.kv_row_offset(1, S) == 0


# ---------------------------------------------------------------- attention pins
@pytest.mark.parametrize("BM,BN", [(4, 4), (8, 4)])
def test_tau_zero_equals_dense_any_maps(BM, BN):
    """No-skip mode performs the same computation as dense attention (paper App. A:
    variants run with threshold -1 are dense-equivalent)."""
    Z, H, Hkv, L, D, S = 1, 2, 1, 64, 8, 16
    Q, K, V = rand_qkv(Z, H, Hkv, L, D)
    dense = orc.dense_attention(Q, K, V)
    p = orc.plan(Q, K, S)
    for tau in (0.0, -1.0):
        O, comp, skip = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, tau)
        np.testing.assert_allclose(O, dense, atol=1e-12)
        for n in range(L // S):
            assert np.all(comp[:, :, n * (S // BM):(n + 1) * (S // BM)] == n * S // BN)
        assert np.all(skip == 0)
    qi, ki = orc.identity_maps(Z, H, L, S)
    np.testing.assert_allclose(orc.attention(Q, K, V, qi, ki, S, BM, BN, 0.0)[0], dense, atol=1e-12)


def test_visit_order_invariance():
    Z, H, Hkv, L, D, S = 1, 1, 1, 64, 8, 16
    Q, K, V = rand_qkv(Z, H, Hkv, L, D)
    dense = orc.dense_attention(Q, K, V)
    qi, ki = orc.identity_maps(Z, H, L, S)
    for n in range(L // S):
        qi[0, 0, n] = RNG.permutation(S)
        o = orc.kv_row_offset(n, S)
        ki[0, 0, o:o + n * S] = RNG.permutation(n * S)
    O, _, _ = orc.attention(Q, K, V, qi, ki, S, 4, 4, 0.0)
    np.testing.assert_allclose(O, dense, atol=1e-12)


@pytest.mark.parametrize("stop_mode", [0, 1])
def test_streaming_equals_visited_set_form(stop_mode):
    Z, H, Hkv, L, D, S = 1, 2, 1, 96, 8, 16
    Q, K, V = rand_qkv(Z, H, Hkv, L, D, scale=1.5)
    p = orc.plan(Q, K, S)
    hit = 0
    for tau in (0.0, 0.02, 0.08, 0.3, 5.0):
        O, comp, skip = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, 8, 4, tau, stop_mode)
        O2, comp2, skip2 = orc.attention_visited_set(Q, K, V, p["q_perm"], p["kv_perm"], S, 8, 4, tau, stop_mode)
        assert np.array_equal(comp, comp2) and np.array_equal(skip, skip2)
        np.testing.assert_allclose(O, O2, atol=1e-12)
        total = orc.prefix_tiles(L, S, 8, 4)
        assert np.all((total - comp - skip >= 0) & (total - comp - skip <= (1 - stop_mode)))
        hit += int((skip > 0).any())
    assert hit >= 2        # the stop rule actually fired in this test


def test_stop_rule_uses_new_scale_when_max_rises():
    """A prefix tile that raises the running maximum has a large gain and must not stop:
    one key aligned with the query dominates everything seen so far."""
    L, S, D = 8, 4, 2
    Q = np.zeros((1, 1, L, D)); K = np.zeros((1, 1, L, D)); V = RNG.standard_normal((1, 1, L, D))
    Q[0, 0, :, 0] = 1.0
    K[0, 0, 1, 0] = 30.0                       # a prefix key with a huge logit
    qi, ki = orc.identity_maps(1, 1, L, S)
    O, comp, _ = orc.attention(Q, K, V, qi, ki, S, 2, 2, tau=0.5, scale=1.0)
    assert comp[0, 0, 2:].tolist() == [1, 1]   # tile 0 (keys 0,1) kept; tile 1 triggers
    assert _[0, 0, 2:].tolist() == [0, 0]
    np.testing.assert_allclose(O[0, 0, 4:], np.broadcast_to(V[0, 0, 1], (4, D)), atol=1e-9)


def test_stop_modes_differ_only_by_the_triggering_tile():
    Z, H, Hkv, L, D, S = 1, 1, 1, 64, 8, 16
    Q, K, V = rand_qkv(Z, H, Hkv, L, D, scale=1.5)
    p = orc.plan(Q, K, S)
    tau = 0.1
    _, c0, s0 = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, 4, 4, tau, 0)
    _, c1, s1 = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, 4, 4, tau, 1)
    assert np.array_equal(s0, s1)              # same decision sequence up to the stop
    trig = orc.prefix_tiles(L, S, 4, 4) - c0 - s0
    assert np.array_equal(c1, c0 + trig) and trig.max() == 1 and trig.min() == 0


def test_exhaustive_tiny_cases_against_literal_model():
    """L in {8}, S=4, tiles 2x2, D=1..2, inputs from a 3-value alphabet: every tie pattern
    the sort and the stop rule can meet, compared with the pure-Python literal model."""
    scale = 0.7
    checked = 0
    rng = np.random.default_rng(7)
    for D in (1, 2):
        for L in (8, 16):
            cases = (itertools.product((-1.0, 0.0, 1.0), repeat=6) if (D == 1 and L == 8)
                     else [None] * 40)
            for case in cases:
                if case is None:
                    q = rng.integers(-1, 2, size=(L, D)).astype(float)
                    k = rng.integers(-1, 2, size=(L, D)).astype(float)
                else:   # 3 free query values + 3 free key values, tiled over the sequence
                    q = np.array([case[i % 3] for i in range(L)], float).reshape(L, D)
                    k = np.array([case[3 + (i * 2) % 3] for i in range(L)], float).reshape(L, D)
                v = rng.standard_normal((L, D))
                Q, K, V = q[None, None], k[None, None], v[None, None]
                p = orc.plan(Q, K, 4)
                for tau in (0.0, 0.2, 0.45, 1.0):
                    for mode in (0, 1):
                        O, comp, skip = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], 4, 2, 2,
                                                      tau, mode, scale=scale)
                        ref, counts, _ = py_s2o(q.tolist(), k.tolist(), v.tolist(), 4, 2, 2,
                                                tau, mode, scale)
                        assert list(zip(comp[0, 0].tolist(), skip[0, 0].tolist())) == counts
                        np.testing.assert_allclose(O[0, 0], np.array(ref), atol=1e-12)
                        checked += 1
    assert checked > 5000


def test_tile_budget_is_masked_softmax_over_the_first_k_ranked_tiles():
    """Fixed budget with no stop rule (top-k selection on the ranked order): the output is
    plain softmax attention under an explicit L x L mask -- own-segment causal keys plus the
    first k*B_N entries of the segment's ranked row -- built here without the oracle."""
    Z, H, Hkv, L, D, S, BM, BN = 1, 2, 1, 96, 8, 16, 8, 4
    Q, K, V = rand_qkv(Z, H, Hkv, L, D, scale=1.3)
    p = orc.plan(Q, K, S)
    scale = 1.0 / math.sqrt(D)
    for k in (0, 1, 3, 7, 1000):
        O, comp, skip = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, tau=0.5, stop_mode=2,
                                      max_tiles=k)
        for h in range(H):
            x = scale * (Q[0, h] @ K[0, 0].T)
            allow = np.zeros((L, L), dtype=bool)
            for n in range(L // S):
                rows = slice(n * S, (n + 1) * S)
                own = np.tril(np.ones((S, S), dtype=bool))
                allow[rows, n * S:(n + 1) * S] = own
                row = p["kv_perm"][0, h, orc.kv_row_offset(n, S):orc.kv_row_offset(n, S) + n * S]
                allow[rows, row[:min(k, n * S // BN) * BN]] = True
            w = scipy_softmax(np.where(allow, x, -np.inf), axis=1)
            np.testing.assert_allclose(O[0, h], w @ V[0, 0], atol=1e-12)
        nK = orc.prefix_tiles(L, S, BM, BN)
        assert np.array_equal(comp[0, 0], np.minimum(nK, k)) and np.array_equal(skip[0, 0], nK - np.minimum(nK, k))
    # a budget that is never reached changes nothing; a stop inside the budget is the usual stop
    for stop_mode in (0, 1):
        ref = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, 0.05, stop_mode)
        big = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, 0.05, stop_mode, max_tiles=10 ** 6)
        for a, b in zip(ref, big):
            assert np.array_equal(a, b)
        cut = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, 0.05, stop_mode, max_tiles=2)
        nK = orc.prefix_tiles(L, S, BM, BN)
        issued_ref, issued_cut = nK - ref[2][0], nK - cut[2][0]
        assert np.array_equal(issued_cut, np.minimum(issued_ref, 2))
        assert np.array_equal(cut[1][0], np.minimum(ref[1][0], 2))
    # stop_mode 2 without a budget is dense attention whatever tau says
    O, comp, skip = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, tau=10.0, stop_mode=2)
    np.testing.assert_allclose(O, orc.dense_attention(Q, K, V), atol=1e-12)
    assert np.all(skip == 0)


def test_monotone_in_tau():
    Z, H, Hkv, L, D, S = 1, 2, 1, 96, 8, 16
    Q, K, V = rand_qkv(Z, H, Hkv, L, D, scale=1.5)
    p = orc.plan(Q, K, S)
    prev = None
    for tau in (0.0, 0.01, 0.05, 0.1, 0.3, 1.0, 1e12):
        _, comp, skip = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, 4, 4, tau)
        if prev is not None:
            assert np.all(comp <= prev[0]) and np.all(skip >= prev[1])
        prev = (comp, skip)
        d = orc.density(skip, L, S, 4, 4)
        assert np.all((d > 0) & (d <= 1))
    assert np.all(prev[0] == 0)                 # tau huge: the first prefix tile triggers
    assert np.array_equal(prev[1][0, 0], np.maximum(orc.prefix_tiles(L, S, 4, 4) - 1, 0))
    _, comp, skip = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, 4, 4, 0.0)
    assert np.all(orc.density(skip, L, S, 4, 4) == 1.0)


def test_gain_profile_predicts_counts_for_every_tau():
    Z, H, Hkv, L, D, S = 1, 1, 1, 64, 8, 16
    Q, K, V = rand_qkv(Z, H, Hkv, L, D, scale=1.5)
    p = orc.plan(Q, K, S)
    for mode in (0, 1):
        gains = orc.gain_profile(Q, K, V, p["q_perm"], p["kv_perm"], S, 4, 4, stop_mode=mode)
        for tau in (0.0, 0.03, 0.1, 0.4):
            _, comp, skip = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, 4, 4, tau, mode)
            for n in range(1, L // S):
                for j in range(S // 4):
                    assert (comp[0, 0, n * 4 + j], skip[0, 0, n * 4 + j]) == \
                        orc.counts_from_gain(gains[(0, 0, n)][j], tau, mode)


def test_replay_reproduces_streaming_run():
    Z, H, Hkv, L, D, S = 1, 2, 2, 64, 8, 16
    Q, K, V = rand_qkv(Z, H, Hkv, L, D, scale=1.5)
    p = orc.plan(Q, K, S)
    for mode in (0, 1):
        O, comp, skip = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, 4, 4, 0.1, mode)
        assert (skip > 0).any()
        O2, comp2, _ = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, 4, 4, 123.0, mode,
                                     forced_computed=comp)
        assert np.array_equal(comp, comp2)
        np.testing.assert_array_equal(O, O2)


def test_two_pass_with_identity_queries_equals_fused_single_pass():
    """Alg. 2 + Alg. 3 with Q_perm = identity is the fused Alg. 4 (paper App. C.3)."""
    Z, H, Hkv, L, D, S = 1, 2, 1, 64, 8, 16
    Q, K, V = rand_qkv(Z, H, Hkv, L, D, scale=1.5)
    p = orc.plan(Q, K, S)
    qi, _ = orc.identity_maps(Z, H, L, S)
    for tau in (0.0, 0.1):
        O, _, _ = orc.attention(Q, K, V, qi, p["kv_perm"], S, 4, 4, tau)
        np.testing.assert_allclose(O, orc.attention_fused_noqperm(Q, K, V, p["kv_perm"], S, 4, 4, tau),
                                   atol=1e-12)


def test_local_window_only_sparsity_matches_paper_table3():
    path = os.path.join(os.path.dirname(__file__), "golden", "table3_local_window_sparsity.txt")
    L, S, B, printed = [ln.split() for ln in open(path) if not ln.startswith("#")][0]
    L, S, B = int(L), int(S), int(B)
    sparsity = 1 - orc.pass1_tiles(L, S, B) / orc.causal_tiles(L, B)
    assert abs(sparsity - (1 - 8704 / 524800)) < 1e-15
    assert f"{sparsity:.3f}" == printed
    # the density helper agrees when no prefix tile is issued
    skip = orc.prefix_tiles(L, S, B, B)[None, None]
    assert abs(1 - orc.density(skip, L, S, B, B)[0, 0] - sparsity) < 1e-15


def _brute_blocks(L, S, BM, BN):
    """Brute force on the explicit L x L causal mask: B_M x B_N score blocks that hold at least
    one causal element (key <= query), split into blocks of the query's own segment and blocks
    of earlier segments (the prefix), per query block."""
    i, j = np.arange(L)[:, None], np.arange(L)[None, :]
    mask = j <= i
    own = np.zeros(L // BM, dtype=np.int64)
    pre = np.zeros(L // BM, dtype=np.int64)
    for b in range(L // BM):
        for t in range(L // BN):
            if mask[b * BM:(b + 1) * BM, t * BN:(t + 1) * BN].any():
                if (t * BN) // S == (b * BM) // S:
                    own[b] += 1
                else:
                    pre[b] += 1
    return own, pre


@pytest.mark.parametrize("L,S,BM,BN", [(64, 16, 8, 4), (96, 32, 16, 4), (512, 256, 128, 64), (1024, 256, 128, 64),
                                       (64, 16, 4, 4)])
def test_density_for_unequal_tile_shapes_matches_brute_force_block_count(L, S, BM, BN):
    """density() in units of B_M x B_N score blocks when B_M != B_N (the 128x64 tiling):
    every block that contains a causal element counts whole; checked against a count on the
    explicit mask, with nothing skipped, everything skipped and random skip counts."""
    own, pre = _brute_blocks(L, S, BM, BN)
    assert np.array_equal(pre, orc.prefix_tiles(L, S, BM, BN))
    total = own.sum() + pre.sum()
    rng = np.random.default_rng(L + BM)
    zero = np.zeros((1, 2, L // BM), dtype=np.int64)
    assert np.all(orc.density(zero, L, S, BM, BN) == 1.0)
    allskip = np.broadcast_to(pre, zero.shape)
    np.testing.assert_allclose(orc.density(allskip, L, S, BM, BN), own.sum() / total, rtol=0, atol=1e-15)
    for _ in range(5):
        skip = rng.integers(0, pre + 1, size=zero.shape)
        want = (own.sum() + (pre[None, None] - skip).sum(axis=-1)) / total
        np.testing.assert_allclose(orc.density(skip, L, S, BM, BN), want, rtol=0, atol=1e-15)
    if BM == BN:
        assert own.sum() == orc.pass1_tiles(L, S, BM) and total == orc.causal_tiles(L, BM)


def test_bf16_conversions_roundtrip():
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    vals = orc.bf16_bits_to_f64(bits)
    finite = np.isfinite(vals)
    assert np.array_equal(orc.f64_to_bf16_bits(vals[finite]), bits[finite])
    assert orc.bf16_bits_to_f64(np.array([0x3F80, 0xC000, 0x3DCD], dtype=np.uint16)).tolist() == \
        [1.0, -2.0, 0.10009765625]
    # ties round to even mantissa
    assert orc.f64_to_bf16_bits(np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8])).tolist() == [0x3F80, 0x3F82]


# ---------------------------------------------------------------- non-causal setting
def py_s2o_noncausal(q, k, v, S, BM, BN, tau, stop_mode, max_tiles, scale):
    """Literal model of the non-causal reading, one head, pure Python lists: every segment
    ranks all L keys by <segment mean of q, k> (score desc, index asc); a permuted query
    tile walks that list in tiles of BN keys from nothing, the first tile is always kept,
    a later tile triggers when every row's (tile weight / weight so far) < tau."""
    L, D = len(q), len(q[0])
    N = L // S
    dot = lambda a, b: sum(x * y for x, y in zip(a, b))
    W = [[math.exp(scale * dot(q[i], k[j])) for j in range(L)] for i in range(L)]
    kguide = [sum(k[s][d] for s in range(S)) / S for d in range(D)]
    out = [None] * L
    counts, rows_of_maps = [], []
    for n in range(N):
        qmean = [sum(q[n * S + s][d] for s in range(S)) / S for d in range(D)]
        sq = [dot(q[n * S + s], kguide) for s in range(S)]
        qperm = sorted(range(S), key=lambda s: (-sq[s], s))
        sk = [dot(qmean, k[t]) for t in range(L)]
        kvperm = sorted(range(L), key=lambda t: (-sk[t], t))
        rows_of_maps.append((qperm, kvperm))
        for j in range(S // BM):
            rows = [n * S + qperm[j * BM + i] for i in range(BM)]
            visited = []
            nK = L // BN
            budget = nK if max_tiles is None else min(nK, max_tiles)
            issued = folded = 0
            for kt in range(budget):
                T = kvperm[kt * BN:(kt + 1) * BN]
                issued += 1
                trig = False
                if visited and stop_mode != 2:
                    trig = all(sum(W[i][t] for t in T) / sum(W[i][t] for t in visited) < tau for i in rows)
                if trig and stop_mode == 0:
                    break
                visited = visited + T
                folded += 1
                if trig:
                    break
            for i in rows:
                tot = sum(W[i][t] for t in visited)
                out[i] = [sum(W[i][t] * v[t][d] for t in visited) / tot for d in range(D)]
            counts.append((folded, nK - issued))
    return out, counts, rows_of_maps


def test_noncausal_dense_matches_torch_sdpa_and_tau_zero_walk():
    """causal=False: the dense reference equals a library attention routine, and the ranked
    walk with tau <= 0 (any maps) equals it."""
    import torch
    Q, K, V = rand_qkv(1, 4, 2, 32, 8)
    ref = orc.dense_attention(Q, K, V, causal=False)
    G = 2
    tq, tk, tv = (torch.from_numpy(x) for x in (Q, np.repeat(K, G, axis=1), np.repeat(V, G, axis=1)))
    lib = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=False).numpy()
    np.testing.assert_allclose(ref, lib, rtol=0, atol=1e-12)
    causal_lib = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).numpy()
    np.testing.assert_allclose(orc.dense_attention(Q, K, V), causal_lib, rtol=0, atol=1e-12)
    assert np.abs(ref - causal_lib).max() > 1e-3          # the flag does something
    S, BM, BN = 8, 4, 4
    p = orc.plan(Q, K, S, causal=False)
    assert p["kv_perm"].shape == (1, 4, (32 // S) * 32)
    for tau in (0.0, -1.0):
        O, c, s = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, tau, causal=False)
        np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)
        assert (c == 32 // BN).all() and (s == 0).all()
    rng = np.random.default_rng(5)
    kv = p["kv_perm"].copy().reshape(1, 4, 32 // S, 32)
    for h in range(4):
        for n in range(32 // S):
            kv[0, h, n] = rng.permutation(32)
    O2, _, _ = orc.attention(Q, K, V, p["q_perm"], kv.reshape(1, 4, -1), S, BM, BN, 0.0, causal=False)
    np.testing.assert_allclose(O2, ref, rtol=0, atol=1e-12)


def test_noncausal_plan_rows_rank_all_tokens():
    Q, K, _ = rand_qkv(1, 2, 1, 48, 4)
    S, L = 16, 48
    p = orc.plan(Q, K, S, causal=False)
    pc = orc.plan(Q, K, S, causal=True)
    np.testing.assert_array_equal(p["q_perm"], pc["q_perm"])          # the query side is unchanged
    np.testing.assert_allclose(p["q_mean"], pc["q_mean"])
    for h in range(2):
        for n in range(L // S):
            row = p["kv_perm"][0, h, n * L:(n + 1) * L]
            sk = p["s_k"][0, h, n * L:(n + 1) * L]
            assert sorted(row.tolist()) == list(range(L))
            np.testing.assert_allclose(sk, K[0, 0] @ Q[0, h, n * S:(n + 1) * S].mean(axis=0), atol=1e-12)
            assert (np.diff(sk[row]) <= 0).all()
            # restricted to the causal prefix, the order is the causal row's order
            if n:
                o = orc.kv_row_offset(n, S)
                np.testing.assert_array_equal(row[row < n * S], pc["kv_perm"][0, h, o:o + n * S])


@pytest.mark.parametrize("stop_mode,max_tiles", [(0, None), (1, None), (2, 3), (0, 4)])
def test_noncausal_against_literal_model(stop_mode, max_tiles):
    rng = np.random.default_rng(77)
    L, D, S, BM, BN = 16, 2, 8, 4, 2
    for trial in range(6):
        Q = rng.choice([-1.0, 0.0, 1.5], size=(1, 1, L, D))
        K = rng.choice([-1.0, 0.5, 1.0], size=(1, 1, L, D))
        V = rng.standard_normal((1, 1, L, D))
        scale = 0.7
        p = orc.plan(Q, K, S, causal=False)
        for tau in (0.0, 0.05, 0.2, 0.6):
            O, c, s = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, tau, stop_mode=stop_mode,
                                    scale=scale, max_tiles=max_tiles, causal=False)
            ref, counts, maps = py_s2o_noncausal(Q[0, 0].tolist(), K[0, 0].tolist(), V[0, 0].tolist(), S, BM, BN,
                                                 tau, stop_mode, max_tiles, scale)
            for n, (qp, kvp) in enumerate(maps):
                assert p["q_perm"][0, 0, n].tolist() == qp
                assert p["kv_perm"][0, 0, n * L:(n + 1) * L].tolist() == kvp
            np.testing.assert_allclose(O[0, 0], np.array(ref), rtol=0, atol=1e-12)
            assert [(int(a), int(b)) for a, b in zip(c[0, 0], s[0, 0])] == counts


@pytest.mark.parametrize("stop_mode", [0, 1])
def test_noncausal_streaming_equals_visited_set_form(stop_mode):
    Q, K, V = rand_qkv(1, 2, 1, 64, 8, scale=1.5)
    S, BM, BN = 16, 8, 4
    p = orc.plan(Q, K, S, causal=False)
    stopped = 0
    for tau in (0.0, 0.02, 0.1, 0.5):
        a = orc.attention(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, tau, stop_mode=stop_mode, causal=False)
        b = orc.attention_visited_set(Q, K, V, p["q_perm"], p["kv_perm"], S, BM, BN, tau, stop_mode=stop_mode,
                                      causal=False)
        np.testing.assert_allclose(a[0], b[0], rtol=0, atol=1e-11)
        np.testing.assert_array_equal(a[1], b[1])
        np.testing.assert_array_equal(a[2], b[2])
        stopped += int((a[2] > 0).sum())
        assert (a[1] >= 1).all()                       # the first tile is always kept
    assert stopped > 0
