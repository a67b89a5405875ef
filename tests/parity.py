"""Parity protocol between the HIP path and the CPU oracle (test infrastructure).

Integer results are compared exactly wherever the fp64 oracle says the answer is
separable from its neighbours, and by admissible-set membership inside a guard band:

  scores      |s_gpu - s_orc| <= e := SCORE_TOL * sum_d |a_d b_d| + 1e-6.  A 128-term fp32
              dot product of exactly representable products has a worst-case error of
              128 * 2^-24 = 7.6e-6 of that sum; the MFMA accumulation measures <= 2.4e-7 of
              it on every workload up to 128K (printed as max_sk_err_over_bound), so 1e-6
              leaves a 4x margin while keeping the near-tie runs below short.
  argsort     (a) perm_gpu == stable_argsort_desc(scores_gpu), bit-exact: checks the sort
                  and its tie-break on the very keys the GPU sorted;
              (b) perm_gpu == perm_orc at every rank outside an oracle near-tie run
                  (adjacent fp64 gap < e_i + e_j, the two scores' error bounds: closer
                  scores can legitimately swap); inside a run the GPU entries must be a
                  permutation of the oracle's.
  stop sets   with the oracle's gain profile on the GPU's own (validated) maps: the GPU
              may stop at tile k only if gain[k] < tau(1+G_STOP) and every earlier gain is
              >= tau(1-G_STOP); it may run on only while gains are >= tau(1-G_STOP).  A
              tile whose decision is the same at tau(1+-G_STOP) is "robust" and is thereby
              compared exactly.
  O           against the oracle replaying the GPU's computed counts:
              max-abs <= 2e-2 and relative MSE <= 1e-4 (bf16 in, fp32 accumulate).
"""
from __future__ import annotations

import numpy as np

from oracle import s2o_oracle as orc
from paper_2602_22575_amd import inputs

SCORE_TOL = 1e-6
G_STOP = 1e-3
O_MAX_ABS = 2e-2
O_REL_MSE = 1e-4


def to_f64(bits):
    return orc.bf16_bits_to_f64(bits)


def score_tol(bound):
    return SCORE_TOL * bound + 1e-6


def run_ids(sorted_scores, sorted_tol):
    """Near-tie run id of every rank of a descending-sorted fp64 score row."""
    gap = sorted_scores[:-1] - sorted_scores[1:]
    return np.concatenate([[0], np.cumsum(gap >= sorted_tol[:-1] + sorted_tol[1:])])


def check_perm_against_oracle(perm_gpu, perm_orc, s_orc, tol):
    """Returns (mismatching ranks, near-tie runs of length > 1); raises if the GPU order
    differs from the oracle's outside a near-tie run."""
    perm_gpu = np.asarray(perm_gpu, dtype=np.int64)
    perm_orc = np.asarray(perm_orc, dtype=np.int64)
    diff = np.nonzero(perm_gpu != perm_orc)[0]
    rid = run_ids(s_orc[perm_orc], tol[perm_orc])
    nruns = int((np.bincount(rid) > 1).sum())
    if diff.size:
        a = perm_gpu[np.lexsort((perm_gpu, rid))]
        b = perm_orc[np.lexsort((perm_orc, rid))]
        assert np.array_equal(a, b), (
            f"order differs from the oracle outside a near-tie run at ranks {diff[:8]}")
    return int(diff.size), nruns


def check_plan(w, Qb, Kb, plan_gpu, heads=None, exact=False, segments=None, causal=True):
    """plan_gpu: dict of numpy arrays (q_perm, kv_perm, s_q, s_k, q_mean, k_guide) from
    the HIP path.  The oracle is run head by head (one query head + its KV head at a time).
    causal=False: the non-causal setting (every row ranks all L tokens).
    Returns a stats dict."""
    S, N, L = w.S, w.N, w.L
    stats = dict(q_mismatch=0, q_runs=0, kv_mismatch=0, kv_runs=0, rows=0, max_sk_err_over_bound=0.0)
    for z in range(w.Z):
        for h in (range(w.H) if heads is None else heads):
            g = h // w.G
            Q = to_f64(Qb[z:z + 1, h:h + 1])
            K = to_f64(Kb[z:z + 1, g:g + 1])
            ref = orc.plan(Q, K, S, causal=causal)
            np.testing.assert_allclose(plan_gpu["k_guide"][z, g], ref["k_guide"][0, 0], rtol=0,
                                       atol=2e-6 * np.abs(K).max())
            np.testing.assert_allclose(plan_gpu["q_mean"][z, h], ref["q_mean"][0, 0], rtol=0,
                                       atol=2e-6 * np.abs(Q).max())
            for n in (range(N) if segments is None else segments):
                # s_Q and Q_perm
                sq_g = plan_gpu["s_q"][z, h, n]
                sq_o = ref["s_q"][0, 0, n]
                bound = np.abs(Q[0, 0, n * S:(n + 1) * S]) @ np.abs(ref["k_guide"][0, 0])
                assert np.all(np.abs(sq_g - sq_o) <= score_tol(bound)), \
                    f"s_Q error {np.abs(sq_g - sq_o).max()} (h={h}, n={n})"
                qp = plan_gpu["q_perm"][z, h, n]
                assert np.array_equal(qp, np.argsort(-sq_g, kind="stable")), "Q_perm is not the stable argsort of s_Q"
                mm, runs = check_perm_against_oracle(qp, ref["q_perm"][0, 0, n], sq_o, score_tol(bound))
                stats["q_mismatch"] += mm
                stats["q_runs"] += runs
                ln = orc.kv_row_len(n, S, L, causal)
                if ln == 0:
                    continue
                o = orc.kv_row_start(n, S, L, causal)
                sk_g = plan_gpu["s_k"][z, h, o:o + ln]
                sk_o = ref["s_k"][0, 0, o:o + ln]
                bound = np.abs(K[0, 0, :ln]) @ np.abs(ref["q_mean"][0, 0, n])
                err = np.abs(sk_g - sk_o)
                stats["max_sk_err_over_bound"] = max(stats["max_sk_err_over_bound"], float((err / bound).max()))
                assert np.all(err <= score_tol(bound)), f"s_K error {err.max()} (h={h}, n={n})"
                kp = plan_gpu["kv_perm"][z, h, o:o + ln]
                assert np.array_equal(kp, np.argsort(-sk_g, kind="stable")), \
                    f"KV_perm is not the stable argsort of s_K (h={h}, n={n})"
                mm, runs = check_perm_against_oracle(kp, ref["kv_perm"][0, 0, o:o + ln], sk_o,
                                                     score_tol(bound))
                stats["kv_mismatch"] += mm
                stats["kv_runs"] += runs
                stats["rows"] += 1
    if exact:
        assert stats["kv_mismatch"] == 0 and stats["q_mismatch"] == 0, stats
    return stats


def check_counts(gain_row, tau, stop_mode, computed, skipped):
    """Admissibility of one tile's (computed, skipped) given the oracle gain row.
    Returns True if the decision was robust (same at both ends of the guard band)."""
    nK = gain_row.size
    lo_c = orc.counts_from_gain(gain_row, tau * (1 + G_STOP), stop_mode)
    hi_c = orc.counts_from_gain(gain_row, tau * (1 - G_STOP), stop_mode)
    if lo_c == hi_c:
        assert (computed, skipped) == lo_c, f"counts {(computed, skipped)} != oracle {lo_c} (robust tile)"
        return True
    issued = nK - skipped
    assert 0 <= computed <= issued <= nK
    stopped = (nK - computed - skipped == 1) if stop_mode == 0 else (skipped > 0)
    if stop_mode == 0:
        assert computed + skipped in (nK, nK - 1)
    else:
        assert computed + skipped == nK
    if stopped:
        k = issued - 1
        assert gain_row[k] < tau * (1 + G_STOP) and np.all(gain_row[:k] >= tau * (1 - G_STOP))
    else:
        upto = nK if stop_mode == 0 else nK - 1
        assert np.all(gain_row[:upto] >= tau * (1 - G_STOP))
    return False


def check_attention(w, Qb, Kb, Vb, q_perm, kv_perm, tau, stop_mode, O_gpu_bits, computed, skipped,
                    heads=None, segments=None, gains=None, use_q_perm=True, max_tiles=0, causal=True):
    """Compares one s2o_attention result with the oracle run on the same maps, one query head
    (with its KV head) at a time.  Returns stats (robust/ambiguous tile counts, max-abs and
    relative MSE of O) and the gain profiles (reusable for another tau).
    max_tiles > 0: the run had a tile budget -- the stop rule is checked on the first
    max_tiles gains of each row and the tiles beyond the budget must be reported skipped.
    stop_mode 2: no stop rule -- every tile inside the budget must be folded in.
    causal=False: the non-causal setting (rows of L keys, no own-segment pass)."""
    S, N, BM, BN = w.S, w.N, w.BM, w.BN
    TJ = S // BM
    hs = list(range(w.H)) if heads is None else list(heads)
    ns = list(range(N)) if segments is None else list(segments)
    gains = {} if gains is None else gains
    robust = ambiguous = 0
    max_abs = num = den = 0.0
    for z in range(w.Z):
        for h in hs:
            g = h // w.G
            Q, K, V = to_f64(Qb[z:z + 1, h:h + 1]), to_f64(Kb[z:z + 1, g:g + 1]), to_f64(Vb[z:z + 1, g:g + 1])
            qp = q_perm[z:z + 1, h:h + 1] if use_q_perm else orc.identity_maps(1, 1, w.L, S)[0]
            kp = kv_perm[z:z + 1, h:h + 1]
            if (z, h) not in gains and stop_mode != 2:
                gains[(z, h)] = orc.gain_profile(Q, K, V, qp, kp, S, BM, BN, stop_mode=stop_mode, segments=ns,
                                                 causal=causal)
            gz = gains.get((z, h))
            for n in ns:
                for j in range(TJ):
                    c = int(computed[z, h, n * TJ + j]); s = int(skipped[z, h, n * TJ + j])
                    nK = orc.kv_row_len(n, S, w.L, causal) // BN
                    if nK == 0:
                        assert (c, s) == (0, 0)
                        continue
                    budget = min(nK, max_tiles) if max_tiles > 0 else nK
                    if stop_mode == 2:
                        assert (c, s) == (budget, nK - budget)
                        robust += 1
                    elif check_counts(gz[(0, 0, n)][j][:budget], tau, stop_mode, c, s - (nK - budget)):
                        robust += 1
                    else:
                        ambiguous += 1
            O_ref, _, _ = orc.attention(Q, K, V, qp, kp, S, BM, BN, tau=0.0, stop_mode=stop_mode,
                                        forced_computed=computed[z:z + 1, h:h + 1], segments=ns, causal=causal)
            O_gpu = to_f64(O_gpu_bits[z, h])
            for n in ns:
                a = O_gpu[n * S:(n + 1) * S]
                b = O_ref[0, 0, n * S:(n + 1) * S]
                max_abs = max(max_abs, float(np.abs(a - b).max()))
                num += float(((a - b) ** 2).sum())
                den += float((b ** 2).sum())
    rel_mse = num / den
    assert max_abs <= O_MAX_ABS, f"O max-abs error {max_abs}"
    assert rel_mse <= O_REL_MSE, f"O relative MSE {rel_mse}"
    return dict(robust=robust, ambiguous=ambiguous, max_abs=max_abs, rel_mse=rel_mse, gains=gains)


def pick_tau(gains, nominal, margin=5 * G_STOP):
    """Nearest threshold >= nominal that no evaluated gain comes within `margin` (relative)
    of, so that every stop decision is robust and counts can be compared exactly."""
    flat = []
    for g in gains.values():
        flat.extend(g.values() if isinstance(g, dict) else [g])
    allg = np.concatenate([g[np.isfinite(g)].ravel() for g in flat if g.size])
    tau = nominal
    for _ in range(1000):
        if not np.any(np.abs(allg / tau - 1.0) <= margin):
            return tau
        tau *= 1.0 + 2 * margin
    raise AssertionError("no robust threshold found")


def _close_rows(s, tol):
    """One row of every adjacent pair closer than twice the near-tie gap (the one with the
    larger index, so that early rows, which feed the pooled vectors, move least)."""
    order = np.argsort(-s, kind="stable")
    ss, tt = s[order], tol[order]
    close = np.nonzero((ss[:-1] - ss[1:]) < 2.0 * (tt[:-1] + tt[1:]))[0]
    return {int(max(order[i], order[i + 1])) for i in close}


def untie(w, Qb, Kb, max_rounds=60):
    """Re-draws query rows, then key rows (in place) until no two ranking scores of any
    segment row lie within twice the near-tie gap; feasible for small workloads only.
    Returns the number of rounds used."""
    for rnd in range(max_rounds):
        Q, K = to_f64(Qb), to_f64(Kb)
        q_mean = Q.reshape(w.Z, w.H, w.N, w.S, w.D).mean(axis=3)
        k_guide = K[:, :, :w.S].mean(axis=2)
        bad_q, bad_k = {}, {}
        for z in range(w.Z):
            for h in range(w.H):
                gk = h // w.G
                for n in range(w.N):
                    seg = Q[z, h, n * w.S:(n + 1) * w.S]
                    rows = _close_rows(seg @ k_guide[z, gk], score_tol(np.abs(seg) @ np.abs(k_guide[z, gk])))
                    bad_q.setdefault((z, h), set()).update(n * w.S + r for r in rows)
        if any(bad_q.values()):          # query scores first: they move q_mean and so every s_K
            for (z, h), rows in bad_q.items():
                inputs.redraw_rows(w, Qb, "q", z, h, rows, rnd, pooled=w.S)
            continue
        for z in range(w.Z):
            for h in range(w.H):
                gk = h // w.G
                for n in range(1, w.N):
                    kp = K[z, gk, :n * w.S]
                    bad_k.setdefault((z, gk), set()).update(
                        _close_rows(kp @ q_mean[z, h, n], score_tol(np.abs(kp) @ np.abs(q_mean[z, h, n]))))
        if not any(bad_k.values()):
            return rnd
        for (z, gk), rows in bad_k.items():
            inputs.redraw_rows(w, Kb, "k", z, gk, rows, rnd, pooled=w.S)
    raise AssertionError("could not remove near-ties")
