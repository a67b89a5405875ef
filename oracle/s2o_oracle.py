"""CPU oracle for S2O causal prefill attention (fp64, numpy).  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain statement of what the hot path computes, written from the
paper.  It shares no code with the HIP path and must never be imported by it: only
tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may call it.

What follows what:
  dense_attention        definition of causal softmax attention (the "Full" reference of
                         Sec. 4.1); brute force, a max-shifted softmax per row.
  plan                   Alg. 1 / Sec. 3.1, Eqs. (1)-(2): segment means, guide vector,
                         query scores + intra-segment Argsort, prefix key scores + Argsort.
  pass1                  Alg. 2: dense causal attention inside each segment, leaving the
                         per-row online-softmax state (m, l, acc).
  attention              Alg. 2 + Alg. 3: gather queries by Q_perm, resume the states, walk
                         the prefix in KV_perm order in tiles of B_N, stop when the
                         marginal normaliser gain drops below tau, normalise, scatter.
  attention_visited_set  the same result written as exact softmax attention restricted to
                         the visited key set (an independent formulation, used as a pin).
  attention_fused_noqperm  Alg. 4 (single pass, no query reorder).
  gain_profile           the per-(query tile, prefix tile) gain the stop rule tests, with
                         stopping disabled.

Readings of points the paper leaves open (each also listed in the design notes):
  * Stop rule (Alg. 3, the `delta l < tau * l` line).  l and l' refer to different running
    maxima when the tile raises the maximum, so the test is evaluated in the new scale:
    gain_i = mass_i / prev_i with mass_i = sum_{t in tile} exp(x_it - m'_i) and
    prev_i = l_i * exp(m_i - m'_i).  It equals the printed form whenever m' = m.
  * Row -> tile reduction: a query tile stops iff max_i gain_i < tau (strict), i.e. every
    row's gain is below tau.  tau <= 0 therefore never stops.  PARITY UNPINNED: the paper
    gives no worked example that fixes the reduction.
  * Triggering tile: stop_mode 0 discards it (Alg. 3 / Alg. 4 break before committing);
    stop_mode 1 commits it and then stops (the deferred check of the appendix kernel D).
    PARITY UNPINNED between the two; each is pinned by the visited-set identity.
    stop_mode 2 evaluates no stop rule (the appendix's kernel C: ranked gather only).
  * Argsort tie-break: stable, equal scores keep ascending index; -0 == +0.
  * GQA: K/V head = h // G; k_guide per KV head; q_mean and both maps per query head.
  * Ranking scores are raw dot products (no softmax scale); attention uses
    softmax_scale = 1/sqrt(D) unless given.
  * KV_perm[n] holds only the n*S valid prefix entries (the -inf tail of Alg. 1 is never
    visited).  Segment 0 has no prefix.
  * The "local window W" listed as an input of Alg. 3/4 is never used in their bodies;
    it is read as W = S, i.e. Pass-1 itself.
  * Non-causal setting (causal=False; the appendix "Why Online Permutation Adds Negligible
    Overhead" runs its decomposition kernels and its top-k comparison on non-causal
    attention too, without spelling the algorithm out): every query attends every key.
    Reading: row n of KV_perm ranks all L tokens by <q_mean[n], K[t]> (rows of L entries,
    for every n, segment 0 included), there is no Pass-1, and each query row starts the
    ranked walk from the empty state (m = -inf, l = 0), so its first tile has infinite gain
    and is always kept.  tau <= 0 (or stop_mode 2 without a budget) reproduces plain softmax
    attention over all keys.  PARITY UNPINNED against the paper (no worked example); pinned
    against the plain definition at tau <= 0, the visited-set identity and the masked
    softmax of a tile budget.
  * Counts, per permuted query tile j of segment n (n*S/B_N prefix tiles exist):
    computed[j] = prefix tiles folded into the state (and so into O); skipped[j] = prefix
    tiles never issued.  A triggering tile that stop_mode 0 discards is in neither, so
    n*S/B_N - computed - skipped is 1 exactly when such a tile exists: the pair tells a
    run that ended on the last tile from one whose last tile triggered.
"""
from __future__ import annotations

import numpy as np

NEG_INF = -np.inf


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns (uint16) as float64."""
    return (np.asarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 -> bf16 (nearest even, via one exact fp32 step when representable)."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    b = f.view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def stable_argsort_desc(s: np.ndarray) -> np.ndarray:
    """Indices sorted by (score descending, index ascending)."""
    return np.argsort(-np.asarray(s, dtype=np.float64), kind="stable")


# ---------------------------------------------------------------------------
# Dense reference
# ---------------------------------------------------------------------------
def dense_attention(Q, K, V, scale=None, rows=None, causal=True):
    """O[z,h,i] = sum_{j<=i} softmax_j(scale <Q[z,h,i], K[z,h//G,j]>) V[z,h//G,j]
    (causal=False: the sum runs over all j).

    Q [Z,H,L,D], K,V [Z,Hkv,L,D] float64.  `rows` (optional 1-D index array) restricts
    the computed query rows; the result then has shape [Z,H,len(rows),D]."""
    Z, H, L, D = Q.shape
    G = H // K.shape[1]
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    rows = np.arange(L) if rows is None else np.asarray(rows)
    O = np.empty((Z, H, rows.size, D))
    for z in range(Z):
        for h in range(H):
            k, v = K[z, h // G], V[z, h // G]
            for c0 in range(0, rows.size, 512):
                r = rows[c0:c0 + 512]
                x = scale * (Q[z, h, r] @ k.T)                 # [r, L]
                if causal:
                    x[np.arange(L)[None, :] > r[:, None]] = NEG_INF
                x -= x.max(axis=1, keepdims=True)
                p = np.exp(x)
                O[z, h, c0:c0 + r.size] = (p @ v) / p.sum(axis=1, keepdims=True)
    return O


# ---------------------------------------------------------------------------
# Step 1: ranking (Alg. 1)
# ---------------------------------------------------------------------------
def kv_row_offset(n: int, S: int) -> int:
    """Start of row n inside the packed KV_perm / s_K arrays of one head: rows 1..n-1 hold
    S, 2S, ... entries, so row n starts at S*n(n-1)/2."""
    return S * n * (n - 1) // 2


def kv_row_start(n: int, S: int, L: int, causal: bool = True) -> int:
    """Start of row n in one head's KV_perm / s_K: packed prefix rows, or rows of L."""
    return kv_row_offset(n, S) if causal else n * L


def kv_row_len(n: int, S: int, L: int, causal: bool = True) -> int:
    """Keys row n ranks: the n*S tokens before segment n, or all L without causality."""
    return n * S if causal else L


def plan(Q, K, S, causal=True):
    """Alg. 1 (causal=False: every row ranks all L tokens, see the header).  Returns a dict with
         q_mean [Z,H,N,D], k_guide [Z,Hkv,D], s_q [Z,H,N,S], q_perm int32 [Z,H,N,S]
         (segment-local offsets), s_k [Z,H,P] and kv_perm int32 [Z,H,P] where
         P = S*N(N-1)/2 packs row n (length n*S, absolute token indices) at
         kv_row_offset(n, S); s_k is indexed by token t, not by rank."""
    Z, H, L, D = Q.shape
    Hkv = K.shape[1]
    G = H // Hkv
    N = L // S
    assert N * S == L and G * Hkv == H
    q_mean = Q.reshape(Z, H, N, S, D).mean(axis=3)
    k_guide = K[:, :, :S, :].mean(axis=2)                          # k_mean[0]
    s_q = np.empty((Z, H, N, S))
    q_perm = np.empty((Z, H, N, S), dtype=np.int32)
    P = kv_row_start(N, S, L, causal)
    s_k = np.empty((Z, H, P))
    kv_perm = np.empty((Z, H, P), dtype=np.int32)
    for z in range(Z):
        for h in range(H):
            g = h // G
            for n in range(N):
                s_q[z, h, n] = Q[z, h, n * S:(n + 1) * S] @ k_guide[z, g]
                q_perm[z, h, n] = stable_argsort_desc(s_q[z, h, n])
                ln = kv_row_len(n, S, L, causal)
                if ln == 0:
                    continue
                o = kv_row_start(n, S, L, causal)
                sk = K[z, g, :ln] @ q_mean[z, h, n]                # causal: the prefix only
                s_k[z, h, o:o + ln] = sk
                kv_perm[z, h, o:o + ln] = stable_argsort_desc(sk)
    return dict(q_mean=q_mean, k_guide=k_guide, s_q=s_q, q_perm=q_perm, s_k=s_k,
                kv_perm=kv_perm)


def identity_maps(Z, H, L, S, causal=True):
    """Maps that visit queries and keys in their original order."""
    N = L // S
    q_perm = np.broadcast_to(np.arange(S, dtype=np.int32), (Z, H, N, S)).copy()
    P = kv_row_start(N, S, L, causal)
    kv_perm = np.empty((Z, H, P), dtype=np.int32)
    for n in range(N):
        o, ln = kv_row_start(n, S, L, causal), kv_row_len(n, S, L, causal)
        kv_perm[:, :, o:o + ln] = np.arange(ln, dtype=np.int32)
    return q_perm, kv_perm


# ---------------------------------------------------------------------------
# Step 2: attention (Alg. 2 + Alg. 3)
# ---------------------------------------------------------------------------
def online_softmax_update(state, x, v):
    """One step of the online-softmax recurrence on rows with logits x [R,T] (masked
    entries = -inf) and values v [T,D]; state = (m [R], l [R], acc [R,D]).  Returns the
    candidate state and (mass, prev): the tile's mass and the old normaliser, both
    expressed relative to the new maximum."""
    m, l, acc = state
    m_new = np.maximum(m, x.max(axis=1))
    with np.errstate(invalid="ignore"):
        alpha = np.where(np.isneginf(m_new), 0.0, np.exp(m - m_new))
        p = np.where(np.isneginf(m_new)[:, None], 0.0, np.exp(x - m_new[:, None]))
    mass = p.sum(axis=1)
    prev = l * alpha
    return (m_new, prev + mass, acc * alpha[:, None] + p @ v), mass, prev


def pass1(q, k, v, scale, BM, BN):
    """Alg. 2 for one (head, segment): q,k,v [S,D] of the segment.  Returns (m,l,acc) per
    row after a dense causal scan of the segment's own key tiles."""
    S, D = q.shape
    m = np.full(S, NEG_INF)
    l = np.zeros(S)
    acc = np.zeros((S, D))
    for b in range(S // BM):
        r = slice(b * BM, (b + 1) * BM)
        st = (m[r], l[r], acc[r])
        rows = np.arange(b * BM, (b + 1) * BM)
        for t in range(S // BN):
            cols = np.arange(t * BN, (t + 1) * BN)
            x = scale * (q[r] @ k[cols].T)
            x[cols[None, :] > rows[:, None]] = NEG_INF             # CausalMask
            st, _, _ = online_softmax_update(st, x, v[cols])
        m[r], l[r], acc[r] = st
    return m, l, acc


def attention(Q, K, V, q_perm, kv_perm, S, BM, BN, tau, stop_mode=0, scale=None,
              forced_computed=None, heads=None, segments=None, return_gain=False, max_tiles=None,
              causal=True):
    """Alg. 2 + Alg. 3.  Returns (O [Z,H,L,D] float64, computed int32 [Z,H,L/BM],
    skipped int32 [Z,H,L/BM]); counts are indexed by permuted tile: entry n*(S/BM)+j is
    the j-th tile of Q~_n.

    forced_computed: replay mode -- tile j folds in exactly the first forced_computed[j]
      prefix tiles of its row (same layout as `computed`) and the stop rule is not
      evaluated; skipped is then reported as the remainder.
    max_tiles: fixed budget (the top-k selection of the appendix's matched-sparsity
      comparison, "Why Online Permutation Adds Negligible Overhead"): a query tile visits
      at most the first max_tiles tiles of its ranked row; the stop rule still applies
      inside the budget, and stop_mode 2 (no stop rule at all, the appendix's kernel C)
      makes it visit exactly min(max_tiles, n*S/B_N).  skipped counts every tile never
      issued, budgeted-out ones included.
    heads / segments: optional subsets (others are left zero) for sampled checks.
    return_gain: also return a dict {(z,h,n): array [S/BM, n*S/BN]} of max-row gains for
      the tiles that were evaluated (nan elsewhere).
    causal=False: no Pass-1; row n of kv_perm lists all L tokens and every query row starts
      from the empty state (see the header)."""
    Z, H, L, D = Q.shape
    G = H // K.shape[1]
    N = L // S
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    TJ = S // BM
    O = np.zeros((Z, H, L, D))
    computed = np.zeros((Z, H, L // BM), dtype=np.int32)
    skipped = np.zeros((Z, H, L // BM), dtype=np.int32)
    gains = {}
    for z in range(Z):
        for h in (range(H) if heads is None else heads):
            g = h // G
            k_all, v_all = K[z, g], V[z, g]
            for n in (range(N) if segments is None else segments):
                seg = slice(n * S, (n + 1) * S)
                qp = q_perm[z, h, n].astype(np.int64)
                qt = Q[z, h, seg][qp]                               # Gather(Q_n, Q_perm[n])
                if causal:
                    m1, l1, a1 = pass1(Q[z, h, seg], k_all[seg], v_all[seg], scale, BM, BN)
                    m, l, acc = m1[qp].copy(), l1[qp].copy(), a1[qp].copy()
                else:
                    m, l, acc = np.full(S, NEG_INF), np.zeros(S), np.zeros((S, D))
                o_row, ln = kv_row_start(n, S, L, causal), kv_row_len(n, S, L, causal)
                nK = ln // BN
                row = kv_perm[z, h, o_row:o_row + ln].astype(np.int64)
                gn = np.full((TJ, nK), np.nan)
                for j in range(TJ):
                    r = slice(j * BM, (j + 1) * BM)
                    st = (m[r], l[r], acc[r])
                    forced = None if forced_computed is None else int(forced_computed[z, h, n * TJ + j])
                    committed, issued = 0, 0
                    budget = nK if max_tiles is None else min(nK, int(max_tiles))
                    for kt in range(budget if forced is None else forced):
                        T = row[kt * BN:(kt + 1) * BN]
                        x = scale * (qt[r] @ k_all[T].T)
                        cand, mass, prev = online_softmax_update(st, x, v_all[T])
                        with np.errstate(divide="ignore"):           # prev = 0: an empty state, gain = inf
                            gain = float((mass / prev).max())
                        gn[j, kt] = gain
                        issued += 1
                        stop = forced is None and stop_mode != 2 and gain < tau
                        if stop and stop_mode == 0:
                            break                                   # triggering tile dropped
                        st = cand
                        committed += 1
                        if stop:
                            break
                    m[r], l[r], acc[r] = st
                    computed[z, h, n * TJ + j] = committed
                    skipped[z, h, n * TJ + j] = nK - issued
                O[z, h, n * S + qp] = acc / l[:, None]              # normalise + Scatter
                gains[(z, h, n)] = gn
    if return_gain:
        return O, computed, skipped, gains
    return O, computed, skipped


def gain_profile(Q, K, V, q_perm, kv_perm, S, BM, BN, stop_mode=0, scale=None,
                 heads=None, segments=None, causal=True):
    """Max-row gain of every (query tile, prefix tile) with stopping disabled.  In both
    stop modes the state before a stop does not depend on tau, so for any tau the stop
    position of tile j is the first k with gain[j,k] < tau."""
    out = attention(Q, K, V, q_perm, kv_perm, S, BM, BN, tau=0.0, stop_mode=stop_mode,
                    scale=scale, heads=heads, segments=segments, return_gain=True, causal=causal)
    return out[3]


def counts_from_gain(gain_row: np.ndarray, tau: float, stop_mode: int = 0):
    """(computed, skipped) implied by a gain row: the first k with gain < tau triggers."""
    nK = int(gain_row.size)
    below = np.nonzero(gain_row < tau)[0]
    if below.size == 0:
        return nK, 0
    k = int(below[0])
    return (k if stop_mode == 0 else k + 1), nK - (k + 1)


def attention_visited_set(Q, K, V, q_perm, kv_perm, S, BM, BN, tau, stop_mode=0, scale=None, causal=True):
    """Independent formulation: at step k the gain of row i is
         sum_{t in T_k} e^{x_it} / sum_{t in J0(i) u T_0..T_{k-1}} e^{x_it},
    J0(i) = own-segment keys up to i, and the output is exact softmax attention over the
    visited set.  No running maximum, no rescaling: one global shift per row.
    causal=False: J0 is empty, the rows list all L keys and the first tile is always kept."""
    Z, H, L, D = Q.shape
    G = H // K.shape[1]
    N = L // S
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    TJ = S // BM
    O = np.zeros((Z, H, L, D))
    computed = np.zeros((Z, H, L // BM), dtype=np.int32)
    skipped = np.zeros((Z, H, L // BM), dtype=np.int32)
    for z in range(Z):
        for h in range(H):
            g = h // G
            k, v = K[z, g], V[z, g]
            for n in range(N):
                o_row, ln = kv_row_start(n, S, L, causal), kv_row_len(n, S, L, causal)
                nK = ln // BN
                kv_row = kv_perm[z, h, o_row:o_row + ln].astype(np.int64)
                span = (n + 1) * S if causal else L                           # keys a row may see
                for j in range(TJ):
                    rows = n * S + q_perm[z, h, n, j * BM:(j + 1) * BM].astype(np.int64)
                    x = scale * (Q[z, h, rows] @ k[:span].T)                  # [BM, span]
                    if causal:
                        x[np.arange(span)[None, :] > rows[:, None]] = NEG_INF
                    e = np.exp(x - x.max(axis=1, keepdims=True))
                    denom = e[:, n * S:].sum(axis=1) if causal else np.zeros(BM)   # J0 mass
                    issued = nK
                    ncommit = nK
                    for kt in range(nK):
                        T = kv_row[kt * BN:(kt + 1) * BN]
                        mass = e[:, T].sum(axis=1)
                        with np.errstate(divide="ignore"):
                            gain = (mass / denom).max()
                        if gain < tau:
                            issued = kt + 1
                            ncommit = kt if stop_mode == 0 else kt + 1
                            break
                        denom = denom + mass
                    own = np.arange(n * S, (n + 1) * S) if causal else np.arange(0)
                    vis = np.concatenate([kv_row[:ncommit * BN], own])
                    O[z, h, rows] = (e[:, vis] @ v[vis]) / e[:, vis].sum(axis=1, keepdims=True)
                    computed[z, h, n * TJ + j] = ncommit
                    skipped[z, h, n * TJ + j] = nK - issued
    return O, computed, skipped


def attention_fused_noqperm(Q, K, V, kv_perm, S, BM, BN, tau, scale=None):
    """Alg. 4: queries in original order; per query tile one state that first scans the
    segment's own key tiles with the causal mask and then the ranked prefix with the
    stop rule (triggering tile discarded, as printed)."""
    Z, H, L, D = Q.shape
    G = H // K.shape[1]
    N = L // S
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    O = np.zeros((Z, H, L, D))
    for z in range(Z):
        for h in range(H):
            g = h // G
            k, v = K[z, g], V[z, g]
            for n in range(N):
                kv_row = kv_perm[z, h, kv_row_offset(n, S):kv_row_offset(n, S) + n * S].astype(np.int64)
                for b in range(S // BM):
                    rows = np.arange(n * S + b * BM, n * S + (b + 1) * BM)
                    q = Q[z, h, rows]
                    st = (np.full(BM, NEG_INF), np.zeros(BM), np.zeros((BM, D)))
                    for t in range(S // BN):
                        cols = np.arange(n * S + t * BN, n * S + (t + 1) * BN)
                        x = scale * (q @ k[cols].T)
                        x[cols[None, :] > rows[:, None]] = NEG_INF
                        st, _, _ = online_softmax_update(st, x, v[cols])
                    for kt in range(n * S // BN):
                        T = kv_row[kt * BN:(kt + 1) * BN]
                        cand, mass, prev = online_softmax_update(st, scale * (q @ k[T].T), v[T])
                        if (mass / prev).max() < tau:
                            break
                        st = cand
                    O[z, h, rows] = st[2] / st[1][:, None]
    return O


# ---------------------------------------------------------------------------
# Bookkeeping (density convention)
# ---------------------------------------------------------------------------
def causal_tiles(L, B):
    """Tiles of a BxB tiling of the causal L x L triangle (diagonal tiles count whole)."""
    t = L // B
    return t * (t + 1) // 2


def pass1_tiles(L, S, B):
    """Tiles Pass-1 computes per head: N segments, each a (S/B)(S/B+1)/2 triangle."""
    s = S // B
    return (L // S) * s * (s + 1) // 2


def prefix_tiles(L, S, BM, BN):
    """int array [L/BM]: prefix tiles that exist for each permuted query tile."""
    return np.repeat(np.arange(L // S) * (S // BN), S // BM)


def density(skipped, L, S, BM, BN):
    """Issued fraction of the causal score area, per head: Pass-1 tiles (closed form)
    plus every prefix tile that was issued (folded in or triggering), in units of
    BM x BN score elements.  sparsity = 1 - density."""
    t1 = (L // S) * sum(-(-((b + 1) * BM) // BN) for b in range(S // BM))
    tc = sum(-(-((b + 1) * BM) // BN) for b in range(L // BM))
    issued = prefix_tiles(L, S, BM, BN) - np.asarray(skipped)
    return (t1 + issued.sum(axis=-1)) / tc
