"""Brute-force re-derivation of the H2O process on tiny inputs (NumPy).

Written independently of ``oracle/``: it works on the whole token sequence at
once with dense boolean membership masks, takes the eviction decision by
literally evaluating the set function F_score(G \\ {v}) for every allowed v and
choosing the arg-max (Definition 4.3 / Algorithm 1, the argmax line), computes
prompt column sums with an explicit double loop, and selects the prompt's heavy
hitters by sorting instead of by repeated eviction.  It is only usable for a
few dozen tokens.
"""
import math

import numpy as np


def _store(x, dtype):
    return np.asarray(x, dtype=dtype).astype(np.float64)


def _rank(acc, members, last_q, policy, score_dtype):
    """What ranks each member after the query at position last_q: its score, or
    (policy 1) its score divided by the number of queries that scored it."""
    if policy == 0:
        return {s: acc[s] for s in members}
    if score_dtype == np.float32:
        return {s: float(np.float32(acc[s]) / np.float32(last_q - s + 1)) for s in members}
    return {s: acc[s] / (last_q - s + 1) for s in members}


def nearest_level_quantise(row, group):
    """Group-wise 4-bit storage of one row, by search: per group of `group`
    elements the 16 levels are evenly spaced from the group's minimum to its
    maximum (spacing and minimum held in binary32) and every element is replaced
    by the level closest to it.  Returns (stored row float64, codes, every
    element's distance to the nearest half-way point in units of the spacing)."""
    row = np.asarray(row, np.float64)
    out, codes = np.empty_like(row), np.empty(row.shape, np.int64)
    margin = np.full(row.shape, np.inf)
    for g0 in range(0, row.size, group):
        x = row[g0:g0 + group]
        mn, mx = np.float32(x.min()), np.float32(x.max())
        step = np.float32(np.float32(mx - mn) / np.float32(15))
        levels = np.float64(mn) + np.arange(16) * np.float64(step)
        dist = np.abs(x[:, None] - levels[None, :])
        c = dist.argmin(axis=1)
        if step > 0:
            frac = (x - np.float64(mn)) / np.float64(step)
            margin[g0:g0 + group] = np.where(frac < 15, np.abs(frac - np.floor(frac) - 0.5), np.inf)
        codes[g0:g0 + group] = c
        out[g0:g0 + group] = levels[c]
    return out, codes, margin


def pattern_cover(pattern, recent, t):
    """The set of positions <= t a sparse-attention pattern lets the query at position t
    attend to, by enumeration (Sparse Transformer's two patterns, each the union of a local
    part and a periodic part).  pattern = ("strided", s): the last `recent` positions, and
    every s-th position counted back from t.  pattern = ("fixed", s): the block of s
    positions that contains t, and the last `recent` positions of every block."""
    kind, s = pattern
    cover = set()
    if kind == "strided":
        cover.update(range(max(0, t - recent + 1), t + 1))
        cover.update(range(t, -1, -s))
    elif kind == "fixed":
        b0 = (t // s) * s
        cover.update(range(b0, t + 1))
        for start in range(0, t + 1, s):
            cover.update(j for j in range(start + s - recent, start + s) if 0 <= j <= t)
    else:
        raise ValueError(kind)
    return cover


def brute_h2o(Q, K, V, n, heavy, recent, scale, score_dtype=np.float64, policy=0, store=None, pattern=None):
    """Q, K, V: [N, d] for all N = n + T tokens.  Returns a dict with
    per-decode-step outputs, resident sets after every call, evicted tokens,
    prompt column sums and final scores.  `store` (row -> row) is what the cache
    does to a key or value row when the token enters it (after the prompt phase,
    or after the token's own step); the token's own step sees the row as given."""
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64).copy(); V = np.asarray(V, np.float64).copy()
    N, d = Q.shape
    k = heavy + recent
    S = scale * (Q @ K.T)                       # every logit there is (rows are redone if rows change)

    acc = np.zeros(N)
    member = np.zeros(N, dtype=bool)
    sets, outs, evicted = [], [], []
    colsum = np.zeros(n)
    attn_prompt = np.zeros((n, d))
    if n > 0:
        P = np.zeros((n, n))
        for i in range(n):
            row = S[i, : i + 1]
            e = np.exp(row - row.max())
            P[i, : i + 1] = e / e.sum()
        for j in range(n):                       # column sums, double loop
            c = 0.0
            for i in range(j, n):
                c += P[i, j]
            colsum[j] = c
        attn_prompt = P @ V[:n]
        acc[:n] = _store(colsum, score_dtype)
        if n <= k:
            member[:n] = True
        elif pattern is not None:
            # what the pattern covers for the last prompt query stays, topped up with the best
            # of the rest; if it covers more than the budget, the best of what it covers
            cover = sorted(pattern_cover(pattern, recent, n - 1))
            rest = [j for j in range(n) if j not in set(cover)]
            r = _rank(acc, list(range(n)), n - 1, policy, score_dtype)
            best_first = lambda js: sorted(js, key=lambda j: (r[j], j), reverse=True)
            kept = cover + best_first(rest)[:k - len(cover)] if len(cover) <= k else best_first(cover)[:k]
            member[kept] = True
        else:
            member[n - recent:n] = True
            older = list(range(n - recent))
            r = _rank(acc, older, n - 1, policy, score_dtype)
            # best first: higher score, then higher position (so that what is
            # dropped is the lowest score and, among equals, the lowest position)
            older.sort(key=lambda j: (r[j], j), reverse=True)
            member[older[:heavy]] = True
        sets.append(set(np.flatnonzero(member).tolist()))
        if store is not None:
            for j in np.flatnonzero(member):
                K[j], V[j] = store(K[j]), store(V[j])

    for t in range(n, N):
        G = member.copy()
        G[t] = True
        if store is not None:
            S[t] = scale * (K @ Q[t])             # against the rows as the cache holds them now
        row = np.where(G, S[t], -np.inf)
        e = np.exp(row - row.max())
        p = e / e.sum()                           # zero outside G
        outs.append(p @ V)
        if score_dtype == np.float32:
            acc = (acc.astype(np.float32) + p.astype(np.float32)).astype(np.float64)
        else:
            acc = acc + p
        u = -1
        if G.sum() > k:
            members = np.flatnonzero(G).tolist()
            if pattern is None:
                allowed = [v for v in members if v <= t - recent]
            else:
                cover = pattern_cover(pattern, recent, t)
                allowed = [v for v in members if v not in cover] or [v for v in members if v != t]
            r = _rank(acc, members, t, policy, score_dtype)
            best_f = None
            for v in allowed:                     # ascending position
                f = math.fsum(r[s] for s in members if s != v)
                if best_f is None or f > best_f:
                    best_f, u = f, v
            G[u] = False
        evicted.append(u)
        member = G
        if store is not None and member[t]:
            K[t], V[t] = store(K[t]), store(V[t])
        sets.append(set(np.flatnonzero(member).tolist()))
    return dict(outs=np.array(outs), sets=sets, evicted=evicted, colsum=colsum,
                attn_prompt=attn_prompt, acc=acc)


def brute_chunked(Q, K, V, chunks, heavy, recent, scale, score_dtype=np.float64, policy=0):
    """Chunked prompt processing on the whole sequence at once: `chunks` lists
    the chunk lengths.  Every token of a chunk attends to the tokens kept so far
    and, causally, to its own chunk; the chunk's column sums are added to the
    scores; then the kept set is cut to the budget by SORTING (last `recent`
    positions stay, of the rest the `heavy` best by (rank value, position)).
    Returns outputs [N, d], the kept set after every chunk and the final scores."""
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    N, d = Q.shape
    assert sum(chunks) == N
    k = heavy + recent
    S = scale * (Q @ K.T)
    acc = np.zeros(N)
    member = np.zeros(N, dtype=bool)
    outs = np.zeros((N, d))
    sets = []
    t0 = 0
    for m in chunks:
        t1 = t0 + m
        csum = np.zeros(N)
        for i in range(t0, t1):
            G = member.copy()
            G[t0:i + 1] = True
            row = np.where(G, S[i], -np.inf)
            e = np.exp(row - row.max())
            p = e / e.sum()
            outs[i] = p @ V
            csum += p
        if score_dtype == np.float32:
            acc = (acc.astype(np.float32) + csum.astype(np.float32)).astype(np.float64)
        else:
            acc = acc + csum
        member[t0:t1] = True
        if member.sum() > k:
            members = np.flatnonzero(member).tolist()
            window = [j for j in members if j >= t1 - recent]
            older = [j for j in members if j < t1 - recent]
            r = _rank(acc, older, t1 - 1, policy, score_dtype)
            older.sort(key=lambda j: (r[j], j), reverse=True)
            member[:] = False
            member[window] = True
            member[older[:heavy]] = True
        sets.append(set(np.flatnonzero(member).tolist()))
        t0 = t1
    return dict(outs=outs, sets=sets, acc=acc)
