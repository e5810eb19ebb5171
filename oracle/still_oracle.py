"""Float64 CPU oracle for STILL's intra-layer hybrid attention forward (arXiv 2602.02180).

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file; it is
used by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg.  It
shares no code with the HIP kernels and imports nothing from them.

Everything here works on ONE (batch, query-head) problem at a time: q, k, v are
[N, d] float64 arrays (k, v already taken from the kv-head that the query head maps
to), tokens are 0-indexed in code (the paper counts from 1; token t here is the
paper's token t+1, chunk c here is the paper's chunk c+1).

The same operator is written three ways, each from a different passage of the paper:

  * still_definition  - Sec. 3.3 recurrent form (cache-routing and output equations)
                        unrolled per output row into explicit index sets, O(N^2);
  * still_recurrent   - the same equations stepped token by token with the salient
                        cache h, and the state (s, z), routing one chunk at the
                        first token of a new chunk (delayed selection);
  * still_chunkwise   - Algorithm 1 (chunk-wise parallel form), chunk tensors,
                        cumulative sum of per-chunk states delayed by two chunks.

They must agree to rounding; tests/ pins them further against textbook softmax
attention (all tokens kept), plain linear attention (quadratic vs state form),
closed forms of the score, norm preservation of the feature map and brute-force
selection.

Readings of the paper used here (each is listed with its reason in the design notes):
  - one scalar `scale` multiplies every q.k logit (score window and softmax branch);
  - the window of token t holds the W keys t-W+1..t clipped at the sequence start;
  - masked positions are excluded from softmax/exp sums (not multiplied by zero);
  - a one-token window gives a_nodiag = 0, so Score = ln((1+eps)/eps);
  - only full chunks are ranked; ties go to the lower index; indices kept ascending;
  - the state sums only the un-selected tokens; the gate multiplies N_LA only;
  - f(x) = x W + b (one linear layer), phi = [softmax(u), softmax(-u)];
  - optional budget on the retained tokens (the long-context evaluations of Sec. 4 cap the
    number of selected tokens; the policy is not stated): chunks are served in order, chunk c
    keeps min(lambda, budget left) tokens, the rest of the chunk goes to the state like any
    un-selected token.  Unused slots of an index list hold -1;
  - optional group-shared selection (a variant, not the paper's method, which ranks per head
    and never mentions grouped-query attention): the query heads that read one kv head rank
    each chunk by the SUM of their scores and all keep the same tokens, so the retained keys
    and values exist once per kv head.

parity unpinned: the whole operator on random inputs at general lambda has no value
printed in the paper; beyond the special cases above its correctness rests on the
agreement of the three independent forms and on the readings listed.
"""
from __future__ import annotations

from typing import Dict, Optional, Tuple

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------
# Sec. 3.1: Self-Saliency Score (window set, the two window softmaxes, the score)
# ----------------------------------------------------------------------------

def _softmax(x: np.ndarray) -> np.ndarray:
    e = np.exp(x - np.max(x))
    return e / np.sum(e)


def self_saliency_scores(q: np.ndarray, k: np.ndarray, W: int, scale: float, eps: float) -> np.ndarray:
    """Score_t for every token: sum over the window of a_diag * ln((a_diag+eps)/(a_nodiag+eps)).

    Window of token t = keys max(0, t-W+1) .. t.  a_diag is the softmax over the whole
    window; a_nodiag the softmax over the window without t itself and 0 at t.
    """
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    N = q.shape[0]
    score = np.empty(N, F64)
    for t in range(N):
        lo = max(0, t - W + 1)
        logit = scale * (k[lo:t + 1] @ q[t])
        a_diag = _softmax(logit)
        a_nodiag = np.zeros_like(a_diag)
        if t > lo:
            a_nodiag[:-1] = _softmax(logit[:-1])
        score[t] = np.sum(a_diag * np.log((a_diag + eps) / (a_nodiag + eps)))
    return score


def alg1_scores(q: np.ndarray, k: np.ndarray, C: int, scale: float, eps: float) -> np.ndarray:
    """Scores as Algorithm 1 builds them (its window is exactly one chunk long, W = C).

    Per chunk: s_in = q k^T within the chunk, s_prev = q against the previous chunk's
    keys; the diag softmax runs over [s_in where key<=query, s_prev where key>query],
    the nodiag one over [s_in where key<query, s_prev where key>query].  The first
    chunk has no previous keys.  N must be a multiple of C here.
    """
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    N, d = q.shape
    assert N % C == 0
    T = N // C
    qc = q.reshape(T, C, d)
    kc = k.reshape(T, C, d)
    row = np.arange(C)[:, None]
    col = np.arange(C)[None, :]
    m_down, m_up, m_diag = row >= col, row < col, row > col
    out = np.empty((T, C), F64)
    for c in range(T):
        s_in = scale * (qc[c] @ kc[c].T)
        if c > 0:
            s_prev = scale * (qc[c] @ kc[c - 1].T)
            prev_ok = m_up
        else:
            s_prev = np.zeros((C, C), F64)
            prev_ok = np.zeros((C, C), bool)
        logits = np.concatenate([s_in, s_prev], axis=1)
        keep_diag = np.concatenate([m_down, prev_ok], axis=1)
        keep_nodiag = np.concatenate([m_diag, prev_ok], axis=1)

        def masked_softmax(keep):
            neg = np.where(keep, logits, -np.inf)
            mx = np.max(neg, axis=1, keepdims=True)
            mx = np.where(np.isfinite(mx), mx, 0.0)
            e = np.where(keep, np.exp(neg - mx), 0.0)
            den = np.sum(e, axis=1, keepdims=True)
            return np.where(den > 0, e / np.where(den > 0, den, 1.0), 0.0)

        a_diag = masked_softmax(keep_diag)
        a_nodiag = masked_softmax(keep_nodiag)
        term = np.where(keep_diag, a_diag * np.log((a_diag + eps) / (a_nodiag + eps)), 0.0)
        out[c] = term.sum(axis=1)
    return out.reshape(N)


# ----------------------------------------------------------------------------
# Sec. 3.3: delayed selection (Top-lambda per completed chunk)
# ----------------------------------------------------------------------------

def chunk_quota(c: int, lam: int, max_retained: Optional[int]) -> int:
    """Tokens chunk c (0-indexed) may keep: lam, or what is left of the budget after chunks 0..c-1."""
    if max_retained is None:
        return lam
    return int(min(lam, max(0, max_retained - c * lam)))


def select_top_lambda(score: np.ndarray, C: int, lam: int, max_retained: Optional[int] = None) -> np.ndarray:
    """Indices (global, ascending) of the highest scores of every FULL chunk: lam of them, or fewer
    once a budget on the total number of retained tokens runs out (chunks are served in order).

    Ties go to the lower index.  Returns int64 [N // C, lam]; slots a chunk does not use hold -1.
    """
    N = score.shape[0]
    ncf = N // C
    sel = np.full((ncf, lam), -1, np.int64)
    kept = 0
    for c in range(ncf):
        quota = lam if max_retained is None else min(lam, max(0, max_retained - kept))
        s = score[c * C:(c + 1) * C]
        order = sorted(range(C), key=lambda i: (-s[i], i))
        sel[c, :quota] = np.sort(np.asarray(order[:quota], np.int64)) + c * C
        kept += quota
    return sel


def retained_sets_evict(score: np.ndarray, sel: np.ndarray, max_retained: int):
    """Budget policy "evict" (an invention: Sec. 4's long-context settings cap the cached tokens, the policy is not
    stated).  Every routed chunk offers its Top-lambda tokens (`sel`, one row per full chunk, -1 = unused slot).
    After routing step s the retained set is the union of the previous set and chunk s's offer, cut back to
    max_retained members by removing the lowest score first (between equal scores the higher index goes first, so
    the lower index is kept, as in the Top-lambda rule).  A removed token, whether it was retained earlier or has
    just been offered, is handed to the linear-attention state AT THIS STEP.

    Returns (retained, released): retained[s] = sorted token indices kept after step s, released[s] = sorted token
    indices removed at step s."""
    kept: list = []
    retained, released = [], []
    for s in range(sel.shape[0]):
        kept = kept + [int(i) for i in sel[s] if i >= 0]
        kept.sort(key=lambda i: (-score[i], i))            # best first
        out = kept[max_retained:]
        kept = kept[:max_retained]
        retained.append(np.asarray(sorted(kept), np.int64))
        released.append(np.asarray(sorted(out), np.int64))
    return retained, released


def eviction_margins(score: np.ndarray, sel: np.ndarray, max_retained: int) -> np.ndarray:
    """Test helper for the "evict" policy: per routing step, the lowest score that stays minus the highest score
    that leaves (+inf when nothing leaves).  A comparison of two implementations is only meaningful at steps
    whose margin exceeds their score tolerance."""
    kept, out = retained_sets_evict(score, sel, max_retained)
    m = np.full(len(kept), np.inf)
    for s in range(len(kept)):
        if out[s].size and kept[s].size:
            m[s] = score[kept[s]].min() - score[out[s]].max()
    return m


def global_scores(q: np.ndarray, k: np.ndarray, scale: float, eps: float) -> np.ndarray:
    """The score with the window set replaced by the whole causal prefix {0..t}: the "global" reference of the
    local-versus-global consistency study of Sec. 3.1.  Same two softmaxes, same formula."""
    return self_saliency_scores(q, k, W=max(1, q.shape[0]), scale=scale, eps=eps)


def selection_overlap(score_a: np.ndarray, score_b: np.ndarray, C: int, lam: int) -> np.ndarray:
    """Per full chunk: how many tokens the Top-lambda sets under two scores have in common (int64 [N // C])."""
    sa = select_top_lambda(score_a, C, lam)
    sb = select_top_lambda(score_b, C, lam)
    return np.asarray([len(set(sa[c].tolist()) & set(sb[c].tolist())) for c in range(sa.shape[0])], np.int64)


def group_rank_score(scores: np.ndarray) -> np.ndarray:
    """Score that a group of query heads sharing one kv head ranks by: the sum of their Self-Saliency Scores.
    scores [G, N] -> [N].  Feeding it to select_top_lambda gives the one index list all G heads use."""
    return np.sum(np.asarray(scores, F64), axis=0)


def selection_gaps(score: np.ndarray, C: int, lam: int, max_retained: Optional[int] = None) -> np.ndarray:
    """Per full chunk: (last kept score) - (first score not kept); +inf if the chunk keeps none or all."""
    ncf = score.shape[0] // C
    gaps = np.full(ncf, np.inf)
    for c in range(ncf):
        quota = chunk_quota(c, lam, max_retained)
        if 0 < quota < C:
            s = np.sort(score[c * C:(c + 1) * C])[::-1]
            gaps[c] = s[quota - 1] - s[quota]
    return gaps


# ----------------------------------------------------------------------------
# Sec. 3.2: Norm-Preserved Feature Map
# ----------------------------------------------------------------------------

def np_map(x: np.ndarray, Wm: np.ndarray, b: Optional[np.ndarray] = None) -> np.ndarray:
    """phi_NP(x) for rows of x: u = f(x) / ||f(x)|| * ||x||, phi = softmax(u) (+) softmax(-u).

    f(x) = x Wm + b.  A zero f(x) gives u = 0 (uniform phi).
    """
    x = np.atleast_2d(np.asarray(x, F64))
    f = x @ np.asarray(Wm, F64)
    if b is not None:
        f = f + np.asarray(b, F64)
    nx = np.sqrt(np.sum(x * x, axis=1, keepdims=True))
    nf = np.sqrt(np.sum(f * f, axis=1, keepdims=True))
    u = np.where(nf > 0, f / np.where(nf > 0, nf, 1.0) * nx, 0.0)
    ep = np.exp(u - u.max(axis=1, keepdims=True))
    en = np.exp(-u - (-u).max(axis=1, keepdims=True))
    return np.concatenate([ep / ep.sum(axis=1, keepdims=True),
                           en / en.sum(axis=1, keepdims=True)], axis=1)


def np_map_u(x: np.ndarray, Wm: np.ndarray, b: Optional[np.ndarray] = None) -> np.ndarray:
    """The rescaled pre-activation u of the feature map (exposed for the norm test)."""
    x = np.atleast_2d(np.asarray(x, F64))
    f = x @ np.asarray(Wm, F64)
    if b is not None:
        f = f + np.asarray(b, F64)
    nx = np.sqrt(np.sum(x * x, axis=1, keepdims=True))
    nf = np.sqrt(np.sum(f * f, axis=1, keepdims=True))
    return np.where(nf > 0, f / np.where(nf > 0, nf, 1.0) * nx, 0.0)


# ----------------------------------------------------------------------------
# Rotary position embedding of q and k (the layer applies it before the operator; not part of the paper's method)
# ----------------------------------------------------------------------------

def rope_rotate(x: np.ndarray, positions: np.ndarray, base: float = 10000.0) -> np.ndarray:
    """Rotate rows of x [N, d] (d even) by their positions: channel pair (i, i + d/2) of row t turns by the angle
    positions[t] * base**(-2 i / d), the half-split pairing of the Llama family that the paper converts."""
    x = np.asarray(x, F64)
    N, d = x.shape
    half = d // 2
    theta = base ** (-2.0 * np.arange(half) / d)
    ang = np.asarray(positions, F64)[:, None] * theta[None, :]
    z = (x[:, :half] + 1j * x[:, half:]) * np.exp(1j * ang)
    return np.concatenate([z.real, z.imag], axis=1)


# ----------------------------------------------------------------------------
# shared result container
# ----------------------------------------------------------------------------

def gate_activate(g: Optional[np.ndarray], gate_activation: str = "none") -> Optional[np.ndarray]:
    """The gate as it multiplies the linear numerator (Sec. 3.2: g comes from a projection W_g; the paper names no
    activation).  "none": g is used as given (already activated by the caller); "sigmoid": g holds the
    pre-activation x W_g and the gate is its logistic function."""
    if g is None:
        return None
    g = np.asarray(g, F64)
    if gate_activation == "none":
        return g
    if gate_activation == "sigmoid":
        return 1.0 / (1.0 + np.exp(-g))
    raise ValueError(f"unknown gate activation {gate_activation!r}")


def _prep(q, k, v, g, Wq, Wk, bq, bk, gate_activation="none"):
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    v = np.asarray(v, F64)
    return q, k, v, gate_activate(g, gate_activation)


def _result(N, d, rows):
    return {
        "rows": rows,
        "out": np.zeros((N, d), F64),
        "M": np.zeros(N, F64),       # max softmax-branch logit of the row
        "N_SA": np.zeros((N, d), F64),  # sum exp(l - M) v   over the salient cache
        "D_SA": np.zeros(N, F64),       # sum exp(l - M)
        "N_LA": np.zeros((N, d), F64),  # gate * phi_q(q) s   (not shifted)
        "D_LA": np.zeros(N, F64),       # phi_q(q) z          (not shifted)
    }


def _merge(res, t):
    """y = (N_SA + N_LA) / (D_SA + D_LA) with the common factor exp(-M) applied to both."""
    f = np.exp(-res["M"][t])
    res["out"][t] = (res["N_SA"][t] + f * res["N_LA"][t]) / (res["D_SA"][t] + f * res["D_LA"][t])


def _scores_and_sel(q, k, C, W, lam, scale, eps, sel, score, max_retained=None, budget_policy="stop"):
    if score is None:
        score = self_saliency_scores(q, k, W, scale, eps)
    if sel is None:
        sel = select_top_lambda(score, C, lam, None if budget_policy == "evict" else max_retained)
    sel = np.asarray(sel, np.int64)
    sel = sel.reshape(q.shape[0] // C, sel.size // max(1, q.shape[0] // C))
    return score, sel


# ----------------------------------------------------------------------------
# Form 1: per-row index sets (the recurrent equations unrolled), O(N^2)
# ----------------------------------------------------------------------------

def still_definition(q, k, v, g, Wq, Wk, C, W, lam, scale, eps, bq=None, bk=None,
                     sel=None, score=None, rows: Optional[Tuple[int, int]] = None,
                     max_retained: Optional[int] = None, gate_activation: str = "none",
                     budget_policy: str = "stop", rank_score=None) -> Dict:
    """Row t in chunk c sees, through exp: the local span (previous chunk and own chunk up to t)
    plus the selected tokens of chunks <= c-2; through phi_q.phi_k: every other token of
    chunks <= c-2.  One division merges them.  (budget_policy "evict": the selected tokens are those
    retained after routing step c-2, see retained_sets_evict; rank_score overrides the score they are ranked by.)"""
    q, k, v, g = _prep(q, k, v, g, Wq, Wk, bq, bk, gate_activation)
    N, d = q.shape
    score, sel = _scores_and_sel(q, k, C, W, lam, scale, eps, sel, score, max_retained, budget_policy)
    evict = budget_policy == "evict" and max_retained is not None
    if evict:
        kept_after, _ = retained_sets_evict(score if rank_score is None else rank_score, sel, max_retained)
    phi_q = np_map(q, Wq, bq)
    phi_k = np_map(k, Wk, bk)
    rows = (0, N) if rows is None else rows
    res = _result(N, v.shape[1], rows)
    res["score"], res["sel"] = score, sel
    for t in range(*rows):
        c = t // C
        local = list(range(max(0, (c - 1) * C), t + 1))
        ret, lin = [], []
        if evict and c >= 2:
            chosen = set(int(i) for i in kept_after[c - 2])
            for i in range(0, (c - 1) * C):
                (ret if i in chosen else lin).append(i)
        for cc in range(0, c - 1 if not evict else 0):
            chosen = set(int(i) for i in sel[cc] if i >= 0)
            for i in range(cc * C, (cc + 1) * C):
                (ret if i in chosen else lin).append(i)
        sa = np.asarray(ret + local, np.int64)
        logit = scale * (k[sa] @ q[t])
        M = logit.max()
        e = np.exp(logit - M)
        res["M"][t] = M
        res["N_SA"][t] = e @ v[sa]
        res["D_SA"][t] = e.sum()
        if lin:
            li = np.asarray(lin, np.int64)
            wgt = phi_k[li] @ phi_q[t]
            n_la = wgt @ v[li]
            res["N_LA"][t] = n_la * (g[t] if g is not None else 1.0)
            res["D_LA"][t] = wgt.sum()
        _merge(res, t)
    return res


# ----------------------------------------------------------------------------
# Form 2: token-by-token recurrence with the salient cache and the (s, z) state
# ----------------------------------------------------------------------------

def still_recurrent(q, k, v, g, Wq, Wk, C, W, lam, scale, eps, bq=None, bk=None,
                    sel=None, score=None, rows: Optional[Tuple[int, int]] = None,
                    return_state: bool = False, max_retained: Optional[int] = None, gate_activation: str = "none",
                    budget_policy: str = "stop", rank_score=None) -> Dict:
    """Step t (1-indexed as in the paper) is written t = (a+1)C + b with 1 <= b <= C.
    When b == 1 and a >= 1 the chunk a (tokens (a-1)C+1 .. aC) is routed: its top-lambda
    keys/values join the retained part of the cache, the others are added to (s, z).
    The cache also always holds the local span aC < i <= t."""
    q, k, v, g = _prep(q, k, v, g, Wq, Wk, bq, bk, gate_activation)
    N, d = q.shape
    score, sel = _scores_and_sel(q, k, C, W, lam, scale, eps, sel, score, max_retained, budget_policy)
    evict = budget_policy == "evict" and max_retained is not None
    rk = score if rank_score is None else rank_score
    dprime = 2 * np.asarray(Wq).shape[1]
    s = np.zeros((dprime, v.shape[1]), F64)
    z = np.zeros(dprime, F64)
    retained: list = []           # token indices (0-indexed) in routing order
    rows = (0, N) if rows is None else rows
    res = _result(N, v.shape[1], rows)
    res["score"], res["sel"] = score, sel
    for t1 in range(1, N + 1):
        a = (t1 - 1) // C - 1
        b = t1 - (a + 1) * C
        if a >= 1 and b == 1:
            chunk0 = a - 1                      # 0-indexed chunk being routed
            chosen = [int(i) for i in sel[chunk0] if i >= 0]
            retained.extend(chosen)
            cs = set(chosen)
            rest = [i for i in range(chunk0 * C, (chunk0 + 1) * C) if i not in cs]
            if evict:
                # the cache is over its budget: the lowest scores leave it (between equal scores the higher index
                # first) and join the chunk's unselected tokens on their way into the state
                while len(retained) > max_retained:
                    worst = min(retained, key=lambda i: (rk[i], -i))
                    retained.remove(worst)
                    rest.append(worst)
            rest = np.asarray(sorted(rest), np.int64)
            if rest.size:
                pk = np_map(k[rest], Wk, bk)
                s = s + pk.T @ v[rest]
                z = z + pk.sum(axis=0)
        t = t1 - 1
        if not (rows[0] <= t < rows[1]):
            continue
        local = np.arange(max(0, a * C), t1, dtype=np.int64)     # paper: a*C < i <= t, 1-indexed
        h = np.concatenate([np.asarray(retained, np.int64), local])
        logit = scale * (k[h] @ q[t])
        M = logit.max()
        e = np.exp(logit - M)
        pq = np_map(q[t], Wq, bq)[0]
        res["M"][t] = M
        res["N_SA"][t] = e @ v[h]
        res["D_SA"][t] = e.sum()
        res["N_LA"][t] = (pq @ s) * (g[t] if g is not None else 1.0)
        res["D_LA"][t] = pq @ z
        _merge(res, t)
    if return_state:
        res["state"] = {"s": s, "z": z, "retained": np.asarray(retained, np.int64)}
    return res


# ----------------------------------------------------------------------------
# Form 3: Algorithm 1, chunk-wise parallel
# ----------------------------------------------------------------------------

def still_chunkwise(q, k, v, g, Wq, Wk, C, W, lam, scale, eps, bq=None, bk=None,
                    sel=None, score=None, rows: Optional[Tuple[int, int]] = None,
                     max_retained: Optional[int] = None, gate_activation: str = "none",
                     budget_policy: str = "stop", rank_score=None) -> Dict:
    """Chunk tensors; per-chunk states phi_k(k_LA)^T v_LA cumulated over chunks and delayed by
    two; chunk c attends with exp to the flattened selected keys of chunks <= c-2, to the whole
    previous chunk and causally to itself; a single division merges both branches.
    (budget_policy "evict": chunk c's selected keys are the set retained after routing step c-2, and a token
    released at step s is part of chunk s's contribution to the state.)"""
    q, k, v, g = _prep(q, k, v, g, Wq, Wk, bq, bk, gate_activation)
    N, d = q.shape
    score, sel = _scores_and_sel(q, k, C, W, lam, scale, eps, sel, score, max_retained, budget_policy)
    evict = budget_policy == "evict" and max_retained is not None
    T = -(-N // C)
    ncf = N // C
    dprime = 2 * np.asarray(Wq).shape[1]
    rows = (0, N) if rows is None else rows
    res = _result(N, v.shape[1], rows)
    res["score"], res["sel"] = score, sel

    # selected / unselected split per full chunk (a chunk may keep fewer tokens than it has slots: slots of -1)
    kept = [sel[c][sel[c] >= 0] for c in range(ncf)]
    n_kept = np.concatenate([[0], np.cumsum([len(x) for x in kept])]).astype(np.int64)   # before chunk c
    flat = np.concatenate(kept) if ncf else np.zeros(0, np.int64)
    k_sa_flat = k[flat]
    v_sa_flat = v[flat]
    if evict:
        kept_after, released = retained_sets_evict(score if rank_score is None else rank_score, sel, max_retained)
    ds = np.zeros((T, dprime, v.shape[1]), F64)
    dz = np.zeros((T, dprime), F64)
    for c in range(ncf):
        keep = np.ones(C, bool)
        keep[kept[c] - c * C] = False
        idx = np.nonzero(keep)[0] + c * C
        if evict:
            idx = np.concatenate([idx, released[c]])
        if idx.size:
            pk = np_map(k[idx], Wk, bk)
            ds[c] = pk.T @ v[idx]
            dz[c] = pk.sum(axis=0)
    s_cum = np.cumsum(ds, axis=0)
    z_cum = np.cumsum(dz, axis=0)

    c_lo, c_hi = rows[0] // C, -(-rows[1] // C)
    for c in range(c_lo, c_hi):
        t0, t1 = c * C, min(N, (c + 1) * C)
        qc = q[t0:t1]
        n_vis = int(n_kept[min(max(0, c - 1), ncf)])     # selected keys of chunks 0..c-2
        blocks_k = [k_sa_flat[:n_vis]]
        blocks_v = [v_sa_flat[:n_vis]]
        if evict:
            alive = kept_after[min(c - 2, ncf - 1)] if c >= 2 and ncf else np.zeros(0, np.int64)
            n_vis = alive.size
            blocks_k, blocks_v = [k[alive]], [v[alive]]
        masks = [np.ones((t1 - t0, n_vis), bool)]
        if c >= 1:
            blocks_k.append(k[t0 - C:t0])
            blocks_v.append(v[t0 - C:t0])
            masks.append(np.ones((t1 - t0, C), bool))
        blocks_k.append(k[t0:t1])
        blocks_v.append(v[t0:t1])
        r = np.arange(t1 - t0)
        masks.append(r[:, None] >= r[None, :])
        kk = np.concatenate(blocks_k, axis=0)
        vv = np.concatenate(blocks_v, axis=0)
        keep = np.concatenate(masks, axis=1)
        logit = np.where(keep, scale * (qc @ kk.T), -np.inf)
        M = logit.max(axis=1)
        o = np.where(keep, np.exp(logit - M[:, None]), 0.0)
        pq = np_map(qc, Wq, bq)
        if c >= 2:
            s_shift, z_shift = s_cum[c - 2], z_cum[c - 2]
        else:
            s_shift, z_shift = np.zeros((dprime, v.shape[1]), F64), np.zeros(dprime, F64)
        n_la = pq @ s_shift
        if g is not None:
            n_la = n_la * g[t0:t1]
        d_la = pq @ z_shift
        f = np.exp(-M)
        n_sa = o @ vv
        d_sa = o.sum(axis=1)
        y = (n_sa + f[:, None] * n_la) / (d_sa + f * d_la)[:, None]
        res["M"][t0:t1] = M
        res["N_SA"][t0:t1] = n_sa
        res["D_SA"][t0:t1] = d_sa
        res["N_LA"][t0:t1] = n_la
        res["D_LA"][t0:t1] = d_la
        res["out"][t0:t1] = y
    res["s_cum"], res["z_cum"] = s_cum, z_cum
    return res


# ----------------------------------------------------------------------------
# batch / head driver
# ----------------------------------------------------------------------------

def still_forward_units(inputs: Dict[str, np.ndarray], kv_map: np.ndarray, units, C, W, lam, scale, eps,
                        form: str = "chunkwise", sel: Optional[np.ndarray] = None,
                        rows: Optional[Tuple[int, int]] = None,
                        max_retained: Optional[int] = None,
                        shared_selection: bool = False,
                        gate_activation: str = "none", budget_policy: str = "stop",
                        rank_scores: Optional[np.ndarray] = None) -> Dict[Tuple[int, int], Dict]:
    """Run one form on the listed (b, hq) units of a batched problem.

    inputs: q [B,N,Hq,d], k,v [B,N,Hkv,d], Wq,Wk [Hq,d,d_f], optional g [B,N,Hq,d],
    optional bq,bk [Hq,d_f].  sel (optional) [B,Hq,N//C,lam] overrides the selection.
    shared_selection: the heads that read one kv head rank by the sum of their scores and share one list.
    Every result carries "rank_score": the score its selection was ranked by (its own, or the group's sum).
    budget_policy "evict" (with max_retained): see retained_sets_evict; rank_scores (optional) [B,Hq,N] overrides the
    score the evictions are ranked by (tests pass the device's fp32 scores, so both sides decide in one precision).
    """
    fn = {"chunkwise": still_chunkwise, "recurrent": still_recurrent, "definition": still_definition}[form]
    out = {}
    group_cache: Dict[Tuple[int, int], np.ndarray] = {}
    for (b, h) in units:
        kh = int(kv_map[h])
        rank = None
        if shared_selection:
            if (b, kh) not in group_cache:
                members = [hh for hh in range(len(kv_map)) if int(kv_map[hh]) == kh]
                group_cache[(b, kh)] = group_rank_score(np.stack([
                    self_saliency_scores(np.asarray(inputs["q"][b, :, hh], F64), np.asarray(inputs["k"][b, :, kh], F64),
                                         W, scale, eps) for hh in members]))
            rank = group_cache[(b, kh)]
        g = inputs["g"][b, :, h] if inputs.get("g") is not None else None
        bq = inputs["bq"][h] if inputs.get("bq") is not None else None
        bk = inputs["bk"][h] if inputs.get("bk") is not None else None
        s_in = None if sel is None else sel[b, h]
        if s_in is None and rank is not None:
            s_in = select_top_lambda(rank, C, lam, None if budget_policy == "evict" else max_retained)
        extra = {}
        if budget_policy == "evict":
            if shared_selection:
                raise ValueError("the evict policy is defined per query head")
            extra = dict(budget_policy="evict", rank_score=None if rank_scores is None else rank_scores[b, h])
        out[(b, h)] = fn(inputs["q"][b, :, h], inputs["k"][b, :, kh], inputs["v"][b, :, kh], g,
                         inputs["Wq"][h], inputs["Wk"][h], C, W, lam, scale, eps, bq=bq, bk=bk,
                         sel=s_in, rows=rows, max_retained=max_retained, gate_activation=gate_activation, **extra)
        out[(b, h)]["rank_score"] = out[(b, h)]["score"] if rank is None else rank
    return out
