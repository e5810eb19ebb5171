"""Pins of the float64 oracle against what the paper and the mathematics fix.

None of these tests touches the HIP path.  Each pin is chosen so that one class of
mistake in oracle/still_oracle.py (a dropped term, a wrong sign, an off-by-one chunk
delay, a transposed operand, a wrong tie-break) fails it:

  * all tokens kept  -> textbook causal softmax attention (appendix softmax-attention eq.)
  * nothing kept     -> plain normalised linear attention over the routed prefix, in its
                        quadratic and its running-state form (appendix linear-attention eqs.)
  * one-hot values   -> every past token is seen exactly once, by exactly one branch, with the
                        two-chunk delay of Sec. 3.3 / Algorithm 1
  * the recurrent equations and Algorithm 1 are two separate statements of the operator in the
    paper; a third form enumerates the index sets row by row - all three must agree
  * score: closed value for a one-token window, closed value for a uniform window, closed form
    through the self-weight p as eps -> 0, and Algorithm 1's mask construction (W = C)
  * NP-Map: ||u|| = ||x||, halves sum to 1, identity MLP gives softmax(x) (+) softmax(-x)
  * selection: brute force over all subsets on tiny chunks, lowest-index tie-break
  * causality: appending tokens never changes earlier rows (prefill/decode consistency)
  * budget on the retained tokens: never exceeded at any row; a budget nobody reaches changes
    nothing; rows before the budget fills are those of the unlimited operator; every token is
    still seen exactly once; with whole chunks kept it is softmax attention over the first
    chunks plus the local span, linear attention over the rest, written out independently

The paper prints no worked numeric example of the operator, so there are no golden values
from it; tests/golden/ says so.
"""
import itertools

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

from oracle import still_oracle as O

EPS = 1e-6


def rand_problem(seed, N, d, df=None, scale_in=1.0):
    rng = np.random.default_rng(seed)
    df = df or d
    q = rng.standard_normal((N, d)) * scale_in
    k = rng.standard_normal((N, d)) * scale_in
    v = rng.standard_normal((N, d))
    g = 1.0 / (1.0 + np.exp(-rng.standard_normal((N, d))))
    Wq = rng.standard_normal((d, df)) / np.sqrt(d)
    Wk = rng.standard_normal((d, df)) / np.sqrt(d)
    return q, k, v, g, Wq, Wk


def causal_softmax_attention(q, k, v, scale):
    """Textbook: y_t = sum_{i<=t} softmax_i(scale q_t.k_i) v_i, through scipy's softmax."""
    N = q.shape[0]
    logits = scale * (q @ k.T)
    logits[np.triu_indices(N, 1)] = -np.inf
    return sp_softmax(logits, axis=1) @ v


FORMS = [O.still_definition, O.still_recurrent, O.still_chunkwise]


# --------------------------------------------------------------------------- all kept
@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("N,C", [(48, 8), (50, 8), (37, 16), (16, 16), (5, 8)])
def test_all_tokens_kept_is_causal_softmax_attention(form, N, C):
    q, k, v, g, Wq, Wk = rand_problem(1, N, 8)
    scale = 1 / np.sqrt(8)
    r = form(q, k, v, g, Wq, Wk, C=C, W=C, lam=C, scale=scale, eps=EPS)
    ref = causal_softmax_attention(q, k, v, scale)
    np.testing.assert_allclose(r["out"], ref, rtol=1e-11, atol=1e-12)
    assert np.all(r["D_LA"] == 0) and np.all(r["N_LA"] == 0)


def test_all_kept_is_chunk_size_invariant_and_stable_for_large_logits():
    q, k, v, g, Wq, Wk = rand_problem(2, 64, 8, scale_in=12.0)   # logits of several hundred
    outs = [O.still_chunkwise(q, k, v, None, Wq, Wk, C=C, W=4, lam=C, scale=1.0, eps=EPS)["out"]
            for C in (4, 8, 32)]
    ref = causal_softmax_attention(q, k, v, 1.0)
    for o in outs:
        assert np.all(np.isfinite(o))
        np.testing.assert_allclose(o, ref, rtol=1e-10, atol=1e-12)


# --------------------------------------------------------------------------- none kept
@pytest.mark.parametrize("form", FORMS)
def test_nothing_kept_linear_branch_is_plain_linear_attention(form):
    """lam = 0: the state seen by a row of chunk c is the sum over ALL tokens of chunks <= c-2,
    so N_LA / D_LA must equal normalised linear attention over that prefix, evaluated here in
    the quadratic form sum_i (phi(q_t).phi(k_i)) v_i with phi recomputed from its definition."""
    N, C, d = 40, 8, 6
    q, k, v, g, Wq, Wk = rand_problem(3, N, d, df=5)
    r = form(q, k, v, None, Wq, Wk, C=C, W=8, lam=0, scale=0.4, eps=EPS)

    def phi(x, Wm):
        f = x @ Wm
        u = f / np.linalg.norm(f, axis=1, keepdims=True) * np.linalg.norm(x, axis=1, keepdims=True)
        return np.concatenate([sp_softmax(u, axis=1), sp_softmax(-u, axis=1)], axis=1)

    pq, pk = phi(q, Wq), phi(k, Wk)
    A = pq @ pk.T                                    # quadratic form weights
    for t in range(N):
        n_prefix = max(0, (t // C - 1)) * C          # tokens of chunks <= c-2
        w = A[t, :n_prefix]
        np.testing.assert_allclose(r["D_LA"][t], w.sum(), rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(r["N_LA"][t], w @ v[:n_prefix], rtol=1e-11, atol=1e-14)
        # the softmax branch then covers exactly the local span
        lo = max(0, (t // C - 1) * C)
        e = np.exp(0.4 * (k[lo:t + 1] @ q[t]) - r["M"][t])
        np.testing.assert_allclose(r["D_SA"][t], e.sum(), rtol=1e-12)


def test_state_recurrence_matches_running_sum():
    """The (s, z) left after the last token equals the token-by-token recurrence
    s += phi(k)^T v, z += phi(k)^T over the routed, un-selected tokens."""
    N, C, d, lam = 48, 8, 6, 3
    q, k, v, g, Wq, Wk = rand_problem(4, N, d)
    r = O.still_recurrent(q, k, v, None, Wq, Wk, C=C, W=8, lam=lam, scale=0.4, eps=EPS, return_state=True)
    n_routed_chunks = (N - 1) // C - 1               # chunks <= c(last) - 2
    chosen = set(r["sel"][:n_routed_chunks].reshape(-1).tolist())
    s = np.zeros((2 * d, d))
    z = np.zeros(2 * d)
    for i in range(n_routed_chunks * C):
        if i in chosen:
            continue
        p = O.np_map(k[i], Wk)[0]
        s += np.outer(p, v[i])
        z += p
    np.testing.assert_allclose(r["state"]["s"], s, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(r["state"]["z"], z, rtol=1e-12, atol=1e-14)
    assert sorted(r["state"]["retained"].tolist()) == sorted(chosen)


# --------------------------------------------------------------------------- each token exactly once
@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("N,C,lam", [(24, 4, 1), (23, 4, 2), (20, 5, 0), (18, 6, 6)])
def test_every_past_token_contributes_once_with_two_chunk_delay(form, N, C, lam):
    """With v = identity (d = N) the numerators list each key's weight separately.  Row t
    (chunk c) must give: exp-weights exactly on the local span [(c-1)C, t] and on the selected
    tokens of chunks <= c-2; phi-weights exactly on the other tokens of chunks <= c-2; nothing
    on the future; never both."""
    rng = np.random.default_rng(5)
    dq = 4
    q = rng.standard_normal((N, dq))
    k = rng.standard_normal((N, dq))
    v = np.eye(N)
    Wq = rng.standard_normal((dq, 3))
    Wk = rng.standard_normal((dq, 3))
    # v has d = N columns while q,k have dq: the operator never mixes those dimensions
    r = form(q, k, v, None, Wq, Wk, C=C, W=3, lam=lam, scale=0.5, eps=EPS)
    sel = r["sel"]
    for t in range(N):
        c = t // C
        sa = r["N_SA"][t] > 0
        la = r["N_LA"][t] > 0
        assert not np.any(sa & la)
        assert np.all((sa | la)[: t + 1]) and not np.any((sa | la)[t + 1:])
        expect_sa = np.zeros(N, bool)
        expect_sa[max(0, (c - 1) * C): t + 1] = True
        for cc in range(0, c - 1):
            expect_sa[sel[cc]] = True
        assert np.array_equal(sa, expect_sa)
        # weights themselves
        e = np.exp(0.5 * (k @ q[t]) - r["M"][t])
        np.testing.assert_allclose(r["N_SA"][t][sa], e[sa], rtol=1e-12)


# --------------------------------------------------------------------------- three forms agree
@pytest.mark.parametrize("N,C,W,lam,df", [(64, 8, 8, 2, 8), (61, 8, 12, 3, 4), (40, 16, 5, 4, 8),
                                          (33, 4, 9, 1, 6), (7, 8, 8, 2, 8)])
def test_recurrent_chunkwise_and_definition_forms_agree(N, C, W, lam, df):
    q, k, v, g, Wq, Wk = rand_problem(6, N, 8, df=df)
    rng = np.random.default_rng(7)
    bq, bk = rng.standard_normal(df) * 0.1, rng.standard_normal(df) * 0.1
    rs = [f(q, k, v, g, Wq, Wk, C=C, W=W, lam=lam, scale=0.35, eps=EPS, bq=bq, bk=bk) for f in FORMS]
    for key in ("out", "M", "N_SA", "D_SA", "N_LA", "D_LA"):
        np.testing.assert_allclose(rs[0][key], rs[1][key], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(rs[0][key], rs[2][key], rtol=1e-11, atol=1e-13)
    assert all(np.all(r["D_SA"] > 0) for r in rs)


def test_row_range_mode_matches_full_run():
    q, k, v, g, Wq, Wk = rand_problem(8, 80, 8)
    full = O.still_chunkwise(q, k, v, g, Wq, Wk, C=8, W=8, lam=2, scale=0.35, eps=EPS)
    part = O.still_chunkwise(q, k, v, g, Wq, Wk, C=8, W=8, lam=2, scale=0.35, eps=EPS, rows=(40, 56))
    np.testing.assert_array_equal(full["out"][40:56], part["out"][40:56])
    rec = O.still_recurrent(q, k, v, g, Wq, Wk, C=8, W=8, lam=2, scale=0.35, eps=EPS, rows=(43, 50))
    np.testing.assert_allclose(full["out"][43:50], rec["out"][43:50], rtol=1e-11)


# --------------------------------------------------------------------------- gate
def test_gate_multiplies_linear_numerator_only():
    q, k, v, g, Wq, Wk = rand_problem(9, 48, 8)
    kw = dict(C=8, W=8, lam=2, scale=0.35, eps=EPS)
    r0 = O.still_chunkwise(q, k, v, None, Wq, Wk, **kw)
    r1 = O.still_chunkwise(q, k, v, g, Wq, Wk, **kw)
    np.testing.assert_allclose(r1["N_LA"], r0["N_LA"] * g, rtol=1e-13)
    np.testing.assert_array_equal(r1["D_LA"], r0["D_LA"])
    f = np.exp(-r0["M"])[:, None]
    y = (r0["N_SA"] + f * g * r0["N_LA"]) / (r0["D_SA"][:, None] + f * r0["D_LA"][:, None])
    np.testing.assert_allclose(r1["out"], y, rtol=1e-12)
    # a gate of zeros removes the linear numerator but keeps its share of the normaliser
    rz = O.still_recurrent(q, k, v, np.zeros_like(g), Wq, Wk, **kw)
    np.testing.assert_allclose(rz["out"], r0["N_SA"] / (r0["D_SA"][:, None] + f * r0["D_LA"][:, None]),
                               rtol=1e-10, atol=1e-14)


@pytest.mark.parametrize("form", FORMS)
def test_sigmoid_gate_literals(form):
    """Gate given as a pre-activation (Sec. 3.2: the gate comes from a projection W_g; sigmoid is this build's
    option, the paper names no activation): literal values of the logistic function, no formula retyped.
    sigmoid(0) = 1/2 halves the linear numerator; +-40 are 1 and 0 to machine precision; ln 3 gives 3/4."""
    q, k, v, g, Wq, Wk = rand_problem(23, 48, 8)
    kw = dict(C=8, W=8, lam=2, scale=0.35, eps=EPS)
    r0 = form(q, k, v, None, Wq, Wk, **kw)
    for x, val in ((0.0, 0.5), (40.0, 1.0), (-40.0, 0.0), (np.log(3.0), 0.75), (-np.log(3.0), 0.25)):
        r = form(q, k, v, np.full_like(g, x), Wq, Wk, gate_activation="sigmoid", **kw)
        np.testing.assert_allclose(r["N_LA"], val * r0["N_LA"], rtol=1e-12, atol=1e-16)
        np.testing.assert_array_equal(r["D_LA"], r0["D_LA"])
    # without the option the same numbers are used as they stand
    r = form(q, k, v, np.full_like(g, 0.5), Wq, Wk, **kw)
    ra = form(q, k, v, np.zeros_like(g), Wq, Wk, gate_activation="sigmoid", **kw)
    np.testing.assert_allclose(r["out"], ra["out"], rtol=1e-13)
    with pytest.raises(ValueError):
        form(q, k, v, g, Wq, Wk, gate_activation="tanh", **kw)


# --------------------------------------------------------------------------- score
def test_score_of_one_token_window_is_closed_value():
    q, k, *_ = rand_problem(10, 12, 8)
    s = O.self_saliency_scores(q, k, W=5, scale=0.3, eps=EPS)
    assert s[0] == pytest.approx(np.log((1 + EPS) / EPS), rel=1e-14)
    s1 = O.self_saliency_scores(q, k, W=1, scale=0.3, eps=EPS)      # every window has one token
    np.testing.assert_allclose(s1, np.log((1 + EPS) / EPS), rtol=1e-14)
    assert np.all(s <= np.log((1 + EPS) / EPS) * (1 + 1e-12))       # the largest value it can take


def test_score_of_uniform_window_is_closed_value():
    rng = np.random.default_rng(11)
    k = rng.standard_normal((20, 8))
    q = np.zeros((20, 8))
    Wn = 6
    s = O.self_saliency_scores(q, k, W=Wn, scale=1.0, eps=EPS)
    for t in range(1, 20):
        n = min(t + 1, Wn)
        expect = ((n - 1) / n) * np.log((1 / n + EPS) / (1 / (n - 1) + EPS)) + (1 / n) * np.log((1 / n + EPS) / EPS)
        assert s[t] == pytest.approx(expect, rel=1e-12)


def test_score_closed_form_through_self_weight():
    """With p the softmax weight the token gives itself, a_nodiag_j = a_diag_j / (1 - p), hence for
    eps -> 0:  Score -> p ln((p + eps)/eps) + (1 - p) ln(1 - p)."""
    q, k, *_ = rand_problem(12, 64, 8)
    eps = 1e-13
    Wn = 9
    s = O.self_saliency_scores(q, k, W=Wn, scale=0.5, eps=eps)
    for t in range(1, 64):
        lo = max(0, t - Wn + 1)
        p = sp_softmax(0.5 * (k[lo:t + 1] @ q[t]))[-1]
        expect = p * np.log((p + eps) / eps) + (1 - p) * np.log1p(-p)
        assert s[t] == pytest.approx(expect, rel=1e-8, abs=1e-9)


def test_score_matches_algorithm1_mask_construction_when_window_is_one_chunk():
    q, k, *_ = rand_problem(13, 96, 8)
    for C in (8, 16, 32):
        a = O.self_saliency_scores(q, k, W=C, scale=0.4, eps=EPS)
        b = O.alg1_scores(q, k, C=C, scale=0.4, eps=EPS)
        np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)


def test_score_ignores_keys_outside_window_and_future():
    q, k, *_ = rand_problem(14, 40, 8)
    s = O.self_saliency_scores(q, k, W=6, scale=0.4, eps=EPS)
    k2 = k.copy()
    k2[:10] += 5.0          # outside the window of token 20
    k2[21:] -= 3.0          # future of token 20
    s2 = O.self_saliency_scores(q, k2, W=6, scale=0.4, eps=EPS)
    assert s2[20] == s[20]
    assert s2[12] != s[12]


# --------------------------------------------------------------------------- NP-Map
def test_np_map_preserves_norm_and_is_two_distributions():
    rng = np.random.default_rng(15)
    x = rng.standard_normal((50, 16)) * np.exp(rng.standard_normal((50, 1)))
    Wm = rng.standard_normal((16, 12)) * 3.0      # an MLP that would rescale norms a lot
    b = rng.standard_normal(12)
    u = O.np_map_u(x, Wm, b)
    np.testing.assert_allclose(np.linalg.norm(u, axis=1), np.linalg.norm(x, axis=1), rtol=1e-14)
    phi = O.np_map(x, Wm, b)
    assert phi.shape == (50, 24) and np.all(phi > 0)
    np.testing.assert_allclose(phi[:, :12].sum(1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(phi[:, 12:].sum(1), 1.0, rtol=1e-14)
    # direction is that of f(x)
    f = x @ Wm + b
    cos = np.sum(u * f, axis=1) / (np.linalg.norm(u, axis=1) * np.linalg.norm(f, axis=1))
    np.testing.assert_allclose(cos, 1.0, rtol=1e-13)


def test_np_map_with_identity_mlp_is_hedgehog_softmax_pair():
    rng = np.random.default_rng(16)
    x = rng.standard_normal((9, 7))
    phi = O.np_map(x, np.eye(7))
    np.testing.assert_allclose(phi[:, :7], sp_softmax(x, axis=1), rtol=1e-13)
    np.testing.assert_allclose(phi[:, 7:], sp_softmax(-x, axis=1), rtol=1e-13)
    # scaling the MLP changes nothing: only its direction is used
    np.testing.assert_allclose(O.np_map(x, 7.5 * np.eye(7)), phi, rtol=1e-13)
    # zero MLP output -> uniform
    np.testing.assert_allclose(O.np_map(x, np.zeros((7, 4))), 0.25)


# --------------------------------------------------------------------------- selection
def test_selection_brute_force_and_tie_break():
    rng = np.random.default_rng(17)
    C = 9
    for trial in range(30):
        score = rng.standard_normal(3 * C + 4)          # ragged tail is never ranked
        if trial % 2:
            score = np.round(score * 2) / 2             # plant many exact ties
        for lam in (0, 1, 3, 8, 9):
            sel = O.select_top_lambda(score, C, lam)
            assert sel.shape == (3, lam)
            for c in range(3):
                s = score[c * C:(c + 1) * C]
                best = None
                for comb in itertools.combinations(range(C), lam):    # lexicographic order
                    tot = sum(s[i] for i in comb)
                    if best is None or tot > best[0] + 1e-15:
                        best = (tot, comb)
                # first maximiser in lexicographic order == ties broken toward low indices
                assert tuple(sel[c] - c * C) == best[1]
                assert np.all(np.diff(sel[c]) > 0)


def test_uniform_scores_select_lowest_indices():
    rng = np.random.default_rng(18)
    N, C, lam, Wn = 64, 8, 3, 8
    k = rng.standard_normal((N, 4))
    v = rng.standard_normal((N, 4))
    q = np.zeros((N, 4))
    r = O.still_chunkwise(q, k, v, None, np.eye(4), np.eye(4), C=C, W=Wn, lam=lam, scale=1.0, eps=EPS)
    for c in range(1, N // C):                  # chunks whose windows are all full: exact ties
        assert r["sel"][c].tolist() == [c * C, c * C + 1, c * C + 2]
    # first chunk: shorter windows score higher (token 0 highest), still the first three
    assert r["sel"][0].tolist() == [0, 1, 2]
    gaps = O.selection_gaps(r["score"], C, lam)
    assert gaps[1] == 0.0 and gaps[0] > 0


def test_selection_gap_and_chunk_quota_literals():
    """Hand-written values (no formula of the oracle is repeated here).  The gap of a chunk is the score of its
    last kept token minus the score of its best dropped token; a budget on the retained tokens is served chunk by
    chunk in order (Sec. 3.3 delayed selection; Sec. 4 long-context settings for the budget)."""
    # one chunk of four tokens, two kept
    assert O.selection_gaps(np.array([5.0, 3.0, 3.0, 1.0]), 4, 2).tolist() == [0.0]        # tie across the cut
    assert O.selection_gaps(np.array([5.0, 4.0, 2.0, 1.0]), 4, 2).tolist() == [2.0]        # 4 kept, 2 dropped
    assert O.selection_gaps(np.array([1.0, 5.0, 2.0, 4.0]), 4, 2).tolist() == [2.0]        # order in the chunk is irrelevant
    assert O.selection_gaps(np.array([5.0, 4.0, 2.0, 1.0]), 4, 1).tolist() == [1.0]        # 5 kept, 4 dropped
    assert O.selection_gaps(np.array([5.0, 4.0, 2.0, 1.0]), 4, 3).tolist() == [1.0]        # 2 kept, 1 dropped
    # nothing kept / everything kept: no cut, the gap is +inf
    assert O.selection_gaps(np.array([5.0, 4.0, 2.0, 1.0]), 4, 0).tolist() == [np.inf]
    assert O.selection_gaps(np.array([5.0, 4.0, 2.0, 1.0]), 4, 4).tolist() == [np.inf]
    # two chunks, the trailing partial chunk (one token) is never ranked
    s = np.array([9.0, 7.0, 4.0, 1.0, 2.0, 8.0, 3.0, 6.5, 100.0])
    assert O.selection_gaps(s, 4, 2).tolist() == [3.0, 3.5]                                # 7-4, 6.5-3
    # budget of three tokens, two per chunk: chunk 0 keeps two, chunk 1 keeps one, chunk 2 none
    s3 = np.concatenate([s[:8], [4.0, 3.0, 2.0, 1.0]])
    assert [O.chunk_quota(c, 2, 3) for c in range(4)] == [2, 1, 0, 0]
    assert [O.chunk_quota(c, 2, None) for c in range(3)] == [2, 2, 2]
    assert [O.chunk_quota(c, 2, 0) for c in range(2)] == [0, 0]
    assert [O.chunk_quota(c, 3, 7) for c in range(4)] == [3, 3, 1, 0]
    assert O.selection_gaps(s3, 4, 2, 3).tolist() == [3.0, 1.5, np.inf]                     # chunk 1: 8 kept, 6.5 best dropped
    sel = O.select_top_lambda(s3, 4, 2, 3)
    assert sel.tolist() == [[0, 1], [5, -1], [-1, -1]]
    # the gap and the selection agree: the kept set is exactly the tokens above the cut
    sel_all = O.select_top_lambda(s, 4, 2)
    assert sel_all.tolist() == [[0, 1], [5, 7]]


# --------------------------------------------------------------------------- causality
@pytest.mark.parametrize("form", [O.still_recurrent, O.still_chunkwise])
def test_appending_tokens_never_changes_earlier_rows(form):
    q, k, v, g, Wq, Wk = rand_problem(19, 70, 8)
    kw = dict(C=8, W=10, lam=2, scale=0.35, eps=EPS)
    full = form(q, k, v, g, Wq, Wk, **kw)
    for n in (1, 8, 9, 37, 64):
        part = form(q[:n], k[:n], v[:n], g[:n], Wq, Wk, **kw)
        np.testing.assert_allclose(part["out"], full["out"][:n], rtol=1e-12, atol=1e-14)
        np.testing.assert_array_equal(part["score"], full["score"][:n])


# --------------------------------------------------------------------------- batched driver
def test_unit_driver_uses_gqa_map():
    rng = np.random.default_rng(20)
    B, N, Hq, Hkv, d = 2, 24, 4, 2, 8
    inp = {"q": rng.standard_normal((B, N, Hq, d)), "k": rng.standard_normal((B, N, Hkv, d)),
           "v": rng.standard_normal((B, N, Hkv, d)), "Wq": rng.standard_normal((Hq, d, d)),
           "Wk": rng.standard_normal((Hq, d, d))}
    kv_map = np.array([0, 0, 1, 1])
    res = O.still_forward_units(inp, kv_map, [(1, 2)], C=4, W=4, lam=1, scale=0.3, eps=EPS)
    direct = O.still_chunkwise(inp["q"][1, :, 2], inp["k"][1, :, 1], inp["v"][1, :, 1], None,
                               inp["Wq"][2], inp["Wk"][2], C=4, W=4, lam=1, scale=0.3, eps=EPS)
    np.testing.assert_array_equal(res[(1, 2)]["out"], direct["out"])


# --------------------------------------------------------------------------- budget on retained tokens
@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("N,C,lam,cap", [(40, 4, 2, 5), (41, 4, 3, 6), (30, 5, 2, 0), (36, 6, 6, 9)])
def test_budget_is_never_exceeded_and_every_token_is_seen_once(form, N, C, lam, cap):
    """One-hot values again: with a budget, row t sees through exp the local span and at most `cap`
    selected tokens (chunks served in order until the budget is used up), every other routed token
    through phi, nothing twice."""
    rng = np.random.default_rng(15)
    q = rng.standard_normal((N, 4))
    k = rng.standard_normal((N, 4))
    Wq = rng.standard_normal((4, 3))
    Wk = rng.standard_normal((4, 3))
    r = form(q, k, np.eye(N), None, Wq, Wk, C=C, W=3, lam=lam, scale=0.5, eps=EPS, max_retained=cap)
    sel = r["sel"]
    counts = (sel >= 0).sum(axis=1)
    assert counts.sum() == min(cap, lam * (N // C))
    assert np.array_equal(counts, [min(lam, max(0, cap - c * lam)) for c in range(N // C)])
    for c in range(N // C):            # the kept ones are the best of the chunk, slots filled from the left
        kept = sel[c][: counts[c]]
        assert np.all(sel[c][counts[c]:] == -1) and np.all(np.diff(kept) > 0)
        order = sorted(range(C), key=lambda i: (-r["score"][c * C + i], i))
        assert sorted(kept.tolist()) == sorted(c * C + i for i in order[: counts[c]])
    for t in range(N):
        c = t // C
        sa, la = r["N_SA"][t] > 0, r["N_LA"][t] > 0
        assert not np.any(sa & la)
        assert np.all((sa | la)[: t + 1]) and not np.any((sa | la)[t + 1:])
        lo = max(0, (c - 1) * C)
        assert sa[:lo].sum() == min(cap, max(0, c - 1) * lam)      # retained part within the budget
        expect = np.zeros(N, bool)
        expect[lo: t + 1] = True
        for cc in range(0, c - 1):
            expect[sel[cc][sel[cc] >= 0]] = True
        assert np.array_equal(sa, expect)


@pytest.mark.parametrize("form", FORMS)
def test_budget_nobody_reaches_changes_nothing_and_early_rows_are_unlimited(form):
    q, k, v, g, Wq, Wk = rand_problem(16, 64, 8)
    kw = dict(C=8, W=6, lam=3, scale=0.35, eps=EPS)
    free = form(q, k, v, g, Wq, Wk, **kw)
    roomy = form(q, k, v, g, Wq, Wk, max_retained=3 * 8, **kw)
    np.testing.assert_array_equal(free["out"], roomy["out"])
    np.testing.assert_array_equal(free["sel"], roomy["sel"])
    tight = form(q, k, v, g, Wq, Wk, max_retained=7, **kw)     # chunks 0,1 keep 3, chunk 2 keeps 1
    # rows of chunk c see chunks <= c-2: identical while those chunks kept their full lam (c <= 3)
    np.testing.assert_array_equal(free["out"][: 4 * 8], tight["out"][: 4 * 8])
    assert np.abs(free["out"][4 * 8:] - tight["out"][4 * 8:]).max() > 1e-6
    # a budget of zero is the operator with nothing kept
    none = form(q, k, v, g, Wq, Wk, C=8, W=6, lam=0, scale=0.35, eps=EPS)
    zero = form(q, k, v, g, Wq, Wk, max_retained=0, **kw)
    np.testing.assert_allclose(zero["out"], none["out"], rtol=1e-13)


def test_budget_forms_agree():
    q, k, v, g, Wq, Wk = rand_problem(17, 70, 8, df=6)
    rs = [f(q, k, v, g, Wq, Wk, C=8, W=11, lam=3, scale=0.35, eps=EPS, max_retained=10) for f in FORMS]
    for key in ("out", "M", "N_SA", "D_SA", "N_LA", "D_LA"):
        np.testing.assert_allclose(rs[0][key], rs[1][key], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(rs[0][key], rs[2][key], rtol=1e-11, atol=1e-13)
    assert np.array_equal(rs[0]["sel"], rs[1]["sel"]) and np.array_equal(rs[0]["sel"], rs[2]["sel"])


# --------------------------------------------------------------------------- budget policy "evict"
def test_evict_policy_retained_sets_literals():
    """Hand example, C = 4, lam = 2, budget 3.  Scores by token:
         chunk 0: 5 1 4 0   -> offers tokens 0, 2
         chunk 1: 9 8 0 0   -> offers 4, 5
         chunk 2: 1 2 0 0   -> offers 8, 9
         chunk 3: 5 5 5 0   -> offers 12, 13 (tie of three: the lower indices)
    step 0: {0, 2}, nothing leaves.  step 1: {0:5, 2:4, 4:9, 5:8} -> 2 leaves.  step 2: 8 and 9 (scores 1, 2) are
    below everything kept and leave at once.  step 3: {0:5, 4:9, 5:8, 12:5, 13:5}: two of the three 5s must go,
    the higher indices first -> 13 and 12 leave, 0 stays."""
    score = np.array([5, 1, 4, 0, 9, 8, 0, 0, 1, 2, 0, 0, 5, 5, 5, 0], float)
    sel = O.select_top_lambda(score, 4, 2)
    assert sel.tolist() == [[0, 2], [4, 5], [8, 9], [12, 13]]
    kept, out = O.retained_sets_evict(score, sel, 3)
    assert [x.tolist() for x in kept] == [[0, 2], [0, 4, 5], [0, 4, 5], [0, 4, 5]]
    assert [x.tolist() for x in out] == [[], [2], [8, 9], [12, 13]]
    # margins: step 1 keeps {5, 9, 8}, releases 4 -> 5 - 4 = 1; step 2: 5 - 2 = 3; step 3: a tie, margin 0
    assert O.eviction_margins(score, sel, 3).tolist() == [np.inf, 1.0, 3.0, 0.0]
    kept1, out1 = O.retained_sets_evict(score, sel, 1)
    assert [x.tolist() for x in kept1] == [[0], [4], [4], [4]]
    assert [x.tolist() for x in out1] == [[2], [0, 5], [8, 9], [12, 13]]


@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("N,C,lam,cap", [(40, 4, 2, 5), (41, 4, 3, 4), (36, 6, 6, 9), (33, 4, 2, 1)])
def test_evict_policy_budget_never_exceeded_and_every_token_seen_once(form, N, C, lam, cap):
    """One-hot values: row t of chunk c sees through exp the local span and the `cap` best-scored offers of chunks
    <= c-2 (brute force over all offers made so far), every other routed token through phi, nothing twice."""
    rng = np.random.default_rng(41)
    q = rng.standard_normal((N, 4))
    k = rng.standard_normal((N, 4))
    Wq = rng.standard_normal((4, 3))
    Wk = rng.standard_normal((4, 3))
    r = form(q, k, np.eye(N), None, Wq, Wk, C=C, W=3, lam=lam, scale=0.5, eps=EPS, max_retained=cap,
             budget_policy="evict")
    sel, score = r["sel"], r["score"]
    assert np.all(sel >= 0)                       # every chunk offers its full Top-lambda
    for t in range(N):
        c = t // C
        sa, la = r["N_SA"][t] > 0, r["N_LA"][t] > 0
        assert not np.any(sa & la)
        assert np.all((sa | la)[: t + 1]) and not np.any((sa | la)[t + 1:])
        lo = max(0, (c - 1) * C)
        offers = [int(i) for cc in range(0, c - 1) for i in sel[cc]]
        best = sorted(offers, key=lambda i: (-score[i], i))[:cap]
        assert sa[:lo].sum() == len(best) <= cap
        expect = np.zeros(N, bool)
        expect[lo: t + 1] = True
        expect[best] = True
        assert np.array_equal(sa, expect)


@pytest.mark.parametrize("form", FORMS)
def test_evict_policy_special_cases(form):
    q, k, v, g, Wq, Wk = rand_problem(42, 64, 8)
    kw = dict(C=8, W=6, lam=3, scale=0.35, eps=EPS)
    free = form(q, k, v, g, Wq, Wk, **kw)
    # a budget nobody reaches is no budget
    roomy = form(q, k, v, g, Wq, Wk, max_retained=3 * 8, budget_policy="evict", **kw)
    np.testing.assert_array_equal(free["out"], roomy["out"])
    # budget zero: every offer leaves at once = nothing is ever kept
    none = form(q, k, v, g, Wq, Wk, C=8, W=6, lam=0, scale=0.35, eps=EPS)
    zero = form(q, k, v, g, Wq, Wk, max_retained=0, budget_policy="evict", **kw)
    np.testing.assert_allclose(zero["out"], none["out"], rtol=1e-12)
    # scores that fall from chunk to chunk: a later offer never beats a kept token, so evicting the lowest score
    # is the stop-adding policy (the offers that do not fit leave at once)
    N = 64
    falling = -np.arange(N, dtype=float)
    stop = form(q, k, v, g, Wq, Wk, max_retained=7, score=falling, **kw)
    evict = form(q, k, v, g, Wq, Wk, max_retained=7, score=falling, budget_policy="evict", **kw)
    np.testing.assert_allclose(stop["out"], evict["out"], rtol=1e-12)
    # scores that rise: the cache always holds the newest offers, i.e. a budget of whole offers is a sliding set
    rising = np.arange(N, dtype=float)
    ev = form(q, k, v, g, Wq, Wk, max_retained=6, score=rising, budget_policy="evict", **kw)
    # the same operator without a budget, fed for every row the two newest offers: only checkable row by row, so
    # compare one row of chunk 6 (sees offers of chunks 0..4, keeps those of chunks 3 and 4) against the definition
    t = 6 * 8 + 5
    keep = [int(i) for cc in (3, 4) for i in ev["sel"][cc]]
    local = list(range(5 * 8, t + 1))
    lin = [i for i in range(0, 5 * 8) if i not in keep]
    sa = np.asarray(keep + local)
    logit = 0.35 * (k[sa] @ q[t])
    e = np.exp(logit - logit.max())
    pq, pk = O.np_map(q, Wq), O.np_map(k, Wk)
    wgt = pk[lin] @ pq[t] * np.exp(-logit.max())
    y = (e @ v[sa] + (wgt @ v[lin]) * g[t]) / (e.sum() + wgt.sum())
    np.testing.assert_allclose(ev["out"][t], y, rtol=1e-11)


def test_evict_policy_forms_agree_and_rank_score_override():
    q, k, v, g, Wq, Wk = rand_problem(43, 70, 8, df=6)
    kw = dict(C=8, W=11, lam=3, scale=0.35, eps=EPS, max_retained=10, budget_policy="evict")
    rs = [f(q, k, v, g, Wq, Wk, **kw) for f in FORMS]
    for key in ("out", "M", "N_SA", "D_SA", "N_LA", "D_LA"):
        np.testing.assert_allclose(rs[0][key], rs[1][key], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(rs[0][key], rs[2][key], rtol=1e-11, atol=1e-13)
    stop = O.still_chunkwise(q, k, v, g, Wq, Wk, C=8, W=11, lam=3, scale=0.35, eps=EPS, max_retained=10)
    assert np.abs(stop["out"] - rs[2]["out"]).max() > 1e-6          # the two policies differ on random scores
    # ranking the evictions by another score changes who stays, not who is offered
    other = np.random.default_rng(5).standard_normal(70)
    alt = [f(q, k, v, g, Wq, Wk, rank_score=other, **kw) for f in FORMS]
    assert np.array_equal(alt[0]["sel"], rs[0]["sel"])
    assert np.abs(alt[0]["out"] - rs[0]["out"]).max() > 1e-6
    np.testing.assert_allclose(alt[0]["out"], alt[1]["out"], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(alt[0]["out"], alt[2]["out"], rtol=1e-11, atol=1e-13)


def test_budget_with_whole_chunks_kept_is_attention_sink_plus_window_plus_linear_rest():
    """lam = C and a budget of m chunks: the first m chunks stay under softmax for good, the local span
    slides, everything between goes through phi.  Written out directly with scipy's softmax weights and
    the kernel-feature weights, one normaliser."""
    N, C, m, scale = 56, 8, 2, 0.4
    q, k, v, g, Wq, Wk = rand_problem(18, N, 8)
    r = O.still_chunkwise(q, k, v, g, Wq, Wk, C=C, W=5, lam=C, scale=scale, eps=EPS, max_retained=m * C)
    pq, pk = O.np_map(q, Wq), O.np_map(k, Wk)
    for t in range(N):
        c = t // C
        lo = max(0, (c - 1) * C)
        n_routed = max(0, c - 1) * C
        sink = np.arange(min(m * C, n_routed))
        sm = np.concatenate([sink, np.arange(lo, t + 1)])
        lin = np.arange(min(m * C, n_routed), n_routed)
        logit = scale * (k[sm] @ q[t])
        a = sp_softmax(logit)                       # softmax weights inside the exp set
        zexp = np.exp(logit - logit.max()).sum()    # their normaliser, up to exp(max)
        w = (pk[lin] @ pq[t]) * np.exp(-logit.max())
        y = (zexp * (a @ v[sm]) + g[t] * (w @ v[lin])) / (zexp + w.sum())
        np.testing.assert_allclose(r["out"][t], y, rtol=1e-11, atol=1e-13)


# --------------------------------------------------------------------------- group-shared selection (variant)
def _gqa_inputs(seed, B, N, Hq, Hkv, d):
    rng = np.random.default_rng(seed)
    return {"q": rng.standard_normal((B, N, Hq, d)), "k": rng.standard_normal((B, N, Hkv, d)),
            "v": rng.standard_normal((B, N, Hkv, d)), "Wq": rng.standard_normal((Hq, d, d)) / np.sqrt(d),
            "Wk": rng.standard_normal((Hq, d, d)) / np.sqrt(d)}


def test_group_shared_selection_ranks_by_the_summed_score_and_is_one_list_per_kv_head():
    B, N, Hq, Hkv, d, C, lam = 2, 40, 6, 2, 4, 5, 2
    inp = _gqa_inputs(19, B, N, Hq, Hkv, d)
    kv_map = np.array([0, 1, 0, 1, 1, 0])                     # an irregular map: groups {0,2,5} and {1,3,4}
    units = [(b, h) for b in range(B) for h in range(Hq)]
    kw = dict(C=C, W=4, lam=lam, scale=0.5, eps=EPS)
    own = O.still_forward_units(inp, kv_map, units, **kw)
    shared = O.still_forward_units(inp, kv_map, units, shared_selection=True, **kw)
    for b in range(B):
        for kh in range(Hkv):
            members = [h for h in range(Hq) if kv_map[h] == kh]
            total = sum(own[(b, h)]["score"] for h in members)           # per-head scores are untouched
            for h in members:
                np.testing.assert_array_equal(shared[(b, h)]["score"], own[(b, h)]["score"])
                np.testing.assert_allclose(shared[(b, h)]["rank_score"], total, rtol=1e-14)
                np.testing.assert_array_equal(shared[(b, h)]["sel"], shared[(b, members[0])]["sel"])
            # brute force: no other lam-subset of a chunk has a larger summed score
            sel = shared[(b, members[0])]["sel"]
            for c in range(N // C):
                best = max(itertools.combinations(range(c * C, (c + 1) * C), lam), key=lambda s: total[list(s)].sum())
                assert sorted(sel[c].tolist()) == sorted(best)
    # the outputs are those of the per-head operator run with the shared lists
    for (b, h) in units:
        again = O.still_forward_units(inp, kv_map, [(b, h)],
                                      sel=np.broadcast_to(shared[(b, h)]["sel"], (B, Hq) + shared[(b, h)]["sel"].shape),
                                      **kw)[(b, h)]
        np.testing.assert_array_equal(again["out"], shared[(b, h)]["out"])
    assert any(not np.array_equal(own[u]["sel"], shared[u]["sel"]) for u in units)


def test_group_shared_selection_with_one_head_per_group_is_the_per_head_operator():
    inp = _gqa_inputs(20, 1, 48, 3, 3, 4)
    kv_map = np.arange(3)
    units = [(0, h) for h in range(3)]
    kw = dict(C=8, W=5, lam=3, scale=0.5, eps=EPS, max_retained=7)
    own = O.still_forward_units(inp, kv_map, units, **kw)
    shared = O.still_forward_units(inp, kv_map, units, shared_selection=True, **kw)
    for u in units:
        np.testing.assert_array_equal(own[u]["sel"], shared[u]["sel"])
        np.testing.assert_array_equal(own[u]["out"], shared[u]["out"])


# --------------------------------------------------------------------------- global score, overlap of selections
def test_global_score_is_the_score_over_the_whole_prefix():
    """Closed form through the self-weight over ALL earlier keys, and the uniform closed value with n = t + 1."""
    q, k, *_ = rand_problem(21, 50, 8)
    eps = 1e-13
    s = O.global_scores(q, k, scale=0.5, eps=eps)
    for t in range(1, 50):
        p = sp_softmax(0.5 * (k[:t + 1] @ q[t]))[-1]
        assert s[t] == pytest.approx(p * np.log((p + eps) / eps) + (1 - p) * np.log1p(-p), rel=1e-8, abs=1e-9)
    k1 = np.ones((30, 8))
    u = O.global_scores(q[:30], k1, scale=0.3, eps=EPS)
    for t in range(1, 30):
        n = t + 1
        expect = ((n - 1) / n) * np.log((1 / n + EPS) / (1 / (n - 1) + EPS)) + (1 / n) * np.log((1 / n + EPS) / EPS)
        assert u[t] == pytest.approx(expect, rel=1e-10)
    assert u[0] == pytest.approx(np.log((1 + EPS) / EPS), rel=1e-12)
    # a window that already covers the prefix gives the same numbers
    np.testing.assert_array_equal(O.global_scores(q, k, 0.5, EPS), O.self_saliency_scores(q, k, W=50, scale=0.5, eps=EPS))
    np.testing.assert_array_equal(O.global_scores(q, k, 0.5, EPS)[:7], O.self_saliency_scores(q, k, W=7, scale=0.5, eps=EPS)[:7])


def test_selection_overlap_counts_common_tokens():
    rng = np.random.default_rng(22)
    a = rng.standard_normal(40)
    assert O.selection_overlap(a, a, C=8, lam=3).tolist() == [3] * 5
    assert O.selection_overlap(a, -a, C=8, lam=3).tolist() == [0] * 5          # best three vs worst three of eight
    assert O.selection_overlap(a, -a, C=8, lam=8).tolist() == [8] * 5
    b = rng.standard_normal(40)
    got = O.selection_overlap(a, b, C=8, lam=4)
    for c in range(5):
        ta = set(np.argsort(-a[8 * c:8 * c + 8], kind="stable")[:4].tolist())
        tb = set(np.argsort(-b[8 * c:8 * c + 8], kind="stable")[:4].tolist())
        assert got[c] == len(ta & tb)
    assert O.selection_overlap(a[:37], b[:37], C=8, lam=4).shape == (4,)        # the partial chunk is not ranked


def test_rope_rotation_literals_norms_and_relative_positions():
    """The rotary embedding helper: a pair turned by a quarter turn, position 0 is the identity, norms are kept, and
    the product of a rotated query and a rotated key depends on their positions only through the difference."""
    # d = 2: one pair, theta = 1: position pi/2 turns (1, 0) into (0, 1)
    got = O.rope_rotate(np.array([[1.0, 0.0]]), np.array([np.pi / 2]), base=10000.0)
    assert np.allclose(got, [[0.0, 1.0]], atol=1e-15)
    # d = 4, base 100: pair (0, 2) turns by pos, pair (1, 3) by pos / 10
    x = np.array([[1.0, 2.0, 0.0, 0.0]])
    got = O.rope_rotate(x, np.array([3.0]), base=100.0)
    assert np.allclose(got, [[np.cos(3.0), 2 * np.cos(0.3), np.sin(3.0), 2 * np.sin(0.3)]], atol=1e-15)
    rng = np.random.default_rng(5)
    q, k = rng.normal(size=(7, 8)), rng.normal(size=(7, 8))
    assert np.array_equal(O.rope_rotate(q, np.zeros(7)), q)
    pos = np.array([0, 1, 2, 5, 9, 100, 4000])
    assert np.allclose(np.linalg.norm(O.rope_rotate(q, pos), axis=1), np.linalg.norm(q, axis=1), rtol=1e-13)
    a = O.rope_rotate(q[:1], np.array([12.0])) @ O.rope_rotate(k[:1], np.array([5.0])).T
    b = O.rope_rotate(q[:1], np.array([1007.0])) @ O.rope_rotate(k[:1], np.array([1000.0])).T
    assert np.allclose(a, b, rtol=1e-10)
    assert not np.allclose(a, q[:1] @ k[:1].T)
