"""Pins of the backward oracle (oracle/still_backward.py) against things other than itself: central finite
differences of the forward definition (Sec. 3.3 output equation, routing held fixed), the textbook gradient of
causal softmax attention when every token is kept, and the Jacobian structure of the NP-Map (Sec. 3.2)."""
import numpy as np
import pytest
import torch

from oracle import still_oracle as O
from oracle import still_backward as OB


def tiny(seed, N=20, d=3, F=4, C=4, gate=True, bias=True):
    r = np.random.default_rng(seed)
    p = dict(q=r.normal(size=(N, d)), k=r.normal(size=(N, d)), v=r.normal(size=(N, d)),
             g=r.normal(size=(N, d)) if gate else None,
             Wq=r.normal(size=(d, F)), Wk=r.normal(size=(d, F)),
             bq=0.3 * r.normal(size=F) if bias else None, bk=0.3 * r.normal(size=F) if bias else None)
    dy = r.normal(size=(N, d))
    return p, dy


def loss(p, dy, sel, C, W, lam, scale, eps, **kw):
    res = O.still_definition(p["q"], p["k"], p["v"], p["g"], p["Wq"], p["Wk"], C, W, lam, scale, eps,
                             bq=p["bq"], bk=p["bk"], sel=sel, **kw)
    return float(np.sum(res["out"] * dy))


@pytest.mark.parametrize("lam,max_retained,act", [(1, None, "none"), (2, None, "sigmoid"), (2, 3, "none"),
                                                   (0, None, "sigmoid")])
def test_every_gradient_matches_central_differences_of_the_forward_definition(lam, max_retained, act):
    C, W, scale, eps = 4, 3, 0.6, 1e-6
    p, dy = tiny(11 + lam)
    fwd = O.still_definition(p["q"], p["k"], p["v"], p["g"], p["Wq"], p["Wk"], C, W, lam, scale, eps,
                             bq=p["bq"], bk=p["bk"], max_retained=max_retained, gate_activation=act)
    sel = fwd["sel"]
    kw = dict(max_retained=max_retained, gate_activation=act)
    got = OB.still_backward_definition(p["q"], p["k"], p["v"], p["g"], p["Wq"], p["Wk"], C, W, lam, scale, eps, dy,
                                       bq=p["bq"], bk=p["bk"], sel=sel, **kw)
    h = 1e-5
    for name, key in (("q", "dq"), ("k", "dk"), ("v", "dv"), ("g", "dg"), ("Wq", "dWq"), ("Wk", "dWk"),
                      ("bq", "dbq"), ("bk", "dbk")):
        base = p[name]
        fd = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = base[i]
            base[i] = old + h
            up = loss(p, dy, sel, C, W, lam, scale, eps, **kw)
            base[i] = old - h
            dn = loss(p, dy, sel, C, W, lam, scale, eps, **kw)
            base[i] = old
            fd[i] = (up - dn) / (2 * h)
        err = np.max(np.abs(fd - got[key]))
        ref = max(1.0, np.max(np.abs(fd)))
        assert err <= 1e-6 * ref, (name, err, ref)
    # with lambda >= 1 and 5 chunks both branches are live: none of the gradients is identically zero
    if lam > 0:
        for key in ("dq", "dk", "dv", "dg", "dWq", "dWk", "dbq", "dbk"):
            assert np.max(np.abs(got[key])) > 1e-6, key
    # the normaliser the backward reports is the forward's: log(D_SA + D_LA) with the common shift undone
    lse_fwd = fwd["M"] + np.log(fwd["D_SA"] + np.exp(-fwd["M"]) * fwd["D_LA"])
    assert np.allclose(got["lse"], lse_fwd, rtol=1e-12, atol=1e-12)


def test_all_tokens_kept_gives_the_gradient_of_causal_softmax_attention():
    """lambda = C: no token ever reaches the linear state, so the operator is causal softmax attention and its
    gradients are the library's (torch autograd on float64); the feature-map parameters get none."""
    C, W, scale, eps = 4, 4, 0.5, 1e-6
    p, dy = tiny(5, N=16, gate=True, bias=False)
    sel = np.arange(16).reshape(4, 4)
    got = OB.still_backward_definition(p["q"], p["k"], p["v"], p["g"], p["Wq"], p["Wk"], C, W, C, scale, eps, dy,
                                       sel=sel)
    tq, tk, tv = (torch.tensor(p[n], dtype=torch.float64, requires_grad=True) for n in ("q", "k", "v"))
    logits = scale * tq @ tk.T
    mask = torch.tril(torch.ones(16, 16, dtype=torch.bool))
    y = torch.softmax(logits.masked_fill(~mask, float("-inf")), dim=1) @ tv
    (y * torch.tensor(dy)).sum().backward()
    for key, t in (("dq", tq), ("dk", tk), ("dv", tv)):
        assert np.allclose(got[key], t.grad.numpy(), rtol=1e-10, atol=1e-12), key
    for key in ("dWq", "dWk", "dg"):
        assert np.max(np.abs(got[key])) == 0.0


def test_np_map_backward_against_differences_and_its_invariants():
    """phi's two halves each sum to one, so a constant added to either half of dphi changes nothing; the map sees
    f only through its direction, so the gradient along (W, b) itself vanishes; the rest by central differences."""
    r = np.random.default_rng(3)
    x, Wm, b = r.normal(size=(5, 3)), r.normal(size=(3, 4)), 0.2 * r.normal(size=4)
    dphi = r.normal(size=(5, 8))
    dx, dW, db = OB.np_map_backward(x, Wm, b, dphi)
    shifted = dphi.copy()
    shifted[:, :4] += 1.7
    shifted[:, 4:] -= 0.4
    for a_, b_ in zip(OB.np_map_backward(x, Wm, b, shifted), (dx, dW, db)):
        assert np.allclose(a_, b_, rtol=1e-10, atol=1e-12)
    h = 1e-6
    for arr, grad in ((x, dx), (Wm, dW), (b, db)):
        fd = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + h
            up = np.sum(O.np_map(x, Wm, b) * dphi)
            arr[i] = old - h
            dn = np.sum(O.np_map(x, Wm, b) * dphi)
            arr[i] = old
            fd[i] = (up - dn) / (2 * h)
        assert np.allclose(fd, grad, rtol=1e-6, atol=1e-8)
    # scaling f (W and b together) leaves phi unchanged: the gradient along (W, b) itself vanishes
    assert abs(np.sum(dW * Wm) + np.sum(db * b)) < 1e-10


def test_units_driver_adds_nothing_of_its_own():
    r = np.random.default_rng(9)
    B, N, Hq, Hkv, d, F, C = 1, 12, 2, 1, 3, 3, 4
    inputs = dict(q=r.normal(size=(B, N, Hq, d)), k=r.normal(size=(B, N, Hkv, d)), v=r.normal(size=(B, N, Hkv, d)),
                  Wq=r.normal(size=(Hq, d, F)), Wk=r.normal(size=(Hq, d, F)))
    dy = r.normal(size=(B, N, Hq, d))
    sel = np.array([[[[1], [6], [9]], [[0], [5], [11]]]])
    res = OB.still_backward_units(inputs, dy, np.array([0, 0]), [(0, 0), (0, 1)], C, 3, 1, 0.5, 1e-6, sel)
    one = OB.still_backward_definition(inputs["q"][0, :, 1], inputs["k"][0, :, 0], inputs["v"][0, :, 0], None,
                                       inputs["Wq"][1], inputs["Wk"][1], C, 3, 1, 0.5, 1e-6, dy[0, :, 1], sel=sel[0, 1])
    assert np.array_equal(res[(0, 1)]["dk"], one["dk"]) and res[(0, 1)]["dg"] is None


def test_attention_map_rows_sum_to_one_reproduce_the_output_and_reduce_to_softmax():
    """A v equals the forward definition's output when the gate is one; every row sums to one and sees no future
    token; with every token kept the map is the causal softmax map (scipy's softmax, row by row); a token that went
    to the linear state carries the phi_q . phi_k weight, written out for one entry."""
    from scipy.special import softmax

    C, W, lam, scale, eps = 4, 3, 1, 0.6, 1e-6
    p, _ = tiny(21, N=22, gate=False)
    fwd = O.still_definition(p["q"], p["k"], p["v"], None, p["Wq"], p["Wk"], C, W, lam, scale, eps, bq=p["bq"], bk=p["bk"])
    A = OB.attention_map(p["q"], p["k"], p["Wq"], p["Wk"], C, W, lam, scale, eps, bq=p["bq"], bk=p["bk"], sel=fwd["sel"])
    assert np.allclose(A.sum(axis=1), 1.0, rtol=1e-13) and np.all(np.triu(A, 1) == 0.0) and np.all(A >= 0.0)
    assert np.allclose(A @ p["v"], fwd["out"], rtol=1e-11, atol=1e-13)
    # row 21 (chunk 5): token 2 of chunk 0 is un-selected unless the list says otherwise
    t = 21
    j = next(i for i in range(0, 4) if i not in set(fwd["sel"][0]))
    den = np.exp(fwd["M"][t]) * fwd["D_SA"][t] + fwd["D_LA"][t]
    w = O.np_map(p["q"][t], p["Wq"], p["bq"])[0] @ O.np_map(p["k"][j], p["Wk"], p["bk"])[0]
    assert np.isclose(A[t, j], w / den, rtol=1e-12)
    # everything kept: the causal softmax map
    sel_all = np.arange(20).reshape(5, 4)
    A2 = OB.attention_map(p["q"], p["k"], p["Wq"], p["Wk"], C, W, C, scale, eps, sel=sel_all)
    for t in range(22):
        assert np.allclose(A2[t, :t + 1], softmax(scale * p["k"][:t + 1] @ p["q"][t]), rtol=1e-12)


@pytest.mark.parametrize("lam,max_retained", [(1, None), (2, 3)])
def test_attention_map_backward_matches_central_differences(lam, max_retained):
    C, W, scale, eps = 4, 3, 0.6, 1e-6
    p, _ = tiny(31 + lam, N=20, gate=False)
    rng = np.random.default_rng(32)
    dA = np.tril(rng.normal(size=(20, 20)))
    fwd = O.still_definition(p["q"], p["k"], p["v"], None, p["Wq"], p["Wk"], C, W, lam, scale, eps, bq=p["bq"], bk=p["bk"],
                             max_retained=max_retained)
    sel = fwd["sel"]

    def loss():
        A = OB.attention_map(p["q"], p["k"], p["Wq"], p["Wk"], C, W, lam, scale, eps, bq=p["bq"], bk=p["bk"], sel=sel,
                             max_retained=max_retained)
        return float(np.sum(A * dA))

    got = OB.attention_map_backward(p["q"], p["k"], p["Wq"], p["Wk"], C, W, lam, scale, eps, dA, bq=p["bq"], bk=p["bk"],
                                    sel=sel, max_retained=max_retained)
    h = 1e-5
    for name, key in (("Wq", "dWq"), ("Wk", "dWk"), ("bq", "dbq"), ("bk", "dbk")):
        base = p[name]
        fd = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = base[i]
            base[i] = old + h
            up = loss()
            base[i] = old - h
            dn = loss()
            base[i] = old
            fd[i] = (up - dn) / (2 * h)
        assert np.max(np.abs(fd)) > 1e-6, name
        assert np.max(np.abs(fd - got[key])) <= 1e-6 * max(1.0, np.max(np.abs(fd))), name
