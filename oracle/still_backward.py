"""Float64 CPU oracle for the BACKWARD pass of STILL's hybrid attention (arXiv 2602.02180).

TEST INFRASTRUCTURE ONLY (same rules as still_oracle.py: used by tests/, smoke() and the benchmark's
cpu_baseline leg; shares no code with the HIP kernels).

The paper trains the operator in two stages (Sec. 4.1: attention transfer for the feature maps and the gate,
then low-rank adaptation of the projections), so its gradients are part of the method, but the paper prints no
backward equations.  What is differentiated here is the output equation of Sec. 3.3,

    y_t = (N_SA + g_t * N_LA) / (D_SA + D_LA),

row by row over the explicit index sets of still_oracle.still_definition, with the routing (the Top-lambda
index lists) held fixed: the selection is a discrete decision and passes no gradient, and the Self-Saliency
Score only feeds that decision.  Every derivative below is the chain rule on that one equation, on the softmax
branch's exponentials, on the linear branch's phi_q . phi_k weights, and on the NP-Map of Sec. 3.2.

Pins (tests/test_oracle_backward.py): central finite differences of still_definition for every input, the
textbook causal-softmax gradient when every token is kept, the NP-Map's Jacobian and invariances.
attention_map (the weights under the shared normaliser, what the first training stage compares with the teacher's
map) is pinned by A v = y, unit row sums, scipy's softmax when every token is kept and one written-out entry;
attention_map_backward (its gradient w.r.t. the feature-map parameters) by central differences of attention_map.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from .still_oracle import F64, _scores_and_sel, gate_activate, np_map


def np_map_backward(x: np.ndarray, Wm: np.ndarray, b: Optional[np.ndarray], dphi: np.ndarray):
    """Gradient of phi_NP (Sec. 3.2) for rows of x: returns (dx, dW, db).

    Forward: f = x W + b, u = f / ||f|| * ||x||, phi = [softmax(u), softmax(-u)].
    """
    x = np.atleast_2d(np.asarray(x, F64))
    Wm = np.asarray(Wm, F64)
    dphi = np.atleast_2d(np.asarray(dphi, F64))
    F = Wm.shape[1]
    f = x @ Wm
    if b is not None:
        f = f + np.asarray(b, F64)
    nx = np.sqrt(np.sum(x * x, axis=1, keepdims=True))
    nf = np.sqrt(np.sum(f * f, axis=1, keepdims=True))
    ok = (nf > 0) & (nx > 0)
    fh = np.where(ok, f / np.where(nf > 0, nf, 1.0), 0.0)
    u = fh * nx
    ep = np.exp(u - u.max(axis=1, keepdims=True))
    en = np.exp(-u - (-u).max(axis=1, keepdims=True))
    pp = ep / ep.sum(axis=1, keepdims=True)
    pn = en / en.sum(axis=1, keepdims=True)
    dpp, dpn = dphi[:, :F], dphi[:, F:]
    # softmax(u):  du = p * (dp - <p, dp>);  softmax(-u): the same with the sign of u flipped
    du = pp * (dpp - np.sum(pp * dpp, axis=1, keepdims=True)) - pn * (dpn - np.sum(pn * dpn, axis=1, keepdims=True))
    # u = fh * nx with fh = f / nf
    dnx = np.sum(fh * du, axis=1, keepdims=True)
    dfh = du * nx
    df = np.where(ok, (dfh - fh * np.sum(fh * dfh, axis=1, keepdims=True)) / np.where(nf > 0, nf, 1.0), 0.0)
    dx = df @ Wm.T + np.where(nx > 0, dnx * x / np.where(nx > 0, nx, 1.0), 0.0)
    dW = x.T @ df
    db = df.sum(axis=0)
    return dx, dW, db


def still_backward_definition(q, k, v, g, Wq, Wk, C, W, lam, scale, eps, dy, bq=None, bk=None,
                              sel=None, score=None, max_retained: Optional[int] = None,
                              gate_activation: str = "none") -> Dict[str, np.ndarray]:
    """Gradients of sum(dy * y) for ONE (batch, query-head) problem, the routing held fixed.

    Returns dq, dk, dv [N, d]; dg [N, d] (w.r.t. g as passed in: the pre-activation when gate_activation is
    "sigmoid"; None without a gate); dWq, dWk [d, d_f]; dbq, dbk [d_f] (None without biases); and "lse", the
    log of the shared normaliser D_SA + D_LA of every row (natural log, no shift).
    dk and dv are this query head's contribution; heads that share a kv head add theirs up.
    """
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    v = np.asarray(v, F64)
    dy = np.asarray(dy, F64)
    N, d = q.shape
    ga = gate_activate(g, gate_activation)
    score, sel = _scores_and_sel(q, k, C, W, lam, scale, eps, sel, score, max_retained, "stop")
    phi_q = np_map(q, Wq, bq)
    phi_k = np_map(k, Wk, bk)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    dga = np.zeros((N, v.shape[1]), F64)
    dphi_q = np.zeros_like(phi_q)
    dphi_k = np.zeros_like(phi_k)
    lse = np.zeros(N, F64)
    for t in range(N):
        c = t // C
        local = list(range(max(0, (c - 1) * C), t + 1))
        ret, lin = [], []
        for cc in range(0, c - 1):
            chosen = set(int(i) for i in sel[cc] if i >= 0)
            for i in range(cc * C, (cc + 1) * C):
                (ret if i in chosen else lin).append(i)
        sa = np.asarray(ret + local, np.int64)
        li = np.asarray(lin, np.int64)
        e = np.exp(scale * (k[sa] @ q[t]))
        w = phi_k[li] @ phi_q[t] if lin else np.zeros(0, F64)
        gt = ga[t] if ga is not None else np.ones(v.shape[1], F64)
        n_raw = w @ v[li] if lin else np.zeros(v.shape[1], F64)
        den = e.sum() + w.sum()
        y = (e @ v[sa] + gt * n_raw) / den
        lse[t] = np.log(den)
        dnum = dy[t] / den
        dden = -np.dot(dy[t], y) / den
        # softmax branch: weights e_j = exp(scale q.k_j)
        dl = e * (v[sa] @ dnum + dden)
        dv[sa] += np.outer(e, dnum)
        dq[t] += scale * (dl @ k[sa])
        dk[sa] += scale * np.outer(dl, q[t])
        # linear branch: weights w_j = phi_q(q_t) . phi_k(k_j), numerator gated per channel
        if lin:
            dga[t] = dnum * n_raw
            dw = v[li] @ (dnum * gt) + dden
            dv[li] += np.outer(w, dnum * gt)
            dphi_q[t] += dw @ phi_k[li]
            dphi_k[li] += np.outer(dw, phi_q[t])
    dxq, dWq, dbq_ = np_map_backward(q, Wq, bq, dphi_q)
    dxk, dWk, dbk_ = np_map_backward(k, Wk, bk, dphi_k)
    out = {"dq": dq + dxq, "dk": dk + dxk, "dv": dv, "dWq": dWq, "dWk": dWk,
           "dbq": dbq_ if bq is not None else None, "dbk": dbk_ if bk is not None else None,
           "lse": lse, "sel": sel, "dg": None}
    if g is not None:
        if gate_activation == "sigmoid":
            out["dg"] = dga * ga * (1.0 - ga)
        else:
            out["dg"] = dga
    return out


def still_backward_units(inputs: Dict[str, np.ndarray], dy: np.ndarray, kv_map: np.ndarray, units, C, W, lam,
                         scale, eps, sel: np.ndarray, max_retained: Optional[int] = None,
                         gate_activation: str = "none") -> Dict:
    """The listed (b, hq) units of a batched problem (shapes as still_oracle.still_forward_units; dy [B,N,Hq,d];
    sel [B,Hq,N//C,lam] is required: the backward pass never re-ranks)."""
    out = {}
    for (b, h) in units:
        kh = int(kv_map[h])
        g = inputs["g"][b, :, h] if inputs.get("g") is not None else None
        bq = inputs["bq"][h] if inputs.get("bq") is not None else None
        bk = inputs["bk"][h] if inputs.get("bk") is not None else None
        out[(b, h)] = still_backward_definition(
            inputs["q"][b, :, h], inputs["k"][b, :, kh], inputs["v"][b, :, kh], g, inputs["Wq"][h], inputs["Wk"][h],
            C, W, lam, scale, eps, dy[b, :, h], bq=bq, bk=bk, sel=sel[b, h], max_retained=max_retained,
            gate_activation=gate_activation)
    return out


def attention_map(q, k, Wq, Wk, C, W, lam, scale, eps, bq=None, bk=None, sel=None, score=None,
                  max_retained: Optional[int] = None) -> np.ndarray:
    """The operator's attention map for ONE (batch, query-head) problem: A[t, j] = weight of v_j in row t under the
    shared normaliser of the Sec. 3.3 output equation: exp(scale q_t.k_j) / (D_SA + D_LA) for the keys the softmax
    branch sees (local span and retained tokens), phi_q(q_t).phi_k(k_j) / (D_SA + D_LA) for the tokens that went to
    the linear state, 0 for the future.  Every row sums to one; with a gate of ones, y = A v.  (This is the map the
    paper's first training stage compares with the teacher's softmax map, Sec. 4.1; the per-channel gate scales the
    linear part of the numerator only and is not part of a scalar map.)"""
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    N = q.shape[0]
    score, sel = _scores_and_sel(q, k, C, W, lam, scale, eps, sel, score, max_retained, "stop")
    phi_q = np_map(q, Wq, bq)
    phi_k = np_map(k, Wk, bk)
    A = np.zeros((N, N), F64)
    for t in range(N):
        c = t // C
        for j in range(max(0, (c - 1) * C), t + 1):
            A[t, j] = np.exp(scale * np.dot(q[t], k[j]))
        for cc in range(0, c - 1):
            chosen = set(int(i) for i in sel[cc] if i >= 0)
            for j in range(cc * C, (cc + 1) * C):
                A[t, j] = np.exp(scale * np.dot(q[t], k[j])) if j in chosen else np.dot(phi_q[t], phi_k[j])
        A[t] /= A[t].sum()
    return A


def attention_map_backward(q, k, Wq, Wk, C, W, lam, scale, eps, dA, bq=None, bk=None, sel=None, score=None,
                           max_retained: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Gradient of sum(dA * A) (A = attention_map) w.r.t. the feature-map parameters W_q, W_k, b_q, b_k, with q, k
    and the routing held fixed: what the first training stage of Sec. 4.1 updates (q and k come from the frozen
    teacher there).  A_tj = a_tj / s_t with s_t the row's sum, so da_tj = (dA_tj - <dA_t, A_t>) / s_t; only the
    pairs owned by the linear branch depend on the parameters, through a_tj = phi_q(q_t) . phi_k(k_j)."""
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    dA = np.asarray(dA, F64)
    N = q.shape[0]
    score, sel = _scores_and_sel(q, k, C, W, lam, scale, eps, sel, score, max_retained, "stop")
    phi_q = np_map(q, Wq, bq)
    phi_k = np_map(k, Wk, bk)
    dphi_q = np.zeros_like(phi_q)
    dphi_k = np.zeros_like(phi_k)
    for t in range(N):
        c = t // C
        a = np.zeros(N, F64)
        lin = []
        for j in range(max(0, (c - 1) * C), t + 1):
            a[j] = np.exp(scale * np.dot(q[t], k[j]))
        for cc in range(0, c - 1):
            chosen = set(int(i) for i in sel[cc] if i >= 0)
            for j in range(cc * C, (cc + 1) * C):
                if j in chosen:
                    a[j] = np.exp(scale * np.dot(q[t], k[j]))
                else:
                    a[j] = np.dot(phi_q[t], phi_k[j])
                    lin.append(j)
        if not lin:
            continue
        s = a.sum()
        da = (dA[t] - np.dot(dA[t], a / s)) / s
        li = np.asarray(lin, np.int64)
        dphi_q[t] += da[li] @ phi_k[li]
        dphi_k[li] += np.outer(da[li], phi_q[t])
    _, dWq, dbq_ = np_map_backward(q, Wq, bq, dphi_q)
    _, dWk, dbk_ = np_map_backward(k, Wk, bk, dphi_k)
    return {"dWq": dWq, "dWk": dWk, "dbq": dbq_ if bq is not None else None, "dbk": dbk_ if bk is not None else None}
