"""GPU parity of the decode step (recurrent form) against the oracle.

The oracle for decode is the prefill oracle on the concatenated sequence (causality: appending tokens
never changes earlier rows, pinned in test_oracle_pins.py); the rows of the decoded tokens are compared.
The indices the HIP path kept at each routing step are read back from the state and injected into the
oracle after being checked against the oracle's own Top-lambda (exact wherever the score gap > 1e-5).
"""
import numpy as np
import pytest

from oracle import still_oracle as O
from paper_2602_02180_amd import binding as S
from paper_2602_02180_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def run_decode(w, inp, n_prefill, n_total, kv_map=None, with_gate=False, gate_activation=0, budget_policy=0):
    """Prefill tokens [0, n_prefill) with state_out (or start from an empty state), then decode up to n_total."""
    import torch

    dev = "cuda"
    full = {k: synth.to_torch(inp[k], w.dtype, dev) for k in ("q", "k", "v", "Wq", "Wk")}
    g_full = synth.to_torch(inp["g"], w.dtype, dev) if with_gate else None
    bq = synth.to_torch(inp["bq"], w.dtype, dev) if inp.get("bq") is not None else None
    bk = synth.to_torch(inp["bk"], w.dtype, dev) if inp.get("bk") is not None else None
    B = w.B
    out = torch.full((B, n_total, w.Hq, w.d), float("nan"), dtype=full["q"].dtype, device=dev)
    base = dict(B=B, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps, dtype=w.dtype,
                d_f=w.df, kv_head_of_q=kv_map, max_tokens=n_total, max_retained=w.max_retained, shared_selection=w.shared_selection,
                gate_activation=gate_activation, budget_policy=budget_policy)
    ps = S.make_params(N=1, **base)
    state = torch.empty(S.still_state_bytes(ps), dtype=torch.uint8, device=dev)
    S.still_state_init(ps, state)
    if n_prefill > 0:
        q0, k0, v0 = (full[n][:, :n_prefill].contiguous() for n in ("q", "k", "v"))
        g0 = g_full[:, :n_prefill].contiguous() if with_gate else None
        o0 = torch.empty_like(q0)
        p0 = S.make_params(N=n_prefill, q=q0, k=k0, v=v0, out=o0, g=g0, **base)
        ws = torch.empty(S.still_fwd_workspace_bytes(p0), dtype=torch.uint8, device=dev)
        S.still_hybrid_attn_fwd(p0, q0, k0, v0, g0, full["Wq"], bq, full["Wk"], bk, o0, state_out=state,
                                workspace=ws)
        out[:, :n_prefill] = o0
    for t in range(n_prefill, n_total):
        qt = full["q"][:, t].contiguous()
        kt = full["k"][:, t].contiguous()
        vt = full["v"][:, t].contiguous()
        gt = g_full[:, t].contiguous() if with_gate else None
        ot = torch.empty_like(qt)
        S.still_hybrid_attn_decode_step(ps, state, t, qt, kt, vt, gt, full["Wq"], bq, full["Wk"], bk, ot)
        out[:, t] = ot
    torch.cuda.synchronize()
    L = S.still_state_layout(ps)
    n_routed = max(0, (n_total - 1) // w.C - 1)
    sel = state[L.sel:L.sel + B * w.Hq * L.n_chunks * max(w.lam, 1) * 4].view(torch.int32)
    sel = sel.reshape(B, w.Hq, L.n_chunks, max(w.lam, 1)).cpu().numpy().astype(np.int64)[:, :, :n_routed, :w.lam]
    return synth.from_torch(out), sel


def run_decode_staggered(w, inp, n_total, offsets, tight_bound=True, budget_policy=0):
    """Sequence b joins at step offsets[b] with an empty state and then appends one token per step through
    still_hybrid_attn_decode_step_at; before joining and after its last token it sits the step out (-1)."""
    import torch

    dev = "cuda"
    full = {k: synth.to_torch(inp[k], w.dtype, dev) for k in ("q", "k", "v", "Wq", "Wk")}
    B = w.B
    out = torch.full((B, n_total, w.Hq, w.d), float("nan"), dtype=full["q"].dtype, device=dev)
    ps = S.make_params(B=B, N=1, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                       dtype=w.dtype, d_f=w.df, max_tokens=n_total, max_retained=w.max_retained, shared_selection=w.shared_selection,
                       budget_policy=budget_policy)
    state = torch.empty(S.still_state_bytes(ps), dtype=torch.uint8, device=dev)
    S.still_state_init(ps, state)
    ar = torch.arange(B, device=dev)
    sentinel = torch.full((B, w.Hq, w.d), 12345.0, dtype=full["q"].dtype, device=dev)
    for s in range(n_total + max(offsets)):
        pos = [s - o if 0 <= s - o < n_total else -1 for o in offsets]
        live = [b for b in range(B) if pos[b] >= 0]
        t_dev = torch.tensor(pos, dtype=torch.int32, device=dev)
        rd = torch.tensor([max(p, 0) for p in pos], device=dev)
        qt, kt, vt = (full[n][ar, rd].contiguous() for n in ("q", "k", "v"))
        ot = sentinel.clone()
        t_max = max(pos) if tight_bound else n_total - 1
        S.still_hybrid_attn_decode_step_at(ps, state, t_dev, t_max, qt, kt, vt, None, full["Wq"], None, full["Wk"],
                                           None, ot)
        for b in range(B):
            if pos[b] >= 0:
                out[b, pos[b]] = ot[b]
            else:
                assert torch.equal(ot[b], sentinel[b]), f"step {s}: idle sequence {b} was written"
        assert live
    torch.cuda.synchronize()
    L = S.still_state_layout(ps)
    n_routed = max(0, (n_total - 1) // w.C - 1)
    sel = state[L.sel:L.sel + B * w.Hq * L.n_chunks * max(w.lam, 1) * 4].view(torch.int32)
    sel = sel.reshape(B, w.Hq, L.n_chunks, max(w.lam, 1)).cpu().numpy().astype(np.int64)[:, :, :n_routed, :w.lam]
    return synth.from_torch(out), sel


def check_decode(w, inp, n_prefill, n_total, with_gate=False, result=None, gate_activation=0, budget_policy=0):
    got, sel_h = result if result is not None else run_decode(w, inp, n_prefill, n_total, with_gate=with_gate,
                                                              gate_activation=gate_activation,
                                                              budget_policy=budget_policy)
    act = "sigmoid" if gate_activation else "none"
    policy = "evict" if budget_policy else "stop"
    offer_budget = None if budget_policy else U.budget(w)      # under eviction every chunk offers its full Top-lambda
    kv_map = synth.kv_head_map(w)
    sub = {k: (v[:, :n_total] if k in ("q", "k", "v", "g") else v) for k, v in inp.items() if k != "heavy"}
    if not with_gate:
        sub.pop("g", None)
    worst = 0.0
    for b in range(w.B):
        for h in range(w.Hq):
            own = O.still_forward_units(sub, kv_map, [(b, h)], C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                                        max_retained=U.budget(w), shared_selection=w.shared_selection,
                                        budget_policy=policy)[(b, h)]
            n_routed = sel_h.shape[2]
            ncf = n_total // w.C
            sel_full = own["sel"].copy()
            # routed chunks: the HIP path's choice must be the oracle's wherever the gap is clear
            gaps = O.selection_gaps(own["rank_score"], w.C, w.lam, offer_budget)
            if budget_policy:      # the case must be well-posed: no eviction decided by less than the score tolerance
                margins = O.eviction_margins(own["rank_score"], own["sel"], w.max_retained)[:n_routed]
                assert margins.min() > 1e-5, f"ill-posed eviction case (margin {margins.min():.2e}): pick another seed"
            for c in range(n_routed):
                if gaps[c] > 1e-5:
                    assert np.array_equal(sel_h[b, h, c], own["sel"][c]), (b, h, c)
                quota = O.chunk_quota(c, w.lam, offer_budget)
                assert np.all(sel_h[b, h, c][:quota] >= 0) and np.all(sel_h[b, h, c][quota:] == -1), (b, h, c)
                sel_full[c] = sel_h[b, h, c]
            ref = O.still_forward_units(sub, kv_map, [(b, h)], C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                                        sel=sel_full[None, None].repeat(w.B, 0).repeat(w.Hq, 1),
                                        gate_activation=act, budget_policy=policy,
                                        max_retained=U.budget(w) if budget_policy else None)[(b, h)]
            x = got[b, n_prefill:n_total, h].astype(np.float64)
            y = ref["out"][n_prefill:n_total]
            assert np.all(np.isfinite(x))
            if w.dtype == "f32":
                err = max(U.rel_err(x, y), U.row_rel_err(x, y))
                assert err <= 1e-4, (b, h, err)
            else:
                err = U.assert_bf16_bar(x, y, f"decode unit {(b, h)}")["bar_fraction"]
            worst = max(worst, err)
    print(f"[decode {w.name} prefill={n_prefill} total={n_total}] worst error measure {worst:.3e}")


def wl(name, **kw):
    base = dict(B=1, N=512, Hq=2, Hkv=1, d=64, C=64, W=64, lam=16, dtype="f32")
    base.update(kw)
    return synth.Workload(name, **base)


@pytest.mark.parametrize("kw,n_total", [
    (dict(dtype="f32", d=64, C=64, W=64), 300),
    (dict(dtype="bf16", d=128, C=64, W=128, Hq=4, Hkv=2, B=2), 330),
    (dict(dtype="f32", d=64, C=128, W=100, lam=5), 400),
])
def test_decode_from_empty_state(kw, n_total):
    w = wl("dec0", **kw)
    inp = synth.make_inputs(w, seed=21, n_tokens=n_total)
    check_decode(w, inp, 0, n_total)


@pytest.mark.parametrize("kw,n_prefill,n_total", [
    (dict(dtype="f32", d=64, C=64, W=64), 200, 340),            # prefill ends inside a chunk
    (dict(dtype="f32", d=64, C=64, W=64), 256, 400),            # prefill ends on a chunk boundary
    (dict(dtype="bf16", d=128, C=128, W=128, Hq=4, Hkv=2), 700, 1000),
    (dict(dtype="bf16", d=64, C=64, W=33, lam=0), 130, 300),
    (dict(dtype="f32", d=64, C=64, W=64, lam=64), 130, 300),
    (dict(dtype="f32", d=64, C=64, W=64), 50, 200),             # prefill shorter than a chunk
])
def test_decode_continues_prefill(kw, n_prefill, n_total):
    w = wl("dec1", **kw)
    inp = synth.make_inputs(w, seed=22, n_tokens=n_total)
    check_decode(w, inp, n_prefill, n_total)


@pytest.mark.parametrize("kw,n_prefill,n_total", [
    (dict(dtype="f32", d=64, C=64, W=64, lam=16, max_retained=40), 0, 520),        # budget fills during decode
    (dict(dtype="f32", d=64, C=64, W=64, lam=16, max_retained=40), 300, 600),      # fills across the hand-over
    (dict(dtype="bf16", d=128, C=128, W=128, lam=16, max_retained=24, Hq=4, Hkv=2), 700, 1100),  # full at prefill
])
def test_decode_with_retained_budget(kw, n_prefill, n_total):
    _decode_with_retained_budget(kw, n_prefill, n_total)


@pytest.mark.parametrize("kw,n_prefill,n_total", [
    (dict(dtype="f32", d=64, C=64, W=64, Hq=4, Hkv=2), 0, 330),
    (dict(dtype="f32", d=64, C=64, W=64, Hq=4, Hkv=2, max_retained=40), 200, 460),
    (dict(dtype="bf16", d=128, C=128, W=128, Hq=8, Hkv=2, B=2), 700, 1000),
])
def test_decode_with_group_shared_selection(kw, n_prefill, n_total):
    """Variant: one list per kv head, ranked by the summed score of its query heads, in prefill and decode alike."""
    w = wl("decs", shared_selection=True, **kw)
    inp = synth.make_inputs(w, seed=26, n_tokens=n_total)
    check_decode(w, inp, n_prefill, n_total)


def _decode_with_retained_budget(kw, n_prefill, n_total):
    """The state's retained rows stop growing at the budget; outputs keep following the oracle."""
    w = wl("decb", **kw)
    inp = synth.make_inputs(w, seed=23, n_tokens=n_total)
    check_decode(w, inp, n_prefill, n_total)
    p = S.make_params(B=w.B, N=1, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, max_tokens=1 << 20, max_retained=w.max_retained, shared_selection=w.shared_selection)
    assert S.still_state_layout(p).cap <= (w.max_retained + 63) // 64 * 64 + 64


@pytest.mark.parametrize("kw,n_prefill,n_total", [
    (dict(dtype="f32", d=128, C=128, W=128, lam=8), 0, 420),      # routing update: two image pieces x two parts
    (dict(dtype="f32", d=128, C=64, W=64, lam=8), 150, 300),
    (dict(dtype="bf16", d=64, C=128, W=96, lam=12), 300, 560),
])
def test_decode_with_feature_map_biases(kw, n_prefill, n_total):
    """The NP-Map's linear layers with biases (Sec. 3.2: f is a learnable layer), prefill hand-over and routing."""
    w = wl("decbias", **kw)
    inp = synth.make_inputs(w, seed=27, n_tokens=n_total)
    rng = np.random.default_rng(5)
    inp["bq"] = synth.round_to_dtype(rng.standard_normal((w.Hq, w.df)) * 0.1, w.dtype)
    inp["bk"] = synth.round_to_dtype(rng.standard_normal((w.Hq, w.df)) * 0.1, w.dtype)
    check_decode(w, inp, n_prefill, n_total)


@pytest.mark.parametrize("kw,n_total", [
    (dict(dtype="f32", d=64, C=64, W=64, lam=16, max_retained=40), 700),          # fills at chunk 2, then evicts
    (dict(dtype="f32", d=64, C=64, W=48, lam=16, max_retained=5), 400),           # budget below one chunk's offer
    (dict(dtype="bf16", d=128, C=128, W=128, lam=16, max_retained=24, Hq=4, Hkv=2, B=2), 1300),
    (dict(dtype="f32", d=128, C=64, W=64, lam=8, max_retained=16), 600),
])
def test_decode_with_eviction_policy(kw, n_total):
    """Budget policy 1 (a variant of this library): the retained rows are the best-scored offers so far, a row that
    leaves enters the state at that routing step; decode from an empty state against the oracle's same policy."""
    w = wl("decev", **kw)
    inp = synth.make_inputs(w, seed=29, n_tokens=n_total)
    check_decode(w, inp, 0, n_total, budget_policy=1)


@pytest.mark.parametrize("kw,n_prefill,n_total", [
    (dict(dtype="f32", d=64, C=64, W=64, lam=16, max_retained=40), 300, 700),     # the budget is full at the hand-over
    (dict(dtype="f32", d=64, C=64, W=64, lam=16, max_retained=40), 130, 500),     # fills during decode
    (dict(dtype="bf16", d=128, C=128, W=128, lam=16, max_retained=24, Hq=4, Hkv=2), 700, 1200),
])
def test_decode_continues_prefill_with_eviction_policy(kw, n_prefill, n_total):
    """The prefill exports the set retained after its last routed step, with scores and token indices; the decode
    steps go on evicting from it."""
    w = wl("decev2", **kw)
    inp = synth.make_inputs(w, seed=30, n_tokens=n_total)
    check_decode(w, inp, n_prefill, n_total, budget_policy=1)


@pytest.mark.parametrize("kw,n_prefill,n_total", [
    (dict(dtype="f32", d=64, C=64, W=200), 0, 420),             # 256 threads score the new token
    (dict(dtype="f32", d=64, C=64, W=256, lam=8), 300, 600),    # the window spans the whole ring
    (dict(dtype="bf16", d=128, C=128, W=160, Hq=4, Hkv=2), 500, 900),
])
def test_decode_with_wide_score_windows(kw, n_prefill, n_total):
    w = wl("decwide", **kw)
    inp = synth.make_inputs(w, seed=31, n_tokens=n_total)
    check_decode(w, inp, n_prefill, n_total)


def test_decode_with_gate():
    w = wl("decg", dtype="f32", d=64, C=64, W=64, lam=8)
    inp = synth.make_inputs(w, seed=23, n_tokens=280, with_gate=True)
    check_decode(w, inp, 150, 280, with_gate=True)


def test_decode_with_sigmoid_gate_from_preactivation():
    """gate_activation = 1 through prefill, hand-over and decode steps: the gate arrives as a pre-activation."""
    w = wl("decsg", dtype="f32", d=64, C=64, W=64, lam=8)
    inp = synth.make_inputs(w, seed=29, n_tokens=280)
    rng = np.random.default_rng(30)
    inp["g"] = synth.round_to_dtype(2.0 * rng.standard_normal(inp["q"].shape), w.dtype)
    check_decode(w, inp, 150, 280, with_gate=True, gate_activation=1)


def test_decode_rejects_token_beyond_capacity():
    import torch

    w = wl("deccap")
    ps = S.make_params(B=1, N=1, Hq=2, Hkv=1, d=64, C=64, W=64, lam=16, scale=0.125, eps=1e-6, dtype="f32",
                       max_tokens=128)
    state = torch.empty(S.still_state_bytes(ps), dtype=torch.uint8, device="cuda")
    S.still_state_init(ps, state)
    x = torch.zeros((1, 2, 64), device="cuda")
    kx = torch.zeros((1, 1, 64), device="cuda")
    Wm = torch.zeros((2, 64, 64), device="cuda")
    with pytest.raises(S.StillError) as e:
        S.still_hybrid_attn_decode_step(ps, state, 128, x, kx, kx, None, Wm, None, Wm, None, torch.empty_like(x))
    assert e.value.code == S.STILL_ERR_STATE


def test_decode_at_long_context_sampled_unit():
    """The benchmark's decode shape (8B layer, 32K context, C = W = 128, heavy-hitter keys) with a small batch:
    prefill 32768 tokens with state_out, 130 decode steps (one routing step), one sampled (batch, head) unit
    against the oracle."""
    w = synth.workload("c4", B=2)
    n_prefill, n_total = w.N, w.N + 130
    inp = synth.make_inputs(w, n_tokens=n_total)
    got, sel_h = run_decode(w, inp, n_prefill, n_total)
    kv_map = synth.kv_head_map(w)
    b, h = 1, 21
    own = O.still_forward_units(inp, kv_map, [(b, h)], C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                                rows=(n_prefill, n_total))[(b, h)]
    gaps = O.selection_gaps(own["rank_score"], w.C, w.lam, U.budget(w))
    n_routed = sel_h.shape[2]
    sel_full = own["sel"].copy()
    mism = 0
    for c in range(n_routed):
        same = np.array_equal(sel_h[b, h, c], own["sel"][c])
        assert same or gaps[c] <= 1e-5, c
        mism += not same
        sel_full[c] = sel_h[b, h, c]
    sel_arr = np.zeros((w.B, w.Hq) + sel_full.shape, np.int64)
    sel_arr[b, h] = sel_full
    ref = O.still_forward_units(inp, kv_map, [(b, h)], C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                                sel=sel_arr, rows=(n_prefill, n_total))[(b, h)]
    x = got[b, n_prefill:n_total, h].astype(np.float64)
    y = ref["out"][n_prefill:n_total]
    print(f"[decode long] routed chunks {n_routed}, near-tie flips {mism}")
    assert np.all(np.isfinite(x))
    U.assert_bf16_bar(x, y, "decode long")


@pytest.mark.parametrize("kw,n_total,offsets,tight", [
    (dict(dtype="f32", d=64, C=64, W=64, B=3), 300, [0, 37, 100], True),
    (dict(dtype="f32", d=64, C=64, W=64, B=3, lam=16, max_retained=24), 300, [64, 0, 1], False),
    (dict(dtype="bf16", d=128, C=128, W=128, B=4, Hq=4, Hkv=2), 520, [0, 128, 5, 300], True),
])
def test_decode_sequences_at_their_own_positions(kw, n_total, offsets, tight):
    """Continuous batching: every sequence of the batch is at a different token, routes its chunks at its own
    steps, and some sequences sit steps out; each must still follow the oracle on its own tokens."""
    w = wl("decat", **kw)
    inp = synth.make_inputs(w, seed=24, n_tokens=n_total)
    check_decode(w, inp, 0, n_total, result=run_decode_staggered(w, inp, n_total, offsets, tight_bound=tight))


def test_decode_sequences_at_their_own_positions_with_eviction_policy():
    """The same with the budget held by eviction: every sequence evicts at its own routing steps."""
    w = wl("decatev", dtype="f32", d=64, C=64, W=64, B=3, lam=16, max_retained=24)
    n_total, offsets = 420, [64, 0, 1]
    inp = synth.make_inputs(w, seed=32, n_tokens=n_total)
    check_decode(w, inp, 0, n_total, budget_policy=1,
                 result=run_decode_staggered(w, inp, n_total, offsets, tight_bound=False, budget_policy=1))


def test_decode_step_at_replays_from_a_hip_graph():
    """One captured step, replayed for every token: the positions live on the device and are advanced there, the
    token inputs are copied into the captured buffers.  Every replay must give the bits of the eager lock-step run
    (same kernels, same launch shape: the bound passed at capture is the last position)."""
    import torch

    n_total = 200
    w = wl("decgraph", dtype="bf16", d=128, C=64, W=64, B=2, Hq=4, Hkv=2)
    inp = synth.make_inputs(w, seed=25, n_tokens=n_total)
    dev = "cuda"
    full = {k: synth.to_torch(inp[k], w.dtype, dev) for k in ("q", "k", "v", "Wq", "Wk")}
    ps = S.make_params(B=w.B, N=1, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                       dtype=w.dtype, d_f=w.df, max_tokens=n_total)

    def fresh_state():
        st = torch.empty(S.still_state_bytes(ps), dtype=torch.uint8, device=dev)
        S.still_state_init(ps, st)
        return st

    # eager reference with the same launch shape (t_max = n_total - 1 at every step)
    state = fresh_state()
    eager = torch.empty(w.B, n_total, w.Hq, w.d, dtype=full["q"].dtype, device=dev)
    for t in range(n_total):
        t_dev = torch.full((w.B,), t, dtype=torch.int32, device=dev)
        ot = torch.empty(w.B, w.Hq, w.d, dtype=full["q"].dtype, device=dev)
        S.still_hybrid_attn_decode_step_at(ps, state, t_dev, n_total - 1, full["q"][:, t].contiguous(),
                                           full["k"][:, t].contiguous(), full["v"][:, t].contiguous(), None,
                                           full["Wq"], None, full["Wk"], None, ot)
        eager[:, t] = ot
    torch.cuda.synchronize()

    state = fresh_state()
    t_dev = torch.zeros(w.B, dtype=torch.int32, device=dev)
    qt, kt, vt = (full[n][:, 0].contiguous() for n in ("q", "k", "v"))
    ot = torch.empty_like(qt)

    def call():
        S.still_hybrid_attn_decode_step_at(ps, state, t_dev, n_total - 1, qt, kt, vt, None, full["Wq"], None,
                                           full["Wk"], None, ot, stream=torch.cuda.current_stream())

    t_dev.fill_(-1)          # warm-up call in which every sequence sits out: the state stays empty
    call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    t_dev.fill_(0)
    for t in range(n_total):
        qt.copy_(full["q"][:, t]); kt.copy_(full["k"][:, t]); vt.copy_(full["v"][:, t])
        ot.fill_(float("nan"))
        graph.replay()
        if t % 50 == 0:
            torch.cuda.synchronize()       # the program's own synchronisations between replays
        assert torch.equal(ot, eager[:, t]), f"replay for token {t} differs from the eager step"
        t_dev.add_(1)


@pytest.mark.parametrize("kw,lens,steps", [
    (dict(dtype="f32", d=64, C=64, W=64, B=3), [1000, 517, 130], 70),
    (dict(dtype="bf16", d=128, C=128, W=128, B=4, Hq=4, Hkv=2), [900, 1300, 128, 40], 140),
    (dict(dtype="f32", d=64, C=64, W=64, B=2, lam=16, max_retained=40, shared_selection=True, Hq=4, Hkv=2),
     [640, 300], 70),
])
def test_right_padded_prefill_then_decode_at_own_positions(kw, lens, steps):
    """A batch of sequences of different lengths, right-padded (the padding holds NaN): every real row must equal
    the oracle on that sequence alone, padding rows of `out` stay untouched, and the exported state lets every
    sequence go on decoding from its own length."""
    import torch

    w = wl("varlen", **kw)
    dev = "cuda"
    n_pad = max(lens)
    n_all = n_pad + steps
    inp = synth.make_inputs(w, seed=27, n_tokens=n_all)
    full = {k: synth.to_torch(inp[k], w.dtype, dev) for k in ("q", "k", "v", "Wq", "Wk")}
    q0, k0, v0 = (full[n][:, :n_pad].clone() for n in ("q", "k", "v"))
    for b, n in enumerate(lens):
        for x in (q0, k0, v0):
            x[b, n:] = float("nan")
    o0 = torch.full_like(q0, 768.0)
    seq_len = torch.tensor(lens, dtype=torch.int32, device=dev)
    base = dict(B=w.B, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps, dtype=w.dtype,
                d_f=w.df, max_tokens=n_all, max_retained=w.max_retained, shared_selection=w.shared_selection)
    ps = S.make_params(N=1, **base)
    state = torch.empty(S.still_state_bytes(ps), dtype=torch.uint8, device=dev)
    S.still_state_init(ps, state)
    p0 = S.make_params(N=n_pad, q=q0, k=k0, v=v0, out=o0, seq_len=seq_len, **base)
    ws = torch.empty(S.still_fwd_workspace_bytes(p0), dtype=torch.uint8, device=dev)
    S.still_hybrid_attn_fwd(p0, q0, k0, v0, None, full["Wq"], None, full["Wk"], None, o0, state_out=state,
                            workspace=ws)
    dec = torch.empty(w.B, steps, w.Hq, w.d, dtype=q0.dtype, device=dev)
    ar = torch.arange(w.B, device=dev)
    for s in range(steps):
        t_dev = seq_len + s
        idx = t_dev.long()
        qt, kt, vt = (full[n][ar, idx].contiguous() for n in ("q", "k", "v"))
        ot = torch.empty_like(qt)
        S.still_hybrid_attn_decode_step_at(ps, state, t_dev, max(lens) + s, qt, kt, vt, None, full["Wq"], None,
                                           full["Wk"], None, ot)
        dec[:, s] = ot
    torch.cuda.synchronize()
    pre, dec = synth.from_torch(o0), synth.from_torch(dec)
    L = S.still_state_layout(ps)
    sel_state = state[L.sel:L.sel + w.B * w.Hq * L.n_chunks * w.lam * 4].view(torch.int32)
    sel_state = sel_state.reshape(w.B, w.Hq, L.n_chunks, w.lam).cpu().numpy().astype(np.int64)
    kv_map = synth.kv_head_map(w)
    worst = 0.0
    for b, n in enumerate(lens):
        assert np.all(pre[b, n:] == 768.0), f"sequence {b}: padding rows of out were written"
        total = n + steps
        one = {k: (v[b:b + 1, :total] if k in ("q", "k", "v") else v) for k, v in inp.items() if k != "heavy"}
        for h in range(w.Hq):
            own = O.still_forward_units(one, kv_map, [(0, h)], C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                                        max_retained=U.budget(w), shared_selection=w.shared_selection)[(0, h)]
            n_routed = max(0, (total - 1) // w.C - 1)
            gaps = O.selection_gaps(own["rank_score"], w.C, w.lam, U.budget(w))
            sel_full = own["sel"].copy()
            for c in range(n_routed):
                if gaps[c] > 1e-5:
                    assert np.array_equal(sel_state[b, h, c], own["sel"][c]), (b, h, c)
                sel_full[c] = sel_state[b, h, c]
            ref = O.still_forward_units(one, kv_map, [(0, h)], C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                                        sel=np.broadcast_to(sel_full, (1, w.Hq) + sel_full.shape))[(0, h)]
            x = np.concatenate([pre[b, :n, h], dec[b, :, h]]).astype(np.float64)
            y = ref["out"][:total]
            assert np.all(np.isfinite(x)), (b, h)
            if w.dtype == "f32":
                err = max(U.rel_err(x, y), U.row_rel_err(x, y))
                assert err <= 1e-4, (b, h, err)
            else:
                err = U.assert_bf16_bar(x, y, f"decode unit {(b, h)}")["bar_fraction"]
            worst = max(worst, err)
    print(f"[varlen {lens} + {steps} decode steps] worst error measure {worst:.3e}")


def test_decode_in_the_benchmark_launch_configuration():
    """Config 5's launch shape (B = 64 sequences, 32K context, one workgroup per (sequence, head) and no split of the
    cache rows): the state of two prefilled sequences is replicated 32 times, 130 steps are decoded for all 64, and
    a sampled unit of a late copy is compared with the oracle."""
    import torch

    w = synth.workload("c4", B=2)
    n_prefill, steps, B = w.N, 130, 64
    n_total = n_prefill + steps
    inp = synth.make_inputs(w, n_tokens=n_total)
    dev = "cuda"
    full = {k: synth.to_torch(inp[k], w.dtype, dev) for k in ("q", "k", "v", "Wq", "Wk")}
    base = dict(Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps, dtype=w.dtype,
                d_f=w.df, max_tokens=n_total)
    p2 = S.make_params(B=2, N=1, **base)
    p64 = S.make_params(B=B, N=1, **base)
    L2, L64 = S.still_state_layout(p2), S.still_state_layout(p64)
    st2 = torch.empty(S.still_state_bytes(p2), dtype=torch.uint8, device=dev)
    q0, k0, v0 = (full[n][:, :n_prefill].contiguous() for n in ("q", "k", "v"))
    o0 = torch.empty_like(q0)
    pf = S.make_params(B=2, N=n_prefill, q=q0, k=k0, v=v0, out=o0, **base)
    ws = torch.empty(S.still_fwd_workspace_bytes(pf), dtype=torch.uint8, device=dev)
    S.still_hybrid_attn_fwd(pf, q0, k0, v0, None, full["Wq"], None, full["Wk"], None, o0, state_out=st2, workspace=ws)
    del ws, o0
    st = torch.empty(S.still_state_bytes(p64), dtype=torch.uint8, device=dev)
    S.still_state_init(p64, st)
    es, d, Hq, Hkv = 2, w.d, w.Hq, w.Hkv
    assert L2.cap == L64.cap and L2.R == L64.R
    per_seq = {"S": 4 * 2 * d * (d + 1) * Hq, "kret": es * L64.cap * d * Hq, "vret": es * L64.cap * d * Hq,
               "sel": 4 * L64.n_chunks * w.lam * Hq, "kring": es * L64.R * d * Hkv, "vring": es * L64.R * d * Hkv,
               "score": 4 * L64.R * Hq}
    for name, n in per_seq.items():
        src = st2[getattr(L2, name): getattr(L2, name) + 2 * n].reshape(2, n)
        st[getattr(L64, name): getattr(L64, name) + B * n].reshape(B // 2, 2, n).copy_(src.unsqueeze(0).expand(B // 2, 2, n))
    nsplit_rows = (n_prefill // w.C - 1) * w.lam + 2 * w.C
    assert (1024 + B * Hq - 1) // (B * Hq) == 1 and nsplit_rows > 64      # one workgroup per unit, as in the bench
    b_probe, h = 37, 21                                                   # a copy of sequence 1
    got = torch.empty(steps, w.d, dtype=full["q"].dtype, device=dev)
    for s in range(steps):
        t = n_prefill + s
        qt, kt, vt = (full[n][:, t].repeat(B // 2, 1, 1).contiguous() for n in ("q", "k", "v"))
        ot = torch.empty_like(qt)
        S.still_hybrid_attn_decode_step(p64, st, t, qt, kt, vt, None, full["Wq"], None, full["Wk"], None, ot)
        got[s] = ot[b_probe, h]
    torch.cuda.synchronize()
    n_routed = max(0, (n_total - 1) // w.C - 1)
    sel_state = st[L64.sel: L64.sel + B * Hq * L64.n_chunks * w.lam * 4].view(torch.int32)
    sel_state = sel_state.reshape(B, Hq, L64.n_chunks, w.lam)[b_probe, h, :n_routed].cpu().numpy().astype(np.int64)
    kv_map = synth.kv_head_map(w)
    own = O.still_forward_units(inp, kv_map, [(1, h)], C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                                rows=(n_prefill, n_total))[(1, h)]
    gaps = O.selection_gaps(own["rank_score"], w.C, w.lam)
    sel_full = own["sel"].copy()
    for c in range(n_routed):
        assert np.array_equal(sel_state[c], own["sel"][c]) or gaps[c] <= 1e-5, c
        sel_full[c] = sel_state[c]
    sel_arr = np.zeros((2, Hq) + sel_full.shape, np.int64)
    sel_arr[1, h] = sel_full
    ref = O.still_forward_units(inp, kv_map, [(1, h)], C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                                sel=sel_arr, rows=(n_prefill, n_total))[(1, h)]
    x = synth.from_torch(got).astype(np.float64)
    y = ref["out"][n_prefill:n_total]
    assert np.all(np.isfinite(x))
    U.assert_bf16_bar(x, y, "decode B=64")
