"""GPU parity of the backward pass (still_hybrid_attn_bwd through the C ABI) against the float64 backward oracle on
the same seeded, dtype-rounded inputs, with the index lists the HIP forward pass chose.

Bars: every gradient tensor within 1e-4 of its largest magnitude on fp32 (measured ~1e-6), within 1e-2 of it on
bf16 (measured 2-5e-3: the operands of the matrix core and the stored results carry 8 bits of mantissa, the sums are
fp32); the log normaliser that the forward pass leaves for the backward pass within 1e-5 relative (fp32) / 2e-2
absolute (bf16).  dk, dv are compared after the oracle's per-head parts are added up over the query heads of a kv
head, parameter gradients after adding up the batch."""
import numpy as np
import pytest

from oracle import still_backward as OB
from paper_2602_02180_amd import binding as S
from paper_2602_02180_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

BAR = {"f32": 1e-4, "bf16": 1e-2}


def small(name, **kw):
    base = dict(B=1, N=512, Hq=2, Hkv=1, d=64, C=64, W=64, lam=16, dtype="f32")
    base.update(kw)
    return synth.Workload(name, **base)


def make_dy(w, inp, seed):
    rng = np.random.default_rng(seed)
    return synth.round_to_dtype(rng.standard_normal(inp["q"].shape).astype(np.float32), w.dtype)


def oracle_grads(w, inp, dy, sel, kv_map, gate_activation="none"):
    B, N = inp["q"].shape[:2]
    units = [(b, h) for b in range(B) for h in range(w.Hq)]
    ref = OB.still_backward_units(inp, dy.astype(np.float64), kv_map, units, w.C, w.W, w.lam, w.scale, w.eps,
                                  sel, max_retained=U.budget(w), gate_activation=gate_activation)
    g = {"dq": np.zeros(inp["q"].shape), "dk": np.zeros(inp["k"].shape), "dv": np.zeros(inp["v"].shape),
         "dWq": np.zeros(inp["Wq"].shape), "dWk": np.zeros(inp["Wk"].shape),
         "lse": np.zeros((B, w.Hq, N)),
         "dg": np.zeros(inp["q"].shape) if inp.get("g") is not None else None,
         "dbq": np.zeros((w.Hq, w.df)) if inp.get("bq") is not None else None,
         "dbk": np.zeros((w.Hq, w.df)) if inp.get("bk") is not None else None}
    for (b, h) in units:
        r = ref[(b, h)]
        kh = int(kv_map[h])
        g["dq"][b, :, h] = r["dq"]
        g["dk"][b, :, kh] += r["dk"]
        g["dv"][b, :, kh] += r["dv"]
        g["dWq"][h] += r["dWq"]
        g["dWk"][h] += r["dWk"]
        g["lse"][b, h] = r["lse"]
        for name in ("dg",):
            if g[name] is not None:
                g[name][b, :, h] = r[name]
        for name in ("dbq", "dbk"):
            if g[name] is not None:
                g[name][h] += r[name]
    return g


def check_backward(w, inp, seed, kv_map=None, gate_activation=0):
    kv = synth.kv_head_map(w) if kv_map is None else kv_map
    dy = make_dy(w, inp, seed)
    hip = U.run_hip_backward(w, inp, dy, kv_map=kv_map, gate_activation=gate_activation)
    ref = oracle_grads(w, inp, dy, hip["sel"], kv, "sigmoid" if gate_activation else "none")
    lse_err = float(np.max(np.abs(hip["lse"] - ref["lse"])))
    print(f"[{w.name}] lse max-abs err {lse_err:.3e}")
    assert lse_err <= (1e-5 * max(1.0, float(np.max(np.abs(ref["lse"])))) if w.dtype == "f32" else 2e-2)
    worst = {}
    for name in ("dq", "dk", "dv", "dg", "dWq", "dWk", "dbq", "dbk"):
        if ref[name] is None:
            assert hip[name] is None
            continue
        x = hip[name].astype(np.float64)
        assert np.all(np.isfinite(x)), name
        scale = float(np.max(np.abs(ref[name])))
        err = float(np.max(np.abs(x - ref[name])))
        worst[name] = err / max(scale, 1e-30) if scale > 0 else err
        print(f"[{w.name}] {name}: max |ref| {scale:.3e}  max-abs err {err:.3e}  ratio {worst[name]:.3e}")
    for name, r in worst.items():
        assert r <= BAR[w.dtype], (name, r)
    return hip, ref


def with_bias(w, inp, seed):
    rng = np.random.default_rng(seed)
    inp["bq"] = synth.round_to_dtype(rng.standard_normal((w.Hq, w.df)) * 0.1, w.dtype)
    inp["bk"] = synth.round_to_dtype(rng.standard_normal((w.Hq, w.df)) * 0.1, w.dtype)
    return inp


def test_backward_fp32_gate_bias_gqa_ragged_tail():
    w = small("bwd", N=600, Hq=4, Hkv=2, lam=8, B=2)
    inp = with_bias(w, synth.make_inputs(w, seed=31, with_gate=True), 32)
    hip, ref = check_backward(w, inp, 33)
    # both branches are live: no gradient is identically zero
    for name in ("dq", "dk", "dv", "dg", "dWq", "dWk", "dbq", "dbk"):
        assert np.max(np.abs(ref[name])) > 1e-4, name


@pytest.mark.parametrize("kw", [
    dict(N=512, lam=16, max_retained=40),                 # the budget runs out in chunk 2
    dict(N=384, lam=0),                                   # nothing retained: local span + linear state only
    dict(N=320, lam=64),                                  # everything retained: no linear branch at all
    dict(N=50),                                           # shorter than one chunk
    dict(N=1024, C=128, W=128, lam=16, Hq=2, Hkv=2),      # the wide chunk
    dict(N=2304, lam=4, Hq=1),                            # many chunks: several segments of the state scan
], ids=["budget", "lam0", "all-kept", "short", "C128", "segments"])
def test_backward_fp32_cases(kw):
    w = small("bwd-" + "-".join(f"{k}{v}" for k, v in kw.items()), **kw)
    check_backward(w, synth.make_inputs(w, seed=41, with_gate=True), 42)


def test_backward_fp32_sigmoid_gate_and_custom_head_map():
    w = small("bwd-sg", N=448, Hq=4, Hkv=2, lam=8)
    inp = synth.make_inputs(w, seed=51)
    rng = np.random.default_rng(52)
    inp["g"] = synth.round_to_dtype(2.0 * rng.standard_normal(inp["q"].shape), w.dtype)
    check_backward(w, inp, 53, kv_map=np.array([1, 0, 0, 1], np.int32), gate_activation=1)


@pytest.mark.parametrize("kw", [
    dict(d=128, C=128, W=128, N=1024, Hq=4, Hkv=2),
    dict(d=64, C=64, W=64, N=1100, Hq=4, Hkv=1, B=2),
    dict(d=128, C=64, W=128, N=900, Hq=2, Hkv=1, max_retained=96),
    dict(d=64, C=128, W=256, N=1500, Hq=3, Hkv=1, B=3, lam=32, max_retained=70),
], ids=["d128-C128", "d64-ragged", "d128-budget", "d64-C128-budget-wide-window"])
def test_backward_bf16(kw):
    w = small("bwd16-" + "-".join(f"{k}{v}" for k, v in kw.items()), dtype="bf16", **kw)
    inp = with_bias(w, synth.make_inputs(w, seed=61, with_gate=True), 62)
    check_backward(w, inp, 63)


def test_backward_at_the_training_shape_sampled_units():
    """Config c6 (the shape bench.py --backward times: 16 sequences of 1024 tokens, 32 query heads over 8 kv heads,
    d = 128, bf16), in the launch configuration the benchmark uses.  The oracle covers what it can reach in seconds:
    dq and dg of the four query heads of kv head 2 in sequence 5, dk and dv of that kv head (the sum over exactly
    those four heads), and dWq, dWk, of query head 9 (sums over all 16 sequences)."""
    w = synth.workload("c6")
    inp = synth.make_inputs(w, with_gate=True)
    dy = make_dy(w, inp, 71)
    hip = U.run_hip_backward(w, inp, dy)
    kv = synth.kv_head_map(w)
    b, kh = 5, 2
    heads = [h for h in range(w.Hq) if kv[h] == kh]
    units = [(b, h) for h in heads] + [(bb, 9) for bb in range(w.B)]
    ref = OB.still_backward_units(inp, dy.astype(np.float64), kv, units, w.C, w.W, w.lam, w.scale, w.eps, hip["sel"])
    bar = BAR[w.dtype]

    def check(name, x, y):
        scale = float(np.max(np.abs(y)))
        err = float(np.max(np.abs(x.astype(np.float64) - y)))
        print(f"[c6] {name}: max |ref| {scale:.3e}  max-abs err {err:.3e}  ratio {err / scale:.3e}")
        assert np.all(np.isfinite(x)) and err <= bar * scale, (name, err, scale)

    for h in heads:
        check(f"dq head {h}", hip["dq"][b, :, h], ref[(b, h)]["dq"])
        check(f"dg head {h}", hip["dg"][b, :, h], ref[(b, h)]["dg"])
    check("dk", hip["dk"][b, :, kh], sum(ref[(b, h)]["dk"] for h in heads))
    check("dv", hip["dv"][b, :, kh], sum(ref[(b, h)]["dv"] for h in heads))
    check("dWq head 9", hip["dWq"][9], sum(ref[(bb, 9)]["dWq"] for bb in range(w.B)))
    check("dWk head 9", hip["dWk"][9], sum(ref[(bb, 9)]["dWk"] for bb in range(w.B)))


def test_backward_with_group_shared_selection_bf16():
    """The selection variant only changes WHICH tokens are kept (one list per kv head); the backward pass takes the
    lists as they are."""
    w = small("bwd-shared", dtype="bf16", d=64, N=768, Hq=4, Hkv=2, lam=8, shared_selection=True)
    inp = synth.make_inputs(w, seed=81, with_gate=True)
    hip, _ = check_backward(w, inp, 82)
    assert np.array_equal(hip["sel"][:, 0], hip["sel"][:, 1]) and np.array_equal(hip["sel"][:, 2], hip["sel"][:, 3])


def test_backward_twice_on_a_user_stream_gives_the_same_gradients():
    """Nothing in the workspace has to start at zero and nothing survives a call: a second call into the same
    (dirty) workspace on a non-default stream reproduces the first to rounding (dk, dv and the parameter gradients
    are summed with atomic adds, so not bit for bit)."""
    import torch

    w = small("bwd-twice", N=700, Hq=4, Hkv=2, lam=8)
    inp = synth.make_inputs(w, seed=91, with_gate=True)
    dy = make_dy(w, inp, 92)
    dev = "cuda"
    q, k, v, g, Wq, Wk = (synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v", "g", "Wq", "Wk"))
    dout = synth.to_torch(dy, w.dtype, dev)
    out = torch.empty_like(q)
    p = S.make_params(B=w.B, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, q=q, k=k, v=v, out=out, g=g)
    sel = torch.zeros(w.B, w.Hq, w.N // w.C, w.lam, dtype=torch.int32, device=dev)
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    bws = torch.empty(S.still_bwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    L = S.still_fwd_workspace_layout(p)
    lse = ws[L.lse:L.lse + w.B * w.Hq * w.N * 4].view(torch.float32)
    stream = torch.cuda.Stream()
    results = []
    with torch.cuda.stream(stream):
        S.still_hybrid_attn_fwd(p, q, k, v, g, Wq, None, Wk, None, out, sel_idx=sel, workspace=ws, stream=stream)
        for _ in range(2):
            grads = [torch.full_like(t, float("nan")) for t in (q, k, v, g)]
            dWq = torch.full((w.Hq, w.d, w.d), float("nan"), dtype=torch.float32, device=dev)
            dWk = torch.full_like(dWq, float("nan"))
            S.still_hybrid_attn_bwd(p, q, k, v, g, Wq, None, Wk, None, out, dout, lse, sel, grads[0], grads[1], grads[2],
                                    grads[3], dWq, None, dWk, None, bws, stream=stream)
            results.append([t.clone() for t in grads + [dWq, dWk]])
    stream.synchronize()
    for a_, b_ in zip(*results):
        a_, b_ = a_.float(), b_.float()
        assert torch.isfinite(a_).all() and torch.isfinite(b_).all()
        assert float((a_ - b_).abs().max()) <= 1e-5 * float(a_.abs().max())


@pytest.mark.parametrize("kw", [
    dict(dtype="f32", N=600, Hq=4, Hkv=2, lam=8, B=2),
    dict(dtype="f32", N=512, lam=16, max_retained=40),
    dict(dtype="bf16", d=128, C=128, W=128, N=1024, Hq=4, Hkv=2),
    dict(dtype="f32", N=50),                               # shorter than a chunk: no linear branch, 56-column rows
    dict(dtype="bf16", d=64, N=330, lam=4, Hq=3, Hkv=3, B=3),
], ids=["f32-gqa-ragged", "f32-budget", "bf16-d128", "f32-short", "bf16-odd-sizes"])
def test_attention_map_against_the_oracle(kw):
    """still_attention_map for the forward call's lists and normalisers: element-wise against the oracle's map
    (weights are at most one: absolute bars 2e-6 on fp32, 4e-3 on bf16, whose logits and features carry 8 bits),
    rows sum to one, nothing above the diagonal, and map x v reproduces the forward output (no gate)."""
    import torch

    w = small("map-" + "-".join(f"{k}{v}" for k, v in kw.items()), **kw)
    inp = with_bias(w, synth.make_inputs(w, seed=101), 102)
    dev = "cuda"
    up = lambda n: synth.to_torch(inp[n], w.dtype, dev)
    q, k, v, Wq, Wk, bq, bk = (up(n) for n in ("q", "k", "v", "Wq", "Wk", "bq", "bk"))
    B, N = q.shape[:2]
    out = torch.empty_like(q)
    p = S.make_params(B=B, N=N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, q=q, k=k, v=v, out=out, max_retained=w.max_retained)
    sel = torch.full((B, w.Hq, N // w.C, w.lam), -1, dtype=torch.int32, device=dev)
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    S.still_hybrid_attn_fwd(p, q, k, v, None, Wq, bq, Wk, bk, out, sel_idx=sel, workspace=ws)
    L = S.still_fwd_workspace_layout(p)
    lse = ws[L.lse:L.lse + B * w.Hq * N * 4].view(torch.float32)
    amap = torch.full((B, w.Hq, N, N), float("nan"), dtype=torch.float32, device=dev)
    bws = torch.empty(S.still_bwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    S.still_attention_map(p, q, k, Wq, bq, Wk, bk, lse, sel, amap, bws)
    torch.cuda.synchronize()
    A = amap.cpu().numpy().astype(np.float64)
    sel_h = sel.cpu().numpy().astype(np.int64)
    y = synth.from_torch(out).astype(np.float64)
    kv = synth.kv_head_map(w)
    bar = 2e-6 if w.dtype == "f32" else 4e-3
    assert np.all(np.isfinite(A)) and np.all(np.triu(A, 1) == 0.0)
    worst = 0.0
    for b in range(B):
        for h in range(w.Hq):
            ref = OB.attention_map(inp["q"][b, :, h], inp["k"][b, :, kv[h]], inp["Wq"][h], inp["Wk"][h], w.C, w.W, w.lam,
                                   w.scale, w.eps, bq=inp["bq"][h], bk=inp["bk"][h], sel=sel_h[b, h],
                                   max_retained=U.budget(w))
            worst = max(worst, float(np.max(np.abs(A[b, h] - ref))))
            assert np.max(np.abs(A[b, h].sum(axis=1) - 1.0)) <= (1e-5 if w.dtype == "f32" else 1e-2)
            yv = A[b, h] @ inp["v"][b, :, kv[h]].astype(np.float64)
            if w.dtype == "f32":
                assert U.rel_err(yv, y[b, :, h]) <= 1e-4
    print(f"[{w.name}] attention map: max-abs err {worst:.3e}")
    assert worst <= bar, worst
    # and its backward pass to the feature-map parameters, for a random dmap
    rng = np.random.default_rng(103)
    dA = np.tril(rng.standard_normal((B, w.Hq, N, N)).astype(np.float32))
    dmap = torch.from_numpy(dA).to(dev)
    f32 = dict(dtype=torch.float32, device=dev)
    dWq, dWk = torch.full((w.Hq, w.d, w.df), float("nan"), **f32), torch.full((w.Hq, w.d, w.df), float("nan"), **f32)
    dbq, dbk = torch.full((w.Hq, w.df), float("nan"), **f32), torch.full((w.Hq, w.df), float("nan"), **f32)
    mws = torch.empty(S.still_attention_map_bwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    S.still_attention_map_bwd(p, q, k, Wq, bq, Wk, bk, lse, sel, amap, dmap, dWq, dbq, dWk, dbk, mws)
    torch.cuda.synchronize()
    ref = {n: np.zeros(s_) for n, s_ in (("dWq", (w.Hq, w.d, w.df)), ("dWk", (w.Hq, w.d, w.df)), ("dbq", (w.Hq, w.df)),
                                         ("dbk", (w.Hq, w.df)))}
    for b in range(B):
        for h in range(w.Hq):
            r = OB.attention_map_backward(inp["q"][b, :, h], inp["k"][b, :, kv[h]], inp["Wq"][h], inp["Wk"][h], w.C, w.W,
                                          w.lam, w.scale, w.eps, dA[b, h].astype(np.float64), bq=inp["bq"][h],
                                          bk=inp["bk"][h], sel=sel_h[b, h], max_retained=U.budget(w))
            for n in ref:
                ref[n][h] += r[n]
    for n, t in (("dWq", dWq), ("dWk", dWk), ("dbq", dbq), ("dbk", dbk)):
        x = t.cpu().numpy().astype(np.float64)
        scale_ = float(np.max(np.abs(ref[n])))
        err = float(np.max(np.abs(x - ref[n])))
        print(f"[{w.name}] map backward {n}: max |ref| {scale_:.3e}  max-abs err {err:.3e}")
        assert np.all(np.isfinite(x)) and err <= BAR[w.dtype] * max(scale_, 1e-30), (n, err, scale_)
