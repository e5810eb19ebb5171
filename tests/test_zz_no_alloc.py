"""The allocation-free prefill entry point (still_hybrid_attn_fwd_static: workspace = the library's built-in scratch
array) against the ordinary entry point, through the C ABI: same kernels, same order, so the results must be equal
bit for bit; two calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

from paper_2602_02180_amd import binding as S
from paper_2602_02180_amd import synth

pytestmark = pytest.mark.gpu


def both_ways(w, seed, with_state):
    import torch

    dev = "cuda"
    inp = synth.make_inputs(w, seed=seed, with_gate=True)
    ten = {n: synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v", "Wq", "Wk", "g")}
    ncf = max(w.N // w.C, 1)
    res = []
    for static in (False, True):
        out = torch.full_like(ten["q"], float("nan"))
        score = torch.full((w.B, w.Hq, w.N), float("nan"), dtype=torch.float32, device=dev)
        sel = torch.full((w.B, w.Hq, ncf, w.lam), -7, dtype=torch.int32, device=dev)
        p = S.make_params(B=w.B, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                          dtype=w.dtype, d_f=w.df, q=ten["q"], k=ten["k"], v=ten["v"], out=out, g=ten["g"],
                          max_tokens=w.N + 8 if with_state else 0)
        state = torch.zeros(S.still_state_bytes(p), dtype=torch.uint8, device=dev) if with_state else None
        assert S.still_fwd_workspace_bytes(p) <= S.STILL_STATIC_WORKSPACE_BYTES
        if static:
            S.still_hybrid_attn_fwd_static(p, ten["q"], ten["k"], ten["v"], ten["g"], ten["Wq"], None, ten["Wk"], None,
                                           out, score_out=score, sel_idx=sel, state_out=state)
        else:
            ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
            S.still_hybrid_attn_fwd(p, ten["q"], ten["k"], ten["v"], ten["g"], ten["Wq"], None, ten["Wk"], None,
                                    out, score_out=score, sel_idx=sel, state_out=state, workspace=ws)
        torch.cuda.synchronize()
        res.append((synth.from_torch(out), score.cpu().numpy(), sel.cpu().numpy(),
                    None if state is None else state.cpu().numpy()))
    return res


def test_static_workspace_entry_point_matches_the_ordinary_one_twice_in_a_row():
    big = synth.Workload("static-a", B=2, N=1500, Hq=4, Hkv=2, d=128, C=128, W=128, lam=16, dtype="bf16")
    small = synth.Workload("static-b", B=1, N=333, Hq=2, Hkv=1, d=64, C=64, W=64, lam=16, dtype="f32")
    for w, seed, with_state in ((big, 61, False), (small, 62, True), (big, 63, True)):
        (o0, s0, i0, st0), (o1, s1, i1, st1) = both_ways(w, seed, with_state)
        assert np.all(np.isfinite(o0))
        assert np.array_equal(o0, o1), f"{w.name}: outputs differ"
        assert np.array_equal(s0, s1), f"{w.name}: scores differ"
        assert np.array_equal(i0, i1), f"{w.name}: selections differ"
        if with_state:
            L = S.still_state_layout(S.make_params(B=w.B, N=1, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam,
                                                   scale=w.scale, eps=w.eps, dtype=w.dtype, max_tokens=w.N + 8))
            # everything but the split partials of the decode step (scratch inside the state, never written here)
            assert np.array_equal(st0[:L.part], st1[:L.part]), f"{w.name}: exported decode states differ"


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    import torch

    w = synth.Workload("static-big", B=1, N=32768, Hq=8, Hkv=2, d=128, C=128, W=128, lam=16, dtype="bf16")
    dev = "cuda"
    q = torch.zeros((1, w.N, w.Hq, w.d), dtype=torch.bfloat16, device=dev)
    k = torch.zeros((1, w.N, w.Hkv, w.d), dtype=torch.bfloat16, device=dev)
    Wm = torch.zeros((w.Hq, w.d, w.d), dtype=torch.bfloat16, device=dev)
    out = torch.full_like(q, 3.0)
    p = S.make_params(B=1, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, q=q, k=k, v=k, out=out)
    assert S.still_fwd_workspace_bytes(p) > S.STILL_STATIC_WORKSPACE_BYTES
    with pytest.raises(S.StillError) as e:
        S.still_hybrid_attn_fwd_static(p, q, k, k, None, Wm, None, Wm, None, out)
    assert e.value.code == S.STILL_ERR_WORKSPACE_TOO_SMALL and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool(torch.all(out == 3.0))
