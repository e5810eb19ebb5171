#!/usr/bin/env python3
"""Benchmark of the STILL hybrid-attention prefill hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c4] [--no-cpu-baseline]

One step = one still_hybrid_attn_fwd call (score + selection + gather + NP-Map linear-attention state scan +
sparse softmax + merge) over one batch of seeded synthetic input that is already resident in HBM.
Prints ONE JSON line: whole-job tokens/s, the roofline record of the dominant kernel (the sparse
softmax + merge kernel, timed with HIP events inside the timed steps on the stream it runs on), and
the float64 oracle timed on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2602_02180_amd import synth  # noqa: E402

PEAK_MFMA = {"bf16": 2.5e15, "f32": 157.3e12}   # dense MFMA peaks of MI355X, flop/s
PEAK_HBM = 8.0e12


# HBM bytes per launch of the dominant prefill kernel (sparse_attn_merge), measured with rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE and scaled by the plain-copy calibration (two counter runs plus two --calibrate-copy runs; FETCH_SIZE
# counts 2 KiB and WRITE_SIZE 1 KiB per unit on this machine).  Other configs: null.
MEASURED_TRAFFIC = {"c4": 1.866e9}


def sparse_branch_flops(w: synth.Workload, N: int) -> float:
    """Algorithmic flops of the sparse softmax branch for one launch: every query row does
    4*d flops (q.k and p.v, 2 per MAC) per visible key: retained keys of chunks <= c-2 plus the
    local span (previous chunk and own chunk up to the row)."""
    t = np.arange(N, dtype=np.int64)
    c = t // w.C
    n_ret = np.maximum(0, c - 1) * w.lam
    if w.max_retained > 0:
        n_ret = np.minimum(n_ret, w.max_retained)
    n_loc = t - np.maximum(0, c - 1) * w.C + 1
    return float(4 * w.d * np.sum(n_ret + n_loc)) * w.B * w.Hq


def linear_rows_flops(w: synth.Workload, N: int) -> float:
    """Algorithmic flops of the rows' linear terms, which the same kernel computes: NP-Map of q (2 d d_f) and
    phi_q S (2 * 2 d_f * d) for every row that has a state (chunks >= 2)."""
    rows = max(0, N - 2 * w.C)
    return float((2 * w.d * w.df + 2 * (2 * w.df) * w.d) * rows) * w.B * w.Hq


def path_flops(w: synth.Workload, N: int) -> float:
    """Useful flops of the whole path per step (score band, both NP-Maps, state update, linear
    output, sparse branch)."""
    d, df = w.d, w.df
    nc = N // w.C
    kept = w.lam * max(0, nc - 2)
    if w.max_retained > 0:
        kept = min(kept, w.max_retained)
    per_head = (2 * d * min(w.W, N) * N            # score logits
                + 2 * (2 * d * df) * N             # NP-Map of q and k
                + 2 * (2 * df) * d * (w.C * max(0, nc - 2) - kept)    # state update, routed chunks
                + 2 * (2 * df) * d * N)            # phi_q S
    return per_head * w.B * w.Hq + sparse_branch_flops(w, N)


def compulsory_bytes(w: synth.Workload, N: int) -> float:
    es = 2 if w.dtype == "bf16" else 4
    return float(w.B * N * w.d * es * (2 * w.Hq + 2 * w.Hkv))


_POOL = {}   # what the forked oracle workers read: set before the pool starts, inherited copy-on-write


def _oracle_worker_init():
    try:
        from threadpoolctl import threadpool_limits
        _POOL["limit"] = threadpool_limits(limits=1)   # one BLAS thread per worker: the pool is the parallelism
    except Exception:  # pragma: no cover
        pass


def _oracle_unit(unit):
    from oracle import still_oracle as O

    w, inp = _POOL["w"], _POOL["inp"]
    t0 = time.perf_counter()
    O.still_forward_units(inp, synth.kv_head_map(w), [unit], C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                          max_retained=w.max_retained if w.max_retained > 0 else None,
                          shared_selection=w.shared_selection, budget_policy="evict" if w.budget_policy else "stop")
    return time.perf_counter() - t0


def host_cores() -> int:
    """Worker processes for the oracle leg: the cores this process may run on, at most 16 (a GPU machine's share)."""
    try:
        n = len(os.sched_getaffinity(0))
    except Exception:  # pragma: no cover
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def cpu_baseline(w: synth.Workload, inp, budget_s: float = 15.0):
    """The oracle as it stands (numpy float64, chunk-wise form; its per-chunk Python loops are single-threaded) on
    whole (batch, head) units of the same inputs, one unit at a time per worker process, one worker per host core,
    until ~budget_s.  Must run before this process touches the GPU: the workers are forked."""
    import itertools
    import multiprocessing as mp

    cores = host_cores()
    _POOL["w"], _POOL["inp"] = w, inp
    order = [(b, h) for h in range(w.Hq) for b in range(w.B)]
    done, busy = 0, 0.0
    t0 = time.perf_counter()
    pool = mp.get_context("fork").Pool(cores, initializer=_oracle_worker_init)
    try:
        for dt in pool.imap_unordered(_oracle_unit, itertools.islice(itertools.cycle(order), 100000)):
            done += 1
            busy += dt
            if time.perf_counter() - t0 > budget_s:
                break
    finally:
        el = time.perf_counter() - t0
        pool.terminate()
        pool.join()
    N = inp["q"].shape[1]
    # one unit = N tokens of one of B*Hq heads; the layer needs all B*Hq units for its B*N tokens
    tok_s = (done * N / el) / w.Hq
    return {"value": tok_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{done} (batch, head) units of the same inputs (of {w.B * w.Hq}; repeated when all are done), all "
                      f"{N} rows each, numpy float64 chunk-wise form, {cores} forked worker processes with one BLAS "
                      f"thread each, {el:.1f} s wall, {busy / max(done, 1):.2f} s per unit on one core; scaled by 1/Hq "
                      f"to whole-layer tokens/s"}


def budget_tag(w: synth.Workload) -> str:
    return (f" max_retained={w.max_retained}" if w.max_retained > 0 else "") + \
        (" budget_policy=evict" if w.budget_policy else "") + \
        (" shared_selection" if w.shared_selection else "")


def global_score_bench(args) -> int:
    """Second workload on the score step (consistency study of Sec. 3.1): still_global_score over the whole causal
    prefix at the shape of the chosen config, then the overlap of the local and the global Top-lambda sets."""
    import torch
    from paper_2602_02180_amd import binding as S

    w = synth.workload(args.config if args.config != "c5" else "c4")
    inp = synth.make_inputs(w)
    dev = "cuda"
    q, k, v = (synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v"))
    Wq, Wk = synth.to_torch(inp["Wq"], w.dtype, dev), synth.to_torch(inp["Wk"], w.dtype, dev)
    out = torch.empty_like(q)
    N = w.N
    p = S.make_params(B=w.B, N=N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, d_f=w.df, q=q, k=k, v=v, out=out)
    glob = torch.empty(w.B, w.Hq, N, dtype=torch.float32, device=dev)
    steps = args.steps if args.steps else 5
    for _ in range(min(args.warmup, 2)):
        S.still_global_score(p, q, k, glob)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        S.still_global_score(p, q, k, glob)
    ev1.record()
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    ker_ms = ev0.elapsed_time(ev1) / steps
    # local scores from one prefill call, then the overlap of the two selections
    local = torch.empty_like(glob)
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    S.still_hybrid_attn_fwd(p, q, k, v, None, Wq, None, Wk, None, out, score_out=local, workspace=ws)
    ov = torch.zeros(w.B, w.Hq, N // w.C, dtype=torch.int32, device=dev)
    S.still_selection_overlap(p, local, glob, ov)
    torch.cuda.synchronize()
    overlap = float(ov.float().mean().item()) / max(w.lam, 1)
    # The method's own work, independent of how the kernel does it: one logit (2 d flops) per causal query-key pair,
    # and per pair the three transcendentals the score equation names (one exponential, two logarithms).  The
    # matrix work is priced against the bf16 MFMA peak, the transcendentals against the vector ALU (256 CUs x 4
    # SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane operations/s; a transcendental occupies a lane for four of them),
    # and the LARGER of the two times is the bound the kernel is measured against.  (The kernel itself walks the
    # logits twice, because every a_j sits inside a logarithm: that is its choice, not the method's.)
    pairs = float(N) * (N + 1) / 2 * w.B * w.Hq
    flops = 2 * w.d * pairs
    peak_alu = 256 * 4 * 16 * 2.4e9
    t_mfma = flops / PEAK_MFMA[w.dtype]
    t_alu = 3 * 4 * pairs / peak_alu
    bound_s = max(t_mfma, t_alu)
    rec = {
        "metric": f"global-score tokens/s ({w.name} shape)", "value": w.B * N * steps / el, "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": min(args.warmup, 2), "ms_per_step": el / steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"global score + overlap, {w.name}: B={w.B} N={N} Hq={w.Hq} Hkv={w.Hkv} d={w.d} "
                               f"C={w.C} W={w.W} lambda={w.lam} heavy_frac={w.heavy_frac}",
                   "overlap_at_lambda_local_vs_global": overlap},
        "roofline": {"bound": "alu" if t_alu >= t_mfma else "mfma", "kernel": "global_score",
                     "achieved": 3 * pairs / (ker_ms * 1e-3) / 1e12, "peak": peak_alu / 4 / 1e12,
                     "unit": "T transcendentals/s", "frac": bound_s / (ker_ms * 1e-3), "traffic": None,
                     "algorithmic_pairs_per_launch": pairs, "mfma_flops_per_launch": flops,
                     "time_at_alu_peak_ms": t_alu * 1e3, "time_at_mfma_peak_ms": t_mfma * 1e3,
                     "mfma_frac": flops / (ker_ms * 1e-3) / PEAK_MFMA[w.dtype], "avg_launch_ms": ker_ms},
    }
    if not args.no_cpu_baseline:
        from oracle import still_oracle as O
        n_s = min(N, 4096)
        qq, kk = inp["q"][0, :n_s, 0].astype(np.float64), inp["k"][0, :n_s, 0].astype(np.float64)
        t0 = time.perf_counter()
        O.global_scores(qq, kk, w.scale, w.eps)
        el_c = time.perf_counter() - t0
        pair_rate = n_s * (n_s + 1) / 2 / el_c
        rec["cpu_baseline"] = {"value": pair_rate / ((N + 1) / 2 * w.Hq), "unit": "tokens/s", "cores": 1,
                               "kind": "oracle",
                               "sample": f"rows 0..{n_s - 1} of one (batch, head) unit, {el_c:.1f} s; its query-key pair "
                                         f"rate scaled to all {N} rows of {w.Hq} heads"}
    print(json.dumps(rec))
    return 0


def backward_flops(w: synth.Workload, N: int) -> float:
    """Algorithmic flops of one backward call.  Softmax branch: five products per visible (row, key) pair (logits and
    dy.v again, then dv, dk, dq), 2 d flops each.  Linear branch, per token and head: on the query side f = x W, phi_q S,
    S A, phi_q^T A, df W^T and x^T df; on the key side f = x W, the state update again, dS v, dS^T phi_k, df W^T and
    x^T df: 36 d d_f flops together."""
    return 2.5 * sparse_branch_flops(w, N) + 36.0 * w.d * w.df * N * w.B * w.Hq


def backward_bench(args) -> int:
    """Side figure: one training step of the operator, still_hybrid_attn_fwd + still_hybrid_attn_bwd, on the
    training shape (config c6: sequences of 1024 tokens, Sec. 4.1) or on the chosen config."""
    import torch
    from paper_2602_02180_amd import binding as S

    w = synth.workload(args.config if args.config in ("c2", "c3", "c4", "c6") else "c6")
    inp = synth.make_inputs(w, with_gate=True)
    dev = "cuda"
    q, k, v, g = (synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v", "g"))
    Wq, Wk = synth.to_torch(inp["Wq"], w.dtype, dev), synth.to_torch(inp["Wk"], w.dtype, dev)
    rng = np.random.default_rng(w.seed + 1000)
    dout = synth.to_torch(synth.round_to_dtype(rng.standard_normal(inp["q"].shape, dtype=np.float32), w.dtype), w.dtype, dev)
    N = w.N
    out = torch.empty_like(q)
    p = S.make_params(B=w.B, N=N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, d_f=w.df, q=q, k=k, v=v, out=out, g=g)
    sel = torch.full((w.B, w.Hq, N // w.C, w.lam), -1, dtype=torch.int32, device=dev)
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    L = S.still_fwd_workspace_layout(p)
    lse = ws[L.lse:L.lse + w.B * w.Hq * N * 4].view(torch.float32)
    dq, dk, dv, dg = (torch.empty_like(t) for t in (q, k, v, g))
    dWq = torch.empty(w.Hq, w.d, w.df, dtype=torch.float32, device=dev)
    dWk = torch.empty_like(dWq)
    bws = torch.empty(S.still_bwd_workspace_bytes(p), dtype=torch.uint8, device=dev)

    def fwd():
        S.still_hybrid_attn_fwd(p, q, k, v, g, Wq, None, Wk, None, out, sel_idx=sel, workspace=ws)

    def bwd():
        S.still_hybrid_attn_bwd(p, q, k, v, g, Wq, None, Wk, None, out, dout, lse, sel, dq, dk, dv, dg, dWq, None,
                                dWk, None, bws)

    steps = args.steps if args.steps else 10
    for _ in range(max(1, min(args.warmup, 3))):
        fwd()
        bwd()
    torch.cuda.synchronize()
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    f_ms = b_ms = 0.0
    t0 = time.perf_counter()
    for _ in range(steps):
        e[0].record()
        fwd()
        e[1].record()
        bwd()
        e[2].record()
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    # the last step's split (events are reused: only the last recording survives), the mean from the wall clock
    f_ms, b_ms = e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2])
    # the attention map and its backward pass (the first training stage's pair), where the N x N maps fit comfortably
    map_ms = map_bwd_ms = None
    if N <= 2048:
        amap = torch.empty(w.B, w.Hq, N, N, dtype=torch.float32, device=dev)
        dmap = torch.randn(w.B, w.Hq, N, N, dtype=torch.float32, device=dev).tril_()
        mws = torch.empty(S.still_attention_map_bwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
        dbq = dbk = None
        for _ in range(2):
            S.still_attention_map(p, q, k, Wq, None, Wk, None, lse, sel, amap, mws)
            S.still_attention_map_bwd(p, q, k, Wq, None, Wk, None, lse, sel, amap, dmap, dWq, dbq, dWk, dbk, mws)
        torch.cuda.synchronize()
        m = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        m[0].record()
        S.still_attention_map(p, q, k, Wq, None, Wk, None, lse, sel, amap, mws)
        m[1].record()
        S.still_attention_map_bwd(p, q, k, Wq, None, Wk, None, lse, sel, amap, dmap, dWq, dbq, dWk, dbk, mws)
        m[2].record()
        torch.cuda.synchronize()
        map_ms, map_bwd_ms = m[0].elapsed_time(m[1]), m[1].elapsed_time(m[2])
        del amap, dmap, mws
    flops = backward_flops(w, N)
    rec = {
        "metric": f"hybrid-attn fwd+bwd tokens/s ({w.name} shape)", "value": w.B * N * steps / el, "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": max(1, min(args.warmup, 3)), "ms_per_step": el / steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"forward + backward, {w.name}: B={w.B} N={N} Hq={w.Hq} Hkv={w.Hkv} d={w.d} C={w.C} "
                               f"W={w.W} lambda={w.lam}, gate given",
                   "fwd_ms": f_ms, "bwd_ms": b_ms, "bwd_workspace_gb": bws.numel() / 1e9,
                   "attention_map_ms": map_ms, "attention_map_bwd_ms": map_bwd_ms},
        "roofline": {"bound": "mfma", "kernel": "still_hybrid_attn_bwd (whole call)",
                     "achieved": flops / (b_ms * 1e-3) / 1e12, "peak": PEAK_MFMA[w.dtype] / 1e12, "unit": "TFLOP/s",
                     "frac": flops / (b_ms * 1e-3) / PEAK_MFMA[w.dtype], "traffic": None,
                     "algorithmic_flops_per_call": flops, "avg_launch_ms": b_ms},
    }
    if not args.no_cpu_baseline:
        from oracle import still_backward as OB
        sel_h = sel.cpu().numpy().astype(np.int64)
        n_s = min(N, 1024)
        t0 = time.perf_counter()
        OB.still_backward_definition(inp["q"][0, :n_s, 0], inp["k"][0, :n_s, 0], inp["v"][0, :n_s, 0],
                                     inp["g"][0, :n_s, 0], inp["Wq"][0], inp["Wk"][0], w.C, w.W, w.lam, w.scale, w.eps,
                                     np.asarray(synth.from_torch(dout[0, :n_s, 0]), np.float64),
                                     sel=sel_h[0, 0, :n_s // w.C])
        el_c = time.perf_counter() - t0
        rec["cpu_baseline"] = {"value": n_s / el_c / w.Hq * (n_s / N), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "sample": f"backward oracle on rows 0..{n_s - 1} of one (batch, head) unit, {el_c:.1f} s; "
                                         f"scaled to {w.Hq} heads (and quadratically to {N} rows)"}
    print(json.dumps(rec))
    return 0


def decode_bench(args) -> int:
    print(json.dumps(decode_record(args, args.steps if args.steps else 0, with_cpu=not args.no_cpu_baseline)))
    return 0


def decode_record(args, steps: int, with_cpu: bool):
    """Config 5: B sequences with a prefilled 32K context, then single-token steps.  The contexts are drawn
    on the GPU (seeded torch generator, same distributions as synth.make_inputs) and prefilled in slices of
    8 sequences through still_hybrid_attn_fwd with state_out; one timed step = one decode step for all B."""
    import torch
    from paper_2602_02180_amd import binding as S

    w = synth.workload("c5", max_retained=args.max_retained, shared_selection=args.shared_selection,
                       budget_policy=int(args.evict))
    dev = "cuda"
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    B, N, Hq, Hkv, d = w.B, w.N, w.Hq, w.Hkv, w.d
    n_steps = steps if steps else w.decode_steps
    max_tokens = N + n_steps + args.warmup + 8
    bf = torch.bfloat16

    def lognormal(*shape):
        return torch.exp(0.5 * torch.randn(*shape, generator=gen, device=dev))

    sq, sk, sv = lognormal(Hq, d), lognormal(Hkv, d), lognormal(Hkv, d)
    Wq = (torch.randn(Hq, d, d, generator=gen, device=dev) / d ** 0.5).to(bf)
    Wk = (torch.randn(Hq, d, d, generator=gen, device=dev) / d ** 0.5).to(bf)
    base = dict(B=B, Hq=Hq, Hkv=Hkv, d=d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps, dtype="bf16",
                max_tokens=max_tokens, max_retained=w.max_retained, shared_selection=w.shared_selection,
                budget_policy=w.budget_policy)
    ps = S.make_params(N=1, **base)
    L = S.still_state_layout(ps)
    state = torch.empty(S.still_state_bytes(ps), dtype=torch.uint8, device=dev)
    S.still_state_init(ps, state)
    # prefill in slices of SB sequences into per-slice states, then scatter into the batch state
    SB = 8
    pslice = S.make_params(N=1, **{**base, "B": SB})
    Ls = S.still_state_layout(pslice)
    st_slice = torch.empty(S.still_state_bytes(pslice), dtype=torch.uint8, device=dev)
    slices = Hkv if w.shared_selection else Hq      # retained rows: per query head, or once per kv head
    regions = [("S", 4 * 2 * d * (d + 1) * Hq), ("kret", 2 * L.cap * d * slices), ("vret", 2 * L.cap * d * slices),
               ("sel", 4 * L.n_chunks * w.lam * Hq), ("kring", 2 * L.R * d * Hkv), ("vring", 2 * L.R * d * Hkv),
               ("score", 4 * L.R * Hq), ("part", 4 * 32 * (d + 2) * Hq)]
    t_prefill = 0.0
    for b0 in range(0, B, SB):
        q = (torch.randn(SB, N, Hq, d, generator=gen, device=dev) * sq).to(bf)
        k = torch.randn(SB, N, Hkv, d, generator=gen, device=dev) * sk
        v = (torch.randn(SB, N, Hkv, d, generator=gen, device=dev) * sv).to(bf)
        n_heavy = int(w.heavy_frac * N)
        for i in range(SB):
            idx = torch.randperm(N, generator=gen, device=dev)[:n_heavy]
            k[i, idx] *= w.heavy_mult
        k = k.to(bf)
        o = torch.empty_like(q)
        pf = S.make_params(N=N, q=q, k=k, v=v, out=o, **{**base, "B": SB})
        ws = torch.empty(S.still_fwd_workspace_bytes(pf), dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        S.still_hybrid_attn_fwd(pf, q, k, v, None, Wq, None, Wk, None, o, state_out=st_slice, workspace=ws)
        torch.cuda.synchronize()
        t_prefill += time.perf_counter() - t0
        if b0 == 0 and with_cpu:   # sequence 0 of the batch, for the oracle leg below
            cpu_ctx = {"q": q[0, :, :8].float().cpu().numpy(), "k": k[0].float().cpu().numpy(),
                       "v": v[0].float().cpu().numpy()}
        for name, per_seq in regions:   # every region is [B, ...]: copy the slice's sequences into place
            src0, dst0 = getattr(Ls, name), getattr(L, name)
            state[dst0 + b0 * per_seq: dst0 + (b0 + SB) * per_seq] = st_slice[src0: src0 + SB * per_seq]
        del q, k, v, o, ws
    torch.cuda.empty_cache()

    def draw_step():
        q = (torch.randn(B, Hq, d, generator=gen, device=dev) * sq).to(bf)
        k = (torch.randn(B, Hkv, d, generator=gen, device=dev) * sk).to(bf)
        v = (torch.randn(B, Hkv, d, generator=gen, device=dev) * sv).to(bf)
        return q, k, v

    toks = [draw_step() for _ in range(args.warmup + n_steps)]
    out = torch.empty(B, Hq, d, dtype=bf, device=dev)
    t = N
    for i in range(args.warmup):
        S.still_hybrid_attn_decode_step(ps, state, t, *toks[i], None, Wq, None, Wk, None, out)
        t += 1
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_steps)]
    t0 = time.perf_counter()
    for i in range(n_steps):
        ev[i][0].record()
        S.still_hybrid_attn_decode_step(ps, state, t, *toks[args.warmup + i], None, Wq, None, Wk, None, out)
        ev[i][1].record()
        t += 1
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    lat = np.array([a.elapsed_time(b) for a, b in ev])
    routing = np.array([((N + args.warmup + i) % w.C) == 0 for i in range(n_steps)])
    c = (N + args.warmup) // w.C
    n_ret = (c - 1) * w.lam if w.max_retained <= 0 else min((c - 1) * w.lam, w.max_retained)
    rows = n_ret + (N + args.warmup - (c - 1) * w.C + 1)
    bytes_step = B * (slices * rows * 2 * d * 2 + Hq * (2 * d * (d + 1)) * 4)
    ordinary = float(np.median(lat[~routing])) if (~routing).any() else float("nan")
    rec = {
        "metric": "hybrid-attn decode tokens/s @32K context, Llama-3-8B layer shape", "value": B * n_steps / el,
        "unit": "tokens/s", "n_gpus": 1, "steps": n_steps, "warmup": args.warmup, "ms_per_step": el / n_steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"c5: B={B} context={N} Hq={Hq} Hkv={Hkv} d={d} C={w.C} W={w.W} lambda={w.lam}" + budget_tag(w),
                   "median_ordinary_step_ms": ordinary,
                   "routing_step_ms": [float(x) for x in lat[routing]],
                   "prefill_of_contexts_s": t_prefill, "state_gb": state.numel() / 1e9},
        "roofline": {"bound": "hbm", "kernel": "decode step (attend + finish)", "achieved": bytes_step / (ordinary * 1e-3) / 1e9,
                     "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": bytes_step / (ordinary * 1e-3) / PEAK_HBM,
                     "traffic": args.traffic_bytes, "algorithmic_bytes_per_step": bytes_step},
    }
    if with_cpu:
        rec["cpu_baseline"] = decode_cpu_baseline(w, cpu_ctx, toks, Wq, Wk, args.warmup, n_steps)
    del state, st_slice, toks
    torch.cuda.empty_cache()
    return rec


def decode_cpu_baseline(w, ctx, toks, Wq, Wk, warmup, n_steps, budget_s: float = 20.0):
    """The oracle has no incremental form: its decode is the chunk-wise form on the concatenated sequence with only the
    decoded rows requested (scores, selection and states of the whole prefix are recomputed).  Timed on query heads of
    sequence 0 until ~budget_s."""
    from oracle import still_oracle as O

    n_dec = warmup + n_steps
    G = w.Hq // w.Hkv
    units_done, t0, c0 = 0, time.perf_counter(), time.process_time()
    for h in range(ctx["q"].shape[1]):
        qd = np.stack([toks[i][0][0, h].float().cpu().numpy() for i in range(n_dec)])
        kd = np.stack([toks[i][1][0, h // G].float().cpu().numpy() for i in range(n_dec)])
        vd = np.stack([toks[i][2][0, h // G].float().cpu().numpy() for i in range(n_dec)])
        q = np.concatenate([ctx["q"][:, h], qd]).astype(np.float64)
        k = np.concatenate([ctx["k"][:, h // G], kd]).astype(np.float64)
        v = np.concatenate([ctx["v"][:, h // G], vd]).astype(np.float64)
        O.still_chunkwise(q, k, v, None, Wq[h].float().cpu().numpy().astype(np.float64),
                          Wk[h].float().cpu().numpy().astype(np.float64), w.C, w.W, w.lam, w.scale, w.eps,
                          rows=(w.N, w.N + n_dec), max_retained=w.max_retained if w.max_retained > 0 else None,
                          budget_policy="evict" if w.budget_policy else "stop")
        units_done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    el = time.perf_counter() - t0
    # threads actually kept busy: the Python loops of the oracle run on one core, numpy's BLAS pool adds to it
    # only inside the matrix products (this leg runs after the GPU was initialised, so it does not fork workers)
    cores = max(1, int(round((time.process_time() - c0) / el)))
    # one decoded token of one sequence needs one row from each of the Hq heads
    return {"value": units_done * n_dec / el / w.Hq, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{units_done} query heads of sequence 0, {n_dec} decoded rows each after the {w.N}-token context, "
                      f"chunk-wise form with a row range (the prefix's scores, selection and states are recomputed every "
                      f"time: the oracle has no incremental state), one process, {el:.1f} s wall (cores = CPU time / "
                      f"wall time); scaled by 1/Hq to tokens/s"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default: 20 prefill calls, 128 decode steps)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="c4", choices=["c1", "c2", "c3", "c4", "c5", "c6"])
    ap.add_argument("--backward", action="store_true",
                    help="side figure: forward + backward of the operator (default shape: c6, the training shape)")
    ap.add_argument("--max-retained", type=int, default=0,
                    help="budget on the retained tokens per (sequence, head); 0 (default) = none, the headline workload")
    ap.add_argument("--evict", action="store_true",
                    help="with --max-retained: hold the budget by evicting the lowest score (budget policy 1) instead "
                         "of not adding (side figures only)")
    ap.add_argument("--shared-selection", action="store_true",
                    help="variant: the query heads of one kv head rank by their summed score and share one retained "
                         "set (not the paper's method; side figures only)")
    ap.add_argument("--global-score", action="store_true",
                    help="second workload: the score over the whole causal prefix and its overlap with the local "
                         "selection (consistency study), at the prefill shape of --config")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true",
                    help="default (config 4) line only: skip the config-5 decode measurement that fills the "
                         "decode_c5_* keys of `config`")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="measured HBM bytes per launch of the dominant kernel (from rocprofv3 --pmc runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run plain device-to-device copies of 1 GiB and exit: the known-size reference against "
                         "which the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU only (the path shards over heads or batch with no exchange "
              "between GPUs). Run with --gpus 1.", file=sys.stderr)
        return 2

    from paper_2602_02180_amd import binding as S

    S.lib()  # fail loudly if the HIP library is missing
    prefill_run = not (args.calibrate_copy or args.global_score or args.config == "c5")
    w = inp = cpu_rec = None
    if prefill_run:
        w = synth.workload(args.config, max_retained=args.max_retained, shared_selection=args.shared_selection,
                           budget_policy=int(args.evict))
        inp = synth.make_inputs(w)
        # The oracle leg forks worker processes, so it runs before this process initialises the GPU (a forked copy
        # of an initialised HIP runtime is not something to rely on); it is outside every timed GPU region anyway.
        if not args.no_cpu_baseline:
            cpu_rec = cpu_baseline(w, inp)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 1 << 30, "launches": 4}))
        return 0

    if args.backward:
        if args.config == "c4" and "--config" not in sys.argv:
            args.config = "c6"
        return backward_bench(args)
    if args.global_score:
        return global_score_bench(args)
    if args.config == "c5":
        return decode_bench(args)
    if not args.steps:
        args.steps = 20
    dev = "cuda"
    q, k, v = (synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v"))
    Wq, Wk = synth.to_torch(inp["Wq"], w.dtype, dev), synth.to_torch(inp["Wk"], w.dtype, dev)
    out = torch.empty_like(q)
    N = w.N
    p = S.make_params(B=w.B, N=N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, d_f=w.df, q=q, k=k, v=v, out=out, max_retained=w.max_retained,
                      shared_selection=w.shared_selection, budget_policy=w.budget_policy)
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        S.still_hybrid_attn_fwd(p, q, k, v, None, Wq, None, Wk, None, out, workspace=ws, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # Timed region: the calls run back to back.  The library records a (begin, end) HIP event pair around the
    # dominant kernel of every call, on the stream it is launched on, without synchronising; the mean over the
    # timed calls is read afterwards (the library keeps the last 64 calls).
    S.still_profile_enable(2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    dom_ms = S.still_profile_read()["sparse_attn_merge"]
    # Per-kernel breakdown from a second, untimed pass with event pairs around every kernel (sixteen stream
    # markers per call slow a call down by a few per cent).  transpose_v and transpose_w run on a second stream
    # next to score_select, so these three overlap.
    S.still_profile_enable(1)
    for _ in range(min(args.steps, 10)):
        step()
    per_kernel = S.still_profile_read()
    S.still_profile_enable(False)

    ms_step = el / args.steps * 1e3
    tok_s = w.B * N * args.steps / el
    dom = "sparse_attn_merge"
    dom_s = dom_ms * 1e-3
    flops = sparse_branch_flops(w, N) + linear_rows_flops(w, N)
    peak = PEAK_MFMA[w.dtype]
    roofline = {"bound": "mfma", "kernel": dom, "achieved": flops / dom_s / 1e12, "peak": peak / 1e12,
                "unit": "TFLOP/s", "frac": flops / dom_s / peak,
                "traffic": args.traffic_bytes if args.traffic_bytes is not None else
                (MEASURED_TRAFFIC.get(args.config) if w.max_retained <= 0 and not w.shared_selection else None),
                "algorithmic_flops_per_launch": flops, "sparse_branch_flops": sparse_branch_flops(w, N),
                "linear_rows_flops": linear_rows_flops(w, N), "avg_launch_ms": dom_ms}
    rec = {
        "metric": "hybrid-attn fwd tokens/s @32K, Llama-3-8B layer shape" if args.config == "c4"
        else f"hybrid-attn fwd tokens/s ({args.config})",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} N={N} Hq={w.Hq} Hkv={w.Hkv} d={w.d} C={w.C} W={w.W} "
                               f"lambda={w.lam} heavy_frac={w.heavy_frac}" + budget_tag(w),
                   "path_gflop_per_step": path_flops(w, N) / 1e9,
                   "compulsory_hbm_mb_per_step": compulsory_bytes(w, N) / 1e6,
                   "path_frac_of_mfma_peak": path_flops(w, N) / (ms_step * 1e-3) / peak,
                   "kernel_ms": per_kernel,
                   "kernel_ms_note": "separate untimed pass; transpose_v/transpose_w overlap score_select on a second stream"},
        "roofline": roofline,
    }
    if cpu_rec is not None:
        rec["cpu_baseline"] = cpu_rec
    if args.config == "c4" and not args.no_decode and w.max_retained <= 0 and not w.shared_selection:
        # the benchmark spec names prefill AND decode: the decode step of config 5 (B = 64 sequences behind a 32K context
        # each, one chunk of 128 steps, one of them routing) rides along as flat keys; the headline fields above
        # stay those of config 4.  `python bench.py --config c5` prints the full decode record.
        del q, k, v, out, ws
        torch.cuda.empty_cache()
        dargs = argparse.Namespace(**vars(args))
        dargs.warmup = 3
        drec = decode_record(dargs, 0, with_cpu=False)
        rt = drec["config"]["routing_step_ms"]
        rec["config"].update({
            "decode_c5_workload": drec["config"]["workload"],
            "decode_c5_steps": drec["steps"],
            "decode_c5_ordinary_step_ms": drec["config"]["median_ordinary_step_ms"],
            "decode_c5_routing_step_ms": float(np.mean(rt)) if rt else None,
            "decode_c5_tokens_per_s": drec["value"],
            "decode_c5_bytes_per_step": drec["roofline"]["algorithmic_bytes_per_step"],
            "decode_c5_hbm_gb_per_s": drec["roofline"]["achieved"],
            "decode_c5_hbm_frac": drec["roofline"]["frac"],
        })
    print(json.dumps(rec))
    return 0


if __name__ == "__main__":
    sys.exit(main())
