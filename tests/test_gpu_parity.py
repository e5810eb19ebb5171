"""GPU parity: the HIP path (through the C ABI) against the float64 oracle on the same seeded,
dtype-rounded inputs.

Bars (from the benchmark spec):
  * selected-index sets bit-exact wherever the oracle's gap between the lambda-th and the
    (lambda+1)-th score exceeds 1e-5; the mismatch rate among near-ties is printed;
  * outputs within 1e-4 relative on fp32 (max-normalised and per row); on bf16 within the stated
    2e-2 absolute wherever |ref| < 4, and elsewhere within 2e-2 plus the half unit in the last
    place that storing ANY result in bf16 adds (tests/gpu_util.py: assert_bf16_bar, the one place
    where that bar is written down); the plain max-abs error and the share of elements under the
    plain bar are printed too.
Output parity is run twice: with the oracle's indices injected into the HIP path (isolates the
gather / linear / softmax / merge kernels) and end to end, where the oracle is re-run with the
HIP path's own indices after those were checked to be a valid Top-lambda set.
"""
import numpy as np
import pytest

from paper_2602_02180_amd import binding as S
from paper_2602_02180_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

F32_REL = 1e-4


def small(name, **kw):
    base = dict(B=1, N=512, Hq=2, Hkv=1, d=64, C=64, W=64, lam=16, dtype="f32")
    base.update(kw)
    return synth.Workload(name, **base)


def all_units(w):
    return [(b, h) for b in range(w.B) for h in range(w.Hq)]


def check_outputs(w, hip, ref_units, units, what):
    worst_rel = worst_row = worst_abs = 0.0
    reports = []
    for (b, h) in units:
        ref = ref_units[(b, h)]
        r0, r1 = ref["rows"]
        x = hip["out"][b, r0:r1, h].astype(np.float64)
        y = ref["out"][r0:r1]
        assert np.all(np.isfinite(x)), f"{what}: non-finite output in unit {(b, h)}"
        worst_rel = max(worst_rel, U.rel_err(x, y))
        worst_row = max(worst_row, U.row_rel_err(x, y))
        worst_abs = max(worst_abs, float(np.max(np.abs(x - y))))
        if w.dtype != "f32":
            reports.append(U.bf16_bar_report(x, y))
    print(f"[{w.name}:{what}] out: max-rel {worst_rel:.3e} row-rel {worst_row:.3e} max-abs {worst_abs:.3e}")
    if w.dtype == "f32":
        assert worst_rel <= F32_REL and worst_row <= F32_REL, (worst_rel, worst_row)
    else:
        rep = U.merge_bf16_reports(reports)
        print(f"[{w.name}:{what}] bf16 bar: {U.bf16_report_text(rep)}")
        assert rep["bar_fraction"] <= 1.0, rep


def check_terms(w, hip, ref_units, units, what):
    """N_LA and D_LA of the linear branch, as left in the workspace."""
    tol = 1e-4 if w.dtype == "f32" else 1e-2
    for (b, h) in units:
        ref = ref_units[(b, h)]
        r0, r1 = ref["rows"]
        e_n = U.rel_err(hip["N_LA"][b, h, r0:r1].astype(np.float64), ref["N_LA"][r0:r1]) if np.any(ref["N_LA"]) else \
            float(np.max(np.abs(hip["N_LA"][b, h, r0:r1])))
        e_d = U.rel_err(hip["D_LA"][b, h, r0:r1].astype(np.float64), ref["D_LA"][r0:r1]) if np.any(ref["D_LA"]) else \
            float(np.max(np.abs(hip["D_LA"][b, h, r0:r1])))
        print(f"[{w.name}:{what}] unit {(b, h)} N_LA rel {e_n:.3e}  D_LA rel {e_d:.3e}")
        assert e_n <= tol and e_d <= tol, (e_n, e_d)


def check_scores_and_selection(w, hip, ref_units, units, what):
    stot = sclear = sbad = stie = 0
    worst = 0.0
    for (b, h) in units:
        ref = ref_units[(b, h)]
        err = float(np.max(np.abs(hip["score"][b, h] - ref["score"])))
        worst = max(worst, err)
        n, clear, bad, tie = U.selection_report(ref["rank_score"], ref["sel"], hip["sel"][b, h], w.C, w.lam,
                                                max_retained=U.budget(w))
        stot, sclear, sbad, stie = stot + n, sclear + clear, sbad + bad, stie + tie
        assert U.selection_is_valid(ref["rank_score"], hip["sel"][b, h], w.C, tol=1e-4, max_retained=U.budget(w)), \
            f"unit {(b, h)}: not a top set"
    print(f"[{w.name}:{what}] score max-abs err {worst:.3e}; chunks {stot}, clear-gap {sclear}, "
          f"mismatch on clear {sbad}, mismatch on near-ties {stie} "
          f"(rate {stie / max(1, stot - sclear):.3f} of near-tie chunks)")
    assert worst <= 5e-5, worst
    assert sbad == 0


def run_case(w, inp, units=None, kv_map=None, rows=None):
    units = all_units(w) if units is None else units
    # 1) oracle with its own selection
    ref = U.oracle_units(w, inp, units, kv_map=kv_map, rows=rows)
    # 2) HIP end to end
    hip = U.run_hip(w, inp, kv_map=kv_map)
    check_scores_and_selection(w, hip, ref, units, "e2e")
    # oracle re-run with the HIP path's indices (identical unless a near-tie flipped)
    sel_h = hip["sel"]
    ref_h = U.oracle_units(w, inp, units, sel=sel_h, kv_map=kv_map, rows=rows)
    check_terms(w, hip, ref_h, units, "e2e")
    check_outputs(w, hip, ref_h, units, "e2e")
    # 3) HIP with the oracle's indices injected
    B, N = inp["q"].shape[0], inp["q"].shape[1]
    ncf = N // w.C
    if w.lam > 0 and ncf > 0:
        sel_full = hip["sel"].copy()
        for (b, h) in units:
            sel_full[b, h] = ref[(b, h)]["sel"]
        hip2 = U.run_hip(w, inp, sel_in=sel_full, kv_map=kv_map)
        ref2 = U.oracle_units(w, inp, units, sel=sel_full, kv_map=kv_map, rows=rows)
        check_terms(w, hip2, ref2, units, "injected")
        check_outputs(w, hip2, ref2, units, "injected")
    return hip


# ------------------------------------------------------------------ config 1 (fp32, full problem)
def test_c1_fp32_full():
    w = synth.CONFIGS["c1"]
    run_case(w, synth.make_inputs(w))


# ------------------------------------------------------------------ small shapes: tiles, ragged tails, edge cases
@pytest.mark.parametrize("kw", [
    dict(dtype="f32", d=64, C=64, W=64, N=512),
    dict(dtype="f32", d=64, C=128, W=100, N=700),            # ragged tail, W not a multiple of 32
    dict(dtype="f32", d=128, C=64, W=128, N=333),            # W > C, ragged
    dict(dtype="bf16", d=64, C=64, W=64, N=640, Hq=4, Hkv=2),
    dict(dtype="bf16", d=128, C=128, W=128, N=1000, Hq=4, Hkv=2, B=2),
    dict(dtype="bf16", d=128, C=64, W=128, N=777),
    dict(dtype="bf16", d=64, C=128, W=33, N=1024, lam=5),
    # window lengths around the band tiles of the score kernel (a one-key window gives every token the same score:
    # the selection is then decided by the tie-break alone)
    dict(dtype="f32", d=64, C=64, W=1, N=200),
    dict(dtype="f32", d=64, C=64, W=5, N=300),
    dict(dtype="f32", d=64, C=64, W=31, N=300),
    dict(dtype="f32", d=64, C=128, W=32, N=400),
    dict(dtype="f32", d=128, C=64, W=65, N=300),
    dict(dtype="bf16", d=128, C=128, W=66, N=600),
    # long retained sets: the sparse-attention kernel's steady-state loop over fully visible retained tiles,
    # with workgroups spanning two chunks (C = 64) and ragged ends
    dict(dtype="f32", d=64, C=64, W=64, N=1500, lam=32),
    dict(dtype="f32", d=128, C=64, W=128, N=1700, lam=32, Hq=1, Hkv=1),
    dict(dtype="bf16", d=128, C=64, W=64, N=1900, lam=48, Hq=2, Hkv=1),
    dict(dtype="bf16", d=64, C=64, W=64, N=1333, lam=40, Hq=2, Hkv=2),
], ids=lambda k: "-".join(f"{a}{b}" for a, b in k.items()))
def test_small_shapes(kw):
    """(shapes listed above; see also test_wide_score_windows)"""
    w = small("small", **kw)
    run_case(w, synth.make_inputs(w, seed=1234))


# budget on the retained tokens: chunks keep lam until it is used up (one chunk may keep a part), then nothing
@pytest.mark.parametrize("kw", [
    dict(dtype="f32", d=64, C=64, W=64, N=1024, lam=16, max_retained=40),           # 16, 16, 8, 0, ...
    dict(dtype="f32", d=64, C=64, W=64, N=900, lam=16, max_retained=1000),          # never reached
    dict(dtype="f32", d=128, C=64, W=128, N=1100, lam=32, max_retained=192, Hq=1, Hkv=1),
    dict(dtype="bf16", d=128, C=128, W=128, N=2000, lam=16, max_retained=100, Hq=4, Hkv=2, B=2),
    dict(dtype="bf16", d=64, C=64, W=64, N=1900, lam=48, max_retained=300, Hq=2, Hkv=2),
    dict(dtype="bf16", d=128, C=64, W=64, N=1500, lam=64, max_retained=128),        # whole chunks kept: sink
], ids=lambda k: "-".join(f"{a}{b}" for a, b in k.items()))
def test_retained_budget(kw):
    w = small("budget", **kw)
    hip = run_case(w, synth.make_inputs(w, seed=4321))
    kept = (hip["sel"] >= 0).sum(axis=(2, 3))
    assert np.all(kept == min(w.max_retained, w.lam * (w.N // w.C)))


# variant: the query heads of one kv head rank by their summed score and share one list
@pytest.mark.parametrize("kw", [
    dict(N=640, lam=16, max_retained=40),                                  # fp32 d=64 C=64: fills at chunk 2, then evicts
    dict(N=500, lam=16, max_retained=5, W=48),                             # budget below one chunk's offer, ragged end
    dict(dtype="bf16", d=128, C=128, W=128, N=1536, lam=16, max_retained=24, Hq=4, Hkv=2, B=2),
    dict(d=128, C=64, W=64, N=700, lam=8, max_retained=16),
    dict(dtype="bf16", d=64, C=64, N=2048, lam=16, max_retained=96, Hq=4, Hkv=1),   # several scan segments
], ids=lambda k: "-".join(f"{a}{b}" for a, b in k.items()))
def test_eviction_policy_prefill(kw):
    """Budget policy 1 (a variant of this library): rows of chunk c see the best-scored offers of chunks <= c-2, a
    token that leaves enters the state at the step it leaves.  The evictions are ranked by the device's own fp32
    scores on both sides (one precision decides); scores and offers are checked against the oracle's as usual."""
    w = small("evict", **kw)
    inp = synth.make_inputs(w, seed=37)
    units = all_units(w)
    hip = U.run_hip(w, inp, budget_policy=1)
    ref_own = U.oracle_units(w, inp, units, budget_policy="evict")
    for (b, h) in units:
        assert float(np.max(np.abs(hip["score"][b, h] - ref_own[(b, h)]["score"]))) <= 5e-5
        n, clear, bad, tie = U.selection_report(ref_own[(b, h)]["rank_score"], ref_own[(b, h)]["sel"], hip["sel"][b, h],
                                                w.C, w.lam)
        assert bad == 0 and np.all(hip["sel"][b, h] >= 0)
    ref = U.oracle_units(w, inp, units, sel=hip["sel"], budget_policy="evict", rank_scores=hip["score"].astype(np.float64))
    check_terms(w, hip, ref, units, "evict")
    check_outputs(w, hip, ref, units, "evict")
    # and the policy is not a no-op here: the stop-adding operator gives other rows
    stop = U.oracle_units(w, inp, units[:1])
    b, h = units[0]
    assert np.abs(stop[(b, h)]["out"] - ref[(b, h)]["out"]).max() > 1e-4


@pytest.mark.parametrize("kw,kv_map", [
    (dict(dtype="f32", d=64, C=64, W=64, N=700, Hq=4, Hkv=2), None),
    (dict(dtype="f32", d=64, C=128, W=100, N=900, Hq=6, Hkv=2, lam=20, max_retained=50), [0, 1, 0, 1, 1, 0]),
    (dict(dtype="bf16", d=128, C=128, W=128, N=1300, Hq=8, Hkv=2, B=2), None),
], ids=["f32-regular", "f32-irregular-map-budget", "bf16-groups-of-4"])
def test_group_shared_selection(kw, kv_map):
    w = small("shared", shared_selection=True, **kw)
    kv = None if kv_map is None else np.asarray(kv_map, np.int32)
    hip = run_case(w, synth.make_inputs(w, seed=555), kv_map=kv)
    kv = synth.kv_head_map(w) if kv is None else kv
    for h in range(w.Hq):
        first = int(np.nonzero(kv == kv[h])[0][0])
        assert np.array_equal(hip["sel"][:, h], hip["sel"][:, first]), "lists of one group differ"


def test_full_size_config4_with_budget_and_group_shared_selection():
    """Config 4 at full size in the launch configuration of the bench, with the budget of the paper's long-context
    setting (896 retained tokens, chunk 128) and one retained set per kv head: sampled units against the oracle."""
    w = synth.workload("c4", max_retained=896, shared_selection=True)
    inp = synth.make_inputs(w)
    units = [(0, 2), (0, 29)]
    ref = U.oracle_units(w, inp, units)
    hip = U.run_hip(w, inp)
    check_scores_and_selection(w, hip, ref, units, "e2e")
    ref_h = U.oracle_units(w, inp, units, sel=hip["sel"])
    check_terms(w, hip, ref_h, units, "e2e")
    check_outputs(w, hip, ref_h, units, "e2e")
    assert np.all(np.isfinite(hip["out"]))
    kept = (hip["sel"] >= 0).sum(axis=(2, 3))
    assert np.all(kept == 896)
    assert np.array_equal(hip["sel"][0, 0], hip["sel"][0, 3]) and np.array_equal(hip["sel"][0, 28], hip["sel"][0, 31])


def test_full_length_config4_shape_with_budget_held_by_eviction_fp32():
    """The config-4 sequence (32768 tokens, chunk 128, 256 routing steps) with the budget of the paper's long-context
    setting (896 retained tokens) held by evicting the lowest score, in fp32 (four query heads on one kv head) so that
    the plan over all steps, the masks over 4096 offers and the redirected state scan are held to the fp32 bar on
    every row of a unit.  (In bf16 the same run is within the bf16 bar on most sampled units; rows that two heavy
    keys with far-apart values share can miss it by the rounding of the weights themselves: a kernel that hands the
    weights to the matrix core in bf16 is off by up to 2^-9 max_j |v_j - y| whatever else it does.)"""
    w = synth.workload("c4", max_retained=896, dtype="f32", Hq=4, Hkv=1)
    inp = synth.make_inputs(w)
    units = [(0, 1)]
    hip = U.run_hip(w, inp, budget_policy=1)
    ref_own = U.oracle_units(w, inp, units, budget_policy="evict")
    b, h = units[0]
    assert float(np.max(np.abs(hip["score"][b, h] - ref_own[(b, h)]["score"]))) <= 5e-5
    n, clear, bad, tie = U.selection_report(ref_own[(b, h)]["rank_score"], ref_own[(b, h)]["sel"], hip["sel"][b, h],
                                            w.C, w.lam)
    assert bad == 0
    ref = U.oracle_units(w, inp, units, sel=hip["sel"], budget_policy="evict",
                         rank_scores=hip["score"].astype(np.float64))
    check_terms(w, hip, ref, units, "evict-32k")
    check_outputs(w, hip, ref, units, "evict-32k")
    assert np.all(np.isfinite(hip["out"]))


@pytest.mark.parametrize("kw", [
    dict(N=700, W=129),                                     # fp32 d=64 C=64: nine band tiles
    dict(N=900, W=256, C=64, lam=8),                        # the widest window: four chunks
    dict(N=1000, W=200, C=128, d=128, lam=16),
    dict(dtype="bf16", N=1200, W=255, C=128, d=128, Hq=4, Hkv=2, lam=16),
], ids=lambda k: "-".join(f"{a}{b}" for a, b in k.items()))
def test_wide_score_windows(kw):
    """Score windows of more than 128 keys (Sec. 3.1 leaves the window length free): the band of the score kernel
    grows to nine tiles."""
    w = small("wide", **kw)
    run_case(w, synth.make_inputs(w, seed=39))


@pytest.mark.parametrize("lam", [0, 1, 64])
def test_lambda_extremes(lam):
    w = small("lam", lam=lam, N=448, dtype="f32")
    run_case(w, synth.make_inputs(w, seed=77))


@pytest.mark.parametrize("N", [1, 31, 64, 65, 128, 129, 191])
def test_short_sequences(N):
    w = small("short", N=N, dtype="bf16", d=128, C=64, W=128, Hq=2, Hkv=2)
    run_case(w, synth.make_inputs(w, seed=5))


def test_gate_bias_and_custom_head_map():
    w = small("gate", N=600, Hq=4, Hkv=2, dtype="f32", d=64, C=64, W=64, lam=8, B=2)
    inp = synth.make_inputs(w, seed=9, with_gate=True)
    rng = np.random.default_rng(10)
    inp["bq"] = synth.round_to_dtype(rng.standard_normal((w.Hq, w.df)) * 0.1, w.dtype)
    inp["bk"] = synth.round_to_dtype(rng.standard_normal((w.Hq, w.df)) * 0.1, w.dtype)
    kv_map = np.array([1, 0, 0, 1], np.int32)
    run_case(w, inp, kv_map=kv_map)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sigmoid_gate_from_preactivation(dtype):
    """gate_activation = 1: g holds the pre-activation and the kernel applies the logistic function where it reads
    the gate (prefill: the prologue of the sparse-attention kernel)."""
    w = small("sgate", N=700, Hq=2, Hkv=1, dtype=dtype, d=128 if dtype == "bf16" else 64, C=64, W=64, lam=8)
    inp = synth.make_inputs(w, seed=19)
    rng = np.random.default_rng(20)
    inp["g"] = synth.round_to_dtype(2.0 * rng.standard_normal(inp["q"].shape), w.dtype)
    units = all_units(w)
    hip = U.run_hip(w, inp, gate_activation=1)
    ref = U.oracle_units(w, inp, units, sel=hip["sel"], gate_activation="sigmoid")
    check_terms(w, hip, ref, units, "sigmoid gate")
    check_outputs(w, hip, ref, units, "sigmoid gate")
    # and it is not the identity: the same numbers taken as they stand give something else
    raw = U.run_hip(w, inp, gate_activation=0)
    assert np.max(np.abs(raw["out"].astype(np.float64) - hip["out"].astype(np.float64))) > 1e-3


def test_heavy_hitter_keys_bf16():
    w = small("heavy", N=2048, Hq=2, Hkv=1, dtype="bf16", d=128, C=128, W=128, heavy_frac=0.01)
    run_case(w, synth.make_inputs(w, seed=11))


def test_all_kept_equals_dense_causal_attention_fp32():
    """lambda = C through the HIP path against torch-free dense causal softmax attention."""
    w = small("dense", N=320, lam=64, dtype="f32")
    inp = synth.make_inputs(w, seed=3)
    hip = U.run_hip(w, inp)
    for h in range(w.Hq):
        q = inp["q"][0, :, h].astype(np.float64)
        k = inp["k"][0, :, 0].astype(np.float64)
        v = inp["v"][0, :, 0].astype(np.float64)
        logit = w.scale * (q @ k.T)
        logit[np.triu_indices(w.N, 1)] = -np.inf
        p = np.exp(logit - logit.max(axis=1, keepdims=True))
        ref = (p / p.sum(axis=1, keepdims=True)) @ v
        assert U.rel_err(hip["out"][0, :, h], ref) <= F32_REL


# ------------------------------------------------------------------ full-size configs on sampled units
@pytest.mark.parametrize("name,units,rows", [
    ("c2", [(0, 0), (3, 31), (1, 13)], None),
    ("c3", [(0, 5), (1, 30)], None),
    ("c4", [(0, 0), (0, 17)], None),
])
def test_full_size_configs_sampled_units(name, units, rows):
    w = synth.CONFIGS[name]
    inp = synth.make_inputs(w)
    ref = U.oracle_units(w, inp, units)
    hip = U.run_hip(w, inp)
    check_scores_and_selection(w, hip, ref, units, "e2e")
    ref_h = U.oracle_units(w, inp, units, sel=hip["sel"])
    check_terms(w, hip, ref_h, units, "e2e")
    check_outputs(w, hip, ref_h, units, "e2e")
    # properties that hold for every unit at any size
    out = hip["out"]
    assert np.all(np.isfinite(out))
    assert np.all(np.isfinite(hip["score"])) and hip["score"].max() <= np.log((1 + w.eps) / w.eps) * (1 + 1e-5)
    sel = hip["sel"]
    assert np.all(np.diff(sel, axis=-1) > 0)
    chunk_of = sel // w.C
    assert np.all(chunk_of == np.arange(sel.shape[2])[None, None, :, None])
    # token 0 has a one-token window: the largest possible score, hence always kept
    assert np.all(sel[:, :, 0, 0] == 0)


# ------------------------------------------------------------------ long segments of the chunk scan in fp32
@pytest.mark.parametrize("kw", [
    dict(d=64, C=64, W=64),            # one sub-unit per unit
    dict(d=64, C=128, W=128),          # two sub-units per unit
    dict(d=128, C=64, W=128),
], ids=lambda k: "-".join(f"{a}{b}" for a, b in k.items()))
def test_many_chunks_per_segment_fp32(kw):
    """Enough (batch, head, chunk) work that a segment of the linear-attention scan spans several chunks, so the
    output pass fetches several staged key-feature units per segment, in fp32 (tight tolerance)."""
    w = small("segs", N=4096 if kw["C"] == 64 else 8192, Hq=32, Hkv=8, dtype="f32", lam=16, **kw)
    inp = synth.make_inputs(w, seed=321)
    hip = U.run_hip(w, inp)
    assert hip["layout"].seg_chunks >= 3 and hip["layout"].nseg >= 2
    units = [(0, 3), (0, 30)]
    ref = U.oracle_units(w, inp, units, sel=hip["sel"])
    check_terms(w, hip, ref, units, "segs")
    check_outputs(w, hip, ref, units, "segs")


# ------------------------------------------------------------------ stream ordering of the two-stream launch sequence
def test_back_to_back_calls_on_a_user_stream_are_ordered():
    """The layout kernels run on a library-owned second stream.  Work enqueued on the caller's stream before a
    call (here: copies that replace v and Wk in place) must still precede them, and the next call must not start
    overwriting the workspace while the previous one reads it: three calls with changing inputs, enqueued back
    to back on one non-default stream with a single workspace, must each give exactly what a lone call gives."""
    import torch

    w = small("order", N=2048, Hq=4, Hkv=2, dtype="bf16", d=128, C=128, W=128)
    dev = "cuda"
    inps = [synth.make_inputs(w, seed=100 + i) for i in range(3)]
    lone = [U.run_hip(w, inp, want_terms=False)["out"] for inp in inps]

    tens = [{n: synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v", "Wq", "Wk")} for inp in inps]
    cur = {n: torch.empty_like(tens[0][n]) for n in tens[0]}
    outs = [torch.full_like(cur["q"], float("nan")) for _ in range(3)]
    p = S.make_params(B=1, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, d_f=w.df, q=cur["q"], k=cur["k"], v=cur["v"], out=outs[0])
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        for i in range(3):
            for n in cur:
                cur[n].copy_(tens[i][n], non_blocking=True)       # on `stream`, right before the call
            S.still_hybrid_attn_fwd(p, cur["q"], cur["k"], cur["v"], None, cur["Wq"], None, cur["Wk"], None, outs[i],
                                    workspace=ws, stream=stream)
    stream.synchronize()
    for i in range(3):
        got = synth.from_torch(outs[i])
        assert np.array_equal(got, lone[i]), f"call {i} differs from the lone call"


def test_rejected_call_enqueues_nothing():
    """state_out + injected indices without score_out is an argument error: the call must return INVALID_ARG with
    nothing enqueued, i.e. a sentinel-filled `out` (and state) stays untouched; the same call with score_out works."""
    import torch

    w = small("reject", N=512, Hq=2, Hkv=1, dtype="f32")
    inp = synth.make_inputs(w, seed=41)
    dev = "cuda"
    ten = {n: synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v", "Wq", "Wk")}
    out = torch.full_like(ten["q"], -123.0)
    p = S.make_params(B=1, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, d_f=w.df, q=ten["q"], k=ten["k"], v=ten["v"], out=out, max_tokens=w.N)
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    state = torch.full((S.still_state_bytes(p),), 0x5A, dtype=torch.uint8, device=dev)
    good = U.run_hip(w, inp, want_terms=False)
    sel = torch.from_numpy(good["sel"].astype(np.int32)).to(dev)
    torch.cuda.synchronize()
    with pytest.raises(S.StillError) as e:
        S.still_hybrid_attn_fwd(p, ten["q"], ten["k"], ten["v"], None, ten["Wq"], None, ten["Wk"], None, out,
                                sel_idx=sel, sel_idx_is_input=True, state_out=state, workspace=ws)
    assert e.value.code == S.STILL_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert bool(torch.all(out == -123.0)), "a rejected call wrote to out"
    assert bool(torch.all(state == 0x5A)), "a rejected call wrote to the state"
    score = torch.empty((1, w.Hq, w.N), dtype=torch.float32, device=dev)
    S.still_hybrid_attn_fwd(p, ten["q"], ten["k"], ten["v"], None, ten["Wq"], None, ten["Wk"], None, out,
                            score_out=score, sel_idx=sel, sel_idx_is_input=True, state_out=state, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(synth.from_torch(out), good["out"])


def test_prefill_call_replays_from_a_hip_graph():
    """The call enqueues kernels, a device-to-device copy and event fork/join only, so it can be captured (after one
    eager call has created the library's helper stream).  Every replay must reproduce the eager result, also after
    the inputs changed in place."""
    import torch

    w = small("graph", N=1024, Hq=4, Hkv=2, dtype="bf16", d=128, C=128, W=128)
    dev = "cuda"
    inps = [synth.make_inputs(w, seed=200 + i) for i in range(3)]
    lone = [U.run_hip(w, inp, want_terms=False)["out"] for inp in inps]
    tens = [{n: synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v", "Wq", "Wk")} for inp in inps]
    cur = {n: tens[0][n].clone() for n in tens[0]}
    out = torch.full_like(cur["q"], float("nan"))
    p = S.make_params(B=1, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, d_f=w.df, q=cur["q"], k=cur["k"], v=cur["v"], out=out)
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)

    def call():
        S.still_hybrid_attn_fwd(p, cur["q"], cur["k"], cur["v"], None, cur["Wq"], None, cur["Wk"], None, out,
                                workspace=ws, stream=torch.cuda.current_stream())

    call()                                   # eager: creates the helper stream, warms everything up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for i in (1, 2, 0, 1):
        for n in cur:
            cur[n].copy_(tens[i][n])
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(synth.from_torch(out), lone[i]), f"replay with inputs {i} differs from the eager call"


def test_profile_modes_report_kernel_times():
    """Timing events: every-kernel mode gives a positive time for every kernel of the call; the dominant-kernel mode
    gives the sparse-attention kernel only (the others read 0); the mean is over the calls since enabling."""
    import torch

    w = small("prof", N=2048, Hq=4, Hkv=2, dtype="bf16", d=128, C=128, W=128)
    inp = synth.make_inputs(w, seed=7)
    dev = "cuda"
    ten = {n: synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v", "Wq", "Wk")}
    out = torch.empty_like(ten["q"])
    p = S.make_params(B=1, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, d_f=w.df, q=ten["q"], k=ten["k"], v=ten["v"], out=out)
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)

    def call():
        S.still_hybrid_attn_fwd(p, ten["q"], ten["k"], ten["v"], None, ten["Wq"], None, ten["Wk"], None, out,
                                workspace=ws)

    call()
    torch.cuda.synchronize()
    try:
        S.still_profile_enable(1)
        for _ in range(3):
            call()
        every = S.still_profile_read()
        assert set(every) == {S.still_profile_kernel_name(i) for i in range(S.STILL_PROFILE_SLOTS)}
        assert all(0.0 < ms < 100.0 for ms in every.values()), every
        S.still_profile_enable(2)
        for _ in range(70):                      # more calls than the ring of event sets holds
            call()
        last = S.still_profile_read()
        assert 0.0 < last["sparse_attn_merge"] < 100.0
        assert all(ms == 0.0 for name, ms in last.items() if name != "sparse_attn_merge"), last
        # same kernel, same input: the two means agree within a generous factor
        assert 0.5 < last["sparse_attn_merge"] / every["sparse_attn_merge"] < 2.0
    finally:
        S.still_profile_enable(0)
    with pytest.raises(S.StillError):
        S.still_profile_read()


# ------------------------------------------------------------------ local-versus-global consistency workload
@pytest.mark.parametrize("kw", [
    dict(dtype="f32", d=64, N=700, Hq=2, Hkv=1),
    dict(dtype="f32", d=128, N=333, Hq=2, Hkv=2),
    dict(dtype="bf16", d=128, N=1500, Hq=4, Hkv=2, B=2, C=128, W=128),
    dict(dtype="bf16", d=64, N=129, Hq=2, Hkv=1),
    dict(dtype="f32", d=64, N=1, Hq=1, Hkv=1),
    dict(dtype="f32", d=128, N=400, Hq=2, Hkv=1, C=128, W=128),
], ids=lambda k: "-".join(f"{a}{b}" for a, b in k.items()))
def test_global_score_and_selection_overlap(kw):
    """Score over the whole causal prefix against the oracle's two-softmax form, then the per-chunk overlap of the
    Top-lambda sets under the local and the global score (exact wherever both oracle gaps are clear)."""
    import torch
    from oracle import still_oracle as O

    w = small("gscore", **kw)
    inp = synth.make_inputs(w, seed=31)
    dev = "cuda"
    q, k = synth.to_torch(inp["q"], w.dtype, dev), synth.to_torch(inp["k"], w.dtype, dev)
    p = S.make_params(B=w.B, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, q=q, k=k)
    glob = torch.full((w.B, w.Hq, w.N), float("nan"), dtype=torch.float32, device=dev)
    S.still_global_score(p, q, k, glob)
    kv = synth.kv_head_map(w)
    local = torch.from_numpy(U.run_hip(w, inp, want_terms=False)["score"]).to(dev)
    ncf = w.N // w.C
    ov = torch.full((w.B, w.Hq, max(ncf, 1)), -1, dtype=torch.int32, device=dev)
    S.still_selection_overlap(p, local, glob, ov)
    torch.cuda.synchronize()
    glob_h, ov_h, local_h = glob.cpu().numpy(), ov.cpu().numpy(), local.cpu().numpy()
    worst, exact, total = 0.0, 0, 0
    for b in range(w.B):
        for h in range(w.Hq):
            qq, kk = inp["q"][b, :, h].astype(np.float64), inp["k"][b, :, kv[h]].astype(np.float64)
            ref_g = O.global_scores(qq, kk, w.scale, w.eps)
            worst = max(worst, float(np.max(np.abs(glob_h[b, h] - ref_g))))
            if ncf == 0:
                continue
            ref_l = O.self_saliency_scores(qq, kk, w.W, w.scale, w.eps)
            ref_ov = O.selection_overlap(ref_l, ref_g, w.C, w.lam)
            clear = (O.selection_gaps(ref_l, w.C, w.lam) > 1e-5) & (O.selection_gaps(ref_g, w.C, w.lam) > 1e-4)
            assert np.array_equal(ov_h[b, h, :ncf][clear], ref_ov[clear]), (b, h)
            # whatever the near-ties do, the count is that of the device's own two rankings
            own = O.selection_overlap(local_h[b, h].astype(np.float64), glob_h[b, h].astype(np.float64), w.C, w.lam)
            assert np.array_equal(ov_h[b, h, :ncf], own), (b, h)
            exact += int(clear.sum()); total += ncf
    print(f"[gscore {w.dtype} d={w.d} N={w.N}] global score max-abs err {worst:.3e}; chunks with clear gaps {exact}/{total}")
    assert worst <= 5e-5, worst      # the bar of the window-local score


def test_global_score_over_a_long_prefix_keeps_relative_accuracy():
    """Over thousands of keys a_j and n_j differ by the factor 1 - a_diag with a_diag ~ 1e-3 .. 1e-4, and the score
    itself is of that size: an absolute bar says nothing there.  Every row's score must match the float64 oracle to
    1e-3 of its own value plus 2e-8 (the kernel takes the logarithm of the ratio as log(1 - a_diag) + log(1 + small) rather
    than as the difference of two fp32 logarithms, which resolves it to a few per cent only)."""
    import torch
    from oracle import still_oracle as O

    w = small("gslong", dtype="bf16", d=128, N=6144, Hq=1, Hkv=1, C=128, W=128)
    inp = synth.make_inputs(w, seed=33)
    dev = "cuda"
    q, k = synth.to_torch(inp["q"], w.dtype, dev), synth.to_torch(inp["k"], w.dtype, dev)
    p = S.make_params(B=w.B, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, q=q, k=k)
    glob = torch.full((w.B, w.Hq, w.N), float("nan"), dtype=torch.float32, device=dev)
    S.still_global_score(p, q, k, glob)
    torch.cuda.synchronize()
    got = glob.cpu().numpy()[0, 0].astype(np.float64)
    ref = O.global_scores(inp["q"][0, :, 0].astype(np.float64), inp["k"][0, :, 0].astype(np.float64), w.scale, w.eps)
    err = np.abs(got - ref)
    tail = slice(1024, None)
    bar = 1e-3 * np.abs(ref) + 2e-8                  # (a score can pass through zero: a small absolute floor)
    frac = (err / bar)[tail]
    print(f"[gscore long prefix] rows >= 1024: median |score| {np.median(np.abs(ref[tail])):.3e}, "
          f"worst error / (1e-3 |ref| + 2e-8) = {frac.max():.3f}, max-abs error {err.max():.3e}")
    assert err.max() <= 5e-5
    assert frac.max() <= 1.0, frac.max()


def test_128k_context_last_rows_and_selection():
    """Four times the longest benchmark context (N = 131072 at the config-4 layer shape, 5.4 GB of workspace): 64-bit
    offsets, grid sizes and the retained prefix of 16 K rows per head hold; the last rows of a unit, which see all
    of it, match the oracle, and the selection of all 1024 chunks is exact where the gap is clear."""
    import torch

    w = synth.workload("c4", N=131072)
    inp = synth.make_inputs(w)
    dev = "cuda"
    q, k, v = (synth.to_torch(inp[n], w.dtype, dev) for n in ("q", "k", "v"))
    Wq, Wk = synth.to_torch(inp["Wq"], w.dtype, dev), synth.to_torch(inp["Wk"], w.dtype, dev)
    out = torch.full_like(q, float("nan"))
    p = S.make_params(B=w.B, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, d_f=w.df, q=q, k=k, v=v, out=out)
    ws = torch.empty(S.still_fwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    sel = torch.full((w.B, w.Hq, w.N // w.C, w.lam), -1, dtype=torch.int32, device=dev)
    S.still_hybrid_attn_fwd(p, q, k, v, None, Wq, None, Wk, None, out, sel_idx=sel, workspace=ws)
    torch.cuda.synchronize()
    o = synth.from_torch(out)
    assert np.all(np.isfinite(o))
    sel_h = sel.cpu().numpy().astype(np.int64)
    rows, unit = (w.N - 200, w.N), (0, 21)
    own = U.oracle_units(w, inp, [unit], rows=(0, 1))[unit]
    n, clear, bad, tie = U.selection_report(own["rank_score"], own["sel"], sel_h[unit], w.C, w.lam)
    print(f"[128k] chunks {n}, clear-gap {clear}, mismatch on clear {bad}, on near-ties {tie}")
    assert bad == 0
    ref = U.oracle_units(w, inp, [unit], sel=sel_h, rows=rows)[unit]
    x = o[0, rows[0]:rows[1], unit[1]].astype(np.float64)
    y = ref["out"][rows[0]:rows[1]]
    U.assert_bf16_bar(x, y, "128k last rows")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rope_pre_pass_matches_the_oracle_and_composes_with_the_prefill(dtype):
    """still_rope_apply rotates q and k in place (per-sequence start positions, GQA, strided tensors); the rotated
    tensors then go through the prefill like any other input."""
    import torch

    w = small("rope", N=300, Hq=4, Hkv=2, B=2, dtype=dtype, d=128 if dtype == "bf16" else 64, lam=8)
    inp = synth.make_inputs(w, seed=23)
    dev = "cuda"
    q, k = synth.to_torch(inp["q"], w.dtype, dev), synth.to_torch(inp["k"], w.dtype, dev)
    pos0 = torch.tensor([0, 4000], dtype=torch.int32, device=dev)
    p = S.make_params(B=w.B, N=w.N, Hq=w.Hq, Hkv=w.Hkv, d=w.d, C=w.C, W=w.W, lam=w.lam, scale=w.scale, eps=w.eps,
                      dtype=w.dtype, q=q, k=k, v=k, out=q)
    S.still_rope_apply(p, q, k, pos0, base=10000.0)
    torch.cuda.synchronize()
    gq, gk = synth.from_torch(q).astype(np.float64), synth.from_torch(k).astype(np.float64)
    from oracle import still_oracle as O
    tol = 2e-5 if dtype == "f32" else 2.0 ** -8      # relative to the row's largest magnitude: one rounding on bf16
    for b in range(w.B):
        pos = np.arange(w.N) + int(pos0[b])
        for name, got, H in (("q", gq, w.Hq), ("k", gk, w.Hkv)):
            for h in range(H):
                ref = O.rope_rotate(inp[name][b, :, h], pos)
                err = np.max(np.abs(got[b, :, h] - ref)) / np.max(np.abs(ref))
                assert err <= tol, (name, b, h, err)
    # position 0 of sequence 0 is untouched, everything else moved
    assert np.array_equal(gq[0, 0], inp["q"][0, 0].astype(np.float64))
    assert np.max(np.abs(gq[1] - inp["q"][1])) > 0.1
    # the rotated tensors are ordinary inputs of the prefill
    inp2 = dict(inp)
    inp2["q"], inp2["k"] = synth.from_torch(q), synth.from_torch(k)
    run_case(w, inp2)
