"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/still.h declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2602_02180_amd import binding as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "still.h")).read()
    return sorted(set(re.findall(r"STILL_API\s+[\w\s\*]+?\b(still_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"still_hybrid_attn_fwd", "still_hybrid_attn_decode_step", "still_fwd_workspace_bytes",
            "still_state_bytes", "still_state_init", "still_last_error", "still_version",
            "still_hybrid_attn_decode_step_at", "still_hybrid_attn_fwd_static", "still_hybrid_attn_bwd",
            "still_bwd_workspace_bytes", "still_bwd_workspace_layout", "still_attention_map",
            "still_attention_map_bwd", "still_attention_map_bwd_workspace_bytes", "still_rope_apply"} <= set(names)
    lib = S.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert S.still_version() >= 100


def params(**kw):
    base = dict(B=1, N=1024, Hq=4, Hkv=2, d=64, C=64, W=64, lam=16, scale=0.125, eps=1e-6, dtype="bf16")
    base.update(kw)
    return S.make_params(**base)


def test_workspace_layout_is_consistent():
    p = params()
    L = S.still_fwd_workspace_layout(p)
    assert S.still_fwd_workspace_bytes(p) == L.total
    offs = [L.score, L.sel, L.vt, L.kret, L.vrett, L.wqt, L.wkf, L.seg, L.snap, L.zsnap, L.pimg, L.zpre, L.kmask, L.n_la, L.d_la, L.vfr, L.ev_src, L.ev_alive, L.ev_fin, L.ev_vfr, L.lse, L.total]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert L.n_pad % 128 == 0 and L.n_pad >= 1024
    assert L.cap % 64 == 0 and L.cap >= (1024 // 64) * 16
    assert L.nseg * L.seg_chunks >= 16
    assert L.snap - L.seg >= 1 * 4 * L.nseg * (2 * 64 * 65) * 4
    assert L.zsnap - L.snap >= 1 * 4 * 16 * 64 * 128 * 2           # one bf16 state per (head, chunk)
    assert L.zpre - L.pimg >= 1 * 4 * L.nseg * 64 * 128 * 2        # and one per (head, segment)
    assert L.d_la - L.n_la <= 256                                   # the inspection regions are empty by default
    Lt = S.still_fwd_workspace_layout(params(emit_terms=1))
    assert Lt.d_la - Lt.n_la >= 1 * 4 * 1024 * 64 * 4 and Lt.total > L.total


def test_retained_budget_bounds_the_retained_rows_of_workspace_and_state():
    free = S.still_fwd_workspace_layout(params(N=8192))
    tight = S.still_fwd_workspace_layout(params(N=8192, max_retained=100))
    assert free.cap == (8192 // 64) * 16 and tight.cap == 128
    assert tight.total < free.total
    roomy = S.still_fwd_workspace_layout(params(N=8192, max_retained=1 << 20))
    assert roomy.cap == free.cap and roomy.total == free.total
    # a decode state no longer grows with the context once the budget is set
    s_free = S.still_state_layout(params(N=1, max_tokens=1 << 20))
    s_tight = S.still_state_layout(params(N=1, max_tokens=1 << 20, max_retained=896))
    assert s_free.cap >= (1 << 20) // 64 * 16 and s_tight.cap == 896 + 64
    assert s_tight.kret < s_tight.vret and s_tight.vret - s_tight.kret == 1 * 4 * s_tight.cap * 64 * 2


def test_eviction_policy_layouts():
    """Budget policy 1: the workspace holds ALL offers (the sparse kernel walks them under masks) plus the plan's
    regions; the decode state holds max_retained rows plus their scores and token indices."""
    stop = S.still_fwd_workspace_layout(params(N=8192, max_retained=100))
    ev = S.still_fwd_workspace_layout(params(N=8192, max_retained=100, budget_policy=1))
    assert stop.cap == 128 and ev.cap == (8192 // 64) * 16
    assert stop.ev_alive - stop.ev_src <= 256 and stop.lse - stop.ev_vfr <= 256      # empty without the policy
    assert ev.ev_alive - ev.ev_src >= 1 * 4 * 8192 * 4
    assert ev.ev_fin - ev.ev_alive >= 1 * 4 * (8192 // 64) * (ev.cap // 64) * 8
    assert ev.ev_vfr - ev.ev_fin >= 1 * 4 * (2 * 100 + 1) * 4
    assert ev.lse - ev.ev_vfr >= 1 * 4 * 64 * ev.n_pad * 2 and ev.total - ev.lse >= 1 * 4 * 8192 * 4
    s_stop = S.still_state_layout(params(N=1, max_tokens=1 << 20, max_retained=896))
    s_ev = S.still_state_layout(params(N=1, max_tokens=1 << 20, max_retained=896, budget_policy=1))
    assert s_ev.cap == s_stop.cap == 896 + 64
    assert s_stop.ret_tok - s_stop.ret_score <= 256
    assert s_ev.ret_tok - s_ev.ret_score >= 1 * 4 * s_ev.cap * 4 and s_ev.total - s_ev.ret_tok >= 1 * 4 * s_ev.cap * 4


@pytest.mark.parametrize("kw,code", [
    (dict(d=96), S.STILL_ERR_UNSUPPORTED),
    (dict(C=32), S.STILL_ERR_UNSUPPORTED),
    (dict(W=257, C=128), S.STILL_ERR_UNSUPPORTED),
    (dict(d_f=32), S.STILL_ERR_UNSUPPORTED),
    (dict(lam=65), S.STILL_ERR_INVALID_ARG),
    (dict(lam=-1), S.STILL_ERR_INVALID_ARG),
    (dict(N=0), S.STILL_ERR_INVALID_ARG),
    (dict(Hq=5), S.STILL_ERR_INVALID_ARG),
    (dict(eps=0.0), S.STILL_ERR_INVALID_ARG),
    (dict(kv_head_of_q=[0, 1, 2, 0]), S.STILL_ERR_INVALID_ARG),
    (dict(budget_policy=2, max_retained=64), S.STILL_ERR_INVALID_ARG),
    (dict(budget_policy=1), S.STILL_ERR_INVALID_ARG),                       # eviction needs a budget to hold
    (dict(budget_policy=1, max_retained=64, shared_selection=1), S.STILL_ERR_UNSUPPORTED),
    (dict(budget_policy=1, max_retained=5000), S.STILL_ERR_UNSUPPORTED),    # the retained set is ranked in LDS
])
def test_bad_params_are_rejected_on_the_host(kw, code):
    p = params(**kw)
    with pytest.raises(S.StillError) as e:
        S.still_fwd_workspace_layout(p)
    assert e.value.code == code
    assert S.still_last_error() != ""


def test_backward_entry_point_validates_on_the_host():
    """The backward pass covers budget_policy 0 without padding; fp32 only at d = 64; its workspace holds a forward
    workspace plus its own regions; null pointers are refused before any launch."""
    for kw in (dict(dtype="f32", d=128, C=128), dict(max_retained=64, budget_policy=1)):
        with pytest.raises(S.StillError) as e:
            S.still_bwd_workspace_layout(params(**kw))
        assert e.value.code == S.STILL_ERR_UNSUPPORTED
    p = params()
    BL = S.still_bwd_workspace_layout(p)
    assert S.still_bwd_workspace_bytes(p) == BL.total
    names = [n for n, t in S.StillBwdWsLayout._fields_ if t is ctypes.c_size_t]
    offs = [getattr(BL, n) for n in names]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert BL.e_row - BL.fwd >= S.still_fwd_workspace_bytes(p)
    assert BL.dz - BL.ds >= 1 * 4 * 16 * 128 * 64 * 2 and BL.total - BL.dv32 >= 1 * 2 * 1024 * 64 * 4
    p.q_st = p.k_st = p.v_st = p.o_st = 64
    null, fake = ctypes.c_void_p(None), ctypes.c_void_p(0x1000)
    rc = S.lib().still_hybrid_attn_bwd(ctypes.byref(p), fake, fake, fake, null, fake, null, fake, null, fake, fake,
                                        null, fake, fake, fake, fake, null, fake, null, fake, null, fake, 1 << 40, null)
    assert rc == S.STILL_ERR_INVALID_ARG and "pointer" in S.still_last_error()
    rc = S.lib().still_hybrid_attn_bwd(ctypes.byref(p), fake, fake, fake, null, fake, null, fake, null, fake, fake,
                                        fake, fake, fake, fake, fake, null, fake, null, fake, null, fake, 16, null)
    assert rc == S.STILL_ERR_WORKSPACE_TOO_SMALL
    rc = S.lib().still_hybrid_attn_bwd(ctypes.byref(p), fake, fake, fake, fake, fake, null, fake, null, fake, fake,
                                        fake, fake, fake, fake, fake, null, fake, null, fake, null, fake, 1 << 40, null)
    assert rc == S.STILL_ERR_INVALID_ARG and "dg" in S.still_last_error()


def test_rope_entry_point_validates_on_the_host():
    lib = S.lib()
    null, fake = ctypes.c_void_p(None), ctypes.c_void_p(0x1000)
    p = params()
    p.q_st = p.k_st = 64
    assert lib.still_rope_apply(ctypes.byref(p), null, null, null, ctypes.c_float(10000.0), null) == S.STILL_ERR_INVALID_ARG
    assert lib.still_rope_apply(ctypes.byref(p), fake, fake, null, ctypes.c_float(1.0), null) == S.STILL_ERR_INVALID_ARG
    assert "base" in S.still_last_error()
    p.q_st = 32
    assert lib.still_rope_apply(ctypes.byref(p), fake, null, null, ctypes.c_float(10000.0), null) == S.STILL_ERR_INVALID_ARG


def test_fwd_rejects_null_and_misaligned_pointers_without_launching():
    p = params()
    lib = S.lib()
    null = ctypes.c_void_p(None)
    rc = lib.still_hybrid_attn_fwd(ctypes.byref(p), null, null, null, null, null, null, null, null, null, null,
                                   null, 0, null, null, 0, null)
    assert rc == S.STILL_ERR_INVALID_ARG
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    p.q_st = p.k_st = p.v_st = p.o_st = 64
    rc = lib.still_hybrid_attn_fwd(ctypes.byref(p), odd, fake, fake, null, fake, null, fake, null, fake, null,
                                   null, 0, null, fake, 1 << 40, null)
    assert rc == S.STILL_ERR_INVALID_ARG and "aligned" in S.still_last_error()
    p.q_st = 63   # not a multiple of 16 bytes
    rc = lib.still_hybrid_attn_fwd(ctypes.byref(p), fake, fake, fake, null, fake, null, fake, null, fake, null,
                                   null, 0, null, fake, 1 << 40, null)
    assert rc == S.STILL_ERR_INVALID_ARG
    p = params()
    p.q_st = p.k_st = p.v_st = p.o_st = 64
    rc = lib.still_hybrid_attn_fwd(ctypes.byref(p), fake, fake, fake, null, fake, null, fake, null, fake, null,
                                   null, 0, null, fake, 16, null)
    assert rc == S.STILL_ERR_WORKSPACE_TOO_SMALL


def test_state_export_with_injected_indices_needs_scores_and_is_rejected_before_any_launch():
    """state_out carries the scores of the local span; with injected indices the scores are only computed when
    score_out is given.  The combination without score_out is refused by the host checks (fake pointers: a launch
    would fault), as the header promises for every failure."""
    p = params(max_tokens=1024)
    p.q_st = p.k_st = p.v_st = p.o_st = 64
    lib = S.lib()
    null, fake = ctypes.c_void_p(None), ctypes.c_void_p(0x1000)
    rc = lib.still_hybrid_attn_fwd(ctypes.byref(p), fake, fake, fake, null, fake, null, fake, null, fake, null,
                                   fake, 1, fake, fake, 1 << 40, null)
    assert rc == S.STILL_ERR_INVALID_ARG and "score" in S.still_last_error()


def test_side_entry_points_validate_only_what_they_read():
    """The global score and the overlap count do not touch the linear branch: its restrictions (d_f == d, W <= 256,
    no fp32 with d = C = 128) must not be applied to them.  Null pointers make the calls stop right after the
    parameter checks, with the pointer message."""
    lib = S.lib()
    null = ctypes.c_void_p(None)
    for kw in (dict(dtype="f32", d=128, C=128), dict(d_f=32), dict(W=4096), dict(C=32, lam=0)):
        p = params(**kw)
        p.q_st = p.k_st = kw.get("d", 64)
        rc = lib.still_global_score(ctypes.byref(p), null, null, null, null)
        assert rc == S.STILL_ERR_INVALID_ARG and "pointer" in S.still_last_error(), (kw, S.still_last_error())
    p = params(C=32, lam=7, d_f=5, W=999)
    rc = lib.still_selection_overlap(ctypes.byref(p), null, null, null, null)
    assert rc == S.STILL_ERR_INVALID_ARG and "pointer" in S.still_last_error()
    for kw, code in ((dict(d=96), S.STILL_ERR_UNSUPPORTED), (dict(eps=0.0), S.STILL_ERR_INVALID_ARG)):
        p = params(**kw)
        assert lib.still_global_score(ctypes.byref(p), null, null, null, null) == code
    for kw, code in ((dict(C=256), S.STILL_ERR_UNSUPPORTED), (dict(lam=65), S.STILL_ERR_INVALID_ARG)):
        p = params(**kw)
        assert lib.still_selection_overlap(ctypes.byref(p), null, null, null, null) == code


def test_public_header_is_plain_c_and_matches_the_binding(tmp_path):
    """include/still.h compiles as C99 on its own, and the struct sizes the C compiler sees are the ones the ctypes
    binding marshals (a field added on one side only would shift every later field)."""
    import shutil
    import subprocess

    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "still.h"\n'
                   'int main(void) { printf("%zu %zu %zu %zu %zu\\n", sizeof(still_params_t), sizeof(still_ws_layout_t),\n'
                   '  sizeof(still_state_layout_t), offsetof(still_params_t, q_sb), offsetof(still_params_t, seq_len));\n'
                   '  return 0; }\n')
    exe = tmp_path / "sizes"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got == [ctypes.sizeof(S.StillParams), ctypes.sizeof(S.StillWsLayout), ctypes.sizeof(S.StillStateLayout),
                   S.StillParams.q_sb.offset, S.StillParams.seq_len.offset]
