"""ctypes binding of libstill's C ABI (include/still.h): same names, argument marshalling only.

Every step of the path runs inside the library's HIP kernels.  torch is used for device
memory and streams; tensors are passed as raw device pointers.  There is no CPU fallback:
if the library has not been built the import of the native handle raises.
"""
from __future__ import annotations

import ctypes as ct
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libstill.so")   # the in-tree build, nothing else

STILL_OK, STILL_ERR_INVALID_ARG, STILL_ERR_UNSUPPORTED, STILL_ERR_WORKSPACE_TOO_SMALL, STILL_ERR_HIP, \
    STILL_ERR_STATE = range(6)
STILL_F32, STILL_BF16 = 0, 1
DTYPE_CODE = {"f32": STILL_F32, "bf16": STILL_BF16}


class StillParams(ct.Structure):
    _fields_ = [
        ("B", ct.c_int32), ("N", ct.c_int32), ("Hq", ct.c_int32), ("Hkv", ct.c_int32), ("d", ct.c_int32),
        ("d_f", ct.c_int32), ("C", ct.c_int32), ("W", ct.c_int32), ("lam", ct.c_int32),
        ("scale", ct.c_float), ("eps", ct.c_float), ("dtype", ct.c_int32), ("max_tokens", ct.c_int32),
        ("max_retained", ct.c_int32), ("shared_selection", ct.c_int32), ("emit_terms", ct.c_int32),
        ("gate_activation", ct.c_int32), ("budget_policy", ct.c_int32),
        ("q_sb", ct.c_int64), ("q_st", ct.c_int64), ("q_sh", ct.c_int64),
        ("k_sb", ct.c_int64), ("k_st", ct.c_int64), ("k_sh", ct.c_int64),
        ("v_sb", ct.c_int64), ("v_st", ct.c_int64), ("v_sh", ct.c_int64),
        ("o_sb", ct.c_int64), ("o_st", ct.c_int64), ("o_sh", ct.c_int64),
        ("g_sb", ct.c_int64), ("g_st", ct.c_int64), ("g_sh", ct.c_int64),
        ("kv_head_of_q", ct.POINTER(ct.c_int32)),
        ("seq_len", ct.c_void_p),
    ]


class StillWsLayout(ct.Structure):
    _fields_ = [(n, ct.c_size_t) for n in
                ("score", "sel", "vt", "kret", "vrett", "wqt", "wkf", "seg", "snap", "zsnap", "pimg", "zpre", "kmask", "n_la", "d_la", "vfr", "ev_src", "ev_alive", "ev_fin", "ev_vfr", "lse", "total")] + \
               [(n, ct.c_int32) for n in ("n_pad", "cap", "nseg", "seg_chunks")]


class StillStateLayout(ct.Structure):
    _fields_ = [(n, ct.c_size_t) for n in
                ("S", "kret", "vret", "sel", "kring", "vring", "score", "part", "ret_score", "ret_tok", "total")] + \
               [(n, ct.c_int32) for n in ("cap", "R", "n_chunks")]


class StillBwdWsLayout(ct.Structure):
    _fields_ = [(n, ct.c_size_t) for n in
                ("fwd", "e_row", "delta", "ed", "a", "phi_q", "phi_k", "uq", "uk", "stq", "stk", "nraw", "gq",
                 "dphi_k", "ds", "dz", "dfq", "dfk", "dq32", "dk32", "dv32", "cxq", "cxk", "qt", "dot", "kt", "kret", "krett", "total")] + \
               [(n, ct.c_int32) for n in ("n_pad_t", "cap_t")]


class StillError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libstill status {code}: {text}")
        self.code = code


_lib = None


def lib() -> ct.CDLL:
    """The loaded library; raises if it was never built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2602_02180_amd.build`")
        # torch first: its wheel carries its own copy of the HIP runtime, and the process must end up with ONE
        # runtime.  Loaded after torch, this library's runtime dependency resolves to the copy torch brought;
        # loaded before it, the system copy comes in as a second runtime and every launch from here fails with
        # "no ROCm-capable device".  Importing torch does not touch the GPU.
        import torch  # noqa: F401

        L = ct.CDLL(LIB_PATH)
        vp, pp = ct.c_void_p, ct.POINTER(StillParams)
        L.still_version.restype = ct.c_int32
        L.still_last_error.restype = ct.c_char_p
        L.still_fwd_workspace_bytes.restype = ct.c_size_t
        L.still_fwd_workspace_bytes.argtypes = [pp]
        L.still_fwd_workspace_layout.restype = ct.c_int
        L.still_fwd_workspace_layout.argtypes = [pp, ct.POINTER(StillWsLayout)]
        L.still_hybrid_attn_fwd.restype = ct.c_int
        L.still_hybrid_attn_fwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ct.c_int32, vp, vp,
                                            ct.c_size_t, vp]
        L.still_hybrid_attn_fwd_static.restype = ct.c_int
        L.still_hybrid_attn_fwd_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ct.c_int32, vp, vp]
        L.still_state_bytes.restype = ct.c_size_t
        L.still_state_bytes.argtypes = [pp]
        L.still_state_layout.restype = ct.c_int
        L.still_state_layout.argtypes = [pp, ct.POINTER(StillStateLayout)]
        L.still_state_init.restype = ct.c_int
        L.still_state_init.argtypes = [pp, vp, vp]
        L.still_hybrid_attn_decode_step.restype = ct.c_int
        L.still_hybrid_attn_decode_step.argtypes = [pp, vp, ct.c_int32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.still_hybrid_attn_decode_step_at.restype = ct.c_int
        L.still_hybrid_attn_decode_step_at.argtypes = [pp, vp, vp, ct.c_int32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.still_global_score.restype = ct.c_int
        L.still_global_score.argtypes = [pp, vp, vp, vp, vp]
        L.still_selection_overlap.restype = ct.c_int
        L.still_selection_overlap.argtypes = [pp, vp, vp, vp, vp]
        L.still_bwd_workspace_bytes.restype = ct.c_size_t
        L.still_bwd_workspace_bytes.argtypes = [pp]
        L.still_bwd_workspace_layout.restype = ct.c_int
        L.still_bwd_workspace_layout.argtypes = [pp, ct.POINTER(StillBwdWsLayout)]
        L.still_hybrid_attn_bwd.restype = ct.c_int
        L.still_hybrid_attn_bwd.argtypes = [pp] + [vp] * 20 + [vp, ct.c_size_t, vp]
        L.still_attention_map.restype = ct.c_int
        L.still_attention_map.argtypes = [pp] + [vp] * 9 + [vp, ct.c_size_t, vp]
        L.still_attention_map_bwd_workspace_bytes.restype = ct.c_size_t
        L.still_attention_map_bwd_workspace_bytes.argtypes = [pp]
        L.still_attention_map_bwd.restype = ct.c_int
        L.still_attention_map_bwd.argtypes = [pp] + [vp] * 14 + [vp, ct.c_size_t, vp]
        L.still_rope_apply.restype = ct.c_int
        L.still_rope_apply.argtypes = [pp, vp, vp, vp, ct.c_float, vp]
        L.still_profile_enable.restype = None
        L.still_profile_enable.argtypes = [ct.c_int32]
        L.still_profile_read.restype = ct.c_int
        L.still_profile_read.argtypes = [ct.POINTER(ct.c_float), ct.c_int32]
        L.still_profile_kernel_name.restype = ct.c_char_p
        L.still_profile_kernel_name.argtypes = [ct.c_int32]
        _lib = L
    return _lib


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _check(code: int) -> None:
    if code != STILL_OK:
        raise StillError(code, still_last_error())


def _strides(t):
    if t is None:
        return 0, 0, 0
    assert t.dim() == 4 and t.stride(3) == 1, "tensors are [B, N, H, d] with a contiguous last dim"
    return t.stride(0), t.stride(1), t.stride(2)


def make_params(*, B, N, Hq, Hkv, d, C, W, lam, scale, eps, dtype, d_f=None, q=None, k=None, v=None, out=None,
                g=None, kv_head_of_q=None, max_tokens=0, max_retained=0, shared_selection=0, seq_len=None,
                emit_terms=0, gate_activation=0, budget_policy=0) -> StillParams:
    """Fill a still_params_t; strides are taken from the torch tensors ([B, N, H, d])."""
    p = StillParams()
    p.B, p.N, p.Hq, p.Hkv, p.d, p.d_f = B, N, Hq, Hkv, d, (d_f or d)
    p.C, p.W, p.lam, p.scale, p.eps = C, W, lam, scale, eps
    p.dtype = DTYPE_CODE[dtype] if isinstance(dtype, str) else dtype
    p.max_tokens = max_tokens
    p.max_retained = max_retained
    p.shared_selection = int(shared_selection)
    p.emit_terms = int(emit_terms)
    p.gate_activation = int(gate_activation)
    p.budget_policy = int(budget_policy)
    if seq_len is not None:   # int32 device tensor [B]; kept alive by the params object
        assert seq_len.is_cuda and seq_len.is_contiguous() and seq_len.numel() == B and str(seq_len.dtype) == "torch.int32"
        p._seq_len_keepalive = seq_len
        p.seq_len = seq_len.data_ptr()
    p.q_sb, p.q_st, p.q_sh = _strides(q)
    p.k_sb, p.k_st, p.k_sh = _strides(k)
    p.v_sb, p.v_st, p.v_sh = _strides(v)
    p.o_sb, p.o_st, p.o_sh = _strides(out)
    p.g_sb, p.g_st, p.g_sh = _strides(g)
    if kv_head_of_q is not None:
        arr = (C_int32_array(len(kv_head_of_q)))(*[int(x) for x in kv_head_of_q])
        p._keepalive = arr
        p.kv_head_of_q = ct.cast(arr, ct.POINTER(ct.c_int32))
    return p


def C_int32_array(n):
    return ct.c_int32 * n


# ------------------------------------------------------------------ entry points (same names as still.h)

def still_version() -> int:
    return int(lib().still_version())


def still_last_error() -> str:
    return lib().still_last_error().decode()


def still_fwd_workspace_bytes(p: StillParams) -> int:
    n = int(lib().still_fwd_workspace_bytes(ct.byref(p)))
    if n == 0:
        raise StillError(-1, still_last_error())
    return n


def still_fwd_workspace_layout(p: StillParams) -> StillWsLayout:
    L = StillWsLayout()
    _check(lib().still_fwd_workspace_layout(ct.byref(p), ct.byref(L)))
    return L


def still_hybrid_attn_fwd(p: StillParams, q, k, v, g, Wq, bq, Wk, bk, out, score_out=None, sel_idx=None,
                          sel_idx_is_input: bool = False, state_out=None, workspace=None, stream=None) -> None:
    """Enqueue the prefill on `stream` (a torch.cuda.Stream; default: torch's current stream)."""
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_hybrid_attn_fwd(
        ct.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(Wq), _ptr(bq), _ptr(Wk), _ptr(bk), _ptr(out),
        _ptr(score_out), _ptr(sel_idx), 1 if sel_idx_is_input else 0, _ptr(state_out), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), stream.cuda_stream))


STILL_STATIC_WORKSPACE_BYTES = 32 << 20


def still_hybrid_attn_fwd_static(p: StillParams, q, k, v, g, Wq, bq, Wk, bk, out, score_out=None, sel_idx=None,
                                 sel_idx_is_input: bool = False, state_out=None, stream=None) -> None:
    """The prefill with the library's built-in scratch array as workspace (allocates nothing)."""
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_hybrid_attn_fwd_static(
        ct.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(Wq), _ptr(bq), _ptr(Wk), _ptr(bk), _ptr(out),
        _ptr(score_out), _ptr(sel_idx), 1 if sel_idx_is_input else 0, _ptr(state_out), stream.cuda_stream))


def still_bwd_workspace_bytes(p: StillParams) -> int:
    n = lib().still_bwd_workspace_bytes(ct.byref(p))
    if n == 0:
        raise StillError(STILL_ERR_INVALID_ARG, still_last_error())
    return n


def still_bwd_workspace_layout(p: StillParams) -> StillBwdWsLayout:
    L = StillBwdWsLayout()
    _check(lib().still_bwd_workspace_layout(ct.byref(p), ct.byref(L)))
    return L


def still_hybrid_attn_bwd(p: StillParams, q, k, v, g, Wq, bq, Wk, bk, out, dout, lse, sel_idx, dq, dk, dv, dg,
                          dWq, dbq, dWk, dbk, workspace, stream=None) -> None:
    """Enqueue the backward pass of the prefill on `stream` (default: torch's current stream)."""
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_hybrid_attn_bwd(
        ct.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(Wq), _ptr(bq), _ptr(Wk), _ptr(bk), _ptr(out),
        _ptr(dout), _ptr(lse), _ptr(sel_idx), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dg), _ptr(dWq), _ptr(dbq),
        _ptr(dWk), _ptr(dbk), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), stream.cuda_stream))


def still_attention_map(p: StillParams, q, k, Wq, bq, Wk, bk, lse, sel_idx, map_out, workspace, stream=None) -> None:
    """The operator's attention map [B, Hq, N, N] (float32) for the forward call that produced lse and sel_idx."""
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_attention_map(
        ct.byref(p), _ptr(q), _ptr(k), _ptr(Wq), _ptr(bq), _ptr(Wk), _ptr(bk), _ptr(lse), _ptr(sel_idx), _ptr(map_out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), stream.cuda_stream))


def still_attention_map_bwd_workspace_bytes(p: StillParams) -> int:
    n = lib().still_attention_map_bwd_workspace_bytes(ct.byref(p))
    if n == 0:
        raise StillError(STILL_ERR_INVALID_ARG, still_last_error())
    return n


def still_attention_map_bwd(p: StillParams, q, k, Wq, bq, Wk, bk, lse, sel_idx, amap, dmap, dWq, dbq, dWk, dbk,
                            workspace, stream=None) -> None:
    """Gradient of a loss on the attention map w.r.t. the feature-map parameters (float32 outputs)."""
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_attention_map_bwd(
        ct.byref(p), _ptr(q), _ptr(k), _ptr(Wq), _ptr(bq), _ptr(Wk), _ptr(bk), _ptr(lse), _ptr(sel_idx), _ptr(amap),
        _ptr(dmap), _ptr(dWq), _ptr(dbq), _ptr(dWk), _ptr(dbk), _ptr(workspace),
        workspace.numel() * workspace.element_size(), stream.cuda_stream))


def still_rope_apply(p: StillParams, q, k, pos0=None, base: float = 10000.0, stream=None) -> None:
    """Rotate q and / or k in place by their positions (pos0: int32 device tensor [B] or None)."""
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_rope_apply(ct.byref(p), _ptr(q), _ptr(k), _ptr(pos0), ct.c_float(base), stream.cuda_stream))


def still_state_bytes(p: StillParams) -> int:
    n = int(lib().still_state_bytes(ct.byref(p)))
    if n == 0:
        raise StillError(-1, still_last_error())
    return n


def still_state_layout(p: StillParams) -> StillStateLayout:
    L = StillStateLayout()
    _check(lib().still_state_layout(ct.byref(p), ct.byref(L)))
    return L


def still_state_init(p: StillParams, state, stream=None) -> None:
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_state_init(ct.byref(p), _ptr(state), stream.cuda_stream))


def still_hybrid_attn_decode_step(p: StillParams, state, t: int, q_t, k_t, v_t, g_t, Wq, bq, Wk, bk, out_t,
                                  stream=None) -> None:
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_hybrid_attn_decode_step(ct.byref(p), _ptr(state), t, _ptr(q_t), _ptr(k_t), _ptr(v_t),
                                               _ptr(g_t), _ptr(Wq), _ptr(bq), _ptr(Wk), _ptr(bk), _ptr(out_t),
                                               stream.cuda_stream))


def still_hybrid_attn_decode_step_at(p: StillParams, state, t_dev, t_max: int, q_t, k_t, v_t, g_t, Wq, bq, Wk, bk,
                                     out_t, stream=None) -> None:
    """t_dev: int32 device tensor [B] with each sequence's token index; t_max: host upper bound of them."""
    import torch

    assert t_dev.dtype == torch.int32 and t_dev.is_cuda and t_dev.is_contiguous()
    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_hybrid_attn_decode_step_at(ct.byref(p), _ptr(state), _ptr(t_dev), t_max, _ptr(q_t), _ptr(k_t),
                                                  _ptr(v_t), _ptr(g_t), _ptr(Wq), _ptr(bq), _ptr(Wk), _ptr(bk),
                                                  _ptr(out_t), stream.cuda_stream))


def still_global_score(p: StillParams, q, k, score_out, stream=None) -> None:
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_global_score(ct.byref(p), _ptr(q), _ptr(k), _ptr(score_out), stream.cuda_stream))


def still_selection_overlap(p: StillParams, score_a, score_b, overlap, stream=None) -> None:
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    _check(lib().still_selection_overlap(ct.byref(p), _ptr(score_a), _ptr(score_b), _ptr(overlap),
                                         stream.cuda_stream))


STILL_PROFILE_SLOTS = 8


def still_profile_enable(on) -> None:
    """False/0 = off, True/1 = every kernel, 2 = the last (dominant) kernel only."""
    lib().still_profile_enable(int(on))


def still_profile_read():
    """Milliseconds per kernel of the last profiled prefill call on this thread: {name: ms}."""
    arr = (ct.c_float * STILL_PROFILE_SLOTS)()
    _check(lib().still_profile_read(arr, STILL_PROFILE_SLOTS))
    return {still_profile_kernel_name(i): float(arr[i]) for i in range(STILL_PROFILE_SLOTS)}


def still_profile_kernel_name(i: int):
    s = lib().still_profile_kernel_name(i)
    return None if s is None else s.decode()
