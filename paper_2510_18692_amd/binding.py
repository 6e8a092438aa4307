"""ctypes binding of libmoga.so: argument marshalling only.

Every function has the name and the argument order of its C entry point in
include/moga.h.  torch is used for device memory (`torch.empty`, `.data_ptr()`)
and for the current HIP stream; every step of the path runs in the library's
kernels.  There is no fallback: if the library cannot be loaded the import of
any entry point raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoga.so")

MOGA_F32, MOGA_BF16 = 0, 1
(OP_ROUTE, OP_PERMUTE, OP_ATTN_FWD, OP_ATTN_BWD, OP_ROUTE_BWD, OP_BALANCE_LOSS, OP_VARLEN_ATTN_FWD,
 OP_VARLEN_ATTN_BWD) = range(8)

_c = ctypes
_vp, _i64, _i32, _f32, _sz = _c.c_void_p, _c.c_int64, _c.c_int, _c.c_float, _c.c_size_t
_SIGNATURES = {
    "moga_status_string": (_c.c_char_p, [_i32]),
    "moga_version": (_i32, []),
    "moga_workspace_bytes": (_sz, [_i32, _i64, _i32, _i32, _i32, _i32, _i32]),
    "moga_route": (_i32, [_vp, _i32, _vp, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moga_permute": (_i32, [_vp, _i64, _i32, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp,
                            _vp, _vp, _vp, _vp, _sz, _vp]),
    "moga_permute_static": (_i32, [_vp, _i64, _i32, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp,
                                   _vp, _vp, _vp, _vp, _vp]),
    "moga_group_attn_fwd": (_i32, [_vp, _vp, _vp, _i32, _i64, _i32, _i32, _vp, _i32, _f32, _vp, _vp,
                                   _vp, _sz, _vp]),
    "moga_unpermute": (_i32, [_vp, _i32, _vp, _vp, _i64, _i32, _i32, _vp, _vp]),
    "moga_unpermute_bwd": (_i32, [_vp, _vp, _i32, _vp, _vp, _i64, _i32, _i32, _vp, _vp, _vp]),
    "moga_group_attn_bwd": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i64, _i32, _i32, _vp, _i32,
                                   _f32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moga_attn_bwd_status_offset": (_sz, [_i64, _i32]),
    "moga_debug_set_spin_limit": (None, [_i32]),
    "moga_debug_set_small_group_rows": (None, [_i64]),
    "moga_permute_bwd": (_i32, [_vp, _vp, _vp, _i32, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp]),
    "moga_route_bwd": (_i32, [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _vp, _vp,
                              _sz, _vp]),
    "moga_fused_attn_fwd": (_i32, [_vp, _vp, _vp, _i32, _i64, _i32, _i32, _vp, _vp, _vp, _i32, _f32, _vp, _vp, _vp]),
    "moga_fused_attn_bwd": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _i32, _f32,
                                   _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moga_varlen_attn_fwd": (_i32, [_vp, _vp, _vp, _i32, _i64, _i64, _i32, _i32, _vp, _vp, _i32, _f32, _vp, _vp,
                                    _vp, _sz, _vp]),
    "moga_varlen_attn_bwd": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i64, _i64, _i32, _i32, _vp, _vp, _i32,
                                    _f32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moga_stga_index_sizes": (_i32, [_i32, _i32, _i32, _i32, _i32, _i32, _vp, _i32, _i32, _vp, _vp]),
    "moga_stga_build_index": (_i32, [_i32, _i32, _i32, _i32, _i32, _i32, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp,
                                     _vp, _vp]),
    "moga_gather_rows": (_i32, [_vp, _i32, _vp, _i64, _i32, _i32, _vp, _vp]),
    "moga_gather_rows_bwd": (_i32, [_vp, _i32, _vp, _vp, _i64, _i64, _i32, _i32, _i32, _vp, _vp]),
    "moga_gather3_bwd": (_i32, [_vp, _vp, _vp, _vp, _vp, _i64, _vp, _vp, _i32, _i64, _i32, _i32, _vp, _vp]),
    "moga_merge3_fwd": (_i32, [_vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _vp]),
    "moga_merge3_bwd": (_i32, [_vp, _vp, _i32, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _vp]),
    "moga_balance_loss": (_i32, [_vp, _vp, _i64, _i32, _f32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moga_balance_loss_bwd": (_i32, [_vp, _vp, _i64, _i32, _f32, _f32, _vp, _i32, _vp, _vp]),
}
EXPORTS = tuple(_SIGNATURES)

_lib = None


class MogaError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__(f"{fn} failed: {status_string(status)} ({status})")


def load():
    """Load libmoga.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)   # AttributeError if an export is missing: fail loudly
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().moga_status_string(int(status)).decode()


def version() -> int:
    return load().moga_version()


def workspace_bytes(op, N, H, D, M, d_model, dtype) -> int:
    return int(load().moga_workspace_bytes(op, N, H, D, M, d_model, dtype))


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MOGA_F32
    if t.dtype == torch.bfloat16:
        return MOGA_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _p(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def _stream(stream):
    return (stream if stream is not None else torch.cuda.current_stream()).cuda_stream


def _ws(nbytes, device):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def _check(fn, status):
    if status != 0:
        raise MogaError(fn, status)


def moga_route(x, w, bias=None, want_probs=True, want_logits=False, stream=None):
    """-> (group int32 [N], gate f32 [N], probs f32 [N, M] | None, logits f32 [N, M] | None)"""
    N, d = x.shape
    M = w.shape[0]
    dev = x.device
    group = torch.empty(N, dtype=torch.int32, device=dev)
    gate = torch.empty(N, dtype=torch.float32, device=dev)
    probs = torch.empty((N, M), dtype=torch.float32, device=dev) if want_probs else None
    logits = torch.empty((N, M), dtype=torch.float32, device=dev) if want_logits else None
    st = load().moga_route(_p(x), _dt(x), _p(w), _p(bias), N, d, M, _p(group), _p(gate), _p(probs),
                           _p(logits), None, 0, _stream(stream))
    _check("moga_route", st)
    return group, gate, probs, logits


def moga_permute(group, M, q=None, k=None, v=None, stream=None):
    """-> dict(counts, cu_seqlens, max_seqlen, perm, inv_perm[, qh, kh, vh])"""
    N = group.shape[0]
    dev = group.device
    i32 = dict(dtype=torch.int32, device=dev)
    out = {
        "counts": torch.empty(M, **i32), "cu_seqlens": torch.empty(M + 1, **i32),
        "max_seqlen": torch.empty(1, **i32), "perm": torch.empty(N, **i32),
        "inv_perm": torch.empty(N, **i32),
    }
    H = D = 0
    dt = MOGA_F32
    if q is not None:
        _, H, D = q.shape
        dt = _dt(q)
        for name, t in (("qh", q), ("kh", k), ("vh", v)):
            out[name] = torch.empty((H, N, D), dtype=t.dtype, device=dev)
    nws = workspace_bytes(OP_PERMUTE, N, H, D, M, 0, dt)
    ws = _ws(nws, dev)
    st = load().moga_permute(_p(group), N, M, _p(q), _p(k), _p(v), dt, H, D, _p(out["counts"]),
                             _p(out["cu_seqlens"]), _p(out["max_seqlen"]), _p(out["perm"]),
                             _p(out["inv_perm"]), _p(out.get("qh")), _p(out.get("kh")),
                             _p(out.get("vh")), _p(ws), ws.numel(), _stream(stream))
    _check("moga_permute", st)
    return out


def moga_permute_static(group, M, out, q=None, k=None, v=None, stream=None):
    """moga_permute without a workspace and without any allocation, here or in the library:
    `out` holds the caller's tensors counts [M], cu_seqlens [M+1], max_seqlen [1], perm [N],
    inv_perm [N] (and qh, kh, vh [H, N, D] when q, k, v are given); they are written in place."""
    N = group.shape[0]
    H = D = 0
    dt = MOGA_F32
    if q is not None:
        _, H, D = q.shape
        dt = _dt(q)
    st = load().moga_permute_static(_p(group), N, M, _p(q), _p(k), _p(v), dt, H, D, _p(out["counts"]),
                                    _p(out["cu_seqlens"]), _p(out["max_seqlen"]), _p(out["perm"]),
                                    _p(out["inv_perm"]), _p(out.get("qh")), _p(out.get("kh")),
                                    _p(out.get("vh")), _stream(stream))
    _check("moga_permute_static", st)
    return out


def moga_group_attn_fwd(qh, kh, vh, cu_seqlens, softmax_scale, stream=None, out=None, lse=None):
    """-> (oh [H, N, D], lse f32 [H, N])"""
    H, N, D = qh.shape
    M = cu_seqlens.shape[0] - 1
    oh = out if out is not None else torch.empty_like(qh)
    lse = lse if lse is not None else torch.empty((H, N), dtype=torch.float32, device=qh.device)
    st = load().moga_group_attn_fwd(_p(qh), _p(kh), _p(vh), _dt(qh), N, H, D, _p(cu_seqlens), M,
                                    float(softmax_scale), _p(oh), _p(lse), None, 0, _stream(stream))
    _check("moga_group_attn_fwd", st)
    return oh, lse


def moga_unpermute(oh, perm, gate=None, stream=None, out=None):
    """-> o [N, H, D]"""
    H, N, D = oh.shape
    o = out if out is not None else torch.empty((N, H, D), dtype=oh.dtype, device=oh.device)
    st = load().moga_unpermute(_p(oh), _dt(oh), _p(perm), _p(gate), N, H, D, _p(o), _stream(stream))
    _check("moga_unpermute", st)
    return o


def moga_unpermute_bwd(d_o, oh, perm, gate, stream=None):
    """-> (d_oh [H, N, D], d_gate f32 [N])"""
    H, N, D = oh.shape
    d_oh = torch.empty_like(oh)
    d_gate = torch.empty(N, dtype=torch.float32, device=oh.device)
    st = load().moga_unpermute_bwd(_p(d_o), _p(oh), _dt(oh), _p(perm), _p(gate), N, H, D, _p(d_oh),
                                   _p(d_gate), _stream(stream))
    _check("moga_unpermute_bwd", st)
    return d_oh, d_gate


def attn_bwd_status(ws, Nq, H):
    """The int32 status word of a backward workspace (0 after every correct run), as a 1-element view."""
    off = int(load().moga_attn_bwd_status_offset(Nq, H))
    return ws[off:off + 4].view(torch.int32)


def set_small_group_rows(rows: int) -> None:
    """Mean group size below which the bf16 attention calls use their small-group kernels (< 0: defaults)."""
    load().moga_debug_set_small_group_rows(int(rows))


def set_spin_limit(polls: int) -> None:
    load().moga_debug_set_spin_limit(int(polls))


def moga_group_attn_bwd(d_oh, qh, kh, vh, oh, lse, cu_seqlens, softmax_scale, stream=None, ws=None):
    """-> (d_qh, d_kh, d_vh) each [H, N, D].  `ws`: the caller's workspace (uint8), else one is allocated."""
    H, N, D = qh.shape
    M = cu_seqlens.shape[0] - 1
    d_qh, d_kh, d_vh = torch.empty_like(qh), torch.empty_like(kh), torch.empty_like(vh)
    if ws is None:
        ws = _ws(workspace_bytes(OP_ATTN_BWD, N, H, D, M, 0, _dt(qh)), qh.device)
    st = load().moga_group_attn_bwd(_p(d_oh), _p(qh), _p(kh), _p(vh), _p(oh), _p(lse), _dt(qh), N, H, D,
                                    _p(cu_seqlens), M, float(softmax_scale), _p(d_qh), _p(d_kh),
                                    _p(d_vh), _p(ws), ws.numel(), _stream(stream))
    _check("moga_group_attn_bwd", st)
    return d_qh, d_kh, d_vh


def moga_permute_bwd(d_qh, d_kh, d_vh, perm, stream=None):
    """-> (d_q, d_k, d_v) each [N, H, D]"""
    H, N, D = d_qh.shape
    mk = lambda t: torch.empty((N, H, D), dtype=t.dtype, device=t.device)
    d_q, d_k, d_v = mk(d_qh), mk(d_kh), mk(d_vh)
    st = load().moga_permute_bwd(_p(d_qh), _p(d_kh), _p(d_vh), _dt(d_qh), _p(perm), N, H, D, _p(d_q),
                                 _p(d_k), _p(d_v), _stream(stream))
    _check("moga_permute_bwd", st)
    return d_q, d_k, d_v


def moga_route_bwd(x, w, probs, group, gate, d_gate, want_dx=False, stream=None):
    """-> (d_w f32 [M, d_model], d_x f32 [N, d_model] | None)"""
    N, d = x.shape
    M = w.shape[0]
    d_w = torch.empty((M, d), dtype=torch.float32, device=x.device)
    d_x = torch.empty((N, d), dtype=torch.float32, device=x.device) if want_dx else None
    ws = _ws(workspace_bytes(OP_ROUTE_BWD, N, 0, 0, M, d, _dt(x)), x.device)
    st = load().moga_route_bwd(_p(x), _dt(x), _p(w), _p(probs), _p(group), _p(gate), _p(d_gate), N, d, M,
                               _p(d_w), _p(d_x), _p(ws), ws.numel(), _stream(stream))
    _check("moga_route_bwd", st)
    return d_w, d_x


def moga_fused_attn_fwd(q, k, v, perm, gate, cu_seqlens, softmax_scale, stream=None):
    """q, k, v [N, H, D] token order -> (o [N, H, D] gated, token order; lse f32 [H, N] sorted order)"""
    N, H, D = q.shape
    M = cu_seqlens.shape[0] - 1
    o = torch.empty_like(q)
    lse = torch.empty((H, N), dtype=torch.float32, device=q.device)
    st = load().moga_fused_attn_fwd(_p(q), _p(k), _p(v), _dt(q), N, H, D, _p(perm), _p(gate), _p(cu_seqlens), M,
                                    float(softmax_scale), _p(o), _p(lse), _stream(stream))
    _check("moga_fused_attn_fwd", st)
    return o, lse


def moga_fused_attn_bwd(d_o, q, k, v, o, lse, perm, inv_perm, gate, cu_seqlens, softmax_scale, stream=None):
    """Token-order tensors -> (d_q, d_k, d_v [N, H, D], d_gate f32 [N])"""
    N, H, D = q.shape
    M = cu_seqlens.shape[0] - 1
    d_q, d_k, d_v = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    d_gate = torch.empty(N, dtype=torch.float32, device=q.device)
    ws = _ws(workspace_bytes(OP_ATTN_BWD, N, H, D, M, 0, _dt(q)), q.device)
    st = load().moga_fused_attn_bwd(_p(d_o), _p(q), _p(k), _p(v), _p(o), _p(lse), _dt(q), N, H, D, _p(perm),
                                    _p(inv_perm), _p(gate), _p(cu_seqlens), M, float(softmax_scale), _p(d_q),
                                    _p(d_k), _p(d_v), _p(d_gate), _p(ws), ws.numel(), _stream(stream))
    _check("moga_fused_attn_bwd", st)
    return d_q, d_k, d_v, d_gate


def moga_varlen_attn_fwd(qh, kh, vh, cu_seqlens_q, cu_seqlens_k, softmax_scale, stream=None):
    """qh [H, Nq, D]; kh, vh [H, Nk, D] -> (oh [H, Nq, D], lse f32 [H, Nq])"""
    H, Nq, D = qh.shape
    Nk = kh.shape[1]
    G = cu_seqlens_q.shape[0] - 1
    oh = torch.empty_like(qh)
    lse = torch.empty((H, Nq), dtype=torch.float32, device=qh.device)
    ws = _ws(workspace_bytes(OP_VARLEN_ATTN_FWD, Nq, H, D, G, 0, _dt(qh)), qh.device)
    st = load().moga_varlen_attn_fwd(_p(qh), _p(kh), _p(vh), _dt(qh), Nq, Nk, H, D, _p(cu_seqlens_q),
                                     _p(cu_seqlens_k), G, float(softmax_scale), _p(oh), _p(lse), _p(ws),
                                     ws.numel(), _stream(stream))
    _check("moga_varlen_attn_fwd", st)
    return oh, lse


def moga_varlen_attn_bwd(d_oh, qh, kh, vh, oh, lse, cu_seqlens_q, cu_seqlens_k, softmax_scale, stream=None):
    """-> (d_qh [H, Nq, D], d_kh, d_vh [H, Nk, D])"""
    H, Nq, D = qh.shape
    Nk = kh.shape[1]
    G = cu_seqlens_q.shape[0] - 1
    d_qh, d_kh, d_vh = torch.empty_like(qh), torch.empty_like(kh), torch.empty_like(vh)
    ws = _ws(workspace_bytes(OP_VARLEN_ATTN_BWD, Nq, H, D, G, 0, _dt(qh)), qh.device)
    st = load().moga_varlen_attn_bwd(_p(d_oh), _p(qh), _p(kh), _p(vh), _p(oh), _p(lse), _dt(qh), Nq, Nk, H, D,
                                     _p(cu_seqlens_q), _p(cu_seqlens_k), G, float(softmax_scale), _p(d_qh),
                                     _p(d_kh), _p(d_vh), _p(ws), ws.numel(), _stream(stream))
    _check("moga_varlen_attn_bwd", st)
    return d_qh, d_kh, d_vh


def moga_stga_build_index(T, Hh, Ww, wh, ww, tg, shot_of_frame, a_prev=1, a_next=1, device="cuda"):
    """Static index lists (host builder), uploaded to `device` (None keeps them as numpy arrays)."""
    import numpy as np
    shots = np.ascontiguousarray(np.asarray(shot_of_frame, dtype=np.int32))
    assert shots.shape == (T,)
    G, Nk = ctypes.c_int64(0), ctypes.c_int64(0)
    sp = shots.ctypes.data_as(ctypes.c_void_p)
    st = load().moga_stga_index_sizes(T, Hh, Ww, wh, ww, tg, sp, a_prev, a_next, ctypes.byref(G), ctypes.byref(Nk))
    _check("moga_stga_index_sizes", st)
    N, G, Nk = T * Hh * Ww, G.value, Nk.value
    out = {"q_index": np.empty(N, np.int32), "q_slot": np.empty(N, np.int32), "cu_q": np.empty(G + 1, np.int32),
           "kv_index": np.empty(Nk, np.int32), "cu_k": np.empty(G + 1, np.int32),
           "inv_cu": np.empty(N + 1, np.int32), "inv_slots": np.empty(Nk, np.int32)}
    hp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    st = load().moga_stga_build_index(T, Hh, Ww, wh, ww, tg, sp, a_prev, a_next, hp(out["q_index"]),
                                      hp(out["q_slot"]), hp(out["cu_q"]), hp(out["kv_index"]), hp(out["cu_k"]),
                                      hp(out["inv_cu"]), hp(out["inv_slots"]))
    _check("moga_stga_build_index", st)
    if device is not None:
        out = {k: torch.from_numpy(v).to(device) for k, v in out.items()}
    out["n_groups"], out["n_keys"] = G, Nk
    return out


def moga_gather_rows(src, index, stream=None):
    """src [N, H, D], index [Nk] -> [H, Nk, D]"""
    N, H, D = src.shape
    Nk = index.shape[0]
    dst = torch.empty((H, Nk, D), dtype=src.dtype, device=src.device)
    st = load().moga_gather_rows(_p(src), _dt(src), _p(index), Nk, H, D, _p(dst), _stream(stream))
    _check("moga_gather_rows", st)
    return dst


def moga_gather_rows_bwd(d_dst, inv_cu, inv_slots, N, d_src=None, stream=None):
    """d_dst [H, Nk, D] -> d_src [N, H, D]; adds into `d_src` when given."""
    H, Nk, D = d_dst.shape
    accumulate = d_src is not None
    if d_src is None:
        d_src = torch.empty((N, H, D), dtype=d_dst.dtype, device=d_dst.device)
    st = load().moga_gather_rows_bwd(_p(d_dst), _dt(d_dst), _p(inv_cu), _p(inv_slots), N, Nk, H, D,
                                     int(accumulate), _p(d_src), _stream(stream))
    _check("moga_gather_rows_bwd", st)
    return d_src


def moga_gather3_bwd(g_moga, inv_moga, g_stga, inv_cu, inv_slots, g_frame, inv_frame=None, stream=None):
    """g_moga, g_frame [H, N, D], g_stga [H, Nk, D] -> their token-order sum [N, H, D] (one pass)."""
    H, N, D = g_moga.shape
    Nk = g_stga.shape[1]
    d_src = torch.empty((N, H, D), dtype=g_moga.dtype, device=g_moga.device)
    st = load().moga_gather3_bwd(_p(g_moga), _p(inv_moga), _p(g_stga), _p(inv_cu), _p(inv_slots), Nk,
                                 _p(g_frame), _p(inv_frame), _dt(g_moga), N, H, D, _p(d_src), _stream(stream))
    _check("moga_gather3_bwd", st)
    return d_src


def moga_merge3_fwd(a_moga, a_stga, a_frame, inv_moga, inv_stga, inv_frame, gate, stream=None):
    """Three [H, N, D] branch outputs -> their mean [N, H, D] in token order (dynamic branch gated)."""
    H, N, D = a_moga.shape
    o = torch.empty((N, H, D), dtype=a_moga.dtype, device=a_moga.device)
    st = load().moga_merge3_fwd(_p(a_moga), _p(a_stga), _p(a_frame), _dt(a_moga), _p(inv_moga), _p(inv_stga),
                                _p(inv_frame), _p(gate), N, H, D, _p(o), _stream(stream))
    _check("moga_merge3_fwd", st)
    return o


def moga_merge3_bwd(d_o, a_moga, inv_moga, inv_stga, inv_frame, gate, stream=None):
    """-> (d_a_moga, d_a_stga, d_a_frame [H, N, D], d_gate f32 [N])"""
    N, H, D = d_o.shape
    mk = lambda: torch.empty((H, N, D), dtype=d_o.dtype, device=d_o.device)
    d_m, d_s, d_f = mk(), mk(), mk()
    d_gate = torch.empty(N, dtype=torch.float32, device=d_o.device)
    st = load().moga_merge3_bwd(_p(d_o), _p(a_moga), _dt(d_o), _p(inv_moga), _p(inv_stga), _p(inv_frame), _p(gate),
                                N, H, D, _p(d_m), _p(d_s), _p(d_f), _p(d_gate), _stream(stream))
    _check("moga_merge3_bwd", st)
    return d_m, d_s, d_f, d_gate


def moga_balance_loss(group, gate, M, alpha, stream=None):
    """Eqs. 6-8 -> (loss f32 [1], frac f32 [M], prob f32 [M]), all on the device."""
    N = group.shape[0]
    dev = group.device
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    frac = torch.empty(M, dtype=torch.float32, device=dev)
    prob = torch.empty(M, dtype=torch.float32, device=dev)
    ws = _ws(workspace_bytes(OP_BALANCE_LOSS, N, 0, 0, M, 0, MOGA_F32), dev)
    st = load().moga_balance_loss(_p(group), _p(gate), N, M, float(alpha), _p(loss), _p(frac), _p(prob),
                                  _p(ws), ws.numel(), _stream(stream))
    _check("moga_balance_loss", st)
    return loss, frac, prob


def moga_balance_loss_bwd(group, frac, alpha, d_loss=1.0, d_gate=None, stream=None):
    """Adds d_loss * dL/d gate to `d_gate` (in place) or returns a new tensor when d_gate is None.
    `d_loss`: a Python number, or a one-element fp32 device tensor (read by the kernel: no host sync)."""
    N, M = group.shape[0], frac.shape[0]
    accumulate = d_gate is not None
    if d_gate is None:
        d_gate = torch.empty(N, dtype=torch.float32, device=group.device)
    host, dev = (1.0, d_loss) if isinstance(d_loss, torch.Tensor) else (float(d_loss), None)
    if dev is not None:
        dev = dev.reshape(1).to(torch.float32)
    st = load().moga_balance_loss_bwd(_p(group), _p(frac), N, M, float(alpha), host, _p(dev),
                                      int(accumulate), _p(d_gate), _stream(stream))
    _check("moga_balance_loss_bwd", st)
    return d_gate


def moga_forward(x, w, q, k, v, softmax_scale, want_probs=True, stream=None):
    """Alg. 1 end to end: the four forward calls in order on one stream.  Returns a dict."""
    group, gate, probs, _ = moga_route(x, w, want_probs=want_probs, stream=stream)
    pm = moga_permute(group, w.shape[0], q, k, v, stream=stream)
    oh, lse = moga_group_attn_fwd(pm["qh"], pm["kh"], pm["vh"], pm["cu_seqlens"], softmax_scale,
                                  stream=stream)
    o = moga_unpermute(oh, pm["perm"], gate, stream=stream)
    pm.update({"group": group, "gate": gate, "probs": probs, "oh": oh, "lse": lse, "o": o})
    return pm


def moga_backward(fwd, x, w, d_o, softmax_scale, want_dx=False, stream=None):
    """Backward of `moga_forward`: the four backward calls in reverse order.  Returns a dict."""
    d_oh, d_gate = moga_unpermute_bwd(d_o, fwd["oh"], fwd["perm"], fwd["gate"], stream=stream)
    d_qh, d_kh, d_vh = moga_group_attn_bwd(d_oh, fwd["qh"], fwd["kh"], fwd["vh"], fwd["oh"], fwd["lse"],
                                           fwd["cu_seqlens"], softmax_scale, stream=stream)
    d_q, d_k, d_v = moga_permute_bwd(d_qh, d_kh, d_vh, fwd["perm"], stream=stream)
    d_w, d_x = moga_route_bwd(x, w, fwd["probs"], fwd["group"], fwd["gate"], d_gate, want_dx=want_dx,
                              stream=stream)
    return {"d_q": d_q, "d_k": d_k, "d_v": d_v, "d_w": d_w, "d_x": d_x, "d_gate": d_gate,
            "d_oh": d_oh, "d_qh": d_qh, "d_kh": d_kh, "d_vh": d_vh}


def visual_forward(x, w, q, k, v, softmax_scale, grid, static_index, stream=None):
    """The three-branch attention block of Section 3.2: MoGA (Alg. 1, gated by Eq. 5), the
    spatial-temporal groups of `static_index` (from moga_stga_build_index) and the per-frame groups,
    averaged by moga_merge3_fwd.  Returns a dict with everything the backward needs."""
    T, Hh, Ww = grid
    N = T * Hh * Ww
    si = static_index
    dev = q.device
    group, gate, probs, _ = moga_route(x, w, want_probs=True, stream=stream)
    pm = moga_permute(group, w.shape[0], q, k, v, stream=stream)
    a_m, lse_m = moga_group_attn_fwd(pm["qh"], pm["kh"], pm["vh"], pm["cu_seqlens"], softmax_scale, stream=stream)
    qs = moga_gather_rows(q, si["q_index"], stream=stream)
    ks = moga_gather_rows(k, si["kv_index"], stream=stream)
    vs = moga_gather_rows(v, si["kv_index"], stream=stream)
    a_s, lse_s = moga_varlen_attn_fwd(qs, ks, vs, si["cu_q"], si["cu_k"], softmax_scale, stream=stream)
    ident = torch.arange(N + 1, dtype=torch.int32, device=dev)
    cu_f = torch.arange(T + 1, dtype=torch.int32, device=dev) * (Hh * Ww)
    qf, kf, vf = (moga_gather_rows(t, ident[:N], stream=stream) for t in (q, k, v))
    a_f, lse_f = moga_varlen_attn_fwd(qf, kf, vf, cu_f, cu_f, softmax_scale, stream=stream)
    o = moga_merge3_fwd(a_m, a_s, a_f, pm["inv_perm"], si["q_slot"], None, gate, stream=stream)
    return {"o": o, "group": group, "gate": gate, "probs": probs, "pm": pm, "a_m": a_m, "lse_m": lse_m,
            "qs": qs, "ks": ks, "vs": vs, "a_s": a_s, "lse_s": lse_s, "qf": qf, "kf": kf, "vf": vf,
            "a_f": a_f, "lse_f": lse_f, "cu_f": cu_f, "ident": ident, "si": si}


def visual_backward(fwd, x, w, d_o, softmax_scale, stream=None):
    """Backward of `visual_forward` -> dict(d_q, d_k, d_v [N, H, D], d_w [M, d_model], d_gate [N])."""
    pm, si, ident = fwd["pm"], fwd["si"], fwd["ident"]
    d_m, d_s, d_f, d_gate = moga_merge3_bwd(d_o, fwd["a_m"], pm["inv_perm"], si["q_slot"], None, fwd["gate"],
                                            stream=stream)
    dqm, dkm, dvm = moga_group_attn_bwd(d_m, pm["qh"], pm["kh"], pm["vh"], fwd["a_m"], fwd["lse_m"],
                                        pm["cu_seqlens"], softmax_scale, stream=stream)
    del d_m
    dqs, dks, dvs = moga_varlen_attn_bwd(d_s, fwd["qs"], fwd["ks"], fwd["vs"], fwd["a_s"], fwd["lse_s"],
                                         si["cu_q"], si["cu_k"], softmax_scale, stream=stream)
    del d_s
    dqf, dkf, dvf = moga_varlen_attn_bwd(d_f, fwd["qf"], fwd["kf"], fwd["vf"], fwd["a_f"], fwd["lse_f"],
                                         fwd["cu_f"], fwd["cu_f"], softmax_scale, stream=stream)
    del d_f
    # every token-order gradient is written once: MoGA rows through inv_perm, the static rows through
    # their slot lists (queries are listed once, keys possibly several times), the frame rows in place
    d_q = moga_gather3_bwd(dqm, pm["inv_perm"], dqs, ident, si["q_slot"], dqf, stream=stream)
    d_k = moga_gather3_bwd(dkm, pm["inv_perm"], dks, si["inv_cu"], si["inv_slots"], dkf, stream=stream)
    d_v = moga_gather3_bwd(dvm, pm["inv_perm"], dvs, si["inv_cu"], si["inv_slots"], dvf, stream=stream)
    del dqm, dkm, dvm, dqs, dks, dvs, dqf, dkf, dvf
    d_w, _ = moga_route_bwd(x, w, fwd["probs"], fwd["group"], fwd["gate"], d_gate, stream=stream)
    return {"d_q": d_q, "d_k": d_k, "d_v": d_v, "d_w": d_w, "d_gate": d_gate}
