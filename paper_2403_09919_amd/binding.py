"""Thin ctypes binding of librd.so (the C ABI declared in include/rd.h).

Argument marshalling only: torch tensors supply device memory and the current stream;
every step of the verification path runs in the library's HIP kernels.  There is no CPU
fallback: importing this module fails if the library has not been built
(`python -m paper_2403_09919_amd.build`).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librd.so")

RD_F32, RD_BF16, RD_F16 = 0, 1, 2
RD_OK = 0
RD_MAX_W, RD_MAX_N = 128, 384

if not os.path.exists(LIB_PATH):
    raise ImportError("librd.so is not built: run `python -m paper_2403_09919_amd.build` "
                      "(hipcc, gfx950); there is no fallback path")

_lib = ctypes.CDLL(LIB_PATH)

_vp, _i, _sz, _f = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_float

EXPORTS = {
    "rd_strerror": (ctypes.c_char_p, [_i]),
    "rd_version": (_i, []),
    "rd_debug_stream_read": (_i, [_vp, _sz, _i, _vp, _vp]),
    "rd_dedup": (_i, [_vp, _vp, _i, _i, _i] + [_vp] * 8 + [_vp]),
    "rd_tree_attn_workspace": (_sz, [_i, _i, _i, _i, _i, _i]),
    "rd_tree_attn": (_i, [_vp] * 8 + [_i, _i, _i, _i, _i, _i, _f, _vp, _vp, _sz, _vp]),
    "rd_tree_attn_bounded": (_i, [_vp] * 8 + [_i, _i, _i, _i, _i, _i, _i, _f, _vp, _vp, _sz, _vp]),
    "rd_tree_attn_rope": (_i, [_vp] * 8 + [_vp, _vp, _vp, _i] + [_i, _i, _i, _i, _i, _i, _f, _vp, _vp, _vp, _sz, _vp]),
    "rd_tree_attn_paged_workspace": (_sz, [_i, _i, _i, _i, _i, _i, _i]),
    "rd_tree_attn_paged": (_i, [_vp] * 4 + [_i, _i, _i] + [_vp] * 5 + [_i, _i, _i, _i, _i, _f, _vp, _vp, _sz, _vp]),
    "rd_accept_workspace": (_sz, [_i, _i, _i, _i]),
    "rd_accept": (_i, [_vp] * 5 + [_i, _i, _i, _i] + [_vp] * 6 + [_vp, _sz, _vp]),
    "rd_accept_static": (_i, [_vp] * 5 + [_i, _i, _i, _i] + [_vp] * 6 + [_vp]),
    "rd_accept_sample_workspace": (_sz, [_i, _i, _i, _i]),
    "rd_accept_sample": (_i, [_vp] * 3 + [_i] + [_vp] * 6 + [_f, _i, _i, _i, _i] + [_vp] * 5 + [_vp, _sz, _vp]),
    "rd_commit": (_i, [_vp] * 5 + [_i] * 7 + [_vp] * 4 + [_vp, _i, _vp, _vp]),
    "rd_draft_workspace": (_sz, [_i, _i, _i, _i, _i]),
    "rd_draft_packed_elems": (_sz, [_i, _i]),
    "rd_draft_pack_weights": (_i, [_vp, _i, _i, _vp, _vp]),
    "rd_draft": (_i, [_vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "rd_rope": (_i, [_vp] * 6 + [_i] * 6 + [_vp]),
    "rd_commit_paged": (_i, [_vp] * 5 + [_i] * 6 + [_vp] * 3 + [_i, _i, _i] + [_vp, _vp] + [_vp, _i, _vp, _vp]),
}
for _name, (_res, _args) in EXPORTS.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


class RdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, rd_strerror(code), code))


def rd_strerror(code: int) -> str:
    return _lib.rd_strerror(int(code)).decode()


def rd_version() -> int:
    return int(_lib.rd_version())


def raw():
    """The ctypes library handle (for tests of the C ABI's argument checks)."""
    return _lib


def _ptr(t: Optional[torch.Tensor], dtype=None, shape=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live in device memory" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(code: int, where: str):
    if code != RD_OK:
        raise RdError(code, where)


def new_workspace(nbytes: int, device) -> torch.Tensor:
    """Zero-filled scratch buffer (the completion counters must start at zero)."""
    return torch.zeros(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ------------------------------------------------------------------------------------------
def rd_dedup(beams: torch.Tensor, ctx_len: Optional[torch.Tensor] = None, *,
             want_prefix_tree: bool = True, want_mask: bool = True, out: Optional[dict] = None) -> dict:
    """beams int32 [B,W,L] -> dict of device tensors (see include/rd.h, rd_dedup)."""
    B, W, L = beams.shape
    N = W * L
    words = (N + 63) // 64
    dev = beams.device
    i32 = torch.int32
    if out is None:
        out = dict(
            prefix_tree=torch.empty((B, W, L), dtype=i32, device=dev) if want_prefix_tree else None,
            packed_tokens=torch.empty((B, N), dtype=i32, device=dev),
            n_packed=torch.empty((B,), dtype=i32, device=dev),
            unpack_index=torch.empty((B, W, L), dtype=i32, device=dev),
            parent=torch.empty((B, N), dtype=i32, device=dev),
            position_ids=torch.empty((B, N), dtype=i32, device=dev),
            tree_mask=torch.empty((B, N, N), dtype=torch.uint8, device=dev) if want_mask else None,
            tree_mask_bits=torch.empty((B, N, words), dtype=torch.int64, device=dev),
        )
    code = _lib.rd_dedup(
        _ptr(beams, i32, (B, W, L), "beams"), _ptr(ctx_len, i32, (B,), "ctx_len"), B, W, L,
        _ptr(out["prefix_tree"], i32, (B, W, L), "prefix_tree"),
        _ptr(out["packed_tokens"], i32, (B, N), "packed_tokens"),
        _ptr(out["n_packed"], i32, (B,), "n_packed"),
        _ptr(out["unpack_index"], i32, (B, W, L), "unpack_index"),
        _ptr(out["parent"], i32, (B, N), "parent"),
        _ptr(out["position_ids"], i32, (B, N), "position_ids"),
        _ptr(out["tree_mask"], torch.uint8, (B, N, N), "tree_mask"),
        _ptr(out["tree_mask_bits"], torch.int64, (B, N, words), "tree_mask_bits"),
        _stream())
    _check(code, "rd_dedup")
    return out


def _dt_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return RD_F32
    if t.dtype == torch.bfloat16:
        return RD_BF16
    if t.dtype == torch.float16:
        return RD_F16
    raise ValueError("unsupported element type %s (float32, bfloat16 or float16)" % t.dtype)


def rd_tree_attn_workspace(B: int, H: int, N: int, D: int, Cmax: int, dt: int) -> int:
    return int(_lib.rd_tree_attn_workspace(B, H, N, D, Cmax, dt))


def rd_tree_attn(q, k_cache, v_cache, ctx_len, k_new, v_new, n_packed, tree_mask_bits, scale: float,
                 out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                 ctx_bound: Optional[int] = None) -> torch.Tensor:
    """q/k_new/v_new [B,H,N,D], k_cache/v_cache [B,H,Cmax,D] -> out [B,H,N,D] (see include/rd.h).  With
    ctx_bound (an upper bound of ctx_len known to the caller) the call is rd_tree_attn_bounded."""
    B, H, N, D = q.shape
    Cmax = k_cache.shape[2]
    dt = _dt_code(q)
    words = (N + 63) // 64
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = new_workspace(rd_tree_attn_workspace(B, H, N, D, Cmax if ctx_bound is None else min(ctx_bound, Cmax), dt), q.device)
    if ctx_bound is not None:
        code = _lib.rd_tree_attn_bounded(
            _ptr(q, q.dtype, (B, H, N, D), "q"),
            _ptr(k_cache, q.dtype, (B, H, Cmax, D), "k_cache") if Cmax > 0 else None,
            _ptr(v_cache, q.dtype, (B, H, Cmax, D), "v_cache") if Cmax > 0 else None,
            _ptr(ctx_len, torch.int32, (B,), "ctx_len"),
            _ptr(k_new, q.dtype, (B, H, N, D), "k_new"), _ptr(v_new, q.dtype, (B, H, N, D), "v_new"),
            _ptr(n_packed, torch.int32, (B,), "n_packed"),
            _ptr(tree_mask_bits, torch.int64, (B, N, words), "tree_mask_bits"),
            B, H, N, D, Cmax, int(ctx_bound), dt, float(scale),
            _ptr(out, q.dtype, (B, H, N, D), "out"),
            _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream())
        _check(code, "rd_tree_attn_bounded")
        return out
    code = _lib.rd_tree_attn(
        _ptr(q, q.dtype, (B, H, N, D), "q"),
        _ptr(k_cache, q.dtype, (B, H, Cmax, D), "k_cache") if Cmax > 0 else None,
        _ptr(v_cache, q.dtype, (B, H, Cmax, D), "v_cache") if Cmax > 0 else None,
        _ptr(ctx_len, torch.int32, (B,), "ctx_len"),
        _ptr(k_new, q.dtype, (B, H, N, D), "k_new"), _ptr(v_new, q.dtype, (B, H, N, D), "v_new"),
        _ptr(n_packed, torch.int32, (B,), "n_packed"),
        _ptr(tree_mask_bits, torch.int64, (B, N, words), "tree_mask_bits"),
        B, H, N, D, Cmax, dt, float(scale),
        _ptr(out, q.dtype, (B, H, N, D), "out"),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream())
    _check(code, "rd_tree_attn")
    return out


def rd_tree_attn_rope(q, k_cache, v_cache, ctx_len, k_new, v_new, n_packed, tree_mask_bits, position_ids,
                      cos_tab, sin_tab, scale: float, out: Optional[torch.Tensor] = None,
                      k_new_rot: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                      want_k_rot: bool = True):
    """rd_tree_attn with the rotary embedding of q and k_new applied inside the call (see include/rd.h,
    rd_tree_attn_rope); returns (out, k_new_rot)."""
    B, H, N, D = q.shape
    Cmax = k_cache.shape[2]
    dt = _dt_code(q)
    words = (N + 63) // 64
    max_pos = cos_tab.shape[0]
    if out is None:
        out = torch.empty_like(q)
    if k_new_rot is None and want_k_rot:
        k_new_rot = torch.zeros_like(k_new)
    if workspace is None:
        workspace = new_workspace(rd_tree_attn_workspace(B, H, N, D, Cmax, dt), q.device)
    code = _lib.rd_tree_attn_rope(
        _ptr(q, q.dtype, (B, H, N, D), "q"),
        _ptr(k_cache, q.dtype, (B, H, Cmax, D), "k_cache") if Cmax > 0 else None,
        _ptr(v_cache, q.dtype, (B, H, Cmax, D), "v_cache") if Cmax > 0 else None,
        _ptr(ctx_len, torch.int32, (B,), "ctx_len"),
        _ptr(k_new, q.dtype, (B, H, N, D), "k_new"), _ptr(v_new, q.dtype, (B, H, N, D), "v_new"),
        _ptr(n_packed, torch.int32, (B,), "n_packed"),
        _ptr(tree_mask_bits, torch.int64, (B, N, words), "tree_mask_bits"),
        _ptr(position_ids, torch.int32, (B, N), "position_ids"),
        _ptr(cos_tab, torch.float32, (max_pos, D // 2), "cos_tab"), _ptr(sin_tab, torch.float32, (max_pos, D // 2), "sin_tab"),
        max_pos, B, H, N, D, Cmax, dt, float(scale),
        _ptr(out, q.dtype, (B, H, N, D), "out"),
        _ptr(k_new_rot, q.dtype, (B, H, N, D), "k_new_rot") if k_new_rot is not None else None,
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream())
    _check(code, "rd_tree_attn_rope")
    return out, k_new_rot


def rd_tree_attn_paged_workspace(B: int, H: int, N: int, D: int, page_size: int, max_pages: int, dt: int) -> int:
    return int(_lib.rd_tree_attn_paged_workspace(B, H, N, D, page_size, max_pages, dt))


def rd_tree_attn_paged(q, k_pages, v_pages, block_table, ctx_len, k_new, v_new, n_packed, tree_mask_bits,
                       scale: float, out: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """As rd_tree_attn with k_pages/v_pages [n_pages,H,page_size,D] and block_table int32 [B,max_pages]
    (see include/rd.h, rd_tree_attn_paged)."""
    B, H, N, D = q.shape
    n_pages, Hp, page_size, Dp = k_pages.shape
    max_pages = block_table.shape[1]
    dt = _dt_code(q)
    words = (N + 63) // 64
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = new_workspace(rd_tree_attn_paged_workspace(B, H, N, D, page_size, max_pages, dt), q.device)
    code = _lib.rd_tree_attn_paged(
        _ptr(q, q.dtype, (B, H, N, D), "q"), _ptr(k_pages, q.dtype, (n_pages, H, page_size, D), "k_pages"),
        _ptr(v_pages, q.dtype, (n_pages, H, page_size, D), "v_pages"),
        _ptr(block_table, torch.int32, (B, max_pages), "block_table"), page_size, max_pages, n_pages,
        _ptr(ctx_len, torch.int32, (B,), "ctx_len"), _ptr(k_new, q.dtype, (B, H, N, D), "k_new"),
        _ptr(v_new, q.dtype, (B, H, N, D), "v_new"), _ptr(n_packed, torch.int32, (B,), "n_packed"),
        _ptr(tree_mask_bits, torch.int64, (B, N, words), "tree_mask_bits"), B, H, N, D, dt, float(scale),
        _ptr(out, q.dtype, (B, H, N, D), "out"), _ptr(workspace, torch.uint8, None, "workspace"),
        workspace.numel(), _stream())
    _check(code, "rd_tree_attn_paged")
    return out


def rd_debug_stream_read(src: torch.Tensor, workgroups: int, nbytes: Optional[int] = None) -> None:
    """One launch that reads `src` (or its first nbytes) once and discards it: the streaming floor."""
    n = src.numel() * src.element_size() if nbytes is None else int(nbytes)
    _check(_lib.rd_debug_stream_read(_ptr(src, None, None, "src"), n, int(workgroups), None, _stream()),
           "rd_debug_stream_read")


def rd_accept_workspace(B: int, W: int, L: int, V: int) -> int:
    return int(_lib.rd_accept_workspace(B, W, L, V))


def rd_accept(logits, beams, unpack_index, n_packed, root_token: Optional[torch.Tensor] = None,
              out: Optional[dict] = None, workspace: Optional[torch.Tensor] = None) -> dict:
    """logits float32 [B,N,V] -> dict(argmax, n_accept, best_beam, best_len, next_token, accepted_idx)."""
    B, W, L = beams.shape
    N = W * L
    V = logits.shape[2]
    dev = logits.device
    i32 = torch.int32
    if out is None:
        out = dict(
            argmax=torch.empty((B, N), dtype=i32, device=dev),
            n_accept=torch.empty((B, W), dtype=i32, device=dev),
            best_beam=torch.empty((B,), dtype=i32, device=dev),
            best_len=torch.empty((B,), dtype=i32, device=dev),
            next_token=torch.empty((B,), dtype=i32, device=dev),
            accepted_idx=torch.empty((B, L), dtype=i32, device=dev),
        )
    if workspace is None:
        workspace = new_workspace(rd_accept_workspace(B, W, L, V), dev)
    code = _lib.rd_accept(
        _ptr(logits, torch.float32, (B, N, V), "logits"), _ptr(beams, i32, (B, W, L), "beams"),
        _ptr(unpack_index, i32, (B, W, L), "unpack_index"), _ptr(n_packed, i32, (B,), "n_packed"),
        _ptr(root_token, i32, (B,), "root_token"), B, W, L, V,
        _ptr(out["argmax"], i32, (B, N), "argmax"), _ptr(out["n_accept"], i32, (B, W), "n_accept"),
        _ptr(out["best_beam"], i32, (B,), "best_beam"), _ptr(out["best_len"], i32, (B,), "best_len"),
        _ptr(out["next_token"], i32, (B,), "next_token"),
        _ptr(out["accepted_idx"], i32, (B, L), "accepted_idx"),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream())
    _check(code, "rd_accept")
    return out


def rd_accept_static(logits, beams, unpack_index, n_packed, out: dict, root_token: Optional[torch.Tensor] = None) -> dict:
    """rd_accept without a workspace and without any allocation (see include/rd.h, rd_accept_static):
    the caller passes every output tensor in `out`."""
    B, W, L = beams.shape
    N = W * L
    V = logits.shape[2]
    i32 = torch.int32
    code = _lib.rd_accept_static(
        _ptr(logits, torch.float32, (B, N, V), "logits"), _ptr(beams, i32, (B, W, L), "beams"),
        _ptr(unpack_index, i32, (B, W, L), "unpack_index"), _ptr(n_packed, i32, (B,), "n_packed"),
        _ptr(root_token, i32, (B,), "root_token"), B, W, L, V,
        _ptr(out["argmax"], i32, (B, N), "argmax"), _ptr(out["n_accept"], i32, (B, W), "n_accept"),
        _ptr(out["best_beam"], i32, (B,), "best_beam"), _ptr(out["best_len"], i32, (B,), "best_len"),
        _ptr(out["next_token"], i32, (B,), "next_token"),
        _ptr(out["accepted_idx"], i32, (B, L), "accepted_idx"), _stream())
    _check(code, "rd_accept_static")
    return out


def rd_accept_sample_workspace(B: int, W: int, L: int, V: int) -> int:
    return int(_lib.rd_accept_sample_workspace(B, W, L, V))


def rd_accept_sample(logits, draft_logits, beams, unpack_index, n_packed, u_accept, u_next, temperature: float,
                     root_token: Optional[torch.Tensor] = None, out: Optional[dict] = None,
                     workspace: Optional[torch.Tensor] = None, step_row: Optional[torch.Tensor] = None) -> dict:
    """Rejection-sampling acceptance: logits, draft_logits float32 [B,N,V]; u_accept float32 [B,N];
    u_next float32 [B] -> dict(n_accept, best_beam, best_len, next_token, accepted_idx).  With
    `step_row` (rd_draft's), draft_logits is rd_draft's step_logits [L-1, rows, V]."""
    B, W, L = beams.shape
    N = W * L
    V = logits.shape[2]
    rows = 0
    draft_shape = (B, N, V)
    if step_row is not None:
        rows = draft_logits.shape[1]
        draft_shape = (L - 1, rows, V)
    dev = logits.device
    i32, f32 = torch.int32, torch.float32
    if out is None:
        out = dict(
            n_accept=torch.empty((B, W), dtype=i32, device=dev),
            best_beam=torch.empty((B,), dtype=i32, device=dev),
            best_len=torch.empty((B,), dtype=i32, device=dev),
            next_token=torch.empty((B,), dtype=i32, device=dev),
            accepted_idx=torch.empty((B, L), dtype=i32, device=dev),
        )
    if workspace is None:
        workspace = new_workspace(rd_accept_sample_workspace(B, W, L, V), dev)
    code = _lib.rd_accept_sample(
        _ptr(logits, f32, (B, N, V), "logits"), _ptr(draft_logits, f32, draft_shape, "draft_logits"),
        _ptr(step_row, i32, (B, W, L - 1), "step_row"), rows,
        _ptr(beams, i32, (B, W, L), "beams"), _ptr(unpack_index, i32, (B, W, L), "unpack_index"),
        _ptr(n_packed, i32, (B,), "n_packed"), _ptr(root_token, i32, (B,), "root_token"),
        _ptr(u_accept, f32, (B, N), "u_accept"), _ptr(u_next, f32, (B,), "u_next"), float(temperature),
        B, W, L, V,
        _ptr(out["n_accept"], i32, (B, W), "n_accept"), _ptr(out["best_beam"], i32, (B,), "best_beam"),
        _ptr(out["best_len"], i32, (B,), "best_len"), _ptr(out["next_token"], i32, (B,), "next_token"),
        _ptr(out["accepted_idx"], i32, (B, L), "accepted_idx"),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream())
    _check(code, "rd_accept_sample")
    return out


def rd_commit(k_new, v_new, accepted_idx, best_len, ctx_len, k_cache, v_cache,
              ctx_len_out: Optional[torch.Tensor] = None, n_committed: Optional[torch.Tensor] = None,
              hidden: Optional[torch.Tensor] = None, hidden_last: Optional[torch.Tensor] = None) -> dict:
    """Appends the accepted packed tokens' K/V rows to the caches IN PLACE (see include/rd.h,
    rd_commit); returns dict(ctx_len, n_committed, hidden_last)."""
    B, H, N, D = k_new.shape
    Cmax = k_cache.shape[2]
    L = accepted_idx.shape[1]
    dev = k_new.device
    i32 = torch.int32
    dt = _dt_code(k_new)
    if ctx_len_out is None:
        ctx_len_out = torch.empty((B,), dtype=i32, device=dev)
    if n_committed is None:
        n_committed = torch.empty((B,), dtype=i32, device=dev)
    Dh = 0
    if hidden is not None:
        Dh = hidden.shape[2]
        if hidden_last is None:
            hidden_last = torch.zeros((B, Dh), dtype=hidden.dtype, device=dev)
    code = _lib.rd_commit(
        _ptr(k_new, None, (B, H, N, D), "k_new"), _ptr(v_new, k_new.dtype, (B, H, N, D), "v_new"),
        _ptr(accepted_idx, i32, (B, L), "accepted_idx"), _ptr(best_len, i32, (B,), "best_len"),
        _ptr(ctx_len, i32, (B,), "ctx_len"), B, H, N, D, Cmax, L, dt,
        _ptr(k_cache, k_new.dtype, (B, H, Cmax, D), "k_cache"), _ptr(v_cache, k_new.dtype, (B, H, Cmax, D), "v_cache"),
        _ptr(ctx_len_out, i32, (B,), "ctx_len_out"), _ptr(n_committed, i32, (B,), "n_committed"),
        _ptr(hidden, k_new.dtype, (B, N, Dh), "hidden") if hidden is not None else None, Dh,
        _ptr(hidden_last, k_new.dtype, (B, Dh), "hidden_last") if hidden is not None else None, _stream())
    _check(code, "rd_commit")
    return dict(ctx_len=ctx_len_out, n_committed=n_committed, hidden_last=hidden_last)


def rd_commit_paged(k_new, v_new, accepted_idx, best_len, ctx_len, k_pages, v_pages, block_table,
                    ctx_len_out: Optional[torch.Tensor] = None, n_committed: Optional[torch.Tensor] = None) -> dict:
    """rd_commit into a paged cache IN PLACE (see include/rd.h, rd_commit_paged)."""
    B, H, N, D = k_new.shape
    n_pages, _, page_size, _ = k_pages.shape
    max_pages = block_table.shape[1]
    L = accepted_idx.shape[1]
    i32 = torch.int32
    dev = k_new.device
    if ctx_len_out is None:
        ctx_len_out = torch.empty((B,), dtype=i32, device=dev)
    if n_committed is None:
        n_committed = torch.empty((B,), dtype=i32, device=dev)
    code = _lib.rd_commit_paged(
        _ptr(k_new, None, (B, H, N, D), "k_new"), _ptr(v_new, k_new.dtype, (B, H, N, D), "v_new"),
        _ptr(accepted_idx, i32, (B, L), "accepted_idx"), _ptr(best_len, i32, (B,), "best_len"),
        _ptr(ctx_len, i32, (B,), "ctx_len"), B, H, N, D, L, _dt_code(k_new),
        _ptr(k_pages, k_new.dtype, (n_pages, H, page_size, D), "k_pages"),
        _ptr(v_pages, k_new.dtype, (n_pages, H, page_size, D), "v_pages"),
        _ptr(block_table, i32, (B, max_pages), "block_table"), page_size, max_pages, n_pages,
        _ptr(ctx_len_out, i32, (B,), "ctx_len_out"), _ptr(n_committed, i32, (B,), "n_committed"),
        None, 0, None, _stream())
    _check(code, "rd_commit_paged")
    return dict(ctx_len=ctx_len_out, n_committed=n_committed)


def rd_rope(q, k_new, position_ids, n_packed, cos_tab, sin_tab) -> None:
    """Rotates q and k_new [B,H,N,D] IN PLACE at position_ids [B,N] (see include/rd.h, rd_rope);
    cos_tab/sin_tab float32 [max_pos, D/2]."""
    ref = q if q is not None else k_new
    B, H, N, D = ref.shape
    max_pos = cos_tab.shape[0]
    code = _lib.rd_rope(
        _ptr(q, ref.dtype, (B, H, N, D), "q") if q is not None else None,
        _ptr(k_new, ref.dtype, (B, H, N, D), "k_new") if k_new is not None else None,
        _ptr(position_ids, torch.int32, (B, N), "position_ids"), _ptr(n_packed, torch.int32, (B,), "n_packed"),
        _ptr(cos_tab, torch.float32, (max_pos, D // 2), "cos_tab"), _ptr(sin_tab, torch.float32, (max_pos, D // 2), "sin_tab"),
        max_pos, B, H, N, D, _dt_code(ref), _stream())
    _check(code, "rd_rope")


class _DraftParams(ctypes.Structure):
    _fields_ = [("emb", _vp), ("rnn_u", _vp), ("rnn_w", _vp), ("rnn_b", _vp), ("mlp_w", _vp), ("mlp_b", _vp),
                ("head_w", _vp), ("n_mlp", _i), ("Dm", _i), ("V", _i), ("dtype", _i), ("tiled", _i)]


def rd_draft_workspace(B: int, W: int, L: int, Dm: int, V: int) -> int:
    return int(_lib.rd_draft_workspace(B, W, L, Dm, V))


def rd_draft_pack(params: dict) -> dict:
    """One-time layout change at model load: returns a copy of `params` whose matrices rnn_u, rnn_w,
    mlp_w and head_w are in rd_draft's operand-tiled layout (see include/rd.h, rd_draft_pack_weights),
    marked with "tiled": True.  emb and the biases are shared with the input dict."""
    def pack(w, n_mats, N, K):
        w = w.contiguous()
        per = int(_lib.rd_draft_packed_elems(N, K))
        dst = torch.empty((n_mats * per,), dtype=w.dtype, device=w.device)
        for k in range(n_mats):
            _check(_lib.rd_draft_pack_weights(w.data_ptr() + k * N * K * 2, N, K, dst.data_ptr() + k * per * 2, _stream()),
                   "rd_draft_pack_weights")
        return dst

    V, Dm = params["emb"].shape
    K = params["mlp_w"].shape[0]
    G = 2 * Dm
    out = dict(params)
    out["rnn_u"] = pack(params["rnn_u"], 1, Dm, Dm)
    out["rnn_w"] = pack(params["rnn_w"], 1, Dm, Dm)
    out["mlp_w"] = pack(params["mlp_w"], K, G, G) if K else params["mlp_w"]
    out["head_w"] = pack(params["head_w"], 1, V, G)
    out["tiled"] = True
    out["n_mlp"] = K
    return out


def rd_draft(params: dict, h, last_token, W: int, L: int, out: Optional[dict] = None,
             workspace: Optional[torch.Tensor] = None, steps: bool = False) -> dict:
    """Draft model + beam search (see include/rd.h, rd_draft).  params: device tensors emb [V,Dm],
    rnn_u, rnn_w [Dm,Dm], mlp_w [K,2Dm,2Dm], head_w [V,2Dm] (all bfloat16 or all float16), rnn_b [Dm], mlp_b [K,2Dm]
    (float32); h bfloat16 [B,Dm]; last_token int32 [B] -> dict(beams int32 [B,W,L], beam_logp [B,W]);
    with `steps` (or an `out` that holds them) also step_logits float32 [L-1,B*W,V] and step_row int32
    [B,W,L-1], the record of the search that rd_accept_sample takes."""
    bf = params["emb"].dtype                  # bfloat16 or float16: the model's 16-bit storage type
    if bf not in (torch.bfloat16, torch.float16):
        raise ValueError("draft model weights must be bfloat16 or float16, got %s" % bf)
    V, Dm = params["emb"].shape
    tiled = bool(params.get("tiled", False))      # matrices packed by rd_draft_pack: flat tensors
    K = params["n_mlp"] if tiled else params["mlp_w"].shape[0]
    G = 2 * Dm
    B = h.shape[0]
    dev = h.device

    def mat(name, n_mats, N, Kc):
        shape = (n_mats * int(_lib.rd_draft_packed_elems(N, Kc)),) if tiled else ((N, Kc) if n_mats == 1 and name != "mlp_w" else (n_mats, N, Kc))
        return _ptr(params[name], bf, shape, name)

    p = _DraftParams(
        _ptr(params["emb"], bf, (V, Dm), "emb"), mat("rnn_u", 1, Dm, Dm), mat("rnn_w", 1, Dm, Dm),
        _ptr(params["rnn_b"], torch.float32, (Dm,), "rnn_b"),
        mat("mlp_w", K, G, G) if K else None,
        _ptr(params["mlp_b"], torch.float32, (K, G), "mlp_b") if K else None,
        mat("head_w", 1, V, G), K, Dm, V, RD_BF16 if bf == torch.bfloat16 else RD_F16, 1 if tiled else 0)
    if out is None:
        out = dict(beams=torch.empty((B, W, L), dtype=torch.int32, device=dev),
                   beam_logp=torch.empty((B, W), dtype=torch.float32, device=dev))
    if steps and out.get("step_logits") is None:
        out["step_logits"] = torch.empty((max(L - 1, 0), B * W, V), dtype=torch.float32, device=dev)
        out["step_row"] = torch.empty((B, W, max(L - 1, 0)), dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(rd_draft_workspace(B, W, L, Dm, V), 256), dtype=torch.uint8, device=dev)
    sl, sr = out.get("step_logits"), out.get("step_row")
    code = _lib.rd_draft(ctypes.byref(p), _ptr(h, bf, (B, Dm), "h"), _ptr(last_token, torch.int32, (B,), "last_token"),
                         B, W, L, _ptr(out["beams"], torch.int32, (B, W, L), "beams"),
                         _ptr(out["beam_logp"], torch.float32, (B, W), "beam_logp"),
                         _ptr(sl, torch.float32, (max(L - 1, 0), B * W, V), "step_logits"),
                         _ptr(sr, torch.int32, (B, W, max(L - 1, 0)), "step_row"),
                         _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream())
    _check(code, "rd_draft")
    return out
