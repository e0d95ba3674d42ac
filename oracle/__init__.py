"""ctypes front end of the CPU oracle (oracle/rd_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It takes and returns numpy arrays, never touches a GPU, and imports
nothing from the HIP package.  bf16 tensors travel as uint16 bit patterns, fp16
tensors as numpy float16.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rd_oracle.c")
_LIB = os.path.join(_HERE, "librd_oracle.so")

DTYPES = {"f32": 0, "bf16": 1, "f16": 2}
NP_DTYPES = {"f32": np.float32, "bf16": np.uint16, "f16": np.float16}


def build(force: bool = False) -> str:
    """Compile rd_oracle.c with gcc (-O2, OpenMP) into oracle/librd_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized(out_dir: str) -> str:
    """The same source with gcc's address and undefined-behaviour sanitizers (-O1, no recovery from
    undefined behaviour), for the tests that run the oracle's pins under them.  The process that loads
    it must have gcc's libasan preloaded."""
    out = os.path.join(out_dir, "librd_oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-shared", "-fPIC", "-Wall", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-o", out, _SRC, "-lm"])
    return out


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        # RD_ORACLE_LIB: a sanitizer build of this same source (tests/test_sanitizers.py)
        _lib = ctypes.CDLL(os.environ.get("RD_ORACLE_LIB") or build())
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def dedup(beams: np.ndarray, ctx_len: Optional[np.ndarray] = None) -> dict:
    """dedup_prefix + pack_beam + tree structure for beams [B,W,L] (or [W,L])."""
    beams = _i32(beams)
    squeeze = beams.ndim == 2
    if squeeze:
        beams = beams[None]
    B, W, L = beams.shape
    N = W * L
    words = (N + 63) // 64
    ctx = None if ctx_len is None else _i32(np.reshape(ctx_len, (B,)))
    out = dict(
        prefix_tree=np.empty((B, W, L), np.int32),
        packed_tokens=np.empty((B, N), np.int32),
        n_packed=np.empty((B,), np.int32),
        unpack_index=np.empty((B, W, L), np.int32),
        parent=np.empty((B, N), np.int32),
        position_ids=np.empty((B, N), np.int32),
        tree_mask=np.empty((B, N, N), np.uint8),
        tree_mask_bits=np.empty((B, N, words), np.uint64),
    )
    lib().orc_dedup(_p(beams), _p(ctx), B, W, L, _p(out["prefix_tree"]), _p(out["packed_tokens"]),
                    _p(out["n_packed"]), _p(out["unpack_index"]), _p(out["parent"]),
                    _p(out["position_ids"]), _p(out["tree_mask"]), _p(out["tree_mask_bits"]))
    if squeeze:
        out = {k: v[0] for k, v in out.items()}
    return out


def _check_attn(q, k_cache, v_cache, k_new, v_new, dtype):
    want = NP_DTYPES[dtype]
    arrs = []
    for a in (q, k_cache, v_cache, k_new, v_new):
        a = np.ascontiguousarray(a)
        assert a.dtype == want, (a.dtype, want)
        arrs.append(a)
    B, H, N, D = arrs[0].shape
    Cmax = arrs[1].shape[2]
    assert arrs[1].shape == (B, H, Cmax, D) and arrs[2].shape == (B, H, Cmax, D)
    assert arrs[3].shape == (B, H, N, D) and arrs[4].shape == (B, H, N, D)
    return arrs, (B, H, N, D, Cmax)


def tree_attn(q, k_cache, v_cache, ctx_len, k_new, v_new, n_packed, tree_mask,
              dtype: str, scale: float) -> np.ndarray:
    """Tree-masked attention, whole tensor; returns [B,H,N,D] in the storage dtype."""
    (q, k_cache, v_cache, k_new, v_new), (B, H, N, D, Cmax) = _check_attn(
        q, k_cache, v_cache, k_new, v_new, dtype)
    ctx_len, n_packed = _i32(ctx_len), _i32(n_packed)
    tree_mask = np.ascontiguousarray(tree_mask, dtype=np.uint8)
    assert tree_mask.shape == (B, N, N)
    out = np.empty_like(q)
    lib().orc_tree_attn(_p(q), _p(k_cache), _p(v_cache), _p(ctx_len), _p(k_new), _p(v_new),
                        _p(n_packed), _p(tree_mask), B, H, N, D, Cmax, DTYPES[dtype],
                        ctypes.c_float(scale), _p(out))
    return out


def tree_attn_paged(q, k_pages, v_pages, block_table, ctx_len, k_new, v_new, n_packed, tree_mask,
                    dtype: str, scale: float) -> np.ndarray:
    """Tree-masked attention over a paged cache: pages [n_pages,H,page_size,D], block_table [B,max_pages].
    Context key c of sequence b is row c % page_size of page block_table[b][c // page_size]; the keys
    are laid out one by one into a dense cache with exactly that rule and the dense routine is run."""
    k_pages, v_pages = np.ascontiguousarray(k_pages), np.ascontiguousarray(v_pages)
    block_table, ctx_len = _i32(block_table), _i32(ctx_len)
    n_pages, H, ps, D = k_pages.shape
    B = block_table.shape[0]
    Cmax = max(int(ctx_len.max()), 1)
    kc = np.zeros((B, H, Cmax, D), k_pages.dtype)
    vc = np.zeros((B, H, Cmax, D), v_pages.dtype)
    for b in range(B):
        for c in range(int(ctx_len[b])):
            page = block_table[b, c // ps]
            kc[b, :, c, :] = k_pages[page, :, c % ps, :]
            vc[b, :, c, :] = v_pages[page, :, c % ps, :]
    return tree_attn(q, kc, vc, ctx_len, k_new, v_new, n_packed, tree_mask, dtype, scale)


def tree_attn_rows(q, k_cache, v_cache, ctx_len, k_new, v_new, n_packed, tree_mask,
                   dtype: str, scale: float, rows) -> np.ndarray:
    """Attention output of selected (b, h, p) rows as unrounded float64 [n_rows, D]."""
    (q, k_cache, v_cache, k_new, v_new), (B, H, N, D, Cmax) = _check_attn(
        q, k_cache, v_cache, k_new, v_new, dtype)
    ctx_len, n_packed = _i32(ctx_len), _i32(n_packed)
    tree_mask = np.ascontiguousarray(tree_mask, dtype=np.uint8)
    rows = _i32(rows).reshape(-1, 3)
    for b, h, p in rows:
        assert 0 <= b < B and 0 <= h < H and 0 <= p < n_packed[b]
    out = np.empty((rows.shape[0], D), np.float64)
    lib().orc_tree_attn_rows(_p(q), _p(k_cache), _p(v_cache), _p(ctx_len), _p(k_new), _p(v_new),
                             _p(n_packed), _p(tree_mask), B, H, N, D, Cmax, DTYPES[dtype],
                             ctypes.c_float(scale), _p(rows), rows.shape[0], _p(out))
    return out


def argmax(logits: np.ndarray, n_packed: np.ndarray) -> np.ndarray:
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    B, N, V = logits.shape
    n_packed = _i32(n_packed)
    out = np.empty((B, N), np.int32)
    lib().orc_argmax(_p(logits), _p(n_packed), B, N, V, _p(out))
    return out


def accept(beams, unpack_index, argmax_in, root_token=None) -> dict:
    beams, unpack_index, argmax_in = _i32(beams), _i32(unpack_index), _i32(argmax_in)
    B, W, L = beams.shape
    root = None if root_token is None else _i32(root_token)
    out = dict(
        n_accept=np.empty((B, W), np.int32),
        best_beam=np.empty((B,), np.int32),
        best_len=np.empty((B,), np.int32),
        next_token=np.empty((B,), np.int32),
        accepted_idx=np.empty((B, L), np.int32),
    )
    lib().orc_accept(_p(beams), _p(unpack_index), _p(argmax_in), _p(root), B, W, L,
                     _p(out["n_accept"]), _p(out["best_beam"]), _p(out["best_len"]),
                     _p(out["next_token"]), _p(out["accepted_idx"]))
    return out


def accept_sample(logits, draft_logits, beams, unpack_index, u_accept, u_next, temperature: float,
                  root_token=None, diagnostics: bool = False, step_row=None) -> dict:
    """Acceptance by rejection sampling (Sec. 3.4's other selection mode).  logits, draft_logits float32
    [B,N,V]; u_accept float32 [B,N] (one uniform number per packed slot); u_next float32 [B].  With
    `step_row` int32 [B,W,L-1], draft_logits is [L-1,rows,V] as the beam search recorded it
    (oracle.draft(..., steps=True)).  With `diagnostics`, also accept_ratio float64 [B,W,L] and
    next_weights float64 [B,V]."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    draft_logits = np.ascontiguousarray(draft_logits, dtype=np.float32)
    beams, unpack_index = _i32(beams), _i32(unpack_index)
    B, W, L = beams.shape
    V = logits.shape[2]
    assert logits.shape == (B, W * L, V)
    rows_per_step = 0
    if step_row is None:
        assert draft_logits.shape == logits.shape
    else:                                     # draft logits as the beam search recorded them: [L-1, rows, V]
        step_row = _i32(step_row)
        rows_per_step = draft_logits.shape[1]
        assert draft_logits.shape == (L - 1, rows_per_step, V) and step_row.shape == (B, W, L - 1)
    u_accept = np.ascontiguousarray(u_accept, dtype=np.float32)
    u_next = np.ascontiguousarray(u_next, dtype=np.float32)
    assert u_accept.shape == (B, W * L) and u_next.shape == (B,)
    root = None if root_token is None else _i32(root_token)
    out = dict(
        n_accept=np.empty((B, W), np.int32),
        best_beam=np.empty((B,), np.int32),
        best_len=np.empty((B,), np.int32),
        next_token=np.empty((B,), np.int32),
        accepted_idx=np.empty((B, L), np.int32),
    )
    ratio = np.empty((B, W, L), np.float64) if diagnostics else None
    weights = np.empty((B, V), np.float64) if diagnostics else None
    fn = lib().orc_accept_sample
    fn.argtypes = ([ctypes.c_void_p] * 3 + [ctypes.c_int] + [ctypes.c_void_p] * 5 + [ctypes.c_double] + [ctypes.c_int] * 4
                   + [ctypes.c_void_p] * 7)
    fn.restype = None
    fn(_p(logits), _p(draft_logits), _p(step_row), rows_per_step, _p(beams), _p(unpack_index), _p(root), _p(u_accept), _p(u_next),
       float(temperature), B, W, L, V, _p(out["n_accept"]), _p(out["best_beam"]), _p(out["best_len"]),
       _p(out["next_token"]), _p(out["accepted_idx"]), _p(ratio), _p(weights))
    if diagnostics:
        out["accept_ratio"], out["next_weights"] = ratio, weights
    return out


def commit(k_new, v_new, accepted_idx, best_len, ctx_len, k_cache, v_cache, dtype: str,
           hidden=None) -> dict:
    """Commit of the accepted tokens: returns updated COPIES of the caches, ctx_len_out,
    n_committed and (if `hidden` [B,N,Dh] is given) hidden_last [B,Dh] (zeros where best_len == 0)."""
    np_dt = NP_DTYPES[dtype]
    k_new = np.ascontiguousarray(k_new, dtype=np_dt)
    v_new = np.ascontiguousarray(v_new, dtype=np_dt)
    kc = np.array(k_cache, dtype=np_dt, order="C", copy=True)
    vc = np.array(v_cache, dtype=np_dt, order="C", copy=True)
    B, H, N, D = k_new.shape
    Cmax = kc.shape[2]
    assert v_new.shape == k_new.shape and kc.shape == (B, H, Cmax, D) and vc.shape == kc.shape
    accepted_idx = _i32(accepted_idx)
    L = accepted_idx.shape[1]
    best_len, ctx_len = _i32(best_len), _i32(ctx_len)
    ctx_out = np.zeros(B, np.int32)
    n_comm = np.zeros(B, np.int32)
    hid_last = None
    Dh = 0
    if hidden is not None:
        hidden = np.ascontiguousarray(hidden, dtype=np_dt)
        Dh = hidden.shape[2]
        assert hidden.shape == (B, N, Dh)
        hid_last = np.zeros((B, Dh), np_dt)
    lib().orc_commit(_p(k_new), _p(v_new), _p(accepted_idx), _p(best_len), _p(ctx_len),
                     B, H, N, D, Cmax, L, DTYPES[dtype], _p(kc), _p(vc), _p(ctx_out), _p(n_comm),
                     _p(hidden), Dh, _p(hid_last))
    return {"k_cache": kc, "v_cache": vc, "ctx_len": ctx_out, "n_committed": n_comm,
            "hidden_last": hid_last}


def rope(x, position_ids, n_packed, cos_tab, sin_tab, dtype: str) -> np.ndarray:
    """Rotary embedding ("rotate half" pairing) of rows p < n_packed[b] of x [B,H,N,D]; returns a copy."""
    x = np.array(x, dtype=NP_DTYPES[dtype], order="C", copy=True)
    B, H, N, D = x.shape
    position_ids, n_packed = _i32(position_ids), _i32(n_packed)
    cos_tab = np.ascontiguousarray(cos_tab, dtype=np.float32)
    sin_tab = np.ascontiguousarray(sin_tab, dtype=np.float32)
    max_pos = cos_tab.shape[0]
    assert position_ids.shape == (B, N) and cos_tab.shape == (max_pos, D // 2) and sin_tab.shape == cos_tab.shape
    lib().orc_rope(_p(x), _p(position_ids), _p(n_packed), _p(cos_tab), _p(sin_tab), max_pos,
                   B, H, N, D, DTYPES[dtype])
    return x


def _bits16(x, dtype: str) -> np.ndarray:
    """16-bit storage as bit patterns: bf16 arrives as uint16 bit patterns, float16 as numpy float16."""
    if dtype == "f16":
        return np.ascontiguousarray(x, np.float16).view(np.uint16)
    return np.ascontiguousarray(x, np.uint16)


def _draft_args(params, h, Dm, dtype):
    emb = _bits16(params["emb"], dtype)
    V = emb.shape[0]
    mlp_w = _bits16(params["mlp_w"], dtype)
    n_mlp = mlp_w.shape[0]
    assert emb.shape == (V, Dm) and params["rnn_u"].shape == (Dm, Dm) and params["rnn_w"].shape == (Dm, Dm)
    assert mlp_w.shape == (n_mlp, 2 * Dm, 2 * Dm) and params["head_w"].shape == (V, 2 * Dm)
    arrs = dict(emb=emb, rnn_u=_bits16(params["rnn_u"], dtype), rnn_w=_bits16(params["rnn_w"], dtype),
                rnn_b=np.ascontiguousarray(params["rnn_b"], np.float32), mlp_w=mlp_w,
                mlp_b=np.ascontiguousarray(params["mlp_b"], np.float32),
                head_w=_bits16(params["head_w"], dtype), h=_bits16(h, dtype))
    return arrs, V, n_mlp


def draft(params: dict, h, last_token, W: int, L: int, steps: bool = False, dtype: str = "bf16") -> dict:
    """Draft model + beam search (Sec. 3.1, 3.2).  params: bf16 bit patterns (dtype "f16": numpy float16)
    emb [V,Dm], rnn_u, rnn_w [Dm,Dm], mlp_w [K,2Dm,2Dm], head_w [V,2Dm]; float32 rnn_b [Dm], mlp_b
    [K,2Dm].  h of the same 16-bit type [B,Dm],
    last_token int32 [B].  Returns beams int32 [B,W,L] (position 0 = last_token) and beam_logp [B,W];
    with `steps` also step_logp float32 [L-1,B*W,V] (the log-probabilities computed during the search) and
    step_row int32 [B,W,L-1] (the row of step t-1 behind token t of final candidate w)."""
    B, Dm = np.asarray(h).shape
    a, V, n_mlp = _draft_args(params, h, Dm, dtype)
    last_token = _i32(last_token)
    assert 1 <= W <= V and L >= 1
    beams = np.empty((B, W, L), np.int32)
    logp = np.empty((B, W), np.float32)
    step_logp = np.zeros((max(L - 1, 0), B * W, V), np.float32) if steps else None
    step_row = np.zeros((B, W, max(L - 1, 0)), np.int32) if steps else None
    lib().orc_draft(_p(a["emb"]), _p(a["rnn_u"]), _p(a["rnn_w"]), _p(a["rnn_b"]), _p(a["mlp_w"]), _p(a["mlp_b"]),
                    n_mlp, _p(a["head_w"]), _p(a["h"]), _p(last_token), B, Dm, V, W, L, DTYPES[dtype], _p(beams), _p(logp),
                    _p(step_logp), _p(step_row))
    out = {"beams": beams, "beam_logp": logp}
    if steps:
        out["step_logp"], out["step_row"] = step_logp, step_row
    return out


def draft_path_logp(params: dict, h, paths, dtype: str = "bf16") -> np.ndarray:
    """Cumulative log probability (float64 [B,n]) of candidate paths int32 [B,n,L] under the draft model."""
    B, Dm = np.asarray(h).shape
    a, V, n_mlp = _draft_args(params, h, Dm, dtype)
    paths = _i32(paths)
    n, L = paths.shape[1:]
    out = np.empty((B, n), np.float64)
    lib().orc_draft_path_logp(_p(a["emb"]), _p(a["rnn_u"]), _p(a["rnn_w"]), _p(a["rnn_b"]), _p(a["mlp_w"]),
                              _p(a["mlp_b"]), n_mlp, _p(a["head_w"]), _p(a["h"]), _p(paths), B, n, Dm, V, L, DTYPES[dtype], _p(out))
    return out


def verify_step(beams, ctx_len, q, k_cache, v_cache, k_new, v_new, logits, dtype, scale,
                root_token=None) -> dict:
    """The whole path in order: dedup -> tree attention -> argmax -> accept."""
    d = dedup(beams, ctx_len)
    out = dict(d)
    out["attn_out"] = tree_attn(q, k_cache, v_cache, ctx_len, k_new, v_new, d["n_packed"],
                                d["tree_mask"], dtype, scale)
    out["argmax"] = argmax(logits, d["n_packed"])
    out.update(accept(beams, d["unpack_index"], out["argmax"], root_token))
    return out
