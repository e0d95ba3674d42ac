"""Host-only checks of the C ABI: the library loads, exports every symbol that
include/rd.h declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2403_09919_amd", "librd.so")
HDR = os.path.join(ROOT, "include", "rd.h")

OK, INVALID, UNSUPPORTED, WORKSPACE = 0, -1, -2, -3
FAKE = 0x10000   # never dereferenced on the host: all these calls must fail before any launch


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("librd.so missing: run `python -m paper_2403_09919_amd.build`")
    from paper_2403_09919_amd import binding
    other = os.environ.get("RD_TEST_LIB")           # a sanitizer build of the host code (tests/test_sanitizers.py)
    if other:
        san = ctypes.CDLL(other)
        for name, (res, args) in binding.EXPORTS.items():
            fn = getattr(san, name)
            fn.restype, fn.argtypes = res, args
        return san
    return binding.raw()


def _declared_symbols():
    src = open(HDR).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(rd_[a-z_]+)\s*\(", src)))


def test_header_symbols_exported(lib):
    names = _declared_symbols()
    assert names == sorted(["rd_strerror", "rd_version", "rd_dedup", "rd_tree_attn_workspace",
                            "rd_tree_attn", "rd_tree_attn_bounded", "rd_tree_attn_rope", "rd_tree_attn_paged_workspace", "rd_tree_attn_paged",
                            "rd_accept_workspace", "rd_accept", "rd_accept_static", "rd_accept_sample_workspace", "rd_accept_sample", "rd_commit", "rd_commit_paged", "rd_rope",
                            "rd_draft_workspace", "rd_draft", "rd_draft_packed_elems", "rd_draft_pack_weights"])
    raw = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(raw, n), n
    from paper_2403_09919_amd import binding
    # the binding also reaches the calibration entry point, which is declared in the library's own
    # csrc/rd_debug.h, not in the public header
    assert sorted(set(binding.EXPORTS) - {"rd_debug_stream_read"}) == names
    assert hasattr(raw, "rd_debug_stream_read")


def test_version_and_strerror(lib):
    assert lib.rd_version() >= 100
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -99):
        s = lib.rd_strerror(code)
        assert s and len(s) > 1
        seen.add(s)
    assert len(seen) == 7


def _dedup(lib, B, W, L, beams=FAKE, req=FAKE, mask=FAKE, bits=FAKE):
    return lib.rd_dedup(beams, None, B, W, L, FAKE, req, req, req, req, req, mask, bits, None)


def test_dedup_argument_errors(lib):
    assert _dedup(lib, 0, 4, 4) == INVALID
    assert _dedup(lib, 1, 0, 4) == INVALID
    assert _dedup(lib, 1, 4, -1) == INVALID
    assert _dedup(lib, 1, 129, 1) == UNSUPPORTED
    assert _dedup(lib, 1, 77, 5) == UNSUPPORTED          # N = 385 > 384
    assert _dedup(lib, 1, 4, 4, beams=None) == INVALID
    assert _dedup(lib, 1, 4, 4, req=None) == INVALID
    assert _dedup(lib, 1, 4, 4, bits=FAKE + 4) == INVALID   # uint64 rows need 8-byte alignment


def _attn(lib, B=1, H=2, N=16, D=64, Cmax=32, dt=0, q=FAKE, kc=FAKE, ws=FAKE, ws_bytes=None, out=FAKE):
    need = lib.rd_tree_attn_workspace(B, H, N, D, Cmax, dt)
    if ws_bytes is None:
        ws_bytes = need
    return lib.rd_tree_attn(q, kc, kc, FAKE, FAKE, FAKE, FAKE, FAKE, B, H, N, D, Cmax, dt, 0.125,
                            out, ws, ws_bytes, None)


def test_tree_attn_argument_errors(lib):
    assert lib.rd_tree_attn_workspace(1, 2, 16, 64, 32, 0) > 0
    assert lib.rd_tree_attn_workspace(1, 2, 16, 96, 32, 0) == 0
    assert _attn(lib, B=0) == INVALID
    assert _attn(lib, Cmax=-1) == INVALID
    assert _attn(lib, D=96) == UNSUPPORTED
    assert _attn(lib, N=385) == UNSUPPORTED
    assert _attn(lib, dt=7) == UNSUPPORTED
    assert _attn(lib, q=None) == INVALID
    assert _attn(lib, kc=None) == INVALID
    assert _attn(lib, q=FAKE + 8) == INVALID              # 16-byte alignment
    assert _attn(lib, out=None) == INVALID
    assert _attn(lib, ws=None) == WORKSPACE
    assert _attn(lib, ws=FAKE + 16) == WORKSPACE          # 256-byte alignment
    assert _attn(lib, ws_bytes=16) == WORKSPACE


def test_tree_attn_bounded_argument_errors(lib):
    def call(B=1, H=2, N=16, D=64, Cmax=4096, bound=600, dt=1, q=FAKE, ws=FAKE, ws_bytes=None):
        need = lib.rd_tree_attn_workspace(B, H, N, D, min(max(bound, 0), Cmax), dt)
        return lib.rd_tree_attn_bounded(q, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, B, H, N, D, Cmax, bound, dt, 0.125,
                                        FAKE, ws, need if ws_bytes is None else ws_bytes, None)
    assert call(B=0) == INVALID
    assert call(bound=-1) == INVALID
    assert call(D=96) == UNSUPPORTED
    assert call(q=None) == INVALID
    assert call(ws=None) == WORKSPACE
    assert call(ws_bytes=16) == WORKSPACE


def test_tree_attn_rope_argument_errors(lib):
    def call(B=1, H=2, N=16, D=64, Cmax=32, dt=1, q=FAKE, pos=FAKE, cos=FAKE, max_pos=64, krot=FAKE + 4096, ws=FAKE, ws_bytes=None):
        need = lib.rd_tree_attn_workspace(B, H, N, D, Cmax, dt if dt in (0, 1, 2) else 1)
        return lib.rd_tree_attn_rope(q, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, pos, cos, cos, max_pos,
                                     B, H, N, D, Cmax, dt, 0.125, FAKE, krot, ws, need if ws_bytes is None else ws_bytes, None)
    assert call(B=0) == INVALID
    assert call(D=96) == UNSUPPORTED
    assert call(dt=0) == UNSUPPORTED                      # 16-bit element types only
    assert call(dt=7) == UNSUPPORTED
    assert call(q=None) == INVALID
    assert call(pos=None) == INVALID
    assert call(cos=None) == INVALID
    assert call(max_pos=0) == INVALID
    assert call(krot=FAKE) == INVALID                     # the rotated keys must not overwrite q / k_new
    assert call(krot=FAKE + 8) == INVALID                 # 16-byte alignment
    assert call(ws=None) == WORKSPACE
    assert call(ws_bytes=16) == WORKSPACE


def test_workspace_sizes(lib):
    # The attention workspace holds one counter per (sequence, head) plus the partial results
    # of the launch plan chosen for the shape; a plan with one workgroup per head needs no
    # partials, so the size is not monotone in the problem size -- but it is never zero for a
    # valid shape, is a multiple of 256 bytes, and covers the counters.
    for shape in [(1, 32, 40, 128, 1024, 1), (8, 32, 40, 128, 2048, 1), (4, 40, 80, 128, 4096, 1),
                  (16, 52, 80, 128, 2048, 1), (1, 4, 16, 64, 128, 0), (2, 3, 128, 64, 0, 0)]:
        n = lib.rd_tree_attn_workspace(*shape)
        assert n >= shape[0] * shape[1] * 4 and n % 256 == 0, shape
    # the fp32 path always exchanges partials: one per context range plus the packed keys
    assert lib.rd_tree_attn_workspace(1, 4, 16, 64, 128, 0) >= 256 + 4 * 2 * 16 * (2 + 64) * 4
    assert lib.rd_tree_attn_workspace(1, 32, 40, 96, 1024, 1) == 0        # unsupported head size
    assert lib.rd_accept_workspace(1, 8, 5, 32000) < lib.rd_accept_workspace(16, 16, 5, 32000)
    assert lib.rd_accept_workspace(1, 129, 1, 10) == 0


def _accept(lib, B=1, W=4, L=4, V=100, logits=FAKE, req=FAKE, ws=FAKE, ws_bytes=None):
    need = lib.rd_accept_workspace(B, W, L, V)
    if ws_bytes is None:
        ws_bytes = need
    return lib.rd_accept(logits, FAKE, FAKE, FAKE, None, B, W, L, V, req, req, req, req, req, req,
                         ws, ws_bytes, None)


def test_stream_read_argument_errors(lib):
    assert lib.rd_debug_stream_read(None, 1024, 4, None, None) == INVALID
    assert lib.rd_debug_stream_read(FAKE, 8, 4, None, None) == INVALID
    assert lib.rd_debug_stream_read(FAKE, 1024, 0, None, None) == INVALID
    assert lib.rd_debug_stream_read(FAKE + 4, 1024, 4, None, None) == INVALID


def test_accept_static_argument_errors(lib):
    """The entry point without a workspace rejects what rd_accept rejects, and sizes beyond its static
    scratch array, all before anything is launched (the pointers here are not device memory)."""
    def call(B=1, W=4, L=4, V=100, logits=FAKE, req=FAKE):
        return lib.rd_accept_static(logits, FAKE, FAKE, FAKE, None, B, W, L, V, req, req, req, req, req, req, None)
    assert call(B=0) == INVALID
    assert call(V=0) == INVALID
    assert call(W=129, L=1) == UNSUPPORTED
    assert call(logits=None) == INVALID
    assert call(logits=FAKE + 4) == INVALID
    assert call(req=None) == INVALID
    SCRATCH_LIMIT = -5
    assert lib.rd_accept_workspace(300, 128, 3, 1000) > (1 << 20)
    assert call(B=300, W=128, L=3, V=1000) == SCRATCH_LIMIT
    assert b"static scratch" in lib.rd_strerror(SCRATCH_LIMIT)


def test_accept_argument_errors(lib):
    assert _accept(lib, B=0) == INVALID
    assert _accept(lib, V=0) == INVALID
    assert _accept(lib, W=129, L=1) == UNSUPPORTED
    assert _accept(lib, logits=None) == INVALID
    assert _accept(lib, logits=FAKE + 4) == INVALID
    assert _accept(lib, req=None) == INVALID
    assert _accept(lib, ws=None) == WORKSPACE
    assert _accept(lib, ws_bytes=8) == WORKSPACE


def _sample(lib, B=1, W=4, L=4, V=100, logits=FAKE, draft=FAKE, req=FAKE, u=FAKE, t=1.0, ws=FAKE, ws_bytes=None,
            step_row=None, rows=0):
    import ctypes
    need = lib.rd_accept_sample_workspace(B, W, L, V)
    if ws_bytes is None:
        ws_bytes = need
    return lib.rd_accept_sample(logits, draft, step_row, rows, FAKE, FAKE, FAKE, None, u, u, ctypes.c_float(t), B, W, L, V,
                                req, req, req, req, req, ws, ws_bytes, None)


def test_accept_sample_argument_errors(lib):
    assert lib.rd_accept_sample_workspace(1, 8, 5, 32000) >= 8 * 40 * 16
    assert lib.rd_accept_sample_workspace(1, 129, 1, 10) == 0
    assert _sample(lib, B=0) == INVALID
    assert _sample(lib, V=0) == INVALID
    assert _sample(lib, t=0.0) == INVALID
    assert _sample(lib, t=-1.0) == INVALID
    assert _sample(lib, t=float("nan")) == INVALID
    assert _sample(lib, t=float("inf")) == INVALID
    assert _sample(lib, W=129, L=1) == UNSUPPORTED
    assert _sample(lib, V=(1 << 20) + 4) == UNSUPPORTED
    assert _sample(lib, logits=None) == INVALID
    assert _sample(lib, draft=FAKE + 4) == INVALID
    assert _sample(lib, u=None) == INVALID
    assert _sample(lib, step_row=FAKE, rows=0) == INVALID
    assert _sample(lib, req=None) == INVALID
    assert _sample(lib, ws=None) == WORKSPACE
    assert _sample(lib, ws_bytes=8) == WORKSPACE


def _paged(lib, B=1, H=2, N=8, D=64, ps=64, mp=4, npg=8, dt=1, q=FAKE, pages=FAKE, table=FAKE, ws=FAKE, ws_bytes=None):
    import ctypes
    need = lib.rd_tree_attn_paged_workspace(B, H, N, D, ps, mp, dt)
    if ws_bytes is None:
        ws_bytes = need
    return lib.rd_tree_attn_paged(q, pages, pages, table, ps, mp, npg, FAKE, FAKE, FAKE, FAKE, FAKE,
                                  B, H, N, D, dt, ctypes.c_float(0.125), FAKE, ws, ws_bytes, None)


def test_paged_attention_argument_errors(lib):
    assert _paged(lib, ps=0) == INVALID
    assert _paged(lib, mp=0) == INVALID
    assert _paged(lib, npg=0) == INVALID
    assert _paged(lib, ps=48) == UNSUPPORTED              # a 32-key tile must not straddle pages
    assert _paged(lib, dt=0) == UNSUPPORTED               # 16-bit caches only
    assert _paged(lib, D=96) == UNSUPPORTED
    assert _paged(lib, N=385) == UNSUPPORTED
    assert _paged(lib, q=None) == INVALID
    assert _paged(lib, pages=None) == INVALID
    assert _paged(lib, table=None) == INVALID
    assert _paged(lib, pages=FAKE + 8) == INVALID
    assert _paged(lib, ws=None) == WORKSPACE
    assert _paged(lib, ws_bytes=16) == WORKSPACE
    assert lib.rd_tree_attn_paged_workspace(1, 2, 8, 64, 48, 4, 1) == 0
    assert lib.rd_tree_attn_paged_workspace(1, 2, 8, 64, 64, 4, 1) >= 256


def _commit(lib, B=1, H=2, N=8, D=64, Cmax=16, L=4, dt=0, src=FAKE, cache=FAKE, ctx=FAKE, ctx_out=FAKE + 64,
            hidden=None, Dh=0, hid_last=None):
    return lib.rd_commit(src, src, FAKE, FAKE, ctx, B, H, N, D, Cmax, L, dt, cache, cache, ctx_out, None,
                         hidden, Dh, hid_last, None)


def test_commit_argument_errors(lib):
    assert _commit(lib, B=0) == INVALID
    assert _commit(lib, Cmax=0) == INVALID
    assert _commit(lib, D=96) == UNSUPPORTED
    assert _commit(lib, N=385) == UNSUPPORTED
    assert _commit(lib, dt=5) == UNSUPPORTED
    assert _commit(lib, src=None) == INVALID
    assert _commit(lib, cache=None) == INVALID
    assert _commit(lib, cache=FAKE + 8) == INVALID            # 16-byte alignment
    assert _commit(lib, ctx_out=None) == INVALID
    assert _commit(lib, ctx_out=FAKE) == INVALID              # must not be ctx_len itself
    assert _commit(lib, hidden=FAKE, Dh=0, hid_last=FAKE) == INVALID
    assert _commit(lib, hidden=FAKE, Dh=6, hid_last=FAKE) == INVALID   # 24 bytes: not a multiple of 16
    assert _commit(lib, hidden=FAKE, Dh=8, hid_last=None) == INVALID


def test_commit_paged_argument_errors(lib):
    def call(B=1, H=2, N=8, D=64, L=4, dt=1, ps=64, mp=2, npg=4, pages=FAKE, table=FAKE, ctx_out=FAKE + 64):
        return lib.rd_commit_paged(FAKE, FAKE, FAKE, FAKE, FAKE, B, H, N, D, L, dt, pages, pages, table, ps, mp, npg,
                                   ctx_out, None, None, 0, None, None)
    assert call(ps=0) == INVALID
    assert call(npg=0) == INVALID
    assert call(D=96) == UNSUPPORTED
    assert call(dt=9) == UNSUPPORTED
    assert call(pages=None) == INVALID
    assert call(table=None) == INVALID
    assert call(ctx_out=FAKE) == INVALID                     # must not be ctx_len itself
    assert call(pages=FAKE + 8) == INVALID


def test_rope_argument_errors(lib):
    def call(q=FAKE, k=FAKE, pos=FAKE, tab=FAKE, max_pos=16, B=1, H=2, N=8, D=64, dt=1):
        return lib.rd_rope(q, k, pos, FAKE, tab, tab, max_pos, B, H, N, D, dt, None)
    assert call(B=0) == INVALID
    assert call(max_pos=0) == INVALID
    assert call(D=96) == UNSUPPORTED
    assert call(N=385) == UNSUPPORTED
    assert call(dt=4) == UNSUPPORTED
    assert call(q=None, k=None) == INVALID
    assert call(pos=None) == INVALID
    assert call(tab=None) == INVALID
    assert call(q=FAKE + 16) == INVALID                      # 32-byte alignment


def test_draft_argument_errors(lib):
    import ctypes
    from paper_2403_09919_amd.binding import _DraftParams

    def call(Dm=64, V=100, K=1, B=1, W=4, L=5, emb=FAKE, mlp=FAKE, h=FAKE, ws=FAKE, ws_bytes=None, params=True,
             sl=None, sr=None, dt=1):
        p = _DraftParams(emb, FAKE, FAKE, FAKE, mlp, mlp, FAKE, K, Dm, V, dt, 0)
        need = lib.rd_draft_workspace(B, W, L, Dm, V)
        return lib.rd_draft(ctypes.byref(p) if params else None, h, FAKE, B, W, L, FAKE, FAKE, sl, sr, ws,
                            need if ws_bytes is None else ws_bytes, None)
    assert call(dt=0) == UNSUPPORTED                         # weights are bf16 (1) or fp16 (2)
    assert call(dt=3) == UNSUPPORTED
    assert call(sl=FAKE) == INVALID                          # the record of the search: both outputs or neither
    assert call(sr=FAKE) == INVALID
    assert call(sl=FAKE + 4, sr=FAKE) == INVALID
    assert call(params=False) == INVALID
    assert call(B=0) == INVALID
    assert call(Dm=0) == INVALID
    assert call(Dm=96) == UNSUPPORTED                        # multiple of 64
    assert call(W=129, V=1000) == UNSUPPORTED
    assert call(B=200, W=4) == UNSUPPORTED                   # B*W <= 512
    assert call(V=300000) == UNSUPPORTED
    assert call(V=3, W=4) == UNSUPPORTED                     # W <= V
    assert call(emb=None) == INVALID
    assert call(mlp=None) == INVALID
    assert call(h=None) == INVALID
    assert call(emb=FAKE + 8) == INVALID
    assert call(ws=None) == WORKSPACE
    assert call(ws_bytes=64) == WORKSPACE
    assert lib.rd_draft_workspace(1, 4, 5, 96, 100) == 0


def test_pack_weights_argument_errors(lib):
    assert lib.rd_draft_packed_elems(100, 64) == 112 * 64
    assert lib.rd_draft_packed_elems(100, 40) == 0            # K a multiple of 32
    assert lib.rd_draft_pack_weights(None, 16, 32, FAKE, None) == INVALID
    assert lib.rd_draft_pack_weights(FAKE, 16, 32, None, None) == INVALID
    assert lib.rd_draft_pack_weights(FAKE, 0, 32, FAKE, None) == INVALID
    assert lib.rd_draft_pack_weights(FAKE, 16, 40, FAKE, None) == UNSUPPORTED
    assert lib.rd_draft_pack_weights(FAKE + 2, 16, 32, FAKE, None) == INVALID


def test_binding_rejects_host_tensors():
    import torch
    from paper_2403_09919_amd import binding
    with pytest.raises(ValueError):
        binding.rd_dedup(torch.zeros((1, 2, 2), dtype=torch.int32))
