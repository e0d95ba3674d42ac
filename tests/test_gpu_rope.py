"""GPU parity for rd_rope against the CPU oracle, and the rotated step: rd_dedup -> rd_rope ->
rd_tree_attn equals the oracle's dedup -> rope -> attention."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import announce, dev, host
from paper_2403_09919_amd import synth
from test_oracle_rope import tables

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rd():
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2403_09919_amd import binding
    return binding


def _tol(dtype, ref64, src64):
    # fp32 arithmetic (each product and the sum rounded) then one rounding to the storage type on the
    # GPU, fp64 then one rounding in the oracle: one unit in the last place of the storage type where
    # the double rounding matters, plus the fp32 rounding of the products, which is relative to the
    # operands (|x[i]| + |x[i+D/2]|), not to a result that may have cancelled
    ulp = {"f32": 2.0 ** -23, "bf16": 2.0 ** -7, "f16": 2.0 ** -10}[dtype]
    half = src64.shape[-1] // 2
    mag = np.abs(src64[..., :half]) + np.abs(src64[..., half:])
    mag = np.concatenate([mag, mag], axis=-1)
    return np.abs(ref64) * ulp + mag * 2.0 ** -22 + 1e-30


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("D,B,H,W,L", [(128, 2, 3, 8, 5), (64, 3, 2, 4, 4), (128, 1, 32, 70, 5), (64, 1, 1, 1, 1)])
def test_rope_matches_oracle(rd, dtype, D, B, H, W, L):
    announce(f"rope {dtype} D={D} B={B} H={H} W={W} L={L}")
    seed = D + W
    ctx = np.array([0, 1000, 4090][:B], np.int32)
    beams = synth.make_beams(B, W, L, 7, seed)
    d = oracle.dedup(beams, ctx)
    q, kn, _ = synth.make_qkv_new(B, H, W * L, D, dtype, seed)
    max_pos = 4096
    cos, sin = tables(max_pos, D)
    pos = d["position_ids"].copy()
    pos[pos < 0] = 0
    ref_q = oracle.rope(q, pos, d["n_packed"], cos, sin, dtype)
    ref_k = oracle.rope(kn, pos, d["n_packed"], cos, sin, dtype)
    q_d, k_d = dev(q), dev(kn)
    dd = rd.rd_dedup(dev(beams), dev(ctx))
    rd.rd_rope(q_d, k_d, dd["position_ids"], dd["n_packed"], dev(cos), dev(sin))
    torch.cuda.synchronize()
    for got, ref, src in ((host(q_d), ref_q, q), (host(k_d), ref_k, kn)):
        g64, r64 = synth.to_f64(got, dtype), synth.to_f64(ref, dtype)
        assert (np.abs(g64 - r64) <= _tol(dtype, r64, synth.to_f64(src, dtype))).all()
        if dtype != "f32":
            mism = float((g64 != r64).mean())
            assert mism < 1e-3, mism                               # and almost everywhere the same bits
        for b in range(B):                                         # rows beyond the packed count untouched
            P = int(d["n_packed"][b])
            assert np.array_equal(got[b, :, P:], src[b, :, P:])
    # q only / k only
    q2, k2 = dev(q), dev(kn)
    rd.rd_rope(q2, None, dd["position_ids"], dd["n_packed"], dev(cos), dev(sin))
    rd.rd_rope(None, k2, dd["position_ids"], dd["n_packed"], dev(cos), dev(sin))
    torch.cuda.synchronize()
    assert np.array_equal(host(q2), host(q_d)) and np.array_equal(host(k2), host(k_d))


def test_rotated_step_matches_oracle(rd):
    announce("dedup -> rope -> tree attention, config 2 shape")
    cfg = synth.CONFIGS[2]
    t = synth.make_attn_inputs(cfg, poison=False)
    scale = float(1.0 / np.sqrt(cfg.D))
    cos, sin = tables(2048, cfg.D)
    d = oracle.dedup(t["beams"], t["ctx_len"])
    pos = np.maximum(d["position_ids"], 0)
    q_r = oracle.rope(t["q"], pos, d["n_packed"], cos, sin, cfg.dtype)
    k_r = oracle.rope(t["k_new"], pos, d["n_packed"], cos, sin, cfg.dtype)
    ref = oracle.tree_attn(q_r, t["k_cache"], t["v_cache"], t["ctx_len"], k_r, t["v_new"], d["n_packed"],
                           d["tree_mask"], cfg.dtype, scale)
    ctx_d = dev(t["ctx_len"])
    dd = rd.rd_dedup(dev(t["beams"]), ctx_d)
    q_d, k_d = dev(t["q"]), dev(t["k_new"])
    rd.rd_rope(q_d, k_d, dd["position_ids"], dd["n_packed"], dev(cos), dev(sin))
    out = rd.rd_tree_attn(q_d, dev(t["k_cache"]), dev(t["v_cache"]), ctx_d, k_d, dev(t["v_new"]), dd["n_packed"],
                          dd["tree_mask_bits"], scale)
    torch.cuda.synchronize()
    err = np.abs(synth.to_f64(host(out), cfg.dtype) - synth.to_f64(ref, cfg.dtype)).max()
    assert err <= 2e-2, err


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("D,B,H,W,L,ctx", [(128, 1, 32, 8, 5, [1024]),            # the Vicuna-7B-shaped layer
                                           (128, 3, 2, 8, 5, [0, 517, 129]),      # ragged, an empty context
                                           (64, 2, 3, 16, 6, [700, 33]),          # D = 64, six row tiles
                                           (128, 2, 4, 16, 5, [5000, 2311]),      # long contexts: packed keys fused into the last range
                                           (128, 2, 2, 70, 5, [97, 640]),         # the widest beams: row groups, three packed-key blocks
                                           (128, 2, 8, 16, 5, [4096, 4096])])
def test_fused_rope_equals_rope_then_attention(rd, dtype, D, B, H, W, L, ctx):
    """rd_tree_attn_rope (q and k_new unrotated, rotation inside the attention call) against rd_rope
    followed by rd_tree_attn -- bit for bit, the rotation arithmetic is the same -- and against the
    oracle's rope -> tree attention chain within the attention tolerance; the rotated keys it hands back
    equal rd_rope's."""
    announce(f"fused rope {dtype} D={D} B={B} H={H} W={W} L={L}")
    N = W * L
    ctx = np.asarray(ctx, np.int32)
    Cmax = int(ctx.max())
    seed = D + W + B
    beams = synth.make_beams(B, W, L, 6 if W > 16 else 32000, seed, "high" if W > 16 else "uniform")
    q, kn, vn = synth.make_qkv_new(B, H, N, D, dtype, seed)
    kc, vc = synth.make_kv_cache(B, H, Cmax, D, dtype, seed, ctx, True)
    max_pos = 8192
    cos, sin = tables(max_pos, D)
    d = oracle.dedup(beams, ctx)
    pos = np.maximum(d["position_ids"], 0)
    scale = float(1.0 / np.sqrt(D))
    q_r = oracle.rope(q, pos, d["n_packed"], cos, sin, dtype)
    k_r = oracle.rope(kn, pos, d["n_packed"], cos, sin, dtype)
    ref = oracle.tree_attn(q_r, kc, vc, ctx, k_r, vn, d["n_packed"], d["tree_mask"], dtype, scale)

    ctx_d = dev(ctx)
    dd = rd.rd_dedup(dev(beams), ctx_d)
    cos_d, sin_d = dev(cos), dev(sin)
    kc_d, vc_d, vn_d = dev(kc), dev(vc), dev(vn)
    fused, k_rot = rd.rd_tree_attn_rope(dev(q), kc_d, vc_d, ctx_d, dev(kn), vn_d, dd["n_packed"], dd["tree_mask_bits"],
                                        dd["position_ids"], cos_d, sin_d, scale)
    q2, k2 = dev(q), dev(kn)
    rd.rd_rope(q2, k2, dd["position_ids"], dd["n_packed"], cos_d, sin_d)
    sep = rd.rd_tree_attn(q2, kc_d, vc_d, ctx_d, k2, vn_d, dd["n_packed"], dd["tree_mask_bits"], scale)
    torch.cuda.synchronize()
    assert np.array_equal(host(fused), host(sep))
    kr, k2h = host(k_rot), host(k2)
    for b in range(B):
        P = int(d["n_packed"][b])
        assert np.array_equal(kr[b, :, :P], k2h[b, :, :P])
        assert not kr[b, :, P:].any()                              # rows beyond the packed count untouched (allocated as zeros)
    err = np.abs(synth.to_f64(host(fused), dtype) - synth.to_f64(ref, dtype)).max()
    assert err <= (5e-3 if dtype == "f16" else 2e-2), err
    # without the rotated-keys output
    fused2, none = rd.rd_tree_attn_rope(dev(q), kc_d, vc_d, ctx_d, dev(kn), vn_d, dd["n_packed"], dd["tree_mask_bits"],
                                        dd["position_ids"], cos_d, sin_d, scale, want_k_rot=False)
    torch.cuda.synchronize()
    assert none is None and np.array_equal(host(fused2), host(fused))
