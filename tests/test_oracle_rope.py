"""Pins for the oracle's rotary embedding: the same rotation written with complex numbers in numpy,
what it must leave alone, and the property rotary embeddings exist for (scores depend on the
distance between positions only)."""
import numpy as np

import oracle
from paper_2403_09919_amd import synth


def tables(max_pos, D, base=10000.0):
    inv = base ** (-np.arange(D // 2, dtype=np.float64) * 2.0 / D)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def test_rope_equals_complex_rotation_and_leaves_the_rest_alone():
    rng = np.random.default_rng(4)
    B, H, N, D, max_pos = 3, 2, 9, 16, 300
    x = rng.standard_normal((B, H, N, D)).astype(np.float32)
    pos = rng.integers(0, max_pos, (B, N)).astype(np.int32)
    pos[0, 0] = 0                                     # angle 0: identity
    pos[1, 2] = max_pos + 50                          # clamped to the last table row
    npk = np.array([9, 4, 0], np.int32)
    cos, sin = tables(max_pos, D)
    y = oracle.rope(x, pos, npk, cos, sin, "f32")
    half = D // 2
    z = x[..., :half].astype(np.float64) + 1j * x[..., half:].astype(np.float64)
    pc = np.clip(pos, 0, max_pos - 1)
    rot = (cos[pc].astype(np.float64) + 1j * sin[pc].astype(np.float64))[:, None, :, :]      # [B,1,N,half]
    zr = z * rot
    want = np.concatenate([zr.real, zr.imag], axis=-1).astype(np.float32)
    for b in range(B):
        assert np.array_equal(y[b, :, :npk[b]], want[b, :, :npk[b]])
        assert np.array_equal(y[b, :, npk[b]:], x[b, :, npk[b]:])            # rows beyond the packed count untouched
    assert np.array_equal(y[0, :, 0], x[0, :, 0])                             # position 0
    assert not np.array_equal(y[0, :, 1], x[0, :, 1])


def test_rope_scores_depend_on_distance_only_and_norms_are_kept():
    rng = np.random.default_rng(5)
    D, max_pos = 32, 4000
    cos, sin = tables(max_pos, D)
    q = rng.standard_normal((1, 1, 1, D)).astype(np.float32)
    k = rng.standard_normal((1, 1, 1, D)).astype(np.float32)
    one = np.array([1], np.int32)
    def score(m, n):
        qr = oracle.rope(q, np.array([[m]], np.int32), one, cos, sin, "f32").astype(np.float64)
        kr = oracle.rope(k, np.array([[n]], np.int32), one, cos, sin, "f32").astype(np.float64)
        assert abs(np.linalg.norm(qr) - np.linalg.norm(q.astype(np.float64))) < 1e-5
        return float((qr * kr).sum())
    base = score(7, 3)
    for shift in (1, 100, 2500, 3900):
        assert abs(score(7 + shift, 3 + shift) - base) < 2e-3 * max(1.0, abs(base))   # fp32 tables at large angles
    assert abs(score(8, 3) - base) > 1e-3


def test_rope_rounds_once_to_the_storage_type():
    rng = np.random.default_rng(6)
    B, H, N, D, max_pos = 1, 2, 5, 8, 64
    cos, sin = tables(max_pos, D)
    pos = rng.integers(0, max_pos, (B, N)).astype(np.int32)
    npk = np.array([N], np.int32)
    half = D // 2
    for dtype in ("bf16", "f16"):
        x32 = rng.standard_normal((B, H, N, D)).astype(np.float32)
        x = synth.f32_to_bf16_bits(x32) if dtype == "bf16" else x32.astype(np.float16)
        xd = synth.to_f64(x, dtype)
        c, s = cos[pos].astype(np.float64)[:, None], sin[pos].astype(np.float64)[:, None]
        want64 = np.concatenate([xd[..., :half] * c - xd[..., half:] * s, xd[..., half:] * c + xd[..., :half] * s], -1)
        y = oracle.rope(x, pos, npk, cos, sin, dtype)
        if dtype == "f16":
            assert np.array_equal(y, want64.astype(np.float16))              # numpy: one rounding from double
        else:
            err = np.abs(synth.to_f64(y, dtype) - want64)
            assert (err <= np.abs(want64) * 2.0 ** -8 + 1e-30).all()          # within half a bf16 ulp (8 significand bits)
