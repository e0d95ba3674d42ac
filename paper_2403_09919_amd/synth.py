"""Seeded synthetic workloads for the ReDrafter verification step.

This module only draws random inputs (beams, context lengths, Q/K/V tensors,
logits) and converts between fp32 and bf16 bit patterns.  It holds none of the
method's arithmetic: wherever a generator needs the result of the dedup step
(the planted-argmax logits need to know which packed node is a child of which),
that result is passed in by the caller.  It is shared by the CPU oracle's tests
and by the HIP path's tests and benchmark, and imports neither.

Workload shapes follow the paper's setting: beam length 5 and beam widths 8-16
(Sec. 4.3, Table 3), Vicuna 7B/13B/33B attention geometry (Sec. 4), and a
sharing level that removes 30-60% of the beam tokens (Sec. 4.3.2, Fig. 5).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

SEED_BASE = 0x5EED0000

# stream ids: every tensor group has its own counter-based child stream so a
# test can draw only what it needs and still see the same values.
_S_CTX, _S_BEAM, _S_QNEW, _S_KCACHE, _S_VCACHE, _S_LOGITS, _S_DRAFT, _S_UNIFORM = range(8)


@dataclass(frozen=True)
class Config:
    idx: int
    name: str
    B: int
    ctx_lo: int          # context length is U{ctx_lo..ctx_hi} per sequence
    ctx_hi: int
    H: int
    D: int
    dtype: str           # "f32", "bf16" (or "f16" in tests)
    W: int
    L: int
    V: int
    share: str           # "uniform": s ~ U{0..L};  "high": s = L-1 w.p. 0.5 else U{0..L}
    p_plant: float

    @property
    def N(self) -> int:
        return self.W * self.L

    @property
    def Cmax(self) -> int:
        return self.ctx_hi

    @property
    def seed(self) -> int:
        return SEED_BASE + self.idx


CONFIGS: Dict[int, Config] = {
    1: Config(1, "tiny", 1, 128, 128, 4, 64, "f32", 4, 4, 1000, "uniform", 0.7),
    2: Config(2, "vicuna7b_layer", 1, 1024, 1024, 32, 128, "bf16", 8, 5, 32000, "uniform", 0.7),
    3: Config(3, "batched7b", 8, 1024, 2048, 32, 128, "bf16", 8, 5, 32000, "uniform", 0.7),
    4: Config(4, "vicuna13b", 4, 4096, 4096, 40, 128, "bf16", 16, 5, 32000, "uniform", 0.6),
    5: Config(5, "vicuna33b", 16, 2048, 2048, 52, 128, "bf16", 16, 5, 32000, "high", 0.8),
}


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream)])


# ----------------------------------------------------------------------------
# bf16 bit-pattern helpers (storage format only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    r = np.where(nan, (u >> 16) | 0x0040, r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact upcast of a stored tensor (fp32 values, bf16 bit patterns or numpy float16) to float64."""
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    if dtype == "f16":
        return np.asarray(x, dtype=np.float16).astype(np.float64)
    return np.asarray(x, dtype=np.float32).astype(np.float64)


def _normal(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    if dtype == "f16":
        return x.astype(np.float16)          # numpy rounds to nearest even
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def poison_value(dtype: str):
    """A NaN in the storage format, used to fill cache entries that must never be read."""
    if dtype == "f16":
        return np.float16(np.nan)
    return np.uint16(0x7FC1) if dtype == "bf16" else np.float32(np.nan)


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------
def make_ctx_len(B: int, lo: int, hi: int, seed: int) -> np.ndarray:
    rng = _rng(seed, _S_CTX)
    if lo == hi:
        return np.full((B,), lo, dtype=np.int32)
    return rng.integers(lo, hi + 1, size=B).astype(np.int32)


def make_beams(B: int, W: int, L: int, V: int, seed: int, share: str = "uniform") -> np.ndarray:
    """Beam-search-like candidates: beam 0 is uniform over the vocabulary; each later
    beam copies a prefix of s tokens from a random earlier beam and continues with
    uniform tokens.  s = L yields an exact duplicate beam, s = 0 a new root."""
    rng = _rng(seed, _S_BEAM)
    beams = np.empty((B, W, L), dtype=np.int32)
    for b in range(B):
        beams[b, 0] = rng.integers(0, V, size=L)
        for i in range(1, W):
            if share == "high" and rng.random() < 0.5:
                s = L - 1
            else:
                s = int(rng.integers(0, L + 1))
            src = int(rng.integers(0, i))
            beams[b, i, :s] = beams[b, src, :s]
            beams[b, i, s:] = rng.integers(0, V, size=L - s)
    return beams


def make_qkv_new(B: int, H: int, N: int, D: int, dtype: str, seed: int
                 ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    rng = _rng(seed, _S_QNEW)
    q = _normal(rng, (B, H, N, D), dtype)
    k = _normal(rng, (B, H, N, D), dtype)
    v = _normal(rng, (B, H, N, D), dtype)
    return q, k, v


def make_kv_cache(B: int, H: int, Cmax: int, D: int, dtype: str, seed: int,
                  ctx_len: Optional[np.ndarray] = None, poison: bool = False
                  ) -> Tuple[np.ndarray, np.ndarray]:
    """K and V caches [B,H,Cmax,D] ~ N(0,1).  With poison=True the entries at
    positions >= ctx_len[b] are NaN (they must never influence a result)."""
    out = []
    for stream in (_S_KCACHE, _S_VCACHE):
        rng = _rng(seed, stream)
        t = np.empty((B, H, Cmax, D), dtype={"bf16": np.uint16, "f16": np.float16}.get(dtype, np.float32))
        for b in range(B):               # chunked: the 33B-shaped cache is 436 MB per tensor
            t[b] = _normal(rng, (H, Cmax, D), dtype)
            if poison and ctx_len is not None and int(ctx_len[b]) < Cmax:
                t[b, :, int(ctx_len[b]):, :] = poison_value(dtype)
        out.append(t)
    return out[0], out[1]


def make_logits(B: int, N: int, V: int, seed: int,
                packed_tokens: np.ndarray, parent: np.ndarray, n_packed: np.ndarray,
                p_plant: float, bump: float = 8.0) -> np.ndarray:
    """LLM-output stand-in: fp32 N(0,1) rows; for each packed node that has children,
    with probability p_plant one child (uniform) gets +bump at its token, so the row's
    argmax usually, not always, continues that branch.  `packed_tokens`, `parent`
    and `n_packed` are the dedup step's outputs, supplied by the caller."""
    rng = _rng(seed, _S_LOGITS)
    logits = rng.standard_normal((B, N, V), dtype=np.float32)
    for b in range(B):
        P = int(n_packed[b])
        for p in range(P):
            kids = [c for c in range(P) if int(parent[b, c]) == p]
            if not kids:
                continue
            u = rng.random()
            pick = int(rng.integers(0, len(kids)))
            if u < p_plant:
                tok = int(packed_tokens[b, kids[pick]])
                if 0 <= tok < V:
                    logits[b, p, tok] += np.float32(bump)
    return logits


def make_draft_logits(logits: np.ndarray, seed: int, noise: float = 1.0) -> np.ndarray:
    """Draft-model stand-in for sampling-mode acceptance: the LLM's logits plus N(0, noise^2), so the
    two distributions agree roughly, as a distilled drafter's do."""
    rng = _rng(seed, _S_DRAFT)
    return (logits + np.float32(noise) * rng.standard_normal(logits.shape, dtype=np.float32)).astype(np.float32)


def make_uniforms(shape, seed: int) -> np.ndarray:
    """Uniform numbers in [0, 1) as float32 (the random draws of sampling-mode acceptance)."""
    rng = _rng(seed, _S_UNIFORM)
    u = rng.random(shape, dtype=np.float32)
    return np.minimum(u, np.float32(1.0 - 2.0 ** -24))


def make_attn_inputs(cfg: Config, seed: Optional[int] = None, poison: bool = True) -> dict:
    """All tensors of one verification step except the logits (which need the dedup result)."""
    seed = cfg.seed if seed is None else seed
    ctx_len = make_ctx_len(cfg.B, cfg.ctx_lo, cfg.ctx_hi, seed)
    beams = make_beams(cfg.B, cfg.W, cfg.L, cfg.V, seed, cfg.share)
    q, k_new, v_new = make_qkv_new(cfg.B, cfg.H, cfg.N, cfg.D, cfg.dtype, seed)
    k_cache, v_cache = make_kv_cache(cfg.B, cfg.H, cfg.Cmax, cfg.D, cfg.dtype, seed, ctx_len, poison)
    return dict(ctx_len=ctx_len, beams=beams, q=q, k_new=k_new, v_new=v_new,
                k_cache=k_cache, v_cache=v_cache)
