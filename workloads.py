"""Seeded synthetic inputs for blockwise parallel decoding.

This module is the only code shared by the CPU oracle's tests and the HIP path's
tests/bench: it draws random numbers and lays them out, and holds none of the
method's arithmetic (no attention, no argmax, no acceptance test).  Everything is
generated with ``numpy.random.default_rng(seed)`` so both sides see identical
arrays.

The five workloads mirror the shapes of the paper's two tasks (Section 7.1:
subword translation with a ~32k vocabulary; Section 7.2: 8x8 -> 32x32 image
super-resolution, 3072 output intensity tokens).  The datasets themselves are
not used: token ids follow a bounded Zipf law, source lengths a clipped
log-normal, weights are N(0, 0.02).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional, Tuple

import numpy as np

BASE_SEED = 181103115


@dataclasses.dataclass(frozen=True)
class Config:
    """Shape of one workload.  ``k`` counts all heads, p_1 included (Section 3)."""
    name: str
    index: int
    n_enc: int
    n_dec: int
    d_model: int
    n_heads: int
    d_ff: int
    vocab: int
    k: int
    batch: int
    max_src: int
    max_out: int
    dtype: str            # "f32" or "bf16" (bf16 weights / cache, fp32 accumulate)
    eos_id: int           # < 0: fixed-length decoding (Section 2, image generation)
    pad_id: int = 0
    ln_eps: float = 1e-6
    src_kind: str = "zipf"      # "uniform3" (ids in [3,V)), "zipf", "uniform0" (ids in [0,V))
    src_len_kind: str = "fixed"  # "fixed" or "lognormal"
    local_q: int = 0            # 1D local self-attention in the decoder (Section 7.2): query block length, 0 = full causal
    local_m: int = 0            # ... and the number of positions before the query block that stay visible

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    @property
    def cache_slots(self) -> int:
        """Decoder positions that can ever be touched: 0..max_out-1+k."""
        return self.max_out + self.k + 1


C0 = Config("C0-tiny-f32", 0, 2, 2, 64, 4, 256, 256, 4, 1, 16, 32, "f32", 2,
            src_kind="uniform3")
C1 = Config("C1-base-bf16", 1, 6, 6, 512, 8, 2048, 32000, 8, 1, 32, 64, "bf16", 2)
C2 = Config("C2-big-bf16-b1", 2, 6, 6, 1024, 16, 4096, 32768, 10, 1, 128, 128, "bf16", 2,
            src_len_kind="lognormal")
C3 = Config("C3-big-bf16-b32", 3, 6, 6, 1024, 16, 4096, 32768, 10, 32, 128, 128, "bf16", 2,
            src_len_kind="lognormal")
C4 = Config("C4-superres-bf16-b8", 4, 6, 6, 512, 8, 2048, 256, 10, 8, 192, 3072, "bf16", -1,
            src_kind="uniform0")
# C4 with the decoder's self-attention as 1D local attention, the layer the paper names for its image model (Section
# 7.2).  The paper gives no block lengths: 256 query positions + 256 of memory are this build's example.
C4L = dataclasses.replace(C4, name="C4L-superres-local-bf16-b8", index=5, local_q=256, local_m=256)
CONFIGS = {c.name.split("-")[0]: c for c in (C0, C1, C2, C3, C4, C4L)}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of ``cfg`` with some fields replaced (used for reduced-size test cases)."""
    return dataclasses.replace(cfg, **kw)


# ----------------------------------------------------------------------------- bf16

def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


# ----------------------------------------------------------------------------- weights

def weight_shapes(cfg: Config) -> Dict[str, Tuple[int, ...]]:
    """Name -> shape of every tensor of the combined scoring-and-proposal model.

    Projection matrices are stored input-major: ``y = x @ W`` with ``W[in, out]``.
    """
    d, f, v, k = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.k
    s: Dict[str, Tuple[int, ...]] = {
        "emb": (v, d),
        "pos_src": (cfg.max_src, d),
        "pos_tgt": (cfg.cache_slots, d),
    }

    def ln(prefix):
        s[prefix + ".g"] = (d,)
        s[prefix + ".b"] = (d,)

    def attn(prefix):
        for m in ("wq", "wk", "wv", "wo"):
            s[f"{prefix}.{m}"] = (d, d)

    def ffn(prefix):
        s[prefix + ".w1"] = (d, f)
        s[prefix + ".b1"] = (f,)
        s[prefix + ".w2"] = (f, d)
        s[prefix + ".b2"] = (d,)

    for l in range(cfg.n_enc):
        ln(f"enc.{l}.ln1"); attn(f"enc.{l}.self"); ln(f"enc.{l}.ln2"); ffn(f"enc.{l}.ffn")
    ln("enc.lnf")
    for l in range(cfg.n_dec):
        ln(f"dec.{l}.ln1"); attn(f"dec.{l}.self")
        ln(f"dec.{l}.ln2"); attn(f"dec.{l}.cross")
        ln(f"dec.{l}.ln3"); ffn(f"dec.{l}.ffn")
    ln("dec.lnf")
    s["head.w1"] = (k, d, f)
    s["head.b1"] = (k, f)
    s["head.w2"] = (k, f, d)
    s["head.b2"] = (k, d)
    return s


def make_weights(cfg: Config, seed: Optional[int] = None, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Every tensor ~ N(0, std); LayerNorm gains are 1 + N(0, std).  fp32 arrays;
    for bf16 workloads the values are rounded to bf16 first so that both sides
    start from bit-identical numbers."""
    rng = np.random.default_rng(BASE_SEED + 10 * cfg.index if seed is None else seed)
    out = {}
    for name, shape in weight_shapes(cfg).items():
        w = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if name.endswith(".g"):
            w = w + np.float32(1.0)
        if cfg.dtype == "bf16":
            w = round_bf16(w)
        out[name] = w
    return out


# ----------------------------------------------------------------------------- sources

def _zipf_ids(rng, n: int, vocab: int, s: float = 1.1) -> np.ndarray:
    """ids = 2 + rank, rank in 1..V-3 with P(rank) ~ rank^-s (inverse CDF on the finite table)."""
    ranks = np.arange(1, vocab - 2, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-s))
    cdf /= cdf[-1]
    r = np.searchsorted(cdf, rng.random(n), side="left") + 1
    return (2 + np.minimum(r, vocab - 3)).astype(np.int32)


def make_sources(cfg: Config, seed: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """(src_ids[B, max_src] padded with pad_id, src_len[B])."""
    base = BASE_SEED + 10 * cfg.index if seed is None else seed
    rng_len = np.random.default_rng(base + 2)
    rng_ids = np.random.default_rng(base + 1)
    B, S = cfg.batch, cfg.max_src
    if cfg.src_len_kind == "lognormal":
        ln_ = np.exp(rng_len.normal(math.log(27.0), 0.6, size=B))
        src_len = np.clip(np.rint(ln_), 1, S).astype(np.int32)
    else:
        src_len = np.full(B, S, dtype=np.int32)
    ids = np.full((B, S), cfg.pad_id, dtype=np.int32)
    for b in range(B):
        n = int(src_len[b])
        if cfg.src_kind == "uniform3":
            ids[b, :n] = rng_ids.integers(3, cfg.vocab, size=n)
        elif cfg.src_kind == "uniform0":
            ids[b, :n] = rng_ids.integers(0, cfg.vocab, size=n)
        else:
            ids[b, :n] = _zipf_ids(rng_ids, n, cfg.vocab)
    return ids, src_len


def make_max_len(cfg: Config, src_len: np.ndarray) -> np.ndarray:
    """Per-sequence output budget.  Batched translation workloads get a
    length-dependent budget so that sequences finish at different steps."""
    if cfg.batch > 1 and cfg.src_len_kind == "lognormal":
        return np.clip(np.rint(1.1 * src_len) + 4, 1, cfg.max_out).astype(np.int32)
    return np.full(cfg.batch, cfg.max_out, dtype=np.int32)


def make_tokens(cfg: Config, n: int, seed: int) -> np.ndarray:
    """[B, n] target-side token ids for teacher-forced states (never EOS/PAD)."""
    rng = np.random.default_rng(seed)
    lo = 3 if cfg.eos_id >= 0 else 0
    return rng.integers(lo, cfg.vocab, size=(cfg.batch, n)).astype(np.int32)


# ----------------------------------------------------------------------------- schedules

def geometric_ratio(k: int, mean: float) -> float:
    """r such that pmf(a) ~ r^(a-1), a in 1..k, has the requested mean."""
    if not (1.0 < mean < k):
        raise ValueError("mean must lie strictly between 1 and k")

    def m(r):
        a = np.arange(1, k + 1, dtype=np.float64)
        p = r ** (a - 1)
        return float((a * p).sum() / p.sum())

    lo, hi = 1e-9, 1e3
    for _ in range(200):
        mid = math.sqrt(lo * hi)
        if m(mid) < mean:
            lo = mid
        else:
            hi = mid
    return math.sqrt(lo * hi)


def make_schedule(cfg: Config, mean: float, steps: int, seed: Optional[int] = None,
                  k: Optional[int] = None) -> np.ndarray:
    """[steps, B] imposed accepted lengths in 1..k, truncated geometric with the given mean."""
    k = cfg.k if k is None else k
    base = BASE_SEED + 10 * cfg.index if seed is None else seed
    rng = np.random.default_rng(base + 3)
    if mean <= 1.0:
        return np.ones((steps, cfg.batch), dtype=np.int32)
    if mean >= k:
        return np.full((steps, cfg.batch), k, dtype=np.int32)
    r = geometric_ratio(k, mean)
    a = np.arange(1, k + 1, dtype=np.float64)
    p = r ** (a - 1)
    p /= p.sum()
    return rng.choice(np.arange(1, k + 1), size=(steps, cfg.batch), p=p).astype(np.int32)
