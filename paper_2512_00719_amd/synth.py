"""Seeded synthetic inputs for the sampling hot path (numpy only).

This module only *generates inputs* (logits, token histories, per-row
sampling parameters, hot sets).  It contains none of the sampling method's
arithmetic and is the one module that both the CPU oracle's tests and the
HIP path's tests/benchmarks may share.

The shapes follow the vocabulary sizes the paper lists for current model
families (section 2.3) and its workload description (section 7.1: all
sampling controls enabled).  The paper's real prompts and model logits are
not available, so every array here is synthetic:

* logits: a Zipf(s)-shaped base profile ``-s*ln(rank+1)`` laid over a seeded
  random permutation of the vocabulary, plus i.i.d. Gaussian noise;
* history: token ids drawn i.i.d. from the Zipf(1.1) law over the same
  permutation (duplicates are intended, they exercise counts above one);
* hot set: the ``H`` ids of lowest profile rank.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

# Layout of one row's sampling parameters (32 bytes, little endian).  It is the
# in-memory record the C boundary consumes; field meaning is documented there.
ROW_PARAMS_DTYPE = np.dtype(
    [
        ("temperature", "<f4"),
        ("top_k", "<i4"),
        ("top_p", "<f4"),
        ("min_p", "<f4"),
        ("rep_penalty", "<f4"),
        ("freq_penalty", "<f4"),
        ("pres_penalty", "<f4"),
        ("n_prompt", "<i4"),
    ],
    align=False,
)
assert ROW_PARAMS_DTYPE.itemsize == 32

SAMPLER_SEED = 0x2512007190000001  # default 64-bit sampler seed used by tests and the benchmark
DATA_SEED_BASE = 20251200


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    """One batch of synthetic input for the sampling call."""

    name: str
    B: int
    V: int
    dtype: str  # "f32" or "bf16"
    logits: np.ndarray  # [B, V] float32 (dtype f32) or uint16 bf16 bit patterns (dtype bf16)
    params: np.ndarray  # [B] ROW_PARAMS_DTYPE
    hist_ptr: np.ndarray  # [B+1] int64 CSR offsets
    hist_ids: np.ndarray  # [nnz] int32
    perm: Optional[np.ndarray] = None  # rank -> token id, when a Zipf profile was used
    hot_ids: Optional[np.ndarray] = None  # [H] int32 or None
    seed: int = SAMPLER_SEED
    meta: dict = field(default_factory=dict)

    def logits_f32(self) -> np.ndarray:
        """Logits as float32 values (exact upcast for bf16)."""
        if self.dtype == "bf16":
            return bf16_bits_to_f32(self.logits)
        return self.logits

    def with_hot(self, H: int) -> "Workload":
        """Copy of this workload whose hot set is the ``H`` lowest-rank ids of the profile."""
        assert self.perm is not None
        w = Workload(**{**self.__dict__})
        w.hot_ids = np.ascontiguousarray(self.perm[:H], dtype=np.int32)
        w.meta = dict(self.meta, H=int(H))
        return w


def make_params(B: int, **kw) -> np.ndarray:
    """Per-row parameter records; scalars broadcast, arrays are taken per row.

    Defaults disable everything: temperature 1, no top-k, top-p 1, min-p 0,
    repetition 1, frequency 0, presence 0, n_prompt 0.
    """
    p = np.zeros(B, dtype=ROW_PARAMS_DTYPE)
    p["temperature"] = 1.0
    p["top_k"] = 0
    p["top_p"] = 1.0
    p["min_p"] = 0.0
    p["rep_penalty"] = 1.0
    p["freq_penalty"] = 0.0
    p["pres_penalty"] = 0.0
    p["n_prompt"] = 0
    for k, v in kw.items():
        p[k] = v
    return p


def zipf_profile_logits(B: int, V: int, s: float, sigma: float, rng: np.random.Generator,
                        dtype: str, perm: np.ndarray, chunk_rows: int = 64) -> np.ndarray:
    """``logits[b, perm[r]] = -s*ln(r+1) + sigma*eps`` with eps ~ N(0,1); cast to ``dtype``."""
    base_by_rank = (-s * np.log(np.arange(1, V + 1, dtype=np.float64))).astype(np.float32)
    base_by_id = np.empty(V, dtype=np.float32)
    base_by_id[perm] = base_by_rank
    out = np.empty((B, V), dtype=np.float32 if dtype == "f32" else np.uint16)
    for r0 in range(0, B, chunk_rows):
        r1 = min(B, r0 + chunk_rows)
        x = rng.standard_normal((r1 - r0, V), dtype=np.float32)
        x *= np.float32(sigma)
        x += base_by_id[None, :]
        out[r0:r1] = x if dtype == "f32" else f32_to_bf16_bits(x)
    return out


def zipf_history(B: int, nnz: int, V: int, s: float, rng: np.random.Generator,
                 perm: Optional[np.ndarray]) -> tuple[np.ndarray, np.ndarray]:
    """CSR history with ``nnz`` ids per row, ranks drawn with P(r) proportional to (r+1)^-s."""
    pmf = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(pmf)
    cdf /= cdf[-1]
    ranks = np.searchsorted(cdf, rng.random(B * nnz), side="right")
    np.minimum(ranks, V - 1, out=ranks)
    ids = ranks if perm is None else perm[ranks]
    hist_ptr = (np.arange(B + 1, dtype=np.int64) * nnz).astype(np.int64)
    return hist_ptr, np.ascontiguousarray(ids, dtype=np.int32)


def _mixed_filter_params(B: int, rng: np.random.Generator, **fixed) -> np.ndarray:
    """Heterogeneous per-row controls: temp U[0.5,1.2], top-k in {0,20,50,1000},
    top-p U[0.8,1.0], min-p in {0,0.05}, 10 % greedy rows (temperature 0)."""
    temp = rng.uniform(0.5, 1.2, B).astype(np.float32)
    top_k = rng.choice(np.array([0, 20, 50, 1000], dtype=np.int32), B)
    top_p = rng.uniform(0.8, 1.0, B).astype(np.float32)
    min_p = rng.choice(np.array([0.0, 0.05], dtype=np.float32), B)
    greedy = rng.random(B) < 0.10
    temp[greedy] = 0.0
    return make_params(B, temperature=temp, top_k=top_k, top_p=top_p, min_p=min_p, **fixed)


def make_config(idx: int, B: Optional[int] = None, V: Optional[int] = None,
                nnz: Optional[int] = None, H: Optional[int] = None) -> Workload:
    """The five benchmark configurations (1-based ``idx``); B/V/nnz/H may be overridden
    to obtain a reduced case with the same value distributions and structure."""
    rng = np.random.default_rng(DATA_SEED_BASE + idx)
    if idx == 1:  # Tiny
        B = B or 4
        V = V or 1024
        nnz = 64 if nnz is None else nnz
        logits = rng.standard_normal((B, V), dtype=np.float32)
        hist_ptr = (np.arange(B + 1, dtype=np.int64) * nnz)
        hist_ids = rng.integers(0, V, B * nnz).astype(np.int32)
        params = make_params(B, temperature=0.8, top_k=50, top_p=0.9,
                             rep_penalty=1.1, freq_penalty=0.2, pres_penalty=0.1)
        return Workload("C1-tiny", B, V, "f32", logits, params, hist_ptr, hist_ids)
    if idx == 2:
        B = B or 256
        V = V or 151_936
        nnz = 2048 if nnz is None else nnz
        s, sigma, dtype = 1.1, 1.5, "bf16"
        params = make_params(B, temperature=0.7, top_k=20, top_p=0.8, rep_penalty=1.05)
    elif idx == 3:
        B = B or 1024
        V = V or 128_256
        nnz = 4096 if nnz is None else nnz
        s, sigma, dtype = 1.1, 1.5, "f32"
        params = _mixed_filter_params(B, rng, rep_penalty=1.1, freq_penalty=0.2, pres_penalty=0.1)
    elif idx == 4:
        B = B or 512
        V = V or 201_088
        nnz = 0 if nnz is None else nnz
        s, sigma, dtype = 1.2, 1.0, "bf16"
        params = make_params(B, temperature=1.0, top_p=0.95)
    elif idx == 5:
        B = B or 4096
        V = V or 256_000
        nnz = 8192 if nnz is None else nnz
        s, sigma, dtype = 1.1, 1.5, "bf16"
        params = _mixed_filter_params(B, rng, rep_penalty=1.1, freq_penalty=0.3, pres_penalty=0.2)
    else:
        raise ValueError("config index must be 1..5")
    perm = rng.permutation(V).astype(np.int64)
    logits = zipf_profile_logits(B, V, s, sigma, rng, dtype, perm)
    if nnz > 0:
        hist_ptr, hist_ids = zipf_history(B, nnz, V, 1.1, rng, perm)
    else:
        hist_ptr, hist_ids = np.zeros(B + 1, dtype=np.int64), np.zeros(0, dtype=np.int32)
    w = Workload(f"C{idx}", B, V, dtype, logits, params, hist_ptr, hist_ids, perm=perm,
                 meta={"zipf_s": s, "sigma": sigma, "nnz_per_row": nnz})
    if idx == 4:
        w = w.with_hot(H or 16384)
    if idx == 5:
        w = w.with_hot(min(H or 16384, V))
    return w
