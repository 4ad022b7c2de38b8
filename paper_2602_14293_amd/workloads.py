"""Seeded synthetic knowledge-base workloads (inputs only; none of the retrieval arithmetic).

The paper's own knowledge base is a ~50 KB text document searched by an LLM state-matcher
(Section 3; Section 5, "Distribution of Optimization Usage"); it has no vector form.  These
generators produce the stand-in workloads for the numeric retrieval model: key matrices with
the stated sizes, dtypes, cluster structure and tag statistics.  Both the HIP path and the CPU
checker are fed from here; nothing in this module scores, filters or ranks anything.

Storage conventions (what the arrays hold):
  keys     torch.float32 / torch.bfloat16 / torch.float8_e4m3fn, row-major [N, d]
  scale    torch.float32 [N] (fp8 workloads only): stored value = scale[i] * code value
  tags     torch.int64 [N] holding the 64 tag bits of each entry (bit pattern, sign is meaningless)
  queries  torch.float32 / torch.bfloat16 / torch.float8_e4m3fn [Q, d] (fp8 queries carry no scale: it cancels)
  qmask    torch.int64 [Q] holding each query's 64 filter bits
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np
import torch

E4M3_MAX = 448.0


@dataclasses.dataclass
class Workload:
    name: str
    keys: torch.Tensor
    queries: torch.Tensor
    k: int
    scale: Optional[torch.Tensor] = None
    tags: Optional[torch.Tensor] = None
    qmask: Optional[torch.Tensor] = None
    seed: int = 0

    @property
    def N(self) -> int:
        return self.keys.shape[0]

    @property
    def d(self) -> int:
        return self.keys.shape[1]

    @property
    def Q(self) -> int:
        return self.queries.shape[0]


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _unit_rows(x: torch.Tensor) -> torch.Tensor:
    return x / x.norm(dim=1, keepdim=True).clamp_min(1e-30)


def random_bits64(n: int, p: float, g: torch.Generator, device) -> torch.Tensor:
    """n 64-bit words whose bits are iid Bernoulli(p), returned as int64 bit patterns."""
    out = torch.zeros(n, dtype=torch.int64, device=device)
    for b in range(64):
        bit = (torch.rand(n, generator=g, device=device) < p).to(torch.int64)
        # bit 63 set makes the int64 negative; shifts on int64 keep the pattern
        out |= bit << b
    return out


def clustered_keys(n: int, d: int, centers: int, noise: float, g: torch.Generator, device,
                   chunk: int = 1 << 17, center_rows: Optional[torch.Tensor] = None):
    """Rows = unit-vector centre (chosen uniformly) + iid N(0, noise^2) per coordinate, re-normalised (fp32)."""
    if center_rows is None:
        center_rows = _unit_rows(torch.randn(centers, d, generator=g, device=device))
    out = torch.empty(n, d, dtype=torch.float32, device=device)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        u = torch.randint(0, center_rows.shape[0], (e - s,), generator=g, device=device)
        x = center_rows[u] + noise * torch.randn(e - s, d, generator=g, device=device)
        out[s:e] = _unit_rows(x)
    return out, center_rows


def perturbed_queries(keys_f32_rows: torch.Tensor, sigma: float, g: torch.Generator) -> torch.Tensor:
    return keys_f32_rows + sigma * torch.randn(keys_f32_rows.shape, generator=g, device=keys_f32_rows.device)


def quantize_e4m3_rows(x: torch.Tensor):
    """Per-row scale = max|x| / 448, codes = round-to-nearest-even of x / scale onto the E4M3 grid."""
    amax = x.abs().amax(dim=1).clamp_min(1e-30)
    scale = (amax / E4M3_MAX).to(torch.float32)
    y = (x / scale[:, None]).clamp(-E4M3_MAX, E4M3_MAX)
    return y.to(torch.float8_e4m3fn), scale


def tiny(seed: int = 0, N: int = 4096, d: int = 256, Q: int = 8, k: int = 8, device="cpu") -> Workload:
    """fp32 keys and queries iid N(0,1), L2-normalised; no tags."""
    g = _gen(seed, device)
    keys = _unit_rows(torch.randn(N, d, generator=g, device=device))
    queries = _unit_rows(torch.randn(Q, d, generator=g, device=device))
    return Workload("tiny", keys, queries, k, seed=seed)


def clustered(seed: int = 0, N: int = 65536, d: int = 768, Q: int = 64, k: int = 16, centers: int = 256,
              device="cpu") -> Workload:
    """bf16 clustered keys (noise sigma 0.1 per coordinate); queries = random keys + N(0, 0.05^2) noise."""
    g = _gen(seed, device)
    kf, _ = clustered_keys(N, d, centers, 0.1, g, device)
    keys = kf.to(torch.bfloat16)
    del kf
    v = torch.randint(0, N, (Q,), generator=g, device=device)
    queries = perturbed_queries(keys[v].float(), 0.05, g).to(torch.bfloat16)
    return Workload("clustered", keys, queries, k, seed=seed)


def filtered(seed: int = 0, N: int = 1 << 20, d: int = 1024, Q: int = 256, k: int = 32, centers: int = 1024,
             p_tag: float = 0.3, p_qmask: Optional[float] = None, single_bit_qmask: bool = False,
             device="cpu") -> Workload:
    """Clustered bf16 keys with 64-bit tags (bits Bernoulli(p_tag)); each query has its own 64-bit mask.

    single_bit_qmask=True gives the sparse variant (one random bit per query) that makes the filter bite.
    """
    g = _gen(seed, device)
    kf, _ = clustered_keys(N, d, centers, 0.1, g, device)
    keys = kf.to(torch.bfloat16)
    del kf
    tags = random_bits64(N, p_tag, g, device)
    v = torch.randint(0, N, (Q,), generator=g, device=device)
    queries = perturbed_queries(keys[v].float(), 0.05, g).to(torch.bfloat16)
    if single_bit_qmask:
        qmask = torch.ones(Q, dtype=torch.int64, device=device) << torch.randint(0, 64, (Q,), generator=g, device=device)
    else:
        qmask = random_bits64(Q, p_tag if p_qmask is None else p_qmask, g, device)
    return Workload("filtered", keys, queries, k, tags=tags, qmask=qmask, seed=seed)


def compressed(seed: int = 0, N: int = 1 << 22, d: int = 768, Q: int = 1024, k: int = 64, centers: int = 4096,
               device="cpu", fp8_queries: bool = False) -> Workload:
    """E4M3 keys with an fp32 per-row scale, quantised from normalised Gaussian-mixture rows; bf16 queries, or
    (fp8_queries) the same queries quantised to E4M3 row by row like the keys."""
    g = _gen(seed, device)
    center_rows = _unit_rows(torch.randn(centers, d, generator=g, device=device))
    keys = torch.empty(N, d, dtype=torch.float8_e4m3fn, device=device)
    scale = torch.empty(N, dtype=torch.float32, device=device)
    chunk = 1 << 17
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        kf, _ = clustered_keys(e - s, d, centers, 0.1, g, device, center_rows=center_rows)
        keys[s:e], scale[s:e] = quantize_e4m3_rows(kf)
    v = torch.randint(0, N, (Q,), generator=g, device=device)
    base = keys[v].float() * scale[v][:, None]
    queries = perturbed_queries(base, 0.05, g).to(torch.bfloat16)
    if fp8_queries:
        queries = quantize_e4m3_rows(queries.float())[0]
    return Workload("compressed-q8" if fp8_queries else "compressed", keys, queries, k, scale=scale, seed=seed)


def grouped(seed: int = 0, C: int = 64, mean_size: int = 300, d: int = 256, spread: float = 0.03, Q: int = 8, k: int = 16,
            dtype=torch.bfloat16, device="cpu", p_tag: Optional[float] = None):
    """A knowledge base whose rows are grouped by cluster, for two-stage retrieval: C unit centres, cluster c holds
    size_c rows = normalised (centre_c + spread * N(0,1) per coordinate), sizes uniform in [mean/4, 7 mean/4] with one
    empty cluster; queries are perturbed copies of stored rows.  Returns (Workload, centroids [C, d] in `dtype` (fp8:
    bf16), cluster_offsets int64 [C + 1])."""
    g = _gen(seed, device)
    centres = _unit_rows(torch.randn(C, d, generator=g, device=device))
    sizes = torch.randint(max(mean_size // 4, 1), max(7 * mean_size // 4, 2), (C,), generator=g, device=device)
    if C > 2:
        sizes[C // 3] = 0
    offsets = torch.zeros(C + 1, dtype=torch.int64, device=device)
    offsets[1:] = torch.cumsum(sizes, 0)
    N = int(offsets[-1])
    owner = torch.repeat_interleave(torch.arange(C, device=device), sizes)
    rows = _unit_rows(centres[owner] + spread * torch.randn(N, d, generator=g, device=device))
    v = torch.randint(0, N, (Q,), generator=g, device=device)
    queries = perturbed_queries(rows[v], spread / 2, g)
    tags = qmask = scale = None
    if p_tag is not None:
        tags, qmask = random_bits64(N, p_tag, g, device), random_bits64(Q, p_tag, g, device)
    if dtype == torch.float8_e4m3fn:
        keys, scale = quantize_e4m3_rows(rows)
        queries, cent = queries.to(torch.bfloat16), centres.to(torch.bfloat16)
    else:
        keys, queries, cent = rows.to(dtype), queries.to(dtype), centres.to(dtype)
    return Workload("grouped", keys, queries, k, scale=scale, tags=tags, qmask=qmask, seed=seed), cent, offsets


def growing_round(seed: int, round_index: int, n_new: int, d: int, Q: int, center_rows: torch.Tensor,
                  device="cpu", p_tag: float = 0.3):
    """One append round of the growing workload: n_new clustered bf16 rows + tags, and Q masked queries.

    Queries are perturbed copies of rows of the new block (the caller may mix in older rows).
    """
    g = _gen(seed * 1000003 + round_index + 1, device)
    kf, _ = clustered_keys(n_new, d, center_rows.shape[0], 0.1, g, device, center_rows=center_rows)
    rows = kf.to(torch.bfloat16)
    tags = random_bits64(n_new, p_tag, g, device)
    v = torch.randint(0, n_new, (Q,), generator=g, device=device)
    queries = perturbed_queries(rows[v].float(), 0.05, g).to(torch.bfloat16)
    qmask = random_bits64(Q, p_tag, g, device)
    return rows, tags, queries, qmask


def growing_base(seed: int = 0, N0: int = 1 << 20, d: int = 1024, centers: int = 1024, device="cpu",
                 p_tag: float = 0.3):
    """Initial state of the growing workload: N0 clustered bf16 rows + tags, and the cluster centres."""
    g = _gen(seed, device)
    kf, center_rows = clustered_keys(N0, d, centers, 0.1, g, device)
    keys = kf.to(torch.bfloat16)
    del kf
    tags = random_bits64(N0, p_tag, g, device)
    return keys, tags, center_rows


# ---- stored bits as numpy arrays (what the CPU checker consumes) -----------------------------

def key_bits(t: torch.Tensor) -> np.ndarray:
    """The stored bits of a float32 / bfloat16 / float8_e4m3fn tensor as float32 / uint16 / uint8."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).numpy()
    raise TypeError(t.dtype)


def word_bits(t: Optional[torch.Tensor]) -> Optional[np.ndarray]:
    """int64 bit patterns -> uint64."""
    if t is None:
        return None
    return t.detach().cpu().contiguous().numpy().view(np.uint64)


def checksum(*tensors) -> int:
    """64-bit checksum of the generated bits (recorded with results; RNG streams differ across devices)."""
    import hashlib

    h = hashlib.blake2b(digest_size=8)
    for t in tensors:
        if t is None:
            continue
        h.update(t.detach().cpu().contiguous().view(torch.uint8).numpy().tobytes())
    return int.from_bytes(h.digest(), "little")
