"""Seeded synthetic KV-cache workloads (inputs only -- none of GEAR's arithmetic).

Both the CPU oracle's tests and the HIP path's tests/bench draw their inputs
from here, so the two sides always see identical bytes.  The value laws stand
in for real LLaMA/Mistral KV caches, which the paper measures on (Sec. 4) and
which are not available offline:

* Key entries are N(0,1) except a few fixed channels per KV head whose scale is
  drawn from U(lo, hi): the "fixed channels with very large magnitudes" the
  paper's background section attributes to Key caches.
* Value entries are Student-t with nu degrees of freedom (heavy-tailed,
  per-token outliers).
* Queries are N(0,1).

Everything is rounded to fp16 (round-to-nearest-even).  Generation runs in
torch on whichever device is asked for; a CPU tensor and a GPU tensor of the
same seed are different draws, so a test always generates once and hands the
same tensor (or a host copy of a slice of it) to both sides.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import torch

D_HEAD = 128


@dataclass(frozen=True)
class Workload:
    """One row of the benchmark's config list (shapes + hyper-parameters)."""
    name: str
    B: int                 # batch
    H_kv: int              # KV heads
    H_q: int               # query heads (multiple of H_kv)
    n: int                 # prefill tokens
    bits: int              # b
    group: int             # g
    outlier_ppm: int       # s as parts per million of a vector (2 % = 20000)
    rank: int              # r for the prefill segment
    rank_chunk: int        # r for each flushed buffer chunk
    n_b: int               # streaming-buffer capacity
    steps: int             # decode steps the config asks for
    iters: int = 3         # power-iteration rounds L
    k_out_channels: int = 4
    k_out_scale: Tuple[float, float] = (10.0, 20.0)
    v_nu: int = 4
    seed: int = 0
    d_h: int = D_HEAD
    v_per_head: bool = False   # Filter_s of the Values per head (group = 0 selects the per-vector grouping)
    lowrank_recent_pct: int = 100   # low-rank term on this share of the prefill tokens, the most recent ones


# The five configurations of the benchmark definition (index = seed base).
CONFIGS = [
    Workload("c0_tiny", B=1, H_kv=32, H_q=32, n=512, bits=4, group=64, outlier_ppm=20000,
             rank=4, rank_chunk=2, n_b=20, steps=1, seed=0),
    Workload("c1_llama2_7b", B=16, H_kv=32, H_q=32, n=4096, bits=2, group=64, outlier_ppm=20000,
             rank=4, rank_chunk=2, n_b=20, steps=256, seed=1),
    Workload("c2_llama2_13b", B=32, H_kv=40, H_q=40, n=2048, bits=4, group=128, outlier_ppm=20000,
             rank=8, rank_chunk=2, n_b=20, steps=128, k_out_channels=6, k_out_scale=(8.0, 25.0),
             v_nu=3, seed=2),
    Workload("c3_long", B=1, H_kv=32, H_q=32, n=32768, bits=2, group=128, outlier_ppm=10000,
             rank=8, rank_chunk=2, n_b=64, steps=64, seed=3),
    Workload("c4_llama3_8b_gqa", B=64, H_kv=8, H_q=32, n=8192, bits=2, group=64, outlier_ppm=20000,
             rank=4, rank_chunk=2, n_b=20, steps=128, seed=4),
    Workload("c4L_llama3_8b_gqa_gearl", B=64, H_kv=8, H_q=32, n=8192, bits=2, group=64, outlier_ppm=0,
             rank=4, rank_chunk=2, n_b=20, steps=128, seed=4),
]


# Variants of the follow-up scope, measured beside the five configurations: the paper's 4-bit backbone
# (per-vector groups, "KCVT") on the 13B layer shape, and the per-head Value Filter on the 7B layer shape.
VARIANTS = [
    Workload("c2_kcvt_4bit", B=32, H_kv=40, H_q=40, n=2048, bits=4, group=0, outlier_ppm=20000,
             rank=4, rank_chunk=2, n_b=20, steps=128, k_out_channels=6, k_out_scale=(8.0, 25.0), v_nu=3, seed=2),
    Workload("c1_v_filter_per_head", B=16, H_kv=32, H_q=32, n=4096, bits=2, group=64, outlier_ppm=20000,
             rank=4, rank_chunk=2, n_b=20, steps=256, seed=1, v_per_head=True),
    # the ablations on where the error reduction is applied: prefill tokens only (GEAR-L, flushed buffers with
    # rank 0), and the most recent quarter of the prefill tokens only
    Workload("c1_gearl_prefill_only", B=16, H_kv=32, H_q=32, n=4096, bits=2, group=64, outlier_ppm=0,
             rank=4, rank_chunk=0, n_b=20, steps=256, seed=1),
    Workload("c1_gearl_recent_25pct", B=16, H_kv=32, H_q=32, n=4096, bits=2, group=64, outlier_ppm=0,
             rank=4, rank_chunk=2, n_b=20, steps=256, seed=1, lowrank_recent_pct=25),
]


def _gen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + stream * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    return g


def key_channel_scales(w: Workload, device="cpu") -> torch.Tensor:
    """sigma[h, c]: 1 everywhere except k_out_channels channels per head."""
    g = _gen(w.seed, 3, "cpu")
    sig = torch.ones(w.H_kv, w.d_h, dtype=torch.float32)
    lo, hi = w.k_out_scale
    for h in range(w.H_kv):
        ch = torch.randperm(w.d_h, generator=g)[: w.k_out_channels]
        sig[h, ch] = lo + (hi - lo) * torch.rand(w.k_out_channels, generator=g)
    return sig.to(device)


def make_keys(w: Workload, n: int, stream: int, device="cpu", B: Optional[int] = None) -> torch.Tensor:
    """fp16 [B, H_kv, n, d_h]; `stream` separates prefill (0) from decode tokens."""
    B = w.B if B is None else B
    g = _gen(w.seed, 10 + stream, device)
    sig = key_channel_scales(w, device)
    out = torch.empty(B, w.H_kv, n, w.d_h, dtype=torch.float16, device=device)
    for b in range(B):      # per batch element keeps the fp32 temporary small
        z = torch.randn(w.H_kv, n, w.d_h, generator=g, device=device, dtype=torch.float32)
        out[b] = (z * sig[:, None, :]).to(torch.float16)
    return out


def make_values(w: Workload, n: int, stream: int, device="cpu", B: Optional[int] = None) -> torch.Tensor:
    """fp16 [B, H_kv, n, d_h], Student-t(nu) = z / sqrt(chi2_nu / nu)."""
    B = w.B if B is None else B
    g = _gen(w.seed, 20 + stream, device)
    out = torch.empty(B, w.H_kv, n, w.d_h, dtype=torch.float16, device=device)
    for b in range(B):
        z = torch.randn(w.H_kv, n, w.d_h, generator=g, device=device, dtype=torch.float32)
        chi = torch.zeros_like(z)
        for _ in range(w.v_nu):
            chi += torch.randn(w.H_kv, n, w.d_h, generator=g, device=device, dtype=torch.float32) ** 2
        out[b] = (z / torch.sqrt(chi / w.v_nu)).clamp_(-6.0e4, 6.0e4).to(torch.float16)
    return out


def make_queries(w: Workload, stream: int, device="cpu", B: Optional[int] = None) -> torch.Tensor:
    """fp16 [B, H_q, 1, d_h]."""
    B = w.B if B is None else B
    g = _gen(w.seed, 30 + stream, device)
    return torch.randn(B, w.H_q, 1, w.d_h, generator=g, device=device, dtype=torch.float32).to(torch.float16)


def make_init_B(w: Workload, rank: int, stream: int, device="cpu", B: Optional[int] = None) -> torch.Tensor:
    """Power-iteration start B0: fp32 [2 (K,V), B, H_kv, d_h, rank], i.i.d. U(-1,1)
    on a 24-bit grid (exactly representable in fp32)."""
    B = w.B if B is None else B
    g = _gen(w.seed, 40 + stream, "cpu")
    k = torch.randint(0, 1 << 24, (2, B, w.H_kv, w.d_h, max(rank, 1)), generator=g, dtype=torch.int64)
    b0 = (k.to(torch.float64) / float(1 << 23) - 1.0).to(torch.float32)
    return b0[..., :rank].contiguous().to(device)


def make_init_B_hashed(seed: int, B: int, H_kv: int, rank: int, device="cpu", d_h: int = D_HEAD) -> torch.Tensor:
    """The start array the library draws itself when it is given a seed instead of an array
    (include/gear.h, gear_compress): fp32 [2, B, H_kv, d_h, rank], entry i (row-major) =
    ((z >> 40) - 2^23) / 2^23, z = mix(seed + (i + 1) * 0x9E3779B97F4A7C15) with the SplitMix64
    finalizer.  Integers only, so this mirror gives the same floats bit for bit; handing it to the
    oracle (and to the library as an explicit array) is how the seeded path is checked."""
    import numpy as np
    n = 2 * B * H_kv * d_h * max(rank, 1)
    with np.errstate(over="ignore"):
        z = np.uint64(seed) + np.uint64(0x9E3779B97F4A7C15) * (np.arange(n, dtype=np.uint64) + np.uint64(1))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    k = (z >> np.uint64(40)).astype(np.int64) - (1 << 23)
    b0 = (k.astype(np.float64) / float(1 << 23)).astype(np.float32).reshape(2, B, H_kv, d_h, max(rank, 1))
    return torch.from_numpy(b0[..., :rank].copy()).to(device)
