"""Seeded synthetic inputs for the table-batched embedding path.

This module only *draws inputs*: table shapes, procedural initial weights, bag lengths, ids,
upstream gradients.  It holds none of the method's arithmetic (no pooling, no sorting, no
optimizer step) and is the one module that both the CPU oracle's tests and the HIP path's
tests/benchmark import.  Everything is a pure function of (config, seed, step, table), written
with torch ops only so that the same code runs on the host or on the device; large configs are
drawn directly in HBM because their tables (100-200 GB) cannot be staged through the host.

The five named configs stand in for the paper's private production workloads (hundreds of
embedding tables, Zipf-skewed categorical ids, thousands of samples per GPU; Section 4 of the
paper quotes 896-4096 samples per GPU and 0.5-1.7 TB of tables over 256-1024 GPUs).
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import torch

_M32 = 0xFFFFFFFF
_MIXMUL = 0x45D9F3B           # < 2**27, so (x < 2**32) * _MIXMUL stays below 2**59: no int64 overflow
_GOLD = 0x9E3779B1            # odd 32-bit constant used to spread the column index


# --------------------------------------------------------------------------------------
# counter-based integer hash (python-int and tensor flavours give identical values)
# --------------------------------------------------------------------------------------
def _mix32_int(x: int) -> int:
    x &= _M32
    x = ((x ^ (x >> 16)) * _MIXMUL) & _M32
    x = ((x ^ (x >> 16)) * _MIXMUL) & _M32
    return x ^ (x >> 16)


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """x: int64 tensor with values in [0, 2**32).  Returns the same range."""
    x = ((x ^ (x >> 16)) * _MIXMUL) & _M32
    x = ((x ^ (x >> 16)) * _MIXMUL) & _M32
    return x ^ (x >> 16)


def _stream_seed(seed: int, *parts: int) -> int:
    """Deterministic 62-bit seed for one (purpose, table, step, ...) random stream."""
    h = _mix32_int(seed * 1000003 + 0x5BD1E995)
    g = _mix32_int(seed * 7919 + 0x27D4EB2F)
    for p in parts:
        h = _mix32_int(h ^ _mix32_int(p + 0x165667B1))
        g = _mix32_int(g + _mix32_int(p * 31 + 0x85EBCA6B))
    return ((h << 30) ^ g) & ((1 << 62) - 1)


# --------------------------------------------------------------------------------------
# configs
# --------------------------------------------------------------------------------------
@dataclass
class Config:
    name: str
    rows: List[int]                 # R_t
    D: List[int]                    # D_t
    weight_dtype: str               # "f32" | "f16"
    B: int
    pooling: str                    # "sum" | "mean"
    length_dist: Tuple              # ("fixed", L) | ("poisson1", lam) | ("lognormal", mu, sigma, cap)
    id_dist: Tuple                  # ("uniform",) | ("zipf", s)
    lr: float = 0.01
    eps: float = 1e-8
    c: float = 1.0                  # the moment scaling factor of Algorithm 1
    seed: int = 0
    w_scale: float = 0.01           # weights ~ U(-w_scale, w_scale)

    @property
    def T(self) -> int:
        return len(self.rows)

    @property
    def sum_D(self) -> int:
        return int(sum(self.D))

    @property
    def total_rows(self) -> int:
        return int(sum(self.rows))

    @property
    def total_elems(self) -> int:
        return int(sum(r * d for r, d in zip(self.rows, self.D)))

    @property
    def torch_weight_dtype(self) -> torch.dtype:
        return torch.float32 if self.weight_dtype == "f32" else torch.float16

    @property
    def weight_bytes(self) -> int:
        return self.total_elems * (4 if self.weight_dtype == "f32" else 2)

    def D_offsets(self) -> List[int]:
        o = [0]
        for d in self.D:
            o.append(o[-1] + d)
        return o

    def row_base(self) -> List[int]:
        o = [0]
        for r in self.rows:
            o.append(o[-1] + r)
        return o

    def w_offsets(self) -> List[int]:
        o = [0]
        for r, d in zip(self.rows, self.D):
            o.append(o[-1] + r * d)
        return o

    def expected_L(self) -> float:
        k = self.length_dist[0]
        if k == "fixed":
            return float(self.length_dist[1])
        if k == "poisson1":
            return float(self.length_dist[1]) + 1.0
        if k == "lognormal":
            _, mu, sigma, cap = self.length_dist
            return min(float(cap), math.exp(mu + 0.5 * sigma * sigma))
        raise ValueError(k)


def _log_uniform_rows(seed: int, T: int, lo_exp: float, hi_exp: float) -> List[int]:
    g = torch.Generator(device="cpu")
    g.manual_seed(_stream_seed(seed, 101))
    u = torch.rand(T, generator=g, dtype=torch.float64)
    return [max(1, int(round(10.0 ** (lo_exp + (hi_exp - lo_exp) * float(x))))) for x in u]


def _choice(seed: int, purpose: int, T: int, values: Sequence[int], probs: Optional[Sequence[float]] = None) -> List[int]:
    g = torch.Generator(device="cpu")
    g.manual_seed(_stream_seed(seed, purpose))
    u = torch.rand(T, generator=g, dtype=torch.float64).tolist()
    if probs is None:
        probs = [1.0 / len(values)] * len(values)
    out = []
    for x in u:
        acc = 0.0
        pick = values[-1]
        for v, p in zip(values, probs):
            acc += p
            if x < acc:
                pick = v
                break
        out.append(pick)
    return out


def config(name: str, *, T: Optional[int] = None, B: Optional[int] = None, rows_scale: float = 1.0,
           seed: int = 0, c: float = 1.0, weight_dtype: Optional[str] = None,
           pooling: Optional[str] = None) -> Config:
    """One of the five benchmark workloads, optionally shrunk (fewer tables, smaller batch, rows scaled)
    for parity tests that a CPU oracle must finish in seconds.  Distributions are never changed."""
    name = name.upper()

    def sc(rows):
        return [max(4, int(round(r * rows_scale))) for r in rows]

    if name == "C1":
        t = T or 1
        cfg = Config("C1", sc([100_000] * t), [64] * t, "f32", B or 512, "sum", ("fixed", 20), ("uniform",))
    elif name == "C2":
        t = T or 26
        cfg = Config("C2", sc(_log_uniform_rows(seed, t, 3.0, 6.0)), [64] * t, "f32", B or 4096, "sum",
                     ("poisson1", 10.0), ("zipf", 1.05))
    elif name == "C3":
        t = T or 128
        cfg = Config("C3", sc(_log_uniform_rows(seed, t, 4.0, 7.0)), _choice(seed, 102, t, [64, 128, 256]), "f32",
                     B or 16384, "sum", ("poisson1", 20.0), ("zipf", 1.2))
    elif name == "C4":
        t = T or 256
        raw = _log_uniform_rows(seed, t, 5.0, 7.0)
        tot = float(sum(raw))
        target = 4.0e8 * t / 256.0
        rows = [max(1000, int(round(r * target / tot))) for r in raw]
        cfg = Config("C4", sc(rows), _choice(seed, 103, t, [128, 256], [0.25, 0.75]), "f16", B or 32768, "sum",
                     ("poisson1", 30.0), ("zipf", 1.1))
    elif name in ("C5", "C5I"):
        # C5: the big tables first; C5I: the same tables with the big ones spread evenly among the small ones
        t = T or 128
        nbig = max(1, t // 16)
        if name == "C5":
            big = [i < nbig for i in range(t)]
        else:
            big = [i % (t // nbig) == (t // nbig) // 2 and i // (t // nbig) < nbig for i in range(t)]
        rows = [50_000_000 if b else 100_000 for b in big]
        D = [128 if b else 32 for b in big]
        cfg = Config(name, sc(rows), D, "f32", B or 65536, "mean", ("lognormal", 2.0, 1.0, 500), ("zipf", 1.3))
    else:
        raise ValueError(f"unknown config {name!r}")
    cfg.seed = seed
    cfg.c = c
    if weight_dtype is not None:
        cfg.weight_dtype = weight_dtype
    if pooling is not None:
        cfg.pooling = pooling
    return cfg


# --------------------------------------------------------------------------------------
# procedural initial weights  w[t, r, j] ~ U(-w_scale, w_scale)
# --------------------------------------------------------------------------------------
def _table_key(cfg: Config, t: int) -> int:
    return _mix32_int(_mix32_int(cfg.seed * 2654435761 + 0x3C6EF372) ^ _mix32_int(t + 0x1B873593))


def weight_rows(cfg: Config, t: int, row_ids: torch.Tensor) -> torch.Tensor:
    """Initial values of rows `row_ids` (int64, any device) of table t, as float32 [n, D_t].
    Element (t, r, j) depends only on (seed, t, r, j), so any row can be re-derived anywhere."""
    D = cfg.D[t]
    dev = row_ids.device
    r = row_ids.to(torch.int64)
    hr = _mix32((r & _M32) ^ _table_key(cfg, t))
    hr = _mix32((hr + (r >> 32)) & _M32)
    jm = (torch.arange(D, dtype=torch.int64, device=dev) * _GOLD) & _M32
    he = _mix32((hr[:, None] + jm[None, :]) & _M32)
    u24 = he >> 8
    w = (u24 - 8388608).to(torch.float32) * (cfg.w_scale / 8388608.0)
    return w


def fill_weights(cfg: Config, flat: torch.Tensor, chunk_elems: int = 1 << 25) -> None:
    """Fill the flat weight buffer (tables concatenated, row-major) in place, in bounded chunks."""
    assert flat.numel() == cfg.total_elems and flat.dtype == cfg.torch_weight_dtype
    woff = cfg.w_offsets()
    for t in range(cfg.T):
        R, D = cfg.rows[t], cfg.D[t]
        view = flat[woff[t]:woff[t + 1]].view(R, D)
        step = max(1, chunk_elems // D)
        for r0 in range(0, R, step):
            r1 = min(R, r0 + step)
            ids = torch.arange(r0, r1, dtype=torch.int64, device=flat.device)
            view[r0:r1].copy_(weight_rows(cfg, t, ids))
        _drain(flat.device)


def state_rows(cfg: Config, keys: torch.Tensor, scale: float = 4.0) -> torch.Tensor:
    """Procedural positive second-moment start values for linearised row keys (float32), in (0, scale]."""
    k = keys.to(torch.int64)
    h = _mix32((k & _M32) ^ _mix32_int(cfg.seed + 0x2545F491))
    h = _mix32((h + (k >> 32)) & _M32)
    return ((h >> 8) + 1).to(torch.float32) * (scale / 16777216.0)


def fill_state(cfg: Config, state: torch.Tensor, kind: str = "zeros", chunk: int = 1 << 26) -> None:
    if kind == "zeros":
        state.zero_()
        return
    n = state.numel()
    for k0 in range(0, n, chunk):
        k1 = min(n, k0 + chunk)
        state[k0:k1].copy_(state_rows(cfg, torch.arange(k0, k1, dtype=torch.int64, device=state.device)))


# --------------------------------------------------------------------------------------
# bag lengths, ids, upstream gradient
# --------------------------------------------------------------------------------------
def _drain(device) -> None:
    """Keep the launch queue short: generation issues tens of thousands of small kernels, and a profiler that
    intercepts every dispatch has been seen to fall over when thousands of them are outstanding at once."""
    if torch.device(device).type == "cuda":
        torch.cuda.synchronize()


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _lengths(cfg: Config, g: torch.Generator, device) -> torch.Tensor:
    kind = cfg.length_dist[0]
    B = cfg.B
    if kind == "fixed":
        return torch.full((B,), int(cfg.length_dist[1]), dtype=torch.int64, device=device)
    if kind == "poisson1":
        lam = torch.full((B,), float(cfg.length_dist[1]), dtype=torch.float32, device=device)
        return torch.poisson(lam, generator=g).to(torch.int64) + 1
    if kind == "lognormal":
        _, mu, sigma, cap = cfg.length_dist
        z = torch.randn(B, generator=g, dtype=torch.float32, device=device)
        L = torch.round(torch.exp(mu + sigma * z)).to(torch.int64)
        return L.clamp_(1, int(cap))
    raise ValueError(kind)


def _coprime_multiplier(seed: int, R: int) -> Tuple[int, int]:
    if R <= 2:
        return 1, 0
    a = 1 + (seed % (R - 1))
    while math.gcd(a, R) != 1:
        a += 1
        if a >= R:
            a = 1
    b = (seed // 7) % R
    return a, b


class _IdSampler:
    """Per-table id sampler.  Zipf: exact bounded pmf p(k) ~ k**-s on ranks 1..R, sampled by inverse CDF;
    rank k is mapped to row (a*(k-1)+b) mod R with gcd(a,R)=1 so that hot rows are scattered."""

    def __init__(self, cfg: Config, t: int, device):
        self.R = cfg.rows[t]
        self.kind = cfg.id_dist[0]
        self.device = device
        if self.kind == "zipf":
            s = float(cfg.id_dist[1])
            k = torch.arange(1, self.R + 1, dtype=torch.float64, device=device)
            cdf = torch.cumsum(k.pow_(-s), 0)
            self.cdf = cdf / cdf[-1]
            self.a, self.b = _coprime_multiplier(_stream_seed(cfg.seed, 104, t), self.R)

    def draw(self, n: int, g: torch.Generator) -> torch.Tensor:
        if n == 0:
            return torch.empty(0, dtype=torch.int64, device=self.device)
        if self.kind == "uniform":
            return torch.randint(0, self.R, (n,), generator=g, dtype=torch.int64, device=self.device)
        u = torch.rand(n, generator=g, dtype=torch.float64, device=self.device)
        rank = torch.searchsorted(self.cdf, u).clamp_(max=self.R - 1)
        return (rank * self.a + self.b) % self.R


def make_batches(cfg: Config, steps: Sequence[int], device="cpu") -> List[Tuple[torch.Tensor, torch.Tensor]]:
    """[(indices int64 [nnz], offsets int64 [T*B+1])] for each requested step number.
    Layout: table-major CSR, bag (t, b) owns indices[offsets[t*B+b] : offsets[t*B+b+1]]; ids are table-local."""
    per_step_len: List[List[torch.Tensor]] = [[] for _ in steps]
    per_step_ids: List[List[torch.Tensor]] = [[] for _ in steps]
    for t in range(cfg.T):
        sampler = _IdSampler(cfg, t, device)
        for k, step in enumerate(steps):
            g = _gen(device, _stream_seed(cfg.seed, 105, t, step))
            L = _lengths(cfg, g, device)
            n = int(L.sum().item())
            per_step_len[k].append(L)
            per_step_ids[k].append(sampler.draw(n, g))
        del sampler
        _drain(device)
    out = []
    for k in range(len(steps)):
        L = torch.cat(per_step_len[k])
        offsets = torch.zeros(L.numel() + 1, dtype=torch.int64, device=device)
        torch.cumsum(L, 0, out=offsets[1:])
        out.append((torch.cat(per_step_ids[k]), offsets))
    return out


def make_batch(cfg: Config, step: int = 0, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    return make_batches(cfg, [step], device)[0]


def make_grad_out(cfg: Config, step: int = 0, device="cpu") -> torch.Tensor:
    """Upstream gradient of the pooled activations, N(0,1), float32 [B, sum(D)]."""
    g = _gen(device, _stream_seed(cfg.seed, 106, step))
    return torch.randn(cfg.B, cfg.sum_D, generator=g, dtype=torch.float32, device=device)


def as_sequence(cfg: Config, indices: torch.Tensor, offsets: torch.Tensor):
    """The same ids read as a non-pooled (sequence) feature: table t owns positions offsets[t*B] .. offsets[(t+1)*B].
    Returns (indices, table_offsets [T+1], number of output elements sum_t n_t * D_t)."""
    toff = offsets[:: cfg.B].contiguous()
    n_t = (toff[1:] - toff[:-1]).tolist()
    return indices, toff, int(sum(n * d for n, d in zip(n_t, cfg.D)))


def make_grad_seq(cfg: Config, total_elems: int, step: int = 0, device="cpu") -> torch.Tensor:
    """Upstream gradient of a non-pooled lookup, N(0,1), float32, flat (one [n_t, D_t] block per table)."""
    g = _gen(device, _stream_seed(cfg.seed, 107, step))
    return torch.randn(max(1, total_elems), generator=g, dtype=torch.float32, device=device)[:total_elems]


def describe(cfg: Config) -> str:
    return (f"{cfg.name}: T={cfg.T} rows={cfg.total_rows:,} sumD={cfg.sum_D} {cfg.weight_dtype} "
            f"weights={cfg.weight_bytes / 1e9:.2f}GB B={cfg.B} E[L]={cfg.expected_L():.1f} "
            f"ids={cfg.id_dist} pooling={cfg.pooling}")
