"""Seeded synthetic embedding-lookup payloads (the five benchmark workloads).

Shapes and distributions borrow from what the paper describes of its Criteo
batches (Section IV-A: 26 categorical tables; Section III-C: table sizes from
under ten to over a million rows; Section III-B: skewed queries, values between
Gaussian and uniform).  No dataset record is used or reproduced.

This module holds input generation only: none of the compressor's arithmetic
lives here.  It serves the CPU oracle and the HIP library alike.

Seeds: 20240704 + 1000*cfg + table (+ iteration for workload 5).
Zipf over a finite table: weights k^-alpha for k = 1..rows, float64 cumulative
sum, inverse CDF by searchsorted; rank k maps to row k-1.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20240704


def seed_for(cfg: int, table: int = 0, iteration: int = 0) -> int:
    return BASE_SEED + 1000 * cfg + table + 1_000_000 * iteration


def sha256(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


# ----------------------------------------------------------------------------
# numpy generators (workloads 1 and 2)
# ----------------------------------------------------------------------------
def zipf_indices_np(rng: np.random.Generator, rows: int, alpha: float, size) -> np.ndarray:
    w = np.arange(1, rows + 1, dtype=np.float64) ** (-alpha)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = rng.random(size)
    return np.minimum(np.searchsorted(cdf, u, side="left"), rows - 1).astype(np.int64)


@dataclass
class Workload:
    name: str
    payload: object            # [T, B, D] array (numpy) or tensor (torch)
    meta: dict = field(default_factory=dict)


def workload1() -> Workload:
    """1 table 1000x16 fp32 N(0, sigma=0.01); 256 single-hot Zipf(1.1) lookups; abs eb 1e-3."""
    rng = np.random.default_rng(seed_for(1, 0))
    table = (rng.standard_normal((1000, 16)) * 0.01).astype(np.float32)
    idx = zipf_indices_np(rng, 1000, 1.1, 256)
    return Workload("cfg1", table[idx][None].copy(), {"eb": 1e-3, "mode": "abs-explicit"})


def workload2(T: int = 26, B: int = 4096, D: int = 64) -> Workload:
    """26 tables, rows log-uniform in [1e3,1e6], D=64, U(+-1/sqrt(rows)); B=4096 Zipf(1.05)."""
    meta_rng = np.random.default_rng(seed_for(2, 999))
    rows = np.round(10.0 ** meta_rng.uniform(3.0, 6.0, T)).astype(np.int64)
    out = np.empty((T, B, D), np.float32)
    for t in range(T):
        rng = np.random.default_rng(seed_for(2, t))
        idx = zipf_indices_np(rng, int(rows[t]), 1.05, B)
        uniq, inv = np.unique(idx, return_inverse=True)
        # only looked-up rows are materialised; each row's values depend on (table seed, row id) alone
        a = 1.0 / np.sqrt(float(rows[t]))
        vals = np.empty((uniq.size, D), np.float32)
        for j, r in enumerate(uniq):
            rr = np.random.default_rng([seed_for(2, t), int(r)])
            vals[j] = rr.uniform(-a, a, D).astype(np.float32)
        out[t] = vals[inv]
    return Workload("cfg2", out, {"rows": rows, "global_eb": 3e-3, "alpha": 5.0 / 3.0, "beta": 3.0,
                                  "eb_min": 1e-4, "eb_max": 1e-2, "mode": "abs"})


# ----------------------------------------------------------------------------
# torch generators (workloads 3-5; device-selectable, the CPU oracle gets a host copy)
# ----------------------------------------------------------------------------
def _torch():
    import torch
    return torch


def zipf_indices_t(gen, rows: int, alpha: float, size, device):
    torch = _torch()
    w = torch.arange(1, rows + 1, dtype=torch.float64, device=device) ** (-alpha)
    cdf = torch.cumsum(w, 0)
    cdf = cdf / cdf[-1]
    u = torch.rand(size, dtype=torch.float64, device=device, generator=gen)
    return torch.clamp(torch.searchsorted(cdf, u), max=rows - 1)


def _gen(device, seed):
    torch = _torch()
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def workload3(T: int = 128, B: int = 8192, D: int = 128, rows: int = 100_000, device="cpu",
              dtype=None) -> Workload:
    """One rank's all-to-all share: N(0, sigma_t), sigma_t log-uniform in [1e-3,1e-1]; Zipf(1.05)."""
    torch = _torch()
    meta_rng = np.random.default_rng(seed_for(3, 999))
    sigma = 10.0 ** meta_rng.uniform(-3.0, -1.0, T)
    out = torch.empty((T, B, D), dtype=torch.float32, device=device)
    for t in range(T):
        g = _gen(device, seed_for(3, t))
        table = torch.randn((rows, D), dtype=torch.float32, device=device, generator=g) * float(sigma[t])
        idx = zipf_indices_t(g, rows, 1.05, (B,), device)
        out[t] = table[idx]
        del table
    if dtype is not None:
        out = out.to(dtype)
    return Workload("cfg3", out, {"sigma": sigma, "global_eb": 0.03, "alpha": 5.0 / 3.0, "beta": 3.0,
                                  "mode": "range-rel"})


def workload4(T: int = 64, B: int = 16384, D: int = 128, rows: int = 100_000, max_pool: int = 20,
              device="cpu") -> Workload:
    """Multi-hot sum-pooled lookups of Laplace(0, 0.02) rows; pooling factor U{1..20}; Zipf(1.2).

    payload is fp32; ``meta['payload_f16']`` is the same sums rounded to fp16."""
    torch = _torch()
    out = torch.empty((T, B, D), dtype=torch.float32, device=device)
    for t in range(T):
        g = _gen(device, seed_for(4, t))
        u = torch.rand((rows, D), dtype=torch.float32, device=device, generator=g) - 0.5
        table = -0.02 * torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.49999997))
        L = torch.randint(1, max_pool + 1, (B,), device=device, generator=g)
        idx = zipf_indices_t(g, rows, 1.2, (B, max_pool), device)
        acc = torch.zeros((B, D), dtype=torch.float32, device=device)
        for j in range(max_pool):  # fixed summation order
            acc += table[idx[:, j]] * (L > j).to(torch.float32)[:, None]
        out[t] = acc
        del table, u
    return Workload("cfg4", out, {"payload_f16": out.to(torch.float16), "global_eb": 0.03, "alpha": 5.0 / 3.0,
                                  "beta": 3.0, "rel_floor_f16": 2.0 ** -10, "mode": "range-rel"})


class Workload5:
    """Iteration-wise run at workload-3 shapes.

    Tables are stored at their iteration-0 scale; iteration i's forward payload is
    gather(table) * float32(0.99**i) (the drift), after 1 % of the rows were redrawn
    (at stored scale, i.e. N(0, sigma_t * 0.99**i) in payload units) and with fresh
    Zipf(1.05) lookups.  The backward payload is iid N(0, 1e-4) of the same shape."""

    def __init__(self, T: int = 128, B: int = 8192, D: int = 128, rows: int = 100_000, device="cpu"):
        torch = _torch()
        self.T, self.B, self.D, self.rows, self.device = T, B, D, rows, device
        meta_rng = np.random.default_rng(seed_for(5, 999))
        self.sigma = 10.0 ** meta_rng.uniform(-3.0, -1.0, T)
        self.tables = torch.empty((T, rows, D), dtype=torch.float32, device=device)
        for t in range(T):
            g = _gen(device, seed_for(5, t))
            self.tables[t] = torch.randn((rows, D), dtype=torch.float32, device=device, generator=g) * float(
                self.sigma[t])
        self.iteration = -1
        self.meta = {"global_eb": 0.03, "alpha": 5.0 / 3.0, "beta": 3.0, "mode": "range-rel", "decay_mult0": 2.0,
                     "decay_steps": 5, "decay_len": 100}

    def step(self):
        """Advance one iteration; -> (forward payload, backward payload), both [T,B,D] fp32."""
        torch = _torch()
        self.iteration += 1
        i = self.iteration
        T, B, D, rows, dev = self.T, self.B, self.D, self.rows, self.device
        fwd = torch.empty((T, B, D), dtype=torch.float32, device=dev)
        scale = float(np.float32(0.99 ** i))
        n_new = max(1, rows // 100)
        for t in range(T):
            g = _gen(dev, seed_for(5, t, i + 1))
            if i > 0:
                which = torch.randint(0, rows, (n_new,), device=dev, generator=g)
                self.tables[t, which] = torch.randn((n_new, D), dtype=torch.float32, device=dev, generator=g) * float(
                    self.sigma[t])
            idx = zipf_indices_t(g, rows, 1.05, (B,), dev)
            fwd[t] = self.tables[t, idx] * scale
        gb = _gen(dev, seed_for(5, 998, i + 1))
        bwd = torch.randn((T, B, D), dtype=torch.float32, device=dev, generator=gb) * 1e-4
        return fwd, bwd
