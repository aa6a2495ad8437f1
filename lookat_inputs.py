"""Seeded synthetic inputs for LOOKAT tests and benchmarks.

This module only DRAWS data (Gaussian arrays, permutations, slicing).  It holds
none of the method's arithmetic: no distances, no argmin, no tables, no softmax.
The CPU oracle and the HIP library are both fed from the arrays made here.

Recipe (stands in for the GPT-2 / Llama key-value caches the paper measures on,
which are not available offline):
  * keys: per head h a fixed mixing matrix A_h [r, d_k] ~ N(0,1); every key is
    z A_h + noise * eps with z ~ N(0,1)^r and eps ~ N(0,1)^{d_k}  (low intrinsic
    dimension, r = 8 for d_k = 64 and r = 16 for d_k = 128, noise = 0.1);
  * calibration keys: separate draws from the same per-head generator;
  * values: fp16 N(0,1);  queries: N(0,1)/8 (fp16 unless stated);
  * codebook initialisation: for every head the first K rows of a seeded
    permutation of that head's calibration keys, cut into m sub-vectors.
    (Lloyd iterations are NOT done here: they are the method's arithmetic.)
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 0x10AC47


@dataclass(frozen=True)
class Config:
    name: str
    B: int          # batch
    H: int          # heads
    L: int          # cached keys per (b,h)
    T: int          # queries per (b,h): 1 for decode
    d_k: int
    m: int
    rank: int
    n_calib: int    # calibration keys per head
    layers: int = 1
    K: int = 256
    noise: float = 0.1
    key_dtype: str = "float32"
    q_dtype: str = "float16"
    index: int = 0

    @property
    def d_sub(self) -> int:
        return self.d_k // self.m

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


# The five workload shapes this build is specified on.
CONFIGS = {
    "C0": Config("C0", B=1, H=1, L=256, T=1, d_k=64, m=4, rank=8, n_calib=256, q_dtype="float32", index=0),
    "C1": Config("C1", B=1, H=12, L=1024, T=1, d_k=64, m=2, rank=8, n_calib=4096, layers=12, index=1),
    "C2": Config("C2", B=32, H=12, L=1024, T=1, d_k=64, m=4, rank=8, n_calib=4096, layers=12, index=2),
    "C3": Config("C3", B=8, H=32, L=32768, T=1, d_k=128, m=8, rank=16, n_calib=16384, index=3),
    "C4": Config("C4", B=4, H=32, L=2048, T=2048, d_k=128, m=16, rank=16, n_calib=4096,
                 key_dtype="float16", index=4),
}


def shrink(cfg: Config, **kw) -> Config:
    """Same recipe at a smaller shape (for cases the oracle must finish in seconds)."""
    return replace(cfg, **kw)


def mixing_matrices(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    return rng.standard_normal((cfg.H, cfg.rank, cfg.d_k)).astype(np.float32)


def lowrank_keys(A: np.ndarray, lead: tuple, n: int, noise: float, rng: np.random.Generator) -> np.ndarray:
    """A [H,r,d_k] -> keys [*lead, H, n, d_k] fp32 = z A_h + noise * eps."""
    H, r, d_k = A.shape
    z = rng.standard_normal(lead + (H, n, r)).astype(np.float32)
    eps = rng.standard_normal(lead + (H, n, d_k)).astype(np.float32)
    return (np.einsum("...hnr,hrd->...hnd", z, A) + np.float32(noise) * eps).astype(np.float32)


def codebook_init(calib: np.ndarray, m: int, K: int, rng: np.random.Generator) -> np.ndarray:
    """calib [H,Nc,d_k] -> initial codebooks [H,m,K,d_sub]: K distinct calibration rows per head."""
    H, Nc, d_k = calib.shape
    d_sub = d_k // m
    out = np.empty((H, m, K, d_sub), dtype=np.float32)
    for h in range(H):
        rows = rng.permutation(Nc)[:K]
        out[h] = calib[h, rows].reshape(K, m, d_sub).transpose(1, 0, 2)
    return out


def make_case(cfg: Config, seed: int | None = None, calib_is_cache: bool = False) -> dict:
    """All host arrays of one workload.  Keys 'A','keys','calib','cb_init','values','q'.

    keys   [B,H,L,d_k] (cfg.key_dtype)     calib [H,n_calib,d_k] fp32
    values [B,H,L,d_k] fp16                q     [B,H,T,d_k] (cfg.q_dtype)
    With calib_is_cache (config C0: "initialised from the seeded keys") the
    calibration set is the cache of batch 0 itself.
    """
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    A = mixing_matrices(cfg, rng)
    keys = lowrank_keys(A, (cfg.B,), cfg.L, cfg.noise, rng)
    if calib_is_cache:
        calib = np.ascontiguousarray(keys[0][:, : cfg.n_calib])
    else:
        calib = lowrank_keys(A, (), cfg.n_calib, cfg.noise, rng)
    cb_init = codebook_init(calib, cfg.m, cfg.K, rng)
    values = rng.standard_normal((cfg.B, cfg.H, cfg.L, cfg.d_k)).astype(np.float16)
    q = (rng.standard_normal((cfg.B, cfg.H, cfg.T, cfg.d_k)) / 8.0).astype(cfg.q_dtype)
    return {"cfg": cfg, "A": A, "keys": keys.astype(cfg.key_dtype), "calib": calib,
            "cb_init": cb_init, "values": values, "q": q}


# ---- device-side generation for the full-size workloads ---------------------
# Same recipe drawn with torch's seeded generator directly in HBM (the large
# configurations are several GB; drawing them on the host and copying would
# dominate the run).  Streams differ from the numpy ones; each consumer reads
# the arrays it is given, never re-draws them.

def torch_generator(cfg: Config, device, salt: int = 0):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed * 1000003 + salt)
    return g


def torch_lowrank_keys(A, lead: tuple, n: int, noise: float, gen, dtype, chunk: int = 1 << 20):
    """A [H,r,d_k] device fp32 -> keys [*lead,H,n,d_k] of `dtype`, drawn in chunks."""
    import torch
    H, r, d_k = A.shape
    out = torch.empty(lead + (H, n, d_k), dtype=dtype, device=A.device)
    flat = out.view(-1, H, n, d_k)
    rows = max(1, chunk // d_k)
    for b in range(flat.shape[0]):
        for h in range(H):
            for s in range(0, n, rows):
                e = min(n, s + rows)
                z = torch.randn((e - s, r), generator=gen, device=A.device, dtype=torch.float32)
                eps = torch.randn((e - s, d_k), generator=gen, device=A.device, dtype=torch.float32)
                # z A_h as broadcast-multiply + reduce: plain elementwise kernels, no BLAS call
                mix = (z.unsqueeze(2) * A[h].unsqueeze(0)).sum(dim=1)
                flat[b, h, s:e] = (mix + noise * eps).to(dtype)
    return out


def torch_case(cfg: Config, device, layer: int = 0) -> dict:
    """Device tensors of one layer of a workload: 'A','keys','calib','cb_init','values','q'."""
    import torch
    gen = torch_generator(cfg, device, salt=layer)
    kd = getattr(torch, cfg.key_dtype)
    qd = getattr(torch, cfg.q_dtype)
    A = torch.randn((cfg.H, cfg.rank, cfg.d_k), generator=gen, device=device, dtype=torch.float32)
    keys = torch_lowrank_keys(A, (cfg.B,), cfg.L, cfg.noise, gen, kd)
    calib = torch_lowrank_keys(A, (), cfg.n_calib, cfg.noise, gen, torch.float32)
    d_sub = cfg.d_sub
    cb_init = torch.empty((cfg.H, cfg.m, cfg.K, d_sub), device=device, dtype=torch.float32)
    for h in range(cfg.H):
        rows = torch.randperm(cfg.n_calib, generator=gen, device=device)[: cfg.K]
        cb_init[h] = calib[h, rows].reshape(cfg.K, cfg.m, d_sub).permute(1, 0, 2)
    values = torch.empty((cfg.B, cfg.H, cfg.L, cfg.d_k), device=device, dtype=torch.float16)
    for b in range(cfg.B):
        values[b] = torch.randn((cfg.H, cfg.L, cfg.d_k), generator=gen, device=device,
                                dtype=torch.float32).to(torch.float16)
    q = (torch.randn((cfg.B, cfg.H, cfg.T, cfg.d_k), generator=gen, device=device,
                     dtype=torch.float32) / 8.0).to(qd)
    return {"cfg": cfg, "A": A, "keys": keys, "calib": calib, "cb_init": cb_init, "values": values, "q": q}
