"""Seeded synthetic workloads for xKV SR decode.

Input generators only: random draws, an orthonormalisation for the recipe of
B, and the one rounding of generated values to the storage type.  None of the
method's arithmetic lives here, so both the CPU oracle's tests and the GPU
tests may use it.

Recipe (stands in for the factors a cross-layer SVD of a real model's KV cache
would give; shapes follow Llama-3.1-8B and Qwen2.5-7B):
  A^K, A^V  [batch][L][r]        iid N(0,1) * a_scale
  B^K_l, B^V_l [batch][G][r][d]  diag(sigma) Q, Q with orthonormal rows drawn
                                 independently per (sequence, layer, K/V),
                                 sigma_i = i^(-decay), i = 1..r
  q         [G][batch][H_q][d_h] iid N(0,1) * q_scale (one query set per layer)
Values are rounded once to the storage dtype (fp32 or bf16) at generation.
bf16 arrays are carried on the host as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    G: int          # layers per group (the paper's window size W)
    H_kv: int
    H_q: int
    d_h: int
    r_k: int
    r_v: int
    L: int
    k: int
    batch: int
    dtype: str      # "f32" or "bf16"
    n_groups: int = 1       # layer groups of the model shape (n_layers = n_groups * G)
    a_scale: float = 1.0
    sigma_decay: float = 1.0
    q_scale: float = 1.0

    @property
    def d(self) -> int:
        return self.H_kv * self.d_h

    @property
    def n_layers(self) -> int:
        return self.n_groups * self.G

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


def _inv_sqrt(x):
    return 1.0 / float(np.sqrt(x))


# The configurations named by the benchmark definition.
TINY = Workload("tiny_f32", G=2, H_kv=1, H_q=4, d_h=64, r_k=32, r_v=32, L=512, k=32, batch=1,
                dtype="f32", a_scale=1.0, sigma_decay=1.0, q_scale=1.0)
LLAMA_GROUP = Workload("llama31_8b_group_L32k_b1", G=4, H_kv=8, H_q=32, d_h=128, r_k=512, r_v=512,
                       L=32768, k=2048, batch=1, dtype="bf16", n_groups=1,
                       a_scale=_inv_sqrt(512), sigma_decay=0.8, q_scale=_inv_sqrt(128))
LLAMA_FULL = Workload("llama31_8b_32layers_L64k_b16", G=4, H_kv=8, H_q=32, d_h=128, r_k=512, r_v=512,
                      L=65536, k=4096, batch=16, dtype="bf16", n_groups=8,
                      a_scale=_inv_sqrt(512), sigma_decay=0.8, q_scale=_inv_sqrt(128))
QWEN = Workload("qwen25_7b_28layers_L128k_b4", G=4, H_kv=4, H_q=28, d_h=128, r_k=384, r_v=384,
                L=131072, k=4096, batch=4, dtype="bf16", n_groups=7,
                a_scale=_inv_sqrt(384), sigma_decay=1.0, q_scale=_inv_sqrt(128))

WORKLOADS = {w.name: w for w in (TINY, LLAMA_GROUP, LLAMA_FULL, QWEN)}


def llama_sweep_point(L: int, batch: int, r: int, k_frac: float) -> Workload:
    """One point of the Llama-shaped sweep (32 layers, G=4, d=1024, 32 query heads)."""
    k = max(1, int(round(L * k_frac)))
    return LLAMA_FULL.with_(name=f"llama_sweep_L{L}_b{batch}_r{r}_k{k}", L=L, batch=batch, r_k=r, r_v=r, k=k,
                            a_scale=_inv_sqrt(r))


# ---------------------------------------------------------------- storage types
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns.  Finite inputs."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_to_f64(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


# ---------------------------------------------------------------- host generator
def _orthonormal_rows(rng: np.random.Generator, r: int, d: int) -> np.ndarray:
    """Q [r][d] with orthonormal rows: transpose of the Q factor of a d x r Gaussian."""
    if r > d:
        raise ValueError("orthonormal rows need r <= d")
    g = rng.standard_normal((d, r))
    qf, rf = np.linalg.qr(g)
    qf = qf * np.sign(np.diag(rf))[None, :]
    return np.ascontiguousarray(qf.T)


def make_B(rng: np.random.Generator, r: int, d: int, decay: float) -> np.ndarray:
    sigma = np.arange(1, r + 1, dtype=np.float64) ** (-decay)
    return sigma[:, None] * _orthonormal_rows(rng, r, d)


def make_case(w: Workload, seed: int) -> dict:
    """Host (numpy) inputs of one layer group for every sequence of the batch.

    Returns storage-dtype arrays: A_k [batch][L][r_k], A_v [batch][L][r_v],
    B_k [batch][G][r_k][d], B_v [batch][G][r_v][d], q [G][batch][H_q][d_h].
    """
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x584B56]))
    A_k = rng.standard_normal((w.batch, w.L, w.r_k)) * w.a_scale
    A_v = rng.standard_normal((w.batch, w.L, w.r_v)) * w.a_scale
    B_k = np.empty((w.batch, w.G, w.r_k, w.d))
    B_v = np.empty((w.batch, w.G, w.r_v, w.d))
    for b in range(w.batch):
        for l in range(w.G):
            B_k[b, l] = make_B(rng, w.r_k, w.d, w.sigma_decay)
            B_v[b, l] = make_B(rng, w.r_v, w.d, w.sigma_decay)
    q = rng.standard_normal((w.G, w.batch, w.H_q, w.d_h)) * w.q_scale
    return {
        "A_k": to_storage(A_k, w.dtype), "A_v": to_storage(A_v, w.dtype),
        "B_k": to_storage(B_k, w.dtype), "B_v": to_storage(B_v, w.dtype),
        "q": to_storage(q, w.dtype),
    }


def make_cache(rng: np.random.Generator, G: int, H_kv: int, d_h: int, L: int, decay: float, rank: int | None = None,
               dtype: str = "bf16") -> np.ndarray:
    """One sequence's uncompressed cache of a layer group, X [G][H_kv][L][d_h] in storage form (stands in for
    the keys or values a model would have written at prefill).

    Read as X_cat [L][n], n = G * H_kv * d_h (column l*H_kv*d_h + g*d_h + j), it is Z diag(i^-decay) Q with Z an
    L x rank Gaussian and Q rank orthonormal rows of length n: a power-law spectrum shared by the layers of the
    group, exactly of rank `rank` when rank < n (before rounding to the storage type).
    """
    n = G * H_kv * d_h
    rank = n if rank is None else rank
    z = rng.standard_normal((L, rank)) * (np.arange(1, rank + 1, dtype=np.float64) ** (-decay))[None, :]
    x_cat = z @ _orthonormal_rows(rng, rank, n)
    x = x_cat.reshape(L, G, H_kv, d_h).transpose(1, 2, 0, 3)
    return to_storage(np.ascontiguousarray(x), dtype)


def cache_as_matrix(x: np.ndarray) -> np.ndarray:
    """X [G][H_kv][L][d_h] (storage form) -> X_cat [L][n] in float64."""
    G, H_kv, L, d_h = x.shape
    return np.ascontiguousarray(storage_to_f64(x).transpose(2, 0, 1, 3).reshape(L, G * H_kv * d_h))


# ---------------------------------------------------------------- device generator
def torch_dtype(dtype: str):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def to_device(case: dict, dtype: str, device="cuda") -> dict:
    """Upload a host case; bf16 bit patterns are reinterpreted, not converted."""
    import torch
    out = {}
    for name, arr in case.items():
        t = torch.from_numpy(np.ascontiguousarray(arr))
        if dtype == "bf16":
            t = t.view(torch.int16).to(device).view(torch.bfloat16)
        else:
            t = t.to(device)
        out[name] = t
    return out


def to_host(t) -> np.ndarray:
    """Download a device tensor; bf16 comes back as uint16 bit patterns."""
    import torch
    t = t.detach()
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def make_group_device(w: Workload, seed: int, device="cuda", n_seq: int | None = None) -> dict:
    """One layer group's inputs generated on the device (for sizes too large for the host path).

    Same recipe as make_case, drawn from torch's device generator; deterministic for a given
    seed on a given software stack.  Any slice can be downloaded for the CPU oracle with to_host.
    """
    import torch
    n_seq = w.batch if n_seq is None else n_seq
    dt = torch_dtype(w.dtype)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)

    def normal(shape, scale):
        out = torch.empty(shape, dtype=dt, device=device)
        # generate in fp32 chunks along the first axis, round once to the storage type
        for b in range(shape[0]):
            out[b] = (torch.randn(shape[1:], generator=gen, device=device, dtype=torch.float32) * scale).to(dt)
        return out

    def orthonormal_columns(g):
        # Cholesky-QR, applied twice: Q = X R^-1 with R^T R = X^T X.  A d x r Gaussian is well conditioned, so two
        # rounds are orthonormal to fp32 rounding; far fewer kernel launches than a Householder QR.
        for _ in range(2):
            gram = g.transpose(1, 2) @ g
            chol = torch.linalg.cholesky(gram)                       # lower, gram = chol chol^T
            g = torch.linalg.solve_triangular(chol, g.transpose(1, 2), upper=False).transpose(1, 2)
        return g

    def make_Bs(r):
        sigma = torch.arange(1, r + 1, device=device, dtype=torch.float32) ** (-w.sigma_decay)
        out = torch.empty((n_seq, w.G, r, w.d), dtype=dt, device=device)
        for b in range(n_seq):
            g = torch.randn((w.G, w.d, r), generator=gen, device=device, dtype=torch.float32)
            qf = orthonormal_columns(g)
            out[b] = (sigma[None, :, None] * qf.transpose(1, 2)).to(dt)
        return out

    return {
        "A_k": normal((n_seq, w.L, w.r_k), w.a_scale),
        "A_v": normal((n_seq, w.L, w.r_v), w.a_scale),
        "B_k": make_Bs(w.r_k),
        "B_v": make_Bs(w.r_v),
        "q": normal((w.G, n_seq, w.H_q, w.d_h), w.q_scale),
    }
