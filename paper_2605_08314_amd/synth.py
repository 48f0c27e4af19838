"""Seeded synthetic inputs with the shapes of the paper's LLaMA-7B / 13B low-rank layers.

This module holds no arithmetic of the method itself: it only draws random tensors,
builds factor pairs with a prescribed singular spectrum, and converts between float64
and the bit patterns (bf16 as uint16, fp32) that the GPU library consumes.  Both the
parity tests (which feed the same arrays to the CPU oracle and to the HIP path) and the
benchmark use it.  The paper evaluates on compressed LLaMA-7B checkpoints (Section 4.1,
Table 2); those are not available offline, so these tensors stand in for them: same
shapes (d=4096, ffn=11008, 32 heads x 128; 13B: d=5120, 40 heads), factors obtained as
the exact truncated SVD of a random matrix whose singular values decay as i^-1/2.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

BASE_SEED = 260508314


def seed_for(cfg: int, i: int = 0) -> int:
    return BASE_SEED + 1000 * cfg + i


# ----------------------------------------------------------------------------- dtype plumbing
def f64_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float64/float32 values to bfloat16 (nearest-even) and return the uint16 bits."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16).reshape(f.shape)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64).reshape(bits.shape)


@dataclass
class Tensor:
    """One input tensor: ``dev`` is what the GPU gets (uint16 bf16 bits or float32),
    ``f64`` is exactly the same values widened to float64 for the oracle."""
    dev: np.ndarray
    f64: np.ndarray


def to_dtype(a: np.ndarray, dtype: str) -> Tensor:
    if dtype == "bf16":
        bits = f64_to_bf16_bits(a)
        return Tensor(bits, bf16_bits_to_f64(bits))
    if dtype == "f32":
        f = np.ascontiguousarray(a, dtype=np.float32)
        return Tensor(f, f.astype(np.float64))
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- factor recipes
def spectrum(n: int, d_out: int) -> np.ndarray:
    """sigma_i = c * i^-1/2, i = 1..n, with c chosen so that sum sigma_i^2 = d_out
    (a unit-variance input row then gives a roughly unit-variance output row)."""
    i = np.arange(1, n + 1, dtype=np.float64)
    s = i ** -0.5
    return s * np.sqrt(d_out / np.sum(s * s))


def orthonormal(rows: int, cols: int, rng: np.random.Generator) -> np.ndarray:
    """rows x cols matrix with orthonormal columns (thin QR of a Gaussian matrix)."""
    q, _ = np.linalg.qr(rng.standard_normal((rows, cols)))
    return q


def svd_factors(d_in: int, d_out: int, r: int, rng: np.random.Generator,
                q1: Optional[np.ndarray] = None):
    """Factor pair of the rank-r truncated SVD of W = Q1 diag(sigma) Q2^T.

    W is built from its SVD (Q1, Q2 orthonormal, sigma distinct and decreasing), so its
    best rank-r approximation is Q1[:, :r] diag(sigma[:r]) Q2[:, :r]^T; sqrt(sigma) goes to
    each side.  Only the r leading columns are ever needed.  Returns float64 (U, V).
    ``q1`` lets several layers share one input-side basis."""
    sig = spectrum(r, d_out)
    if q1 is None:
        q1 = orthonormal(d_in, r, rng)
    q2 = orthonormal(d_out, r, rng)
    root = np.sqrt(sig)
    return q1 * root[None, :], root[:, None] * q2.T


def full_svd_matrix(d_in: int, d_out: int, rng: np.random.Generator):
    """(W, Q1, sigma, Q2) with W = Q1 diag(sigma) Q2^T of full rank min(d_in, d_out)."""
    n = min(d_in, d_out)
    q1, q2 = orthonormal(d_in, n, rng), orthonormal(d_out, n, rng)
    sig = spectrum(n, d_out)
    return (q1 * sig[None, :]) @ q2.T, q1, sig, q2


# ----------------------------------------------------------------------------- workloads
@dataclass
class Workload:
    name: str
    dtype: str
    t: Dict[str, Tensor] = field(default_factory=dict)   # named tensors
    meta: Dict[str, object] = field(default_factory=dict)


def config1(seed: int = seed_for(1)) -> Workload:
    """Single factorized linear, fp32: x[16,512], U[512,128], V[128,512]; entries normal with
    standard deviation fan_in^-1/2 (fan_in = 512 for x and U, 128 for V); no bias."""
    rng = np.random.default_rng(seed)
    w = Workload("cfg1_linear_f32", "f32")
    w.t["x"] = to_dtype(rng.standard_normal((16, 512)) / np.sqrt(512), "f32")
    w.t["U"] = to_dtype(rng.standard_normal((512, 128)) / np.sqrt(512), "f32")
    w.t["V"] = to_dtype(rng.standard_normal((128, 512)) / np.sqrt(128), "f32")
    w.meta.update(M=16, d_in=512, r=128, d_out=512)
    return w


def attention_layer(B: int, d: int = 4096, r: int = 384, n_heads: int = 32, S_max: int = 64,
                    T: int = 1, seed: int = seed_for(2), dtype: str = "bf16") -> Workload:
    """Q/K/V/O factor pairs of one attention block (config 2 at d=4096, r=384).

    x[B*T, d] ~ N(0,1) feeds Q, K and V; the O projection takes an independent a[B*T, d]
    ~ N(0,1) standing in for the attention output, which this path does not compute.
    ``pos`` holds one seeded write position per sequence with pos[b] + T <= S_max."""
    rng = np.random.default_rng(seed)
    w = Workload(f"attn_d{d}_r{r}_M{B*T}", dtype)
    for name in ("q", "k", "v", "o"):
        U, V = svd_factors(d, d, r, rng)
        w.t["U_" + name], w.t["V_" + name] = to_dtype(U, dtype), to_dtype(V, dtype)
    w.t["x"] = to_dtype(rng.standard_normal((B * T, d)), dtype)
    w.t["a"] = to_dtype(rng.standard_normal((B * T, d)), dtype)
    pos = rng.integers(0, S_max - T + 1, size=B).astype(np.int32)
    w.meta.update(B=B, T=T, M=B * T, d=d, r=r, n_heads=n_heads, head_dim=d // n_heads,
                  S_max=S_max, pos=pos)
    return w


def mlp_layer(M: int, d: int = 4096, ffn: int = 11008, r_g: int = 768, r_u: int = 768,
              r_d: int = 768, seed: int = seed_for(3), dtype: str = "bf16",
              with_bias: bool = False) -> Workload:
    """Packed-MLP factors (config 3 at d=4096, ffn=11008, r=768): U_gu = [U_gate | U_up]."""
    rng = np.random.default_rng(seed)
    w = Workload(f"mlp_d{d}_f{ffn}_r{r_g}-{r_u}-{r_d}_M{M}", dtype)
    Ug, Vg = svd_factors(d, ffn, r_g, rng)
    Uu, Vu = svd_factors(d, ffn, r_u, rng)
    Ud, Vd = svd_factors(ffn, d, r_d, rng)
    w.t["U_g"], w.t["U_u"] = to_dtype(Ug, dtype), to_dtype(Uu, dtype)
    w.t["U_gu"] = Tensor(np.concatenate([w.t["U_g"].dev, w.t["U_u"].dev], axis=1),
                         np.concatenate([w.t["U_g"].f64, w.t["U_u"].f64], axis=1))
    w.t["V_g"], w.t["V_u"] = to_dtype(Vg, dtype), to_dtype(Vu, dtype)
    w.t["U_d"], w.t["V_d"] = to_dtype(Ud, dtype), to_dtype(Vd, dtype)
    w.t["x"] = to_dtype(rng.standard_normal((M, d)), dtype)
    if with_bias:
        w.t["b_g"] = to_dtype(0.1 * rng.standard_normal(ffn), dtype)
        w.t["b_u"] = to_dtype(0.1 * rng.standard_normal(ffn), dtype)
        w.t["b_d"] = to_dtype(0.1 * rng.standard_normal(d), dtype)
    w.meta.update(M=M, d=d, ffn=ffn, r_g=r_g, r_u=r_u, r_d=r_d)
    return w


def shared_basis(M: int, d: int = 5120, r: int = 512, n_layers: int = 2,
                 seed: int = seed_for(5), dtype: str = "bf16") -> Workload:
    """Config 5: one basis U_shared[d, r] reused by ``n_layers`` layers, each with its own
    V_i[r, d] (W_i ~ U_shared V_i): one orthonormal Q1 and independent Q2_i."""
    rng = np.random.default_rng(seed)
    w = Workload(f"shared_d{d}_r{r}_M{M}", dtype)
    q1 = orthonormal(d, r, rng)
    root = np.sqrt(spectrum(r, d))
    w.t["U_sh"] = to_dtype(q1 * root[None, :], dtype)
    for i in range(n_layers):
        q2 = orthonormal(d, r, rng)
        w.t[f"V_{i}"] = to_dtype(root[:, None] * q2.T, dtype)
    w.t["x"] = to_dtype(rng.standard_normal((M, d)), dtype)
    w.meta.update(M=M, d=d, r=r, n_layers=n_layers)
    return w


def prefill_row_sample(S: int, tile: int = 128, per_tile: int = 2,
                       seed: int = seed_for(4, 99)) -> np.ndarray:
    """Rows the oracle checks at prefill sizes: first and last row of every ``tile``-row
    block plus ``per_tile`` seeded rows inside it (rows are independent, so a row sample
    checks every column of those rows exactly)."""
    rng = np.random.default_rng(seed)
    rows: List[int] = []
    for lo in range(0, S, tile):
        hi = min(S, lo + tile)
        rows += [lo, hi - 1]
        rows += list(rng.integers(lo, hi, size=per_tile))
    return np.unique(np.asarray(rows, dtype=np.int64))
