"""fp64 CPU oracle for the factorized-linear hot path -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It never imports the HIP package and shares nothing with it.

The arithmetic lives in ``lowrank_oracle.c`` (plain C loops in binary64, following the
paper's Section 3.1); this module compiles it with gcc on first use and marshals numpy
float64 arrays through ctypes.  Every function takes and returns float64; callers widen
the bf16 / fp32 inputs the GPU sees exactly to float64 before calling.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lowrank_oracle.c")
_LIB = os.path.join(_HERE, "liblr_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc, -O2, OpenMP, no FP contraction).  Returns the .so path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call([
            "gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11",
            "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


_i64 = ctypes.c_int64


def num_threads() -> int:
    """Threads the OpenMP row loop uses (reported as ``cores`` by the benchmark)."""
    return int(_load().lr_oracle_num_threads())


def linear(x, U, V, bias=None) -> np.ndarray:
    """y = (x U) V (+ bias): the factor-pair linear layer of Section 3.1."""
    x, U, V = _f64(x), _f64(U), _f64(V)
    M, d_in = x.shape
    r, d_out = V.shape
    assert U.shape == (d_in, r), (U.shape, d_in, r)
    b = None if bias is None else _f64(bias)
    assert b is None or b.shape == (d_out,)
    y = np.empty((M, d_out), dtype=np.float64)
    rc = _load().lr_oracle_linear(_p(x), _p(U), _p(V), _p(b), _p(y),
                                  _i64(M), _i64(d_in), _i64(r), _i64(d_out))
    assert rc == 0, rc
    return y


def stage1(x, U) -> np.ndarray:
    """t = x U, the rank-space intermediate."""
    x, U = _f64(x), _f64(U)
    M, d_in = x.shape
    assert U.shape[0] == d_in
    r = U.shape[1]
    t = np.empty((M, r), dtype=np.float64)
    _load().lr_oracle_stage1(_p(x), _p(U), _p(t), _i64(M), _i64(d_in), _i64(r))
    return t


def stage2(t, V, bias=None) -> np.ndarray:
    """y = t V (+ bias)."""
    t, V = _f64(t), _f64(V)
    M, r = t.shape
    assert V.shape[0] == r
    d_out = V.shape[1]
    b = None if bias is None else _f64(bias)
    y = np.empty((M, d_out), dtype=np.float64)
    _load().lr_oracle_stage2(_p(t), _p(V), _p(b), _p(y), _i64(M), _i64(r), _i64(d_out))
    return y


def cache_write(proj, cache: np.ndarray, pos, T: int) -> None:
    """Scatter rows of ``proj`` [B*T, H*E] into the dense cache [B, S_max, H, E] in place
    at positions pos[b] .. pos[b]+T-1 (Section 3.1, dense KV cache)."""
    proj = _f64(proj)
    assert cache.dtype == np.float64 and cache.flags.c_contiguous and cache.ndim == 4
    B, S_max, H, E = cache.shape
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    assert pos.shape == (B,) and proj.shape == (B * T, H * E)
    rc = _load().lr_oracle_cache_write(_p(proj), _p(cache), _p(pos), _i64(B), _i64(T),
                                       _i64(S_max), _i64(H), _i64(E))
    if rc != 0:
        raise ValueError("cache position out of range")


def qkv(x, Us: Sequence, Vs: Sequence, biases: Optional[Sequence] = None, kv: Optional[dict] = None):
    """Several projections of the same x (Q, K, V; or the layers that share one basis).

    Projections whose U is the *same object* share one stage-1 product t = x U (the
    shared basis is used once, Section 3.1).  ``kv`` (optional) is a dict with float64
    arrays ``k_cache``/``v_cache`` [B, S_max, H, E], int ``pos`` [B], ``T`` tokens per
    sequence and ``k_index``/``v_index`` naming which projections are K and V; those
    outputs are also scattered into the caches in place.  Returns the list of outputs.
    """
    n = len(Us)
    assert len(Vs) == n
    outs = []
    t_by_basis = {}
    for i in range(n):
        key = id(Us[i])
        if key not in t_by_basis:
            t_by_basis[key] = stage1(x, Us[i])
        b = None if biases is None else biases[i]
        outs.append(stage2(t_by_basis[key], Vs[i], b))
    if kv is not None:
        cache_write(outs[kv["k_index"]], kv["k_cache"], kv["pos"], kv["T"])
        cache_write(outs[kv["v_index"]], kv["v_cache"], kv["pos"], kv["T"])
    return outs


def packed_mlp(x, U_gu, V_g, V_u, U_d, V_d, b_g=None, b_u=None, b_d=None) -> np.ndarray:
    """out = down(SiLU(gate(x)) * up(x)) with the packed gate|up input factor (Section 3.1)."""
    x, U_gu, V_g, V_u, U_d, V_d = map(_f64, (x, U_gu, V_g, V_u, U_d, V_d))
    M, d = x.shape
    r_g, ffn = V_g.shape
    r_u = V_u.shape[0]
    r_d = U_d.shape[1]
    assert U_gu.shape == (d, r_g + r_u) and V_u.shape == (r_u, ffn)
    assert U_d.shape == (ffn, r_d) and V_d.shape == (r_d, d)
    bg = None if b_g is None else _f64(b_g)
    bu = None if b_u is None else _f64(b_u)
    bd = None if b_d is None else _f64(b_d)
    out = np.empty((M, d), dtype=np.float64)
    rc = _load().lr_oracle_packed_mlp(_p(x), _p(U_gu), _p(V_g), _p(V_u), _p(U_d), _p(V_d),
                                      _p(bg), _p(bu), _p(bd), _p(out),
                                      _i64(M), _i64(d), _i64(ffn), _i64(r_g), _i64(r_u), _i64(r_d))
    assert rc == 0, rc
    return out


def pack_concat(U_list: Sequence[np.ndarray]) -> np.ndarray:
    """Offline prepack: [U_0 | U_1 | ...] along the rank axis, bit-exact for any dtype."""
    Us = [np.ascontiguousarray(u) for u in U_list]
    d_in = Us[0].shape[0]
    dt = Us[0].dtype
    assert all(u.shape[0] == d_in and u.dtype == dt and u.ndim == 2 for u in Us)
    n = len(Us)
    ptrs = (ctypes.c_void_p * n)(*[u.ctypes.data for u in Us])
    rs = (ctypes.c_int64 * n)(*[u.shape[1] for u in Us])
    packed = np.empty((d_in, sum(u.shape[1] for u in Us)), dtype=dt)
    _load().lr_oracle_pack_concat(ptrs, rs, ctypes.c_int(n), _i64(d_in), _i64(dt.itemsize), _p(packed))
    return packed


def pack_panels(W: np.ndarray) -> np.ndarray:
    """Decode prepack (a pure re-layout, Section 3.1 first paragraph leaves the native layout to the runtime): the row-major
    factor W[K, N], N a multiple of 64, as N / 64 panels of 64 columns; returns an array [N / 64, K, 64] whose flat order is
    the layout: panel p holds columns 64 p .. 64 p + 63 of every row, rows in order.  Bit-exact for any dtype."""
    W = np.ascontiguousarray(W)
    K, N = W.shape
    assert N % 64 == 0
    out = np.empty((N // 64, K, 64), dtype=W.dtype)
    for p in range(N // 64):
        for k in range(K):
            out[p, k, :] = W[k, 64 * p:64 * p + 64]
    return out


def rope(x, positions, H: int, E: int, base: float = 10000.0) -> np.ndarray:
    """Rotary position embedding, rotate-half pairing (i, i + E/2), angle p * base**(-2i/E);
    x [rows, H*E], positions [rows] (Section 4: RoPE on q and k)."""
    x = _f64(x)
    rows = x.shape[0]
    assert x.shape == (rows, H * E)
    p = np.ascontiguousarray(positions, dtype=np.int64)
    assert p.shape == (rows,)
    y = np.empty_like(x)
    rc = _load().lr_oracle_rope(_p(x), _p(y), _p(p), _i64(rows), _i64(H), _i64(E), ctypes.c_double(base))
    assert rc == 0, rc
    return y


def decode_attention(q, k_cache: np.ndarray, v_cache: np.ndarray, pos, T: int, scale: float,
                     rope_base: float = 0.0) -> np.ndarray:
    """Causal attention of T new tokens per sequence over the dense cache [B, S_max, H, E]
    (Section 3.1, decode attention).  Rows pos[b]..pos[b]+T-1 of the caches hold the new raw k / v;
    with rope_base > 0 the new k rows are rotated in place in ``k_cache`` and q is rotated first.
    Returns out [B*T, H*E]."""
    q = _f64(q)
    assert k_cache.dtype == np.float64 and k_cache.flags.c_contiguous and k_cache.ndim == 4
    v_cache = _f64(v_cache)
    B, S_max, H, E = k_cache.shape
    assert v_cache.shape == k_cache.shape and q.shape == (B * T, H * E)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    assert pos.shape == (B,)
    out = np.empty((B * T, H * E), dtype=np.float64)
    rc = _load().lr_oracle_decode_attention(_p(q), _p(k_cache), _p(v_cache), _p(pos), _p(out), _i64(B), _i64(T),
                                            _i64(S_max), _i64(H), _i64(E), ctypes.c_double(scale),
                                            ctypes.c_double(rope_base))
    if rc == -1:
        raise ValueError("cache position out of range")
    assert rc == 0, rc
    return out


# ---------------------------------------------------------------------------------------------
# Diagnostic-only "rounding-faithful" mode.  The definitions above round nothing; a bf16 kernel
# rounds the rank-space rows t, the hidden rows h and the outputs to bfloat16 (nearest-even).
# The functions below take the same steps in the same order with those three roundings put in, in
# float64 otherwise, so that a kernel result can be compared with something that differs from it by
# accumulation order only.  They gate nothing: tests report the distance to them next to the
# distance to the exact definition, to tell rounding from a systematic error inside the tolerance.
# ---------------------------------------------------------------------------------------------
def round_bf16(a) -> np.ndarray:
    """Nearest bfloat16 (8 significant bits, ties to even) of float64 values, returned as float64.
    Written on the float64 value itself: scale to an integer significand, round half to even, scale back."""
    a = _f64(a)
    out = np.zeros_like(a)
    nz = np.isfinite(a) & (a != 0.0)
    m, e = np.frexp(a[nz])                 # a = m * 2**e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0)                 # 8 significant bits; numpy rounds half to even
    out[nz] = np.ldexp(q, e - 8)
    out[~np.isfinite(a)] = a[~np.isfinite(a)]
    return out


def diag_linear(x, U, V, bias=None, rnd=round_bf16) -> np.ndarray:
    """linear() with t and y rounded by ``rnd`` (identity ``rnd`` gives linear() again)."""
    return rnd(stage2(rnd(stage1(x, U)), V, bias))


def diag_qkv(x, Us: Sequence, Vs: Sequence, biases: Optional[Sequence] = None, rnd=round_bf16):
    """qkv() without the cache scatter, with t and the outputs rounded by ``rnd``."""
    t_by_basis = {}
    outs = []
    for i in range(len(Us)):
        key = id(Us[i])
        if key not in t_by_basis:
            t_by_basis[key] = rnd(stage1(x, Us[i]))
        outs.append(rnd(stage2(t_by_basis[key], Vs[i], None if biases is None else biases[i])))
    return outs


def diag_packed_mlp(x, U_gu, V_g, V_u, U_d, V_d, b_g=None, b_u=None, b_d=None, rnd=round_bf16) -> np.ndarray:
    """packed_mlp() step by step (Section 3.1, packed gate/up) with t_gu, h, t_d and out rounded by ``rnd``."""
    V_g, V_u = _f64(V_g), _f64(V_u)
    r_g = V_g.shape[0]
    t = rnd(stage1(x, U_gu))
    g = stage2(np.ascontiguousarray(t[:, :r_g]), V_g, b_g)
    u = stage2(np.ascontiguousarray(t[:, r_g:]), V_u, b_u)
    h = rnd(g / (1.0 + np.exp(-g)) * u)
    return rnd(stage2(rnd(stage1(h, U_d)), V_d, b_d))
