"""ctypes binding of liblowrank.so -- argument marshalling only.

Every function has the name and the argument order of its C entry point in
``include/lowrank.h``; tensors are torch tensors on the GPU whose ``data_ptr()`` is passed
through (PyTorch serves as device-memory allocator and stream provider, nothing else).  All
arithmetic happens in the HIP kernels.  Importing this module loads the library and raises
``ImportError`` if it has not been built (``python -m paper_2605_08314_amd.build``): there is
no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch  # imported before the library so that the HIP runtime torch ships is the one in use

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblowrank.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_08314_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)

LR_F32, LR_BF16, LR_BF16_PANELS = 0, 1, 2
LR_PHASE_DECODE, LR_PHASE_PREFILL, LR_PHASE_AUTO = 0, 1, 2
LR_OP_LINEAR, LR_OP_QKV, LR_OP_PACKED_MLP, LR_OP_DECODE_ATTENTION = 0, 1, 2, 3
PHASES = {"decode": LR_PHASE_DECODE, "prefill": LR_PHASE_PREFILL, "auto": LR_PHASE_AUTO}

_vp, _i64, _int, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t


class lr_kv_target(ctypes.Structure):
    _fields_ = [("k_cache", _vp), ("v_cache", _vp), ("pos", _vp),
                ("B", _i64), ("S_max", _i64), ("n_heads", _i64), ("head_dim", _i64),
                ("tokens_per_seq", _i64), ("k_index", ctypes.c_int32), ("v_index", ctypes.c_int32)]


_lib.lowrank_linear.argtypes = [_vp] * 5 + [_i64] * 4 + [_int, _int, _vp, _sz, _vp]
_lib.lowrank_linear.restype = _int
_lib.lowrank_linear_noalloc.argtypes = [_vp] * 5 + [_i64] * 4 + [_int, _vp]
_lib.lowrank_linear_noalloc.restype = _int
_lib.lowrank_qkv.argtypes = [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_vp),
                             ctypes.POINTER(_vp), ctypes.POINTER(_i64), ctypes.POINTER(_i64), _int,
                             _i64, _i64, ctypes.POINTER(lr_kv_target), _int, _int, _vp, _sz, _vp]
_lib.lowrank_qkv.restype = _int
_lib.lowrank_packed_mlp.argtypes = [_vp] * 10 + [_i64] * 6 + [_int, _int, _vp, _sz, _vp]
_lib.lowrank_packed_mlp.restype = _int
_lib.lowrank_decode_attention.argtypes = [_vp, ctypes.POINTER(lr_kv_target), _vp, ctypes.c_float, ctypes.c_float, _int, _vp, _sz, _vp]
_lib.lowrank_decode_attention.restype = _int
_lib.lowrank_prefill_attention.argtypes = [_vp, ctypes.POINTER(lr_kv_target), _vp, ctypes.c_float, ctypes.c_float, _int, _vp]
_lib.lowrank_prefill_attention.restype = _int
_lib.lowrank_prefill_factorized_attention.argtypes = [_vp, _vp, _vp, _i64, ctypes.POINTER(lr_kv_target), _vp, ctypes.c_float, ctypes.c_float, _int, _vp]
_lib.lowrank_prefill_factorized_attention.restype = _int
_lib.lowrank_rank_project.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _int, _vp, _sz, _vp]
_lib.lowrank_rank_project.restype = _int
_lib.lowrank_pack_concat.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(_i64), _int, _i64, _int, _vp, _vp]
_lib.lowrank_pack_concat.restype = _int
_lib.lowrank_pack_panels.argtypes = [_vp, _i64, _i64, _vp, _int, _vp]
_lib.lowrank_pack_panels.restype = _int
_lib.lowrank_workspace_bytes.argtypes = [_int, _i64, _i64, _i64, _i64, _int, _int]
_lib.lowrank_workspace_bytes.restype = _sz
_lib.lowrank_workspace_init.argtypes = [_vp, _sz, _vp]
_lib.lowrank_workspace_init.restype = _int
_lib.lowrank_workspace_status.argtypes = [_vp, _vp]
_lib.lowrank_workspace_status.restype = _int
_lib.lowrank_configure.argtypes = [_int, _i64]
_lib.lowrank_configure.restype = _int
_lib.lowrank_plan_name.argtypes = [_int, _i64, _i64, _i64, _i64, _int, _int, _int]
_lib.lowrank_plan_name.restype = ctypes.c_char_p
_lib.lowrank_prefill_tile.argtypes = [_i64, _i64, _i64, _int, _int] + [ctypes.POINTER(_int)] * 3
_lib.lowrank_prefill_tile.restype = _int
_lib.lowrank_last_error.restype = ctypes.c_char_p
_lib.lowrank_version.restype = ctypes.c_char_p


class LowrankError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"liblowrank status {status}: {lowrank_last_error()}")


def _check(st: int) -> None:
    if st != 0:
        raise LowrankError(st)


def _dtype_code(t: torch.Tensor, panels: bool = False) -> int:
    if panels:
        assert t.dtype == torch.bfloat16, "panel layout is bf16 only"
        return LR_BF16_PANELS
    return _plain_dtype_code(t)


def _plain_dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LR_F32
    if t.dtype == torch.bfloat16:
        return LR_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors must be contiguous"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _phase(phase) -> int:
    return PHASES[phase] if isinstance(phase, str) else int(phase)


def lowrank_last_error() -> str:
    return _lib.lowrank_last_error().decode()


def lowrank_version() -> str:
    return _lib.lowrank_version().decode()


def lowrank_prefill_tile(M: int, K: int, N: int, n_products: int = 1, gate_up: bool = False):
    """(tile_m, tile_n, share_k) the prefill dispatcher picks for n_products products [M, K] x [K, N];
    share_k: 0 = none, 1 = shared-K walk, n >= 2 = K cut into n chunks (split-K with a reduction launch)."""
    bm, bn, sk = _int(0), _int(0), _int(0)
    _check(_lib.lowrank_prefill_tile(M, K, N, n_products, int(gate_up), ctypes.byref(bm), ctypes.byref(bn), ctypes.byref(sk)))
    return bm.value, bn.value, sk.value


def lowrank_workspace_bytes(op: int, M: int, d_in: int, r_total: int, d_out: int, dtype: int, phase) -> int:
    return int(_lib.lowrank_workspace_bytes(op, M, d_in, r_total, d_out, dtype, _phase(phase)))


def lowrank_plan_name(op: int, M: int, d_in: int, r_total: int, d_out: int, dtype: int, phase, aligned: bool = True) -> str:
    return _lib.lowrank_plan_name(op, M, d_in, r_total, d_out, dtype, _phase(phase), int(aligned)).decode()


def lowrank_workspace_init(workspace: torch.Tensor, stream=None) -> None:
    _check(_lib.lowrank_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def lowrank_workspace_status(workspace: torch.Tensor, stream=None) -> None:
    """Synchronises the stream; raises if a fused decode call on this workspace gave up waiting."""
    _check(_lib.lowrank_workspace_status(_ptr(workspace), _stream(stream)))


LR_CFG_DEVICE_SHARED, LR_CFG_WAIT_LIMIT = 0, 1


def lowrank_configure(option: int, value: int) -> None:
    _check(_lib.lowrank_configure(option, value))


def new_workspace(op: int, M: int, d_in: int, r_total: int, d_out: int, dtype: int, phase="auto",
                  device="cuda", prepare: bool = False) -> torch.Tensor:
    """Allocate (with torch) a workspace big enough for the given call.  The library prepares a workspace
    itself on first use, so nothing else is needed; ``prepare=True`` also calls lowrank_workspace_init.
    The part in which the library keeps state is filled with random bytes first, so that no caller (or
    test) can come to depend on fresh memory happening to be zero."""
    n = max(lowrank_workspace_bytes(op, M, d_in, r_total, d_out, dtype, phase), 4096)
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    ws[: min(n, 17 << 20)].random_(0, 256)
    if prepare:
        lowrank_workspace_init(ws)
    return ws


def lowrank_linear(x, U, V, bias, y, phase, workspace, stream=None, panels: bool = False) -> None:
    """panels=True: U and V hold 64-column panels (lowrank_pack_panels); their shapes are still (d_in, r), (r, d_out)."""
    M, d_in = x.shape
    r, d_out = V.shape
    assert U.shape == (d_in, r) and y.shape == (M, d_out)
    _check(_lib.lowrank_linear(_ptr(x), _ptr(U), _ptr(V), _ptr(bias), _ptr(y), M, d_in, r, d_out,
                               _dtype_code(x, panels), _phase(phase), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream(stream)))


def lowrank_linear_noalloc(x, U, V, bias, y, stream=None) -> None:
    M, d_in = x.shape
    r, d_out = V.shape
    assert U.shape == (d_in, r) and y.shape == (M, d_out)
    _check(_lib.lowrank_linear_noalloc(_ptr(x), _ptr(U), _ptr(V), _ptr(bias), _ptr(y), M, d_in, r, d_out,
                                       _dtype_code(x), _stream(stream)))


def lowrank_qkv(x, U: Sequence, V: Sequence, bias: Optional[Sequence], out: Sequence, kv: Optional[dict],
                phase, workspace, stream=None, panels: bool = False) -> None:
    """``kv``: dict(k_cache, v_cache, pos, tokens_per_seq, k_index, v_index) or None; the caches
    are [B, S_max, n_heads, head_dim] tensors, pos an int32 device tensor [B]."""
    n = len(U)
    M, d_in = x.shape
    arr = lambda items: (_vp * n)(*[_ptr(t) for t in items])
    rs = (_i64 * n)(*[v.shape[0] for v in V])
    ns = (_i64 * n)(*[v.shape[1] for v in V])
    kvs = None
    if kv is not None:
        kc = kv["k_cache"]
        B, S_max, H, E = kc.shape
        assert kv["pos"].dtype == torch.int32
        kvs = ctypes.pointer(lr_kv_target(_ptr(kc), _ptr(kv["v_cache"]), _ptr(kv["pos"]), B, S_max, H, E,
                                          kv["tokens_per_seq"], kv["k_index"], kv["v_index"]))
    _check(_lib.lowrank_qkv(_ptr(x), arr(U), arr(V), None if bias is None else arr(bias), arr(out), rs, ns, n,
                            M, d_in, kvs, _dtype_code(x, panels), _phase(phase), _ptr(workspace),
                            workspace.numel() * workspace.element_size(), _stream(stream)))


def lowrank_packed_mlp(x, U_gu, V_g, V_u, U_d, V_d, b_g, b_u, b_d, out, phase, workspace, stream=None,
                       panels: bool = False) -> None:
    M, d = x.shape
    r_g, ffn = V_g.shape
    r_u = V_u.shape[0]
    r_d = U_d.shape[1]
    assert U_gu.shape == (d, r_g + r_u) and V_u.shape == (r_u, ffn)
    assert U_d.shape == (ffn, r_d) and V_d.shape == (r_d, d) and out.shape == (M, d)
    _check(_lib.lowrank_packed_mlp(_ptr(x), _ptr(U_gu), _ptr(V_g), _ptr(V_u), _ptr(U_d), _ptr(V_d),
                                   _ptr(b_g), _ptr(b_u), _ptr(b_d), _ptr(out), M, d, ffn, r_g, r_u, r_d,
                                   _dtype_code(x, panels), _phase(phase), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)))


def lowrank_decode_attention(q, k_cache, v_cache, pos, tokens_per_seq: int, out, scale: float, rope_base: float,
                             workspace, stream=None) -> None:
    """q, out [B * tokens_per_seq, n_heads * head_dim]; caches [B, S_max, n_heads, head_dim]; pos int32 [B].
    Rotates the new k rows in place in ``k_cache`` when rope_base > 0."""
    B, S_max, H, E = k_cache.shape
    assert v_cache.shape == k_cache.shape and pos.dtype == torch.int32
    assert q.shape == (B * tokens_per_seq, H * E) and out.shape == q.shape
    kvs = lr_kv_target(_ptr(k_cache), _ptr(v_cache), _ptr(pos), B, S_max, H, E, tokens_per_seq, 0, 0)
    _check(_lib.lowrank_decode_attention(_ptr(q), ctypes.byref(kvs), _ptr(out), scale, rope_base, _dtype_code(q),
                                         _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def lowrank_prefill_attention(q, k_cache, v_cache, pos, tokens_per_seq: int, out, scale: float, rope_base: float,
                              stream=None) -> None:
    """Same operation and shapes as ``lowrank_decode_attention``, on the matrix cores (bf16, head_dim 128); no workspace."""
    B, S_max, H, E = k_cache.shape
    assert v_cache.shape == k_cache.shape and pos.dtype == torch.int32
    assert q.shape == (B * tokens_per_seq, H * E) and out.shape == q.shape
    kvs = lr_kv_target(_ptr(k_cache), _ptr(v_cache), _ptr(pos), B, S_max, H, E, tokens_per_seq, 0, 0)
    _check(_lib.lowrank_prefill_attention(_ptr(q), ctypes.byref(kvs), _ptr(out), scale, rope_base, _dtype_code(q), _stream(stream)))


def lowrank_prefill_factorized_attention(t_q, V_q, b_q, k_cache, v_cache, pos, tokens_per_seq: int, out, scale: float,
                                         rope_base: float, stream=None) -> None:
    """Prefill attention whose queries arrive as rank-space rows t_q [M, r] and the factor V_q [r, H * E] (+ optional b_q)."""
    B, S_max, H, E = k_cache.shape
    r = V_q.shape[0]
    assert v_cache.shape == k_cache.shape and pos.dtype == torch.int32
    assert t_q.shape == (B * tokens_per_seq, r) and V_q.shape == (r, H * E) and out.shape == (B * tokens_per_seq, H * E)
    kvs = lr_kv_target(_ptr(k_cache), _ptr(v_cache), _ptr(pos), B, S_max, H, E, tokens_per_seq, 0, 0)
    _check(_lib.lowrank_prefill_factorized_attention(_ptr(t_q), _ptr(V_q), _ptr(b_q), r, ctypes.byref(kvs), _ptr(out), scale,
                                                     rope_base, _dtype_code(t_q), _stream(stream)))


def lowrank_rank_project(x, U, t, workspace, stream=None) -> None:
    M, d_in = x.shape
    r = U.shape[1]
    assert U.shape == (d_in, r) and t.shape == (M, r)
    _check(_lib.lowrank_rank_project(_ptr(x), _ptr(U), _ptr(t), M, d_in, r, _dtype_code(x), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)))


def lowrank_pack_panels(W: torch.Tensor, W_panels: torch.Tensor, stream=None) -> None:
    """W [K, N] row-major bf16 -> W_panels (same shape and size): N / 64 panels of 64 columns, each [K, 64] contiguous."""
    K, N = W.shape
    assert W_panels.numel() == W.numel() and W_panels.dtype == W.dtype
    _check(_lib.lowrank_pack_panels(_ptr(W), K, N, _ptr(W_panels), _plain_dtype_code(W), _stream(stream)))


def lowrank_pack_concat(U_list: Sequence[torch.Tensor], U_packed: torch.Tensor, stream=None) -> None:
    n = len(U_list)
    d_in = U_list[0].shape[0]
    ptrs = (_vp * n)(*[_ptr(u) for u in U_list])
    rs = (_i64 * n)(*[u.shape[1] for u in U_list])
    assert U_packed.shape == (d_in, sum(u.shape[1] for u in U_list))
    _check(_lib.lowrank_pack_concat(ptrs, rs, n, d_in, _dtype_code(U_list[0]), _ptr(U_packed), _stream(stream)))
