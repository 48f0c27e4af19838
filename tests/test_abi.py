"""CPU-only checks of the C-ABI library: it loads, exports every function the header declares,
and its host-side logic (workspace sizing, argument validation, plan names) behaves.  No kernel
is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lowrank.h")


@pytest.fixture(scope="module")
def B():
    from paper_2605_08314_amd import binding
    return binding


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lowrank_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol(B):
    names = declared_functions()
    assert {"lowrank_linear", "lowrank_qkv", "lowrank_packed_mlp"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in lowrank.h but not exported"
    assert "gfx950" in B.lowrank_version()


def test_workspace_bytes_host_function(B):
    assert B.lowrank_workspace_bytes(B.LR_OP_LINEAR, 0, 4096, 384, 4096, B.LR_BF16, "decode") >= 4096
    a = B.lowrank_workspace_bytes(B.LR_OP_LINEAR, 32, 4096, 384, 4096, B.LR_BF16, "decode")
    b = B.lowrank_workspace_bytes(B.LR_OP_LINEAR, 64, 4096, 384, 4096, B.LR_BF16, "decode")
    assert b > a >= 4096 + 32 * 384 * 4
    m = B.lowrank_workspace_bytes(B.LR_OP_PACKED_MLP, 32, 4096, 2304, 11008, B.LR_BF16, "decode")
    assert m >= 32 * (2304 + 11008) * 4
    # monotone in the row count: a workspace for M rows serves fewer rows of the same call
    sizes = [B.lowrank_workspace_bytes(B.LR_OP_PACKED_MLP, M, 4096, 2304, 11008, B.LR_BF16, "auto") for M in (1, 8, 9, 32, 33, 512, 8192)]
    assert sizes == sorted(sizes)
    assert B.lowrank_workspace_bytes(9, 1, 1, 1, 1, B.LR_BF16, "decode") == 0
    assert B.lowrank_workspace_bytes(B.LR_OP_QKV, -1, 1, 1, 1, B.LR_BF16, "decode") == 0
    assert B.lowrank_workspace_bytes(B.LR_OP_QKV, 1, 1, 1, 1, 5, "decode") == 0


def test_validation_errors_without_launch(B):
    lib = ctypes.CDLL(B.LIB_PATH)
    lib.lowrank_linear.argtypes = B._lib.lowrank_linear.argtypes
    lib.lowrank_last_error.restype = ctypes.c_char_p
    fake = 0x1000  # never dereferenced: every call below fails validation first
    call = lambda **kw: lib.lowrank_linear(kw.get("x", fake), fake, fake, None, kw.get("y", fake),
                                           kw.get("M", 4), 64, 8, 64, kw.get("dtype", 1), kw.get("phase", 0),
                                           kw.get("ws", 0x10000), kw.get("wsb", 1 << 30), None)
    assert call(M=-1) == -2
    assert call(dtype=3) == -3
    assert call(phase=9) == -5
    assert call(ws=None) == -6
    assert call(ws=0x10010) == -4
    assert call(wsb=16) == -6 and b"workspace" in lib.lowrank_last_error()
    assert call(y=None) == -1
    assert call(M=0, ws=None) == 0          # empty batch: legal no-op, needs no workspace
    assert call(dtype=2) == -8 and b"panel" in lib.lowrank_last_error()    # panel layout outside the decode fast path (r = 8)
    lib.lowrank_pack_panels.argtypes = B._lib.lowrank_pack_panels.argtypes
    assert lib.lowrank_pack_panels(fake, 8, 100, 0x2000, 1, None) == -2      # N not a multiple of 64
    assert lib.lowrank_pack_panels(fake, 8, 128, 0x2000, 0, None) == -3      # bf16 only
    assert lib.lowrank_pack_panels(fake, 8, 128, fake, 1, None) == -2        # not in place
    assert lib.lowrank_pack_panels(None, 0, 128, None, 1, None) == 0         # empty: no-op


def test_plan_names(B):
    for args in [(B.LR_OP_LINEAR, 1, 4096, 384, 4096), (B.LR_OP_PACKED_MLP, 8192, 4096, 2304, 11008),
                 (B.LR_OP_QKV, 3, 37, 5, 19)]:
        for phase in ("decode", "prefill", "auto"):
            assert B.lowrank_plan_name(*args, B.LR_BF16, phase) in {"generic", "decode_mfma", "prefill_mfma"}
    # ragged shapes, fp32 and unaligned pointers always take the generic kernels
    assert B.lowrank_plan_name(B.LR_OP_QKV, 3, 37, 5, 19, B.LR_BF16, "decode") == "generic"
    assert B.lowrank_plan_name(B.LR_OP_LINEAR, 16, 512, 128, 512, B.LR_F32, "decode") == "generic"
    assert B.lowrank_plan_name(B.LR_OP_LINEAR, 16, 4096, 384, 4096, B.LR_BF16, "decode", aligned=False) == "generic"
    # factors stored as 64-column panels: the decode kernels or nothing
    assert B.lowrank_plan_name(B.LR_OP_LINEAR, 16, 4096, 384, 4096, B.LR_BF16_PANELS, "decode") == "decode_mfma"
    assert B.lowrank_plan_name(B.LR_OP_LINEAR, 512, 4096, 384, 4096, B.LR_BF16_PANELS, "auto") == "unsupported"
    assert B.lowrank_plan_name(B.LR_OP_LINEAR, 3, 37, 5, 19, B.LR_BF16_PANELS, "decode") == "unsupported"
    assert B.lowrank_workspace_bytes(B.LR_OP_LINEAR, 16, 4096, 384, 4096, B.LR_BF16_PANELS, "decode") == \
        B.lowrank_workspace_bytes(B.LR_OP_LINEAR, 16, 4096, 384, 4096, B.LR_BF16, "decode")


def _dry_lib(B):
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in ("lowrank_linear", "lowrank_qkv", "lowrank_packed_mlp", "lowrank_workspace_bytes"):
        getattr(lib, n).argtypes = getattr(B._lib, n).argtypes
        getattr(lib, n).restype = getattr(B._lib, n).restype
    lib.lowrank_last_error.restype = ctypes.c_char_p
    return lib


def test_qkv_cache_argument_validation_without_launch(B):
    """lowrank_qkv rejects inconsistent cache descriptions before anything is launched."""
    lib = _dry_lib(B)
    fake = 0x10000
    vp, i64 = ctypes.c_void_p, ctypes.c_int64

    def call(M=4, Bn=2, T=2, S_max=16, H=2, E=4, k_index=1, v_index=2, d_out=(8, 8, 8), cache=fake):
        U = (vp * 3)(fake, fake, fake); V = (vp * 3)(fake, fake, fake); out = (vp * 3)(fake, fake, fake)
        r = (i64 * 3)(4, 4, 4); n = (i64 * 3)(*d_out)
        kv = B.lr_kv_target(cache, cache, fake, Bn, S_max, H, E, T, k_index, v_index)
        return lib.lowrank_qkv(fake, U, V, None, out, r, n, 3, M, 16, ctypes.pointer(kv), B.LR_BF16, 0,
                               fake, 1 << 44, None)      # workspace size only compared, never touched

    assert call(k_index=3) == -2                      # index outside the projections
    assert call(Bn=3) == -2                           # B * tokens_per_seq != M
    assert call(S_max=1) == -2                        # cache shorter than one call's tokens
    assert call(d_out=(8, 8, 16)) == -2               # V width != n_heads * head_dim
    assert call(S_max=1 << 30) == -2                  # cache rows are 32-bit indices
    assert call(M=1 << 21, Bn=1 << 20, S_max=1 << 12) == -2 and b"2^31" in lib.lowrank_last_error()
    assert call(cache=None) == -1                     # NULL cache
    assert call(M=0, Bn=0, cache=None) == 0           # empty batch: no-op


def test_prefill_tile_selection_over_the_benchmark_shapes(B):
    """Host-side tile choice of the prefill phase (pure integer logic): every product of the mixed-rank layers
    (ranks 384/768, 256, 512, 1024 at S = 512, 2048, 8192) and of the shared-basis layer (13B shape, S = 4096)
    gets one of the three tile kernels, tall tiles only when there are rows for them, shared K only for the long-K
    product with few tiles, and the choices the measurements settled on at S = 8192 are the ones made."""
    shapes = []
    for S in (512, 2048, 8192):
        for ra, rm in ((384, 768), (256, 256), (512, 512), (1024, 1024)):
            shapes += [(S, 4096, ra, 3), (S, ra, 4096, 3), (S, 4096, ra, 1), (S, ra, 4096, 1),
                       (S, 4096, 2 * rm, 1), (S, 11008, rm, 1), (S, rm, 4096, 1)]
    shapes += [(4096, 5120, 512, 1), (4096, 512, 5120, 2), (4096, 13824, 512, 1)]
    for M, K, N, n in shapes:
        bm, bn, sk = B.lowrank_prefill_tile(M, K, N, n)
        assert (bm, bn) in {(256, 256), (256, 192), (128, 128)}, (M, K, N, n)
        t128 = n * ((M + 127) // 128) * ((N + 127) // 128)
        if sk == 1:      # shared-K walk: tall tiles, long K, few tiles
            assert bm == 256 and K >= 4096 and n * ((M + 255) // 256) * ((N + 255) // 256) <= 128, (M, K, N, n)
        elif sk >= 2:    # K cut into sk chunks: only when the 128 x 128 tiles leave most of the 512 workgroup slots empty
            assert (bm, bn) == (128, 128) and t128 <= 192 and t128 * sk <= 512 and K // sk >= 512 and n * sk <= 16, (M, K, N, n, sk)
        else:
            assert sk == 0
        if bn == 192:
            assert N % 192 == 0 or ((N + 191) // 192) * 192 - N < ((N + 255) // 256) * 256 - N      # 192-wide only where it wastes fewer columns
        assert B.lowrank_prefill_tile(M, K, N, n) == (bm, bn, sk)                                       # deterministic
    # S = 8192, ranks 384/768 (the benchmark's layer): reconstruction products on 256x256, the rank-space products
    # of width 1152 / 1536 on 256x192, h U_d (K = 11008, 96 tiles for 256 CUs) shares K on 256x192
    assert B.lowrank_prefill_tile(8192, 384, 4096, 3) == (256, 256, 0)
    assert B.lowrank_prefill_tile(8192, 4096, 384, 3) == (256, 192, 0)
    assert B.lowrank_prefill_tile(8192, 4096, 1536, 1) == (256, 192, 0)
    assert B.lowrank_prefill_tile(8192, 11008, 768, 1) == (256, 192, 1)
    assert B.lowrank_prefill_tile(8192, 768, 4096, 1) == (256, 256, 0)
    # few rows: the rank-space products (long K, 24..36 tiles of 128x128 for 512 slots) cut K into chunks,
    # the reconstruction products (K = rank) run as they are
    assert B.lowrank_prefill_tile(512, 4096, 384, 3) == (128, 128, 5)      # 36 tiles: 16 products at most -> 5 chunks
    assert B.lowrank_prefill_tile(512, 11008, 768, 1) == (128, 128, 8)
    assert B.lowrank_prefill_tile(512, 384, 4096, 3) == (128, 128, 0)
    assert B.lowrank_prefill_tile(2048, 11008, 768, 1) == (128, 128, 5)     # 96 tiles x 5 <= 512
    # the fused gate/up kernel has one shape; shapes outside the matrix-core rule are refused
    assert B.lowrank_prefill_tile(8192, 768, 11008, 1, gate_up=True) == (128, 128, 0)
    with pytest.raises(B.LowrankError):
        B.lowrank_prefill_tile(8192, 100, 4096, 1)


def test_configure_validates_its_arguments(B):
    B.lowrank_configure(B.LR_CFG_WAIT_LIMIT, 1 << 20)
    B.lowrank_configure(B.LR_CFG_DEVICE_SHARED, 0)
    with pytest.raises(B.LowrankError):
        B.lowrank_configure(99, 1)
    with pytest.raises(B.LowrankError):
        B.lowrank_configure(B.LR_CFG_WAIT_LIMIT, -1)
