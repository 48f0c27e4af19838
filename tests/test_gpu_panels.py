"""Factors stored as 64-column panels (lowrank_pack_panels, dtype LR_BF16_PANELS): the layout itself, and the decode calls
on panel factors against the oracle, which only ever sees the row-major matrices."""
import numpy as np
import pytest

from paper_2605_08314_amd import synth
from util import TOL, max_rel_err

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def G():
    import gpu_util
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return gpu_util


def _panels_host(oracle, t):
    """Row-major bf16 factor (synth.Tensor) -> the same bits in panel order, shaped [K, N] again for the binding."""
    bits = t.dev                                                # uint16 bit patterns [K, N]
    return oracle.pack_panels(bits).reshape(bits.shape)


@pytest.mark.parametrize("K,N", [(32, 64), (384, 4096), (4096, 1152), (11008, 768), (100, 192)])
def test_pack_panels_bit_exact(G, oracle, K, N):
    rng = np.random.default_rng(K + N)
    W = rng.integers(0, 65536, size=(K, N)).astype(np.uint16)
    Wd = G.dev(W)
    Pd = torch.zeros_like(Wd)
    G.B.lowrank_pack_panels(Wd, Pd)
    torch.cuda.synchronize()
    assert np.array_equal(G.bits(Pd).reshape(-1), oracle.pack_panels(W).reshape(-1))


@pytest.mark.parametrize("M", [1, 8, 17, 32])
def test_decode_calls_on_panel_factors(G, oracle, M):
    B = G.B
    # QKV with cache + O projection (benchmark shape)
    w = synth.attention_layer(M, S_max=64)
    m, t = w.meta, w.t
    d, r, H, E, S_max, T = m["d"], m["r"], m["n_heads"], m["head_dim"], m["S_max"], m["T"]
    x = G.dev(t["x"])
    Us = [G.dev(_panels_host(oracle, t["U_" + n])) for n in "qkv"]
    Vs = [G.dev(_panels_host(oracle, t["V_" + n])) for n in "qkv"]
    outs = [torch.full((M, d), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(3)]
    kc = torch.zeros((m["B"], S_max, H, E), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    ws = B.new_workspace(B.LR_OP_QKV, M, d, 3 * r, 3 * d, B.LR_BF16, "decode")
    B.lowrank_qkv(x, Us, Vs, None, outs, dict(k_cache=kc, v_cache=vc, pos=G.dev(m["pos"]), tokens_per_seq=T, k_index=1, v_index=2),
                  "decode", ws, panels=True)
    B.lowrank_workspace_status(ws)
    want = oracle.qkv(t["x"].f64, [t["U_" + n].f64 for n in "qkv"], [t["V_" + n].f64 for n in "qkv"])
    for i in range(3):
        assert max_rel_err(G.host64(outs[i]), want[i]) <= TOL["bf16"], f"projection {i}"
    kb, ob = G.bits(kc), G.bits(outs[1])
    for b in range(m["B"]):
        for s in range(T):
            assert np.array_equal(kb[b, m["pos"][b] + s].reshape(-1), ob[b * T + s])
    y = torch.full((M, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    wo = B.new_workspace(B.LR_OP_LINEAR, M, d, r, d, B.LR_BF16, "decode")
    B.lowrank_linear(G.dev(t["a"]), G.dev(_panels_host(oracle, t["U_o"])), G.dev(_panels_host(oracle, t["V_o"])), None, y, "decode", wo,
                     panels=True)
    B.lowrank_workspace_status(wo)
    assert max_rel_err(G.host64(y), oracle.linear(t["a"].f64, t["U_o"].f64, t["V_o"].f64)) <= TOL["bf16"]
    # packed MLP (benchmark shape); the packed gate/up factor goes through both prepacks on the device
    w = synth.mlp_layer(M)
    t, mm = w.t, w.meta
    pk = lambda name: G.dev(_panels_host(oracle, t[name]))
    U_gu_rm = G.dev(t["U_gu"])
    U_gu_p = torch.zeros_like(U_gu_rm)
    B.lowrank_pack_panels(U_gu_rm, U_gu_p)
    out = torch.full((M, mm["d"]), float("nan"), dtype=torch.bfloat16, device="cuda")
    wm = B.new_workspace(B.LR_OP_PACKED_MLP, M, mm["d"], mm["r_g"] + mm["r_u"] + mm["r_d"], mm["ffn"], B.LR_BF16, "decode")
    bias = lambda n: G.dev(t[n]) if n in t else None
    B.lowrank_packed_mlp(G.dev(t["x"]), U_gu_p, pk("V_g"), pk("V_u"), pk("U_d"), pk("V_d"), bias("b_g"), bias("b_u"), bias("b_d"),
                         out, "decode", wm, panels=True)
    B.lowrank_workspace_status(wm)
    kw = {k: t[k].f64 for k in ("b_g", "b_u", "b_d") if k in t}
    want = oracle.packed_mlp(t["x"].f64, t["U_gu"].f64, t["V_g"].f64, t["V_u"].f64, t["U_d"].f64, t["V_d"].f64, **kw)
    assert max_rel_err(G.host64(out), want) <= TOL["bf16"]


@pytest.mark.parametrize("M,d_in,r,d_out", [(1, 4096, 384, 4096), (7, 1024, 256, 2048), (25, 4096, 384, 4096), (32, 2048, 128, 1024)])
def test_panel_factors_small_integers_exact(G, oracle, M, d_in, r, d_out):
    """Inputs of -1 / 0 / +1 whose every partial sum is a small integer: the result must equal the oracle's bit for bit, so a tile
    or row taken from the wrong place of the panel layout cannot hide under a tolerance."""
    B = G.B
    rng = np.random.default_rng(77 * M + r)
    x = np.zeros((M, d_in)); U = rng.choice([-1.0, 0.0, 1.0], size=(d_in, r)); V = np.zeros((r, d_out))
    for i in range(M):
        x[i, rng.choice(d_in, 8, replace=False)] = rng.choice([-1.0, 1.0], 8)
    for j in range(d_out):
        V[rng.choice(r, 16, replace=False), j] = rng.choice([-1.0, 1.0], 16)
    bias = rng.integers(-3, 4, size=d_out).astype(np.float64)
    xt, Ut, Vt, bt = (synth.to_dtype(a, "bf16") for a in (x, U, V, bias))
    y = torch.full((M, d_out), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = B.new_workspace(B.LR_OP_LINEAR, M, d_in, r, d_out, B.LR_BF16, "decode")
    B.lowrank_linear(G.dev(xt), G.dev(_panels_host(oracle, Ut)), G.dev(_panels_host(oracle, Vt)), G.dev(bt), y, "decode", ws, panels=True)
    B.lowrank_workspace_status(ws)
    assert np.array_equal(G.host64(y), oracle.linear(x, U, V, bias))


def test_panel_factors_outside_the_decode_kernels_are_refused(G):
    B = G.B
    x = torch.zeros((64, 256), dtype=torch.bfloat16, device="cuda")
    U = torch.zeros((256, 128), dtype=torch.bfloat16, device="cuda"); V = torch.zeros((128, 256), dtype=torch.bfloat16, device="cuda")
    y = torch.full((64, 256), 7.0, dtype=torch.bfloat16, device="cuda")
    ws = B.new_workspace(B.LR_OP_LINEAR, 64, 256, 128, 256, B.LR_BF16, "prefill")
    with pytest.raises(B.LowrankError):
        B.lowrank_linear(x, U, V, None, y, "prefill", ws, panels=True)      # 64 rows: prefill kernels do not read panels
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())                                           # nothing was launched
