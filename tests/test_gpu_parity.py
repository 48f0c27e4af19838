"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element,
on the same seeded inputs.  Bar: normwise-max relative error <= 1e-5 (fp32), <= 2e-2 (bf16);
cache writes, packing and untouched memory bit-exact."""
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


# ------------------------------------------------------------------ config 1: fp32 linear
@pytest.mark.parametrize("phase", ["decode", "prefill", "auto"])
def test_config1_linear_f32(G, oracle, phase):
    w = synth.config1()
    y = G.run_linear(w.t["x"], w.t["U"], w.t["V"], None, phase, "f32")
    want = oracle.linear(w.t["x"].f64, w.t["U"].f64, w.t["V"].f64)
    assert max_rel_err(G.host64(y), want) <= TOL["f32"]


# ------------------------------------------------------------------ config 2: decode QKV + O with cache
def run_attention(G, oracle, w, phase):
    B = G.B
    m, t = w.meta, w.t
    M, d, r, H, E, S_max, T = m["M"], m["d"], m["r"], m["n_heads"], m["head_dim"], m["S_max"], m["T"]
    x = G.dev(t["x"])
    Us = [G.dev(t["U_" + n]) for n in "qkv"]
    Vs = [G.dev(t["V_" + n]) for n in "qkv"]
    outs = [torch.full((M, d), float("nan"), dtype=G.tdtype(w.dtype), device="cuda") for _ in range(3)]
    SENT = -65536.0
    kc = torch.full((m["B"], S_max, H, E), SENT, dtype=G.tdtype(w.dtype), device="cuda")
    vc = torch.full((m["B"], S_max, H, E), SENT, dtype=G.tdtype(w.dtype), device="cuda")
    pos = G.dev(m["pos"])
    ws = B.new_workspace(B.LR_OP_QKV, M, d, 3 * r, 3 * d, G.code(w.dtype), phase)
    B.lowrank_qkv(x, Us, Vs, None, outs, dict(k_cache=kc, v_cache=vc, pos=pos, tokens_per_seq=T, k_index=1, v_index=2),
                  phase, ws)
    B.lowrank_workspace_status(ws)
    want = oracle.qkv(t["x"].f64, [t["U_" + n].f64 for n in "qkv"], [t["V_" + n].f64 for n in "qkv"])
    for i in range(3):
        assert max_rel_err(G.host64(outs[i]), want[i]) <= TOL[w.dtype], f"projection {i}"
    # cache: the written slots hold exactly the bits of the k / v outputs, every other slot is untouched
    for cache, o in ((kc, outs[1]), (vc, outs[2])):
        cb, ob = G.bits(cache), G.bits(o)
        expect = G.bits(torch.full_like(cache, SENT))
        for b in range(m["B"]):
            for s in range(T):
                expect[b, m["pos"][b] + s] = ob[b * T + s].reshape(H, E)
        assert np.array_equal(cb, expect)
    # O projection on the independent input a
    y = G.run_linear(t["a"], t["U_o"], t["V_o"], None, phase, w.dtype)
    assert max_rel_err(G.host64(y), oracle.linear(t["a"].f64, t["U_o"].f64, t["V_o"].f64)) <= TOL[w.dtype]


@pytest.mark.parametrize("Bsz", [1, 4, 16, 24, 25, 32])  # 24 / 25: atomics / bf16 finalisation of the split-K stage
def test_config2_decode_attention(G, oracle, Bsz):
    run_attention(G, oracle, synth.attention_layer(Bsz, S_max=64), "decode")


# ------------------------------------------------------------------ config 3: decode packed MLP
@pytest.mark.parametrize("Bsz", [1, 8, 9, 32])        # 8 / 9: the last row count with atomics, the first with bf16 finalisation
def test_config3_decode_packed_mlp(G, oracle, Bsz):
    w = synth.mlp_layer(Bsz)
    out = G.run_mlp(w, "decode")
    t = w.t
    want = oracle.packed_mlp(t["x"].f64, t["U_gu"].f64, t["V_g"].f64, t["V_u"].f64, t["U_d"].f64, t["V_d"].f64)
    assert max_rel_err(G.host64(out), want) <= TOL["bf16"]


# ------------------------------------------------------------------ config 4: prefill, mixed ranks, row-sampled oracle
PREFILL_CASES = [  # (S, attention rank, mlp rank)
    (512, 384, 768), (512, 256, 256), (2048, 512, 512), (2048, 1024, 1024), (8192, 384, 768), (8192, 1024, 1024)]


@pytest.mark.parametrize("S,r_attn,r_mlp", PREFILL_CASES)
def test_config4_prefill_layer(G, oracle, S, r_attn, r_mlp):
    B = G.B
    rows = synth.prefill_row_sample(S, tile=256 if S > 2048 else 128, per_tile=1)
    # attention projections: one sequence of S tokens, cache [1, S, 32, 128], pos 0
    w = synth.attention_layer(1, r=r_attn, S_max=S, T=S, seed=synth.seed_for(4, r_attn))
    m, t = w.meta, w.t
    d, H, E = m["d"], m["n_heads"], m["head_dim"]
    x = G.dev(t["x"])
    Us = [G.dev(t["U_" + n]) for n in "qkv"]
    Vs = [G.dev(t["V_" + n]) for n in "qkv"]
    outs = [torch.full((S, d), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(3)]
    kc = torch.full((1, S, H, E), -65536.0, dtype=torch.bfloat16, device="cuda")
    vc = torch.full((1, S, H, E), -65536.0, dtype=torch.bfloat16, device="cuda")
    ws = B.new_workspace(B.LR_OP_QKV, S, d, 3 * r_attn, 3 * d, B.LR_BF16, "prefill")
    B.lowrank_qkv(x, Us, Vs, None, outs, dict(k_cache=kc, v_cache=vc, pos=G.dev(m["pos"]), tokens_per_seq=S,
                                              k_index=1, v_index=2), "prefill", ws)
    torch.cuda.synchronize()
    assert int(m["pos"][0]) == 0
    xs = t["x"].f64[rows]
    want = oracle.qkv(xs, [t["U_" + n].f64 for n in "qkv"], [t["V_" + n].f64 for n in "qkv"])
    for i in range(3):
        assert max_rel_err(G.host64(outs[i][rows]), want[i]) <= TOL["bf16"], f"projection {i}"
    assert np.array_equal(G.bits(kc).reshape(S, d), G.bits(outs[1]))     # whole cache, bit-exact
    assert np.array_equal(G.bits(vc).reshape(S, d), G.bits(outs[2]))
    y = G.run_linear(t["a"], t["U_o"], t["V_o"], None, "prefill", "bf16")
    assert max_rel_err(G.host64(y[rows]), oracle.linear(t["a"].f64[rows], t["U_o"].f64, t["V_o"].f64)) <= TOL["bf16"]
    del outs, kc, vc, x, y
    # packed MLP at the same S
    wm = synth.mlp_layer(S, r_g=r_mlp, r_u=r_mlp, r_d=r_mlp, seed=synth.seed_for(4, 500 + r_mlp))
    out = G.run_mlp(wm, "prefill")
    tm = wm.t
    want = oracle.packed_mlp(tm["x"].f64[rows], tm["U_gu"].f64, tm["V_g"].f64, tm["V_u"].f64, tm["U_d"].f64, tm["V_d"].f64)
    assert max_rel_err(G.host64(out[rows]), want) <= TOL["bf16"]


# ------------------------------------------------------------------ config 5: shared basis (13B shape)
@pytest.mark.parametrize("M,phase", [(16, "decode"), (4096, "prefill")])
def test_config5_shared_basis(G, oracle, M, phase):
    B = G.B
    w = synth.shared_basis(M)
    t, d, r = w.t, w.meta["d"], w.meta["r"]
    x, U = G.dev(t["x"]), G.dev(t["U_sh"])
    Vs = [G.dev(t["V_0"]), G.dev(t["V_1"])]
    outs = [torch.full((M, d), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    ws = B.new_workspace(B.LR_OP_QKV, M, d, 2 * r, 2 * d, B.LR_BF16, phase)
    B.lowrank_qkv(x, [U, U], Vs, None, outs, None, phase, ws)          # same pointer twice: basis used once
    B.lowrank_workspace_status(ws)
    rows = np.arange(M) if M <= 32 else synth.prefill_row_sample(M, tile=256, per_tile=1)
    Uf = t["U_sh"].f64
    want = oracle.qkv(t["x"].f64[rows], [Uf, Uf], [t["V_0"].f64, t["V_1"].f64])
    for i in range(2):
        assert max_rel_err(G.host64(outs[i][rows]), want[i]) <= TOL["bf16"]
    # the aliased call equals two independent single-layer calls up to the order of the fp32
    # split-K additions (a few bf16 ulps at most)
    for i in range(2):
        y = G.run_linear(t["x"], t["U_sh"], t[f"V_{i}"], None, phase, "bf16")
        assert max_rel_err(G.host64(y), G.host64(outs[i])) <= 2.0 ** -6
