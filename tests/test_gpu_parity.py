"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element,
on the same seeded inputs.  Bar: normwise-max relative error <= 1e-5 (fp32), <= 2e-2 (bf16);
cache writes, packing and untouched memory bit-exact."""
import numpy as np
import pytest

from paper_2605_08314_amd import synth
from util import TOL, diag_report, max_rel_err

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
    faithful = oracle.diag_qkv(t["x"].f64, [t["U_" + n].f64 for n in "qkv"], [t["V_" + n].f64 for n in "qkv"])
    for i in range(3):
        diag_report(f"config 2 {phase} B={M} projection {'qkv'[i]}", G.host64(outs[i]), want[i], faithful[i])
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
    diag_report(f"config 2 {phase} B={M} O projection", G.host64(y), oracle.linear(t["a"].f64, t["U_o"].f64, t["V_o"].f64),
                oracle.diag_linear(t["a"].f64, t["U_o"].f64, t["V_o"].f64))
    assert max_rel_err(G.host64(y), oracle.linear(t["a"].f64, t["U_o"].f64, t["V_o"].f64)) <= TOL[w.dtype]


@pytest.mark.parametrize("Bsz", [1, 4, 16, 17, 25, 32])  # 16 / 17: one / two 16-row blocks per wave
def test_config2_decode_attention(G, oracle, Bsz):
    run_attention(G, oracle, synth.attention_layer(Bsz, S_max=64), "decode")


# ------------------------------------------------------------------ config 3: decode packed MLP
@pytest.mark.parametrize("Bsz", [1, 8, 16, 17, 24, 25, 32])   # 16 / 17: one / two 16-row blocks per wave; 24 / 25: the last row count with atomics, the first with bf16 finalisation
def test_config3_decode_packed_mlp(G, oracle, Bsz):
    w = synth.mlp_layer(Bsz)
    out = G.run_mlp(w, "decode")
    t = w.t
    want = oracle.packed_mlp(t["x"].f64, t["U_gu"].f64, t["V_g"].f64, t["V_u"].f64, t["U_d"].f64, t["V_d"].f64)
    diag_report(f"config 3 decode B={Bsz} packed MLP", G.host64(out), want,
                oracle.diag_packed_mlp(t["x"].f64, t["U_gu"].f64, t["V_g"].f64, t["V_u"].f64, t["U_d"].f64, t["V_d"].f64))
    assert max_rel_err(G.host64(out), want) <= TOL["bf16"]


# ------------------------------------------------------------------ config 4: prefill, mixed ranks, row-sampled oracle
PREFILL_RANKS = [(384, 768), (256, 256), (512, 512), (1024, 1024)]   # the four layers of the mixed-rank stack
PREFILL_CASES = [(S, ra, rm) for S in (512, 2048, 8192) for ra, rm in PREFILL_RANKS]


def prefill_rows(S):
    """Rows compared with the oracle: every row at S = 512; for longer inputs the first and last row of every tile
    of the tallest kernel tile in use plus one seeded row per tile (rows are independent of each other)."""
    if S <= 512:
        return np.arange(S)
    return synth.prefill_row_sample(S, tile=256 if S > 2048 else 128, per_tile=1)


@pytest.mark.parametrize("S,r_attn,r_mlp", PREFILL_CASES)
def test_config4_prefill_layer(G, oracle, S, r_attn, r_mlp):
    B = G.B
    rows = prefill_rows(S)
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
    B.lowrank_workspace_status(ws)
    assert int(m["pos"][0]) == 0
    xs = t["x"].f64[rows]
    Uf, Vf = [t["U_" + n].f64 for n in "qkv"], [t["V_" + n].f64 for n in "qkv"]
    want = oracle.qkv(xs, Uf, Vf)
    faithful = oracle.diag_qkv(xs, Uf, Vf)
    for i in range(3):
        got = G.host64(outs[i])
        assert np.isfinite(got).all()
        diag_report(f"config 4 S={S} r={r_attn} projection {'qkv'[i]}", got[rows], want[i], faithful[i])
        assert max_rel_err(got[rows], want[i]) <= TOL["bf16"], f"projection {i}"
    assert np.array_equal(G.bits(kc).reshape(S, d), G.bits(outs[1]))     # whole cache, bit-exact
    assert np.array_equal(G.bits(vc).reshape(S, d), G.bits(outs[2]))
    y = G.run_linear(t["a"], t["U_o"], t["V_o"], None, "prefill", "bf16")
    want_o = oracle.linear(t["a"].f64[rows], t["U_o"].f64, t["V_o"].f64)
    diag_report(f"config 4 S={S} r={r_attn} O projection", G.host64(y[rows]), want_o,
                oracle.diag_linear(t["a"].f64[rows], t["U_o"].f64, t["V_o"].f64))
    assert max_rel_err(G.host64(y[rows]), want_o) <= TOL["bf16"]
    del outs, kc, vc, x, y
    # packed MLP at the same S
    wm = synth.mlp_layer(S, r_g=r_mlp, r_u=r_mlp, r_d=r_mlp, seed=synth.seed_for(4, 500 + r_mlp))
    out = G.run_mlp(wm, "prefill")
    tm = wm.t
    margs = [tm[n].f64 for n in ("U_gu", "V_g", "V_u", "U_d", "V_d")]
    want = oracle.packed_mlp(tm["x"].f64[rows], *margs)
    got = G.host64(out)
    assert np.isfinite(got).all()
    diag_report(f"config 4 S={S} r={r_mlp} packed MLP", got[rows], want, oracle.diag_packed_mlp(tm["x"].f64[rows], *margs))
    assert max_rel_err(got[rows], want) <= TOL["bf16"]


def test_config4_four_layer_stack(G, oracle):
    """The four layers of the mixed-rank stack (ranks 384/768, 256, 512, 1024) run back to back at S = 512, each
    consuming what the one before produced, on ONE workspace per entry point shared by all layers (sized for the
    largest rank).  Every call's output is checked against the oracle applied to the very input that call
    received on the GPU (bf16 bits widened exactly), so each layer is judged on its own while running in the
    stack; the drift of the whole chain against an fp64 chain is reported, and bounded by the sum of its steps.
    (The attention between the projections is not part of this path: the O projection takes q.)"""
    B = G.B
    S, d, H, E = 512, 4096, 32, 128
    layers = []
    for li, (ra, rm) in enumerate(PREFILL_RANKS):
        wa = synth.attention_layer(1, r=ra, S_max=S, T=S, seed=synth.seed_for(4, 700 + li))
        wm = synth.mlp_layer(1, r_g=rm, r_u=rm, r_d=rm, seed=synth.seed_for(4, 800 + li))
        layers.append((ra, rm, wa.t, wm.t))
    x0 = synth.to_dtype(np.random.default_rng(synth.seed_for(4, 900)).standard_normal((S, d)), "bf16")
    ws_q = B.new_workspace(B.LR_OP_QKV, S, d, 3 * 1024, 3 * d, B.LR_BF16, "prefill")
    ws_o = B.new_workspace(B.LR_OP_LINEAR, S, d, 1024, d, B.LR_BF16, "prefill")
    ws_m = B.new_workspace(B.LR_OP_PACKED_MLP, S, d, 3 * 1024, 11008, B.LR_BF16, "prefill")
    pos = torch.zeros((1,), dtype=torch.int32, device="cuda")
    dev_layers = []
    for ra, rm, ta, tm in layers:
        dev_layers.append(dict(Us=[G.dev(ta["U_" + n]) for n in "qkv"], Vs=[G.dev(ta["V_" + n]) for n in "qkv"],
                               Uo=G.dev(ta["U_o"]), Vo=G.dev(ta["V_o"]),
                               mlp=[G.dev(tm[n]) for n in ("U_gu", "V_g", "V_u", "U_d", "V_d")],
                               kc=torch.full((1, S, H, E), -65536.0, dtype=torch.bfloat16, device="cuda"),
                               vc=torch.full((1, S, H, E), -65536.0, dtype=torch.bfloat16, device="cuda")))
    h = G.dev(x0)
    trace = []                                  # (input, outputs) of every call, kept on the device until the stack has run
    for L in dev_layers:
        q, k, v = (torch.full((S, d), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(3))
        B.lowrank_qkv(h, L["Us"], L["Vs"], None, [q, k, v],
                      dict(k_cache=L["kc"], v_cache=L["vc"], pos=pos, tokens_per_seq=S, k_index=1, v_index=2), "prefill", ws_q)
        o = torch.full((S, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.lowrank_linear(q, L["Uo"], L["Vo"], None, o, "prefill", ws_o)
        hn = torch.full((S, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.lowrank_packed_mlp(o, *L["mlp"], None, None, None, hn, "prefill", ws_m)
        trace.append((h, q, k, v, o, hn))
        h = hn
    for w in (ws_q, ws_o, ws_m):
        B.lowrank_workspace_status(w)
    rows = synth.prefill_row_sample(S, tile=128, per_tile=1)
    chain = x0.f64[rows]                        # the fp64 chain on the sampled rows (rows never mix on this path)
    for li, ((ra, rm, ta, tm), L, (hin, q, k, v, o, hn)) in enumerate(zip(layers, dev_layers, trace)):
        Uf, Vf = [ta["U_" + n].f64 for n in "qkv"], [ta["V_" + n].f64 for n in "qkv"]
        want = oracle.qkv(G.host64(hin)[rows], Uf, Vf)
        for name, got, wnt in zip("qkv", (q, k, v), want):
            assert max_rel_err(G.host64(got)[rows], wnt) <= TOL["bf16"], (li, name)
        assert np.array_equal(G.bits(L["kc"]).reshape(S, d), G.bits(k)) and np.array_equal(G.bits(L["vc"]).reshape(S, d), G.bits(v))
        assert max_rel_err(G.host64(o)[rows], oracle.linear(G.host64(q)[rows], ta["U_o"].f64, ta["V_o"].f64)) <= TOL["bf16"], li
        margs = [tm[n].f64 for n in ("U_gu", "V_g", "V_u", "U_d", "V_d")]
        assert max_rel_err(G.host64(hn)[rows], oracle.packed_mlp(G.host64(o)[rows], *margs)) <= TOL["bf16"], li
        chain = oracle.packed_mlp(oracle.linear(oracle.qkv(chain, Uf, Vf)[0], ta["U_o"].f64, ta["V_o"].f64), *margs)
        drift = max_rel_err(G.host64(hn)[rows], chain)
        diag_report(f"config 4 stack S={S}: after layer {li} (ranks {ra}/{rm}), whole chain", G.host64(hn)[rows], chain, gate_blocks=False)
        assert drift <= 3 * (li + 1) * TOL["bf16"]          # three calls per layer, each within the tolerance


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
    faithful = oracle.diag_qkv(t["x"].f64[rows], [Uf, Uf], [t["V_0"].f64, t["V_1"].f64])
    for i in range(2):
        diag_report(f"config 5 {phase} M={M} shared basis, layer {i}", G.host64(outs[i][rows]), want[i], faithful[i])
        assert max_rel_err(G.host64(outs[i][rows]), want[i]) <= TOL["bf16"]
    # the aliased call equals two independent single-layer calls up to the order of the fp32
    # split-K additions (a few bf16 ulps at most)
    for i in range(2):
        y = G.run_linear(t["x"], t["U_sh"], t[f"V_{i}"], None, phase, "bf16")
        assert max_rel_err(G.host64(y), G.host64(outs[i])) <= 2.0 ** -6
