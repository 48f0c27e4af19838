"""HIP-graph capture of the decode calls: every replay must reproduce the eager result.
The library records no memset nodes (workspace areas are cleared by its own kernels)."""
import numpy as np
import pytest

from paper_2605_08314_amd import synth
from util import TOL, max_rel_err

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def test_graph_replays_match_eager_and_oracle(oracle):
    import gpu_util as G
    B = G.B
    wa = synth.attention_layer(4, d=1024, r=128, n_heads=8, S_max=8, seed=41)
    wm = synth.mlp_layer(4, d=1024, ffn=2816, r_g=192, r_u=192, r_d=192, seed=42)
    ta, tm, m = wa.t, wm.t, wa.meta
    x = G.dev(ta["x"])
    Us, Vs = [G.dev(ta["U_" + n]) for n in "qkv"], [G.dev(ta["V_" + n]) for n in "qkv"]
    mlp_w = [G.dev(tm[n]) for n in ("U_gu", "V_g", "V_u", "U_d", "V_d")]
    xm = G.dev(tm["x"])
    outs = [torch.zeros((4, 1024), dtype=torch.bfloat16, device="cuda") for _ in range(3)]
    om = torch.zeros((4, 1024), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((4, 8, 8, 128), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    pos = G.dev(m["pos"])
    ws1 = B.new_workspace(B.LR_OP_QKV, 4, 1024, 384, 3072, B.LR_BF16, "decode")
    ws2 = B.new_workspace(B.LR_OP_PACKED_MLP, 4, 1024, 576, 2816, B.LR_BF16, "decode")

    def body():
        B.lowrank_qkv(x, Us, Vs, None, outs, dict(k_cache=kc, v_cache=vc, pos=pos, tokens_per_seq=1, k_index=1, v_index=2),
                      "decode", ws1)
        B.lowrank_packed_mlp(xm, *mlp_w, None, None, None, om, "decode", ws2)

    body()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs] + [om.clone()]
    want = oracle.qkv(ta["x"].f64, [ta["U_" + n].f64 for n in "qkv"], [ta["V_" + n].f64 for n in "qkv"])
    want.append(oracle.packed_mlp(tm["x"].f64, tm["U_gu"].f64, tm["V_g"].f64, tm["V_u"].f64, tm["U_d"].f64, tm["V_d"].f64))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        body()
    for rep in range(4):
        for o in outs + [om]:
            o.fill_(float("nan"))                       # eager work between the replays
        kc.zero_(); vc.zero_()
        if rep == 2:
            body()                                      # an eager call on the same workspaces in between
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        B.lowrank_workspace_status(ws1)
        B.lowrank_workspace_status(ws2)
        for got, e, w in zip(outs + [om], eager, want):
            assert max_rel_err(G.host64(got), w) <= TOL["bf16"], rep
            assert max_rel_err(G.host64(got), G.host64(e)) <= 2.0 ** -6, rep
        for b in range(4):
            assert np.array_equal(G.bits(kc)[b, m["pos"][b]].reshape(-1), G.bits(outs[1])[b])


@pytest.mark.parametrize("M", [1, 4, 12])
def test_back_to_back_calls_with_different_inputs_inside_one_graph(oracle, M):
    """Six calls per entry point on ONE workspace, inputs cycling through three different ones, recorded in a graph: the
    calls follow each other without any host synchronisation, and the accumulator area a call uses was last used two
    calls earlier with another input.  Anything of that earlier call that survived -- in the area, or as a cached copy of
    its lines -- would make calls 2 .. 5 wrong.  (After the barrier of a stage its input is read with plain cached loads.)"""
    import gpu_util as G
    B = G.B
    wm = [synth.mlp_layer(M, d=1024, ffn=2816, r_g=192, r_u=192, r_d=192, seed=300 + k) for k in range(3)]
    wa = [synth.attention_layer(M, d=1024, r=128, n_heads=8, S_max=8, seed=310 + k) for k in range(3)]
    mlp_w = [G.dev(wm[0].t[n]) for n in ("U_gu", "V_g", "V_u", "U_d", "V_d")]           # one set of factors,
    Us = [G.dev(wa[0].t["U_" + n]) for n in "qkv"]; Vs = [G.dev(wa[0].t["V_" + n]) for n in "qkv"]
    xm = [G.dev(w.t["x"]) for w in wm]                                                      # three different inputs
    xa = [G.dev(w.t["x"]) for w in wa]
    om = [torch.zeros((M, 1024), dtype=torch.bfloat16, device="cuda") for _ in range(6)]
    oq = [[torch.zeros((M, 1024), dtype=torch.bfloat16, device="cuda") for _ in range(3)] for _ in range(6)]
    ws_m = B.new_workspace(B.LR_OP_PACKED_MLP, M, 1024, 576, 2816, B.LR_BF16, "decode")
    ws_q = B.new_workspace(B.LR_OP_QKV, M, 1024, 384, 3072, B.LR_BF16, "decode")
    t0 = wm[0].t
    want_m = [oracle.packed_mlp(w.t["x"].f64, t0["U_gu"].f64, t0["V_g"].f64, t0["V_u"].f64, t0["U_d"].f64, t0["V_d"].f64) for w in wm]
    a0 = wa[0].t
    want_q = [oracle.qkv(w.t["x"].f64, [a0["U_" + n].f64 for n in "qkv"], [a0["V_" + n].f64 for n in "qkv"]) for w in wa]

    def body():
        for i in range(6):
            B.lowrank_packed_mlp(xm[i % 3], *mlp_w, None, None, None, om[i], "decode", ws_m)
            B.lowrank_qkv(xa[i % 3], Us, Vs, None, oq[i], None, "decode", ws_q)

    body()                                             # eager once (also warms everything up)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        body()
    for rep in range(3):
        for o in om: o.fill_(float("nan"))
        for os_ in oq:
            for o in os_: o.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        B.lowrank_workspace_status(ws_m)
        B.lowrank_workspace_status(ws_q)
        for i in range(6):
            assert max_rel_err(G.host64(om[i]), want_m[i % 3]) <= TOL["bf16"], (rep, i)
            for p in range(3):
                assert max_rel_err(G.host64(oq[i][p]), want_q[i % 3][p]) <= TOL["bf16"], (rep, i, p)


def test_back_to_back_calls_at_the_benchmark_layer_size(oracle):
    """The same at the benchmark's layer size (d = 4096, ffn = 11008, ranks 768, one row): the full grid of 256 workgroups on
    all XCDs, three different inputs cycling over six calls of the packed MLP inside one graph."""
    import gpu_util as G
    B = G.B
    ws = [synth.mlp_layer(1, seed=400 + k) for k in range(3)]
    t0 = ws[0].t
    mlp_w = [G.dev(t0[n]) for n in ("U_gu", "V_g", "V_u", "U_d", "V_d")]
    xs = [G.dev(w.t["x"]) for w in ws]
    d, ffn = t0["x"].f64.shape[1], t0["V_g"].f64.shape[1]
    outs = [torch.zeros((1, d), dtype=torch.bfloat16, device="cuda") for _ in range(6)]
    wsp = B.new_workspace(B.LR_OP_PACKED_MLP, 1, d, t0["U_gu"].f64.shape[1] + t0["U_d"].f64.shape[1], ffn, B.LR_BF16, "decode")
    want = [oracle.packed_mlp(w.t["x"].f64, t0["U_gu"].f64, t0["V_g"].f64, t0["V_u"].f64, t0["U_d"].f64, t0["V_d"].f64) for w in ws]

    def body():
        for i in range(6):
            B.lowrank_packed_mlp(xs[i % 3], *mlp_w, None, None, None, outs[i], "decode", wsp)

    body()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        body()
    for rep in range(3):
        for o in outs: o.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        B.lowrank_workspace_status(wsp)
        for i in range(6):
            assert max_rel_err(G.host64(outs[i]), want[i % 3]) <= TOL["bf16"], (rep, i)
