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
