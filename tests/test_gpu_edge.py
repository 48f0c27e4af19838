"""GPU edge cases through the C ABI: degenerate sizes, ragged and unaligned shapes, biases,
multi-token cache writes, packing, phase AUTO, error codes."""
import numpy as np
import pytest

from paper_2605_08314_amd import synth
from util import TOL, max_rel_err

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def G():
    import gpu_util
    assert torch.cuda.is_available()
    return gpu_util


def rand_t(rng, shape, dtype, scale=1.0):
    return synth.to_dtype(rng.standard_normal(shape) * scale, dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (3, 37, 5, 19), (7, 130, 33, 257), (33, 512, 64, 512),
                                   (2, 4096, 384, 4096), (5, 1000, 24, 72), (32, 264, 72, 136)])
@pytest.mark.parametrize("phase", ["decode", "prefill"])
def test_linear_shapes_with_bias(G, oracle, dtype, shape, phase):
    M, d_in, r, d_out = shape
    rng = np.random.default_rng(hash(shape) % 2**31)
    x = rand_t(rng, (M, d_in), dtype)
    U = rand_t(rng, (d_in, r), dtype, d_in ** -0.5)
    V = rand_t(rng, (r, d_out), dtype, r ** -0.5)
    b = rand_t(rng, (d_out,), dtype)
    for bias in (None, b):
        y = G.run_linear(x, U, V, bias, phase, dtype)
        want = oracle.linear(x.f64, U.f64, V.f64, None if bias is None else bias.f64)
        assert max_rel_err(G.host64(y), want) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_sizes(G, oracle, dtype):
    B = G.B
    td = G.tdtype(dtype)
    rng = np.random.default_rng(5)
    ws = B.new_workspace(B.LR_OP_LINEAR, 4, 64, 8, 32, G.code(dtype))
    # M == 0: no-op, output untouched
    x0 = torch.empty((0, 64), dtype=td, device="cuda")
    U, V = G.dev(rand_t(rng, (64, 8), dtype)), G.dev(rand_t(rng, (8, 32), dtype))
    y0 = torch.empty((0, 32), dtype=td, device="cuda")
    B.lowrank_linear(x0, U, V, None, y0, "auto", ws)
    # r == 0: y = bias, or zeros
    x = rand_t(rng, (4, 64), dtype)
    b = rand_t(rng, (32,), dtype)
    U0 = torch.empty((64, 0), dtype=td, device="cuda")
    V0 = torch.empty((0, 32), dtype=td, device="cuda")
    for bias in (None, b):
        y = torch.full((4, 32), float("nan"), dtype=td, device="cuda")
        B.lowrank_linear(G.dev(x), U0, V0, None if bias is None else G.dev(bias), y, "decode", ws)
        torch.cuda.synchronize()
        want = np.zeros((4, 32)) if bias is None else np.broadcast_to(bias.f64, (4, 32))
        assert np.array_equal(G.host64(y), want)


def test_unaligned_pointers_take_generic_path(G, oracle):
    B = G.B
    rng = np.random.default_rng(6)
    M, d_in, r, d_out = 4, 256, 64, 256
    x, U, V = rand_t(rng, (M, d_in), "bf16"), rand_t(rng, (d_in, r), "bf16", d_in ** -0.5), rand_t(rng, (r, d_out), "bf16", r ** -0.5)
    def shifted(t):           # same values at an address that is only 2-byte aligned
        flat = torch.empty(t.dev.size + 1, dtype=torch.bfloat16, device="cuda")
        view = flat[1:].view(t.dev.shape)
        view.copy_(G.dev(t))
        return view
    y = torch.empty((M, d_out), dtype=torch.bfloat16, device="cuda")
    ws = B.new_workspace(B.LR_OP_LINEAR, M, d_in, r, d_out, B.LR_BF16)
    B.lowrank_linear(shifted(x), shifted(U), shifted(V), None, y, "decode", ws)
    torch.cuda.synchronize()
    assert max_rel_err(G.host64(y), oracle.linear(x.f64, U.f64, V.f64)) <= TOL["bf16"]


@pytest.mark.parametrize("phase", ["decode", "prefill"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_qkv_multi_token_cache_bias_and_null_out(G, oracle, phase, dtype):
    B = G.B
    rng = np.random.default_rng(7)
    Bn, T, H, E, S_max, d_in = 3, 4, 4, 32, 16, 256
    M, d_out = Bn * T, H * E
    ranks = (64, 128, 64)
    x = rand_t(rng, (M, d_in), dtype)
    Us = [rand_t(rng, (d_in, r), dtype, d_in ** -0.5) for r in ranks]
    Vs = [rand_t(rng, (r, d_out), dtype, r ** -0.5) for r in ranks]
    bs = [rand_t(rng, (d_out,), dtype), None, rand_t(rng, (d_out,), dtype)]
    pos = np.array([0, 12, 5], dtype=np.int32)
    td = G.tdtype(dtype)
    kc = torch.full((Bn, S_max, H, E), -65536.0, dtype=td, device="cuda")
    vc = torch.full((Bn, S_max, H, E), -65536.0, dtype=td, device="cuda")
    q = torch.full((M, d_out), float("nan"), dtype=td, device="cuda")
    k = torch.full((M, d_out), float("nan"), dtype=td, device="cuda")
    ws = B.new_workspace(B.LR_OP_QKV, M, d_in, sum(ranks), 3 * d_out, G.code(dtype), phase)
    B.lowrank_qkv(G.dev(x), [G.dev(u) for u in Us], [G.dev(v) for v in Vs],
                  [None if b is None else G.dev(b) for b in bs], [q, k, None],       # V only to the cache
                  dict(k_cache=kc, v_cache=vc, pos=G.dev(pos), tokens_per_seq=T, k_index=1, v_index=2), phase, ws)
    torch.cuda.synchronize()
    SENT = -65536.0
    okc = np.full((Bn, S_max, H, E), SENT)
    ovc = np.full((Bn, S_max, H, E), SENT)
    want = oracle.qkv(x.f64, [u.f64 for u in Us], [v.f64 for v in Vs], [None if b is None else b.f64 for b in bs],
                      kv=dict(k_cache=okc, v_cache=ovc, pos=pos, T=T, k_index=1, v_index=2))
    assert max_rel_err(G.host64(q), want[0]) <= TOL[dtype]
    assert max_rel_err(G.host64(k), want[1]) <= TOL[dtype]
    written = okc != SENT
    assert np.array_equal(G.host64(kc) != SENT, written)             # same slots as the oracle's scatter
    assert np.array_equal(G.host64(vc) != SENT, ovc != SENT)
    assert max_rel_err(G.host64(vc)[ovc != SENT], ovc[ovc != SENT]) <= TOL[dtype]
    kb = G.bits(kc)
    for b in range(Bn):
        for s in range(T):
            assert np.array_equal(kb[b, pos[b] + s].reshape(-1), G.bits(k)[b * T + s])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_pack_concat_bit_exact(G, oracle, dtype):
    B = G.B
    rng = np.random.default_rng(8)
    d_in = 192
    Us = [rand_t(rng, (d_in, r), dtype, d_in ** -0.5) for r in (64, 128, 64)]
    Ud = [G.dev(u) for u in Us]
    packed = torch.zeros((d_in, 256), dtype=G.tdtype(dtype), device="cuda")
    B.lowrank_pack_concat(Ud, packed)
    torch.cuda.synchronize()
    want = oracle.pack_concat([u.dev for u in Us])
    want_bits = want.view(np.uint32) if want.dtype == np.float32 else want
    assert np.array_equal(G.bits(packed), want_bits)


@pytest.mark.parametrize("M,phase", [(1, "decode"), (8, "decode"), (20, "decode"), (300, "prefill")])
def test_pack_concat_output_feeds_packed_mlp_and_qkv(G, oracle, M, phase):
    """The offline prepack in use: U_gu = lowrank_pack_concat(U_gate, U_up) goes into lowrank_packed_mlp, and a
    rank-concatenated factor [U_a | U_b] (with V_a stacked on V_b) goes into lowrank_qkv as one projection next to
    an ordinary one.  Expected values come from the oracle on the separate factors."""
    B = G.B
    w = synth.mlp_layer(M, d=1024, ffn=2816, r_g=192, r_u=320, r_d=128, seed=515 + M, dtype="bf16", with_bias=True)
    t = w.t
    U_gu = torch.full((1024, 512), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.lowrank_pack_concat([G.dev(t["U_g"]), G.dev(t["U_u"])], U_gu)
    out = torch.full((M, 1024), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = B.new_workspace(B.LR_OP_PACKED_MLP, M, 1024, 192 + 320 + 128, 2816, B.LR_BF16, phase)
    B.lowrank_packed_mlp(G.dev(t["x"]), U_gu, G.dev(t["V_g"]), G.dev(t["V_u"]), G.dev(t["U_d"]), G.dev(t["V_d"]),
                         G.dev(t["b_g"]), G.dev(t["b_u"]), G.dev(t["b_d"]), out, phase, ws)
    B.lowrank_workspace_status(ws)
    want = oracle.packed_mlp(t["x"].f64, oracle.pack_concat([t["U_g"].f64, t["U_u"].f64]), t["V_g"].f64, t["V_u"].f64,
                             t["U_d"].f64, t["V_d"].f64, t["b_g"].f64, t["b_u"].f64, t["b_d"].f64)
    assert max_rel_err(G.host64(out), want) <= TOL["bf16"]
    # qkv: projection 0 uses the packed pair, projection 1 an ordinary factor pair
    rng = np.random.default_rng(616 + M)
    d_in, d_out = 512, 1024
    Ua, Ub, Uc = (rand_t(rng, (d_in, r), "bf16", d_in ** -0.5) for r in (64, 128, 192))
    Va, Vb, Vc = (rand_t(rng, (r, d_out), "bf16", r ** -0.5) for r in (64, 128, 192))
    x = rand_t(rng, (M, d_in), "bf16")
    Uab = torch.full((d_in, 192), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.lowrank_pack_concat([G.dev(Ua), G.dev(Ub)], Uab)
    Vab = torch.cat([G.dev(Va), G.dev(Vb)], dim=0).contiguous()
    outs = [torch.full((M, d_out), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    ws = B.new_workspace(B.LR_OP_QKV, M, d_in, 384, 2 * d_out, B.LR_BF16, phase)
    B.lowrank_qkv(G.dev(x), [Uab, G.dev(Uc)], [Vab, G.dev(Vc)], None, outs, None, phase, ws)
    B.lowrank_workspace_status(ws)
    want0 = oracle.linear(x.f64, Ua.f64, Va.f64) + oracle.linear(x.f64, Ub.f64, Vb.f64)     # separate factors, summed
    assert max_rel_err(G.host64(outs[0]), want0) <= TOL["bf16"]
    assert max_rel_err(G.host64(outs[1]), oracle.linear(x.f64, Uc.f64, Vc.f64)) <= TOL["bf16"]


@pytest.mark.parametrize("M", [1, 5, 32, 40, 300])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_packed_mlp_small_with_bias_and_uneven_ranks(G, oracle, M, dtype):
    w = synth.mlp_layer(M, d=256, ffn=448, r_g=64, r_u=128, r_d=64, seed=99 + M, dtype=dtype, with_bias=True)
    t = w.t
    for phase in ("decode", "prefill"):
        out = G.run_mlp(w, phase)
        want = oracle.packed_mlp(t["x"].f64, t["U_gu"].f64, t["V_g"].f64, t["V_u"].f64, t["U_d"].f64, t["V_d"].f64,
                                 t["b_g"].f64, t["b_u"].f64, t["b_d"].f64)
        assert max_rel_err(G.host64(out), want) <= TOL[dtype], phase


def test_packed_mlp_ragged_generic(G, oracle):
    w = synth.mlp_layer(3, d=100, ffn=77, r_g=5, r_u=9, r_d=6, seed=123, dtype="bf16", with_bias=True)
    t = w.t
    out = G.run_mlp(w, "decode")
    want = oracle.packed_mlp(t["x"].f64, t["U_gu"].f64, t["V_g"].f64, t["V_u"].f64, t["U_d"].f64, t["V_d"].f64,
                             t["b_g"].f64, t["b_u"].f64, t["b_d"].f64)
    assert max_rel_err(G.host64(out), want) <= TOL["bf16"]


@pytest.mark.parametrize("M", [1, 32, 33, 200])
def test_phase_auto_equals_explicit(G, M):
    rng = np.random.default_rng(9)
    x, U, V = rand_t(rng, (M, 512), "bf16"), rand_t(rng, (512, 128), "bf16", 512 ** -0.5), rand_t(rng, (128, 512), "bf16", 128 ** -0.5)
    ya = G.run_linear(x, U, V, None, "auto", "bf16")
    ye = G.run_linear(x, U, V, None, "decode" if M <= 32 else "prefill", "bf16")
    # same kernels either way; split-K sums may be added in a different order between two runs
    assert max_rel_err(G.host64(ya), G.host64(ye)) <= 2.0 ** -6
    B = G.B
    want = "decode" if M <= 32 else "prefill"
    assert B.lowrank_plan_name(B.LR_OP_LINEAR, M, 512, 128, 512, B.LR_BF16, "auto") == \
        B.lowrank_plan_name(B.LR_OP_LINEAR, M, 512, 128, 512, B.LR_BF16, want)


def test_repeat_calls_same_workspace_are_bit_identical(G):
    B = G.B
    w = synth.attention_layer(8, d=1024, r=128, n_heads=8, S_max=8)
    t = w.t
    x, U, V = G.dev(t["x"]), G.dev(t["U_q"]), G.dev(t["V_q"])
    ws = B.new_workspace(B.LR_OP_LINEAR, 8, 1024, 128, 1024, B.LR_BF16)
    ys = []
    for _ in range(4):
        y = torch.empty((8, 1024), dtype=torch.bfloat16, device="cuda")
        B.lowrank_linear(x, U, V, None, y, "decode", ws)
        ys.append(y)
    torch.cuda.synchronize()
    # same workspace reused: later calls must not see leftovers of earlier ones
    for y in ys[1:]:
        assert max_rel_err(G.host64(y), G.host64(ys[0])) <= 1e-2
    # a smaller call after a larger one on the same workspace
    y2 = torch.empty((2, 1024), dtype=torch.bfloat16, device="cuda")
    B.lowrank_linear(x[:2].contiguous(), U, V, None, y2, "decode", ws)
    torch.cuda.synchronize()
    assert max_rel_err(G.host64(y2), G.host64(ys[0][:2])) <= 1e-2


def test_mixed_calls_share_one_workspace(G, oracle):
    """qkv, linear and MLP calls of different sizes interleaved on ONE workspace: the split-K
    accumulator areas must be clean for every call whatever ran before."""
    B = G.B
    wa = synth.attention_layer(8, d=1024, r=128, n_heads=8, S_max=8, seed=31)
    wm = synth.mlp_layer(8, d=1024, ffn=2816, r_g=192, r_u=192, r_d=192, seed=32)
    ta, tm = wa.t, wm.t
    nbytes = max(B.lowrank_workspace_bytes(B.LR_OP_QKV, 8, 1024, 384, 3072, B.LR_BF16, "decode"),
                 B.lowrank_workspace_bytes(B.LR_OP_PACKED_MLP, 8, 1024, 576, 2816, B.LR_BF16, "decode"))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 256)     # never prepared: the first call does it
    x = G.dev(ta["x"])
    Us, Vs = [G.dev(ta["U_" + n]) for n in "qkv"], [G.dev(ta["V_" + n]) for n in "qkv"]
    mlp_w = [G.dev(tm[n]) for n in ("U_gu", "V_g", "V_u", "U_d", "V_d")]
    xm = G.dev(tm["x"])
    want_qkv = oracle.qkv(ta["x"].f64, [ta["U_" + n].f64 for n in "qkv"], [ta["V_" + n].f64 for n in "qkv"])
    want_mlp = oracle.packed_mlp(tm["x"].f64, tm["U_gu"].f64, tm["V_g"].f64, tm["V_u"].f64, tm["U_d"].f64, tm["V_d"].f64)
    want_lin2 = oracle.linear(ta["x"].f64[:2], ta["U_q"].f64, ta["V_q"].f64)
    for rep in range(3):
        outs = [torch.full((8, 1024), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(3)]
        B.lowrank_qkv(x, Us, Vs, None, outs, None, "decode", ws)
        om = torch.full((8, 1024), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.lowrank_packed_mlp(xm, *mlp_w, None, None, None, om, "decode", ws)
        y2 = torch.full((2, 1024), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.lowrank_linear(x[:2].contiguous(), Us[0], Vs[0], None, y2, "decode", ws)
        om2 = torch.full((8, 1024), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.lowrank_packed_mlp(xm, *mlp_w, None, None, None, om2, "decode", ws)
        B.lowrank_workspace_status(ws)
        for i in range(3):
            assert max_rel_err(G.host64(outs[i]), want_qkv[i]) <= TOL["bf16"], (rep, i)
        assert max_rel_err(G.host64(om), want_mlp) <= TOL["bf16"], rep
        assert max_rel_err(G.host64(om2), want_mlp) <= TOL["bf16"], rep
        assert max_rel_err(G.host64(y2), want_lin2) <= TOL["bf16"], rep


@pytest.mark.parametrize("M", [4, 16, 32])
def test_alternating_inputs_on_one_workspace(G, oracle, M):
    """Calls with DIFFERENT inputs alternate on one workspace: intermediates of an earlier call that
    survived anywhere (accumulator areas, bf16 copies, caches) would show up as a wrong result."""
    B = G.B
    ws_n = max(B.lowrank_workspace_bytes(B.LR_OP_QKV, M, 1024, 384, 3072, B.LR_BF16, "decode"),
               B.lowrank_workspace_bytes(B.LR_OP_PACKED_MLP, M, 1024, 576, 2816, B.LR_BF16, "decode"))
    ws = torch.empty(ws_n, dtype=torch.uint8, device="cuda").random_(0, 256)      # never prepared: the first call does it
    sets = []
    for k in range(2):
        wa = synth.attention_layer(M, d=1024, r=128, n_heads=8, S_max=8, seed=70 + k)
        wm = synth.mlp_layer(M, d=1024, ffn=2816, r_g=192, r_u=192, r_d=192, seed=80 + k)
        ta, tm = wa.t, wm.t
        sets.append(dict(
            x=G.dev(ta["x"]), Us=[G.dev(ta["U_" + n]) for n in "qkv"], Vs=[G.dev(ta["V_" + n]) for n in "qkv"],
            xm=G.dev(tm["x"]), mlp=[G.dev(tm[n]) for n in ("U_gu", "V_g", "V_u", "U_d", "V_d")],
            want_qkv=oracle.qkv(ta["x"].f64, [ta["U_" + n].f64 for n in "qkv"], [ta["V_" + n].f64 for n in "qkv"]),
            want_mlp=oracle.packed_mlp(tm["x"].f64, tm["U_gu"].f64, tm["V_g"].f64, tm["V_u"].f64, tm["U_d"].f64, tm["V_d"].f64)))
    for rep in range(6):
        sset = sets[rep % 2]
        outs = [torch.full((M, 1024), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(3)]
        om = torch.full((M, 1024), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.lowrank_qkv(sset["x"], sset["Us"], sset["Vs"], None, outs, None, "decode", ws)
        B.lowrank_packed_mlp(sset["xm"], *sset["mlp"], None, None, None, om, "decode", ws)
        B.lowrank_workspace_status(ws)
        for i in range(3):
            assert max_rel_err(G.host64(outs[i]), sset["want_qkv"][i]) <= TOL["bf16"], (rep, i)
        assert max_rel_err(G.host64(om), sset["want_mlp"]) <= TOL["bf16"], rep


def test_error_codes(G):
    B = G.B
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    U = torch.zeros((64, 8), dtype=torch.bfloat16, device="cuda")
    V = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    small = torch.zeros(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.LowrankError) as e:
        B.lowrank_linear(x, U, V, None, y, "decode", small)
    assert e.value.status == -6 and "workspace" in str(e.value)
    ws = B.new_workspace(B.LR_OP_LINEAR, 4, 64, 8, 64, B.LR_BF16)
    with pytest.raises(B.LowrankError) as e:
        B.lowrank_linear(x, U, V, None, y, 7, ws)
    assert e.value.status == -5
    with pytest.raises(B.LowrankError) as e:
        B.lowrank_linear(x, U, V, None, y, "decode", ws[1:])
    assert e.value.status == -4


# ------------------------------------------------------------------ prefill fast path: ragged tiles, several sequences, biases
@pytest.mark.parametrize("case", [
    # (sequences, tokens per sequence, d_in, ranks, heads, head_dim): M = sequences * tokens
    (3, 50, 256, (128, 256, 128), 2, 128),       # small tiles, sequence borders inside a 32-row block, ragged M
    (30, 5, 256, (128, 128, 128), 2, 128),       # fewer than 32 tokens per sequence: per-row cache positions
    (3, 1000, 256, (128, 128, 256), 41, 128),    # 3000 x 5248 outputs: big tiles, ragged in M and in N, mixed ranks
    (600, 5, 256, (128, 128, 128), 41, 128),     # the same with short sequences
])
def test_prefill_qkv_fast_path_cache_bias_ragged(G, oracle, case):
    B = G.B
    Bn, T, d_in, ranks, H, E = case
    M, d_out, S_max = Bn * T, H * E, T + 24
    rng = np.random.default_rng(1000 + M + H)
    x = rand_t(rng, (M, d_in), "bf16")
    Us = [rand_t(rng, (d_in, r), "bf16", d_in ** -0.5) for r in ranks]
    Vs = [rand_t(rng, (r, d_out), "bf16", r ** -0.5) for r in ranks]
    bs = [rand_t(rng, (d_out,), "bf16"), None, rand_t(rng, (d_out,), "bf16")]
    pos = rng.integers(0, 24, size=Bn).astype(np.int32)
    assert B.lowrank_plan_name(B.LR_OP_QKV, M, d_in, sum(ranks), 3 * d_out, B.LR_BF16, "prefill", 1) == "prefill_mfma"
    SENT = -65536.0
    kc = torch.full((Bn, S_max, H, E), SENT, dtype=torch.bfloat16, device="cuda")
    vc = torch.full((Bn, S_max, H, E), SENT, dtype=torch.bfloat16, device="cuda")
    q = torch.full((M, d_out), float("nan"), dtype=torch.bfloat16, device="cuda")
    v = torch.full((M, d_out), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = B.new_workspace(B.LR_OP_QKV, M, d_in, sum(ranks), 3 * d_out, B.LR_BF16, "prefill")
    B.lowrank_qkv(G.dev(x), [G.dev(u) for u in Us], [G.dev(w) for w in Vs],
                  [None if b is None else G.dev(b) for b in bs], [q, None, v],        # K only to the cache
                  dict(k_cache=kc, v_cache=vc, pos=G.dev(pos), tokens_per_seq=T, k_index=1, v_index=2), "prefill", ws)
    B.lowrank_workspace_status(ws)
    # the oracle on a row sample: tile borders, sequence borders, the ragged tail, and seeded rows
    rows = sorted(set([0, 1, 31, 32, 127, 128, 255, 256, M - 257, M - 129, M - 2, M - 1] +
                      [b * T for b in range(0, Bn, max(1, Bn // 7))] + [b * T + T - 1 for b in range(0, Bn, max(1, Bn // 5))] +
                      list(rng.integers(0, M, size=24))))
    rows = [r for r in rows if 0 <= r < M]
    want = oracle.qkv(x.f64[rows], [u.f64 for u in Us], [w.f64 for w in Vs], [None if b is None else b.f64 for b in bs])
    assert max_rel_err(G.host64(q[rows]), want[0]) <= TOL["bf16"]
    assert max_rel_err(G.host64(v[rows]), want[2]) <= TOL["bf16"]
    kh, vh = G.host64(kc), G.host64(vc)
    for i, m in enumerate(rows):
        b, s = divmod(m, T)
        assert max_rel_err(kh[b, pos[b] + s].reshape(1, -1), want[1][i:i + 1]) <= TOL["bf16"]
    # every slot: written exactly where a token belongs, V cache bit-identical to the V output
    written = np.zeros((Bn, S_max), dtype=bool)
    for b in range(Bn):
        written[b, pos[b]:pos[b] + T] = True
    assert np.array_equal((kh != SENT).all(axis=(2, 3)), written) and np.array_equal((kh != SENT).any(axis=(2, 3)), written)
    assert np.array_equal((vh != SENT).any(axis=(2, 3)), written)
    vb, ob = G.bits(vc), G.bits(v)
    for b in range(0, Bn, max(1, Bn // 11)):
        assert np.array_equal(vb[b, pos[b]:pos[b] + T].reshape(T, d_out), ob[b * T:(b + 1) * T])


@pytest.mark.parametrize("M", [300, 1000])
def test_prefill_mlp_fast_path_with_bias(G, oracle, M):
    w = synth.mlp_layer(M, d=512, ffn=1024, r_g=128, r_u=256, r_d=128, seed=321 + M, dtype="bf16", with_bias=True)
    out = G.run_mlp(w, "prefill")          # every dimension fits the MFMA path: K % 64 == 0, N % 128 == 0
    t = w.t
    want = oracle.packed_mlp(t["x"].f64, t["U_gu"].f64, t["V_g"].f64, t["V_u"].f64, t["U_d"].f64, t["V_d"].f64,
                             t["b_g"].f64, t["b_u"].f64, t["b_d"].f64)
    assert max_rel_err(G.host64(out), want) <= TOL["bf16"]


def _prefill_shapes():
    """Seeded shapes for the MFMA prefill path: K in steps of 64, N in steps of 128, any M > 32; chosen so that
    every tile kernel (128 x 128, 256 x 192, 256 x 256, ragged in both directions) and both k-step parities occur."""
    rng = np.random.default_rng(2605)
    shapes = [(33, 64, 128, 128), (257, 128, 256, 384), (1000, 192, 384, 1536), (2049, 64, 128, 4224),
              (4100, 320, 256, 4096 + 128), (8192, 128, 128, 2048), (3000, 64, 128, 5248)]
    for _ in range(9):
        M = int(rng.integers(34, 2500))
        d_in = 64 * int(rng.integers(1, 9))
        r = 128 * int(rng.integers(1, 7))
        d_out = 128 * int(rng.integers(1, 33))
        shapes.append((M, d_in, r, d_out))
    return shapes


@pytest.mark.parametrize("shape", _prefill_shapes())
def test_prefill_linear_shape_sweep(G, oracle, shape):
    M, d_in, r, d_out = shape
    rng = np.random.default_rng(M * 7 + d_out)
    x = rand_t(rng, (M, d_in), "bf16")
    U = rand_t(rng, (d_in, r), "bf16", d_in ** -0.5)
    V = rand_t(rng, (r, d_out), "bf16", r ** -0.5)
    b = rand_t(rng, (d_out,), "bf16")
    assert G.B.lowrank_plan_name(G.B.LR_OP_LINEAR, M, d_in, r, d_out, G.B.LR_BF16, "prefill", 1) == "prefill_mfma"
    y = G.run_linear(x, U, V, b, "prefill", "bf16")
    rows = sorted(set([0, M // 2, M - 1] + [m for m in (127, 128, 255, 256, 511, 512, M - 129, M - 257) if 0 <= m < M] +
                      list(rng.integers(0, M, size=40))))
    want = oracle.linear(x.f64[rows], U.f64, V.f64, b.f64)
    got = G.host64(y)
    assert np.isfinite(got).all()                 # every element was written (the output starts as NaN)
    assert max_rel_err(got[rows], want) <= TOL["bf16"]


# ------------------------------------------------------------------ workspace contract
def _mlp_case(M, seed):
    w = synth.mlp_layer(M, d=1024, ffn=2816, r_g=192, r_u=192, r_d=192, seed=seed)
    t = w.t
    return ([t[n] for n in ("x", "U_gu", "V_g", "V_u", "U_d", "V_d")],
            lambda o: o.packed_mlp(*[t[n].f64 for n in ("x", "U_gu", "V_g", "V_u", "U_d", "V_d")]))


def test_row_counts_change_on_one_workspace(G, oracle):
    """One workspace sized for the largest batch serves calls whose row count crosses every internal threshold
    (atomics / bf16 finalisation at 8|9 rows, one / two row blocks at 16|17, decode / prefill at 32|33), in an order in
    which a layout that moved with the row count would add onto stale sums: 12, 12, 4, 12, then a prefill call and a
    decode call after it.  Every result is checked against the oracle."""
    B = G.B
    nbytes = B.lowrank_workspace_bytes(B.LR_OP_PACKED_MLP, 300, 1024, 576, 2816, B.LR_BF16, "auto")
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 256)
    cases = {M: _mlp_case(M, 900 + M) for M in (12, 4, 32, 300, 17, 1)}
    dev = {M: [G.dev(a) for a in cases[M][0]] for M in cases}
    want = {M: cases[M][1](oracle) for M in cases}
    for M in (12, 12, 4, 12, 300, 12, 32, 17, 300, 1, 12):
        x, U_gu, V_g, V_u, U_d, V_d = dev[M]
        out = torch.full((M, 1024), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.lowrank_packed_mlp(x, U_gu, V_g, V_u, U_d, V_d, None, None, None, out, "auto", ws)
        B.lowrank_workspace_status(ws)
        assert max_rel_err(G.host64(out), want[M]) <= TOL["bf16"], M
    # the two-stage entry point on the same buffer, rows 25 (bf16 finalisation) then 3 (atomics) then 25
    wa = synth.attention_layer(25, d=1024, r=128, n_heads=8, S_max=8, seed=931).t
    x, U, V = G.dev(wa["x"]), G.dev(wa["U_q"]), G.dev(wa["V_q"])
    wantl = oracle.linear(wa["x"].f64, wa["U_q"].f64, wa["V_q"].f64)
    for M in (25, 3, 25):
        y = torch.full((M, 1024), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.lowrank_linear(x[:M].contiguous(), U, V, None, y, "decode", ws)
        B.lowrank_workspace_status(ws)
        assert max_rel_err(G.host64(y), wantl[:M]) <= TOL["bf16"], M


@pytest.mark.parametrize("M", [1, 12, 300])
def test_unprepared_workspace_with_arbitrary_contents(G, oracle, M):
    """A workspace straight from the allocator, filled with 0xFF bytes, random bytes, or the 'being prepared' word
    left behind by nobody: the first call prepares it on the stream and returns correct results, a second call reuses it."""
    B = G.B
    args, want_fn = _mlp_case(M, 950 + M)
    dev = [G.dev(a) for a in args]
    want = want_fn(oracle)
    nbytes = B.lowrank_workspace_bytes(B.LR_OP_PACKED_MLP, M, 1024, 576, 2816, B.LR_BF16, "auto")
    for fill in ("ff", "random", "zero"):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        if fill == "ff":
            ws.fill_(255)
        elif fill == "random":
            ws.random_(0, 256)
        else:
            ws.zero_()
        for _ in range(2):
            out = torch.full((M, 1024), float("nan"), dtype=torch.bfloat16, device="cuda")
            B.lowrank_packed_mlp(*dev, None, None, None, out, "auto", ws)
            B.lowrank_workspace_status(ws)
            assert max_rel_err(G.host64(out), want) <= TOL["bf16"], fill


def test_device_shared_setting_uses_one_launch_per_stage(G, oracle):
    """lowrank_configure(LR_CFG_DEVICE_SHARED, 1): no launch depends on co-resident workgroups; same results."""
    B = G.B
    args, want_fn = _mlp_case(8, 970)
    dev = [G.dev(a) for a in args]
    ws = B.new_workspace(B.LR_OP_PACKED_MLP, 8, 1024, 576, 2816, B.LR_BF16)
    B.lowrank_configure(B.LR_CFG_DEVICE_SHARED, 1)
    try:
        out = torch.full((8, 1024), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.lowrank_packed_mlp(*dev, None, None, None, out, "decode", ws)
        B.lowrank_workspace_status(ws)
        wa = synth.attention_layer(8, d=1024, r=128, n_heads=8, S_max=8, seed=971).t
        y = G.run_linear(wa["x"], wa["U_q"], wa["V_q"], None, "decode", "bf16")
    finally:
        B.lowrank_configure(B.LR_CFG_DEVICE_SHARED, 0)
    assert max_rel_err(G.host64(out), want_fn(oracle)) <= TOL["bf16"]
    assert max_rel_err(G.host64(y), oracle.linear(wa["x"].f64, wa["U_q"].f64, wa["V_q"].f64)) <= TOL["bf16"]


def test_wait_that_gives_up_poisons_results_and_is_reported(G, oracle):
    """The bounded device-side wait is made to give up from the host (a limit of zero polls: a workgroup that does not
    find the barrier complete at its first look stops waiting), so every kernel still runs to its end.  The call must
    not deliver plausible numbers: the workgroups that gave up write NaN, the status call reports the failure, every
    later call on that workspace returns NaN only, and preparing the workspace again restores normal service."""
    B = G.B
    args, want_fn = _mlp_case(4, 980)
    dev = [G.dev(a) for a in args]
    want = want_fn(oracle)
    ws = B.new_workspace(B.LR_OP_PACKED_MLP, 4, 1024, 576, 2816, B.LR_BF16)
    def call():
        out = torch.zeros((4, 1024), dtype=torch.bfloat16, device="cuda")
        B.lowrank_packed_mlp(*dev, None, None, None, out, "decode", ws)
        torch.cuda.synchronize()
        return G.host64(out)
    assert max_rel_err(call(), want) <= TOL["bf16"]
    B.lowrank_configure(B.LR_CFG_WAIT_LIMIT, 0)
    try:
        got = call()
    finally:
        B.lowrank_configure(B.LR_CFG_WAIT_LIMIT, 1 << 20)
    assert np.isnan(got).any()                                   # at least the workgroups that gave up
    ok = ~np.isnan(got)
    if ok.any():                                                 # whoever did pass every barrier had complete inputs
        assert np.max(np.abs(got[ok] - want[ok])) <= TOL["bf16"] * np.max(np.abs(want))
    with pytest.raises(B.LowrankError) as e:
        B.lowrank_workspace_status(ws)
    assert e.value.status == -7
    assert np.isnan(call()).all()                                # the failure sticks to the workspace
    B.lowrank_workspace_init(ws)
    assert max_rel_err(call(), want) <= TOL["bf16"]
    B.lowrank_workspace_status(ws)


# ------------------------------------------------------------------ exact arithmetic: indexing errors cannot hide under a tolerance
def _sparse_int(rng, shape, nnz_axis, nnz):
    """Matrix of -1 / 0 / +1 with exactly `nnz` nonzeros along `nnz_axis` of every slice."""
    a = np.zeros(shape)
    n = shape[nnz_axis]
    other = shape[1 - nnz_axis]
    for i in range(other):
        idx = rng.choice(n, size=nnz, replace=False)
        sgn = rng.choice([-1.0, 1.0], size=nnz)
        if nnz_axis == 0:
            a[idx, i] = sgn
        else:
            a[i, idx] = sgn
    return a


@pytest.mark.parametrize("M,d_in,r,d_out,phase", [
    (1, 4096, 384, 4096, "decode"), (7, 4096, 384, 4096, "decode"), (16, 1024, 256, 2048, "decode"),
    (25, 4096, 384, 4096, "decode"), (32, 2048, 128, 1024, "decode"),
    (300, 1024, 256, 2048, "prefill"), (2048, 4096, 384, 4096, "prefill"), (1000, 512, 128, 640, "prefill"),
    (333, 2112, 256, 640, "prefill"),        # ragged rows; K cut into chunks of 576, 576, 576 and 384 (split-K with a shorter last chunk)
])
def test_small_integer_inputs_give_exact_results(G, oracle, M, d_in, r, d_out, phase):
    """x, U, V hold only -1, 0, +1, sparse enough that every partial sum, every rank-space value and every output is a small
    integer: exactly representable in bf16 and in every accumulation order.  The tuned kernels must then reproduce the oracle
    bit for bit (through the tolerance of the ordinary parity tests a misplaced tile of small values could slip)."""
    B = G.B
    rng = np.random.default_rng(31 * M + r)
    x = _sparse_int(rng, (M, d_in), 1, 8)            # 8 nonzeros per row of x           -> |t| <= 8
    U = rng.choice([-1.0, 0.0, 1.0], size=(d_in, r))
    V = _sparse_int(rng, (r, d_out), 0, 16)          # 16 nonzeros per column of V       -> |y| <= 128
    bias = rng.integers(-3, 4, size=d_out).astype(np.float64)
    xt, Ut, Vt, bt = (synth.to_dtype(a, "bf16") for a in (x, U, V, bias))
    assert B.lowrank_plan_name(B.LR_OP_LINEAR, M, d_in, r, d_out, B.LR_BF16, phase) != "generic"
    y = G.run_linear(xt, Ut, Vt, bt, phase, "bf16")
    want = oracle.linear(x, U, V, bias)
    assert np.array_equal(G.host64(y), want)
    # and the same through lowrank_qkv with a cache (three projections of different rank, V twice)
    if M <= 32:
        V2 = _sparse_int(rng, (r // 2, d_out), 0, 16)
        U2 = rng.choice([-1.0, 0.0, 1.0], size=(d_in, r // 2))
        H, E, S_max = d_out // 128, 128, 8
        pos = rng.integers(0, S_max, size=M).astype(np.int32)
        kc = torch.zeros((M, S_max, H, E), dtype=torch.bfloat16, device="cuda")
        vc = torch.zeros_like(kc)
        outs = [torch.full((M, d_out), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(3)]
        ws = B.new_workspace(B.LR_OP_QKV, M, d_in, 2 * r + r // 2, 3 * d_out, B.LR_BF16, phase)
        Ud, Vd, U2d, V2d = G.dev(Ut), G.dev(Vt), G.dev(synth.to_dtype(U2, "bf16")), G.dev(synth.to_dtype(V2, "bf16"))
        B.lowrank_qkv(G.dev(xt), [Ud, U2d, Ud], [Vd, V2d, Vd], None, outs,
                      dict(k_cache=kc, v_cache=vc, pos=G.dev(pos), tokens_per_seq=1, k_index=1, v_index=2), phase, ws)
        B.lowrank_workspace_status(ws)
        assert np.array_equal(G.host64(outs[0]), oracle.linear(x, U, V))
        assert np.array_equal(G.host64(outs[1]), oracle.linear(x, U2, V2))
        assert np.array_equal(G.host64(outs[2]), oracle.linear(x, U, V))
        kh = G.host64(kc)
        for b in range(M):
            assert np.array_equal(kh[b, pos[b]].reshape(-1), oracle.linear(x[b:b + 1], U2, V2)[0])
