"""Decode attention over the dense KV cache (with rotary embedding) against the fp64 oracle, through the C ABI."""
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


def make_case(rng, B, T, H, E, S_max, pos, dtype):
    """Caches filled with history (already-rotated keys are just numbers), new raw k / v rows at pos .. pos+T-1."""
    q = synth.to_dtype(rng.standard_normal((B * T, H * E)), dtype)
    kc = synth.to_dtype(rng.standard_normal((B, S_max, H, E)), dtype)
    vc = synth.to_dtype(rng.standard_normal((B, S_max, H, E)), dtype)
    return q, kc, vc, np.asarray(pos, dtype=np.int32)


def run_gpu(G, q, kc, vc, pos, T, scale, base, dtype, ws=None):
    B = G.B
    qd, kd, vd = G.dev(q), G.dev(kc), G.dev(vc)
    Bn, S_max, H, E = kd.shape
    out = torch.full(qd.shape, float("nan"), dtype=G.tdtype(dtype), device="cuda")
    if ws is None:
        ws = B.new_workspace(B.LR_OP_DECODE_ATTENTION, Bn * T, H * E, H, 0, G.code(dtype))
    B.lowrank_decode_attention(qd, kd, vd, G.dev(pos), T, out, scale, base, ws)
    torch.cuda.synchronize()
    return out, kd, ws


CASES = [  # (B, T, H, E, S_max, positions, dtype)  -- head_dim 64 / 128 / 256 in bf16 take the fast kernel
    (1, 1, 32, 128, 2048, [2047], "bf16"),          # one long sequence: 24 splits per head
    (1, 1, 32, 128, 8192, [5000], "bf16"),
    (4, 1, 8, 128, 600, [0, 1, 37, 599], "bf16"),   # lengths 1, 2, 38, 600: mostly empty splits
    (2, 3, 4, 64, 100, [0, 50], "bf16"),            # three new tokens per sequence, causal among them
    (3, 1, 2, 256, 50, [49, 7, 20], "bf16"),
    (32, 1, 32, 128, 300, list(range(100, 132)), "bf16"),   # a full decode batch: one split per (row, head)
    (2, 2, 3, 32, 70, [5, 60], "bf16"),             # head_dim 32: generic kernel
    (2, 2, 3, 16, 1100, [1000, 3], "f32"),          # fp32: generic kernel, several LDS chunks
    (1, 1, 2, 128, 40, [39], "f32"),
]


@pytest.mark.parametrize("base", [0.0, 10000.0])
@pytest.mark.parametrize("case", CASES)
def test_decode_attention_matches_oracle(G, oracle, case, base):
    Bn, T, H, E, S_max, pos, dtype = case
    rng = np.random.default_rng(77 + S_max + H)
    q, kc, vc, pos = make_case(rng, Bn, T, H, E, S_max, pos, dtype)
    scale = E ** -0.5
    out, kd, _ = run_gpu(G, q, kc, vc, pos, T, scale, base, dtype)
    ok = kc.f64.copy()
    want = oracle.decode_attention(q.f64, ok, vc.f64, pos, T, scale, rope_base=base)
    assert max_rel_err(G.host64(out), want) <= TOL[dtype]
    # the key cache: new rows rotated (rounded to the storage type), every other row untouched bit for bit
    kb_in, kb_out, kh = kc.dev, G.bits(kd), G.host64(kd)
    for b in range(Bn):
        new = np.zeros(S_max, dtype=bool); new[pos[b]:pos[b] + T] = True
        assert np.array_equal(kb_out[b][~new], (kb_in[b][~new].view(np.uint32) if dtype == "f32" else kb_in[b][~new]))
        if base > 0:
            assert max_rel_err(kh[b][new].reshape(T, -1), ok[b][new].reshape(T, -1)) <= (2.0 ** -8 if dtype == "bf16" else 1e-6)
        else:
            assert np.array_equal(kb_out[b][new], (kb_in[b][new].view(np.uint32) if dtype == "f32" else kb_in[b][new]))


def test_repeated_calls_share_a_workspace(G, oracle):
    """Counters and partials of the split reduction are left clean: long, short, long on one workspace."""
    rng = np.random.default_rng(5)
    H, E, S_max = 8, 128, 3000
    ws = None
    for n in (2999, 3, 1500):
        q, kc, vc, pos = make_case(rng, 1, 1, H, E, S_max, [n - 1], "bf16")
        out, _, ws = run_gpu(G, q, kc, vc, pos, 1, E ** -0.5, 10000.0, "bf16", ws)
        want = oracle.decode_attention(q.f64, kc.f64.copy(), vc.f64, pos, 1, E ** -0.5, rope_base=10000.0)
        assert max_rel_err(G.host64(out), want) <= TOL["bf16"]


def test_single_position_returns_its_value_row(G):
    rng = np.random.default_rng(6)
    q, kc, vc, pos = make_case(rng, 2, 1, 4, 128, 16, [0, 0], "bf16")
    out, _, _ = run_gpu(G, q, kc, vc, pos, 1, 0.1, 10000.0, "bf16")
    assert np.array_equal(G.bits(out).reshape(2, 4, 128), vc.dev[:, 0])          # softmax over one position = 1: exact


def test_decode_layer_chain_qkv_cache_rope_attention_o(G, oracle):
    """lowrank_qkv writes raw k, v into the cache; attention rotates, attends; lowrank_linear projects."""
    B = G.B
    rng = np.random.default_rng(8)
    Bn, H, E, S_max, d, r = 3, 4, 64, 40, 256, 64
    pos = np.array([0, 17, 39], dtype=np.int32)
    bf = lambda a: synth.to_dtype(a, "bf16")
    x = bf(rng.standard_normal((Bn, d)))
    Us = [bf(rng.standard_normal((d, r)) * d ** -0.5) for _ in range(4)]
    Vs = [bf(rng.standard_normal((r, d)) * r ** -0.5) for _ in range(4)]
    kc = bf(rng.standard_normal((Bn, S_max, H, E))); vc = bf(rng.standard_normal((Bn, S_max, H, E)))
    kd, vd, pd = G.dev(kc), G.dev(vc), G.dev(pos)
    qd = torch.empty((Bn, d), dtype=torch.bfloat16, device="cuda")
    ad = torch.empty_like(qd); yd = torch.empty_like(qd)
    w1 = B.new_workspace(B.LR_OP_QKV, Bn, d, 3 * r, 3 * d, B.LR_BF16, "decode")
    w2 = B.new_workspace(B.LR_OP_DECODE_ATTENTION, Bn, d, H, 0, B.LR_BF16)
    w3 = B.new_workspace(B.LR_OP_LINEAR, Bn, d, r, d, B.LR_BF16, "decode")
    B.lowrank_qkv(G.dev(x), [G.dev(u) for u in Us[:3]], [G.dev(v) for v in Vs[:3]], None, [qd, None, None],
                  dict(k_cache=kd, v_cache=vd, pos=pd, tokens_per_seq=1, k_index=1, v_index=2), "decode", w1)
    B.lowrank_decode_attention(qd, kd, vd, pd, 1, ad, E ** -0.5, 10000.0, w2)
    B.lowrank_linear(ad, G.dev(Us[3]), G.dev(Vs[3]), None, yd, "decode", w3)
    for w in (w1, w3):
        B.lowrank_workspace_status(w)
    okc, ovc = kc.f64.copy(), vc.f64.copy()
    qkv = oracle.qkv(x.f64, [u.f64 for u in Us[:3]], [v.f64 for v in Vs[:3]],
                     kv=dict(k_cache=okc, v_cache=ovc, pos=pos, T=1, k_index=1, v_index=2))
    att = oracle.decode_attention(qkv[0], okc, ovc, pos, 1, E ** -0.5, rope_base=10000.0)
    want = oracle.linear(att, Us[3].f64, Vs[3].f64)
    assert max_rel_err(G.host64(ad), att) <= TOL["bf16"]
    assert max_rel_err(G.host64(yd), want) <= TOL["bf16"]


def test_attention_error_codes(G):
    B = G.B
    q = torch.zeros((1, 6), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((1, 4, 2, 3), dtype=torch.bfloat16, device="cuda")        # odd head_dim
    pos = torch.zeros((1,), dtype=torch.int32, device="cuda")
    ws = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.LowrankError):
        B.lowrank_decode_attention(q, kc, kc.clone(), pos, 1, torch.empty_like(q), 1.0, 0.0, ws)
    q = torch.zeros((1, 8), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((1, 4, 2, 4), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.LowrankError):                                            # workspace too small
        B.lowrank_decode_attention(q, kc, kc.clone(), pos, 1, torch.empty_like(q), 1.0, 0.0, ws[:256])
    assert B.lowrank_workspace_bytes(B.LR_OP_DECODE_ATTENTION, 1, 8, 3, 0, B.LR_BF16, "decode") == 0   # 8 % 3 != 0


PREFILL_CASES = [  # (B, T, H, S_max, positions): bf16, head_dim 128 -- the matrix-core prefill kernel
    (1, 1, 2, 8, [0]),                       # a single token: sees only itself
    (1, 65, 2, 80, [0]),                     # one partial query block, keys cross one tile border
    (1, 128, 1, 128, [0]),                   # exactly one query block
    (2, 200, 2, 300, [0, 37]),               # two query blocks, a ragged one; a history of 37 positions
    (3, 130, 3, 400, [5, 0, 200]),           # histories longer than the new tokens
    (1, 700, 2, 1000, [250]),                # many key tiles; unmasked tiles, then the diagonal
]


@pytest.mark.parametrize("base", [0.0, 10000.0])
@pytest.mark.parametrize("case", PREFILL_CASES)
def test_prefill_attention_matches_oracle(G, oracle, case, base):
    B = G.B
    Bn, T, H, S_max, pos = case
    E = 128
    rng = np.random.default_rng(500 + T + H)
    q, kc, vc, pos = make_case(rng, Bn, T, H, E, S_max, pos, "bf16")
    scale = E ** -0.5
    qd, kd, vd = G.dev(q), G.dev(kc), G.dev(vc)
    out = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    B.lowrank_prefill_attention(qd, kd, vd, G.dev(pos), T, out, scale, base)
    torch.cuda.synchronize()
    ok = kc.f64.copy()
    want = oracle.decode_attention(q.f64, ok, vc.f64, pos, T, scale, rope_base=base)
    got = G.host64(out)
    assert np.isfinite(got).all()
    assert max_rel_err(got, want) <= TOL["bf16"]
    kb_in, kb_out, kh = kc.dev, G.bits(kd), G.host64(kd)
    for b in range(Bn):
        new = np.zeros(S_max, dtype=bool); new[pos[b]:pos[b] + T] = True
        assert np.array_equal(kb_out[b][~new], kb_in[b][~new])
        if base > 0:
            assert max_rel_err(kh[b][new].reshape(T, -1), ok[b][new].reshape(T, -1)) <= 2.0 ** -8
        else:
            assert np.array_equal(kb_out[b][new], kb_in[b][new])


@pytest.mark.parametrize("profile", ["rising", "falling", "jumps"])
def test_prefill_attention_scores_far_from_the_first_tile(G, oracle, profile):
    """Score profiles along the keys that make a row's running maximum move by many powers of two in later tiles
    (rising), never again after the first (falling), or now and then (jumps): the kernel keeps its exponentials
    relative to a reference that it moves only when needed, so every one of those paths has to give the plain softmax."""
    B = G.B
    rng = np.random.default_rng(777)
    Bn, T, H, E, S_max = 1, 300, 2, 128, 512
    pos = np.asarray([130], dtype=np.int32)                   # 130 keys of history, 300 new rows: 7 key tiles
    u = rng.standard_normal(E); u /= np.linalg.norm(u)
    j = np.arange(S_max, dtype=np.float64)
    if profile == "rising":
        amp = 0.35 * j                                        # about +22 per 64-key tile in log2 units after scaling
    elif profile == "falling":
        amp = 60.0 - 0.35 * j
    else:
        amp = 40.0 * ((j // 97) % 2) + 25.0 * (j % 131 == 0)
    k = 0.3 * rng.standard_normal((Bn, S_max, H, E)) + amp[None, :, None, None] * u[None, None, None, :]
    qv = 0.3 * rng.standard_normal((Bn * T, H, E)) + 3.0 * u[None, None, :]
    q = synth.to_dtype(qv.reshape(Bn * T, H * E), "bf16")
    kc = synth.to_dtype(k, "bf16")
    vc = synth.to_dtype(rng.standard_normal((Bn, S_max, H, E)), "bf16")
    scale = E ** -0.5
    out = torch.full((Bn * T, H * E), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.lowrank_prefill_attention(G.dev(q), G.dev(kc), G.dev(vc), G.dev(pos), T, out, scale, 0.0)
    torch.cuda.synchronize()
    want = oracle.decode_attention(q.f64, kc.f64.copy(), vc.f64, pos, T, scale, rope_base=0.0)
    got = G.host64(out)
    assert np.isfinite(got).all()
    assert max_rel_err(got, want) <= TOL["bf16"]


def test_prefill_attention_equals_decode_attention_rotation(G):
    """The two entry points rotate new key rows with the same arithmetic: bit-identical caches."""
    B = G.B
    rng = np.random.default_rng(91)
    Bn, T, H, E, S_max = 2, 40, 2, 128, 64
    q, kc, vc, pos = make_case(rng, Bn, T, H, E, S_max, [3, 20], "bf16")
    qd, vd = G.dev(q), G.dev(vc)
    k1, k2 = G.dev(kc), G.dev(kc)
    o1 = torch.empty_like(qd); o2 = torch.empty_like(qd)
    B.lowrank_prefill_attention(qd, k1, vd, G.dev(pos), T, o1, E ** -0.5, 10000.0)
    ws = B.new_workspace(B.LR_OP_DECODE_ATTENTION, Bn * T, H * E, H, 0, B.LR_BF16)
    B.lowrank_decode_attention(qd, k2, vd, G.dev(pos), T, o2, E ** -0.5, 10000.0, ws)
    torch.cuda.synchronize()
    assert np.array_equal(G.bits(k1), G.bits(k2))
    assert max_rel_err(G.host64(o1), G.host64(o2)) <= TOL["bf16"]


def test_prefill_attention_error_codes(G):
    B = G.B
    q = torch.zeros((4, 2 * 64), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((1, 8, 2, 64), dtype=torch.bfloat16, device="cuda")
    pos = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.LowrankError):      # head_dim 64 is not covered by the matrix-core kernel
        B.lowrank_prefill_attention(q, kc, kc.clone(), pos, 4, torch.empty_like(q), 1.0, 0.0)


def test_prefill_layer_chain_qkv_cache_rope_attention_o(G, oracle):
    """The prefill attention half of a layer: lowrank_qkv writes raw k, v for 300 new tokens behind a history,
    lowrank_prefill_attention rotates and attends, lowrank_linear projects."""
    B = G.B
    rng = np.random.default_rng(18)
    Bn, T, H, E, S_max, r = 2, 300, 2, 128, 400, 128
    d = H * E
    pos = np.array([0, 90], dtype=np.int32)
    bf = lambda a: synth.to_dtype(a, "bf16")
    x = bf(rng.standard_normal((Bn * T, d)))
    Us = [bf(rng.standard_normal((d, r)) * d ** -0.5) for _ in range(4)]
    Vs = [bf(rng.standard_normal((r, d)) * r ** -0.5) for _ in range(4)]
    kc = bf(rng.standard_normal((Bn, S_max, H, E))); vc = bf(rng.standard_normal((Bn, S_max, H, E)))
    kd, vd, pd = G.dev(kc), G.dev(vc), G.dev(pos)
    qd = torch.empty((Bn * T, d), dtype=torch.bfloat16, device="cuda")
    ad = torch.empty_like(qd); yd = torch.empty_like(qd)
    w1 = B.new_workspace(B.LR_OP_QKV, Bn * T, d, 3 * r, 3 * d, B.LR_BF16, "prefill")
    w3 = B.new_workspace(B.LR_OP_LINEAR, Bn * T, d, r, d, B.LR_BF16, "prefill")
    B.lowrank_qkv(G.dev(x), [G.dev(u) for u in Us[:3]], [G.dev(v) for v in Vs[:3]], None, [qd, None, None],
                  dict(k_cache=kd, v_cache=vd, pos=pd, tokens_per_seq=T, k_index=1, v_index=2), "prefill", w1)
    B.lowrank_prefill_attention(qd, kd, vd, pd, T, ad, E ** -0.5, 10000.0)
    B.lowrank_linear(ad, G.dev(Us[3]), G.dev(Vs[3]), None, yd, "prefill", w3)
    for w in (w1, w3):
        B.lowrank_workspace_status(w)
    okc, ovc = kc.f64.copy(), vc.f64.copy()
    qkv = oracle.qkv(x.f64, [u.f64 for u in Us[:3]], [v.f64 for v in Vs[:3]],
                     kv=dict(k_cache=okc, v_cache=ovc, pos=pos, T=T, k_index=1, v_index=2))
    att = oracle.decode_attention(qkv[0], okc, ovc, pos, T, E ** -0.5, rope_base=10000.0)
    want = oracle.linear(att, Us[3].f64, Vs[3].f64)
    assert max_rel_err(G.host64(ad), att) <= TOL["bf16"]
    assert max_rel_err(G.host64(yd), want) <= TOL["bf16"]


def test_prefill_attention_full_size_sampled_rows(G, oracle):
    """The benchmark's shape (8192 new tokens, 32 heads of 128, empty history): sampled rows of two heads against the
    oracle.  The oracle sees a two-head slice of the caches whose key rows below the sampled token are rotated by the
    oracle itself; the token's own key row is left raw for the oracle call to rotate, as the entry point does."""
    B = G.B
    T, H, E = 8192, 32, 128
    gen = torch.Generator(device="cuda"); gen.manual_seed(99)
    q = torch.randn((T, H * E), device="cuda", dtype=torch.bfloat16, generator=gen)
    kc = torch.randn((1, T, H, E), device="cuda", dtype=torch.bfloat16, generator=gen)
    vc = torch.randn((1, T, H, E), device="cuda", dtype=torch.bfloat16, generator=gen)
    k_raw = kc.clone()
    out = torch.full_like(q, float("nan"))
    pos = torch.zeros((1,), dtype=torch.int32, device="cuda")
    B.lowrank_prefill_attention(q, kc, vc, pos, T, out, E ** -0.5, 10000.0)
    torch.cuda.synchronize()
    got = G.host64(out)
    assert np.isfinite(got).all()
    heads = [0, 21]
    hs = np.array(heads)
    k2 = G.host64(k_raw)[0][:, hs, :]                    # [T, 2, E] raw keys of two heads
    v2 = G.host64(vc)[0][:, hs, :]
    q2 = G.host64(q).reshape(T, H, E)[:, hs, :].reshape(T, 2 * E)
    k_rot = oracle.rope(k2.reshape(T, 2 * E), np.arange(T), 2, E, 10000.0).reshape(T, 2, E)
    rng = np.random.default_rng(5)
    rows = sorted(set([0, 1, 63, 64, 127, 128, 129, 4095, 4096, 8063, 8064, 8191] + list(rng.integers(0, T, size=12))))
    for srow in rows:
        kcache = np.ascontiguousarray(k_rot[None, :srow + 1].copy())
        kcache[0, srow] = k2[srow]                        # the new token's key: raw, rotated by the call
        want = oracle.decode_attention(q2[srow:srow + 1], kcache, np.ascontiguousarray(v2[None, :srow + 1]),
                                       np.array([srow], dtype=np.int32), 1, E ** -0.5, rope_base=10000.0)
        sel = got[srow].reshape(H, E)[hs].reshape(1, 2 * E)
        assert max_rel_err(sel, want) <= TOL["bf16"], srow
    # the rotated cache rows of those heads, bf16-rounded
    kh = G.host64(kc)[0][:, hs, :]
    assert max_rel_err(kh.reshape(T, -1), k_rot.reshape(T, -1)) <= 2.0 ** -8


# ------------------------------------------------------------------ factorized queries (rank-space rows into the attention kernel)
@pytest.mark.parametrize("base", [0.0, 10000.0])
@pytest.mark.parametrize("with_bias", [False, True])
@pytest.mark.parametrize("case,r_q", [(c, r) for c, r in zip(PREFILL_CASES, (64, 128, 384, 64, 256, 192))])
def test_prefill_factorized_attention_matches_oracle(G, oracle, case, r_q, with_bias, base):
    """lowrank_prefill_factorized_attention takes t_q [M, r] and V_q [r, H * 128] and rebuilds its query tiles inside the
    kernel.  Expected values: the oracle's second stage q = t_q V_q (+ b_q) followed by the oracle's attention over the
    dense cache; the cache must end up exactly as after the dense-query entry point."""
    B = G.B
    Bn, T, H, S_max, pos = case
    E = 128
    rng = np.random.default_rng(900 + T + H + r_q)
    _, kc, vc, pos = make_case(rng, Bn, T, H, E, S_max, pos, "bf16")
    tq = synth.to_dtype(rng.standard_normal((Bn * T, r_q)), "bf16")
    Vq = synth.to_dtype(rng.standard_normal((r_q, H * E)) * r_q ** -0.5, "bf16")
    bq = synth.to_dtype(0.3 * rng.standard_normal(H * E), "bf16") if with_bias else None
    scale = E ** -0.5
    kd, vd = G.dev(kc), G.dev(vc)
    out = torch.full((Bn * T, H * E), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.lowrank_prefill_factorized_attention(G.dev(tq), G.dev(Vq), None if bq is None else G.dev(bq), kd, vd, G.dev(pos), T, out, scale, base)
    torch.cuda.synchronize()
    q64 = oracle.stage2(tq.f64, Vq.f64, None if bq is None else bq.f64)
    ok = kc.f64.copy()
    want = oracle.decode_attention(q64, ok, vc.f64, pos, T, scale, rope_base=base)
    got = G.host64(out)
    assert np.isfinite(got).all()
    assert max_rel_err(got, want) <= TOL["bf16"]
    # same cache as after the dense-query entry point (the key rotation does not depend on the queries)
    kd2 = G.dev(kc)
    qd = G.dev(synth.to_dtype(q64, "bf16"))
    out2 = torch.empty_like(out)
    B.lowrank_prefill_attention(qd, kd2, G.dev(vc), G.dev(pos), T, out2, scale, base)
    torch.cuda.synchronize()
    assert np.array_equal(G.bits(kd), G.bits(kd2))
    assert max_rel_err(got, G.host64(out2)) <= TOL["bf16"]


def test_factorized_attention_chain_without_dense_q(G, oracle):
    """The prefill chain as the paper draws it: rank-space rows t_q = x U_q (lowrank_rank_project), K and V through
    lowrank_qkv into the dense cache only, then attention straight from t_q and V_q -- no dense q anywhere.  Checked against
    the oracle's linear layers + attention."""
    B = G.B
    Bn, T, H, E, d, r = 1, 384, 4, 128, 512, 128
    S_max = T + 16
    rng = np.random.default_rng(4242)
    x = synth.to_dtype(rng.standard_normal((T, d)), "bf16")
    Us = [synth.to_dtype(rng.standard_normal((d, r)) * d ** -0.5, "bf16") for _ in range(3)]
    Vs = [synth.to_dtype(rng.standard_normal((r, H * E)) * r ** -0.5, "bf16") for _ in range(3)]
    pos = np.asarray([9], dtype=np.int32)
    hist_k = synth.to_dtype(rng.standard_normal((Bn, S_max, H, E)), "bf16")
    hist_v = synth.to_dtype(rng.standard_normal((Bn, S_max, H, E)), "bf16")
    kd, vd, xd = G.dev(hist_k), G.dev(hist_v), G.dev(x)
    ws = B.new_workspace(B.LR_OP_QKV, T, d, 3 * r, 3 * H * E, B.LR_BF16, "prefill")
    tq = torch.full((T, r), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.lowrank_rank_project(xd, G.dev(Us[0]), tq, ws)
    B.lowrank_qkv(xd, [G.dev(Us[1]), G.dev(Us[2])], [G.dev(Vs[1]), G.dev(Vs[2])], None, [None, None],
                  dict(k_cache=kd, v_cache=vd, pos=G.dev(pos), tokens_per_seq=T, k_index=0, v_index=1), "prefill", ws)
    out = torch.full((T, H * E), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.lowrank_prefill_factorized_attention(tq, G.dev(Vs[0]), None, kd, vd, G.dev(pos), T, out, E ** -0.5, 10000.0)
    B.lowrank_workspace_status(ws)
    # rank-space rows against the oracle's first stage
    assert max_rel_err(G.host64(tq), oracle.stage1(x.f64, Us[0].f64)) <= TOL["bf16"]
    # the whole chain in fp64
    okc, ovc = hist_k.f64.copy(), hist_v.f64.copy()
    q, k, v = oracle.qkv(x.f64, [u.f64 for u in Us], [w.f64 for w in Vs],
                         kv=dict(k_cache=okc, v_cache=ovc, pos=pos, T=T, k_index=1, v_index=2))
    want = oracle.decode_attention(q, okc, ovc, pos, T, E ** -0.5, rope_base=10000.0)
    assert max_rel_err(G.host64(out), want) <= TOL["bf16"]


def test_factorized_attention_rejects_what_it_cannot_run(G):
    B = G.B
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    pos = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.LowrankError) as e:          # rank not a multiple of 64
        B.lowrank_prefill_factorized_attention(z(4, 96), z(96, 128), None, z(1, 8, 1, 128), z(1, 8, 1, 128), pos, 4, z(4, 128), 1.0, 0.0)
    assert e.value.status == -8
    with pytest.raises(B.LowrankError) as e:          # head_dim 64
        B.lowrank_prefill_factorized_attention(z(4, 64), z(64, 64), None, z(1, 8, 1, 64), z(1, 8, 1, 64), pos, 4, z(4, 64), 1.0, 0.0)
    assert e.value.status == -8
