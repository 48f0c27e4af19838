"""Pins for the fp64 oracle: each test checks it against something that is not the oracle --
a brute-force loop written independently here, a library routine (numpy's BLAS/LAPACK), a
closed form, or an invariant of the mathematics.  The paper prints no worked numeric example
of a factorized layer (it has no equations), so no value of the paper's can serve as a pin.
A plausible mistake in the oracle (dropped bias, transposed operand, wrong pack order,
wrong cache stride, SiLU sign) fails at least one test below.
"""
import math

import numpy as np
import pytest

from paper_2605_08314_amd import synth
from util import max_rel_err


# ---------------------------------------------------------------- brute force, exact on integers
def brute_linear(x, U, V, bias):
    M, d_in = len(x), len(x[0])
    r = len(V)
    d_out = len(V[0]) if r else (len(bias) if bias is not None else 0)
    y = [[0] * d_out for _ in range(M)]
    for m in range(M):
        for n in range(d_out):
            acc = 0
            for j in range(r):
                tj = 0
                for k in range(d_in):
                    tj += x[m][k] * U[k][j]
                acc += tj * V[j][n]
            y[m][n] = acc + (bias[n] if bias is not None else 0)
    return y


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 3, 1, 4), (3, 5, 2, 4), (4, 8, 3, 7), (5, 2, 6, 3)])
@pytest.mark.parametrize("with_bias", [False, True])
def test_linear_brute_force_exact(oracle, shape, with_bias):
    M, d_in, r, d_out = shape
    rng = np.random.default_rng(sum(shape) + with_bias)
    x = rng.integers(-9, 10, size=(M, d_in))
    U = rng.integers(-9, 10, size=(d_in, r))
    V = rng.integers(-9, 10, size=(r, d_out))
    b = rng.integers(-99, 100, size=d_out) if with_bias else None
    want = np.array(brute_linear(x.tolist(), U.tolist(), V.tolist(), None if b is None else b.tolist()),
                    dtype=np.float64).reshape(M, d_out)
    got = oracle.linear(x, U, V, b)
    assert np.array_equal(got, want)          # integers are exact in binary64


# ---------------------------------------------------------------- library and closed-form pins
def test_linear_matches_dense_reconstruction(oracle):
    rng = np.random.default_rng(11)
    x, U, V = rng.standard_normal((7, 96)), rng.standard_normal((96, 20)), rng.standard_normal((20, 53))
    b = rng.standard_normal(53)
    want = x @ (U @ V) + b                    # other association, numpy's BLAS
    assert max_rel_err(oracle.linear(x, U, V, b), want) <= 1e-12
    assert max_rel_err(oracle.linear(x, U, V), x @ U @ V) <= 1e-12


def test_full_rank_svd_recovers_dense_layer(oracle):
    rng = np.random.default_rng(12)
    W = rng.standard_normal((40, 28))
    P, s, Qt = np.linalg.svd(W, full_matrices=False)
    U, V = P * np.sqrt(s)[None, :], np.sqrt(s)[:, None] * Qt
    x = rng.standard_normal((6, 40))
    assert max_rel_err(oracle.linear(x, U, V), x @ W) <= 1e-10


def test_generator_is_truncated_svd_eckart_young(oracle):
    """The factor recipe really is the rank-r truncated SVD: residual^2 = sum of dropped sigma^2,
    and LAPACK's SVD of W returns the same leading singular values."""
    rng = np.random.default_rng(13)
    W, q1, sig, q2 = synth.full_svd_matrix(48, 36, rng)
    r = 10
    root = np.sqrt(sig[:r])
    U, V = q1[:, :r] * root[None, :], root[:, None] * q2[:, :r].T
    resid = np.linalg.norm(W - U @ V, "fro") ** 2
    assert abs(resid - np.sum(sig[r:] ** 2)) <= 1e-10 * np.sum(sig ** 2)
    assert np.allclose(np.linalg.svd(W, compute_uv=False), sig, rtol=1e-10)
    x = rng.standard_normal((3, 48))
    P, s, Qt = np.linalg.svd(W, full_matrices=False)
    want = ((x @ P[:, :r]) * s[:r]) @ Qt[:r]              # x times LAPACK's truncated SVD
    assert max_rel_err(oracle.linear(x, U, V), want) <= 1e-10


def test_svd_factors_recipe_norm():
    rng = np.random.default_rng(14)
    U, V = synth.svd_factors(64, 80, 16, rng)
    assert U.shape == (64, 16) and V.shape == (16, 80)
    assert abs(np.linalg.norm(U @ V, "fro") ** 2 - 80) <= 1e-9
    s = np.linalg.svd(U @ V, compute_uv=False)[:16]
    assert np.allclose(s * np.sqrt(np.arange(1, 17)), s[0], rtol=1e-9)    # sigma_i ~ i^-1/2


def test_linearity_zero_rank_zero_input(oracle):
    rng = np.random.default_rng(15)
    U, V = rng.standard_normal((30, 9)), rng.standard_normal((9, 17))
    x1, x2 = rng.standard_normal((4, 30)), rng.standard_normal((4, 30))
    a, b = 1.75, -0.5
    lhs = oracle.linear(a * x1 + b * x2, U, V)
    rhs = a * oracle.linear(x1, U, V) + b * oracle.linear(x2, U, V)
    assert max_rel_err(lhs, rhs) <= 1e-12
    bias = rng.standard_normal(17)
    y0 = oracle.linear(x1, np.zeros((30, 0)), np.zeros((0, 17)), bias)
    assert np.array_equal(y0, np.broadcast_to(bias, (4, 17)))
    assert np.array_equal(oracle.linear(x1, np.zeros((30, 0)), np.zeros((0, 17))), np.zeros((4, 17)))
    assert np.array_equal(oracle.linear(np.zeros((4, 30)), U, V, bias), np.broadcast_to(bias, (4, 17)))
    assert oracle.linear(np.zeros((0, 30)), U, V).shape == (0, 17)


def test_rank_one_and_identity_factors(oracle):
    rng = np.random.default_rng(16)
    x = rng.standard_normal((5, 12))
    u, v = rng.standard_normal(12), rng.standard_normal(8)
    want = np.outer(x @ u, v)
    assert max_rel_err(oracle.linear(x, u[:, None], v[None, :]), want) <= 1e-13
    V = rng.standard_normal((12, 8))
    assert max_rel_err(oracle.linear(x, np.eye(12), V), x @ V) <= 1e-13
    U = rng.standard_normal((12, 8))
    assert max_rel_err(oracle.linear(x, U, np.eye(8)), x @ U) <= 1e-13
    # a permutation as V must permute columns exactly (catches a transposed V)
    perm = rng.permutation(8)
    Pm = np.eye(8)[perm]                       # (t Pm)[n] = t[j] with perm[j] = n
    t = oracle.stage1(x, U)
    y = oracle.linear(x, U, Pm)
    assert np.array_equal(y[:, perm], t)


def test_stage_split_equals_fused(oracle):
    rng = np.random.default_rng(17)
    x, U, V = rng.standard_normal((3, 21)), rng.standard_normal((21, 5)), rng.standard_normal((5, 11))
    b = rng.standard_normal(11)
    assert np.array_equal(oracle.stage2(oracle.stage1(x, U), V, b), oracle.linear(x, U, V, b))
    assert max_rel_err(oracle.stage1(x, U), x @ U) <= 1e-13


# ---------------------------------------------------------------- packing (index work, bitwise)
def test_pack_concat_bitwise_and_order(oracle):
    rng = np.random.default_rng(18)
    for dt in (np.uint16, np.float32, np.float64):
        Us = [rng.integers(0, 60000, size=(13, r)).astype(dt) for r in (3, 1, 6)]
        packed = oracle.pack_concat(Us)
        assert packed.dtype == dt and packed.shape == (13, 10)
        assert np.array_equal(packed, np.concatenate(Us, axis=1))
        assert np.array_equal(packed[:, 0:3], Us[0]) and np.array_equal(packed[:, 4:10], Us[2])


def test_pack_panels_layout(oracle):
    # hand example: K = 2, N = 128, W[k, n] = 128 k + n.  Panel 0 is columns 0..63 of row 0, then of row 1; panel 1 columns 64..127.
    W = np.arange(256, dtype=np.uint16).reshape(2, 128)
    flat = oracle.pack_panels(W).reshape(-1)
    want = list(range(0, 64)) + list(range(128, 192)) + list(range(64, 128)) + list(range(192, 256))
    assert flat.tolist() == want
    # the flat index of element (k, n) as the boundary states it, element by element on a ragged-looking shape
    rng = np.random.default_rng(181)
    K, N = 7, 192
    W = rng.integers(0, 60000, size=(K, N)).astype(np.uint16)
    flat = oracle.pack_panels(W).reshape(-1)
    for k in range(K):
        for n in range(N):
            assert flat[((n // 64) * K + k) * 64 + n % 64] == W[k, n]
    # undoing it is a concatenation of the panels along the columns; panels of a concatenation are the panels side by side
    for dt in (np.uint16, np.float32):
        A = rng.integers(0, 60000, size=(5, 128)).astype(dt)
        Bm = rng.integers(0, 60000, size=(5, 64)).astype(dt)
        P = oracle.pack_panels(A)
        assert P.dtype == dt and np.array_equal(np.concatenate(list(P), axis=1), A)
        assert np.array_equal(oracle.pack_panels(np.concatenate([A, Bm], axis=1)),
                              np.concatenate([oracle.pack_panels(A), oracle.pack_panels(Bm)], axis=0))


def test_packed_projection_equals_separate_bitwise(oracle):
    rng = np.random.default_rng(19)
    x = rng.standard_normal((4, 33))
    Us = [rng.standard_normal((33, r)) for r in (5, 7, 2)]
    t_packed = oracle.stage1(x, oracle.pack_concat(Us))
    col = 0
    for U in Us:
        assert np.array_equal(t_packed[:, col:col + U.shape[1]], oracle.stage1(x, U))
        col += U.shape[1]


# ---------------------------------------------------------------- qkv, cache, shared basis
def test_qkv_equals_separate_and_cache_scatter(oracle):
    rng = np.random.default_rng(20)
    B, T, H, E, S_max, d_in = 3, 2, 4, 5, 9, 14
    d_out = H * E
    x = rng.standard_normal((B * T, d_in))
    Us = [rng.standard_normal((d_in, r)) for r in (3, 4, 2)]
    Vs = [rng.standard_normal((U.shape[1], d_out)) for U in Us]
    bs = [rng.standard_normal(d_out), None, rng.standard_normal(d_out)]
    pos = np.array([0, 7, 3], dtype=np.int32)
    SENT = -12345.0
    kc = np.full((B, S_max, H, E), SENT)
    vc = np.full((B, S_max, H, E), SENT)
    outs = oracle.qkv(x, Us, Vs, bs, kv=dict(k_cache=kc, v_cache=vc, pos=pos, T=T, k_index=1, v_index=2))
    for i in range(3):
        assert np.array_equal(outs[i], oracle.linear(x, Us[i], Vs[i], bs[i]))
    # independent re-statement of the cache addressing with numpy indexing
    for cache, o in ((kc, outs[1]), (vc, outs[2])):
        expect = np.full_like(cache, SENT)
        for b in range(B):
            for s in range(T):
                expect[b, pos[b] + s] = o[b * T + s].reshape(H, E)
        assert np.array_equal(cache, expect)
        assert np.count_nonzero(cache != SENT) == B * T * H * E
    with pytest.raises(ValueError):
        oracle.cache_write(outs[1], kc, np.array([0, 8, 3], dtype=np.int32), T)


def test_shared_basis_alias_equals_independent(oracle):
    rng = np.random.default_rng(21)
    x = rng.standard_normal((4, 18))
    U = rng.standard_normal((18, 6))
    V1, V2 = rng.standard_normal((6, 10)), rng.standard_normal((6, 10))
    shared = oracle.qkv(x, [U, U], [V1, V2])
    assert np.array_equal(shared[0], oracle.linear(x, U, V1))
    assert np.array_equal(shared[1], oracle.linear(x, U.copy(), V2))


# ---------------------------------------------------------------- packed MLP
def silu_via_mlp(oracle, z):
    """out = SiLU(z) through the MLP entry point: d = ffn = 1, gate = identity, up = 0*x + 1."""
    one = np.ones((1, 1))
    out = oracle.packed_mlp(np.array([[z]]), np.array([[1.0, 0.0]]), one, one, one, one,
                            b_u=np.array([1.0]))
    return float(out[0, 0])


def test_silu_closed_forms(oracle):
    assert silu_via_mlp(oracle, 0.0) == 0.0
    # sigmoid(ln a) = a / (1 + a)  =>  SiLU(ln 3) = (3/4) ln 3,  SiLU(-ln 3) = -(1/4) ln 3
    assert abs(silu_via_mlp(oracle, math.log(3.0)) - 0.75 * math.log(3.0)) <= 1e-15
    assert abs(silu_via_mlp(oracle, -math.log(3.0)) + 0.25 * math.log(3.0)) <= 1e-15
    # SiLU(z) - SiLU(-z) = z for every z
    for z in (0.3, 1.0, 2.5, 7.0, 30.0):
        assert abs(silu_via_mlp(oracle, z) - silu_via_mlp(oracle, -z) - z) <= 1e-14 * max(1.0, z)
    assert silu_via_mlp(oracle, 50.0) == pytest.approx(50.0, rel=1e-15)
    assert -1e-18 < silu_via_mlp(oracle, -50.0) < 0.0
    assert silu_via_mlp(oracle, -800.0) == 0.0 or abs(silu_via_mlp(oracle, -800.0)) < 1e-300
    # the global minimum of SiLU sits where 1 + e^-z (1 + z) = 0, z* ~ -1.27846, value ~ -0.27846
    zs = np.linspace(-3, 0, 3001)
    vals = np.array([silu_via_mlp(oracle, float(z)) for z in zs])
    zmin = zs[np.argmin(vals)]
    assert abs(zmin + 1.2785) < 2e-3 and abs(vals.min() + 0.27846) < 1e-5


def test_packed_mlp_matches_dense_reference(oracle):
    rng = np.random.default_rng(22)
    M, d, ffn, r_g, r_u, r_d = 5, 24, 37, 6, 4, 7
    x = rng.standard_normal((M, d))
    Ug, Uu = rng.standard_normal((d, r_g)) / 4, rng.standard_normal((d, r_u)) / 4
    Vg, Vu = rng.standard_normal((r_g, ffn)), rng.standard_normal((r_u, ffn))
    Ud, Vd = rng.standard_normal((ffn, r_d)) / 4, rng.standard_normal((r_d, d))
    bg, bu, bd = rng.standard_normal(ffn), rng.standard_normal(ffn), rng.standard_normal(d)
    Wg, Wu, Wd = Ug @ Vg, Uu @ Vu, Ud @ Vd
    for use_b in (False, True):
        g = x @ Wg + (bg if use_b else 0)
        u = x @ Wu + (bu if use_b else 0)
        sig = 0.5 * (1.0 + np.tanh(0.5 * g))                     # logistic via tanh, not via exp
        want = (g * sig * u) @ Wd + (bd if use_b else 0)
        got = oracle.packed_mlp(x, np.concatenate([Ug, Uu], 1), Vg, Vu, Ud, Vd,
                                *( (bg, bu, bd) if use_b else (None, None, None)))
        assert max_rel_err(got, want) <= 1e-12


def test_packed_mlp_pack_order_and_special_cases(oracle):
    rng = np.random.default_rng(23)
    M, d, ffn, r_g, r_u, r_d = 3, 10, 12, 2, 5, 4
    x = rng.standard_normal((M, d))
    Ug, Uu = rng.standard_normal((d, r_g)), rng.standard_normal((d, r_u))
    Vg, Vu = rng.standard_normal((r_g, ffn)), rng.standard_normal((r_u, ffn))
    Ud, Vd = rng.standard_normal((ffn, r_d)), rng.standard_normal((r_d, d))
    U_gu = oracle.pack_concat([Ug, Uu])
    out = oracle.packed_mlp(x, U_gu, Vg, Vu, Ud, Vd)
    # chain built from the single-layer oracle: gate columns first, then up
    g, u = oracle.linear(x, Ug, Vg), oracle.linear(x, Uu, Vu)
    h = g * (0.5 * (1.0 + np.tanh(0.5 * g))) * u
    assert max_rel_err(out, oracle.linear(h, Ud, Vd)) <= 1e-12
    # up branch switched off and b_u = 1: out = down(SiLU(g))
    out1 = oracle.packed_mlp(x, oracle.pack_concat([Ug, np.zeros_like(Uu)]), Vg, Vu, Ud, Vd, b_u=np.ones(ffn))
    hg = g * (0.5 * (1.0 + np.tanh(0.5 * g)))
    assert max_rel_err(out1, oracle.linear(hg, Ud, Vd)) <= 1e-12
    # x = 0 and no bias: SiLU(0) * 0 = 0 everywhere
    assert np.array_equal(oracle.packed_mlp(np.zeros((2, d)), U_gu, Vg, Vu, Ud, Vd), np.zeros((2, d)))
    # swapping gate and up factors must change the result (SiLU is not symmetric)
    swapped = oracle.packed_mlp(x, oracle.pack_concat([Uu, Ug]), Vu, Vg, Ud, Vd)
    assert max_rel_err(swapped, out) > 1e-3


# ---------------------------------------------------------------- dtype plumbing of the generators
def test_bf16_round_trip_and_rounding():
    vals = np.array([0.0, 1.0, -1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -9, 3.140625, 1e-3])
    bits = synth.f64_to_bf16_bits(vals)
    back = synth.bf16_bits_to_f64(bits)
    assert back[0] == 0.0 and back[1] == 1.0 and back[2] == -1.0
    assert back[3] == 1.0                         # tie rounds to even mantissa
    assert back[4] == 1.0 + 2.0 ** -7             # representable
    assert back[5] == 1.0 + 2.0 ** -7             # 1 + 3*2^-9 is nearer to 1 + 2^-7 than to 1
    assert back[6] == 3.140625
    assert np.all(np.abs(back - vals) <= np.abs(vals) * 2.0 ** -8)
    assert np.array_equal(synth.f64_to_bf16_bits(back), bits)   # idempotent


def test_workload_shapes_match_configs():
    w = synth.config1()
    assert w.t["x"].dev.shape == (16, 512) and w.t["U"].dev.shape == (512, 128) and w.t["V"].dev.shape == (128, 512)
    assert w.t["x"].dev.dtype == np.float32
    a = synth.attention_layer(2, d=256, r=24, n_heads=4, S_max=16)
    assert a.t["U_q"].dev.dtype == np.uint16 and a.t["U_q"].dev.shape == (256, 24)
    assert np.array_equal(synth.bf16_bits_to_f64(a.t["V_o"].dev), a.t["V_o"].f64)
    m = synth.mlp_layer(2, d=64, ffn=96, r_g=8, r_u=16, r_d=8)
    assert m.t["U_gu"].dev.shape == (64, 24)
    assert np.array_equal(m.t["U_gu"].dev[:, :8], m.t["U_g"].dev)
    rows = synth.prefill_row_sample(300)
    assert rows[0] == 0 and rows[-1] == 299 and 127 in rows and 128 in rows and 255 in rows and 256 in rows


# ---------------------------------------------------------------- rotary embedding (Section 4: RoPE on q and k)
def test_rope_unit_vectors_pin_pairing_frequency_and_sign(oracle):
    H, E, base, p = 2, 8, 10000.0, 7
    for h in range(H):
        for i in range(E // 2):
            a = p * base ** (-2.0 * i / E)
            x = np.zeros((1, H * E)); x[0, h * E + i] = 1.0                 # low partner of pair i
            y = oracle.rope(x, [p], H, E, base)
            want = np.zeros_like(x); want[0, h * E + i] = math.cos(a); want[0, h * E + i + E // 2] = math.sin(a)
            assert np.allclose(y, want, rtol=0, atol=1e-15)
            x = np.zeros((1, H * E)); x[0, h * E + i + E // 2] = 1.0        # high partner
            y = oracle.rope(x, [p], H, E, base)
            want = np.zeros_like(x); want[0, h * E + i] = -math.sin(a); want[0, h * E + i + E // 2] = math.cos(a)
            assert np.allclose(y, want, rtol=0, atol=1e-15)


def test_rope_identity_norm_composition_and_relative_property(oracle):
    rng = np.random.default_rng(11)
    H, E = 3, 16
    x = rng.standard_normal((5, H * E)); k = rng.standard_normal((5, H * E))
    assert np.array_equal(oracle.rope(x, [0] * 5, H, E), x)                                  # position 0: identity
    pos = np.array([1, 17, 300, 4095, 8191])
    y = oracle.rope(x, pos, H, E)
    pair_norm = lambda z: z.reshape(5, H, 2, E // 2)[:, :, 0] ** 2 + z.reshape(5, H, 2, E // 2)[:, :, 1] ** 2
    assert np.allclose(pair_norm(y), pair_norm(x), rtol=1e-12)                               # a rotation of every pair
    assert np.allclose(oracle.rope(oracle.rope(x, pos, H, E), [5] * 5, H, E), oracle.rope(x, pos + 5, H, E), atol=1e-9)
    # scores depend on the position difference only
    dots = lambda m, n: (oracle.rope(x, m, H, E).reshape(5, H, E) * oracle.rope(k, n, H, E).reshape(5, H, E)).sum(-1)
    assert np.allclose(dots(pos, pos - 1), dots(pos + 100, pos + 99), atol=1e-9)
    assert not np.allclose(dots(pos, pos - 1), dots(pos, pos - 2), atol=1e-3)
    # E = 2: the plain planar rotation by p radians
    z = oracle.rope(np.array([[1.0, 0.0], [0.0, 1.0]]), [2, 3], 1, 2)
    assert np.allclose(z, [[math.cos(2), math.sin(2)], [-math.sin(3), math.cos(3)]], atol=1e-15)


# ---------------------------------------------------------------- attention over the dense cache (Section 3.1)
def _attention_brute(q, kc, vc, pos, T, scale):
    """Pure-Python loops, no numpy arithmetic: softmax(q K^T scale) V, causal."""
    B, S_max, H, E = kc.shape
    out = [[0.0] * (H * E) for _ in range(B * T)]
    for b in range(B):
        for s in range(T):
            n = int(pos[b]) + s + 1
            for h in range(H):
                sc = [scale * sum(float(q[b * T + s, h * E + e]) * float(kc[b, j, h, e]) for e in range(E)) for j in range(n)]
                mx = max(sc)
                w = [math.exp(v - mx) for v in sc]
                den = sum(w)
                for e in range(E):
                    out[b * T + s][h * E + e] = sum(w[j] / den * float(vc[b, j, h, e]) for j in range(n))
    return np.array(out)


def test_attention_brute_force_and_causality(oracle):
    rng = np.random.default_rng(12)
    B, T, S_max, H, E = 2, 3, 9, 2, 4
    q = rng.standard_normal((B * T, H * E))
    kc = rng.standard_normal((B, S_max, H, E)); vc = rng.standard_normal((B, S_max, H, E))
    pos = np.array([4, 0], dtype=np.int32)
    want = _attention_brute(q, kc, vc, pos, T, 0.5)
    got = oracle.decode_attention(q, kc.copy(), vc, pos, T, 0.5)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-14)
    # positions a row may not see do not matter: poison them
    kp, vp = kc.copy(), vc.copy()
    for b in range(B):
        kp[b, pos[b] + T:] = np.nan; vp[b, pos[b] + T:] = np.nan
    assert np.array_equal(oracle.decode_attention(q, kp, vp, pos, T, 0.5), got)
    # causal inside the new tokens: row s of sequence 1 (pos 0) sees exactly s + 1 positions; row 0 returns v[0]
    assert np.allclose(got[T * 1 + 0].reshape(H, E), vc[1, 0], rtol=1e-14)
    with pytest.raises(ValueError):
        oracle.decode_attention(q, kc.copy(), vc, np.array([7, 0], dtype=np.int32), T, 0.5)     # 7 + 3 > S_max


def test_attention_closed_forms(oracle):
    from scipy.special import softmax
    rng = np.random.default_rng(13)
    B, S_max, H, E, n = 1, 40, 2, 8, 33
    q = rng.standard_normal((1, H * E))
    kc = rng.standard_normal((B, S_max, H, E)); vc = rng.standard_normal((B, S_max, H, E))
    pos = np.array([n - 1], dtype=np.int32)
    scale = E ** -0.5
    out = oracle.decode_attention(q, kc.copy(), vc, pos, 1, scale)
    # library softmax + matmul
    for h in range(H):
        w = softmax(scale * kc[0, :n, h] @ q[0, h * E:(h + 1) * E])
        assert np.allclose(out[0, h * E:(h + 1) * E], w @ vc[0, :n, h], rtol=1e-12)
    # weights sum to one: V = const -> out = const;  identical keys -> plain mean of V
    assert np.allclose(oracle.decode_attention(q, kc.copy(), np.full_like(vc, 3.25), pos, 1, scale), 3.25, rtol=1e-14)
    same = np.broadcast_to(kc[:, :1], kc.shape).copy()
    assert np.allclose(oracle.decode_attention(q, same, vc, pos, 1, scale).reshape(H, E), vc[0, :n].mean(axis=0), rtol=1e-13)
    # adding one vector to every key shifts every score equally: same output
    shifted = kc + rng.standard_normal((1, 1, H, E))
    assert np.allclose(oracle.decode_attention(q, shifted, vc, pos, 1, scale), out, rtol=1e-10)
    # huge scores: no overflow, the best key wins
    big = oracle.decode_attention(q * 1e4, kc.copy(), vc, pos, 1, 1.0)
    for h in range(H):
        j = int(np.argmax(kc[0, :n, h] @ q[0, h * E:(h + 1) * E]))
        assert np.allclose(big[0, h * E:(h + 1) * E], vc[0, j, h], rtol=1e-12)
    # scale really multiplies the scores: scale 0 -> uniform weights
    assert np.allclose(oracle.decode_attention(q, kc.copy(), vc, pos, 1, 0.0).reshape(H, E), vc[0, :n].mean(axis=0), rtol=1e-13)


def test_attention_with_rope_rotates_new_keys_in_place_and_queries(oracle):
    rng = np.random.default_rng(14)
    B, T, S_max, H, E = 2, 2, 12, 2, 8
    q = rng.standard_normal((B * T, H * E))
    kc = rng.standard_normal((B, S_max, H, E)); vc = rng.standard_normal((B, S_max, H, E))
    pos = np.array([5, 9], dtype=np.int32)
    k_in = kc.copy()
    out = oracle.decode_attention(q, kc, vc, pos, T, E ** -0.5, rope_base=10000.0)
    # the cache: only the new rows changed, and they are the rotated raw rows
    for b in range(B):
        for j in range(S_max):
            if pos[b] <= j < pos[b] + T:
                assert np.allclose(kc[b, j].reshape(1, -1), oracle.rope(k_in[b, j].reshape(1, -1), [j], H, E), rtol=0, atol=1e-15)
            else:
                assert np.array_equal(kc[b, j], k_in[b, j])
    # same as: rotate by hand, then attention without RoPE
    rows_pos = np.array([pos[b] + s for b in range(B) for s in range(T)])
    want = oracle.decode_attention(oracle.rope(q, rows_pos, H, E), kc.copy(), vc, pos, T, E ** -0.5, rope_base=0.0)
    assert np.allclose(out, want, rtol=1e-13, atol=1e-15)
    assert not np.allclose(out, oracle.decode_attention(q, k_in.copy(), vc, pos, T, E ** -0.5), atol=1e-3)


# ------------------------------------------------------------------ diagnostic rounding-faithful mode
def test_round_bf16_known_values_and_grid():
    import oracle as o
    # ties to even at 8 significant bits: 1 + 2^-8 is half-way between 1 and 1 + 2^-7
    assert o.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert o.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert o.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    assert o.round_bf16(np.array([-3.0, 0.0, 0.15625, 255.0, 256.5]))[::1].tolist() == [-3.0, 0.0, 0.15625, 255.0, 256.0]
    rng = np.random.default_rng(11)
    a = rng.standard_normal(4096) * np.exp(rng.uniform(-20, 20, 4096))
    r = o.round_bf16(a)
    assert np.array_equal(o.round_bf16(r), r)                                  # idempotent: results are on the grid
    assert np.max(np.abs(r - a) / np.abs(a)) <= 2.0 ** -8                      # half a unit in the 8th significant bit
    # independent statement of the same rounding: through the float32 bit pattern (inputs exactly float32 here)
    f = a.astype(np.float32)
    assert np.array_equal(o.round_bf16(f.astype(np.float64)), synth.bf16_bits_to_f64(synth.f64_to_bf16_bits(f)))


def test_diag_mode_is_the_exact_definition_when_nothing_rounds(oracle):
    rng = np.random.default_rng(12)
    ident = lambda a: a
    x = rng.standard_normal((5, 24)); U = rng.standard_normal((24, 6)); V = rng.standard_normal((6, 10)); b = rng.standard_normal(10)
    assert np.array_equal(oracle.diag_linear(x, U, V, b, rnd=ident), oracle.linear(x, U, V, b))
    ya = oracle.diag_qkv(x, [U, U], [V, 2 * V], [b, None], rnd=ident)
    yb = oracle.qkv(x, [U, U], [V, 2 * V], [b, None])
    assert all(np.array_equal(p, q) for p, q in zip(ya, yb))
    w = synth.mlp_layer(3, d=32, ffn=40, r_g=4, r_u=6, r_d=5, seed=5, dtype="f32", with_bias=True).t
    args = [w[n].f64 for n in ("x", "U_gu", "V_g", "V_u", "U_d", "V_d", "b_g", "b_u", "b_d")]
    assert max_rel_err(oracle.diag_packed_mlp(*args, rnd=ident), oracle.packed_mlp(*args)) <= 1e-13
    # integer-valued eighths: every intermediate of the linear layer is exactly representable, so rounding changes nothing
    xi = rng.integers(-4, 5, (4, 8)) / 8.0; Ui = rng.integers(-2, 3, (8, 3)).astype(float); Vi = rng.integers(-2, 3, (3, 5)).astype(float)
    assert np.array_equal(oracle.diag_linear(xi, Ui, Vi), oracle.linear(xi, Ui, Vi))


def test_diag_mode_differs_from_exact_by_rounding_only(oracle):
    w = synth.mlp_layer(4, d=256, ffn=448, r_g=64, r_u=64, r_d=64, seed=6, dtype="bf16", with_bias=True).t
    args = [w[n].f64 for n in ("x", "U_gu", "V_g", "V_u", "U_d", "V_d", "b_g", "b_u", "b_d")]
    e = max_rel_err(oracle.diag_packed_mlp(*args), oracle.packed_mlp(*args))
    assert 0.0 < e <= 4 * 2.0 ** -8                                             # four roundings of at most 2^-8 each
    wa = synth.attention_layer(4, d=256, r=32, n_heads=2, S_max=8, seed=7).t
    e = max_rel_err(oracle.diag_linear(wa["x"].f64, wa["U_q"].f64, wa["V_q"].f64), oracle.linear(wa["x"].f64, wa["U_q"].f64, wa["V_q"].f64))
    assert 0.0 < e <= 2 * 2.0 ** -8
