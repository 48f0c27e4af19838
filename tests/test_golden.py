"""Stored expected values (tests/golden/): hand-worked integer examples that the oracle must reproduce exactly, and
regression values written by tests/golden/make_golden.py from the oracle alone, which the oracle must still reproduce
(CPU) and which the HIP path is compared with directly (GPU, without running the oracle)."""
import json
import os

import numpy as np
import pytest

from util import TOL, max_rel_err

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


@pytest.fixture(scope="module")
def hand():
    return json.load(open(os.path.join(GOLD, "hand_examples.json")))


@pytest.fixture(scope="module")
def stored():
    d = json.load(open(os.path.join(GOLD, "oracle_regression.json")))
    return {name: {k: (np.asarray(v) if isinstance(v, list) else v) for k, v in case.items()} for name, case in d.items()}


A = lambda v: np.asarray(v, dtype=np.float64)


def test_hand_linear_and_stages(oracle, hand):
    c = hand["linear"]
    assert np.array_equal(oracle.stage1(A(c["x"]), A(c["U"])), A(c["t"]))
    assert np.array_equal(oracle.linear(A(c["x"]), A(c["U"]), A(c["V"]), A(c["bias"])), A(c["y"]))
    assert np.array_equal(oracle.stage2(A(c["t"]), A(c["V"]), A(c["bias"])), A(c["y"]))


def test_hand_shared_basis(oracle, hand):
    c = hand["shared_basis"]
    U = A(c["U"])
    ya, yb = oracle.qkv(A(c["x"]), [U, U], [A(c["V_a"]), A(c["V_b"])])
    assert np.array_equal(ya, A(c["y_a"])) and np.array_equal(yb, A(c["y_b"]))


def test_hand_cache_write(oracle, hand):
    c = hand["cache_write"]
    cache = np.zeros((c["B"], c["S_max"], c["H"], c["E"]))
    oracle.cache_write(A(c["proj"]), cache, np.asarray(c["pos"], dtype=np.int32), c["T"])
    assert np.array_equal(cache, A(c["cache_after"]))


def test_hand_attention_equal_scores_average_the_values(oracle, hand):
    c = hand["attention"]
    out = oracle.decode_attention(A(c["q"]), A(c["k_cache"]), A(c["v_cache"]), np.asarray(c["pos"], dtype=np.int32),
                                  c["T"], c["scale"], rope_base=0.0)
    assert np.allclose(out, A(c["out"]), rtol=0, atol=1e-15)


def test_oracle_reproduces_the_stored_regression_values(oracle, stored):
    c = stored["linear"]
    assert max_rel_err(oracle.linear(c["x"], c["U"], c["V"], c["bias"]), c["y"]) <= 1e-14
    c = stored["packed_mlp"]
    got = oracle.packed_mlp(c["x"], c["U_gu"], c["V_g"], c["V_u"], c["U_d"], c["V_d"], c["b_g"], c["b_u"], c["b_d"])
    assert max_rel_err(got, c["out"]) <= 1e-14
    c = stored["attention"]
    k = c["k_cache"].copy()
    got = oracle.decode_attention(c["q"], k, c["v_cache"], c["pos"].astype(np.int32), c["T"], c["scale"], rope_base=c["rope_base"])
    assert max_rel_err(got, c["out"]) <= 1e-14 and max_rel_err(k, c["k_cache_after"]) <= 1e-14


def test_stored_inputs_are_exact_in_bf16(stored):
    for case in stored.values():
        for k, v in case.items():
            if isinstance(v, np.ndarray) and v.dtype == np.float64 and k not in ("y", "out", "k_cache_after"):
                assert np.array_equal(v * 8, np.round(v * 8)) and np.max(np.abs(v)) <= 2.0, k


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_hip_path_matches_the_stored_values(stored, dtype):
    import torch
    import gpu_util as G
    B = G.B
    td = G.tdtype(dtype)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.float64).to(td).cuda()
    c = stored["linear"]
    M, d_in = c["x"].shape
    r, d_out = c["V"].shape
    y = torch.full((M, d_out), float("nan"), dtype=td, device="cuda")
    ws = B.new_workspace(B.LR_OP_LINEAR, M, d_in, r, d_out, G.code(dtype), "decode")
    B.lowrank_linear(dev(c["x"]), dev(c["U"]), dev(c["V"]), dev(c["bias"]), y, "decode", ws)
    assert max_rel_err(G.host64(y), c["y"]) <= TOL[dtype]
    c = stored["packed_mlp"]
    M, d = c["x"].shape
    ffn = c["V_g"].shape[1]
    out = torch.full((M, d), float("nan"), dtype=td, device="cuda")
    ws = B.new_workspace(B.LR_OP_PACKED_MLP, M, d, c["U_gu"].shape[1] + c["U_d"].shape[1], ffn, G.code(dtype), "decode")
    B.lowrank_packed_mlp(dev(c["x"]), dev(c["U_gu"]), dev(c["V_g"]), dev(c["V_u"]), dev(c["U_d"]), dev(c["V_d"]),
                         dev(c["b_g"]), dev(c["b_u"]), dev(c["b_d"]), out, "decode", ws)
    assert max_rel_err(G.host64(out), c["out"]) <= TOL[dtype]
    c = stored["attention"]
    Bn, S_max, H, E = c["k_cache"].shape
    T = int(c["T"])
    kd, vd = dev(c["k_cache"]), dev(c["v_cache"])
    o = torch.full((Bn * T, H * E), float("nan"), dtype=td, device="cuda")
    ws = B.new_workspace(B.LR_OP_DECODE_ATTENTION, Bn * T, H * E, H, 0, G.code(dtype))
    pos = torch.from_numpy(c["pos"].astype(np.int32)).cuda()
    B.lowrank_decode_attention(dev(c["q"]), kd, vd, pos, T, o, float(c["scale"]), float(c["rope_base"]), ws)
    torch.cuda.synchronize()
    assert max_rel_err(G.host64(o), c["out"]) <= TOL[dtype]
    assert max_rel_err(G.host64(kd), c["k_cache_after"]) <= (2.0 ** -8 if dtype == "bf16" else 1e-6)
