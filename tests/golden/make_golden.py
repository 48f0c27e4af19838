"""Writes tests/golden/oracle_regression.json: outputs of the fp64 oracle for small seeded inputs.

Calls only ``oracle/`` (never the HIP library).  Inputs are multiples of 1/8 with magnitude at most 2, so the same numbers
are exact in bf16, fp32 and fp64 and are stored in the file next to the results."""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import oracle  # noqa: E402


def eighths(rng, shape):
    return rng.integers(-16, 17, size=shape).astype(np.float64) / 8.0


def cases():
    rng = np.random.default_rng(20260508)
    out = {}
    x, U, V, b = eighths(rng, (5, 16)), eighths(rng, (16, 4)), eighths(rng, (4, 12)), eighths(rng, (12,))
    out["linear"] = dict(x=x, U=U, V=V, bias=b, y=oracle.linear(x, U, V, b))
    x = eighths(rng, (3, 16))
    U_gu, V_g, V_u = eighths(rng, (16, 7)), eighths(rng, (3, 24)), eighths(rng, (4, 24))
    U_d, V_d = eighths(rng, (24, 5)), eighths(rng, (5, 16))
    b_g, b_u, b_d = eighths(rng, (24,)), eighths(rng, (24,)), eighths(rng, (16,))
    out["packed_mlp"] = dict(x=x, U_gu=U_gu, V_g=V_g, V_u=V_u, U_d=U_d, V_d=V_d, b_g=b_g, b_u=b_u, b_d=b_d,
                             out=oracle.packed_mlp(x, U_gu, V_g, V_u, U_d, V_d, b_g, b_u, b_d))
    Bn, T, H, E, S_max = 2, 2, 2, 8, 6
    q = eighths(rng, (Bn * T, H * E))
    kc, vc = eighths(rng, (Bn, S_max, H, E)), eighths(rng, (Bn, S_max, H, E))
    pos = np.asarray([3, 0], dtype=np.int32)
    k_after = kc.copy()
    o = oracle.decode_attention(q, k_after, vc, pos, T, E ** -0.5, rope_base=10000.0)
    out["attention"] = dict(q=q, k_cache=kc, v_cache=vc, pos=pos, T=T, scale=E ** -0.5, rope_base=10000.0,
                            out=o, k_cache_after=k_after)
    return out


def to_json(v):
    if isinstance(v, np.ndarray):
        return v.tolist()
    if isinstance(v, (np.floating, np.integer)):
        return v.item()
    return v


if __name__ == "__main__":
    data = {name: {k: to_json(v) for k, v in case.items()} for name, case in cases().items()}
    path = os.path.join(HERE, "oracle_regression.json")
    with open(path, "w") as f:
        json.dump(data, f, indent=1)
    print("wrote", path)
