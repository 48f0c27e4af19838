"""The entry point that allocates nothing (lowrank_linear_noalloc, scratch inside the library image) against
lowrank_linear with a caller-provided workspace: same results to the parity bar, on two calls in a row of which the
second is smaller (the shared scratch keeps the first call's contents), plus the size limit."""
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


def _case(rng, M, d_in, r, d_out, dtype):
    x = synth.to_dtype(rng.standard_normal((M, d_in)), dtype)
    U = synth.to_dtype(rng.standard_normal((d_in, r)) * d_in ** -0.5, dtype)
    V = synth.to_dtype(rng.standard_normal((r, d_out)) * r ** -0.5, dtype)
    b = synth.to_dtype(rng.standard_normal(d_out), dtype)
    return x, U, V, b


@pytest.mark.parametrize("dtype,shapes", [
    ("bf16", [(32, 4096, 384, 4096), (3, 1024, 128, 2048)]),          # decode kernels, larger then smaller
    ("bf16", [(200, 512, 256, 640), (7, 130, 33, 257)]),              # more than 32 rows / ragged: generic kernels
    ("f32", [(16, 512, 128, 512), (2, 64, 8, 32)]),
])
def test_noalloc_matches_workspace_entry_point(G, oracle, dtype, shapes):
    B = G.B
    rng = np.random.default_rng(2605)
    for M, d_in, r, d_out in shapes:                                  # two calls in a row on the same scratch
        x, U, V, b = _case(rng, M, d_in, r, d_out, dtype)
        xd, Ud, Vd, bd = G.dev(x), G.dev(U), G.dev(V), G.dev(b)
        y_ref = G.run_linear(x, U, V, b, "decode" if M <= 32 else "prefill", dtype)
        y = torch.full((M, d_out), float("nan"), dtype=G.tdtype(dtype), device="cuda")
        B.lowrank_linear_noalloc(xd, Ud, Vd, bd, y)
        torch.cuda.synchronize()
        want = oracle.linear(x.f64, U.f64, V.f64, b.f64)
        assert max_rel_err(G.host64(y), want) <= TOL[dtype], (M, d_in, r, d_out)
        assert max_rel_err(G.host64(y), G.host64(y_ref)) <= TOL[dtype], (M, d_in, r, d_out)


def test_noalloc_rejects_what_does_not_fit(G):
    B = G.B
    M, d_in, r, d_out = 64, 64, 4096, 64                              # 64 * 4096 floats = 1 MiB > 512 KiB
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    y = z(M, d_out)
    with pytest.raises(B.LowrankError) as e:
        B.lowrank_linear_noalloc(z(M, d_in), z(d_in, r), z(r, d_out), None, y)
    assert e.value.status == -6 and "scratch" in str(e.value)
    B.lowrank_linear_noalloc(z(0, d_in), z(d_in, r), z(r, d_out), None, z(0, d_out))      # empty batch: no-op
