"""Host<->device plumbing for the GPU parity tests (imports torch and the HIP binding)."""
import numpy as np
import torch

from paper_2605_08314_amd import binding as B
from paper_2605_08314_amd import synth


def dev(t, device="cuda"):
    """synth.Tensor (or raw numpy array of uint16 bf16 bits / float32 / int32) -> device tensor."""
    a = t.dev if isinstance(t, synth.Tensor) else t
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def host64(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> float64 numpy, exactly."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw bit patterns of a device tensor as unsigned integers (for bit-exact comparisons)."""
    c = t.detach().to("cpu").contiguous()
    if c.dtype == torch.bfloat16:
        return c.view(torch.int16).numpy().view(np.uint16)
    if c.dtype == torch.float32:
        return c.view(torch.int32).numpy().view(np.uint32)
    return c.numpy()


def tdtype(name: str):
    return {"bf16": torch.bfloat16, "f32": torch.float32}[name]


def code(name: str) -> int:
    return {"bf16": B.LR_BF16, "f32": B.LR_F32}[name]


def run_linear(x, U, V, bias, phase, dtype):
    xd, Ud, Vd = dev(x), dev(U), dev(V)
    bd = None if bias is None else dev(bias)
    M, d_in = xd.shape
    r, d_out = Vd.shape
    y = torch.full((M, d_out), float("nan"), dtype=tdtype(dtype), device="cuda")
    ws = B.new_workspace(B.LR_OP_LINEAR, M, d_in, r, d_out, code(dtype), phase)
    B.lowrank_linear(xd, Ud, Vd, bd, y, phase, ws)
    B.lowrank_workspace_status(ws)
    return y


def run_mlp(w, phase, x=None, biases=True):
    t = w.t
    xd = dev(t["x"]) if x is None else x
    M, d = xd.shape
    m = w.meta
    out = torch.full((M, d), float("nan"), dtype=tdtype(w.dtype), device="cuda")
    ws = B.new_workspace(B.LR_OP_PACKED_MLP, M, d, m["r_g"] + m["r_u"] + m["r_d"], m["ffn"], code(w.dtype), phase)
    bg = dev(t["b_g"]) if biases and "b_g" in t else None
    bu = dev(t["b_u"]) if biases and "b_u" in t else None
    bd = dev(t["b_d"]) if biases and "b_d" in t else None
    B.lowrank_packed_mlp(xd, dev(t["U_gu"]), dev(t["V_g"]), dev(t["V_u"]), dev(t["U_d"]), dev(t["V_d"]),
                         bg, bu, bd, out, phase, ws)
    B.lowrank_workspace_status(ws)
    return out
