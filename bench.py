#!/usr/bin/env python3
"""Benchmark of the factorized-linear hot path on one MI355X.

A *step* is one decode token step through a stack of L LLaMA-7B-shaped low-rank layers: per layer
one `lowrank_qkv` (Q/K/V at rank 384, K and V also written into the dense cache), one
`lowrank_linear` (O projection, rank 384) and one `lowrank_packed_mlp` (rank 768, ffn 11008), on
B token rows (configs 2 and 3 of the baseline).  Every layer has its own factors (L x 94.8 MB, far
more than the 256 MB last-level cache), so each step streams every factor byte from HBM.
`value` = algorithmic GB/s of the step: factor bytes + activations read + outputs written, each
counted once, divided by the wall time of the step (launch gaps included).

The same JSON line also carries
  roofline      the dominant kernel family (decode packed MLP) timed alone with HIP events,
  prefill       TFLOP/s of one layer (QKV + O + MLP, config 4) at S rows, algorithmic flops,
  decode_ops    per-entry-point GB/s for each batch size,
  prefill_ranks the four layers of the mixed-rank stack (ranks 384/768, 256, 512, 1024) at S = 512, 2048, 8192,
  shared_basis  the shared-basis layer pair of the 13B shape: decode B = 16 and prefill S = 4096,
  decode_attention  attention over the dense cache (with rotary embedding) at several cached lengths,
  cpu_baseline  the fp64 oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

D, FFN, R_ATTN, R_MLP, HEADS, HEAD_DIM = 4096, 11008, 384, 768, 32, 128
HBM_PEAK_GBS = 8000.0
# HBM bytes per decode-MLP launch at B=1 from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the
# same counters read for the 256 MiB copy of --pmc-mode (profiles/decode_mlp_pmc_traffic.txt).
MLP_TRAFFIC_BYTES = 70926778
TRAFFIC_SOURCE = "profiles/decode_mlp_pmc_traffic.txt (rocprofv3 --pmc run of `bench.py --pmc-mode`; not measured in this run)"
MFMA_BF16_PEAK_TFLOPS = 2500.0


def attn_bytes(B, r=R_ATTN, d=D):
    """Algorithmic bytes of QKV (+cache write) and O for B token rows."""
    factors_qkv = 3 * 2 * d * r * 2
    factors_o = 2 * d * r * 2
    act_qkv = B * d * 2 * (1 + 3 + 2)        # x read; q,k,v written; k,v written to the cache
    act_o = B * d * 2 * 2                    # a read, o written
    return factors_qkv + act_qkv, factors_o + act_o


def mlp_bytes(B, r=R_MLP, d=D, ffn=FFN):
    factors = (d * 2 * r + 2 * r * ffn + ffn * r + r * d) * 2
    return factors + B * d * 2 * 2


def attn_flops(M, r=R_ATTN, d=D):
    return 4 * 2 * r * (d + d) * M


def mlp_flops(M, r=R_MLP, d=D, ffn=FFN):
    return 2 * (d * 2 * r + ffn * 2 * r + ffn * r + r * d) * M


class Layer:
    """Device-resident factors of one layer (random values; timing does not depend on them)."""

    def __init__(self, torch, r_attn=R_ATTN, r_mlp=R_MLP, d=D, ffn=FFN, gen=None):
        def w(rows, cols, fan):
            return (torch.randn((rows, cols), device="cuda", dtype=torch.float32, generator=gen) * fan ** -0.5).to(torch.bfloat16)
        self.U = [w(d, r_attn, d) for _ in range(4)]          # q, k, v, o
        self.V = [w(r_attn, d, r_attn) for _ in range(4)]
        self.U_gu = w(d, 2 * r_mlp, d)
        self.V_g, self.V_u = w(r_mlp, ffn, r_mlp), w(r_mlp, ffn, r_mlp)
        self.U_d, self.V_d = w(ffn, r_mlp, ffn), w(r_mlp, d, r_mlp)
        self.P = None

    def make_panels(self, torch, B):
        """The decode copy of every factor: 64-column panels (lowrank_pack_panels), made once at load time."""
        def pk(W):
            P = torch.empty_like(W)
            B.lowrank_pack_panels(W, P)
            return P
        self.P = dict(U=[pk(u) for u in self.U], V=[pk(v) for v in self.V], U_gu=pk(self.U_gu), V_g=pk(self.V_g),
                      V_u=pk(self.V_u), U_d=pk(self.U_d), V_d=pk(self.V_d))


def capture(torch, fn):
    """Record fn()'s launches into a HIP graph (after one eager run) and return its replay()."""
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    torch.cuda.synchronize()
    return g.replay


def time_region(torch, fn, iters, warmup):
    """Average milliseconds per call of fn() over `iters` calls, HIP events on the current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def run_prefill(torch, B, gen, ly, S, R_ATTN=R_ATTN, R_MLP=R_MLP, iters=10):
    """One layer at S rows (QKV with cache write, O, packed MLP): time and TFLOP/s (algorithmic flops)."""
    bf = torch.bfloat16
    xs = torch.randn((S, D), device="cuda", generator=gen).to(bf)
    qs, os_, ms_ = (torch.empty((S, D), device="cuda", dtype=bf) for _ in range(3))
    kcs = torch.zeros((1, S, HEADS, HEAD_DIM), device="cuda", dtype=bf)
    vcs = torch.zeros_like(kcs)
    pos0 = torch.zeros((1,), device="cuda", dtype=torch.int32)
    wq = B.new_workspace(B.LR_OP_QKV, S, D, 3 * R_ATTN, 3 * D, B.LR_BF16, "prefill")
    wo = B.new_workspace(B.LR_OP_LINEAR, S, D, R_ATTN, D, B.LR_BF16, "prefill")
    wm = B.new_workspace(B.LR_OP_PACKED_MLP, S, D, 3 * R_MLP, FFN, B.LR_BF16, "prefill")

    def prefill_layer():
        # K and V go where attention reads them: the dense cache only
        B.lowrank_qkv(xs, ly.U[:3], ly.V[:3], None, [qs, None, None],
                      dict(k_cache=kcs, v_cache=vcs, pos=pos0, tokens_per_seq=S, k_index=1, v_index=2), "prefill", wq)
        B.lowrank_linear(xs, ly.U[3], ly.V[3], None, os_, "prefill", wo)
        B.lowrank_packed_mlp(xs, ly.U_gu, ly.V_g, ly.V_u, ly.U_d, ly.V_d, None, None, None, ms_, "prefill", wm)

    plan = B.lowrank_plan_name(B.LR_OP_PACKED_MLP, S, D, 3 * R_MLP, FFN, B.LR_BF16, "prefill")
    iters = iters if plan != "generic" else 1
    # replayed as a HIP graph like the decode step: at a few hundred rows the eight launches of a layer are
    # otherwise bound by the host's launch rate, not by the GPU
    pms = time_region(torch, capture(torch, prefill_layer) if plan != "generic" else prefill_layer, iters, 2)
    for w in (wq, wo, wm):
        B.lowrank_workspace_status(w)
    pfl = attn_flops(S, R_ATTN) + mlp_flops(S, R_MLP)
    tf = pfl / (pms * 1e-3) / 1e12
    return {"workload": f"one layer, S={S}, ranks {R_ATTN}/{R_MLP}", "plan": plan, "ms": round(pms, 3),
            "TFLOPs": round(tf, 1), "frac_mfma_bf16_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
            "tokens_per_s": round(S / (pms * 1e-3), 1)}


def run_prefill_ranks(torch, B, gen, S_list=(512, 2048, 8192), ranks=((384, 768), (256, 256), (512, 512), (1024, 1024))):
    """The four layers of the mixed-rank stack (attention rank, MLP rank), each at S rows: time, TFLOP/s of the
    algorithmic flops (156,160 * rho * S when all seven pairs have rank rho) and the tiles the dispatcher picked."""
    rows = {}
    for ra, rm in ranks:
        ly = Layer(torch, r_attn=ra, r_mlp=rm, gen=gen)
        for S in S_list:
            r = run_prefill(torch, B, gen, ly, S, ra, rm, iters=6 if S >= 8192 else 10)
            tiles = {"x*U_qkv": B.lowrank_prefill_tile(S, D, ra, 3), "t*V_qkv": B.lowrank_prefill_tile(S, ra, D, 3),
                     "x*U_gu": B.lowrank_prefill_tile(S, D, 2 * rm, 1), "h*U_d": B.lowrank_prefill_tile(S, FFN, rm, 1),
                     "t*V_d": B.lowrank_prefill_tile(S, rm, D, 1)}
            r["tiles"] = {k: f"{v[0]}x{v[1]}" + ("+shareK" if v[2] == 1 else (f"+splitK{v[2]}" if v[2] > 1 else "")) for k, v in tiles.items()}
            rows[f"r{ra}-{rm}_S{S}"] = r
        del ly
    return rows


def run_shared_basis(torch, B, gen, groups=20, d=5120, r=512):
    """Shared-basis layer pair (13B shape): one basis U_sh[d, r] used by two layers with their own V_i[r, d], through
    lowrank_qkv with the same U pointer twice (x * U_sh is formed once).  Decode at B = 16 rotating over `groups`
    distinct groups (15.7 MB each, far more than the last-level cache in total); prefill at S = 4096."""
    bf = torch.bfloat16
    def w(rows, cols, fan):
        return (torch.randn((rows, cols), device="cuda", dtype=torch.float32, generator=gen) * fan ** -0.5).to(bf)
    sets = [(w(d, r, d), w(r, d, r), w(r, d, r)) for _ in range(groups)]
    out = {}
    Bn = 16
    x = torch.randn((Bn, d), device="cuda", generator=gen).to(bf)
    y0, y1 = torch.empty((Bn, d), device="cuda", dtype=bf), torch.empty((Bn, d), device="cuda", dtype=bf)
    ws = B.new_workspace(B.LR_OP_QKV, Bn, d, 2 * r, 2 * d, B.LR_BF16, "decode")

    def sweep_dec():
        for U, V0, V1 in sets:
            B.lowrank_qkv(x, [U, U], [V0, V1], None, [y0, y1], None, "decode", ws)

    ms = time_region(torch, capture(torch, sweep_dec), 10, 2) / groups
    B.lowrank_workspace_status(ws)
    nbytes = 3 * d * r * 2 + Bn * d * 2 * 3                       # U_sh once, V_1, V_2; x read, two outputs written
    out["decode_B16"] = {"plan": B.lowrank_plan_name(B.LR_OP_QKV, Bn, d, 2 * r, 2 * d, B.LR_BF16, "decode"),
                         "us": round(ms * 1e3, 2), "bytes": nbytes, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                         "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         "unshared_bytes": 4 * d * r * 2 + Bn * d * 2 * 3}
    S = 4096
    xs = torch.randn((S, d), device="cuda", generator=gen).to(bf)
    z0, z1 = torch.empty((S, d), device="cuda", dtype=bf), torch.empty((S, d), device="cuda", dtype=bf)
    wp = B.new_workspace(B.LR_OP_QKV, S, d, 2 * r, 2 * d, B.LR_BF16, "prefill")
    U, V0, V1 = sets[0]

    def pre():
        B.lowrank_qkv(xs, [U, U], [V0, V1], None, [z0, z1], None, "prefill", wp)

    ms = time_region(torch, pre, 10, 2)
    B.lowrank_workspace_status(wp)
    fl = 2.0 * S * (d * r + 2 * r * d)
    t1, t2 = B.lowrank_prefill_tile(S, d, r, 1), B.lowrank_prefill_tile(S, r, d, 2)
    out["prefill_S4096"] = {"plan": B.lowrank_plan_name(B.LR_OP_QKV, S, d, 2 * r, 2 * d, B.LR_BF16, "prefill"),
                            "tiles": {"x*U_sh": f"{t1[0]}x{t1[1]}", "t*V_i": f"{t2[0]}x{t2[1]}"},
                            "ms": round(ms, 4), "GFLOP": round(fl / 1e9, 1), "TFLOPs": round(fl / (ms * 1e-3) / 1e12, 1),
                            "frac_mfma_bf16_peak": round(fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
    return out


def run_decode_attention(torch, B, gen, cases=((1, 512), (1, 2048), (1, 8192), (32, 2048)), layers=8):
    """Attention over the dense cache with rotary embedding, one new token per sequence: us per call and GB/s of
    the K and V rows it has to read (plus q and out), rotated over `layers` distinct caches, HIP-graph replay."""
    bf = torch.bfloat16
    rows = {}
    for Bn, n in cases:
        kcs = [torch.randn((Bn, n, HEADS, HEAD_DIM), device="cuda", dtype=bf, generator=gen) for _ in range(layers)]
        vcs = [torch.randn((Bn, n, HEADS, HEAD_DIM), device="cuda", dtype=bf, generator=gen) for _ in range(layers)]
        q = torch.randn((Bn, D), device="cuda", dtype=bf, generator=gen)
        out = torch.empty_like(q)
        pos = torch.full((Bn,), n - 1, device="cuda", dtype=torch.int32)
        ws = B.new_workspace(B.LR_OP_DECODE_ATTENTION, Bn, D, HEADS, 0, B.LR_BF16)

        def sweep_attn():
            for i in range(layers):
                B.lowrank_decode_attention(q, kcs[i], vcs[i], pos, 1, out, HEAD_DIM ** -0.5, 10000.0, ws)

        ms = time_region(torch, capture(torch, sweep_attn), 10, 2) / layers
        by = 2 * Bn * n * D * 2 + 2 * Bn * D * 2
        rows[f"B{Bn}_len{n}"] = {"us": round(ms * 1e3, 2), "GBps": round(by / (ms * 1e-3) / 1e9, 1),
                                 "frac_hbm_peak": round(by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del kcs, vcs
    return rows


def run_prefill_attention(torch, B, gen, S):
    """Causal attention of S new tokens over the cache they were just written to (rotary embedding on q and k):
    time and TFLOP/s; algorithmic flops = 4 * head_dim per visible (query, key) pair and head."""
    bf = torch.bfloat16
    q = torch.randn((S, D), device="cuda", dtype=bf, generator=gen)
    kc = torch.randn((1, S, HEADS, HEAD_DIM), device="cuda", dtype=bf, generator=gen)
    vc = torch.randn((1, S, HEADS, HEAD_DIM), device="cuda", dtype=bf, generator=gen)
    out = torch.empty_like(q)
    pos0 = torch.zeros((1,), device="cuda", dtype=torch.int32)

    def call():
        # every call rotates the new key rows again; the values drift but the work is the same
        B.lowrank_prefill_attention(q, kc, vc, pos0, S, out, HEAD_DIM ** -0.5, 10000.0)

    ms = time_region(torch, call, 5, 2)
    fl = 4.0 * HEAD_DIM * HEADS * (S * (S + 1) / 2)
    tf = fl / (ms * 1e-3) / 1e12
    return {"workload": f"S={S} new tokens, {HEADS} heads x {HEAD_DIM}, causal, RoPE", "ms": round(ms, 3),
            "TFLOPs": round(tf, 1), "frac_mfma_bf16_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)}


def run_prefill_factorized_attention(torch, B, gen, S, r=R_ATTN):
    """The same attention with factorized queries (rank-space rows t_q and V_q; the kernel rebuilds its query tiles), and the
    two ways from x to the attention output: dense (lowrank_linear writes q, lowrank_prefill_attention reads it) against
    factorized (lowrank_rank_project writes t_q, the attention kernel does the rest)."""
    bf = torch.bfloat16
    x = torch.randn((S, D), device="cuda", dtype=bf, generator=gen)
    U = (torch.randn((D, r), device="cuda", generator=gen) * D ** -0.5).to(bf)
    V = (torch.randn((r, D), device="cuda", generator=gen) * r ** -0.5).to(bf)
    kc = torch.randn((1, S, HEADS, HEAD_DIM), device="cuda", dtype=bf, generator=gen)
    vc = torch.randn((1, S, HEADS, HEAD_DIM), device="cuda", dtype=bf, generator=gen)
    pos0 = torch.zeros((1,), device="cuda", dtype=torch.int32)
    q, out = torch.empty((S, D), device="cuda", dtype=bf), torch.empty((S, D), device="cuda", dtype=bf)
    tq = torch.empty((S, r), device="cuda", dtype=bf)
    ws = B.new_workspace(B.LR_OP_LINEAR, S, D, r, D, B.LR_BF16, "prefill")
    B.lowrank_rank_project(x, U, tq, ws)
    scale = HEAD_DIM ** -0.5

    def fact_only():
        B.lowrank_prefill_factorized_attention(tq, V, None, kc, vc, pos0, S, out, scale, 10000.0)

    def chain_dense():
        B.lowrank_linear(x, U, V, None, q, "prefill", ws)
        B.lowrank_prefill_attention(q, kc, vc, pos0, S, out, scale, 10000.0)

    def chain_fact():
        B.lowrank_rank_project(x, U, tq, ws)
        B.lowrank_prefill_factorized_attention(tq, V, None, kc, vc, pos0, S, out, scale, 10000.0)

    ms_f = time_region(torch, fact_only, 5, 2)
    ms_cd = time_region(torch, chain_dense, 5, 2)
    ms_cf = time_region(torch, chain_fact, 5, 2)
    B.lowrank_workspace_status(ws)
    fl = 4.0 * HEAD_DIM * HEADS * (S * (S + 1) / 2) + 2.0 * S * r * D          # attention + the in-kernel q = t_q V_q
    return {"workload": f"S={S}, rank {r}: queries as rank-space rows", "ms": round(ms_f, 3),
            "TFLOPs": round(fl / (ms_f * 1e-3) / 1e12, 1), "frac_mfma_bf16_peak": round(fl / (ms_f * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "chain_dense_q_ms": round(ms_cd, 3), "chain_factorized_q_ms": round(ms_cf, 3)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--batch", type=int, default=1, help="token rows B of the timed decode step")
    ap.add_argument("--prefill-rows", type=int, default=8192)
    ap.add_argument("--eager", action="store_true", help="plain launches instead of HIP-graph replay")
    ap.add_argument("--row-major", action="store_true", help="decode on the row-major factors instead of their prepacked 64-column panels")
    ap.add_argument("--quick", action="store_true", help="skip the per-batch table, prefill and the CPU baseline")
    ap.add_argument("--prefill-only", action="store_true", help="only the prefill layer (for profiling): one JSON line with its numbers")
    ap.add_argument("--attention-only", action="store_true", help="only the decode-attention rows (for profiling)")
    ap.add_argument("--pmc-mode", action="store_true",
                    help="for rocprofv3 --pmc runs: a 256 MiB plain copy (known traffic) and 32 eager decode-MLP launches, nothing else")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_08314_amd import binding as B
    from paper_2605_08314_amd import bench_probe as probe

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(260508314)
    L, Bt = args.layers, args.batch
    if args.pmc_mode:
        L = min(L, 8)
    if args.attention_only:
        print(json.dumps({"attention_only": True, "decode_attention": run_decode_attention(torch, B, gen)}))
        return
    if args.prefill_only:
        print(json.dumps({"prefill_only": True, "prefill": run_prefill(torch, B, gen, Layer(torch, gen=gen), args.prefill_rows),
                          "prefill_attention": run_prefill_attention(torch, B, gen, args.prefill_rows),
                          "prefill_factorized_attention": run_prefill_factorized_attention(torch, B, gen, args.prefill_rows)}))
        return
    layers = [Layer(torch, gen=gen) for _ in range(L)]
    panels = not args.row_major
    if panels:
        for ly in layers:
            ly.make_panels(torch, B)
        torch.cuda.synchronize()
    S_max = 64
    bf = torch.bfloat16

    def decode_buffers(Bn):
        x = torch.randn((Bn, D), device="cuda", generator=gen).to(bf)
        a = torch.randn((Bn, D), device="cuda", generator=gen).to(bf)
        q, k, v, o, m = (torch.empty((Bn, D), device="cuda", dtype=bf) for _ in range(5))
        kc = torch.zeros((L, Bn, S_max, HEADS, HEAD_DIM), device="cuda", dtype=bf)
        vc = torch.zeros_like(kc)
        pos = torch.randint(0, S_max, (Bn,), device="cuda", dtype=torch.int32, generator=gen)
        ws_qkv = B.new_workspace(B.LR_OP_QKV, Bn, D, 3 * R_ATTN, 3 * D, B.LR_BF16, "decode")
        ws_o = B.new_workspace(B.LR_OP_LINEAR, Bn, D, R_ATTN, D, B.LR_BF16, "decode")
        ws_mlp = B.new_workspace(B.LR_OP_PACKED_MLP, Bn, D, 3 * R_MLP, FFN, B.LR_BF16, "decode")
        return dict(x=x, a=a, q=q, k=k, v=v, o=o, m=m, kc=kc, vc=vc, pos=pos, ws_qkv=ws_qkv, ws_o=ws_o, ws_mlp=ws_mlp)

    def make_ops(pan):
        def fac(ly):
            return ly.P if pan else dict(U=ly.U, V=ly.V, U_gu=ly.U_gu, V_g=ly.V_g, V_u=ly.V_u, U_d=ly.U_d, V_d=ly.V_d)

        def op_qkv(buf, li):
            f = fac(layers[li])
            B.lowrank_qkv(buf["x"], f["U"][:3], f["V"][:3], None, [buf["q"], buf["k"], buf["v"]],
                          dict(k_cache=buf["kc"][li], v_cache=buf["vc"][li], pos=buf["pos"], tokens_per_seq=1, k_index=1, v_index=2),
                          "decode", buf["ws_qkv"], panels=pan)

        def op_o(buf, li):
            f = fac(layers[li])
            B.lowrank_linear(buf["a"], f["U"][3], f["V"][3], None, buf["o"], "decode", buf["ws_o"], panels=pan)

        def op_mlp(buf, li):
            f = fac(layers[li])
            B.lowrank_packed_mlp(buf["x"], f["U_gu"], f["V_g"], f["V_u"], f["U_d"], f["V_d"], None, None, None, buf["m"], "decode",
                                 buf["ws_mlp"], panels=pan)
        return op_qkv, op_o, op_mlp

    op_qkv, op_o, op_mlp = make_ops(panels)

    def sweep(buf, ops):
        for li in range(L):
            for op in ops:
                op(buf, li)

    if args.pmc_mode:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        buf = decode_buffers(Bt)
        for _ in range(4):
            probe.copy(dst, src)
        for _ in range(4):
            sweep(buf, (op_mlp,))
        torch.cuda.synchronize()
        B.lowrank_workspace_status(buf["ws_mlp"])
        print(json.dumps({"pmc_mode": True, "copy_bytes": 256 << 20, "mlp_launches": 4 * L, "mlp_bytes_per_launch": mlp_bytes(Bt)}))
        return

    # ---- the timed step: exactly --steps passes over the L-layer stack at B = --batch.
    # The step's 3L launches are recorded once into a HIP graph and replayed (the paper's
    # per-layer graph replay, Section 3.1, is the same idea); --eager times plain launches.
    buf = decode_buffers(Bt)
    step_eager = lambda: sweep(buf, (op_qkv, op_o, op_mlp))
    step = step_eager if args.eager else capture(torch, step_eager)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step = e0.elapsed_time(e1) / args.steps
    for k in ("ws_qkv", "ws_o", "ws_mlp"):
        B.lowrank_workspace_status(buf[k])
    qkv_b, o_b = attn_bytes(Bt)
    step_bytes = L * (qkv_b + o_b + mlp_bytes(Bt))
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- dominant kernel family alone: decode packed MLP, rotated over the L layers
    mlp_sweep = (lambda: sweep(buf, (op_mlp,))) if args.eager else capture(torch, lambda: sweep(buf, (op_mlp,)))
    mlp_ms = time_region(torch, mlp_sweep, max(3, args.steps // 2), 2) / L
    mlp_gbs = mlp_bytes(Bt) / (mlp_ms * 1e-3) / 1e9
    # what a kernel that only streams a buffer of the same size reaches on this machine (context for `frac`)
    big = torch.empty(L * mlp_bytes(Bt) // 16 * 16, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    per = mlp_bytes(Bt) // 16 * 16
    slices = [big[i * per:(i + 1) * per] for i in range(L)]
    def read_sweep():
        for sl in slices:
            probe.read(sl, sink)
    read_ms = time_region(torch, read_sweep if args.eager else capture(torch, read_sweep), max(3, args.steps // 2), 2) / L
    del big, slices
    roofline = {"bound": "hbm", "kernel": "lowrank_packed_mlp decode (k_decode_fused_mlp, all four stages of one call)",
                "achieved": round(mlp_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(mlp_gbs / HBM_PEAK_GBS, 4), "traffic": MLP_TRAFFIC_BYTES if Bt == 1 else None,
                "traffic_source": TRAFFIC_SOURCE if Bt == 1 else None,
                "bytes_per_launch": mlp_bytes(Bt), "us_per_launch": round(mlp_ms * 1e3, 2),
                "stream_read_same_size_GBps": round(per / (read_ms * 1e-3) / 1e9, 1)}

    out = {
        "metric": "decode GB/s (% HBM peak) + prefill TFLOP/s, Llama-7B-shaped rank-r layers",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"decode step, {L} LLaMA-7B-shaped low-rank layers (QKV+cache r=384, O r=384, packed MLP r=768), B={Bt}",
                   "layers": L, "batch": Bt, "d": D, "ffn": FFN, "r_attn": R_ATTN, "r_mlp": R_MLP,
                   "factor_layout": ("64-column panels, prepacked once with lowrank_pack_panels (decode); row-major (prefill)" if panels
                                     else "row-major")},
        "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
        "tokens_per_s": round(Bt / (ms_per_step * 1e-3), 1),
        "host_wall_ms_per_step": round(wall_ms, 4), "launch": "eager" if args.eager else "hip_graph_replay",
        "roofline": roofline,
    }

    if not args.quick:
        # ---- per-entry-point decode table (in the factor layout of the step; on the row-major factors for two batch sizes as well)
        def ops_table(batches, ops):
            table = {}
            for Bn in batches:
                b2 = buf if Bn == Bt else decode_buffers(Bn)
                row = {}
                for name, op, nbytes in (("qkv", ops[0], attn_bytes(Bn)[0]), ("o", ops[1], attn_bytes(Bn)[1]), ("mlp", ops[2], mlp_bytes(Bn))):
                    fn = (lambda: sweep(b2, (op,))) if args.eager else capture(torch, lambda: sweep(b2, (op,)))
                    ms = time_region(torch, fn, 10, 2) / L
                    row[name] = {"us": round(ms * 1e3, 2), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}
                for k in ("ws_qkv", "ws_o", "ws_mlp"):
                    B.lowrank_workspace_status(b2[k])
                table[f"B{Bn}"] = row
                if b2 is not buf:
                    del b2
            return table
        out["decode_ops"] = ops_table(sorted({1, 4, 8, 16, 32}), (op_qkv, op_o, op_mlp))
        if panels:
            out["decode_ops_row_major"] = ops_table([1, 32], make_ops(False))

        out["prefill"] = run_prefill(torch, B, gen, layers[0], args.prefill_rows)
        out["prefill_ranks"] = run_prefill_ranks(torch, B, gen)
        out["shared_basis"] = run_shared_basis(torch, B, gen)
        out["prefill_attention"] = run_prefill_attention(torch, B, gen, args.prefill_rows)
        out["prefill_factorized_attention"] = run_prefill_factorized_attention(torch, B, gen, args.prefill_rows)
        out["decode_attention"] = run_decode_attention(torch, B, gen)

        # ---- CPU baseline: the oracle as it stands, on this machine's host cores, bounded sample
        import numpy as np
        import oracle
        from paper_2605_08314_amd import synth
        Bs = 32
        wa = synth.attention_layer(Bs)
        wmlp = synth.mlp_layer(Bs)
        ta, tm = wa.t, wmlp.t
        t_start = time.perf_counter()
        reps = 0
        while True:
            oracle.qkv(ta["x"].f64, [ta["U_" + n].f64 for n in "qkv"], [ta["V_" + n].f64 for n in "qkv"])
            oracle.linear(ta["a"].f64, ta["U_o"].f64, ta["V_o"].f64)
            oracle.packed_mlp(tm["x"].f64, tm["U_gu"].f64, tm["V_g"].f64, tm["V_u"].f64, tm["U_d"].f64, tm["V_d"].f64)
            reps += 1
            el = time.perf_counter() - t_start
            if el > 12.0 or reps >= 2000:      # about 12 s of CPU work
                break
        # the same layer at B = 1 (the batch of the timed step): one row, hence one thread
        x1, a1, m1 = ta["x"].f64[:1], ta["a"].f64[:1], tm["x"].f64[:1]
        t1 = time.perf_counter()
        reps1 = 0
        while True:
            oracle.qkv(x1, [ta["U_" + n].f64 for n in "qkv"], [ta["V_" + n].f64 for n in "qkv"])
            oracle.linear(a1, ta["U_o"].f64, ta["V_o"].f64)
            oracle.packed_mlp(m1, tm["U_gu"].f64, tm["V_g"].f64, tm["V_u"].f64, tm["U_d"].f64, tm["V_d"].f64)
            reps1 += 1
            el1 = time.perf_counter() - t1
            if el1 > 4.0 or reps1 >= 200:
                break
        layer_bytes = sum(attn_bytes(Bs)) + mlp_bytes(Bs)
        out["cpu_baseline"] = {"value": round(reps * layer_bytes / el / 1e9, 3), "unit": "GB/s",
                               "cores": min(Bs, oracle.num_threads()), "kind": "oracle",
                               "sample": f"{reps} layer(s) of the same stack at B={Bs} (fp64 oracle, rows parallel over OpenMP threads)",
                               "tokens_per_s": round(reps * Bs / el / L, 3),
                               "B1": {"ms_per_layer": round(el1 / reps1 * 1e3, 2), "cores": 1,
                                      "GBps": round(reps1 * (sum(attn_bytes(1)) + mlp_bytes(1)) / el1 / 1e9, 3),
                                      "tokens_per_s": round(reps1 / el1 / L, 3)}}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
