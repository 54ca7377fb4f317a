#!/usr/bin/env python3
"""Benchmark of the Cartridge hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic inputs already
resident in HBM: cartridge attention forward + backward at the Llama-8B-shaped layer (cfg3), the
fused context-distillation loss (cfg4) and one serve-time decode step over a shared cartridge
(cfg5).  Prints ONE JSON line.  `value` is the attention forward+backward throughput in
algorithmic TFLOP/s (4*D flops per visible (query,key) pair forward, 10*D backward); the loss
and decode rates in algorithmic GB/s ride along in "parts".

python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "bench_step_hbm_traffic.md")


def profiled_traffic(kernel: str, lib_version: int):
    """HBM bytes per launch of `kernel` at the bench workload, from the committed rocprofv3 --pmc
    summary (FETCH_SIZE and WRITE_SIZE runs of this command, scaled as the summary states), or
    None when the summary is missing or was taken with another version of the library."""
    try:
        text = open(TRAFFIC_FILE).read()
    except OSError:
        return None
    import re
    m = re.search(r"library version (\d+)", text)
    if not m or int(m.group(1)) != lib_version:
        return None
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 5 and cells[0].startswith(kernel + " (cfg3"):
            try:
                return round((float(cells[3]) + float(cells[4])) * 1e9)
            except ValueError:
                return None
    return None


def attn_pairs(cfg) -> int:
    return cfg.S * cfg.P + cfg.S * (cfg.S + 1) // 2


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2506_06266_amd import binding as cb
    from paper_2506_06266_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    cb.load()   # fails loudly when the HIP library is missing
    dev = "cuda"
    acfg, kcfg, dcfg = synth.ATTN_CONFIGS["cfg3"], synth.KL_CONFIGS["cfg4"], synth.DECODE_CONFIGS["cfg5"]

    # ---- inputs and every output / workspace buffer, allocated before the timed region ----
    a = synth.attn_inputs(acfg, dev)
    o = torch.empty_like(a["q"])
    lse = torch.empty(acfg.B, acfg.Hq, acfg.S, dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(a["q"]), torch.empty_like(a["k_own"]), torch.empty_like(a["v_own"])
    dzk = torch.empty(a["z_k"].shape, dtype=torch.float32, device=dev)
    dzv = torch.empty(a["z_v"].shape, dtype=torch.float32, device=dev)
    import ctypes as C
    lib = cb.load()
    ad = cb.attn_desc(a["q"], a["k_own"], acfg.P)
    ws_attn = torch.empty(max(lib.cart_attn_bwd_workspace(C.byref(ad)), lib.cart_attn_fwd_workspace(C.byref(ad)), 16),
                          dtype=torch.uint8, device=dev)
    kl = synth.kl_inputs(kcfg, dev)
    dlogits = torch.empty_like(kl["logits"])
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    ws_kl = torch.empty(kcfg.N * 4 + 256, dtype=torch.uint8, device=dev)
    dc = synth.decode_inputs(dcfg, dev)
    dec_o = torch.empty_like(dc["q"])
    dec_lse = torch.empty(dcfg.B, dcfg.Hq, dtype=torch.float32, device=dev)
    dd = cb.DecodeDesc(dcfg.B, dcfg.Hq, dcfg.Hkv, dcfg.D, dcfg.P, dc["k_own"].shape[0], dcfg.max_len,
                       cb.CART_BF16, 0.0, cb.IMPL_AUTO)
    ws_dec = torch.empty(max(lib.cart_decode_workspace(C.byref(dd)), 16), dtype=torch.uint8, device=dev)
    own_tokens = int(dc["k_own"].shape[0])

    def attn_fwd():
        cb.cart_attn_fwd(a["q"], a["k_own"], a["v_own"], a["z_k"], a["z_v"], o=o, lse=lse, workspace=ws_attn)

    def attn_bwd():
        cb.cart_attn_bwd(a["q"], a["k_own"], a["v_own"], a["z_k"], a["z_v"], o, lse, a["d_o"], d_q=dq,
                         d_k_own=dk, d_v_own=dv, d_z_k=dzk, d_z_v=dzv, workspace=ws_attn)

    def kl_step():
        cb.cart_distill_kl_fwd_bwd(kl["logits"], kl["teacher_idx"], kl["teacher_logp"], kcfg.scale,
                                   d_logits=dlogits, loss=loss, workspace=ws_kl)

    def dec_step():
        cb.cart_decode(dc["q"], dc["z_k"], dc["z_v"], dc["k_own"], dc["v_own"], dc["cu_lens"], dcfg.max_len,
                       o=dec_o, lse=dec_lse, workspace=ws_dec)

    parts = [("attn_fwd", attn_fwd), ("attn_bwd", attn_bwd), ("kl", kl_step), ("decode", dec_step)]

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)          # a plain copy kernel: 1 GiB read, 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        for _, f in parts:
            f()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; events on the launch stream bracket every part, and
    # the library records an event at every kernel boundary of the backward call (trace hook)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(parts) + 1)] for _ in range(args.steps)]
    traces = [cb.KernelTrace(8) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        ev[s][0].record()
        for i, (name, f) in enumerate(parts):
            if name == "attn_bwd":
                with traces[s]:
                    f()
            else:
                f()
            ev[s][i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    part_ms = {name: sum(ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(args.steps)) / args.steps
               for i, (name, _) in enumerate(parts)}
    bwd_kernels = ["dq", "dkv", "dz_reduce"]
    k_ms = {n: 0.0 for n in bwd_kernels}
    for tr in traces:
        iv = tr.intervals_ms(4)
        for n, v in zip(bwd_kernels, iv):
            k_ms[n] += v / args.steps
        tr.close()

    # ---- rows past the step (not part of ms_per_step): the loss kernel's other two modes on the
    # same cfg4 buffers -- rest-bucket KL, and next-token cross-entropy (K = 1, no teacher_logp)
    def timed(f, n=5):
        f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n
    labels = kl["teacher_idx"][:, :1].contiguous()
    rest_ms = timed(lambda: cb.cart_distill_kl_fwd_bwd(kl["logits"], kl["teacher_idx"], kl["teacher_logp"],
                                                       kcfg.scale, mode=cb.KL_REST, d_logits=dlogits, loss=loss,
                                                       workspace=ws_kl))
    ntp_ms = timed(lambda: cb.cart_distill_kl_fwd_bwd(kl["logits"], labels, None, kcfg.scale, d_logits=dlogits,
                                                      loss=loss, workspace=ws_kl))

    # teacher records: top-20 tokens and log-probabilities of every cfg4 row
    tk_idx = torch.empty(kcfg.N, kcfg.K, dtype=torch.int32, device=dev)
    tk_lp = torch.empty(kcfg.N, kcfg.K, dtype=torch.float32, device=dev)
    topk_ms = timed(lambda: cb.cart_teacher_topk(kl["logits"], kcfg.K, teacher_idx=tk_idx, teacher_logp=tk_lp))

    # decode with the cartridge in pieces: cfg5's 8192 slots as four shared segments, and the
    # paper's serving protocol of one cartridge per request (128 requests x 2048 slots)
    quarter = dcfg.P // 4
    segs = [(dc["z_k"][:, i * quarter:(i + 1) * quarter].contiguous(), dc["z_v"][:, i * quarter:(i + 1) * quarter].contiguous())
            for i in range(4)]
    seg_ms = timed(lambda: cb.cart_decode_composed(dc["q"], segs, None, None, None, dc["k_own"], dc["v_own"],
                                                   dc["cu_lens"], dcfg.max_len, o=dec_o, lse=dec_lse))
    gen = torch.Generator(device=dev).manual_seed(77)
    pool_p = 2048
    pool_k = (0.02 * torch.randn(dcfg.B, dcfg.Hkv, pool_p, dcfg.D, generator=gen, device=dev)).to(torch.bfloat16)
    pool_v = (0.02 * torch.randn(dcfg.B, dcfg.Hkv, pool_p, dcfg.D, generator=gen, device=dev)).to(torch.bfloat16)
    cart_id = torch.arange(dcfg.B, dtype=torch.int32, device=dev)
    pool_ms = timed(lambda: cb.cart_decode_composed(dc["q"], [], pool_k, pool_v, cart_id, dc["k_own"], dc["v_own"],
                                                    dc["cu_lens"], dcfg.max_len, o=dec_o, lse=dec_lse))
    pool_bytes = 2 * pool_k.numel() * 2 + 2 * own_tokens * dcfg.Hkv * dcfg.D * 2 + 2 * dcfg.B * dcfg.Hq * dcfg.D * 2
    del pool_k, pool_v

    # the decode call as a serving loop would issue it: captured once into a HIP graph (the library
    # neither allocates nor synchronises), ten calls per replay
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dec_step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    dec_graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(dec_graph):
        for _ in range(10):
            dec_step()
    graph_ms = timed(dec_graph.replay) / 10
    del dec_graph

    # the same call through the entry point that keeps its partial results in the library's own
    # device array (one launch less to set up for the caller, the same kernels), and alone in a
    # loop (in the timed step the call follows 8 GB of loss traffic)
    static_ms = timed(lambda: cb.cart_decode_static(dc["q"], dc["z_k"], dc["z_v"], dc["k_own"], dc["v_own"],
                                                    dc["cu_lens"], dcfg.max_len, o=dec_o, lse=dec_lse), n=20)
    alone_ms = timed(dec_step, n=20)

    # the serving comparison run: no cartridge, 8 requests that each carry a 131072-token KV cache
    lcfg = synth.DECODE_CONFIGS["cfg5_long"]
    lg = synth.decode_inputs(lcfg, dev)
    lg_o, lg_lse = cb.cart_decode(lg["q"], None, None, lg["k_own"], lg["v_own"], lg["cu_lens"], lcfg.max_len)
    long_ms = timed(lambda: cb.cart_decode(lg["q"], None, None, lg["k_own"], lg["v_own"], lg["cu_lens"], lcfg.max_len,
                                           o=lg_o, lse=lg_lse))
    long_bytes = 2 * lg["k_own"].numel() * 2
    del lg, lg_o, lg_lse

    # the same decode call with the last-level cache cold: 512 MiB written between the calls
    flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    cold = []
    for i in range(6):
        flush.fill_(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dec_step()
        e1.record()
        torch.cuda.synchronize()
        cold.append(e0.elapsed_time(e1))
    decode_cold_ms = sorted(cold[1:])[len(cold[1:]) // 2]
    del flush

    # the Llama-3B-shaped layer (cfg2), forward and backward
    c2 = synth.ATTN_CONFIGS["cfg2"]
    a2 = synth.attn_inputs(c2, dev)
    o2, lse2 = cb.cart_attn_fwd(a2["q"], a2["k_own"], a2["v_own"], a2["z_k"], a2["z_v"])
    g2 = cb.cart_attn_bwd(a2["q"], a2["k_own"], a2["v_own"], a2["z_k"], a2["z_v"], o2, lse2, a2["d_o"])
    ad2 = cb.attn_desc(a2["q"], a2["k_own"], c2.P)
    ws2 = torch.empty(max(lib.cart_attn_bwd_workspace(C.byref(ad2)), lib.cart_attn_fwd_workspace(C.byref(ad2)), 16),
                      dtype=torch.uint8, device=dev)
    c2_fwd_ms = timed(lambda: cb.cart_attn_fwd(a2["q"], a2["k_own"], a2["v_own"], a2["z_k"], a2["z_v"], o=o2,
                                               lse=lse2, workspace=ws2), n=10)
    c2_bwd_ms = timed(lambda: cb.cart_attn_bwd(a2["q"], a2["k_own"], a2["v_own"], a2["z_k"], a2["z_v"], o2, lse2,
                                               a2["d_o"], d_q=g2[0], d_k_own=g2[1], d_v_own=g2[2], d_z_k=g2[3],
                                               d_z_v=g2[4], workspace=ws2), n=10)
    c2_pairs = attn_pairs(c2) * c2.B * c2.Hq
    del a2, o2, lse2, g2, ws2

    # the cfg3 step's attention kernels on all-zero inputs: the same instruction streams with no
    # switching activity in the data paths -- what the schedules would run at if the chip were not
    # power-limited under them (a statement about the machine, not a throughput claim)
    zq, zk_, zv_, zdo = (torch.zeros_like(a[n]) for n in ("q", "k_own", "v_own", "d_o"))
    zzk, zzv = torch.zeros_like(a["z_k"]), torch.zeros_like(a["z_v"])
    zero_fwd_ms = timed(lambda: cb.cart_attn_fwd(zq, zk_, zv_, zzk, zzv, o=o, lse=lse, workspace=ws_attn))
    zero_bwd_ms = timed(lambda: cb.cart_attn_bwd(zq, zk_, zv_, zzk, zzv, o, lse, zdo, d_q=dq, d_k_own=dk, d_v_own=dv,
                                                 d_z_k=dzk, d_z_v=dzv, workspace=ws_attn))
    del zq, zk_, zv_, zdo, zzk, zzv

    # what this machine gives a kernel with nothing else to do, measured in this run: a matrix-core-only
    # loop of the attention kernels' instruction, a 4 GiB device copy and a 4 GiB device read
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    peak_fl = [0.0]
    def mfma_loop():
        peak_fl[0] = cb.cart_calib_mfma(sink, 20000, 1)
    mfma_ms = timed(mfma_loop, n=3)
    peak_mfma_tflops = peak_fl[0] / mfma_ms / 1e9
    big_a = torch.empty(4 << 30, dtype=torch.uint8, device=dev).fill_(1)
    big_b = torch.empty_like(big_a)
    copy_ms = timed(lambda: cb.cart_calib_copy(big_b, big_a), n=3)
    read_ms = timed(lambda: cb.cart_calib_read(big_a, sink), n=3)
    peak_copy_gbs = 2 * big_a.numel() / copy_ms / 1e6
    peak_read_gbs = big_a.numel() / read_ms / 1e6
    del big_a, big_b

    # one packed global batch of 64 ragged conversations (<= 1024 tokens) at the same layer shape
    pcfg = synth.PACKED_CONFIGS["cfg3_packed"]
    pk = synth.attn_packed_inputs(pcfg, dev)
    plens = synth.packed_lengths(pcfg)
    pmax = int(plens.max())
    pk_o, pk_lse = cb.cart_attn_varlen_fwd(pk["q"], pk["k_own"], pk["v_own"], pk["z_k"], pk["z_v"],
                                           pk["cu_seqlens"], pmax)
    pk_g = cb.cart_attn_varlen_bwd(pk["q"], pk["k_own"], pk["v_own"], pk["z_k"], pk["z_v"], pk["cu_seqlens"], pmax,
                                   pk_o, pk_lse, pk["d_o"])
    def packed_step():
        cb.cart_attn_varlen_fwd(pk["q"], pk["k_own"], pk["v_own"], pk["z_k"], pk["z_v"], pk["cu_seqlens"], pmax,
                                o=pk_o, lse=pk_lse)
        cb.cart_attn_varlen_bwd(pk["q"], pk["k_own"], pk["v_own"], pk["z_k"], pk["z_v"], pk["cu_seqlens"], pmax,
                                pk_o, pk_lse, pk["d_o"], d_q=pk_g[0], d_k_own=pk_g[1], d_v_own=pk_g[2],
                                d_z_k=pk_g[3], d_z_v=pk_g[4])
    packed_ms = timed(packed_step)
    packed_pairs = sum(int(n) * acfg.P + int(n) * (int(n) + 1) // 2 for n in plens.tolist()) * acfg.Hq
    packed_tflops = packed_pairs * 14 * acfg.D / packed_ms / 1e9
    del pk, pk_o, pk_lse, pk_g

    pairs = attn_pairs(acfg) * acfg.B * acfg.Hq
    fwd_flop, bwd_flop = pairs * 4 * acfg.D, pairs * 10 * acfg.D
    attn_ms = part_ms["attn_fwd"] + part_ms["attn_bwd"]
    attn_tflops = (fwd_flop + bwd_flop) / (attn_ms * 1e-3) / 1e12
    kl_bytes = 2 * kcfg.N * kcfg.V * 2 + kcfg.N * kcfg.K * 8 + 4
    dec_bytes = (2 * dcfg.Hkv * dcfg.P * dcfg.D * 2 + 2 * own_tokens * dcfg.Hkv * dcfg.D * 2
                 + 2 * dcfg.B * dcfg.Hq * dcfg.D * 2)
    kl_gbs = kl_bytes / (part_ms["kl"] * 1e-3) / 1e9
    dec_gbs = dec_bytes / (part_ms["decode"] * 1e-3) / 1e9

    # Roofline of the step's dominant kernel, the slowest kernel of the backward call.  The
    # call's kernels share the algorithmic work of the gradient (10*D flops per visible pair:
    # recomputing S, then dP, dV, dQ, dK), whatever they recompute between them, so `achieved`
    # prices the call: algorithmic flops of the backward / time of its kernels.  What the dominant
    # kernel itself executes per second is reported beside it.
    units = {"dq": 3, "dkv": 4}                  # contractions each kernel performs per pair
    dom = max(units, key=lambda n: k_ms[n])
    bwd_kernel_ms = sum(k_ms.values())
    bwd_alg_tflops = bwd_flop / (bwd_kernel_ms * 1e-3) / 1e12
    dom_exec_tflops = pairs * units[dom] * 2 * acfg.D / (k_ms[dom] * 1e-3) / 1e12
    dom_name = {"dq": "attn_bwd_dq_kernel", "dkv": "attn_bwd_kv_kernel"}[dom]
    roofline = {"kernel": dom_name, "bound": "mfma", "achieved": round(bwd_alg_tflops, 1),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(bwd_alg_tflops / PEAK_BF16_TFLOPS, 4),
                "traffic": profiled_traffic(dom_name, lib.cart_version()),
                "basis": "algorithmic flops of the backward call (10*D per visible pair) / time of its kernels",
                "call_kernel_ms": round(bwd_kernel_ms, 4), "avg_launch_ms": round(k_ms[dom], 4),
                "executed_units_per_pair": sum(units.values()), "algorithmic_units_per_pair": 5,
                "kernel_executed_tflops": round(dom_exec_tflops, 1),
                "kernel_executed_frac": round(dom_exec_tflops / PEAK_BF16_TFLOPS, 4),
                "frac_of_measured_peak": round(bwd_alg_tflops / peak_mfma_tflops, 4)}

    out = {
        "metric": "cartridge attn fwd+bwd TFLOP/s (MFMA util) @Llama-8B shape; KL loss HBM GB/s",
        "value": round(attn_tflops, 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg3 attention B16 S2048 Hq32 Hkv8 D128 P4096 fwd+bwd; cfg4 loss N16384 "
                               "V128256 K20; cfg5 decode B128 P8192 own U[1,1024]"},
        "parts": {"attn_fwd_ms": round(part_ms["attn_fwd"], 4), "attn_bwd_ms": round(part_ms["attn_bwd"], 4),
                  "attn_fwd_tflops": round(fwd_flop / part_ms["attn_fwd"] / 1e9, 1),
                  "attn_bwd_tflops": round(bwd_flop / part_ms["attn_bwd"] / 1e9, 1),
                  "attn_mfma_frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                  "attn_fwd_frac": round(fwd_flop / part_ms["attn_fwd"] / 1e9 / PEAK_BF16_TFLOPS, 4),
                  "attn_bwd_frac": round(bwd_flop / part_ms["attn_bwd"] / 1e9 / PEAK_BF16_TFLOPS, 4),
                  "attn_frac_of_measured_peak": round(attn_tflops / peak_mfma_tflops, 4),
                  "bwd_kernel_ms": {n: round(v, 4) for n, v in k_ms.items()},
                  "kl_ms": round(part_ms["kl"], 4), "kl_gbs": round(kl_gbs, 1),
                  "kl_hbm_frac": round(kl_gbs / PEAK_HBM_GBS, 4),
                  "decode_ms": round(part_ms["decode"], 4), "decode_gbs": round(dec_gbs, 1),
                  "decode_hbm_frac": round(dec_gbs / PEAK_HBM_GBS, 4),
                  "decode_cold_ms": round(decode_cold_ms, 4),
                  "decode_cold_gbs": round(dec_bytes / decode_cold_ms / 1e6, 1),
                  "kl_frac_of_measured_copy": round(kl_gbs / peak_copy_gbs, 4),
                  "decode_frac_of_measured_read": round(dec_gbs / peak_read_gbs, 4),
                  "cfg2": {"workload": "Llama-3B-shaped layer B32 S1024 Hq24 Hkv8 D128 P2048",
                           "attn_fwd_ms": round(c2_fwd_ms, 4), "attn_bwd_ms": round(c2_bwd_ms, 4),
                           "attn_fwd_tflops": round(c2_pairs * 4 * c2.D / c2_fwd_ms / 1e9, 1),
                           "attn_bwd_tflops": round(c2_pairs * 10 * c2.D / c2_bwd_ms / 1e9, 1),
                           "attn_fwd_bwd_tflops": round(c2_pairs * 14 * c2.D / (c2_fwd_ms + c2_bwd_ms) / 1e9, 1),
                           "attn_mfma_frac": round(c2_pairs * 14 * c2.D / (c2_fwd_ms + c2_bwd_ms) / 1e9
                                                   / PEAK_BF16_TFLOPS, 4)}},
        "measured_peaks": {"attn_fwd_ms_on_zero_inputs": round(zero_fwd_ms, 4),
                           "attn_bwd_ms_on_zero_inputs": round(zero_bwd_ms, 4),
                           "mfma_bf16_tflops": round(peak_mfma_tflops, 1), "copy_4GiB_gbs": round(peak_copy_gbs, 1),
                           "read_4GiB_gbs": round(peak_read_gbs, 1),
                           "note": "timed in this run: the cfg3 attention calls on all-zero inputs (same instruction streams, no "
                                   "switching activity: the chip is power-limited under these kernels); plain kernels of "
                                   "this library (matrix-core-only loop; "
                                   "16-byte-per-lane copy and read of 4 GiB)"},
        "roofline": roofline,
        "next_rows": {"kl_rest_bucket_ms": round(rest_ms, 4),
                      "kl_rest_bucket_gbs": round((2 * kcfg.N * kcfg.V * 2 + kcfg.N * kcfg.K * 8) / rest_ms / 1e6, 1),
                      "ntp_cross_entropy_ms": round(ntp_ms, 4),
                      "ntp_cross_entropy_gbs": round((2 * kcfg.N * kcfg.V * 2 + kcfg.N * 4) / ntp_ms / 1e6, 1),
                      "teacher_topk_ms": round(topk_ms, 4),
                      "teacher_topk_gbs": round(kcfg.N * kcfg.V * 2 / topk_ms / 1e6, 1),
                      "decode_4_shared_segments_ms": round(seg_ms, 4),
                      "decode_cartridge_per_request_ms": round(pool_ms, 4),
                      "decode_cartridge_per_request_gbs": round(pool_bytes / pool_ms / 1e6, 1),
                      "decode_graph_replay_ms": round(graph_ms, 4),
                      "decode_alone_in_a_loop_ms": round(alone_ms, 4),
                      "decode_static_scratch_ms": round(static_ms, 4),
                      "decode_no_cartridge_8x131072_ms": round(long_ms, 4),
                      "decode_no_cartridge_8x131072_gbs": round(long_bytes / long_ms / 1e6, 1),
                      "attn_packed_64_conversations_fwd_bwd_ms": round(packed_ms, 4),
                      "attn_packed_64_conversations_tflops": round(packed_tflops, 1)},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a, acfg)
    print(json.dumps(out))
    return 0


def cpu_baseline(a, acfg):
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample of cfg3: four
    sequences x four KV groups (16 query heads), forward + backward."""
    import numpy as np
    from oracle import cartridge_oracle as orc
    try:
        allowed = len(os.sched_getaffinity(0))
    except AttributeError:
        allowed = os.cpu_count() or 1
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = allowed
    cores = min(threads, allowed)      # the BLAS pool's threads, no more than the CPUs this process may use
    G = acfg.Hq // acfg.Hkv
    f64 = lambda t: t.detach().to("cpu").double().numpy()
    NB, NK = 4, 4                      # sequences x KV groups in the sample
    q = f64(a["q"][:NB, :, :NK * G]); do = f64(a["d_o"][:NB, :, :NK * G])
    k = f64(a["k_own"][:NB, :, :NK]); v = f64(a["v_own"][:NB, :, :NK])
    zk = f64(a["z_k"][:NK]); zv = f64(a["z_v"][:NK])
    t0 = time.perf_counter()
    orc.attn_fwd(q, k, v, zk, zv)
    orc.attn_bwd(q, k, v, zk, zv, do)
    dt = time.perf_counter() - t0
    flop = attn_pairs(acfg) * NB * NK * G * 14 * acfg.D
    return {"value": round(flop / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "blas_threads": int(threads), "affinity_cpus": int(allowed),
            "sample": "cfg3 shape, 4 of 16 sequences x 16 of 32 query heads (4 KV groups), fwd+bwd, "
                      "%.1f s" % dt}


if __name__ == "__main__":
    sys.exit(main())
