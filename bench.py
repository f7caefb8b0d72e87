#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One step = one pass of the hot path over one batch of the named synthetic
workload: gate -> permute -> grouped FFN forward -> combine, plus (for the
workloads that train) combine backward -> grouped FFN backward -> permute
backward -> gate backward.  Inputs are resident in HBM before the timed region.
The default workload is the Mixtral-8x7B-shaped layer at 16K tokens per device,
forward + backward (the largest configuration that the metric is quoted on).
Prints ONE JSON line.  `value` is tokens/s of the whole step; `roofline` prices
the grouped-FFN kernels (the dominant ones) against the dense bf16 MFMA peak
with HIP events recorded around them inside the timed steps; `roofline_hbm`
prices the row-copy stages against the HBM peak; `other_workloads` holds the
same figures for the other configurations (fewer steps); `ceilings` are what a
plain device copy and a dense one-expert problem through the same GEMM kernel
reach on this machine in this run (with the vendor library's plain GEMM beside
them); `saved_as` is a short run of the same workload with the other form of
saved activations (--saved); `cpu_baseline` is the CPU oracle timed on a
bounded sample of the same workload.
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
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def cpu_baseline(w, inp, target_seconds=15.0):
    """The oracle (fp32 instantiation, as it stands) on the first Ts tokens of the same workload."""
    import numpy as np
    from oracle import oracle as O
    from paper_2602_11686_amd import inputs as I
    cores = min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "1000000")))
    f = {n: I.widen(v, np.float32) for n, v in inp.items()}

    def run(ts):
        t0 = time.perf_counter()
        fw = O.layer_fwd(f["x"][:ts], f["w_gate"], f["bias"], f["w1"], f["w3"], f["w2"], w.k)
        if w.backward:
            O.layer_bwd(f["x"][:ts], f["w_gate"], f["w1"], f["w3"], f["w2"], fw, f["dy"][:ts])
        return time.perf_counter() - t0

    run(min(w.T, 64))                              # warms the library and the thread pool
    ts, dt = min(w.T, 256), None
    for _ in range(4):                             # grow the sample until it takes >= 10 s or is the whole batch
        dt = run(ts)
        if dt >= 10.0 or ts >= w.T:
            break
        ts = int(min(w.T, max(2 * ts, ts * target_seconds / max(dt, 1e-3)))) // 64 * 64
    reps, total = 1, dt
    while total < 10.0 and reps < 64:              # whole batch still short: repeat it
        total += run(ts)
        reps += 1
    return {"value": ts * reps / total, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"first {ts} of {w.T} tokens of {w.name} (all {w.E} experts' weights), "
                      f"{'fwd+bwd' if w.backward else 'fwd'}, fp32 oracle, {reps} pass(es), {total:.1f} s"}


def cold_leg(w, s, g, buf, perm_bytes, comb_bytes, sets=4, rounds=6):
    """permute and combine with their row buffers rotated over several sets (together well beyond the
    256 MB memory-side cache plus the L2s), so that every call streams from and to HBM."""
    import torch
    from paper_2602_11686_amd import binding as B
    xs = [torch.empty_like(g["x"]).copy_(g["x"]) for _ in range(sets)]
    xps = [torch.empty_like(buf.x_perm) for _ in range(sets)]
    ys = [torch.empty_like(buf.y) for _ in range(sets)]
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn):
        for q in range(sets):
            fn(q)
        e0, e1 = ev(), ev()
        e0.record()
        for r in range(rounds):
            for q in range(sets):
                fn(q)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (rounds * sets)

    p_ms = timed(lambda q: B.moe_permute(s, xs[q], buf.topk_ids, buf.counts, buf.offsets, buf.row_of_pair,
                                         buf.pair_of_row, xps[q], buf.ws))
    c_ms = timed(lambda q: B.moe_unpermute_combine(s, xps[q], buf.row_of_pair, buf.topk_w, ys[q]))
    mb = sets * (xs[0].numel() + xps[0].numel() + ys[0].numel()) * xs[0].element_size() / 1e6
    return {"buffer_sets": sets, "rotated_MB": round(mb, 1),
            "permute": {"ms": round(p_ms, 4), "gbs": round(perm_bytes / (p_ms * 1e-3) / 1e9, 1)},
            "combine": {"ms": round(c_ms, 4), "gbs": round(comb_bytes / (c_ms * 1e-3) / 1e9, 1)}}


def dispatcher_leg(w, s, g, buf, counts, N=32, D=8):
    """The planner and the token dispatcher on this workload's routing, for a synthetic cluster of N devices
    in nodes of D (the paper's testbed: 4 nodes of 8): layout search on the host (C++), then the permutation
    with the lite routing folded in and the grouped FFN over replica groups, timed like the other stages."""
    import numpy as np
    import torch
    from paper_2602_11686_amd import binding as B
    from paper_2602_11686_amd import planner as P
    C = max(-(-w.E // N), min(2 if w.E <= 16 else 8, 256 // N))
    while N * C > 256:
        C -= 1
    ps = P.PlanShape(N, w.E, C, D)
    rng = np.random.default_rng(w.seed)
    Rm = rng.poisson(np.maximum(counts, 1)[None, :] * rng.uniform(0.7, 1.3, size=(N, 1))).astype(np.int64)
    Rm[0] = counts
    # cost model constants: tokens of d bf16 values over 64 GB/s links inside a node, 25 GB/s between nodes,
    # 6 d f FLOPs per token at 1 PFLOP/s
    cost = P.PlanCost(v_comm=2.0 * w.d, b_intra=64e9, b_inter=25e9, v_comp=6.0 * w.d * w.f, b_comp=1e15, f_ckpt=0)
    t0 = time.perf_counter()
    A, T_model, best = P.moe_plan_expert_layout(ps, cost, Rm, 2, w.seed)
    planner_ms = (time.perf_counter() - t0) * 1e3
    received = P.moe_plan_lite_routing(ps, Rm, A).sum(axis=(0, 1))
    # static expert parallelism for comparison: EP groups of E/C consecutive devices, device i holds the C
    # experts of its position in the group (the same layout on every group)
    static = np.zeros((N, w.E), np.int32)
    if w.E % C == 0 and N % (w.E // C) == 0:
        for i in range(N):
            p_ep = w.E // C
            static[i, (i % p_ep) * C:(i % p_ep) * C + C] = 1
    else:
        static[np.arange(w.E) % N, np.arange(w.E)] = 1
    received_static = P.moe_plan_lite_routing(ps, Rm, static).sum(axis=(0, 1))
    G, eog, dog, rb, rg = P.moe_plan_dispatch_table(ps, A, 0)
    dev = lambda a: torch.tensor(a, dtype=torch.int32, device="cuda")
    eog_d, rb_d, rg_d = dev(eog), dev(rb), dev(rg)
    ec = torch.empty(w.E, dtype=torch.int32, device="cuda")
    gc = torch.empty(G, dtype=torch.int32, device="cuda")
    go = torch.empty(G + 1, dtype=torch.int32, device="cuda")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn, n):
        for _ in range(3):
            fn()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    perm = lambda: B.moe_permute_lite(s, G, g["x"], buf.topk_ids, rb_d, rg_d, ec, gc, go, buf.row_of_pair,
                                      buf.pair_of_row, buf.x_perm, err, buf.ws)
    ffn = lambda: B.moe_grouped_ffn_fwd_groups(s, G, eog_d, buf.x_perm, go, g["w1"], g["w3"], g["w2"], buf.y_perm,
                                               None, None, buf.ws)
    perm_ms = timed(perm, 20)
    ffn_ms = timed(ffn, 5)
    return {"cluster": {"N": N, "D": D, "C": C, "G": G}, "planner_layout_ms": round(planner_ms, 3),
            "modelled_T_s": T_model, "device_load_max_over_mean": {"static_ep": float(received_static.max() / received_static.mean()),
                                                                    "after_relayout": float(received.max() / received.mean())},
            "permute_lite_ms": round(perm_ms, 4), "ffn_fwd_groups_ms": round(ffn_ms, 4),
            "table_errors": int(err.item())}


def fsep_leg(w, counts, N=8, D=8):
    """The FSEP parameter layout kernels on this workload's expert size, for the buffers of N ranks held
    in this GPU's memory (one node of the paper's testbed): unshard restores C experts per rank, reshard
    reduces their gradients back to shards.  GB/s = bytes read + written / time."""
    import numpy as np
    import torch
    from paper_2602_11686_amd import fsep as F
    from paper_2602_11686_amd import planner as P
    C = max(1, 2 * w.E // N)
    psi = 3 * w.d * w.f
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    el = 2 if w.dtype == "bf16" else 4
    ps = P.PlanShape(N, w.E, C, D)
    rng = np.random.default_rng(w.seed)
    Rm = rng.poisson(np.maximum(counts, 1)[None, :] * rng.uniform(0.7, 1.3, size=(N, 1))).astype(np.int64)
    cost = P.PlanCost(v_comm=2.0 * w.d, b_intra=64e9, b_inter=25e9, v_comp=6.0 * w.d * w.f, b_comp=1e15, f_ckpt=0)
    A, _, _ = P.moe_plan_expert_layout(ps, cost, Rm, 2, w.seed)
    hosted = np.full((N, C), -1, np.int32)
    for i in range(N):
        hosted[i, :A[i].sum()] = np.repeat(np.arange(w.E), A[i])
    hd = torch.tensor(hosted, device="cuda")
    shards = torch.zeros(N, w.E, psi // N, dtype=dt, device="cuda")
    restored = torch.empty(N, C, psi, dtype=dt, device="cuda")
    gsh = torch.empty(N, w.E, psi // N, dtype=dt, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn, n=5):
        fn()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    un_ms = timed(lambda: F.moe_fsep_unshard(shards, hd, restored))
    restored.normal_()
    re_ms = timed(lambda: F.moe_fsep_reshard(restored, hd, gsh))
    slots = int((hosted >= 0).sum())
    return {"ranks": N, "C": C, "psi": psi, "unshard_ms": round(un_ms, 4),
            "unshard_gbs": round(2.0 * slots * psi * el / (un_ms * 1e-3) / 1e9, 1),
            "reshard_ms": round(re_ms, 4),
            "reshard_gbs": round((slots + w.E) * psi * el / (re_ms * 1e-3) / 1e9, 1),
            "v_fsep_bytes_per_rank": C * (N - 1) * (psi // N) * el}


def run_workload(w, steps, warmup, inp=None, keep=False):
    """`warmup` untimed steps, then `steps` timed steps of the hot path on workload w.
    Returns the figures of the run (and, with keep, the device tensors for the legs that follow)."""
    import numpy as np
    import torch
    from paper_2602_11686_amd import binding as B
    from paper_2602_11686_amd import inputs as I
    from paper_2602_11686_amd.layer import MoeLayerBuffers, to_device

    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    s = B.Shape(w.T, w.d, w.f, w.E, w.k, dt)
    if inp is None:
        inp = I.layer_inputs(w)
    g = {n: (to_device(v, dt) if n != "bias" else torch.from_numpy(v).cuda()) for n, v in inp.items()}
    buf = MoeLayerBuffers(s, backward=w.backward, save_products=SAVED_AS == "products")
    torch.cuda.synchronize()

    ev = lambda: torch.cuda.Event(enable_timing=True)
    stage_names = ["gate", "permute", "ffn_fwd", "combine"] + (
        ["combine_bwd", "ffn_bwd", "permute_bwd", "gate_bwd"] if w.backward else [])
    marks = [[ev() for _ in range(len(stage_names) + 1)] for _ in range(steps)]

    def step(m=None):
        def mark(i):
            if m is not None:
                m[i].record()
        mark(0)
        B.moe_gate_topk(s, g["x"], g["w_gate"], g["bias"], buf.topk_ids, buf.topk_w, None, buf.ws); mark(1)
        B.moe_permute(s, g["x"], buf.topk_ids, buf.counts, buf.offsets, buf.row_of_pair, buf.pair_of_row,
                      buf.x_perm, buf.ws); mark(2)
        buf.ffn_fwd(g["w1"], g["w3"], g["w2"]); mark(3)
        B.moe_unpermute_combine(s, buf.y_perm, buf.row_of_pair, buf.topk_w, buf.y); mark(4)
        if w.backward:
            B.moe_combine_bwd(s, g["dy"], buf.y_perm, buf.row_of_pair, buf.topk_w, buf.dy_perm, buf.dtopk_w); mark(5)
            buf.ffn_bwd(g["w1"], g["w3"], g["w2"]); mark(6)
            B.moe_unpermute_combine(s, buf.dx_perm, buf.row_of_pair, None, buf.dx); mark(7)
            B.moe_gate_topk_bwd(s, g["x"], g["w_gate"], buf.topk_ids, buf.topk_w, buf.dtopk_w, buf.dx,
                                buf.dw_gate, buf.ws); mark(8)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(marks[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / steps
    # the same steps replayed from a HIP graph (the calls only enqueue kernels, so a step captures as it is):
    # what the launch path costs, which matters for the short layers
    graph_ms = None
    if GRAPH_LEG:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / steps
        del graph
    stage_ms = {n: float(np.mean([marks[i][j].elapsed_time(marks[i][j + 1]) for i in range(steps)]))
                for j, n in enumerate(stage_names)}
    counts = buf.counts.cpu().numpy()
    R, el = w.T * w.k, (2 if w.dtype == "bf16" else 4)

    # algorithmic work (not padded tiles, not recomputation)
    ffn_fwd_flops = 6.0 * w.d * w.f * R
    ffn_bwd_flops = 12.0 * w.d * w.f * R
    flops = ffn_fwd_flops + (ffn_bwd_flops if w.backward else 0.0)
    ffn_ms = stage_ms["ffn_fwd"] + (stage_ms["ffn_bwd"] if w.backward else 0.0)
    achieved = flops / (ffn_ms * 1e-3) / 1e12
    perm_bytes = (1 + w.k) * w.T * w.d * el + R * 12
    comb_bytes = (1 + w.k) * w.T * w.d * el + R * 8
    cbwd_bytes = (1 + 2 * w.k) * w.T * w.d * el
    stages = {n: {"ms": round(v, 4)} for n, v in stage_ms.items()}
    stages["ffn_fwd"]["tflops"] = round(ffn_fwd_flops / (stage_ms["ffn_fwd"] * 1e-3) / 1e12, 2)
    hbm = {}

    def hbm_stage(name, nbytes):
        gbs = nbytes / (stage_ms[name] * 1e-3) / 1e9
        stages[name]["gbs"] = round(gbs, 1)
        hbm[name] = {"achieved": round(gbs, 1), "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes_per_launch": nbytes}
    hbm_stage("permute", perm_bytes)
    hbm_stage("combine", comb_bytes)
    if w.backward:
        stages["ffn_bwd"]["tflops"] = round(ffn_bwd_flops / (stage_ms["ffn_bwd"] * 1e-3) / 1e12, 2)
        hbm_stage("permute_bwd", comb_bytes)
        hbm_stage("combine_bwd", cbwd_bytes)
    res = {"ms_per_step": ms_per_step, "tokens_per_s": w.T / (ms_per_step * 1e-3), "stages": stages, "hbm": hbm,
           "achieved": achieved, "flops": flops, "ffn_ms": ffn_ms, "counts": counts,
           "perm_bytes": perm_bytes, "comb_bytes": comb_bytes, "graph_ms": graph_ms,
           "config": {"workload": w.name, "T": w.T, "d": w.d, "f": w.f, "E": w.E, "k": w.k,
                      "pass": "fwd+bwd" if w.backward else "fwd", "seed": w.seed,
                      "max_over_mean_load": float(counts.max() / counts.mean()),
                      "empty_experts": int((counts == 0).sum())}}
    if keep:
        res["live"] = (s, g, buf, inp)
    return res


def ceilings_leg():
    """What this machine gives, in this run, to (i) a plain device-to-device copy of 1 GiB (read + write, beyond the
    256 MB memory-side cache) and (ii) a dense one-expert problem (8192 rows, d = f = 4096, forward and
    backward) through the same grouped-GEMM kernels: the measured ceilings beside the vendor peaks."""
    import torch
    from paper_2602_11686_amd import binding as B
    ev = lambda: torch.cuda.Event(enable_timing=True)
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * (1 << 30) * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    T, d, f = 8192, 4096, 4096
    s = B.Shape(T, d, f, 1, 1, torch.bfloat16)
    gen = torch.Generator(device="cuda").manual_seed(7)
    rn = lambda *sh: (torch.randn(sh, device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
    xp, dyp, w1, w3, w2 = rn(T, d) * 50, rn(T, d) * 50, rn(1, d, f), rn(1, d, f), rn(1, f, d)
    off = torch.tensor([0, T], dtype=torch.int32, device="cuda")
    ws = torch.empty(B.moe_workspace_bytes(s), dtype=torch.uint8, device="cuda")
    yp, dxp = torch.empty_like(xp), torch.empty_like(xp)
    a, b = torch.empty(T, f, dtype=torch.bfloat16, device="cuda"), torch.empty(T, f, dtype=torch.bfloat16, device="cuda")
    dw1, dw3, dw2 = torch.empty_like(w1), torch.empty_like(w3), torch.empty_like(w2)
    fwd = lambda: B.moe_grouped_ffn_fwd(s, xp, off, w1, w3, w2, yp, a, b, ws)
    bwd = lambda: B.moe_grouped_ffn_bwd(s, xp, off, w1, w3, w2, a, b, dyp, dxp, dw1, dw3, dw2, ws)
    out = {"copy_1GiB_gbs": round(copy_gbs, 1), "copy_frac_of_hbm_peak": round(copy_gbs / PEAK_HBM_GBS, 4)}
    for name, fn, fl in (("dense_gemm_fwd_tflops", fwd, 6.0 * T * d * f), ("dense_gemm_bwd_tflops", bwd, 12.0 * T * d * f)):
        for _ in range(3):
            fn()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(fl * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    out["dense_gemm_shape"] = {"rows": T, "d": d, "f": f, "experts": 1}
    # The vendor library's plain bf16 GEMM (torch.matmul, no epilogue) in this run, as context for the dense
    # figures above: the forward's operand layout (B row-major [K, N]) and the backward's (B as [N, K]).
    del xp, dyp, w1, w3, w2, yp, dxp, a, b, dw1, dw3, dw2
    M, K, N = 8192, 4096, 8192
    am, bn, bt = rn(M, K), rn(K, N), rn(N, K)
    for name, fn in (("library_gemm_nn_tflops", lambda: am @ bn), ("library_gemm_nt_tflops", lambda: am @ bt.t())):
        for _ in range(3):
            fn()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(20):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(2.0 * M * K * N * 20 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    out["library_gemm_shape"] = {"M": M, "K": K, "N": N}
    return out


# What the forward pass keeps for the backward pass: "ab" = A and B (moe_grouped_ffn_fwd/_bwd), "products" = H,
# B*silu'(A) and silu(A) (moe_grouped_ffn_fwd_products/_bwd_products: one more saved tensor, a cheaper backward)
SAVED_AS = "ab"
# also time the steps replayed from a captured HIP graph (off for the runs the profiles are taken on)
GRAPH_LEG = True

OTHER_WORKLOADS = ["cfg2_e64k4", "cfg4_finegrained", "cfg5_skewed", "cfg5_balanced"]


def main():
    global SAVED_AS, GRAPH_LEG
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3_mixtral")
    ap.add_argument("--saved", choices=["ab", "products"], default=SAVED_AS,
                    help="what the forward pass keeps for the backward pass (see SAVED_AS)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the other configurations (other_workloads)")
    ap.add_argument("--hot-path-only", action="store_true",
                    help="time the layer only: no cold-cache, dispatcher, FSEP, ceiling, other-workload or CPU legs "
                         "(what the profiles are taken on)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device copy a few times (reference for the HBM byte counters)")
    args = ap.parse_args()
    SAVED_AS = args.saved
    GRAPH_LEG = not args.hot_path_only
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (the hot path of one device's token share); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_11686_amd import binding as B
    from paper_2602_11686_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    B.lib()  # fail loudly if the HIP library is not built

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "repeats": 5}))
        return

    w = I.WORKLOADS[args.workload]
    r = run_workload(w, args.steps, args.warmup, keep=True)
    s, g, buf, inp = r.pop("live")
    counts = r["counts"]

    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):  # bytes between L2 and the fabric for the grouped-FFN kernels, rocprofv3 --pmc (profiles/)
        with open(tpath) as fh:
            rec = json.load(fh).get(w.name, {})
        traffic = rec.get("ffn_hbm_bytes_per_step")
        if traffic is not None:
            traffic_source = "profiles/traffic.json (committed rocprofv3 --pmc run, not measured in this run): " + rec.get("source", "")

    out = {
        "metric": "MoE-layer tokens/s; grouped-GEMM bf16 TFLOP/s and % MFMA peak, 1 GPU",
        "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": r["config"],
        "roofline": {"bound": "mfma", "achieved": r["achieved"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": r["achieved"] / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "grouped FFN (moe_grouped_ffn_fwd" + ("+bwd" if w.backward else "") + ")",
                     "flops_per_launch": r["flops"], "ms_per_launch": r["ffn_ms"]},
        "roofline_hbm": {"bound": "hbm", "peak": PEAK_HBM_GBS, "unit": "GB/s", "stages": r["hbm"]},
        "stages": r["stages"],
    }
    if r["graph_ms"] is not None:
        out["hip_graph_replay"] = {"ms_per_step": round(r["graph_ms"], 4), "steps": args.steps,
                                   "note": "the same step captured once and replayed; the headline is the eager loop"}
    if not args.hot_path_only:
        out["cold_cache"] = cold_leg(w, s, g, buf, r["perm_bytes"], r["comb_bytes"])
        for n in ("permute", "combine"):
            out["cold_cache"][n]["frac"] = round(out["cold_cache"][n]["gbs"] / PEAK_HBM_GBS, 4)
        out["dispatcher"] = dispatcher_leg(w, s, g, buf, counts)
        out["fsep_layout"] = fsep_leg(w, counts)
    cpu = None
    if not args.no_cpu_baseline and not args.hot_path_only:
        cpu = cpu_baseline(w, inp)
    if not args.hot_path_only and w.backward:
        # the same workload with the other form of saved activations, as a short leg beside the headline
        del buf
        torch.cuda.empty_cache()
        headline_form = SAVED_AS
        SAVED_AS = "products" if headline_form == "ab" else "ab"
        o = run_workload(w, steps=20, warmup=5, inp=inp)
        out["saved_as"] = {"headline": headline_form,
                           SAVED_AS: {"ms_per_step": round(o["ms_per_step"], 4), "ffn_tflops": round(o["achieved"], 1),
                                      "frac": round(o["achieved"] / PEAK_BF16_TFLOPS, 4), "steps": 20, "warmup": 5,
                                      "ffn_fwd_ms": o["stages"]["ffn_fwd"]["ms"], "ffn_bwd_ms": o["stages"]["ffn_bwd"]["ms"]}}
        SAVED_AS = headline_form
        buf = None
    del s, g, buf, inp
    torch.cuda.empty_cache()
    if not args.hot_path_only:
        out["ceilings"] = ceilings_leg()
        torch.cuda.empty_cache()
    if not args.hot_path_only and not args.no_other_workloads:
        others, shared = {}, {}
        for name in OTHER_WORKLOADS:
            if name == w.name:
                continue
            ow = I.WORKLOADS[name]
            # the two routings of the re-layout comparison share tokens and weights (same seed); only the bias differs
            key = (ow.seed, ow.T, ow.d, ow.f, ow.E, ow.k, ow.dtype)
            oinp = shared.get(key)
            if oinp is None:
                shared.clear()
                oinp = shared[key] = I.layer_inputs(ow)
            oinp = dict(oinp, bias=I.gate_bias(ow))
            # short layers get more steps, so that every timed region is some 0.2 s long (the clocks settle)
            o_steps = 200 if ow.d * ow.f * ow.T * ow.k < 2 ** 40 else (60 if not ow.backward or ow.d * ow.f < 2 ** 24 else 20)
            o = run_workload(ow, steps=o_steps, warmup=10, inp=oinp)
            others[name] = {"ms_per_step": round(o["ms_per_step"], 4), "tokens_per_s": round(o["tokens_per_s"], 1),
                            "pass": o["config"]["pass"], "max_over_mean_load": o["config"]["max_over_mean_load"],
                            "empty_experts": o["config"]["empty_experts"], "steps": o_steps, "warmup": 10,
                            "ffn_tflops": round(o["achieved"], 1), "frac": round(o["achieved"] / PEAK_BF16_TFLOPS, 4),
                            "hip_graph_replay_ms_per_step": None if o["graph_ms"] is None else round(o["graph_ms"], 4),
                            "hbm": {n: {"gbs": v["achieved"], "frac": v["frac"]} for n, v in o["hbm"].items()}}
            torch.cuda.empty_cache()
        if "cfg5_skewed" in others and "cfg5_balanced" in others:
            others["cfg5_skewed_over_balanced_step_time"] = round(
                others["cfg5_skewed"]["ms_per_step"] / others["cfg5_balanced"]["ms_per_step"], 4)
        out["other_workloads"] = others
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
