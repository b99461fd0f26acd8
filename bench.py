#!/usr/bin/env python3
"""Benchmark of the sparse fully-connected training step on one MI355X.

A step is one pass of the hot path over one batch: for every layer of the workload the
forward product, the input gradient and the weight gradient at the active positions;
every Delta_t-th step (Table "Private hyperparameters of MST": topology update interval
100) each layer also runs one Mixed-Growing update (dense gradient on the matrix cores,
prune / grow selection, rebuild of the index views).  Inputs are synthetic, seeded, and
resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
ALU_FP32_PEAK_TFLOPS = 157.3   # fp32 vector peak (256 CUs x 4 SIMD x 16 lanes x 2 flop x 2 (packed) x 2.4 GHz)
MFMA_FP32_PEAK_TFLOPS = 157.3
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA peak
METRIC = "effective sparse TFLOP/s + HBM GB/s (% peak) per FC train step, 1 MI355X"


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=100)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C4", "C5"])
    p.add_argument("--update-interval", type=int, default=100, help="Delta_t; 0 = never update")
    p.add_argument("--allocation", default="uniform", choices=["uniform", "erdos_renyi"],
                   help="C5 only: every layer at the sweep's density, or the Erdos-Renyi shares of it (Sec. 3.2)")
    p.add_argument("--update-streams", type=int, default=1,
                   help="C5 only: 1 = the layers' mask updates run on one stream per layer, 0 = all on the main stream")
    p.add_argument("--fused-update", type=int, default=1,
                   help="C5 only: 1 = weight gradient and update from one dense gradient "
                        "(mst_sparse_fc_bwd_weight_update), 0 = separate calls")
    p.add_argument("--separate-bwd", action="store_true",
                   help="time mst_sparse_fc_bwd_input and mst_sparse_fc_bwd_weight as two calls instead of "
                        "mst_sparse_fc_bwd (both gradients from one walk)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--seed", type=int, default=2024)
    p.add_argument("--attention-mask", type=int, nargs=2, metavar=("L", "STRIDE"), default=None,
                   help="time the strided attention mask of Sec. 3.3 instead of a config (its own JSON line)")
    p.add_argument("--pmc-probe", action="store_true",
                   help="short run for rocprofv3 --pmc: a 1 GiB device copy (calibration), then each product twice")
    return p.parse_args()


class LayerRun:
    """Device state of one layer of the workload."""

    def __init__(self, mst, synth, torch, seed, lid, name, I, O, T, density, mask, act):
        import numpy as np
        self.name, self.I, self.O, self.T = name, I, O, T
        W, M = synth.make_layer(seed, lid, I, O, density, mask)
        self.W, self.M = W, M
        to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        if act == "f32":
            X, dY = synth.make_activations(seed, lid, T, I, O)
            self.X, self.dY, self.act = to(X), to(dY), mst.MST_F32
            self.act_bytes = 4
        else:
            Xf, dYf, xb, yb = synth.make_activations(seed, lid, T, I, O, "bf16")
            X, dY = Xf, dYf
            self.X, self.dY, self.act = to(xb.view(np.int16)), to(yb.view(np.int16)), mst.MST_BF16
            self.act_bytes = 2
        self.X_host, self.dY_host = X, dY
        self.nnz = int(M.sum())
        cap = min(O * I, self.nnz + self.nnz // 2 + 64)
        self.layer = mst.Layer(O, I, cap, "cuda:0")
        self.ws = torch.empty(mst.mst_workspace_bytes(O, I, cap, T), dtype=torch.uint8, device="cuda:0")
        self.layer.load_dense(to(W), to(M), self.ws)
        self.Y = torch.empty((T, O), dtype=torch.float32, device="cuda:0")
        self.dX = torch.empty((T, I), dtype=torch.float32, device="cuda:0")
        self.dW = torch.empty(cap, dtype=torch.float32, device="cuda:0")
        self.density = density

    # algorithmic (compulsory) bytes and flops of each product
    def bytes_fwd(self):
        return self.act_bytes * self.T * self.I + 4 * self.T * self.O + 8 * self.nnz + 4 * (self.O + 1)

    def bytes_bwd_input(self):
        return self.act_bytes * self.T * self.O + 4 * self.T * self.I + 8 * self.nnz + 4 * (self.I + 1)

    def bytes_bwd_weight(self):
        return self.act_bytes * self.T * (self.I + self.O) + 8 * self.nnz + 4 * self.nnz

    def bytes_bwd(self):
        # both gradients in one call: dY and X read once, dX and dW written, the entries read once
        return (self.act_bytes * self.T * (self.I + self.O) + 4 * self.T * self.I + 8 * self.nnz + 4 * self.nnz +
                4 * (self.I + 1))

    def flops_product(self):
        return 2 * self.nnz * self.T


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); no multi-GPU path exists", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2408_11746_amd as mst
    import synth

    if args.attention_mask:
        return attention_mask(args, mst, torch)
    cfg = synth.CONFIGS[args.config]
    if args.config == "C5":
        return sweep(args, cfg, mst, synth, torch)
    T, act, density = cfg["T"], cfg["act"], cfg["densities"][0]
    layers = [LayerRun(mst, synth, torch, args.seed, lid + 1, name, I, O, T, density, cfg["mask"], act)
              for lid, (name, I, O) in enumerate(cfg["layers"])]
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()

    if args.pmc_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)                      # 1 GiB read + 1 GiB written per launch
        # a one-element torch kernel after every call: the boundary between the calls' dispatches
        mark = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        mark.add_(1)
        for L in layers:
            for _ in range(2):
                mst.mst_sparse_fc_fwd(L.layer, L.X, L.Y, T, L.act, stream)
                mark.add_(1)
                if args.separate_bwd:
                    mst.mst_sparse_fc_bwd_input(L.layer, L.dY, L.dX, T, L.act, stream)
                    mark.add_(1)
                    mst.mst_sparse_fc_bwd_weight(L.layer, L.dY, L.X, L.dW, T, L.ws, L.act, stream)
                else:
                    mst.mst_sparse_fc_bwd(L.layer, L.dY, L.X, L.dX, L.dW, T, L.ws, L.act, stream)
                mark.add_(1)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "copy_bytes_each_way": 1 << 30,
                          "layers": {L.name: dict(I=L.I, O=L.O, nnz=L.nnz) for L in layers}}))
        return

    products = ("fwd", "bwd_input", "bwd_weight") if args.separate_bwd else ("fwd", "bwd")
    kinds = products + ("sync_values", "mask_update")
    ev = {(L.name, k): [] for L in layers for k in kinds}

    def run_step(t, record):
        # one event between consecutive calls: the end of a call is the start of the next
        def mark():
            e = torch.cuda.Event(enable_timing=True)
            e.record(stream)
            return e

        last = mark() if record else None
        for L in layers:
            # the three products, then the hand-over of the (optimiser-updated) active weights
            # to the index views, which a training step pays once per layer
            for kind in products + ("sync_values",):
                if kind == "fwd":
                    mst.mst_sparse_fc_fwd(L.layer, L.X, L.Y, T, L.act, stream)
                elif kind == "bwd":
                    mst.mst_sparse_fc_bwd(L.layer, L.dY, L.X, L.dX, L.dW, T, L.ws, L.act, stream)
                elif kind == "bwd_input":
                    mst.mst_sparse_fc_bwd_input(L.layer, L.dY, L.dX, T, L.act, stream)
                elif kind == "bwd_weight":
                    mst.mst_sparse_fc_bwd_weight(L.layer, L.dY, L.X, L.dW, T, L.ws, L.act, stream)
                else:
                    L.layer.sync_values(stream)
                if record:
                    nxt = mark()
                    ev[(L.name, kind)].append((last, nxt))
                    last = nxt
        if args.update_interval and (t + 1) % args.update_interval == 0:
            for li, L in enumerate(layers):
                mst.mst_mask_update(L.layer, L.dY, L.X, T, density, cfg["zeta"], cfg["R"],
                                    args.seed * 1000003 + t * 131 + li, L.ws, L.act, stream)
                if record:
                    nxt = mark()
                    ev[(L.name, "mask_update")].append((last, nxt))
                    last = nxt

    t = 0
    for _ in range(args.warmup):
        run_step(t, False)
        t += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step(t, True)
        t += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    n_updates = sum(len(ev[(L.name, "mask_update")]) for L in layers) // max(1, len(layers))
    ms_per_step = 1e3 * elapsed / args.steps
    sparse_flops_step = sum(3 * L.flops_product() for L in layers)
    bytes_step = sum(L.bytes_fwd() + (L.bytes_bwd_input() + L.bytes_bwd_weight() if args.separate_bwd else L.bytes_bwd())
                     for L in layers)
    value = sparse_flops_step / (elapsed / args.steps) / 1e12

    # per-call device times from the events recorded inside the timed region
    table, dominant = [], None
    for L in layers:
        for kind in kinds:
            pairs = ev[(L.name, kind)]
            if not pairs:
                continue
            ms = sum(a.elapsed_time(b) for a, b in pairs) / len(pairs)
            row = dict(layer=L.name, call=kind, launches=len(pairs), avg_ms=round(ms, 5))
            if kind in products:
                by = getattr(L, "bytes_" + kind)()
                fl = L.flops_product() * (2 if kind == "bwd" else 1)
                row.update(eff_tflops=round(fl / ms / 1e9, 3), hbm_gbs=round(by / ms / 1e6, 1),
                           hbm_frac=round(by / ms / 1e6 / HBM_PEAK_GBS, 4),
                           alu_frac=round(fl / ms / 1e9 / ALU_FP32_PEAK_TFLOPS, 4),
                           alg_bytes=by, alg_flops=fl)
                tot = ms * len(pairs)
                if dominant is None or tot > dominant[0]:
                    dominant = (tot, row, L)
            elif kind == "mask_update":
                row.update(dense_grad_gflop=round(2 * T * L.O * L.I / 1e9, 2))
            table.append(row)

    _, drow, dL = dominant
    t_hbm = drow["alg_bytes"] / (HBM_PEAK_GBS * 1e9)
    t_alu = drow["alg_flops"] / (ALU_FP32_PEAK_TFLOPS * 1e12)
    # fwd / bwd_input are one k_spmm launch; bwd_weight is k_sddmm followed by the small k_sddmm_reduce
    dense_bww = act == "bf16" and density > 0.045 and T >= 2048
    if dense_bww:          # the bf16 MFMA weight gradient is faster than any sparse kernel here
        bwd_kernels = "k_spmm64 + k_gemm_tn_bf16 + k_gather_flat (separate kernels)"
    else:
        bwd_kernels = "k_bwd_fused + k_bwd_fused_reduce"
    kernel = {"fwd": "k_spmm / k_spmm64 (launch shape chosen per call)",
              "bwd_input": "k_spmm / k_spmm64 (launch shape chosen per call)",
              "bwd_weight": "k_sddmm+k_sddmm_reduce", "bwd": bwd_kernels}[drow["call"]]
    # with bfloat16 activations the library computes the weight gradient as the full MFMA
    # product dY^T X read at the active positions from a density of 0.045 on (T >= 2048)
    mfma_bww = drow["call"] == "bwd_weight" and act == "bf16" and density > 0.045 and T >= 2048
    if mfma_bww:
        kernel = "k_gemm_tn_bf16+k_gather_flat"
        dense_tf = 2.0 * T * dL.O * dL.I / drow["avg_ms"] / 1e9
        roof = dict(bound="mfma", achieved=round(dense_tf, 1), peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=round(dense_tf / MFMA_BF16_PEAK_TFLOPS, 4))
    elif t_hbm >= t_alu:
        roof = dict(bound="hbm", achieved=drow["hbm_gbs"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(drow["hbm_gbs"] / HBM_PEAK_GBS, 4))
    else:
        roof = dict(bound="alu", achieved=drow["eff_tflops"], peak=ALU_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=round(drow["eff_tflops"] / ALU_FP32_PEAK_TFLOPS, 4))
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s.json" % args.config.lower())
    if os.path.exists(tpath):        # counter-based HBM bytes of this call, measured by the commands in profiles/
        traffic = json.load(open(tpath)).get("calls", {}).get("%s/%s" % (dL.name, drow["call"]))
    roof.update(traffic=traffic, kernel=kernel, call="%s/%s" % (dL.name, drow["call"]),
                avg_launch_ms=drow["avg_ms"], alg_bytes_per_launch=drow["alg_bytes"],
                alg_flops_per_launch=drow["alg_flops"], hbm_frac=drow["hbm_frac"], alu_frac=drow["alu_frac"])

    out = {
        "metric": METRIC, "value": round(value, 4), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if act == "f32" else "bf16-in/f32-acc",
        "data": "synthetic",
        "config": {"workload": "%s: %s FC set (%s), density %.2f %s mask, T=%d tokens, %s "
                               "+ value hand-over to the index views per layer, Mixed-Growing update every %d steps"
                               % (args.config, "GPT-2-small block" if len(layers) > 1 else "single layer",
                                  ", ".join("%s %d->%d" % (L.name, L.I, L.O) for L in layers), density,
                                  cfg["mask"], T,
                                  "fwd+bwd_input+bwd_weight" if args.separate_bwd
                                  else "fwd + bwd (input and weight gradient in one call)", args.update_interval),
                   "nnz": {L.name: L.nnz for L in layers}, "mask_updates_in_timed_region": n_updates},
        "hbm_gbs_step": round(bytes_step / (elapsed / args.steps) / 1e9, 1),
        "hbm_frac_step": round(bytes_step / (elapsed / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
        "roofline": roof,
        "calls": table,
    }

    # MFMA utilisation of the dense gradient G = dY^T X that scores gradient growth (outside the
    # timed region: it runs once per update inside mst_mask_update)
    G = torch.empty(max(L.O * L.I for L in layers), dtype=torch.float32, device="cuda:0")
    dg = {}
    peak = MFMA_BF16_PEAK_TFLOPS if act == "bf16" else MFMA_FP32_PEAK_TFLOPS
    for L in layers:
        for _ in range(2):
            mst.mst_dense_grad(L.dY, L.X, G, T, L.O, L.I, L.act, L.ws, stream)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(5):
            mst.mst_dense_grad(L.dY, L.X, G, T, L.O, L.I, L.act, L.ws, stream)
        b.record(stream)
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / 5
        tf = 2.0 * T * L.O * L.I / ms / 1e9
        dg[L.name] = dict(avg_ms=round(ms, 4), tflops=round(tf, 1), mfma_frac=round(tf / peak, 4))
    out["dense_grad_gemm"] = dict(dtype="bf16" if act == "bf16" else "f32", peak_tflops=peak, layers=dg)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layers, T)
    print(json.dumps(out))


def attention_mask(args, mst, torch):
    """The [L x L] byte mask of the strided pattern: a write-only kernel, L * L algorithmic bytes."""
    L, stride = args.attention_mask
    stream = torch.cuda.current_stream()
    M = torch.empty(L * L, dtype=torch.uint8, device="cuda:0")
    for _ in range(max(1, args.warmup)):
        mst.mst_strided_attention_mask(M, L, stride, stream)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    a.record(stream)
    for _ in range(args.steps):
        mst.mst_strided_attention_mask(M, L, stride, stream)
    b.record(stream)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / args.steps
    ms = a.elapsed_time(b) / args.steps
    gbs = L * L / ms / 1e6
    kept = mst.mst_strided_attention_count(L, stride)
    assert int(M.sum(dtype=torch.int64).item()) == kept
    print(json.dumps({
        "metric": "strided attention mask build, HBM GB/s written", "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(1e3 * wall, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "strided attention mask, L=%d, stride=%d" % (L, stride), "q_atten": kept / (L * L)},
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "kernel": "k_strided_mask16",
                     "avg_launch_ms": round(ms, 5), "alg_bytes_per_launch": L * L}}))


def sweep(args, cfg, mst, synth, torch):
    """Config C5: one GPT-2-large block (of 36 identical ones) swept through the densities
    1.0, 0.5, 0.1, 0.02, 0.1, 0.5; every transition is produced by the fused mask update itself
    and every step also runs one update at the current density (mask update every step)."""
    import numpy as np
    T = cfg["T"]
    stream = torch.cuda.current_stream()
    layers = []
    for lid, (name, I, O) in enumerate(cfg["layers"]):
        L = LayerRun.__new__(LayerRun)
        L.name, L.I, L.O, L.T, L.act, L.act_bytes = name, I, O, T, mst.MST_F32, 4
        W = synth.normal(args.seed, 1000 * (lid + 1) + 2, (O, I), 0.02)
        M = np.ones((O, I), np.uint8)
        X, dY = synth.make_activations(args.seed, lid + 1, T, I, O)
        L.X, L.dY = torch.from_numpy(X).cuda(), torch.from_numpy(dY).cuda()
        cap = O * I
        L.layer = mst.Layer(O, I, cap, "cuda:0")
        L.ws = torch.empty(mst.mst_workspace_bytes(O, I, cap, T), dtype=torch.uint8, device="cuda:0")
        L.layer.load_dense(torch.from_numpy(W).cuda(), torch.from_numpy(M).cuda(), L.ws)
        L.Y = torch.empty((T, O), dtype=torch.float32, device="cuda:0")
        L.dX = torch.empty((T, I), dtype=torch.float32, device="cuda:0")
        L.dW = torch.empty(cap, dtype=torch.float32, device="cuda:0")
        layers.append(L)
    torch.cuda.synchronize()
    steps = max(1, args.steps // len(cfg["densities"]))
    rows, tot_time, tot_flops, seed = [], 0.0, 0.0, args.seed * 7919

    # The products of the block run in order on one stream.  The updates of different layers
    # are independent (each has its own workspace): they are issued on one stream per layer,
    # so that the many small selection and format kernels of one layer fill the gaps of the
    # others; the next step's products wait for all of them.  All streams at default priority.
    side = [torch.cuda.Stream() for _ in layers] if args.update_streams else [stream] * len(layers)

    def one_step(dl):
        nonlocal seed
        for L in layers:
            mst.mst_sparse_fc_fwd(L.layer, L.X, L.Y, T, L.act, stream)
            mst.mst_sparse_fc_bwd_input(L.layer, L.dY, L.dX, T, L.act, stream)
            if not args.fused_update:
                mst.mst_sparse_fc_bwd_weight(L.layer, L.dY, L.X, L.dW, T, L.ws, L.act, stream)
                L.layer.sync_values(stream)
        fork = torch.cuda.Event()
        fork.record(stream)
        for L, d, s in zip(layers, dl, side):
            seed += 1
            if s is not stream:
                s.wait_event(fork)
            if args.fused_update:
                # every step updates the topology: the dense gradient the update needs also
                # gives the weight gradient (no separate SDDMM / dense product, and the update
                # rebuilds the views, so no separate hand-over of the values)
                mst.mst_sparse_fc_bwd_weight_update(L.layer, L.dY, L.X, L.dW, T, d, cfg["zeta"], cfg["R"], seed, L.ws,
                                                    L.act, s)
            else:
                mst.mst_mask_update(L.layer, L.dY, L.X, T, d, cfg["zeta"], cfg["R"], seed, L.ws, L.act, s)
            if s is not stream:
                done = torch.cuda.Event()
                done.record(s)
                stream.wait_event(done)

    for d in cfg["densities"]:
        if args.allocation == "erdos_renyi":
            dl = mst.mst_erdos_renyi_density([(L.O, L.I) for L in layers], d)
        else:
            dl = [d] * len(layers)
        for L, dk in zip(layers, dl):          # transition to this density (untimed)
            seed += 1
            mst.mst_mask_update(L.layer, L.dY, L.X, T, dk, cfg["zeta"], cfg["R"], seed, L.ws, L.act, stream)
        for _ in range(min(2, args.warmup)):
            one_step(dl)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            one_step(dl)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        flops = sum(6 * L.layer.nnz * T for L in layers)
        rows.append(dict(density=d, ms_per_step=round(1e3 * dt, 4), eff_tflops=round(flops / dt / 1e12, 3),
                         nnz={L.name: L.layer.nnz for L in layers},
                         path="dense-mfma" if d > 0.30 else "sparse"))
        tot_time += dt
        tot_flops += flops
    out = {"metric": METRIC, "value": round(tot_flops / tot_time / 1e12, 4), "unit": "TFLOP/s", "n_gpus": 1,
           "steps": steps * len(cfg["densities"]), "warmup": args.warmup,
           "ms_per_step": round(1e3 * tot_time / len(cfg["densities"]), 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "C5: one GPT-2-large block (1280/5120; 1 of 36 identical blocks), T=%d, densities %s "
                                  "(%s over the layers) reached by the mask update itself, products + fused "
                                  "Mixed-Growing update every step (updates of the four layers on %s; %s)"
                                  % (T, cfg["densities"], args.allocation,
                                     "one stream per layer" if args.update_streams else "the main stream",
                                     "weight gradient and update share one dense gradient" if args.fused_update
                                     else "weight gradient and update as separate calls")},
           "sweep": rows}
    print(json.dumps(out))


def cpu_baseline(layers, T):
    """The oracle as it stands (dense masked fp64 products with numpy) on the host cores."""
    import numpy as np
    from oracle import products as opr
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    Ts = min(T, 8192)            # bounded sample of the same batch: the first Ts tokens
    t0 = time.perf_counter()
    flops, reps = 0, 0
    while time.perf_counter() - t0 < 10.0 and reps < 50:      # about 10-30 s of CPU work
        for L in layers:
            X, dY = L.X_host[:Ts], L.dY_host[:Ts]
            opr.fc_fwd(X, L.W, L.M)
            opr.fc_bwd_input(dY, L.W, L.M)
            opr.fc_bwd_weight(dY, X, L.M)
            flops += 3 * 2 * L.nnz * Ts
        reps += 1
    dt = time.perf_counter() - t0
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": "first %d of %d tokens, all layers, fwd+bwd_input+bwd_weight, %d repetitions (%.1f s); "
                      "effective (nonzero-only) FLOPs over the oracle's dense masked fp64 numpy products"
                      % (Ts, T, reps, dt)}


if __name__ == "__main__":
    main()
