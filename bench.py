#!/usr/bin/env python3
"""Benchmark of the sparse fully-connected training step on one MI355X.

A step is one pass of the hot path over one batch: for every layer of the workload the
forward product, the input gradient and the weight gradient at the active positions, plus the
Mixed-Growing topology update (Algorithm 1: dense gradient on the matrix cores, prune / grow
selections, rebuild of the index views) on the steps that carry one.

Default run (what `python bench.py --gpus 1 --steps K --warmup W` prints as ONE JSON line):
  * headline = the schedule sweep of the GPT-2-large block (the largest single-GPU workload):
    the layers are driven through the densities 1.0, 0.5, 0.1, 0.02, 0.1, 0.5 of the warm-up /
    ultra-sparse / restoration phases (Sec. 3.1), every step runs the products at the current
    density and then one update per layer that moves it to the next density of the cycle;
  * `per_config`: the other four workloads (single layer, GPT-2-small block at density 0.10,
    the same block at 0.02 with power-law rows, GPT-2-medium block with bfloat16 activations),
    K steps each with a topology update every `--update-interval` steps, and the step between two
    updates replayed from a HIP graph (`graph_replay`: no host launch time, checked bit for bit
    against the same step issued call by call).
`--config Cx` runs one workload alone.  Inputs are synthetic, seeded, and resident in HBM
before the timed region.  Every library call of the timed region is bracketed by events on
the launch stream.
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

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
ALU_FP32_PEAK_TFLOPS = 157.3    # published fp32 vector peak: 256 CUs x 4 SIMD x 16 lanes x 2 flop x 2 (packed) x 2.4 GHz
ALU_FP32_UNPACKED_TFLOPS = 78.6  # the same without packed-fp32 instructions, which this build switches off
MFMA_FP32_PEAK_TFLOPS = 157.3
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA peak
CLOCK_HZ, N_CU = 2.4e9, 256
METRIC = "effective sparse TFLOP/s + HBM GB/s (% peak) per FC train step, 1 MI355X"


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=24)
    p.add_argument("--warmup", type=int, default=6)
    p.add_argument("--config", default="all", choices=["all", "C1", "C2", "C3", "C4", "C5"],
                   help="all = headline on the schedule sweep (C5) plus a per_config table of C1..C4")
    p.add_argument("--update-interval", type=int, default=10,
                   help="block workloads C1..C4: steps between topology updates (the paper's Delta_t is 100; the "
                        "default puts updates inside a short timed region); 0 = never update")
    p.add_argument("--allocation", default="uniform", choices=["uniform", "erdos_renyi"],
                   help="C5 only: every layer at the sweep's density, or the Erdos-Renyi shares of it (Sec. 3.2)")
    p.add_argument("--update-streams", type=int, default=3, choices=[0, 1, 2, 3],
                   help="C5 only: 0 = everything on the main stream; 3 (default) = after the four dense gradients the "
                        "layers' gathers and SGD steps run on one stream per layer and the four updates in ONE "
                        "mst_mask_update_from_scores_multi call on those streams (chains of small dependent kernels "
                        "side by side; their per-call times overlap); 1, 2 = the same streams with per-layer calls")
    p.add_argument("--fused-update", type=int, default=0,
                   help="C5 only: 1 = weight gradient and update in ONE call (mst_sparse_fc_bwd_weight_update); "
                        "0 = the same work as three calls (mst_dense_grad, mst_gather_active, "
                        "mst_mask_update_from_scores) so that the dense-gradient kernel is timed on its own")
    p.add_argument("--separate-bwd", action="store_true",
                   help="block workloads: time mst_sparse_fc_bwd_input and mst_sparse_fc_bwd_weight as two calls "
                        "instead of mst_sparse_fc_bwd (both gradients from one walk)")
    p.add_argument("--path", default="auto", choices=["auto", "sparse", "dense"],
                   help="pin every layer to the sparse kernels or to the masked dense MFMA contractions "
                        "(mst_layer_set_path); auto = the library chooses per call from density, batch and dtype")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-per-config", action="store_true")
    p.add_argument("--lr", type=float, default=1e-5,
                   help="step size of the caller-side SGD on the active weights between backward and hand-over "
                        "(without it grown weights would stay exactly 0 and magnitude pruning would degenerate "
                        "into a tie-break by index); 0 = no optimiser step")
    p.add_argument("--seed", type=int, default=2024)
    p.add_argument("--attention-mask", type=int, nargs=2, metavar=("L", "STRIDE"), default=None,
                   help="time the strided attention mask of Sec. 3.3 instead of a config (its own JSON line)")
    p.add_argument("--lds-probe", action="store_true",
                   help="time the LDS read probe (4-, 8- and 16-byte conflict-free reads on every CU) instead of a "
                        "config: the on-chip roofline of the sparse walk, as its own JSON line")
    p.add_argument("--pmc-probe", action="store_true",
                   help="short run for rocprofv3 --pmc: a 1 GiB device copy (calibration), then each call twice")
    return p.parse_args()


class LayerRun:
    """Device state of one layer of a workload."""

    def __init__(self, mst, synth, torch, seed, lid, name, I, O, T, density, mask, act, cap=None, dense_start=False):
        import numpy as np
        self.name, self.I, self.O, self.T = name, I, O, T
        if dense_start:
            W = synth.normal(seed, 1000 * lid + 2, (O, I), 0.02)
            M = np.ones((O, I), np.uint8)
        else:
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
        if cap is None:
            cap = min(O * I, self.nnz + self.nnz // 2 + 64)
        self.layer = mst.Layer(O, I, cap, "cuda:0")
        self.ws = torch.empty(mst.mst_workspace_bytes(O, I, cap, T), dtype=torch.uint8, device="cuda:0")
        self.layer.load_dense(to(W), to(M), self.ws)
        self.Y = torch.empty((T, O), dtype=torch.float32, device="cuda:0")
        self.dX = torch.empty((T, I), dtype=torch.float32, device="cuda:0")
        self.dW = torch.empty(cap, dtype=torch.float32, device="cuda:0")
        self.density = density

    def sgd(self, lr):
        """The caller's optimiser (not part of the library): plain SGD on the active-weight
        vector with the weight gradient of this step, a torch kernel on the current stream."""
        n = self.layer.nnz
        if n:
            self.layer.values().add_(self.dW[:n], alpha=-lr)

    # algorithmic (compulsory) bytes and flops of each product at nnz active weights
    def bytes_fwd(self, nnz=None):
        nnz = self.nnz if nnz is None else nnz
        return self.act_bytes * self.T * self.I + 4 * self.T * self.O + 8 * nnz + 4 * (self.O + 1)

    def bytes_bwd_input(self, nnz=None):
        nnz = self.nnz if nnz is None else nnz
        return self.act_bytes * self.T * self.O + 4 * self.T * self.I + 8 * nnz + 4 * (self.I + 1)

    def bytes_bwd_weight(self, nnz=None):
        nnz = self.nnz if nnz is None else nnz
        return self.act_bytes * self.T * (self.I + self.O) + 8 * nnz + 4 * nnz

    def bytes_bwd(self, nnz=None):
        # both gradients in one call: dY and X read once, dX and dW written, the entries read once
        nnz = self.nnz if nnz is None else nnz
        return (self.act_bytes * self.T * (self.I + self.O) + 4 * self.T * self.I + 8 * nnz + 4 * nnz +
                4 * (self.I + 1))

    def bytes_dense_grad(self):
        return self.act_bytes * self.T * (self.I + self.O) + 4 * self.O * self.I

    def flops_product(self, nnz=None):
        return 2 * (self.nnz if nnz is None else nnz) * self.T

    def flops_dense_grad(self):
        return 2 * self.T * self.O * self.I


def lds_peak_bytes_per_s(mst, torch, stream):
    """LDS read rate of the chip with 16-byte conflict-free reads, measured now (the on-chip
    roofline of the walk: one 4-byte LDS operand per multiply-add)."""
    blocks, iters, width = N_CU, 2000, 16
    out = torch.empty(blocks * 1024, dtype=torch.float32, device="cuda:0")
    mst.mst_probe_lds_read(out, width, 200, blocks, stream)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    mst.mst_probe_lds_read(out, width, iters, blocks, stream)
    b.record(stream)
    torch.cuda.synchronize()
    return blocks * 1024 * iters * 8 * width / (a.elapsed_time(b) * 1e-3)


def lds_probe(mst, torch, stream):
    """The LDS read rate by read width, each width timed over three launches."""
    blocks, iters = N_CU, 2000
    out = torch.empty(blocks * 1024, dtype=torch.float32, device="cuda:0")
    res = {}
    for width in (4, 8, 16):
        mst.mst_probe_lds_read(out, width, 200, blocks, stream)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(3):
            mst.mst_probe_lds_read(out, width, iters, blocks, stream)
        b.record(stream)
        torch.cuda.synchronize()
        rate = 3 * blocks * 1024 * iters * 8 * width / (a.elapsed_time(b) * 1e-3)
        res["%d-byte reads" % width] = dict(tb_per_s=round(rate / 1e12, 2),
                                            bytes_per_clk_per_cu=round(rate / N_CU / 2.4e9, 1))
    print(json.dumps({"lds_probe": True, "workgroups": blocks, "threads_per_workgroup": 1024,
                      "reads_per_thread": iters * 8, "clock_ghz_assumed": 2.4, "rates": res}))


def product_row_numbers(row, ms, by, fl, lds_bytes, lds_peak):
    row.update(eff_tflops=round(fl / ms / 1e9, 3), hbm_gbs=round(by / ms / 1e6, 1),
               hbm_frac=round(by / ms / 1e6 / HBM_PEAK_GBS, 4),
               alu_frac=round(fl / ms / 1e9 / ALU_FP32_PEAK_TFLOPS, 4), alg_bytes=by, alg_flops=fl)
    if lds_bytes and lds_peak:
        row.update(lds_frac=round(lds_bytes / (ms * 1e-3) / lds_peak, 4))


def split_gemm_applies(M, N, K):
    """Shapes of whole tiles take the kernel that forms an fp32 product from three bf16 MFMA
    products of the operands' bf16 halves (include/mst.h, mst_gemm_force_fp32_mfma)."""
    return M % 128 == 0 and N % 128 == 0 and K % 64 == 0


def dense_gemm_roofline(flops, ms, act, M, N, K, bf16_products=1.0):
    """A dense contraction: the matrix cores' peak for the dtype of the MFMA instructions that
    run.  fp32 operands on whole tiles run as 3 bf16 MFMA products per term: executed flops =
    3 x the product's 2 M N K, against the bf16 peak.  With bfloat16 activations the weight
    gradient is one product per term, Y and dX (fp32 weights split hi + lo) two."""
    tf = flops / ms / 1e9
    if act == "bf16":
        return dict(bound="mfma", achieved=round(bf16_products * tf, 2), peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=round(bf16_products * tf / MFMA_BF16_PEAK_TFLOPS, 4),
                    mfma_dtype="bf16 (%.3g MFMA products per term)" % bf16_products)
    if split_gemm_applies(M, N, K):
        return dict(bound="mfma", achieved=round(3 * tf, 2), peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=round(3 * tf / MFMA_BF16_PEAK_TFLOPS, 4), mfma_dtype="bf16 (fp32 operands split hi + lo, 3 products)",
                    fp32_equivalent_tflops=round(tf, 2), frac_of_fp32_mfma_peak=round(tf / MFMA_FP32_PEAK_TFLOPS, 4))
    return dict(bound="mfma", achieved=round(tf, 2), peak=MFMA_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                frac=round(tf / MFMA_FP32_PEAK_TFLOPS, 4), mfma_dtype="fp32")


def roofline_of(row, L, act, kernel, traffic_cfg):
    """The roofline object of one (layer, call) row."""
    if row["call"] == "dense_grad":
        roof = dense_gemm_roofline(row["alg_flops"], row["avg_ms"], act, L.O, L.I, L.T)
    else:
        t_hbm = row["alg_bytes"] / (HBM_PEAK_GBS * 1e9)
        t_alu = row["alg_flops"] / (ALU_FP32_PEAK_TFLOPS * 1e12)
        if row.get("path") == "dense-mfma":
            mnk = row.get("dense_mnk") or ((L.T, L.O, L.I) if row["call"] == "fwd" else (L.T, L.I, L.O))
            roof = dense_gemm_roofline(row["dense_flops"], row["avg_ms"], act, *mnk,
                                       bf16_products=row.get("bf16_products", 1.0))
        elif t_hbm >= t_alu:
            roof = dict(bound="hbm", achieved=row["hbm_gbs"], peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(row["hbm_gbs"] / HBM_PEAK_GBS, 4))
        else:
            roof = dict(bound="alu", achieved=row["eff_tflops"], peak=ALU_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=round(row["eff_tflops"] / ALU_FP32_PEAK_TFLOPS, 4),
                        frac_of_unpacked_peak=round(row["eff_tflops"] / ALU_FP32_UNPACKED_TFLOPS, 4))
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s.json" % traffic_cfg.lower())
    if os.path.exists(tpath):        # counter-based HBM bytes of this call, measured by the commands in profiles/
        traffic = json.load(open(tpath)).get("calls", {}).get("%s/%s" % (L.name, row["call"]))
    roof.update(traffic=traffic, kernel=kernel, call="%s/%s" % (L.name, row["call"]), avg_launch_ms=row["avg_ms"],
                alg_bytes_per_launch=row["alg_bytes"], alg_flops_per_launch=row["alg_flops"])
    if traffic and row["call"] == "dense_grad":
        # FETCH_SIZE counts what the eight L2s fetch from the fabric (Infinity Cache hits included): every XCD
        # reads all of X and its share of dY, and the partial outputs of the k ranges are written and read back
        roof["traffic_note"] = ("bytes per call from profiles/hbm_traffic_%s.json: L2 fills and write-backs of all 8 XCDs "
                                "(operands re-read per XCD, k-range partial outputs), not unique HBM bytes"
                                % traffic_cfg.lower())
    for k in ("hbm_frac", "alu_frac", "lds_frac"):
        if k in row:
            roof[k] = row[k]
    return roof


def sustained_clock_mhz(run_call, torch, seconds=1.2):
    """The shader clock while `run_call` (the roofline's call) runs back to back: the driver's
    pp_dpm_sclk file of this GPU (what rocm-smi --showclocks prints) read from a second thread,
    median of the samples taken after the first 0.4 s.  Under a chip-wide matrix-core load the part
    runs below the 2.4 GHz that the published peaks assume.  None where the file cannot be found."""
    import glob
    import re
    import threading
    files = glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")
    if len(files) > 1:                                # several cards in sysfs: the one torch's device 0 sits on
        pr = torch.cuda.get_device_properties(0)
        want = "%04x:%02x:%02x" % (getattr(pr, "pci_domain_id", 0), getattr(pr, "pci_bus_id", -1) & 0xFF,
                                    getattr(pr, "pci_device_id", 0))
        files = [f for f in files if want in os.path.realpath(os.path.dirname(f)).lower()]
    if len(files) != 1:
        return None
    samples, stop = [], threading.Event()

    def sampler():
        time.sleep(0.4)
        while not stop.is_set():
            try:
                m = re.search(r"(\d+)Mhz \*", open(files[0]).read())
            except OSError:
                return
            if m:
                samples.append(int(m.group(1)))
            stop.wait(0.05)

    th = threading.Thread(target=sampler)
    th.start()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(50):
            run_call()
        torch.cuda.synchronize()
    stop.set()
    th.join()
    return sorted(samples)[len(samples) // 2] if samples else None


def free_layers(torch, layers):
    for L in layers:
        L.layer.close()
    layers.clear()
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ block workloads C1..C4

def run_block(args, name, mst, synth, torch, lds_peak, with_cpu_baseline):
    cfg = synth.CONFIGS[name]
    T, act, density = cfg["T"], cfg["act"], cfg["densities"][0]
    layers = [LayerRun(mst, synth, torch, args.seed, lid + 1, lname, I, O, T, density, cfg["mask"], act)
              for lid, (lname, I, O) in enumerate(cfg["layers"])]
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    fstats = {L.name: L.layer.format_stats(stream) for L in layers}
    for L in layers:
        L.layer.set_path({"auto": mst.MST_PATH_AUTO, "sparse": mst.MST_PATH_SPARSE, "dense": mst.MST_PATH_DENSE}[args.path])
    # which contraction serves each call (asked of the library, not re-derived here)
    dense_prod = {L.name: L.layer.uses_dense(L.act, T) for L in layers}
    dense_wgrad = {L.name: L.layer.uses_dense(L.act, T, True) for L in layers}
    dense_bwd = {L.name: L.layer.uses_dense(L.act, T, 2) for L in layers}      # the one-call backward's own rule

    def path_of(L, kind):
        a, b = dense_prod[L.name], dense_wgrad[L.name]
        if kind in ("fwd", "bwd_input"):
            return "dense-mfma" if a else "sparse"
        if kind == "bwd_weight":
            return "dense-mfma" if b else "sparse"
        return "dense-mfma" if dense_bwd[L.name] else "sparse"

    if args.pmc_probe:
        pmc_probe_block(args, mst, torch, layers, T, stream)
        free_layers(torch, layers)
        return None

    products = ("fwd", "bwd_input", "bwd_weight") if args.separate_bwd else ("fwd", "bwd")
    kinds = products + ("caller_sgd", "sync_values", "mask_update")
    ev = {(L.name, k): [] for L in layers for k in kinds}

    def run_step(t, record):
        # one event between consecutive calls: the end of a call is the start of the next
        def mark():
            e = torch.cuda.Event(enable_timing=True)
            e.record(stream)
            return e

        last = mark() if record else None
        for L in layers:
            # the products, then the hand-over of the (optimiser-updated) active weights to the
            # index views, which a training step pays once per layer
            for kind in products + ("caller_sgd", "sync_values"):
                if kind == "caller_sgd":
                    if not args.lr:
                        continue
                    L.sgd(args.lr)
                elif kind == "fwd":
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
        if args.update_interval and mst.mst_update_due(t + 1, args.update_interval):
            for li, L in enumerate(layers):
                mst.mst_mask_update(L.layer, L.dY, L.X, T, density, cfg["zeta"], cfg["R"],
                                    mst.mst_update_seed(args.seed, t, len(layers), li), L.ws, L.act, stream)
                if record:
                    nxt = mark()
                    ev[(L.name, "mask_update")].append((last, nxt))
                    last = nxt

    clock_ramp(mst, torch, stream)
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
    update_ms = []
    for L in layers:
        fs = fstats[L.name]
        for kind in kinds:
            pairs = ev[(L.name, kind)]
            if not pairs:
                continue
            ms = sum(a.elapsed_time(b) for a, b in pairs) / len(pairs)
            row = dict(layer=L.name, call=kind, launches=len(pairs), avg_ms=round(ms, 5))
            if kind in products:
                row["path"] = path_of(L, kind)
                by = getattr(L, "bytes_" + kind)()
                fl = L.flops_product() * (2 if kind == "bwd" else 1)
                # LDS operand bytes of the walk: 4 bytes per token and stored entry slot of the view walked
                slots = fs["row_view_slots"] if kind == "fwd" else fs["col_view_slots"] if kind in ("bwd", "bwd_input") else 0
                product_row_numbers(row, ms, by, fl, 4 * slots * T if row["path"] == "sparse" else 0, lds_peak)
                tot = ms * len(pairs)
                if dominant is None or tot > dominant[0]:
                    dominant = (tot, row, L)
            elif kind == "mask_update":
                row.update(dense_grad_gflop=round(2 * T * L.O * L.I / 1e9, 2))
                update_ms.append(ms)
            table.append(row)

    _, drow, dL = dominant
    # fwd / bwd_input are one SpMM launch or one masked dense product; bwd is the shared walk followed by its
    # small second kernel, or the two dense contractions
    dp, dw = dense_prod[dL.name], dense_wgrad[dL.name]
    spmm_k = "k_spmm / k_spmm64 (launch shape chosen per call) + k_heavy_fwd after the forward (heavy rows as a dense product; returns at once without any)"
    gemm_k = "k_gemm_split256 / k_gemm_split_n160 / k_gemm_split (fp32 operands as bf16 hi + lo)" if act == "f32" else \
        "k_gemm_a16_256 (bfloat16 activations x fp32 weights as bf16 hi + lo, 2 products per term)"
    wgrad_dense_k = ("k_gemm_tn_bf16" if act == "bf16" else "k_gemm_split256<TN> / k_gemm_split<TN>") + " + k_gather_flat"
    kernel = {"fwd": gemm_k if dp else spmm_k,
              "bwd_input": gemm_k if dp else spmm_k,
              "bwd_weight": wgrad_dense_k if dw else "k_sddmm + k_sddmm_reduce",
              "bwd": "k_bwd_fused + k_bwd_fused_reduce" if not dense_bwd[dL.name] else
                     "%s, then %s" % (gemm_k, wgrad_dense_k)}[drow["call"]]
    if drow["path"] == "dense-mfma":
        # every leg of the call is a dense contraction: priced against the matrix cores
        legs = 2 if drow["call"] == "bwd" else 1
        drow["dense_flops"] = legs * 2.0 * T * dL.O * dL.I
        drow["dense_mnk"] = {"fwd": (T, dL.O, dL.I), "bwd_input": (T, dL.I, dL.O)}.get(drow["call"], (dL.O, dL.I, T))
        # bfloat16 activations: Y, dX = 2 MFMA products per term, weight gradient 1, the one-call backward both
        drow["bf16_products"] = {"fwd": 2.0, "bwd_input": 2.0, "bwd_weight": 1.0, "bwd": 1.5}[drow["call"]]
    roof = roofline_of(drow, dL, act, kernel, name)

    out = {
        "metric": METRIC, "value": round(value, 4), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "clock_ramp_ms": 40, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if act == "f32" else "bf16-in/f32-acc",
        "data": "synthetic",
        "config": {"workload": "%s: %s FC set (%s), density %.2f %s mask, T=%d tokens, %s "
                               "+ value hand-over to the index views per layer, Mixed-Growing update every %d steps"
                               % (name, "GPT-2 block" if len(layers) > 1 else "single layer",
                                  ", ".join("%s %d->%d" % (L.name, L.I, L.O) for L in layers), density,
                                  cfg["mask"], T,
                                  "fwd+bwd_input+bwd_weight" if args.separate_bwd
                                  else "fwd + bwd (input and weight gradient in one call)", args.update_interval),
                   "path": args.path,
                   "nnz": {L.name: L.nnz for L in layers}, "mask_updates_in_timed_region": n_updates,
                   "caller_sgd_lr": args.lr,
                   "ell_efficiency": {L.name: dict(row_view=round(fstats[L.name]["row_view_efficiency"], 4),
                                                   col_view=round(fstats[L.name]["col_view_efficiency"], 4),
                                                   heavy_rows=fstats[L.name]["heavy_rows"],
                                                   heavy_entries=fstats[L.name]["heavy_entries"])
                                      for L in layers}},
        "hbm_gbs_step": round(bytes_step / (elapsed / args.steps) / 1e9, 1),
        "hbm_frac_step": round(bytes_step / (elapsed / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
        "alu_frac_step": round(value / ALU_FP32_PEAK_TFLOPS, 4),
        "ms_per_mask_update": round(sum(update_ms) / len(update_ms), 4) if update_ms else None,
        "lds_peak_measured_tbs": round(lds_peak / 1e12, 1) if lds_peak else None,
        "roofline": roof,
        "calls": table,
    }

    # MFMA utilisation of the dense gradient G = dY^T X that scores gradient growth (it runs once per
    # update inside mst_mask_update; here on its own, after the timed region)
    G = torch.empty(max(L.O * L.I for L in layers), dtype=torch.float32, device="cuda:0")
    dg = {}
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
        r = dense_gemm_roofline(2.0 * T * L.O * L.I, ms, act, L.O, L.I, T)
        dg[L.name] = dict(avg_ms=round(ms, 4), tflops=round(2.0 * T * L.O * L.I / ms / 1e9, 1), mfma_tflops=r["achieved"],
                          mfma_peak=r["peak"], mfma_frac=r["frac"], mfma_dtype=r["mfma_dtype"])
    out["dense_grad_gemm"] = dict(operands="bf16" if act == "bf16" else "f32", layers=dg)

    out["graph_replay"] = graph_replay_block(args, mst, torch, layers, T, products)
    if with_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_block(layers, T)
    free_layers(torch, layers)
    return out


def graph_replay_block(args, mst, torch, layers, T, products):
    """Everything a step does between two topology updates (the products, the caller's SGD, the value
    hand-over, for every layer) recorded ONCE into a HIP graph and replayed: the step without the
    host's per-launch time, which is what a training loop pays while the topology stands still (the
    update itself sizes its launches on the host and stays outside; after it the graph is recorded
    again).  The first replay is compared bit for bit with the same step issued call by call."""
    main = torch.cuda.current_stream()

    def step(s):
        for L in layers:
            for kind in products:
                if kind == "fwd":
                    mst.mst_sparse_fc_fwd(L.layer, L.X, L.Y, T, L.act, s)
                elif kind == "bwd":
                    mst.mst_sparse_fc_bwd(L.layer, L.dY, L.X, L.dX, L.dW, T, L.ws, L.act, s)
                elif kind == "bwd_input":
                    mst.mst_sparse_fc_bwd_input(L.layer, L.dY, L.dX, T, L.act, s)
                else:
                    mst.mst_sparse_fc_bwd_weight(L.layer, L.dY, L.X, L.dW, T, L.ws, L.act, s)
            if args.lr:
                L.sgd(args.lr)
            L.layer.sync_values(s)

    def outputs():
        return [t.clone() for L in layers for t in (L.Y, L.dX, L.dW[:L.layer.nnz], L.layer.values())]

    start = [L.layer.values().clone() for L in layers]

    def rewind():
        for L, v in zip(layers, start):
            L.layer.values().copy_(v)
            L.layer.sync_values(main)

    step(main)
    torch.cuda.synchronize()
    eager = outputs()
    rewind()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(main)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for L in layers:                              # (recording runs nothing: whatever a replay leaves is its own)
        for t in (L.Y, L.dX, L.dW):
            t.fill_(float("nan"))
    graph.replay()
    torch.cuda.synchronize()
    same = all(torch.equal(a, b) for a, b in zip(eager, outputs()))
    n = max(50, args.steps)
    for _ in range(5):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        graph.replay()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / n
    rewind()
    torch.cuda.synchronize()
    return dict(ms_per_step=round(ms, 4), replays=n, matches_call_by_call=bool(same),
                holds="%s%s + value hand-over of every layer; no topology update" % (" + ".join(products), " + caller's SGD" if args.lr else ""))


def pmc_probe_block(args, mst, torch, layers, T, stream):
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


# ------------------------------------------------------------------ schedule sweep C5

def run_sweep(args, mst, synth, torch, lds_peak, with_cpu_baseline):
    """One GPT-2-large block (of 36 identical ones) driven round the density cycle by the update
    itself: step t computes the products at cycle position t mod 6 and then updates every layer
    to the density of position t + 1 (a topology update every step)."""
    import numpy as np
    cfg = synth.CONFIGS["C5"]
    T, cyc = cfg["T"], cfg["densities"]
    ncyc = len(cyc)
    stream = torch.cuda.current_stream()
    layers = [LayerRun(mst, synth, torch, args.seed, lid + 1, lname, I, O, T, 1.0, "uniform", "f32", cap=O * I,
                       dense_start=True)
              for lid, (lname, I, O) in enumerate(cfg["layers"])]
    for L in layers:
        L.layer.set_path({"auto": mst.MST_PATH_AUTO, "sparse": mst.MST_PATH_SPARSE, "dense": mst.MST_PATH_DENSE}[args.path])
    G = [torch.empty(L.O * L.I, dtype=torch.float32, device="cuda:0") for L in layers]
    shapes = [(L.O, L.I) for L in layers]
    torch.cuda.synchronize()

    def targets(pos):
        d = cyc[pos % ncyc]
        return mst.mst_erdos_renyi_density(shapes, d) if args.allocation == "erdos_renyi" else [d] * len(layers)

    if args.pmc_probe:
        pmc_probe_sweep(args, mst, torch, layers, G, T, cyc, targets, cfg, stream)
        free_layers(torch, layers)
        return None

    # (the box gives a process four hardware queues: three side streams and the main one for the last layer)
    side = ([torch.cuda.Stream() for _ in layers[:-1]] + [stream]) if args.update_streams == 3 else \
        [torch.cuda.Stream() for _ in layers] if args.update_streams else [stream] * len(layers)
    upd_start = {}
    step_ev = {}       # position -> (first, last) events of its steps on the main stream
    phase_ev = []      # (fork, join) of the layers' update chains when they run side by side
    ev = []            # (position, layer index, call, start event, end event)
    nnz_at = {}        # position -> per-layer active counts (host arithmetic of the update, no read-back)
    dense_at = {}      # position -> per layer: does the library route Y and dX to the masked dense contraction

    def run_step(t, record):
        pos = t % ncyc
        nnz_at[pos] = [L.layer.nnz for L in layers]
        dense_at[pos] = [L.layer.uses_dense(L.act, T) for L in layers]

        def mark(s):
            e = torch.cuda.Event(enable_timing=True)
            e.record(s)
            return e

        last = mark(stream) if record else None
        step_begin = last
        for li, L in enumerate(layers):
            for call in ("fwd", "bwd_input"):
                if call == "fwd":
                    mst.mst_sparse_fc_fwd(L.layer, L.X, L.Y, T, L.act, stream)
                else:
                    mst.mst_sparse_fc_bwd_input(L.layer, L.dY, L.dX, T, L.act, stream)
                if record:
                    nxt = mark(stream)
                    ev.append((pos, li, call, last, nxt))
                    last = nxt
        fork = None
        grads_first = args.update_streams >= 2 and not args.fused_update
        multi = args.update_streams == 3 and not args.fused_update
        if grads_first:
            # the four dense gradients (each fills the chip) one after the other on the main stream; only
            # then the layers' chains of small kernels (gather, SGD, update), side by side on their streams
            for li, L in enumerate(layers):
                mst.mst_dense_grad(L.dY, L.X, G[li], T, L.O, L.I, L.act, L.ws, stream)
                if record:
                    nxt = mark(stream)
                    ev.append((pos, li, "dense_grad", last, nxt))
                    last = nxt
        if args.update_streams:
            fork = torch.cuda.Event(enable_timing=True)
            fork.record(stream)
        dl = targets(pos + 1)
        for li, (L, d, s) in enumerate(zip(layers, dl, side)):
            seed = mst.mst_update_seed(args.seed, t, len(layers), li)
            if s is not stream:
                s.wait_event(fork)
            if args.update_streams:
                last = mark(s) if record else None       # every layer's chain is timed on its own stream
            if args.fused_update:
                # weight gradient (at the positions active now) and update from one dense gradient
                mst.mst_sparse_fc_bwd_weight_update(L.layer, L.dY, L.X, L.dW, T, d, cfg["zeta"], cfg["R"], seed, L.ws,
                                                    L.act, s)
                calls = ("bwd_weight_update",)
            else:
                calls = ("dense_grad", "gather_active", "caller_sgd", "mask_update") if args.lr else \
                        ("dense_grad", "gather_active", "mask_update")
            for call in calls:
                if call == "dense_grad" and grads_first:
                    continue
                if call == "dense_grad":
                    mst.mst_dense_grad(L.dY, L.X, G[li], T, L.O, L.I, L.act, L.ws, s)
                elif call == "gather_active":
                    mst.mst_gather_active(L.layer, G[li], L.dW, s)
                elif call == "caller_sgd":
                    with torch.cuda.stream(s):
                        L.sgd(args.lr)
                elif call == "mask_update":
                    if multi:
                        if record:
                            upd_start[li] = last
                        continue
                    mst.mst_mask_update_from_scores(L.layer, G[li], d, cfg["zeta"], cfg["R"], seed, L.ws, s)
                if record:
                    nxt = mark(s)
                    ev.append((pos, li, call, last, nxt))
                    last = nxt
            if s is not stream and not multi:
                done = torch.cuda.Event()
                done.record(s)
                stream.wait_event(done)
        if multi:
            # the four updates in ONE native call, each on its layer's stream
            mst.mst_mask_update_from_scores_multi([L.layer for L in layers], G, dl, cfg["zeta"], cfg["R"],
                                                  [mst.mst_update_seed(args.seed, t, len(layers), li) for li in range(len(layers))],
                                                  [L.ws for L in layers], side)
            for li, s in enumerate(side):
                if record:
                    ev.append((pos, li, "mask_update", upd_start[li], mark(s)))
                if s is not stream:
                    done = torch.cuda.Event()
                    done.record(s)
                    stream.wait_event(done)
        if record:
            step_end = mark(stream)                                          # (after the side streams have joined)
            step_ev.setdefault(pos, []).append((step_begin, step_end))
            if grads_first:
                phase_ev.append((fork, step_end))

    clock_ramp(mst, torch, stream)
    t = 0
    for _ in range(args.warmup):
        run_step(t, False)
        t += 1
    torch.cuda.synchronize()
    t_first = t
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step(t, True)
        t += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # after the timed region: one more pass of the cycle to read the views' stored entry counts at every
    # position (a read-back that must not sit between timed calls); the LDS operand bytes of a sparse walk
    t_end = t
    slots_at = {}
    for _ in range(ncyc):
        fs = [L.layer.format_stats(stream) for L in layers]
        slots_at[t % ncyc] = [dict(fwd=f["row_view_slots"], bwd_input=f["col_view_slots"]) for f in fs]
        run_step(t, False)
        t += 1
    torch.cuda.synchronize()
    t = t_end

    # ---- per (position, layer, call) device times
    acc = {}
    for pos, li, call, a, b in ev:
        acc.setdefault((pos, li, call), []).append(a.elapsed_time(b))
    steps_at = {p: sum(1 for tt in range(t_first, t) if tt % ncyc == p) for p in range(ncyc)}
    tot_flops = sum(6 * n * T for tt in range(t_first, t) for n in nnz_at[tt % ncyc])
    value = tot_flops / elapsed / 1e12
    tot_bytes = 0.0
    sweep_rows, calls, dominant = [], [], None
    by_layer_call = {}
    for p in range(ncyc):
        if not steps_at[p]:
            continue
        d = cyc[p]
        ms_pos = 0.0
        for li, L in enumerate(layers):
            nnz = nnz_at[p][li]
            dense_path = dense_at[p][li]
            for call in ("fwd", "bwd_input"):
                xs = acc.get((p, li, call), [])
                if not xs:
                    continue
                ms = sum(xs) / len(xs)
                ms_pos += ms
                row = dict(density=d, position=p, layer=L.name, call=call, launches=len(xs), avg_ms=round(ms, 5),
                           min_ms=round(min(xs), 5), max_ms=round(max(xs), 5),
                           path="dense-mfma" if dense_path else "sparse")
                by = L.bytes_fwd(nnz) if call == "fwd" else L.bytes_bwd_input(nnz)
                lds_bytes = 0 if dense_path else 4 * slots_at[p][li][call] * T
                product_row_numbers(row, ms, by, L.flops_product(nnz), lds_bytes, lds_peak)
                if dense_path:
                    mnk = (T, L.O, L.I) if call == "fwd" else (T, L.I, L.O)
                    r = dense_gemm_roofline(L.flops_dense_grad(), ms, "f32", *mnk)
                    row.update(dense_flops=L.flops_dense_grad(), mfma_tflops=r["achieved"], mfma_frac=r["frac"],
                               mfma_dtype=r["mfma_dtype"])
                calls.append(row)
                if dominant is None or ms * len(xs) > dominant[0]:
                    dominant = (ms * len(xs), row, L)
            for call in ("dense_grad", "gather_active", "caller_sgd", "mask_update", "bwd_weight_update"):
                xs = acc.get((p, li, call), [])
                if xs:
                    ms_pos += sum(xs) / len(xs)
                    by_layer_call.setdefault((li, call), []).extend(xs)
        # the step's own span on the main stream (with side streams the calls' times overlap and their sum overstates)
        ms_pos = sum(a.elapsed_time(b) for a, b in step_ev[p]) / len(step_ev[p])
        step_bytes = sum(L.bytes_fwd(n) + L.bytes_bwd_input(n) + L.bytes_bwd_weight(n)
                         for L, n in zip(layers, nnz_at[p]))
        step_flops = sum(6 * n * T for n in nnz_at[p])
        tot_bytes += step_bytes * steps_at[p]
        sweep_rows.append(dict(position=p, density=d, next_density=cyc[(p + 1) % ncyc], steps=steps_at[p],
                               ms_per_step_device=round(ms_pos, 4), eff_tflops=round(step_flops / ms_pos / 1e9, 3),
                               hbm_frac=round(step_bytes / ms_pos / 1e6 / HBM_PEAK_GBS, 4),
                               alu_frac=round(step_flops / ms_pos / 1e9 / ALU_FP32_PEAK_TFLOPS, 4),
                               nnz={L.name: n for L, n in zip(layers, nnz_at[p])},
                               path="dense-mfma" if all(dense_at[p]) else "sparse" if not any(dense_at[p]) else "mixed"))
    # the update's calls do the same work at every position (the dense gradient) or nearly so: one row per layer
    for (li, call), xs in sorted(by_layer_call.items()):
        L = layers[li]
        ms = sum(xs) / len(xs)
        row = dict(layer=L.name, call=call, launches=len(xs), avg_ms=round(ms, 5), min_ms=round(min(xs), 5),
                   max_ms=round(max(xs), 5))
        if call == "dense_grad":
            r = dense_gemm_roofline(L.flops_dense_grad(), ms, "f32", L.O, L.I, T)
            row.update(alg_flops=L.flops_dense_grad(), alg_bytes=L.bytes_dense_grad(),
                       tflops=round(L.flops_dense_grad() / ms / 1e9, 2), mfma_tflops=r["achieved"],
                       mfma_frac=r["frac"], mfma_dtype=r["mfma_dtype"])
            if dominant is None or ms * len(xs) > dominant[0]:
                dominant = (ms * len(xs), row, L)
        calls.append(row)

    _, drow, dL = dominant
    if drow["call"] == "dense_grad":
        kernel = ("k_gemm_split256<TN> (256 x 256 tiles; fp32 operands split into bf16 hi + lo, 3 x "
                  "v_mfma_f32_32x32x16_bf16 per term) + k_splitk_reduce4 (ordered sum of its split partial outputs)")
    elif drow.get("path") == "dense-mfma":
        kernel = ("k_gemm_split256 (masked dense product, bf16 hi + lo split on v_mfma_f32_32x32x16_bf16; preceded by the "
                  "scatter of the dense weight copy after an update)")
    else:
        kernel = "k_spmm / k_spmm64 (launch shape chosen per call)"
    roof = roofline_of(drow, dL, "f32", kernel, "C5")
    if drow["call"] == "dense_grad" and roof["bound"] == "mfma":
        gi = layers.index(dL)
        mhz = sustained_clock_mhz(lambda: mst.mst_dense_grad(dL.dY, dL.X, G[gi], T, dL.O, dL.I, dL.act, dL.ws, stream), torch)
        if mhz:
            # `frac` stays against the published peak; this is the same rate against what the matrix cores can
            # issue at the clock the chip actually holds under this load
            pk = roof["peak"] * mhz / (CLOCK_HZ / 1e6)
            roof["sustained_clock"] = dict(sclk_mhz=mhz, peak_at_that_clock=round(pk, 1), frac=round(roof["achieved"] / pk, 4),
                                           how="the driver's pp_dpm_sclk (what rocm-smi --showclocks prints) sampled while this call runs "
                                               "back to back for 1.2 s after the timed region (median); published peaks "
                                               "assume %.1f GHz" % (CLOCK_HZ / 1e9))
    upd = [x for (li, call), xs in by_layer_call.items() if call in ("mask_update", "bwd_weight_update") for x in xs]
    out = {"metric": METRIC, "value": round(value, 4), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "clock_ramp_ms": 40, "ms_per_step": round(1e3 * elapsed / args.steps, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None,
           "dtype": "f32 (dense contractions: fp32 operands as bf16 hi + lo, fp32 accumulation)", "data": "synthetic",
           "config": {"workload": "C5: schedule sweep of one GPT-2-large block (qkv 1280->3840, proj 1280->1280, fc1 "
                                  "1280->5120, fc2 5120->1280; 1 of 36 identical blocks), T=%d tokens, fp32; step t runs "
                                  "fwd + bwd_input of the four layers at density cycle[t mod 6], cycle = %s (%s over the "
                                  "layers), then per layer the dense gradient, the weight gradient read from it, the caller's SGD "
                                  "step on the active weights and one Mixed-Growing update to cycle[(t+1) mod 6] (%s; %s)"
                                  % (T, cyc, args.allocation,
                                     "one call" if args.fused_update else "three calls so that the dense-gradient kernel "
                                     "is timed on its own",
                                     {0: "one stream",
                                      1: "every layer's dense gradient, gather, SGD and update on a stream of its own",
                                      2: "the dense gradients on the main stream, then the layers' chains (gather, SGD, "
                                         "update) on one stream per layer",
                                      3: "the dense gradients on the main stream, then gather and SGD per layer on its "
                                         "stream and the four updates in one mst_mask_update_from_scores_multi call, side "
                                         "by side on four streams (the mask_update rows are times on a layer's stream and "
                                         "overlap; update_phase_ms is the span of all of it)"}[args.update_streams]),
                      "mask_updates_in_timed_region": args.steps * len(layers),
                      "layers": {L.name: [L.I, L.O] for L in layers},
                      "caller_sgd_lr": args.lr},
           "hbm_gbs_step": round(tot_bytes / elapsed / 1e9, 1),
           "hbm_frac_step": round(tot_bytes / elapsed / 1e9 / HBM_PEAK_GBS, 4),
           "alu_frac_step": round(value / ALU_FP32_PEAK_TFLOPS, 4),
           "ms_per_mask_update": round(sum(upd) / len(upd), 4) if upd else None,
           "update_phase_ms": round(sum(a.elapsed_time(b) for a, b in phase_ev) / len(phase_ev), 4) if phase_ev else None,
           "lds_peak_measured_tbs": round(lds_peak / 1e12, 1) if lds_peak else None,
           "roofline": roof, "sweep": sweep_rows, "calls": calls}
    if with_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_sweep(synth, args.seed, cfg)
    free_layers(torch, layers)
    return out


def pmc_probe_sweep(args, mst, torch, layers, G, T, cyc, targets, cfg, stream):
    """Counter run of the sweep: the calibration copy, then one step at every cycle position with
    a one-element kernel after each call."""
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    mark = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    mark.add_(1)
    order = []
    for t in range(len(cyc)):
        for L in layers:
            mst.mst_sparse_fc_fwd(L.layer, L.X, L.Y, T, L.act, stream)
            mark.add_(1)
            mst.mst_sparse_fc_bwd_input(L.layer, L.dY, L.dX, T, L.act, stream)
            mark.add_(1)
            order += ["%s/fwd@%d" % (L.name, t), "%s/bwd_input@%d" % (L.name, t)]
        for li, (L, d) in enumerate(zip(layers, targets(t + 1))):
            mst.mst_dense_grad(L.dY, L.X, G[li], T, L.O, L.I, L.act, L.ws, stream)
            mark.add_(1)
            mst.mst_gather_active(L.layer, G[li], L.dW, stream)
            mark.add_(1)
            mst.mst_mask_update_from_scores(L.layer, G[li], d, cfg["zeta"], cfg["R"], 1000 + t * 4 + li, L.ws, stream)
            mark.add_(1)
            order += ["%s/dense_grad@%d" % (L.name, t), "%s/gather_active@%d" % (L.name, t),
                      "%s/mask_update@%d" % (L.name, t)]
    torch.cuda.synchronize()
    print(json.dumps({"pmc_probe": True, "copy_bytes_each_way": 1 << 30, "calls_in_order": order,
                      "layers": {L.name: dict(I=L.I, O=L.O) for L in layers}}))


def clock_ramp(mst, torch, stream, ms=40.0):
    """The GPU's clocks take tens of milliseconds to come up after an idle period (layer set-up on the
    host); a short workload timed right after one reads 5-40 % slow.  Before the W warm-up steps of a
    timed region this runs a dense contraction on scratch buffers for `ms` milliseconds.  It touches no
    layer state, so the W warm-up steps and the K timed steps are the same steps with or without it."""
    n = 4096
    a = torch.randn(n, n, device="cuda:0")
    b = torch.randn(n, n, device="cuda:0")
    c = torch.empty(n, n, device="cuda:0")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while 1e3 * (time.perf_counter() - t0) < ms:
        for _ in range(4):
            mst.mst_dense_grad(a, b, c, n, n, n, mst.MST_F32, None, stream)
        torch.cuda.synchronize()


# ------------------------------------------------------------------ other modes

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


def _oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline_block(layers, T):
    """The oracle as it stands (dense masked fp64 products with numpy) on the host cores."""
    from oracle import products as opr
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
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": _oracle_threads(), "kind": "oracle",
            "sample": "first %d of %d tokens, all layers, fwd+bwd_input+bwd_weight, %d repetitions (%.1f s); "
                      "effective (nonzero-only) FLOPs over the oracle's dense masked fp64 numpy products"
                      % (Ts, T, reps, dt)}


def cpu_baseline_sweep(synth, seed, cfg):
    """The oracle on a bounded sample of the sweep: the three products of the four layers at
    every density of the cycle on the whole batch, and the Mixed-Growing update of the
    smallest layer (1280 x 1280) at every transition."""
    import numpy as np
    from oracle import mixed_growing as omg
    from oracle import products as opr
    T, cyc = cfg["T"], cfg["densities"]
    Ts = T
    acts, Ws, Ms = [], [], []
    for lid, (_, I, O) in enumerate(cfg["layers"]):          # inputs first: drawing them is not the oracle's work
        acts.append(synth.make_activations(seed, lid + 1, Ts, I, O))
        Ws.append(synth.normal(seed, 100000 + lid, (O, I), 0.02))
        Ms.append(synth.nested_uniform_masks(seed, 200000 + lid, O, I, cyc))
    t0 = time.perf_counter()
    flops, n_upd = 0, 0
    Wp = Mp = Gp = None
    for p, d in enumerate(cyc + cyc):                       # two passes of the cycle: 10-15 s of host work
        p %= len(cyc)
        for lid, (lname, I, O) in enumerate(cfg["layers"]):
            W, M = Ws[lid], Ms[lid][p]
            X, dY = acts[lid]
            opr.fc_fwd(X, W, M)
            opr.fc_bwd_input(dY, W, M)
            opr.fc_bwd_weight(dY, X, M)
            flops += 3 * 2 * int(M.sum()) * Ts
            if lname == "proj":
                if Wp is None:
                    Wp, Mp = W * M, M
                    Gp = opr.dense_grad(dY, X).astype(np.float32)
        r = omg.update(Wp, Mp, Gp, cyc[(p + 1) % len(cyc)], cfg["zeta"], cfg["R"], seed + p)
        Wp, Mp = r["W"], r["M"]
        n_upd += 1
    dt = time.perf_counter() - t0
    # the same products on ONE thread, on a smaller token sample (one pass of the cycle)
    single = None
    try:
        from threadpoolctl import threadpool_limits
        T1 = 256
        with threadpool_limits(limits=1):
            t1 = time.perf_counter()
            f1 = 0
            for p in range(len(cyc)):
                for lid in range(len(cfg["layers"])):
                    W, M = Ws[lid], Ms[lid][p]
                    X, dY = acts[lid][0][:T1], acts[lid][1][:T1]
                    opr.fc_fwd(X, W, M)
                    opr.fc_bwd_input(dY, W, M)
                    opr.fc_bwd_weight(dY, X, M)
                    f1 += 3 * 2 * int(M.sum()) * T1
            d1 = time.perf_counter() - t1
        single = {"value": round(f1 / d1 / 1e12, 5), "unit": "TFLOP/s", "cores": 1,
                  "sample": "one pass of the cycle, products only, first %d tokens, %.1f s" % (T1, d1)}
    except ImportError:
        pass
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": _oracle_threads(), "kind": "oracle",
            "single_thread": single,
            "sample": "two passes of the density cycle %s: fwd+bwd_input+bwd_weight of the four layers on the first %d of "
                      "%d tokens (dense masked fp64 numpy products, masks drawn per density) plus %d Mixed-Growing "
                      "updates of the 1280x1280 layer, %.1f s in all; effective (nonzero-only) FLOPs of the products "
                      "over that time" % (cyc, Ts, T, n_upd, dt)}


def compact(out, name):
    """One row of the per_config table from a block workload's full result."""
    r = out["roofline"]
    return dict(config=name, workload=out["config"]["workload"], dtype=out["dtype"], steps=out["steps"],
                ms_per_step=out["ms_per_step"], eff_tflops=out["value"], hbm_gbs_step=out["hbm_gbs_step"],
                hbm_frac=out["hbm_frac_step"], alu_frac=out["alu_frac_step"],
                alu_frac_of_unpacked_peak=round(out["value"] / ALU_FP32_UNPACKED_TFLOPS, 4),
                mask_updates_in_timed_region=out["config"]["mask_updates_in_timed_region"],
                ms_per_mask_update=out["ms_per_mask_update"], graph_replay=out["graph_replay"], ell_efficiency=out["config"]["ell_efficiency"],
                slowest_call=dict(call=r["call"], avg_ms=r["avg_launch_ms"], bound=r["bound"], frac=r["frac"],
                                  hbm_frac=r.get("hbm_frac"), alu_frac=r.get("alu_frac"), lds_frac=r.get("lds_frac")),
                path=out["config"]["path"],
                calls=[{k: c[k] for k in ("layer", "call", "path", "avg_ms", "eff_tflops", "hbm_frac", "alu_frac", "lds_frac")
                        if k in c} for c in out["calls"]],
                dense_grad_gemm=out["dense_grad_gemm"])


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); no multi-GPU path exists", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2408_11746_amd as mst
    import synth

    if args.attention_mask:
        return attention_mask(args, mst, torch)
    stream = torch.cuda.current_stream()
    if args.lds_probe:
        return lds_probe(mst, torch, stream)
    lds_peak = None if args.pmc_probe else lds_peak_bytes_per_s(mst, torch, stream)
    cpu = not args.no_cpu_baseline
    if args.config == "C5" or args.config == "all":
        out = run_sweep(args, mst, synth, torch, lds_peak, cpu)
        if out is None:
            return
        if args.config == "all" and not args.no_per_config:
            rows = []
            for name in ("C1", "C2", "C3", "C4"):
                row = compact(run_block(args, name, mst, synth, torch, lds_peak, False), name)
                if args.path == "auto" and any(c.get("path", "sparse") != "sparse" for c in row["calls"]):
                    # the library sends some call of this workload to a dense contraction: the same workload with
                    # every layer pinned to the sparse kernels, so that those stay measured
                    pinned = argparse.Namespace(**dict(vars(args), path="sparse"))
                    sp = compact(run_block(pinned, name, mst, synth, torch, lds_peak, False), name)
                    row["sparse_pinned"] = {k: sp[k] for k in ("ms_per_step", "eff_tflops", "hbm_frac", "alu_frac",
                                                               "slowest_call", "calls")}
                rows.append(row)
            out["per_config"] = rows
        print(json.dumps(out))
        return
    out = run_block(args, args.config, mst, synth, torch, lds_peak, cpu)
    if out is not None:
        print(json.dumps(out))


if __name__ == "__main__":
    main()
