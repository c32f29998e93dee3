#!/usr/bin/env python3
"""Benchmark of the expert-pruning hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic batch of the Mixtral-shaped
layer (E=8, top-2, H=4096, F=14336):
    moe_expert_outputs on T=262144 calibration tokens            (router + expert GEMMs)
    prune_enumerate_multi for r=6 (28 subsets) and r=4 (70)      (one Gram pass + scoring + argmin per r)
    moe_forward_skip on the first 32768 tokens, beta = median    (dynamic skipping forward)
Inputs are generated on the device before the timed region.  `value` is
(28 + 70) * T subset-token pairs per second of whole-step time.

Prints ONE JSON line.  `roofline` is for the dominant kernel (the gate/up GEMM), timed per
launch with HIP events on the launch stream inside the timed steps; `kernels` carries the same
figures for every kernel; `cpu_baseline` times the fp64 numpy oracle on a bounded sample.
"""
from __future__ import annotations

import argparse
import glob
import json
import math
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0     # MI355X dense bf16
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E

# Fabric-side traffic per launch of the dominant kernel (dense gate/up GEMM) measured with
# rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE runs of this script with --copy-calibration, each
# scaled by what the 1 GiB copy reads on the same counter: x2.000 and x1.000); the figures are in
# profiles/hot_path_C3_hbm_traffic.txt.  None = not measured for that workload.
MEASURED_TRAFFIC_BYTES = {"C3": 97.7e9, "C2": None, "C4": 82.7e9}   # re-measured on commit 83adbb7, unchanged (C4: one launch over 16 experts)
PEAK_ALU_LANE_OPS = 256 * 64 * 2.4e9   # CUs x lanes x clock: plain (non-packed) fp32/int lane operations per second
PEAK_LDS_LOOKUPS = 256 * 32 * 2.4e9    # CUs x LDS banks x clock: 4-byte LDS look-ups per second without bank conflicts


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="C3", choices=["C2", "C3", "C4"],
                    help="C3 = Mixtral-shaped layer (the headline); C2 = mid layer (quick check); "
                         "C4 = enumeration stress (16 experts, top-4, 12870 + 1820 subsets; no skip leg)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-rank-limited", action="store_true",
                    help="skip the extra, separately timed leg that redoes expert outputs + enumeration with "
                         "the rank-limited expert pass")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy before the timed region, so that a "
                         "rocprofv3 --pmc run of this command holds a kernel of known traffic to scale "
                         "FETCH_SIZE / WRITE_SIZE by")
    return ap.parse_args()


class PowerSampler(threading.Thread):
    """Reads the board's own telemetry (sysfs, read-only: socket power, power cap, current shader clock) every half
    second while the timed steps run; reports nothing where the files are not there."""

    def __init__(self):
        super().__init__(daemon=True)
        self.stop_flag = threading.Event()
        self.power_w, self.sclk_mhz, self.cap_w, self.dev = [], [], None, None
        for d in sorted(glob.glob("/sys/class/drm/card*/device")):
            if glob.glob(os.path.join(d, "hwmon", "hwmon*", "power1_input")):
                self.dev = d
                break

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return f.read()
        except OSError:
            return None

    def run(self):
        if self.dev is None:
            return
        hw = glob.glob(os.path.join(self.dev, "hwmon", "hwmon*"))[0]
        cap = self._read(os.path.join(hw, "power1_cap"))
        self.cap_w = float(cap) / 1e6 if cap else None
        while not self.stop_flag.wait(0.5):
            p = self._read(os.path.join(hw, "power1_input"))
            if p:
                self.power_w.append(float(p) / 1e6)
            for line in (self._read(os.path.join(self.dev, "pp_dpm_sclk")) or "").splitlines():
                if line.rstrip().endswith("*"):
                    self.sclk_mhz.append(float(line.split(":")[1].strip().rstrip("*").strip().lower().rstrip("mhz")))

    def summary(self):
        if not self.power_w:
            return None
        return {"socket_power_w_mean": sum(self.power_w) / len(self.power_w), "socket_power_w_max": max(self.power_w),
                "power_cap_w": self.cap_w,
                "shader_clock_mhz_mean": sum(self.sclk_mhz) / len(self.sclk_mhz) if self.sclk_mhz else None,
                "shader_clock_mhz_max_of_part": 2400, "samples": len(self.power_w),
                "source": "sysfs hwmon power1_input / power1_cap and pp_dpm_sclk, every 0.5 s during the timed steps"}


def cpu_baseline(cfg, layer, Y, logits, torch, wl):
    """The oracle as it stands, on a bounded sample of the same workload (host cores)."""
    import numpy as np

    import oracle

    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    n1 = 512 if cfg.H >= 4096 else 1024         # tokens through all E experts (fp64 GEMMs)
    n_sub_all = sum(math.comb(cfg.E, r) for r in cfg.rs)
    # tokens through the enumeration, all r: bounded so that the oracle needs ten to fifteen seconds
    n2 = min(6144 if cfg.H >= 4096 else 8192, max(32, int(2e6 / n_sub_all)))
    x = wl.to_f64(layer["x"][:n1])
    Wg = wl.to_f64(layer["Wgate"])
    t_o1 = 0.0
    for e in range(cfg.E):                       # one expert at a time: fp64 weights are large
        W1, W3, W2 = (wl.to_f64(layer[n][e:e + 1]) for n in ("W1", "W3", "W2"))
        t0 = time.perf_counter()
        oracle.expert_outputs(x, Wg, W1, W3, W2)
        t_o1 += time.perf_counter() - t0
    l64, Y64 = wl.to_f64(logits[:n2]), wl.to_f64(Y[:, :n2])
    t0 = time.perf_counter()
    for r in cfg.rs:
        oracle.prune_enumerate(l64, Y64, cfg.k, r)
    t_o2 = time.perf_counter() - t0
    n_sub = sum(math.comb(cfg.E, r) for r in cfg.rs)
    per_token = t_o1 / n1 + t_o2 / n2
    return {
        "value": n_sub / per_token, "unit": "subset·tokens/s", "cores": int(cores), "kind": "oracle",
        "sample": f"expert_outputs on {n1} tokens x {cfg.E} experts ({t_o1:.2f} s) + prune_enumerate "
                  f"r={list(cfg.rs)} on {n2} tokens ({t_o2:.2f} s), scaled per token",
        "expert_outputs_tokens_per_s": n1 / t_o1, "enumerate_subset_tokens_per_s": n_sub * n2 / t_o2,
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus N with N > 1 is not supported "
              "(the path would shard over tokens with one small all-reduce of the loss vector).", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2402_14800_amd as pkg
    from paper_2402_14800_amd import binding
    from paper_2402_14800_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.workload]
    T_skip = min(32768, cfg.T)
    do_skip = cfg.k == 2                               # the top-2 skipping forward is defined for k = 2
    layer = wl.make_layer(cfg, device=dev)            # torch generator on the device
    x, Wg, W1, W3, W2 = (layer[n] for n in ("x", "Wgate", "W1", "W3", "W2"))
    E, H, F, T, k = cfg.E, cfg.H, cfg.F, cfg.T, cfg.k
    dt = binding.MOEP_BF16

    # All buffers are allocated once, outside the timed region.
    logits = torch.empty((T, E), dtype=torch.float32, device=dev)
    Y = torch.empty((E, T, H), dtype=torch.bfloat16, device=dev)
    ws_exp = torch.empty(binding.moe_expert_outputs_workspace(T, E, H, F, dt), dtype=torch.uint8, device=dev)
    ws_enum = torch.empty(max(binding.prune_enumerate_workspace(T, E, H, k, r, dt) for r in cfg.rs),
                          dtype=torch.uint8, device=dev)
    x_skip = x[:T_skip]
    beta = None
    if do_skip:
        ws_skip = torch.empty(binding.moe_forward_skip_workspace(T_skip, E, H, F, dt), dtype=torch.uint8, device=dev)
        # beta = median of w_e1 / w_e0 over the skip batch (Sec. 3.3), calibrated on the device up front.
        _, _, lg, _ = pkg.moe_forward_skip(x_skip, Wg, W1, W3, W2, 0.0, workspace=ws_skip)
        beta = float(pkg.skip_calibrate_beta(lg).item())
        del lg
    bias = layer.get("bias")                           # config 4: per-expert logit bias, added by the harness
    logits_b = torch.empty_like(logits) if bias is not None else logits

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                                  # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    results = {}

    def step():
        pkg.moe_expert_outputs(x, Wg, W1, W3, W2, logits=logits, Y=Y, workspace=ws_exp)
        if bias is not None:
            torch.add(logits, bias, out=logits_b)
        for r, res in zip(cfg.rs, pkg.prune_enumerate_multi(logits_b, Y, k, cfg.rs, workspace=ws_enum)):
            results[r] = res                         # one Gram pass for every r
        if do_skip:
            results["skip"] = pkg.moe_forward_skip(x_skip, Wg, W1, W3, W2, beta, workspace=ws_skip,
                                                   want_logits=False, want_top2=False)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    pkg.kernel_timing_enable(True)
    pkg.kernel_timing_reset()
    torch.cuda.synchronize()
    sampler = PowerSampler()
    sampler.start()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    sampler.stop_flag.set()
    sampler.join()
    records = pkg.kernel_timing_records()        # (kernel, ms) launch by launch, HIP events on the launch stream
    pkg.kernel_timing_enable(False)
    per_launch = {}
    for name, ms in records:
        per_launch.setdefault(name, []).append(ms)
    timing = {name: (float(sum(v)), len(v)) for name, v in per_launch.items()}

    ms_per_step = 1e3 * elapsed / args.steps
    n_sub = sum(math.comb(E, r) for r in cfg.rs)
    value = n_sub * T / (elapsed / args.steps)

    # ---- per-kernel figures: algorithmic work per launch / measured launch time ----
    es = 2
    slots = float(2 * T_skip - int(results["skip"][1].sum().item())) if do_skip else 0.0
    # scorer: selection steps and multiply-adds per (subset, token) pair, summed over the r of this workload
    def pair_ops(r):
        n_act = min(E, min(k, r) + E - r)
        return 4 * n_act + n_act * (n_act + 3) // 2 + 8
    # (the library scores through per-token selection tables when there are many subsets and few selections per token;
    #  those launches are timed under another name and are bound by LDS look-ups: per pair half a look-up per nibble of
    #  the kept mask (one 32-bit entry serves two tokens), one for the selection index, one for the error)
    def uses_tables(r):
        n_act, kk = min(E, min(k, r) + E - r), min(k, r)
        return math.comb(E, r) >= 512 and n_act <= 12 and math.comb(n_act, kk) <= 512
    score_ops = float(sum(math.comb(E, r) * T * pair_ops(r) for r in cfg.rs if not uses_tables(r)))
    lookups = float(sum(math.comb(E, r) * T * ((E + 3) // 4 / 2 + 2) for r in cfg.rs if uses_tables(r)))
    work_per_step = {   # kernel -> (bound, algorithmic flops, bytes or lane operations per STEP, all launches together)
        "gemm_gate_up_swiglu": ("mfma", 4.0 * T * H * F * E),
        "gemm_down": ("mfma", 2.0 * T * H * F * E),
        "gemm_gate_up_swiglu_routed": ("mfma", 4.0 * slots * H * F),
        "gemm_down_routed": ("mfma", 2.0 * slots * H * F),
        "gram": ("hbm", float(E) * T * H * es + 4.0 * T * E * E),
        "subset_score": ("alu", score_ops),
        "subset_score_tables": ("lds", lookups),
        "router_logits": ("hbm", None),      # launched with two different T: reported as time only
    }
    kernels = {}
    for name, (total_ms, n) in sorted(timing.items()):
        avg_ms = total_ms / n
        ms_sorted = sorted(per_launch[name])
        entry = {"launches_per_step": n / args.steps, "avg_ms": avg_ms,
                 "median_ms": ms_sorted[len(ms_sorted) // 2] if len(ms_sorted) % 2 else
                 0.5 * (ms_sorted[len(ms_sorted) // 2 - 1] + ms_sorted[len(ms_sorted) // 2]),
                 "min_ms": ms_sorted[0]}
        bound, w = work_per_step.get(name, (None, None))
        if w:
            w = w * args.steps / n            # algorithmic work of the average launch
            if bound == "alu":
                a = w / (avg_ms * 1e-3)
                entry.update(bound="alu", achieved=a, peak=PEAK_ALU_LANE_OPS, unit="lane-op/s", frac=a / PEAK_ALU_LANE_OPS)
            elif bound == "lds":
                a = w / (avg_ms * 1e-3)
                entry.update(bound="lds", achieved=a, peak=PEAK_LDS_LOOKUPS, unit="look-up/s", frac=a / PEAK_LDS_LOOKUPS)
            elif bound == "mfma":
                a = w / (avg_ms * 1e-3) / 1e12
                entry.update(bound="mfma", achieved=a, peak=PEAK_MFMA_BF16_TFLOPS, unit="TFLOP/s",
                             frac=a / PEAK_MFMA_BF16_TFLOPS)
            else:
                a = w / (avg_ms * 1e-3) / 1e9
                entry.update(bound="hbm", achieved=a, peak=PEAK_HBM_GBS, unit="GB/s", frac=a / PEAK_HBM_GBS)
        kernels[name] = entry
    # Empirical ceiling next to the nominal peak: the MFMA stream of the GEMM's K loop alone (no LDS, memory or
    # barrier traffic), operand bits taken from this layer's x and W1, launches of about the dominant kernel's length.
    sink = torch.empty((1 << 17,), dtype=torch.float32, device=dev)
    pkg.mfma_ceiling(x, W1, 2000, sink)
    torch.cuda.synchronize()
    pkg.kernel_timing_enable(True)
    pkg.kernel_timing_reset()
    ceiling_flop = [pkg.mfma_ceiling(x, W1, 40000, sink) for _ in range(5)][0]
    ceiling_ms = sorted(ms for name, ms in pkg.kernel_timing_records() if name == "mfma_ceiling")
    pkg.kernel_timing_enable(False)
    empirical_peak = ceiling_flop / (ceiling_ms[len(ceiling_ms) // 2] * 1e-3) / 1e12
    dom = kernels["gemm_gate_up_swiglu"]
    roofline = {"kernel": "gemm_gate_up_swiglu", "bound": "mfma", "achieved": dom["achieved"],
                "peak": dom["peak"], "unit": "TFLOP/s", "frac": dom["frac"],
                "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload),
                "launches_per_step": dom["launches_per_step"], "median_ms": dom["median_ms"], "min_ms": dom["min_ms"],
                "empirical_peak": empirical_peak, "frac_of_empirical_peak": dom["achieved"] / empirical_peak,
                "empirical_peak_kind": "MFMA-only launch of the same loop shape on this layer's operand bits, "
                                       "median of 5 launches of %.1f ms" % ceiling_ms[len(ceiling_ms) // 2]}

    gemm_ms = sum(timing[n][0] for n in ("gemm_gate_up_swiglu", "gemm_down")) / args.steps
    enum_names = ("gram", "routing_prep", "subset_score", "subset_score_tables", "loss_reduce_argmin")
    enum_ms = sum(timing[n][0] for n in enum_names if n in timing) / args.steps
    skip_names = ("gemm_gate_up_swiglu_routed", "gemm_down_routed", "skip_route_dispatch", "skip_combine")
    skip_ms = sum(timing[n][0] for n in skip_names if n in timing) / args.steps
    out = {
        "metric": "subset·tokens scored/sec (whole hot path: expert outputs + enumeration for every r"
                  + (" + skip forward)" if do_skip else ")"),
        "value": value, "unit": "subset·tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: E={E} top-{k} H={H} F={F} T={T} r={list(cfg.rs)}; "
                               + (f"skip forward on {T_skip} tokens, beta={beta:.4f}" if do_skip else
                                  f"logit bias variance {cfg.gate_bias_var}"),
                   "input_backend": layer["backend"], "seed": cfg.seed},
        "expert_gemm_tflops": 6.0 * T * H * F * E / (gemm_ms * 1e-3) / 1e12,
        "expert_gemm_ms": gemm_ms,
        "enumerate_subset_tokens_per_s": n_sub * T / (enum_ms * 1e-3),
        "enumerate_ms": enum_ms,                     # one Gram pass shared by every r (prune_enumerate_multi)
        "skip_forward_tokens_per_s": T_skip / (skip_ms * 1e-3) if skip_ms else None,
        "skip_forward_ms": skip_ms,
        "skip_fraction": 1.0 - (slots - T_skip) / T_skip if do_skip else None,
        "argmin": {str(r): int(results[r][1].item()) for r in cfg.rs},
        "roofline": roofline,
        "power": sampler.summary(),          # the GEMMs run at the board's power cap: see the clock it leaves them
        "kernels": kernels,
    }
    # Extra leg, not part of `value`: the same forward with beta = 0 (nothing skipped), for the speedup
    # dynamic skipping buys on this batch.
    if do_skip:
        def forward(b):
            pkg.moe_forward_skip(x_skip, Wg, W1, W3, W2, b, workspace=ws_skip, want_logits=False, want_top2=False)

        def timed_forward(fn, b):
            fn(b)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn(b)
            torch.cuda.synchronize()
            return 1e3 * (time.perf_counter() - t0) / args.steps

        unskipped_ms = timed_forward(forward, 0.0)
        skipped_ms = timed_forward(forward, beta)
        # the same two on expert weights packed once, outside the timed region (a serving loop's case)
        packed = pkg.moe_pack_weights(W1, W3, W2)

        def forward_packed(b):
            pkg.moe_forward_pruned_skip_packed(x_skip, Wg, packed, F, b, workspace=ws_skip, want_logits=False,
                                               want_top2=False)

        unskipped_packed_ms = timed_forward(forward_packed, 0.0)
        skipped_packed_ms = timed_forward(forward_packed, beta)
        del packed
        out["skip_forward_vs_unskipped"] = {"tokens": T_skip, "unskipped_ms": unskipped_ms, "skipped_ms": skipped_ms,
                                            "speedup": unskipped_ms / skipped_ms,
                                            "unskipped_tokens_per_s": T_skip / (unskipped_ms * 1e-3),
                                            "skipped_tokens_per_s": T_skip / (skipped_ms * 1e-3),
                                            "prepacked_weights": {
                                                "unskipped_ms": unskipped_packed_ms, "skipped_ms": skipped_packed_ms,
                                                "speedup": unskipped_packed_ms / skipped_packed_ms,
                                                "skipped_tokens_per_s": T_skip / (skipped_packed_ms * 1e-3)}}
    n_rank_needed = max(min(E, min(k, r) + E - r) for r in cfg.rs)
    # (not with a harness-side logit bias: the rank-limited pass ranks by its own router logits)
    if not args.no_rank_limited and n_rank_needed <= 8 and bias is None:
        # Extra leg, timed on its own and NOT part of `value`: the same enumeration results from the
        # rank-limited pass (each token through its n_rank best-ranked experts only).
        n_rank = n_rank_needed
        ws_rk = torch.empty(binding._lib.moe_expert_outputs_ranked_workspace(T, E, H, F, dt, n_rank),
                            dtype=torch.uint8, device=dev)
        rk_out = (logits, torch.empty((T, n_rank), dtype=torch.int32, device=dev),
                  torch.empty((T, n_rank), dtype=torch.int32, device=dev),
                  torch.empty((T * n_rank, H), dtype=torch.bfloat16, device=dev))
        rk_res = {}

        def ranked_step():
            pkg.moe_expert_outputs_ranked(x, Wg, W1, W3, W2, n_rank, workspace=ws_rk, out=rk_out)
            for r in cfg.rs:
                rk_res[r] = pkg.prune_enumerate_ranked(*rk_out, k, r, workspace=ws_enum)

        ranked_step()
        torch.cuda.synchronize()
        pkg.kernel_timing_enable(True)
        pkg.kernel_timing_reset()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ranked_step()
        torch.cuda.synchronize()
        rk_elapsed = (time.perf_counter() - t0) / args.steps
        rk_timing = pkg.kernel_timing_collect()
        pkg.kernel_timing_enable(False)
        rk_gemm_ms = sum(rk_timing[n][0] for n in ("gemm_gate_up_swiglu_routed", "gemm_down_routed")) / args.steps
        out["rank_limited"] = {
            "n_rank": n_rank, "ms_per_pass": 1e3 * rk_elapsed,
            "dense_ms_per_pass": gemm_ms + enum_ms,
            "expert_gemm_ms": rk_gemm_ms,
            "expert_gemm_tflops": 6.0 * T * n_rank * H * F / (rk_gemm_ms * 1e-3) / 1e12,
            "subset_tokens_per_s_with_skip_leg": n_sub * T / (rk_elapsed + skip_ms * 1e-3),
            "same_argmin": all(int(rk_res[r][1].item()) == int(results[r][1].item()) for r in cfg.rs),
            "kernels_ms": {n: v[0] / v[1] for n, v in sorted(rk_timing.items())},
        }
        del ws_rk, rk_out
    if all(math.comb(E, r) <= 128 for r in cfg.rs) and k <= 4 and E * H * 2 <= 148 * 1024:
        # Extra leg, NOT part of `value`: Eq. 3 as written (no Gram matrices; every token's rows read once and kept in
        # LDS while all subsets are scored) against the Gram path, each r on its own, same logits and Y.
        ws_dir = torch.empty(max(binding._lib.prune_enumerate_direct_workspace(T, E, H, k, r, dt) for r in cfg.rs),
                             dtype=torch.uint8, device=dev)
        leg = {"what": "Eq. 3 as written (prune_enumerate_direct) against the Gram path (prune_enumerate), each r on its "
                       "own, same logits and Y; not part of `value`"}
        for r in cfg.rs:
            d = pkg.prune_enumerate_direct(logits_b, Y, k, r, workspace=ws_dir)
            g = pkg.prune_enumerate(logits_b, Y, k, r, workspace=ws_enum)
            torch.cuda.synchronize()
            pkg.kernel_timing_enable(True)
            pkg.kernel_timing_reset()
            for _ in range(3):
                pkg.prune_enumerate_direct(logits_b, Y, k, r, workspace=ws_dir)
                pkg.prune_enumerate(logits_b, Y, k, r, workspace=ws_enum)
            torch.cuda.synchronize()
            tm = pkg.kernel_timing_collect()
            pkg.kernel_timing_enable(False)
            direct_ms = tm["direct_gather_weight_reduce"][0] / tm["direct_gather_weight_reduce"][1]
            gram_ms = sum(tm[n][0] / tm[n][1] for n in ("gram", "routing_prep", "subset_score", "subset_score_tables")
                          if n in tm)
            leg[f"r={r}"] = {"direct_ms": direct_ms, "gram_path_ms": gram_ms,
                             "bytes_of_Y": float(E) * T * H * es,
                             "direct_GBps": float(E) * T * H * es / (direct_ms * 1e-3) / 1e9,
                             "max_rel_difference": float(((d[0] - g[0]).abs() / g[0].abs().clamp_min(1e-30)).max().item()),
                             "same_argmin": int(d[1].item()) == int(g[1].item())}
        leg["all_r"] = {"direct_ms": sum(v["direct_ms"] for v in leg.values() if isinstance(v, dict)),
                        "gram_path_ms_one_shared_gram_pass": enum_ms}
        out["direct_path"] = leg
        del ws_dir
    if args.workload == "C3":
        # The paper's own figures for this path, as context only: other hardware, the whole 32-layer model, and its wall
        # times include the calibration forward (Sec. 4.1 for the pruning times, the speed-up table of Sec. 4 for skipping).
        out["paper_context"] = {
            "expert_pruning_wall_time": "about 30 min (r=6) and 90 min (r=4) for all 32 MoE layers of Mixtral 8x7B on "
                                        "128 x 2048 calibration tokens; hardware not stated for that run (A100-80G "
                                        "elsewhere in the paper)",
            "derived_subset_tokens_per_s_per_layer": {"r=6": 28 * 262144 / (1800.0 / 32), "r=4": 70 * 262144 / (5400.0 / 32)},
            "dynamic_skipping_generation_speedup": 1.08,
            "note": "context, not a target: vs_baseline stays null",
        }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, layer, Y, logits_b, torch, wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
