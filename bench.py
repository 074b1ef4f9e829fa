#!/usr/bin/env python3
"""Benchmark of the MoE-layer forward hot path on one MI355X.

A "step" is one pass of the whole path (router -> permute -> grouped SwiGLU
expert GEMMs -> un-permute/combine, plus the shared expert where the workload
has one) over one batch of seeded synthetic tokens that already sit in HBM.
Default workload: the Mixtral-8x22B-shaped layer (T=8192, H=6144, E=8, K=2,
F=16384, bf16, dropless, skewed router).

Prints ONE JSON line: whole-path tokens/s (`value`), the roofline figures of
the dominant kernel (the gate/up grouped GEMM) measured with HIP events on the
launch stream inside the timed region, per-stage figures (`stages`) and the CPU
oracle timed on a bounded sample of the same workload (`cpu_baseline`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense fp8 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
NSETS = 4                   # rotating activation/workspace sets (defeats the 256 MB Infinity Cache)



def measured_traffic(workload):
    """Bytes one gate/up GEMM launch moves past the L2 (fetched + written), from the rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE summary of this workload under profiles/ (its line `roofline.traffic gate_up = <bytes>`); None when
    that workload was not profiled."""
    import re
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_hbm_traffic.txt")
    try:
        m = re.search(r"^roofline\.traffic gate_up = ([0-9.eE+]+)", open(path).read(), flags=re.M)
    except OSError:
        return None
    return float(m.group(1)) if m else None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="mixtral8x22b")
    ap.add_argument("--precision", default="bf16", choices=["bf16", "fp8"],
                    help="fp8: expert FFN on E4M3 operands with delayed per-tensor scaling (weights quantised "
                         "beforehand and resident, activations quantised inside the timed step); a separate "
                         "experiment, the headline metric is the bf16 run")
    ap.add_argument("--ffn-backward", action="store_true",
                    help="also time the backward of the grouped expert FFN (and the one-off weight transposes it "
                         "needs) on the same routing; reported in a separate object, not part of the step")
    ap.add_argument("--backward", action="store_true",
                    help="also time the backward of the whole layer (combine, expert FFN, router, permute backward in "
                         "mirrored order) and report it under 'backward' (bf16 workloads without a shared expert)")
    ap.add_argument("--dispatch-backward", action="store_true",
                    help="also time the backward of the dispatcher's two data movements (combine backward, permute "
                         "backward) on the same routing; reported in a separate object, not part of the step")
    ap.add_argument("--permute-variants", action="store_true",
                    help="also time moe_permute_variant (drop by score, pad to capacity) on the same routing; "
                         "workloads with a capacity factor only")
    ap.add_argument("--ep-share", type=int, default=0, metavar="S",
                    help="also time what ONE GPU of an S-rank expert-parallel group of this workload does between the "
                         "two All-to-All-Vs: gather the received chunks by expert, run its E/S experts, gather back "
                         "by source (every rank holding this workload's token count; no collective is run)")
    ap.add_argument("--library-gemm", action="store_true",
                    help="also time the two expert GEMMs on UNIFORM experts (every expert the same whole number of "
                         "256-row tiles, the workload's weights and token values) against the vendor library's GEMM "
                         "(torch.matmul, one call per expert, no grouping, no SwiGLU) on the same operands: context "
                         "for the roofline fraction, bf16 workloads only")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="moe_set_option knob for sweeps, e.g. gemm_variant=40 (repeatable)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true",
                    help="skip the bare-MFMA probe (what this box sustains on zero and on workload-like operands)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target wall time of the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy 5 times (scale reference for rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    return ap.parse_args()


class PowerSampler:
    """Average board power over a region, from the amdgpu hwmon file (microwatts), read by a host thread every
    couple of milliseconds; reports None where the file is not readable."""

    def __init__(self):
        import glob
        self.path = None
        for pat in ("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input",
                    "/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"):
            for f in sorted(glob.glob(pat)):
                try:
                    int(open(f).read())
                    self.path = f
                    break
                except (OSError, ValueError):
                    pass
            if self.path:
                break
        self.samples = []
        self._stop = None
        self._thread = None

    def start(self):
        import threading
        self.samples = []
        if self.path is None:
            return
        self._stop = threading.Event()

        def loop():
            while not self._stop.is_set():
                try:
                    self.samples.append(int(open(self.path).read()) * 1e-6)
                except (OSError, ValueError):
                    pass
                time.sleep(0.002)
        self._thread = threading.Thread(target=loop, daemon=True)
        self._thread.start()

    def stop(self):
        if self._thread is not None:
            self._stop.set()
            self._thread.join()
            self._thread = None
        v = self.samples
        if len(v) >= 4:
            v = v[len(v) // 4:]          # the reading lags the load: keep the later three quarters
        return round(sum(v) / len(v), 0) if v else None


def cpu_baseline(inp, capacity, target_s):
    """Time the CPU oracle (as it stands) on the first S tokens of the batch."""
    import numpy as np
    import oracle
    cfg = inp.cfg
    t = inp.tensors

    def run(S):
        x = np.ascontiguousarray(t["x"][:S])
        t0 = time.perf_counter()
        oracle.layer_forward(x, t["w_router"], inp.bias, t["w_gate"], t["w_up"], t["w_down"], K=cfg.K,
                             renormalize=cfg.renormalize, capacity_rows=capacity,
                             ws_gate=t.get("ws_gate"), ws_up=t.get("ws_up"), ws_down=t.get("ws_down"))
        return time.perf_counter() - t0

    S = 8
    dt = run(S)
    S2 = int(max(S, min(cfg.T, S * target_s / max(dt, 1e-3))))
    if S2 > 2 * S:
        S, dt = S2, run(S2)
    return {"value": S / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {S} tokens of the batch through oracle.layer_forward with the full weights, {dt:.1f} s"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all experts local, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2504_14960_amd as moe
    from moe_inputs import get_config, make_layer_inputs

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    if args.copy_calibration:
        src = torch.full((1 << 30,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": 1 << 30, "copy_calibration_bytes_written": 1 << 30, "launches": 5}))
        return
    for opt in args.option:
        nm, val = opt.split("=")
        moe.set_option(nm, int(val))
    cfg = get_config(args.config)
    T, H, E, K, F, Fs = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F, cfg.shared_F
    bf16 = cfg.dtype == "bf16"
    es = 2 if bf16 else 4
    tdt = torch.bfloat16 if bf16 else torch.float32
    capacity = moe.capacity_from_factor(cfg.capacity_factor, T, K, E) if cfg.capacity_factor else 0
    r_max = moe.max_rows(T, K, E, capacity)

    t_gen = time.perf_counter()
    inp = make_layer_inputs(cfg)
    t_gen = time.perf_counter() - t_gen

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    w = {k: dev(v) for k, v in inp.tensors.items() if k != "x"}
    bias = None if inp.bias is None else dev(inp.bias)
    x_host = inp.tensors["x"]
    sets = []
    for i in range(NSETS):
        xs = dev(np.roll(x_host, i * 17, axis=0)) if i else dev(x_host)
        s = dict(
            x=xs,
            logits=torch.empty((T, E), dtype=torch.float32, device="cuda"),
            idx=torch.empty((T, K), dtype=torch.int32, device="cuda"),
            gate=torch.empty((T, K), dtype=torch.float32, device="cuda"),
            counts=torch.empty((E,), dtype=torch.int32, device="cuda"),
            offsets=torch.empty((E + 1,), dtype=torch.int32, device="cuda"),
            roa=torch.empty((T * K,), dtype=torch.int32, device="cuda"),
            aor=torch.empty((r_max,), dtype=torch.int32, device="cuda"),
            pws=torch.empty((moe.permute_workspace_bytes(T, K, E) + 256,), dtype=torch.uint8, device="cuda"),
            x_perm=torch.empty((r_max, H), dtype=tdt, device="cuda"),
            h=torch.empty((r_max, F), dtype=tdt, device="cuda"),
            y_perm=torch.empty((r_max, H), dtype=tdt, device="cuda"),
            y=torch.empty((T, H), dtype=tdt, device="cuda"),
        )
        if Fs:
            s["s_off"] = torch.tensor([0, T], dtype=torch.int32, device="cuda")
            s["s_h"] = torch.empty((T, Fs), dtype=tdt, device="cuda")
            s["s_y"] = torch.empty((T, H), dtype=tdt, device="cuda")
        sets.append(s)

    fp8 = args.precision == "fp8"
    if fp8:
        if not bf16 or Fs:
            print("bench.py: --precision fp8 needs a bf16 workload without a shared expert", file=sys.stderr)
            sys.exit(2)
        # delayed scaling: the scales come from amax values of an earlier step; here one calibration pass
        # (outside the timed region) plays that earlier step
        def amax_of(t):
            a = torch.zeros(1, dtype=torch.float32, device="cuda")
            moe.fp8_quantize(t, 1.0, torch.empty(t.numel(), dtype=torch.uint8, device="cuda"), a)
            return float(a.item())
        f8 = {"s": {}, "w": {}}
        for k in ("w_gate", "w_up", "w_down"):
            f8["s"][k] = moe.fp8_delayed_scale([amax_of(w[k])])
            f8["w"][k] = torch.empty(w[k].shape, dtype=torch.uint8, device="cuda")
            moe.fp8_quantize(w[k], f8["s"][k], f8["w"][k])
        f8["s"]["x"] = moe.fp8_delayed_scale([amax_of(sets[0]["x"])])
        f8["dq_gate"] = 1.0 / (f8["s"]["x"] * f8["s"]["w_gate"])
        f8["dq_up"] = 1.0 / (f8["s"]["x"] * f8["s"]["w_up"])
        f8["scale_h"] = 1.0
        for s in sets:
            s["xq"] = torch.empty((r_max, H), dtype=torch.uint8, device="cuda")
            s["hq"] = torch.empty((r_max, F), dtype=torch.uint8, device="cuda")
            s["amax"] = torch.zeros(2, dtype=torch.float32, device="cuda")
        del w["w_gate"], w["w_up"], w["w_down"]

    # shader clock the two expert GEMMs run at: workgroup 0 of each launch leaves its shader-clock and 100 MHz
    # reference ticks in these cells (the last launch's values are read after the timed region)
    clk = {nm: torch.zeros(2, dtype=torch.int64, device="cuda") for nm in ("gate_up", "down")}

    stage_names = ["router", "permute", "gate_up", "down"] + (["shared"] if Fs else []) + ["combine"]

    def step(s, events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        moe.router_topk(s["x"], w["w_router"], bias, s["logits"], K, cfg.renormalize, s["idx"], s["gate"])
        mark(1)
        if fp8:
            # the amax cells of this step (x, h) start from zero; the permute writes x_perm as E4M3 directly
            s["amax"].zero_()
            moe.permute_fp8(s["x"], s["idx"], E, capacity, f8["s"]["x"], s["xq"], s["counts"], s["offsets"],
                            s["roa"], s["aor"], s["amax"][0:1], s["pws"])
            mark(2)
            moe.expert_gate_up_fp8(s["xq"], s["offsets"], f8["w"]["w_gate"], f8["w"]["w_up"], f8["dq_gate"],
                                   f8["dq_up"], f8["scale_h"], s["hq"], s["amax"][1:2])
            mark(3)
            moe.expert_down_fp8(s["hq"], s["offsets"], f8["w"]["w_down"],
                                1.0 / (f8["scale_h"] * f8["s"]["w_down"]), s["y_perm"])
            mark(4)
            n = 4
        else:
            moe.permute(s["x"], s["idx"], E, capacity, s["x_perm"], s["counts"], s["offsets"], s["roa"], s["aor"],
                        s["pws"])
            mark(2)
            moe.gemm_clock_sample(clk["gate_up"])
            moe.expert_gate_up(s["x_perm"], s["offsets"], w["w_gate"], w["w_up"], s["h"])
            mark(3)
            moe.gemm_clock_sample(clk["down"])
            moe.expert_down(s["h"], s["offsets"], w["w_down"], s["y_perm"])
            moe.gemm_clock_sample(None)
            mark(4)
            n = 4
        addend = None
        if Fs:
            moe.grouped_gemm_swiglu(s["x"], s["s_off"], w["ws_gate"].unsqueeze(0), w["ws_up"].unsqueeze(0),
                                    w["ws_down"].unsqueeze(0), s["s_h"], s["s_y"])
            addend = s["s_y"]
            n += 1
            mark(n)
        moe.unpermute_combine(s["y_perm"], s["roa"], s["gate"], addend, s["y"])
        mark(n + 1)

    if fp8:
        # calibration step: records max |h| with a neutral scale, as the previous step of a delayed-scaling run would
        step(sets[0])
        torch.cuda.synchronize()
        f8["scale_h"] = moe.fp8_delayed_scale([float(sets[0]["amax"][1].item())])
    for i in range(args.warmup):
        step(sets[i % NSETS])
    torch.cuda.synchronize()
    R = int(sets[0]["offsets"][E].item())          # kept rows (outside the timed region)
    counts = sets[0]["counts"].cpu().tolist()

    nev = len(stage_names) + 1
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(nev)] for _ in range(args.steps)]
    power = PowerSampler()
    torch.cuda.synchronize()
    power.start()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % NSETS], evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_watts = power.stop()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    per_step = {nm: sorted(evs[i][j].elapsed_time(evs[i][j + 1]) for i in range(args.steps))
                for j, nm in enumerate(stage_names)}
    stage_ms = {nm: sum(v) / len(v) for nm, v in per_step.items()}

    # algorithmic work (useful bytes / flops only)
    maps = 8 * T * K
    alg = {
        "router": ("GB/s", T * H * es + T * (4 * E + 8 * K)),
        "permute": ("GB/s", (T + R) * H * es + maps),
        "gate_up": ("TFLOP/s", 4.0 * R * H * F),
        "down": ("TFLOP/s", 2.0 * R * H * F),
        "combine": ("GB/s", (R + T + (T if Fs else 0)) * H * es + maps),
    }
    if Fs:
        alg["shared"] = ("TFLOP/s", 6.0 * T * H * Fs)
    if fp8:
        alg["permute"] = ("GB/s", T * H * es + R * H + maps)   # bf16 rows in, E4M3 rows out
    stages = {}
    for nm in stage_names:
        unit, work = alg[nm]
        ms = stage_ms[nm]
        rate = work / (ms * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9)
        peak = (PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS) if unit == "TFLOP/s" else PEAK_HBM_GBS
        v = per_step[nm]
        stages[nm] = {"ms": round(ms, 4), "ms_median": round(v[len(v) // 2], 4), "ms_min": round(v[0], 4),
                      "achieved": round(rate, 1), "unit": unit, "frac": round(rate / peak, 4)}
    # what the two rooflines allow for the ragged expert GEMMs: per expert the larger of its MFMA time and the
    # time to stream its weights and rows once from HBM, summed over the experts (they share the chip in turn)
    def attainable_ms(flop_per_row, w_bytes, row_bytes):
        t = 0.0
        for n in counts:
            if n > 0:
                t += max(flop_per_row * n / ((PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS) * 1e12),
                         (w_bytes + n * row_bytes) / (PEAK_HBM_GBS * 1e9))
        return round(t * 1e3, 4)
    ges = 1 if fp8 else es   # bytes per GEMM operand element
    if not fp8:
        for nm, cell in clk.items():
            tk = cell.cpu().tolist()
            if tk[1] > 0:
                stages[nm]["shader_mhz"] = round(100.0 * tk[0] / tk[1], 0)
    stages["gate_up"]["attainable_ms"] = attainable_ms(4.0 * H * F, 2 * H * F * ges, (H + F) * ges)
    stages["down"]["attainable_ms"] = attainable_ms(2.0 * H * F, H * F * ges, H * es + F * ges)

    dom = stages["gate_up"]
    roofline = {"kernel": "gate/up grouped GEMM (moe_expert_gate_up)", "bound": "mfma", "achieved": dom["achieved"],
                "peak": PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": dom["frac"],
                "traffic": None if fp8 else measured_traffic(cfg.name)}
    if "shader_mhz" in dom:
        roofline["shader_mhz"] = dom["shader_mhz"]
    # board power averaged over the timed steps (the two expert GEMMs are ~98 % of a step at the default workload)
    roofline["board_power_w"] = step_watts

    out = {
        "metric": "MoE layer fwd tokens/s; grouped-GEMM % bf16 MFMA peak; permute GB/s % HBM",
        "value": round(T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp8e4m3" if fp8 else cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name} layer: T={T} H={H} E={E} K={K} F={F}"
                               + (f" shared_F={Fs}" if Fs else "")
                               + (f" capacity={capacity}" if capacity else " dropless")
                               + (f" bias={cfg.bias}" if cfg.bias else "")
                               + (" [expert FFN in FP8 E4M3, delayed scaling, weights pre-quantised]" if fp8 else ""),
                   "kept_rows": R, "rows_per_expert_min_max": [min(counts), max(counts)],
                   "buffer_sets": NSETS, "input_generation_s": round(t_gen, 1)},
        "roofline": roofline,
        "stages": stages,
        "context": "the paper reports 49.3 % (Mixtral 8x22B) and 39.0 % (Qwen2-57B-A14B) MFU for whole training "
                   "steps on H100 clusters: other hardware, other scope, shown for orientation only",
    }
    if not args.no_probe and bf16:
        # the bare inner loop of the grouped GEMM (MFMA + LDS fragment reads, nothing else) on this machine, with
        # all-zero operands and with operands distributed like the workload's: the second is what power
        # management lets the dense MFMA sustain here, the practical ceiling under roofline.peak
        from moe_inputs import make_tokens
        nwg, iters = 256, 20000
        sink = torch.empty(nwg * 256, dtype=torch.float32, device="cuda")
        ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
        like = dev(np.ascontiguousarray(np.concatenate([make_tokens(4242, 512 if fp8 else 256, 64, True, 1.0),
                                                         make_tokens(4243, 512 if fp8 else 256, 64, True, 0.02)])))
        if fp8:
            # the same values as E4M3 codes under per-tensor scales 448 / amax: [256][128] bytes per operand
            q = torch.empty((2, 32768), dtype=torch.uint8, device="cuda")
            halves = like.view(2, -1)
            for i in range(2):
                a = torch.zeros(1, dtype=torch.float32, device="cuda")
                moe.fp8_quantize(halves[i], 1.0, q[i], a)
                moe.fp8_quantize(halves[i], moe.fp8_delayed_scale([float(a.item())]), q[i])
            images = {"zeros": torch.zeros(65536, dtype=torch.uint8, device="cuda"), "workload_like": q.view(-1)}
            run_probe, flop = moe.probe_mfma_fp8, 16777216.0
        else:
            images = {"zeros": torch.zeros(32768, dtype=torch.int16, device="cuda"), "workload_like": like}
            run_probe, flop = moe.probe_mfma_bf16, 8388608.0
        probe = {}
        for nm, d_img in images.items():
            run_probe(d_img, iters // 10, nwg, sink, ticks)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            power.start()
            e0.record()
            for _ in range(12):
                run_probe(d_img, iters, nwg, sink, ticks)
            e1.record()
            torch.cuda.synchronize()
            watts = power.stop()
            tk = ticks.cpu().tolist()
            probe[nm] = {"tflops": round(12 * nwg * iters * flop / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1),
                         "shader_mhz": round(100.0 * tk[0] / max(tk[1], 1), 0), "board_power_w": watts}
        probe["note"] = ("bare MFMA + LDS fragment loop of the grouped GEMM, 256 workgroups x 4 waves, no global traffic: "
                         "the rate and clock this box sustains; operands ~N(0,1) x N(0,0.02^2) as in the workload"
                         + (", as E4M3 codes" if fp8 else ""))
        roofline["mfma_probe"] = probe
        roofline["frac_of_probe"] = round(dom["achieved"] / probe["workload_like"]["tflops"], 4)
    if args.ffn_backward and not fp8 and bf16:
        s0 = sets[0]
        bfk = dict(dtype=torch.bfloat16, device="cuda")
        wgu_t = torch.empty((E, H, 2 * F), **bfk)
        wd_t = torch.empty((E, F, H), **bfk)
        dwg, dwu, dwd = torch.empty((E, F, H), **bfk), torch.empty((E, F, H), **bfk), torch.empty((E, H, F), **bfk)
        dxp = torch.empty((r_max, H), **bfk)
        bws = torch.empty(moe.expert_backward_workspace_bytes(r_max, H, F, E) + 256, dtype=torch.uint8, device="cuda")

        def timed(fn, n, w):
            for _ in range(w):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n

        n_b, w_b = max(3, args.steps // 4), 2
        t_tr = timed(lambda: moe.expert_weights_transpose(w["w_gate"], w["w_up"], w["w_down"], wgu_t, wd_t), n_b, w_b)
        # y_perm stands in for the incoming gradient dy_perm (same shape and value range)
        t_bw = timed(lambda: moe.grouped_gemm_swiglu_backward(s0["x_perm"], s0["h"], None, s0["y_perm"], s0["offsets"],
                                                              w["w_gate"], w["w_up"], wgu_t, wd_t, dxp, dwg, dwu, dwd,
                                                              bws), n_b, w_b)
        useful = 12.0 * R * H * F            # dh, dx (2 products), three weight gradients
        out["ffn_backward"] = {
            "ms": round(t_bw, 4), "useful_tflops": round(useful / (t_bw * 1e-3) / 1e12, 1),
            "frac_of_bf16_peak": round(useful / (t_bw * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
            "executed_flop_over_useful": round(16.0 / 12.0, 3),   # g and u are recomputed: 4 R H F more
            "weights_transpose_ms": round(t_tr, 4),
            "weights_transpose_gbs": round(2 * 3 * E * H * F * es / (t_tr * 1e-3) / 1e9, 1),
            "workspace_gb": round(bws.numel() / 1e9, 2)}
    if args.backward and not fp8 and bf16 and not Fs:
        s0 = sets[0]
        bfk = dict(dtype=torch.bfloat16, device="cuda")
        f32k = dict(dtype=torch.float32, device="cuda")
        b = dict(wgu_t=torch.empty((E, H, 2 * F), **bfk), wd_t=torch.empty((E, F, H), **bfk),
                 dwg=torch.empty((E, F, H), **bfk), dwu=torch.empty((E, F, H), **bfk), dwd=torch.empty((E, H, F), **bfk),
                 gu=torch.empty((r_max, 2 * F), **bfk),
                 dy_perm=torch.empty((r_max, H), **bfk), dx_perm=torch.empty((r_max, H), **bfk),
                 dgate=torch.empty((T, K), **f32k), dlogits=torch.empty((T, E), **f32k),
                 dx_r=torch.empty((T, H), **bfk), dx=torch.empty((T, H), **bfk),
                 dwr=torch.empty((E, H), **f32k), dbias=torch.empty((E,), **f32k),
                 ews=torch.empty(moe.expert_backward_workspace_bytes(r_max, H, F, E) + 256, dtype=torch.uint8, device="cuda"),
                 rws=torch.empty(moe.router_backward_workspace_bytes(T, H, E) + 256, dtype=torch.uint8, device="cuda"))
        bnames = ["weights_transpose", "combine_backward", "ffn_backward", "router_backward", "permute_backward"]

        def bstep(ev=None):
            def mark(i):
                if ev is not None:
                    ev[i].record()
            mark(0)   # s0["y"] plays dy, the gradient of the layer output (same shape and value range)
            moe.expert_weights_transpose(w["w_gate"], w["w_up"], w["w_down"], b["wgu_t"], b["wd_t"])
            mark(1)
            moe.unpermute_combine_backward(s0["y"], s0["y_perm"], s0["roa"], s0["gate"], b["dy_perm"], b["dgate"])
            mark(2)
            moe.grouped_gemm_swiglu_backward(s0["x_perm"], s0["h"], b["gu"], b["dy_perm"], s0["offsets"], w["w_gate"], w["w_up"],
                                             b["wgu_t"], b["wd_t"], b["dx_perm"], b["dwg"], b["dwu"], b["dwd"], b["ews"])
            mark(3)
            moe.router_backward(s0["x"], w["w_router"], s0["logits"], s0["idx"], b["dgate"], cfg.renormalize,
                                b["dlogits"], b["dx_r"], b["dwr"], b["dbias"], b["rws"])
            mark(4)
            moe.permute_backward(b["dx_perm"], s0["roa"], b["dx_r"], b["dx"], K)
            mark(5)

        def fstep():      # the training forward: as step(), the first GEMM also keeping g | u for the backward
            moe.router_topk(s0["x"], w["w_router"], bias, s0["logits"], K, cfg.renormalize, s0["idx"], s0["gate"])
            moe.permute(s0["x"], s0["idx"], E, capacity, s0["x_perm"], s0["counts"], s0["offsets"], s0["roa"],
                        s0["aor"], s0["pws"])
            moe.expert_gate_up_saving(s0["x_perm"], s0["offsets"], w["w_gate"], w["w_up"], s0["h"], b["gu"])
            moe.expert_down(s0["h"], s0["offsets"], w["w_down"], s0["y_perm"])
            moe.unpermute_combine(s0["y_perm"], s0["roa"], s0["gate"], None, s0["y"])

        n_b = max(3, args.steps // 4)
        for _ in range(2):
            fstep()
        torch.cuda.synchronize()
        tf0 = time.perf_counter()
        for i in range(n_b):
            fstep()
        torch.cuda.synchronize()
        fms = (time.perf_counter() - tf0) * 1e3 / n_b
        for _ in range(2):
            bstep()
        bev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(n_b)]
        torch.cuda.synchronize()
        tb0 = time.perf_counter()
        for i in range(n_b):
            bstep(bev[i])
        torch.cuda.synchronize()
        bms = (time.perf_counter() - tb0) * 1e3 / n_b
        bst = {nm: round(sum(bev[i][j].elapsed_time(bev[i][j + 1]) for i in range(n_b)) / n_b, 4)
               for j, nm in enumerate(bnames)}
        useful = 12.0 * R * H * F
        out["backward"] = {
            "ms_per_step": round(bms, 4), "steps": n_b, "stage_ms": bst,
            "forward_saving_gu_ms": round(fms, 4),
            "tokens_per_s_fwd_bwd": round(T / ((fms + bms) * 1e-3), 1),
            "ffn_backward_useful_tflops": round(useful / (bst["ffn_backward"] * 1e-3) / 1e12, 1),
            "layer_useful_tflops_fwd_bwd": round(18.0 * R * H * F / ((fms + bms) * 1e-3) / 1e12, 1),
            "note": "weights_transpose re-lays the three expert weight tensors once per optimizer step; "
                    "with several micro-batches per step it is paid once, not per backward"}
    if args.library_gemm and bf16 and not fp8:
        s0 = sets[0]
        rows_e = max(256, (R // E) // 256 * 256)          # whole tiles per expert, about the workload's row count
        Ru = rows_e * E
        offs_u = torch.arange(0, Ru + 1, rows_e, dtype=torch.int32, device="cuda")
        xu = s0["x_perm"][:Ru] if Ru <= r_max else s0["x_perm"].repeat((Ru + r_max - 1) // r_max, 1)[:Ru]
        hu = torch.empty((Ru, F), dtype=tdt, device="cuda")
        yu = torch.empty((Ru, H), dtype=tdt, device="cuda")
        gu_lib = torch.empty((rows_e, 2 * F), dtype=tdt, device="cuda")
        y_lib = torch.empty((rows_e, H), dtype=tdt, device="cuda")
        # the library multiplies by one [2F, H] matrix per expert (gate rows, then up rows): same FLOP, no activation
        w_gu = [torch.cat([w["w_gate"][e], w["w_up"][e]]).t() for e in range(min(E, 8))]
        w_dn = [w["w_down"][e].t() for e in range(min(E, 8))]

        def lib_gate_up():
            for e in range(E):
                torch.matmul(xu[e * rows_e:(e + 1) * rows_e], w_gu[e % len(w_gu)], out=gu_lib)

        def lib_down():
            for e in range(E):
                torch.matmul(hu[e * rows_e:(e + 1) * rows_e], w_dn[e % len(w_dn)], out=y_lib)

        def timed_ms(fn, n=8, wu=3):
            for _ in range(wu):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n

        res = {}
        for nm, ours, theirs, flop in (
                ("gate_up", lambda: moe.expert_gate_up(xu, offs_u, w["w_gate"], w["w_up"], hu), lib_gate_up, 4.0 * Ru * H * F),
                ("down", lambda: moe.expert_down(hu, offs_u, w["w_down"], yu), lib_down, 2.0 * Ru * H * F)):
            # interleaved, twice, so that both sides see the same clocks
            t_o = [timed_ms(ours), 0.0]
            t_l = [timed_ms(theirs), 0.0]
            t_o[1], t_l[1] = timed_ms(ours), timed_ms(theirs)
            res[nm] = {"this_tflops": [round(flop / (t * 1e-3) / 1e12, 1) for t in t_o],
                       "library_tflops": [round(flop / (t * 1e-3) / 1e12, 1) for t in t_l]}
        res["shape"] = {"experts": E, "rows_per_expert": rows_e, "H": H, "F": F}
        res["note"] = ("uniform experts; library = torch.matmul (hipBLASLt), one call per expert on the same operands, "
                       "gate and up weights as one [2F, H] matrix, no SwiGLU, its output overwritten by every call")
        out["library_gemm"] = res
    if args.permute_variants and capacity > 0:
        s0 = sets[0]
        vws = torch.empty(moe.permute_variant_workspace_bytes(T, K, E) + 256, dtype=torch.uint8, device="cuda")
        res = {}
        for nm, by_score, pad in (("by_position_packed", False, False), ("by_score_packed", True, False),
                                  ("by_position_padded", False, True), ("by_score_padded", True, True)):
            rows = E * capacity if pad else r_max
            xp = torch.empty((rows, H), dtype=tdt, device="cuda")
            aor = torch.empty((rows,), dtype=torch.int32, device="cuda")
            def run():
                moe.permute_variant(s0["x"], s0["idx"], s0["gate"], E, capacity, by_score, pad, xp, s0["counts"],
                                    s0["offsets"], s0["roa"], aor, vws)
            for _ in range(args.warmup):
                run()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                run()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            kept = int(s0["counts"].sum().item())
            work = (T + (rows if pad else kept)) * H * es + maps      # rows read once; rows written (pad: zeros too)
            res[nm] = {"ms": round(ms, 4), "kept_rows": kept, "rows_written": rows if pad else kept,
                       "achieved": round(work / (ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                       "frac": round(work / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        step(s0)      # leave the plain dispatch's maps behind for what follows
        out["permute_variants"] = res
    if args.ep_share:
        S = args.ep_share
        if E % S or fp8 or not bf16:
            print("bench.py: --ep-share S needs a bf16 workload (not --precision fp8) with E divisible by S", file=sys.stderr)
            sys.exit(2)
        El = E // S
        step(sets[0])
        cnt = sets[0]["counts"].cpu().numpy()
        loads = cnt.reshape(S, El).sum(1)
        d = int(loads.argmax())                          # the rank the group waits for
        # every source sends what this batch sends: i.i.d. batches differ by a few per cent only
        chunk = np.tile(cnt[d * El:(d + 1) * El], S).astype(np.int32)          # chunk (s, e), source-major
        Rr = int(chunk.sum())
        by_expert = np.array([sr * El + e for e in range(El) for sr in range(S)], dtype=np.int32)
        by_source = np.array([e * S + sr for sr in range(S) for e in range(El)], dtype=np.int32)
        g = dict(recv=torch.randn((Rr, H), dtype=tdt, device="cuda"),
                 grouped=torch.empty((Rr, H), dtype=tdt, device="cuda"),
                 h=torch.empty((Rr, F), dtype=tdt, device="cuda"),
                 y=torch.empty((Rr, H), dtype=tdt, device="cuda"),
                 back=torch.empty((Rr, H), dtype=tdt, device="cuda"),
                 chunk=torch.from_numpy(chunk).cuda(), by_expert=torch.from_numpy(by_expert).cuda(),
                 by_source=torch.from_numpy(by_source).cuda(),
                 rows_e=torch.empty(S * El, dtype=torch.int32, device="cuda"),
                 goff=torch.empty(El + 1, dtype=torch.int32, device="cuda"),
                 ws=torch.empty(moe.sort_chunks_workspace_bytes(S * El) + 256, dtype=torch.uint8, device="cuda"))
        wl = {k: w[k][d * El:(d + 1) * El] for k in ("w_gate", "w_up", "w_down")}
        enames = ["gather_by_expert", "gate_up", "down", "gather_by_source"]
        def estep(ev=None):
            def mark(i):
                if ev is not None:
                    ev[i].record()
            mark(0)
            moe.sort_chunks(g["recv"], g["chunk"], g["by_expert"], S, g["grouped"], g["rows_e"], g["goff"], g["ws"])
            mark(1)
            moe.expert_gate_up(g["grouped"], g["goff"], wl["w_gate"], wl["w_up"], g["h"])
            mark(2)
            moe.expert_down(g["h"], g["goff"], wl["w_down"], g["y"])
            mark(3)
            moe.sort_chunks(g["y"], g["rows_e"], g["by_source"], 0, g["back"], None, None, g["ws"])
            mark(4)
        for _ in range(max(2, args.warmup)):
            estep()
        n_e = max(3, args.steps)
        eev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(n_e)]
        torch.cuda.synchronize()
        te0 = time.perf_counter()
        for i in range(n_e):
            estep(eev[i])
        torch.cuda.synchronize()
        ems = (time.perf_counter() - te0) * 1e3 / n_e
        est = {nm: round(sum(eev[i][j].elapsed_time(eev[i][j + 1]) for i in range(n_e)) / n_e, 4)
               for j, nm in enumerate(enames)}
        gbytes = 2.0 * Rr * H * es                      # every row read once and written once
        gms = 0.5 * (est["gather_by_expert"] + est["gather_by_source"])
        out["ep_share"] = {
            "ranks": S, "local_experts": El, "rank": d, "rows_received": Rr, "mean_rows_per_rank": round(float(loads.mean()) * S, 1),
            "chunks": S * El, "ms": round(ems, 4), "steps": n_e, "stage_ms": est,
            "gather": {"bytes": gbytes, "achieved": round(gbytes / (gms * 1e-3) / 1e9, 1), "unit": "GB/s",
                       "frac": round(gbytes / (gms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
            "gemm_tflops": round(6.0 * Rr * H * F / ((est["gate_up"] + est["down"]) * 1e-3) / 1e12, 1),
            "sample": "the most loaded rank of the group; every source sends the chunk sizes of this batch's routing; "
                      "payload N(0,1); the two All-to-All-Vs themselves are not run"}
    if args.dispatch_backward and not fp8:
        # dy plays the gradient of the layer output; the forward's y_perm, maps and gates are reused
        res = {}
        dgs = [torch.empty((T, K), dtype=torch.float32, device="cuda") for _ in sets]
        def cb(i):
            s = sets[i % NSETS]
            moe.unpermute_combine_backward(s["y"], s["y_perm"], s["roa"], s["gate"], s["x_perm"], dgs[i % NSETS])
        def pb(i):
            s = sets[i % NSETS]
            moe.permute_backward(s["x_perm"], s["roa"], None, s["y"], K)
        for nm, fn, work in (("combine_backward", cb, (T + 2 * R) * H * es + 12 * T * K),
                             ("permute_backward", pb, (R + T) * H * es + 4 * T * K)):
            for i in range(args.warmup):
                fn(i)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(args.steps):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            rate = work / (ms * 1e-3) / 1e9
            res[nm] = {"ms": round(ms, 4), "achieved": round(rate, 1), "unit": "GB/s", "frac": round(rate / PEAK_HBM_GBS, 4)}
        out["dispatch_backward"] = res
    if not args.no_cpu_baseline and not fp8:
        out["cpu_baseline"] = cpu_baseline(inp, capacity, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
