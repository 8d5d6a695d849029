#!/usr/bin/env python3
"""Benchmark of the block-masked cross-attention hot path on one MI355X.

One "step" = beagle_xattn_fwd + beagle_xattn_bwd (all projections, masked
attention, every gradient) on one synthetic batch of the named workload, with
all inputs resident in HBM.  Prints ONE JSON line.

  value        TFLOP/s counting only unmasked attention pairs plus the dense
               projection FLOPs (forward + backward): K steps between two
               synchronisations, nothing else on the stream (no event
               bracketing); `step_ms` gives median / min of per-step HIP events
               from a second loop; the per-kernel table comes from a third
               loop in which every launch is bracketed by events
  roofline     the kernel with the largest share of the step, its algorithmic
               FLOPs / its average duration (HIP events on the launch stream)
  other_workloads  the same step at the other two training configurations
  decode       the draft step at M in {1, 8, 32, 64} against L = 4096 cache
               rows, buffers rotated through > 1 GB so each call reads cold
               HBM; eager and HIP-graph replay; `roofline_decode` per M and
               `read_probe` (a kernel that only reads the same bytes)
  cpu_baseline the float64 oracle timed on the host cores on a bounded sample
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import re
import statistics
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_training_c2.md")


TRAINING_KERNEL_SOURCES = ("gemm_bf16.hip", "attn_fwd_bf16.hip", "attn_bwd_bf16.hip", "attn_tiles.h", "common.h",
                           "mask_index.h")


def kernel_source_digest():
    """sha256 over the sources the training step's kernels are compiled from: identifies the kernels a counter
    table was measured on."""
    h = hashlib.sha256()
    for f in TRAINING_KERNEL_SOURCES:
        h.update(f.encode())
        h.update(open(os.path.join(ROOT, "paper_2505_24544_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """HBM-side bytes per launch (fetched + written) from the tracked rocprofv3 --pmc summary, or (None, reason).
    Counters cannot be read from inside this process; the table names the kernel sources it was measured on and
    is ignored when they have changed since."""
    try:
        txt = open(TRAFFIC_TABLE).read()
    except OSError:
        return None, "no tracked counter table"
    m = re.search(r"traffic-table workload=(\S+) kernel-sources=(\S+)", txt)
    if not m or m.group(1) != workload:
        return None, "counter table is for another workload"
    if m.group(2) != kernel_source_digest():
        return None, "kernel sources changed since the counter table was measured (%s)" % m.group(2)
    tab = {}
    for name, f, w in re.findall(r"^\| (\w+) \| ([0-9.]+) \| ([0-9.]+) \|$", txt, re.M):
        tab[name] = (float(f) + float(w)) * 1e6
    return tab, "profiles/" + os.path.basename(TRAFFIC_TABLE) + " @ kernel sources " + m.group(2)


def flops_training(cfg, need_dxkv=True):
    """Algorithmic FLOPs of one forward+backward (unmasked pairs only)."""
    B, S, L, D = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden
    H, G, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    import numpy as np
    p = np.arange(S)
    t = p - cfg.block_offset
    ws = np.where(t < 0, 0, cfg.block_offset + (t // cfg.block_size) * cfg.block_size)
    pairs = int(np.minimum(ws, L).sum())
    proj = {
        "q": 2 * B * S * D * H * d, "k": 2 * B * L * D * G * d, "v": 2 * B * L * D * G * d,
        "o": 2 * B * S * H * d * D,
    }
    proj_fwd = sum(proj.values())
    proj_bwd = 2 * proj_fwd - (0 if need_dxkv else 2 * (2 * B * L * D * G * d))
    attn_fwd = 4 * d * pairs * B * H
    attn_bwd = 10 * d * pairs * B * H
    return dict(total=proj_fwd + proj_bwd + attn_fwd + attn_bwd, proj_fwd=proj_fwd, proj_bwd=proj_bwd,
                attn_fwd=attn_fwd, attn_bwd=attn_bwd, proj=proj, pairs=pairs)


def kernel_flops(cfg, fl, need_dxkv=True):
    """Algorithmic FLOPs per launch of each named kernel of the training step."""
    p = fl["proj"]
    return {
        "proj_qkv": p["q"] + p["k"] + p["v"], "proj_out": p["o"], "bwd_dout": p["o"], "bwd_dwo": p["o"],
        "bwd_dx": p["q"] + ((p["k"] + p["v"]) if need_dxkv else 0), "bwd_dw": p["q"] + p["k"] + p["v"],
        # grouped-query shapes whose three weight gradients would leave a half-empty last round: dWq alone, dWk and dWv as
        # halves of the contraction (+ a pass that adds the halves, bwd_dwkv_sum: no algorithmic FLOPs)
        "bwd_dwq": p["q"], "bwd_dwkv": p["k"] + p["v"],
        "attn_fwd_bf16": fl["attn_fwd"],
        # the backward's five contractions (10 d flops per visible pair): S, dP, dQ are credited to the dQ
        # kernel, dK and dV to the dK/dV kernel; the S and dP that the latter recomputes are not counted
        "attn_bwd_dq_bf16": 0.6 * fl["attn_bwd"], "attn_bwd_dkv_bf16": 0.4 * fl["attn_bwd"],
    }


class ClockSampler:
    """Shader clock and board power while the timed loops run, from the amdgpu sysfs files if this user may read
    them (freq1_input in Hz, power1_average / power1_input in microwatts); otherwise says why not."""

    def __init__(self):
        self.freq, self.power, self.note = [], [], None
        self._stop = threading.Event()
        self._thr = None
        hw = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*"))
        self.ffile = next((os.path.join(h, "freq1_input") for h in hw if os.path.exists(os.path.join(h, "freq1_input"))), None)
        self.pfile = next((os.path.join(h, n) for h in hw for n in ("power1_average", "power1_input")
                           if os.path.exists(os.path.join(h, n))), None)
        if not self.ffile and not self.pfile:
            self.note = "no readable amdgpu hwmon files under /sys/class/drm (clock and power not logged)"

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return float(f.read().strip())
        except (OSError, ValueError):
            return None

    def _run(self):
        while not self._stop.is_set():
            if self.ffile:
                v = self._read(self.ffile)
                if v:
                    self.freq.append(v / 1e6)
            if self.pfile:
                v = self._read(self.pfile)
                if v:
                    self.power.append(v / 1e6)
            time.sleep(0.005)

    def __enter__(self):
        if not self.note:
            self._thr = threading.Thread(target=self._run, daemon=True)
            self._thr.start()
        return self

    def __exit__(self, *a):
        self._stop.set()
        if self._thr:
            self._thr.join()

    def summary(self):
        if self.note:
            return {"note": self.note}
        out = {"samples": max(len(self.freq), len(self.power)), "source": "amdgpu hwmon sysfs, sampled every 5 ms during the timed loops"}
        if self.freq:
            out.update(sclk_mhz_median=round(statistics.median(self.freq)), sclk_mhz_min=round(min(self.freq)),
                       sclk_mhz_max=round(max(self.freq)))
        if self.power:
            out.update(power_w_median=round(statistics.median(self.power)), power_w_max=round(max(self.power)))
        if not self.freq and not self.power:
            out = {"note": "amdgpu hwmon files exist but returned nothing readable"}
        return out


def shader_clock_summary(samples):
    """Mean shader clock per step from consecutive clock samples [n + 1, slots, (cycle counter, 100 MHz clock)]:
    per step the median over the compute units whose slot was written by both samples."""
    import numpy as np
    mhz = []
    for s0, s1 in zip(samples[:-1], samples[1:]):
        both = (s0[:, 1] > 0) & (s1[:, 1] > s0[:, 1])
        if both.any():
            d = (s1[both] - s0[both]).astype(np.float64)
            mhz.append(float(np.median(d[:, 0] / d[:, 1])) * 100.0)
    ok = [m for m in mhz if 300.0 <= m <= 3000.0]
    if not ok:
        return dict(note="no plausible sample pair", raw_mhz=[round(m, 1) for m in mhz[:4]])
    return dict(source="beagle_xattn_probe_clock: per-compute-unit shader-cycle counter over the 100 MHz device clock, one sample per step",
                mhz_median=round(statistics.median(ok)), mhz_min=round(min(ok)), mhz_max=round(max(ok)),
                steps_used=len(ok), steps_dropped=len(samples) - 1 - len(ok), nominal_mhz=2400,
                bf16_mfma_peak_at_median_clock_tflops=round(PEAK_BF16_TFLOPS * statistics.median(ok) / 2400.0, 1))


def run_calib_copy(torch):
    """One plain 1 GiB device-to-device copy: what FETCH_SIZE / WRITE_SIZE read for a known size."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def train_leg(torch, bx, dm, synth, name, steps, warmup, profile=True, sampler=None, calib_copy=False):
    """fwd + bwd at one training configuration.  Returns (summary dict, device tensors for later legs)."""
    dev = "cuda:0"
    cfg = synth.CONFIGS[name]
    desc = dm.desc_of(cfg, bx.BEAGLE_FLAG_NEED_DXKV)
    inp = synth.make_inputs(cfg)
    t = {n: dm.to_dev(a, cfg) for n, a in inp.items()}
    del inp
    B, S, L, D, H, G, hd = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    bf = torch.bfloat16
    E = lambda *s, dt=bf: torch.empty(*s, dtype=dt, device=dev)
    y, lse = E(B, S, D), E(B, H, S, dt=torch.float32)
    q, k, v, o = E(B, S, H, hd), E(B, L, G, hd), E(B, L, G, hd), E(B, S, H, hd)
    dxq, dxkv = E(B, S, D), E(B, L, D)
    dwq, dwk, dwv, dwo = E(D, H * hd), E(D, G * hd), E(D, G * hd), E(H * hd, D)
    ws_f = dm.workspace(desc, bx.BEAGLE_WS_FWD)
    ws_b = dm.workspace(desc, bx.BEAGLE_WS_BWD)
    stream = torch.cuda.current_stream()

    def step():
        bx.beagle_xattn_fwd(desc, t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"], y, lse, q, k, v, o,
                            ws_f, stream)
        bx.beagle_xattn_bwd(desc, t["dy"], t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"], q, k, v, o, lse,
                            dxq, dxkv, dwq, dwk, dwv, dwo, ws_b, stream)

    if calib_copy:
        run_calib_copy(torch)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ctx = sampler if sampler is not None else _Null()
    with ctx:
        # (1) the judged number: exactly `steps` steps between two synchronisations, nothing else enqueued
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # (2) the same loop with one event pair per step: spread of the step time
        # and one sample of the shader-cycle counter against the 100 MHz device clock after every step
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        clk = torch.zeros(steps + 1, bx.BEAGLE_CLOCK_SLOTS, 2, dtype=torch.int64, device=dev)
        bx.beagle_xattn_probe_clock(clk[0], stream)
        for i, (a, b) in enumerate(ev):
            a.record()
            step()
            b.record()
            bx.beagle_xattn_probe_clock(clk[i + 1], stream)
        torch.cuda.synchronize()
        per_step = [a.elapsed_time(b) for a, b in ev]
        shader_clock = shader_clock_summary(clk.cpu().numpy())
        # (3) every launch bracketed by events: the per-kernel table
        prof = {}
        if profile:
            bx.beagle_xattn_profile_begin()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            prof = bx.beagle_xattn_profile_end()
    ms_step = dt / steps * 1e3
    fl = flops_training(cfg, True)
    tflops = fl["total"] / (ms_step * 1e-3) / 1e12
    kf = kernel_flops(cfg, fl, True)
    kernels, roofline = {}, None
    for kn, (cnt, ms) in prof.items():
        avg = ms / cnt
        kernels[kn] = dict(avg_ms=round(avg, 4), launches_per_step=cnt / steps,
                           tflops=round(kf[kn] / (avg * 1e-3) / 1e12, 1) if kn in kf else None)
    if prof:
        dom = max(prof, key=lambda n: prof[n][1])
        avg = prof[dom][1] / prof[dom][0]
        ach = kf.get(dom, 0) / (avg * 1e-3) / 1e12
        tab, src = measured_traffic(cfg.name)
        roofline = dict(bound="mfma", kernel=dom, achieved=round(ach, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=round(ach / PEAK_BF16_TFLOPS, 4), traffic=(tab or {}).get(dom), traffic_measured_at=src,
                        avg_ms=round(avg, 4), flops_per_launch=kf.get(dom))
    summ = dict(workload="%s: B%d S%d D%d H%d/G%d d%d k%d bf16 fwd+bwd (dXkv included)" % (
                    cfg.name, B, S, D, H, G, hd, cfg.block_size),
                ms_per_step=round(ms_step, 4), tflops=round(tflops, 2),
                pct_bf16_mfma_peak=round(100 * tflops / PEAK_BF16_TFLOPS, 2), tokens_per_s=round(B * S / (ms_step * 1e-3)),
                step_ms=dict(mean_wall=round(ms_step, 4), median=round(statistics.median(per_step), 4),
                             min=round(min(per_step), 4), max=round(max(per_step), 4), n=steps),
                shader_clock=shader_clock,
                algorithmic_tflop_per_step=round(fl["total"] / 1e12, 4), roofline=roofline, kernels=kernels)
    keep = dict(cfg=cfg, desc=desc, t=t, fl=fl, y=y, lse=lse, q=q, k=k, v=v, o=o, dxq=dxq, dxkv=dxkv, dwq=dwq, dwk=dwk,
                dwv=dwv, dwo=dwo, ws_f=ws_f, E=E)
    return summ, keep


class _Skip(Exception):
    pass


class _Null:
    def __enter__(self):
        return self

    def __exit__(self, *a):
        return False


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c5"])
    ap.add_argument("--only", default="all", choices=["all", "train", "decode"],
                    help="train: the headline loop only; decode: the draft-step leg only (for profiler runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode, simulation-step and draft-block legs")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (calibrates FETCH_SIZE / WRITE_SIZE under rocprofv3)")
    ap.add_argument("--no-graph", action="store_true",
                    help="decode leg: skip the HIP-graph replays (for counter runs, which look at single dispatches)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_24544_amd import binding as bx, devmem as dm, synth

    bx.lib()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    full = args.only == "all"

    if args.only == "decode":
        if args.calib_copy:
            run_calib_copy(torch)
        print(json.dumps({"decode": bench_decode(torch, bx, dm, synth, not args.no_graph)}))
        return

    sampler = ClockSampler()
    head, keep = train_leg(torch, bx, dm, synth, args.workload, args.steps, args.warmup, not args.no_profile, sampler,
                           args.calib_copy)
    cfg, fl = keep["cfg"], keep["fl"]

    sim = block = decode = None
    if full and not args.no_decode:
        sim = bench_sim(torch, bx, dm, keep, max(1, args.steps // 2))
        block = bench_block(torch, bx, dm, cfg, keep["t"], fl, max(1, args.steps // 2))
    del keep
    torch.cuda.empty_cache()

    # ---- the other two training configurations, compact
    others = {}
    if full:
        for name in ("c2", "c3", "c5"):
            if name == args.workload:
                continue
            s, kp = train_leg(torch, bx, dm, synth, name, max(4, args.steps // 2), 3, not args.no_profile)
            del kp
            torch.cuda.empty_cache()
            others[name] = dict(workload=s["workload"], ms_per_step=s["ms_per_step"], tflops=s["tflops"],
                                pct_bf16_mfma_peak=s["pct_bf16_mfma_peak"], tokens_per_s=s["tokens_per_s"],
                                step_ms=s["step_ms"], shader_clock_mhz=(s["shader_clock"] or {}).get("mhz_median"),
                                algorithmic_tflop_per_step=s["algorithmic_tflop_per_step"],
                                roofline=s["roofline"],
                                kernel_avg_ms={n: k["avg_ms"] for n, k in s["kernels"].items()})

    if full and not args.no_decode:
        decode = bench_decode(torch, bx, dm, synth, not args.no_graph)

    cpu = cpu_other = None
    if full and not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, synth)
        cpu_other = cpu_baseline_other(synth, args.workload)

    out = {
        "metric": "masked xattn fwd+bwd TFLOP/s (% bf16 MFMA peak); draft-step us (% HBM BW)",
        "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": head["workload"]},
        "pct_bf16_mfma_peak": head["pct_bf16_mfma_peak"],
        "tokens_per_s": head["tokens_per_s"],
        "algorithmic_tflop_per_step": head["algorithmic_tflop_per_step"],
        "step_ms": head["step_ms"], "clock": dict(sampler.summary(), shader_clock=head["shader_clock"]),
        "roofline": head["roofline"],
        "roofline_decode": (decode or {}).get("roofline_decode"),
        "cpu_baseline": cpu,
        "kernels": head["kernels"], "other_workloads": others or None, "late_stage_sim": sim, "draft_block": block,
        "decode": decode, "cpu_baseline_other": cpu_other,
    }
    print(json.dumps(out))


def bench_sim(torch, bx, dm, keep, nsim):
    """Late-stage simulation step (true keys + the predicted-state band), same workload, step t = 3."""
    cfg, desc, t, fl, E = keep["cfg"], keep["desc"], keep["t"], keep["fl"], keep["E"]
    B, S, L, D, H, G, hd = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    y, lse, q, k, v, o = (keep[n] for n in ("y", "lse", "q", "k", "v", "o"))
    dxq, dxkv, dwq, dwk, dwv, dwo = (keep[n] for n in ("dxq", "dxkv", "dwq", "dwk", "dwv", "dwo"))
    stream = torch.cuda.current_stream()
    tsim = min(3, cfg.block_size - 1)
    xp = t["xkv"].flip(1).contiguous()             # any states of the right shape: time is value-independent
    kp, vp, dxp = E(B, L, G, hd), E(B, L, G, hd), E(B, L, D)
    ws_s = dm.workspace(desc, bx.BEAGLE_WS_BWD_SIM)

    def sim_step():
        bx.beagle_xattn_fwd_sim(desc, t["xq"], t["xkv"], xp, t["wq"], t["wk"], t["wv"], t["wo"], tsim, y, lse,
                                q, k, v, kp, vp, o, keep["ws_f"], stream)
        # the in-place save of the newly predicted rows (y stands in for the draft block's output); the rows
        # it overwrites are invisible at this step, so the backward below is unaffected
        bx.beagle_xattn_sim_save(desc, y, xp, tsim, stream)
        bx.beagle_xattn_bwd_sim(desc, t["dy"], t["xq"], t["xkv"], xp, t["wq"], t["wk"], t["wv"], t["wo"], q, k, v,
                                kp, vp, o, lse, tsim, dxq, dxkv, dxp, dwq, dwk, dwv, dwo, ws_s, stream)
    for _ in range(3):
        sim_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(nsim):
        sim_step()
    torch.cuda.synchronize()
    ms_sim = (time.perf_counter() - t0) / nsim * 1e3
    # algorithmic FLOPs: the early-stage step + the projections of the predicted states (forward K, V;
    # backward dXpred and their share of dWk, dWv) + the band (4 d forward, 10 d backward per visible pair)
    band_pairs = B * H * sum(min(i, tsim) for i in range(cfg.block_size)) * (S // cfg.block_size)
    fl_sim = fl["total"] + 3 * (fl["proj"]["k"] + fl["proj"]["v"]) + 14 * hd * band_pairs
    return dict(sim_step=tsim, ms_per_step=round(ms_sim, 4), tflops=round(fl_sim / (ms_sim * 1e-3) / 1e12, 1),
                pct_bf16_mfma_peak=round(100 * fl_sim / (ms_sim * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
                algorithmic_tflop_per_step=round(fl_sim / 1e12, 4))


def bench_block(torch, bx, dm, cfg, t, fl, nsteps):
    """Forward + backward of the whole draft block (section 4.1, Eq. 1) at the training workload's shapes with the
    feed-forward width of the matching LLaMA model; random weights (time is value-independent)."""
    dev = "cuda:0"
    B, S, L, D, H, G, hd = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    F = {4096: 11008, 5120: 13824}.get(D, (8 * D // 3 + 63) // 64 * 64)
    if G != H and D == 4096:
        F = 14336                                       # the GQA 8B shape
    bf, f32 = torch.bfloat16, torch.float32
    g = torch.Generator(device=dev).manual_seed(11)
    R = lambda *s, std=0.02: (torch.randn(*s, device=dev, generator=g) * std).to(bf)
    E = lambda *s, dt=bf: torch.empty(*s, dtype=dt, device=dev)
    desc = dm.desc_of(cfg, bx.BEAGLE_FLAG_NEED_DXKV)
    W = dict(wq=t["wq"], wk=t["wk"], wv=t["wv"], wo=t["wo"], w_gate=R(D, F), w_up=R(D, F), w_down=R(F, D),
             g_q=R(D, std=0.1) + 1, g_kv=R(D, std=0.1) + 1, g_mlp=R(D, std=0.1) + 1)
    e, hs, dh = R(B, S, D), R(B, L, D, std=3.0), R(B, S, D, std=1.0)
    sv = dict(xq_n=E(B, S, D), r_q=E(B * S, dt=f32), xkv_n=E(B, L, D), r_kv=E(B * L, dt=f32), q=E(B, S, H, hd),
              k=E(B, L, G, hd), v=E(B, L, G, hd), o=E(B, S, H, hd), lse=E(B, H, S, dt=f32), y=E(B, S, D), z=E(B, S, D),
              r_mlp=E(B * S, dt=f32), u=E(B, S, F), w=E(B, S, F), m=E(B, S, F))
    gr = dict(de=E(B, S, D), dhs=E(B, L, D), dwq=E(D, H * hd), dwk=E(D, G * hd), dwv=E(D, G * hd), dwo=E(H * hd, D),
              dw_gate=E(D, F), dw_up=E(D, F), dw_down=E(F, D), dg_q=E(D, dt=f32), dg_kv=E(D, dt=f32), dg_mlp=E(D, dt=f32))
    h = E(B, S, D)
    params, saved, grads = bx.make_block_params(F, 1e-5, **W), bx.make_block_saved(**sv), bx.make_block_grads(**gr)
    ws = torch.empty(bx.beagle_xattn_block_workspace_bytes(desc, F, bx.BEAGLE_WS_BLOCK_BWD), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        bx.beagle_xattn_block_fwd(desc, params, e, hs, h, saved, None, stream)
        bx.beagle_xattn_block_bwd(desc, params, dh, e, hs, saved, grads, ws, stream)
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(nsteps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / nsteps * 1e3
    bx.beagle_xattn_profile_begin()
    for _ in range(nsteps):
        step()
    torch.cuda.synchronize()
    prof = bx.beagle_xattn_profile_end()
    # the attention op's FLOPs + the feed-forward's three GEMMs forward and six backward (2 M D F each)
    fl_blk = fl["total"] + 18 * B * S * D * F
    # bytes the streaming kernels must move at least (bf16): norm fwd r+w, norm bwd 3r+w, gate fwd 2r+w, bwd 3r+2w
    MD, MF = B * S * D * 2, B * S * F * 2
    stream_bytes = {"norm_q": 2 * MD, "norm_kv": 2 * B * L * D * 2, "norm_mlp": 2 * MD, "mlp_gate": 3 * MF,
                    "bwd_mlp_gate": 5 * MF, "bwd_norm_mlp": 4 * MD, "bwd_norm_q": 4 * MD, "bwd_norm_kv": 3 * B * L * D * 2}
    kern = {}
    for n, (c, tot) in prof.items():
        kern[n] = dict(avg_ms=round(tot / c, 4))
        if n in stream_bytes:
            kern[n]["gbs"] = round(stream_bytes[n] / (tot / c * 1e-3) / 1e9, 1)
    return dict(ffn=F, ms_per_step=round(ms, 4), tflops=round(fl_blk / (ms * 1e-3) / 1e12, 1),
                pct_bf16_mfma_peak=round(100 * fl_blk / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
                algorithmic_tflop_per_step=round(fl_blk / 1e12, 4), tokens_per_s=round(B * S / (ms * 1e-3)), kernels=kern)


def _time_calls(torch, fn, n_sets, reps, spread=None):
    """Average microseconds per call of fn(r), r cycling through the buffer sets, by HIP events on the stream:
    n_sets warm-up calls, then `reps` timed ones.  An event is also recorded after every n_sets calls; with `spread`
    (a dict) the per-call averages of those groups go into it as median / min / max."""
    for r in range(n_sets):
        fn(r)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True)]
    marks[0].record()
    for r in range(reps):
        fn(r)
        if (r + 1) % n_sets == 0 or r + 1 == reps:
            marks.append(torch.cuda.Event(enable_timing=True))
            marks[-1].record()
    torch.cuda.synchronize()
    if spread is not None:
        sizes = [n_sets] * (reps // n_sets) + ([reps % n_sets] if reps % n_sets else [])
        per = [a.elapsed_time(b) / n * 1e3 for a, b, n in zip(marks[:-1], marks[1:], sizes)]
        spread.update(groups=len(per), calls_per_group=n_sets, median=round(statistics.median(per), 2),
                      min=round(min(per), 2), max=round(max(per), 2))
    return marks[0].elapsed_time(marks[-1]) / reps * 1e3


def bench_decode(torch, bx, dm, synth, graphs=True):
    """Draft step at the decode config (L=4096, D=4096, H=32, d=128): random bf16 cache rows and weights of those
    shapes (time is value-independent), ten buffer sets so that every call reads cold HBM."""
    cfg = synth.CONFIGS["c4"]
    dev = "cuda:0"
    L, D, H, G, hd = cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    nset = 10                      # 10 x 134 MB > 1 GB: defeats the 256 MB Infinity Cache
    g = torch.Generator(device=dev).manual_seed(4)
    # one allocation per kind so that the read probe can walk the same bytes: [K | V | Wq | Wo] per set
    per = L * G * hd
    slab = torch.empty(nset, 4, per, dtype=torch.bfloat16, device=dev)
    assert D * H * hd == per, "the decode config has square projections"
    sets = []
    for i in range(nset):
        slab[i, 0].copy_((torch.randn(per, device=dev, generator=g) * 1.28).to(torch.bfloat16))
        slab[i, 1].copy_((torch.randn(per, device=dev, generator=g) * 1.28).to(torch.bfloat16))
        slab[i, 2].copy_((torch.randn(per, device=dev, generator=g) * 0.02).to(torch.bfloat16))
        slab[i, 3].copy_((torch.randn(per, device=dev, generator=g) * 0.02).to(torch.bfloat16))
        sets.append((slab[i, 0].view(L, G, hd), slab[i, 1].view(L, G, hd), slab[i, 2].view(D, H * hd),
                     slab[i, 3].view(H * hd, D)))
    # the two projections once more in the decode-time layout (packed once per model load):
    # the same bytes per call, streamed from these buffers instead
    wq_pk = torch.empty(nset, D * H * hd, dtype=torch.bfloat16, device=dev)
    wo_pk = torch.empty(nset, D * H * hd, dtype=torch.bfloat16, device=dev)
    for i in range(nset):
        bx.beagle_xattn_prepare_weights(dm.desc_of(cfg.with_(seq_q=1)), wq=sets[i][2], wo=sets[i][3], wq_pk=wq_pk[i], wo_pk=wo_pk[i])
    res, roof = {}, {}
    stream = torch.cuda.current_stream()

    # ---- what a kernel that only reads gets out of the memory system, on the same (cold) bytes
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    set_bytes = 4 * per * 2
    probe = {}
    for label, off, nb in (("whole_step_134MB", 0, set_bytes), ("kv_cache_67MB", 0, 2 * per * 2),
                           ("one_weight_matrix_34MB", 2 * per * 2, per * 2)):
        us = _time_calls(torch, lambda r: bx.beagle_xattn_probe_read(slab[r % nset].data_ptr() + off, nb, 512, sink, stream),
                         nset, 50)
        probe[label] = dict(bytes=nb, us=round(us, 2), gbs=round(nb / us / 1e3, 1),
                            pct_hbm_peak=round(100 * nb / us / 1e3 / PEAK_HBM_GBS, 2))
    probe["three_separate_reads_us"] = round(probe["kv_cache_67MB"]["us"] + 2 * probe["one_weight_matrix_34MB"]["us"], 2)
    probe["note"] = ("beagle_xattn_probe_read, 512 workgroups, 16-byte loads, nothing else: the ceiling for one kernel "
                     "streaming the step's bytes, and for three kernels streaming them one after the other")
    res["read_probe"] = probe

    for M in (1, 8, 32, 64):
        c = cfg.with_(seq_q=M)
        desc = dm.desc_of(c)
        x = torch.randn(M, D, device=dev, generator=g)
        x = (x / x.pow(2).mean(-1, keepdim=True).add(1e-5).sqrt()).to(torch.bfloat16)
        y = torch.empty(M, D, dtype=torch.bfloat16, device=dev)
        lse = torch.empty(H, M, dtype=torch.float32, device=dev)
        ws = dm.workspace(desc, bx.BEAGLE_WS_DRAFT)
        call = lambda r, st=stream: bx.beagle_xattn_draft_step(desc, x, *sets[r % nset], y, lse, ws, st)
        spread = {}
        us = _time_calls(torch, call, nset, 50, spread)
        prep_us = None
        if M <= bx.BEAGLE_PREPARED_MAX_QUERIES:
            prep = lambda r: bx.beagle_xattn_draft_step_prepared(desc, x, sets[r % nset][0], sets[r % nset][1],
                                                                 wq_pk[r % nset], wo_pk[r % nset], L, None, 0, y, lse, ws, stream)
            prep_us = _time_calls(torch, prep, nset, 50)
        # the same fifty calls as five replays of a HIP graph that holds one call per buffer set
        graph_us = None
        try:
            if not graphs:
                raise _Skip()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                cs = torch.cuda.current_stream()
                for r in range(nset):
                    call(r, cs)
            gr.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                gr.replay()
            e1.record()
            torch.cuda.synchronize()
            graph_us = e0.elapsed_time(e1) / (5 * nset) * 1e3
            del gr
        except _Skip:
            pass
        except Exception as ex:        # reported, not hidden: the eager figure stands
            graph_us = None
            res.setdefault("graph_errors", []).append("M%d: %r" % (M, ex))
        # second pass with every kernel bracketed by events (adds gaps; used for the breakdown only)
        bx.beagle_xattn_profile_begin()
        for r in range(50):
            call(r)
        torch.cuda.synchronize()
        prof = bx.beagle_xattn_profile_end()
        core_bytes = 2 * L * G * hd * 2 + 2 * M * H * hd * 2
        call_bytes = core_bytes + 2 * D * H * hd * 2
        kern = {n: round(ms / cnt * 1e3, 2) for n, (cnt, ms) in prof.items()}
        best = min(us, graph_us) if graph_us else us
        res["M%d" % M] = dict(us_per_call=round(us, 2), graph_us_per_call=round(graph_us, 2) if graph_us else None,
                              gbs=round(call_bytes / us / 1e3, 1),
                              pct_hbm_peak=round(100 * call_bytes / us / 1e3 / PEAK_HBM_GBS, 2),
                              us_per_call_groups=spread,
                              draft_tokens_per_s=round(M / (us * 1e-6)), bytes=call_bytes,
                              kernel_us_bracketed=kern)
        if prep_us:
            res["M%d" % M]["packed_weights"] = dict(us_per_call=round(prep_us, 2), gbs=round(call_bytes / prep_us / 1e3, 1),
                                                 pct_hbm_peak=round(100 * call_bytes / prep_us / 1e3 / PEAK_HBM_GBS, 2))
        att = kern.get("draft_attn")
        roof["M%d" % M] = dict(
            bound="hbm", kernel="beagle_xattn_draft_step (whole call: projections, attention, merges)",
            bytes=call_bytes, avg_us=round(us, 2), median_us=spread.get("median"), min_us=spread.get("min"), achieved=round(call_bytes / us / 1e3, 1), peak=PEAK_HBM_GBS,
            unit="GB/s", frac=round(call_bytes / us / 1e3 / PEAK_HBM_GBS, 4),
            graph_replay=dict(avg_us=round(graph_us, 2), frac=round(call_bytes / graph_us / 1e3 / PEAK_HBM_GBS, 4)) if graph_us else None,
            packed_weights=dict(entry="beagle_xattn_draft_step_prepared (wq, wo packed once per model load; same bytes per call)",
                             avg_us=round(prep_us, 2), achieved=round(call_bytes / prep_us / 1e3, 1),
                             frac=round(call_bytes / prep_us / 1e3 / PEAK_HBM_GBS, 4)) if prep_us else None,
            frac_of_read_probe=round(probe["whole_step_134MB"]["us"] / min(best, prep_us or best), 4),
            attention_core=dict(kernel="decode_attn_kernel", bytes=core_bytes, avg_us_bracketed=att,
                                frac_bracketed=round(core_bytes / att / 1e3 / PEAK_HBM_GBS, 4) if att else None,
                                note="event-bracketed (includes the bracket's own gaps); the kernel-trace duration is in profiles/"))
    res["roofline_decode"] = roof

    # ---- the same step with drafted states in the cache under a draft tree (50 drafted rows: five finished
    # depths of top-k 10; the 10 queries of the next depth), and appending 10 drafted states to the cache
    import numpy as np
    M, T = 10, 50
    rng = np.random.default_rng(5)
    tm = np.zeros((M, 2), np.uint32)
    for m in range(M):
        for dpt in range(5):                       # one ancestor per finished depth
            t = 10 * dpt + int(rng.integers(0, 10))
            tm[m, t // 32] |= np.uint32(1) << np.uint32(t % 32)
    tmd = torch.from_numpy(tm.view(np.int32)).to(dev)
    c = cfg.with_(seq_q=M, seq_kv=L)
    desc = dm.desc_of(c)
    x = torch.randn(M, D, device=dev, generator=g).to(torch.bfloat16)
    y = torch.empty(M, D, dtype=torch.bfloat16, device=dev)
    lse = torch.empty(H, M, dtype=torch.float32, device=dev)
    ws = dm.workspace(desc, bx.BEAGLE_WS_DRAFT)
    wk = (torch.randn(D, G * hd, device=dev, generator=g) * 0.02).to(torch.bfloat16)
    wv = (torch.randn(D, G * hd, device=dev, generator=g) * 0.02).to(torch.bfloat16)
    adesc = dm.desc_of(cfg.with_(seq_q=M, seq_kv=L))
    aws = dm.workspace(adesc, bx.BEAGLE_WS_APPEND)

    def tree_call(r):
        kc, vc, wq, wo = sets[r % nset]
        bx.beagle_xattn_draft_step_tree(desc, x, kc, vc, wq, wo, L - T, tmd, 2, y, lse, ws, stream)

    def tree_prepared_call(r):
        kc, vc, _, _ = sets[r % nset]
        bx.beagle_xattn_draft_step_prepared(desc, x, kc, vc, wq_pk[r % nset], wo_pk[r % nset], L - T, tmd, 2, y, lse, ws, stream)

    def append_call(r):
        kc, vc, _, _ = sets[r % nset]
        bx.beagle_xattn_kv_append(adesc, x, wk, wv, kc, vc, L - T, aws, stream)

    wk_pk, wv_pk = torch.empty_like(wk).view(-1), torch.empty_like(wv).view(-1)
    bx.beagle_xattn_prepare_weights(adesc, wk=wk, wv=wv, wk_pk=wk_pk, wv_pk=wv_pk)

    def append_packed_call(r):
        kc, vc, _, _ = sets[r % nset]
        bx.beagle_xattn_kv_append_prepared(adesc, x, wk_pk, wv_pk, kc, vc, L - T, stream)

    # the whole draft block per draft step (Eq. 1): the tree step above + RMSNorm, residuals and the feed-forward
    # layer of the 7B shape; its three matrices rotate through four sets (1.1 GB) like the rest
    F = 11008
    R = lambda *sh, std=0.02: (torch.randn(*sh, device=dev, generator=g) * std).to(torch.bfloat16)
    mlps = [(R(D, F), R(D, F), R(F, D)) for _ in range(4)]
    gq, gm = R(D, std=0.1) + 1, R(D, std=0.1) + 1
    hb = torch.empty(M, D, dtype=torch.bfloat16, device=dev)
    bws = torch.empty(bx.beagle_xattn_block_workspace_bytes(desc, F, bx.BEAGLE_WS_BLOCK_DRAFT), dtype=torch.uint8, device=dev)

    def block_call(r):
        kc, vc, wq, wo = sets[r % nset]
        wg, wu, wd = mlps[r % 4]
        prm = bx.make_block_params(F, 1e-5, wq=wq, wo=wo, w_gate=wg, w_up=wu, w_down=wd, g_q=gq, g_mlp=gm)
        bx.beagle_xattn_block_draft_step(desc, prm, x, kc, vc, L - T, tmd, 2, hb, lse, bws, stream)

    # ... and with all four streamed matrices in the decode-time layout (packed once per model load)
    mlps_t = []
    for i, (wg, wu, wd) in enumerate(mlps):
        tw = dict(wq_pk=wq_pk[i], wo_pk=wo_pk[i], w_gate_pk=torch.empty(D * F, dtype=torch.bfloat16, device=dev),
                  w_up_pk=torch.empty(D * F, dtype=torch.bfloat16, device=dev), w_down_pk=torch.empty(F * D, dtype=torch.bfloat16, device=dev))
        prm = bx.make_block_params(F, 1e-5, wq=sets[i][2], wo=sets[i][3], w_gate=wg, w_up=wu, w_down=wd, g_q=gq, g_mlp=gm)
        bx.beagle_xattn_block_prepare_weights(desc, prm, bx.make_block_decode_weights(**tw))
        mlps_t.append(tw)

    def block_prepared_call(r):
        kc, vc, _, _ = sets[r % nset]
        tw = dict(mlps_t[r % 4], wq_pk=wq_pk[r % nset], wo_pk=wo_pk[r % nset])
        prm = bx.make_block_params(F, 1e-5, g_q=gq, g_mlp=gm)
        bx.beagle_xattn_block_draft_step_prepared(desc, prm, bx.make_block_decode_weights(**tw), x, kc, vc, L - T, tmd, 2,
                                                  hb, lse, bws, stream)

    for name, fn in (("tree_M10_T50", tree_call), ("tree_M10_T50_packed_weights", tree_prepared_call),
                     ("kv_append_n10", append_call), ("kv_append_n10_packed_weights", append_packed_call),
                     ("block_M10_T50_F11008", block_call),
                     ("block_M10_T50_F11008_prepared", block_prepared_call)):
        us = _time_calls(torch, fn, nset, 50)
        if name.startswith("tree"):
            nbytes = 2 * L * G * hd * 2 + 2 * M * H * hd * 2 + 2 * D * H * hd * 2
        elif name.startswith("block"):
            nbytes = 2 * L * G * hd * 2 + 2 * M * H * hd * 2 + 2 * D * H * hd * 2 + 3 * D * F * 2 + 2 * M * D * 2
        else:
            nbytes = 2 * D * G * hd * 2 + M * D * 2 + 2 * M * G * hd * 2
        res[name] = dict(us_per_call=round(us, 2), gbs=round(nbytes / us / 1e3, 1),
                         pct_hbm_peak=round(100 * nbytes / us / 1e3 / PEAK_HBM_GBS, 2), bytes=nbytes)
    return res


def _host_cores():
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count()


def cpu_baseline(cfg, synth):
    """The float64 oracle, as it stands, on the host cores: forward+backward on
    every sequence of the workload's batch, one at a time, each cut to its
    first 2048 positions (all heads, full width).  For c2 that is the whole
    workload: about 12 s on the GPU machine's 16 host cores."""
    from oracle import beagle_oracle as orc
    S = min(2048, cfg.seq_q)
    c = cfg.with_(batch=1, seq_q=S, seq_kv=S)
    mask = orc.dense_mask(S, S, c.block_size, c.block_offset)
    dt = 0.0
    for b in range(cfg.batch):
        inp = synth.make_inputs(c.with_(seed_base=c.seed_base + 1000 * b))
        t0 = time.perf_counter()
        orc.xattn_backward(inp["dy"], inp["xq"], inp["xkv"], inp["wq"], inp["wk"], inp["wv"], inp["wo"],
                           n_q_heads=c.n_q_heads, n_kv_heads=c.n_kv_heads, mask=mask)
        dt += time.perf_counter() - t0
    fl = flops_training(c, True)["total"] * cfg.batch
    return dict(value=round(fl / dt / 1e12, 5), unit="TFLOP/s", cores=_host_cores(), kind="oracle",
                seconds=round(dt, 2), tokens_per_s=round(cfg.batch * S / dt, 1),
                sample="%s shape, %d sequence(s) one at a time, first %d positions each, float64 NumPy, "
                       "fwd+bwd incl. dXkv" % (c.name, cfg.batch, S))


def cpu_baseline_other(synth, headline):
    """The oracle on the remaining configurations, each on a bounded sample (one sequence cut to its first 2048
    positions; the tiny fp32 problem whole, with all host threads and with one)."""
    from oracle import beagle_oracle as orc
    out = {}

    def run(c):
        inp = synth.make_inputs(c)
        mask = orc.dense_mask(c.seq_q, c.seq_kv, c.block_size, c.block_offset)
        t0 = time.perf_counter()
        orc.xattn_backward(inp["dy"], inp["xq"], inp["xkv"], inp["wq"], inp["wk"], inp["wv"], inp["wo"],
                           n_q_heads=c.n_q_heads, n_kv_heads=c.n_kv_heads, mask=mask)
        return time.perf_counter() - t0

    c1 = synth.CONFIGS["c1"]
    run(c1)                                           # first call: imports, thread pool start-up
    dt = run(c1)
    fl = flops_training(c1, True)["total"]
    out["c1"] = dict(seconds=round(dt, 4), gflops=round(fl / dt / 1e9, 2), cores=_host_cores(), sample="whole problem, fwd+bwd")
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            dt1 = run(c1)
        out["c1_one_thread"] = dict(seconds=round(dt1, 4), gflops=round(fl / dt1 / 1e9, 2), cores=1, sample="whole problem, fwd+bwd")
    except Exception as ex:
        out["c1_one_thread"] = dict(note="threadpoolctl unavailable: %r" % (ex,))
    for name in ("c2", "c3", "c5"):
        if name == headline:
            continue
        cfg = synth.CONFIGS[name]
        S = min(2048, cfg.seq_q)
        c = cfg.with_(batch=1, seq_q=S, seq_kv=S)
        dt = run(c)
        fl = flops_training(c, True)["total"]
        out[name] = dict(seconds=round(dt, 2), tflops=round(fl / dt / 1e12, 5), cores=_host_cores(),
                         tokens_per_s=round(S / dt, 1),
                         sample="%s shape, one sequence cut to its first %d positions, fwd+bwd incl. dXkv" % (name, S))
    return out


if __name__ == "__main__":
    main()
