#!/usr/bin/env python3
"""Benchmark of the LoRDO hot path on one MI355X.

A "step" is one local step over every matrix of the workload (down-projection, fused low-rank
Adam, up-projection with the weight update), plus, at the workload's cadence, the outer step on
a generated averaged pseudo-gradient (every `outer_every` steps) and the subspace refresh with
moment rotation (every `refresh_every` steps).  With the default K = 200 steps on workload c2 the
timed region holds exactly one refresh and six outer steps.  Inputs are synthetic, seeded and
resident in HBM before the timed region starts.

Prints ONE JSON line: the whole-path time per step, the roofline of the dominant kernel (event-
timed through the library's profiling hooks on the stream the kernels run on) and the float64
oracle timed on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix peak

WORKLOAD_TEXT = {
    "c1": "c1: single 256x256 fp32 matrix, r=16",
    "c2": "c2: ~125M transformer set, 12 layers x {4 of 768x768, 768x3072, 3072x768}, r=128, bf16 grads, fp32 weights and moments",
    "c3": "c3: ~1B set, 24 layers x {4 of 2048x2048, 2 of 2048x5632, 5632x2048}, r=256, bf16 Student-t grads",
    "c4": "c4: ~7B set, 32 layers x {4 of 4096x4096, 2 of 4096x11008, 11008x4096}, r=512, bf16 grads",
    "c5": "c5: single 8192x28672 bf16 matrix",
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c2")
    ap.add_argument("--rank", type=int, default=None)
    ap.add_argument("--grad-sets", type=int, default=None, help="distinct gradient sets cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="skip the event-timed second pass")
    ap.add_argument("--refresh-every", type=int, default=None)
    ap.add_argument("--outer-every", type=int, default=None)
    ap.add_argument("--rayleigh-ritz", action="store_true",
                    help="end every refresh with the Rayleigh-Ritz step (basis ordered as singular vectors; ranks up to 1024)")
    ap.add_argument("--update", default="plain", choices=["plain", "low-qhm", "full-qhm", "ef", "global", "local", "uplink"],
                    help="update case of the local step: plain (default, the headline), low-rank / full-rank QHM (omega 0.9), "
                         "error feedback, global = full-rank QHM + error feedback (the paper's LoRDO-Global), local = low-rank QHM + error "
                         "feedback with the refresh of Alg. 2, uplink = plain with the r x q up-link buffer and the outer step fed from it")
    ap.add_argument("--short-side", action="store_true",
                    help="project every matrix with more rows than columns on the right (shape field side = 1); "
                         "update cases plain and low-qhm")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run plain 1 GiB device copies (known traffic) to scale the FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


KERNEL_OF_CLASS = {"down": "k_proj_down", "adam": "k_adam", "up": "k_proj_up", "outer": "k_pq<0>"}


def measured_traffic(cfg, rank, kernel_class, update="plain"):
    """HBM bytes per launch of a kernel class from the committed rocprofv3 counter summary of this
    workload (FETCH_SIZE and WRITE_SIZE runs, scaled by a plain copy), or None if there is none."""
    if rank is not None or update != "plain":
        return None
    path = os.path.join(ROOT, "profiles", f"{cfg}_hbm_traffic_pmc.txt")
    prefix = KERNEL_OF_CLASS.get(kernel_class)
    if prefix is None or not os.path.exists(path):
        return None
    best = None
    with open(path) as f:
        for line in f:
            if line.startswith("#") or line.startswith("kernel,"):
                continue
            parts = line.strip().rsplit(",", 4)          # kernel names may hold commas
            if len(parts) == 5 and parts[0].startswith(prefix):
                try:
                    n, tb = int(parts[1]), float(parts[4])
                except ValueError:
                    continue
                if best is None or n > best[0]:
                    best = (n, tb)
    return best[1] if best else None


def algorithmic_work(shapes, grad_bytes=2, ef=False, qhm_full=False):
    """Algorithmic bytes and flops per step of each kernel class (unpadded sizes).  With error feedback
    the down-projection also reads the residual E, Adam also writes g as operand planes and the "up"
    class holds a second launch (E <- G + E - Q g: E read and written, G read); the full-rank QHM
    update reads G in the weight update."""
    spq = sum(p * q for p, q, r in shapes)
    spr = sum(p * r for p, q, r in shapes)
    srq = sum(r * q for p, q, r in shapes)
    flops = sum(2 * p * q * r for p, q, r in shapes)
    up_bytes = 8 * spq + 4 * spr + 4 * srq + (grad_bytes * spq if qhm_full else 0)
    up_flops = flops
    if ef:
        up_bytes += 8 * spq + grad_bytes * spq + 4 * spr + 4 * srq
        up_flops += flops
    return {
        "down": dict(bytes=grad_bytes * spq + 4 * spr + 4 * srq + (4 * spq if ef else 0), flops=flops),
        "adam": dict(bytes=(28 if ef else 24) * srq, flops=0),
        "up": dict(bytes=up_bytes, flops=up_flops),
        "outer": dict(bytes=24 * spq, flops=0),
    }


def refresh_flops(shapes, q_it, rotate=True):
    """Algorithmic flops of one subspace refresh: 2 q_it + 1 products with the source, CholeskyQR passes
    (symmetric Gram r^2 rows, factorisation r^3 / 3, triangular apply r^2 rows; one pass per intermediate
    block, two for the final basis) and the moment rotation (R = Q_new^T Q_old, R u, (R o R) w)."""
    total = 0
    for p, q, r in shapes:
        total += (2 * q_it + 1) * 2 * p * q * r
        y_passes = (q_it + 2) if q_it > 0 else 2
        total += y_passes * (2 * p * r * r + r ** 3 // 3) + q_it * (2 * q * r * r + r ** 3 // 3)
        if rotate:
            total += 2 * p * r * r + 4 * r * r * q
    return total


def build_workload(torch, lordo, synth, cfg, rank, n_sets):
    shapes = synth.config_shapes(cfg, rank)
    d = synth.CONFIG_DEFAULTS[cfg]
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.seed_for(int(cfg[1:]), 999))
    W = [(0.02 * torch.randn(p, q, generator=gen, device=dev)).contiguous() for p, q, r in shapes]
    grad_dtype = torch.float32 if cfg == "c1" else torch.bfloat16
    draws = [synth.device_spiked_gradient(torch, p, q, d["n_spike"], synth.seed_for(int(cfg[1:]), i), noise=d["noise"],
                                          dtype=grad_dtype, device=dev) for i, (p, q, r) in enumerate(shapes)]
    G = [[dr(s) for dr in draws] for s in range(n_sets)]
    Omega = [torch.randn(q, r, generator=gen, device=dev) for p, q, r in shapes]
    # stand-in for the cross-worker mean of the pseudo-gradients: same structure as a gradient,
    # scaled by eta * H (what H local steps move a weight by)
    scale = 1e-3 * max(d["outer_every"], 1)
    D = [(scale * 1e3 * draws[i](10_000).float()).contiguous() for i in range(len(shapes))]
    return shapes, W, G, Omega, D, grad_dtype


def run_steps(opt, Wp, Gp, Dp, Op, steps, outer_every, refresh_every, lr, start=0, local_variant=False, Ap=None):
    n_sets = len(Gp)
    for i in range(start, start + steps):
        g = Gp[i % n_sets]
        if local_variant and refresh_every and (i + 1) % refresh_every == 0:
            opt.refresh_subspace_local(g, Op)        # Alg. 2: projection from this step's gradient plus the error buffer
        opt.local_step(Wp, g, lr)
        if outer_every and (i + 1) % outer_every == 0:
            if Ap is not None:
                opt.outer_step_lowrank(Wp, Ap)       # App. A.5.1: Delta = Q mean(A), no p x q pseudo-gradient
            else:
                opt.outer_step(Wp, Dp)
        if not local_variant and refresh_every and (i + 1) % refresh_every == 0:
            opt.refresh_subspace(g, Op)


def cpu_baseline(cfg, shapes, outer_every, refresh_every, power_iters):
    """Time the float64 oracle on the host on a bounded sample: local steps on the leading matrices
    (one transformer layer's worth per distinct shape), one refresh and one outer step on the same
    sample; scale by element counts to the whole set and amortise at the workload's cadence."""
    import numpy as np
    from oracle import lordo_oracle as orc
    from paper_2602_04396_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    d = synth.CONFIG_DEFAULTS[cfg]
    # sample: one matrix per distinct shape, then further matrices in layer order until the
    # local-step work of the sample reaches a fixed float64 flop budget (or the set is exhausted)
    n_local = 2
    budget = 1.0e11
    seen, sample = set(), []
    for i, s in enumerate(shapes):
        if s not in seen:
            seen.add(s)
            sample.append(i)
    flops = sum(4 * r * p * q for p, q, r in (shapes[i] for i in sample)) * n_local
    for i, s in enumerate(shapes):
        if flops >= budget:
            break
        if i not in sample:
            sample.append(i)
            flops += 4 * s[2] * s[0] * s[1] * n_local
    sample.sort()
    hp = orc.Hyper(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=power_iters)
    states, Ws, gens = [], [], []
    for i in sample:
        p, q, r = shapes[i]
        rng = np.random.default_rng(synth.seed_for(int(cfg[1:]), 300 + i))
        W0 = synth.weights(rng, p, q).astype(np.float64)
        states.append(orc.init_state(W0, r, synth.orthonormal(rng, p, r)))
        Ws.append(W0)
        gens.append(synth.SpikedGradient(p, q, d["n_spike"], synth.seed_for(int(cfg[1:]), i), noise=d["noise"]))
    grads = [[g.draw(t).astype(np.float64) for g in gens] for t in range(2)]
    omegas = [synth.omega(np.random.default_rng(synth.seed_for(int(cfg[1:]), 400 + i)), shapes[i][1], shapes[i][2]).astype(np.float64)
              for i in sample]
    # weights of the sample in the whole set: by shape count
    counts = {}
    for s in shapes:
        counts[s] = counts.get(s, 0) + 1
    in_sample = {}
    for i in sample:
        in_sample[shapes[i]] = in_sample.get(shapes[i], 0) + 1
    t_local = t_refresh = t_outer = 0.0
    for k, i in enumerate(sample):
        w = counts[shapes[i]] / in_sample[shapes[i]]
        t0 = time.perf_counter()
        for t in range(n_local):
            Ws[k] = orc.local_step(states[k], Ws[k], grads[t][k], 1e-3, hp)
        t1 = time.perf_counter()
        orc.refresh_subspace(states[k], grads[1][k], omegas[k], hp)
        t2 = time.perf_counter()
        D = orc.pseudo_gradient(states[k], Ws[k])
        Ws[k] = orc.outer_step(states[k], D, hp)
        t3 = time.perf_counter()
        t_local += w * (t1 - t0) / n_local
        t_refresh += w * (t2 - t1)
        t_outer += w * (t3 - t2)
    ms = 1e3 * (t_local + (t_refresh / refresh_every if refresh_every else 0.0) + (t_outer / outer_every if outer_every else 0.0))
    return {
        "value": ms, "unit": "ms/step", "cores": int(cores), "kind": "oracle",
        "sample": (f"{len(sample)} of {len(shapes)} matrices (every distinct shape present), "
                   f"{n_local} local steps + 1 refresh + 1 outer step each, scaled by shape counts to the full set; "
                   f"local {1e3 * t_local:.1f} ms, refresh {1e3 * t_refresh:.1f} ms, outer {1e3 * t_outer:.1f} ms"),
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_04396_amd import lordo, synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")        # 1 GiB, far beyond every cache
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "5 device copies of 1 GiB: 1048576 KiB read and 1048576 KiB written each"}))
        return
    lordo.load()
    cfg = args.config.lower()
    d = synth.CONFIG_DEFAULTS[cfg]
    outer_every = d["outer_every"] if args.outer_every is None else args.outer_every
    refresh_every = d["refresh_every"] if args.refresh_every is None else args.refresh_every
    n_sets = args.grad_sets or (4 if cfg in ("c1", "c2") else 2)
    shapes, W, G, Omega, D, grad_dtype = build_workload(torch, lordo, synth, cfg, args.rank, n_sets)
    qhm_mode = {"plain": 0, "ef": 0, "low-qhm": 1, "full-qhm": 2, "global": 2, "local": 1, "uplink": 0}[args.update]
    uplink = args.update == "uplink"
    if uplink and outer_every and refresh_every:       # the buffer is tied to Q: refresh only right after an outer step
        refresh_every = max(outer_every, refresh_every // outer_every * outer_every)
    use_ef = args.update in ("ef", "global", "local")
    local_variant = args.update == "local"
    hp = lordo.hparams(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=d["power_iters"],
                       grad_dtype=lordo.F32 if grad_dtype == torch.float32 else lordo.BF16,
                       qhm_mode=qhm_mode, omega=0.9 if qhm_mode else 1.0, error_feedback=use_ef, uplink_buffer=uplink,
                       rayleigh_ritz=args.rayleigh_ritz)
    if args.short_side:
        if args.update not in ("plain", "low-qhm", "uplink", "ef", "local"):
            sys.exit("--short-side: the projection on the right is built for --update plain, low-qhm, ef, local and uplink")
        gen = torch.Generator(device="cuda")
        gen.manual_seed(synth.seed_for(int(cfg[1:]), 997))
        lib_shapes = [(p, q, r, 1) if p > q else (p, q, r) for p, q, r in shapes]
        Omega = [torch.randn(p if p > q else q, r, generator=gen, device="cuda") for p, q, r in shapes]
        shapes = [(q, p, r) if p > q else (p, q, r) for p, q, r in shapes]      # the transposed problems, for the work counts
    else:
        lib_shapes = shapes
    opt = lordo.Lordo(lib_shapes, hp, W, torch)
    Wp = opt.ptrs(W)
    Gp = [opt.ptrs(g, grad_dtype) for g in G]
    Dp = opt.ptrs(D)
    Op = opt.ptrs(Omega, torch.float32, "qr")
    Ap = None
    if uplink:    # stand-in for the mean of the workers' buffers: eta * H times a unit-scale low-rank update
        gen = torch.Generator(device="cuda")
        gen.manual_seed(synth.seed_for(int(cfg[1:]), 998))
        # (`shapes` holds the transposed problems of right-projected matrices: their buffers are r x rows)
        Ap = opt.ptrs([(1e-3 * max(outer_every, 1)) * torch.randn(r, q, generator=gen, device="cuda") for p, q, r in shapes],
                      torch.float32, "rq")
    lr = 1e-3
    # a first projection from the first gradient set, as a training run would have
    opt.refresh_subspace(Gp[0], Op)
    opt.poll_status()

    run_steps(opt, Wp, Gp, Dp, Op, args.warmup, outer_every, refresh_every, lr, start=0, local_variant=local_variant, Ap=Ap)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(opt, Wp, Gp, Dp, Op, args.steps, outer_every, refresh_every, lr, start=0, local_variant=local_variant, Ap=Ap)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = 1e3 * (t1 - t0) / args.steps
    opt.poll_status()

    work = algorithmic_work(shapes, 4 if grad_dtype == torch.float32 else 2, ef=use_ef, qhm_full=qhm_mode == 2)
    kernels = {}
    roofline = None
    if not args.no_events:
        opt.profile_enable(True)
        run_steps(opt, Wp, Gp, Dp, Op, args.steps, outer_every, refresh_every, lr, start=0, local_variant=local_variant, Ap=Ap)
        if not outer_every:          # workloads that time the outer step and the refresh on their own
            opt.outer_step_lowrank(Wp, Ap) if uplink else opt.outer_step(Wp, Dp)
        if not refresh_every:
            opt.refresh_subspace(Gp[0], Op)
        torch.cuda.synchronize()
        total_by = {}
        for name, kc in (("down", lordo.K_DOWN), ("adam", lordo.K_ADAM), ("up", lordo.K_UP), ("outer", lordo.K_OUTER),
                         ("refresh", lordo.K_REFRESH)):
            ms, cnt = opt.profile_read(kc)
            if cnt == 0:
                continue
            avg = ms / cnt
            entry = {"avg_ms": avg, "launches": cnt}
            if name in work:
                entry["GBps"] = work[name]["bytes"] / (avg * 1e-3) / 1e9
                if work[name]["flops"]:
                    entry["TFLOPps"] = work[name]["flops"] / (avg * 1e-3) / 1e12
            if name == "refresh":
                entry["TFLOPps"] = refresh_flops(shapes, d["power_iters"]) / (avg * 1e-3) / 1e12
            kernels[name] = entry
            total_by[name] = ms
        opt.profile_enable(False)
        dom = max((k for k in total_by if k in work), key=lambda k: total_by[k])
        w = work[dom]
        avg_s = kernels[dom]["avg_ms"] * 1e-3
        t_hbm = w["bytes"] / (HBM_PEAK_GBS * 1e9)
        t_mfma = w["flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        if t_mfma > t_hbm:
            ach = w["flops"] / avg_s / 1e12
            roofline = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": measured_traffic(cfg, args.rank, dom, args.update)}
        else:
            ach = w["bytes"] / avg_s / 1e9
            roofline = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": ach / HBM_PEAK_GBS, "traffic": measured_traffic(cfg, args.rank, dom, args.update)}

    if args.rayleigh_ritz and not args.no_events and not use_ef:
        # the spectrum metrics (Sec. 5.1) on their own: the gap program is a second pass of the size of a refresh
        opt.spectral_gap(Gp[0], Op)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(3):
            opt.spectral_gap(Gp[0], Op)
        torch.cuda.synchronize()
        kernels["spectral_gap"] = {"avg_ms": 1e3 * (time.perf_counter() - t2) / 3, "launches": 3}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = None if args.short_side else cpu_baseline(cfg, shapes, outer_every, refresh_every, d["power_iters"])

    out = {
        "metric": "full-model low-rank optimizer step ms",
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 MFMA operands (fp32 state split hi+lo), f32 accumulate and state",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[cfg] + (f", rank override {args.rank}" if args.rank else ""),
                   "matrices": len(shapes), "params": sum(p * q for p, q, r in shapes),
                   "refresh_every": refresh_every, "outer_every": outer_every, "power_iters": d["power_iters"],
                   "grad_sets": n_sets, "outer": "nesterov lr 0.7 momentum 0.9 on a generated averaged pseudo-gradient",
                   "update": args.update, "rayleigh_ritz": bool(args.rayleigh_ritz), "short_side": bool(args.short_side)},
        "roofline": roofline,
        "kernels": kernels,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
