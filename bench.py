#!/usr/bin/env python3
"""Benchmark of the LoRDO hot path on one MI355X.

Default workload: c4, the ~7B-shaped set (224 matrices, r = 512), the largest one that is a whole model.  A "step"
is one local step over every matrix (down-projection, fused low-rank Adam, up-projection with the weight update);
workloads with a cadence (c2: refresh every 200, outer step every 32 steps) also run the outer step on a generated
averaged pseudo-gradient and the subspace refresh with moment rotation inside the timed region at that cadence.
c4 times them apart from the local step: whatever --steps is, one outer step and one refresh are event-timed after
the loop, so `kernels` always holds down, adam, up, outer and refresh.  Inputs are synthetic, seeded and resident
in HBM before the timed region starts.

Prints ONE JSON line: the time per step, the time of one refresh and of one outer step, the roofline of the
dominant kernel of the local step (event-timed through the library's profiling hooks on the stream the kernels run
on), the per-class times of the other workloads (c2, c3, the rank sweep on the 8192 x 28672 matrix with one and two
power iterations) and the float64 oracle timed on the host cores with one thread and with all of them.
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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c4")
    ap.add_argument("--rank", type=int, default=None)
    ap.add_argument("--grad-sets", type=int, default=None, help="distinct gradient sets cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="skip the event-timed second pass")
    ap.add_argument("--no-extra", dest="extra", action="store_false",
                    help="skip the per-class times of the other workloads (c2, c3, rank sweep on c5)")
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
    ap.add_argument("--param-dtype", default="f32", choices=["f32", "bf16"],
                    help="storage type of the weights (bf16: updates formed in fp32 and rounded once; update cases plain, low-qhm, ef, local)")
    ap.add_argument("--err-dtype", default="f32", choices=["f32", "bf16"],
                    help="storage type of the error-feedback residual E (update cases ef and global)")
    ap.add_argument("--calibrate-gemm", action="store_true",
                    help="only time the library's plain bf16 GEMM (torch.matmul / bmm) at the shapes of the c4 projections and at "
                         "8192^3: what a library contraction reaches on this box with random operands (context for the issued rates)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run plain 1 GiB device copies (known traffic) to scale the FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


KERNEL_OF_CLASS = {"down": "k_proj_down", "adam": "k_adam", "up": "k_proj_up", "outer": "k_pq<0>"}


def measured_traffic(cfg, rank, kernel_class, update="plain", param_dtype="f32"):
    """HBM bytes per launch of a kernel class from the committed rocprofv3 counter summary of this
    workload (FETCH_SIZE and WRITE_SIZE runs, scaled by a plain copy), or None if there is none."""
    if rank is not None or update != "plain" or param_dtype != "f32":
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


def measured_mfma_counters(cfg, rank, kernel_class, update="plain", param_dtype="f32"):
    """Matrix-core busy cycles over elapsed cycles and the clock the chip ran at, for a projection kernel of this
    workload, from the committed rocprofv3 counter summary (its "derived" lines), or {} if it does not cover the case."""
    if update != "plain" or param_dtype != "f32" or cfg not in ("c4", "c5"):
        return {}
    label = "c4 r=512" if cfg == "c4" else f"c5 r={rank}"
    path = os.path.join(ROOT, "profiles", "c4_c5_projection_mfma_counters_pmc.txt")
    prefix = KERNEL_OF_CLASS.get(kernel_class)
    if prefix is None or not os.path.exists(path):
        return {}
    with open(path) as f:
        for line in f:
            parts = line.lstrip("# ").strip().split(",")
            if len(parts) == 6 and parts[0] == label and parts[1].startswith(prefix):
                try:
                    return {"mfma_busy_frac_of_elapsed_cycles": float(parts[5]), "clock_GHz": float(parts[4])}
                except ValueError:
                    return {}
    return {}


def algorithmic_work(shapes, grad_bytes=2, ef=False, qhm_full=False, w_bytes=4, e_bytes=4):
    """Algorithmic bytes and flops per step of each kernel class (unpadded sizes).  With error feedback
    the down-projection also reads the residual E, Adam also writes g as operand planes and the "up"
    class holds a second launch (E <- G + E - Q g: E read and written, G read); the full-rank QHM
    update reads G in the weight update."""
    spq = sum(p * q for p, q, r in shapes)
    spr = sum(p * r for p, q, r in shapes)
    srq = sum(r * q for p, q, r in shapes)
    flops = sum(2 * p * q * r for p, q, r in shapes)
    up_bytes = 2 * w_bytes * spq + 4 * spr + 4 * srq + (grad_bytes * spq if qhm_full else 0)
    up_flops = flops
    if ef:
        up_bytes += 2 * e_bytes * spq + grad_bytes * spq + 4 * spr + 4 * srq
        up_flops += flops
    return {
        "down": dict(bytes=grad_bytes * spq + 4 * spr + 4 * srq + (e_bytes * spq if ef else 0), flops=flops),
        "adam": dict(bytes=(28 if ef else 24) * srq, flops=0),
        "up": dict(bytes=up_bytes, flops=up_flops),
        "outer": dict(bytes=(20 + w_bytes) * spq, flops=0),
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


def build_workload(torch, lordo, synth, cfg, rank, n_sets, w_dtype=None):
    shapes = synth.config_shapes(cfg, rank)
    d = synth.CONFIG_DEFAULTS[cfg]
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.seed_for(int(cfg[1:]), 999))
    W = [(0.02 * torch.randn(p, q, generator=gen, device=dev)).to(w_dtype or torch.float32).contiguous() for p, q, r in shapes]
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


def _oracle_sample(cfg, shapes, power_iters, sample, n_local, thread_settings):
    """Wall-clock of the float64 oracle on the matrices `sample`: for every entry of `thread_settings` (BLAS pool
    limited to that many threads; None: as many as it takes by itself) a dict matrix index -> (local step, refresh,
    outer step) seconds.  The inputs of a matrix are generated once and serve every setting."""
    import numpy as np
    from oracle import lordo_oracle as orc
    from paper_2602_04396_amd import synth
    from threadpoolctl import threadpool_limits
    d = synth.CONFIG_DEFAULTS[cfg]
    hp = orc.Hyper(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=power_iters)
    out = [dict() for _ in thread_settings]
    for i in sample:
        p, q, r = shapes[i]
        rng = np.random.default_rng(synth.seed_for(int(cfg[1:]), 300 + i))
        W0 = synth.weights(rng, p, q).astype(np.float64)
        Q0 = synth.orthonormal(rng, p, r)
        gen = synth.SpikedGradient(p, q, d["n_spike"], synth.seed_for(int(cfg[1:]), i), noise=d["noise"])
        grads = [gen.draw(t).astype(np.float64) for t in range(n_local)]
        om = synth.omega(np.random.default_rng(synth.seed_for(int(cfg[1:]), 400 + i)), q, r).astype(np.float64)
        for k, threads in enumerate(thread_settings):
            W = W0.copy()
            st = orc.init_state(W, r, Q0)
            with threadpool_limits(limits=threads):
                t0 = time.perf_counter()
                for t in range(n_local):
                    W = orc.local_step(st, W, grads[t], 1e-3, hp)
                t1 = time.perf_counter()
                orc.refresh_subspace(st, grads[-1], om, hp)
                t2 = time.perf_counter()
                W = orc.outer_step(st, orc.pseudo_gradient(st, W), hp)
                t3 = time.perf_counter()
            out[k][i] = ((t1 - t0) / n_local, t2 - t1, t3 - t2)
    return out


def cpu_baseline(cfg, shapes, outer_every, refresh_every, power_iters):
    """The float64 oracle, as it stands, timed on the host cores: once with one thread and once with every core
    the BLAS pool takes.  Small sets (c1, c2) are timed in full; for the larger ones the oracle runs one matrix
    per distinct shape at full size and its time is multiplied by the number of matrices of that shape
    ("extrapolated").  The value is per step: the local step plus, where the workload has a cadence, the refresh
    and the outer step amortised over it; the three parts are also given on their own."""
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    full = cfg in ("c1", "c2")
    counts = {}
    for sh in shapes:
        counts[sh] = counts.get(sh, 0) + 1
    if full:
        sample = list(range(len(shapes)))
        weight = {i: 1.0 for i in sample}
    else:
        seen, sample = set(), []
        for i, sh in enumerate(shapes):
            if sh not in seen:
                seen.add(sh)
                sample.append(i)
        weight = {i: float(counts[shapes[i]]) for i in sample}
    n_local = 2 if full else 1

    def total(per):
        t_local = sum(weight[i] * per[i][0] for i in sample)
        t_refresh = sum(weight[i] * per[i][1] for i in sample)
        t_outer = sum(weight[i] * per[i][2] for i in sample)
        ms = 1e3 * (t_local + (t_refresh / refresh_every if refresh_every else 0.0) + (t_outer / outer_every if outer_every else 0.0))
        return {"value": ms, "local_step_ms": 1e3 * t_local, "refresh_ms": 1e3 * t_refresh, "outer_step_ms": 1e3 * t_outer}

    per_all, per_one = _oracle_sample(cfg, shapes, power_iters, sample, n_local, [None, 1])
    multi, single = total(per_all), total(per_one)
    label = ("full set" if full else "extrapolated (one matrix per distinct shape x counts)")
    return {
        "value": multi["value"], "unit": "ms/step", "cores": int(cores), "kind": "oracle",
        "sample": (f"{label}: {len(sample)} of {len(shapes)} matrices at full size, {n_local} local step(s) + 1 refresh + 1 outer step "
                   f"each; value = local step" + (" + refresh / refresh_every" if refresh_every else "")
                   + (" + outer step / outer_every" if outer_every else "") + " (ms); the three parts are given separately"),
        "threads_all": dict(multi, cores=int(cores)),
        "threads_1": dict(single, cores=1),
    }


class Workload:
    """One workload resident in HBM, its library context, and the pointer tables of every call."""

    def __init__(self, torch, lordo, synth, cfg, rank, n_sets, args, power_iters=None, base=None):
        self.torch, self.lordo, self.cfg, self.rank = torch, lordo, cfg, rank
        d = synth.CONFIG_DEFAULTS[cfg]
        self.defaults = d
        self.power_iters = d["power_iters"] if power_iters is None else power_iters
        w_bf16 = getattr(args, "param_dtype", "f32") == "bf16"
        if base is None:
            base = build_workload(torch, lordo, synth, cfg, rank, n_sets, torch.bfloat16 if w_bf16 else None)
        shapes, W, G, Omega, D, grad_dtype = base
        self.base = base
        self.grad_dtype = grad_dtype
        self.qhm_mode = {"plain": 0, "ef": 0, "low-qhm": 1, "full-qhm": 2, "global": 2, "local": 1, "uplink": 0}[args.update]
        self.uplink = args.update == "uplink"
        self.use_ef = args.update in ("ef", "global", "local")
        self.local_variant = args.update == "local"
        hp = lordo.hparams(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=self.power_iters,
                           grad_dtype=lordo.F32 if grad_dtype == torch.float32 else lordo.BF16,
                           qhm_mode=self.qhm_mode, omega=0.9 if self.qhm_mode else 1.0, error_feedback=self.use_ef,
                           uplink_buffer=self.uplink, rayleigh_ritz=args.rayleigh_ritz,
                           param_dtype=lordo.BF16 if w_bf16 else lordo.F32,
                           err_dtype=lordo.BF16 if getattr(args, "err_dtype", "f32") == "bf16" and self.use_ef else lordo.F32)
        if args.short_side:
            gen = torch.Generator(device="cuda")
            gen.manual_seed(synth.seed_for(int(cfg[1:]), 997))
            lib_shapes = [(p, q, r, 1) if p > q else (p, q, r) for p, q, r in shapes]
            Omega = [torch.randn(p if p > q else q, r, generator=gen, device="cuda") for p, q, r in shapes]
            shapes = [(q, p, r) if p > q else (p, q, r) for p, q, r in shapes]      # the transposed problems, for the work counts
        else:
            lib_shapes = shapes
        self.shapes = shapes
        self.opt = opt = lordo.Lordo(lib_shapes, hp, W, torch)
        self.Wp = opt.ptrs(W, torch.bfloat16 if w_bf16 else torch.float32)
        self.Gp = [opt.ptrs(g, grad_dtype) for g in G]
        self.Dp = opt.ptrs(D)
        self.Op = opt.ptrs(Omega, torch.float32, "qr")
        self.Ap = None
        if self.uplink:    # stand-in for the mean of the workers' buffers: eta * H times a unit-scale low-rank update
            gen = torch.Generator(device="cuda")
            gen.manual_seed(synth.seed_for(int(cfg[1:]), 998))
            # (`shapes` holds the transposed problems of right-projected matrices: their buffers are r x rows)
            self.Ap = opt.ptrs([(1e-3 * max(d["outer_every"], 1)) * torch.randn(r, q, generator=gen, device="cuda") for p, q, r in shapes],
                               torch.float32, "rq")
        # a first projection from the first gradient set, as a training run would have
        opt.refresh_subspace(self.Gp[0], self.Op)
        opt.poll_status()

    def steps(self, n, outer_every, refresh_every, lr=1e-3):
        run_steps(self.opt, self.Wp, self.Gp, self.Dp, self.Op, n, outer_every, refresh_every, lr, start=0,
                  local_variant=self.local_variant, Ap=self.Ap)

    def outer_once(self):
        self.opt.outer_step_lowrank(self.Wp, self.Ap) if self.uplink else self.opt.outer_step(self.Wp, self.Dp)

    def refresh_once(self):
        self.opt.refresh_subspace(self.Gp[0], self.Op)

    def profiled(self, n, outer_every, refresh_every, work):
        """`n` steps at the given cadence with every kernel class bracketed by HIP events on the launch stream, then
        -- whatever the cadence and n -- one outer step and one refresh, so that both always have a time of their own."""
        lordo, opt = self.lordo, self.opt
        opt.profile_enable(True)
        self.steps(n, outer_every, refresh_every)
        self.outer_once()
        self.refresh_once()
        self.torch.cuda.synchronize()
        kernels, total_by = {}, {}
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
                entry["TFLOPps"] = refresh_flops(self.shapes, self.power_iters) / (avg * 1e-3) / 1e12
            kernels[name] = entry
            total_by[name] = ms
        # When no matrix needs split-K the moment update runs in the epilogue of the down-projection and the "adam" span
        # holds nothing that moves the state (a rate beyond anything the memory system can do tells): its bytes then
        # belong to the down-projection
        if "adam" in kernels and "down" in kernels and kernels["adam"].get("GBps", 0.0) > 2 * HBM_PEAK_GBS:
            avg = kernels["down"]["avg_ms"]
            kernels["down"]["GBps"] = (work["down"]["bytes"] + work["adam"]["bytes"]) / (avg * 1e-3) / 1e9
            kernels["down"]["includes"] = "adam (fused epilogue)"
            kernels["adam"] = {"avg_ms": kernels["adam"]["avg_ms"], "launches": kernels["adam"]["launches"], "fused_into": "down"}
        opt.profile_enable(False)
        opt.poll_status()
        return kernels, total_by

    def close(self):
        self.opt.close()


def roofline_of(kernels, total_by, work, cfg, rank, update, param_dtype="f32"):
    """Roofline entry of the kernel class that takes most of the local step."""
    dom = max((k for k in total_by if k in ("down", "adam", "up")), key=lambda k: total_by[k])
    w = work[dom]
    avg_s = kernels[dom]["avg_ms"] * 1e-3
    nbytes = w["bytes"] + (work["adam"]["bytes"] if dom == "down" and "includes" in kernels[dom] else 0)
    t_hbm = nbytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = w["flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    # the fp32 operands (Q, N) enter the matrix cores as bf16 hi + lo planes: 2 passes over the contraction for the
    # down-projection of a bf16 gradient (3 with error feedback), 3 for the up-projection.  Reported next to the
    # algorithmic roofline: the matrix-core rate on issued passes.
    passes = {"down": 3 if update in ("ef", "global", "local") else 2, "up": 3}.get(dom, 0)
    issued = {"mfma_passes": passes, "issued_TFLOPps": passes * w["flops"] / avg_s / 1e12,
              "issued_frac_of_mfma_peak": passes * w["flops"] / avg_s / 1e12 / MFMA_BF16_PEAK_TFLOPS} if passes and w["flops"] else {}
    issued.update(measured_mfma_counters(cfg, rank, dom, update, param_dtype))
    if t_mfma > t_hbm:
        ach = w["flops"] / avg_s / 1e12
        return dict({"kernel": dom, "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": measured_traffic(cfg, rank, dom, update, param_dtype)}, **issued)
    ach = nbytes / avg_s / 1e9
    return dict({"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": ach / HBM_PEAK_GBS, "traffic": measured_traffic(cfg, rank, dom, update, param_dtype)}, **issued)


def class_ms(kernels):
    return {k: round(v["avg_ms"], 5) for k, v in kernels.items()}


def graph_replay_ms(torch, wl, n):
    """Milliseconds per local step when the step is recorded once per gradient set into a HIP graph and replayed (the
    step count and the bias corrections advance on the device, so replays are successive steps)."""
    graphs = []
    for Gp in wl.Gp:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            wl.opt.local_step(wl.Wp, Gp, 1e-3)
        graphs.append(g)
    for g in graphs:
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n):
        graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    return 1e3 * (time.perf_counter() - t0) / n


def extra_variants(torch, lordo, synth, args, cfg):
    """The headline workload under the configuration the paper's experiments use, LoRDO-Global (full-rank QHM with error
    feedback, Sec. 3.2 and Alg. 1), with fp32 storage and with the weights and the residual stored in bf16: time per
    local step and per kernel class."""
    import copy
    import gc
    out = []
    for storage in ("f32", "bf16"):
        a = copy.copy(args)
        a.update, a.param_dtype, a.err_dtype, a.rayleigh_ritz, a.short_side = "global", storage, storage, False, False
        wl = Workload(torch, lordo, synth, cfg, None, 2, a)
        wl.steps(2, 0, 0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        wl.steps(6, 0, 0)
        torch.cuda.synchronize()
        step_ms = 1e3 * (time.perf_counter() - t0) / 6
        work = algorithmic_work(wl.shapes, 2, ef=True, qhm_full=True, w_bytes=2 if storage == "bf16" else 4, e_bytes=2 if storage == "bf16" else 4)
        kernels, _ = wl.profiled(4, 0, 0, work)
        out.append({"workload": cfg, "update": "global (full-rank QHM + error feedback)", "storage_of_W_and_E": storage,
                    "step_ms": round(step_ms, 4), "ms": class_ms({k: v for k, v in kernels.items() if k in ("down", "adam", "up")})})
        wl.close()
        del wl
        gc.collect()
        torch.cuda.empty_cache()
    return out


def extra_configs(torch, lordo, synth, args, skip_cfg):
    """Per-class times of the other workloads of the table, so that one run covers it: c2, c3 and the rank sweep on
    the single largest matrix (c5) with one and two power iterations in the refresh.  Kernel-class averages only."""
    import gc
    out = []
    # (warm-up long enough for the clocks to settle: some tens of milliseconds of steps)
    for cfg, warm, steps in (("c1", 200, 500), ("c2", 100, 200), ("c3", 5, 20), ("c4", 3, 6)):
        if cfg == skip_cfg:
            continue
        wl = Workload(torch, lordo, synth, cfg, None, 4 if cfg == "c2" else 2, args)
        wl.steps(warm, 0, 0)
        work = algorithmic_work(wl.shapes, 4 if cfg == "c1" else 2, w_bytes=2 if args.param_dtype == "bf16" else 4)
        kernels, _ = wl.profiled(steps, 0, 0, work)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        wl.steps(steps, 0, 0)
        torch.cuda.synchronize()
        step_ms = 1e3 * (time.perf_counter() - t0) / steps
        out.append({"workload": cfg, "rank": wl.shapes[0][2], "power_iters": wl.power_iters, "ms": class_ms(kernels),
                    "step_ms": round(step_ms, 5),
                    "step_ms_graph_replay": round(graph_replay_ms(torch, wl, steps), 5) if cfg in ("c1", "c2") else None,
                    "GBps": {k: round(v["GBps"]) for k, v in kernels.items() if "GBps" in v},
                    "adam_fused": "fused_into" in kernels.get("adam", {}),
                    "TFLOPps": {k: round(v["TFLOPps"], 1) for k, v in kernels.items() if "TFLOPps" in v}})
        wl.close()
        del wl
        gc.collect()
        torch.cuda.empty_cache()
    if skip_cfg != "c5":
        base = None
        for rank in (64, 128, 256, 512, 1024):
            if base is None:
                base = build_workload(torch, lordo, synth, "c5", rank, 2, torch.bfloat16 if args.param_dtype == "bf16" else None)
            shapes = synth.config_shapes("c5", rank)
            gen = torch.Generator(device="cuda")
            gen.manual_seed(synth.seed_for(5, 999))
            Omega = [torch.randn(q, r, generator=gen, device="cuda") for p, q, r in shapes]
            this = (shapes, base[1], base[2], Omega, base[4], base[5])
            entry = {"workload": "c5", "rank": rank}
            for q_it in (1, 2):
                wl = Workload(torch, lordo, synth, "c5", rank, 2, args, power_iters=q_it, base=this)
                wl.steps(20 if q_it == 1 else 3, 0, 0)
                work = algorithmic_work(wl.shapes, 2, w_bytes=2 if args.param_dtype == "bf16" else 4)
                kernels, _ = wl.profiled(50 if q_it == 1 else 0, 0, 0, work)
                if q_it == 1:
                    entry["ms"] = class_ms({k: v for k, v in kernels.items() if k != "refresh"})
                    entry["GBps"] = {k: round(v["GBps"]) for k, v in kernels.items() if "GBps" in v}
                    entry["adam_fused"] = "fused_into" in kernels.get("adam", {})
                    entry["TFLOPps"] = {k: round(v["TFLOPps"], 1) for k, v in kernels.items() if "TFLOPps" in v and k != "refresh"}
                entry[f"refresh_ms_q{q_it}"] = round(kernels["refresh"]["avg_ms"], 4)
                wl.close()
                del wl
                gc.collect()
            out.append(entry)
            del Omega, this
            torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import gc
    import torch
    from paper_2602_04396_amd import lordo, synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate_gemm:
        def rate(fn, flops, reps):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return flops / ((time.perf_counter() - t0) / reps) / 1e12
        bf = dict(device="cuda", dtype=torch.bfloat16)
        out = {"calibration": "library bf16 GEMM (torch.matmul / torch.bmm, fp32 accumulate, bf16 output, standard-normal operands), TFLOP/s"}
        a, b = torch.randn(8192, 8192, **bf), torch.randn(8192, 8192, **bf)
        out["square_8192"] = rate(lambda: a @ b, 2 * 8192 ** 3, 10)
        a, b = torch.randn(128, 4096, 512, **bf), torch.randn(128, 512, 4096, **bf)       # the 128 matrices of 4096 x 4096 of c4
        out["up_shape_128x(4096x512x4096)"] = rate(lambda: torch.bmm(a, b), 2 * 128 * 4096 * 512 * 4096, 5)
        a, b = torch.randn(64, 512, 4096, **bf), torch.randn(64, 4096, 11008, **bf)       # the 64 matrices of 4096 x 11008
        out["down_shape_64x(512x4096x11008)"] = rate(lambda: torch.bmm(a, b), 2 * 64 * 512 * 4096 * 11008, 5)
        print(json.dumps(out))
        return
    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")        # 1 GiB, far beyond every cache
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            b.copy_(a)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 10
        # the same memory under a read-modify-write pass (torch's in-place add: 1 GiB read, 1 GiB written), the access
        # pattern of the weight update and of the outer step
        for _ in range(5):
            a.add_(1.0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            a.add_(1.0)
        torch.cuda.synchronize()
        dt_rmw = (time.perf_counter() - t0) / 10
        print(json.dumps({"calibration": "device copies of 1 GiB: 1048576 KiB read and 1048576 KiB written each; then in-place adds over 1 GiB",
                          "copy_GBps": 2 * (1 << 30) / dt / 1e9, "read_modify_write_GBps": 2 * (1 << 30) / dt_rmw / 1e9}))
        return
    lordo.load()
    cfg = args.config.lower()
    d = synth.CONFIG_DEFAULTS[cfg]
    outer_every = d["outer_every"] if args.outer_every is None else args.outer_every
    refresh_every = d["refresh_every"] if args.refresh_every is None else args.refresh_every
    n_sets = args.grad_sets or (4 if cfg in ("c1", "c2") else 2)
    if args.short_side and args.update not in ("plain", "low-qhm", "uplink", "ef", "local"):
        sys.exit("--short-side: the projection on the right is built for --update plain, low-qhm, ef, local and uplink")
    wl = Workload(torch, lordo, synth, cfg, args.rank, n_sets, args)
    if wl.uplink and outer_every and refresh_every:       # the buffer is tied to Q: refresh only right after an outer step
        refresh_every = max(outer_every, refresh_every // outer_every * outer_every)
    shapes, grad_dtype = wl.shapes, wl.grad_dtype

    wl.steps(args.warmup, outer_every, refresh_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    wl.steps(args.steps, outer_every, refresh_every)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = 1e3 * (t1 - t0) / args.steps
    wl.opt.poll_status()

    w_bytes = 2 if args.param_dtype == "bf16" else 4
    work = algorithmic_work(shapes, 4 if grad_dtype == torch.float32 else 2, ef=wl.use_ef, qhm_full=wl.qhm_mode == 2, w_bytes=w_bytes,
                            e_bytes=2 if args.err_dtype == "bf16" else 4)
    kernels = {}
    roofline = None
    if not args.no_events:
        kernels, total_by = wl.profiled(args.steps, outer_every, refresh_every, work)
        roofline = roofline_of(kernels, total_by, work, cfg, args.rank, args.update, args.param_dtype)

    if args.rayleigh_ritz and not args.no_events and not wl.use_ef:
        # the spectrum metrics (Sec. 5.1) on their own: the gap program is a second pass of the size of a refresh
        wl.opt.spectral_gap(wl.Gp[0], wl.Op)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(3):
            wl.opt.spectral_gap(wl.Gp[0], wl.Op)
        torch.cuda.synchronize()
        kernels["spectral_gap"] = {"avg_ms": 1e3 * (time.perf_counter() - t2) / 3, "launches": 3}
    power_iters = wl.power_iters
    wl.close()
    del wl
    gc.collect()
    torch.cuda.empty_cache()

    extra = None
    if args.extra and not args.no_events:
        extra = {"configs": extra_configs(torch, lordo, synth, args, cfg),
                 "variants": extra_variants(torch, lordo, synth, args, cfg) if args.update == "plain" and not args.short_side else None,
                 "note": "HIP-event averages per kernel class and call (ms); down/up TFLOP/s on 2pqr flops, GB/s on algorithmic bytes"}

    cpu = None
    if not args.no_cpu_baseline and not args.short_side:
        cpu = cpu_baseline(cfg, shapes, outer_every, refresh_every, power_iters)

    out = {
        "metric": "full-model low-rank optimizer step ms",
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[cfg] + (f", rank override {args.rank}" if args.rank else ""),
                   "arithmetic": "bf16 matrix-core products with fp32 accumulation; fp32 operands (Q, N, the moments' inputs) enter as "
                                 "bf16 hi + lo planes, so that results hold the 1e-4 bound against the float64 oracle; state and weights fp32"
                                 + (" (weights stored in bf16)" if args.param_dtype == "bf16" else ""),
                   "matrices": len(shapes), "params": sum(p * q for p, q, r in shapes),
                   "timed_region": ("local steps only; one refresh and one outer step are event-timed on their own after it"
                                    if not (refresh_every or outer_every) else
                                    f"local steps with a refresh every {refresh_every} and an outer step every {outer_every} steps"),
                   "refresh_every": refresh_every, "outer_every": outer_every, "power_iters": power_iters,
                   "grad_sets": n_sets, "outer": "nesterov lr 0.7 momentum 0.9 on a generated averaged pseudo-gradient",
                   "update": args.update, "rayleigh_ritz": bool(args.rayleigh_ritz), "short_side": bool(args.short_side),
                   "param_dtype": args.param_dtype, "err_dtype": args.err_dtype if args.update in ("ef", "global", "local") else None},
        "ms_per_refresh": kernels.get("refresh", {}).get("avg_ms"),
        "ms_per_outer": kernels.get("outer", {}).get("avg_ms"),
        "roofline": roofline,
        "kernels": kernels,
        "extra": extra,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
