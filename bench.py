#!/usr/bin/env python3
"""Benchmark of the basis-rotation optimizer step on one MI355X.

A "step" is one pass of the whole hot path over one pipeline stage's matrices: take the
delayed gradient from the ring, first moment + Kronecker statistics, basis refresh when
t mod freq == 0, rotate, Adam in the rotated basis, rotate back and apply.  Inputs are
synthetic and resident in HBM before the timed region starts.

Prints ONE JSON line: throughput in parameters per second for the whole stage ("value"), the
milliseconds per step, "roofline" (the dominant contraction kernel against the matrix-core peak of
its input type, timed with HIP events on the launch stream), "roofline_elementwise", a per-kernel
table, the other math modes' short runs ("modes") and the CPU oracle timed on a bounded sample
("cpu_baseline").
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # MI355X dense matrix-core peaks (FP32, BF16)
MATH = {"f32": 0, "bf16": 1, "bf16x3": 2}
PEAK_HBM_GBS = 8000.0
TAU = 3
FREQ = 10


def workload(name):
    from paper_2602_03515_amd import synth
    if name == "stage3b":
        return list(synth.STAGE_3B), "3B-class pipeline stage: 8 layers x (4x 2560x2560, 2x 2560x6912, 1x 6912x2560) = 56 matrices"
    if name == "stage3b_emb":
        return (list(synth.STAGE_3B) + [synth.EMBEDDING_SHARD],
                "refresh-heavy stress: the 56 stage matrices + the 32000x2560 embedding shard, unilateral rotation, "
                "refresh every step with 2 power iterations + QR")
    if name == "layer3b":
        return list(synth.STAGE_3B_LAYER), "one layer of the 3B-class stage (7 matrices)"
    if name == "layer2048":
        return list(synth.LLAMA_LAYER_2048), "one Llama-style layer, hidden 2048 (7 matrices)"
    if name == "small":
        return [(256, 256)], "single 256x256 matrix"
    raise SystemExit(f"unknown workload {name}")


def make_inputs(shapes, slots, seed, device, sigma=0.01, rank=64):
    """Low-rank-plus-noise gradients generated on the device: G = A diag(1/i) B^T + sigma N, one
    tensor per ring slot and matrix; weights ~ 0.02 N(0,1)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    params, ring = [], [[] for _ in range(slots)]
    s = 1.0 / torch.arange(1, rank + 1, device=device, dtype=torch.float32)
    for (m, n) in shapes:
        A, _ = torch.linalg.qr(torch.randn(m, rank, generator=gen, device=device))
        Bm, _ = torch.linalg.qr(torch.randn(n, rank, generator=gen, device=device))
        signal = (A * s[None, :]) @ Bm.T
        params.append(0.02 * torch.randn(m, n, generator=gen, device=device))
        for k in range(slots):
            ring[k].append((signal + sigma * torch.randn(m, n, generator=gen, device=device)).contiguous())
        del A, Bm, signal
    return params, ring


def cpu_baseline(seconds_hint=20.0):
    """The float64 oracle as it stands, timed on this host's cores on a bounded sample of the same workload: one
    layer of the stage (7 matrices), three ordinary (non-refresh) steps each, plus ONE refresh (both factors of a
    2560 x 2560 matrix, the oracle's Power step with LAPACK's QR plugged into its `qr` hook, as the full-size parity
    tests run it) and the oracle's own Householder loop at order 1024.  The stage figure is EXTRAPOLATED from those:
    8 layers, the refresh scaled to the stage's factor orders by k^3 and amortised over `FREQ` steps."""
    import numpy as np
    from oracle import br_oracle as oc
    from paper_2602_03515_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1

    def lapack_qr(P):
        q, r = np.linalg.qr(P)
        d = np.where(np.diag(r) < 0, -1.0, 1.0)
        return q * d[None, :], r * d[:, None]

    hp = oc.Hyper().rounded_to_f32()
    rng = np.random.default_rng(2)
    shapes = list(synth.STAGE_3B_LAYER)
    t_total, params, reps = 0.0, 0, 3
    done = []
    refresh_state = None
    for (m, n) in shapes:
        G = (0.01 * rng.standard_normal((m, n))).astype(np.float32)
        W = (0.02 * rng.standard_normal((m, n))).astype(np.float32)
        st = oc.MatrixState(m, n, hp)
        t0 = time.perf_counter()
        for _ in range(reps):
            W = oc.optimizer_step(st, W, G, 1e-3, hp, freq=0)
        t_total += time.perf_counter() - t0
        params += reps * m * n
        done.append(f"{m}x{n}")
        if refresh_state is None and m == n:
            refresh_state = st
        if t_total > 1.5 * seconds_hint:
            break
    layer_params = sum(m * n for m, n in shapes)
    plain_layer_s = t_total / params * layer_params                 # one non-refresh step of one layer
    # one refresh of a 2560 x 2560 matrix: two factors of order 2560 (well-conditioned statistics: shifted noise Gram)
    k = refresh_state.m
    refresh_state.L = refresh_state.L + 1e-4 * np.eye(k)
    refresh_state.R = refresh_state.R + 1e-4 * np.eye(k)
    t0 = time.perf_counter()
    oc.refresh(refresh_state, hp, lapack_qr)
    t_refresh = time.perf_counter() - t0
    cubes_measured = 2.0 * k ** 3
    cubes_layer = sum(float(m) ** 3 + float(n) ** 3 for m, n in shapes)
    refresh_layer_s = t_refresh * cubes_layer / cubes_measured
    P = rng.standard_normal((1024, 1024))
    t0 = time.perf_counter()
    oc.householder_qr(P)
    t_house = time.perf_counter() - t0
    stage_s = 8.0 * (plain_layer_s + refresh_layer_s / FREQ)
    return {"value": 8.0 * layer_params / stage_s, "unit": "params/s", "cores": int(cores), "kind": "oracle",
            "extrapolated": True,
            "sample": f"{len(done)} matrices of one stage layer ({', '.join(done)}), {reps} non-refresh steps each, "
                      f"float64 numpy, {t_total:.1f} s; one refresh of a {k}x{k} matrix (2 factors of order {k}, LAPACK QR "
                      f"through the oracle's qr hook) {t_refresh:.1f} s; stage figure = 8 layers x (step + refresh scaled "
                      f"by k^3 to the layer's factor orders / {FREQ})",
            "non_refresh_params_per_s": params / t_total,
            "refresh_step_s_one_2560_matrix": t_refresh,
            "refresh_s_one_layer_extrapolated": refresh_layer_s,
            "stage_ms_per_step_extrapolated": 1e3 * stage_s,
            "oracle_householder_qr_order_1024_s": t_house}


def counter_traffic(workload_name, kernel):
    """HBM bytes per launch of the dominant kernel, from the hardware-counter runs summarised in
    profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size).  Counters cannot be
    read from inside this process; the value is the one measured for the library at the commit the
    file names ("counted_at"), by the commands that file lists.  (None, None) when no such measurement exists."""
    if workload_name != "stage3b":
        return None, None
    name = "gemm_bf16_mfma_stage3b_hbm_traffic.txt" if "bf16" in kernel else "gemm_f32_mfma_stage3b_hbm_traffic.txt"
    value, stamp = None, None
    base = kernel.replace(",adam", "")      # the fused-Adam launches are the same kernel symbol family
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("traffic_bytes_per_launch") and f"[{base}]" in line:
                value = float(line.rsplit("=", 1)[1])
            if line.startswith("counted_at"):
                stamp = line.split(":", 1)[1].strip()
    except OSError:
        pass
    return value, (f"profiles/{name}; {stamp}" if stamp else f"profiles/{name}")


def run_mode(B, BasisRotationAdam, torch, params, ring, math, warmup, steps, freq=FREQ, **hparams):
    """Times `steps` optimizer steps in one math mode on copies of the parameters; returns
    (elapsed seconds, profile entries, optimizer)."""
    work = [p.clone() for p in params]
    grad_dtype = hparams.pop("grad_dtype", None)
    opt = BasisRotationAdam(work, freq=freq, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, math=MATH[math],
                            grad_dtype=grad_dtype, **hparams)
    torch.cuda.synchronize()
    t = 0
    for _ in range(warmup):
        t += 1
        opt.step(ring[t % (TAU + 1)])          # the ring hands over the slot filled tau steps ago
    torch.cuda.synchronize()
    B.br_profile_begin(opt.ctx)
    t0 = time.perf_counter()
    for _ in range(steps):
        t += 1
        opt.step(ring[t % (TAU + 1)])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = B.br_profile_end(opt.ctx)
    return elapsed, prof, opt


def stream_ceiling(torch, dev):
    """What this machine's memory system sustains for a 2-read 1-write stream (c = a + b on 1 GiB arrays, a library
    elementwise kernel), measured here: the ceiling next to which the step's elementwise kernels are judged, beside
    the 8 TB/s datasheet figure."""
    n = 1 << 28
    a = torch.ones(n, dtype=torch.float32, device=dev)
    b = torch.ones(n, dtype=torch.float32, device=dev)
    c = torch.empty_like(a)
    for _ in range(3):
        torch.add(a, b, out=c)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        torch.add(a, b, out=c)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 10
    return {"gbs": 3 * 4 * n / (ms * 1e-3) / 1e9, "what": "torch.add(a, b, out=c) on 3 x 1 GiB, HIP events, 10 launches"}


def elementwise_kernels(B, BasisRotationAdam, torch, params, ring):
    """Achieved GB/s (algorithmic bytes / HIP-event time) of the elementwise kernels outside the rotated step:
    plain Adam for unrotated tensors, global-norm clipping (sum of squares, scaling) and Delay Compensation, on the
    stage's 56 tensors (634 M entries)."""
    work = [p.clone() for p in params]
    stale = [p.clone() for p in params]
    grads = [g.clone() for g in ring[0]]
    opt = BasisRotationAdam(work, freq=0, lr=1e-3, rotate=[False] * len(work))
    for timed in (False, True):
        if timed:
            B.br_profile_begin(opt.ctx)
        for _ in range(3):
            for g, src in zip(grads, ring[0]):       # fresh gradients (norm about 250): the scaling pass really scales
                g.copy_(src)
            opt.delay_compensate(grads, stale, 0.5)
            opt.clip_gradients(grads, 1.0)
            opt.accumulate_stats(grads)
            opt.apply(grads)
    prof = B.br_profile_end(opt.ctx)
    factor = float(opt.clip_result()[1])
    assert factor < 1.0, factor
    out = {p["kernel"]: {"gbs": p["bytes"] / (p["ms"] * 1e-3) / 1e9, "frac_of_8tbs": p["bytes"] / (p["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                         "launches": p["launches"]} for p in prof if p["bytes"] > 0 and p["ms"] > 0}
    opt.close()
    return out


def layer2048(B, BasisRotationAdam, torch, dev):
    """One Llama-style layer at hidden 2048, BF16 parameters and gradients with FP32 master weights and state,
    refresh every 10 steps: ms per step in each math mode (2 warm-up + 10 timed steps, one refresh inside)."""
    from paper_2602_03515_amd import synth
    shapes = list(synth.LLAMA_LAYER_2048)
    params, ring = make_inputs(shapes, TAU + 1, seed=3, device=dev)
    params = [p.to(torch.bfloat16).contiguous() for p in params]
    ring = [[g.to(torch.bfloat16).contiguous() for g in slot] for slot in ring]
    n_params = sum(m * n for m, n in shapes)
    out = {"params": n_params, "param_dtype": "bf16", "grad_dtype": "bf16", "refresh_every": FREQ, "steps": 10, "warmup": 2}
    for math in ("f32", "bf16x3", "bf16"):
        el, pr, o = run_mode(B, BasisRotationAdam, torch, params, ring, math, 2, 10, grad_dtype=torch.bfloat16)
        out[math] = {"ms_per_step": 1e2 * el, "params_per_s": n_params * 10 / el, "state_bytes": o.state_bytes}
        o.close()
    return out


def refresh_heavy(B, BasisRotationAdam, torch, dev, params, ring):
    """Refresh-heavy stress: the 56 stage matrices + the 32000 x 2560 embedding shard, unilateral rotation (every
    factor has order 2560), refresh EVERY step with 2 power iterations + one QR, FP32 math: 1 warm-up + 5 timed steps."""
    from paper_2602_03515_amd import synth
    ep, er = make_inputs([synth.EMBEDDING_SHARD], TAU + 1, seed=5, device=dev)
    shapes = list(synth.STAGE_3B) + [synth.EMBEDDING_SHARD]
    all_params = list(params) + ep
    all_ring = [ring[k] + er[k] for k in range(TAU + 1)]
    torch.cuda.reset_peak_memory_stats(dev)
    steps = 5
    el, prof, opt = run_mode(B, BasisRotationAdam, torch, all_params, all_ring, "f32", 1, steps, freq=1,
                             geometry=B.BR_UNILATERAL, power_iters=2)
    qr = next((p for p in prof if p["kernel"].startswith("qr_householder")), None)
    closed = 4 * sum(2 * m * n + 2 * min(m, n) ** 2 for m, n in shapes)
    out = {"params": sum(m * n for m, n in shapes), "ms_per_step": 1e3 * el / steps, "steps": steps, "warmup": 1,
           "qr_per_step": len(shapes), "factor_order": 2560,
           "qr_ms_per_step": qr["ms"] / steps, "qr_per_s": len(shapes) * steps / (qr["ms"] * 1e-3),
           "qr_tflops_nominal": qr["flops"] / (qr["ms"] * 1e-3) / 1e12,
           "state_bytes_closed_form": closed, "state_bytes": opt.state_bytes, "scratch_bytes": opt.scratch_bytes,
           "peak_allocated_bytes": int(torch.cuda.max_memory_allocated(dev)),
           "note": "closed form = 4 (2 mn + 2 min(m,n)^2) per matrix; state_bytes adds the cached rotated moment; peak includes "
                   "parameters, their working copies and the gradient ring"}
    opt.close()
    return out


def issue_factor(kernel):
    """Matrix instructions issued per algorithmic product: 3 and 4 for the hi + lo split kernels."""
    return 3 if kernel.endswith("<3>") else 4 if kernel.endswith("<4>") else 1


def dominant_gemm(prof):
    gemm = [p for p in prof if p["kernel"].startswith("br_gemm")]
    return max(gemm, key=lambda p: p["ms"]) if gemm else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="stage3b")
    ap.add_argument("--math", default="f32", choices=sorted(MATH),
                    help="input precision of the step's contractions: f32 (FP32 MFMA, default), "
                         "bf16x3 (hi+lo BF16 split, same 1e-4 bar), bf16 (2e-2 bar)")
    ap.add_argument("--refresh-math", default="auto", choices=["auto", "f32", "f16x3"],
                    help="arithmetic of the refresh's large products: f32 (FP32 MFMA), f16x3 (hi+lo FP16 split products, FP32 "
                         "accumulation), auto (f32 under --math f32, f16x3 under the BF16 math modes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--single-mode", action="store_true",
                    help="skip the short runs of the other math modes (10 steps each, reported under 'modes') that "
                         "otherwise follow the timed run")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) so that HBM byte counters "
                         "collected by a profiler can be scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (one pipeline stage's share); --gpus must be 1", file=sys.stderr)
        raise SystemExit(2)

    import torch
    from paper_2602_03515_amd import binding as B
    from paper_2602_03515_amd.optimizer import BasisRotationAdam

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        raise SystemExit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    shapes, desc = workload(args.workload)
    n_params = sum(m * n for m, n in shapes)
    params, ring = make_inputs(shapes, TAU + 1, seed=2, device=dev)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    stress = args.workload == "stage3b_emb"
    freq = 1 if stress else FREQ
    extra = {"geometry": B.BR_UNILATERAL, "power_iters": 2} if stress else {}
    extra["refresh_math"] = {"auto": B.BR_REFRESH_AUTO, "f32": B.BR_REFRESH_F32, "f16x3": B.BR_REFRESH_F16X3}[args.refresh_math]
    split_refresh = args.refresh_math == "f16x3" or (args.refresh_math == "auto" and args.math != "f32")
    elapsed, prof, opt = run_mode(B, BasisRotationAdam, torch, params, ring, args.math, args.warmup, args.steps, freq=freq, **extra)

    ms_per_step = 1e3 * elapsed / args.steps
    refreshes = sum(1 for k in range(args.warmup + 1, args.warmup + args.steps + 1) if k % freq == 0)
    dom = dominant_gemm(prof)
    roofline = None
    if dom:
        avg_ms = dom["ms"] / dom["launches"]
        achieved = dom["flops"] / dom["launches"] / (avg_ms * 1e-3) / 1e12
        peak = PEAK_TFLOPS["bf16" if "bf16" in dom["kernel"] else "f32"]
        roofline = {"bound": "mfma", "kernel": dom["kernel"], "achieved": achieved, "peak": peak,
                    "unit": "TFLOP/s", "frac": achieved / peak,
                    "traffic": counter_traffic(args.workload, dom["kernel"])[0],
                    "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE of a separate counter run)",
                    "traffic_source": counter_traffic(args.workload, dom["kernel"])[1],
                    "launches": dom["launches"], "avg_launch_ms": avg_ms}
        issue = issue_factor(dom["kernel"])
        if issue > 1:   # hi + lo split: each algorithmic product is 3 (4) matrix instructions
            roofline["issue_factor"] = issue
            roofline["frac_issued"] = issue * achieved / peak
    breakdown = {p["kernel"]: {"launches": p["launches"], "ms_per_step": p["ms"] / args.steps,
                               "tflops": (p["flops"] / (p["ms"] * 1e-3) / 1e12) if p["ms"] > 0 else None,
                               "gbs": (p["bytes"] / (p["ms"] * 1e-3) / 1e9) if p["ms"] > 0 and p["bytes"] > 0 else None}
                 for p in prof}
    out = {
        "metric": "rotated-optimizer steps/sec per stage (params/s)",
        "value": n_params * args.steps / elapsed,
        "unit": "params/s",
        "steps_per_s": args.steps / elapsed,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.math, "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc}", "params": n_params, "geometry": "unilateral" if stress else "bilateral",
                   "source": "second", "refresh_every": freq, "refreshes_in_timed_region": refreshes,
                   "power_iters": 2 if stress else 1, "delay_tau": TAU, "param_dtype": "f32", "grad_dtype": "f32",
                   "math": {"f32": "fp32 MFMA", "bf16": "bf16 MFMA", "bf16x3": "bf16 MFMA, hi+lo split (3 products)"}[args.math],
                   "refresh_math": "f16 MFMA, hi+lo split (3 products), FP32 accumulation" if split_refresh else "fp32 MFMA",
                   "state_bytes": None, "scratch_bytes": None},
        "roofline": roofline,
        "kernels": breakdown,
    }
    out["config"]["state_bytes"], out["config"]["scratch_bytes"] = opt.state_bytes, opt.scratch_bytes
    # the HBM-bound part of the step: its busiest kernel against the 8 TB/s datasheet figure
    ew = [p for p in prof if p["bytes"] > 0 and p["ms"] > 0]
    if ew:
        e = max(ew, key=lambda p: p["ms"])
        gbs = e["bytes"] / (e["ms"] * 1e-3) / 1e9
        out["roofline_elementwise"] = {"bound": "hbm", "kernel": e["kernel"], "achieved": gbs, "peak": PEAK_HBM_GBS,
                                       "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "launches": e["launches"]}
    if stress:
        # what the refresh-heavy configuration is for: QR throughput and the optimizer state's size
        qr = next((p for p in prof if p["kernel"].startswith("qr_householder")), None)
        orders = [min(m, n) for m, n in shapes]
        closed = 4 * sum(2 * m * n + 2 * min(m, n) ** 2 for m, n in shapes)
        out["refresh"] = {
            "factor_orders": sorted(set(orders)), "qr_per_step": len(orders),
            "qr_ms_per_step": qr["ms"] / args.steps if qr else None,
            "qr_per_s": (len(orders) * args.steps / (qr["ms"] * 1e-3)) if qr else None,
            "qr_tflops_nominal": (qr["flops"] / (qr["ms"] * 1e-3) / 1e12) if qr else None,
            "state_bytes_closed_form": closed, "state_bytes": opt.state_bytes, "scratch_bytes": opt.scratch_bytes,
            "peak_allocated_bytes": int(torch.cuda.max_memory_allocated(dev)),
            "note": "closed form = 4 (2 mn + 2 min(m,n)^2) per matrix: M, S~ and the smaller side's statistic and basis; "
                    "state_bytes adds the cached rotated moment and alignment; peak includes parameters and the gradient ring"}
    del opt
    if not args.single_mode:
        out["modes"] = {}
        for math in sorted(MATH):
            if math == args.math:
                continue
            torch.cuda.empty_cache()
            el, pr, o2 = run_mode(B, BasisRotationAdam, torch, params, ring, math, 1, 10)
            d2 = dominant_gemm(pr)
            ach = d2["flops"] / (d2["ms"] * 1e-3) / 1e12
            pk = PEAK_TFLOPS["bf16" if "bf16" in d2["kernel"] else "f32"]
            out["modes"][math] = {"value": n_params * 10 / el, "unit": "params/s", "ms_per_step": 1e2 * el, "steps": 10,
                                  "warmup": 1, "dominant_kernel": d2["kernel"], "achieved_tflops": ach, "frac": ach / pk,
                                  "frac_issued": issue_factor(d2["kernel"]) * ach / pk,
                                  "state_bytes": o2.state_bytes, "scratch_bytes": o2.scratch_bytes}
            del o2
        if args.math == "f32" and not stress and not split_refresh:
            # the same FP32 step with the refresh's large products as split FP16 products (BR_REFRESH_F16X3)
            torch.cuda.empty_cache()
            el, pr, o2 = run_mode(B, BasisRotationAdam, torch, params, ring, "f32", 1, 10, refresh_math=B.BR_REFRESH_F16X3)
            qr = next((p for p in pr if p["kernel"].startswith("qr_householder")), None)
            lq = next((p for p in pr if p["kernel"].startswith("br_gemm_f16")), None)
            out["modes"]["f32+f16x3_refresh"] = {
                "value": n_params * 10 / el, "unit": "params/s", "ms_per_step": 1e2 * el, "steps": 10, "warmup": 1,
                "what": "BR_MATH_F32 step contractions (FP32 MFMA); A Q and the QR's large updates as hi + lo FP16 split products",
                "qr_region_ms_per_step": qr["ms"] / 10 if qr else None,
                "qr_tflops_nominal": (qr["flops"] / (qr["ms"] * 1e-3) / 1e12) if qr else None,
                "power_product_ms_per_step": lq["ms"] / 10 if lq else None,
                "state_bytes": o2.state_bytes, "scratch_bytes": o2.scratch_bytes}
            del o2
    if not args.single_mode and args.workload == "stage3b":
        out["stream_2r1w"] = stream_ceiling(torch, dev)
        if "roofline_elementwise" in out:
            out["roofline_elementwise"]["frac_of_measured_2r1w_stream"] = (
                out["roofline_elementwise"]["achieved"] / out["stream_2r1w"]["gbs"])
        out["elementwise_kernels"] = elementwise_kernels(B, BasisRotationAdam, torch, params, ring)
        out["layer2048"] = layer2048(B, BasisRotationAdam, torch, dev)
        out["refresh_heavy"] = refresh_heavy(B, BasisRotationAdam, torch, dev, params, ring)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
