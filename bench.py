#!/usr/bin/env python3
"""Benchmark of the 4-bit AdamW step on one MI355X.

A "step" is one pass of the whole hot path over every tensor of the workload: for each quantized
tensor the two-kernel 4-bit step (decompress, Adam rule, parameter update, compress), for each small
tensor the fp32-state AdamW kernel.  All inputs are synthetic, seeded and resident in HBM before the
timed region starts.  Prints ONE JSON line (see the keys at the bottom).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c5_llama_7b] [--no-cpu-baseline]

With --second-moment b128 every quantized tensor is taken flat and its second moment is compressed
block-wise (what the method uses for 1-dimensional and flattened parameters): the step is then one
kernel that touches every byte once.  The default (rank1) is the configuration the headline metric
is quoted on.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
# Algorithmic bytes per quantized parameter (every stream touched once per kernel):
#   pass 1: param read+write 8, grad 4 or 2, m codes read+write 1, v codes read 0.5, block scales
#           read+write 8/128
#   pass 2: grad 4 or 2 again, v codes read+write 1
def bytes_per_param(bf16: bool):
    g = 2.0 if bf16 else 4.0
    p1 = 8.0 + g + 1.0 + 0.5 + 8.0 / 128.0
    p2 = g + 1.0
    return p1, p2


# block-wise second moment, one pass: param read+write 8, grad 4 or 2, both moments' codes read+write 2,
# both moments' block scales read+write 16/128
def bytes_per_param_b128(bf16: bool):
    return 8.0 + (2.0 if bf16 else 4.0) + 2.0 + 16.0 / 128.0


# factorized second moment, two passes.  Update pass: param read+write 8, grad 4 or 2, m codes read+write 1, block
# scales read+write 8/128.  Statistics pass: grad 4 or 2.
def bytes_per_param_factor(bf16: bool):
    g = 2.0 if bf16 else 4.0
    return 8.0 + g + 1.0 + 8.0 / 128.0, g



class Workload:
    """One synthetic parameter set resident on the device, with the closure that runs one optimizer step over it."""
    pass


def build_workload(config, second_moment, optimizer, grad_dtype, launch, seed, deterministic=False):
    import torch
    import paper_2309_01507_amd as lpmm
    import workloads

    dev = torch.device("cuda:0")
    specs = workloads.param_set(config)
    bf16 = workloads.GRAD_BF16[config] if grad_dtype == "config" else grad_dtype == "bf16"
    recipe = workloads.GRAD_RECIPE[config]
    lr, b1, b2, eps, wd = 1e-3, 0.9, 0.999, 1e-8, 0.01

    # ---- synthetic workload, generated on the device ------------------------------------------------
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    n_grad_sets = 2                              # the timed steps alternate between two gradient sets
    tensors = []
    max_rc = 2
    for tid, sp in enumerate(specs):
        p = torch.randn(sp.numel, generator=gen, device=dev, dtype=torch.float32) * 0.02
        if recipe == "col_lognormal":
            sigma = 1e-3 * torch.exp(torch.randn(sp.cols, generator=gen, device=dev))
        gs = []
        for k in range(n_grad_sets):
            z = torch.randn(sp.rows, sp.cols, generator=gen, device=dev, dtype=torch.float32)
            if recipe == "col_lognormal":
                z *= sigma[None, :]
            elif recipe == "iid":
                z *= 1e-3
            else:                                # outlier_sparse (config 3)
                z *= 1e-4
                hot_r = torch.randperm(sp.rows, generator=gen, device=dev)[:max(1, sp.rows // 100)]
                hot_c = torch.randperm(sp.cols, generator=gen, device=dev)[:max(1, sp.cols // 200)]
                z[hot_r, :] *= 1e3
                z[:, hot_c] *= 1e3
                zero = torch.rand(sp.rows, generator=gen, device=dev) < 0.9
                z[zero, :] = 0.0
            gs.append(z.reshape(-1).to(torch.bfloat16) if bf16 else z.reshape(-1).contiguous())
            del z
        if optimizer == "sgdm":
            tensors.append(("q", sp, p, gs, lpmm.new_state_sgdm(sp.numel, dev)) if sp.quantized else
                           ("f", sp, p, gs, torch.zeros(sp.numel, device=dev)))
        elif sp.quantized and second_moment == "b128":
            tensors.append(("q", sp, p, gs, lpmm.new_state_b128(sp.numel, dev)))
        elif sp.quantized:
            st = (lpmm.new_state_factor if second_moment == "factor" else lpmm.new_state)(sp.rows, sp.cols, dev)
            max_rc = max(max_rc, sp.rows + sp.cols)
            tensors.append(("q", sp, p, gs, st))
        else:
            m = torch.zeros(sp.numel, device=dev)
            v = torch.zeros(sp.numel, device=dev)
            tensors.append(("f", sp, p, gs, (m, v)))
    lpmm.ensure_init(max_rc)
    torch.cuda.synchronize()

    sgdm = optimizer == "sgdm"
    b128 = second_moment == "b128" and not sgdm
    factor = second_moment == "factor" and not sgdm
    momentum = 0.9
    if sgdm:
        step4 = lpmm.lpmm_sgdm4_step_bf16g if bf16 else lpmm.lpmm_sgdm4_step
    elif factor:
        step4 = lpmm.lpmm_adamw4_factor_step_bf16g if bf16 else lpmm.lpmm_adamw4_factor_step
    elif b128:
        step4 = lpmm.lpmm_adamw4_b128_step_bf16g if bf16 else lpmm.lpmm_adamw4_b128_step
    else:
        step4 = lpmm.lpmm_adamw4_step_bf16g if bf16 else lpmm.lpmm_adamw4_step

    # one plan per gradient set (a plan refers to its buffers by address)
    def make_plans():
        out = []
        for k in range(n_grad_sets):
            if sgdm:
                descs = [lpmm.make_desc_sgdm(p, gs[k], st, sp.numel) for kind, sp, p, gs, st in tensors]
            else:
                det = lambda sp: deterministic and factor and sp.quantized and sp.cols % 128 == 0
                descs = [lpmm.make_desc(p, gs[k], st, sp.rows, sp.cols, deterministic=det(sp)) for kind, sp, p, gs, st in tensors]
            out.append(lpmm.new_plan(descs, 1 if bf16 else 0, dev))
        return out

    plans = make_plans() if launch == "multi" else []

    def one_step(t, use=None):
        k = t % n_grad_sets
        if plans:
            pl = (use or plans)[k]
            if sgdm:
                lpmm.lpmm_sgdm4_step_multi(pl, lr, momentum)
            else:
                lpmm.lpmm_adamw4_step_multi(pl, lr, b1, b2, eps, wd, t)
            return
        for kind, sp, p, gs, st in tensors:
            if sgdm:
                if kind == "q":
                    step4(p, gs[k], st, lr, momentum)
                else:
                    lpmm.lpmm_sgdm32_step(p, gs[k], st, sp.numel, 1 if bf16 else 0, lr, momentum)
            elif kind == "q":
                step4(p, gs[k], st, lr, b1, b2, eps, wd, t)
            else:
                lpmm.lpmm_adamw32_step(p, gs[k], st[0], st[1], sp.numel, 1 if bf16 else 0, lr, b1, b2, eps,
                                       wd, t)

    def release():
        for pl in plans:
            lpmm.lpmm_adamw4_plan_release(pl)

    wl = Workload()
    wl.specs, wl.tensors, wl.plans, wl.one_step, wl.release = specs, tensors, plans, one_step, release
    wl.make_plans = make_plans
    wl.bf16, wl.recipe, wl.sgdm, wl.b128, wl.factor = bf16, recipe, sgdm, b128, factor
    wl.n_params = sum(sp.numel for sp in specs)
    wl.n_quant = sum(sp.numel for sp in specs if sp.quantized)
    wl.hyper = (lr, b1, b2, eps, wd, momentum)
    # bp1: the recorded (dominant) kernel, bp2: the other pass
    wl.bp1, wl.bp2 = ((bytes_per_param_b128(bf16), 0.0) if b128 else bytes_per_param_factor(bf16) if factor
                      else (bytes_per_param_factor(bf16)[0], 0.0) if sgdm    # param 8, grad, m codes 1, block scales 8/128
                      else bytes_per_param(bf16))
    n_small = wl.n_params - wl.n_quant
    wl.small_bytes = ((16.0 if sgdm else 24.0) + (2.0 if bf16 else 4.0)) * n_small   # fp32 states: p, m (, v) read+write, g read
    return wl


def time_steps(wl, steps, warmup, t0=0):
    """`warmup` untimed steps, then exactly `steps` steps between two device synchronizations; returns (seconds, t)."""
    import torch
    t = t0
    for _ in range(warmup):
        t += 1
        wl.one_step(t)
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    for _ in range(steps):
        t += 1
        wl.one_step(t)
    torch.cuda.synchronize()
    return time.perf_counter() - c0, t


# The other configurations and variants, timed after the headline leg (outside its timed region) and reported under
# "secondary": (workload, second moment, optimizer).
SECONDARY = [("c1_single_1024", "rank1", "adamw"), ("c2_bert_base", "rank1", "adamw"),
             ("c3_outlier_32000x4096", "rank1", "adamw"), ("c4_gpt2_medium", "rank1", "adamw"),
             ("c5_llama_7b", "b128", "adamw"), ("c5_llama_7b", "factor", "adamw"), ("c5_llama_7b", "b128", "sgdm")]


def secondary_leg(config, second_moment, optimizer, seed):
    import gc
    import torch
    wl = build_workload(config, second_moment, optimizer, "config", "multi", seed)
    probe, t = time_steps(wl, 3, 3)                        # sizes the timed run: about 0.2 s, 20 to 2000 steps
    steps = int(min(2000, max(20, 0.2 / max(probe / 3, 1e-6))))
    elapsed, t = time_steps(wl, steps, 0, t)
    per_step = elapsed / steps
    step_bytes = (wl.bp1 + wl.bp2) * wl.n_quant + wl.small_bytes
    out = {"workload": config,
           "variant": ("sgdm, flattened, one pass" if wl.sgdm else "block-wise second moment, flattened, one pass" if wl.b128
                       else "factorized second moment, two passes" if wl.factor else "rank-1/Linear, two passes"),
           "grad_dtype": "bf16" if wl.bf16 else "f32", "params": wl.n_params, "steps": steps,
           "ms_per_step": round(per_step * 1e3, 4), "params_per_s": round(wl.n_params / per_step, 1),
           "bytes_per_param": wl.bp1 + wl.bp2, "hbm_gbps": round(step_bytes / per_step / 1e9, 1),
           "hbm_frac": round(step_bytes / per_step / 1e9 / HBM_PEAK_GBPS, 4)}
    wl.release()
    del wl
    gc.collect()
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c5_llama_7b")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip what is timed after the headline leg: the other configurations and variants, and the serial "
                         "leg behind roofline.alone")
    ap.add_argument("--grad-dtype", choices=["config", "bf16", "f32"], default="config",
                    help="override the gradient type of the configuration (experiments)")
    ap.add_argument("--second-moment", choices=["rank1", "b128", "factor"], default="rank1",
                    help="rank1: rank-1/Linear second moment of 2-D tensors (two passes, the headline "
                         "configuration); b128: every tensor flat with a block-wise second moment (one pass); "
                         "factor: row / column statistics instead of a per-element second moment (two passes)")
    ap.add_argument("--optimizer", choices=["adamw", "sgdm"], default="adamw",
                    help="adamw: the 4-bit AdamW step (the headline metric); sgdm: SGD with momentum and 4-bit "
                         "momentum (App. E Alg. 2), every tensor flat, one pass")
    ap.add_argument("--deterministic", action="store_true",
                    help="with --second-moment factor: row / column sums in a fixed order instead of float atomics")
    ap.add_argument("--launch", choices=["multi", "per-tensor"], default="multi",
                    help="multi: one plan, pass 1 / pass 2 of neighbouring tensor groups share launches; "
                         "per-tensor: two launches per quantized tensor")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2309_01507_amd as lpmm
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    lpmm.lib()                                   # fail loudly if lpmm4.so is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = build_workload(args.config, args.second_moment, args.optimizer, args.grad_dtype, args.launch, args.seed,
                        args.deterministic)
    specs, tensors, plans, one_step = wl.specs, wl.tensors, wl.plans, wl.one_step
    bf16, recipe, sgdm, b128, factor = wl.bf16, wl.recipe, wl.sgdm, wl.b128, wl.factor
    n_params, n_quant = wl.n_params, wl.n_quant
    lr, b1, b2, eps, wd, momentum = wl.hyper

    # ---- warm-up, then the timed region ---------------------------------------------------------------
    t = 0
    for _ in range(args.warmup):
        t += 1
        one_step(t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        t += 1
        one_step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    value = n_params / (elapsed / args.steps)

    # ---- the same K steps again with HIP events around every launch of the step -------------------------
    bp1, bp2, small_bytes = wl.bp1, wl.bp2, wl.small_bytes
    one_pass = b128 or sgdm
    n_q_tensors = sum(1 for x in tensors if x[0] == "q")
    n_tensors, has_plans = len(tensors), bool(plans)
    lpmm.lpmm_profile_begin(max(n_q_tensors, 64) * args.steps)
    for _ in range(args.steps):
        t += 1
        one_step(t)
    torch.cuda.synchronize()
    p1_ms, p2_ms, n_calls = lpmm.lpmm_profile_end()
    launches = max(n_calls, 1)
    if factor and not plans:
        p1_ms, p2_ms = p2_ms, p1_ms          # per tensor the statistics pass is recorded first; the update pass dominates
    if plans:
        # the recorded launches are the pass-1 kernels (pass 1 of a tensor group plus the fp32-state
        # tensors); pass 2 of the previous group runs beside them on the plan's second stream
        # (a factorized plan's recorded launches are its update passes; its launches run one after the other on the
        # caller's stream, and the fp32-state tensors ride with the statistics passes)
        bytes_per_launch = (bp1 * n_quant + (0.0 if factor else small_bytes)) * args.steps / launches
        avg_ms = p1_ms / launches
        achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
        roofline = {
            "bound": "hbm", "kernel": ("sgdm_phase_kernel (the whole step)" if sgdm else
                                       "phase_kernel<roles=3> (the whole block-wise step)" if b128 else
                                       "factor_phase_kernel<roles=2> (update pass)" if factor else
                                       "phase_kernel<roles=1> (pass 1)"),
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
            "bytes_per_param": bp1, "launches": n_calls, "avg_launch_ms": round(avg_ms, 5),
            "bytes_per_launch": round(bytes_per_launch),
            "traffic_source": None,
            "note": ("one pass: this kernel is the whole step" if one_pass else
                     "the statistics pass (%.1f B/param) is a launch of its own before it on the same stream; "
                     "whole-step figures are in config" % bp2 if factor else
                     "pass 2 of the neighbouring tensor group (%.1f B/param) runs concurrently and shares "
                     "the bandwidth; whole-step figures are in config" % bp2),
        }
        if not one_pass and not factor and not args.no_secondary:
            # The same steps once more with every launch on the caller's stream, one after the other (plans built
            # under LPMM_MULTI_STREAMS=0): the dominant kernel's rate when it has the chip to itself.  The step as a
            # whole is slower that way, which is why the timed region above overlaps the passes.
            os.environ["LPMM_MULTI_STREAMS"] = "0"
            try:
                serial = wl.make_plans()
            finally:
                del os.environ["LPMM_MULTI_STREAMS"]
            for _ in range(2):
                t += 1
                one_step(t, serial)
            torch.cuda.synchronize()
            lpmm.lpmm_profile_begin(max(n_q_tensors, 64) * args.steps)
            c0 = time.perf_counter()
            for _ in range(args.steps):
                t += 1
                one_step(t, serial)
            torch.cuda.synchronize()
            serial_ms = (time.perf_counter() - c0) * 1e3 / args.steps
            s1_ms, _, s_calls = lpmm.lpmm_profile_end()
            for pl in serial:
                lpmm.lpmm_adamw4_plan_release(pl)
            if s_calls == n_calls and s1_ms > 0:
                alone = bytes_per_launch / (s1_ms / s_calls * 1e-3) / 1e9
                roofline["alone"] = {"achieved": round(alone, 1), "frac": round(alone / HBM_PEAK_GBPS, 4),
                                     "avg_launch_ms": round(s1_ms / s_calls, 5), "ms_per_step": round(serial_ms, 4),
                                     "note": "same kernels and tiles, every launch on the caller's stream one after "
                                             "the other: this kernel with the chip to itself (events included in the step time)"}
        # HBM bytes per launch measured offline with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/)
        tpath = os.path.join(ROOT, "profiles", "traffic_phase_kernel_%s%s.json" % (args.config, "_sgdm" if sgdm else "_b128" if b128 else "_factor" if factor else ""))
        if os.path.exists(tpath):
            tr = json.load(open(tpath))
            if tr.get("launches_per_step") == n_calls // max(args.steps, 1):
                roofline["traffic"] = tr["hbm_bytes_per_launch"]
                roofline["traffic_source"] = "profiles/" + os.path.basename(tpath)
    else:
        p1_avg_ms = p1_ms / launches
        p1_bytes_per_launch = bp1 * n_quant * args.steps / launches
        achieved = p1_bytes_per_launch / (p1_avg_ms * 1e-3) / 1e9
        roofline = {
            "bound": "hbm", "kernel": "sgdm4_kernel" if sgdm else "b128_kernel" if b128 else "factor_update_fast" if factor else "pass1_fast",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
            "bytes_per_param": bp1, "launches": n_calls, "avg_launch_ms": round(p1_avg_ms, 5),
            "bytes_per_launch": round(p1_bytes_per_launch),
            ("statistics_pass" if factor else "pass2"): {"bytes_per_param": bp2, "avg_launch_ms": round(p2_ms / launches, 5),
                      "achieved": round(bp2 * n_quant * args.steps / max(p2_ms, 1e-9) / 1e6, 1)},
        }

    # ---- CPU baseline: the oracle as it stands, one thread, on a bounded sample of the workload -----------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        big = max((sp for sp in specs if sp.quantized), key=lambda s: s.numel)
        rows = min(big.rows, max(1, (24 << 20) // big.cols))        # about 25 M parameters of that tensor
        cols = big.cols
        w = workloads.weights(args.seed, 0, rows, cols).reshape(-1)
        st = (oracle.state_zero_sgdm(rows * cols) if sgdm else oracle.state_zero_b128(rows * cols) if b128
              else oracle.state_zero_factor(rows, cols) if factor else oracle.state_zero(rows, cols))
        if sgdm:
            cpu_step = lambda w_, g_, st_, hp_, s_: oracle.sgdm4_step(w_, g_, st_, lr, momentum)
        else:
            cpu_step = oracle.adamw4_b128_step if b128 else oracle.adamw4_factor_step if factor else oracle.adamw4_step
        hp = oracle.Hyper(lr, b1, b2, eps, wd)
        n_cpu_steps = 20
        gs = [workloads.grads(args.seed, 0, s, rows, cols, recipe, bf16).reshape(-1) for s in (1, 2)]
        c0 = time.perf_counter()
        for s in range(1, n_cpu_steps + 1):
            cpu_step(w, gs[s % 2], st, hp, s)
        cdt = time.perf_counter() - c0
        cpu = {"value": round(rows * cols * n_cpu_steps / cdt, 1), "unit": "params/s", "cores": 1,
               "kind": "oracle",
               "sample": f"{n_cpu_steps} steps on the first {rows} rows of '{big.name}' ({rows}x{cols}, "
                         f"{rows * cols} params), {cdt:.1f} s; host has {os.cpu_count()} logical cpus"}

    # For scale: what a plain device-to-device copy reaches on this machine (torch's copy kernel, 1 GiB read + 1 GiB
    # written per call), outside every timed region above.
    copy_gbps = None
    try:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbps = round(10 * 2.0 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        del src, dst
    except RuntimeError:
        pass

    # ---- the other configurations and variants, for the record (after and outside the headline's timed region) ----
    secondary = None
    if not args.no_secondary and args.config == "c5_llama_7b" and args.second_moment == "rank1" and not sgdm \
            and args.launch == "multi" and args.grad_dtype == "config":
        import gc
        wl.release()
        del wl, specs, tensors, plans, one_step
        gc.collect()
        torch.cuda.empty_cache()
        secondary = []
        for cfg, sm, opt in SECONDARY:
            try:
                secondary.append(secondary_leg(cfg, sm, opt, args.seed))
            except Exception as e:            # a failing side leg must not take the headline line with it
                secondary.append({"workload": cfg, "variant": sm + "/" + opt, "error": repr(e)[:200]})

    total_gbps = ((bp1 + bp2) * n_quant + small_bytes) / (elapsed / args.steps) / 1e9
    # the same roofline for all kernels of a step together (they overlap on two streams, so a single kernel's
    # duration includes the slow-down from its neighbour): algorithmic bytes of the step / wall time of the step
    roofline["whole_step"] = {"achieved": round(total_gbps, 1), "frac": round(total_gbps / HBM_PEAK_GBPS, 4),
                              "bytes_per_param": bp1 + bp2, "ms": round(ms_per_step, 4)}
    roofline["plain_copy_gbps_on_this_box"] = copy_gbps
    # every stream touched once (what a single pass would move): param 8, grad, codes 2, block scales and,
    # for the rank-1 form, one more float per 128 elements standing in for the row / column maxima
    floor_bpp = 8.0 + (2.0 if bf16 else 4.0) + (1.0 if factor or sgdm else 2.0) + (16.0 if b128 else 8.0) / 128.0
    floor_gbps = (floor_bpp * n_quant + small_bytes) / (elapsed / args.steps) / 1e9
    if has_plans:
        kernels_per_step = (n_calls // max(args.steps, 1)) * (1 if one_pass else 2)     # as many A as B launches
    else:
        kernels_per_step = n_q_tensors * (1 if one_pass else 2) + (n_tensors - n_q_tensors)
    out = {
        "metric": "params updated/sec per 4-bit SGDM step" if sgdm else "params updated/sec per 4-bit AdamW step", "value": round(value, 1), "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.config, "tensors": n_tensors, "params": n_params,
                   "quantized_params": n_quant, "grad_dtype": "bf16" if bf16 else "f32",
                   "second_moment": "none (SGD with momentum, App. E Alg. 2), flattened tensors, one pass" if sgdm
                   else "block-wise B128/Linear on flattened tensors, one pass" if b128
                   else "factorized (row and column statistics), two passes" if factor
                   else "rank-1/Linear, two passes",
                   "grad_recipe": recipe,
                   "launch": (("multi-tensor plan, %d launches per step" if one_pass else
                               "multi-tensor plan, %d update launches per step, each behind its statistics launch "
                               "on the caller's stream" if factor else
                               "multi-tensor plan, %d pass-1 launches per step on the caller's stream, "
                               "pass 2 on a second stream") % (n_calls // max(args.steps, 1)))
                   if has_plans else "per-tensor, %d kernel%s per quantized tensor" % ((1, "") if one_pass else (2, "s")),
                   "kernels_per_step": kernels_per_step,
                   "hbm_gbps_one_touch_floor": round(floor_gbps, 1),
                   ("hbm_gbps_one_pass_model" if one_pass else "hbm_gbps_two_pass_model"): round(total_gbps, 1),
                   ("hbm_frac_one_pass_model" if one_pass else "hbm_frac_two_pass_model"):
                       round(total_gbps / HBM_PEAK_GBPS, 4)},
        "roofline": roofline, "cpu_baseline": cpu, "secondary": secondary,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
