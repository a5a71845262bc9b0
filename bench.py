#!/usr/bin/env python3
"""Benchmark of the DVM hot path on one MI355X.

A step is one pass of the whole hot path over the configured workload: every instance of the
dynamic-shape stream is encoded by dvm_encode (host: shape inference, fusion, register allocation,
tile plan, bytecode), consecutive instances are merged eight at a time into one launch by dvm_stack
(temporal stacking), and dvm_run executes each launch (device: the bytecode interpreter), all on one
stream.  Inputs and outputs of all instances are resident in HBM before the timed region.  The same
stream is also run with every instance as its own launch; that figure is reported beside the main one.

Workload (default): fused RMSNorm with learned scale, bf16 in/out with fp32 accumulation,
x = [B, S, 4096] ~ N(0,1), weight ~ N(1, 0.1), eps 1e-6, 200 instances with B uniform in 1..32 and
S uniform in 1..2048, all shapes distinct, drawn from a seed (synthetic data).

Prints ONE JSON line: whole-job throughput in GB/s of algorithmic bytes (one read of every input
element + one write of every output element), the roofline record of the interpreter kernel
(per-launch HIP-event durations on the launch stream), the encode latency per instance, and the
CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# rocprofv3 summaries of this command (kernel trace and the two HBM byte counters) per workload
PROFILE_SUMMARY = {w: f"profiles/dvm_vm_kernel_{w}.md"
                   for w in ("c1_gelu", "c2_rmsnorm", "c3_masked_softmax", "c4_chain", "c5_layers", "layernorm_bf16", "column_sum")}


def measured_traffic(workload: str):
    """HBM bytes per interpreter launch from the committed counter summary (FETCH_SIZE + WRITE_SIZE, each scaled
    by what the same counter reads for a plain copy of known size), or None if there is no such summary."""
    path = os.path.join(ROOT, PROFILE_SUMMARY.get(workload, ""))
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(line.split(":", 1)[1])
    except (OSError, ValueError):
        pass
    return None


def bench_fuser(args, B, gen, W, ctx, dev) -> int:
    """The paper's dynamic control-flow workload (Table 2): (a > b ? 2x : 4x) + y over [b, s, f] with the branch
    decided on the host, issued operator by operator through the streaming fuser (dvm_fuser_*)."""
    import numpy as np
    import torch
    shapes = [sh for sh in gen.if_else_add_shapes(60) if sh[0] * sh[1] * sh[2] <= 2.7e8][: args.instances or None]
    insts = []
    for k, (b, s, f_, flag) in enumerate(shapes):
        x = gen.randn((b, s, f_), gen.BASE_SEED + 7000 + 2 * k, dev)
        y = gen.randn((b, s, f_), gen.BASE_SEED + 7001 + 2 * k, dev)
        insts.append((x, y, torch.empty_like(x), torch.empty_like(x), flag, B.shape_of_tensor(x)))
    torch.cuda.synchronize()
    total_bytes = sum(3 * x.numel() * 4 for x, *_ in insts)
    stream = torch.cuda.current_stream()
    fuser = B.Fuser(ctx, stream.cuda_stream)
    perf = time.perf_counter

    def one_step(events=None, host_us=None):
        for k, (x, y, tmp, out, flag, shp) in enumerate(insts):
            t0 = perf()
            vx = fuser.tensor(x.data_ptr(), "f32", shp)
            vy = fuser.tensor(y.data_ptr(), "f32", shp)
            t = fuser.op("muls", [vx], "f32", tmp.data_ptr(), imm=2.0 if flag else 4.0)
            o = fuser.op("add", [t, vy], "f32", out.data_ptr())
            fuser.release(t)
            if events is not None:
                events[k][0].record(stream)
            fuser.flush()
            if events is not None:
                events[k][1].record(stream)
            for v in (vx, vy, o):
                fuser.release(v)
            if host_us is not None:
                host_us.append((perf() - t0) * 1e6)

    for _ in range(args.warmup):
        one_step()
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in insts] for _ in range(args.steps)]
    host_us = []
    torch.cuda.synchronize()
    t0 = perf()
    for s_ in range(args.steps):
        one_step(evs[s_], host_us)
    torch.cuda.synchronize()
    elapsed = perf() - t0
    kern_ms = [a.elapsed_time(b) for e in evs for (a, b) in e]
    avg_launch_ms = float(np.mean(kern_ms))
    bytes_per_launch = total_bytes / len(insts)
    achieved = bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9
    value = total_bytes * args.steps / elapsed / 1e9
    hu = np.array(host_us)
    st = fuser.stats()
    result = {
        "metric": "achieved HBM GB/s of VM-run fused ops (algorithmic bytes / wall time, encode included)",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "if-else-add (a > b ? 2x : 4x) + y fp32 over [b, s, f] (the paper's Table 2 range, instances up to "
                               "2.7e8 elements), branch taken on the host, operators issued one by one through the streaming fuser",
                   "instances": len(insts)},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "fuser_host_us_per_instance": {"median": round(float(np.median(hu)), 2), "p99": round(float(np.percentile(hu, 99)), 2),
                                       "max": round(float(hu.max()), 2), "mean": round(float(hu.mean()), 2),
                                       "note": "two tensor registrations, two operators, releases, flush (program build, "
                                               "encode, launch), through ctypes"},
        "fuser": st,
        "roofline": {"bound": "hbm", "kernel": "dvm_vm_kernel (bytecode interpreter)", "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "bytes_per_launch": int(bytes_per_launch), "avg_launch_ms": round(avg_launch_ms, 5),
                     "launches": len(kern_ms), "instances_per_launch": 1, "traffic": None},
    }
    if not args.no_cpu_baseline:
        from oracle import interp
        used, worst, cpu_bytes = 0, 0.0, 0
        t_cpu = 0.0
        for (x, y, tmp, out, flag, shp) in insts:
            if x.numel() > 6e7 - used:
                continue
            desc = W.get_program("if_else_add_true" if flag else "if_else_add_false")
            hx, hy = x.cpu().to(torch.float64).numpy(), y.cpu().to(torch.float64).numpy()
            t1 = perf()
            rounded, exact = interp.run(desc, {"x": hx, "y": hy})
            t_cpu += perf() - t1
            ref = rounded[desc.outputs[0][0]]
            got = out.cpu().to(torch.float64).numpy()
            tol = 1e-5 * np.abs(ref) + 1e-5 * interp.row_scale(exact[desc.outputs[0][0]])
            worst = max(worst, float(np.max(np.abs(got - ref) / np.maximum(tol, 1e-300))))
            used += x.numel()
            cpu_bytes += 3 * x.numel() * 4
        result["cpu_baseline"] = {"value": round(cpu_bytes / max(t_cpu, 1e-9) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": f"instances of the same stream with {used} elements in all, {t_cpu:.1f} s of NumPy float64",
                                  "max_err_over_tol_vs_gpu": round(worst, 4)}
        if worst > 1.0:
            print(json.dumps(result))
            return 1
    print(json.dumps(result))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c2_rmsnorm",
                    choices=["c1_gelu", "c2_rmsnorm", "c3_masked_softmax", "c4_chain", "c5_layers", "layernorm_bf16", "if_else_add",
                             "column_sum"])
    ap.add_argument("--instances", type=int, default=0, help="use only the first N instances (0 = the workload's default)")
    ap.add_argument("--stack", type=int, default=0,
                    help="consecutive instances merged into one launch by temporal stacking (default 8, capped by the "
                         "launch's tensor table; 1 = every instance its own launch; config 5 always stacks a layer)")
    ap.add_argument("--stacking", default="", choices=["", "temporal", "spatial"],
                    help="how the parts of a launch share it: one after the other on all workgroups (temporal) or side by "
                         "side on shares of the workgroups (spatial); default temporal (it measured faster on every workload here)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--skip-unstacked", action="store_true",
                    help="leave out the second pass that launches every program on its own (profiler runs use this so "
                         "that the kernel statistics cover the stacked launches only)")
    ap.add_argument("--dump-launches", default="", help="write per-program bytes and mean launch time to this CSV file")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region run a plain 256 MiB device copy (a known-size kernel that scales "
                         "the HBM byte counters of a profiler run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path needs no exchange between devices); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2603_24239_amd import binding as B
    from workloads import gen
    from workloads import programs as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    lib = B.load()          # raises if libdvm.so has not been built: there is no fallback path
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ctx = B.Context(0)
    if args.workload == "if_else_add":
        return bench_fuser(args, B, gen, W, ctx, dev)
    progs = {}

    def program(name):
        if name not in progs:
            progs[name] = (W.get_program(name), B.Program(W.get_program(name)))
        return progs[name]

    # ---- synthetic inputs, resident in HBM -----------------------------------------------------
    # a part is one program applied to one set of tensors; `groups` lists the parts of each launch
    parts = []

    def add_part(name, ins_d, nbytes, shape, outs=None):
        desc, prog = program(name)
        ins = [ins_d[n] for n, _ in desc.inputs]
        if outs is None:
            shapes = [tuple(t.shape) for t in ins]
            full = max(shapes, key=lambda sh: (len(sh), int(np.prod(sh))))
            out_shape = tuple(np.broadcast_shapes(*shapes)) if len(shapes) > 1 else full
            outs_l = [torch.empty(out_shape, dtype=torch.bfloat16 if dt == "bf16" else torch.float32, device=dev)
                      for _, dt in desc.outputs]
            layout = None
        else:
            outs_l = [outs[n] for n, _ in desc.outputs]
            layout = (B.dvm_shape * len(outs_l))(*[B.shape_of_tensor(t) for t in outs_l])
        parts.append({"name": name, "desc": desc, "prog": prog, "ins": ins, "outs": outs_l, "bytes": nbytes, "shape": shape,
                      "shapes": (B.dvm_shape * len(ins))(*[B.shape_of_tensor(t) for t in ins]), "layout": layout})

    fixed_groups = None
    default_budget = 4e8        # elements of the first input the CPU oracle is given (about 10-30 s)
    if args.workload == "c2_rmsnorm":
        shapes = gen.c2_shapes()[: args.instances or None]
        for i, (b, s) in enumerate(shapes):
            add_part("c2_rmsnorm", gen.c2_inputs(b, s, gen.BASE_SEED + 2000 + i, dev), gen.c2_bytes(b, s), (b, s))
        wl = {"workload": "config 2: fused RMSNorm bf16, x[B,S,4096], 200 dynamic instances (B 1..32, S 1..2048)",
              "instances": len(parts), "hidden": 4096, "eps": 1e-6}
    elif args.workload == "layernorm_bf16":
        # the LayerNorm subgraph range of the paper's Table 2 ([b, 8192, h]); the first 24 of the seeded stream
        shapes = gen.layernorm_paper_shapes()[: args.instances or 24]
        for i, (b, s_, h) in enumerate(shapes):
            add_part("layernorm_bf16", gen.layernorm_inputs(b, s_, h, gen.BASE_SEED + 6000 + 3 * i, dev),
                     gen.layernorm_bytes(b, s_, h), (b, s_, h))
        wl = {"workload": "LayerNorm bf16 over [b, 8192, h], b 1..60, h in {1024, 2048, 3072, 4096} (the paper's Table 2 range), eps 1e-5",
              "instances": len(parts)}
    elif args.workload == "column_sum":
        # Table 1's Sum in its general form: [M, size, N] reduced along `size` to [M, 1, N], fp32
        shapes = gen.column_sum_shapes()[: args.instances or None]
        for i, (m, size, n) in enumerate(shapes):
            x = gen.randn((m, size, n), gen.BASE_SEED + 8000 + i, dev)
            add_part("colsum", {"x": x}, gen.column_sum_bytes(m, size, n), (m, size, n),
                     {"s": torch.empty((m, 1, n), dtype=torch.float32, device=dev)})
        wl = {"workload": "sum along the penultimate axis fp32, [M,size,N] -> [M,1,N], 48 dynamic instances "
                          "(M 1..256, size 16..4096, N 512..4096)", "instances": len(parts)}
    elif args.workload == "c4_chain":
        shapes = gen.c4_shapes()[: args.instances or None]
        for i, t in enumerate(shapes):
            add_part("c4_chain", gen.c4_inputs(t, gen.BASE_SEED + 4000 + i, dev), gen.c4_bytes(t), (t,))
        wl = {"workload": "config 4: 12-op transformer non-GEMM chain bf16 over [T,8192], 100 dynamic instances",
              "instances": len(parts), "hidden": 8192}
        default_budget = 2e8
    elif args.workload == "c1_gelu":
        add_part("c1_gelu_erf", gen.c1_inputs(gen.BASE_SEED + 1, dev), 4 * 1000 * 4 * 2 + 2 * 1000 * 4, (4, 1000))
        wl = {"workload": "config 1: gelu(x*a+b) fp32 on [4,1000] (latency-bound)", "instances": 1}
    elif args.workload == "c3_masked_softmax":
        # the first 16 instances of the seeded stream (the whole stream is 185 GB of traffic)
        shapes = gen.c3_shapes()[: args.instances or 16]
        for i, (b, s) in enumerate(shapes):
            add_part("c3_masked_softmax", gen.c3_inputs(b, s, gen.BASE_SEED + 3000 + i, dev), gen.c3_bytes(b, s), (b, s))
        wl = {"workload": "config 3: causal-masked softmax fp32 over [B,32,S,S] (B 1..4, S 128..4096), mask [S,S] broadcast",
              "instances": len(parts)}
        default_budget = 1.5e8
    else:
        # config 5: 64 steps of a 32-layer stack, six programs per layer, T log-normal; one buffer set per
        # step shared by its 32 layers; every layer is one launch (its six programs stacked)
        ctx.set_limits(16, 6)       # parts that share a launch must fit one interpreter variant
        steps_T = gen.c5_steps()[: args.instances or None]
        fixed_groups = []
        for si, T in enumerate(steps_T):
            d = gen.c5_inputs(T, gen.BASE_SEED + 5000 + 100 * si, dev)
            rope_out = torch.empty((T, 32, 128), dtype=torch.bfloat16, device=dev)
            L = T // 8 + 1
            first = len(parts)
            add_part("c5_rmsnorm", d["c5_rmsnorm"], (2 * T * 4096 + 4096) * 2, (T,))
            add_part("c5_rope", d["c5_rope"], 2 * T * 32 * 128 * 2 + 2 * T * 64 * 4, (T,),
                     {"y1": rope_out[..., :64], "y2": rope_out[..., 64:]})
            add_part("c5_softmax", d["c5_softmax"], 2 * 32 * T * L * 2, (T,))
            add_part("c5_residual", d["c5_residual_a"], 3 * T * 4096 * 2, (T,))
            add_part("c5_silu_gate", d["c5_silu_gate"], 3 * T * 14336 * 2, (T,))
            add_part("c5_residual", d["c5_residual_b"], 3 * T * 4096 * 2, (T,))
            layer = list(range(first, first + 6))
            fixed_groups += [layer] * 32
        wl = {"workload": "config 5: 64 steps x 32 layers x {rmsnorm, rope, softmax, residual, silu-gate, residual} bf16, "
                          "T log-normal (median 512, 1..8192); one launch per layer",
              "instances": len(fixed_groups), "steps_of_the_stream": len(steps_T)}
        default_budget = 1.5e8
    torch.cuda.synchronize()

    # ---- launches: lists of part indices -------------------------------------------------------
    enc_cap = 8192
    if fixed_groups is not None:
        groups_idx = fixed_groups
        group = 6
        singles_idx = [[i] for g in fixed_groups for i in g]
    else:
        n_t_part = len(parts[0]["ins"]) + len(parts[0]["outs"])
        max_group = max(1, min(32 // n_t_part, 10))
        # default: eight per launch; config 3's instances are gigabytes each and differ in row length (a stacked
        # launch runs all its parts with the largest tile register size among them), so they stay apart
        # (and a column sum's workgroup and tile register size depend on its shape: one launch each as well)
        default_stack = 1 if args.workload in ("c3_masked_softmax", "column_sum") else 8
        group = max(1, min(args.stack if args.stack > 0 else default_stack, max_group))
        groups_idx = [list(range(lo, min(lo + group, len(parts)))) for lo in range(0, len(parts), group)]
        singles_idx = [[i] for i in range(len(parts))]
    total_bytes = sum(parts[i]["bytes"] for g in groups_idx for i in g)

    def marshal(groups):
        out = []
        for idx in groups:
            tens = [t for i in idx for t in parts[i]["ins"] + parts[i]["outs"]]
            out.append((idx, (C.c_void_p * len(tens))(*[t.data_ptr() for t in tens]), len(tens)))
        return out

    max_parts = max(len(g) for g in groups_idx)
    part_bufs = [C.create_string_buffer(enc_cap) for _ in range(max_parts)]
    part_ptrs = (C.c_void_p * max_parts)(*[C.cast(b, C.c_void_p) for b in part_bufs])
    part_lens = (C.c_size_t * max_parts)()
    stacked = C.create_string_buffer(enc_cap)
    ln = C.c_size_t()
    stream = torch.cuda.current_stream()
    stream_h = C.c_void_p(stream.cuda_stream)
    perf = time.perf_counter

    stacking = args.stacking or "temporal"
    stack_fn = lib.dvm_stack_spatial if stacking == "spatial" else lib.dvm_stack

    def one_step(groups, events=None, enc_us=None):
        """Encode every part, stack the parts of each launch (temporal stacking; a single part is launched
        as it is), run."""
        for k, (idx, ptrs, n_t) in enumerate(groups):
            for j, i in enumerate(idx):
                pt = parts[i]
                t0 = perf()
                st = lib.dvm_encode(ctx._h, pt["prog"]._h, pt["shapes"], len(pt["ins"]), pt["layout"], part_bufs[j], enc_cap,
                                    C.byref(ln), None)
                t1 = perf()
                if st != 0:
                    raise B.DvmError(st, "dvm_encode")
                part_lens[j] = ln.value
                if enc_us is not None:
                    enc_us.append((t1 - t0) * 1e6)
            if len(idx) == 1:
                code, code_len = part_bufs[0], part_lens[0]
            else:
                st = stack_fn(part_ptrs, part_lens, len(idx), stacked, enc_cap, C.byref(ln))
                if st != 0:
                    raise B.DvmError(st, "dvm_stack")
                code, code_len = stacked, ln.value
            if events is not None:
                events[k][0].record(stream)
            st = lib.dvm_run(ctx._h, code, code_len, ptrs, n_t, stream_h)
            if st != 0:
                raise B.DvmError(st, "dvm_run")
            if events is not None:
                events[k][1].record(stream)

    def timed(groups, steps, warmup, enc_us=None):
        for _ in range(warmup):
            one_step(groups)
        evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in groups]
               for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = perf()
        for s in range(steps):
            one_step(groups, evs[s], enc_us)
        torch.cuda.synchronize()
        return perf() - t0, evs

    groups = marshal(groups_idx)
    enc_us = []
    elapsed, all_events = timed(groups, args.steps, args.warmup, enc_us)

    # the same stream with every program as its own launch (no stacking): per-program launch times
    unstacked = not args.skip_unstacked
    if unstacked:
        singles = marshal(singles_idx)
        elapsed1, events1 = timed(singles, args.steps, 1) if group > 1 else (elapsed, all_events)

    if args.calibrate_copy:
        src = torch.empty(256 * 2**20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    ms_per_step = elapsed / args.steps * 1e3
    value = total_bytes * args.steps / elapsed / 1e9
    kern_ms = [a.elapsed_time(b) for evs in all_events for (a, b) in evs]
    avg_launch_ms = float(np.mean(kern_ms))
    bytes_per_launch = total_bytes / len(groups)
    achieved = bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9
    large = single = None
    if unstacked:
        one_ms = [float(np.mean([events1[s][k][0].elapsed_time(events1[s][k][1]) for s in range(args.steps)]))
                  for k in range(len(singles_idx))]
        one_bytes = [parts[g[0]]["bytes"] for g in singles_idx]
        if args.dump_launches:
            with open(args.dump_launches, "w") as f:
                f.write("launch,program,shape,bytes,mean_launch_us,GBps\n")
                for k, g in enumerate(singles_idx):
                    pt = parts[g[0]]
                    f.write(f"{k},{pt['name']},{'x'.join(map(str, pt['shape']))},{pt['bytes']},{one_ms[k] * 1e3:.2f},"
                            f"{pt['bytes'] / one_ms[k] / 1e6:.1f}\n")
        # the large launches (beyond the 256 MB Infinity Cache), each program on its own
        big = [k for k, b in enumerate(one_bytes) if b >= 256e6]
        if big:
            large = {"launches": len(big),
                     "GBps": round(sum(one_bytes[k] for k in big) / sum(one_ms[k] for k in big) / 1e6, 1)}
        single = {"value": round(total_bytes * args.steps / elapsed1 / 1e9, 2), "unit": "GB/s",
                  "ms_per_step": round(elapsed1 / args.steps * 1e3, 4),
                  "avg_launch_ms": round(float(np.mean(one_ms)), 5),
                  "achieved": round(sum(one_bytes) / sum(one_ms) / 1e6, 2),
                  "note": "same stream, every program its own launch, HIP events around every launch"}
    enc = np.array(enc_us)

    wl["instances_per_launch"] = group
    wl["stacking"] = stacking if group > 1 else "none"
    result = {
        "metric": "achieved HBM GB/s of VM-run fused ops (algorithmic bytes / wall time, encode included)",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic", "config": wl,
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "encode_us_per_instance": {"median": round(float(np.median(enc)), 2), "p99": round(float(np.percentile(enc, 99)), 2),
                                   "max": round(float(enc.max()), 2), "note": "dvm_encode timed through ctypes"},
        "large_instances": large, "one_launch_per_instance": single,
        "roofline": {"bound": "hbm", "kernel": "dvm_vm_kernel (bytecode interpreter)", "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "bytes_per_launch": int(bytes_per_launch), "avg_launch_ms": round(avg_launch_ms, 5),
                     "launches": len(kern_ms), "instances_per_launch": group,
                     "traffic": measured_traffic(args.workload) if not args.instances and not args.stack and not args.stacking else None},
    }

    # ---- the CPU oracle on a bounded sample of the same workload (a baseline, not the target) -----
    if not args.no_cpu_baseline:
        from oracle import interp
        budget = default_budget
        # distinct parts in stream order while they fit the budget (elements of the first input); if none
        # fits, the leading rows of the first part (its rows are independent and its other inputs are vectors)
        used, sample, seen = 0.0, [], set()
        for g in groups_idx:
            for i in g:
                n_el = parts[i]["ins"][0].numel()
                if i in seen or n_el > budget - used:
                    continue
                seen.add(i)
                sample.append((i, None))
                used += n_el
            if len(sample) >= 40 or used >= 0.9 * budget:
                break
        if not sample:
            x = parts[0]["ins"][0]
            sample.append((0, max(1, int(budget // x.shape[-1]))))
            used = sample[0][1] * x.shape[-1]

        def head_rows(t, lead, n):
            """The first n rows of a tensor with the full leading shape; broadcast vectors stay whole."""
            if n is None or t.dim() < 2 or tuple(t.shape[:-1]) != lead:
                return t
            return t.reshape(-1, t.shape[-1])[:n]
        host_inputs = []
        for i, n in sample:
            pt = parts[i]
            lead = tuple(pt["ins"][0].shape[:-1])
            host_inputs.append({nm: head_rows(t, lead, n).detach().cpu().to(torch.float64).numpy()
                                for (nm, _), t in zip(pt["desc"].inputs, pt["ins"])})
        t0 = perf()
        refs = [interp.run(parts[i]["desc"], hi) for (i, _), hi in zip(sample, host_inputs)]
        cpu_s = perf() - t0
        cpu_bytes = sum(parts[i]["bytes"] * (1.0 if n is None else n / (parts[i]["ins"][0].numel() // parts[i]["ins"][0].shape[-1]))
                        for i, n in sample)
        # the same sample doubles as an end-to-end check of the benchmarked path
        worst = 0.0
        for (i, n), (rounded, exact) in zip(sample, refs):
            pt = parts[i]
            for (nm, dt), out_t in zip(pt["desc"].outputs, pt["outs"]):
                got = out_t.detach().cpu().to(torch.float64).numpy()
                ref = rounded[nm]
                if n is not None:
                    got = got.reshape(-1, got.shape[-1])[:n]
                    ref = ref.reshape(-1, ref.shape[-1])
                rtol = 2e-2 if dt == "bf16" else 1e-4
                scale = np.broadcast_to(interp.row_scale(exact[nm]).reshape(ref.shape[:-1] + (1,)), ref.shape)
                tol = rtol * np.abs(ref) + rtol * scale
                fin = np.isfinite(ref)
                worst = max(worst, float(np.max(np.where(fin, np.abs(got - ref) / np.maximum(tol, 1e-300), 0.0))))
        result["cpu_baseline"] = {"value": round(cpu_bytes / cpu_s / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": f"{len(sample)} programs (or their leading rows) of the same stream, "
                                            f"{int(used)} elements of their first inputs, "
                                            f"{cpu_s:.1f} s of NumPy float64 per-op evaluation",
                                  "max_err_over_tol_vs_gpu": round(worst, 4)}
        if worst > 1.0:
            print(f"bench.py: GPU output differs from the oracle on the sample (x{worst:.3g} of tolerance)", file=sys.stderr)
            print(json.dumps(result))
            return 1
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
