#!/usr/bin/env python3
"""Benchmark of the DVM hot path on one MI355X.

A step is one pass of the whole hot path over the configured workloads: every instance of a
dynamic-shape stream is encoded by dvm_encode (host: shape inference, fusion, register allocation, tile
plan, bytecode), consecutive instances are merged into one launch by dvm_stack (temporal stacking), and
dvm_run executes each launch (device: the bytecode interpreter), all on one stream.  Inputs and outputs
of a stream are resident in HBM before its timed region starts.

Default (`--workload suite`): the four dynamic streams of the benchmark configuration, one after the
other (they do not fit the device together): config 2 (RMSNorm bf16, 200 instances), config 3 (causal
masked softmax fp32, all 50 instances), config 4 (12-op chain bf16, 100 instances) and config 5 (64 steps
of a 32-layer stack), plus the latency of config 1.  The headline `value` and the `roofline` record are
the aggregate over the large memory-bound configs 2-4; `per_config` holds every stream's own figures.
`--workload <name>` runs one stream alone (the committed rocprofv3 summaries are made that way).

Prints ONE JSON line: throughput in GB/s of algorithmic bytes (one read of every input element + one
write of every output element), the roofline record of the interpreter kernel (per-launch HIP-event
durations on the launch stream), the copy-kernel ceiling measured in the same job, the encode latency per
instance measured inside the library (dvm_encode_timed), and the CPU oracle timed on a bounded sample of
the same workloads on all host cores and on one.
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
SUITE = ["c2_rmsnorm", "c3_masked_softmax", "c4_chain", "c5_layers"]
LARGE_CLASS = ["c2_rmsnorm", "c3_masked_softmax", "c4_chain"]
ALL_WORKLOADS = ["c1_gelu", "c2_rmsnorm", "c3_masked_softmax", "c4_chain", "c5_layers", "layernorm_bf16", "if_else_add", "column_sum"]

# rocprofv3 summaries (kernel trace and the two HBM byte counters) of `bench.py --workload <name>`
PROFILE_SUMMARY = {w: f"profiles/dvm_vm_kernel_{w}.md" for w in ALL_WORKLOADS}


def measured_traffic_ratio(workload: str):
    """HBM bytes / algorithmic bytes of the interpreter launches of a workload, from the committed counter summary
    (two rocprofv3 --pmc runs of this command, FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter
    reads for a plain copy of known size), or None if there is no such summary."""
    path = os.path.join(ROOT, PROFILE_SUMMARY.get(workload, ""))
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_ratio:"):
                    return float(line.split(":", 1)[1])
    except (OSError, ValueError):
        pass
    return None


# ------------------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands, one row block per worker process.  The pool is forked before the
# process touches the GPU; workers use NumPy only.
# ------------------------------------------------------------------------------------------------------

def _np_from_raw(path, dtype, shape):
    """A storage-dtype array written by the parent into shared memory, widened to float64 (bf16 travels as uint16)."""
    import numpy as np
    if dtype == "bf16":
        u = np.fromfile(path, dtype=np.uint16).reshape(shape)
        return (u.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return np.fromfile(path, dtype=np.float32).reshape(shape).astype(np.float64)


def _oracle_worker(task):
    import numpy as np
    from oracle import interp
    from workloads import programs as W
    name, ins_spec, got_spec, rtol, start_at = task
    desc = W.get_program(name)
    ins = {k: _np_from_raw(p, dt, sh) for k, (p, dt, sh) in ins_spec.items()}
    while time.monotonic() < start_at:      # all workers of a leg start together
        time.sleep(0.0005)
    t0 = time.monotonic()
    rounded, exact = interp.run(desc, ins)
    t1 = time.monotonic()
    worst = 0.0
    for nm, (p, dt, sh) in got_spec.items():
        got = _np_from_raw(p, dt, sh)
        ref = rounded[nm]
        scale = np.broadcast_to(interp.row_scale(exact[nm]), ref.shape)
        tol = rtol * np.abs(ref) + rtol * scale
        fin = np.isfinite(ref)
        if not np.array_equal(np.isnan(got), np.isnan(ref)):
            worst = float("inf")
        worst = max(worst, float(np.max(np.where(fin, np.abs(got - ref) / np.maximum(tol, 1e-300), 0.0))))
    return t0, t1, worst


class CpuBaseline:
    def __init__(self, enabled: bool):
        self.enabled = enabled
        self.cores = 0
        self.pool = None
        self.legs = []
        if not enabled:
            return
        import multiprocessing as mp
        self.cores = max(1, min(len(os.sched_getaffinity(0)), 16))
        self.pool = mp.get_context("fork").Pool(self.cores)
        self.dir = f"/dev/shm/dvm_bench_{os.getpid()}"
        os.makedirs(self.dir, exist_ok=True)
        self.n_files = 0

    def _put(self, t):
        """Write a CPU tensor's storage bits to shared memory; returns (path, storage dtype, shape)."""
        import torch
        p = os.path.join(self.dir, f"t{self.n_files}.bin")
        self.n_files += 1
        t = t.contiguous()
        if t.dtype == torch.bfloat16:
            t.view(torch.int16).numpy().tofile(p)
            return p, "bf16", tuple(t.shape)
        t.numpy().tofile(p)
        return p, "f32", tuple(t.shape)

    def leg(self, name: str, desc_name: str, blocks, bytes_per_block: float, rtol: float):
        """blocks: list of (inputs dict name -> CPU tensor, GPU outputs dict name -> CPU tensor), one per worker."""
        if not self.enabled or not blocks:
            return
        tasks = [(desc_name, {k: self._put(v) for k, v in ins.items()}, {k: self._put(v) for k, v in got.items()}, rtol)
                 for ins, got in blocks]
        # one block on one core, the others idle
        t0, t1, w1 = self.pool.apply(_oracle_worker, (tasks[0] + (0.0,),))
        one = bytes_per_block / max(t1 - t0, 1e-9)
        start_at = time.monotonic() + 0.5
        res = self.pool.map(_oracle_worker, [t + (start_at,) for t in tasks], chunksize=1)
        wall = max(r[1] for r in res) - min(r[0] for r in res)
        self.legs.append({"config": name, "blocks": len(blocks), "bytes": bytes_per_block * len(blocks), "wall_s": wall,
                          "cpu_s_1core": t1 - t0, "GBps_1core": one / 1e9, "worst": max([w1] + [r[2] for r in res])})
        for f in os.listdir(self.dir):
            os.unlink(os.path.join(self.dir, f))

    def result(self):
        if not self.enabled or not self.legs:
            return None
        tot_b = sum(l["bytes"] for l in self.legs)
        tot_t = sum(l["wall_s"] for l in self.legs)
        one_b = sum(l["bytes"] / l["blocks"] for l in self.legs)
        one_t = sum(l["cpu_s_1core"] for l in self.legs)
        return {"value": round(tot_b / tot_t / 1e9, 4), "unit": "GB/s", "cores": self.cores, "kind": "oracle",
                "one_core_GBps": round(one_b / one_t / 1e9, 4),
                "sample": "leading row blocks of one instance per config (" + ", ".join(
                    f"{l['config']}: {l['blocks']} blocks, {l['bytes'] / 1e6:.0f} MB, {l['wall_s']:.1f} s" for l in self.legs) +
                    f"), the blocks dealt out to {self.cores} worker processes, one per core (count from sched_getaffinity, capped at 16), "
                    "NumPy float64 per-op evaluation; one_core_GBps: one block alone on one core",
                "per_config_GBps": {l["config"]: round(l["bytes"] / l["wall_s"] / 1e9, 4) for l in self.legs},
                "max_err_over_tol_vs_gpu": round(max(l["worst"] for l in self.legs), 4)}

    def close(self):
        if self.pool is not None:
            self.pool.close()
            self.pool.join()
            try:
                os.rmdir(self.dir)
            except OSError:
                pass


# ------------------------------------------------------------------------------------------------------
# the streaming fuser workload
# ------------------------------------------------------------------------------------------------------

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


# ------------------------------------------------------------------------------------------------------
# one dynamic stream: inputs, launches, timing
# ------------------------------------------------------------------------------------------------------

class Stream:
    """The parts (one program applied to one set of tensors) of a workload and how they group into launches."""

    def __init__(self, name, args, B, gen, W, ctx, dev):
        import numpy as np
        import torch
        self.name, self.args, self.B, self.ctx, self.dev = name, args, B, ctx, dev
        self.parts = []
        self.fixed_groups = None
        self.set_counts = None        # per launch: how many sets of tensors it runs over (dvm_run_batched), None: one each
        self.dtype = "bf16 storage, f32 arithmetic"
        progs = {}

        def program(pname):
            if pname not in progs:
                progs[pname] = (W.get_program(pname), B.Program(W.get_program(pname)))
            return progs[pname]

        def add_part(pname, ins_d, nbytes, shape, outs=None):
            desc, prog = program(pname)
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
            self.parts.append({"name": pname, "desc": desc, "prog": prog, "ins": ins, "outs": outs_l, "bytes": nbytes, "shape": shape,
                               "shapes": (B.dvm_shape * len(ins))(*[B.shape_of_tensor(t) for t in ins]), "layout": layout})

        n_inst = args.instances or None
        self.default_stack = 8
        if name == "c2_rmsnorm":
            for i, (b, s) in enumerate(gen.c2_shapes()[:n_inst]):
                add_part("c2_rmsnorm", gen.c2_inputs(b, s, gen.BASE_SEED + 2000 + i, dev), gen.c2_bytes(b, s), (b, s))
            self.wl = {"workload": "config 2: fused RMSNorm bf16, x[B,S,4096], 200 dynamic instances (B 1..32, S 1..2048), eps 1e-6"}
        elif name == "layernorm_bf16":
            # the LayerNorm subgraph range of the paper's Table 2 ([b, 8192, h]); the first 24 of the seeded stream
            for i, (b, s_, h) in enumerate(gen.layernorm_paper_shapes()[: args.instances or 24]):
                add_part("layernorm_bf16", gen.layernorm_inputs(b, s_, h, gen.BASE_SEED + 6000 + 3 * i, dev),
                         gen.layernorm_bytes(b, s_, h), (b, s_, h))
            self.wl = {"workload": "LayerNorm bf16 over [b, 8192, h], b 1..60, h in {1024, 2048, 3072, 4096} (the paper's Table 2 range), eps 1e-5"}
        elif name == "column_sum":
            # Table 1's Sum in its general form: [M, size, N] reduced along `size` to [M, 1, N], fp32
            for i, (m, size, n) in enumerate(gen.column_sum_shapes()[:n_inst]):
                x = gen.randn((m, size, n), gen.BASE_SEED + 8000 + i, dev)
                add_part("colsum", {"x": x}, gen.column_sum_bytes(m, size, n), (m, size, n),
                         {"s": torch.empty((m, 1, n), dtype=torch.float32, device=dev)})
            self.wl = {"workload": "sum along the penultimate axis fp32, [M,size,N] -> [M,1,N], 48 dynamic instances "
                                   "(M 1..256, size 16..4096, N 512..4096)"}
            self.default_stack = 1      # (workgroup and tile register size depend on the shape: one launch each)
            self.dtype = "f32"
        elif name == "c4_chain":
            for i, t in enumerate(gen.c4_shapes()[:n_inst]):
                add_part("c4_chain", gen.c4_inputs(t, gen.BASE_SEED + 4000 + i, dev), gen.c4_bytes(t), (t,))
            self.wl = {"workload": "config 4: 12-op transformer non-GEMM chain bf16 over [T,8192], 100 dynamic instances (T 1..16384)"}
        elif name == "c1_gelu":
            add_part("c1_gelu_erf", gen.c1_inputs(gen.BASE_SEED + 1, dev), 4 * 1000 * 4 * 2 + 2 * 1000 * 4, (4, 1000))
            self.wl = {"workload": "config 1: gelu(x*a+b) fp32 on [4,1000] (latency-bound)"}
            self.dtype = "f32"
        elif name == "c3_masked_softmax":
            # all 50 instances of the seeded stream (92 GB of scores, as much again of outputs); the causal mask of a
            # given S is one tensor shared by the instances of that S
            masks = {}
            for i, (b, s) in enumerate(gen.c3_shapes()[:n_inst]):
                d = gen.c3_inputs(b, s, gen.BASE_SEED + 3000 + i, dev)
                d["mask"] = masks.setdefault(s, d["mask"])
                add_part("c3_masked_softmax", d, gen.c3_bytes(b, s), (b, s))
            self.wl = {"workload": "config 3: causal-masked softmax fp32 over [B,32,S,S] (B 1..4, S 128..4096), mask [S,S] broadcast, "
                                   "50 dynamic instances"}
            self.default_stack = 1      # (instances are gigabytes each and differ in row length)
            self.dtype = "f32"
        elif name == "c5_layers":
            # config 5: 64 steps of a 32-layer stack, six programs per layer, T log-normal; one buffer set per
            # step shared by its 32 layers; every layer is one launch (its six programs stacked)
            # parts that share a launch must fit one interpreter variant: five of the six programs need one tile register
            # at most and run in the 64-element variant; RoPE needs two and is a launch of its own (32 elements)
            ctx_rope = ctx
            if not args.limits:
                ctx.set_limits(64, 1)
                ctx_rope = B.Context(0)
                ctx_rope.set_limits(32, 2)
                if args.assignment:
                    ctx_rope.set_assignment(args.assignment)
                self.extra_ctx = [ctx_rope]
            steps_T = gen.c5_steps()[:n_inst]
            self.fixed_groups = []
            self.set_counts = []
            for si, T in enumerate(steps_T):
                d = gen.c5_inputs(T, gen.BASE_SEED + 5000 + 100 * si, dev)
                rope_out = torch.empty((T, 32, 128), dtype=torch.bfloat16, device=dev)
                L = T // 8 + 1
                first = len(self.parts)
                add_part("c5_rmsnorm", d["c5_rmsnorm"], (2 * T * 4096 + 4096) * 2, (T,))
                add_part("c5_rope", d["c5_rope"], 2 * T * 32 * 128 * 2 + 2 * T * 64 * 4, (T,),
                         {"y1": rope_out[..., :64], "y2": rope_out[..., 64:]})
                add_part("c5_softmax", d["c5_softmax"], 2 * 32 * T * L * 2, (T,))
                add_part("c5_residual", d["c5_residual_a"], 3 * T * 4096 * 2, (T,))
                add_part("c5_silu_gate", d["c5_silu_gate"], 3 * T * 14336 * 2, (T,))
                add_part("c5_residual", d["c5_residual_b"], 3 * T * 4096 * 2, (T,))
                # (layers_per_launch of the 32 layers share a launch: dvm_run_batched runs the layer's bytecode once
                # per layer, the encode of the six programs serves all of them -- the layers have the same shapes)
                lpl = max(1, min(32, args.layers_per_launch))
                if ctx_rope is not ctx:
                    self.parts[first + 1]["ctx"] = ctx_rope
                    launches = [[first, first + 2, first + 3, first + 4, first + 5], [first + 1]]
                else:
                    launches = [list(range(first, first + 6))]
                for g_ in launches:
                    self.fixed_groups += [g_] * (32 // lpl)
                    self.set_counts += [lpl] * (32 // lpl)
                    if 32 % lpl:
                        self.fixed_groups += [g_]
                        self.set_counts += [32 % lpl]
            self.wl = {"workload": "config 5: 64 steps x 32 layers x {rmsnorm, rope, softmax, residual, silu-gate, residual} bf16, "
                                   "T log-normal (median 512, 1..8192); five programs of a layer stacked and RoPE beside them, %d layer(s) per launch, "
                                   "every step's wall time includes its encodes" % max(1, min(32, args.layers_per_launch)),
                       "launches_per_32_layer_step": len(self.fixed_groups) // max(1, len(steps_T)),
                       "steps_of_the_stream": len(steps_T)}
            self.steps_T = steps_T
        else:
            raise ValueError(name)
        torch.cuda.synchronize()

        # launches: lists of part indices
        if self.fixed_groups is not None:
            self.groups_idx = self.fixed_groups
            self.group = 6
            self.singles_idx = [[i] for g, c in zip(self.fixed_groups, self.set_counts or [1] * len(self.fixed_groups)) for _ in range(c) for i in g]
        else:
            n_t_part = len(self.parts[0]["ins"]) + len(self.parts[0]["outs"])
            max_group = max(1, min(32 // n_t_part, 10))
            self.group = max(1, min(args.stack if args.stack > 0 else self.default_stack, max_group))
            n = len(self.parts)
            self.groups_idx = [list(range(lo, min(lo + self.group, n))) for lo in range(0, n, self.group)]
            self.singles_idx = [[i] for i in range(n)]
        counts = self.set_counts if (self.set_counts is not None and self.fixed_groups is not None) else [1] * len(self.groups_idx)
        self.group_sets = counts
        self.total_bytes = sum(self.parts[i]["bytes"] * c for g, c in zip(self.groups_idx, counts) for i in g)
        self.wl["instances"] = len(self.groups_idx) if self.fixed_groups is not None else len(self.parts)
        self.wl["instances_per_launch"] = self.group
        self.stacking = args.stacking or "temporal"
        self.wl["stacking"] = self.stacking if self.group > 1 else "none"
        # the planner is told how many copies of a program share a launch (it prices the tiles that many times)
        # (sets of a batched launch; stacking 8 large instances of config 2 or 4 measured the same with and without)
        self.copies = args.copies_hint if args.copies_hint > 0 else (max(self.set_counts) if self.set_counts else 1)
        for c_ in [ctx] + getattr(self, "extra_ctx", []):
            c_.set_copies_in_flight(self.copies)
        self.wl["planned_for_copies_in_flight"] = self.copies

    def ctx_restore(self):
        self.ctx.set_copies_in_flight(1)
        if self.name == "c5_layers" and not self.args.limits:
            self.ctx.set_limits(64, 6)

    def run(self, lib, steps, warmup, unstacked=True):
        """Time `steps` passes over the stream (after `warmup` untimed ones); returns the stream's figures."""
        import numpy as np
        import torch
        B, ctx, parts = self.B, self.ctx, self.parts
        enc_cap = 8192
        max_parts = max(len(g) for g in self.groups_idx)
        part_bufs = [C.create_string_buffer(enc_cap) for _ in range(max_parts)]
        part_ptrs = (C.c_void_p * max_parts)(*[C.cast(b, C.c_void_p) for b in part_bufs])
        part_lens = (C.c_size_t * max_parts)()
        stacked = C.create_string_buffer(enc_cap)
        ln = C.c_size_t()
        ns = (C.c_int64 * 1)()
        stream = torch.cuda.current_stream()
        stream_h = C.c_void_p(stream.cuda_stream)
        perf = time.perf_counter
        stack_fn = lib.dvm_stack_spatial if self.stacking == "spatial" else lib.dvm_stack

        def marshal(groups, counts=None):
            out = []
            for k, idx in enumerate(groups):
                tens = [t for i in idx for t in parts[i]["ins"] + parts[i]["outs"]]
                n_sets = counts[k] if counts else 1
                ptrs = [t.data_ptr() for t in tens] * n_sets
                out.append((idx, (C.c_void_p * len(ptrs))(*ptrs), len(tens), n_sets))
            return out

        max_table = max(len([t for i in idx for t in parts[i]["ins"] + parts[i]["outs"]]) * c
                        for idx, c in zip(self.groups_idx, self.group_sets))
        table = torch.empty(max_table, dtype=torch.int64, device=self.dev)      # dvm_run_batched's address table

        def one_step(groups, events=None, enc_ns=None):
            """Encode every part, stack the parts of each launch (a single part is launched as it is), run."""
            for k, (idx, ptrs, n_t, n_sets) in enumerate(groups):
                for j, i in enumerate(idx):
                    pt = parts[i]
                    st = lib.dvm_encode_timed(pt.get("ctx", ctx)._h, pt["prog"]._h, pt["shapes"], len(pt["ins"]), pt["layout"], part_bufs[j], enc_cap,
                                              C.byref(ln), 1, ns)
                    if st != 0:
                        raise B.DvmError(st, "dvm_encode")
                    part_lens[j] = ln.value
                    if enc_ns is not None:
                        enc_ns.append(ns[0])
                if len(idx) == 1:
                    code, code_len = part_bufs[0], part_lens[0]
                else:
                    st = stack_fn(part_ptrs, part_lens, len(idx), stacked, enc_cap, C.byref(ln))
                    if st != 0:
                        raise B.DvmError(st, "dvm_stack")
                    code, code_len = stacked, ln.value
                if events is not None:
                    events[k][0].record(stream)
                if n_sets > 1:
                    st = lib.dvm_run_batched(ctx._h, code, code_len, ptrs, n_t, n_sets, C.c_void_p(table.data_ptr()), table.numel() * 8, stream_h)
                else:
                    st = lib.dvm_run(ctx._h, code, code_len, ptrs, n_t, stream_h)
                if st != 0:
                    raise B.DvmError(st, "dvm_run")
                if events is not None:
                    events[k][1].record(stream)

        def timed(groups, n_steps, n_warm, enc_ns=None):
            for _ in range(n_warm):
                one_step(groups)
            evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in groups]
                   for _ in range(n_steps)]
            torch.cuda.synchronize()
            t0 = perf()
            for s in range(n_steps):
                one_step(groups, evs[s], enc_ns)
            torch.cuda.synchronize()
            return perf() - t0, evs

        groups = marshal(self.groups_idx, self.group_sets)
        enc_ns = []
        elapsed, all_events = timed(groups, steps, warmup, enc_ns)
        kern_ms = [a.elapsed_time(b) for evs in all_events for (a, b) in evs]
        group_bytes = [sum(parts[i]["bytes"] for i in g) * c for g, c in zip(self.groups_idx, self.group_sets)]
        big_groups = [k for k, b in enumerate(group_bytes) if b >= 256e6]
        group_ms = [float(np.mean([all_events[s][k][0].elapsed_time(all_events[s][k][1]) for s in range(steps)])) for k in range(len(groups))]
        r = {"config": dict(self.wl), "dtype": self.dtype, "total_bytes": self.total_bytes, "elapsed_s": elapsed, "steps": steps,
             "kernel_ms_sum_per_step": sum(kern_ms) / steps, "launches_per_step": len(groups),
             "whole_job_GBps": self.total_bytes * steps / elapsed / 1e9,
             "kernel_GBps": self.total_bytes / (sum(kern_ms) / steps) / 1e6,
             "large_launches": None, "unstacked": None}
        if big_groups:
            r["large_launches"] = {"launches": len(big_groups),
                                   "GBps": sum(group_bytes[k] for k in big_groups) / sum(group_ms[k] for k in big_groups) / 1e6,
                                   "bytes": sum(group_bytes[k] for k in big_groups), "ms": sum(group_ms[k] for k in big_groups)}
        # first-call encode of every distinct part (cold) and the steady state inside the timed steps
        enc = np.array(enc_ns, dtype=np.float64) / 1e3
        r["encode_us"] = {"median": round(float(np.median(enc)), 2), "p99": round(float(np.percentile(enc, 99)), 2),
                          "max": round(float(enc.max()), 2), "calls": int(enc.size),
                          "note": "every dvm_encode call of the timed steps, CLOCK_MONOTONIC inside the library (dvm_encode_timed)"}
        # the same stream with every program as its own launch (no stacking): per-program launch times
        if unstacked:
            if self.group > 1:
                for c_ in [ctx] + getattr(self, "extra_ctx", []):
                    c_.set_copies_in_flight(1)
                singles = marshal(self.singles_idx)
                elapsed1, events1 = timed(singles, steps, 1)
                for c_ in [ctx] + getattr(self, "extra_ctx", []):
                    c_.set_copies_in_flight(self.copies)
            else:
                elapsed1, events1 = elapsed, all_events
            one_ms = [float(np.mean([events1[s][k][0].elapsed_time(events1[s][k][1]) for s in range(steps)]))
                      for k in range(len(self.singles_idx))]
            one_bytes = [parts[g[0]]["bytes"] for g in self.singles_idx]
            if self.args.dump_launches:
                with open(self.args.dump_launches, "a") as f:
                    f.write("launch,program,shape,bytes,mean_launch_us,GBps\n")
                    for k, g in enumerate(self.singles_idx):
                        pt = parts[g[0]]
                        f.write(f"{k},{pt['name']},{'x'.join(map(str, pt['shape']))},{pt['bytes']},{one_ms[k] * 1e3:.2f},"
                                f"{pt['bytes'] / one_ms[k] / 1e6:.1f}\n")
            rates = np.array([b / m / 1e6 for b, m in zip(one_bytes, one_ms)])
            big = [k for k, b in enumerate(one_bytes) if b >= 256e6]
            r["unstacked"] = {"whole_job_GBps": round(self.total_bytes * steps / elapsed1 / 1e9, 1),
                              "kernel_GBps": round(sum(one_bytes) / sum(one_ms) / 1e6, 1),
                              "per_instance_GBps_median": round(float(np.median(rates)), 1),
                              "per_instance_GBps_p10": round(float(np.percentile(rates, 10)), 1),
                              "large_only_GBps": round(sum(one_bytes[k] for k in big) / sum(one_ms[k] for k in big) / 1e6, 1) if big else None,
                              "large_instances": len(big), "avg_launch_ms": round(float(np.mean(one_ms)), 5),
                              "note": "same stream, every program its own launch; large = at least 256 MB of algorithmic bytes"}
        if self.name == "c5_layers":
            n_steps_stream = len(self.steps_T)
            r["ms_per_32_layer_step"] = round(elapsed / steps / n_steps_stream * 1e3, 4)
        return r


def copy_ceiling(lib, ctx, dev, B):
    """The library's own copy kernel on 512 MiB (beyond the last-level cache), both tile assignments; GB/s read + written."""
    import torch
    n = 512 * 2**20
    src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    stream = torch.cuda.current_stream()
    out = {}
    for mode, label in ((1, "interleaved"), (0, "blocked")):
        for _ in range(2):
            st = lib.dvm_copy_kernel(ctx._h, dst.data_ptr(), src.data_ptr(), n, mode, C.c_void_p(stream.cuda_stream))
            if st != 0:
                raise B.DvmError(st, "dvm_copy_kernel")
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        torch.cuda.synchronize()
        for a, b in evs:
            a.record(stream)
            lib.dvm_copy_kernel(ctx._h, dst.data_ptr(), src.data_ptr(), n, mode, C.c_void_p(stream.cuda_stream))
            b.record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in evs)
        out[label] = round(2.0 * n / (ms[len(ms) // 2] * 1e-3) / 1e9, 1)
    ok = bool(torch.equal(src, dst))
    del src, dst
    return {"GBps": max(out.values()), "by_tile_assignment": out, "bytes_copied": n, "verified": ok,
            "kernel": "dvm_copy_tiles (csrc/dvm_bench.hip): 16 B per lane and access, streaming hints; median of 10 launches"}


def condition_memory(torch, dev, gib, chunk_mib):
    """Bring the device's free memory into the state it has in a process that has been allocating and freeing for a while:
    allocate `gib` GiB in blocks of `chunk_mib` MiB and hand them back to the driver in a scrambled order, so that the
    tensors allocated afterwards lie on physical pages scattered over the memory instead of on one pristine contiguous
    stretch.  On this machine the same launches (the library's copy kernel included) run 4-10 % faster over such pages
    than in the first process on a freshly booted box, and later processes on a box see them anyway; doing it here
    makes the figures independent of what ran on the box before.  Nothing of it is timed."""
    import random
    import time
    if gib <= 0:
        return {"conditioned": False}
    t0 = time.perf_counter()
    chunk = int(chunk_mib * 2**20)
    blocks = []
    try:
        for _ in range(int(gib * 2**30 // chunk)):
            blocks.append(torch.empty(chunk, dtype=torch.uint8, device=dev))
    except RuntimeError:            # (less free memory than asked for: scramble what there is)
        pass
    got = len(blocks)
    torch.cuda.synchronize()
    random.Random(1).shuffle(blocks)
    while blocks:
        blocks.pop()
        if len(blocks) % 1024 == 0:
            torch.cuda.empty_cache()
    torch.cuda.empty_cache()
    return {"conditioned": True, "GiB": round(got * chunk / 2**30, 1), "block_MiB": chunk_mib, "seconds": round(time.perf_counter() - t0, 1),
            "note": "device memory allocated in blocks and freed in a scrambled order before the inputs are allocated (untimed): "
                    "physical pages as in a long-running process; --shuffle-memory-gib 0 gives the pristine-box figures"}


def single_launch_extras(B, gen, W, dev):
    """Single launches of the forms beyond the five configurations: a reduction along the penultimate axis split over a
    workspace (a bias gradient) and rows longer than a tile (softmax and RMSNorm at 32768 and 100000 columns).  GB/s of
    algorithmic bytes (one read of every input element, one write of every output element) over the median of 10 timed runs
    (a split reduction is two kernel launches per run)."""
    import torch
    from workloads.programs import _p, single_op_program
    stream = torch.cuda.current_stream()

    def timed(ctx, desc, ins, n_bytes):
        code = B.encode_for(ctx, B.Program(desc), ins)
        outs = [torch.empty(s_, dtype=torch.bfloat16 if dt == "bf16" else torch.float32, device=dev) for s_, (_, dt) in zip(code.out_shapes, desc.outputs)]
        ptrs = [t.data_ptr() for t in ins + outs]
        if code.needs_workspace():
            ws = torch.empty(code.tensor(code.info().n_tensors - 1)[0] // 4, dtype=torch.int32, device=dev)
            ptrs.append(ws.data_ptr())
        for _ in range(3):
            B.dvm_run(ctx, code, ptrs, stream.cuda_stream)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        torch.cuda.synchronize()
        for a, b in evs:
            a.record(stream)
            B.dvm_run(ctx, code, ptrs, stream.cuda_stream)
            b.record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in evs)[len(evs) // 2]
        inf = code.info()
        return {"GBps": round(n_bytes / ms / 1e6, 1), "us": round(ms * 1e3, 1), "kernel_launches": inf.n_launches, "segments": inf.n_segments}

    out = {}
    ctx = B.Context(0)
    ctx.set_workspace_limit(4 << 20)
    g = gen.randn((8192, 4096), gen.BASE_SEED + 9001, dev, "f32")
    desc = _p("bias_gradient", [("g", "f32")], [("s", "csum", ["g"], {})], [("s", "f32")])
    r = timed(ctx, desc, [g], g.numel() * 4 + 4096 * 4)
    plain = timed(B.Context(0), desc, [g], g.numel() * 4 + 4096 * 4)
    r["unsplit_GBps"] = plain["GBps"]
    out["bias_gradient_f32_8192x4096"] = r
    del g
    ctx = B.Context(0)
    for cols in (32768, 100000):
        rows = (1 << 28) // (cols * 4)
        z = gen.randn((rows, cols), gen.BASE_SEED + 9002, dev, "f32")
        out[f"softmax_f32_{rows}x{cols}"] = timed(ctx, single_op_program("softmax", 1, "f32"), [z], 2 * z.numel() * 4)
        del z
        x = gen.randn((rows, cols), gen.BASE_SEED + 9003, dev, "bf16")
        w = gen.randn((cols,), gen.BASE_SEED + 9004, dev, "bf16")
        out[f"rmsnorm_bf16_{rows}x{cols}"] = timed(ctx, W.get_program("c2_rmsnorm"), [x, w], 2 * x.numel() * 2 + cols * 2)
        del x, w
    torch.cuda.empty_cache()
    return out


def baseline_blocks(stream, name, cores, gen):
    """Row blocks (up to four per worker) of one instance of a stream for the CPU oracle, with the GPU's outputs for the same rows."""
    import torch
    parts = stream.parts
    blocks = []
    if name == "c2_rmsnorm":
        rows_per = 3072
        i = max(range(len(parts)), key=lambda k: parts[k]["ins"][0].shape[0] * parts[k]["ins"][0].shape[1])
        x, w = parts[i]["ins"]
        y = parts[i]["outs"][0]
        x2, y2 = x.reshape(-1, x.shape[-1]), y.reshape(-1, y.shape[-1])
        nb = min(4 * cores, x2.shape[0] // rows_per)
        for b in range(nb):
            sl = slice(b * rows_per, (b + 1) * rows_per)
            blocks.append(({"x": x2[sl].cpu(), "w": w.cpu()}, {"y": y2[sl].cpu()}))
        return "c2_rmsnorm", blocks, rows_per * 4096 * 2 * 2 + 4096 * 2, 2e-2
    if name == "c4_chain":
        rows_per = 512
        i = max(range(len(parts)), key=lambda k: parts[k]["ins"][0].shape[0])
        x, r, gamma, beta, bias, mask = parts[i]["ins"]
        y = parts[i]["outs"][0]
        nb = min(4 * cores, x.shape[0] // rows_per)
        for b in range(nb):
            sl = slice(b * rows_per, (b + 1) * rows_per)
            blocks.append(({"x": x[sl].cpu(), "r": r[sl].cpu(), "gamma": gamma.cpu(), "beta": beta.cpu(), "bias": bias.cpu(),
                            "mask": mask[sl].cpu()}, {"y": y[sl].cpu()}))
        return "c4_chain", blocks, rows_per * 8192 * 2 * 4 + 3 * 8192 * 2, 2e-2
    if name == "c3_masked_softmax":
        # one [S, S] plane (one batch index and head) per worker, of the instance whose S is nearest 2048
        i = min(range(len(parts)), key=lambda k: abs(parts[k]["ins"][0].shape[-1] - 2048))
        z, mask = parts[i]["ins"]
        p = parts[i]["outs"][0]
        S = z.shape[-1]
        z3, p3 = z.reshape(-1, S, S), p.reshape(-1, S, S)
        nb = min(4 * cores, z3.shape[0])
        mh = mask.cpu()
        for b in range(nb):
            blocks.append(({"z": z3[b].cpu(), "mask": mh}, {"p": p3[b].cpu()}))
        return "c3_masked_softmax", blocks, S * S * 4 * 2 + S * S * 4, 1e-4
    return name, [], 0, 0.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="suite", choices=["suite"] + ALL_WORKLOADS)
    ap.add_argument("--instances", type=int, default=0, help="use only the first N instances (0 = the workload's default)")
    ap.add_argument("--stack", type=int, default=0,
                    help="consecutive instances merged into one launch by temporal stacking (default 8, capped by the "
                         "launch's tensor table; 1 = every instance its own launch; config 5 always stacks a layer)")
    ap.add_argument("--layers-per-launch", type=int, default=32,
                    help="config 5: how many of a step's 32 layers share one launch (dvm_run_batched over the layers' tensor sets)")
    ap.add_argument("--stacking", default="", choices=["", "temporal", "spatial"],
                    help="how the parts of a launch share it: one after the other on all workgroups (temporal) or side by "
                         "side on shares of the workgroups (spatial); default temporal (it measured faster on every workload here)")
    ap.add_argument("--assignment", default="", choices=["", "blocked", "interleaved"],
                    help="how tiles are dealt out to workgroups: Algorithm 2's blocked ranges or round-robin (the library's default)")
    ap.add_argument("--limits", default="", help="K,NR: bound the interpreter variant the planner may choose (dvm_ctx_set_limits), for tuning")
    ap.add_argument("--copies-hint", type=int, default=0,
                    help="dvm_ctx_set_copies_in_flight for the stream's programs (0 = the tensor sets of a batched launch, else 1)")
    ap.add_argument("--shuffle-memory-gib", type=float, default=240.0,
                    help="before the inputs are allocated, allocate this much device memory in blocks and free them in a scrambled order (0: off)")
    ap.add_argument("--shuffle-chunk-mib", type=float, default=2.0, help="block size of that step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--skip-unstacked", action="store_true",
                    help="leave out the second pass that launches every program on its own (profiler runs use this so "
                         "that the kernel statistics cover the stacked launches only)")
    ap.add_argument("--dump-launches", default="", help="append per-program bytes and mean launch time to this CSV file")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region run a plain 256 MiB device copy (a known-size kernel that scales "
                         "the HBM byte counters of a profiler run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path needs no exchange between devices); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    # worker processes of the CPU baseline are forked before anything touches the GPU
    names = SUITE if args.workload == "suite" else [args.workload]
    want_cpu = not args.no_cpu_baseline and args.workload != "if_else_add" and any(n in LARGE_CLASS for n in names)
    cpu = CpuBaseline(want_cpu)
    try:
        return run(args, names, cpu)
    finally:
        cpu.close()


def run(args, names, cpu) -> int:
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
    if args.assignment:
        ctx.set_assignment(args.assignment)
    if args.limits:
        k_, nr_ = (int(v) for v in args.limits.split(","))
        ctx.set_limits(k_, nr_)
    else:
        # the caller allows the 64-element variant (the library's default bound is 32): programs over bf16 tensors that need
        # one tile register at most are planned for it
        ctx.set_limits(64, 6)
    placement = condition_memory(torch, dev, args.shuffle_memory_gib, args.shuffle_chunk_mib)
    if args.workload == "if_else_add":
        return bench_fuser(args, B, gen, W, ctx, dev)

    per = {}
    cpu_legs = []
    for name in names:
        print(f"bench.py: {name}: generating inputs", file=sys.stderr, flush=True)
        s = Stream(name, args, B, gen, W, ctx, dev)
        print(f"bench.py: {name}: timing {args.steps} step(s)", file=sys.stderr, flush=True)
        r = s.run(lib, args.steps, args.warmup, unstacked=not args.skip_unstacked)
        if cpu.enabled and name in LARGE_CLASS:
            # (the sample is taken now; the oracle runs on it after all GPU timing, so that the device never idles
            # between two timed workloads)
            cpu_legs.append((name,) + tuple(baseline_blocks(s, name, cpu.cores, gen)))
        s.ctx_restore()
        per[name] = r
        del s
        torch.cuda.empty_cache()

    if args.workload == "suite":
        # config 1 is latency-bound: time per launch and per encode + launch + synchronise
        s = Stream("c1_gelu", args, B, gen, W, ctx, dev)
        r1 = s.run(lib, 200, 20, unstacked=False)
        per["c1_gelu"] = r1
        del s

    ceiling = copy_ceiling(lib, ctx, dev, B)
    extras = single_launch_extras(B, gen, W, dev) if args.workload == "suite" else None
    for name, dn, blocks, bpb, rtol in cpu_legs:
        print(f"bench.py: {name}: CPU oracle on {len(blocks)} row blocks", file=sys.stderr, flush=True)
        cpu.leg(name, dn, blocks, bpb, rtol)

    if args.calibrate_copy:
        src = torch.empty(256 * 2**20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # ---- aggregate: the large memory-bound configs ----------------------------------------------------
    head = [n for n in names if n in LARGE_CLASS] or names
    tot_bytes_step = sum(per[n]["total_bytes"] for n in head)
    wall_step = sum(per[n]["elapsed_s"] / per[n]["steps"] for n in head)
    kern_step_ms = sum(per[n]["kernel_ms_sum_per_step"] for n in head)
    launches_step = sum(per[n]["launches_per_step"] for n in head)
    value = tot_bytes_step / wall_step / 1e9
    achieved = tot_bytes_step / kern_step_ms / 1e6
    ratios = {n: measured_traffic_ratio(n) for n in head}
    traffic = None
    if all(v is not None for v in ratios.values()) and not args.instances and not args.stack and not args.stacking and not args.assignment and not args.limits:
        traffic = int(sum(per[n]["total_bytes"] * ratios[n] for n in head) / launches_step)
    ms_per_step = sum(per[n]["elapsed_s"] / per[n]["steps"] for n in names if n in per) * 1e3

    per_config = {}
    for n, r in per.items():
        frac = r["kernel_GBps"] / HBM_PEAK_GBS
        pc = {"workload": r["config"]["workload"], "instances": r["config"]["instances"],
              "instances_per_launch": r["config"]["instances_per_launch"], "dtype": r["dtype"],
              "whole_job_GBps": round(r["whole_job_GBps"], 1), "kernel_GBps": round(r["kernel_GBps"], 1), "frac": round(frac, 4),
              "pct_of_copy_ceiling": round(100.0 * r["kernel_GBps"] / ceiling["GBps"], 1),
              "ms_per_pass": round(r["elapsed_s"] / r["steps"] * 1e3, 4), "launches_per_pass": r["launches_per_step"],
              "large_launches_GBps": round(r["large_launches"]["GBps"], 1) if r["large_launches"] else None,
              "traffic_ratio": measured_traffic_ratio(n), "encode_us": r["encode_us"], "unstacked": r["unstacked"]}
        if "ms_per_32_layer_step" in r:
            pc["ms_per_32_layer_step"] = r["ms_per_32_layer_step"]
        if n == "c1_gelu":
            pc["us_per_encode_and_launch"] = round(r["elapsed_s"] / r["steps"] * 1e6, 2)
        per_config[n] = pc
    big_b = sum(per[n]["large_launches"]["bytes"] for n in head if per[n]["large_launches"])
    big_ms = sum(per[n]["large_launches"]["ms"] for n in head if per[n]["large_launches"])

    dtypes = sorted({per[n]["dtype"] for n in head})
    if args.workload == "suite":
        wl = {"workload": "configs 2, 3 and 4 (the large memory-bound dynamic streams: RMSNorm bf16 x 200, causal-masked softmax fp32 x 50, "
                          "12-op chain bf16 x 100), run one after the other; config 5 (32-layer model stream) and config 1 (latency) "
                          "are timed in the same job and reported under per_config",
              "instances": sum(per[n]["config"]["instances"] for n in head)}
    else:
        wl = per[names[0]]["config"]
    result = {
        "metric": "achieved HBM GB/s of VM-run fused ops (algorithmic bytes / wall time, encode included)",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "; ".join(dtypes), "data": "synthetic", "config": wl,
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "roofline": {"bound": "hbm", "kernel": "dvm_vm_kernel (bytecode interpreter)", "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "bytes_per_launch": int(tot_bytes_step / launches_step), "avg_launch_ms": round(kern_step_ms / launches_step, 5),
                     "launches": launches_step * args.steps,
                     "large_launches_GBps": round(big_b / big_ms / 1e6, 1) if big_ms else None,
                     "pct_of_copy_ceiling": round(100.0 * achieved / ceiling["GBps"], 1),
                     "traffic": traffic,
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of `bench.py --workload <config>`, summaries under profiles/"
                                       if traffic is not None else None},
        "copy_ceiling": ceiling,
        "memory_placement": placement,
        "per_config": per_config,
    }
    if extras is not None:
        result["single_launches"] = extras
    base = cpu.result()
    rc = 0
    if base is not None:
        result["cpu_baseline"] = base
        if base["max_err_over_tol_vs_gpu"] > 1.0:
            print(f"bench.py: GPU output differs from the oracle on the sample (x{base['max_err_over_tol_vs_gpu']:.3g} of tolerance)",
                  file=sys.stderr)
            rc = 1
    print(json.dumps(result))
    return rc


if __name__ == "__main__":
    sys.exit(main())
