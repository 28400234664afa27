#!/usr/bin/env python3
"""Benchmark of the LP hot path on one MI355X.

One "step" = one LP denoising step over one latent: lp_partition of the global
latent along the step's rotating dimension, lp_attention over every sub-latent
(the K partitions in turn on this one GPU, `layers` attention calls each), then
lp_reconstruct of the K predictions.  All inputs are synthetic, seeded, and
resident in device memory before the timed region starts.

Prints ONE JSON line.  The headline (`value`, `roofline`, `latent_ops`,
`cpu_baseline`) is the 81-frame 720p workload of the 40-head model (the largest
configuration that is one step on one GPU); `other_configs` carries the same
figures, in short, for the other benchmark configurations, among them the
50-step denoising loop with its per-step latency and per-kernel breakdown.
`value` is attention TFLOP/s of the whole step stream (attention flops / wall
time of the timed steps, partition and reconstruct time included).
"""
from __future__ import annotations

import argparse
import concurrent.futures
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0        # MI355X HBM3E
METRIC = "lp_attention TFLOP/s (% bf16 MFMA peak); partition+stitch GB/s (% HBM)"
HEADLINE = 3                  # dit14b-81f-720p
LOOP = 4                      # the 50-step loop on the 81-frame 480p latent
LOOP_STEPS = 50
ATTENTION_SOURCE = os.path.join(ROOT, "paper_2512_07350_amd", "csrc", "lp_attention.hip")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--spinup-ms", type=float, default=200.0,
                    help="run untimed steps for this long before the warm-up steps: the GPU needs some tens of "
                         "milliseconds of load to settle at its running clock")
    ap.add_argument("--workload", type=int, default=HEADLINE,
                    help="index into the benchmark configurations for the headline (default %d)" % HEADLINE)
    ap.add_argument("--layers", type=int, default=0, help="attention calls per partition per step (0 = the workload's)")
    ap.add_argument("--guided", action="store_true",
                    help="time the guided step instead (Eq. 4-6): attention on the conditional / unconditional pair "
                         "in one lp_attention_batch call per partition and layer, then "
                         "lp_reconstruct_guided_step_partition, which also writes the next step's sub-latents "
                         "(so the step has no lp_partition launch of its own)")
    ap.add_argument("--only", action="store_true", help="the headline workload only: no other_configs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "attention_traffic.json"),
                    help="measured HBM bytes per attention launch (written from rocprofv3 --pmc runs; see profiles/)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain device copy of 256 MiB (known size) so that a rocprofv3 --pmc run "
                         "of this command holds the reference dispatch the byte counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a single-GPU hot path; run it with --gpus 1 (got %d). "
              "No multi-GPU figure exists." % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2512_07350_amd import binding as lp
    from paper_2512_07350_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    ctx = Ctx(lp, synth, np, torch)

    cfg = args.workload
    w = synth.WORKLOADS[cfg]
    loop = w.layers > 1 and not args.guided and not args.layers
    run = Run(ctx, cfg, guided=args.guided, layers=args.layers or w.layers, carry=loop)
    steps = LOOP_STEPS if loop and args.steps == ap.get_default("steps") else args.steps
    m = run.measure(steps, args.warmup, args.spinup_ms)
    latent_dims = latent_per_dim(ctx, run)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                       # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()

    result = {
        "metric": METRIC, "value": round(m["value"], 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "spinup_steps": m["spinup_steps"],
        "events": ctx.event_kind, "ms_per_step": round(m["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": run.config(),
        "roofline": dict(m["roofline"], traffic=traffic_record(args.traffic_json, w.name, args.guided)),
        "latent_ops": dict(m["latent_ops"], per_dim=latent_dims),
        "time_split_ms_per_step": m["time_split_ms_per_step"],
    }
    if loop:
        result["loop"] = m["loop"]
    if not args.guided:
        result["block_ops"] = block_ops(ctx, run, check=not args.no_cpu_baseline)
    if not args.no_cpu_baseline and not args.guided:
        result["cpu_baseline"] = cpu_baseline(ctx, run)
    del run
    torch.cuda.empty_cache()

    if not args.only and not args.guided and cfg == HEADLINE:
        result["other_configs"] = other_configs(ctx, args)
    print(json.dumps(result), flush=True)
    return 0


class Ctx:
    """What every part of the benchmark needs: the binding, the input generator, the stream, events."""

    def __init__(self, lp, synth, np, torch):
        self.lp, self.synth, self.np, self.torch = lp, synth, np, torch
        self.stream = torch.cuda.current_stream().cuda_stream
        self.ev, self.event_kind = event_factory(torch, self.stream)
        self.pool = concurrent.futures.ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1))

    def qkv_to_device(self, jobs):
        """jobs: list of (seed, n, heads, head_dim).  -> list of [q, k, v] device tensors (bf16 bits as int16).
        The draws are numpy's (which releases the interpreter lock), one task per tensor."""
        synth, np, torch = self.synth, self.np, self.torch

        def one(seed, n, heads, hd, t):
            return synth.f32_to_bf16_bits(synth.normal_f32(seed, (n, heads, hd), substream=t + 1))

        futs = [[self.pool.submit(one, seed, n, heads, hd, t) for t in range(3)] for seed, n, heads, hd in jobs]
        out = []
        for trio in futs:
            out.append([torch.from_numpy(f.result().view(np.int16)).cuda() for f in trio])
        return out


class Run:
    """Device-resident state of one workload and its step."""

    def __init__(self, ctx, cfg, guided=False, layers=1, carry=False):
        lp, synth, np, torch = ctx.lp, ctx.synth, ctx.np, ctx.torch
        self.ctx, self.cfg, self.guided, self.layers, self.carry = ctx, cfg, guided, layers, carry
        self.w = w = synth.WORKLOADS[cfg]
        self.z = torch.from_numpy(synth.latent(synth.seed_for(cfg, 0, 0, tensor=9), w.latent)).cuda()
        self.out = torch.empty_like(self.z)
        self.state = {}
        jobs, where = [], []
        for dim in sorted(set(w.dims)):
            plan = lp.lp_plan_create(w.latent, w.patch, w.K, dim, **w.overlap_args())
            parts = plan.parts()
            subs = torch.empty(plan.total_elems, dtype=torch.float32, device="cuda")
            preds = torch.from_numpy(synth.normal_f32(synth.seed_for(cfg, dim, 0, tensor=10), (plan.total_elems,))).cuda()
            preds_u = None
            if guided or carry:
                preds_u = torch.from_numpy(synth.normal_f32(synth.seed_for(cfg, dim, 0, tensor=11), (plan.total_elems,))).cuda()
            self.state[dim] = dict(plan=plan, parts=parts, subs=subs, preds=preds, preds_u=preds_u, qkv=[None] * len(parts))
            for kp, part in enumerate(parts):
                if part.n_tokens:
                    jobs.append((synth.seed_for(cfg, dim, kp), part.n_tokens, w.heads, w.head_dim))
                    where.append((dim, kp, 0))
                    if guided:    # second item of the pair
                        jobs.append((synth.seed_for(cfg, dim, kp, tensor=12), part.n_tokens, w.heads, w.head_dim))
                        where.append((dim, kp, 1))
        dev = ctx.qkv_to_device(jobs)
        for (dim, kp, item), trio in zip(where, dev):
            slot = self.state[dim]["qkv"]
            if item == 0:
                slot[kp] = [trio[0].shape[0]] + trio
            else:                 # [2, n, heads, d]
                slot[kp] = [slot[kp][0]] + [torch.stack([a, b]) for a, b in zip(slot[kp][1:], trio)]
        for st in self.state.values():
            for item in st["qkv"]:
                if item is not None:
                    item.append(torch.empty_like(item[1]))
        self.ws_bytes = lp.lp_attention_workspace_size(w.head_dim)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()

    def flops_of(self, n):
        return 4.0 * n * n * self.w.head_dim * self.w.heads * (2 if self.guided else 1)

    def config(self):
        w, synth = self.w, self.ctx.synth
        return {"workload": w.name, "index": self.cfg, "latent": list(w.latent), "patch": list(w.patch), "K": w.K,
                "overlap_patches": w.overlap_patches, "overlap_ratio": w.overlap_ratio,
                "dims": [synth.DIM_NAMES[d] for d in w.dims], "heads": w.heads, "head_dim": w.head_dim,
                "tokens_per_partition": {synth.DIM_NAMES[d]: [int(p.n_tokens) for p in st["parts"]] for d, st in self.state.items()},
                "attention_layers_per_partition": self.layers, "guided_pair": bool(self.guided),
                "latent_carried_between_steps": bool(self.carry)}

    def step(self, step_1based, rec=None):
        """Enqueue one step.  carry: the step ends with the guided sampler update of z in place
        (Eq. 4-6), so step i + 1 partitions what step i wrote."""
        ctx, lp, w = self.ctx, self.ctx.lp, self.w
        stream, ev = ctx.stream, ctx.ev
        dim = w.dims[(step_1based - 1) % len(w.dims)]
        if len(w.dims) == 3:
            assert dim == lp.lp_rotation_dim(step_1based)
        st = self.state[dim]
        # one event between consecutive launches: the end of one interval is the start of the next
        e0 = ev(); e0.record()
        if not self.guided:           # guided: the previous step's fused call has written these sub-latents
            lp.lp_partition(st["plan"], self.z, st["subs"], stream)
        e1 = ev(); e1.record()
        att = []
        last = e1
        hd, heads = w.head_dim, w.heads
        for item in st["qkv"]:
            if item is None:
                continue
            n, qd, kd, vd, od = item
            for _ in range(self.layers):
                if self.guided:
                    lp.lp_attention_batch(qd, kd, vd, od, 2, n, heads, hd, n * heads * hd, heads * hd, hd, 0.0,
                                          self.ws, self.ws_bytes, stream)
                else:
                    lp.lp_attention(qd, kd, vd, od, n, heads, hd, heads * hd, hd, 0.0, self.ws, self.ws_bytes, stream)
                a1 = ev(); a1.record()
                att.append((last, a1, n))
                last = a1
        e2 = last
        next_dim = w.dims[step_1based % len(w.dims)]
        if self.guided:
            nxt = self.state[next_dim]
            lp.lp_reconstruct_guided_step_partition(st["plan"], st["preds"], st["preds_u"], 5.0, self.z, 1.0, -0.02,
                                                    self.z if self.carry else self.out, nxt["plan"], nxt["subs"], stream)
        elif self.carry:
            lp.lp_reconstruct_guided_step(st["plan"], st["preds"], st["preds_u"], 5.0, self.z, 1.0, -0.02, self.z, stream)
        else:
            lp.lp_reconstruct(st["plan"], st["preds"], self.out, stream)
        e3 = ev(); e3.record()
        if rec is not None:
            rec.append((dim, next_dim, e0, e1, att, e2, e3))

    def measure(self, steps, warmup, spinup_ms):
        torch, synth, w = self.ctx.torch, self.ctx.synth, self.w
        t_spin = time.perf_counter() + spinup_ms * 1e-3
        spin_steps = 0
        while time.perf_counter() < t_spin:
            for i in range(len(w.dims)):
                self.step(i + 1)
            torch.cuda.synchronize()
            spin_steps += len(w.dims)
        for i in range(warmup):
            self.step(i + 1)
        torch.cuda.synchronize()
        if self.carry:       # the timed loop starts from the seeded latent, at step 1
            self.z.copy_(torch.from_numpy(synth.latent(synth.seed_for(self.cfg, 0, 0, tensor=9), w.latent)))
            torch.cuda.synchronize()
        first = 1 if self.carry else warmup + 1
        records = []
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(first + i, records)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

        att_ms = att_flops = 0.0
        att_launches = 0
        part_ms = rec_ms = part_bytes = rec_bytes = 0.0
        per_dim = {}
        step_ms = []
        for dim, next_dim, e0, e1, att, e2, e3 in records:
            st = self.state[dim]
            tp, tr = e0.elapsed_time(e1), e2.elapsed_time(e3)
            part_ms += tp
            rec_ms += tr
            s_ext = 4.0 * st["plan"].total_elems
            s_z = 4.0 * st["plan"].latent_elems
            part_bytes += 2.0 * s_ext              # read each selected element once, write it once
            # read every prediction once, write the latent once; guided step: both sets and z read;
            # fused with the next partition: the next step's sub-latents written as well
            if self.guided:
                rec_bytes += 2.0 * s_ext + 2.0 * s_z + 4.0 * self.state[next_dim]["plan"].total_elems
            elif self.carry:
                rec_bytes += 2.0 * s_ext + 2.0 * s_z
            else:
                rec_bytes += s_ext + s_z
            d = per_dim.setdefault(synth.DIM_NAMES[dim], dict(ms=0.0, flops=0.0, launches=0, steps=0, part_ms=0.0, rec_ms=0.0, step_ms=0.0))
            d["steps"] += 1; d["part_ms"] += tp; d["rec_ms"] += tr
            t_step = e0.elapsed_time(e3)
            d["step_ms"] += t_step
            step_ms.append(t_step)
            for a0, a1, n in att:
                t = a0.elapsed_time(a1)
                att_ms += t
                att_flops += self.flops_of(n)
                att_launches += 1
                d["ms"] += t; d["flops"] += self.flops_of(n); d["launches"] += 1

        achieved = att_flops / (att_ms * 1e-3) / 1e12
        res = {
            "value": att_flops / wall / 1e12, "ms_per_step": wall * 1e3 / steps, "spinup_steps": spin_steps,
            "roofline": {"kernel": "attention_kernel<%d,%d>, timed per lp_attention call (the interval also holds the "
                                   "combine_kernel<%d> that merges shared query tiles, when there is one, and the launch gap)"
                                   % (w.head_dim, attention_rows_per_wave() // 32, w.head_dim),
                         "bound": "mfma", "achieved": round(achieved, 3), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                         "launches": att_launches, "avg_launch_ms": round(att_ms / max(att_launches, 1), 5),
                         "avg_flops_per_launch": att_flops / max(att_launches, 1),
                         "per_dim_tflops": {k: round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) for k, v in per_dim.items()}},
            "latent_ops": {"bound": "hbm", "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                           "in_step": "partition / reconstruct as timed inside the steps (buffers reused every step: warm)",
                           "partition": rate(part_bytes, part_ms, steps),
                           "reconstruct": rate(rec_bytes, rec_ms, steps)},
            "time_split_ms_per_step": {"partition": round(part_ms / steps, 5), "attention": round(att_ms / steps, 4),
                                       "reconstruct": round(rec_ms / steps, 5)},
        }
        if self.guided:
            res["latent_ops"].pop("partition")     # no partition launch of its own in the guided step
        if self.carry:
            srt = sorted(step_ms)
            res["loop"] = {
                "steps": steps, "latent": "step i+1 partitions the latent step i wrote (guided sampler update in place, Eq. 4-6)",
                "step_latency_ms": {"median": round(srt[len(srt) // 2], 3), "min": round(srt[0], 3), "max": round(srt[-1], 3),
                                    "mean": round(sum(srt) / len(srt), 3)},
                "step_latency_ms_each": [round(t, 3) for t in step_ms],
                "per_dim_ms_per_step": {k: {"step": round(v["step_ms"] / v["steps"], 3),
                                            "partition_kernel": round(v["part_ms"] / v["steps"], 5),
                                            "attention_kernel+combine_kernel": round(v["ms"] / v["steps"], 3),
                                            "attention_calls": v["launches"] // v["steps"],
                                            "reconstruct_kernel (guided step)": round(v["rec_ms"] / v["steps"], 5)}
                                        for k, v in per_dim.items()},
                "final_latent_checksum": float(self.z.double().sum().item()),
            }
        return res


def rate(nbytes, ms, steps):
    if ms <= 0:
        return None
    gbps = nbytes / (ms * 1e-3) / 1e9
    return {"GBps": round(gbps, 1), "avg_us": round(ms * 1e3 / steps, 2), "frac": round(gbps / PEAK_HBM_GBPS, 4)}


def attention_rows_per_wave():
    """Query rows one wavefront of attention_kernel owns (read from the kernel source, for the label only)."""
    import re
    m = re.search(r"constexpr int blocks_per_wave\([^)]*\) \{ return (\d+); \}", open(ATTENTION_SOURCE).read())
    return 32 * int(m.group(1)) if m else 32


def traffic_record(path, workload, guided):
    """HBM bytes per lp_attention launch from the tracked rocprofv3 --pmc record of this workload -- only if the
    record was taken with the attention source as it is now (it names the file's SHA-256); else null."""
    if guided or not path or not os.path.exists(path):
        return None
    sha = hashlib.sha256(open(ATTENTION_SOURCE, "rb").read()).hexdigest()
    doc = json.load(open(path))
    for rec in doc.get("records", [doc]):
        if rec.get("workload") == workload and rec.get("attention_source_sha256") == sha:
            return rec.get("attention_bytes_per_launch")
    return None


def other_configs(ctx, args):
    """The other benchmark configurations, each in short: tiny, 33-frame rotating, 81-frame H step with the
    K = 1 full sequence beside it, and the 50-step loop."""
    torch, lp, synth = ctx.torch, ctx.lp, ctx.synth
    out = []
    for cfg, steps, warmup in ((0, 200, 20), (1, 60, 10), (2, 20, 3), (LOOP, LOOP_STEPS, 3)):
        w = synth.WORKLOADS[cfg]
        carry = cfg == LOOP
        run = Run(ctx, cfg, layers=w.layers, carry=carry)
        m = run.measure(steps, warmup, 100.0 if not carry else 0.0)
        entry = {"config": run.config(), "steps": steps, "value": round(m["value"], 3), "unit": "TFLOP/s",
                 "ms_per_step": round(m["ms_per_step"], 4),
                 "roofline": {k: m["roofline"][k] for k in ("achieved", "frac", "launches", "avg_launch_ms", "per_dim_tflops")},
                 "latent_ops": {d: {c: {k: v[c][k]["frac"] for k in ("partition", "reconstruct", "guided_step")} for c in ("warm", "cold")}
                                for d, v in latent_per_dim(ctx, run, total_bytes=1 << 30, reps=2).items()},
                 "time_split_ms_per_step": m["time_split_ms_per_step"]}
        if carry:
            entry["loop"] = m["loop"]
        if cfg == 2:
            entry["K1_full_sequence"] = k1_comparison(ctx, run)
            entry["block_ops"] = block_ops(ctx, run, check=False)      # the 12-head block: d_model 1536
        out.append(entry)
        del run
        torch.cuda.empty_cache()
    return out


def block_ops(ctx, run, calls=5, check=True):
    """The DiT-block operations around the attention core at the shape of the workload's largest sub-latent:
    lp_qkv_projection (projection with q / k normalisation and rotation in its epilogue), lp_attention on what it
    wrote, lp_linear as the output projection -- each timed alone, back to back calls between two events; a few
    tokens of q, k, v are compared with the oracle.  (The paper fixes none of the block's internals; see lp.h.)"""
    lp, synth, np, torch, w = ctx.lp, ctx.synth, ctx.np, ctx.torch, run.w
    dim = sorted(run.state)[0]
    st = run.state[dim]
    kp = max(range(len(st["parts"])), key=lambda i: st["parts"][i].n_tokens)
    part = st["parts"][kp]
    n, heads, hd = int(part.n_tokens), w.heads, w.head_dim
    dm = heads * hd
    grid = tuple(int(part.shape[1 + d]) // w.patch[d] for d in range(3))
    offset = [0, 0, 0]
    offset[dim] = int(part.alpha_ext)
    seed = synth.seed_for(run.cfg, dim, kp, tensor=30)

    def bf16_dev(sub, shape, scale):
        parts = [ctx.pool.submit(lambda r=r: synth.f32_to_bf16_bits(np.float32(scale) * synth.normal_f32(seed, (r[1] - r[0],) + shape[1:], substream=sub * 64 + i)))
                 for i, r in enumerate(_row_chunks(shape[0], 16))]
        host = np.concatenate([f.result() for f in parts])
        return host, torch.from_numpy(host.view(np.int16)).cuda()

    x_h, x = bf16_dev(1, (n, dm), 1.0)
    wq_h, w_qkv = bf16_dev(2, (3 * dm, dm), dm ** -0.5)
    _, w_o = bf16_dev(3, (dm, dm), dm ** -0.5)
    bias_h = 0.5 * synth.normal_f32(seed, (3 * dm,), substream=250)
    gq_h = 1.0 + 0.2 * synth.normal_f32(seed, (heads, hd), substream=251)
    gk_h = 1.0 + 0.2 * synth.normal_f32(seed, (heads, hd), substream=252)
    bias, gq, gk = (torch.from_numpy(a).cuda() for a in (bias_h, gq_h, gk_h))
    q, k, v, o = (torch.empty((n, heads, hd), dtype=torch.bfloat16, device="cuda") for _ in range(4))
    y = torch.empty((n, dm), dtype=torch.bfloat16, device="cuda")
    rope = lp.make_rope(grid, offset, head_dim=hd)
    stream = ctx.stream
    ops = {
        "qkv_projection": (lambda: lp.lp_qkv_projection(x, w_qkv, bias, gq, gk, 1e-6, rope, q, k, v, n, heads, hd, stream), 2.0 * n * dm * 3 * dm),
        "attention": (lambda: lp.lp_attention(q, k, v, o, n, heads, hd, heads * hd, hd, 0.0, run.ws, run.ws_bytes, stream), 4.0 * n * n * hd * heads),
        "out_projection": (lambda: lp.lp_linear(o, w_o, bias[:dm], y, n, dm, dm, stream), 2.0 * n * dm * dm),
    }
    res = {"tokens": n, "heads": heads, "head_dim": hd, "d_model": dm, "patch_grid": list(grid), "grid_offset": offset}
    total_ms = total_flops = 0.0
    for name, (fn, flops) in ops.items():
        fn(); fn()
        a, b = ctx.ev(), ctx.ev()
        a.record()
        for _ in range(calls):
            fn()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / calls
        total_ms += ms
        total_flops += flops
        res[name] = {"ms": round(ms, 4), "tflops": round(flops / ms / 1e9, 1), "frac": round(flops / ms / 1e9 / PEAK_BF16_TFLOPS, 4)}
    res["block_attention_path"] = {"ms": round(total_ms, 4), "tflops": round(total_flops / total_ms / 1e9, 1),
                                   "frac": round(total_flops / total_ms / 1e9 / PEAK_BF16_TFLOPS, 4)}
    if check:
        from oracle import lp_oracle as orc
        rows = [0, n // 3, n - 1]
        worst = 0.0
        got = [t.view(torch.int16).cpu().numpy().view(np.uint16) for t in (q, k, v)]
        for r in rows:
            c = [r // (grid[1] * grid[2]) + offset[0], (r // grid[2]) % grid[1] + offset[1], r % grid[2] + offset[2]]
            want = orc.qkv_block(x_h[r:r + 1], wq_h, bias_h, gq_h, gk_h, 1e-6, heads, hd, (1, 1, 1), c)
            for g_bits, e in zip(got, want):
                worst = max(worst, float(np.max(np.abs(synth.bf16_bits_to_f32(g_bits[r:r + 1]) - e) / (2.0 ** -8 * np.abs(e) + 3e-4))))
        res["qkv_vs_oracle_on_3_tokens"] = {"worst_error_over_bound": round(worst, 3), "bound": "2^-8 |want| + 3e-4"}
    return res


def _row_chunks(rows, n):
    step = (rows + n - 1) // n
    return [(i, min(rows, i + step)) for i in range(0, rows, step)]


def k1_comparison(ctx, run, calls=5):
    """The non-LP comparison of the 81-frame configuration: one lp_attention call over all tokens of the latent."""
    lp, synth, torch, w = ctx.lp, ctx.synth, ctx.torch, run.w
    plan1 = lp.lp_plan_create(w.latent, w.patch, 1, w.dims[0], overlap_patches=0)
    n = plan1.parts()[0].n_tokens
    q, k, v = ctx.qkv_to_device([(synth.seed_for(run.cfg, w.dims[0], 15), n, w.heads, w.head_dim)])[0]
    o = torch.empty_like(q)
    call = lambda: lp.lp_attention(q, k, v, o, n, w.heads, w.head_dim, w.heads * w.head_dim, w.head_dim, 0.0, run.ws, run.ws_bytes, ctx.stream)
    call(); call()
    a, b = ctx.ev(), ctx.ev()
    a.record()
    for _ in range(calls):
        call()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / calls
    flops = 4.0 * n * n * w.head_dim * w.heads
    lp_flops = sum(run.flops_of(p.n_tokens) for st in run.state.values() for p in st["parts"])
    return {"n_tokens": int(n), "ms_per_call": round(ms, 4), "tflops": round(flops / ms / 1e9, 2),
            "frac": round(flops / ms / 1e9 / PEAK_BF16_TFLOPS, 4),
            "lp_flops_over_full_sequence_flops": round(lp_flops / flops, 4)}


def event_factory(torch, stream):
    """Timing events for the marks between launches.  Preferred: HIP events created with
    hipEventDisableSystemFence (for events that only measure time), recorded on `stream`; a
    default event makes the device flush its caches at every mark, which costs the step a few
    per cent.  Falls back to torch events if the HIP runtime cannot be bound."""
    import ctypes as C

    class TorchEvent:
        def __init__(self):
            self.e = torch.cuda.Event(enable_timing=True)

        def record(self):
            self.e.record()

        def elapsed_time(self, other):
            return self.e.elapsed_time(other.e)

    try:
        hip = C.CDLL("libamdhip64.so")       # the runtime torch has loaded
        hip.hipEventCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
        hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        hip.hipEventDestroy.argtypes = [C.c_void_p]
        k_disable_system_fence = 0x20000000

        class HipEvent:
            def __init__(self):
                self.h = C.c_void_p()
                if hip.hipEventCreateWithFlags(C.byref(self.h), k_disable_system_fence) != 0:
                    raise RuntimeError("hipEventCreateWithFlags")

            def record(self):
                if hip.hipEventRecord(self.h, C.c_void_p(stream)) != 0:
                    raise RuntimeError("hipEventRecord")

            def elapsed_time(self, other):
                ms = C.c_float()
                if hip.hipEventElapsedTime(C.byref(ms), self.h, other.h) != 0:
                    raise RuntimeError("hipEventElapsedTime")
                return ms.value

            def __del__(self):
                try:
                    if self.h:
                        hip.hipEventDestroy(self.h)
                except Exception:       # interpreter shutdown: the runtime may already be gone
                    pass

        a, b = HipEvent(), HipEvent()          # check the binding on a known piece of work
        a.record()
        torch.empty(1 << 20, device="cuda").zero_()
        b.record()
        torch.cuda.synchronize()
        if not a.elapsed_time(b) > 0.0:
            raise RuntimeError("no time between two events")
        return HipEvent, "hip events without system fence"
    except (OSError, AttributeError, RuntimeError):
        return TorchEvent, "torch events"


def latent_per_dim(ctx, run, total_bytes=2 << 30, reps=3):
    """lp_partition, lp_reconstruct and lp_reconstruct_guided_step per partition dimension, each timed as a run of launches
    back to back between two HIP events.  "warm": every call on the same buffers (operands in L2 / Infinity Cache).  "cold": each
    call on its own copy of the buffers, the copies together (about total_bytes) several times the
    last-level cache, so that operands come from HBM."""
    lp, torch, synth, state, w, z, stream = ctx.lp, ctx.torch, ctx.synth, run.state, run.w, run.z, ctx.stream
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn, n):             # n launches back to back between one pair of events
        best = 1e9
        for _ in range(reps):
            a, b = ev(), ev()
            a.record()
            for c in range(n):
                fn(c)
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b) / n)
        return best

    res = {}
    for dim in sorted(state):
        st = state[dim]
        plan = st["plan"]
        s_ext, s_z = 4 * plan.total_elems, 4 * plan.latent_elems
        copies = int(max(2, min(256, total_bytes // (2 * (s_ext + s_z)))))
        zs = [z.clone() for _ in range(copies)]
        subs = [torch.empty_like(st["subs"]) for _ in range(copies)]
        preds = [st["preds"].clone() for _ in range(copies)]
        outs = [torch.empty_like(z) for _ in range(copies)]
        # the guided step reads a second prediction set: the sub-latent buffers stand in for it
        guided = lambda c0, c1: lp.lp_reconstruct_guided_step(plan, preds[c0], subs[c0], 5.0, zs[c1], 1.0, -0.02,
                                                              outs[c1], stream)
        # fused with the partition for the following step (the next dim of the rotation); the
        # second prediction set's buffer cannot double as the destination here
        nxt_plan = state[w.dims[(w.dims.index(dim) + 1) % len(w.dims)]]["plan"]
        nxt_subs = [torch.empty(nxt_plan.total_elems, dtype=torch.float32, device="cuda") for _ in range(copies)]
        fused = lambda c0, c1: lp.lp_reconstruct_guided_step_partition(plan, preds[c0], subs[c0], 5.0, zs[c1], 1.0, -0.02,
                                                                       outs[c1], nxt_plan, nxt_subs[c1], stream)
        t = {"warm": {"partition": timed(lambda c: lp.lp_partition(plan, zs[0], subs[0], stream), 50),
                      "reconstruct": timed(lambda c: lp.lp_reconstruct(plan, preds[0], outs[0], stream), 50),
                      "guided_step": timed(lambda c: guided(0, 0), 50),
                      "guided_step_partition": timed(lambda c: fused(0, 0), 50),
                      "device_copy": timed(lambda c: subs[0].copy_(preds[0]), 50)},
             "cold": {"partition": timed(lambda c: lp.lp_partition(plan, zs[c], subs[c], stream), copies),
                      "reconstruct": timed(lambda c: lp.lp_reconstruct(plan, preds[c], outs[c], stream), copies),
                      "guided_step": timed(lambda c: guided(c, c), copies),
                      "guided_step_partition": timed(lambda c: fused(c, c), copies),
                      "device_copy": timed(lambda c: subs[c].copy_(preds[c]), copies)}}
        nbytes = {"partition": 2.0 * s_ext, "reconstruct": float(s_ext + s_z), "guided_step": 2.0 * s_ext + 2.0 * s_z,
                  "guided_step_partition": 2.0 * s_ext + 2.0 * s_z + 4.0 * nxt_plan.total_elems,
                  "device_copy": 2.0 * s_ext}       # the runtime's own copy of the packed sub-latents: what a plain copy of this size reaches
        entry = {"gamma": round(s_ext / s_z, 4), "copies": copies}
        for cache in ("warm", "cold"):
            entry[cache] = {}
            for name in ("partition", "reconstruct", "guided_step", "guided_step_partition", "device_copy"):
                gbps = nbytes[name] / (t[cache][name] * 1e-3) / 1e9
                entry[cache][name] = {"us": round(t[cache][name] * 1e3, 2), "GBps": round(gbps, 1),
                                      "frac": round(gbps / PEAK_HBM_GBPS, 4)}
        res[synth.DIM_NAMES[dim]] = entry
        del zs, subs, preds, outs, nxt_subs
    return res


def cpu_baseline(ctx, run):
    """Time the CPU oracle, as it stands, on a bounded sample of this workload: one step along
    every partition dimension the workload visits, partition and reconstruct in full and attention
    on every `stride`-th query row of every partition (each row over all keys, all heads; at least
    256 rows per partition).  Also compares the GPU's attention output on those rows with the
    oracle's.  The oracle's time for the whole attention problem is the measured time scaled by
    the share of rows and is labelled as an extrapolation."""
    from oracle import lp_oracle as orc
    synth, np, w, cfg, state = ctx.synth, ctx.np, run.w, run.cfg, run.state
    dims = sorted(state)
    plans = {d: orc.plan(w.latent, w.patch, w.K, d, **w.overlap_args()) for d in dims}
    total_flops = sum(4.0 * p.n_tokens ** 2 * w.head_dim * w.heads for d in dims for p in plans[d].parts)
    budget_flops = 1.5e12                     # 10-30 s of oracle work on the 16 host cores of a GPU machine at the 40-head shapes
    stride = max(1, int(np.ceil(total_flops / budget_flops)))
    z_h = synth.latent(synth.seed_for(cfg, 0, 0, tensor=9), w.latent)
    t_part = t_rec = t_att = 0.0
    flops = bytes_part = bytes_rec = 0.0
    max_err = sum_err = 0.0
    n_cmp = 0
    min_rows = None
    parity_latent = True
    for dim in dims:
        st, ref_plan = state[dim], plans[dim]
        preds_h = st["preds"].cpu().numpy()
        t0 = time.perf_counter()
        subs_ref = orc.partition(ref_plan, z_h)
        t_part += time.perf_counter() - t0
        t0 = time.perf_counter()
        orc.reconstruct(ref_plan, preds_h)
        t_rec += time.perf_counter() - t0
        bytes_part += 2 * 4.0 * ref_plan.total_elems
        bytes_rec += 4.0 * (ref_plan.total_elems + int(np.prod(w.latent)))
        if not run.carry:     # (a carried latent has moved on from the seeded one)
            parity_latent = parity_latent and bool(np.array_equal(st["subs"].cpu().numpy(), subs_ref))
        for kp, part in enumerate(ref_plan.parts):
            n = part.n_tokens
            if n == 0:
                continue
            # the seeded inputs, as uploaded (drawing them again on the host takes longer than the oracle)
            q, k, v = (t.cpu().numpy().view(np.uint16) for t in st["qkv"][kp][1:4])
            rows = np.arange(0, n, min(stride, max(1, n // 256)), dtype=np.int64)
            min_rows = len(rows) if min_rows is None else min(min_rows, len(rows))
            t0 = time.perf_counter()
            want = orc.attention(q, k, v, rows=rows)
            t_att += time.perf_counter() - t0
            flops += 4.0 * len(rows) * n * w.head_dim * w.heads
            got_bits = st["qkv"][kp][4].cpu().numpy().view(np.uint16)
            err = np.abs(synth.bf16_bits_to_f32(got_bits[rows]) - want)
            max_err = max(max_err, float(err.max()))
            sum_err += float(err.sum()); n_cmp += err.size
    return {"value": round(flops / t_att / 1e12, 5), "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "one step along each of %s of %s: attention on every %d-th query row of all %d partitions (at least %d rows "
                      "per partition; all keys, all heads; %.3g of %.3g flop) in %.1f s; partition %.1f ms and reconstruct %.1f ms in full"
                      % ("/".join(synth.DIM_NAMES[d] for d in dims), w.name, stride, w.K, min_rows or 0, flops, total_flops, t_att,
                         t_part * 1e3, t_rec * 1e3),
            "attention_seconds_measured": round(t_att, 2),
            "attention_seconds_full_problem_extrapolated": round(t_att * total_flops / flops, 1),
            "partition_GBps": round(bytes_part / t_part / 1e9, 2),
            "reconstruct_GBps": round(bytes_rec / t_rec / 1e9, 2),
            "gpu_vs_oracle_on_sample": {"attention_max_abs": max_err, "attention_mean_abs": sum_err / max(n_cmp, 1),
                                        "partition_bit_exact": parity_latent}}


if __name__ == "__main__":
    sys.exit(main())
