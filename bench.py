#!/usr/bin/env python3
"""Benchmark of the LP hot path on one MI355X.

One "step" = one LP denoising step over one latent: lp_partition of the global
latent along the step's rotating dimension, lp_attention over every sub-latent
(the K partitions in turn on this one GPU, `layers` attention calls each), then
lp_reconstruct of the K predictions.  All inputs are synthetic, seeded, and
resident in device memory before the timed region starts.

Prints ONE JSON line.  `value` is attention TFLOP/s of the whole step stream
(attention flops / wall time of the timed steps, partition and reconstruct time
included).  `roofline` describes the attention kernel (its flops over its own
HIP-event time inside the timed region), `latent_ops` the two HBM-bound kernels,
`cpu_baseline` the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--spinup-ms", type=float, default=200.0,
                    help="run untimed steps for this long before the warm-up steps: the GPU needs some tens of "
                         "milliseconds of load to settle at its running clock")
    ap.add_argument("--workload", type=int, default=1, help="index into the benchmark configurations (default 1)")
    ap.add_argument("--layers", type=int, default=0, help="attention calls per partition per step (0 = the workload's)")
    ap.add_argument("--guided", action="store_true",
                    help="time the guided step instead (Eq. 4-6): attention on the conditional / unconditional pair "
                         "in one lp_attention_batch call per partition and layer, then "
                         "lp_reconstruct_guided_step_partition, which also writes the next step's sub-latents "
                         "(so the step has no lp_partition launch of its own)")
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
    stream = torch.cuda.current_stream().cuda_stream
    cfg = args.workload
    w = synth.WORKLOADS[cfg]
    layers = args.layers or w.layers

    # ---- plans and device-resident inputs for every partition dim the workload visits
    z = torch.from_numpy(synth.latent(synth.seed_for(cfg, 0, 0, tensor=9), w.latent)).cuda()
    out = torch.empty_like(z)
    state = {}
    for dim in sorted(set(w.dims)):
        plan = lp.lp_plan_create(w.latent, w.patch, w.K, dim, **w.overlap_args())
        parts = plan.parts()
        subs = torch.empty(plan.total_elems, dtype=torch.float32, device="cuda")
        preds = torch.from_numpy(synth.normal_f32(synth.seed_for(cfg, dim, 0, tensor=10), (plan.total_elems,))).cuda()
        qkv = []
        for kp, part in enumerate(parts):
            n = part.n_tokens
            if n == 0:
                qkv.append(None)
                continue
            host = synth.qkv_bf16(synth.seed_for(cfg, dim, kp), n, w.heads, w.head_dim)
            if args.guided:   # second item of the pair: [2, n, heads, d]
                other = synth.qkv_bf16(synth.seed_for(cfg, dim, kp, tensor=12), n, w.heads, w.head_dim)
                host = [np.stack([a, b]) for a, b in zip(host, other)]
            dev = [torch.from_numpy(a.view(np.int16)).cuda() for a in host]
            qkv.append((n, dev[0], dev[1], dev[2], torch.empty_like(dev[0])))
        preds_u = None
        if args.guided:
            preds_u = torch.from_numpy(synth.normal_f32(synth.seed_for(cfg, dim, 0, tensor=11), (plan.total_elems,))).cuda()
        state[dim] = dict(plan=plan, parts=parts, subs=subs, preds=preds, preds_u=preds_u, qkv=qkv)
    ws_bytes = lp.lp_attention_workspace_size(w.head_dim)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()

    n_items = 2 if args.guided else 1

    def flops_of(n):
        return 4.0 * n * n * w.head_dim * w.heads * n_items

    ev, event_kind = event_factory(torch, stream)

    def run_step(step_1based, rec=None):
        dim = w.dims[(step_1based - 1) % len(w.dims)]
        if len(w.dims) == 3:
            assert dim == lp.lp_rotation_dim(step_1based)
        st = state[dim]
        # one event between consecutive launches: the end of one interval is the start of the next
        e0 = ev(); e0.record()
        if not args.guided:           # guided: the previous step's fused call has written these sub-latents
            lp.lp_partition(st["plan"], z, st["subs"], stream)
        e1 = ev(); e1.record()
        att = []
        last = e1
        for item in st["qkv"]:
            if item is None:
                continue
            n, qd, kd, vd, od = item
            for _ in range(layers):
                if args.guided:
                    lp.lp_attention_batch(qd, kd, vd, od, 2, n, w.heads, w.head_dim, n * w.heads * w.head_dim,
                                          w.heads * w.head_dim, w.head_dim, 0.0, ws, ws_bytes, stream)
                else:
                    lp.lp_attention(qd, kd, vd, od, n, w.heads, w.head_dim, w.heads * w.head_dim, w.head_dim, 0.0, ws, ws_bytes, stream)
                a1 = ev(); a1.record()
                att.append((last, a1, n))
                last = a1
        e2 = last
        if args.guided:
            nxt = state[w.dims[step_1based % len(w.dims)]]
            lp.lp_reconstruct_guided_step_partition(st["plan"], st["preds"], st["preds_u"], 5.0, z, 1.0, -0.02, out,
                                                    nxt["plan"], nxt["subs"], stream)
        else:
            lp.lp_reconstruct(st["plan"], st["preds"], out, stream)
        e3 = ev(); e3.record()
        if rec is not None:
            rec.append((dim, w.dims[step_1based % len(w.dims)], e0, e1, att, e2, e3))

    t_spin = time.perf_counter() + args.spinup_ms * 1e-3
    spin_steps = 0
    while time.perf_counter() < t_spin:
        for i in range(len(w.dims)):
            run_step(i + 1)
        torch.cuda.synchronize()
        spin_steps += len(w.dims)
    for i in range(args.warmup):
        run_step(i + 1)
    torch.cuda.synchronize()
    records = []
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_step(args.warmup + i + 1, records)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    att_ms = att_flops = 0.0
    att_launches = 0
    part_ms = rec_ms = part_bytes = rec_bytes = 0.0
    per_dim = {}
    for dim, next_dim, e0, e1, att, e2, e3 in records:
        st = state[dim]
        part_ms += e0.elapsed_time(e1)
        rec_ms += e2.elapsed_time(e3)
        s_ext = 4.0 * st["plan"].total_elems
        s_z = 4.0 * st["plan"].latent_elems
        part_bytes += 2.0 * s_ext              # read each selected element once, write it once
        # read every prediction once, write the latent once; guided: both sets and z read, and the
        # next step's sub-latents written as well
        if args.guided:
            rec_bytes += 2.0 * s_ext + 2.0 * s_z + 4.0 * state[next_dim]["plan"].total_elems
        else:
            rec_bytes += s_ext + s_z
        d = per_dim.setdefault(synth.DIM_NAMES[dim], dict(ms=0.0, flops=0.0, launches=0))
        for a0, a1, n in att:
            t = a0.elapsed_time(a1)
            att_ms += t
            att_flops += flops_of(n)
            att_launches += 1
            d["ms"] += t; d["flops"] += flops_of(n); d["launches"] += 1

    latent_dims = latent_per_dim(lp, torch, state, w, z, stream, synth)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                       # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()

    ms_per_step = wall * 1e3 / args.steps
    value = att_flops / wall / 1e12
    achieved = att_flops / (att_ms * 1e-3) / 1e12
    traffic = None
    if args.traffic_json and os.path.exists(args.traffic_json):
        rec = json.load(open(args.traffic_json))
        if rec.get("workload") == w.name and not args.guided:
            traffic = rec.get("attention_bytes_per_launch")

    result = {
        "metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "spinup_steps": spin_steps,
        "events": event_kind, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "index": cfg, "latent": list(w.latent), "patch": list(w.patch), "K": w.K,
                   "overlap_patches": w.overlap_patches, "overlap_ratio": w.overlap_ratio, "dims": [synth.DIM_NAMES[d] for d in w.dims],
                   "heads": w.heads, "head_dim": w.head_dim, "attention_layers_per_partition": layers,
                   "guided_pair": bool(args.guided)},
        "roofline": {"kernel": "attention_kernel<%d>" % w.head_dim, "bound": "mfma",
                     "achieved": round(achieved, 3), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                     "launches": att_launches, "avg_launch_ms": round(att_ms / max(att_launches, 1), 5),
                     "avg_flops_per_launch": att_flops / max(att_launches, 1),
                     "per_dim_tflops": {k: round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) for k, v in per_dim.items()}},
        "latent_ops": {"bound": "hbm", "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                       "in_step": "partition / reconstruct as timed inside the steps (buffers reused every step: warm)",
                       "per_dim": latent_dims,
                       "partition": {"GBps": round(part_bytes / (part_ms * 1e-3) / 1e9, 1), "avg_us": round(part_ms * 1e3 / args.steps, 2),
                                     "frac": round(part_bytes / (part_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)},
                       "reconstruct": {"GBps": round(rec_bytes / (rec_ms * 1e-3) / 1e9, 1), "avg_us": round(rec_ms * 1e3 / args.steps, 2),
                                       "frac": round(rec_bytes / (rec_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)}},
        "time_split_ms_per_step": {"partition": round(part_ms / args.steps, 5), "attention": round(att_ms / args.steps, 4),
                                   "reconstruct": round(rec_ms / args.steps, 5)},
    }

    if not args.no_cpu_baseline and not args.guided:
        result["cpu_baseline"] = cpu_baseline(w, cfg, state, synth, np, torch)
    print(json.dumps(result), flush=True)
    return 0


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


def latent_per_dim(lp, torch, state, w, z, stream, synth, total_bytes=2 << 30, reps=3):
    """lp_partition, lp_reconstruct and lp_reconstruct_guided_step per partition dimension, each timed as a run of launches
    back to back between two HIP events.  "warm": every call on the same buffers (operands in L2 / Infinity Cache).  "cold": each
    call on its own copy of the buffers, the copies together (about total_bytes) several times the
    last-level cache, so that operands come from HBM."""
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
        dims_sorted = sorted(state)
        nxt_plan = state[w.dims[(w.dims.index(dim) + 1) % len(w.dims)]]["plan"]
        nxt_subs = [torch.empty(nxt_plan.total_elems, dtype=torch.float32, device="cuda") for _ in range(copies)]
        fused = lambda c0, c1: lp.lp_reconstruct_guided_step_partition(plan, preds[c0], subs[c0], 5.0, zs[c1], 1.0, -0.02,
                                                                       outs[c1], nxt_plan, nxt_subs[c1], stream)
        t = {"warm": {"partition": timed(lambda c: lp.lp_partition(plan, zs[0], subs[0], stream), 50),
                      "reconstruct": timed(lambda c: lp.lp_reconstruct(plan, preds[0], outs[0], stream), 50),
                      "guided_step": timed(lambda c: guided(0, 0), 50),
                      "guided_step_partition": timed(lambda c: fused(0, 0), 50)},
             "cold": {"partition": timed(lambda c: lp.lp_partition(plan, zs[c], subs[c], stream), copies),
                      "reconstruct": timed(lambda c: lp.lp_reconstruct(plan, preds[c], outs[c], stream), copies),
                      "guided_step": timed(lambda c: guided(c, c), copies),
                      "guided_step_partition": timed(lambda c: fused(c, c), copies)}}
        nbytes = {"partition": 2.0 * s_ext, "reconstruct": float(s_ext + s_z), "guided_step": 2.0 * s_ext + 2.0 * s_z,
                  "guided_step_partition": 2.0 * s_ext + 2.0 * s_z + 4.0 * nxt_plan.total_elems}
        entry = {"gamma": round(s_ext / s_z, 4), "copies": copies}
        for cache in ("warm", "cold"):
            entry[cache] = {}
            for name in ("partition", "reconstruct", "guided_step", "guided_step_partition"):
                gbps = nbytes[name] / (t[cache][name] * 1e-3) / 1e9
                entry[cache][name] = {"us": round(t[cache][name] * 1e3, 2), "GBps": round(gbps, 1),
                                      "frac": round(gbps / PEAK_HBM_GBPS, 4)}
        res[synth.DIM_NAMES[dim]] = entry
        del zs, subs, preds, outs, nxt_subs
    return res


def cpu_baseline(w, cfg, state, synth, np, torch):
    """Time the CPU oracle, as it stands, on a bounded sample of this workload: one step along
    every partition dimension the workload visits, partition and reconstruct in full and attention
    on every `stride`-th query row of every partition (each row over all keys).  Also compares
    the GPU's attention output on those rows with the oracle's."""
    from oracle import lp_oracle as orc
    dims = sorted(state)
    plans = {d: orc.plan(w.latent, w.patch, w.K, d, **w.overlap_args()) for d in dims}
    total_flops = sum(4.0 * p.n_tokens ** 2 * w.head_dim * w.heads for d in dims for p in plans[d].parts)
    budget_flops = 2.5e12                     # 15-20 s of oracle work on 16 cores
    stride = max(1, int(np.ceil(total_flops / budget_flops)))
    z_h = synth.latent(synth.seed_for(cfg, 0, 0, tensor=9), w.latent)
    t_part = t_rec = t_att = 0.0
    flops = bytes_part = bytes_rec = 0.0
    max_err = sum_err = 0.0
    n_cmp = 0
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
        parity_latent = parity_latent and bool(np.array_equal(st["subs"].cpu().numpy(), subs_ref))
        for kp, part in enumerate(ref_plan.parts):
            n = part.n_tokens
            if n == 0:
                continue
            q, k, v = synth.qkv_bf16(synth.seed_for(cfg, dim, kp), n, w.heads, w.head_dim)
            rows = np.arange(0, n, stride, dtype=np.int64)
            t0 = time.perf_counter()
            want = orc.attention(q, k, v, rows=rows)
            t_att += time.perf_counter() - t0
            flops += 4.0 * len(rows) * n * w.head_dim * w.heads
            got_bits = st["qkv"][kp][4].cpu().numpy().view(np.uint16)
            err = np.abs(synth.bf16_bits_to_f32(got_bits[rows]) - want)
            max_err = max(max_err, float(err.max()))
            sum_err += float(err.sum()); n_cmp += err.size
    return {"value": round(flops / t_att / 1e12, 5), "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "one step along each of %s of %s: attention on every %d-th query row of all %d partitions (all keys, "
                      "all heads; %.3g of %.3g flop) in %.1f s; partition %.1f ms and reconstruct %.1f ms in full"
                      % ("/".join(synth.DIM_NAMES[d] for d in dims), w.name, stride, w.K, flops, total_flops, t_att,
                         t_part * 1e3, t_rec * 1e3),
            "partition_GBps": round(bytes_part / t_part / 1e9, 2),
            "reconstruct_GBps": round(bytes_rec / t_rec / 1e9, 2),
            "gpu_vs_oracle_on_sample": {"attention_max_abs": max_err, "attention_mean_abs": sum_err / max(n_cmp, 1),
                                        "partition_bit_exact": parity_latent}}


if __name__ == "__main__":
    sys.exit(main())
