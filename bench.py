#!/usr/bin/env python3
"""Benchmark of the fused FlashOptim optimizer step on one MI355X.

Default workload (the one the headline metric is quoted on): FlashAdamW over the Llama-3.1-8B parameter list
(291 tensors, 8,030,261,248 parameters, 57.2 GB of resident state), one fused multi-tensor call per step
(issued as 30 back-to-back kernel launches), synthetic values.  A "step" is one pass of the whole path:
reconstruct master weights and states, AdamW update from BF16 gradients, re-quantise states, re-split
weights.  Inputs are resident in HBM before the timed region starts.

The timed call is flashoptim_adamw_step_exact, the entry point that is bit-identical to the oracle
(--rounding default times flashoptim_adamw_step instead, whose division is faithfully rounded).

Prints ONE JSON line: params/s (value), ms per step, the HBM roofline of the step kernel (algorithmic bytes
per step / time per step measured with HIP events on the launch stream; equivalently mean bytes per kernel
launch / mean launch duration), an `also` array with the other configurations measured in the same process
(the faithful entry point, gradient release, checkpoint pack / unpack, SGD and Lion on the same list, the
ResNet-50 and GPT-2 lists, each beside the arithmetic-free probe of its traffic), and the CPU oracle's
throughput on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak
BYTES_PER_PARAM = {"adamw": 12.25, "sgd": 10.125, "lion": 10.125}   # read + written, incl. FP16 scales
HYPER = {
    "adamw": dict(lr=1e-3, wd=0.01, beta1=0.9, beta2=0.999, eps=1e-8),
    "sgd": dict(lr=1e-2, wd=5e-4, momentum=0.9),
    "lion": dict(lr=1e-4, wd=0.1, beta1=0.9, beta2=0.99),
}
WORKLOADS = {
    # name: (optimizer, shapes function name, gradient distribution, gradient scale / per-tensor sigma)
    "llama31_8b_adamw": ("adamw", "llama31_8b", "normal", 1e-4),
    "llama31_8b_sgd": ("sgd", "llama31_8b", "normal", 1e-4),
    "llama31_8b_lion": ("lion", "llama31_8b", "normal", 1e-4),
    "gpt2_sgd": ("sgd", "gpt2_small", "normal", None),
    "gpt2_lion": ("lion", "gpt2_small", "normal", None),
    "resnet50_adamw": ("adamw", "resnet50", "student3", 1e-3),
    "flat_adamw": ("adamw", "flat_tensor", "normal", 1e-3),
    "llama31_8b_flat_adamw": ("adamw", "llama31_8b_flat", "normal", 1e-4),
    "llama31_8b_flat_sgd": ("sgd", "llama31_8b_flat", "normal", 1e-4),
    "llama31_8b_flat_lion": ("lion", "llama31_8b_flat", "normal", 1e-4),
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama31_8b_adamw", choices=sorted(WORKLOADS))
    ap.add_argument("--mode", default="fused", choices=["fused", "grad_release", "ckpt_pack", "ckpt_unpack"],
                    help="fused: one multi-tensor launch per step; grad_release: one call per tensor in "
                         "reverse list order with a single reused gradient buffer; ckpt_pack / ckpt_unpack: "
                         "a 'step' is one checkpoint gather / scatter of the whole list (a plain copy)")
    ap.add_argument("--variant", default="flash", choices=["flash", "wsplit", "oquant", "ref"],
                    help="flash: both techniques on (the product path); wsplit: split weights + FP32 states; "
                         "oquant: FP32 weights + 8-bit states; ref: plain FP32 optimizer (BF16 gradients). "
                         "The last three are the ablation entry points (fused mode only).")
    ap.add_argument("--rounding", default="exact", choices=["default", "exact"],
                    help="AdamW only: exact = flashoptim_adamw_step_exact (bit-identical to the oracle; what `value` "
                         "is); default = flashoptim_adamw_step (faithfully rounded division, inside the parity bar)")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the `also` measurements that the default run appends (other entry points, modes, "
                         "optimizers and lists)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true",
                    help="skip the two side measurements taken after the timed region: the arithmetic-free stream "
                         "probe (same traffic as the step) and, for AdamW, the bit-exact entry point")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


VARIANT_FLAGS = {"flash": (True, True), "wsplit": (True, False), "oquant": (False, True), "ref": (False, False)}


def variant_bytes(kind, variant):
    """Algorithmic bytes read + written per parameter."""
    split, quant = VARIANT_FLAGS[variant]
    nstate = 2 if kind == "adamw" else 1
    w = (2 + 1) * 2 if split else 4 * 2                       # weights (+ correction), in and out
    st = (1 + 2 / 32) * 2 * nstate if quant else 4 * 2 * nstate
    return w + st + 2                                         # + BF16 gradient, read once


def build_state(fo, W, torch, specs, kind, hp, dist, scale, seed, with_grads, variant="flash"):
    """Device buffers for the whole list: theta_0 is drawn per tensor in FP32 on the device and split by
    the library; gradients are drawn in BF16 on the device."""
    split, quant = VARIANT_FLAGS[variant]
    bufs = []
    for i, sp in enumerate(specs):
        b = fo.ParamBuffers(sp.numel, kind, device="cuda", with_grad=with_grads, split_weights=split,
                            quantize_states=quant)
        th = W.theta0(sp, i, seed=seed, device="cuda")
        if split:
            fo.split_weights(th, b.param, b.rho)
        else:
            b.theta.copy_(th)
        del th
        if with_grads:
            sc = W.tensor_sigma(i, seed) if scale is None else scale
            b.grad.copy_(W.grad_bf16(sp, i, 1, seed=seed, device="cuda", dist=dist, scale=sc))
        b.lr, b.weight_decay = hp["lr"], (hp["wd"] if sp.role == "matrix" else 0.0)
        bufs.append(b)
    torch.cuda.synchronize()
    return bufs


def step_call(fo, kind, tl, hp, t, exact=False):
    if isinstance(tl, fo.TensorListEx):
        if kind == "adamw":
            fo.adamw_step_ex(tl, hp["beta1"], hp["beta2"], hp["eps"], t)
        elif kind == "sgd":
            fo.sgd_step_ex(tl, hp["momentum"])
        else:
            fo.lion_step_ex(tl, hp["beta1"], hp["beta2"])
    elif kind == "adamw":
        (fo.adamw_step_exact if exact else fo.adamw_step)(tl, hp["beta1"], hp["beta2"], hp["eps"], t)
    elif kind == "sgd":
        fo.sgd_step(tl, hp["momentum"])
    else:
        fo.lion_step(tl, hp["beta1"], hp["beta2"])


def cpu_baseline(W, specs, kind, hp, dist, scale, seed, target_seconds):
    """The oracle, as it stands, on a bounded sample of the same workload, on this host's cores."""
    import numpy as np
    import torch
    import oracle

    # sample: the first tensors of the list up to ~64M parameters (for the Llama list: the leading
    # 64M-element slice of the embedding plus nothing else would be unrepresentative, so take one
    # decoder layer's tensors when the list has them)
    names = [s.name for s in specs]
    if any(n.startswith("layers.0.") for n in names):
        sample = [(i, s) for i, s in enumerate(specs) if s.name.startswith("layers.0.")]
        what = "decoder layer 0 of the list (9 tensors)"
    else:
        sample, tot = [], 0
        for i, s in enumerate(specs):
            if tot > 64e6:
                break
            sample.append((i, s)); tot += s.numel
        what = f"first {len(sample)} tensors of the list"
        if len(sample) == 1 and sample[0][1].numel > (1 << 26):
            s0 = sample[0][1]
            sample = [(0, W.ParamSpec(s0.name, (1 << 26,), s0.role))]
            what = "leading 2^26 elements of the single tensor"
    n = sum(s.numel for _, s in sample)
    states, grads = [], []
    for i, s in sample:
        states.append(oracle.TensorState(W.theta0(s, i, seed=seed).numpy(), kind))
        sc = W.tensor_sigma(i, seed) if scale is None else scale
        grads.append(W.grad_bf16(s, i, 1, seed=seed, dist=dist, scale=sc).view(torch.int16).numpy().view(np.uint16))
    threads = oracle.max_threads()

    def one(t, nthreads=0):
        for (i, s), st, g in zip(sample, states, grads):
            wd = hp["wd"] if s.role == "matrix" else 0.0
            if kind == "adamw":
                oracle.adamw_step(st, g, hp["lr"], wd, hp["beta1"], hp["beta2"], hp["eps"], t, nthreads=nthreads)
            elif kind == "sgd":
                oracle.sgd_step(st, g, hp["lr"], wd, hp["momentum"], nthreads=nthreads)
            else:
                oracle.lion_step(st, g, hp["lr"], wd, hp["beta1"], hp["beta2"], nthreads=nthreads)

    one(1)                                  # untimed: page in, reach a non-zero state
    t0 = time.perf_counter(); one(2); dt = time.perf_counter() - t0
    reps = max(1, min(200, int(target_seconds / max(dt, 1e-3))))
    t0 = time.perf_counter()
    for r in range(reps):
        one(3 + r)
    total = time.perf_counter() - t0
    # the same sample on one thread, one step
    t0 = time.perf_counter(); one(3 + reps, nthreads=1); single = time.perf_counter() - t0
    return {"value": n * reps / total, "unit": "params/s", "cores": threads, "kind": "oracle",
            "sample": f"{what}: {n} params x {reps} steps, {total:.1f} s",
            "single_thread_value": n / single}


def kernel_source_sha():
    """SHA-256 (first 16 hex digits) of the device code: a counter summary under profiles/ names the sources it
    was measured on, and stops being reported once they have changed."""
    import hashlib
    h = hashlib.sha256()
    for rel in ("paper_2602_23349_amd/csrc/flashoptim_kernels.hip", "paper_2602_23349_amd/csrc/flashoptim_device.h"):
        h.update(open(os.path.join(ROOT, rel), "rb").read())
    return h.hexdigest()[:16]


def read_profile(path):
    vals = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            v = v.split("#")[0].strip()
            try:
                vals[k.strip()] = float(v)
            except ValueError:
                vals[k.strip()] = v
    return vals


def read_traffic(kind, workload, entry="exact"):
    """HBM bytes per step (all kernel launches of one call) RECORDED by rocprofv3 --pmc (FETCH_SIZE,
    WRITE_SIZE) in a separate, committed run: (bytes, source) - or (None, None) when no summary exists for
    this workload or the device code has changed since it was taken."""
    name = f"{kind}_step{'_exact' if (kind == 'adamw' and entry == 'exact') else ''}_{workload}_pmc.txt"
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, None
    vals = read_profile(path)
    if vals.get("KERNEL_SOURCE_SHA") != kernel_source_sha():
        return None, {"file": "profiles/" + name, "stale": True}
    return vals.get("HBM_BYTES_PER_STEP"), {"file": "profiles/" + name, "kernel_source_sha": vals["KERNEL_SOURCE_SHA"],
                                             "recorded_not_measured_in_this_run": True}


def kernel_label(kind, release, exact, ckpt=False):
    """The step kernel's name as rocprofv3 prints it: <KIND, VEC, THREADS, DIRECT, SPLIT, QUANT, EXACT>."""
    if ckpt:
        return "fo::copy_kernel"
    k = ["adamw", "sgd", "lion"].index(kind)
    tf = lambda b: "true" if b else "false"
    # SGD, Lion and every ablation variant are instantiated with EXACT = true (they have no division to shorten)
    return f"fo::step_kernel<{k}, 8, {256 if k == 0 else 512}, {tf(release)}, true, true, {tf(exact or k != 0)}>"


def time_calls(torch, stream, fn, steps, warmup=2):
    """ms per call of fn(), HIP events on `stream` around `steps` calls after `warmup` untimed ones."""
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(steps):
        fn()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def also_measurements(fo, W, torch, stream, specs, bufs, tl, hp, steps, t_start):
    """The other configurations, measured after the timed region on the state that is already resident
    (Llama list) or on small lists built here.  Each entry: what ran, ms per step, algorithmic GB/s, fraction
    of the 8 TB/s peak, and the arithmetic-free probe of the same traffic where one exists."""
    import types
    out = []
    n = sum(s.numel for s in specs)
    t = [t_start]

    def entry(name, entry_point, ms, bytes_per_step, probe_ms=None, **extra):
        g = bytes_per_step / (ms * 1e-3) / 1e9
        d = {"name": name, "entry_point": entry_point, "ms_per_step": ms, "achieved": g, "unit": "GB/s",
             "frac": g / HBM_PEAK_GBPS}
        if probe_ms:
            pg = bytes_per_step / (probe_ms * 1e-3) / 1e9
            d["same_traffic_without_arithmetic"] = pg
            d["frac_of_that"] = g / pg
        d.update(extra)
        out.append(d)

    def adamw(fn, lst):
        def call():
            t[0] += 1
            fn(lst, hp["beta1"], hp["beta2"], hp["eps"], t[0])
        return call

    # the faithful entry point on the same list
    probe_ms = time_calls(torch, stream, lambda: fo.stream_probe("adamw", tl), steps)
    ms = time_calls(torch, stream, adamw(fo.adamw_step, tl), steps)
    entry("llama31_8b_adamw fused, faithful division", "flashoptim_adamw_step", ms, 12.25 * n, probe_ms,
          kernel=kernel_label("adamw", False, False))
    # gradient release: one call per tensor in reverse order through ONE gradient buffer (the largest tensor's)
    gbuf = max((b.grad for b in bufs), key=lambda g: g.numel())
    singles = []
    for i in reversed(range(len(specs))):
        tl.set_grad(i, gbuf)
        singles.append(tl.slice(i))

    def release(fn):
        def call():
            t[0] += 1
            for s1 in singles:
                fn(s1, hp["beta1"], hp["beta2"], hp["eps"], t[0])
        return call

    ms = time_calls(torch, stream, release(fo.adamw_step_exact), steps)
    entry("llama31_8b_adamw gradient release (291 calls per step)", "flashoptim_adamw_step_exact", ms, 12.25 * n,
          kernel=kernel_label("adamw", True, True), resident_bytes_per_param=5.125)
    ms = time_calls(torch, stream, release(fo.adamw_step), steps)
    entry("llama31_8b_adamw gradient release, faithful division", "flashoptim_adamw_step", ms, 12.25 * n,
          kernel=kernel_label("adamw", True, False), resident_bytes_per_param=5.125)
    # per-tensor calls again, alternating between two side streams (and two gradient buffers, so that a gradient is
    # never overwritten while the previous call on the other stream may still read its own): consecutive launches
    # then overlap at their boundaries instead of each waiting for the previous one to drain.  The side streams
    # start after the work already on the main stream and the main stream waits for both at the end of the step.
    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    gbuf2 = gbuf.clone()
    singles2 = []
    for k, i in enumerate(reversed(range(len(specs)))):
        tl.set_grad(i, gbuf if k % 2 == 0 else gbuf2)
        singles2.append(tl.slice(i))

    def release_two_streams():
        t[0] += 1
        for sd in side:
            sd.wait_stream(stream)
        for k, s1 in enumerate(singles2):
            fo.adamw_step_exact(s1, hp["beta1"], hp["beta2"], hp["eps"], t[0], stream=side[k % 2])
        for sd in side:
            stream.wait_stream(sd)

    ms = time_calls(torch, stream, release_two_streams, steps)
    entry("llama31_8b_adamw gradient release, calls alternating between two streams", "flashoptim_adamw_step_exact", ms,
          12.25 * n, kernel=kernel_label("adamw", True, True),
          resident_bytes_per_param=5.125 + 2.0 * gbuf.numel() / n)
    del gbuf2, singles2
    # the same with one call per decoder layer (its 9 tensors as one list; embedding, and final norm + head, apart):
    # 34 calls per step, the layer's gradients carved out of the same single buffer
    groups, cur = [], []
    for i, sp in enumerate(specs):
        layer = sp.name.split(".")[1] if sp.name.startswith("layers.") else sp.name.split(".")[0]
        if cur and cur[0][0] != layer and not (cur[0][0] == "norm" and layer == "lm_head"):
            groups.append([j for _, j in cur]); cur = []
        cur.append((layer, i))
    groups.append([j for _, j in cur])
    layer_lists = []
    need = max(sum((bufs[j].numel + 255) // 256 * 256 for j in g) for g in groups)
    glayer = torch.empty(need, dtype=gbuf.dtype, device=gbuf.device)      # one buffer for a whole layer's gradients
    glayer[:gbuf.numel()].copy_(gbuf[:min(need, gbuf.numel())])
    if need > gbuf.numel():
        glayer[gbuf.numel():].copy_(gbuf[:need - gbuf.numel()])
    for idx in reversed(groups):
        off, lst = 0, []
        for j in idx:
            b = bufs[j]
            lst.append(types.SimpleNamespace(param=b.param, rho=b.rho, grad=glayer[off:off + b.numel], m_q=b.m_q,
                                             m_scale=b.m_scale, v_q=b.v_q, v_scale=b.v_scale, numel=b.numel, lr=b.lr,
                                             weight_decay=b.weight_decay))
            off += (b.numel + 255) // 256 * 256
        assert off <= glayer.numel()
        layer_lists.append(fo.TensorList(lst))

    def release_by_layer():
        t[0] += 1
        for l1 in layer_lists:
            fo.adamw_step_exact(l1, hp["beta1"], hp["beta2"], hp["eps"], t[0])

    ms = time_calls(torch, stream, release_by_layer, steps)
    entry(f"llama31_8b_adamw gradient release by layer ({len(layer_lists)} calls per step)", "flashoptim_adamw_step_exact",
          ms, 12.25 * n, kernel=kernel_label("adamw", False, True),
          resident_bytes_per_param=5.125 + 2.0 * max(sum(bufs[j].numel for j in g) for g in groups) / n)
    del layer_lists, glayer
    for i, b in enumerate(bufs):
        tl.set_grad(i, b.grad)
    # checkpoint gather / scatter of the whole list
    numels = [s.numel for s in specs]
    blob = torch.empty(fo.checkpoint_size("adamw", numels), dtype=torch.uint8, device="cuda")
    payload = sum(5 * m + 4 * ((m + 31) // 32) for m in numels)
    ms = time_calls(torch, stream, lambda: fo.checkpoint_pack("adamw", tl, 1, blob), steps)
    entry("llama31_8b_adamw checkpoint pack", "flashoptim_checkpoint_pack", ms, 2.0 * payload, kernel="fo::copy_kernel")
    ms = time_calls(torch, stream, lambda: fo.checkpoint_unpack("adamw", blob, tl), steps)
    entry("llama31_8b_adamw checkpoint unpack", "flashoptim_checkpoint_unpack", ms, 2.0 * payload, kernel="fo::copy_kernel")
    del blob
    torch.cuda.empty_cache()
    # SGD and Lion over the same list (the AdamW buffers without the variance; momentum restarted from Q(0))
    for kind in ("sgd", "lion"):
        h = HYPER[kind]
        lst = []
        for sp, b in zip(specs, bufs):
            b.m_q.zero_(); b.m_scale.zero_()
            lst.append(types.SimpleNamespace(param=b.param, rho=b.rho, grad=b.grad, m_q=b.m_q, m_scale=b.m_scale,
                                             v_q=None, v_scale=None, numel=b.numel, lr=h["lr"],
                                             weight_decay=h["wd"] if sp.role == "matrix" else 0.0))
        tl2 = fo.TensorList(lst)
        call = (lambda: fo.sgd_step(tl2, h["momentum"])) if kind == "sgd" else (lambda: fo.lion_step(tl2, h["beta1"], h["beta2"]))
        ms = time_calls(torch, stream, call, steps, warmup=3)
        probe_ms = time_calls(torch, stream, lambda: fo.stream_probe(kind, tl2), steps)
        entry(f"llama31_8b_{kind} fused", f"flashoptim_{kind}_step", ms, 10.125 * n, probe_ms,
              kernel=kernel_label(kind, False, True))
    return out


def ablation_measurements(fo, W, torch, stream, specs, steps):
    """The paper's two ablations and the plain FP32 optimizer (Section 4.3) over the Llama list, through the same
    multi-tensor machinery: what the compressed layout buys on this chip.  Each variant builds its own state."""
    out = []
    kind, hp = "adamw", HYPER["adamw"]
    n = sum(s.numel for s in specs)
    names = {"wsplit": "weight split only (FP32 states)", "oquant": "state quantisation only (FP32 weights)",
             "ref": "plain FP32 AdamW with BF16 gradients"}
    for variant in ("wsplit", "oquant", "ref"):
        bufs = build_state(fo, W, torch, specs, kind, hp, "normal", 1e-4, 0, with_grads=True, variant=variant)
        tl = fo.TensorListEx(bufs)
        t = [0]

        def call():
            t[0] += 1
            fo.adamw_step_ex(tl, hp["beta1"], hp["beta2"], hp["eps"], t[0])

        ms = time_calls(torch, stream, call, steps, warmup=2)
        bpp = variant_bytes(kind, variant)
        g = bpp * n / (ms * 1e-3) / 1e9
        out.append({"name": f"llama31_8b_adamw fused, {names[variant]}", "entry_point": "flashoptim_adamw_step_ex",
                    "ms_per_step": ms, "bytes_per_param": bpp, "achieved": g, "unit": "GB/s", "frac": g / HBM_PEAK_GBPS})
        del bufs, tl
        torch.cuda.empty_cache()
    return out


def small_list_measurements(fo, W, torch, stream, steps=200):
    """The small workloads (cache-sized: not roofline points), each beside its probe: the flat 2^20-element tensor,
    the ResNet-50 list and the GPT-2 list."""
    out = []
    for workload in ("flat_adamw", "resnet50_adamw", "gpt2_sgd", "gpt2_lion"):
        kind, shape_fn, dist, scale = WORKLOADS[workload]
        h = HYPER[kind]
        specs = getattr(W, shape_fn)()
        n = sum(s.numel for s in specs)
        bufs = build_state(fo, W, torch, specs, kind, h, dist, scale, 0, with_grads=True)
        tl = fo.TensorList(bufs)
        t = [0]

        def call():
            t[0] += 1
            step_call(fo, kind, tl, h, t[0], exact=True)

        # A step of these lists takes 5-200 us and the state was just built on the host: the first ~15 ms of GPU
        # work after such an idle stretch run ~15 % slower (clocks ramping up), which would cover the whole timed
        # region.  So the untimed warm-up is sized to 100 ms of work from a first rough timing.
        rough = time_calls(torch, stream, call, 20, warmup=10)
        ms = time_calls(torch, stream, call, steps, warmup=max(10, int(100.0 / rough)))
        probe_ms = time_calls(torch, stream, lambda: fo.stream_probe(kind, tl), steps, warmup=10)
        bpp = BYTES_PER_PARAM[kind]
        g = bpp * n / (ms * 1e-3) / 1e9
        pg = bpp * n / (probe_ms * 1e-3) / 1e9
        out.append({"name": f"{workload} fused ({len(specs)} tensors, {n} params; cache-sized, not a roofline point)",
                    "entry_point": "flashoptim_adamw_step_exact" if kind == "adamw" else f"flashoptim_{kind}_step",
                    "ms_per_step": ms, "params_per_s": n / (ms * 1e-3), "achieved": g, "unit": "GB/s",
                    "frac": g / HBM_PEAK_GBPS, "same_traffic_without_arithmetic": pg, "frac_of_that": g / pg,
                    "kernel": kernel_label(kind, len(specs) == 1, True)})
        del bufs, tl
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1. "
              "The step needs no communication: a multi-GPU job runs this same kernel on each rank's shard.",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2602_23349_amd as fo
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    fo.load_library()
    torch.cuda.set_device(0)

    kind, shape_fn, dist, scale = WORKLOADS[args.workload]
    hp = HYPER[kind]
    specs = getattr(W, shape_fn)()
    n_params = sum(s.numel for s in specs)
    seed = 0
    release = args.mode == "grad_release"
    ckpt = args.mode.startswith("ckpt")
    exact = args.rounding == "exact"

    if args.variant != "flash" and args.mode != "fused":
        print("bench.py: --variant other than flash is available in fused mode only", file=sys.stderr)
        sys.exit(2)
    bufs = build_state(fo, W, torch, specs, kind, hp, dist, scale, seed, with_grads=not (release or ckpt),
                       variant=args.variant)
    tl = fo.TensorList(bufs) if args.variant == "flash" else fo.TensorListEx(bufs)
    stream = torch.cuda.current_stream()

    if ckpt:
        blob = torch.empty(fo.checkpoint_size(kind, [s.numel for s in specs]), dtype=torch.uint8, device="cuda")
        fo.checkpoint_pack(kind, tl, 1, blob)

        def do_step(t):
            if args.mode == "ckpt_pack":
                fo.checkpoint_pack(kind, tl, t, blob)
            else:
                fo.checkpoint_unpack(kind, blob, tl)
    elif release:
        # one reusable gradient buffer of the largest tensor's size; per-tensor calls in reverse order
        gmax = max(s.numel for s in specs)
        gbuf = W.grad_bf16(W.ParamSpec("g", (gmax,), "matrix"), 0, 1, seed=seed, device="cuda", dist="normal",
                           scale=scale or 1e-3)
        singles = []
        for i in reversed(range(len(specs))):
            tl.set_grad(i, gbuf)
            singles.append(tl.slice(i))

        def do_step(t):
            for s in singles:
                step_call(fo, kind, s, hp, t, exact)
    else:
        def do_step(t):
            step_call(fo, kind, tl, hp, t, exact)

    t = 0
    for _ in range(args.warmup):
        t += 1
        do_step(t)
    torch.cuda.synchronize()

    # timed region: K steps, HIP events on the stream the kernels are launched on
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    wall0 = time.perf_counter()
    ev[0].record(stream)
    for k in range(args.steps):
        t += 1
        do_step(t)
        ev[k + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    per_step_ms = [ev[k].elapsed_time(ev[k + 1]) for k in range(args.steps)]
    total_ms = ev[0].elapsed_time(ev[args.steps])
    ms_per_step = total_ms / args.steps
    value = n_params * args.steps / (total_ms * 1e-3)

    calls = len(specs) if release else 1
    if ckpt or args.variant != "flash":
        launches = None if args.variant != "flash" else 1
    elif release:
        launches = sum(fo.step_launch_count(kind, [s.numel]) for s in specs)
    else:
        launches = fo.step_launch_count(kind, [s.numel for s in specs])
    bytes_per_param = variant_bytes(kind, args.variant)
    assert args.variant != "flash" or bytes_per_param == BYTES_PER_PARAM[kind]
    algo_bytes = bytes_per_param * n_params                 # per step = per launch in fused mode
    if ckpt:
        payload = sum(2 * s.numel + s.numel * (3 if kind == "adamw" else 2)
                      + 2 * ((s.numel + 31) // 32) * (2 if kind == "adamw" else 1) for s in specs)
        algo_bytes = 2.0 * payload                          # every payload byte is read once and written once
    achieved = algo_bytes / (ms_per_step * 1e-3) / 1e9
    traffic, traffic_source = (None, None) if (release or ckpt or args.variant != "flash") else \
        read_traffic(kind, args.workload, args.rounding)
    # the memory ceiling of this access pattern: the same bytes through the same launch shape with no
    # arithmetic (fused flash mode only; run after the timed region, on the same list)
    probe = None
    if args.variant == "flash" and args.mode == "fused" and not args.no_probe:
        fo.stream_probe(kind, tl)
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record(stream)
        for _ in range(args.steps):
            fo.stream_probe(kind, tl)
        p1.record(stream)
        torch.cuda.synchronize()
        probe = algo_bytes / (p0.elapsed_time(p1) / args.steps * 1e-3) / 1e9
    # the clock the compute units run at during the step and during the probe (the step kernels run under the
    # package power limit): a one-wavefront monitor on a stream of its own samples it while K more steps run
    clocks = None
    if args.variant == "flash" and args.mode == "fused" and not args.no_probe:
        import numpy as np

        def clock_during(fn, approx_ms):
            mon = fo.ClockMonitor(n_samples=max(8, int(0.6 * args.steps * approx_ms)), seconds_per_sample=1e-3)
            mon.start()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return float(np.median(mon.ghz()))

        def one_more_step():
            nonlocal t
            t += 1
            do_step(t)

        idle = fo.ClockMonitor(n_samples=8, seconds_per_sample=1e-3)
        idle.start()
        clocks = {"idle": float(np.median(idle.ghz())),
                  "step": clock_during(one_more_step, ms_per_step),
                  "same_traffic_without_arithmetic": clock_during(lambda: fo.stream_probe(kind, tl), ms_per_step)}
    # the other configurations (default run on the headline workload only)
    also = None
    if (args.workload == "llama31_8b_adamw" and args.variant == "flash" and args.mode == "fused" and exact
            and not args.no_also):
        also = also_measurements(fo, W, torch, stream, specs, bufs, tl, hp, max(5, args.steps // 2), t + 1000)
        also += small_list_measurements(fo, W, torch, stream)
        del bufs, tl
        bufs = tl = None
        torch.cuda.empty_cache()
        also += ablation_measurements(fo, W, torch, stream, specs, max(5, args.steps // 2))
    out = {
        "metric": "optimizer_step_params_per_sec", "value": value, "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "optimizer": kind, "tensors": len(specs), "params": n_params,
                   "mode": args.mode, "variant": args.variant,
                   "entry_point": (("flashoptim_adamw_step_exact" if exact else "flashoptim_adamw_step")
                                   if kind == "adamw" and args.variant == "flash" and not ckpt else
                                   (f"flashoptim_checkpoint_{args.mode[5:]}" if ckpt else
                                    f"flashoptim_{kind}_step{'_ex' if args.variant != 'flash' else ''}")),
                   "rounding": (args.rounding if kind == "adamw" and args.variant == "flash" and not ckpt else None),
                   "calls_per_step": calls,
                   "kernel_launches_per_step": launches,
                   "resident_bytes_per_param": (7.125 if kind == "adamw" else 6.0625) - (2 if release else 0),
                   "min_ms_step": min(per_step_ms), "median_ms_step": sorted(per_step_ms)[len(per_step_ms) // 2],
                   "max_ms_step": max(per_step_ms),
                   "wall_ms_per_step": wall * 1e3 / args.steps},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": (traffic / launches) if (traffic and launches) else None,
                     "traffic_per_step": traffic,
                     "traffic_source": traffic_source,
                     "kernel": (kernel_label(kind, release, exact, ckpt) if args.variant == "flash" else
                                "fo::step_kernel<...> (ablation variant)"),
                     "algorithmic_bytes_per_step": algo_bytes,
                     "algorithmic_bytes_per_launch": (algo_bytes / launches) if launches else None,
                     "bytes_per_param": bytes_per_param,
                     "same_traffic_without_arithmetic": probe,
                     "frac_of_that": (achieved / probe) if probe else None,
                     "shader_clock_ghz": clocks},
    }
    if also is not None:
        out["also"] = also
    if not args.no_cpu_baseline and not ckpt and args.variant == "flash":
        del bufs, tl
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(W, specs, kind, hp, dist, scale, seed, args.cpu_seconds)
        out["cpu_baseline"]["gpu_over_cpu"] = value / out["cpu_baseline"]["value"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
