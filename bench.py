#!/usr/bin/env python3
"""Benchmark of the AGoQ quantization hot path on one MI355X.

One "step" is one pass of the whole path over the LLaMA-8B-shaped workload:
  * quantize the five stored activations of a decoder layer (seq 4096, micro-batch 1:
    three [4096,4096] and two [4096,14336] bf16 tensors) under the bit map
    norm inputs 8-bit, linear / FFN-intermediate inputs 4-bit, group 128 (one launch for
    the layer);
  * store one decoder layer's fp32 gradient (218,103,808 elements) as int8, group 128;
  * local reduce + requantize of K=8 such int8 gradients (the receive buffer of the
    All-to-All), n = 218,103,808;
  * dequantize the five stored activations back to bf16 (one launch).
The order puts ~3 GB of gradient traffic between writing the activation codes and reading
them back, so no launch finds its input in the last-level cache.

The figure of merit is effective HBM bandwidth: algorithmic bytes (read the tensor once,
write codes + scales once, or the reverse) divided by time.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0
# HBM bytes per launch of the K=8 reduce kernel on this workload, from hardware counters
# (FETCH_SIZE and WRITE_SIZE runs scaled by a plain copy; summary under profiles/)
TRAFFIC_REDUCE_K8_BYTES = 2024878722
GROUP = 128
K_CHUNKS = 8
SLOT_NAMES = ("norm1_in", "oproj_in", "norm2_in", "gate", "up")


def algo_bytes_act(numel, bits, group=GROUP):
    return numel * 2 + numel * bits // 8 + 4 * (numel // group)


def algo_bytes_grad_quant(numel, group=GROUP):
    return numel * 4 + numel + 4 * (numel // group)


def algo_bytes_reduce(numel, K, group=GROUP):
    return (K + 1) * (numel + 4 * (numel // group))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device copy a few times and exit: gives the hardware "
                         "counters a kernel of known traffic to be scaled against")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU's share of the path and uses no collective; "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import workloads as wl
    import paper_2605_00539_amd as agoq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    agoq.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.calibrate_copy:
        n = 1 << 28                                   # 1 GiB of fp32 read, 1 GiB written
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "read_bytes_per_launch": 4 * n,
                          "write_bytes_per_launch": 4 * n, "launches": 5}))
        return 0

    # ---- inputs (seeded, synthetic, generated on the device) ---------------------------
    acfg = wl.CONFIGS["llama8b_act"]
    gcfg = wl.CONFIGS["llama8b_grad"]
    rows = acfg["acts"]["A"]["rows"]
    hidden, ffn = acfg["acts"]["A"]["cols"], acfg["acts"]["F"]["cols"]
    bitmap = agoq.layer_bitmap(5)                 # [8, 4, 8, 4, 4]
    acts, act_bits = [], []
    for slot, name in enumerate(SLOT_NAMES):
        cols = ffn if name in ("gate", "up") else hidden
        x = wl.act_device(rows, cols, acfg["seed"] + slot, acfg["dist"],
                          wl.n_outlier_channels(cols, acfg["outlier_frac"]), acfg["outlier_scale"])
        acts.append(x.reshape(-1))
        act_bits.append(bitmap[slot])
    n_grad = gcfg["n"]
    grad = wl.grad_device(n_grad, gcfg["seed"], gcfg["sigma"], gcfg["spike_frac"], gcfg["spike_scale"])
    # the K peers' int8 gradients: quantize K seeded gradients with the library (set-up, untimed)
    n_groups = n_grad // GROUP
    in_codes = torch.empty((K_CHUNKS, n_grad), dtype=torch.int8, device=dev)
    in_scales = torch.empty((K_CHUNKS, n_groups), dtype=torch.float32, device=dev)
    for k in range(K_CHUNKS):
        gk = grad if k == 0 else wl.grad_device(n_grad, gcfg["seed"] + 1 + k, gcfg["sigma"],
                                                gcfg["spike_frac"], gcfg["spike_scale"])
        agoq.grad_quant(gk, GROUP, codes=in_codes[k], scales=in_scales[k])
        torch.cuda.synchronize()
        del gk

    # ---- outputs, allocated once ------------------------------------------------------
    act_codes = [torch.empty(x.numel() * b // 8, dtype=torch.uint8, device=dev) for x, b in zip(acts, act_bits)]
    act_scales = [torch.empty(x.numel() // GROUP, dtype=torch.float32, device=dev) for x in acts]
    act_out = [torch.empty_like(x) for x in acts]
    g_codes = torch.empty(n_grad, dtype=torch.int8, device=dev)
    g_scales = torch.empty(n_groups, dtype=torch.float32, device=dev)
    r_codes = torch.empty(n_grad, dtype=torch.int8, device=dev)
    r_scales = torch.empty(n_groups, dtype=torch.float32, device=dev)

    bytes_quant = sum(algo_bytes_act(x.numel(), b) for x, b in zip(acts, act_bits))
    bytes_dequant = bytes_quant
    bytes_gq = algo_bytes_grad_quant(n_grad)
    bytes_red = algo_bytes_reduce(n_grad, K_CHUNKS)
    bytes_step = bytes_quant + bytes_dequant + bytes_gq + bytes_red

    stream = torch.cuda.current_stream()
    # descriptor arrays of the two layer launches (host memory, marshalled once)
    q_slots = agoq.layer_slots(acts, act_bits, act_codes, act_scales)
    d_slots = agoq.layer_slots(act_out, act_bits, act_codes, act_scales)

    def step(ev=None):
        """One pass of the path.  ev: optional dict of per-kernel-class event lists."""
        def mark(name):
            if ev is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record(stream)
                ev[name].append(e)
        mark("t0")
        agoq.act_quant_layer(acts, GROUP, act_bits, slots=q_slots, stream=stream)
        mark("t1")
        agoq.grad_quant(grad, GROUP, codes=g_codes, scales=g_scales, stream=stream)
        mark("t2")
        agoq.grad_reduce_requant(in_codes, in_scales, n_grad, GROUP, out_codes=r_codes,
                                 out_scales=r_scales, stream=stream)
        mark("t3")
        agoq.act_dequant_layer(act_codes, act_scales, None, GROUP, act_bits, outs=act_out,
                               slots=d_slots, stream=stream)
        mark("t4")

    # ---- warm-up, then the timed region -------------------------------------------------
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # events around the dominant kernel (the K-way reduce) of every timed step, on the
    # stream the kernels are launched on
    red_events = []
    t_start = time.perf_counter()
    for _ in range(args.steps):
        agoq.act_quant_layer(acts, GROUP, act_bits, slots=q_slots, stream=stream)
        agoq.grad_quant(grad, GROUP, codes=g_codes, scales=g_scales, stream=stream)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        agoq.grad_reduce_requant(in_codes, in_scales, n_grad, GROUP, out_codes=r_codes,
                                 out_scales=r_scales, stream=stream)
        e1.record(stream)
        red_events.append((e0, e1))
        agoq.act_dequant_layer(act_codes, act_scales, None, GROUP, act_bits, outs=act_out,
                               slots=d_slots, stream=stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    value = bytes_step / (elapsed / args.steps) / 1e9
    red_ms = sum(a.elapsed_time(b) for a, b in red_events) / len(red_events)
    red_gbps = bytes_red / (red_ms * 1e-3) / 1e9

    # ---- per-kernel-class breakdown (separate, untimed for `value`) ----------------------
    ev = {k: [] for k in ("t0", "t1", "t2", "t3", "t4")}
    for _ in range(min(args.steps, 20)):
        step(ev)
    torch.cuda.synchronize()

    def avg_ms(a, b):
        return sum(x.elapsed_time(y) for x, y in zip(ev[a], ev[b])) / len(ev[a])

    kernels = {}
    for name, a, b, nbytes in (("act_quant_layer", "t0", "t1", bytes_quant),
                               ("grad_quant", "t1", "t2", bytes_gq),
                               ("grad_reduce_requant_k8", "t2", "t3", bytes_red),
                               ("act_dequant_layer", "t3", "t4", bytes_dequant)):
        ms = avg_ms(a, b)
        gbps = nbytes / (ms * 1e-3) / 1e9
        kernels[name] = {"us": round(ms * 1e3, 2), "GB/s": round(gbps, 1),
                         "frac_of_peak": round(gbps / PEAK_HBM_GBPS, 4), "algo_MB": round(nbytes / 1e6, 1)}

    # ---- CPU baseline: the oracle on a bounded sample of the same inputs -------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(torch, acts, act_bits, act_codes, act_scales, act_out, grad, g_codes,
                           g_scales, in_codes, in_scales, r_codes, r_scales, n_grad)

    out = {
        "metric": "effective HBM GB/s (quant, dequant, grad reduce) and % of MI355X peak",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "LLaMA-8B-shaped decoder layer: 5 stored activations seq 4096 mb 1 "
                        "(bits %s, group 128) quant+dequant, fp32 gradient of 218,103,808 -> int8, "
                        "8-chunk local reduce+requant" % (bitmap,),
            "group": GROUP, "K": K_CHUNKS, "algo_bytes_per_step": bytes_step,
        },
        "frac_of_peak": round(value / PEAK_HBM_GBPS, 4),
        "roofline": {
            "bound": "hbm", "kernel": "grad_reduce_kernel<128,8>",
            "achieved": round(red_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
            "frac": round(red_gbps / PEAK_HBM_GBPS, 4), "traffic": TRAFFIC_REDUCE_K8_BYTES,
            "algo_bytes_per_launch": bytes_red, "avg_launch_us": round(red_ms * 1e3, 2),
        },
        "kernels": kernels,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    return 0


def cpu_baseline(torch, acts, act_bits, act_codes, act_scales, act_out, grad, g_codes, g_scales,
                 in_codes, in_scales, r_codes, r_scales, n_grad):
    """Time the oracle (as it stands) on the host, with all its threads, on one whole step of
    the same inputs (three passes, the median counts: some 20 core-seconds of work), and
    check the GPU outputs of the last timed step against it, every byte.  A one-thread
    figure on 1/16 of the step follows."""
    import numpy as np
    import oracle

    def bits_of(t):
        return t.view(torch.int16).cpu().numpy().view(np.uint16)

    threads = oracle.max_threads()
    host_acts = [bits_of(x) for x in acts]
    ng = nr = n_grad
    gh = grad[:ng].cpu().numpy()
    ch = np.ascontiguousarray(in_codes[:, :nr].cpu().numpy())
    sh = np.ascontiguousarray(in_scales[:, :nr // GROUP].cpu().numpy())

    def one_pass():
        nbytes, secs, outs = 0, 0.0, []
        for xb, b in zip(host_acts, act_bits):
            t = time.perf_counter()
            oc, os_ = oracle.act_quant(xb, GROUP, b)
            oy = oracle.act_dequant(oc, os_, xb.size, GROUP, b)
            secs += time.perf_counter() - t
            nbytes += 2 * algo_bytes_act(xb.size, b)
            outs.append((oc, os_, oy))
        t = time.perf_counter()
        gq = oracle.grad_quant(gh, GROUP)
        red = oracle.grad_reduce_requant(ch, sh, nr, GROUP)
        secs += time.perf_counter() - t
        nbytes += algo_bytes_grad_quant(ng) + algo_bytes_reduce(nr, K_CHUNKS)
        return nbytes, secs, outs, gq, red

    passes = sorted((one_pass() for _ in range(3)), key=lambda p: p[1])
    nbytes, secs, outs, gq, red = passes[1]                  # the median pass
    ok = True
    for (oc, os_, oy), c, s, y in zip(outs, act_codes, act_scales, act_out):
        ok &= np.array_equal(c.cpu().numpy(), oc) and np.array_equal(
            s.cpu().numpy().view(np.uint32), os_.view(np.uint32)) and np.array_equal(bits_of(y), oy)
    ok &= np.array_equal(g_codes[:ng].cpu().numpy(), gq[0]) and np.array_equal(
        g_scales[:ng // GROUP].cpu().numpy().view(np.uint32), gq[1].view(np.uint32))
    ok &= np.array_equal(r_codes[:nr].cpu().numpy(), red[0]) and np.array_equal(
        r_scales[:nr // GROUP].cpu().numpy().view(np.uint32), red[1].view(np.uint32))
    # one thread: the first stored activation (quantize + dequantize), 1/16 of the gradient
    # store and 1/16 of the reduce
    oracle.set_threads(1)
    xb = host_acts[0]
    n16 = (n_grad // 16) // GROUP * GROUP
    ch16 = np.ascontiguousarray(ch[:, :n16])
    sh16 = np.ascontiguousarray(sh[:, :n16 // GROUP])
    t = time.perf_counter()
    oc, os_ = oracle.act_quant(xb, GROUP, act_bits[0])
    oracle.act_dequant(oc, os_, xb.size, GROUP, act_bits[0])
    oracle.grad_quant(gh[:n16], GROUP)
    oracle.grad_reduce_requant(ch16, sh16, n16, GROUP)
    secs1 = time.perf_counter() - t
    nbytes1 = 2 * algo_bytes_act(xb.size, act_bits[0]) + algo_bytes_grad_quant(n16) + \
        algo_bytes_reduce(n16, K_CHUNKS)
    oracle.set_threads(threads)
    return {
        "value": round(nbytes / secs / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
        "one_thread_GB/s": round(nbytes1 / secs1 / 1e9, 3),
        "sample": "one whole step (5 activations quant+dequant, gradient store, 8-chunk reduce): "
                  "%.0f MB algorithmic in %.2f s wall on %d threads (median of 3 passes)"
                  % (nbytes / 1e6, secs, threads),
        "gpu_matches_oracle_on_sample": bool(ok),
    }


if __name__ == "__main__":
    sys.exit(main())
