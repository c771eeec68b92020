"""Per-kernel throughput on all five benchmark configurations (one GPU).

    python -m paper_2605_00539_amd.sweep [--launches 200] [--reps 5]

Protocol: for every (kernel, tensor shape, bits, group) case, `launches` back-to-back
launches between two events on one stream, cycling through enough distinct input AND
output buffers that the cycle's footprint on each side exceeds 1 GiB (the chip has a
256 MB last-level cache in front of HBM; without rotation it absorbs re-reads and
overwrites); median of `reps` such runs.  Reported: microseconds per launch, effective
GB/s = algorithmic bytes / time, and the fraction of the 8 TB/s HBM peak.
"""
import argparse
import json
import sys

import torch

from . import binding as agoq

PEAK = 8000.0
GiB = 1 << 30


def algo_act(n, bits, group):
    return n * 2 + n * bits // 8 + 4 * (n // group)


def algo_gq(n, group):
    return 5 * n + 4 * (n // group)


def algo_red(n, K, group):
    return (K + 1) * (n + 4 * (n // group))


def timed(fn, launches, reps):
    for i in range(min(10, launches)):
        fn(i)
    torch.cuda.synchronize()
    out = []
    for _ in range(reps):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(launches):
            fn(i)
        e1.record()
        e1.synchronize()
        out.append(e0.elapsed_time(e1) * 1e3 / launches)
    out.sort()
    return out[len(out) // 2]


def timed_wall(fn, launches, reps):
    """Host-clock variant for launches that go to more than one stream (events on one stream
    would not see the others): device-wide synchronization on both sides of the loop."""
    import time
    for i in range(min(10, launches)):
        fn(i)
    torch.cuda.synchronize()
    out = []
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(launches):
            fn(i)
        torch.cuda.synchronize()
        out.append((time.perf_counter() - t0) * 1e6 / launches)
    out.sort()
    return out[len(out) // 2]


def slots_for(bytes_each, floor=2, cap=128):
    """Buffers needed for a 1.5 GiB rotation, at most `cap` (tiny tensors stay cache-resident
    whatever the rotation; they measure launch latency, not bandwidth)."""
    return min(cap, max(floor, -(-(GiB + GiB // 2) // bytes_each)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--launches", type=int, default=200)
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--configs", default="1,2,3,4,5",
                    help="comma-separated configuration numbers to run (default: all five)")
    ap.add_argument("--messages", action="store_true",
                    help="also time the per-GPU quantize/reduce/dequantize work of one 8-bit "
                         "All-Reduce at message sizes 2^15 .. 2^30 elements")
    args = ap.parse_args()
    wanted = {int(c) for c in args.configs.split(",") if c}
    import workloads as wl

    import ctypes
    L = agoq.load_library()
    P = ctypes.c_void_p
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    st = P(torch.cuda.current_stream().cuda_stream)
    rows = []
    # the two side streams of the "(2 streams)" rows, made once and used first thing, so that
    # every case sees the same pair of hardware queues
    two = [torch.cuda.Stream(), torch.cuda.Stream()]
    sp = [P(t.cuda_stream) for t in two]
    for t in two:
        with torch.cuda.stream(t):
            torch.zeros(1, device=dev)
    torch.cuda.synchronize()

    def report(config, kernel, case, us, nbytes):
        gbps = nbytes / us / 1e3
        rows.append(dict(config=config, kernel=kernel, case=case, us=round(us, 2),
                         algo_MB=round(nbytes / 1e6, 2), GBps=round(gbps, 1),
                         frac=round(gbps / PEAK, 4)))
        print("%-14s %-22s %-34s %10.2f us %10.1f MB %9.1f GB/s %6.1f%%" %
              (config, kernel, case, us, nbytes / 1e6, gbps, 100 * gbps / PEAK), flush=True)

    def act_case(config, label, rows_, cols, dist, frac, scale, seed, group_list, bits_list, fused=False, fp=False):
        n = rows_ * cols
        nx = slots_for(2 * n)
        base = wl.act_device(rows_, cols, seed, dist, wl.n_outlier_channels(cols, frac), scale).reshape(-1)
        xs = [base] + [base.roll(7919 * (i + 1)) for i in range(nx - 1)]
        ys = [torch.empty(n, dtype=torch.bfloat16, device=dev) for _ in range(nx)]
        for group in group_list:
            for bits in bits_list:
                nc = slots_for(n * bits // 8)
                cs = [torch.empty(n * bits // 8, dtype=torch.uint8, device=dev) for _ in range(nc)]
                ss = [torch.empty(n // group, dtype=torch.float32, device=dev) for _ in range(nc)]
                for i in range(nc):
                    agoq.act_quant(xs[i % nx], group, bits, codes=cs[i], scales=ss[i])
                torch.cuda.synchronize()
                nb = algo_act(n, bits, group)
                case = "%s [%d,%d] b%d g%d" % (label, rows_, cols, bits, group)
                # argument tuples are marshalled once, so that the loop issues launches as
                # fast as the host can (small tensors finish in under 10 us)
                m = max(nx, nc)
                qa = [(P(xs[i % nx].data_ptr()), n, group, bits, P(cs[i % nc].data_ptr()),
                       P(ss[i % nc].data_ptr()), st) for i in range(m)]
                da = [(P(cs[i % nc].data_ptr()), P(ss[i % nc].data_ptr()), n, group, bits,
                       P(ys[i % nx].data_ptr()), st) for i in range(m)]
                us = timed(lambda i: L.agoq_act_quant(*qa[i % len(qa)]), args.launches, args.reps)
                report(config, "act_quant", case, us, nb)
                us = timed(lambda i: L.agoq_act_dequant(*da[i % len(da)]), args.launches, args.reps)
                report(config, "act_dequant", case, us, nb)
                if 2 * n <= (64 << 20):
                    # small tensors: each launch lasts under 13 us, about 3 of which are the dispatch
                    # gap between dependent launches of one stream.  Alternating two streams lets
                    # one kernel's ramp overlap the other's drain and shows the kernel's own rate.
                    for t in two:
                        t.wait_stream(torch.cuda.current_stream())
                    us = timed_wall(lambda i: L.agoq_act_quant(*qa[i % len(qa)][:6], sp[i & 1]), 2 * args.launches, args.reps)
                    report(config, "act_quant (2 streams)", case, us, nb)
                    us = timed_wall(lambda i: L.agoq_act_dequant(*da[i % len(da)][:6], sp[i & 1]), 2 * args.launches, args.reps)
                    report(config, "act_dequant (2 streams)", case, us, nb)
                    torch.cuda.synchronize()
                if fp and bits == 4:
                    us = timed(lambda i: L.agoq_fp4_act_quant(qa[i % len(qa)][0], n, group, qa[i % len(qa)][4],
                                                              qa[i % len(qa)][5], st), args.launches, args.reps)
                    report(config, "fp4_act_quant", case.replace(" b4 ", " e2m1 "), us, nb)
                    us = timed(lambda i: L.agoq_fp4_act_dequant(da[i % len(da)][0], da[i % len(da)][1], n, group,
                                                                da[i % len(da)][5], st), args.launches, args.reps)
                    report(config, "fp4_act_dequant", case.replace(" b4 ", " e2m1 "), us, nb)
                    # leave int4 codes behind for the cases that follow
                    for i in range(nc):
                        agoq.act_quant(xs[i % nx], group, bits, codes=cs[i], scales=ss[i])
                    torch.cuda.synchronize()
                if fused and cols <= 16384:
                    # dequantize fused with the RMSNorm recompute (same bytes as a plain dequantize)
                    gamma = torch.ones(cols, dtype=torch.float32, device=dev)
                    rs = [torch.empty(rows_, dtype=torch.float32, device=dev) for _ in range(4)]
                    na = [(P(cs[i % nc].data_ptr()), P(ss[i % nc].data_ptr()), rows_, cols, group, bits,
                           P(gamma.data_ptr()), ctypes.c_float(1e-5), P(ys[i % nx].data_ptr()),
                           P(rs[i % 4].data_ptr()), st) for i in range(m)]
                    us = timed(lambda i: L.agoq_act_dequant_rmsnorm(*na[i % len(na)]), args.launches, args.reps)
                    report(config, "act_dequant_rmsnorm", case, us, nb + 4 * rows_)
                    # forward side: the layer plus the quantization of its input in one pass
                    fa = [(P(xs[i % nx].data_ptr()), rows_, cols, P(gamma.data_ptr()), ctypes.c_float(1e-5), group,
                           bits, P(ys[i % nx].data_ptr()), P(rs[i % 4].data_ptr()), P(cs[i % nc].data_ptr()),
                           P(ss[i % nc].data_ptr()), st) for i in range(m)]
                    us = timed(lambda i: L.agoq_rmsnorm_fwd_quant(*fa[i % len(fa)]), args.launches, args.reps)
                    report(config, "rmsnorm_fwd_quant", case, us, nb + 2 * n + 4 * rows_)
                    ga = [(P(xs[i % nx].data_ptr()), P(xs[(i + 1) % nx].data_ptr()), n, group, bits, bits,
                           P(ys[i % nx].data_ptr()), P(cs[i % nc].data_ptr()), P(ss[i % nc].data_ptr()),
                           P(cs[(i + 1) % nc].data_ptr()), P(ss[(i + 1) % nc].data_ptr()), st) for i in range(m)]
                    us = timed(lambda i: L.agoq_silu_mul_fwd_quant(*ga[i % len(ga)]), args.launches, args.reps)
                    report(config, "silu_mul_fwd_quant", case, us, 2 * nb + 2 * n)
                    # SiLU & Multiply recompute from two stored tensors of this shape and width
                    sa = [(P(cs[i % nc].data_ptr()), P(ss[i % nc].data_ptr()), bits,
                           P(cs[(i + 1) % nc].data_ptr()), P(ss[(i + 1) % nc].data_ptr()), bits, n, group,
                           P(ys[i % nx].data_ptr()), st) for i in range(m)]
                    us = timed(lambda i: L.agoq_act_dequant_silu_mul(*sa[i % len(sa)]), args.launches, args.reps)
                    report(config, "act_dequant_silu_mul", case, us, 2 * (n * bits // 8 + 4 * (n // group)) + 2 * n)
                del cs, ss
        del xs, ys, base

    def layer_case(config, label, rows_, hidden, ffn, dist, frac, scale, seed, group, bitmap):
        """The five stored tensors of one layer in ONE launch (agoq_act_quant_layer /
        agoq_act_dequant_layer); whole layers rotate so that each side's cycle exceeds 1 GiB."""
        cols = [hidden, hidden, hidden, ffn, ffn]
        layer_bytes = 2 * rows_ * sum(cols)
        nl = min(8, max(2, -(-(GiB + GiB // 2) // layer_bytes)))
        base = [wl.act_device(rows_, c, seed + i, dist, wl.n_outlier_channels(c, frac), scale).reshape(-1)
                for i, c in enumerate(cols)]
        xs = [base] + [[b.roll(7919 * (l + 1)) for b in base] for l in range(nl - 1)]
        ys = [[torch.empty_like(b) for b in base] for _ in range(nl)]
        code_bytes = sum(b.numel() * w // 8 for b, w in zip(base, bitmap))
        nc = min(16, max(2, -(-(GiB + GiB // 2) // code_bytes)))
        cs = [[torch.empty(b.numel() * w // 8, dtype=torch.uint8, device=dev) for b, w in zip(base, bitmap)]
              for _ in range(nc)]
        ss = [[torch.empty(b.numel() // group, dtype=torch.float32, device=dev) for b in base] for _ in range(nc)]
        m = max(nl, nc)
        qs = [agoq.layer_slots(xs[i % nl], bitmap, cs[i % nc], ss[i % nc]) for i in range(m)]
        ds = [agoq.layer_slots(ys[i % nl], bitmap, cs[i % nc], ss[i % nc]) for i in range(m)]
        for i in range(nc):
            L.agoq_act_quant_layer(qs[i % m][0], 5, group, st)
        torch.cuda.synchronize()
        nb = sum(algo_act(b.numel(), w, group) for b, w in zip(base, bitmap))
        case = "%s rows %d map %s g%d" % (label, rows_, bitmap, group)
        us = timed(lambda i: L.agoq_act_quant_layer(qs[i % m][0], 5, group, st), args.launches, args.reps)
        report(config, "act_quant_layer (1 launch)", case, us, nb)
        us = timed(lambda i: L.agoq_act_dequant_layer(ds[i % m][0], 5, group, st), args.launches, args.reps)
        report(config, "act_dequant_layer (1 launch)", case, us, nb)
        del xs, ys, cs, ss, base, qs, ds
        torch.cuda.empty_cache()

    def grad_case(config, n, sigma, spike_frac, spike_scale, seed, K, group, share=True, fp8=False, kscan=False):
        g = [wl.grad_device(n, seed + i, sigma, spike_frac, spike_scale) for i in range(2 if n > (1 << 26) else 8)]
        nout = slots_for(n, floor=3)
        ocs = [torch.empty(n, dtype=torch.int8, device=dev) for _ in range(nout)]
        oss = [torch.empty(n // group, dtype=torch.float32, device=dev) for _ in range(nout)]
        launches = max(20, min(args.launches, int(2e9 / n)))
        us = timed(lambda i: agoq.grad_quant(g[i % len(g)], group, codes=ocs[i % nout],
                                             scales=oss[i % nout]), launches, args.reps)
        report(config, "grad_quant", "n=%d g%d" % (n, group), us, algo_gq(n, group))
        if n > (1 << 26):
            # local accumulation (stored int8 gradient + new micro-batch gradient -> int8) and
            # int8 -> fp32 dequantize, on the same tensor size
            mcs = [torch.empty(n, dtype=torch.int8, device=dev) for _ in range(nout)]
            mss = [torch.empty(n // group, dtype=torch.float32, device=dev) for _ in range(nout)]
            for i in range(nout):
                agoq.grad_quant(g[i % len(g)], group, codes=mcs[i], scales=mss[i])
            torch.cuda.synchronize()
            us = timed(lambda i: agoq.grad_accumulate(mcs[i % nout], mss[i % nout], g[i % len(g)], group,
                                                      out_codes=ocs[i % nout], out_scales=oss[i % nout]),
                       launches, args.reps)
            report(config, "grad_accumulate", "fp32 addend n=%d g%d" % (n, group), us,
                   n * 6 + 8 * (n // group))
            gb = [x.to(torch.bfloat16) for x in g]
            us = timed(lambda i: agoq.grad_accumulate(mcs[i % nout], mss[i % nout], gb[i % len(gb)], group,
                                                      out_codes=ocs[i % nout], out_scales=oss[i % nout]),
                       launches, args.reps)
            report(config, "grad_accumulate", "bf16 addend n=%d g%d" % (n, group), us,
                   n * 4 + 8 * (n // group))
            del gb
            fo = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(2)]
            us = timed(lambda i: agoq.grad_dequant(mcs[i % nout], mss[i % nout], group, out=fo[i % 2]),
                       launches, args.reps)
            report(config, "grad_dequant", "n=%d g%d" % (n, group), us, n * 5 + 4 * (n // group))
            del mcs, mss, fo
        if fp8:
            ucs = [t.view(torch.uint8) for t in ocs]
            us = timed(lambda i: agoq.fp8_grad_quant(g[i % len(g)], group, codes=ucs[i % nout],
                                                     scales=oss[i % nout]), launches, args.reps)
            report(config, "fp8_grad_quant", "n=%d g%d" % (n, group), us, algo_gq(n, group))
            fcodes = torch.empty((K, n), dtype=torch.uint8, device=dev)
            fscales = torch.empty((K, n // group), dtype=torch.float32, device=dev)
            for k in range(K):
                gk = wl.grad_device(n, seed + 300 + k, sigma, spike_frac, spike_scale)
                agoq.fp8_grad_quant(gk, group, codes=fcodes[k], scales=fscales[k])
                torch.cuda.synchronize()
                del gk
            us = timed(lambda i: agoq.fp8_grad_reduce_requant(fcodes, fscales, n, group, out_codes=ucs[i % nout],
                                                              out_scales=oss[i % nout]), launches, args.reps)
            report(config, "fp8_grad_reduce_requant", "K=%d n=%d g%d" % (K, n, group), us, algo_red(n, K, group))
            fo = torch.empty(n, dtype=torch.float32, device=dev)
            us = timed(lambda i: agoq.fp8_grad_dequant(fcodes[i % K], fscales[i % K], group, out=fo), launches, args.reps)
            report(config, "fp8_grad_dequant", "n=%d g%d" % (n, group), us, algo_gq(n, group))
            del fcodes, fscales, fo
        nin = 1 if K * n > GiB else -(-GiB // (K * n)) + 1
        ins = []
        for s in range(nin):
            codes = torch.empty((K, n), dtype=torch.int8, device=dev)
            scales = torch.empty((K, n // group), dtype=torch.float32, device=dev)
            for k in range(K):
                gk = wl.grad_device(n, seed + 100 + 17 * s + k, sigma, spike_frac, spike_scale)
                agoq.grad_quant(gk, group, codes=codes[k], scales=scales[k])
                torch.cuda.synchronize()
                del gk
            ins.append((codes, scales))
        us = timed(lambda i: agoq.grad_reduce_requant(ins[i % nin][0], ins[i % nin][1], n, group,
                                                      out_codes=ocs[i % nout], out_scales=oss[i % nout]),
                   launches, args.reps)
        report(config, "grad_reduce_requant", "K=%d n=%d g%d" % (K, n, group), us, algo_red(n, K, group))
        if share:
            ns = n // K
            codes, scales = ins[0]

            # a shard is a strided window of the receive buffer: pass pointers and strides
            # to the C ABI directly

            def shard_raw(i):
                k = i % K
                off = k * ns
                o = ocs[(i // K) % nout]
                osc = oss[(i // K) % nout]
                rc = L.agoq_grad_reduce_requant(P(codes.data_ptr() + off), n,
                                                P(scales.data_ptr() + 4 * (off // group)), n // group,
                                                K, ns, group, P(o.data_ptr() + off),
                                                P(osc.data_ptr() + 4 * (off // group)), st)
                assert rc == 0
            us = timed(shard_raw, args.launches, args.reps)
            report(config, "grad_reduce_requant", "K=%d share n=%d g%d" % (K, ns, group), us,
                   algo_red(ns, K, group))
        if kscan:
            # other chunk counts on the shard size (random codes and scales: timing only)
            ns = n // 8
            for Kx in (1, 2, 3, 5, 12, 32, 64):
                nsl = max(1, -(-(GiB + GiB // 2) // (Kx * ns)))
                bufs = [(torch.randint(-127, 128, (Kx, ns), device=dev, dtype=torch.int8),
                         torch.rand((Kx, ns // group), device=dev, dtype=torch.float32) * 1e-5 + 1e-8)
                        for _ in range(min(nsl, 8))]
                us = timed(lambda i: agoq.grad_reduce_requant(bufs[i % len(bufs)][0], bufs[i % len(bufs)][1], ns, group,
                                                              out_codes=ocs[i % nout][:ns], out_scales=oss[i % nout][:ns // group]),
                           args.launches, args.reps)
                report(config, "grad_reduce_requant", "K=%d n=%d g%d" % (Kx, ns, group), us, algo_red(ns, Kx, group))
                del bufs
        del ins, g, ocs, oss

    C = wl.CONFIGS
    # config 1: tiny (launch-latency bound; parity case, reported for completeness)
    if 1 in wanted:
        c = C["tiny"]
        act_case("1-tiny", "act", c["act"]["rows"], c["act"]["cols"], "normal",
                 c["act"]["outlier_channels"] / c["act"]["cols"], c["act"]["outlier_scale"], c["seed"],
                 [c["group"]], [c["bits"]])
        grad_case("1-tiny", c["grad"]["n"], c["grad"]["sigma"], 0.0, 1.0, 1, c["K"], c["group"], share=False)
    # config 2: LLaMA-8B-shaped activations
    if 2 in wanted:
        c = C["llama8b_act"]
        for name, sh in c["acts"].items():
            act_case("2-8B-act", name, sh["rows"], sh["cols"], c["dist"], c["outlier_frac"],
                     c["outlier_scale"], c["seed"], [c["group"]], [4, 8], fp=True)
        a = c["acts"]
        layer_case("2-8B-act", "layer", a["A"]["rows"], a["A"]["cols"], a["F"]["cols"], c["dist"],
                   c["outlier_frac"], c["outlier_scale"], c["seed"], c["group"], agoq.layer_bitmap(5))
    # config 3: LLaMA-8B-shaped gradients, K = 8
    if 3 in wanted:
        c = C["llama8b_grad"]
        grad_case("3-8B-grad", c["n"], c["sigma"], c["spike_frac"], c["spike_scale"], c["seed"], c["K"],
                  c["group"], fp8=True, kscan=True)
    # config 4: 32B-shaped activations, both group sizes
    if 4 in wanted:
        c = C["llama32b_act"]
        for name, sh in c["acts"].items():
            act_case("4-32B-act", name, sh["rows"], sh["cols"], c["dist"], c["outlier_frac"],
                     c["outlier_scale"], c["seed"], list(c["groups"]), [4, 8])
    # config 5: stage sweep at seq 8192, K = 16
    if 5 in wanted:
        c = C["stage_sweep"]
        per = {}
        for name, cols in (("H", c["hidden"]), ("F", c["ffn"])):
            before = len(rows)
            act_case("5-stage", name, c["rows"], cols, c["dist"], c["outlier_frac"], c["outlier_scale"],
                     c["seed"], [c["group"]], [4, 5, 6, 8], fused=True)
            for r in rows[before:]:
                if r["kernel"] in ("act_quant", "act_dequant"):
                    per[(name, r["kernel"], int(r["case"].split(" b")[1].split()[0]))] = r
        gcfg = c["grad"]
        grad_case("5-stage", gcfg["n"], gcfg["sigma"], gcfg["spike_frac"], gcfg["spike_scale"], c["seed"],
                  c["K"], c["group"])
        # whole-layer figures per stage bit map (sum of the five tensors' launches)
        bf16_bytes = c["rows"] * (3 * c["hidden"] + 2 * c["ffn"]) * 2
        for stage in (1, 2, 3, 4):
            b = agoq.dbca_bits(4, stage)
            for native in (True, False):
                bitmap = agoq.layer_bitmap(b, native=native)
                if not native and bitmap == agoq.layer_bitmap(b, native=True):
                    continue
                stored = agoq.layer_stored_bytes(c["rows"], c["hidden"], c["ffn"], c["group"], bitmap, True)
                for kernel in ("act_quant", "act_dequant"):
                    us = nb = 0.0
                    for slot, bits in enumerate(bitmap):
                        r = per[("F" if slot >= 3 else "H", kernel, bits)]
                        us += r["us"]
                        nb += r["algo_MB"] * 1e6
                    report("5-stage", kernel + "_layer",
                           "stage %d (B=%d) map %s stored %d B (%.1f%% saved vs bf16)" %
                           (stage, b, bitmap, stored, 100.0 * (1 - stored / bf16_bytes)), us, nb)
        seen = []
        for stage in (1, 2, 3, 4):
            b = agoq.dbca_bits(4, stage)
            for native in (True, False):
                bitmap = agoq.layer_bitmap(b, native=native)
                if bitmap in seen:
                    continue
                seen.append(bitmap)
                layer_case("5-stage", "stage %d (B=%d)" % (stage, b), c["rows"], c["hidden"], c["ffn"],
                           c["dist"], c["outlier_frac"], c["outlier_scale"], c["seed"], c["group"], bitmap)
    # message-size sweep: the quantize / reduce / dequantize work one GPU does for one
    # decomposed 8-bit All-Reduce over P = 8 peers on a gradient bucket of n elements
    # (store n as int8; reduce the 8 received chunks of its n/8 shard; dequantize the n
    # gathered elements) -- the work the paper's communication breakdown (Table
    # comm_savings, column "Quant/Dequant") times at message sizes 2^15 .. 2^30
    if args.messages:
        group, K = 128, 8
        for log2n in (15, 20, 25, 28, 30):
            n = 1 << log2n
            ns = n // K
            nrot = max(2, min(16, -(-(GiB + GiB // 2) // (4 * n))))
            g = [wl.grad_device(n, 700 + i, 1e-4, 0.001, 100.0) for i in range(nrot)]
            codes = [torch.empty(n, dtype=torch.int8, device=dev) for _ in range(nrot)]
            scales = [torch.empty(n // group, dtype=torch.float32, device=dev) for _ in range(nrot)]
            out = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(2)]
            rc = torch.randint(-127, 128, (K, ns), device=dev, dtype=torch.int8)
            rs = torch.rand((K, ns // group), device=dev, dtype=torch.float32) * 1e-5 + 1e-8
            oc = torch.empty(ns, dtype=torch.int8, device=dev)
            osc = torch.empty(ns // group, dtype=torch.float32, device=dev)

            # pointers marshalled once: at the small sizes the binding's per-call checks
            # would otherwise be most of the time
            pg = [P(t.data_ptr()) for t in g]
            pc = [P(t.data_ptr()) for t in codes]
            ps = [P(t.data_ptr()) for t in scales]
            po = [P(t.data_ptr()) for t in out]
            prc, prs, poc, pos = P(rc.data_ptr()), P(rs.data_ptr()), P(oc.data_ptr()), P(osc.data_ptr())

            def message(i):
                r = i % nrot
                bad = L.agoq_grad_quant(pg[r], n, group, pc[r], ps[r], st)
                bad |= L.agoq_grad_reduce_requant(prc, ns, prs, ns // group, K, ns, group, poc, pos, st)
                bad |= L.agoq_grad_dequant(pc[r], ps[r], n, group, po[i % 2], st)
                assert bad == 0
            launches = max(5, min(args.launches, int(4e9 / n)))
            us = timed(message, launches, args.reps)
            report("messages", "quant+reduce+dequant", "n=2^%d elements (fp32 %d MiB), K=8" % (log2n, 4 * n >> 20),
                   us, 2 * algo_gq(n, group) + algo_red(ns, K, group))
            del g, codes, scales, out, rc, rs, oc, osc
            torch.cuda.empty_cache()
    print(json.dumps(rows))
    return 0


if __name__ == "__main__":
    sys.exit(main())
