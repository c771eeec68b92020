#!/usr/bin/env python3
"""Benchmark of the AGoQ quantization hot path on one MI355X.

One "step" (the headline `value`) is one pass of the whole path over the LLaMA-8B-shaped
workload:
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

Beside the step, `kernels` carries one row per kernel and tensor of the other benchmark
configurations (sections c2..c5 below), each timed as `--launches` back-to-back launches
over a rotation of inputs AND outputs whose footprint exceeds 1 GiB on each side (the chip
has a 256 MB last-level cache in front of HBM), median of `--reps` runs, and each checked
once, on full tensors, bit for bit against the CPU oracle (`gpu_matches_oracle`).

The figure of merit is effective HBM bandwidth: algorithmic bytes (read the tensor once,
write codes + scales once, or the reverse) divided by time.  Prints ONE JSON line on
stdout; a readable table of the rows goes to stderr as they are measured.

Sections (`--sections`, comma separated; default: all of them, about 80 s):
  step      the headline step, its four kernels, the oracle timed on the host cores
  c2        8B-shaped activations, single-tensor calls
  c3        8B-shaped gradient: the 8-chunk reduce on this GPU's 1/8 shard
  c4        32B-shaped activations (hidden 5120, FFN 27648), groups 64 and 128, single-tensor
            calls and the layer in one launch
  c5        pipeline-stage sweep at seq 8192: the layer under each stage's bit map (4/8-bit
            mixes and native 5/6-bit codes), gradient store, 16-chunk reduce (n = N, N/16)
  fused     dequantize fused with the RMSNorm / SiLU & Multiply recompute and the forward
            forms, 4/5/6/8-bit, on the seq-8192 tensors (outputs checked to the stated bar)
  gradx     local accumulation, int8 -> fp32 dequantize, E4M3 forms
  kscan     the reduce for K = 1..16, 32, 64 on the 27M-element shard
  messages  quantize + 8-chunk reduce + dequantize of one 8-bit All-Reduce at 2^15..2^30 elements
  floor     streaming kernels without arithmetic on the small tensors' footprints, and the
            same calls alternating two streams
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0
GiB = 1 << 30
# HBM bytes per launch of the K=8 reduce kernel on the step's workload, from hardware counters
# (two rocprofv3 --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size)
TRAFFIC_REDUCE_K8_BYTES = 2024896318
TRAFFIC_SOURCE = ("stored figure: rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE of this command, "
                  "profiles/bench_llama8b_step_hbm_traffic.txt")
GROUP = 128
K_CHUNKS = 8
MARK_MAX = 1024          # --mark-rows: most timed runs of one command (every real launch has more workgroups)
SLOT_NAMES = ("norm1_in", "oproj_in", "norm2_in", "gate", "up")
P = ctypes.c_void_p
ALL_SECTIONS = ("step", "c2", "c3", "c4", "c5", "fused", "gradx", "sr", "kscan", "messages", "floor")
DEFAULT_SECTIONS = ",".join(ALL_SECTIONS)


def algo_bytes_act(numel, bits, group=GROUP):
    return numel * 2 + numel * bits // 8 + 4 * (numel // group)


def algo_bytes_grad_quant(numel, group=GROUP):
    return numel * 4 + numel + 4 * (numel // group)


def algo_bytes_reduce(numel, K, group=GROUP):
    return (K + 1) * (numel + 4 * (numel // group))


def rotation(bytes_each, floor=2, cap=128):
    """Buffers needed for a 1.5 GiB rotation."""
    return min(cap, max(floor, -(-(GiB + GiB // 2) // bytes_each)))


class Rows:
    """Per-kernel rows: timing protocol, table on stderr, dict for the JSON line."""

    def __init__(self, torch, launches, reps, mark=None):
        self.torch = torch
        self.launches = launches
        self.reps = reps
        self.rows = {}
        self.mark = mark            # callable(ordinal) or None: see --mark-rows
        self.marks = 0
        self.fresh_mark = False     # a timed run has started since the last row was added

    def _mark(self):
        """With --mark-rows, every timed run starts with one launch of the library's plain copy
        kernel over `ordinal` workgroups: a kernel trace or counter file of the command can
        then be cut into rows by that kernel's grid size, and a row names its ordinal."""
        self.marks += 1
        self.fresh_mark = True
        if self.mark is not None:
            self.mark(self.marks)

    def timed(self, fn, launches=None):
        """Median microseconds per launch over `reps` runs of back-to-back launches, events on
        the current stream (the stream every call here is launched on)."""
        torch = self.torch
        launches = launches or self.launches
        self._mark()
        for i in range(min(10, launches)):
            fn(i)
        torch.cuda.synchronize()
        out = []
        for _ in range(self.reps):
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

    def timed_wall(self, fn, launches=None):
        """Host-clock variant for launches that go to more than one stream."""
        torch = self.torch
        launches = launches or self.launches
        self._mark()
        for i in range(min(10, launches)):
            fn(i)
        torch.cuda.synchronize()
        out = []
        for _ in range(self.reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(launches):
                fn(i)
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t0) * 1e6 / launches)
        out.sort()
        return out[len(out) // 2]

    def add(self, section, kernel, case, us, nbytes, ok=None, **extra):
        gbps = nbytes / us / 1e3
        row = {"us": round(us, 2), "GB/s": round(gbps, 1), "frac_of_peak": round(gbps / PEAK_HBM_GBPS, 4),
               "algo_MB": round(nbytes / 1e6, 1)}
        if ok is not None:
            row["gpu_matches_oracle"] = bool(ok)
        if self.mark is not None and self.fresh_mark:
            row["mark"] = self.marks
        self.fresh_mark = False
        row.update(extra)
        self.rows["%s/%s/%s" % (section, kernel, case)] = row
        print("%-9s %-28s %-46s %9.2f us %9.1f MB %8.1f GB/s %5.1f%%  %s" %
              (section, kernel, case, us, nbytes / 1e6, gbps, 100 * gbps / PEAK_HBM_GBPS,
               "" if ok is None else ("oracle: equal" if ok else "oracle: MISMATCH")),
              file=sys.stderr, flush=True)


def bits_of(torch, t):
    """bf16 device tensor -> uint16 numpy array of its bit patterns."""
    import numpy as np
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def same_u32(torch, dev_f32, host_f32):
    import numpy as np
    return np.array_equal(dev_f32.cpu().numpy().view(np.uint32), host_f32.view(np.uint32))


class Env:
    """What every section needs: torch, the binding, the raw library, the stream, the oracle."""

    def __init__(self, args):
        import torch
        import workloads as wl
        import paper_2605_00539_amd as agoq
        self.torch, self.wl, self.agoq = torch, wl, agoq
        self.L = agoq.load_library()
        self.dev = torch.device("cuda:0")
        torch.cuda.set_device(self.dev)
        self.stream = torch.cuda.current_stream()
        self.st = P(self.stream.cuda_stream)
        self.check = not args.no_check
        self.oracle = None
        if self.check or not args.no_cpu_baseline:
            import oracle
            self.oracle = oracle
        mark = None
        if args.mark_rows:
            # 512 sixteen-byte items per workgroup of the copy kernel: ordinal workgroups
            self._mark_buf = torch.zeros(2 * MARK_MAX * 512 * 16, dtype=torch.uint8, device=self.dev)
            src, dst = P(self._mark_buf.data_ptr()), P(self._mark_buf.data_ptr() + MARK_MAX * 512 * 16)

            def mark(ordinal):
                if ordinal > MARK_MAX:
                    raise RuntimeError("--mark-rows: more than %d timed runs" % MARK_MAX)
                assert self.L.agoq_probe_stream(src, 16, dst, 16, 512 * ordinal, self.st) == 0
        self.rows = Rows(torch, args.launches, args.reps, mark)

    def empty(self, n, dtype):
        return self.torch.empty(n, dtype=dtype, device=self.dev)


# ---------------------------------------------------------------------------------------------
# activations: single-tensor calls and layer launches
# ---------------------------------------------------------------------------------------------

class ActTensor:
    """One synthetic stored tensor: its bf16 data on the device (with rolled copies for the
    rotation) and, on demand, the oracle's codes / scales / dequantized bits per (bits, group)."""

    def __init__(self, env, rows, cols, seed, dist, frac, scale):
        self.env = env
        self.rows, self.cols, self.n = rows, cols, rows * cols
        self.base = env.wl.act_device(rows, cols, seed, dist, env.wl.n_outlier_channels(cols, frac),
                                      scale).reshape(-1)
        self._host = None
        self._oracle = {}

    def copies(self, count):
        return [self.base] + [self.base.roll(7919 * (i + 1)) for i in range(count - 1)]

    def oracle(self, bits, group):
        key = (bits, group)
        if key not in self._oracle:
            env = self.env
            if self._host is None:
                self._host = bits_of(env.torch, self.base)
            oc, os_ = env.oracle.act_quant(self._host, group, bits)
            oy = env.oracle.act_dequant(oc, os_, self.n, group, bits)
            self._oracle[key] = (oc, os_, oy)
        return self._oracle[key]

    def matches(self, bits, group, codes, scales, y):
        """Full-tensor comparison of one quantize + dequantize of the base data."""
        import numpy as np
        env = self.env
        oc, os_, oy = self.oracle(bits, group)
        return (np.array_equal(codes.cpu().numpy(), oc) and same_u32(env.torch, scales, os_) and
                np.array_equal(bits_of(env.torch, y), oy))


def act_single(env, section, label, t, groups, bits_list, fp4=False, two_streams=None):
    """agoq_act_quant / agoq_act_dequant on one tensor, every (group, bits)."""
    torch, L, st, R = env.torch, env.L, env.st, env.rows
    n = t.n
    nx = rotation(2 * n)
    xs = t.copies(nx)
    ys = [env.empty(n, torch.bfloat16) for _ in range(nx)]
    for group in groups:
        for bits in bits_list:
            nc = rotation(n * bits // 8)
            cs = [env.empty(n * bits // 8, torch.uint8) for _ in range(nc)]
            ss = [env.empty(n // group, torch.float32) for _ in range(nc)]
            for i in range(nc):
                env.agoq.act_quant(xs[i % nx], group, bits, codes=cs[i], scales=ss[i])
            torch.cuda.synchronize()
            nb = algo_bytes_act(n, bits, group)
            case = "%s[%d,%d] b%d g%d" % (label, t.rows, t.cols, bits, group)
            m = max(nx, nc)
            # argument tuples are marshalled once, so that the loop issues launches as fast as
            # the host can (the small tensors finish in under 10 us)
            qa = [(P(xs[i % nx].data_ptr()), n, group, bits, P(cs[i % nc].data_ptr()),
                   P(ss[i % nc].data_ptr()), st) for i in range(m)]
            da = [(P(cs[i % nc].data_ptr()), P(ss[i % nc].data_ptr()), n, group, bits,
                   P(ys[i % nx].data_ptr()), st) for i in range(m)]
            ok = None
            if env.check:
                # slot 0 holds the base data: one quantize and one dequantize of it, compared whole
                cs[0].zero_()
                ss[0].zero_()
                ys[0].zero_()
                assert L.agoq_act_quant(*qa[0]) == 0 and L.agoq_act_dequant(*da[0]) == 0
                torch.cuda.synchronize()
                ok = t.matches(bits, group, cs[0], ss[0], ys[0])
            us = R.timed(lambda i: L.agoq_act_quant(*qa[i % m]))
            R.add(section, "act_quant", case, us, nb, ok)
            us = R.timed(lambda i: L.agoq_act_dequant(*da[i % m]))
            R.add(section, "act_dequant", case, us, nb, ok)
            if two_streams is not None and 2 * n <= (64 << 20):
                # each launch of a small tensor pays ~3 us of ramp and drain; alternating two
                # streams lets one launch's ramp overlap the other's drain
                sp = two_streams
                for s_ in sp:
                    s_.wait_stream(env.stream)
                ps = [P(s_.cuda_stream) for s_ in sp]
                us = R.timed_wall(lambda i: L.agoq_act_quant(*qa[i % m][:6], ps[i & 1]), 2 * R.launches)
                R.add(section, "act_quant (2 streams)", case, us, nb)
                us = R.timed_wall(lambda i: L.agoq_act_dequant(*da[i % m][:6], ps[i & 1]), 2 * R.launches)
                R.add(section, "act_dequant (2 streams)", case, us, nb)
                torch.cuda.synchronize()
            if fp4 and bits == 4:
                ok4 = None
                if env.check:
                    import numpy as np
                    assert L.agoq_fp4_act_quant(qa[0][0], n, group, qa[0][4], qa[0][5], st) == 0
                    assert L.agoq_fp4_act_dequant(da[0][0], da[0][1], n, group, da[0][5], st) == 0
                    torch.cuda.synchronize()
                    host = bits_of(torch, t.base)
                    oc, os_ = env.oracle.fp4_act_quant(host, group)
                    oy = env.oracle.fp4_act_dequant(oc, os_, n, group)
                    ok4 = (np.array_equal(cs[0].cpu().numpy(), oc) and same_u32(torch, ss[0], os_) and
                           np.array_equal(bits_of(torch, ys[0]), oy))
                us = R.timed(lambda i: L.agoq_fp4_act_quant(qa[i % m][0], n, group, qa[i % m][4], qa[i % m][5], st))
                R.add(section, "fp4_act_quant", case.replace(" b4 ", " e2m1 "), us, nb, ok4)
                for i in range(nc):
                    L.agoq_fp4_act_quant(qa[i % m][0], n, group, P(cs[i].data_ptr()), P(ss[i].data_ptr()), st)
                us = R.timed(lambda i: L.agoq_fp4_act_dequant(da[i % m][0], da[i % m][1], n, group, da[i % m][5], st))
                R.add(section, "fp4_act_dequant", case.replace(" b4 ", " e2m1 "), us, nb, ok4)
            del cs, ss
    del xs, ys


def act_layer(env, section, label, tensors, group, bitmap):
    """The five stored tensors of one layer in ONE launch (agoq_act_quant_layer /
    agoq_act_dequant_layer); whole layers rotate so that each side's cycle exceeds 1 GiB."""
    torch, L, st, R, agoq = env.torch, env.L, env.st, env.rows, env.agoq
    layer_bytes = 2 * sum(t.n for t in tensors)
    nl = min(8, max(2, -(-(GiB + GiB // 2) // layer_bytes)))
    per = [t.copies(nl) for t in tensors]
    xs = [[per[j][l] for j in range(len(tensors))] for l in range(nl)]
    ys = [[env.empty(t.n, torch.bfloat16) for t in tensors] for _ in range(nl)]
    code_bytes = sum(t.n * w // 8 for t, w in zip(tensors, bitmap))
    nc = min(16, max(2, -(-(GiB + GiB // 2) // code_bytes)))
    cs = [[env.empty(t.n * w // 8, torch.uint8) for t, w in zip(tensors, bitmap)] for _ in range(nc)]
    ss = [[env.empty(t.n // group, torch.float32) for t in tensors] for _ in range(nc)]
    m = max(nl, nc)
    qs = [agoq.layer_slots(xs[i % nl], bitmap, cs[i % nc], ss[i % nc], group) for i in range(m)]
    ds = [agoq.layer_slots(ys[i % nl], bitmap, cs[i % nc], ss[i % nc], group) for i in range(m)]
    count = len(tensors)
    for i in range(nc):
        assert L.agoq_act_quant_layer(qs[i % m].array, count, group, st) == 0
    torch.cuda.synchronize()
    ok = None
    if env.check:
        for c, s, y in zip(cs[0], ss[0], ys[0]):
            c.zero_()
            s.zero_()
            y.zero_()
        assert L.agoq_act_quant_layer(qs[0].array, count, group, st) == 0
        assert L.agoq_act_dequant_layer(ds[0].array, count, group, st) == 0
        torch.cuda.synchronize()
        ok = all(t.matches(w, group, c, s, y) for t, w, c, s, y in zip(tensors, bitmap, cs[0], ss[0], ys[0]))
    nb = sum(algo_bytes_act(t.n, w, group) for t, w in zip(tensors, bitmap))
    stored = sum(t.n * w // 8 + 4 * (t.n // group) for t, w in zip(tensors, bitmap))
    case = "%s map %s g%d" % (label, "".join(str(b) for b in bitmap), group)
    extra = {"stored_bytes": stored, "saved_vs_bf16": round(1.0 - stored / layer_bytes, 4)}
    us = R.timed(lambda i: L.agoq_act_quant_layer(qs[i % m].array, count, group, st))
    R.add(section, "act_quant_layer", case, us, nb, ok, **extra)
    us = R.timed(lambda i: L.agoq_act_dequant_layer(ds[i % m].array, count, group, st))
    R.add(section, "act_dequant_layer", case, us, nb, ok, **extra)
    del xs, ys, cs, ss, qs, ds, per
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------------------------
# gradients
# ---------------------------------------------------------------------------------------------

def quantized_chunks(env, K, n, group, seed, sigma, spike_frac, spike_scale):
    """The receive buffer of an All-to-All: K seeded gradients stored by the library (set-up)."""
    torch = env.torch
    codes = torch.empty((K, n), dtype=torch.int8, device=env.dev)
    scales = torch.empty((K, n // group), dtype=torch.float32, device=env.dev)
    for k in range(K):
        gk = env.wl.grad_device(n, seed + k, sigma, spike_frac, spike_scale)
        env.agoq.grad_quant(gk, group, codes=codes[k], scales=scales[k])
        torch.cuda.synchronize()
        del gk
    return codes, scales


def reduce_rows(env, section, codes, scales, K, n, group, share):
    """agoq_grad_reduce_requant on the whole buffer (n = N) and, with `share`, on this GPU's
    1/K shard of it (a strided window of the same buffer)."""
    import numpy as np
    torch, L, st, R = env.torch, env.L, env.st, env.rows
    nout = rotation(n, floor=3)
    ocs = [env.empty(n, torch.int8) for _ in range(nout)]
    oss = [env.empty(n // group, torch.float32) for _ in range(nout)]
    pc, ps = P(codes.data_ptr()), P(scales.data_ptr())
    ok = None
    if env.check:
        assert L.agoq_grad_reduce_requant(pc, n, ps, n // group, K, n, group, P(ocs[0].data_ptr()),
                                          P(oss[0].data_ptr()), st) == 0
        torch.cuda.synchronize()
        wc, ws = env.oracle.grad_reduce_requant(codes.cpu().numpy(), scales.cpu().numpy(), n, group)
        ok = np.array_equal(ocs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
    launches = max(20, min(R.launches, int(2e9 / n)))
    oa = [(P(ocs[i].data_ptr()), P(oss[i].data_ptr())) for i in range(nout)]
    us = R.timed(lambda i: L.agoq_grad_reduce_requant(pc, n, ps, n // group, K, n, group, oa[i % nout][0],
                                                     oa[i % nout][1], st), launches)
    R.add(section, "grad_reduce_requant", "K=%d n=%d g%d" % (K, n, group), us, algo_bytes_reduce(n, K, group), ok)
    if share:
        ns = n // K
        calls = []
        for k in range(K):
            off = k * ns
            for o in range(nout):
                calls.append((P(codes.data_ptr() + off), n, P(scales.data_ptr() + 4 * (off // group)), n // group,
                              K, ns, group, P(ocs[o].data_ptr() + off), P(oss[o].data_ptr() + 4 * (off // group)), st))
        # order: shard 0 of output set 0, shard 1 of set 0, ... so that inputs and outputs both move on
        calls = [calls[k * nout + o] for o in range(nout) for k in range(K)]
        oks = None
        if env.check:
            # every shard once into output set 0; the K shards side by side are the whole reduce
            for o in (ocs[0], oss[0]):
                o.zero_()
            for k in range(K):
                assert L.agoq_grad_reduce_requant(*calls[k]) == 0
            torch.cuda.synchronize()
            oks = np.array_equal(ocs[0][:K * ns].cpu().numpy(), wc[:K * ns]) and \
                np.array_equal(oss[0][:K * ns // group].cpu().numpy().view(np.uint32), ws[:K * ns // group].view(np.uint32))
        us = R.timed(lambda i: L.agoq_grad_reduce_requant(*calls[i % len(calls)]))
        R.add(section, "grad_reduce_requant", "K=%d share n=%d g%d" % (K, ns, group), us,
              algo_bytes_reduce(ns, K, group), oks)
    del ocs, oss


def grad_quant_row(env, section, n, group, seed, sigma, spike_frac, spike_scale):
    import numpy as np
    torch, L, st, R = env.torch, env.L, env.st, env.rows
    g = [env.wl.grad_device(n, seed + i, sigma, spike_frac, spike_scale) for i in range(2)]
    nout = rotation(n, floor=3)
    ocs = [env.empty(n, torch.int8) for _ in range(nout)]
    oss = [env.empty(n // group, torch.float32) for _ in range(nout)]
    ok = None
    if env.check:
        env.agoq.grad_quant(g[0], group, codes=ocs[0], scales=oss[0])
        torch.cuda.synchronize()
        wc, ws = env.oracle.grad_quant(g[0].cpu().numpy(), group)
        ok = np.array_equal(ocs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
    launches = max(20, min(R.launches, int(2e9 / n)))
    qa = [(P(g[i % 2].data_ptr()), n, group, P(ocs[i % nout].data_ptr()), P(oss[i % nout].data_ptr()), st)
          for i in range(2 * nout)]
    us = R.timed(lambda i: L.agoq_grad_quant(*qa[i % len(qa)]), launches)
    R.add(section, "grad_quant", "n=%d g%d" % (n, group), us, algo_bytes_grad_quant(n, group), ok)
    return g, ocs, oss


# ---------------------------------------------------------------------------------------------
# sections
# ---------------------------------------------------------------------------------------------

def section_c2(env, two_streams=None, section="c2"):
    c = env.wl.CONFIGS["llama8b_act"]
    for name, sh in c["acts"].items():
        t = ActTensor(env, sh["rows"], sh["cols"], c["seed"], c["dist"], c["outlier_frac"], c["outlier_scale"])
        act_single(env, section, name, t, [c["group"]], [4, 8], fp4=(section == "c2"), two_streams=two_streams)
        del t
        env.torch.cuda.empty_cache()


def section_c3(env):
    c = env.wl.CONFIGS["llama8b_grad"]
    codes, scales = quantized_chunks(env, c["K"], c["n"], c["group"], c["seed"] + 100, c["sigma"],
                                     c["spike_frac"], c["spike_scale"])
    # n = N is the step's own reduce (timed there); here: the per-GPU shard of the same buffer
    import numpy as np
    torch, L, st, R = env.torch, env.L, env.st, env.rows
    K, n, group = c["K"], c["n"], c["group"]
    ns = n // K
    nout = rotation(n, floor=3)
    ocs = [env.empty(n, torch.int8) for _ in range(nout)]
    oss = [env.empty(n // group, torch.float32) for _ in range(nout)]
    calls = []
    for o in range(nout):
        for k in range(K):
            off = k * ns
            calls.append((P(codes.data_ptr() + off), n, P(scales.data_ptr() + 4 * (off // group)), n // group,
                          K, ns, group, P(ocs[o].data_ptr() + off), P(oss[o].data_ptr() + 4 * (off // group)), st))
    ok = None
    if env.check:
        for k in range(K):
            assert L.agoq_grad_reduce_requant(*calls[k]) == 0
        torch.cuda.synchronize()
        wc, ws = env.oracle.grad_reduce_requant(codes.cpu().numpy(), scales.cpu().numpy(), n, group)
        ok = np.array_equal(ocs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
    us = R.timed(lambda i: L.agoq_grad_reduce_requant(*calls[i % len(calls)]))
    R.add("c3", "grad_reduce_requant", "K=%d share n=%d g%d" % (K, ns, group), us, algo_bytes_reduce(ns, K, group), ok)
    del codes, scales, ocs, oss
    torch.cuda.empty_cache()


def section_c4(env, two_streams=None, section="c4"):
    c = env.wl.CONFIGS["llama32b_act"]
    sh = c["acts"]
    for name in ("A", "F"):
        t = ActTensor(env, sh[name]["rows"], sh[name]["cols"], c["seed"], c["dist"], c["outlier_frac"],
                      c["outlier_scale"])
        act_single(env, section, name, t, list(c["groups"]), [4, 8], two_streams=two_streams)
        del t
        env.torch.cuda.empty_cache()
    if section != "c4":
        return
    # the 32B-shaped layer in one launch: three [4096,5120] and two [4096,27648] tensors
    bitmap = env.agoq.layer_bitmap(5)                 # [8, 4, 8, 4, 4]
    tensors = [ActTensor(env, sh["F" if slot >= 3 else "A"]["rows"], sh["F" if slot >= 3 else "A"]["cols"],
                         c["seed"] + slot, c["dist"], c["outlier_frac"], c["outlier_scale"])
               for slot in range(5)]
    for group in c["groups"]:
        act_layer(env, "c4", "layer rows %d" % sh["A"]["rows"], tensors, group, bitmap)
    del tensors
    env.torch.cuda.empty_cache()


def stage_maps(agoq):
    """(label, bit map) of the four stages under Eq. (dynamic), realised natively and as 4/8-bit
    mixes.  Stage 1 is the paper's first stage (most stored micro-batches, fewest bits)."""
    out, seen = [], []
    for stage in (1, 2, 3, 4):
        b = agoq.dbca_bits(4, stage)
        for native in (True, False):
            bitmap = agoq.layer_bitmap(b, native=native)
            if bitmap in seen:
                continue
            seen.append(bitmap)
            out.append(("stage %d B=%d %s" % (stage, b, "native" if native else "mix"), bitmap))
    return out


def section_c5(env):
    c = env.wl.CONFIGS["stage_sweep"]
    torch = env.torch
    tensors = [ActTensor(env, c["rows"], c["ffn"] if slot >= 3 else c["hidden"], c["seed"] + slot, c["dist"],
                         c["outlier_frac"], c["outlier_scale"]) for slot in range(5)]
    for label, bitmap in stage_maps(env.agoq):
        act_layer(env, "c5", label + " rows %d" % c["rows"], tensors, c["group"], bitmap)
    del tensors
    torch.cuda.empty_cache()
    gc = c["grad"]
    g, ocs, oss = grad_quant_row(env, "c5", gc["n"], c["group"], c["seed"], gc["sigma"], gc["spike_frac"],
                                 gc["spike_scale"])
    del g, ocs, oss
    torch.cuda.empty_cache()
    codes, scales = quantized_chunks(env, c["K"], gc["n"], c["group"], c["seed"] + 1, gc["sigma"],
                                     gc["spike_frac"], gc["spike_scale"])
    reduce_rows(env, "c5", codes, scales, c["K"], gc["n"], c["group"], share=True)
    del codes, scales
    torch.cuda.empty_cache()


def close_bf16(torch, got, want_bits, min_equal=0.995):
    """The bar of the fused kernels: at most one bf16 step apart, at least 99.5% equal
    (magnitudes below 2^-100 only need to be below 2^-100 on both sides)."""
    import numpy as np
    a = bits_of(torch, got).astype(np.int32)
    b = want_bits.astype(np.int32)
    tiny = ((a & 0x7FFF) < 0x0D80) & ((b & 0x7FFF) < 0x0D80)
    # distance in steps along the ordered bf16 line
    ka = np.where(a & 0x8000, -(a & 0x7FFF), a & 0x7FFF)
    kb = np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    d = np.abs(ka - kb)
    d[tiny] = 0
    return bool(d.max() <= 1 and (d == 0).mean() >= min_equal)


def section_fused(env):
    import numpy as np
    c = env.wl.CONFIGS["stage_sweep"]
    torch, L, st, R, group = env.torch, env.L, env.st, env.rows, c["group"]
    eps = 1e-5
    c32 = env.wl.CONFIGS["llama32b_act"]
    n32 = c32["acts"]["A"]
    # H, F: the seq-8192 tensors of the stage sweep, all four fused calls at every width;
    # N: the norm input of the 32B-shaped layer (5120 wide), the two RMSNorm calls at 4 and 8 bits
    for name, rows_, cols, widths, norm_only, cf in (("H", c["rows"], c["hidden"], (4, 5, 6, 8), False, c),
                                                     ("F", c["rows"], c["ffn"], (4, 5, 6, 8), False, c),
                                                     ("N", n32["rows"], n32["cols"], (4, 8), True, c32)):
        t = ActTensor(env, rows_, cols, cf["seed"], cf["dist"], cf["outlier_frac"], cf["outlier_scale"])
        if not norm_only:
            act_single(env, "fused", name, t, [group], [5, 6])
        n = t.n
        nx = rotation(2 * n)
        xs = t.copies(nx)
        ys = [env.empty(n, torch.bfloat16) for _ in range(nx)]
        gamma = 0.5 + torch.rand(cols, dtype=torch.float32, device=env.dev,
                                 generator=torch.Generator(device=env.dev).manual_seed(c["seed"]))
        rs = [env.empty(rows_, torch.float32) for _ in range(4)]
        for bits in widths:
            nc = rotation(n * bits // 8)
            cs = [env.empty(n * bits // 8, torch.uint8) for _ in range(nc)]
            ss = [env.empty(n // group, torch.float32) for _ in range(nc)]
            for i in range(nc):
                env.agoq.act_quant(xs[i % nx], group, bits, codes=cs[i], scales=ss[i])
            torch.cuda.synchronize()
            nb = algo_bytes_act(n, bits, group)
            case = "%s[%d,%d] b%d g%d" % (name, rows_, cols, bits, group)
            m = max(nx, nc)
            F = ctypes.c_float
            na = [(P(cs[i % nc].data_ptr()), P(ss[i % nc].data_ptr()), rows_, cols, group, bits, P(gamma.data_ptr()),
                   F(eps), P(ys[i % nx].data_ptr()), P(rs[i % 4].data_ptr()), st) for i in range(m)]
            fa = [(P(xs[i % nx].data_ptr()), rows_, cols, P(gamma.data_ptr()), F(eps), group, bits,
                   P(ys[i % nx].data_ptr()), P(rs[i % 4].data_ptr()), P(cs[i % nc].data_ptr()),
                   P(ss[i % nc].data_ptr()), st) for i in range(m)]
            ga = [(P(xs[i % nx].data_ptr()), P(xs[(i + 1) % nx].data_ptr()), n, group, bits, bits,
                   P(ys[i % nx].data_ptr()), P(cs[i % nc].data_ptr()), P(ss[i % nc].data_ptr()),
                   P(cs[(i + 1) % nc].data_ptr()), P(ss[(i + 1) % nc].data_ptr()), st) for i in range(m)]
            sa = [(P(cs[i % nc].data_ptr()), P(ss[i % nc].data_ptr()), bits, P(cs[(i + 1) % nc].data_ptr()),
                   P(ss[(i + 1) % nc].data_ptr()), bits, n, group, P(ys[i % nx].data_ptr()), st) for i in range(m)]
            ok_n = ok_f = ok_g = ok_s = None
            if env.check:
                hx0, hx1 = bits_of(torch, xs[0]), bits_of(torch, xs[1 % nx])
                hg = gamma.cpu().numpy()
                oc0, os0, _ = t.oracle(bits, group)
                if not norm_only:
                    oc1, os1 = env.oracle.act_quant(hx1, group, bits)
                # recompute side (slot 0 holds the codes of xs[0], slot 1 those of xs[1])
                assert L.agoq_act_dequant_rmsnorm(*na[0]) == 0
                torch.cuda.synchronize()
                wy, wr = env.oracle.act_dequant_rmsnorm(oc0, os0, rows_, cols, group, bits, hg, eps)
                ok_n = close_bf16(torch, ys[0], wy) and bool(np.allclose(rs[0].cpu().numpy(), wr, rtol=2e-6, atol=0))
                if nc >= 2 and not norm_only:
                    assert L.agoq_act_dequant_silu_mul(*sa[0]) == 0
                    torch.cuda.synchronize()
                    wz = env.oracle.act_dequant_silu_mul(oc0, os0, bits, oc1, os1, bits, n, group)
                    ok_s = close_bf16(torch, ys[0], wz)
                # forward side: layer output to the bar, stored codes and scales bit for bit
                cs[0].zero_()
                ss[0].zero_()
                assert L.agoq_rmsnorm_fwd_quant(*fa[0]) == 0
                torch.cuda.synchronize()
                wy, wr = env.oracle.rmsnorm_fwd(hx0, rows_, cols, hg, eps)
                ok_f = (close_bf16(torch, ys[0], wy) and np.array_equal(cs[0].cpu().numpy(), oc0) and
                        same_u32(torch, ss[0], os0))
                if nc >= 2 and nx >= 2 and not norm_only:
                    assert L.agoq_silu_mul_fwd_quant(*ga[0]) == 0
                    torch.cuda.synchronize()
                    wz = env.oracle.silu_mul_fwd(hx0, hx1)
                    ok_g = (close_bf16(torch, ys[0], wz) and np.array_equal(cs[0].cpu().numpy(), oc0) and
                            same_u32(torch, ss[0], os0) and np.array_equal(cs[1].cpu().numpy(), oc1) and
                            same_u32(torch, ss[1], os1))
                for i in range(nc):
                    env.agoq.act_quant(xs[i % nx], group, bits, codes=cs[i], scales=ss[i])
                torch.cuda.synchronize()
            if cols <= 16384:
                us = R.timed(lambda i: L.agoq_act_dequant_rmsnorm(*na[i % m]))
                R.add("fused", "act_dequant_rmsnorm", case, us, nb + 4 * rows_, ok_n)
                us = R.timed(lambda i: L.agoq_rmsnorm_fwd_quant(*fa[i % m]))
                R.add("fused", "rmsnorm_fwd_quant", case, us, nb + 2 * n + 4 * rows_, ok_f)
            if not norm_only:
                us = R.timed(lambda i: L.agoq_silu_mul_fwd_quant(*ga[i % m]))
                R.add("fused", "silu_mul_fwd_quant", case, us, 2 * nb + 2 * n, ok_g)
                for i in range(nc):
                    env.agoq.act_quant(xs[i % nx], group, bits, codes=cs[i], scales=ss[i])
                us = R.timed(lambda i: L.agoq_act_dequant_silu_mul(*sa[i % m]))
                R.add("fused", "act_dequant_silu_mul", case, us, 2 * (n * bits // 8 + 4 * (n // group)) + 2 * n, ok_s)
            del cs, ss
        del xs, ys, t
        torch.cuda.empty_cache()


def section_gradx(env):
    import numpy as np
    c = env.wl.CONFIGS["llama8b_grad"]
    torch, L, st, R, agoq = env.torch, env.L, env.st, env.rows, env.agoq
    n, group, K = c["n"], c["group"], c["K"]
    g, ocs, oss = grad_quant_row(env, "gradx", n, group, c["seed"], c["sigma"], c["spike_frac"], c["spike_scale"])
    nout = len(ocs)
    launches = max(20, min(R.launches, int(2e9 / n)))
    mcs = [env.empty(n, torch.int8) for _ in range(nout)]
    mss = [env.empty(n // group, torch.float32) for _ in range(nout)]
    for i in range(nout):
        agoq.grad_quant(g[(i + 1) % 2], group, codes=mcs[i], scales=mss[i])
    torch.cuda.synchronize()
    gb = [x.to(torch.bfloat16) for x in g]
    ok32 = ok16 = okd = None
    if env.check:
        hm, hs = mcs[0].cpu().numpy(), mss[0].cpu().numpy()
        agoq.grad_accumulate(mcs[0], mss[0], g[0], group, out_codes=ocs[0], out_scales=oss[0])
        torch.cuda.synchronize()
        wc, ws = env.oracle.grad_accumulate(hm, hs, g[0].cpu().numpy(), group)
        ok32 = np.array_equal(ocs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
        agoq.grad_accumulate(mcs[0], mss[0], gb[0], group, out_codes=ocs[0], out_scales=oss[0])
        torch.cuda.synchronize()
        wc, ws = env.oracle.grad_accumulate(hm, hs, bits_of(torch, gb[0]), group)
        ok16 = np.array_equal(ocs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
    us = R.timed(lambda i: agoq.grad_accumulate(mcs[i % nout], mss[i % nout], g[i % 2], group,
                                                out_codes=ocs[i % nout], out_scales=oss[i % nout]), launches)
    R.add("gradx", "grad_accumulate", "fp32 addend n=%d g%d" % (n, group), us, n * 6 + 8 * (n // group), ok32)
    us = R.timed(lambda i: agoq.grad_accumulate(mcs[i % nout], mss[i % nout], gb[i % 2], group,
                                                out_codes=ocs[i % nout], out_scales=oss[i % nout]), launches)
    R.add("gradx", "grad_accumulate", "bf16 addend n=%d g%d" % (n, group), us, n * 4 + 8 * (n // group), ok16)
    del gb
    fo = [env.empty(n, torch.float32) for _ in range(2)]
    if env.check:
        agoq.grad_dequant(mcs[0], mss[0], group, out=fo[0])
        torch.cuda.synchronize()
        okd = np.array_equal(fo[0].cpu().numpy().view(np.uint32),
                             env.oracle.grad_dequant(mcs[0].cpu().numpy(), mss[0].cpu().numpy(), group).view(np.uint32))
    us = R.timed(lambda i: agoq.grad_dequant(mcs[i % nout], mss[i % nout], group, out=fo[i % 2]), launches)
    R.add("gradx", "grad_dequant", "n=%d g%d" % (n, group), us, n * 5 + 4 * (n // group), okd)
    del mcs, mss
    # E4M3 code book: store, reduce, dequantize
    ucs = [t.view(torch.uint8) for t in ocs]
    ok8 = None
    if env.check:
        agoq.fp8_grad_quant(g[0], group, codes=ucs[0], scales=oss[0])
        torch.cuda.synchronize()
        wc, ws = env.oracle.fp8_grad_quant(g[0].cpu().numpy(), group)
        ok8 = np.array_equal(ucs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
    us = R.timed(lambda i: agoq.fp8_grad_quant(g[i % 2], group, codes=ucs[i % nout], scales=oss[i % nout]), launches)
    R.add("gradx", "fp8_grad_quant", "n=%d g%d" % (n, group), us, algo_bytes_grad_quant(n, group), ok8)
    fcodes = torch.empty((K, n), dtype=torch.uint8, device=env.dev)
    fscales = torch.empty((K, n // group), dtype=torch.float32, device=env.dev)
    for k in range(K):
        gk = env.wl.grad_device(n, c["seed"] + 300 + k, c["sigma"], c["spike_frac"], c["spike_scale"])
        agoq.fp8_grad_quant(gk, group, codes=fcodes[k], scales=fscales[k])
        torch.cuda.synchronize()
        del gk
    okr = okq = None
    if env.check:
        agoq.fp8_grad_reduce_requant(fcodes, fscales, n, group, out_codes=ucs[0], out_scales=oss[0])
        agoq.fp8_grad_dequant(fcodes[0], fscales[0], group, out=fo[0])
        torch.cuda.synchronize()
        wc, ws = env.oracle.fp8_grad_reduce_requant(fcodes.cpu().numpy(), fscales.cpu().numpy(), n, group)
        okr = np.array_equal(ucs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
        okq = np.array_equal(fo[0].cpu().numpy().view(np.uint32),
                             env.oracle.fp8_grad_dequant(fcodes[0].cpu().numpy(), fscales[0].cpu().numpy(), group).view(np.uint32))
    us = R.timed(lambda i: agoq.fp8_grad_reduce_requant(fcodes, fscales, n, group, out_codes=ucs[i % nout],
                                                        out_scales=oss[i % nout]), launches)
    R.add("gradx", "fp8_grad_reduce_requant", "K=%d n=%d g%d" % (K, n, group), us, algo_bytes_reduce(n, K, group), okr)
    us = R.timed(lambda i: agoq.fp8_grad_dequant(fcodes[i % K], fscales[i % K], group, out=fo[i % 2]), launches)
    R.add("gradx", "fp8_grad_dequant", "n=%d g%d" % (n, group), us, algo_bytes_grad_quant(n, group), okq)
    del fcodes, fscales, fo, g, ocs, oss, ucs
    torch.cuda.empty_cache()


def section_sr(env):
    """The stochastic-rounding entry points (not used by the paper: an extension) on the 8B
    shapes, each compared whole with the oracle's independent implementation of the same
    counter-based generator."""
    import numpy as np
    torch, L, st, R, agoq, wl = env.torch, env.L, env.st, env.rows, env.agoq, env.wl
    seed = 0x5EED1234
    ca = wl.CONFIGS["llama8b_act"]
    sh = ca["acts"]["F"]
    t = ActTensor(env, sh["rows"], sh["cols"], ca["seed"], ca["dist"], ca["outlier_frac"], ca["outlier_scale"])
    n, group = t.n, ca["group"]
    nx = rotation(2 * n)
    xs = t.copies(nx)
    for bits in (4, 8):
        nc = rotation(n * bits // 8)
        cs = [env.empty(n * bits // 8, torch.uint8) for _ in range(nc)]
        ss = [env.empty(n // group, torch.float32) for _ in range(nc)]
        m = max(nx, nc)
        qa = [(P(xs[i % nx].data_ptr()), n, group, bits, seed, P(cs[i % nc].data_ptr()), P(ss[i % nc].data_ptr()), st)
              for i in range(m)]
        ok = None
        if env.check:
            assert L.agoq_act_quant_sr(*qa[0]) == 0
            torch.cuda.synchronize()
            oc, os_ = env.oracle.act_quant_sr(bits_of(torch, t.base), group, bits, seed)
            ok = np.array_equal(cs[0].cpu().numpy(), oc) and same_u32(torch, ss[0], os_)
        us = R.timed(lambda i: L.agoq_act_quant_sr(*qa[i % m]))
        R.add("sr", "act_quant_sr", "F[%d,%d] b%d g%d" % (t.rows, t.cols, bits, group), us,
              algo_bytes_act(n, bits, group), ok)
        del cs, ss
    del xs, t
    torch.cuda.empty_cache()

    c = wl.CONFIGS["llama8b_grad"]
    n, group, K = c["n"], c["group"], c["K"]
    g = [wl.grad_device(n, c["seed"] + i, c["sigma"], c["spike_frac"], c["spike_scale"]) for i in range(2)]
    nout = rotation(n, floor=3)
    ocs = [env.empty(n, torch.int8) for _ in range(nout)]
    oss = [env.empty(n // group, torch.float32) for _ in range(nout)]
    launches = max(20, min(R.launches, int(2e9 / n)))
    ok = None
    if env.check:
        agoq.grad_quant(g[0], group, codes=ocs[0], scales=oss[0], sr_seed=seed)
        torch.cuda.synchronize()
        wc, ws = env.oracle.grad_quant_sr(g[0].cpu().numpy(), group, seed)
        ok = np.array_equal(ocs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
    us = R.timed(lambda i: agoq.grad_quant(g[i % 2], group, codes=ocs[i % nout], scales=oss[i % nout], sr_seed=seed),
                 launches)
    R.add("sr", "grad_quant_sr", "n=%d g%d" % (n, group), us, algo_bytes_grad_quant(n, group), ok)
    # accumulate: the stored gradient is the nearest-rounding store of g[1]
    mc, ms = agoq.grad_quant(g[1], group)
    ok = None
    if env.check:
        agoq.grad_accumulate(mc, ms, g[0], group, out_codes=ocs[0], out_scales=oss[0], sr_seed=seed)
        torch.cuda.synchronize()
        wc, ws = env.oracle.grad_accumulate_sr(mc.cpu().numpy(), ms.cpu().numpy(), g[0].cpu().numpy(), group, seed)
        ok = np.array_equal(ocs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
    us = R.timed(lambda i: agoq.grad_accumulate(mc, ms, g[i % 2], group, out_codes=ocs[i % nout],
                                                out_scales=oss[i % nout], sr_seed=seed), launches)
    R.add("sr", "grad_accumulate_sr", "fp32 addend n=%d g%d" % (n, group), us, n * 6 + 8 * (n // group), ok)
    del g, mc, ms
    torch.cuda.empty_cache()
    codes, scales = quantized_chunks(env, K, n, group, c["seed"] + 100, c["sigma"], c["spike_frac"], c["spike_scale"])
    ok = None
    if env.check:
        agoq.grad_reduce_requant(codes, scales, n, group, out_codes=ocs[0], out_scales=oss[0], sr_seed=seed)
        torch.cuda.synchronize()
        wc, ws = env.oracle.grad_reduce_requant_sr(codes.cpu().numpy(), scales.cpu().numpy(), n, group, seed)
        ok = np.array_equal(ocs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
    us = R.timed(lambda i: agoq.grad_reduce_requant(codes, scales, n, group, out_codes=ocs[i % nout],
                                                    out_scales=oss[i % nout], sr_seed=seed), launches)
    R.add("sr", "grad_reduce_requant_sr", "K=%d n=%d g%d" % (K, n, group), us, algo_bytes_reduce(n, K, group), ok)
    del codes, scales, ocs, oss
    torch.cuda.empty_cache()


def section_kscan(env):
    """Other chunk counts on the 8B shard size (random codes and scales)."""
    import numpy as np
    c = env.wl.CONFIGS["llama8b_grad"]
    torch, L, st, R = env.torch, env.L, env.st, env.rows
    group = c["group"]
    ns = c["n"] // 8
    nout = rotation(ns, floor=3)
    ocs = [env.empty(ns, torch.int8) for _ in range(nout)]
    oss = [env.empty(ns // group, torch.float32) for _ in range(nout)]
    gen = torch.Generator(device=env.dev).manual_seed(c["seed"] + 900)
    for K in list(range(1, 17)) + [32, 64]:
        nsl = max(1, min(8, -(-(GiB + GiB // 2) // (K * ns))))
        bufs = [(torch.randint(-127, 128, (K, ns), device=env.dev, dtype=torch.int8, generator=gen),
                 torch.rand((K, ns // group), device=env.dev, dtype=torch.float32, generator=gen) * 1e-5 + 1e-8)
                for _ in range(nsl)]
        ok = None
        if env.check:
            cc, sc = bufs[0]
            assert L.agoq_grad_reduce_requant(P(cc.data_ptr()), ns, P(sc.data_ptr()), ns // group, K, ns, group,
                                              P(ocs[0].data_ptr()), P(oss[0].data_ptr()), st) == 0
            torch.cuda.synchronize()
            wc, ws = env.oracle.grad_reduce_requant(cc.cpu().numpy(), sc.cpu().numpy(), ns, group)
            ok = np.array_equal(ocs[0].cpu().numpy(), wc) and same_u32(torch, oss[0], ws)
        calls = [(P(bufs[i % nsl][0].data_ptr()), ns, P(bufs[i % nsl][1].data_ptr()), ns // group, K, ns, group,
                  P(ocs[i % nout].data_ptr()), P(oss[i % nout].data_ptr()), st) for i in range(nsl * nout)]
        us = R.timed(lambda i: L.agoq_grad_reduce_requant(*calls[i % len(calls)]))
        R.add("kscan", "grad_reduce_requant", "K=%d n=%d g%d" % (K, ns, group), us, algo_bytes_reduce(ns, K, group), ok)
        del bufs, calls
        torch.cuda.empty_cache()


def section_messages(env):
    """The quantize / reduce / dequantize work one GPU does for one decomposed 8-bit All-Reduce
    over 8 peers on a gradient bucket of n elements (store n as int8; reduce the 8 received
    chunks of its n/8 shard; dequantize the n gathered elements): the work the paper's
    communication breakdown (Table comm_savings, column Quant/Dequant) times at 2^15..2^30."""
    torch, L, st, R, wl = env.torch, env.L, env.st, env.rows, env.wl
    group, K = 128, 8
    for log2n in (15, 20, 25, 28, 30):
        n = 1 << log2n
        ns = n // K
        nrot = max(2, min(16, -(-(GiB + GiB // 2) // (4 * n))))
        g = [wl.grad_device(n, 700 + i, 1e-4, 0.001, 100.0) for i in range(nrot)]
        codes = [env.empty(n, torch.int8) for _ in range(nrot)]
        scales = [env.empty(n // group, torch.float32) for _ in range(nrot)]
        out = [env.empty(n, torch.float32) for _ in range(2)]
        rc = torch.randint(-127, 128, (K, ns), device=env.dev, dtype=torch.int8)
        rs = torch.rand((K, ns // group), device=env.dev, dtype=torch.float32) * 1e-5 + 1e-8
        oc = env.empty(ns, torch.int8)
        osc = env.empty(ns // group, torch.float32)
        pg = [P(t.data_ptr()) for t in g]
        pc = [P(t.data_ptr()) for t in codes]
        ps = [P(t.data_ptr()) for t in scales]
        po = [P(t.data_ptr()) for t in out]
        prc, prs, poc, pos = P(rc.data_ptr()), P(rs.data_ptr()), P(oc.data_ptr()), P(osc.data_ptr())

        def message(i, stream=st):
            r = i % nrot
            bad = L.agoq_grad_quant(pg[r], n, group, pc[r], ps[r], stream)
            bad |= L.agoq_grad_reduce_requant(prc, ns, prs, ns // group, K, ns, group, poc, pos, stream)
            bad |= L.agoq_grad_dequant(pc[r], ps[r], n, group, po[i % 2], stream)
            assert bad == 0
        launches = max(5, min(R.launches, int(4e9 / n)))
        us = R.timed(message, launches)
        nbytes = 2 * algo_bytes_grad_quant(n, group) + algo_bytes_reduce(ns, K, group)
        case = "n=2^%d (fp32 %d MiB) K=8" % (log2n, 4 * n >> 20)
        R.add("messages", "quant+reduce+dequant", case, us, nbytes)
        if log2n <= 20:
            # launch-latency bound: the same three kernels, 16 messages captured in a HIP graph
            # (the library neither allocates nor synchronizes, so a caller may capture it)
            per = 16
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                cap = P(torch.cuda.current_stream().cuda_stream)
                for i in range(per):
                    message(i, cap)
            us = R.timed(lambda i: graph.replay(), max(5, launches // per)) / per
            R.add("messages", "quant+reduce+dequant, graph", case, us, nbytes)
            del graph
        del g, codes, scales, out, rc, rs, oc, osc
        torch.cuda.empty_cache()


def section_floor(env):
    """What a launch of a small tensor's footprint can reach at all: streaming kernels that move
    the same bytes with the same access widths and do no arithmetic, timed under the same
    protocol; then the real calls alternating two streams."""
    torch, L, st, R = env.torch, env.L, env.st, env.rows
    shapes = (("A[4096,4096]", 4096 * 4096), ("A[4096,5120]", 4096 * 5120), ("H[8192,4096]", 8192 * 4096))
    for name, n in shapes:
        items = n // 8                      # one item = the 8 elements a lane owns
        nx = rotation(2 * n)
        src = [torch.randint(0, 255, (2 * n,), dtype=torch.uint8, device=env.dev) for _ in range(nx)]
        dst = [env.empty(2 * n, torch.uint8) for _ in range(nx)]
        for label, lb, sb in (("read 16 B", 16, 0), ("quantize-4 traffic 16 B -> 4 B", 16, 4),
                              ("quantize-8 traffic 16 B -> 8 B", 16, 8), ("dequantize-4 traffic 4 B -> 16 B", 4, 16),
                              ("dequantize-8 traffic 8 B -> 16 B", 8, 16), ("copy 16 B -> 16 B", 16, 16)):
            calls = [(P(src[i].data_ptr()), lb, P(dst[i].data_ptr()), sb, items, st) for i in range(nx)]
            assert L.agoq_probe_stream(*calls[0]) == 0
            us = R.timed(lambda i: L.agoq_probe_stream(*calls[i % nx]))
            R.add("floor", "probe_stream", "%s %s" % (name, label), us, items * (lb + sb))
        del src, dst
        torch.cuda.empty_cache()
    two = [torch.cuda.Stream(), torch.cuda.Stream()]
    for s_ in two:
        with torch.cuda.stream(s_):
            torch.zeros(1, device=env.dev)
    torch.cuda.synchronize()
    check, env.check = env.check, False
    section_c2(env, two_streams=two, section="floor")
    section_c4(env, two_streams=two, section="floor")
    env.check = check


# ---------------------------------------------------------------------------------------------
# the step
# ---------------------------------------------------------------------------------------------

def section_step(env, args):
    torch, wl, agoq = env.torch, env.wl, env.agoq
    dev, stream = env.dev, env.stream
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

    # descriptor arrays of the two layer launches (host memory, marshalled once)
    q_slots = agoq.layer_slots(acts, act_bits, act_codes, act_scales, GROUP)
    d_slots = agoq.layer_slots(act_out, act_bits, act_codes, act_scales, GROUP)

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

    # The same step with the activations as ten single-tensor calls (a forward pass produces
    # the five tensors at five different times, so a caller may not be able to batch them):
    # reported beside `value`, not part of it.
    P_ = ctypes.c_void_p
    L, st = env.L, env.st
    qcalls = [(P_(x.data_ptr()), x.numel(), GROUP, b, P_(c.data_ptr()), P_(s_.data_ptr()), st)
              for x, b, c, s_ in zip(acts, act_bits, act_codes, act_scales)]
    dcalls = [(P_(c.data_ptr()), P_(s_.data_ptr()), y.numel(), GROUP, b, P_(y.data_ptr()), st)
              for y, b, c, s_ in zip(act_out, act_bits, act_codes, act_scales)]

    def step_single():
        bad = 0
        for a in qcalls:
            bad |= L.agoq_act_quant(*a)
        agoq.grad_quant(grad, GROUP, codes=g_codes, scales=g_scales, stream=stream)
        agoq.grad_reduce_requant(in_codes, in_scales, n_grad, GROUP, out_codes=r_codes,
                                 out_scales=r_scales, stream=stream)
        for a in dcalls:
            bad |= L.agoq_act_dequant(*a)
        assert bad == 0
    for _ in range(args.warmup):
        step_single()
    torch.cuda.synchronize()
    t_single = time.perf_counter()
    for _ in range(args.steps):
        step_single()
    torch.cuda.synchronize()
    single_s = (time.perf_counter() - t_single) / args.steps

    # per-kernel breakdown of the step (separate passes, not part of `value`)
    ev = {k: [] for k in ("t0", "t1", "t2", "t3", "t4")}
    for _ in range(min(args.steps, 20)):
        step(ev)
    torch.cuda.synchronize()

    def avg_us(a, b):
        return 1e3 * sum(x.elapsed_time(y) for x, y in zip(ev[a], ev[b])) / len(ev[a])

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(torch, env.oracle, acts, act_bits, act_codes, act_scales, act_out, grad, g_codes,
                           g_scales, in_codes, in_scales, r_codes, r_scales, n_grad)
    ok = None if cpu is None else cpu["gpu_matches_oracle_on_sample"]
    for name, a, b, nbytes in (("act_quant_layer", "t0", "t1", bytes_quant),
                               ("grad_quant", "t1", "t2", bytes_gq),
                               ("grad_reduce_requant", "t2", "t3", bytes_red),
                               ("act_dequant_layer", "t3", "t4", bytes_dequant)):
        env.rows.add("step", name, "8B layer, n=%d K=%d" % (n_grad, K_CHUNKS), avg_us(a, b), nbytes, ok)
    return {
        "value": round(value, 1), "ms_per_step": round(ms_per_step, 4), "bitmap": bitmap,
        "bytes_step": bytes_step, "cpu": cpu,
        "per_tensor_calls": {"value": round(bytes_step / single_s / 1e9, 1), "ms_per_step": round(single_s * 1e3, 4),
                             "launches_per_step": 12,
                             "note": "the same step with the five activations quantized and dequantized by "
                                     "single-tensor calls instead of one layer launch each"},
        "roofline": {
            "bound": "hbm", "kernel": "grad_reduce_kernel<128,8>",
            "achieved": round(red_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
            "frac": round(red_gbps / PEAK_HBM_GBPS, 4), "traffic": TRAFFIC_REDUCE_K8_BYTES,
            "traffic_source": TRAFFIC_SOURCE,
            "algo_bytes_per_launch": bytes_red, "avg_launch_us": round(red_ms * 1e3, 2),
        },
    }


def cpu_baseline(torch, oracle, acts, act_bits, act_codes, act_scales, act_out, grad, g_codes, g_scales,
                 in_codes, in_scales, r_codes, r_scales, n_grad):
    """Time the oracle (as it stands) on the host, with all its threads, on one whole step of
    the same inputs (three passes, the median counts: some 20 core-seconds of work), and
    check the GPU outputs of the last timed step against it, every byte.  A one-thread
    figure on 1/16 of the step follows."""
    import numpy as np

    threads = oracle.max_threads()
    host_acts = [bits_of(torch, x) for x in acts]
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
        ok &= np.array_equal(c.cpu().numpy(), oc) and same_u32(torch, s, os_) and \
            np.array_equal(bits_of(torch, y), oy)
    ok &= np.array_equal(g_codes[:ng].cpu().numpy(), gq[0]) and same_u32(torch, g_scales[:ng // GROUP], gq[1])
    ok &= np.array_equal(r_codes[:nr].cpu().numpy(), red[0]) and same_u32(torch, r_scales[:nr // GROUP], red[1])
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


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--sections", default=DEFAULT_SECTIONS,
                    help="comma-separated subset of: " + ",".join(ALL_SECTIONS) + " (default: all)")
    ap.add_argument("--launches", type=int, default=200, help="back-to-back launches per timed run of a row")
    ap.add_argument("--reps", type=int, default=5, help="timed runs per row (the median counts)")
    ap.add_argument("--no-check", action="store_true",
                    help="skip the full-tensor comparisons of the rows with the oracle (profiler runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mark-rows", action="store_true",
                    help="profiler runs: start every timed run with one launch of the library's copy kernel "
                         "whose workgroup count is the run's ordinal (a row's \"mark\" in the JSON line), so "
                         "that a kernel trace can be cut into rows")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device copy a few times and exit: gives the hardware "
                         "counters a kernel of known traffic to be scaled against")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU's share of the path and uses no collective; "
              "run it with --gpus 1", file=sys.stderr)
        return 2
    sections = ALL_SECTIONS if args.sections == "all" else tuple(s for s in args.sections.split(",") if s)
    for s in sections:
        if s not in ALL_SECTIONS:
            print("bench.py: unknown section %r" % s, file=sys.stderr)
            return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if "step" not in sections:
        args.no_cpu_baseline = True
    env = Env(args)
    if args.calibrate_copy:
        n = 1 << 28                                   # 1 GiB of fp32 read, 1 GiB written
        src = torch.ones(n, dtype=torch.float32, device=env.dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "read_bytes_per_launch": 4 * n,
                          "write_bytes_per_launch": 4 * n, "launches": 5}))
        return 0

    t_all = time.perf_counter()
    step = section_step(env, args) if "step" in sections else None
    torch.cuda.empty_cache()
    for name, fn in (("c2", section_c2), ("c3", section_c3), ("c4", section_c4), ("c5", section_c5),
                     ("fused", section_fused), ("gradx", section_gradx), ("sr", section_sr), ("kscan", section_kscan),
                     ("messages", section_messages), ("floor", section_floor)):
        if name in sections:
            fn(env)
            torch.cuda.empty_cache()
    checked = [r["gpu_matches_oracle"] for r in env.rows.rows.values() if "gpu_matches_oracle" in r]

    out = {
        "metric": "effective HBM GB/s (quant, dequant, grad reduce) and % of MI355X peak",
        "value": step["value"] if step else None,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": step["ms_per_step"] if step else None,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "LLaMA-8B-shaped decoder layer: 5 stored activations seq 4096 mb 1 "
                        "(bits %s, group 128) quant+dequant, fp32 gradient of 218,103,808 -> int8, "
                        "8-chunk local reduce+requant" % (step["bitmap"] if step else "[8, 4, 8, 4, 4]",),
            "group": GROUP, "K": K_CHUNKS, "algo_bytes_per_step": step["bytes_step"] if step else None,
            "sections": list(sections), "launches_per_row": args.launches, "reps_per_row": args.reps,
        },
        "frac_of_peak": round(step["value"] / PEAK_HBM_GBPS, 4) if step else None,
        "roofline": step["roofline"] if step else None,
        "step_per_tensor_calls": step["per_tensor_calls"] if step else None,
        "kernels": env.rows.rows,
        "rows_checked_against_oracle": len(checked),
        "rows_matching_oracle": sum(1 for c in checked if c),
        "cpu_baseline": step["cpu"] if step else None,
        "bench_wall_s": round(time.perf_counter() - t_all, 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
