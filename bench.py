#!/usr/bin/env python3
"""Benchmark of the hot path on ONE MI355X.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--reps N] [--workload NAME]

Without --workload the line's headline (`value`, `roofline`, `cpu_baseline`) is the largest
decoder stage (stage5) and `also` carries every other measurement of the path, each with its
own roofline and the oracle timed beside it:
  stage2 / stage3 / stage5   decoder stages of the benchmark configurations.  A step is the
          steady-state stage step: forward(t), backward(t - tau), delayed SGD update
          (rv_stage_step).  tokens/s; bf16 MFMA roofline.
  avg4    1e9 fp32 elements, C = 16 replicas in HBM, rings R in {1,2,4,8}: ring-partitioned mean
          with one replica's SGD step folded in, to one output (reduce-only) and written back to
          all replicas.  GB/s of algorithmic bytes; HBM roofline.
  avg2 / avg3 / avg5   the mean of the stages' own replica sets (C=4,R=4 / C=8,R=4 / C=8,R=8).
  update  the delayed SGD update with the bf16 weight version on config 3's parameter count
          (14 B per parameter); HBM roofline.
  mlp1    the tiny two-stage fp32 MLP chain (launch bound): samples/s only.
  gemm    one bf16 matrix product alone (--shape M,N,K, --layout fwd|dgrad|wgrad, --operands
          normal|zeros|ones), for counter runs.
Every timing is the median of --reps repetitions of --steps steps (HIP events on the stream
the work is enqueued on).  Inputs are synthetic and seeded (activations N(0,1) and upstream
gradients N(0,1e-3) rounded to bf16, parameters N(0,0.02) with LayerNorm gains 1+N(0,0.02);
replicas x_c = o + n_c with o, n_c ~ N(0,1)) and resident in HBM before the timed region.
The oracle (CPU fp64) is timed beside each on a bounded sample ("cpu_baseline": all host cores,
and one thread).
"""
import argparse
import json
import os
import re
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
BF16_PEAK_TFLOPS = 2500.0    # MI355X published dense bf16 MFMA rate

DECODER_CFG = {
    "stage2": dict(L=4, d=1024, h=16, f=4096, S=512, mb=8, tau=2, eta=1e-3, seed=2, C=4, R=4),
    "stage3": dict(L=8, d=2048, h=16, f=8192, S=1024, mb=4, tau=3, eta=1e-3, seed=3, C=8, R=4),
    "stage5": dict(L=12, d=1600, h=25, f=6400, S=1024, mb=8, tau=4, eta=1e-3, seed=5, C=8, R=8),
}


def n_params(c):
    return c["L"] * (4 * c["d"] ** 2 + 2 * c["d"] * c["f"] + 9 * c["d"] + c["f"])


def host_cores():
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count()


def events_ms(fn, steps, warmup, reps=1):
    """Median over `reps` repetitions of the mean time of `steps` calls of fn, timed with HIP
    events on torch's current stream.  Returns (median ms per call, wall ms per call, all reps)."""
    import torch
    for _ in range(warmup):
        fn()
    per, walls = [], []
    for _ in range(reps):
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        walls.append((time.perf_counter() - t0) * 1e3 / steps)
        per.append(e0.elapsed_time(e1) / steps)
    return statistics.median(per), statistics.median(walls), per


def traffic_table():
    """HBM bytes per launch from the rocprofv3 counter runs, read from the table kept beside the
    profiles that produced them (profiles/hbm_traffic.md: | kernel | shape | bytes | ...)."""
    out = {}
    try:
        for line in open(os.path.join(ROOT, "profiles", "hbm_traffic.md")):
            m = re.match(r"\|\s*`([^`]+)`\s*\|\s*([^|]+?)\s*\|\s*([0-9.eE+]+)\s*\|", line)
            if m:
                out[(m.group(1), m.group(2))] = float(m.group(3))
    except OSError:
        pass
    return out


def mfma_roofline(flops, us, kernel=None, **extra):
    tf = flops / (us * 1e-6) / 1e12
    r = {"bound": "mfma", "achieved": tf, "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / BF16_PEAK_TFLOPS}
    if kernel:
        r["kernel"] = kernel
    r.update(extra)
    return r


def hbm_roofline(nbytes, ms, kernel, shape_key=None):
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
            "traffic": traffic_table().get((kernel, shape_key)) if shape_key else None, "kernel": kernel,
            "us_per_launch": ms * 1e3, "algorithmic_bytes_per_launch": nbytes}


def decoder_flops_per_token(c):
    gemm = 6 * c["L"] * (4 * c["d"] ** 2 + 2 * c["d"] * c["f"])
    attn = 6 * c["S"] * c["d"] * c["L"]
    return gemm + attn


def decoder_params(seed, c):
    """Flat fp32 parameter vector on the device: weights, biases, LN beta ~ N(0, 0.02);
    LN gamma ~ 1 + N(0, 0.02)."""
    import torch
    from paper_2401_01728_amd.inputs import device
    d, f, L = c["d"], c["f"], c["L"]
    per = 4 * d * d + 2 * d * f + 9 * d + f
    w = torch.empty(L * per, dtype=torch.float32, device="cuda")
    device.fill_normal_(w, seed, 0, 0.0, 0.02)
    for l in range(L):
        base = l * per
        w[base:base + d] += 1.0                                   # ln1.gamma
        o2 = base + 2 * d + 3 * d * d + 3 * d + d * d + d          # ln2.gamma
        w[o2:o2 + d] += 1.0
    return w


# ---------------------------------------------------------------------------------------------
# decoder stage step
# ---------------------------------------------------------------------------------------------
def bench_stage(args, name, cpu_seconds=20.0):
    import torch
    import paper_2401_01728_amd as rv
    from paper_2401_01728_amd.inputs import device
    c = DECODER_CFG[name]
    st = rv.Stage.decoder(c["L"], c["d"], c["h"], c["f"], c["S"], c["mb"], c["tau"], c["eta"])
    st.set_params(decoder_params(c["seed"], c))
    shape = (c["mb"], c["S"], c["d"])
    n_in = 4
    xs = [device.fill_normal_(torch.empty(shape, dtype=torch.bfloat16, device="cuda"), c["seed"], 1000 + i) for i in range(n_in)]
    gs = [device.fill_normal_(torch.empty(shape, dtype=torch.bfloat16, device="cuda"), c["seed"], 2000 + i, 0.0, 1e-3) for i in range(n_in)]
    out = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    gin = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    tau = c["tau"]
    state = {"t": 0}
    for t in range(tau):                                   # pipeline fill: forwards only
        st.forward(t, xs[t % n_in], out)
    state["t"] = tau

    def step():
        t = state["t"]
        if args.no_overlap:            # the two halves as separate calls on one stream
            st.forward(t, xs[t % n_in], out)
            st.backward(t - tau, gs[(t - tau) % n_in], gin)
        else:
            st.step(t, xs[t % n_in], t - tau, gs[(t - tau) % n_in], out, gin)
        state["t"] = t + 1

    # Warm-up: at least --warmup steps, then on until the step time is steady.  On the MI355X boxes
    # used here the first 1-2 s of a run of concurrent streams are 4-13 % slower than every step after
    # them (kernels and whole steps alike, on any box, whatever ran before); a training run lives in
    # the steady state, so that is what is timed.  The cold figure is reported beside it.
    import torch as _t
    warm_steps, blocks, t_w0 = 0, [], time.perf_counter()
    for _ in range(max(args.warmup, tau + 3)):
        step()
    warm_steps = max(args.warmup, tau + 3)
    while not args.cold and time.perf_counter() - t_w0 < 15.0:
        e0 = _t.cuda.Event(enable_timing=True); e1 = _t.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            step()
        e1.record(); _t.cuda.synchronize()
        warm_steps += 10
        blocks.append(e0.elapsed_time(e1) / 10)
        if len(blocks) >= 6 and time.perf_counter() - t_w0 > 3.0 and max(blocks[-4:]) <= 1.01 * min(blocks[-4:]):
            break
    # The dominant kernel of the step (largest share of its rocprofv3 trace) is the grouped
    # weight-gradient kernel: dW2 | dW1 | dWo | dWqkv of one block over the microbatch's tokens, in
    # one to three launches per block (the library decides when each product goes out).  The
    # library brackets each of its launches with HIP events on the stream it goes to, here,
    # inside the timed steps, beside everything else the step has running.
    st.profile(True)
    ms, wall_ms, per = events_ms(step, args.steps, 0, args.reps)
    launches, k_us = st.profile_read()
    st.profile(False)
    tokens = c["mb"] * c["S"]
    T, d, f = tokens, c["d"], c["f"]
    flops = decoder_flops_per_token(c) * tokens
    kfl_block = 2.0 * T * (2 * d * f + 4 * d * d)
    blocks_timed = c["L"] * args.steps * args.reps
    per_block = launches / float(blocks_timed) if launches else 1.0   # launches of that kernel per block
    kfl = kfl_block / per_block                                        # mean flops of one launch
    kname = "gemm_dtl_grouped_wgrad_kernel"
    kshape = "%s: K=%d tokens, d=%d, ffn=%d" % (name, T, d, f)
    res = {"metric": "stage tokens/s (fwd+bwd+delayed SGD)", "value": tokens / (ms * 1e-3), "unit": "tokens/s",
           "ms_per_step": ms, "dtype": "bf16",
           "config": {"workload": "%s: %d pre-LN decoder blocks d=%d h=%d ffn=%d seq=%d microbatch=%d tau=%d" % (
               name, c["L"], c["d"], c["h"], c["f"], c["S"], c["mb"], c["tau"]), "tokens_per_step": tokens},
           "wall_ms_per_step": wall_ms, "ms_per_step_reps": per,
           "warmup_steps_run": warm_steps, "cold_ms_per_step": blocks[0] if blocks else None}
    res["roofline"] = mfma_roofline(
        kfl, k_us, kernel="%s (dW2, dW1, dWo, dWqkv of one block in %.3g launches, K=%d tokens), inside the timed steps" % (
            kname, per_block, T),
        traffic=traffic_table().get((kname, kshape)), us_per_launch=k_us, launches_timed=launches,
        launches_per_block=per_block, algorithmic_flops_per_launch=kfl)
    # the whole step against the same peak: model flops of forward + backward (all kernels, three
    # streams) over the step time - the figure the 50 % target is about
    res["roofline_step"] = mfma_roofline(flops, ms * 1e3, algorithmic_flops_per_step=flops)
    del st
    torch.cuda.empty_cache()
    if args.step_only:
        return res
    # the same kernel launched alone (nothing else on the chip), operands with the step's distributions
    from paper_2401_01728_amd import kernels as kk
    act = lambda n: torch.empty(T, n, dtype=torch.bfloat16, device="cuda").normal_()
    grd = lambda n: torch.empty(T, n, dtype=torch.bfloat16, device="cuda").normal_(std=1e-3)
    xa = [act(f), act(d), act(d), act(d)]
    dys = [grd(d), grd(f), grd(d), grd(3 * d)]
    outs = [torch.empty(x.shape[1], y.shape[1], dtype=torch.float32, device="cuda") for x, y in zip(xa, dys)]
    kms, _, _ = events_ms(lambda: kk.gemm_wgrad_grouped(xa, dys, outs), 20, 3, 3)
    res["roofline_kernel_alone"] = mfma_roofline(kfl_block, kms * 1e3, kernel=kname + ", the four products in one launch, alone",
                                                 us_per_launch=kms * 1e3, algorithmic_flops_per_launch=kfl_block)
    # the largest forward product of a block (x W1 with the GELU epilogue), alone
    A = torch.empty(T, d, dtype=torch.bfloat16, device="cuda").normal_()
    B = torch.empty(d, f, dtype=torch.bfloat16, device="cuda").normal_(std=0.02)
    bias = torch.zeros(f, dtype=torch.bfloat16, device="cuda")
    z = torch.empty(T, f, dtype=torch.bfloat16, device="cuda"); gl = torch.empty_like(z)
    kms, _, _ = events_ms(lambda: kk.gemm_bf16(A, 0, B, 1, T, f, d, kk.EPI_BF16_BIAS_GELU, z, out2=gl, bias=bias), 20, 3, 3)
    res["roofline_ffn1_alone"] = mfma_roofline(2.0 * T * d * f, kms * 1e3,
                                               kernel="gemm_dtl_kernel (x W1 + b1, GELU epilogue) M=%d N=%d K=%d" % (T, f, d),
                                               us_per_launch=kms * 1e3, algorithmic_flops_per_launch=2.0 * T * d * f)
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_stage(c, cpu_seconds)
    return res


def cpu_stage(c, budget_s):
    """The oracle's stage step (forward, backward with recomputed forward, update) on a BOUNDED
    sample of the workload: whole sequences of its shape through the first blocks of its stage
    (every block costs the same), sized to the time budget from the box's measured rates;
    tokens/s is scaled by blocks_run / blocks.  Once on all host cores (BLAS threads), once on one."""
    from oracle import stage as ostage
    from paper_2401_01728_amd.inputs import gen
    from threadpoolctl import threadpool_limits
    d, f, L, S = c["d"], c["f"], c["L"], c["S"]
    per = 4 * d * d + 2 * d * f + 9 * d + f
    seq_block_flops = 8.0 * S * (4 * d * d + 2 * d * f)      # forward + backward with recomputed forward

    def run(blocks, seqs, threads):
        w = gen.normal_f32(c["seed"], 0, blocks * per, 0.0, 0.02).astype(np.float64)
        n = seqs * S * d
        x = gen.bf16_bits_to_f32(gen.normal_bf16_bits(c["seed"], 1000, n)).astype(np.float64).reshape(seqs, S, d)
        dy = gen.bf16_bits_to_f32(gen.normal_bf16_bits(c["seed"], 2000, n, 0.0, 1e-3)).astype(np.float64).reshape(seqs, S, d)
        o = ostage.Stage("decoder", 0, c["eta"], w, n_blocks=blocks, d=d, h=c["h"], f=f)
        with threadpool_limits(limits=threads):
            t0 = time.perf_counter()
            o.forward(0, x); o.backward(0, dy)
            dt = time.perf_counter() - t0
        return {"value": seqs * S / dt * blocks / L, "unit": "tokens/s", "cores": threads, "kind": "oracle",
                "sample": "one oracle stage step (numpy fp64) on %d of the %d sequences of a microbatch through %d of "
                          "the %d blocks, %.1f s; tokens/s scaled by %d/%d" % (seqs, c["mb"], blocks, L, dt, blocks, L)}

    cores = host_cores()
    # sized from rates seen on the pool's hosts: ~300 GFLOP/s effective on all cores, ~25 on one
    units_all = max(1.0, budget_s * 0.6 * 300e9 / seq_block_flops)
    units_one = max(1.0, budget_s * 0.4 * 25e9 / seq_block_flops)
    pick = lambda u: (min(L, max(1, int(u))), 1) if u < L else (L, min(c["mb"], max(1, int(u / L))))
    b_all, s_all = pick(units_all)
    b_one, s_one = pick(units_one)
    res = run(b_all, s_all, cores)
    res["one_thread"] = run(b_one, s_one, 1)
    return res


# ---------------------------------------------------------------------------------------------
# cluster average
# ---------------------------------------------------------------------------------------------
def make_replicas(n, C, seed, spread=None):
    import torch
    from paper_2401_01728_amd.inputs import device
    shared = torch.empty(n, dtype=torch.float32, device="cuda")
    device.fill_normal_(shared, seed, 0, 0.0, 1.0 if spread is None else 0.02)
    reps = []
    for c in range(C):
        r = torch.empty(n, dtype=torch.float32, device="cuda")
        device.fill_normal_(r, seed, 1 + c, 0.0, 1.0 if spread is None else spread)
        r += shared
        reps.append(r)
    return reps


def bench_average(args, label, n, C, rings, seed, fused_grad, spread=None, cpu=True):
    """One replica set, every R in `rings`, reduce-only and write-back."""
    import torch
    import paper_2401_01728_amd as rv
    from paper_2401_01728_amd.inputs import device
    reps = make_replicas(n, C, seed, spread)
    grad = None
    if fused_grad:
        grad = torch.empty(n, dtype=torch.float32, device="cuda"); device.fill_normal_(grad, seed, 99, 0.0, 1e-3)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    if args.calib_copy:     # a plain copy of known size (n fp32 read + n fp32 written) to scale the HBM counters
        out.copy_(reps[0])
    eta = 1e-3
    gbytes = 4 * n if fused_grad else 0
    kernel = "average_kernel<%d,%s>" % (C, "true" if fused_grad else "false")
    runs = {}
    for R in rings:
        for mode in ("reduce_only", "write_back"):
            if mode == "write_back" and args.no_write_back:
                continue
            wb = mode == "write_back"
            fn = lambda: rv.cluster_average(reps, R, mean_out=None if wb else out, write_back=wb, grad=grad,
                                            grad_replica=0, eta=eta)
            ms, _, per = events_ms(fn, max(args.avg_calls, 1), 2, args.reps)
            nbytes = (2 * C if wb else C + 1) * 4 * n + gbytes
            key = "%s: N=%d C=%d R=%d %s" % (label, n, C, R, mode)
            runs["R%d_%s" % (R, mode)] = {"ms_per_call": ms, "ms_per_call_reps": per,
                                          "roofline": hbm_roofline(nbytes, ms, kernel, key)}
    res = {"workload": "%s: N=%d fp32, C=%d replicas%s" % (label, n, C, ", SGD step of one replica folded in" if fused_grad else ""),
           "runs": runs}
    del reps, out, grad
    torch.cuda.empty_cache()
    if cpu and not args.no_cpu:
        res["cpu_baseline"] = cpu_average(C, rings[0], eta, seed, fused_grad)
    return res


def cpu_average(C, R, eta, seed, fused_grad):
    """oracle.average.direct_mean (fp64 definition) and the round-by-round ring algorithm on a
    bounded sample; numpy's element-wise kernels are single-threaded, so the all-cores figure is
    the one-thread figure."""
    from oracle import average
    from paper_2401_01728_amd.inputs import gen
    n = 2_000_000
    o = gen.normal_f32(seed, 0, n)
    xs = [(o + gen.normal_f32(seed, 1 + c, n)).astype(np.float32) for c in range(C)]
    g = gen.normal_f32(seed, 99, n, std=1e-3) if fused_grad else None
    nbytes = (C + 1 + (1 if fused_grad else 0)) * 4 * n
    t0 = time.perf_counter(); reps = 0
    while time.perf_counter() - t0 < 2.0:
        average.direct_mean(xs, g, 0, eta); reps += 1
    dt = (time.perf_counter() - t0) / reps
    t0 = time.perf_counter()
    average.multi_ring_allreduce(xs, R, g, 0, eta)
    dt_ring = time.perf_counter() - t0
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "oracle.average.direct_mean (fp64) on N=%d, C=%d, %d calls; numpy element-wise code is "
                      "single-threaded: one thread = all cores" % (n, C, reps),
            "ring_algorithm": {"value": nbytes / dt_ring / 1e9, "unit": "GB/s", "cores": 1,
                               "sample": "oracle.average.multi_ring_allreduce (2(C-1) rounds with message copies) "
                                         "on N=%d, C=%d, R=%d, one call, %.1f s" % (n, C, R, dt_ring)}}


# ---------------------------------------------------------------------------------------------
# delayed update alone
# ---------------------------------------------------------------------------------------------
def bench_update(args):
    import torch
    import paper_2401_01728_amd as rv
    from paper_2401_01728_amd.inputs import device
    n = int(args.n or n_params(DECODER_CFG["stage3"]))
    w = device.fill_normal_(torch.empty(n, dtype=torch.float32, device="cuda"), 3, 0, 0.0, 0.02)
    g = device.fill_normal_(torch.empty(n, dtype=torch.float32, device="cuda"), 3, 1, 0.0, 1e-3)
    v16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    if args.calib_copy:
        g.copy_(w)
    ms, _, per = events_ms(lambda: rv.block_update(w, g, 1e-3, bf16_out=v16), max(args.avg_calls, 1), 3, args.reps)
    res = {"workload": "update: w <- w - eta g with the bf16 weight version, %d parameters (config 3's stage)" % n,
           "ms_per_call": ms, "ms_per_call_reps": per,
           "roofline": hbm_roofline(14 * n, ms, "update_kernel<1>", "update: n=%d" % n)}
    ms32, _, _ = events_ms(lambda: rv.block_update(w, g, 1e-3), max(args.avg_calls, 1), 3, args.reps)
    res["fp32_only"] = {"ms_per_call": ms32, "roofline": hbm_roofline(12 * n, ms32, "update_kernel<0>")}
    del w, g, v16
    torch.cuda.empty_cache()
    if not args.no_cpu:
        from paper_2401_01728_amd.inputs import gen
        m = 4_000_000
        wh = gen.normal_f32(3, 0, m, 0.0, 0.02).astype(np.float64); gh = gen.normal_f32(3, 1, m, 0.0, 1e-3).astype(np.float64)
        t0 = time.perf_counter(); reps = 0
        while time.perf_counter() - t0 < 2.0:
            wh = wh - 1e-3 * gh; reps += 1            # Eq. 2 as oracle/stage.py applies it
        dt = (time.perf_counter() - t0) / reps
        res["cpu_baseline"] = {"value": 14 * m / dt / 1e9, "unit": "GB/s (at the GPU's 14 B/param)", "cores": 1, "kind": "oracle",
                               "sample": "the oracle's update line w - eta*g (numpy fp64) on %d parameters, %d calls" % (m, reps)}
    return res


# ---------------------------------------------------------------------------------------------
# config 1: two chained fp32 MLP stages
# ---------------------------------------------------------------------------------------------
def bench_mlp1(args):
    import torch
    import paper_2401_01728_amd as rv
    from paper_2401_01728_amd.inputs import device
    dims, mb, eta = [64, 128, 64], 8, 0.01
    s0 = rv.Stage.mlp(dims, mb, 1, eta); s1 = rv.Stage.mlp(dims, mb, 0, eta)
    for s, seed in ((s0, 1), (s1, 2)):
        w = torch.empty(s.num_params, dtype=torch.float32, device="cuda")
        device.fill_uniform_(w, seed, 0, -0.2, 0.2)
        s.set_params(w)
    x = device.fill_normal_(torch.empty(mb, 64, dtype=torch.float32, device="cuda"), 1, 100)
    dy = device.fill_normal_(torch.empty(mb, 64, dtype=torch.float32, device="cuda"), 1, 200, 0.0, 1e-2)
    h = torch.empty(mb, 64, device="cuda"); y = torch.empty(mb, 64, device="cuda")
    dh = torch.empty(mb, 64, device="cuda"); dx = torch.empty(mb, 64, device="cuda")
    state = {"t": 0}
    s0.forward(0, x, h)                      # stage 0 runs one microbatch ahead (tau = 1)
    s1.forward(0, h, y); s1.backward(0, dy, dh)
    state["t"] = 1

    def step():                              # one microbatch through both peers, both directions
        t = state["t"]
        s0.forward(t, x, h)
        s0.backward(t - 1, dh, dx)
        s1.forward(t, h, y)
        s1.backward(t, dy, dh)
        state["t"] = t + 1

    ms, wall, per = events_ms(step, max(args.steps, 50), 10, args.reps)
    res = {"workload": "mlp1: two chained fp32 MLP stages 64-128-64, microbatch 8, tau = 1 then 0 (launch bound)",
           "value": mb / (ms * 1e-3), "unit": "samples/s", "ms_per_microbatch": ms, "wall_ms_per_microbatch": wall}
    if not args.no_cpu:
        from oracle import stage as ostage
        rng = np.random.default_rng(1)
        P = 64 * 128 + 128 + 128 * 64 + 64
        w0, w1 = rng.uniform(-0.2, 0.2, P), rng.uniform(-0.2, 0.2, P)
        xh = rng.normal(size=(mb, 64)); dyh = rng.normal(size=(mb, 64)) * 1e-2
        t0 = time.perf_counter(); n = 0
        while time.perf_counter() - t0 < 2.0:
            # 16 microbatches per run, as the configuration has (the same input every time: a longer
            # run on it would drift to overflow)
            o0 = ostage.Stage("mlp", 1, eta, w0, dims=dims); o1 = ostage.Stage("mlp", 0, eta, w1, dims=dims)
            hh = o0.forward(0, xh); o1.forward(0, hh); dhh = o1.backward(0, dyh)
            for t in range(1, 16):
                hh = o0.forward(t, xh); o0.backward(t - 1, dhh); o1.forward(t, hh); dhh = o1.backward(t, dyh)
            n += 16
        res["cpu_baseline"] = {"value": mb * n / (time.perf_counter() - t0), "unit": "samples/s", "cores": 1, "kind": "oracle",
                               "sample": "%d microbatches through the oracle's two stages (numpy fp64)" % n}
    return res


def bench_gemm(args):
    """One matrix product through its per-kernel entry point (automatic tile choice)."""
    import torch
    from paper_2401_01728_amd import kernels as kk
    M, N, K = [int(v) for v in args.shape.split(",")]
    akm, bkm, epi = {"fwd": (0, 1, kk.EPI_BF16_BIAS), "dgrad": (0, 0, kk.EPI_BF16), "wgrad": (1, 1, kk.EPI_F32)}[args.layout]

    def operand(r, c, std):
        t = torch.empty(r, c, dtype=torch.bfloat16, device="cuda")
        return {"normal": lambda: t.normal_(std=std), "zeros": t.zero_, "ones": lambda: t.fill_(1.0)}[args.operands]()
    # --sets > 1: cycle through that many operand/result sets, so a launch does not find its
    # operands in the last-level cache from the launch before
    sets = [(operand(K, M, 1.0) if akm else operand(M, K, 1.0), operand(K, N, 0.02) if bkm else operand(N, K, 0.02),
             torch.empty(M, N, dtype=torch.float32 if epi == kk.EPI_F32 else torch.bfloat16, device="cuda"))
            for _ in range(max(args.sets, 1))]
    bias = torch.zeros(N, dtype=torch.bfloat16, device="cuda")
    turn = {"i": 0}

    def one():
        A, B, out = sets[turn["i"] % len(sets)]
        turn["i"] += 1
        kk.gemm_bf16(A, akm, B, bkm, M, N, K, epi, out, bias=bias)
    ms, _, _ = events_ms(one, args.steps, args.warmup, args.reps)
    tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
    return {"metric": "bf16 matrix product TFLOP/s", "value": tf, "unit": "TFLOP/s", "ms_per_step": ms, "dtype": "bf16",
            "config": {"workload": "gemm: M=%d N=%d K=%d %s, operands %s" % (M, N, K, args.layout, args.operands)},
            "roofline": mfma_roofline(2.0 * M * N * K, ms * 1e3, kernel="gemm_dtl_kernel", traffic=None,
                                      algorithmic_flops_per_launch=2.0 * M * N * K)}


def avg_job(args, name):
    if name == "avg4":
        rings = [int(r) for r in args.rings.split(",")]
        return bench_average(args, "avg4", int(args.n or 1_000_000_000), 16, rings, 4, True)
    c = DECODER_CFG["stage" + name[3:]]
    return bench_average(args, name, int(args.n or n_params(c)), c["C"], [c["R"]], c["seed"], False, spread=0.002)


def as_headline(sub, metric, value, unit, ms, dtype, workload, roofline):
    res = {"metric": metric, "value": value, "unit": unit, "ms_per_step": ms, "dtype": dtype,
           "config": {"workload": workload}, "roofline": roofline}
    res["detail"] = sub
    if "cpu_baseline" in sub:
        res["cpu_baseline"] = sub["cpu_baseline"]
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--reps", type=int, default=5, help="repetitions of the timed region; the median is reported")
    ap.add_argument("--workload", default=None)
    ap.add_argument("--rings", default="1,2,4,8", help="avg4: comma-separated ring counts")
    ap.add_argument("--avg-calls", type=int, default=20, help="calls per repetition of the average / update workloads")
    ap.add_argument("--n", type=float, default=None)
    ap.add_argument("--shape", default="8192,8192,8192", help="gemm: M,N,K")
    ap.add_argument("--layout", default="dgrad", choices=["fwd", "dgrad", "wgrad"])
    ap.add_argument("--sets", type=int, default=1, help="gemm: operand sets cycled through (more than the cache holds: cold operands)")
    ap.add_argument("--operands", default="normal", choices=["normal", "zeros", "ones"])
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--cold", action="store_true", help="stage workloads: time right after --warmup steps (no wait for the steady state)")
    ap.add_argument("--no-write-back", action="store_true")
    ap.add_argument("--step-only", action="store_true",
                    help="stage workloads: the stage steps only, no kernels launched alone afterwards (counter runs)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="average / update: also run one plain 4*n-byte copy (counter calibration)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="issue forward and backward as two calls on one stream (for per-kernel profiles)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr); sys.exit(2)
    from paper_2401_01728_amd import _lib
    _lib.lib()                                              # fail loudly if the HIP library is missing
    wl = args.workload
    if wl is None:
        # the whole measurement: headline on the largest stage, everything else nested
        res = bench_stage(args, "stage5", cpu_seconds=24.0)
        also = {}
        for name in ("stage3", "stage2"):
            also[name] = bench_stage(args, name, cpu_seconds=8.0)
        for name in ("avg4", "avg3", "avg5", "avg2"):
            also[name] = avg_job(args, name)
        also["update"] = bench_update(args)
        also["mlp1"] = bench_mlp1(args)
        res["also"] = also
    elif wl in DECODER_CFG:
        res = bench_stage(args, wl)
    elif wl == "gemm":
        res = bench_gemm(args)
    elif wl in ("avg4", "avg2", "avg3", "avg5"):
        sub = avg_job(args, wl)
        first = next(iter(sub["runs"].values()))
        res = as_headline(sub, "replica-average HBM GB/s (ring-partitioned mean of C replicas)", first["roofline"]["achieved"],
                          "GB/s", first["ms_per_call"], "f32", sub["workload"], first["roofline"])
    elif wl == "update":
        sub = bench_update(args)
        res = as_headline(sub, "delayed SGD update HBM GB/s", sub["roofline"]["achieved"], "GB/s", sub["ms_per_call"], "f32",
                          sub["workload"], sub["roofline"])
    elif wl == "mlp1":
        sub = bench_mlp1(args)
        res = as_headline(sub, "stage samples/s (two chained MLP stages)", sub["value"], "samples/s", sub["ms_per_microbatch"],
                          "f32", sub["workload"], None)
    else:
        print("bench.py: unknown workload %r" % wl, file=sys.stderr); sys.exit(2)
    res.update({"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "reps": args.reps, "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "data": "synthetic"})
    print(json.dumps(res))


if __name__ == "__main__":
    main()
