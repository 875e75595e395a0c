#!/usr/bin/env python3
"""Benchmark of the hot path on ONE MI355X.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Workloads (synthetic, seeded: activations N(0,1) and upstream gradients N(0,1e-3) rounded to bf16,
parameters N(0,0.02) with LayerNorm gains 1+N(0,0.02); replicas x_c = o + n_c with o, n_c ~ N(0,1)):
  stage2  (default) the middle transformer-decoder stage: 4 pre-LN blocks, d_model 1024,
          16 heads, FFN 4096, seq 512, microbatch 8, tau 2.  A step is the steady-state
          stage step: forward(t), backward(t - tau), delayed SGD update.  tokens/s.
  stage3 / stage5   the larger decoder stages, same step.
  gemm    one bf16 matrix product alone (--shape M,N,K, --layout fwd|dgrad|wgrad, --operands
          normal|zeros|ones): the kernel under the stage step, for counter runs.  TFLOP/s.
  avg4    the averaging-dominated case: 1e9 fp32 elements, C = 16 replicas in HBM, ring
          partitioned mean with one replica's SGD step folded in; a step is one call.
The oracle (CPU fp64) is timed beside it on a bounded sample ("cpu_baseline").
"""
import argparse
import json
import os
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


def events_ms(fn, steps, warmup):
    """Times `steps` calls of fn on torch's current stream with HIP events."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall / steps


def decoder_flops_per_token(c):
    gemm = 6 * c["L"] * (4 * c["d"] ** 2 + 2 * c["d"] * c["f"])
    attn = 6 * c["S"] * c["d"] * c["L"]
    return gemm + attn


def decoder_params(seed, c, device_fill=True):
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


def bench_avg4(args):
    import torch
    import paper_2401_01728_amd as rv
    from paper_2401_01728_amd.inputs import device
    n, C, eta, seed = int(args.n or 1_000_000_000), 16, 1e-3, 4
    R = args.rings
    shared = torch.empty(n, dtype=torch.float32, device="cuda")
    device.fill_normal_(shared, seed, 0)
    reps = []
    for c in range(C):
        r = torch.empty(n, dtype=torch.float32, device="cuda")
        device.fill_normal_(r, seed, 1 + c)
        r += shared
        reps.append(r)
    del shared
    grad = torch.empty(n, dtype=torch.float32, device="cuda"); device.fill_normal_(grad, seed, 99, 0.0, 1e-3)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    fn = lambda: rv.cluster_average(reps, R, mean_out=out, grad=grad, grad_replica=0, eta=eta)
    if args.calib_copy:     # a plain copy of known size (n fp32 read + n fp32 written) to scale the HBM counters
        out.copy_(grad)
    ms, wall_ms = events_ms(fn, args.steps, args.warmup)
    alg_bytes = (C + 2) * 4 * n
    gbs = alg_bytes / (ms * 1e-3) / 1e9
    res = {"metric": "replica-average HBM GB/s (ring-partitioned mean of C replicas + folded SGD step)",
           "value": gbs, "unit": "GB/s", "ms_per_step": ms, "dtype": "f32",
           "config": {"workload": "avg4: N=%d fp32, C=16, R=%d, fused grad" % (n, R)},
           "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": gbs / HBM_PEAK_GBS,
                        # counter runs recorded in profiles/avg4_average_kernel.md (default N, R = 4 only)
                        "traffic": 72.0e9 if (n == 1_000_000_000 and R == 4) else None,
                        "kernel": "average_kernel<16,true>",
                        "algorithmic_bytes_per_launch": alg_bytes}}
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_average(C, R, eta, seed)
    return res


def cpu_average(C, R, eta, seed):
    from oracle import average
    from paper_2401_01728_amd.inputs import gen
    n = 4_000_000
    o = gen.normal_f32(seed, 0, n)
    xs = [(o + gen.normal_f32(seed, 1 + c, n)).astype(np.float32) for c in range(C)]
    g = gen.normal_f32(seed, 99, n, std=1e-3)
    t0 = time.perf_counter(); reps = 0
    while time.perf_counter() - t0 < 10.0:
        average.direct_mean(xs, g, 0, eta); reps += 1
    dt = (time.perf_counter() - t0) / reps
    return {"value": (C + 2) * 4 * n / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "oracle.average.direct_mean (fp64) on N=%d, C=%d, %d calls" % (n, C, reps)}


def bench_gemm(args):
    """One matrix product through its per-kernel entry point (automatic tile choice)."""
    import torch
    from paper_2401_01728_amd import kernels as kk
    M, N, K = [int(v) for v in args.shape.split(",")]
    akm, bkm, epi = {"fwd": (0, 1, kk.EPI_BF16_BIAS), "dgrad": (0, 0, kk.EPI_BF16), "wgrad": (1, 1, kk.EPI_F32)}[args.layout]

    def operand(r, c, std):
        t = torch.empty(r, c, dtype=torch.bfloat16, device="cuda")
        return {"normal": lambda: t.normal_(std=std), "zeros": t.zero_, "ones": lambda: t.fill_(1.0)}[args.operands]()
    A = operand(K, M, 1.0) if akm else operand(M, K, 1.0)
    B = operand(K, N, 0.02) if bkm else operand(N, K, 0.02)
    out = torch.empty(M, N, dtype=torch.float32 if epi == kk.EPI_F32 else torch.bfloat16, device="cuda")
    bias = torch.zeros(N, dtype=torch.bfloat16, device="cuda")
    ms, _ = events_ms(lambda: kk.gemm_bf16(A, akm, B, bkm, M, N, K, epi, out, bias=bias), args.steps, args.warmup)
    tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
    return {"metric": "bf16 matrix product TFLOP/s", "value": tf, "unit": "TFLOP/s", "ms_per_step": ms, "dtype": "bf16",
            "config": {"workload": "gemm: M=%d N=%d K=%d %s, operands %s" % (M, N, K, args.layout, args.operands)},
            "roofline": {"bound": "mfma", "achieved": tf, "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": tf / BF16_PEAK_TFLOPS, "traffic": None, "kernel": "gemm_dtl_kernel",
                         "algorithmic_flops_per_launch": 2.0 * M * N * K}}


def bench_stage(args, name):
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

    ms, wall_ms = events_ms(step, args.steps, args.warmup)
    tokens = c["mb"] * c["S"]
    flops = decoder_flops_per_token(c) * tokens
    tflops = flops / (ms * 1e-3) / 1e12
    res = {"metric": "stage tokens/s (fwd+bwd+delayed SGD)", "value": tokens / (ms * 1e-3), "unit": "tokens/s",
           "ms_per_step": ms, "dtype": "bf16",
           "config": {"workload": "%s: %d pre-LN decoder blocks d=%d h=%d ffn=%d seq=%d microbatch=%d tau=%d" % (
               name, c["L"], c["d"], c["h"], c["f"], c["S"], c["mb"], c["tau"]), "tokens_per_step": tokens},
           "wall_ms_per_step": wall_ms}
    # The dominant kernel (largest share of the step in the rocprofv3 trace): the grouped
    # weight-gradient launch of one block, dW2 | dW1 | dWo | dWqkv over the microbatch's tokens.
    # Launched alone through its per-kernel entry point on torch's current stream and timed with
    # HIP events; operands have the step's value distributions.
    from paper_2401_01728_amd import kernels as kk
    T, d, f = tokens, c["d"], c["f"]
    act = lambda n: torch.empty(T, n, dtype=torch.bfloat16, device="cuda").normal_()
    grd = lambda n: torch.empty(T, n, dtype=torch.bfloat16, device="cuda").normal_(std=1e-3)
    xs = [act(f), act(d), act(d), act(d)]
    dys = [grd(d), grd(f), grd(d), grd(3 * d)]
    outs = [torch.empty(x.shape[1], y.shape[1], dtype=torch.float32, device="cuda") for x, y in zip(xs, dys)]
    kms, _ = events_ms(lambda: kk.gemm_wgrad_grouped(xs, dys, outs), 20, 3)
    kfl = 2.0 * T * (2 * d * f + 4 * d * d)
    # bytes per launch through the L2s' fabric ports, from the rocprofv3 counter runs recorded in
    # profiles/stage2_stage_step_kernel_trace.md (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the factors a
    # plain copy of known size gives); measured for the config-2 shapes only
    traffic = 268.7e6 if name == "stage2" else None
    res["roofline"] = {"bound": "mfma", "achieved": kfl / (kms * 1e-3) / 1e12, "peak": BF16_PEAK_TFLOPS,
                       "unit": "TFLOP/s", "frac": kfl / (kms * 1e-3) / 1e12 / BF16_PEAK_TFLOPS, "traffic": traffic,
                       "kernel": "gemm_dtl_grouped_wgrad_kernel (dW2, dW1, dWo, dWqkv of one block, K=%d tokens)" % T,
                       "us_per_launch": kms * 1e3, "algorithmic_flops_per_launch": kfl}
    # the whole step against the same peak (all kernels, three streams)
    res["roofline_step"] = {"bound": "mfma", "achieved": tflops, "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                            "frac": tflops / BF16_PEAK_TFLOPS, "algorithmic_flops_per_step": flops}
    # the largest forward product of a block (x W1 with the GELU epilogue), alone
    A = torch.empty(T, d, dtype=torch.bfloat16, device="cuda").normal_()
    B = torch.empty(d, f, dtype=torch.bfloat16, device="cuda").normal_(std=0.02)
    bias = torch.zeros(f, dtype=torch.bfloat16, device="cuda")
    z = torch.empty(T, f, dtype=torch.bfloat16, device="cuda"); gl = torch.empty_like(z)
    kms, _ = events_ms(lambda: kk.gemm_bf16(A, 0, B, 1, T, f, d, kk.EPI_BF16_BIAS_GELU, z, out2=gl, bias=bias), 20, 3)
    kfl = 2.0 * T * d * f
    res["roofline_ffn1"] = {"kernel": "gemm_dtl_kernel (x W1 + b1, GELU epilogue) M=%d N=%d K=%d" % (T, f, d),
                            "bound": "mfma", "achieved": kfl / (kms * 1e-3) / 1e12, "peak": BF16_PEAK_TFLOPS,
                            "unit": "TFLOP/s", "frac": kfl / (kms * 1e-3) / 1e12 / BF16_PEAK_TFLOPS,
                            "us_per_launch": kms * 1e3, "algorithmic_flops_per_launch": kfl}
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_stage(c)
    return res


def cpu_stage(c):
    """The oracle's stage step (forward, backward with recomputed forward, update) on a BOUNDED
    sample: a few whole sequences of the workload's shape (the full microbatch where that is
    about ten seconds of work)."""
    from oracle import stage as ostage
    from paper_2401_01728_amd.inputs import gen
    d, f, L, S = c["d"], c["f"], c["L"], c["S"]
    mb = c["mb"] if d <= 1024 else min(2, c["mb"])
    P = L * (4 * d * d + 2 * d * f + 9 * d + f)
    w = gen.normal_f32(c["seed"], 0, P, 0.0, 0.02).astype(np.float64)
    n = mb * S * d
    x = gen.bf16_bits_to_f32(gen.normal_bf16_bits(c["seed"], 1000, n)).astype(np.float64).reshape(mb, S, d)
    dy = gen.bf16_bits_to_f32(gen.normal_bf16_bits(c["seed"], 2000, n, 0.0, 1e-3)).astype(np.float64).reshape(mb, S, d)
    o = ostage.Stage("decoder", 0, c["eta"], w, n_blocks=L, d=d, h=c["h"], f=f)
    reps = 2 if d <= 1024 else 1
    t0 = time.perf_counter()
    for r in range(reps):
        o.forward(r, x); o.backward(r, dy)
    dt = time.perf_counter() - t0
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    return {"value": reps * mb * S / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "%d oracle stage step(s) (numpy fp64) on %d of the %d sequences of a microbatch, %.1f s"
                      % (reps, mb, c["mb"], dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default=None)
    ap.add_argument("--rings", type=int, default=4)
    ap.add_argument("--n", type=float, default=None)
    ap.add_argument("--shape", default="8192,8192,8192", help="gemm: M,N,K")
    ap.add_argument("--layout", default="dgrad", choices=["fwd", "dgrad", "wgrad"])
    ap.add_argument("--operands", default="normal", choices=["normal", "zeros", "ones"])
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--calib-copy", action="store_true", help="avg4: also run one plain 4*n-byte copy (counter calibration)")
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
    wl = args.workload or "stage2"
    res = bench_avg4(args) if wl == "avg4" else bench_gemm(args) if wl == "gemm" else bench_stage(args, wl)
    res.update({"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "data": "synthetic"})
    print(json.dumps(res))


if __name__ == "__main__":
    main()
