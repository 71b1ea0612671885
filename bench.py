#!/usr/bin/env python3
"""bench.py -- one GPU, the whole hot path on config 2 of the benchmark spec.

A "step" is one pass of the whole path over one batch of synthetic input: garble the LeNet-5-shaped
network (batch 16, 8-prime CRT base, 128-bit labels), encode the inputs, evaluate the garbled
network, decode.  Inputs, weights and every buffer are resident in HBM before the timed region.
Prints ONE JSON line (Measurement).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8, published
# vector issue rate of the simple 32-bit integer instructions (and, xor, add, shift right, three-input bit operation):
# 256 compute units x 4 SIMDs x 32 lanes x 2.4 GHz = 78.6 T lane-instructions/s, the same unit count that gives the
# published 157.3 TFLOP/s of fp32 FMA.  (Measured with a loop of independent v_add_u32: 70.7 T/s.  Shift left, byte
# permute, three-operand forms and all multiplies issue at half of that.)
ALU_PEAK_TOPS = 256 * 4 * 32 * 2.4e9 / 1e12

# Figures taken from the rocprofv3 --pmc runs of this same command (profiles/k_proj_garble_lenet_b16_pmc.txt):
# vector instructions per ciphertext row of k_proj_garble and of k_digits_garble / per gate of the evaluator's gate kernels, averaged over
# the launches of one config-2 step (SQ_INSTS_VALU * 64 lanes / rows), and the HBM bytes per row (FETCH_SIZE,
# WRITE_SIZE, scaled by what the same counters read for the 1 GiB copy issued in warm-up: 2.0 and 1.0).
PMC = dict(garble_valu_per_row=792.5, digits_valu_per_row=636.8, eval_valu_per_gate=625.1,
           garble_fetch_bytes_per_row=4.27, garble_write_bytes_per_row=29.83,
           digits_fetch_bytes_per_row=4.62, digits_write_bytes_per_row=21.47)


def gate_counts(net, k, n_digits):
    """projection-gate tables per step (the garbler builds each once, the evaluator hashes once per table)"""
    sign = k * n_digits + n_digits
    gates = 0
    for L in net["layers"]:
        if L["kind"] == "relu":
            gates += L["n"] * (sign + 3 * k)
        elif L["kind"] == "sign":
            gates += L["n"] * (sign + k)
        elif L["kind"] == "scale":
            gates += L["n"] * L["repeat"] * ((k - 1) + (sign - n_digits))
    return gates * net["batch"]


def mac_counts(net, lam_sum):
    macs = 0
    for L in net["layers"]:
        if L["kind"] == "conv":
            macs += L["out_h"] * L["out_w"] * L["out_c"] * L["kh"] * L["kw"] * L["in_c"]
    return macs * net["batch"] * lam_sum


def cpu_baseline(net, seconds_target=12.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload: the ReLU +
    scale-by-2^6 activation pipeline (garble and evaluate) over `per_thread` values per thread."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    from oracle import capi

    cores = min(16, os.cpu_count() or 1)
    repeat = next(L["repeat"] for L in net["layers"] if L["kind"] == "scale")
    k, n = len(net["primes"]), len(net["digits"])
    per_value = (k * n + n + 3 * k) + repeat * ((k - 1) + (k - 1) * n + n)

    def work(t, count):
        orc = capi.Oracle(net["primes"], net["digits"], net["seed"], 0)
        g = np.random.default_rng(t)
        X = g.integers(0, orc.P, count)
        zero = [orc.input_labels(t * count, count, i) for i in range(k)]
        act = [orc.encode(i, X, zero[i]) for i in range(k)]
        r0, rt = orc.relu_garble(2, zero, elem_base=t * count)
        s0, st = orc.scale_garble(3, r0, repeat, elem_base=t * count)
        r = orc.relu_eval(2, act, rt, elem_base=t * count)
        orc.scale_eval(3, r, st, repeat, elem_base=t * count)
        return count

    t0 = time.time()
    work(0, 20)                                   # calibrate on one core
    per = (time.time() - t0) / 20
    count = max(20, int(seconds_target / per))
    t0 = time.time()
    with ThreadPoolExecutor(cores) as ex:
        done = sum(ex.map(lambda t: work(t, count), range(cores)))
    dt = time.time() - t0
    return dict(value=2 * done * per_value / dt, unit="projection gates/s (garble+eval)", cores=cores, kind="oracle",
                sample="ReLU + scale-by-2^%d pipeline of config 2 on %d values (%d per thread), garble + evaluate, %.1f s"
                       % (repeat, done, count, dt))


def kernel_line(pr, steps, bytes_per_unit_note=None):
    """per-kernel figures from the library's own HIP-event instrumentation (events recorded around every
    launch on the stream the kernel runs on)"""
    if not pr["ms"]:
        return None
    sec = pr["ms"] * 1e-3
    return dict(ms_per_step=pr["ms"] / steps, launches_per_step=pr["launches"] // steps,
                avg_launch_ms=pr["ms"] / max(pr["launches"], 1), units_per_s=pr["units"] / sec,
                gbytes_per_s=pr["bytes"] / sec / 1e9, units_per_launch=pr["units"] / max(pr["launches"], 1),
                bytes_per_launch=pr["bytes"] / max(pr["launches"], 1))


def read_profiles(ctx):
    return {name: ctx.profile_read(kind) for name, kind in (("garble", 0), ("eval", 1), ("linear", 2), ("garble_digits", 3))}


def micro_projection(torch, workloads, reps=2):
    """Config 3: 2^24 independent gates Z_p -> Z_q over the 12-prime base, grouped by (p, q)."""
    from paper_2302_06361_amd import Context, ProjectionBatch
    mb = workloads.proj_microbench(seed=3)
    ctx = Context(mb["primes"], mb["seed"], workloads.DIGITS[12])
    pb = ProjectionBatch(ctx, mb["pi"], mb["qi"])
    a_all = torch.as_tensor(mb["a"][pb.order].astype("int16")).to(ctx.device)
    gen = torch.Generator(device=ctx.device)
    gen.manual_seed(3)
    for G in pb.groups:
        i, p, n = G["pi"], ctx.primes[G["pi"]], G["count"]
        t = G["in0"].tensors[i]
        t.copy_(torch.randint(0, p, t.shape, dtype=torch.uint8, device=ctx.device, generator=gen))
        R = torch.zeros(t.shape[0] * 16, dtype=torch.int16)
        R[:ctx.lam(p)] = torch.as_tensor(ctx.offset(p).astype("int16"))
        a = a_all[G["start"]:G["start"] + n].view(1, n, 1)
        G["act"].tensors[i].copy_(((t.to(torch.int16) + a * R.to(ctx.device).view(-1, 1, 16)) % p).to(torch.uint8))
        G["phi"].copy_(torch.randint(0, ctx.primes[G["qi"]], G["phi"].shape, dtype=torch.uint8, device=ctx.device, generator=gen))
    pb.garble(); pb.evaluate()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record()
    for _ in range(reps):
        pb.garble()
    ev[1].record()
    for _ in range(reps):
        pb.evaluate()
    ev[2].record()
    torch.cuda.synchronize()
    gms, ems = ev[0].elapsed_time(ev[1]) / reps, ev[1].elapsed_time(ev[2]) / reps
    # the same passes again with the library's per-launch events, for the per-kernel figures (not timed above)
    ctx.profile_enable(True)
    read_profiles(ctx)
    for _ in range(reps):
        pb.garble(serial=True)
    for _ in range(reps):
        pb.evaluate(serial=True)
    torch.cuda.synchronize()
    ctx.profile_enable(False)
    pr = read_profiles(ctx)
    out = dict(workload="config 3: 2^24 gates Z_p->Z_q, (p,q) uniform over the 12-prime base, 144 grouped launches on 4 streams",
               gates=pb.n, rows=pb.rows, table_bytes=pb.table_bytes,
               garble_ms=gms, eval_ms=ems, garble_gates_per_s=pb.n / (gms * 1e-3), eval_gates_per_s=pb.n / (ems * 1e-3),
               garble_rows_per_s=pb.rows / (gms * 1e-3), garble_table_GBps=pb.table_bytes / (gms * 1e-3) / 1e9,
               garble_frac_of_hbm=pb.table_bytes / (gms * 1e-3) / 1e9 / HBM_PEAK_GBS,
               kernels=dict(k_proj_garble=kernel_line(pr["garble"], reps), k_proj_eval=kernel_line(pr["eval"], reps)))
    del pb
    ctx.close()
    torch.cuda.empty_cache()
    return out


def micro_contraction(torch, workloads, reps=5):
    """Config 4: dense 4096 x 4096 on label tensors at batch 128, every prime of the 12-prime base."""
    from paper_2302_06361_amd import DENSE, Context, Labels, Layer
    mb = workloads.gemm_microbench(seed=4)
    ctx = Context(mb["primes"], mb["seed"], workloads.DIGITS[12])
    M, K, Bn = mb["M"], mb["K"], mb["batch"]
    wp = ctx.weights_prepare(mb["W"])
    x, y = Labels(ctx, Bn * K), Labels(ctx, Bn * M)
    gen = torch.Generator(device=ctx.device)
    gen.manual_seed(4)
    for i, p in enumerate(ctx.primes):
        t = x.tensors[i]
        t.copy_(torch.randint(0, p, t.shape, dtype=torch.uint8, device=ctx.device, generator=gen))
    lay = Layer(DENSE, 1, Bn, in_c=K, out_c=M, weights=wp)
    lam = sum(ctx.lam(p) for p in ctx.primes)
    macs = M * K * Bn * lam
    for _ in range(2):
        ctx.eval_layer(lay, x, None, y)
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    read_profiles(ctx)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        ctx.eval_layer(lay, x, None, y)
    e1.record()
    torch.cuda.synchronize()
    ctx.profile_enable(False)
    pr = read_profiles(ctx)["linear"]
    ms = e0.elapsed_time(e1) / reps
    kms = pr["ms"] / max(pr["launches"], 1)
    out = dict(workload="config 4: dense 4096x4096, weights in [-64,63], batch 128, 12 primes (%d label digits per value)" % lam,
               ms=ms, label_mac_per_s=macs / (ms * 1e-3),
               roofline=dict(bound="mfma", kernel="k_dense_mfma", unit="TOP/s", peak=INT8_MFMA_PEAK_TOPS,
                             achieved=2 * macs / (kms * 1e-3) / 1e12, frac=2 * macs / (kms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS,
                             avg_launch_ms=kms, ops_per_launch=2 * macs,
                             # HBM bytes per launch from the rocprofv3 --pmc runs in profiles/k_dense_mfma_dense4096_b128_pmc.txt
                             traffic=1.965e9 + 0.327e9, algorithmic_bytes_per_launch=float(M) * K * len(ctx.primes) + 2.0 * Bn * (M + K) / 2 * 16 * sum((ctx.lam(p) + 15) // 16 for p in ctx.primes)))
    ctx.close()
    torch.cuda.empty_cache()
    return out


def micro_vgg(torch, workloads, images=1, reps=2):
    """Config 5, streamed: garble + evaluate layer by layer, `images` images of the batch of 64 at a time."""
    from paper_2302_06361_amd import Context, StreamedNetwork
    net = workloads.vgg(seed=5, batch=64)
    ctx = Context(net["primes"], net["seed"], net["digits"])
    g = StreamedNetwork(ctx, net, batch=images)
    x = torch.as_tensor(net["x"][:images * net["n_in"]]).to(ctx.device)
    k, n = ctx.k, len(ctx.digits)
    lam_sum = sum(ctx.lam(p) for p in ctx.primes)
    sub = dict(net, batch=images)
    gates, macs = gate_counts(sub, k, n), mac_counts(sub, lam_sum)
    g.run(x)
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    read_profiles(ctx)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.run(x)
    e1.record()
    torch.cuda.synchronize()
    ctx.profile_enable(False)
    pr = read_profiles(ctx)
    ms = e0.elapsed_time(e1) / reps
    out = dict(workload="config 5: VGG shape (12 primes, scale 2^5), %d image(s) of the batch of 64 streamed layer by layer, "
                        "garble + evaluate + decode" % images,
               images=images, ms=ms, ms_per_image=ms / images, outputs_valid=bool(g.valid.all().item()),
               table_bytes_per_image=g.table_bytes // images, gates_per_image=gates // images,
               gates_per_s=2 * gates / (ms * 1e-3), label_macs_per_image=2 * macs // images,
               kernels=dict(k_proj_garble=kernel_line(pr["garble"], reps), k_digits_garble=kernel_line(pr["garble_digits"], reps),
                            eval_kernels=kernel_line(pr["eval"], reps), linear=kernel_line(pr["linear"], reps)))
    ctx.close()
    torch.cuda.empty_cache()
    return out


def micro_paper_models(torch, workloads, reps=5):
    """The shapes of the paper's models A-F (Sec. Model architectures), batch 1, random weights: garbling time
    (offline in the paper) and evaluation time (its online figure, there including a modelled network cost)."""
    from paper_2302_06361_amd import Context, GarbledNetwork
    out = {}
    for name in "ABCDfF":
        net = workloads.paper_model(name, seed=6)
        ctx = Context(net["primes"], net["seed"], net["digits"])
        g = GarbledNetwork(ctx, net)
        x = torch.as_tensor(net["x"]).to(ctx.device)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        for r in range(reps + 1):
            if r == 1:
                torch.cuda.synchronize()
                ev[0].record()
            g.garble()
        ev[1].record()
        g.encode(x)
        for _ in range(reps):
            g.evaluate()
            g.decode()
        ev[2].record()
        torch.cuda.synchronize()
        out[name] = dict(primes=len(net["primes"]), relu_values=sum(L["n"] for L in net["layers"] if L["kind"] == "relu"),
                         table_bytes=g.table_bytes, garble_ms=ev[0].elapsed_time(ev[1]) / reps,
                         eval_ms=ev[1].elapsed_time(ev[2]) / reps, outputs_valid=bool(g.valid.all().item()))
        del g
        ctx.close()
        torch.cuda.empty_cache()
    return dict(workload="paper model shapes A-F, batch 1, random integer weights and biases", models=out,
                paper_online_ms_gpu=dict(A=10, B=32, C=16, D=42, f=1332, F=1443),
                note="the paper's figures (its Table of online runtimes, other hardware) include a modelled 1 Gbit/s transfer; context only")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--batch", type=int, default=16, help="batch elements of config 2 (16 = the config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-micro", action="store_true", help="skip the config-3 and config-4 microbenchmarks")
    ap.add_argument("--only", choices=["config3", "config4", "config5", "paper_models"], help="run one microbenchmark alone (for profiling); prints its JSON object")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build measures ONE GPU (every box has one); --gpus %d is not supported" % a.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    import workloads
    from paper_2302_06361_amd import Context, GarbledNetwork

    if a.only:
        fn = dict(config3=micro_projection, config4=micro_contraction, config5=micro_vgg, paper_models=micro_paper_models)[a.only]
        print(json.dumps(fn(torch, workloads)))
        return

    net = workloads.lenet(seed=2, batch=a.batch)
    ctx = Context(net["primes"], net["seed"], net["digits"])
    g = GarbledNetwork(ctx, net)
    x = torch.as_tensor(net["x"]).to(ctx.device)
    k, n = ctx.k, len(ctx.digits)
    lam_sum = sum(ctx.lam(p) for p in ctx.primes)
    gates = gate_counts(net, k, n)
    macs = mac_counts(net, lam_sum)

    # a plain copy of known size, for scaling the HBM counters of a rocprofv3 --pmc run of this command
    src = torch.empty(1 << 30, dtype=torch.uint8, device=ctx.device)
    dst = torch.empty_like(src)
    dst.copy_(src)
    del src, dst

    def step(ev=None):
        if ev:
            ev[0].record()
        g.garble()
        if ev:
            ev[1].record()
        g.encode(x)
        if ev:
            ev[2].record()
        g.evaluate()
        if ev:
            ev[3].record()
        g.decode()
        if ev:
            ev[4].record()

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(a.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(a.steps):
        step(evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    phase = [sum(e[i].elapsed_time(e[i + 1]) for e in evs) / a.steps for i in range(4)]   # ms: garble, encode, eval, decode
    ok = bool(g.valid.all().item())
    ms_step = wall * 1e3 / a.steps

    # the same steps again with an event pair around every kernel launch (the library's instrumentation,
    # on the launch stream): per-kernel durations for the roofline.  Not part of the timed region above.
    ctx.profile_enable(True)
    read_profiles(ctx)
    for s in range(a.steps):
        step()
    torch.cuda.synchronize()
    ctx.profile_enable(False)
    prof = read_profiles(ctx)

    kg, ke, kl, kd = (kernel_line(prof[n_], a.steps) for n_ in ("garble", "eval", "linear", "garble_digits"))

    def garble_roofline(kernel, kk, valu, traffic_per_row):
        r = dict(kernel=kernel, bound="alu", unit="Tlane-instr/s (32-bit integer vector instructions)", peak=ALU_PEAK_TOPS,
                 achieved=kk["units_per_s"] * valu / 1e12, ms_per_step=kk["ms_per_step"],
                 avg_launch_ms=kk["avg_launch_ms"], launches_per_step=kk["launches_per_step"],
                 rows_per_launch=kk["units_per_launch"], rows_per_s=kk["units_per_s"], lane_ops_per_row=valu,
                 hbm_algorithmic_GBps=kk["gbytes_per_s"], hbm_frac=kk["gbytes_per_s"] / HBM_PEAK_GBS,
                 algorithmic_bytes_per_launch=kk["bytes_per_launch"], traffic=traffic_per_row * kk["units_per_launch"])
        r["frac"] = r["achieved"] / ALU_PEAK_TOPS
        return r
    # the dominant kernel of the step: the general projection-gate garbler (carry chains, half gates, casts); the
    # digit gates of the sign gadgets run in the fused kernel, reported beside it
    roofline = garble_roofline("k_proj_garble", kg, PMC["garble_valu_per_row"],
                               PMC["garble_fetch_bytes_per_row"] + PMC["garble_write_bytes_per_row"])
    roofline_digits = garble_roofline("k_digits_garble", kd, PMC["digits_valu_per_row"],
                                      PMC["digits_fetch_bytes_per_row"] + PMC["digits_write_bytes_per_row"]) if kd else None
    ev_valu = PMC["eval_valu_per_gate"]
    roofline_eval = dict(kernel="k_digits_eval + k_chain_eval + k_cast_halve + k_proj_eval", bound="alu", unit=roofline["unit"], peak=ALU_PEAK_TOPS,
                         achieved=ke["units_per_s"] * ev_valu / 1e12 if ev_valu else None,
                         avg_launch_ms=ke["avg_launch_ms"], launches_per_step=ke["launches_per_step"],
                         gates_per_s=ke["units_per_s"], hbm_algorithmic_GBps=ke["gbytes_per_s"],
                         hbm_frac=ke["gbytes_per_s"] / HBM_PEAK_GBS)
    roofline_eval["frac"] = roofline_eval["achieved"] / ALU_PEAK_TOPS if roofline_eval["achieved"] else None

    out = dict(
        metric="label-MAC/s + projection gates/s (garble & eval); ms/inference, 1 GPU",
        value=2 * gates / (ms_step * 1e-3),
        unit="projection gates/s (garbled + evaluated, whole step: garble+encode+eval+decode)",
        n_gpus=1, steps=a.steps, warmup=a.warmup, ms_per_step=ms_step, higher_is_better=True, scaling="weak",
        vs_baseline=None, dtype="u8 digits, i32 accumulate", data="synthetic",
        config=dict(workload="config 2: LeNet-5 shape, batch %d, 8-prime CRT base, 128-bit labels (ceil rule), "
                             "ReLU + scale 2^6 after every conv/dense but the last" % a.batch,
                    batch=a.batch, primes=ctx.primes, sign_digits=ctx.digits, table_bytes=g.table_bytes),
        outputs_valid=ok,
        garble_gates_per_s=gates / (phase[0] * 1e-3),
        eval_gates_per_s=gates / (phase[2] * 1e-3),
        ms_per_inference=ms_step / a.batch,
        ms_per_inference_eval=phase[2] / a.batch,
        ms_per_inference_garble=phase[0] / a.batch,
        phase_ms=dict(garble=phase[0], encode=phase[1], eval=phase[2], decode=phase[3]),
        gates_per_step=gates, label_macs_per_step=2 * macs,
        roofline=roofline, roofline_digits_kernel=roofline_digits, roofline_eval_kernel=roofline_eval,
        linear_kernels_config2=dict(ms_per_step=kl["ms_per_step"], label_mac_per_s=kl["units_per_s"],
                                    note="config-2 linear layers are tiny (launch-bound); config 4 below is the contraction figure"),
    )
    del g
    ctx.close()
    torch.cuda.empty_cache()
    if not a.no_micro:
        out["config3_projection_gates"] = micro_projection(torch, workloads)
        out["config4_contraction"] = micro_contraction(torch, workloads)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(net)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
