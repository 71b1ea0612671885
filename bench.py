#!/usr/bin/env python3
"""bench.py -- one GPU, the whole hot path.

A "step" is one pass of the whole path over one batch of synthetic input on the second of the five benchmark
configurations, the one the metric is quoted on: garble the LeNet-5-shaped network (batch 16, 8-prime CRT base, 128-bit
labels), encode the inputs, evaluate the garbled network, decode.  Inputs, weights and every buffer are resident
in HBM before the timed region.  The other four configurations are measured after the timed steps and reported
in `configs` of the same JSON line (config 1: batch-1 latency; config 3: projection gates/s; config 4:
label-MAC/s; config 5: streamed over `--images` images of its batch of 64, never extrapolated).
Prints ONE JSON line.
"""
import argparse
import hashlib
import re
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

PMC_FILE = os.path.join(ROOT, "profiles", "gate_kernels_lenet_b16_pmc_per_unit.txt")
GATE_SOURCES = ["dash_core.h", "dash_bodies.h", "dash_tabs.h", "dash_launch.h", "dash_gates.hip", "dash_gates_digits.hip", "dash_gates_eval.hip",
                "dash_gates_digits_eval.hip", "dash_gates_cast.hip", "dash_layers.hip"]


def gate_source_hash():
    """identifies the gate-kernel sources a counter file was taken with: their code, without comments and blank space
    (a reworded comment does not make counters stale)"""
    h = hashlib.sha256()
    for name in GATE_SOURCES:
        text = open(os.path.join(ROOT, "paper_2302_06361_amd", "csrc", name), encoding="utf-8").read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
        text = re.sub(r"//[^\n]*", " ", text)
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:16]


def load_pmc():
    """Per-unit counter figures of the gate kernels (executed vector instructions per ciphertext row / per gate, HBM
    bytes per row) from the committed summary of the rocprofv3 --pmc runs of this same command: `key = value` lines.
    Returns (dict or None, note).  The file names the commit and the hash of the gate-kernel sources it was taken with;
    figures taken with other sources are flagged stale (and still printed: they are counters, not timings)."""
    if not os.path.exists(PMC_FILE):
        return None, "profiles/%s is missing: no executed-instruction or traffic figures" % os.path.basename(PMC_FILE)
    vals = {}
    for line in open(PMC_FILE):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = [t.strip() for t in line.split("=", 1)]
            try:
                vals[k] = float(v)
            except ValueError:
                vals[k] = v
    stale = vals.get("gate_source_hash") != gate_source_hash()
    return vals, "taken at commit %s%s" % (vals.get("commit", "?"), "; STALE: the gate-kernel sources have changed since" if stale else "")


# ---- algorithmic work of one hash, in 32-bit lane operations ---------------------------------------------------
# What the method needs on a 32-bit SIMD lane, however the kernels are written: AES 256 (160 table indices, two
# three-input xors per column and round, 16 for the last round, 4 for the feed-forward); label of value a: 4 per dword;
# compress: 3 per dword + 16 for the wide multiply-adds; base-q digits: 3 per digit + 132 for the long division of the
# 128-bit number; packed modular additions: 4 per dword.
def _lam_ceil(m):
    lam, v = 0, 1
    while v < (1 << 128):
        v *= m
        lam += 1
    return lam


AES_LANE_OPS = 160 + 72 + 4 + 16 + 4      # 160 table indices, 2 three-input xors per column and round (9 rounds), key, last round, feed-forward


def _compress_ops(m, lam):
    dw = (lam + 3) // 4
    return dw if m == 2 else 3 * dw + 16          # bits: one packing per dword; else 2 dot products + 1 fold per dword, 4 x 4 wide multiply-adds


def _decompress_ops(m, lam):
    dw = (lam + 3) // 4
    return 2 * dw if m == 2 else 3 * lam + 132    # bits: one spread per dword; else 3 per digit + the long division of the 128-bit number


def _modadd_ops(m, lam, count):
    dw = (lam + 3) // 4
    return count * dw * (1 if m == 2 else 4)      # packed modular addition of 4 digits: add, compare mask, and, subtract


def alg_ops_garble_row(p, q, lam_p, lam_q, short=False, share=1):
    """one ciphertext row: form the label of a, compress, AES, base-q digits, add payload (zero label + phi(a) R_q).
    share: gates that hash the same input label under different tweaks (the n digit gates of a residue): the label is
    formed and compressed once for all of them."""
    head = (_modadd_ops(p, lam_p, 1) + _compress_ops(p, lam_p)) / share
    if short:
        return head + AES_LANE_OPS + 24 + 4
    return head + AES_LANE_OPS + _decompress_ops(q, lam_q) + _modadd_ops(q, lam_q, 2)


def alg_ops_eval_gate(p, q, lam_p, lam_q, share=1):
    """one evaluated gate: compress, AES, base-q digits, subtract from the row"""
    return _compress_ops(p, lam_p) / share + AES_LANE_OPS + _decompress_ops(q, lam_q) + _modadd_ops(q, lam_q, 1)


def gadget_gates(primes, digits, kind, repeat=1):
    """(p, q, class) of every projection-gate table of one value of an activation layer; class: 'digits' (the fused digit
    kernels), 'gate' (general gate kernels), 'short' (one-digit rows of the half gate)"""
    k, n = len(primes), len(digits)
    m = [digits[0]] + [k * d for d in digits[1:]]

    def sign(first):
        out = [(primes[i], m[j], "digits") for i in range(first, k) for j in range(n)]
        out += [(m[j], m[j - 1], "gate") for j in range(1, n)] + [(m[0], 2, "gate")]
        return out
    if kind == "relu":
        out = sign(0)
        for p in primes:
            out += [(p, p, "gate"), (2, p, "gate"), (2, p, "short")]
        return out
    if kind == "sign":
        return sign(0) + [(2, p, "gate") for p in primes]
    out = []
    for _ in range(repeat):
        out += [(2, p, "gate") for p in primes[1:]] + sign(1)
    return out


def network_work(net):
    """gates, rows and algorithmic lane operations of one pass over `batch` batch elements, split by kernel class"""
    primes, digits = net["primes"], net["digits"]
    w = dict(gates=0, rows=dict(digits=0, gate=0), ops_garble=dict(digits=0.0, gate=0.0), ops_eval=0.0)
    for L in net["layers"]:
        if L["kind"] not in ("relu", "scale", "sign"):
            continue
        per = gadget_gates(primes, digits, L["kind"], L.get("repeat", 1))
        nval = L["n"] * net["batch"]
        for p, q, cls in per:
            lp, lq = _lam_ceil(p), _lam_ceil(q)
            c = "digits" if cls == "digits" else "gate"
            w["gates"] += nval
            w["rows"][c] += nval * p
            share = len(digits) if cls == "digits" else 1
            w["ops_garble"][c] += nval * p * alg_ops_garble_row(p, q, lp, lq, cls == "short", share)
            w["ops_eval"] += nval * alg_ops_eval_gate(p, q, lp, lq, share)
    return w


def mac_counts(net, lam_sum):
    macs = 0
    for L in net["layers"]:
        if L["kind"] == "conv":
            macs += L["out_h"] * L["out_w"] * L["out_c"] * L["kh"] * L["kw"] * L["in_c"]
    return macs * net["batch"] * lam_sum


# ---- the oracle on the host cores ------------------------------------------------------------------------
def cpu_baseline(net, seconds_target=10.0):
    """The oracle as it stands, on the host cores, on bounded samples of the same workloads:
    (1) the ReLU + scale-by-2^6 activation pipeline of config 2 (garble and evaluate), values split over the threads;
    (2) the dense contraction of config 4 on a subset of output rows and batch elements;
    (3) one whole config-1 inference (garble, encode, evaluate, decode) on one thread."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import workloads
    from oracle import capi
    from oracle import net as onet

    cores = min(16, os.cpu_count() or 1)
    repeat = next(L["repeat"] for L in net["layers"] if L["kind"] == "scale")
    k = len(net["primes"])
    per_value = len(gadget_gates(net["primes"], net["digits"], "relu")) + len(gadget_gates(net["primes"], net["digits"], "scale", repeat))

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
    out = dict(value=2 * done * per_value / dt, unit="projection gates/s (garble+eval)", cores=cores, kind="oracle",
               sample="ReLU + scale-by-2^%d pipeline of config 2 on %d values (%d per thread), garble + evaluate, %.1f s"
                      % (repeat, done, count, dt))

    # (2) config 4: R output rows of the 4096 x 4096 layer for one batch element per thread, all 12 primes
    mb = workloads.gemm_microbench(seed=4)
    K, rows = mb["K"], 2048
    orc12 = capi.Oracle(mb["primes"], workloads.DIGITS[12], mb["seed"], 0)
    lam12 = [orc12.lam(p) for p in mb["primes"]]

    def macs(t):
        g = np.random.default_rng(100 + t)
        r0 = (t * rows) % (mb["M"] - rows)
        for i, p in enumerate(mb["primes"]):
            x = workloads.uniform_labels(g, K, lam12[i], p)
            orc12.dense(i, x, 1, K, rows, mb["W"][r0:r0 + rows])
        return rows * K * sum(lam12)
    t0 = time.time()
    with ThreadPoolExecutor(cores) as ex:
        total = sum(ex.map(macs, range(cores)))
    dt = time.time() - t0
    out["label_mac_per_s"] = dict(value=total / dt, cores=cores,
                                  sample="config 4: %d output rows x 4096 inputs x 12 primes for %d batch elements (one per thread), %.1f s" % (rows, cores, dt))

    # (3) config 1: one inference, single thread
    net1 = workloads.mlp(seed=1, batch=1)
    orc1 = onet.make_oracle(net1)
    t0 = time.time()
    gb = onet.garble(orc1, net1)
    t1 = time.time()
    act = onet.encode(orc1, net1, gb["e"], np.asarray(net1["x"]))
    outl = onet.evaluate(orc1, net1, act, gb["tables"])
    orc1.decode(outl, gb["d"])
    t2 = time.time()
    out["config1_inference"] = dict(garble_ms=(t1 - t0) * 1e3, eval_ms=(t2 - t1) * 1e3, cores=1,
                                    sample="config 1 whole (MLP 784-128-10, batch 1): garble; encode + evaluate + decode")
    return out


def kernel_line(pr, steps):
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


def zero_pad_digits(ctx, labels, i):
    """digits past lambda in the last chunk are zero in a LabelTensor (the layout contract)"""
    lam = ctx.lam(ctx.primes[i])
    if lam % 16:
        labels.tensors[i][-1, :, lam % 16:] = 0


# ---- config 3 --------------------------------------------------------------------------------------------
def micro_projection(torch, workloads, reps=2):
    """Config 3: 2^24 independent gates Z_p -> Z_q over the 12-prime base, grouped by (p, q)."""
    from paper_2302_06361_amd import Context, ProjectionBatch
    mb = workloads.proj_microbench(seed=3)
    ctx = Context(mb["primes"], mb["seed"], workloads.DIGITS[12])
    pb = ProjectionBatch(ctx, mb["pi"], mb["qi"])
    a_all = torch.as_tensor(mb["a"][pb.order].astype("int64")).to(ctx.device)
    gen = torch.Generator(device=ctx.device)
    gen.manual_seed(3)
    ops_g = ops_e = 0.0
    for G in pb.groups:
        i, p, q, n = G["pi"], ctx.primes[G["pi"]], ctx.primes[G["qi"]], G["count"]
        t = G["in0"].tensors[i]
        t.copy_(torch.randint(0, p, t.shape, dtype=torch.uint8, device=ctx.device, generator=gen))
        zero_pad_digits(ctx, G["in0"], i)
        ctx.encode(a_all[G["start"]:G["start"] + n], G["in0"], G["act"])           # active label = zero + a R_p
        G["phi"].copy_(torch.randint(0, q, G["phi"].shape, dtype=torch.uint8, device=ctx.device, generator=gen))
        ops_g += n * p * alg_ops_garble_row(p, q, ctx.lam(p), ctx.lam(q))
        ops_e += n * alg_ops_eval_gate(p, q, ctx.lam(p), ctx.lam(q))
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
        pb.garble()
    for _ in range(reps):
        pb.evaluate()
    torch.cuda.synchronize()
    ctx.profile_enable(False)
    pr = read_profiles(ctx)
    kg, ke = kernel_line(pr["garble"], reps), kernel_line(pr["eval"], reps)
    eval_bytes = pr["eval"]["bytes"] / reps
    out = dict(workload="config 3: 2^24 gates Z_p->Z_q, (p,q) uniform over the 12-prime base, grouped by (p,q): one "
                        "dash_garble_layers / dash_eval_layers call over the 144 groups, one stream",
               gates=pb.n, rows=pb.rows, table_bytes=pb.table_bytes, launches_garble=kg["launches_per_step"], launches_eval=ke["launches_per_step"],
               garble_ms=gms, eval_ms=ems, garble_gates_per_s=pb.n / (gms * 1e-3), eval_gates_per_s=pb.n / (ems * 1e-3),
               garble_rows_per_s=pb.rows / (gms * 1e-3),
               garble=dict(hbm_algorithmic_GBps=pr["garble"]["bytes"] / reps / (gms * 1e-3) / 1e9,
                           hbm_frac=pr["garble"]["bytes"] / reps / (gms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           alu_frac_algorithmic=ops_g / (gms * 1e-3) / 1e12 / ALU_PEAK_TOPS),
               eval=dict(hbm_algorithmic_GBps=eval_bytes / (ems * 1e-3) / 1e9, hbm_frac=eval_bytes / (ems * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         alu_frac_algorithmic=ops_e / (ems * 1e-3) / 1e12 / ALU_PEAK_TOPS),
               kernels=dict(k_proj_garble=kg, k_proj_eval=ke))
    pmc, note = load_pmc()
    if pmc and "proj2p24_eval_traffic_bytes_per_gate" in pmc:
        # HBM bytes from the committed counters (FETCH_SIZE + WRITE_SIZE, scaled): the evaluator's row gather moves whole lines
        et, gt = pmc["proj2p24_eval_traffic_bytes_per_gate"] * pb.n, pmc["proj2p24_garble_traffic_bytes_per_row"] * pb.rows
        out["eval"].update(traffic=et, hbm_traffic_GBps=et / (ems * 1e-3) / 1e9, hbm_traffic_frac=et / (ems * 1e-3) / 1e9 / HBM_PEAK_GBS, counters=note)
        out["garble"].update(traffic=gt, hbm_traffic_GBps=gt / (gms * 1e-3) / 1e9, counters=note)
    del pb
    ctx.close()
    torch.cuda.empty_cache()
    return out


# ---- config 4 --------------------------------------------------------------------------------------------
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
        zero_pad_digits(ctx, x, i)
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
    traffic, note = gemm_traffic()
    out = dict(workload="config 4: dense 4096x4096, weights in [-64,63], batch 128, 12 primes (%d label digits per value)" % lam,
               ms=ms, label_mac_per_s=macs / (ms * 1e-3),
               roofline=dict(bound="mfma", kernel="k_dense_mfma", unit="TOP/s", peak=INT8_MFMA_PEAK_TOPS,
                             achieved=2 * macs / (kms * 1e-3) / 1e12, frac=2 * macs / (kms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS,
                             avg_launch_ms=kms, ops_per_launch=2 * macs, traffic=traffic, traffic_note=note,
                             algorithmic_bytes_per_launch=float(M) * K * len(ctx.primes) + 2.0 * Bn * (M + K) / 2 * 16 * sum((ctx.lam(p) + 15) // 16 for p in ctx.primes)))
    ctx.close()
    torch.cuda.empty_cache()
    return out


def gemm_traffic():
    """HBM bytes per launch of k_dense_mfma on config 4 from the committed counter summary (FETCH_SIZE + WRITE_SIZE, scaled by
    the copy kernel), or None"""
    path = os.path.join(ROOT, "profiles", "k_dense_mfma_dense4096_b128_pmc.txt")
    if not os.path.exists(path):
        return None, "profiles/k_dense_mfma_dense4096_b128_pmc.txt is missing"
    for line in open(path):
        if line.startswith("hbm_bytes_per_launch"):
            return float(line.split("=")[1].split("#")[0]), "from profiles/k_dense_mfma_dense4096_b128_pmc.txt"
    return None, "no hbm_bytes_per_launch line in profiles/k_dense_mfma_dense4096_b128_pmc.txt"


# ---- config 5 --------------------------------------------------------------------------------------------
def micro_vgg(torch, workloads, images=2, chunk=2, reps=1):
    """Config 5, streamed: garble + encode + evaluate + decode layer by layer, `chunk` images of the batch of 64 at a
    time (the tables of one image's largest layer take 30 GB), `images` images in all."""
    from paper_2302_06361_amd import Context, StreamedNetwork
    net = workloads.vgg(seed=5, batch=64)
    images = min(images, 64)
    chunk = min(chunk, images)
    ctx = Context(net["primes"], net["seed"], net["digits"])
    g = StreamedNetwork(ctx, net, batch=chunk)
    n_in = net["n_in"]
    xs = [torch.as_tensor(net["x"][b * n_in:(b + chunk) * n_in]).to(ctx.device) for b in range(0, images, chunk) if b + chunk <= images]
    lam_sum = sum(ctx.lam(p) for p in ctx.primes)
    sub = dict(net, batch=len(xs) * chunk)
    work, macs = network_work(sub), mac_counts(sub, lam_sum)
    g.run(xs[0])
    torch.cuda.synchronize()
    valid = True
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        for ci, x in enumerate(xs):
            g.batch_base = ci * chunk
            g.rebase()
            g.run(x)
            valid = valid and bool(g.valid.all().item())
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    # per-kernel figures from one more chunk with the library's events (not timed above)
    ctx.profile_enable(True)
    read_profiles(ctx)
    g.run(xs[0])
    torch.cuda.synchronize()
    ctx.profile_enable(False)
    pr = read_profiles(ctx)
    n_img = len(xs) * chunk
    # table bytes of one image in the working format and in the packed storage format (dash_tables_pack; defined for
    # label lengths by the floor rule, so both are given for a floor-rule context; sizes only, nothing is run)
    from paper_2302_06361_amd import LAMBDA_FLOOR
    from paper_2302_06361_amd.network import build_layers
    fctx = Context(net["primes"], net["seed"], net["digits"], LAMBDA_FLOOR)
    flayers, _, ftb, _ = build_layers(fctx, net, 1, 0)
    floor_bytes = sum(ftb)
    floor_packed = sum(fctx.tables_packed_bytes(l) for l, tb in zip(flayers, ftb) if tb)
    fctx.close()
    out = dict(workload="config 5: VGG shape (12 primes, scale 2^5), %d image(s) of the batch of 64, streamed layer by layer in chunks "
                        "of %d images, garble + encode + evaluate + decode" % (n_img, chunk),
               images=n_img, chunk=chunk, ms=ms, ms_per_image=ms / n_img, outputs_valid=valid,
               table_bytes_per_image=g.table_bytes // chunk, gates_per_image=work["gates"] // n_img,
               table_bytes_per_image_floor_rule=dict(working_format=floor_bytes, packed_format=floor_packed),
               gates_per_s=2 * work["gates"] / (ms * 1e-3), label_macs_per_image=2 * macs // n_img,
               kernels_per_chunk=dict(k_proj_garble=kernel_line(pr["garble"], 1), k_digits_garble=kernel_line(pr["garble_digits"], 1),
                                      eval_kernels=kernel_line(pr["eval"], 1), linear=kernel_line(pr["linear"], 1)))
    ctx.close()
    torch.cuda.empty_cache()
    return out


# ---- config 1 and the paper's model shapes: batch-1 latency ---------------------------------------------------
def latency(torch, net, reps=5):
    from paper_2302_06361_amd import Context, GarbledNetwork
    ctx = Context(net["primes"], net["seed"], net["digits"])
    g = GarbledNetwork(ctx, net)
    x = torch.as_tensor(net["x"]).to(ctx.device)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for r in range(reps + 1):
        if r == 1:
            torch.cuda.synchronize()
            ev[0].record()
        g.garble()
    ev[3].record()
    for r in range(reps + 1):       # one untimed pass first, like the garbler's (the kernels' first launches load their code)
        if r == 1:
            torch.cuda.synchronize()
            ev[1].record()
        g.encode(x)
        g.evaluate()
        g.decode()
    ev[2].record()
    torch.cuda.synchronize()
    work = network_work(net)
    out = dict(primes=len(net["primes"]), activation_values=sum(L["n"] for L in net["layers"] if L["kind"] == "relu") * net["batch"],
               gates=work["gates"], table_bytes=g.table_bytes, garble_ms=ev[0].elapsed_time(ev[3]) / reps,
               eval_ms=ev[1].elapsed_time(ev[2]) / reps, outputs_valid=bool(g.valid.all().item()))
    del g
    ctx.close()
    torch.cuda.empty_cache()
    return out


def micro_mlp(torch, workloads):
    """Config 1: MLP 784-128-10, batch 1, 8 primes, ReLU + scale 2^6: latency of one inference."""
    out = latency(torch, workloads.mlp(seed=1, batch=1), reps=10)
    out["workload"] = "config 1: MLP 784-128-10, batch 1, 8 primes, ReLU + scale 2^6; eval_ms = encode + evaluate + decode of one inference"
    out["ms_per_inference"] = out["eval_ms"]
    return out


def micro_reduced_accuracy(torch, workloads, batch=16):
    """Config 2's network with the reduced-accuracy sign (Appendix, Approximated Garbled Sign): the three-digit set
    (26; 12, 12) instead of the exact seven-digit one: 27 digit and carry gates per sign gadget instead of 63."""
    net = dict(workloads.lenet(seed=2, batch=batch))
    net["digits"] = list(workloads.DIGITS_REDUCED[8])
    out = latency(torch, net, reps=3)
    out["workload"] = ("config 2's network (LeNet-5 shape, batch %d, 8 primes) with the sign digit set %s: the sign is wrong for at "
                       "most 2 k / M = 0.43 %% of the values" % (batch, tuple(net["digits"])))
    out["ms_per_inference_eval"] = out["eval_ms"] / batch
    out["ms_per_inference_garble"] = out["garble_ms"] / batch
    return out


def micro_paper_models(torch, workloads):
    """The shapes of the paper's models A-F (Sec. Model architectures), batch 1, random weights: garbling time
    (offline in the paper) and evaluation time (its online figure, there including a modelled network cost)."""
    out = {name: latency(torch, workloads.paper_model(name, seed=6)) for name in "ABCDfF"}
    return dict(workload="paper model shapes A-F, batch 1, random integer weights and biases", models=out,
                paper_online_ms_gpu=dict(A=10, B=32, C=16, D=42, f=1332, F=1443),
                note="the paper's figures (its table of online runtimes, other hardware) include a modelled 1 Gbit/s transfer; context only")


def micro_aes(torch, workloads, log2_blocks=24, repeat=16, reps=3):
    """AES-128 alone in the forms the library holds (dash_profile.h): the gate kernels' T-table look-ups in LDS
    in both table layouts, the table-free bit-plane form (32 blocks per lane), and all four tables per bank.  2^24 blocks resident in HBM,
    `repeat` encryptions in a row per block so that the 32 bytes of traffic per block do not matter."""
    from paper_2302_06361_amd import Context
    ctx = Context(workloads.PRIMES[:3], bytes(range(16)), workloads.DIGITS[3])
    n = 1 << log2_blocks
    gen = torch.Generator(device=ctx.device)
    gen.manual_seed(3)
    d_in = torch.randint(0, 256, (n, 16), dtype=torch.uint8, device=ctx.device, generator=gen)
    d_out = torch.empty_like(d_in)
    names = ["tables_4KB_per_workgroup", "tables_per_bank_64KB", "bit_planes_32_blocks_per_lane", "four_tables_per_bank_128KB"]
    out = {}
    for v, name in enumerate(names):
        ctx.profile_aes(v, bytes(range(16)), d_in, d_out, repeat)       # warm-up
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(reps):
            ctx.profile_aes(v, bytes(range(16)), d_in, d_out, repeat)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / reps
        out[name] = dict(ms_per_launch=ms, blocks_per_s=n * repeat / (ms * 1e-3))
    ctx.close()
    return dict(workload="AES-128 alone: 2^%d blocks, %d encryptions in a row per block" % (log2_blocks, repeat), forms=out,
                executed_valu_per_block=dict(bit_planes_32_blocks_per_lane=630, note="static count of the kernel's instructions"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--batch", type=int, default=16, help="batch elements of config 2 (16 = the config)")
    ap.add_argument("--images", type=int, default=2, help="images of config 5's batch of 64 to stream (64 = the whole config, about 11 s)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-micro", action="store_true", help="the config-2 step alone")
    ap.add_argument("--only", choices=["config1", "config3", "config4", "config5", "paper_models", "reduced", "aes"],
                    help="run one of the other configurations alone (for profiling); prints its JSON object")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build measures ONE GPU (every box has one); --gpus %d is not supported" % a.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    import workloads
    from paper_2302_06361_amd import Context, GarbledNetwork

    if a.only:
        fn = dict(config1=micro_mlp, config3=micro_projection, config4=micro_contraction,
                  config5=lambda t, w: micro_vgg(t, w, images=a.images), paper_models=micro_paper_models,
                  reduced=lambda t, w: micro_reduced_accuracy(t, w, a.batch), aes=micro_aes)[a.only]
        print(json.dumps(fn(torch, workloads)))
        return

    net = workloads.lenet(seed=2, batch=a.batch)
    ctx = Context(net["primes"], net["seed"], net["digits"])
    g = GarbledNetwork(ctx, net)
    x = torch.as_tensor(net["x"]).to(ctx.device)
    lam_sum = sum(ctx.lam(p) for p in ctx.primes)
    work = network_work(net)
    gates = work["gates"]
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
    pmc, pmc_note = load_pmc()

    def garble_roofline(kernel, kk, cls, key):
        """ALU roofline of a garbling kernel.  achieved = ALGORITHMIC lane operations per launch / average launch duration
        (frac = frac_algorithmic); frac_issue = executed vector instructions (counter SQ_INSTS_VALU of the committed --pmc
        summary) on the same clock; hbm_frac = algorithmic bytes against the HBM peak."""
        alg_per_row = work["ops_garble"][cls] / max(work["rows"][cls], 1)
        r = dict(kernel=kernel, bound="alu", unit="Tlane-op/s (32-bit integer vector operations)", peak=ALU_PEAK_TOPS,
                 achieved=kk["units_per_s"] * alg_per_row / 1e12, ms_per_step=kk["ms_per_step"],
                 avg_launch_ms=kk["avg_launch_ms"], launches_per_step=kk["launches_per_step"],
                 rows_per_launch=kk["units_per_launch"], rows_per_s=kk["units_per_s"], algorithmic_lane_ops_per_row=alg_per_row,
                 hbm_algorithmic_GBps=kk["gbytes_per_s"], hbm_frac=kk["gbytes_per_s"] / HBM_PEAK_GBS,
                 algorithmic_bytes_per_launch=kk["bytes_per_launch"], counters=pmc_note)
        r["frac"] = r["frac_algorithmic"] = r["achieved"] / ALU_PEAK_TOPS
        if pmc and key + "_valu_per_row" in pmc:
            r["executed_lane_instr_per_row"] = pmc[key + "_valu_per_row"]
            r["frac_issue"] = kk["units_per_s"] * pmc[key + "_valu_per_row"] / 1e12 / ALU_PEAK_TOPS
            r["traffic"] = (pmc[key + "_fetch_bytes_per_row"] + pmc[key + "_write_bytes_per_row"]) * kk["units_per_launch"]
        else:
            r["frac_issue"] = r["traffic"] = None
        return r
    # the dominant kernel of the step: the general projection-gate garbler (carry chains, half gates, casts); the
    # digit gates of the sign gadgets run in the fused kernel, reported beside it
    roofline = garble_roofline("k_proj_garble", kg, "gate", "garble")
    roofline_digits = garble_roofline("k_digits_garble", kd, "digits", "digits") if kd else None
    alg_eval = work["ops_eval"] / gates
    roofline_eval = dict(kernel="k_digits_eval + k_chain_eval + k_cast_halve + k_proj_eval", bound="alu", unit=roofline["unit"], peak=ALU_PEAK_TOPS,
                         achieved=ke["units_per_s"] * alg_eval / 1e12, algorithmic_lane_ops_per_gate=alg_eval,
                         ms_per_step=ke["ms_per_step"], avg_launch_ms=ke["avg_launch_ms"], launches_per_step=ke["launches_per_step"],
                         gates_per_s=ke["units_per_s"], hbm_algorithmic_GBps=ke["gbytes_per_s"],
                         hbm_frac=ke["gbytes_per_s"] / HBM_PEAK_GBS)
    roofline_eval["frac"] = roofline_eval["frac_algorithmic"] = roofline_eval["achieved"] / ALU_PEAK_TOPS
    roofline_eval["frac_issue"] = (ke["units_per_s"] * pmc["eval_valu_per_gate"] / 1e12 / ALU_PEAK_TOPS) if pmc and "eval_valu_per_gate" in pmc else None

    config2 = dict(
        workload="config 2: LeNet-5 shape, batch %d, 8-prime CRT base, 128-bit labels (ceil rule), "
                 "ReLU + scale 2^6 after every conv/dense but the last" % a.batch,
        ms_per_step=ms_step, outputs_valid=ok,
        gates_per_s=2 * gates / (ms_step * 1e-3), garble_gates_per_s=gates / (phase[0] * 1e-3), eval_gates_per_s=gates / (phase[2] * 1e-3),
        ms_per_inference=ms_step / a.batch, ms_per_inference_eval=(phase[1] + phase[2] + phase[3]) / a.batch,
        ms_per_inference_garble=phase[0] / a.batch,
        phase_ms=dict(garble=phase[0], encode=phase[1], eval=phase[2], decode=phase[3]),
        gates_per_step=gates, label_macs_per_step=2 * macs, table_bytes=g.table_bytes,
        linear_kernels=dict(ms_per_step=kl["ms_per_step"], label_mac_per_s=kl["units_per_s"],
                            note="config-2 linear layers are tiny (launch-bound); config 4 is the contraction figure"))
    out = dict(
        metric="label-MAC/s + projection gates/s (garble & eval); ms/inference, 1 GPU",
        value=2 * gates / (ms_step * 1e-3),
        unit="projection gates/s (garbled + evaluated, whole step: garble+encode+eval+decode)",
        n_gpus=1, steps=a.steps, warmup=a.warmup, ms_per_step=ms_step, higher_is_better=True, scaling="weak",
        vs_baseline=None, dtype="u8 digits, i32 accumulate", data="synthetic",
        config=dict(workload=config2["workload"] + "; the other four configurations are in `configs`",
                    batch=a.batch, primes=ctx.primes, sign_digits=ctx.digits, table_bytes=g.table_bytes),
        outputs_valid=ok,
        garble_gates_per_s=config2["garble_gates_per_s"], eval_gates_per_s=config2["eval_gates_per_s"],
        ms_per_inference=config2["ms_per_inference"], ms_per_inference_eval=config2["ms_per_inference_eval"],
        ms_per_inference_garble=config2["ms_per_inference_garble"],
        roofline=roofline, roofline_digits_kernel=roofline_digits, roofline_eval_kernel=roofline_eval,
    )
    del g
    ctx.close()
    torch.cuda.empty_cache()
    configs = dict(config2=config2)
    if not a.no_micro:
        configs["config1"] = micro_mlp(torch, workloads)
        configs["config3"] = micro_projection(torch, workloads)
        configs["config4"] = micro_contraction(torch, workloads)
        configs["config5"] = micro_vgg(torch, workloads, images=a.images)
        configs["paper_models"] = micro_paper_models(torch, workloads)
        configs["config2_reduced_accuracy"] = micro_reduced_accuracy(torch, workloads, a.batch)
    out["configs"] = {k: configs[k] for k in sorted(configs)}
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(net)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
