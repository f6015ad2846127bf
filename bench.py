#!/usr/bin/env python3
"""Benchmark of the HISA hot path on one MI355X.

Headline metric of the benchmark definition: key-switched rotLeft per second at N = 2^15,
batch 64 -- the primitive micro-benchmark configuration (16 limbs of 50-bit
primes, dnum 3, rotation steps {1, 7, 64}).  One "step" rotates a batch of 64
synthetic ciphertexts, resident in HBM, by one of the three amounts (cycling).

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      dominant kernel of the step, algorithmic bytes / HIP-event time
  rot_left      whole-operation figures against the staged and strict HBM models
  ops           per-primitive timings of the same configuration
  cpu_baseline  the CPU oracle on a bounded sample of the same workload
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes_rot_left(N, l, K, alpha, B):
    """HBM bytes each kernel of one batched rotLeft must move (reads + writes), per kernel name."""
    LP = 8 * N
    ext = l + K
    digits = (l + alpha - 1) // alpha
    sizes = [min(alpha, l - j * alpha) for j in range(digits)]
    out = {}
    out["automorph_ntt_kernel"] = 2 * l * LP * B
    out["ntt_pass_kernel<true>"] = 2 * LP * B * (l + 2 * K)
    out["ntt_pass_kernel<false>"] = 2 * LP * B * (sum(ext - a for a in sizes) + 2 * l)
    out["base_conv_kernel"] = LP * B * (sum(a + (ext - a) for a in sizes) + 2 * (K + l))
    out["copy_limbs_kernel"] = 2 * l * LP * B
    out["inner_product_kernel"] = LP * (B * (digits * ext + 2 * ext) + digits * 2 * ext)
    out["moddown_final_kernel"] = 7 * l * LP * B
    # fused fp64 pipeline (primes below 2^50): what each launch set must read and write once
    conv_out = sum(ext - a for a in sizes)
    # kernel names as rocprofv3 prints them: ntt_fp_kernel<log2 N - 10, mode>; mode 2 = inverse transform to the
    # conversion input, 3 = base conversion + forward transform, 4 = the same + final combine
    k3 = "%d" % (N.bit_length() - 1 - 10)
    # 2 = stage A (c1 to the conversion input), 5 = stage C (special limbs of the accumulators to the ModDown's
    # conversion input), 6 = stage D (conversion + transform + subtraction from the folded accumulators)
    out["ntt_fp_kernel<%s, 2>" % k3] = 2 * LP * B * l
    out["ntt_fp_kernel<%s, 5>" % k3] = 2 * LP * B * 2 * K
    out["ntt_fp_kernel<%s, 3>" % k3] = LP * B * (l + conv_out)
    out["inner_product_fp_kernel"] = LP * (B * (conv_out + l + 2 * ext) + digits * 2 * ext)
    out["inner_product_fold_fp_kernel"] = LP * (B * (conv_out + l + l + 2 * ext) + digits * 2 * ext)   # + the addend c0
    out["ntt_fp_kernel<%s, 4>" % k3] = LP * B * (2 * K + 2 * l + l + 2 * l)
    out["ntt_fp_kernel<%s, 6>" % k3] = LP * B * (2 * K + 2 * l + 2 * l)
    return out


def algorithmic_flops_rot_left(N, l, K, alpha, B):
    """fp64 operations (an FMA counts two) the fused fp64 kernels of one batched rotLeft must execute, per kernel
    name.  A modular product is mul, fma, mul, round, fma, add = 8; a butterfly is a product, an add and a
    subtract = 10; a base-conversion term is a product and an add = 9.  Twiddle-factor products, range
    normalisations and integer<->double conversions are implementation overhead and are not counted."""
    log_n = N.bit_length() - 1
    ext = l + K
    digits = (l + alpha - 1) // alpha
    sizes = [min(alpha, l - j * alpha) for j in range(digits)]
    ntt = 10 * (N // 2) * log_n
    k3 = "%d" % (log_n - 10)
    out = {}
    out["ntt_fp_kernel<%s, 2>" % k3] = B * l * (ntt + 2 * 8 * N)                    # + untwist and (D/q)^-1 products
    out["ntt_fp_kernel<%s, 5>" % k3] = B * 2 * K * (ntt + 8 * N)                    # + untwist
    out["ntt_fp_kernel<%s, 6>" % k3] = B * 2 * l * (ntt + 9 * K * N + N)            # + acc - conv
    out["inner_product_fold_fp_kernel"] = B * ext * N * 2 * (9 * digits + 8)
    out["ntt_fp_kernel<%s, 3>" % k3] = B * sum((ext - a) * (ntt + 9 * a * N) for a in sizes)
    out["ntt_fp_kernel<%s, 4>" % k3] = B * 2 * l * (ntt + 9 * K * N + 10 * N)       # + (acc - conv) P^-1 + addend
    out["inner_product_fp_kernel"] = B * ext * N * 2 * 9 * digits
    return out


COUNTER_FILE = os.path.join(ROOT, "profiles", "rot_left_n15_l16_dnum3_b64_counters.md")
KERNEL_SOURCES = ("ntt_fp.hip", "fparith.hpp", "elementwise.hip")


def kernel_source_sha():
    """Short hash of the sources of the timed kernels: a counter summary names the hash it was measured on."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_1810_00845_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def read_counters(path=COUNTER_FILE):
    """Per-launch hardware counters of the headline configuration from the committed rocprofv3 summary (a table of
    per-launch averages: FETCH_SIZE and WRITE_SIZE in KiB, SQ counters; the row of the library's copy kernel, which
    moves a known 1 GiB each way, gives the factors that turn the memory counters into bytes).  Returns
    ({kernel: {"traffic": bytes, "valu_issue_busy": share}}, source description) or ({}, reason)."""
    if not os.path.exists(path):
        return {}, {"file": None, "note": "no counter summary committed"}
    rows, sha = {}, None
    for line in open(path):
        if line.startswith("kernel sources sha:"):
            sha = line.split(":", 1)[1].strip()
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 7 and cells[0] not in ("kernel", "") and not set(cells[0]) <= set("-: "):
            try:
                rows[cells[0]] = [float(c) if c not in ("", "-") else None for c in cells[1:]]
            except ValueError:
                pass
    copy = rows.get("copy_kernel")
    if not copy or not copy[1] or not copy[2]:
        return {}, {"file": os.path.relpath(path, ROOT), "note": "no copy_kernel row to scale the memory counters"}
    gib_kib = float(1 << 20)
    f_fetch, f_write = gib_kib / copy[1], gib_kib / copy[2]
    out = {}
    for name, (launches, fetch, write, valu, busy, wait_share) in rows.items():
        d = {}
        if fetch is not None and write is not None:
            d["traffic"] = int((fetch * f_fetch + write * f_write) * 1024)
        if valu is not None and busy:
            d["valu_issue_busy"] = round(valu * 4 / (4 * busy), 3)   # 4 cycles per wave instruction, 4 SIMDs per CU
        if wait_share is not None:
            d["wait_share"] = wait_share
        out[name] = d
    src = {"file": os.path.relpath(path, ROOT), "measured_on_kernel_sources": sha, "current_kernel_sources": kernel_source_sha(),
           "fetch_factor": round(f_fetch, 3), "write_factor": round(f_write, 3)}
    src["stale"] = sha != src["current_kernel_sources"]
    return out, src


def summarize_counters(root):
    """The counter summary read_counters reads, from rocprofv3's csv output under `root`: sub-folders trace
    (--kernel-trace), fetch (--pmc FETCH_SIZE), write (--pmc WRITE_SIZE), sq (--pmc SQ_...) of the headline run with
    --no-ops, and ops_trace / ops_fetch / ops_write of a run with the per-primitive timings (only the streaming
    primitives' rows are taken from those).  Per kernel: launches and mean duration from the trace, per-launch means
    of the counters.  Printed to stdout; the profiling commands themselves are listed in the committed summary."""
    import collections
    import csv
    import glob
    import re

    def load(sub, pattern):
        rows = []
        for f in glob.glob(os.path.join(root, sub, "**", "*" + pattern), recursive=True):
            with open(f) as fh:
                rows += list(csv.DictReader(fh))
        return rows

    def short(name):
        return re.sub(r", (true|false)>$", ">", name.replace("void ", "").split("(")[0])

    def counters(sub):
        agg = collections.defaultdict(lambda: collections.defaultdict(list))
        for r in load(sub, "counter_collection.csv"):
            agg[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
        return agg

    def durations(sub, keep):
        d = collections.defaultdict(list)
        for r in load(sub, "kernel_trace.csv"):
            if keep(short(r["Kernel_Name"])):
                d[short(r["Kernel_Name"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
        return d

    avg = lambda x: sum(x) / len(x) if x else None
    cell = lambda x, fmt="%.1f": (fmt % x) if x is not None else "-"
    ops = ("addsub_kernel", "mul_plain_kernel", "mul_no_relin_kernel")
    dur = durations("trace", lambda n: n.startswith(("ntt_fp_kernel", "inner_product", "copy_kernel")))
    dur.update(durations("ops_trace", lambda n: n in ops))
    cf, cw, cs = counters("fetch"), counters("write"), counters("sq")
    of, ow = counters("ops_fetch"), counters("ops_write")
    for n in ops:
        cf[n], cw[n] = of.get(n, {}), ow.get(n, {})
    print("kernel sources sha: %s" % kernel_source_sha())
    print()
    print("| kernel | launches | FETCH_SIZE_KiB | WRITE_SIZE_KiB | SQ_INSTS_VALU | SQ_BUSY_CU_CYCLES | wait_share |")
    print("|---|---|---|---|---|---|---|")
    for n in sorted(dur):
        wa, wc = avg(cs[n].get("SQ_WAIT_INST_ANY", [])), avg(cs[n].get("SQ_WAVE_CYCLES", []))
        print("| %s | %d | %s | %s | %s | %s | %s |" % (
            n, len(dur[n]), cell(avg(cf[n].get("FETCH_SIZE", []))), cell(avg(cw[n].get("WRITE_SIZE", []))),
            cell(avg(cs[n].get("SQ_INSTS_VALU", [])), "%.0f"), cell(avg(cs[n].get("SQ_BUSY_CU_CYCLES", [])), "%.0f"),
            cell(wa / wc if wa is not None and wc else None, "%.3f")))
    print()
    print("kernel durations from the trace runs (us, mean over launches):")
    for n in sorted(dur):
        print("  %-36s %4d launches  %10.2f" % (n, len(dur[n]), avg(dur[n]) / 1e3))


FP64_PEAK_TFLOPS = 78.6   # 256 CUs x 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz


def staged_bytes_rot_left(N, l, K, alpha, dnum_key, L, B):
    """(11 l + 6 K) LP + key/B: one HBM round trip per change of access pattern, everything else fused."""
    LP = 8 * N
    key = dnum_key * 2 * (L + K) * LP
    return (11 * l + 6 * K) * LP + key / B, 4 * l * LP + key / B


def time_op(ctx, fn, iters, warm=2):
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        fn()
    ctx.sync()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / iters


def cpu_baseline(log_n, q_bits, dnum, special_bits, seed, sample, steps):
    """The oracle's rotLeft on `sample` ciphertexts of the same shape, spread over the host cores."""
    from concurrent.futures import ThreadPoolExecutor
    import numpy as np
    from oracle import Oracle
    from paper_1810_00845_amd import synth
    o = Oracle(log_n, q_bits, dnum, special_bits, seed)
    o.gen_rot_keys(steps[:1])
    cores = min(sample, os.cpu_count() or 1, 16)
    coeff = synth.uniform_residues(seed, (sample, 2, len(q_bits), o.N), o.primes[:len(q_bits)])
    cts = [o.import_ct(coeff[i], 2.0 ** 50) for i in range(sample)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        list(ex.map(lambda c: o.rot_left(c, steps[0]), cts))
    dt = time.perf_counter() - t0
    one = min(4, sample)                       # the same call on one thread, for the per-core figure
    t1 = time.perf_counter()
    for c in cts[:one]:
        o.rot_left(c, steps[0])
    dt1 = time.perf_counter() - t1
    return {"value": sample / dt, "unit": "rotLeft/s", "cores": cores, "kind": "oracle",
            "single_thread_value": one / dt1,
            "sample": "%d ciphertexts of the same N, limbs, dnum, one rotLeft(%d) each, %.1f s on %d threads; %d of them "
                      "again on one thread, %.1f s" % (sample, steps[0], dt, cores, one, dt1)}


def network_latencies():
    """Encrypted inference latency of the benchmark networks (benchmark configurations 3, 4 and 5): encrypt-done to the
    last output ciphertext ready, one image, rotation and relinearisation keys resident, weights converted and
    encoded ahead of time (hisa_conv2d_prepare, hisa_fc_prepare, hisa_matmul_prepare) (median of 3 after one set-up
    pass that generates the keys and the plans).  Every data layout is timed (Sec. "Data Layout Selection":
    HW-tiling throughout, HW-tiling up to the first fully connected layer and CHW-tiling after it, CHW-tiling
    throughout, CHW-tiling with HW-tiled convolutions; the last needs two more levels than the SqueezeNet-style
    parameters have); latency_ms is that of the layout the cost model selects from dry runs on the analysis backend
    (operation counts x micro-benchmarked unit costs), as the paper's compiler does; layouts_ms shows whether that was
    the fastest."""
    from paper_1810_00845_amd import hisa, nets
    out = {}
    for name, paper, layouts in (("lenet_small", "LeNet-5-small: 8 s (HEAAN, 16 Xeon threads)", ("hw", "chw_fc", "chw", "hw_conv")),
                                 ("lenet_medium", "LeNet-5-medium: 51 s (HEAAN, 16 Xeon threads)", ("hw", "chw_fc", "chw", "hw_conv")),
                                 ("squeezenet_cifar", "SqueezeNet-CIFAR: 1342 s (HEAAN, 16 Xeon threads)", ("hw", "chw"))):
        params, layers, x = getattr(nets, name)()
        limbs = len(params["q_bits"])
        border = params.get("border", 0)
        res = {}
        ctx = hisa.Context(params["log_n"], params["q_bits"], params["dnum"], params["special_bits"], seed=11)
        ctx.keygen()
        costs = nets.measure_costs(ctx, limbs)
        selected, est = nets.select_layout(ctx, layers, x, params["scale"], limbs, costs, border=border, layouts=layouts)
        ctx.close()
        for layout in layouts:
            ctx = hisa.Context(params["log_n"], params["q_bits"], params["dnum"], params["special_bits"], seed=11)
            ctx.keygen()
            plans = {}
            kw = dict(border=border, plans=plans, layout=layout)
            t_setup = time.perf_counter()
            nets.run_encrypted(ctx, layers, x, params["scale"], limbs, make_keys=True, **kw)
            ctx.sync()
            t_setup = time.perf_counter() - t_setup      # rotation keys and plans (weights converted and encoded) + one inference
            # latency: the host queues the whole network, one wait at the end; the per-layer times come from one more
            # inference that waits after every layer
            client = {}
            runs = sorted((nets.run_encrypted(ctx, layers, x, params["scale"], limbs, layer_times=False, client_times=client, **kw)
                           for _ in range(3)), key=lambda r: r[1])
            per_layer = nets.run_encrypted(ctx, layers, x, params["scale"], limbs, **kw)[2]
            client["setup_s"] = t_setup
            res[layout] = (runs[1][1], per_layer, None, dict(client))
            if layout == selected:     # one more inference with HIP events around every kernel: where the time goes
                ctx.profile_enable(True)
                nets.run_encrypted(ctx, layers, x, params["scale"], limbs, **kw)
                prof = sorted(ctx.profile_read().items(), key=lambda kv: -kv[1][1])
                ctx.profile_enable(False)
                res[layout] = (runs[1][1], per_layer, {k: [c, round(ms, 3)] for k, (c, ms) in prof[:8]}, dict(client))
            nets.free_plans(ctx, plans)
            ctx.close()
        best = selected
        out[name] = {"latency_ms": round(res[best][0] * 1e3, 2), "layout": best,
                     "layouts_ms": {k: round(v[0] * 1e3, 2) for k, v in res.items()},
                     "cost_model_ms": {k: round(v * 1e3, 2) for k, v in est.items()},
                     "log_n": params["log_n"], "limbs": limbs, "dnum": params["dnum"],
                     "layers_ms": [[k, round(s * 1e3, 2)] for k, s in res[best][1]],
                     "kernels_launches_ms": res[best][2],
                     # the client's side, outside the latency: encode + encrypt of the image, decrypt + decode of the result
                     "client_ms": {k.replace("_s", ""): round(v * 1e3, 3) for k, v in res[best][3].items() if k != "setup_s"},
                     # once per network and key set: rotation keys for the amounts the circuit uses, weights converted
                     # and encoded into plans, and the first inference
                     "setup_ms": round(res[best][3]["setup_s"] * 1e3, 1),
                     "paper_context": paper, "data": "seeded random weights and image"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=15)
    ap.add_argument("--log-n", type=int, default=15)
    ap.add_argument("--limbs", type=int, default=16)
    ap.add_argument("--dnum", type=int, default=3)
    ap.add_argument("--bits", type=int, default=50)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--cpu-sample", type=int, default=64, help="ciphertexts for the oracle baseline (0 = skip)")
    ap.add_argument("--no-ops", action="store_true", help="skip the per-primitive timings")
    ap.add_argument("--no-nets", action="store_true", help="skip the encrypted-network latencies")
    ap.add_argument("--summarize-counters", metavar="DIR", help="no benchmark: print the counter summary of the "
                    "rocprofv3 csv output under DIR (the text committed under profiles/)")
    args = ap.parse_args()
    if args.summarize_counters:
        summarize_counters(args.summarize_counters)
        return
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_1810_00845_amd import hisa
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU; libhisa has no CPU fallback")

    log_n, L, dnum, B = args.log_n, args.limbs, args.dnum, args.batch
    q_bits = [args.bits] * L
    rot_steps = [1, 7, 64]
    ctx = hisa.Context(log_n, q_bits, dnum, args.bits, seed=1)
    ctx.keygen()
    ctx.gen_rot_keys(rot_steps)
    N, K, alpha = ctx.N, ctx.K, ctx.alpha
    cts = ctx.ct_random_batch(B, L, 2.0 ** 50, counter=0)
    ctx.sync()

    def step(i):
        out = ctx.rot_left_batch(cts, rot_steps[i % 3])
        for c in out:
            c.free()

    for i in range(args.warmup):
        step(i)
    ctx.sync(); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    ctx.sync(); torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    value = B * args.steps / dt

    # per-kernel durations with HIP events on the launch stream (separate pass over the same steps)
    prof_steps = 3
    ctx.profile_enable(True)
    for i in range(prof_steps):
        step(i)
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    alg = algorithmic_bytes_rot_left(N, L, K, alpha, B)
    flops = algorithmic_flops_rot_left(N, L, K, alpha, B)
    # the transform kernel's name carries a third template argument (two conversion targets per pass or one); the
    # launches of a stage are summed whatever their form
    merged = {}
    for name, (cnt, ms) in prof.items():
        key = re.sub(r", (true|false)>$", ">", name)
        c0, m0 = merged.get(key, (0, 0.0))
        merged[key] = (c0 + cnt, m0 + ms)
    kernels = {}
    for name, (cnt, ms) in merged.items():
        per_step_ms = ms / prof_steps
        gbs = alg.get(name, 0) / (per_step_ms * 1e-3) / 1e9 if per_step_ms > 0 else 0.0
        kernels[name] = {"launches_per_step": cnt / prof_steps, "ms_per_step": round(per_step_ms, 4),
                         "avg_launch_us": round(1e3 * ms / cnt, 2), "algorithmic_GBs": round(gbs, 1)}
        if name in flops and per_step_ms > 0:
            kernels[name]["algorithmic_TFLOPs"] = round(flops[name] / (per_step_ms * 1e-3) / 1e12, 2)
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    headline = (log_n, L, dnum, B, args.bits) == (15, 16, 3, 64, 50)

    # measured peaks of this GPU (hisa_calibrate: register-only instruction chains, a 1 GiB device-to-device copy)
    cal = ctx.calibrate()
    # An fp64 vector instruction is one lane-operation (an FMA two flops): the datasheet's 78.6 TFLOP/s is
    # 256 CUs x 4 SIMDs x 16 lanes x 2 x 2.4 GHz; the measured counterpart is twice the measured FMA issue rate.
    fp64_measured = 2.0 * cal["fma_f64"]
    counters, counter_src = read_counters() if headline else ({}, {"file": None, "note": "counters exist for the headline configuration only"})

    def counter_key(name):     # the counter summary keeps rocprofv3's names, without the third template argument
        return name

    launches = max(kernels[dom]["launches_per_step"], 1)
    hbm_side = {"achieved_GBs": kernels[dom]["algorithmic_GBs"], "frac": round(kernels[dom]["algorithmic_GBs"] / HBM_PEAK_GBS, 4),
                "frac_of_measured_copy": round(kernels[dom]["algorithmic_GBs"] / cal["copy_GBs"], 4) if cal["copy_GBs"] else None,
                "algorithmic_bytes_per_launch": int(alg.get(dom, 0) / launches)}
    cnt = counters.get(counter_key(dom), {})
    if dom in flops:
        # the transform kernels are bound by the vector ALU, not by HBM (counters: 55-65 % of the issue slots busy,
        # a fifth of the HBM peak), so the roofline is the fp64 vector peak; the HBM reading stays beside it
        tf = kernels[dom]["algorithmic_TFLOPs"]
        roofline = {"kernel": dom, "bound": "alu", "achieved": tf, "peak": FP64_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tf / FP64_PEAK_TFLOPS, 4),
                    "peak_measured": round(fp64_measured, 2), "frac_of_measured": round(tf / fp64_measured, 4),
                    "algorithmic_flops_per_launch": int(flops[dom] / launches),
                    "valu_issue_busy": cnt.get("valu_issue_busy"), "hbm": hbm_side}
    else:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": hbm_side["achieved_GBs"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": hbm_side["frac"],
                    "peak_measured": round(cal["copy_GBs"], 1), "frac_of_measured": hbm_side["frac_of_measured_copy"],
                    "algorithmic_bytes_per_launch": hbm_side["algorithmic_bytes_per_launch"]}
    roofline["traffic"] = cnt.get("traffic")
    roofline["counters_from"] = counter_src
    roofline["avg_launch_us"] = kernels[dom]["avg_launch_us"]
    roofline["share_of_step"] = round(kernels[dom]["ms_per_step"] / sum(k["ms_per_step"] for k in kernels.values()), 3)
    for name, k in kernels.items():      # counter readings of every kernel of the step, where the summary has them
        c = counters.get(counter_key(name))
        if c:
            k["counters_per_launch"] = c
    staged, strict = staged_bytes_rot_left(N, L, K, alpha, dnum, L, B)
    per_ct_s = dt / (B * args.steps)
    rot = {"us_per_ct": round(per_ct_s * 1e6, 2),
           "staged_bytes_per_ct": int(staged), "strict_bytes_per_ct": int(strict),
           "staged_GBs": round(staged / per_ct_s / 1e9, 1), "frac_of_hbm_staged": round(staged / per_ct_s / 1e9 / HBM_PEAK_GBS, 4),
           "frac_of_hbm_strict": round(strict / per_ct_s / 1e9 / HBM_PEAK_GBS, 4),
           "frac_of_measured_copy_staged": round(staged / per_ct_s / 1e9 / cal["copy_GBs"], 4) if cal["copy_GBs"] else None}
    if counters:
        per_step = sum(c.get("traffic", 0) * kernels[n]["launches_per_step"] for n, c in counters.items() if n in kernels)
        rot["counter_bytes_per_ct"] = int(per_step / B)

    nets_out = None
    if not args.no_nets:
        nets_out = network_latencies()

    ops = {}
    if not args.no_ops:
        LP = 8 * N
        buf = torch.zeros((B * 2 * L, N), dtype=torch.int64, device="cuda")
        t = time_op(ctx, lambda: ctx.ntt_raw(buf, 0), 10)
        ops["ntt"] = {"ms": round(t * 1e3, 4), "polys": B * 2 * L, "GBs": round(2 * LP * B * 2 * L / t / 1e9, 1)}
        t = time_op(ctx, lambda: ctx.ntt_raw(buf, 0, inverse=True), 10)
        ops["intt"] = {"ms": round(t * 1e3, 4), "polys": B * 2 * L, "GBs": round(2 * LP * B * 2 * L / t / 1e9, 1)}
        del buf
        pt = ctx.encode([0.5] * 8, 2.0 ** 50, L)

        def free_all(xs):
            for x in xs:
                x.free()
        t = time_op(ctx, lambda: free_all(ctx.add_batch(cts, cts)), 10)
        ops["add"] = {"ms": round(t * 1e3, 4), "GBs": round(3 * 2 * L * LP * B / t / 1e9, 1)}
        t = time_op(ctx, lambda: free_all(ctx.mul_plain_batch(cts, pt)), 10)
        ops["mul_plain"] = {"ms": round(t * 1e3, 4), "GBs": round((4 * L * B + L) * LP / t / 1e9, 1)}

        def resc():
            tmp = ctx.add_batch(cts, cts)
            ctx.rescale_batch(tmp)
            free_all(tmp)
        t_add = ops["add"]["ms"] * 1e-3
        t = time_op(ctx, resc, 5) - t_add
        ops["rescale"] = {"ms": round(t * 1e3, 4), "GBs": round((2 * L + 2 * (L - 1)) * LP * B / t / 1e9, 1)}

        def relin():
            tmp = ctx.mul_no_relin_batch(cts, cts)
            ctx.relinearize_batch(tmp)
            free_all(tmp)
        t_mul = time_op(ctx, lambda: free_all(ctx.mul_no_relin_batch(cts, cts)), 5)
        ops["mul_no_relin"] = {"ms": round(t_mul * 1e3, 4), "GBs": round(7 * L * LP * B / t_mul / 1e9, 1)}
        t = time_op(ctx, relin, 5) - t_mul
        ops["relinearize"] = {"ms": round(t * 1e3, 4), "per_s": round(B / t, 1)}

        def hoisted():
            for row in ctx.rot_left_hoisted_batch(cts, rot_steps):
                for c in row:
                    c.free()
        t = time_op(ctx, hoisted, 5)
        ops["rot_left_hoisted_x3"] = {"ms": round(t * 1e3, 4), "per_s": round(3 * B / t, 1),
                                      "note": "three rotations of each ciphertext sharing one decomposition of c1"}

    # HBM traffic of the streaming primitives from the same counter summary, where it has them
    for op, kname in (("add", "addsub_kernel"), ("mul_plain", "mul_plain_kernel"), ("mul_no_relin", "mul_no_relin_kernel")):
        c = counters.get(kname, {})
        if op in ops and "traffic" in c:
            ops[op]["counter_bytes_per_launch"] = c["traffic"]
            ops[op]["counter_GBs"] = round(c["traffic"] / (ops[op]["ms"] * 1e-3) / 1e9, 1)

    base = None
    if args.cpu_sample > 0:
        base = cpu_baseline(log_n, q_bits, dnum, args.bits, 1, args.cpu_sample, rot_steps)

    print(json.dumps({
        # the benchmark's metric names two figures: `value` is the first, the network latencies are under `networks`
        "metric": "key-switched rotLeft/s at N=2^15 (batch 64); encrypted-network latency ms" if (log_n, B) == (15, 64) else
                  "key-switched rotLeft/s at N=2^%d (batch %d)" % (log_n, B),
        "value": round(value, 1), "unit": "rotLeft/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        # residues are 64-bit words below 2^50; the timed kernels do their modular arithmetic on them exactly in fp64
        "dtype": "f64" if all(b <= 50 for b in q_bits) and args.bits <= 50 and log_n >= 12 else "u64", "data": "synthetic",
        "config": {"workload": "primitive micro-benchmark: rotLeft over a batch of %d random ciphertexts, N=2^%d, "
                               "%d limbs of %d-bit primes, dnum %d, steps {1,7,64}" % (B, log_n, L, args.bits, dnum),
                   "log_n": log_n, "limbs": L, "dnum": dnum, "special_primes": K, "batch": B},
        "roofline": roofline, "rot_left": rot, "kernels": kernels, "calibration": {k: round(v, 3) if isinstance(v, float) else v for k, v in cal.items()},
        "ops": ops, "networks": nets_out,
        "cpu_baseline": base}))


if __name__ == "__main__":
    main()
