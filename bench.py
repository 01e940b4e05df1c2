#!/usr/bin/env python3
"""Benchmark of the integer-only CNN hot path on one MI355X.

A step is one pass of the whole ResNet-50-shaped integer network at batch 64
(every conv with its fused integer epilogue, the skip merges, both pools and
the fully connected layer) over synthetic inputs that already sit in HBM.
Prints one JSON line on stdout; per-layer detail goes to stderr and, with
--layers-json PATH, to that file.
"""
import argparse
import glob
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0     # MI355X dense int8 matrix-core peak, TOP/s
HBM_PEAK_GBS = 8000.0


WORKLOADS = {
    "cfg0": "cfg0: one 3x3 conv layer 1x56x56x64 -> 64",
    "cfg1": "cfg1: VDSR-shaped, 20 conv3x3 layers on one 256x256 luma plane",
    "cfg2": "cfg2: VRCNN-shaped, one 720x1280 luma plane, two concatenations",
    "cfg3": "cfg3: ResNet-50-shaped integer inference, batch 64, 3x224x224 uint8 input, 53 convs + FC, 16 skip merges "
            "(the 4 projection convs fused into their block's last conv)",
    "cfg4": "cfg4: ResNet-152-shaped integer inference, batch 128",
    "cfg5": "cfg5: ResNet-18-shaped (basic blocks) integer inference, batch 64",
    "cfg6": "cfg6: VRCNN-shaped, one 2560x1600 luma plane",
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def layer_work(net, op, images, fused_proj=None, fused_block=None, fused_pool=None, fused_pair=None, fused_projblock=None, fused_twin=None):
    """Algorithmic ops and bytes of one conv launch (true sizes, input counted once).  With a
    projection fused into the launch, its ops, input and weights are added and the int32 skip
    tensor is not counted (it never exists).  With a whole bottleneck block in the launch: the ops of its
    three layers (true sizes: the recomputed halo is not work), the block input once (it is also the skip
    operand), all weights and biases, the block output; the middle tensors are not counted (they never exist)."""
    if fused_projblock is not None:
        # a stage's opening block, projection included, in one launch: the ops of its four layers; the block input once (it
        # feeds the first layer and the projection), all weights, the output; neither middle tensor nor the int32 skip tensor
        o1, o2, proj = fused_projblock
        ops1, b1, m, k1 = layer_work(net, o1, images)
        ops2, b2, _, k2 = layer_work(net, o2, images)
        ops3, b3, _, k3 = layer_work(net, op, images, fused_proj=proj)
        mid = m * o1["cout"]
        x_bytes = images * net["buffers"][o1["src"]]["shape"][1] * net["buffers"][o1["src"]]["shape"][2] * o1["cin"]
        return ops1 + ops2 + ops3, (b1 - mid) + (b2 - 2 * mid) + (b3 - mid - x_bytes), m, k1 + k2 + k3
    if fused_twin is not None:
        # two branches of one input in one launch: both layers' ops, weights and outputs; the input once
        opsa, ba, m, ka = layer_work(net, op, images)
        opsb, bb, _, kb = layer_work(net, fused_twin, images)
        _, h, w, _ = net["buffers"][op["src"]]["shape"]
        return opsa + opsb, ba + bb - images * h * w * op["cin"], m, ka + kb
    if fused_pair is not None:
        # two pointwise layers in one launch: both layers' ops; the first layer's input, skip operand and output, both
        # layers' weights, the second layer's output (the second layer's input is not read back from memory)
        ops3, b3, m, k3 = layer_work(net, op, images)
        ops1, b1, _, k1 = layer_work(net, fused_pair, images)
        return ops3 + ops1, b3 + b1 - m * op["cout"], m, k3 + k1
    if fused_pool is not None:
        # convolution and the max-pool behind it in one launch: the convolution's ops; the picture, the weights and the
        # pooled tensor as bytes (the convolution's own output never exists)
        ops, byts, m, k = layer_work(net, op, images)
        pn, ph, pw, pc = net["buffers"][fused_pool["dst"]]["shape"]
        return ops, byts - m * op["cout"] + images * ph * pw * pc, m, k
    if fused_block is not None:
        o1, o2 = fused_block
        ops1, b1, m, k1 = layer_work(net, o1, images)
        ops2, b2, _, k2 = layer_work(net, o2, images)
        ops3, b3, _, k3 = layer_work(net, dict(op, res=None), images)
        mid = m * o1["cout"]
        return ops1 + ops2 + ops3, (b1 - mid) + (b2 - 2 * mid) + (b3 - mid), m, k1 + k2 + k3
    if fused_proj is not None:
        main = dict(op, res=None)
        o1, b1, m, k1 = layer_work(net, main, images)
        proj = dict(fused_proj, out_mode="brelu")
        o2, b2, _, k2 = layer_work(net, proj, images)
        return o1 + o2, b1 + b2 - m * op["cout"], m, k1 + k2
    n, ho, wo, _ = net["buffers"][op["dst"]]["shape"]
    _, h, w, _ = net["buffers"][op["src"]]["shape"]
    n = images
    m = n * ho * wo
    k = op["kh"] * op["kw"] * op["cin"]
    ops = 2.0 * m * op["cout"] * k
    out_b = 4 if op["out_mode"] == "raw_s32" else 1
    byts = n * h * w * op["cin"] + k * op["cout"] + 4 * op["cout"] + m * op["cout"] * out_b
    if op["res"] is not None:
        byts += m * op["cout"] * (4 if op["res_dtype"] == "s32" else 1)
    return ops, byts, m, k


def cpu_baseline(net, calib, seed, budget_s=20.0):
    """The oracle as it stands, timed on this host: images/s on a bounded sample."""
    from oracle import net as ONet
    from oracle import oracle as O
    from workloads import nets as W
    n_all = net["buffers"]["raw"]["shape"][0]
    x = W.input_tensor(net, seed, n_all)
    t0 = time.time()
    ONet.run(net, seed, calib, images=2, x_raw=x[:2])
    t1 = (time.time() - t0) / 2
    k = int(max(1, min(n_all, budget_s // max(t1, 1e-3))))
    t0 = time.time()
    passes = 0
    while passes == 0 or (time.time() - t0 < 10.0 and passes < 100):      # at least about ten seconds of work
        ONet.run(net, seed, calib, images=k, x_raw=x[:k])
        passes += 1
    dt = time.time() - t0
    return {"value": passes * k / dt, "unit": "images/s", "cores": O.num_threads(), "kind": "oracle",
            "sample": "%d of the %d images of the same batch, every layer of the network, %d pass%s, %.1f s" % (
                k, n_all, passes, "" if passes == 1 else "es", dt)}


def csrc_digest():
    """Hash of the kernel sources: a byte-counter summary under profiles/ is only valid for the build it was taken on."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2006_11735_amd", "csrc", "*"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


def _time_us(torch, fns, reps=20):
    """Average duration of a call.  fns: one callable, or several that are called in turn (the same kernel on
    different buffers, so that no call finds its operands in the 256 MB last-level cache)."""
    if callable(fns):
        fns = [fns]
    for f in fns[:3]:
        f()
    reps = max(reps, len(fns))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(reps):
        fns[i % len(fns)]()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e3


COLD_BYTES = 1.5e9      # buffer sets a cold measurement rotates over: well beyond the 256 MB last-level cache


def _sets(bytes_per_set):
    return max(2, int(COLD_BYTES // bytes_per_set) + 1)


def measured_peaks(torch):
    """The two roofs as this machine delivers them: a register-only loop of the int8 matrix instruction and a
    streaming device copy of 1 GiB (read + written bytes over time)."""
    from paper_2006_11735_amd import binding as B
    blocks, iters = 256 * 8, 4000
    sink = torch.empty(blocks * 256, dtype=torch.int32, device="cuda")
    us = _time_us(torch, lambda: B.icnn_peak_mfma_i8(blocks, iters, sink), reps=5)
    tops = blocks * 4 * iters * 8 * 65536 / us / 1e6
    n = 1 << 30
    src = torch.zeros(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    us_c = _time_us(torch, lambda: B.icnn_peak_copy(src, dst, n), reps=5)
    gbs = 2 * n / us_c / 1e3
    log("measured roofs: int8 MFMA loop %.0f TOP/s (%.1f%% of nominal), 1 GiB copy %.0f GB/s (%.1f%% of nominal)" % (
        tops, 100 * tops / INT8_MFMA_PEAK_TOPS, gbs, 100 * gbs / HBM_PEAK_GBS))
    del src, dst
    return tops, gbs


def add_bandwidth(torch, copy_gbs):
    """Achieved bandwidth of the stand-alone rescaled addition (3 and 6 bytes per element): cold = every call on
    buffers no earlier call left in the last-level cache (the HBM figure); warm = one buffer set back to back."""
    from paper_2006_11735_amd import binding as B
    px, c = 64 * 56 * 56, 256
    out = {}
    for name, a_dt, a_torch, bytes_per in (("u8+u8->u8", B.ICNN_U8, torch.uint8, 3), ("s32+u8->u8", B.ICNN_S32, torch.int32, 6)):
        d = B.add_desc(count_pixels=px, c=c, a_c_stride=c, b_c_stride=c, out_c_stride=c, a_dtype=a_dt,
                       b_dtype=B.ICNN_U8, b_mul=18415, b_shift=5 if a_dt == B.ICNN_S32 else 14, mul=23187,
                       shift=24 if a_dt == B.ICNN_S32 else 15, lo=0, hi=127)   # 8-bit maps: ratios near 1; accumulators: << 1
        sets = []
        for _ in range(_sets(px * c * bytes_per)):
            a = torch.randint(0, 100, (px, c), device="cuda").to(a_torch)
            b = torch.randint(0, 127, (px, c), device="cuda").to(torch.uint8)
            o = torch.empty((px, c), dtype=torch.uint8, device="cuda")
            sets.append((a, b, o))
        fns = [(lambda t=t: B.iadd_rescale(d, t[0], t[1], t[2])) for t in sets]
        us = _time_us(torch, fns, reps=3 * len(fns))
        us_warm = _time_us(torch, fns[0])
        gbs, gbs_warm = px * c * bytes_per / us / 1e3, px * c * bytes_per / us_warm / 1e3
        out[name] = {"elements": px * c, "us": us, "achieved_gbs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS,
                     "frac_of_measured_copy": gbs / copy_gbs, "buffer_sets": len(fns),
                     "warm_us": us_warm, "warm_gbs_cache_assisted": gbs_warm}
        log("iadd_rescale %-11s %d elements: cold %.1f us, %.0f GB/s (%.0f%% of %d GB/s, %.0f%% of the measured copy); "
            "warm (cache-assisted) %.1f us, %.0f GB/s" % (name, px * c, us, gbs, 100 * gbs / HBM_PEAK_GBS, HBM_PEAK_GBS,
                                                         100 * gbs / copy_gbs, us_warm, gbs_warm))
        del sets, fns
    return out


def other_bandwidth(torch, copy_gbs):
    """Achieved bandwidth (algorithmic bytes / time) of the remaining memory-bound kernels at the sizes they have in
    the workloads, cold (rotating over buffer sets larger than the last-level cache) and warm."""
    from paper_2006_11735_amd import binding as B
    out = {}

    def report(name, byts, make):
        sets = [make() for _ in range(_sets(byts))]
        fns = [s_ for s_ in sets]
        us = _time_us(torch, fns, reps=3 * len(fns))
        us_warm = _time_us(torch, fns[0])
        gbs = byts / us / 1e3
        out[name] = {"algorithmic_bytes": byts, "us": us, "achieved_gbs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS,
                     "frac_of_measured_copy": gbs / copy_gbs, "buffer_sets": len(fns), "warm_us": us_warm,
                     "warm_gbs_cache_assisted": byts / us_warm / 1e3}
        log("%-38s %6.1f MB: cold %6.1f us, %5.0f GB/s (%.0f%% of %d GB/s, %.0f%% of the measured copy); warm %6.1f us" % (
            name, byts / 1e6, us, gbs, 100 * gbs / HBM_PEAK_GBS, HBM_PEAK_GBS, 100 * gbs / copy_gbs, us_warm))

    for label, nb in (("64x112x112x64 3x3/2", 64), ("256x112x112x64 3x3/2 (257 MB)", 256)):
        def maxpool():
            x = torch.randint(0, 128, (nb, 112, 112, 64), device="cuda").to(torch.uint8)
            o = torch.empty((nb, 56, 56, 64), dtype=torch.uint8, device="cuda")
            return lambda: B.imaxpool2d_u8(nb, 112, 112, 64, 3, 2, 1, x, o)
        report("imaxpool2d_u8 " + label, nb * 112 * 112 * 64 + nb * 56 * 56 * 64, maxpool)

    def avgpool():
        x = torch.randint(0, 128, (64, 7, 7, 2048), device="cuda").to(torch.uint8)
        o = torch.empty((64, 1, 1, 2048), dtype=torch.uint8, device="cuda")
        return lambda: B.iavgpool_global_u8(64, 7, 7, 2048, 21400, 20, 127, x, o)
    report("iavgpool_global_u8 64x7x7x2048", 64 * 49 * 2048 + 64 * 2048, avgpool)
    for label, px in (("720x1280", 720 * 1280), ("2560x1600 (393 MB)", 2560 * 1600)):
        def concat():
            a = torch.randint(0, 128, (px, 32), device="cuda").to(torch.uint8)
            b = torch.randint(0, 128, (px, 16), device="cuda").to(torch.uint8)
            o = torch.empty((px, 48), dtype=torch.uint8, device="cuda")
            return lambda: B.iconcat([a, b], [32, 16], [32, 16], [20000, 23000], [15, 15], 127, px, o, 48)
        report("iconcat %s 32+16 channels" % label, 2 * px * 48, concat)
    for label, n in (("64x224x224x3", 64 * 224 * 224 * 3), ("128x224x224x3 x4 (77 MB)", 4 * 128 * 224 * 224 * 3)):
        def renorm():
            x = torch.randint(0, 256, (n,), device="cuda").to(torch.uint8)
            o = torch.empty_like(x)
            return lambda: B.irenormalize_u8(n, x, o)
        report("irenormalize_u8 " + label, 2 * n, renorm)
    return out


def summarise_pmc(config, fetch_csv, write_csv):
    """HBM bytes per conv launch from two rocprofv3 --pmc runs.  The counters are in KiB per dispatch; each is scaled
    by what it reads for stream_copy_kernel on 256 MiB (262144 KiB read, 262144 KiB written)."""
    import collections
    import csv

    def load(path):
        agg = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            agg[r["Kernel_Name"].split("(")[0]].append(float(r["Counter_Value"]))
        return agg
    f, w = load(fetch_csv), load(write_csv)
    scale = {}
    for name, agg in (("fetch", f), ("write", w)):
        ref = [v for k, vs in agg.items() if "stream_copy_kernel" in k for v in vs]
        if not ref:
            sys.exit("no stream_copy_kernel dispatch in the %s run: was --copy-calibration given?" % name)
        ref = [v for v in ref if v < 1.5 * min(ref)]      # the 256 MiB calibration copies, not the 1 GiB copies of the roof measurement
        scale[name] = 262144.0 / (sum(ref) / len(ref))
    per_pass = {k: len(v) for k, v in f.items() if "maxpool" in k or "avgpool" in k}
    passes = min(per_pass.values()) if per_pass else 1
    # launches outside the passes (the fused block's warm-up launch at set-up) come first: drop them
    for agg in (f, w):
        for k in list(agg):
            if "conv_" in k and len(agg[k]) % passes:
                agg[k] = agg[k][len(agg[k]) % passes:]
    conv_f = sum(sum(v) for k, v in f.items() if "conv_" in k)
    conv_w = sum(sum(v) for k, v in w.items() if "conv_" in k)
    n_f = sum(len(v) for k, v in f.items() if "conv_" in k)
    rd, wr = conv_f * 1024 * scale["fetch"] / passes, conv_w * 1024 * scale["write"] / passes
    out = {"conv_hbm_bytes_per_launch": (rd + wr) / (n_f / passes), "conv_hbm_read_bytes_per_step": rd,
           "conv_hbm_write_bytes_per_step": wr, "conv_launches_per_step": n_f / passes,
           "fetch_size_scale": scale["fetch"], "write_size_scale": scale["write"], "csrc_digest": csrc_digest(),
           "kernels_kib_per_dispatch": {k: [len(f[k]), sum(f[k]) / len(f[k]), sum(w.get(k, [0])) / max(1, len(w.get(k, [0])))]
                                        for k in sorted(f) if any(t in k for t in ("conv_", "pool", "pad_", "stream_copy"))}}
    path = os.path.join(ROOT, "profiles", "traffic_%s.json" % config)
    json.dump(out, open(path, "w"), indent=1)
    print(json.dumps(out, indent=1))
    print("written", path)


def summarise_trace(stats_csv, passes):
    """No GPU work: the library's kernels out of a rocprofv3 --kernel-trace --stats `*_kernel_stats.csv`, as a
    markdown table (calls per pass of the network, average duration, time per pass, share of the library's time)."""
    import csv
    rows = []
    for r in csv.DictReader(open(stats_csv)):
        name = r["Name"]
        if "icnn::" not in name:
            continue
        short = name.replace("void ", "").replace("icnn::", "").split("(")[0]
        rows.append((short, int(r["Calls"]), float(r["TotalDurationNs"]), float(r["AverageNs"])))
    total = sum(t for _, _, t, _ in rows)
    print("| kernel | calls | calls/pass | avg us | ms/pass | % of the library's GPU time |")
    print("|---|---|---|---|---|---|")
    for short, calls, t, avg in sorted(rows, key=lambda x: -x[2]):
        print("| %s | %d | %.1f | %.2f | %.4f | %.2f |" % (short, calls, calls / passes, avg / 1e3, t / passes / 1e6, 100 * t / total))
    conv = [(c, t) for s_, c, t, _ in rows if s_.startswith("conv_") and "prepack" not in s_]
    nc, tc = sum(c for c, _ in conv), sum(t for _, t in conv)
    print()
    if nc:
        print("conv kernels (names starting conv_): %d calls, %.1f per pass, average %.2f us, %.4f ms per pass" % (
        nc, nc / passes, tc / nc / 1e3, tc / passes / 1e6))


def summarise_mfma(counter_csv):
    """No GPU work: matrix-core utilisation per kernel out of one rocprofv3 --pmc run that collected
    SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE SQ_INSTS_VALU_MFMA_MOPS_I8
    (`*_counter_collection.csv`), as a markdown table.  MFMA-busy cycles are summed over the chip's 1024 SIMDs; they are
    set against (a) the dispatch's duration from its timestamps at the nominal 2.4 GHz and (b) GRBM_GUI_ACTIVE (summed
    over the 8 XCCs, hence / 8), which under the profiler also covers the idle time around a short dispatch.
    SQ_INSTS_VALU_MFMA_MOPS_I8 x 512 = executed int8 operations (padding included)."""
    import collections
    import csv
    per = collections.defaultdict(lambda: collections.defaultdict(float))
    calls = collections.Counter()
    dur = collections.defaultdict(float)
    seen = set()
    for r in csv.DictReader(open(counter_csv)):
        name = r["Kernel_Name"]
        if "icnn::" not in name:
            continue
        short = name.replace("void ", "").replace("icnn::", "").split("(")[0]
        per[short][r["Counter_Name"]] += float(r["Counter_Value"])
        if r["Dispatch_Id"] not in seen:
            seen.add(r["Dispatch_Id"])
            calls[short] += 1
            dur[short] += float(r["End_Timestamp"]) - float(r["Start_Timestamp"])
    print("| kernel | dispatches | avg us (under the profiler) | executed int8 TOP/s | MFMA busy % of duration x 2.4 GHz | MFMA busy % of GPU-active cycles |")
    print("|---|---|---|---|---|---|")
    tot = collections.defaultdict(float)
    tot_dur = 0.0
    for short in sorted(per, key=lambda k: -dur[k]):
        c = per[short]
        act = c["GRBM_GUI_ACTIVE"] / 8
        if act <= 0 or dur[short] <= 0:
            continue
        busy = c["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024
        print("| %s | %d | %.2f | %.0f | %.1f | %.1f |" % (
            short, calls[short], dur[short] / calls[short] / 1e3, c["SQ_INSTS_VALU_MFMA_MOPS_I8"] * 512 / dur[short] / 1e3,
            100 * busy / (dur[short] * 2.4), 100 * busy / act))
        if short.startswith("conv_") and "prepack" not in short:
            for k, v in c.items():
                tot[k] += v
            tot_dur += dur[short]
    if tot_dur:
        busy = tot["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024
        print()
        print("all conv kernels: executed %.0f int8 TOP/s over their durations; MFMA busy %.1f %% of duration x 2.4 GHz, %.1f %% of "
              "GPU-active cycles" % (tot["SQ_INSTS_VALU_MFMA_MOPS_I8"] * 512 / tot_dur / 1e3, 100 * busy / (tot_dur * 2.4),
                                     100 * busy / (tot["GRBM_GUI_ACTIVE"] / 8)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="cfg3", help="workload (cfg3 = ResNet-50-shaped, batch 64)")
    ap.add_argument("--summarise-mfma", metavar="COUNTER_CSV", default=None,
                    help="no GPU work: matrix-core utilisation per kernel from a rocprofv3 --pmc counter file")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers-json", default=None, help="also write the per-layer table to this file")
    ap.add_argument("--layer-reps", type=int, default=20)
    ap.add_argument("--per-channel", action="store_true",
                    help="time the variant with one (mul, shift) per output channel instead of the per-layer workload")
    ap.add_argument("--main-only", action="store_true",
                    help="skip the per-channel variant and the stand-alone bandwidth kernels (clean kernel traces)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 256 MiB device copies (stream_copy_kernel: reference for rocprofv3 byte counters)")
    ap.add_argument("--summarise-pmc", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"), default=None,
                    help="no GPU work: turn the counter_collection.csv files of two rocprofv3 --pmc runs of "
                         "`bench.py --copy-calibration --main-only` (FETCH_SIZE, then WRITE_SIZE) into profiles/traffic_<config>.json")
    ap.add_argument("--summarise-trace", nargs=2, metavar=("STATS_CSV", "PASSES"), default=None,
                    help="no GPU work: the library's kernels of a rocprofv3 --kernel-trace --stats kernel_stats.csv as a markdown "
                         "table; PASSES = passes of the network in the profiled process")
    args = ap.parse_args()
    if args.summarise_mfma:
        return summarise_mfma(args.summarise_mfma)
    if args.summarise_trace:
        return summarise_trace(args.summarise_trace[0], float(args.summarise_trace[1]))
    if args.summarise_pmc:
        return summarise_pmc(args.config, *args.summarise_pmc)
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    from paper_2006_11735_amd.netrun import GpuNet
    from workloads import nets as W
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU (there is no CPU fallback)")
    torch.cuda.set_device(0)

    net = W.CONFIGS[args.config]()
    seed = 0
    calib_path = os.path.join(ROOT, "workloads", "calib", "%s_seed%d.json" % (args.config, seed))
    pc_path = calib_path.replace(".json", "_pc.json")
    if args.per_channel:
        calib_path = pc_path
    calib = json.load(open(calib_path))
    images = net["buffers"]["raw"]["shape"][0]
    g = GpuNet(net, seed, calib)
    g.set_input()
    torch.cuda.synchronize()

    if args.copy_calibration:
        from paper_2006_11735_amd import binding as B
        src = torch.zeros(1 << 28, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            B.icnn_peak_copy(src, dst, 1 << 28)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        g.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g.run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # ---- per-launch durations, measured with HIP events on the launch stream, in network
    # order (so each layer sees the cache state its producer left behind)
    nsteps = len(g.steps)
    reps = max(1, args.layer_reps)
    acc = [0.0] * nsteps
    for _ in range(reps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(nsteps + 1)]
        ev[0].record()
        for i in range(nsteps):
            g.run_step(i)
            ev[i + 1].record()
        torch.cuda.synchronize()
        for i in range(nsteps):
            acc[i] += ev[i].elapsed_time(ev[i + 1])
    layer_ms = [a / reps for a in acc]
    # an event between two launches costs a little stream time itself: the per-launch intervals add
    # up to more than the step measured above without events; spread that excess evenly
    excess = max(0.0, (sum(layer_ms) - ms_per_step) / nsteps)
    layer_ms = [max(m - excess, 1e-4) for m in layer_ms]

    conv_ops = conv_ms = conv_bytes = 0.0
    other_ms = 0.0
    rows = []
    for step, ms in zip(g.steps, layer_ms):
        kind, op = step[0], step[1]
        if kind not in ("conv", "conv_pc", "dual", "dual_pc", "block", "convpool", "pair", "projblock", "twin"):
            other_ms += ms
            rows.append({"name": op["dst"], "kind": kind, "ms": ms})
            continue
        ops, byts, m, k = layer_work(net, op, images, g.fused_proj.get(op["name"]) if kind in ("dual", "dual_pc") else None,
                                     g.fused_block.get(op["name"]) if kind == "block" else None,
                                     g.fused_pool.get(op["name"]) if kind == "convpool" else None,
                                     g.fused_pair.get(op["name"]) if kind == "pair" else None,
                                     g.fused_projblock.get(op["name"]) if kind == "projblock" else None,
                                     g.fused_twin.get(op["name"]) if kind == "twin" else None)
        conv_ops += ops
        conv_ms += ms
        conv_bytes += byts
        tops = ops / (ms * 1e-3) / 1e12
        attain = min(INT8_MFMA_PEAK_TOPS, ops / byts * HBM_PEAK_GBS / 1e3)
        rows.append({"name": (op["name"][:-3] + "_block" if kind == "block" else op["name"]) + ("+proj" if kind in ("dual", "dual_pc") else "") +
                             ("+pool" if kind == "convpool" else "") + ("+next_c1" if kind == "pair" else "") + ("+" + g.fused_twin[op["name"]]["name"] if kind == "twin" else "") + ("_block+proj" if kind == "projblock" else ""), "kind": "conv", "M": m, "N": op["cout"] + (g.fused_twin[op["name"]]["cout"] if kind == "twin" else 0), "K": k, "ms": ms,
                     "tops": tops, "pct_mfma_peak": 100 * tops / INT8_MFMA_PEAK_TOPS,
                     "pct_attainable": 100 * tops / attain, "gbs": byts / (ms * 1e-3) / 1e9})
    for r in rows:
        if r["kind"] == "conv":
            log("%-12s M=%-7d N=%-5d K=%-5d %8.1f us %7.1f TOP/s %5.1f%% peak %5.1f%% attainable %7.0f GB/s" % (
                r["name"], r["M"], r["N"], r["K"], r["ms"] * 1e3, r["tops"], r["pct_mfma_peak"],
                r["pct_attainable"], r["gbs"]))
        else:
            log("%-12s %-8s %8.1f us" % (r["name"], r["kind"], r["ms"] * 1e3))
    conv_tops = conv_ops / (conv_ms * 1e-3) / 1e12
    n_conv = sum(1 for r in rows if r["kind"] == "conv")
    log("conv launches: %d, %.3f ms per step (events, excess %.2f us/launch removed; whole step %.3f ms wall), %.1f TOP/s" % (
        n_conv, conv_ms, excess * 1e3, ms_per_step, conv_tops))

    traffic, traffic_stale = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % args.config)
    if os.path.exists(tpath):          # HBM bytes per conv launch from the committed rocprofv3 --pmc summary
        tj = json.load(open(tpath))
        traffic = tj.get("conv_hbm_bytes_per_launch")
        traffic_stale = tj.get("csrc_digest") != csrc_digest()     # counters were taken on other kernel sources
        if traffic_stale:
            log("note: %s was measured on other kernel sources than this build (traffic_stale)" % tpath)

    peak_tops, copy_gbs = measured_peaks(torch)

    result = {
        "metric": "images/s ResNet-50-shaped b64 (int8 conv TOPS and % of int8 MFMA peak alongside)" if args.config == "cfg3"
                  else "images/s (int8 conv TOPS and % of int8 MFMA peak alongside)",
        "value": images / (ms_per_step * 1e-3),
        "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": WORKLOADS.get(args.config, args.config) + ", stored oracle-side calibration (seed 0)",
                   "batch": images},
        "conv_tops": conv_tops,
        "pct_int8_mfma_peak": 100 * conv_tops / INT8_MFMA_PEAK_TOPS,
        "whole_step_tops": conv_ops / (ms_per_step * 1e-3) / 1e12,
        "roofline": {"kernel": "conv kernels (all %d conv launches of a step: conv_dlds / conv_halo / conv_deep / conv_plane / conv_pic / conv_narrow / conv_dual / conv_block / conv_block64 / conv_pair / conv_stem_pool, every tile shape)" % n_conv,
                     "bound": "mfma", "achieved": conv_tops, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": conv_tops / INT8_MFMA_PEAK_TOPS, "traffic": traffic, "traffic_stale": traffic_stale,
                     "peak_measured": peak_tops, "frac_of_peak_measured": conv_tops / peak_tops,
                     "launches_per_step": n_conv, "avg_launch_us": conv_ms * 1e3 / n_conv,
                     "algorithmic_gop_per_step": conv_ops / 1e9,
                     "algorithmic_gb_per_step": conv_bytes / 1e9},
    }
    if not args.main_only:
        # Throughput with two steps in flight: consecutive steps are independent batches, so a second set of activation
        # buffers (same weights' values, its own copies) and a second stream let one step's small launches fill the
        # compute units another step's leave idle.  Reported beside the headline figure, which stays one step at a time.
        g2 = GpuNet(net, seed, calib)
        g2.set_input()
        pair = [g, g2]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()

        def pipelined(k):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(k):
                with torch.cuda.stream(streams[i & 1]):
                    pair[i & 1].run()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / k * 1e3
        pipelined(2 * max(2, args.warmup))
        ms2 = pipelined(2 * ((args.steps + 1) // 2))
        out_name = net["outputs"][0]
        same = bool(torch.equal(g.buf[out_name], g2.buf[out_name]))
        result["two_steps_in_flight"] = {"ms_per_step": ms2, "images_per_s": images / (ms2 * 1e-3), "streams": 2,
                                         "whole_step_tops": conv_ops / (ms2 * 1e-3) / 1e12, "outputs_identical": same,
                                         "note": "the same steps issued alternately on two streams over two sets of activation "
                                                 "buffers; not the headline value"}
        log("two steps in flight (two streams): %.3f ms per step, %.0f images/s, outputs identical: %s" % (
            ms2, images / (ms2 * 1e-3), same))
        del g2, pair
    if args.per_channel:
        result["config"]["workload"] += "; per-output-channel requantisation (iconv2d_brelu_pc, iconv2d_dual_brelu_pc)"
    elif os.path.exists(pc_path) and args.config == "cfg3" and not args.main_only:
        # the same network with one (mul, shift) and skip rescale per output channel, on both stored calibrations:
        # channels without a positive calibration value keep the layer's pair ("layer"), or get the wide pair of
        # their own statistic ("own": parameters that no kernel's fast form had a say in)
        variants = {}
        for label, path in (("layer", pc_path), ("own", pc_path.replace("_pc.json", "_pc_own.json"))):
            if not os.path.exists(path):
                continue
            g_pc = GpuNet(net, seed, json.load(open(path)))
            g_pc.set_input()
            for _ in range(5):
                g_pc.run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(30):
                g_pc.run()
            torch.cuda.synchronize()
            ms_pc = (time.perf_counter() - t0) / 30 * 1e3
            variants[label] = {"ms_per_step": ms_pc, "images_per_s": images / (ms_pc * 1e-3), "launches_per_step": len(g_pc.steps),
                               "calibration": os.path.relpath(path, ROOT)}
            log("per-channel variant (%s): %.3f ms per step (%d launches)" % (label, ms_pc, len(g_pc.steps)))
            del g_pc
        result["per_channel_variant"] = dict(variants.get("layer", {}), floor_channels_own=variants.get("own"),
                                             note="iconv2d_brelu_pc on every BReLU layer, iconv2d_dual_brelu_pc on the four "
                                                  "projection blocks; the top-level figures are for the calibration in which a "
                                                  "channel without a positive calibration value keeps the layer's pair, "
                                                  "floor_channels_own for the one in which it gets the pair of its own statistic")
    result["hbm_copy_measured_gbs"] = copy_gbs
    if not args.main_only:
        del g
        torch.cuda.empty_cache()
        result["iadd_rescale"] = add_bandwidth(torch, copy_gbs)
        result["bandwidth_kernels"] = other_bandwidth(torch, copy_gbs)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(net, calib, seed)
    if args.layers_json:
        with open(args.layers_json, "w") as f:
            json.dump({"result": result, "layers": rows}, f, indent=1)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
