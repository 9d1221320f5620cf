#!/usr/bin/env python3
"""Benchmark of the compressed-collective hot path on one MI355X.

One step = one pass of the whole path over one message buffer, as a rank in a
compressed ring all-reduce performs it (Sec. IV-A):
    zc_compress(local gradients)            fp32 -> stream
    zc_reduce_compressed([incoming, local]) decompress + add + recompress, fused
    zc_decompress(result)                   stream -> fp32
Headline workload: the data-parallel gradient bucket (2^28 fp32 values with low-rank
structure, rate 4), synthetic and seeded, resident in HBM before timing starts.
`value` is GB/s of uncompressed fp32 pushed through the whole step (4*n / step time).

The same JSON line carries, under `configs`, every kernel on all five workloads
(compress, decompress, 2-way reduce; the ring share as the chain of seven 2-way
reduces plus the final decompress, and as one 8-way reduce), under `error_per_rate`
the round-trip error at every rate, and under `copy_GBps` a timed 1 GiB device copy
(the attainable memory rate on this machine).

Prints ONE JSON line on stdout.
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0                       # MI355X HBM3E, published
INT_ALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12  # 256 CUs x 64 lanes x 2.4 GHz, one int32 op per lane-clock
LLC_BYTES = 256 << 20                       # last-level cache: working sets below this are rotated

HERE = os.path.dirname(os.path.abspath(__file__))
PROFILE = os.path.join(HERE, "profiles", "zc_rate4_gradient_bucket.md")
# the kernels behind the three calls of the headline step at rate 4 (names as rocprofv3 prints them)
KERNEL_NAMES = {"compress": "compress4_wide_kernel<0>", "decompress": "decompress4_wide_kernel<0>",
                "reduce": "reduce_kernel<4, 4, false, false, 2>"}


def profiled_counters(path=PROFILE):
    """HBM bytes per launch and wave-level VALU instructions per launch of the headline
    kernels, read from the rocprofv3 summary of this same workload under profiles/
    (its tables 'Counters' and 'HBM traffic per launch after scaling')."""
    out = {}
    try:
        text = open(path).read()
    except OSError:
        return out
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) < 5 or cells[0] in ("kernel", "---"):
            continue
        entry = out.setdefault(cells[0], {})
        if len(cells) == 6 and re.fullmatch(r"\d+", cells[3] or "") and re.fullmatch(r"\d+", cells[4] or ""):
            entry["traffic_bytes"] = int(cells[3])          # read MiB | written MiB | total bytes | algorithmic | VALU/block
        elif len(cells) >= 12:
            try:
                entry["valu_wave_insts"] = float(cells[4])   # FETCH | WRITE | WAVES | INSTS_VALU | ...
            except ValueError:
                pass
    return out


def algorithmic_bytes(kernel, n, rate, k=2):
    """Bytes the method itself must move per launch: 4 + R/8 per value for
    compress and decompress, (k + 1) * R/8 per value for the k-way reduce."""
    if kernel in ("compress", "decompress"):
        return n * 4 + n * rate // 8
    return (k + 1) * (n * rate // 8)


SETTLE_MS = 60.0   # untimed launches before a kernel is timed on its own (see time_events)


def time_events(fn, reps, torch, skip=0, settle_ms=SETTLE_MS, batch_ms=0.6):
    """Per-launch durations (ms) measured with HIP events on the launch stream; fn gets the
    iteration number.  Before timing, fn is launched untimed for `settle_ms` of wall time:
    back-to-back launches of one kernel go through a clock transient on this GPU (the same
    launch takes up to 40 % longer between about 3 and 15 ms after the load starts, then
    settles), so a kernel timed on its own is timed in its settled state.  An event pair
    costs several microseconds on the stream, so short launches are timed in batches of
    back-to-back launches that last about `batch_ms` between one pair of events; each of
    the `reps` figures returned is a batch's time divided by its launches."""
    i = 0
    per_launch_ms = None
    t0 = time.perf_counter()
    while settle_ms > 0 and (time.perf_counter() - t0) * 1e3 < settle_ms:
        t1 = time.perf_counter()
        for _ in range(10):
            fn(i)
            i += 1
        torch.cuda.synchronize()
        per_launch_ms = (time.perf_counter() - t1) * 1e3 / 10
    batch = 1 if not per_launch_ms else int(min(64, max(1, round(batch_ms / per_launch_ms))))
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        for _ in range(batch):
            fn(i)
            i += 1
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) / batch for a, b in evs][skip:]


def frac(nbytes, ms):
    return round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)


def cpu_baseline(x_host, rate, sample_values, threads):
    """The CPU reference, as it stands, on the first `sample_values` values: the
    same three calls as one GPU step.  Blocks are independent, so `threads`
    workers each take a contiguous run of blocks."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import zc_ref
    n = min(sample_values, x_host.size) // 4 * 4
    xs = x_host[:n]
    peer = np.ascontiguousarray(xs[::-1])

    def work(part):
        cp = zc_ref.compress(part[1], rate)  # the incoming chunk (not timed as part of the step)
        t0 = time.perf_counter()
        c = zc_ref.compress(part[0], rate)
        r = zc_ref.reduce_compressed([cp, c], part[0].size, rate)
        zc_ref.decompress(r, part[0].size, rate)
        return time.perf_counter() - t0

    def run(nthreads):
        bounds = [(n // 4 * i // nthreads) * 4 for i in range(nthreads + 1)]
        parts = [(xs[a:b], peer[a:b]) for a, b in zip(bounds[:-1], bounds[1:])]
        if nthreads == 1:
            inner = [work(parts[0])]
        else:
            with ThreadPoolExecutor(nthreads) as ex:
                inner = list(ex.map(work, parts))
        # the untimed pre-compression of the incoming chunk is excluded via the inner clocks
        return max(inner)

    t1 = run(1)
    out = {"value": round(4 * n / t1 / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": "first %d values of the workload buffer, same three calls as one step" % n}
    if threads > 1:
        tn = run(threads)
        out["all_cores"] = {"value": round(4 * n / tn / 1e9, 4), "cores": threads}
    return out


def error_stats(torch, back, x):
    err = (back - x).double()
    return {"max_abs": float("%.4g" % float(err.abs().max())), "rmse": float("%.4g" % float(err.pow(2).mean().sqrt()))}


def measure_copy(torch, x, y, reps=8):
    """A plain device-to-device copy of the 1 GiB buffer: bytes read + written per second."""
    ms = float(np.median(time_events(lambda i: y.copy_(x), reps, torch)))
    return round(2 * x.numel() * x.element_size() / (ms * 1e-3) / 1e9, 1)


def config_table(torch, zc, workloads, dev, reps=20):
    """compress / decompress / 2-way reduce on each of the five workloads with the library
    as it is.  Buffers whose working set would fit the 256 MB last-level cache are rotated
    through enough copies that every launch reads from and writes to HBM; the ring share is
    reported both ways and says which."""
    out = {}
    for config in (1, 3, 4):
        rate = workloads.CONFIGS[config]["rate"]
        entries = {}
        for label, b in workloads.config_buffers(config):
            n = b.size
            per_set = 4 * n + n * rate // 8
            copies = int(min(96, max(2, np.ceil(1.6 * LLC_BYTES / per_set))))
            x0 = torch.from_numpy(b).to(dev)
            xs = [x0] + [x0.clone() for _ in range(copies - 1)]
            cs = [zc.zc_compress(x, rate) for x in xs]
            rs = [torch.empty_like(c) for c in cs]
            ys = [torch.empty_like(x) for x in xs]
            m = len(xs)
            tc = time_events(lambda i: zc.zc_compress(xs[i % m], rate, d_out=cs[i % m]), reps, torch)
            td = time_events(lambda i: zc.zc_decompress(cs[i % m], n, rate, d_out=ys[i % m]), reps, torch)
            tr = time_events(lambda i: zc.zc_reduce_compressed([cs[i % m], cs[(i + 1) % m]], n, rate, d_out=rs[i % m]),
                             reps, torch)
            mc, md, mr = float(np.median(tc)), float(np.median(td)), float(np.median(tr))
            ab = algorithmic_bytes("compress", n, rate)
            e = {"n": n, "rate": rate, "rotated_copies": m,
                 "compress_ms": round(mc, 4), "compress_hbm_frac": frac(ab, mc),
                 "decompress_ms": round(md, 4), "decompress_hbm_frac": frac(ab, md),
                 "reduce_k2_ms": round(mr, 4), "reduce_k2_hbm_frac": frac(algorithmic_bytes("reduce", n, rate), mr),
                 "reduce_k2_uncompressed_GBps": round(4 * n / (mr * 1e-3) / 1e9, 1)}
            e.update(error_stats(torch, ys[0], xs[0]))
            if config == 1:
                # a 4 MiB message is about 1 us of traffic: the figures are launch costs
                e["note"] = "launch-bound: correctness workload"
            entries[label] = e
            del xs, cs, rs, ys, x0
            torch.cuda.empty_cache()
        out[str(config)] = entries if len(entries) > 1 else next(iter(entries.values()))

    # the ring share: eight pre-compressed peer chunks
    rate = workloads.CONFIGS[5]["rate"]
    bufs = workloads.config_buffers(5)
    n = bufs[0][1].size
    comp0 = [zc.zc_compress(torch.from_numpy(b).to(dev), rate) for _, b in bufs]
    chunk = comp0[0].numel()
    chain_bytes = 7 * 3 * chunk + chunk + 4 * n
    k8_bytes = 9 * chunk + chunk + 4 * n
    share = {"n_per_chunk": n, "rate": rate, "peers": 8}
    for label, nsets in (("llc_resident", 1), ("rotated", 4)):
        sets = [comp0] + [[c.clone() for c in comp0] for _ in range(nsets - 1)]
        accs = [torch.empty_like(comp0[0]) for _ in range(nsets)]
        finals = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(nsets)]

        def chain(i):
            comp, acc, final = sets[i % nsets], accs[i % nsets], finals[i % nsets]
            zc.zc_reduce_compressed([comp[0], comp[1]], n, rate, d_out=acc)
            for j in range(2, 8):
                zc.zc_reduce_compressed([acc, comp[j]], n, rate, d_out=acc)   # in place, as a ring hop forwards it
            zc.zc_decompress(acc, n, rate, d_out=final)

        def direct(i):
            comp, acc, final = sets[i % nsets], accs[i % nsets], finals[i % nsets]
            zc.zc_reduce_compressed(comp, n, rate, d_out=acc)
            zc.zc_decompress(acc, n, rate, d_out=final)

        tch = float(np.median(time_events(chain, reps, torch)))
        tk8 = float(np.median(time_events(direct, reps, torch)))
        share[label] = {"chain_7_reduces_plus_decompress_ms": round(tch, 4), "chain_hbm_frac": frac(chain_bytes, tch),
                        "chain_uncompressed_GBps": round(8 * 4 * n / (tch * 1e-3) / 1e9, 1),
                        "reduce_k8_plus_decompress_ms": round(tk8, 4), "k8_hbm_frac": frac(k8_bytes, tk8)}
        if nsets == 1:
            share[label]["note"] = "16 MiB per chunk: served from the last-level cache, not HBM"
            direct(0)
            torch.cuda.synchronize()
            direct_sum = finals[0].clone()
            chain(0)
            torch.cuda.synchronize()
            chained = finals[0].clone()
            # the same eight launches as one HIP graph (the chain is launch-bound: 18 us kernels)
            side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
            comp, acc, final = sets[0], accs[0], finals[0]
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                zc.zc_reduce_compressed([comp[0], comp[1]], n, rate, d_out=acc, stream=side)
                for j in range(2, 8):
                    zc.zc_reduce_compressed([acc, comp[j]], n, rate, d_out=acc, stream=side)
                zc.zc_decompress(acc, n, rate, d_out=final, stream=side)
            final.zero_()
            tg = float(np.median(time_events(lambda i: graph.replay(), reps, torch)))
            share[label]["chain_as_hip_graph_ms"] = round(tg, 4)
            share[label]["graph_equals_eager"] = bool(torch.equal(final.view(torch.int32), chained.view(torch.int32)))
            del graph
        del sets, accs, finals
    total = torch.zeros(n, dtype=torch.float64, device=dev)
    for _, b in bufs:
        total += torch.from_numpy(b).to(dev).double()
    for key, got in (("ring_chain_error_vs_exact_sum", chained), ("reduce_k8_error_vs_exact_sum", direct_sum)):
        err = got.double() - total
        share[key] = {"max_abs": float("%.4g" % float(err.abs().max())), "rmse": float("%.4g" % float(err.pow(2).mean().sqrt())),
                      "sum_std": float("%.4g" % float(total.std()))}
    out["5"] = share
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="leave out the five-workload table and the error per rate")
    ap.add_argument("--no-extras", action="store_true",
                    help="leave out the ring-hop variants, half precision, 4 x 4 blocks and the lossless codec")
    ap.add_argument("--cpu-sample-log2", type=int, default=26)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain device copies of the 1 GiB input (known traffic, for scaling profiler counters)")
    ap.add_argument("--rates", type=int, nargs="+", default=None,
                    help="instead of the benchmark line: time the same three-call step at these rates on 2^28 values "
                         "(gradient bucket below rate 16, GELU activations from rate 16 up); one JSON list on stdout")
    ap.add_argument("--lossless", action="store_true",
                    help="instead of the benchmark line: time zl_compress / zl_decompress alone on the 2^28-word gradient "
                         "bucket (fp32), 12 pairs of launches; one JSON object on stdout")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2409_02423_amd import workloads, zc
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    zc.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.rates:
        print(json.dumps(rate_loop(torch, zc, workloads, dev, args.rates)))
        return
    if args.lossless:
        print(json.dumps(lossless_loop(torch, zc, workloads, dev, calibrate=args.calibrate_copy)))
        return

    cfg = workloads.CONFIGS[2]
    rate, n = cfg["rate"], cfg["n"]
    x_host = workloads.config_buffers(2)[0][1]
    x = torch.from_numpy(x_host).to(dev)
    peer_host = workloads.gradient_lowrank(6144, 43690, tail=n - 6144 * 43690, config=2, index=1)
    incoming = zc.zc_compress(torch.from_numpy(peer_host).to(dev), rate)
    del peer_host
    c = torch.empty(zc.zc_compressed_size(n, rate), dtype=torch.uint8, device=dev)
    r = torch.empty_like(c)
    y = torch.empty(n, dtype=torch.float32, device=dev)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []

    def step(record):
        e = [ev() for _ in range(4)] if record else None
        if record:
            e[0].record()
        zc.zc_compress(x, rate, d_out=c)
        if record:
            e[1].record()
        zc.zc_reduce_compressed([incoming, c], n, rate, d_out=r)
        if record:
            e[2].record()
        zc.zc_decompress(r, n, rate, d_out=y)
        if record:
            e[3].record()
            marks.append(e)

    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < SETTLE_MS:   # settle the clocks (untimed, see time_events)
        for _ in range(5):
            step(False)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / args.steps
    if args.calibrate_copy:
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
    names = ("compress", "reduce", "decompress")
    avg_ms = {nm: float(np.mean([m[i].elapsed_time(m[i + 1]) for m in marks])) for i, nm in enumerate(names)}
    dominant = max(avg_ms, key=avg_ms.get)
    abytes = algorithmic_bytes(dominant, n, rate, k=2)
    prof = profiled_counters().get(KERNEL_NAMES[dominant], {})
    if dominant == "reduce" and "valu_wave_insts" in prof:
        # two decodes and one encode per 6 bytes of traffic: bound by integer VALU work
        ops = prof["valu_wave_insts"] * 64
        achieved = ops / (avg_ms[dominant] * 1e-3) / 1e12
        roofline = {"kernel": KERNEL_NAMES[dominant], "bound": "alu", "achieved": round(achieved, 2),
                    "peak": round(INT_ALU_PEAK_TOPS, 2), "unit": "Tops/s (int32 lane operations)",
                    "frac": round(achieved / INT_ALU_PEAK_TOPS, 4), "lane_ops_per_launch": ops}
    else:
        achieved = abytes / (avg_ms[dominant] * 1e-3) / 1e9
        roofline = {"kernel": KERNEL_NAMES[dominant], "bound": "hbm", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4)}
    copy_gbps = measure_copy(torch, x, y)
    roofline.update({"traffic": prof.get("traffic_bytes"),
                     "traffic_source": "rocprofv3 FETCH_SIZE + WRITE_SIZE per launch from profiles/%s (null if that "
                                       "summary has no row for this kernel)" % os.path.basename(PROFILE),
                     "avg_launch_ms": round(avg_ms[dominant], 4), "algorithmic_bytes": abytes,
                     "frac_of_measured_copy": round(achieved / copy_gbps, 4) if roofline["bound"] == "hbm" else None,
                     "stream_input": "the 128 MiB stream the decompress kernel reads was written by the reduce kernel just "
                                     "before it with plain stores, so part of it may come from the 256 MB last-level cache "
                                     "(at most 11 % of the kernel's bytes); the fp32 side is 1 GiB and comes from / goes to HBM; "
                                     "`decompress_from_hbm` has the same kernel alone on streams that lie in HBM"})
    kernels = {nm: {"avg_ms": round(avg_ms[nm], 4),
                    "uncompressed_GBps": round(4 * n / (avg_ms[nm] * 1e-3) / 1e9, 1),
                    "algorithmic_GBps": round(algorithmic_bytes(nm, n, rate) / (avg_ms[nm] * 1e-3) / 1e9, 1),
                    "hbm_frac": frac(algorithmic_bytes(nm, n, rate), avg_ms[nm])}
               for nm in names}
    # the fused reduce is bound by integer work, not by bytes: its share of the integer ALU peak, from
    # the instruction count in the tracked profile (absent if that summary has no row for the kernel)
    reduce_prof = profiled_counters().get(KERNEL_NAMES["reduce"], {})
    if "valu_wave_insts" in reduce_prof:
        lane_ops = reduce_prof["valu_wave_insts"] * 64
        kernels["reduce"]["int_alu_frac"] = round(lane_ops / (avg_ms["reduce"] * 1e-3) / 1e12 / INT_ALU_PEAK_TOPS, 4)
        kernels["reduce"]["valu_instructions_per_block"] = round(reduce_prof["valu_wave_insts"] * 64 / (n / 4), 1)

    result = {
        "metric": "compress/decompress/reduce GB/s (uncompressed fp32) and % of HBM peak",
        "value": round(4 * n / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": "configs[1]: DP gradient bucket, 2^28 fp32 (6144x43690 rank-8 + noise), rate 4; "
                               "step = compress + 2-way fused reduce + decompress", "n_values": n, "rate": rate},
        "kernels": kernels,
    }
    back = zc.zc_decompress(c, n, rate)
    quality = error_stats(torch, back, x)
    quality["input_std"] = float("%.4g" % float(x.double().std()))
    del back
    if not args.no_extras:
        result.update(extras(torch, zc, workloads, dev, x, incoming, c, r, y, n, rate))
    result["round_trip_error"] = quality

    if not args.no_configs:
        # error of the lossy round trip against the original input at every rate (reported, not a target)
        per_rate = {}
        for rr in (4, 8, 12, 16, 20, 24, 28, 32):
            cc = zc.zc_compress(x, rr)
            zc.zc_decompress(cc, n, rr, d_out=y)
            per_rate[str(rr)] = error_stats(torch, y, x)
            del cc
        per_rate["data"] = "gradient bucket of configs[1], input std %.4g" % quality["input_std"]
        result["error_per_rate"] = per_rate
    del incoming, c
    torch.cuda.empty_cache()
    if not args.no_configs:
        table = config_table(torch, zc, workloads, dev)
        table["2"] = {"n": n, "rate": rate, "rotated_copies": 1,
                      "compress_ms": kernels["compress"]["avg_ms"], "compress_hbm_frac": kernels["compress"]["hbm_frac"],
                      "decompress_ms": kernels["decompress"]["avg_ms"], "decompress_hbm_frac": kernels["decompress"]["hbm_frac"],
                      "reduce_k2_ms": kernels["reduce"]["avg_ms"], "reduce_k2_hbm_frac": kernels["reduce"]["hbm_frac"],
                      "max_abs": quality["max_abs"], "rmse": quality["rmse"],
                      "note": "1 GiB message: no rotation needed; figures from inside the timed step"}
        result["configs"] = dict(sorted(table.items()))
    result["copy_GBps"] = copy_gbps
    result["roofline"] = roofline

    if not args.no_cpu_baseline:
        del y, r, x
        torch.cuda.empty_cache()
        threads = min(16, len(os.sched_getaffinity(0)))
        result["cpu_baseline"] = cpu_baseline(x_host, rate, 1 << args.cpu_sample_log2, threads)
    print(json.dumps(result))


def extras(torch, zc, workloads, dev, x, incoming, c, r, y, n, rate):
    """Figures outside `value`, on the headline buffer: the two fused ring-hop variants, the
    buffer as a bf16 message, 4 x 4 blocks on a matrix of the same size, the lossless codec."""
    # Compressed inputs of these launches are rotated through three copies, so that every launch
    # finds its stream in HBM and not in the 256 MB last-level cache where its own last launch left it.
    three = lambda s: [s, s.clone(), s.clone()]
    incomings = three(incoming)
    hop_mixed = float(np.median(time_events(lambda i: zc.zc_reduce_mixed([incomings[i % 3]], x, n, rate, d_out=r), 12, torch)))
    hop_raw = float(np.median(time_events(lambda i: zc.zc_reduce_decompress([incomings[i % 3]], x, n, rate, d_out=y), 12, torch)))
    alone = float(np.median(time_events(lambda i: zc.zc_decompress(incomings[i % 3], n, rate, d_out=y), 12, torch)))
    mixed_bytes = n * 4 + 2 * (n * rate // 8)
    raw_bytes = 2 * n * 4 + n * rate // 8
    ring_hop = {"reduce_mixed_ms": round(hop_mixed, 4), "reduce_mixed_hbm_frac": frac(mixed_bytes, hop_mixed),
                "reduce_decompress_ms": round(hop_raw, 4), "reduce_decompress_hbm_frac": frac(raw_bytes, hop_raw),
                "note": "compressed incoming chunk + raw local values -> compressed sum / -> fp32 sum"}
    decompress_from_hbm = {"ms": round(alone, 4), "hbm_frac": frac(algorithmic_bytes("decompress", n, rate), alone),
                           "note": "zc_decompress alone on rotated streams; inside the step its stream was written "
                                   "by the reduce kernel just before and comes from the last-level cache"}
    del incomings

    # the same buffer as a bf16 message
    xh = x.to(torch.bfloat16)
    yh = torch.empty_like(xh)
    ch = torch.empty_like(c)
    hc = float(np.median(time_events(lambda i: zc.zc_compress_half(xh, rate, d_out=ch), 12, torch)))
    zc.zc_compress_half(xh, rate, d_out=ch)
    chs = three(ch)
    hd = float(np.median(time_events(lambda i: zc.zc_decompress_half(chs[i % 3], n, rate, d_out=yh), 12, torch)))
    hb = n * 2 + n * rate // 8
    half_precision = {"dtype": "bf16", "compress_ms": round(hc, 4), "decompress_ms": round(hd, 4),
                      "compress_hbm_frac": frac(hb, hc), "decompress_hbm_frac": frac(hb, hd)}
    del xh, yh, ch, chs

    # 4 x 4 blocks on a matrix of the same size and structure
    m_rows, m_cols = 8192, 32768
    xm = torch.from_numpy(workloads.gradient_lowrank(m_rows, m_cols, config=2, index=0)).to(dev).reshape(m_rows, m_cols)
    ym = y.reshape(m_rows, m_cols)
    blocks_4x4 = {"matrix": "%dx%d rank-8 + noise" % (m_rows, m_cols)}
    for r2 in (4, 8):
        cm = torch.empty(zc.zc2d_compressed_size(m_rows, m_cols, r2), dtype=torch.uint8, device=dev)
        tc = float(np.median(time_events(lambda i: zc.zc2d_compress(xm, r2, d_out=cm), 12, torch)))
        cms = three(cm)
        td = float(np.median(time_events(lambda i: zc.zc2d_decompress(cms[i % 3], m_rows, m_cols, r2, d_out=ym), 12, torch)))
        rm = torch.empty_like(cm)
        tr = float(np.median(time_events(lambda i: zc.zc2d_reduce_compressed([cms[i % 3], cms[(i + 1) % 3]], m_rows, m_cols, r2,
                                                                              d_out=rm), 12, torch)))
        del rm, cms
        mb = 4 * n + cm.numel()
        rel2 = float(((ym - xm).double().pow(2).mean() / xm.double().pow(2).mean()).sqrt())
        one = zc.zc_decompress(zc.zc_compress(xm.reshape(-1), r2), n, r2)
        rel1 = float(((one - xm.reshape(-1)).double().pow(2).mean() / xm.double().pow(2).mean()).sqrt())
        del one, cm
        blocks_4x4["rate_%d" % r2] = {
            "compress_ms": round(tc, 4), "decompress_ms": round(td, 4), "reduce_2way_ms": round(tr, 4),
            "compress_hbm_frac": frac(mb, tc), "decompress_hbm_frac": frac(mb, td),
            "relative_rms_error": round(rel2, 5), "relative_rms_error_blocks_of_4": round(rel1, 5)}
    del xm, ym

    # the lossless codec on the same buffer, as fp32 words and as a bf16 message
    lossless = {}
    cl = torch.empty(zc.zl_max_compressed_size(n), dtype=torch.uint8, device=dev)
    for label, xl in (("fp32", x), ("bf16", x.to(torch.bfloat16))):
        half = xl.element_size() == 2
        comp, decomp = (zc.zl_compress16, zc.zl_decompress16) if half else (zc.zl_compress, zc.zl_decompress)
        yl = torch.empty_like(xl)
        comp(xl, d_out=cl)
        size = zc.zl_stream_bytes(cl)
        tc = float(np.median(time_events(lambda i: comp(xl, d_out=cl), 12, torch)))
        td = float(np.median(time_events(lambda i: decomp(cl[:size], n, d_out=yl), 12, torch)))
        message = xl.element_size() * n
        moved = message + size
        as_int = torch.int16 if half else torch.int32
        lossless[label] = {"stream_over_message": round(size / float(message), 4),
                           "compress_ms": round(tc, 4), "decompress_ms": round(td, 4),
                           "compress_hbm_frac": frac(moved, tc), "decompress_hbm_frac": frac(moved, td),
                           "exact": bool(torch.equal(yl.view(as_int), xl.view(as_int)))}
        del xl, yl
    del cl
    return {"ring_hop": ring_hop, "decompress_from_hbm": decompress_from_hbm, "half_precision": half_precision,
            "blocks_4x4": blocks_4x4, "lossless": lossless}


def lossless_loop(torch, zc, workloads, dev, reps=12, calibrate=False):
    x = torch.from_numpy(workloads.config_buffers(2)[0][1]).to(dev)
    n = x.numel()
    c = torch.empty(zc.zl_max_compressed_size(n), dtype=torch.uint8, device=dev)
    y = torch.empty_like(x)
    zc.zl_compress(x, d_out=c)
    size = zc.zl_stream_bytes(c)
    tc = time_events(lambda i: zc.zl_compress(x, d_out=c), reps, torch)
    td = time_events(lambda i: zc.zl_decompress(c[:size], n, d_out=y), reps, torch)
    if calibrate:
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
    moved = 4 * n + size
    mc, md = float(np.median(tc)), float(np.median(td))
    return {"workload": "configs[1] gradient bucket, 2^28 words", "stream_bytes": size, "stream_over_message": round(size / (4.0 * n), 4),
            "compress_ms": round(mc, 4), "decompress_ms": round(md, 4),
            "compress_hbm_frac": frac(moved, mc), "decompress_hbm_frac": frac(moved, md),
            "exact": bool(torch.equal(y.view(torch.int32), x.view(torch.int32)))}


def rate_loop(torch, zc, workloads, dev, rates, reps=12):
    """compress -> 2-way reduce -> decompress on 2^28 values at each rate, per-kernel
    medians from HIP events on the launch stream."""
    n = 1 << 28
    grad = torch.from_numpy(workloads.config_buffers(2)[0][1]).to(dev)
    act = torch.from_numpy(workloads.activation_gelu(n)).to(dev) if any(r >= 16 for r in rates) else None
    y = torch.empty(n, dtype=torch.float32, device=dev)
    out = []
    for rate in rates:
        x = grad if rate < 16 else act
        c = zc.zc_compress(x, rate)
        peer = zc.zc_compress(torch.flip(x, [0]).contiguous(), rate)
        r = torch.empty_like(c)
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < SETTLE_MS:   # settle the clocks (untimed, see time_events)
            for _ in range(5):
                zc.zc_compress(x, rate, d_out=c)
                zc.zc_reduce_compressed([peer, c], n, rate, d_out=r)
                zc.zc_decompress(r, n, rate, d_out=y)
            torch.cuda.synchronize()
        marks = []
        for _ in range(reps):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            e[0].record()
            zc.zc_compress(x, rate, d_out=c)
            e[1].record()
            zc.zc_reduce_compressed([peer, c], n, rate, d_out=r)
            e[2].record()
            zc.zc_decompress(r, n, rate, d_out=y)
            e[3].record()
            marks.append(e)
        torch.cuda.synchronize()
        ms = [float(np.median([m[i].elapsed_time(m[i + 1]) for m in marks])) for i in range(3)]
        ab = algorithmic_bytes("compress", n, rate)
        out.append({"rate": rate, "data": "gradient bucket" if rate < 16 else "gelu activations",
                    "compress_ms": round(ms[0], 4), "reduce_k2_ms": round(ms[1], 4), "decompress_ms": round(ms[2], 4),
                    "compress_hbm_frac": frac(ab, ms[0]), "decompress_hbm_frac": frac(ab, ms[2]),
                    "reduce_hbm_frac": frac(algorithmic_bytes("reduce", n, rate), ms[1]),
                    "reduce_uncompressed_GBps": round(4 * n / (ms[1] * 1e-3) / 1e9, 1)})
        del c, peer, r
    return out


if __name__ == "__main__":
    main()
