#!/usr/bin/env python3
"""Benchmark of the zc hot path on one MI355X.

One step = one pass of the whole hot path on synthetic data already resident in HBM:
  1. zc_compress    of a 512^3 fp32 Gaussian random field (P(k) ~ k^-3), rel. bound 1e-4
  2. zc_decompress  of a stream of that field
  3. zc_reduce_compressed of 8 compressed rank buffers of 64M values (same generator, other
     seeds, common absolute bound), the local step of a compressed Allreduce.
The step rotates over four stream buffers: it compresses into one and decompresses the one that was
written three steps (about 7 GB of memory traffic) earlier, so that the decompression reads its stream
from HBM and not from what the compression has just left in the 256 MB memory-side cache; the
decompression of the stream just written is reported beside it as `warm`.

`value` is the step's throughput in fp32 gigabytes per second: the fp32 data the step stands for,
4n (compress input) + 4n (decompress output) + 4*8*m (what the 8 reduce operands represent), over the
step time; it is not a count of bytes moved (the reduce moves only compressed bytes).  The bytes the
method itself must move (`algorithmic_bytes`) over the same time are `algorithmic_GBps` and, against
the 8 TB/s peak, `hbm_frac_step`.  Per stage, `roofline` is the main kernel alone (HIP events handed to
its launch) and `call_frac` the whole call as a user pays for it.  The reference CPU codec is timed on
the same buffers as `cpu_baseline` (reported baseline, not a target).
"""
import argparse
import hashlib
import json
import math
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
ROTATION = 4          # stream buffers the step rotates over


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--rel", type=float, default=1e-4, help="value-range-relative error bound of the timed step")
    ap.add_argument("--side", type=int, default=512, help="field side; 512 is the benchmark configuration")
    ap.add_argument("--streams", choices=("plain", "indexed"), default="indexed",
                    help="stream variant of every call; indexed (with the segment index of Section 3.5.2) is the "
                         "library's default, plain is ZC_STREAM_PLAIN")
    ap.add_argument("--tiles", choices=("by_id", "by_ticket"), default="by_id",
                    help="how the kernels that write a stream hand out their tiles; by_ticket is ZC_TILES_BY_TICKET")
    ap.add_argument("--settle-ms", type=float, default=100.0,
                    help="untimed steps run for this long before the warmup steps: the first milliseconds of work on an "
                         "idle GPU run several percent slow")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", choices=("all", "none", "ring"), default="all",
                    help="the untimed measurements after the timed step: all of them, none, or only the ring round and "
                         "the k-way Max (what a profile of those two kernels needs)")
    ap.add_argument("--no-extras", action="store_true", help="the same as --extras none")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run plain device copies of the field (4n B read + 4n B written each): the known "
                         "traffic that calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.no_extras:
        args.extras = "none"
    return args


def source_digest():
    """Digest of the kernel sources: ties the counter figures under profiles/ to the code they were taken on."""
    d = os.path.join(ROOT, "paper_2502_18554_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".h", ".hip")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def profiled(workload_key):
    """What the rocprofv3 counter runs summarised in profiles/traffic.json say about the main kernels of this
    workload (counters cannot be read from inside this script): HBM bytes per launch (`traffic_bytes`) and VALU
    instructions per launch (`valu_instructions`); {} when that file was taken on other kernel sources or
    another workload."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        return {}
    entry = rec.get(workload_key)
    if not entry or entry.get("source_digest") != source_digest():
        return {}
    return entry


def streaming_rate(zc, read_bytes, write_bytes, stage_gbs, reps=12):
    """Times zc_debug_stream on about read_bytes + write_bytes in the nearest mix of 1..16 loads : 1..16 stores per lane."""
    import torch
    unit = 8192
    ratio = read_bytes / write_bytes
    loads, stores = min(((a, b) for a in range(1, 17) for b in range(1, 17)), key=lambda ab: (abs(ab[0] / ab[1] - ratio), -ab[0]))
    tiles = max(1, round((read_bytes + write_bytes) / ((loads + stores) * unit)))
    src = torch.zeros(tiles * loads * unit, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty(tiles * stores * unit, dtype=torch.uint8, device="cuda:0")
    for _ in range(3):
        assert zc.zc_debug_stream(src, dst, tiles, loads, stores) == 0
    torch.cuda.synchronize()
    zc.zc_profile_enable(True, only=["stream"])
    for _ in range(reps):
        zc.zc_debug_stream(src, dst, tiles, loads, stores)
    torch.cuda.synchronize()
    times = [ms for name, ms in zc.zc_profile_collect() if name == "stream"]
    zc.zc_profile_enable(False)
    ms = sum(times) / len(times)
    gbs = tiles * (loads + stores) * unit / ms / 1e6
    return {"loads_per_lane": loads, "stores_per_lane": stores, "workgroups": tiles, "bytes": tiles * (loads + stores) * unit,
            "kernel_ms": round(ms, 4), "GBps": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4),
            "stage_over_streaming": round(stage_gbs / gbs, 4)}


def valu_frac(instructions, kernel_ms):
    """Share of the kernel's duration that its VALU instructions need to issue: a wave64 instruction holds
    the 16 lanes of its SIMD for 4 cycles, there are 256 x 4 SIMDs, and the clock is 2.4 GHz."""
    if not instructions:
        return None
    return round(instructions * 4 / (1024 * 2.4e9) / (kernel_ms * 1e-3), 4)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import paper_2502_18554_amd as zc
    from paper_2502_18554_amd import synth
    from paper_2502_18554_amd.binding import ZC_OK, ZC_STREAM_PLAIN, ZC_TILES_BY_TICKET

    zc.binding.lib()                      # fails loudly if the HIP library is missing
    indexed = args.streams == "indexed"
    variant = 0 if indexed else ZC_STREAM_PLAIN                      # what readers are given
    flags = variant | (ZC_TILES_BY_TICKET if args.tiles == "by_ticket" else 0)   # ... and writers
    dev = "cuda:0"
    torch.cuda.set_device(0)
    side = args.side
    K = 8
    shape_c = (side, side, side)
    shape_r = (side // 2, side, side)

    def u8(nbytes):
        return torch.empty(nbytes + 64, dtype=torch.uint8, device=dev)

    def check(st, what):
        if st != ZC_OK:
            raise zc.ZcError(st, what)

    # ---------------- inputs, resident in HBM ----------------
    x = synth.power_law_field(shape_c, seed=0, device=dev)
    n = x.numel()
    eb = synth.abs_bound(x, args.rel)
    d_streams = [u8(zc.zc_compress_bound(n, variant)) for _ in range(ROTATION)]
    d_ys = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(2)]
    d_stream, d_y = d_streams[0], d_ys[0]
    ws_c, ws_d = u8(zc.zc_workspace_bytes(n, 1)), u8(zc.zc_workspace_bytes(n, 1))

    ranks, chunks, chunk_bytes = [], [], []
    m = shape_r[0] * shape_r[1] * shape_r[2]
    eb_r = float(torch.tensor(args.rel * 2.0, dtype=torch.float32))     # common bound: fields span [-1, 1]
    scratch = u8(zc.zc_compress_bound(m, variant))
    ws_r = u8(zc.zc_workspace_bytes(m, K))
    for r in range(K):
        xr = synth.power_law_field(shape_r, seed=100 + r, device=dev)
        st, total = zc.zc_compress(xr, m, eb_r, scratch, ws_r, flags=flags)
        check(st, f"compress rank {r}")
        chunks.append(scratch[:total].clone())
        chunk_bytes.append(total)
        ranks.append(xr)
    d_red = u8(zc.zc_compress_bound(m, variant))

    for s in d_streams:
        st, c_bytes = zc.zc_compress(x, n, eb, s, ws_c, flags=flags)
        check(st, "compress")
    st, n_out = zc.zc_decompress(d_stream, c_bytes, d_y, ws_d, flags=variant)
    check(st, "decompress")
    st, r_bytes = zc.zc_reduce_compressed(chunks, chunk_bytes, d_red, ws_r, flags=flags)
    check(st, "reduce")
    assert n_out == n
    max_err = float((d_y.double() - x.double()).abs().max())
    assert max_err <= eb, (max_err, eb)

    if args.copy_probe:
        for _ in range(3):
            torch.neg(x, out=d_y)          # one elementwise kernel: reads 4n bytes, writes 4n bytes
        torch.cuda.synchronize()

    stage_names = ("compress", "decompress", "reduce")
    alg_bytes = {
        "compress": 4 * n + c_bytes,
        "decompress": c_bytes + 4 * n,
        "reduce": sum(chunk_bytes) + r_bytes,
    }
    fp32_bytes = {"compress": 4 * n, "decompress": 4 * n, "reduce": 4 * m * K}
    counter = [0]

    def step(events=None, rotate=True):
        j = counter[0]
        counter[0] += 1
        s_out = d_streams[j % ROTATION] if rotate else d_stream
        s_in = d_streams[(j + 1) % ROTATION] if rotate else d_stream     # written ROTATION - 1 steps ago
        if events:
            events[0].record()
        zc.zc_compress(x, n, eb, s_out, ws_c, sync=False, flags=flags)
        if events:
            events[1].record()
        zc.zc_decompress(s_in, c_bytes, d_ys[j % 2], ws_d, sync=False, flags=variant)
        if events:
            events[2].record()
        zc.zc_reduce_compressed(chunks, chunk_bytes, d_red, ws_r, sync=False, flags=flags)
        if events:
            events[3].record()

    def kernel_averages(records):
        return {s: (sum(ms for name, ms in records if name == s) / max(1, sum(1 for name, _ in records if name == s)))
                for s in stage_names}

    def finish_all(what):
        for ws, name in ((ws_c, "compress"), (ws_d, "decompress"), (ws_r, "reduce")):
            st, _ = zc.zc_finish(ws)
            check(st, f"{name} ({what})")

    # untimed, before the warmup steps; the kernels are timed here to learn which one runs longest
    zc.zc_profile_enable(True)
    t_settle = time.perf_counter()
    while True:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        if (time.perf_counter() - t_settle) * 1e3 >= args.settle_ms:
            break
    settled = kernel_averages(zc.zc_profile_collect())
    zc.zc_profile_enable(False)
    dominant = max(stage_names, key=lambda s: settled[s])
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The timed region carries the timing of the dominant kernel only (HIP events handed to its launch, on
    # the stream it runs on): every timed launch costs the step a few microseconds.
    zc.zc_profile_enable(True, only=(dominant,))
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    timed_records = zc.zc_profile_collect()
    zc.zc_profile_enable(False)
    finish_all("timed loop")
    assert len(timed_records) == args.steps and all(name == dominant for name, _ in timed_records), len(timed_records)
    # Per-call times and the other kernels' times come from two more passes over the same steps, one with
    # an event between the calls, one with every main kernel timed: an event record holds back the launch
    # behind it by a few microseconds, which the timed region above should not pay.
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    zc.zc_profile_enable(True)
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    kernel_ms = kernel_averages(zc.zc_profile_collect())
    kernel_ms[dominant] = sum(ms for _, ms in timed_records) / len(timed_records)
    # the decompression of the stream that the compression of the same step has just written
    for i in range(args.steps):
        step(rotate=False)
    torch.cuda.synchronize()
    warm_ms = kernel_averages(zc.zc_profile_collect())["decompress"]
    zc.zc_profile_enable(False)
    finish_all("per-stage passes")

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    stage_ms = {s: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i, s in enumerate(stage_names)}
    workload_key = f"{side}^3 rel {args.rel:g} + reduce {K}x{m}, {args.streams} streams, tiles {args.tiles}"
    counters = profiled(workload_key)
    traffic = counters.get("traffic_bytes", {})
    valu = counters.get("valu_instructions", {})
    stages = {}
    for s in stage_names:
        # roofline = the main kernel alone; ms / call_frac = the whole call (on plain streams: the kernels ahead of it too)
        gbs = alg_bytes[s] / kernel_ms[s] / 1e6
        stages[s] = {
            "ms": round(stage_ms[s], 4),
            "fp32_GBps": round(fp32_bytes[s] / stage_ms[s] / 1e6, 1),
            "call_frac": round(alg_bytes[s] / stage_ms[s] / 1e6 / HBM_PEAK_GBS, 4),
            "kernel_ms": round(kernel_ms[s], 4),
            "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic.get(s)},
            "valu_frac": valu_frac(valu.get(s), kernel_ms[s]),
            "algorithmic_bytes": alg_bytes[s],
        }
    stages["decompress"]["input"] = f"cold: the stream was written {ROTATION - 1} steps earlier"
    stages["decompress"]["just_written"] = {"kernel_ms": round(warm_ms, 4),
                                            "frac": round(alg_bytes["decompress"] / warm_ms / 1e6 / HBM_PEAK_GBS, 4),
                                            "input": "the stream the compression of the same step has just written"}
    # Beside every stage: a kernel that only streams the same bytes in the same read : write mix, with the
    # access shape of the codec's kernels (zc_debug_stream): what the memory system gives such a kernel.
    read_write = {"compress": (4 * n, c_bytes), "decompress": (c_bytes, 4 * n), "reduce": (sum(chunk_bytes), r_bytes)}
    for s in stage_names:
        stages[s]["streaming_kernel"] = streaming_rate(zc, *read_write[s], alg_bytes[s] / kernel_ms[s] / 1e6)
    total_fp32 = sum(fp32_bytes.values())
    total_alg = sum(alg_bytes.values())
    value = total_fp32 / ms_per_step / 1e6

    def timed(fn, reps=10, warm=3):
        for _ in range(warm):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    # ---------------- untimed extras ----------------
    extras = {}
    if args.extras == "all":
        # the three error bounds of the 512^3 configuration; the decompression reads a stream written four
        # compressions earlier (cold, as in the step)
        for rel in (1e-2, 1e-3, 1e-4):
            e = synth.abs_bound(x, rel)
            for s in d_streams:
                st, cb = zc.zc_compress(x, n, e, s, ws_c, flags=flags)
                check(st, "compress extra")
            res = {"ratio": round(4 * n / cb, 3)}
            rot = [0]

            def comp():
                rot[0] += 1
                zc.zc_compress(x, n, e, d_streams[rot[0] % ROTATION], ws_c, sync=False, flags=flags)

            def decomp():
                rot[0] += 1
                zc.zc_decompress(d_streams[rot[0] % ROTATION], cb, d_ys[rot[0] % 2], ws_d, sync=False, flags=variant)

            for name, fn in (("compress", comp), ("decompress", decomp)):
                ms = timed(fn, reps=12, warm=8)
                frac = round((4 * n + cb) / ms / 1e6 / HBM_PEAK_GBS, 4)      # the whole call: it is one launch
                res[name] = {"ms": round(ms, 4), "fp32_GBps": round(4 * n / ms / 1e6, 1), "call_frac": frac, "hbm_frac": frac}
            extras[f"rel_{rel:g}"] = res
        finish_all("error bound sweep")
        for s in d_streams:                  # back to the step's bound
            st, _ = zc.zc_compress(x, n, eb, s, ws_c, flags=flags)
            check(st, "compress")
        st, _ = zc.zc_decompress(d_stream, c_bytes, d_y, ws_d, flags=variant)
        check(st, "decompress")
        # quality sums of the reconstruction (synchronous call: timed on the host)
        st, q4 = zc.zc_quality(x, d_y, n, ws_c)
        check(st, "quality extra")
        torch.cuda.synchronize()
        tq = time.perf_counter()
        for _ in range(5):
            zc.zc_quality(x, d_y, n, ws_c)
        ms = (time.perf_counter() - tq) * 1e3 / 5
        rng_x = q4[3] - q4[2]
        rmse = (q4[1] / n) ** 0.5
        extras["quality"] = {"max_err": q4[0], "nrmse": rmse / rng_x, "psnr_dB": round(20 * math.log10(rng_x / rmse), 2),
                             "ms": round(ms, 4), "call_frac": round(8 * n / ms / 1e6 / HBM_PEAK_GBS, 4)}
        # the step as a HIP graph: the asynchronous calls only launch kernels, so the three calls
        # are captured once and replayed
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(rotate=False)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0g = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_g = (time.perf_counter() - t0g) * 1e3 / args.steps
        finish_all("graph replay")
        extras["hip_graph"] = {"ms_per_step": round(ms_g, 4), "value_GBps": round(total_fp32 / ms_g / 1e6, 1),
                               "note": "one set of buffers (the decompression reads the stream just written)"}
        del graph

        # the same step with the other stream variant, and with the other tile hand-out
        def variant_step(o_variant, o_flags):
            o_streams = [u8(zc.zc_compress_bound(n, o_variant)) for _ in range(ROTATION)]
            o_red = u8(zc.zc_compress_bound(m, o_variant))
            o_chunks, o_bytes = [], []
            for r in range(K):
                st, total = zc.zc_compress(ranks[r], m, eb_r, o_red, ws_r, flags=o_flags)
                check(st, "compress rank (other variant)")
                o_chunks.append(o_red[:total].clone())
                o_bytes.append(total)
            for s in o_streams:
                st, oc_bytes = zc.zc_compress(x, n, eb, s, ws_c, flags=o_flags)
                check(st, "compress (other variant)")
            jj = [0]

            def o_step(events=None):
                j = jj[0]
                jj[0] += 1
                if events:
                    events[0].record()
                zc.zc_compress(x, n, eb, o_streams[j % ROTATION], ws_c, sync=False, flags=o_flags)
                if events:
                    events[1].record()
                zc.zc_decompress(o_streams[(j + 1) % ROTATION], oc_bytes, d_ys[j % 2], ws_d, sync=False, flags=o_variant)
                if events:
                    events[2].record()
                zc.zc_reduce_compressed(o_chunks, o_bytes, o_red, ws_r, sync=False, flags=o_flags)
                if events:
                    events[3].record()

            for _ in range(args.warmup + 3):
                o_step()
            torch.cuda.synchronize()
            t0o = time.perf_counter()
            for _ in range(args.steps):
                o_step()
            torch.cuda.synchronize()
            ms_o = (time.perf_counter() - t0o) * 1e3 / args.steps
            o_evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
            for i in range(args.steps):
                o_step(o_evs[i])
            torch.cuda.synchronize()
            finish_all("other variant")
            calls = {s: round(sum(e[i].elapsed_time(e[i + 1]) for e in o_evs) / args.steps, 4) for i, s in enumerate(stage_names)}
            st, or_bytes = zc.zc_finish(ws_r)                  # the reduced stream's size in this variant
            check(st, "other variant")
            o_alg = {"compress": 4 * n + oc_bytes, "decompress": 4 * n + oc_bytes, "reduce": sum(o_bytes) + or_bytes}
            fracs = {s: round(o_alg[s] / calls[s] / 1e6 / HBM_PEAK_GBS, 4) for s in stage_names}
            return {"ms_per_step": round(ms_o, 4), "value_GBps": round(total_fp32 / ms_o / 1e6, 1), "call_ms": calls,
                    "call_frac": fracs, "hbm_frac_step": round(sum(o_alg.values()) / ms_o / 1e6 / HBM_PEAK_GBS, 4),
                    "compressed_bytes": oc_bytes}

        o_variant = ZC_STREAM_PLAIN if indexed else 0
        extras["other_stream_variant"] = dict(streams="plain" if indexed else "indexed",
                                              **variant_step(o_variant, o_variant | (flags & ZC_TILES_BY_TICKET)))
        extras["other_tile_hand_out"] = dict(tiles="by_id" if flags & ZC_TILES_BY_TICKET else "by_ticket",
                                             **variant_step(variant, flags ^ ZC_TILES_BY_TICKET))
        # the tail of the compressed Allgather at the shape of the reduce above: the 8 rank streams
        # decompressed by 8 calls and by one call
        outs = [torch.empty(m, dtype=torch.float32, device=dev) for _ in range(K)]
        ws_k = [u8(zc.zc_workspace_bytes(m, 1)) for _ in range(K)]

        def eight_calls():
            for i in range(K):
                zc.zc_decompress(chunks[i], chunk_bytes[i], outs[i], ws_k[i], sync=False, flags=variant)

        def one_call():
            zc.zc_decompress_many(chunks, chunk_bytes, outs, ws_r, sync=False, flags=variant)

        res = {"workload": f"{K} streams of {m} values (abs eb {eb_r:g}) -> {K} fp32 buffers"}
        for name, fn in (("eight_calls", eight_calls), ("one_call", one_call)):
            ms = timed(fn, reps=5)
            res[name] = {"ms": round(ms, 4), "fp32_GBps": round(4 * m * K / ms / 1e6, 1),
                         "call_frac": round((sum(chunk_bytes) + 4 * m * K) / ms / 1e6 / HBM_PEAK_GBS, 4)}
        st, _ = zc.zc_finish(ws_r)
        check(st, "decompress_many extra")
        extras["decompress_many"] = res
        del outs, ws_k
    if args.extras in ("all", "ring"):
        # one round of the ring reduce-scatter at the shape of the reduce above: the received
        # stream of rank 0 plus the uncompressed buffer of rank 1 -> stream of the sums
        st, s_bytes = zc.zc_reduce_step(chunks[0], chunk_bytes[0], ranks[1], m, scratch, ws_r, flags=flags)
        check(st, "reduce_step extra")

        def ring_round(op=None):
            if op is None:
                zc.zc_reduce_step(chunks[0], chunk_bytes[0], ranks[1], m, scratch, ws_r, sync=False, flags=flags)
            else:
                zc.zc_reduce_step_op(chunks[0], chunk_bytes[0], ranks[1], m, op, scratch, ws_r, sync=False, flags=flags)

        for _ in range(5):
            ring_round()
        torch.cuda.synchronize()
        ms = timed(ring_round)
        zc.zc_profile_enable(True)
        for _ in range(10):
            ring_round()
        torch.cuda.synchronize()
        kt = [t for name, t in zc.zc_profile_collect() if name == "reduce_step"]
        zc.zc_profile_enable(False)
        alg = chunk_bytes[0] + 4 * m + s_bytes
        k_ms = sum(kt) / len(kt)
        extras["reduce_step"] = {"workload": f"received stream of {m} values + {m} local fp32 values -> stream",
                                 "ms": round(ms, 4), "kernel_ms": round(k_ms, 4),
                                 "algorithmic_bytes": alg, "fp32_GBps": round(8 * m / ms / 1e6, 1),
                                 "hbm_frac": round(alg / k_ms / 1e6 / HBM_PEAK_GBS, 4),
                                 "call_frac": round(alg / ms / 1e6 / HBM_PEAK_GBS, 4),
                                 "valu_frac": valu_frac(valu.get("reduce_step"), k_ms),
                                 "traffic": traffic.get("reduce_step")}
        # the other aggregation functions: a Max round at the same shape, and the averaging
        # decompression of the reduced stream of the step above
        ms_max = timed(lambda: ring_round(zc.binding.ZC_OP_MAX))
        st, _ = zc.zc_finish(ws_r)
        check(st, "reduce_step_op extra")
        # k-way Max of the same compressed rank buffers (Section 3.2), and the k-way Sum and the ring
        # round each done in 4 parts of whole tiles, as a pipeline over a collective's chunks would
        d_red_alt = u8(zc.zc_compress_bound(m, variant))
        st, x_bytes = zc.zc_reduce_compressed_op(chunks, chunk_bytes, zc.binding.ZC_OP_MAX, d_red_alt, ws_r, flags=flags)
        check(st, "reduce_compressed_op extra")
        ms_kmax = timed(lambda: zc.zc_reduce_compressed_op(chunks, chunk_bytes, zc.binding.ZC_OP_MAX, d_red_alt, ws_r,
                                                           sync=False, flags=flags))
        st, _ = zc.zc_finish(ws_r)
        check(st, "reduce_compressed_op extra")
        quarter = m // 4

        def sum_in_parts():
            for i in range(4):
                zc.zc_reduce_compressed_part(chunks, chunk_bytes, m, i * quarter, quarter if i < 3 else m - 3 * quarter,
                                             d_red_alt, ws_r, sync=False, flags=flags)

        def round_in_parts():
            for i in range(4):
                zc.zc_reduce_step_part(chunks[0], chunk_bytes[0], ranks[1], m, zc.binding.ZC_OP_SUM, i * quarter,
                                       quarter if i < 3 else m - 3 * quarter, scratch, ws_r, sync=False, flags=flags)

        parts = None
        if quarter % 8192 == 0:
            ms_sum_parts = timed(sum_in_parts)
            st, b_sum_parts = zc.zc_finish(ws_r)
            check(st, "reduce_compressed_part extra")
            assert b_sum_parts == r_bytes and torch.equal(d_red_alt[:r_bytes], d_red[:r_bytes]), "parts != whole (Sum)"
            ms_round_parts = timed(round_in_parts)
            st, b_round_parts = zc.zc_finish(ws_r)
            check(st, "reduce_step_part extra")
            assert b_round_parts == s_bytes
            parts = {"reduce_in_4_parts_ms": round(ms_sum_parts, 4), "ring_round_in_4_parts_ms": round(ms_round_parts, 4)}
        alg_kmax = sum(chunk_bytes) + x_bytes
        extras["reduce_max"] = {"workload": f"k-way Max of the {K} compressed rank buffers", "ms": round(ms_kmax, 4),
                                "algorithmic_bytes": alg_kmax, "call_frac": round(alg_kmax / ms_kmax / 1e6 / HBM_PEAK_GBS, 4),
                                "valu_frac": valu_frac(valu.get("reduce_max"), ms_kmax)}
        if parts:
            extras["in_parts"] = parts
        extras["reduce_step"]["max_ms"] = round(ms_max, 4)
    if args.extras == "all":
        d_avg = torch.empty(m, dtype=torch.float32, device=dev)      # (d_y keeps the field for the cross-check below)
        ms_avg = timed(lambda: zc.zc_decompress_average(d_red, r_bytes, d_avg, ws_d, sync=False, flags=variant))
        st, n_avg = zc.zc_finish(ws_d)
        check(st, "decompress_average extra")
        # the field compressed in 8 parts (zc_compress_part), and decompressed in 8 chunks (zc_decompress_range)
        part = n // 8

        def in_parts():
            for i in range(8):
                zc.zc_compress_part(x, n, eb, i * part, part if i < 7 else n - 7 * part, d_stream, ws_c, sync=False, flags=flags)

        def in_chunks():
            for i in range(8):
                zc.zc_decompress_range(d_stream, c_bytes, i * part, part, d_y[i * part:(i + 1) * part], ws_d, sync=False,
                                       flags=variant)

        if part % 16384 == 0:
            ms_parts = timed(in_parts)
            st, b_parts = zc.zc_finish(ws_c)
            check(st, "compress_part extra")
            assert b_parts == c_bytes
            d_y.fill_(float("nan"))
            ms_chunks = timed(in_chunks)
            st, _ = zc.zc_finish(ws_d)
            check(st, "decompress_range extra")
            assert float((d_y.double() - x.double()).abs().max()) <= eb, "chunks do not add up to the field"
            extras["pipelined"] = {"compress_in_8_parts_ms": round(ms_parts, 4), "decompress_in_8_chunks_ms": round(ms_chunks, 4)}
        extras["other_ops"] = {"decompress_average": {"ms": round(ms_avg, 4), "values": n_avg,
                                                      "call_frac": round((r_bytes + 4 * m) / ms_avg / 1e6 / HBM_PEAK_GBS, 4)}}

    # ---------------- reference CPU codec on the same buffers (same mix as the step) ----------------
    cpu = None
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import zcref
        zcref.set_indexed(indexed)
        ns = min(n, 1 << 27)
        mr = min(m, 1 << 26)
        st, _ = zc.zc_compress(x, n, eb, d_stream, ws_c, flags=flags)
        check(st, "compress")
        st, _ = zc.zc_decompress(d_stream, c_bytes, d_y, ws_d, flags=variant)
        check(st, "decompress")
        xs = x[:ns].cpu().numpy()
        rs = [r[:mr].cpu().numpy() for r in ranks]
        t = time.perf_counter()
        st, s_ref, _ = zcref.compress(xs, eb)
        t_c = time.perf_counter() - t
        t = time.perf_counter()
        _, y_ref, _ = zcref.decompress(s_ref)
        t_d = time.perf_counter() - t
        ss = [zcref.compress(r, eb_r)[1] for r in rs]      # untimed setup, as on the GPU
        t = time.perf_counter()
        st_r, red_ref, _ = zcref.reduce(ss)
        t_r = time.perf_counter() - t
        assert st == 0 and st_r == 0
        # Cross-check of the GPU results of this run.  The sample is a prefix and blocks are independent: the
        # reconstruction must agree bit for bit; when the sample is the whole buffer, so must the streams.
        assert np.array_equal(d_y[:ns].cpu().numpy().view(np.uint32), y_ref.view(np.uint32)), "GPU != reference"
        if ns == n:
            assert d_stream[:c_bytes].cpu().numpy().tobytes() == s_ref.tobytes(), "compressed stream != reference"
        if mr == m:
            assert d_red[:r_bytes].cpu().numpy().tobytes() == red_ref.tobytes(), "reduced stream != reference"
        zcref.set_indexed(False)
        sample_bytes = 4 * ns + 4 * ns + 4 * mr * K
        cpu = {
            "value": round(sample_bytes / (t_c + t_d + t_r) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"first {ns} values of the field (compress+decompress) and first {mr} values of each of the "
                      f"{K} rank buffers (reduce); {t_c + t_d + t_r:.1f} s of CPU time",
            "compress_GBps": round(4 * ns / t_c / 1e9, 4), "decompress_GBps": round(4 * ns / t_d / 1e9, 4),
            "reduce_GBps": round(4 * mr * K / t_r / 1e9, 4),
        }

    out = {
        "metric": "compress / decompress / fused-reduce GB/s (fp32 input) and % HBM peak",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64+u32", "data": "synthetic",
        "value_is": "fp32 bytes the step stands for (4n + 4n + 4*8*m) per second, not bytes moved",
        "algorithmic_GBps": round(total_alg / ms_per_step / 1e6, 1),
        "hbm_frac_step": round(total_alg / ms_per_step / 1e6 / HBM_PEAK_GBS, 4),
        "config": {"workload": f"{side}^3 fp32 power-law Gaussian field, rel eb {args.rel:g}: compress + decompress (of a "
                               f"stream written {ROTATION - 1} steps earlier); fused reduce of {K} compressed rank buffers of {m} values",
                   "streams": args.streams, "tiles": args.tiles, "settle_ms": args.settle_ms, "block": 32, "abs_eb": eb,
                   "compressed_bytes": c_bytes, "ratio": round(4 * n / c_bytes, 3),
                   "reduce_in_bytes": sum(chunk_bytes), "reduce_out_bytes": r_bytes, "source_digest": source_digest()},
        "roofline": dict(stages[dominant]["roofline"], kernel=dominant + "_kernel"),
        "stages": stages,
        "extras": extras,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
