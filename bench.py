#!/usr/bin/env python3
"""Benchmark of the zc hot path on one MI355X.

One step = one pass of the whole hot path on synthetic data already resident in HBM:
  1. zc_compress    of a 512^3 fp32 Gaussian random field (P(k) ~ k^-3), rel. bound 1e-4
  2. zc_decompress  of that stream
  3. zc_reduce_compressed of 8 compressed rank buffers of 64M values (same generator, other
     seeds, common absolute bound), the local step of a compressed Allreduce.
`value` is fp32 gigabytes moved through the step per second: 4n (compress input) + 4n
(decompress output) + 4*8*m (the fp32 data the 8 reduce operands stand for), over the step
time.  Per-stage throughput and roofline figures are in `stages`; `roofline` repeats the stage
whose kernel runs longest.  The reference CPU codec is timed on a bounded sample of the same
buffers as `cpu_baseline` (reported baseline, not a target).
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of each main kernel on the default workload, from the rocprofv3 counter runs
# summarised under profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by what the counter reads on a plain
# copy of the field in the same run).  Counters cannot be read from inside this script, so the figures are
# carried here and reported only when the run is that workload.
PROFILED_TRAFFIC = {"indexed": {"compress": 755.8e6, "decompress": 746.5e6, "reduce": 973.4e6},
                    "plain": {"compress": 755.1e6, "decompress": 746.9e6, "reduce": 972.0e6}}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--rel", type=float, default=1e-4, help="value-range-relative error bound of the timed step")
    ap.add_argument("--side", type=int, default=512, help="field side; 512 is the benchmark configuration")
    ap.add_argument("--streams", choices=("plain", "indexed"), default="indexed",
                    help="stream variant of every call: indexed streams carry a segment index (zc_set_indexed_streams)")
    ap.add_argument("--settle-ms", type=float, default=100.0,
                    help="untimed steps run for this long before the warmup steps: the first milliseconds of work on an "
                         "idle GPU run several percent slow")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the untimed sweep over the other error bounds")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run plain device copies of the field (4n B read + 4n B written each): the known "
                         "traffic that calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import paper_2502_18554_amd as zc
    from paper_2502_18554_amd import synth
    from paper_2502_18554_amd.binding import ZC_OK

    zc.binding.lib()                      # fails loudly if the HIP library is missing
    indexed = args.streams == "indexed"
    zc.zc_set_indexed_streams(indexed)
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
    d_stream = u8(zc.zc_compress_bound(n))
    d_y = torch.empty(n, dtype=torch.float32, device=dev)
    ws_c, ws_d = u8(zc.zc_workspace_bytes(n, 1)), u8(zc.zc_workspace_bytes(n, 1))

    ranks, chunks, chunk_bytes = [], [], []
    m = shape_r[0] * shape_r[1] * shape_r[2]
    eb_r = float(torch.tensor(args.rel * 2.0, dtype=torch.float32))     # common bound: fields span [-1, 1]
    scratch = u8(zc.zc_compress_bound(m))
    ws_r = u8(zc.zc_workspace_bytes(m, K))
    for r in range(K):
        xr = synth.power_law_field(shape_r, seed=100 + r, device=dev)
        st, total = zc.zc_compress(xr, m, eb_r, scratch, ws_r)
        check(st, f"compress rank {r}")
        chunks.append(scratch[:total].clone())
        chunk_bytes.append(total)
        ranks.append(xr)
    d_red = u8(zc.zc_compress_bound(m))

    st, c_bytes = zc.zc_compress(x, n, eb, d_stream, ws_c)
    check(st, "compress")
    st, n_out = zc.zc_decompress(d_stream, c_bytes, d_y, ws_d)
    check(st, "decompress")
    st, r_bytes = zc.zc_reduce_compressed(chunks, chunk_bytes, d_red, ws_r)
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

    def step(events=None):
        if events:
            events[0].record()
        zc.zc_compress(x, n, eb, d_stream, ws_c, sync=False)
        if events:
            events[1].record()
        zc.zc_decompress(d_stream, c_bytes, d_y, ws_d, sync=False)
        if events:
            events[2].record()
        zc.zc_reduce_compressed(chunks, chunk_bytes, d_red, ws_r, sync=False)
        if events:
            events[3].record()

    def kernel_averages(records):
        return {s: (sum(ms for name, ms in records if name == s) / max(1, sum(1 for name, _ in records if name == s)))
                for s in stage_names}

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
    for ws, what in ((ws_c, "compress"), (ws_d, "decompress"), (ws_r, "reduce")):
        st, _ = zc.zc_finish(ws)
        check(st, what + " (timed loop)")
    assert len(timed_records) == args.steps and all(name == dominant for name, _ in timed_records), len(timed_records)
    # Per-call times (set-up kernels included) and the other kernels' times come from two more passes over
    # the same steps, one with an event between the calls, one with every main kernel timed: an event record
    # holds back the launch behind it by a few microseconds, which the timed region above should not pay.
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    zc.zc_profile_enable(True)
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    kernel_ms = kernel_averages(zc.zc_profile_collect())
    zc.zc_profile_enable(False)
    kernel_ms[dominant] = sum(ms for _, ms in timed_records) / len(timed_records)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    stage_ms = {s: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i, s in enumerate(stage_names)}
    stages = {}
    for s in stage_names:
        # stage = the whole call (set-up kernels included); roofline = its main kernel alone
        gbs = alg_bytes[s] / kernel_ms[s] / 1e6
        stages[s] = {
            "ms": round(stage_ms[s], 4),
            "fp32_GBps": round(fp32_bytes[s] / stage_ms[s] / 1e6, 1),
            "kernel_ms": round(kernel_ms[s], 4),
            "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(gbs / HBM_PEAK_GBS, 4),
                         "traffic": PROFILED_TRAFFIC[args.streams][s] if (side == 512 and args.rel == 1e-4) else None},
            "algorithmic_bytes": alg_bytes[s],
        }
    total_fp32 = sum(fp32_bytes.values())
    value = total_fp32 / ms_per_step / 1e6

    # ---------------- untimed extras: the other error bounds of the 512^3 configuration ----------------
    extras = {}
    if not args.no_extras:
        for rel in (1e-2, 1e-3, 1e-4):
            e = synth.abs_bound(x, rel)
            st, cb = zc.zc_compress(x, n, e, d_stream, ws_c)
            check(st, "compress extra")
            res = {"ratio": round(4 * n / cb, 3)}
            for name, fn in (("compress", lambda: zc.zc_compress(x, n, e, d_stream, ws_c, sync=False)),
                             ("decompress", lambda: zc.zc_decompress(d_stream, cb, d_y, ws_d, sync=False))):
                for _ in range(10):
                    fn()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(10):
                    fn()
                b.record()
                torch.cuda.synchronize()
                ms = a.elapsed_time(b) / 10
                res[name] = {"ms": round(ms, 4), "fp32_GBps": round(4 * n / ms / 1e6, 1),
                             "hbm_frac": round((4 * n + cb) / ms / 1e6 / HBM_PEAK_GBS, 4)}
            extras[f"rel_{rel:g}"] = res
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
        import math
        extras["quality"] = {"max_err": q4[0], "nrmse": rmse / rng_x, "psnr_dB": round(20 * math.log10(rng_x / rmse), 2),
                             "ms": round(ms, 4), "hbm_frac": round(8 * n / ms / 1e6 / HBM_PEAK_GBS, 4)}
        # the step as a HIP graph: the asynchronous calls only launch kernels, so the three calls
        # are captured once and replayed
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0g = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_g = (time.perf_counter() - t0g) * 1e3 / args.steps
        for ws, what in ((ws_c, "compress"), (ws_d, "decompress"), (ws_r, "reduce")):
            st, _ = zc.zc_finish(ws)
            check(st, what + " (graph replay)")
        extras["hip_graph"] = {"ms_per_step": round(ms_g, 4), "value_GBps": round(total_fp32 / ms_g / 1e6, 1)}
        del graph
        # the same step on the other stream variant (plain <-> indexed), inputs compressed anew
        other = not indexed
        zc.zc_set_indexed_streams(other)
        o_stream, o_red = u8(zc.zc_compress_bound(n)), u8(zc.zc_compress_bound(m))
        o_chunks, o_bytes = [], []
        for r in range(K):
            st, total = zc.zc_compress(ranks[r], m, eb_r, o_red, ws_r)
            check(st, "compress rank (other variant)")
            o_chunks.append(o_red[:total].clone())
            o_bytes.append(total)
        st, oc_bytes = zc.zc_compress(x, n, eb, o_stream, ws_c)
        check(st, "compress (other variant)")

        def other_step():
            zc.zc_compress(x, n, eb, o_stream, ws_c, sync=False)
            zc.zc_decompress(o_stream, oc_bytes, d_y, ws_d, sync=False)
            zc.zc_reduce_compressed(o_chunks, o_bytes, o_red, ws_r, sync=False)

        for _ in range(args.warmup):
            other_step()
        torch.cuda.synchronize()
        t0o = time.perf_counter()
        for _ in range(args.steps):
            other_step()
        torch.cuda.synchronize()
        ms_o = (time.perf_counter() - t0o) * 1e3 / args.steps
        for ws, what in ((ws_c, "compress"), (ws_d, "decompress"), (ws_r, "reduce")):
            st, _ = zc.zc_finish(ws)
            check(st, what + " (other variant)")
        extras["other_stream_variant"] = {"streams": "indexed" if other else "plain", "ms_per_step": round(ms_o, 4),
                                          "value_GBps": round(total_fp32 / ms_o / 1e6, 1), "compressed_bytes": oc_bytes}
        zc.zc_set_indexed_streams(indexed)
        del o_stream, o_red, o_chunks
        # the tail of the compressed Allgather at the shape of the reduce above: the 8 rank streams
        # decompressed by 8 calls and by one call
        outs = [torch.empty(m, dtype=torch.float32, device=dev) for _ in range(K)]
        ws_k = [u8(zc.zc_workspace_bytes(m, 1)) for _ in range(K)]

        def eight_calls():
            for i in range(K):
                zc.zc_decompress(chunks[i], chunk_bytes[i], outs[i], ws_k[i], sync=False)

        def one_call():
            zc.zc_decompress_many(chunks, chunk_bytes, outs, ws_r, sync=False)

        res = {"workload": f"{K} streams of {m} values (abs eb {eb_r:g}) -> {K} fp32 buffers"}
        for name, fn in (("eight_calls", eight_calls), ("one_call", one_call)):
            for _ in range(3):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(5):
                fn()
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / 5
            res[name] = {"ms": round(ms, 4), "fp32_GBps": round(4 * m * K / ms / 1e6, 1),
                         "hbm_frac": round((sum(chunk_bytes) + 4 * m * K) / ms / 1e6 / HBM_PEAK_GBS, 4)}
        st, _ = zc.zc_finish(ws_r)
        check(st, "decompress_many extra")
        extras["decompress_many"] = res
        del outs, ws_k
        # one round of the ring reduce-scatter at the shape of the reduce above: the received
        # stream of rank 0 plus the uncompressed buffer of rank 1 -> stream of the sums
        st, s_bytes = zc.zc_reduce_step(chunks[0], chunk_bytes[0], ranks[1], m, scratch, ws_r)
        check(st, "reduce_step extra")
        for _ in range(5):
            zc.zc_reduce_step(chunks[0], chunk_bytes[0], ranks[1], m, scratch, ws_r, sync=False)
        torch.cuda.synchronize()
        zc.zc_profile_enable(True)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            zc.zc_reduce_step(chunks[0], chunk_bytes[0], ranks[1], m, scratch, ws_r, sync=False)
        b.record()
        torch.cuda.synchronize()
        kt = [ms for name, ms in zc.zc_profile_collect() if name == "reduce_step"]
        zc.zc_profile_enable(False)
        ms = a.elapsed_time(b) / 10
        alg = chunk_bytes[0] + 4 * m + s_bytes
        extras["reduce_step"] = {"workload": f"received stream of {m} values + {m} local fp32 values -> stream",
                                 "ms": round(ms, 4), "kernel_ms": round(sum(kt) / len(kt), 4),
                                 "algorithmic_bytes": alg, "fp32_GBps": round(8 * m / ms / 1e6, 1),
                                 "hbm_frac": round(alg / (sum(kt) / len(kt)) / 1e6 / HBM_PEAK_GBS, 4)}
        # the other aggregation functions: a Max round at the same shape, and the averaging
        # decompression of the reduced stream of the step above
        def timed(fn, reps=10):
            for _ in range(3):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        ms_max = timed(lambda: zc.zc_reduce_step_op(chunks[0], chunk_bytes[0], ranks[1], m, zc.binding.ZC_OP_MAX, scratch,
                                                    ws_r, sync=False))
        st, _ = zc.zc_finish(ws_r)
        check(st, "reduce_step_op extra")
        d_avg = torch.empty(m, dtype=torch.float32, device=dev)      # (d_y keeps the field for the cross-check below)
        ms_avg = timed(lambda: zc.zc_decompress_average(d_red, r_bytes, d_avg, ws_d, sync=False))
        st, n_avg = zc.zc_finish(ws_d)
        check(st, "decompress_average extra")
        # the field compressed in 8 parts (zc_compress_part), and decompressed in 8 chunks (zc_decompress_range)
        part = n // 8

        def in_parts():
            for i in range(8):
                zc.zc_compress_part(x, n, eb, i * part, part if i < 7 else n - 7 * part, d_stream, ws_c, sync=False)

        def in_chunks():
            for i in range(8):
                zc.zc_decompress_range(d_stream, c_bytes, i * part, part, d_y[i * part:(i + 1) * part], ws_d, sync=False)

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
        extras["other_ops"] = {"reduce_step_max_ms": round(ms_max, 4),
                               "decompress_average": {"ms": round(ms_avg, 4), "values": n_avg,
                                                      "hbm_frac": round((r_bytes + 4 * m) / ms_avg / 1e6 / HBM_PEAK_GBS, 4)}}

    # ---------------- reference CPU codec on a bounded sample (same mix as the step) ----------------
    cpu = None
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import zcref
        ns = min(n, 1 << 27)
        mr = min(m, 1 << 26)
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
        # the sample is a prefix, blocks are independent: reconstruction and widths must agree bit for bit
        assert np.array_equal(d_y[:ns].cpu().numpy().view(np.uint32), y_ref.view(np.uint32)), "GPU != reference"
        # (the reference writes plain streams; an indexed stream has its width table behind the index)
        def widths_at(n_values):
            nb_all = (n_values + 31) // 32
            return 32 + ((4 * ((nb_all + 63) // 64 + 1) + 15) // 16 * 16 if indexed else 0)
        nbs = ns // 32
        assert np.array_equal(d_stream[widths_at(n):widths_at(n) + nbs].cpu().numpy(), s_ref[32:32 + nbs]), "widths differ"
        assert np.array_equal(d_red[widths_at(m):widths_at(m) + mr // 32].cpu().numpy(), red_ref[32:32 + mr // 32]), \
            "reduce widths differ"
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
        "config": {"workload": f"{side}^3 fp32 power-law Gaussian field, rel eb {args.rel:g}: compress + decompress; "
                               f"fused reduce of {K} compressed rank buffers of {m} values",
                   "streams": args.streams, "settle_ms": args.settle_ms, "block": 32, "abs_eb": eb, "compressed_bytes": c_bytes, "ratio": round(4 * n / c_bytes, 3),
                   "reduce_in_bytes": sum(chunk_bytes), "reduce_out_bytes": r_bytes},
        "roofline": dict(stages[dominant]["roofline"], kernel=dominant + "_kernel"),
        "stages": stages,
        "extras": extras,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
