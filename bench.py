#!/usr/bin/env python3
"""Benchmark of the FastSGD codec on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: for every keep fraction
of the workload's sweep, fastsgd_compress followed by fastsgd_decompress of that stream, inputs
resident in HBM.  Prints ONE JSON line (metric = input GB/s of the round trip, 8 bytes per element:
4-byte key + 4-byte value, the paper's 64 bits per original pair, Section 3.4).
"""
import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "bench_c4_hbm_traffic.md")


def threshold_bits(total, base, tau):
    """Bit pattern of the early-stop threshold sum / b^tau (Algorithm 1 line 2) the way the codec
    evaluates it: the power by repeated float64 multiplication, the quotient rounded up to float32.
    Only used to count, for the byte accounting, the rows the value pass has to read."""
    import numpy as np
    p = 1.0
    for _ in range(tau):
        p = p * base
    t = total / p
    f = np.float32(t)
    if float(f) < t:
        f = np.nextafter(f, np.float32(np.inf))
    return int(np.array([f], np.float32).view(np.uint32)[0])


def committed_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, or None."""
    try:
        for line in open(TRAFFIC_FILE):
            m = re.match(r"\|\s*(\w+)\s*\|.*\|\s*([0-9.eE+]+)\s*\|\s*$", line)
            if m and m.group(1) == kernel:
                return float(m.group(2))
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replays of the per-point timings")
    ap.add_argument("--cpu-sample", type=int, default=0, help="elements the oracle is timed on (0 = the whole workload)")
    ap.add_argument("--widening", action="store_true",
                    help="also time decode-and-aggregate (4 copies of each stream) and decode-and-update (Adam); "
                         "reported under \"widening\", outside the timed step")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run, before anything else, one plain elementwise kernel over the value array "
                         "(out = -in: n*4 bytes read, n*4 bytes written), the dispatch of known HBM traffic the "
                         "rocprofv3 counter runs are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this codec is a single-GPU path (one worker's gradient); --gpus must be 1. "
              "Nothing was run.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2112_04291_amd import binding as B
    from paper_2112_04291_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()

    gen = {"c1": W.config1, "c2": W.config2, "c3": W.config3, "c4": W.config4}[args.workload]
    t0 = time.time()
    if args.scale != 1.0 and args.workload in ("c2", "c4"):
        w = gen(n=int({"c2": 25_600_000, "c4": 124_000_000}[args.workload] * args.scale))
    else:
        w = gen()
    keeps = w.meta["keep"]
    bases = W.solve_bases(w.values, keeps)
    n = int(w.values.size)
    print(f"[bench] workload {w.name}: n={n} keeps={keeps} bases={bases} (generated in {time.time() - t0:.1f}s)",
          file=sys.stderr, flush=True)

    keys = torch.from_numpy(w.keys.view(np.int32)).cuda()
    values = torch.from_numpy(w.values).cuda()
    plist = [B.params(b) for b in bases]

    if args.calibrate:
        ref_copy = torch.empty_like(values)
        torch.neg(values, out=ref_copy)          # n*4 bytes read + n*4 bytes written
        torch.cuda.synchronize()
        del ref_copy

    # one output buffer per sweep point (sized from a first, untimed pass), shared workspace
    probe = B.Buffers(n, plist[0])
    points = []
    for keep, p in zip(keeps, plist):
        rc = B.compress(keys, values, p, probe.out, probe.out_offsets, probe.status, probe.workspace, n=n,
                        out_capacity=probe.out_capacity)
        torch.cuda.synchronize()
        assert rc == B.OK and int(probe.status[0]) == B.OK, (rc, int(probe.status[0]))
        nbytes = int(probe.out_offsets[0])
        hdr = probe.out_bytes_view()[:64].cpu().numpy()
        d = int(hdr[40:48].view("<u8")[0])
        total = float(hdr[24:32].view("<f8")[0])
        out = torch.empty(nbytes // 8 + 8, dtype=torch.int64, device="cuda")
        points.append(dict(keep=keep, p=p, out=out, cap=nbytes, bytes=nbytes, d=d, sum=total,
                           keys_out=torch.empty(max(d, 1), dtype=torch.int32, device="cuda"),
                           vals_out=torch.empty(max(d, 1), dtype=torch.float32, device="cuda")))
    ws, dws = probe.workspace, probe.dec_workspace
    obytes = torch.zeros(2, dtype=torch.int64, device="cuda")
    count = torch.zeros(2, dtype=torch.int64, device="cuda")
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    del probe.out

    # granules (32 elements, 128 bytes) whose bound reaches the threshold: what the value pass has to read.
    # The bound is the largest |v| of the granule as a bit pattern, upper 16 bits, rounded up.
    rows = (n + 255) // 256
    pad = rows * 256 - n
    absbits = values.abs().view(torch.int32)
    if pad:
        absbits = torch.cat([absbits, torch.zeros(pad, dtype=torch.int32, device="cuda")])
    qbound = ((absbits.view(rows * 8, 32).max(dim=1).values.to(torch.int64) + 0xFFFF) >> 16) << 16
    for pt in points:
        pt["granules_active"] = int((qbound >= threshold_bits(pt["sum"], pt["p"].base, pt["p"].tau)).sum())
    del absbits, qbound

    def do_compress(pt):
        rc = B.compress(keys, values, pt["p"], pt["out"], obytes, status, ws, n=n, out_capacity=pt["cap"])
        assert rc == B.OK

    def do_decompress(pt):
        rc = B.decompress(pt["out"], pt["bytes"], pt["keys_out"], pt["vals_out"], count, status, dws, capacity=pt["d"])
        assert rc == B.OK

    def step():
        for pt in points:
            do_compress(pt)
            do_decompress(pt)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert int(status[0]) == B.OK and int(count[0]) == points[-1]["d"]
    ms_per_step = 1e3 * elapsed / args.steps
    in_bytes_step = 8.0 * n * len(points)
    value = in_bytes_step / (elapsed / args.steps) / 1e9

    # per direction and per sweep point, event-timed on the launch stream
    def timed(fn, pt, iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn(pt)
        e0.record()
        for _ in range(iters):
            fn(pt)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    # the same calls replayed from a HIP graph (a call is kernel launches only, so it can be captured):
    # what the kernels take once the launch gaps between them are gone
    def graph_timed(fn, pt, iters):
        if args.no_graph:
            return None
        cur = torch.cuda.current_stream()
        side = torch.cuda.Stream()
        side.wait_stream(cur)
        with torch.cuda.stream(side):
            fn(pt)                                           # warm-up outside the capture
        cur.wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(iters):
                fn(pt)
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    detail = []
    kern_time = {}
    kern_bytes = {}
    for pt in points:
        c_ms = timed(do_compress, pt, args.steps)
        d_ms = timed(do_decompress, pt, args.steps)
        cg_ms = graph_timed(do_compress, pt, args.steps)
        dg_ms = graph_timed(do_decompress, pt, args.steps)
        assert int(status[0]) == B.OK and int(count[0]) == pt["d"] and int(obytes[0]) == pt["bytes"]
        rc, kc = B.profile_compress(keys, values, pt["p"], pt["out"], obytes, status, ws, args.steps, n=n,
                                    out_capacity=pt["cap"])
        assert rc == B.OK
        rc, kd = B.profile_decompress(pt["out"], pt["bytes"], pt["keys_out"], pt["vals_out"], count, status, dws,
                                      args.steps, capacity=pt["d"])
        assert rc == B.OK
        d, sb, qa = pt["d"], pt["bytes"], pt["granules_active"]
        # algorithmic bytes per launch: what each kernel's method has to move
        alg = {
            "abs_sum": 4.0 * n + 16.0 * rows,                    # every value once; eight 16-bit bounds per row out
            "encode_values": 16.0 * rows + 128.0 * qa + 4.0 * d + 5.0 * d,   # bounds; granules that can hold a
                                                                 # survivor; keys of survivors; key + code byte to scratch
            "measure_keys": 4.0 * d,                             # surviving keys
            "pack_keys": 5.0 * d + (sb - 64),                    # surviving keys and code bytes in, stream out
            "decode": sb + 8.0 * d,                              # stream in, (key, value) pairs out
        }
        for k, v in {**kc, **{"decode": kd["decode"], "decode_setup": kd["setup"]}}.items():
            kern_time[k] = kern_time.get(k, 0.0) + v
        for k, v in alg.items():
            kern_bytes[k] = kern_bytes.get(k, 0.0) + v
        comp_alg = 8.0 * n + 18.0 * d + sb                       # two value passes + survivor traffic + stream
        detail.append(dict(keep=pt["keep"], base=pt["p"].base, d=d, stream_bytes=sb, ratio=8.0 * n / sb,
                           bits_per_key=8.0 * (sb - 64 - d) / max(d, 1), granules_read=qa, granules=8 * rows,
                           compress_ms=c_ms, decompress_ms=d_ms,
                           compress_graph_ms=cg_ms, decompress_graph_ms=dg_ms,
                           compress_graph_hbm_frac=None if cg_ms is None else comp_alg / cg_ms / 1e6 / HBM_PEAK_GBPS,
                           decompress_graph_hbm_frac=None if dg_ms is None else (sb + 8.0 * d) / dg_ms / 1e6 / HBM_PEAK_GBPS,
                           compress_input_GBps=8.0 * n / c_ms / 1e6, decompress_input_GBps=8.0 * n / d_ms / 1e6,
                           compress_elements_per_s=n / c_ms * 1e3,
                           compress_hbm_frac=comp_alg / c_ms / 1e6 / HBM_PEAK_GBPS,
                           decompress_hbm_frac=(sb + 8.0 * d) / d_ms / 1e6 / HBM_PEAK_GBPS,
                           kernels_ms={**kc, **{"decode_" + k: v for k, v in kd.items()}}))

    dominant = max(("abs_sum", "encode_values"), key=lambda k: kern_time[k])
    kernels = {k: dict(ms_total=kern_time[k], achieved_GBps=kern_bytes[k] / kern_time[k] / 1e6,
                       frac=kern_bytes[k] / kern_time[k] / 1e6 / HBM_PEAK_GBPS) for k in kern_bytes}
    launches = len(points)
    roofline = dict(bound="hbm", kernel="k_" + dominant,
                    achieved=kern_bytes[dominant] / kern_time[dominant] / 1e6, peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=kern_bytes[dominant] / kern_time[dominant] / 1e6 / HBM_PEAK_GBPS,
                    traffic=committed_traffic("k_" + dominant),
                    traffic_source="profiles/bench_c4_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, "
                                   "separate runs of this command, scaled by a plain elementwise kernel of known size; bytes per launch)",
                    avg_launch_ms=kern_time[dominant] / launches,
                    algorithmic_bytes_per_launch=kern_bytes[dominant] / launches)

    widening = None
    if args.widening:
        widening = []
        dense = torch.zeros(n, dtype=torch.float32, device="cuda")
        theta, m1, v1 = (torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(3))
        aws = torch.empty(B.decompress_workspace_size(4) // 8 + 32, dtype=torch.int64, device="cuda")
        for pt in points:
            sb = pt["bytes"]
            four = torch.cat([pt["out"].view(torch.uint8)[:sb]] * 4 + [torch.zeros(64, dtype=torch.uint8, device="cuda")])
            offs = torch.tensor([0, sb, 2 * sb, 3 * sb, 4 * sb], dtype=torch.int64, device="cuda")

            def do_acc(_):
                assert B.decompress_accumulate(four, 4 * sb, offs, 4, dense, count, status, aws) == B.OK

            def do_adam(_):
                assert B.decompress_adam(pt["out"], sb, theta, m1, v1, 1e-3, 0.9, 0.999, 1e-8, count, status, aws) == B.OK

            a_ms = timed(do_acc, pt, args.steps)
            assert int(status[0]) == B.OK and int(count[0]) == 4 * pt["d"]
            u_ms = timed(do_adam, pt, args.steps)
            assert int(status[0]) == B.OK and int(count[0]) == pt["d"]
            widening.append(dict(keep=pt["keep"], d=pt["d"], accumulate_4_streams_ms=a_ms, adam_ms=u_ms,
                                 accumulate_pairs_per_s=4.0 * pt["d"] / a_ms * 1e3, adam_pairs_per_s=pt["d"] / u_ms * 1e3))
            del four
        del dense, theta, m1, v1
        # variants of the encoder: no key array (keys are the indices), and the paper's base b = 1.1 with
        # the threshold that keeps about the same fraction (b^tau = base^128; above 128 a token is 9 bits)
        cap_all = max(B.compressed_size(n, B.params(1.1, 256)), B.compressed_size(n, plist[0]))
        vout = torch.empty(cap_all // 8 + 8, dtype=torch.int64, device="cuda")
        for pt, wd in zip(points, widening):
            def do_implicit(_):
                assert B.compress(None, values, pt["p"], vout, obytes, status, ws, n=n, out_capacity=cap_all) == B.OK

            i_ms = timed(do_implicit, pt, args.steps)
            assert int(status[0]) == B.OK and int(obytes[0]) == pt["bytes"]
            tau11 = min(256, max(1, int(math.ceil(128.0 * math.log(pt["p"].base) / math.log(1.1)))))
            p11 = B.params(1.1, tau11)

            def do_b11(_):
                assert B.compress(keys, values, p11, vout, obytes, status, ws, n=n, out_capacity=cap_all) == B.OK

            b_ms = timed(do_b11, pt, args.steps)
            assert int(status[0]) == B.OK
            sb11 = int(obytes[0])
            d11 = int(vout.view(torch.uint8)[40:48].cpu().numpy().view("<u8")[0])
            k11 = torch.empty(max(d11, 1), dtype=torch.int32, device="cuda")
            v11 = torch.empty(max(d11, 1), dtype=torch.float32, device="cuda")

            def do_b11_dec(_):
                assert B.decompress(vout, sb11, k11, v11, count, status, dws, capacity=d11) == B.OK

            bd_ms = timed(do_b11_dec, pt, args.steps)
            assert int(status[0]) == B.OK and int(count[0]) == d11
            wd.update(no_key_array_compress_ms=i_ms, base_1p1=dict(tau=tau11, d=d11, stream_bytes=sb11,
                                                                    compress_ms=b_ms, decompress_ms=bd_ms))
            del k11, v11
        del vout

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ref
        m = n if args.cpu_sample <= 0 else min(args.cpu_sample, n)
        sk, sv = w.keys[:m], w.values[:m]
        sbases = bases if m == n else W.solve_bases(sv, keeps)
        t0 = time.perf_counter()
        for b in sbases:
            rc, st = ref.compress(sk, sv, ref.params(b))
            assert rc == ref.OK
            rc, k2, v2 = ref.decompress(st)
            assert rc == ref.OK
        cpu_s = time.perf_counter() - t0
        cpu = dict(value=8.0 * m * len(sbases) / cpu_s / 1e9, unit="GB/s", cores=1, kind="oracle",
                   sample=f"{'all' if m == n else 'first'} {m} elements of {w.name}, all {len(sbases)} keep "
                          f"fractions, compress+decompress once, {cpu_s:.1f} s on one host core")

    line = {
        "metric": "compress & decompress input GB/s (% of HBM peak) on 1 MI355X; compression ratio",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n": n, "keep_fractions": keeps, "tau": 128, "flag_bits": 2,
                   "block_keys": 1024, "step": "compress+decompress at every keep fraction",
                   "arithmetic": "f32 values and u32 keys compared as IEEE bit patterns; f64 boundary table"},
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "detail": detail,
    }
    if widening is not None:
        line["widening"] = widening
    print(json.dumps(line))


if __name__ == "__main__":
    main()
