#!/usr/bin/env python3
"""Benchmark of the FastSGD codec on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: for every keep fraction
of the workload's sweep, fastsgd_compress followed by fastsgd_decompress of that stream (config 5: one
fastsgd_compress_segmented + fastsgd_decompress_segmented over the 160 tensors), inputs resident in HBM.
Prints ONE JSON line (metric = input GB/s of the round trip, 8 bytes per element: 4-byte key + 4-byte
value, the paper's 64 bits per original pair, Section 3.4).

A dense gradient (configs 2, 4, 5: keys 0..n-1) is passed the way a caller holding one passes it, without a
key array (d_keys = NULL: the keys are the indices); the same call WITH the explicit key array 0..n-1 is timed
beside it and reported as `compress_explicit_keys_*`.  Sparse gradients (configs 1, 3) have their key arrays.

Byte counts used below, per call (N elements, d survivors, sb stream bytes, rows = N/256):
  compress, "algorithmic"  no key array: 8N + 14d + sb; key array: 8N + 18d + sb : both value passes in full, key
                           (4d, where there is a key array) + scratch traffic of the survivors (5d scratch out,
                           5d + 4d scratch back in), stream out
  compress, "moved"        what the kernels are built to move: the second pass reads only the 128-byte
                           granules whose bound reaches the threshold (q of them), and with an explicit key array
                           whole 128-byte lines around the surviving keys (key_lines of them):
                           4N + 32 rows + 128 q [+ 128 key_lines] + 14d + sb
  decompress               sb + 8d
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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "bench_c4_all_hbm_traffic.md")


def threshold_bits(total, base, tau):
    """Bit pattern of the early-stop threshold sum / b^tau (Algorithm 1 line 2) the way the codec
    evaluates it: the power by repeated float64 multiplication, the quotient rounded up to float32.
    Only used to count, for the byte accounting, the granules the value pass has to read."""
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


def host_cpu():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return model, os.cpu_count(), usable


class Timer:
    """Event timing on torch's current stream, which is the stream the binding launches on."""

    def __init__(self, torch, use_graph):
        self.torch = torch
        self.use_graph = use_graph

    def eager(self, fn, iters):
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn(0)
        e0.record()
        for i in range(iters):
            fn(i + 1)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    def graph(self, fn, iters):
        """The same calls replayed from a HIP graph (a call is kernel launches only, so it can be
        captured): what the kernels take once the launch gaps between them are gone."""
        if not self.use_graph:
            return None
        torch = self.torch
        cur = torch.cuda.current_stream()
        side = torch.cuda.Stream()
        side.wait_stream(cur)
        with torch.cuda.stream(side):
            fn(0)                                            # warm-up outside the capture
        cur.wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(iters):
                fn(i)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters


class SingleCase:
    """One gradient (configs 1-4): a sweep of keep fractions, one stream per point."""

    def __init__(self, w, keeps, copies=1):
        import numpy as np
        import torch
        from paper_2112_04291_amd import binding as B
        from paper_2112_04291_amd import workloads as W
        self.w, self.B, self.torch = w, B, torch
        self.n = n = int(w.values.size)
        self.keeps = list(keeps)
        self.bases = W.solve_bases(w.values, self.keeps)
        # `copies` copies of the input, used in turn, so that a small input is not served from the caches
        self.keys = [torch.from_numpy(w.keys.view(np.int32)).cuda() for _ in range(copies)]
        self.values = [torch.from_numpy(w.values).cuda() for _ in range(copies)]
        self.dense = bool(n and w.keys[0] == 0 and w.keys[-1] == n - 1)       # keys are the indices
        plist = [B.params(b) for b in self.bases]
        probe = B.Buffers(n, plist[0])
        self.points = []
        for keep, p in zip(self.keeps, plist):
            rc = B.compress(None if self.dense else self.keys[0], self.values[0], p, probe.out, probe.out_offsets,
                            probe.status, probe.workspace, n=n, out_capacity=probe.out_capacity)
            torch.cuda.synchronize()
            assert rc == B.OK and int(probe.status[0]) == B.OK, (rc, int(probe.status[0]))
            nbytes = int(probe.out_offsets[0])
            hdr = probe.out_bytes_view()[:64].cpu().numpy()
            d = int(hdr[40:48].view("<u8")[0])
            total = float(hdr[24:32].view("<f8")[0])
            out = torch.empty(nbytes // 8 + 8, dtype=torch.int64, device="cuda")
            self.points.append(dict(keep=keep, p=p, out=out, cap=nbytes, bytes=nbytes, d=d, sum=total,
                                    keys_out=torch.empty(max(d, 1), dtype=torch.int32, device="cuda"),
                                    vals_out=torch.empty(max(d, 1), dtype=torch.float32, device="cuda")))
        self.ws, self.dws = probe.workspace, probe.dec_workspace
        self.obytes = torch.zeros(2, dtype=torch.int64, device="cuda")
        self.count = torch.zeros(2, dtype=torch.int64, device="cuda")
        self.status = torch.zeros(2, dtype=torch.int32, device="cuda")
        del probe.out

    def count_fetch_units(self):
        """Per point: granules (32 values, 128 bytes) whose bound reaches the threshold -- what the value pass
        has to read -- and, for a dense gradient with an explicit key array, the 128-byte lines of that array
        that hold a surviving key.  The bound is the largest |v| of the granule as a bit pattern, upper 16
        bits, rounded up."""
        torch, n = self.torch, self.n
        rows = (n + 255) // 256
        pad = rows * 256 - n
        absbits = self.values[0].abs().view(torch.int32)
        if pad:
            absbits = torch.cat([absbits, torch.zeros(pad, dtype=torch.int32, device="cuda")])
        qbound = ((absbits.view(rows * 8, 32).max(dim=1).values.to(torch.int64) + 0xFFFF) >> 16) << 16
        for pt in self.points:
            pt["granules_active"] = int((qbound >= threshold_bits(pt["sum"], pt["p"].base, pt["p"].tau)).sum())
            pt["key_lines"] = None
        del absbits, qbound
        if self.dense:
            for pt in self.points:
                self.compress(pt)
                self.decompress(pt)
                torch.cuda.synchronize()
                lines = torch.unique_consecutive(pt["keys_out"][:pt["d"]] >> 5)
                pt["key_lines"] = int(lines.numel())

    def compress(self, pt, i=0, keys=None):
        keys = (not self.dense) if keys is None else keys       # a dense gradient goes without its key array
        k = self.keys[i % len(self.keys)] if keys else None
        rc = self.B.compress(k, self.values[i % len(self.values)], pt["p"], pt["out"], self.obytes, self.status, self.ws,
                             n=self.n, out_capacity=pt["cap"])
        assert rc == self.B.OK

    def decompress(self, pt, i=0):
        rc = self.B.decompress(pt["out"], pt["bytes"], pt["keys_out"], pt["vals_out"], self.count, self.status, self.dws,
                               capacity=pt["d"])
        assert rc == self.B.OK

    def check(self, pt):
        assert int(self.status[0]) == self.B.OK and int(self.count[0]) == pt["d"] and int(self.obytes[0]) == pt["bytes"]

    def stream_bytes_host(self, pt):
        return pt["out"].view(self.torch.uint8)[:pt["bytes"]].cpu().numpy()

    def oracle_streams(self, ref):
        """The oracle over the whole workload, every point: (seconds, [stream per point])."""
        t0 = time.perf_counter()
        streams = []
        for b in self.bases:
            rc, st = ref.compress(self.w.keys, self.w.values, ref.params(b))
            assert rc == ref.OK
            rc, k2, v2 = ref.decompress(st)
            assert rc == ref.OK
            streams.append(st)
        return time.perf_counter() - t0, streams


class BatchCase:
    """Config 5: 160 tensors in one segmented call, every tensor with its own base (1 % kept)."""

    def __init__(self, w, keep, copies=1):
        import numpy as np
        import torch
        from paper_2112_04291_amd import binding as B
        from paper_2112_04291_amd import workloads as W
        self.w, self.B, self.torch = w, B, torch
        self.n = n = int(w.values.size)
        self.keeps = [keep]
        offs = [int(x) for x in w.seg_offsets]
        self.offs = offs
        self.nseg = nseg = len(offs) - 1
        self.bases = [W.solve_bases(w.values[offs[i]:offs[i + 1]], [keep])[0] for i in range(nseg)]
        self.plist = [B.params(b) for b in self.bases]
        self.keys = [torch.from_numpy(w.keys.view(np.int32)).cuda() for _ in range(copies)]
        self.values = [torch.from_numpy(w.values).cuda() for _ in range(copies)]
        self.dense = True                                        # every tensor has the keys 0..n_i-1
        cap = B.compressed_size(max(n, 1), B.params(1.1, 128, 2, 1024)) + (64 + 4096) * nseg
        out = torch.empty(cap // 8 + 8, dtype=torch.int64, device="cuda")
        self.ws = torch.empty(B.workspace_size(n, nseg, 1024) // 8 + 32, dtype=torch.int64, device="cuda")
        self.dws = B.decoder_workspace(nseg)
        self.out_offs = torch.zeros(nseg + 1, dtype=torch.int64, device="cuda")
        self.pair_offs = torch.zeros(nseg + 1, dtype=torch.int64, device="cuda")
        self.status = torch.zeros(2, dtype=torch.int32, device="cuda")
        pt = dict(keep=keep, out=out, p=self.plist[0])
        self.points = [pt]
        self.compress(pt)
        torch.cuda.synchronize()
        assert int(self.status[0]) == B.OK
        so = self.out_offs.cpu().numpy()
        pt["bytes"] = int(so[-1])
        blob = out.view(torch.uint8)[:pt["bytes"]].cpu().numpy()
        pt["d"] = int(sum(int(blob[int(o) + 40:int(o) + 48].view("<u8")[0]) for o in so[:-1]))
        pt["keys_out"] = torch.empty(max(pt["d"], 1), dtype=torch.int32, device="cuda")
        pt["vals_out"] = torch.empty(max(pt["d"], 1), dtype=torch.float32, device="cuda")
        pt["granules_active"] = None
        pt["key_lines"] = None

    def count_fetch_units(self):
        pass

    def compress(self, pt, i=0, keys=None):
        keys = (not self.dense) if keys is None else keys
        k = self.keys[i % len(self.keys)] if keys else None
        rc = self.B.compress_segmented(k, self.values[i % len(self.values)], self.offs, self.plist, pt["out"], self.out_offs,
                                       self.status, self.ws)
        assert rc == self.B.OK

    def decompress(self, pt, i=0):
        rc = self.B.decompress_segmented(pt["out"], pt["bytes"], self.out_offs, self.nseg, pt["keys_out"], pt["vals_out"],
                                         self.pair_offs, self.status, self.dws)
        assert rc == self.B.OK

    def check(self, pt):
        assert int(self.status[0]) == self.B.OK and int(self.pair_offs[self.nseg]) == pt["d"]
        assert int(self.out_offs[self.nseg]) == pt["bytes"]

    def stream_bytes_host(self, pt):
        return pt["out"].view(self.torch.uint8)[:pt["bytes"]].cpu().numpy()

    def oracle_streams(self, ref):
        t0 = time.perf_counter()
        rc, blob, so = ref.compress_segmented(self.w.keys, self.w.values, self.w.seg_offsets,
                                              [ref.params(b) for b in self.bases])
        assert rc == ref.OK
        rc, k2, v2, po = ref.decompress_segmented(blob, so, self.points[0]["d"])
        assert rc == ref.OK
        return time.perf_counter() - t0, [blob]


WORKLOAD_NAMES = {"c1": "c1_tiny_sparse", "c2": "c2_dense_25m", "c3": "c3_sparse_zipf", "c4": "c4_dense_124m",
                  "c5": "c5_segmented"}


def make_case(name, scale=1.0, keeps=None):
    from paper_2112_04291_amd import workloads as W
    t0 = time.time()
    if name == "c5":
        w = W.config5()
        case = BatchCase(w, 0.01, copies=2)
    else:
        gen = {"c1": W.config1, "c2": W.config2, "c3": W.config3, "c4": W.config4}[name]
        if scale != 1.0 and name in ("c2", "c4"):
            w = gen(n=int({"c2": 25_600_000, "c4": 124_000_000}[name] * scale))
        else:
            w = gen()
        in_bytes = 8 * int(w.values.size)
        copies = 1 if in_bytes >= (512 << 20) else min(8, -(-(1 << 30) // max(in_bytes, 1)))
        case = SingleCase(w, keeps or w.meta["keep"], copies=copies)
    print(f"[bench] workload {w.name}: n={case.n} keeps={case.keeps} (ready in {time.time() - t0:.1f}s)",
          file=sys.stderr, flush=True)
    return case


def point_record(case, pt, timer, iters, explicit_keys=True):
    """Timings and rates of one point of a case (compress and decompress each timed on their own)."""
    n, d, sb = case.n, pt["d"], pt["bytes"]
    rows = (n + 255) // 256
    c_ms = timer.eager(lambda i: case.compress(pt, i), iters)
    d_ms = timer.eager(lambda i: case.decompress(pt, i), iters)
    cg_ms = timer.graph(lambda i: case.compress(pt, i), iters)
    dg_ms = timer.graph(lambda i: case.decompress(pt, i), iters)
    case.check(pt)
    key_bytes = 0.0 if case.dense else 4.0 * d                 # key fetch of the survivors, where there is a key array
    comp_alg = 8.0 * n + 14.0 * d + key_bytes + sb             # two value passes + survivor traffic + stream
    dec_alg = sb + 8.0 * d
    rec = dict(keep=pt["keep"], d=d, stream_bytes=sb, ratio=8.0 * n / sb,
               key_array="none (dense gradient: the keys are the indices)" if case.dense else "explicit",
               compress_ms=c_ms, decompress_ms=d_ms, compress_graph_ms=cg_ms, decompress_graph_ms=dg_ms,
               compress_input_GBps=8.0 * n / c_ms / 1e6, decompress_input_GBps=8.0 * n / d_ms / 1e6,
               compress_elements_per_s=n / c_ms * 1e3,
               compress_algorithmic_bytes=comp_alg, decompress_algorithmic_bytes=dec_alg,
               compress_hbm_frac=comp_alg / c_ms / 1e6 / HBM_PEAK_GBPS,
               decompress_hbm_frac=dec_alg / d_ms / 1e6 / HBM_PEAK_GBPS,
               compress_graph_hbm_frac=None if cg_ms is None else comp_alg / cg_ms / 1e6 / HBM_PEAK_GBPS,
               decompress_graph_hbm_frac=None if dg_ms is None else dec_alg / dg_ms / 1e6 / HBM_PEAK_GBPS)
    if pt.get("granules_active") is not None:
        qa = pt["granules_active"]
        moved = 4.0 * n + 32.0 * rows + 128.0 * qa + key_bytes + 14.0 * d + sb
        rec.update(base=pt["p"].base, bits_per_key=8.0 * (sb - 64 - d) / max(d, 1), granules_read=qa, granules=8 * rows,
                   compress_moved_bytes=moved, compress_moved_frac=moved / c_ms / 1e6 / HBM_PEAK_GBPS)
    if case.dense and explicit_keys:
        # the same call with the explicit key array 0..n-1
        e_ms = timer.eager(lambda i: case.compress(pt, i, keys=True), iters)
        case.check(pt)
        ealg = 8.0 * n + 18.0 * d + sb
        rec.update(compress_explicit_keys_ms=e_ms, compress_explicit_keys_algorithmic_bytes=ealg,
                   compress_explicit_keys_hbm_frac=ealg / e_ms / 1e6 / HBM_PEAK_GBPS)
        kl = pt.get("key_lines")
        if kl is not None and pt.get("granules_active") is not None:
            emoved = 4.0 * n + 32.0 * rows + 128.0 * pt["granules_active"] + 128.0 * kl + 14.0 * d + sb
            rec.update(key_lines_read=kl, compress_explicit_keys_moved_bytes=emoved,
                       compress_explicit_keys_moved_frac=emoved / e_ms / 1e6 / HBM_PEAK_GBPS)
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--keeps", default="", help="comma-separated keep fractions instead of the workload's sweep "
                                                  "(profiling one point on its own)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replays of the per-point timings")
    ap.add_argument("--no-explicit-keys", action="store_true",
                    help="do not also time a dense gradient WITH its explicit key array (profiling runs: every "
                         "launch in the trace then belongs to the timed call)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the per-config records of the configurations that are not the timed workload")
    ap.add_argument("--widening", action="store_true",
                    help="also time decode-and-aggregate (8 streams into one dense vector) and decode-and-update (Adam); "
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

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()
    timer = Timer(torch, not args.no_graph)

    keeps = [float(x) for x in args.keeps.split(",") if x] or None
    case = make_case(args.workload, args.scale, keeps)
    n, points = case.n, case.points
    values = case.values[0]

    if args.calibrate:
        ref_copy = torch.empty_like(values)
        torch.neg(values, out=ref_copy)          # n*4 bytes read + n*4 bytes written
        torch.cuda.synchronize()
        del ref_copy

    case.count_fetch_units()

    # ---- the timed step: the whole hot path over the whole sweep
    def step(i):
        for pt in points:
            case.compress(pt, i)
            case.decompress(pt, i)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    case.check(points[-1])
    ms_per_step = 1e3 * elapsed / args.steps
    value = 8.0 * n * len(points) / (elapsed / args.steps) / 1e9

    # ---- what this GPU sustains on a plain streaming read and a plain copy of the value array
    sink = torch.zeros(2, dtype=torch.int64, device="cuda")
    probe_src = values if values.numel() >= (32 << 20) else torch.zeros(124_000_000, dtype=torch.float32, device="cuda")
    probe_bytes = probe_src.numel() * 4
    read_ms = timer.eager(lambda i: B.probe_read(probe_src, sink), args.steps)
    copy_dst = torch.empty_like(probe_src)
    copy_ms = timer.eager(lambda i: copy_dst.copy_(probe_src), args.steps)
    del copy_dst
    peak_measured = dict(read_GBps=probe_bytes / read_ms / 1e6, copy_GBps=2.0 * probe_bytes / copy_ms / 1e6,
                         bytes=probe_bytes, note="fastsgd_probe_read (plain streaming read) and a device-to-device copy "
                                                 "of the same array, timed in this run")

    # ---- per direction and per sweep point, event-timed on the launch stream; per kernel for one gradient
    detail = []
    kern_time, kern_bytes = {}, {}
    rows = (n + 255) // 256
    for pt in points:
        rec = point_record(case, pt, timer, args.steps, not args.no_explicit_keys)
        if isinstance(case, SingleCase):
            rc, kc = B.profile_compress(None if case.dense else case.keys[0], values, pt["p"], pt["out"], case.obytes,
                                        case.status, case.ws, args.steps, n=n, out_capacity=pt["cap"])
            assert rc == B.OK
            rc, kd = B.profile_decompress(pt["out"], pt["bytes"], pt["keys_out"], pt["vals_out"], case.count, case.status,
                                          case.dws, args.steps, capacity=pt["d"])
            assert rc == B.OK
            d, sb, qa = pt["d"], pt["bytes"], pt["granules_active"]
            # bytes each kernel is built to move, per launch: every value once and eight 16-bit bounds per row out;
            # bounds, granules that can hold a survivor, keys of survivors (where there is a key array), key + code
            # byte to scratch; surviving keys; surviving keys and code bytes in, stream out; stream in, pairs out
            alg = {
                "abs_sum": 4.0 * n + 16.0 * rows,
                "encode_values": 16.0 * rows + 128.0 * qa + (0.0 if case.dense else 4.0 * d) + 5.0 * d,
                "measure_keys": 4.0 * d,
                "pack_keys": 5.0 * d + (sb - 64),
                "decode": sb + 8.0 * d,
            }
            for k, v in {**kc, **{"decode": kd["decode"]}}.items():
                kern_time[k] = kern_time.get(k, 0.0) + v
            for k, v in alg.items():
                kern_bytes[k] = kern_bytes.get(k, 0.0) + v
            rec["kernels_ms"] = {**kc, **{"decode_" + k: v for k, v in kd.items()}}
            rec["kernels_moved_bytes"] = alg
        detail.append(rec)

    kernels = None
    big = max(detail, key=lambda r: r["d"])                          # the point with the most survivors
    calls = dict(point=dict(keep=big["keep"], d=big["d"], stream_bytes=big["stream_bytes"]),
                 compress=dict(key_array=big["key_array"], ms=big["compress_ms"],
                               algorithmic_bytes=big["compress_algorithmic_bytes"],
                               frac=big["compress_hbm_frac"], moved_bytes=big.get("compress_moved_bytes"),
                               moved_frac=big.get("compress_moved_frac"),
                               explicit_keys_ms=big.get("compress_explicit_keys_ms"),
                               explicit_keys_frac=big.get("compress_explicit_keys_hbm_frac"),
                               explicit_keys_moved_frac=big.get("compress_explicit_keys_moved_frac")),
                 decompress=dict(ms=big["decompress_ms"], algorithmic_bytes=big["decompress_algorithmic_bytes"],
                                 frac=big["decompress_hbm_frac"]),
                 note="whole calls at the sweep point with the most survivors; frac = algorithmic bytes / time / peak "
                      "(compress 8N+14d+sb without a key array, 8N+18d+sb with one; decompress sb+8d); moved_* counts the "
                      "granules actually read (and the 128-byte key lines actually fetched) instead; explicit_keys_*: "
                      "the same dense gradient passed WITH the key array 0..n-1")
    if kern_time:
        dominant = max(("abs_sum", "encode_values"), key=lambda k: kern_time[k])
        kernels = {k: dict(ms_total=kern_time[k], achieved_GBps=kern_bytes[k] / kern_time[k] / 1e6,
                           frac=kern_bytes[k] / kern_time[k] / 1e6 / HBM_PEAK_GBPS) for k in kern_bytes}
        launches = len(points)
        roofline = dict(bound="hbm", kernel="k_" + dominant,
                        achieved=kern_bytes[dominant] / kern_time[dominant] / 1e6, peak=HBM_PEAK_GBPS, unit="GB/s",
                        frac=kern_bytes[dominant] / kern_time[dominant] / 1e6 / HBM_PEAK_GBPS,
                        traffic=committed_traffic("k_" + dominant) if args.workload == "c4" and not keeps else None,
                        traffic_source="profiles/bench_c4_all_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, "
                                       "separate runs of this command, scaled by a plain elementwise kernel of known size; "
                                       "bytes per launch)",
                        avg_launch_ms=kern_time[dominant] / launches,
                        algorithmic_bytes_per_launch=kern_bytes[dominant] / launches,
                        peak_measured=peak_measured, calls=calls)
    else:
        comp = sum(r["compress_algorithmic_bytes"] for r in detail) / sum(r["compress_ms"] for r in detail) / 1e6
        roofline = dict(bound="hbm", kernel="fastsgd_compress_segmented (whole call)", achieved=comp, peak=HBM_PEAK_GBPS,
                        unit="GB/s", frac=comp / HBM_PEAK_GBPS, traffic=None, peak_measured=peak_measured, calls=calls)

    widening = None
    if args.widening and isinstance(case, SingleCase):
        widening = []
        n_streams = 8
        dense = torch.zeros(n, dtype=torch.float32, device="cuda")
        theta, m1, v1 = (torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(3))
        aws = B.decoder_workspace(n_streams)
        count, status, obytes, ws, dws = case.count, case.status, case.obytes, case.ws, case.dws
        keys = None if case.dense else case.keys[0]
        cap_w = max(B.compressed_size(n, pt["p"]) for pt in points)
        wout = torch.empty(cap_w // 8 + 8, dtype=torch.int64, device="cuda")
        for pt in points:
            sb = pt["bytes"]
            # the workers' gradients: the same values, rotated by a different amount for every worker, so that
            # the streams hold different keys (same keep fraction, same base)
            parts, sizes = [], []
            for wkr in range(n_streams):
                vals_w = torch.roll(case.values[0], wkr * 15485863) if wkr else case.values[0]
                rc = B.compress(keys, vals_w, pt["p"], wout, obytes, status, ws, n=n, out_capacity=cap_w)
                torch.cuda.synchronize()
                assert rc == B.OK and int(status[0]) == B.OK
                sizes.append(int(obytes[0]))
                parts.append(wout.view(torch.uint8)[:sizes[-1]].clone())
                del vals_w
            d_all = sum(int(x[40:48].cpu().numpy().view("<u8")[0]) for x in parts)
            many = torch.cat(parts + [torch.zeros(64, dtype=torch.uint8, device="cuda")])
            offs = torch.tensor([sum(sizes[:i]) for i in range(n_streams + 1)], dtype=torch.int64, device="cuda")
            total_w = sum(sizes)
            del parts

            def do_acc(_):
                assert B.decompress_accumulate(many, total_w, offs, n_streams, dense, count, status, aws) == B.OK

            def do_adam(_):
                assert B.decompress_adam(pt["out"], sb, theta, m1, v1, 1e-3, 0.9, 0.999, 1e-8, count, status, aws) == B.OK

            a_ms = timer.eager(do_acc, args.steps)
            assert int(status[0]) == B.OK and int(count[0]) == d_all
            u_ms = timer.eager(do_adam, args.steps)
            assert int(status[0]) == B.OK and int(count[0]) == pt["d"]
            widening.append(dict(keep=pt["keep"], d=pt["d"], accumulate_streams=n_streams, accumulate_ms=a_ms, adam_ms=u_ms,
                                 accumulate_pairs=d_all, accumulate_pairs_per_s=float(d_all) / a_ms * 1e3,
                                 adam_pairs_per_s=pt["d"] / u_ms * 1e3))
            del many
        del dense, theta, m1, v1, wout
        # the paper's base b = 1.1 with the threshold that keeps about the same fraction (b^tau = base^128;
        # above 128 a token is 9 bits)
        cap_all = max(B.compressed_size(n, B.params(1.1, 256)), B.compressed_size(n, points[0]["p"]))
        vout = torch.empty(cap_all // 8 + 8, dtype=torch.int64, device="cuda")
        for pt, wd in zip(points, widening):
            tau11 = min(256, max(1, int(math.ceil(128.0 * math.log(pt["p"].base) / math.log(1.1)))))
            p11 = B.params(1.1, tau11)

            def do_b11(_):
                assert B.compress(keys, values, p11, vout, obytes, status, ws, n=n, out_capacity=cap_all) == B.OK

            b_ms = timer.eager(do_b11, args.steps)
            assert int(status[0]) == B.OK
            sb11 = int(obytes[0])
            d11 = int(vout.view(torch.uint8)[40:48].cpu().numpy().view("<u8")[0])
            k11 = torch.empty(max(d11, 1), dtype=torch.int32, device="cuda")
            v11 = torch.empty(max(d11, 1), dtype=torch.float32, device="cuda")

            def do_b11_dec(_):
                assert B.decompress(vout, sb11, k11, v11, count, status, dws, capacity=d11) == B.OK

            bd_ms = timer.eager(do_b11_dec, args.steps)
            assert int(status[0]) == B.OK and int(count[0]) == d11
            wd.update(base_1p1=dict(tau=tau11, d=d11, stream_bytes=sb11, compress_ms=b_ms, decompress_ms=bd_ms))
            del k11, v11
        del vout

    # ---- the CPU oracle on the same workload: a baseline, and the check that the timed streams are the oracle's
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ref
        cpu_s, ref_streams = case.oracle_streams(ref)
        same = True
        for pt, st_ref in zip(points, ref_streams):
            case.compress(pt)
            torch.cuda.synchronize()
            got = case.stream_bytes_host(pt)
            same = same and got.size == st_ref.size and bool(np.array_equal(got, st_ref))
        model, nproc, usable = host_cpu()
        cpu = dict(value=8.0 * n * len(points) / cpu_s / 1e9, unit="GB/s", cores=1, kind="oracle",
                   cpu_model=model, nproc=nproc, usable_cores=usable, parity_checked=same,
                   sample=f"all {n} elements of {case.w.name}, all {len(points)} keep fraction(s), compress+decompress "
                          f"once, {cpu_s:.1f} s on one host core; every GPU stream of the timed step compared byte for "
                          f"byte with the oracle's")
        assert same, "a stream of the timed step differs from the oracle's"
        del ref_streams

    # ---- one record per other configuration (one call each, inputs used in turn where they are small)
    configs = None
    keep_fractions = [r["keep"] for r in detail]
    if args.workload == "c4" and not args.no_other_configs and not keeps and args.scale == 1.0:
        del case, values, points, probe_src
        torch.cuda.empty_cache()
        configs = []
        for name in ("c1", "c2", "c3", "c5"):
            c = make_case(name)
            for pt in c.points:
                rec = point_record(c, pt, timer, args.steps)
                in_bytes = 8 * c.n
                rec.update(workload=c.w.name, n=c.n, segments=getattr(c, "nseg", 1), input_copies=len(c.values),
                           residency="cache-resident (inputs under 512 MB in all: rates may exceed HBM peak)"
                           if in_bytes * len(c.values) < (512 << 20) else "HBM (the inputs used in turn exceed the caches)")
                configs.append(rec)
            del c
            torch.cuda.empty_cache()

    line = {
        "metric": "compress & decompress input GB/s (% of HBM peak) on 1 MI355X; compression ratio",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[args.workload], "n": n,
                   "keep_fractions": keep_fractions, "tau": 128, "flag_bits": 2,
                   "block_keys": 1024, "step": "compress+decompress at every keep fraction",
                   "key_array": detail[0]["key_array"],
                   "arithmetic": "f32 values and u32 keys compared as IEEE bit patterns; f64 boundary table"},
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "detail": detail,
    }
    if configs is not None:
        line["configs"] = configs
    if widening is not None:
        line["widening"] = widening
    print(json.dumps(line))


if __name__ == "__main__":
    main()
