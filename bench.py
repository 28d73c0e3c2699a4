#!/usr/bin/env python3
"""Bench of the C-Coll SZx hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic field already resident in HBM:
compress(x) -> decompress(stream) -> reduce_step(local, stream), all through the C ABI's enqueue-only
calls on one stream.  `value` is uncompressed float32 bytes handled per second by the step
(3 calls x 4n bytes / step time).  In the timed steps the library records HIP events around each coding / decoding
kernel itself (`kernel_ms`; the roofline of the slowest kernel comes from these).  The per-call rates come from
the same steps run once more with events recorded between the calls (a call = index scan + kernel + gaps + two
event markers), next to the durations of the same calls launched 20 times in a row and the compression ratio.
The CPU oracle is timed beside it on a bounded sample.

Besides the headline line (the 512^3 field at relative bound 1e-3) the same JSON object carries, unless
--no-extras is given, the other workloads of the benchmark spec: `ring8` (the per-rank compute of a compressed ring
reduce-scatter of 8 simulated ranges held in one GPU's memory: 8 x (1 compress + 7 reduce steps) on chunks of
17,958,405 values), `bcast64` (one 2^28-value field compressed once and decoded as 64 ranges), `sweep`
(20 points of noise fraction x bound) and `pipe` (the headline field written, forwarded and decoded piece by piece
on two HIP streams).

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload field512|vector|field256] [--rel-eb 1e-3]
                       [--no-extras | --extras pipe,ring8,bcast64,sweep] [--cpu-sample N]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, vendor figure


def make_workload(name: str):
    import workloads
    if name == "field512":
        return workloads.blob_field((512, 512, 512)), "3D float32 field 512x512x512, 32 Gaussian blobs + N(0,1e-4) noise"
    if name == "field256":
        return workloads.blob_field((256, 256, 256)), "3D float32 field 256x256x256 (reduced)"
    if name == "vector":
        return workloads.vector_1d(1 << 20), "1D float32 vector n=2^20"
    raise SystemExit(f"unknown workload {name}")


def time_kernel(torch, fn, reps: int) -> float:
    """Average duration in ms of `reps` back-to-back launches, by HIP events on the launch stream."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


class KernelTimer:
    """Pairs of HIP events that the library records around a kernel itself (ccoll_time_next_kernel): the
    dispatch's own start and end, without the marker packets of events recorded between calls."""

    def __init__(self):
        import ctypes
        self.ct = ctypes
        self.hip = ctypes.CDLL("libamdhip64.so.7")     # the runtime the library is linked against (already loaded)
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.all = []

    def pair(self):
        evs = []
        for _ in range(2):
            e = self.ct.c_void_p()
            rc = self.hip.hipEventCreate(self.ct.byref(e)); assert rc == 0, rc
            evs.append(e.value); self.all.append(e.value)
        return tuple(evs)

    def ms(self, pair) -> float:
        out = self.ct.c_float()
        rc = self.hip.hipEventElapsedTime(self.ct.byref(out), pair[0], pair[1]); assert rc == 0, rc
        return out.value

    def close(self):
        for e in self.all:
            self.hip.hipEventDestroy(e)
        self.all = []


def _cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(x, eb, sample_elems: int):
    """The oracle as it stands on the first `sample_elems` values of the same input.  Primary figure: one thread
    pinned to one core, median of three runs per call (the protocol of the paper's single-thread Table I).
    Secondary, labelled: the same unchanged oracle functions called from a thread pool on independent ranges of
    chunks, one per host core this process may use."""
    import statistics
    from concurrent.futures import ThreadPoolExecutor
    import numpy as np
    from oracle import ref
    xs = np.ascontiguousarray(x[:sample_elems])
    loc = np.roll(xs, 1)
    allowed = sorted(os.sched_getaffinity(0))
    core = allowed[len(allowed) // 2]
    os.sched_setaffinity(0, {core})
    try:
        s = ref.compress(xs, eb)
        tc, td, tr = [], [], []
        for _ in range(3):
            t0 = time.perf_counter(); s = ref.compress(xs, eb); t1 = time.perf_counter()
            y = ref.decompress(s, xs.size); t2 = time.perf_counter()
            r = ref.reduce_step(loc, s, eb); t3 = time.perf_counter()
            tc.append(t1 - t0); td.append(t2 - t1); tr.append(t3 - t2)
            del y, r
    finally:
        os.sched_setaffinity(0, set(allowed))
    mc, md, mr = statistics.median(tc), statistics.median(td), statistics.median(tr)
    gb = 4.0 * xs.size / 1e9
    # all host cores: the input cut into ranges of whole chunks, one oracle call per range and thread
    nthreads = max(1, min(len(allowed), 16))
    per = -(-(xs.size // 5120 + 1) // nthreads) * 5120
    pieces = [(i, min(xs.size, i + per)) for i in range(0, xs.size, per)]

    def one(rng):
        a, b = rng
        st = ref.compress(xs[a:b], eb)
        yy = ref.decompress(st, b - a)
        rr = ref.reduce_step(loc[a:b], st, eb)
        return yy.size + rr.size

    with ThreadPoolExecutor(nthreads) as ex:
        list(ex.map(one, pieces[:nthreads]))           # warm
        t0 = time.perf_counter(); list(ex.map(one, pieces)); t1 = time.perf_counter()
    return {
        "value": round(3 * gb / (mc + md + mr), 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"first {xs.size} values of the same field: compress + decompress + reduce_step, one thread pinned to "
                  f"core {core}, median of 3 runs per call",
        "compress_GBps": round(gb / mc, 4), "decompress_GBps": round(gb / md, 4), "reduce_step_GBps": round(gb / mr, 4),
        "cpu_model": _cpu_model(), "host_cores_total": os.cpu_count(), "host_cores_usable": len(allowed),
        "all_cores": {"value": round(3 * gb / (t1 - t0), 4), "unit": "GB/s", "threads": nthreads,
                      "note": "secondary: the unchanged oracle called on independent ranges of chunks from a thread pool"},
    }


def stream_stats(stream_u8, n):
    """Constant / raw block fractions of a CSX1 stream (host side, from the bitmaps and reqlen bytes)."""
    import numpy as np
    b = stream_u8
    nch = int(b[20:24].view(np.uint32)[0])
    idx = b[32:32 + 4 * nch].view(np.uint32).astype(np.int64)
    start = 32 + 4 * nch + np.concatenate(([0], np.cumsum(idx)[:-1]))
    nblocks = (n + 127) // 128
    nonconst = raw = 0
    lo = b[start[:, None] + np.arange(8)[None, :]].astype(np.uint64)
    bitmaps = (lo << (8 * np.arange(8, dtype=np.uint64))[None, :]).sum(axis=1).astype(np.uint64)
    k = np.array([bin(int(v)).count("1") for v in bitmaps], dtype=np.int64)
    nonconst = int(k.sum())
    nbc = np.full(nch, 40, dtype=np.int64)
    if nch:
        nbc[-1] = (n - (nch - 1) * 5120 + 127) // 128
    for c in np.nonzero(k)[0]:
        r0 = int(start[c]) + 8 + 4 * int(nbc[c]) + 2 * int(k[c])
        raw += int((b[r0:r0 + int(k[c])] == 32).sum())
    return 1.0 - nonconst / max(nblocks, 1), raw / max(nblocks, 1)


def run_table(path, pkg, torch, workloads):
    """Throughput, CR and block statistics over the workloads of the paper's tables: written as markdown."""
    import numpy as np
    rows = []
    ctx = pkg.Context(0, reserve_n=1 << 28)

    def point(tag, x, rel):
        n = x.size
        eb = float(workloads.abs_bound(x, rel))
        dx = torch.from_numpy(x).cuda(); dl = torch.roll(dx, 1)
        cap = pkg.max_compressed_bytes(n)
        s1 = torch.empty(cap, dtype=torch.uint8, device="cuda"); s2 = torch.empty(cap, dtype=torch.uint8, device="cuda")
        y = torch.empty(n, dtype=torch.float32, device="cuda")
        fc = lambda: ctx.compress_async(dx, eb, s1)
        fd = lambda: ctx.decompress_async(s1, n, y, in_bytes=cap)
        fr = lambda: ctx.reduce_step_async(dl, s1, eb, s2, cin_bytes=cap)
        fc(); st, cb = ctx.wait(); assert st == 0, st
        tc = time_kernel(torch, fc, 10); td = time_kernel(torch, fd, 10); tr = time_kernel(torch, fr, 10)
        st, rb = ctx.wait(); assert st == 0, st
        err = (y.double() - dx.double()).abs().max().item() / eb
        const, raw = stream_stats(s1[:cb].cpu().numpy(), n)
        gb = 4.0 * n / 1e9
        rows.append((tag, rel, 4.0 * n / cb, const, raw, gb / tc * 1e3, gb / td * 1e3, gb / tr * 1e3, err))
        del dx, dl, s1, s2, y
        torch.cuda.empty_cache()

    point("vector 2^20", workloads.vector_1d(1 << 20), 1e-3)
    f = workloads.blob_field((512, 512, 512))
    for rel in (1e-2, 1e-3, 1e-4):
        point("field 512^3", f, rel)
    del f
    g = workloads.gradient_like(143_667_240 // 8)
    point("gradient chunk 17,958,405", g, 1e-5 / float(np.float64(g.max()) - np.float64(g.min())))
    del g
    for frac in (0.0, 0.25, 0.5, 1.0):
        x = workloads.sweep_mix(frac)
        for rel in (1e-2, 1e-3, 1e-4, 1e-5, 1e-6):
            point("sweep noise %.2f" % frac, x, rel)
        del x
    ctx.close()
    with open(path, "w") as fh:
        fh.write("| workload | rel eb | CR | constant blocks | raw blocks | compress GB/s | decompress GB/s | reduce step GB/s | max err / eb |\n")
        fh.write("|---|---|---|---|---|---|---|---|---|\n")
        for r in rows:
            fh.write("| %s | %.0e | %.2f | %.1f %% | %.1f %% | %.0f | %.0f | %.0f | %.3f |\n" % (r[0], r[1], r[2], 100 * r[3], 100 * r[4], r[5], r[6], r[7], r[8]))
    return rows


def _events(torch, k):
    return [torch.cuda.Event(enable_timing=True) for _ in range(k)]


def bench_ring8(pkg, torch, workloads):
    """Workload 2: ring reduce-scatter of P = 8 simulated ranks (Sec. III-A.2, Fig. 4, Eq. 2) in one GPU's memory.
    The chunk that rank k starts with travels the ring: compressed once, then reduced (decompress + add the local
    chunk + recompress) by the seven other ranks; a "send" is a pointer hand-off.  All eight chains run round by
    round as in the collective: 8 compress calls, then 7 rounds of 8 reduce steps."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    P, n, eb = 8, 143_667_240 // 8, float(np.float32(1e-5))
    t0 = time.perf_counter()
    with ThreadPoolExecutor(8) as ex:          # data[r][k]: chunk k of rank r's gradient-like vector
        host = list(ex.map(lambda i: workloads.gradient_like(n, seed=workloads.SEED_GRAD + 97 * (i // P) + (i % P)), range(P * P)))
    data = [[torch.from_numpy(host[r * P + k]).cuda() for k in range(P)] for r in range(P)]
    del host
    gen_s = time.perf_counter() - t0
    ctx = pkg.Context(0, reserve_n=n)
    cap = pkg.max_compressed_bytes(n)
    S = [[torch.empty(cap, dtype=torch.uint8, device="cuda") for _ in range(2)] for _ in range(P)]

    def run(ev=None):
        i = 0
        for k in range(P):
            if ev: ev[i].record()
            assert ctx.compress_async(data[k][k], eb, S[k][0]) == 0
            i += 1
        for j in range(1, P):
            for k in range(P):
                if ev: ev[i].record()
                assert ctx.reduce_step_async(data[(k + j) % P][k], S[k][(j - 1) & 1], eb, S[k][j & 1], cin_bytes=cap) == 0
                i += 1
        if ev: ev[i].record()

    run(); st, _ = ctx.wait(); assert st == 0, st
    run(); torch.cuda.synchronize()
    reps = 3
    tot, tcomp, tred = [], [], []
    for _ in range(reps):
        ev = _events(torch, P * P + 1)
        run(ev); torch.cuda.synchronize()
        d = [ev[i].elapsed_time(ev[i + 1]) for i in range(P * P)]
        tot.append(ev[0].elapsed_time(ev[-1])); tcomp.append(sum(d[:P]) / P); tred.append(sum(d[P:]) / (P * (P - 1)))
    ms_tot, ms_c, ms_r = min(tot), min(tcomp), min(tred)
    # accuracy of the reduced chunks against the float64 sum, and sizes
    fin = (P - 1) & 1
    worst, inside, count, out_bytes = 0.0, 0, 0, 0
    bound = (2.0 / 3.0) * (P ** 0.5) * eb
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    for k in range(P):
        assert ctx.decompress_async(S[k][fin], n, y, in_bytes=cap) == 0
        st, _ = ctx.wait(); assert st == 0, st
        exact = torch.zeros(n, dtype=torch.float64, device="cuda")
        for r in range(P):
            exact += data[r][k].double()
        err = (y.double() - exact).abs()
        worst = max(worst, err.max().item()); inside += int((err <= bound).sum().item()); count += n
        out_bytes += int(S[k][fin][24:32].view(torch.int64).item())
        del exact, err
    first_bytes = int(S[0][0][24:32].view(torch.int64).item())
    ctx.close()
    gb = 4.0 * n / 1e9
    return {
        "workload": "P=8 simulated ranks x 143,667,240 gradient-like values (Laplace(0,1e-3), 20% zeros), abs eb 1e-5; "
                    "8 chains of 1 compress + 7 reduce steps on chunks of 17,958,405 values",
        "n_per_call": n, "calls": P * P, "ms_total": round(ms_tot, 3),
        "aggregate_GBps": round(P * P * gb / (ms_tot * 1e-3), 1),
        "compress_ms": round(ms_c, 4), "compress_GBps": round(gb / (ms_c * 1e-3), 1),
        "reduce_step_ms": round(ms_r, 4), "reduce_step_GBps": round(gb / (ms_r * 1e-3), 1),
        "CR_first_round": round(4.0 * n / first_bytes, 3), "CR_reduced": round(4.0 * n * P / out_bytes, 3),
        "max_abs_err_over_P_eb": round(worst / (P * eb), 4), "max_abs_err_over_eb": round(worst / eb, 3),
        "frac_within_two_thirds_sqrtP_eb": round(inside / count, 5), "input_generation_s": round(gen_s, 1),
    }


def bench_bcast64(pkg, torch, workloads):
    """Workload 3: one 2^28-value field compressed once (the root of a C-Bcast / C-Scatter), decoded as 64 ranges
    of 2^22 values that start in the middle of chunks: 64 plain range calls, 64 calls over a kept index, and one
    call for all 64 ranges."""
    x = workloads.bcast_field()
    n = x.size
    eb = float(workloads.abs_bound(x, 1e-3))
    dx = torch.from_numpy(x).cuda()
    del x
    ctx = pkg.Context(0, reserve_n=n)
    cap = pkg.max_compressed_bytes(n)
    s = torch.empty(cap, dtype=torch.uint8, device="cuda")
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    assert ctx.compress_async(dx, eb, s) == 0
    st, nb = ctx.wait(); assert st == 0, st
    cnt = n // 64
    firsts, counts = [j * cnt for j in range(64)], [cnt] * 64
    outs = [y[j * cnt:(j + 1) * cnt] for j in range(64)]
    ms_c = time_kernel(torch, lambda: ctx.compress_async(dx, eb, s), 10)
    ms_full = time_kernel(torch, lambda: ctx.decompress_async(s, n, y, in_bytes=nb), 10)

    def plain():
        for j in range(64):
            ctx.decompress_range_async(s[:nb], n, firsts[j], cnt, outs[j])

    def indexed():
        for j in range(64):
            ctx.decompress_range_indexed_async(s[:nb], n, firsts[j], cnt, outs[j])

    ms_plain = time_kernel(torch, plain, 5)
    ctx.index(s[:nb], n)
    ms_idx = time_kernel(torch, indexed, 5)
    ms_batch = time_kernel(torch, lambda: ctx.decompress_ranges_async(s[:nb], n, firsts, counts, outs), 10)
    st, _ = ctx.wait(); assert st == 0, st
    err = (y.double() - dx.double()).abs().max().item()
    ctx.close()
    gb = 4.0 * n / 1e9
    return {
        "workload": "3D float32 field 1024x512x512 (blobs + 8 sinusoidal modes), rel eb 1e-3, 64 ranges of 2^22 values",
        "n": n, "CR": round(4.0 * n / nb, 3), "max_abs_err_over_eb": round(err / eb, 4),
        "compress_ms": round(ms_c, 4), "compress_GBps": round(gb / (ms_c * 1e-3), 1),
        "decompress_full_ms": round(ms_full, 4), "decompress_full_GBps": round(gb / (ms_full * 1e-3), 1),
        "ranges64_plain_calls_ms": round(ms_plain, 4), "ranges64_indexed_calls_ms": round(ms_idx, 4),
        "ranges64_one_call_ms": round(ms_batch, 4), "ranges64_one_call_GBps": round(gb / (ms_batch * 1e-3), 1),
    }


def bench_pipe(pkg, torch, workloads, x, eb, pieces: int = 8):
    """PIPE-SZx on one GPU (Sec. III-E.2): the headline field written as one stream in `pieces` launches on one
    HIP stream while a second HIP stream forwards (device copy: the transport's stand-in) and decodes every piece
    that is final.  Compared with the same three stages one after the other on one stream."""
    n = x.size
    nchunks = -(-n // 5120)
    per = -(-nchunks // pieces // 12) * 12
    bounds = list(range(0, nchunks, per)) + [nchunks]
    k = len(bounds) - 1
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    ca, cb = pkg.Context(0, stream=sa, reserve_n=n), pkg.Context(0, stream=sb, reserve_n=n)
    dx = torch.from_numpy(x).cuda()
    cap = pkg.max_compressed_bytes(n)
    sent = torch.empty(cap, dtype=torch.uint8, device="cuda"); recv = torch.empty(cap, dtype=torch.uint8, device="cuda")
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    prog = torch.zeros(k, 2, dtype=torch.int64, device="cuda")
    res = torch.zeros(2 * k, 2, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()

    def piped():
        # producer first, then consumer: each side's work sits in its HIP stream before the device gets to it, as
        # with a transport thread of its own (launching piece by piece from one host thread starves the device)
        evs = []
        with torch.cuda.stream(sa):
            ca.compress_begin(n, eb, sent)
            for i in range(k):
                ca.compress_chunks_async(dx, bounds[i], bounds[i + 1], prog[i], res[i])
                ev = torch.cuda.Event(); ev.record(sa); evs.append(ev)
        with torch.cuda.stream(sb):
            for i in range(k):
                sb.wait_event(evs[i])
                pkg.forward_async(recv, sent, n, prog[i - 1] if i else None, prog[i], hip_stream=sb.cuda_stream)
                cb.decompress_chunks_async(recv, cap, n, bounds[i], bounds[i + 1], y[bounds[i] * 5120:], res[k + i])

    def serial():
        with torch.cuda.stream(sa):
            ca.compress_async(dx, eb, sent, res[0])
            pkg.forward_async(recv, sent, n, None, prog[k - 1], hip_stream=sa.cuda_stream)
            ca.decompress_async(recv, n, y, res[1], in_bytes=cap)

    def wall(fn, reps):
        fn(); torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps

    ms_p = wall(piped, 10)
    assert (res.cpu().numpy()[:, 1] == 0).all()
    err = (y.double() - dx.double()).abs().max().item()
    assert err <= eb * (1 + 1e-9), (err, eb)
    ms_s = wall(serial, 10)
    ca.close(); cb.close()
    return {"pieces": k, "chunks_per_piece": per, "ms_pipelined_two_streams": round(ms_p, 4), "ms_serial_one_stream": round(ms_s, 4),
            "note": "compress -> forward (device copy) -> decompress of the headline field; wall clock per pass"}


def bench_sweep(pkg, torch, workloads):
    """Workload 4: noise fraction {0, .25, .5, 1} x relative bound {1e-2 .. 1e-6} on 2^27 values."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    fracs = (0.0, 0.25, 0.5, 1.0)
    with ThreadPoolExecutor(4) as ex:
        fields = list(ex.map(workloads.sweep_mix, fracs))
    n = fields[0].size
    ctx = pkg.Context(0, reserve_n=n)
    cap = pkg.max_compressed_bytes(n)
    s1 = torch.empty(cap, dtype=torch.uint8, device="cuda"); s2 = torch.empty(cap, dtype=torch.uint8, device="cuda")
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    rows = []
    gb = 4.0 * n / 1e9
    for frac, x in zip(fracs, fields):
        dx = torch.from_numpy(x).cuda(); dl = torch.roll(dx, 1)
        for rel in (1e-2, 1e-3, 1e-4, 1e-5, 1e-6):
            eb = float(workloads.abs_bound(x, rel))
            assert ctx.compress_async(dx, eb, s1) == 0
            st, cb = ctx.wait(); assert st == 0, st
            tc = time_kernel(torch, lambda: ctx.compress_async(dx, eb, s1), 8)
            td = time_kernel(torch, lambda: ctx.decompress_async(s1, n, y, in_bytes=cb), 8)
            tr = time_kernel(torch, lambda: ctx.reduce_step_async(dl, s1, eb, s2, cin_bytes=cb), 8)
            st, rb = ctx.wait(); assert st == 0, st
            ctx.decompress_async(s1, n, y, in_bytes=cb); st, _ = ctx.wait(); assert st == 0, st
            err = (y.double() - dx.double()).abs().max().item() / eb
            const, raw = stream_stats(s1[:cb].cpu().numpy(), n)
            rows.append({"noise": frac, "rel_eb": rel, "CR": round(4.0 * n / cb, 3), "const_blocks": round(const, 4),
                         "raw_blocks": round(raw, 4), "compress_GBps": round(gb / tc * 1e3, 1),
                         "decompress_GBps": round(gb / td * 1e3, 1), "reduce_step_GBps": round(gb / tr * 1e3, 1),
                         "max_abs_err_over_eb": round(err, 4)})
        del dx, dl
    ctx.close()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=100, help="untimed steps first (the device needs some tens of ms of work to reach its running clocks)")
    ap.add_argument("--workload", default="field512")
    ap.add_argument("--rel-eb", type=float, default=1e-3)
    ap.add_argument("--cpu-sample", type=int, default=1 << 27, help="elements the oracle is timed on (0 = skip)")
    ap.add_argument("--table", default=None, help="also run all workloads and bounds and write a markdown table to this path")
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload (no pipe / ring8 / bcast64 / sweep keys)")
    ap.add_argument("--extras", default="pipe,ring8,bcast64,sweep", help="which of the other workloads to run (comma separated)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    import paper_2304_03890_amd as pkg
    import workloads

    x, desc = make_workload(args.workload)
    n = x.size
    eb = float(workloads.abs_bound(x, args.rel_eb))
    dx = torch.from_numpy(x).cuda()
    dlocal = torch.roll(dx, 1)                       # a second resident field for the reduce step
    ctx = pkg.Context(0, reserve_n=n)
    cap = pkg.max_compressed_bytes(n)
    stream = torch.empty(cap, dtype=torch.uint8, device="cuda")
    stream2 = torch.empty(cap, dtype=torch.uint8, device="cuda")
    y = torch.empty(n, dtype=torch.float32, device="cuda")

    # The timed calls keep {bytes, status} inside the context (no extra launch); they are checked here once.
    def k_compress():
        rc = ctx.compress_async(dx, eb, stream); assert rc == 0, rc

    def k_decompress():
        rc = ctx.decompress_async(stream, n, y, in_bytes=cap); assert rc == 0, rc

    def k_reduce():
        rc = ctx.reduce_step_async(dlocal, stream, eb, stream2, cin_bytes=cap); assert rc == 0, rc

    def step():
        k_compress(); k_decompress(); k_reduce()

    # correctness of what is timed: statuses, bound, and sizes
    k_compress(); st, cbytes = ctx.wait(); assert st == 0, st
    k_decompress(); st, _ = ctx.wait(); assert st == 0, st
    k_reduce(); st, rbytes = ctx.wait(); assert st == 0, st
    err = (y.double() - dx.double()).abs().max().item()
    assert err <= float(np.float64(np.float32(eb))), (err, eb)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The timed region: K steps.  The library records a pair of HIP events around each coding / decoding kernel
    # itself, on the stream it launches on: the kernels' own durations inside the timed region.
    kt = KernelTimer()
    kev = [[kt.pair() for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        ctx.time_next_kernel(*kev[k][0]); k_compress()
        ctx.time_next_kernel(*kev[k][1]); k_decompress()
        ctx.time_next_kernel(*kev[k][2]); k_reduce()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / args.steps
    kms = [sum(kt.ms(kev[k][i]) for k in range(args.steps)) / args.steps for i in range(3)]
    kt.close()

    # The same K steps once more with events recorded between the calls: each call's duration as its caller sees
    # it (index scan + kernel + the gaps around them, and the two event markers).
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for k in range(args.steps):
        ev[k][0].record(); k_compress(); ev[k][1].record(); k_decompress(); ev[k][2].record(); k_reduce(); ev[k][3].record()
    torch.cuda.synchronize()
    ms_c = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    ms_d = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    ms_r = sum(e[2].elapsed_time(e[3]) for e in ev) / args.steps
    # and once more with no events at all
    t0 = time.perf_counter()
    for k in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step_plain = (time.perf_counter() - t0) * 1e3 / args.steps

    # the same calls back to back (20 launches of one kind in a row), for comparison
    reps = max(5, args.steps)
    b2b = {"compress": time_kernel(torch, k_compress, reps), "decompress": time_kernel(torch, k_decompress, reps),
           "reduce_step": time_kernel(torch, k_reduce, reps)}

    # a plain device copy of the same field on the same box, for scale (read + written bytes per second)
    ms_copy = time_kernel(torch, lambda: y.copy_(dx), reps)
    copy_rw = 2 * 4.0 * n / (ms_copy * 1e-3) / 1e9

    gb = 4.0 * n / 1e9
    cr, cr2 = 4.0 * n / cbytes, 4.0 * n / rbytes
    alg = {  # algorithmic HBM bytes per launch: read + write, nothing re-read
        "k_compress": 4.0 * n + cbytes,
        "k_decompress": cbytes + 4.0 * n,
        "k_reduce_step": 4.0 * n + cbytes + rbytes,
    }
    dur = {"k_compress": kms[0], "k_decompress": kms[1], "k_reduce_step": kms[2]}       # the kernels themselves
    call = {"compress": ms_c, "decompress": ms_d, "reduce_step": ms_r}                    # the calls, with event markers
    dom = max(dur, key=dur.get)
    achieved = alg[dom] / (dur[dom] * 1e-3) / 1e9

    line = {
        "metric": "SZx compress / decompress / reduce-step GB/s (uncompressed) at 1 GPU; CR",
        "value": round(3 * gb / (ms_step * 1e-3), 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": desc, "n": n, "rel_eb": args.rel_eb, "abs_eb": eb, "block": 128, "chunk": 5120},
        "compress_GBps": round(gb / (ms_c * 1e-3), 2), "decompress_GBps": round(gb / (ms_d * 1e-3), 2),
        "reduce_step_GBps": round(gb / (ms_r * 1e-3), 2),
        "compress_frac_hbm_peak": round(gb / (ms_c * 1e-3) / HBM_PEAK_GBPS, 4),
        "decompress_frac_hbm_peak": round(gb / (ms_d * 1e-3) / HBM_PEAK_GBPS, 4),
        "reduce_step_frac_hbm_peak": round(gb / (ms_r * 1e-3) / HBM_PEAK_GBPS, 4),
        "CR": round(cr, 3), "CR_reduce_out": round(cr2, 3), "max_abs_err_over_eb": round(err / eb, 4),
        "ms_per_step_without_events": round(ms_step_plain, 4),
        "kernel_ms": {k: round(v, 4) for k, v in dur.items()},
        "kernel_frac_hbm_peak_uncompressed": {k: round(gb / (v * 1e-3) / HBM_PEAK_GBPS, 4) for k, v in dur.items()},
        "call_ms_between_events": {k: round(v, 4) for k, v in call.items()},
        "call_ms_back_to_back": {k: round(v, 4) for k, v in b2b.items()},
        "device_copy_rw_GBps": round(copy_rw, 1),
        "rw_frac_of_device_copy": {k: round(alg[k] / (dur[k] * 1e-3) / 1e9 / copy_rw, 4) for k in dur},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                     "algorithmic_bytes": alg[dom]},
    }
    # HBM bytes per launch measured with rocprofv3 --pmc on this workload, if a summary has been committed
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            tr = json.load(f)
        if tr.get("workload") == args.workload and abs(tr.get("rel_eb", 0) - args.rel_eb) < 1e-12:
            line["roofline"]["traffic"] = tr["kernels"].get(dom)
            line["roofline"]["traffic_measured_at_commit"] = tr.get("commit")
    except (OSError, ValueError):
        pass
    if args.cpu_sample > 0:
        line["cpu_baseline"] = cpu_baseline(x, eb, min(n, args.cpu_sample))
    ctx.close()
    del dx, dlocal, stream, stream2, y
    torch.cuda.empty_cache()
    extras = [] if args.no_extras else [e for e in args.extras.split(",") if e]
    if "pipe" in extras:
        line["pipe"] = bench_pipe(pkg, torch, workloads, x, eb)
        torch.cuda.empty_cache()
    for key, fn in (("ring8", bench_ring8), ("bcast64", bench_bcast64), ("sweep", bench_sweep)):
        if key in extras:
            line[key] = fn(pkg, torch, workloads)
            torch.cuda.empty_cache()
    if args.table:
        run_table(args.table, pkg, torch, workloads)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
