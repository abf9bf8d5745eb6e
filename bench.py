#!/usr/bin/env python3
"""Benchmark of the compression hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic ResNet-50-shaped
gradients for 8 simulated workers (8 sets of buffers in one GPU's HBM), bucket by bucket
("one communication per bucket"):

  flatten            8 workers x B buckets   layer tensors -> contiguous 25 MiB buckets
  compress_minmax    8 workers x B buckets   MinMax-u8 with worker error state (delta)
  drr_minmax         B buckets               decompress, average 8 workers, server error state (epsilon),
                                             recompress, decode to fp32
  ring_fp            B buckets               ring averaging of 8 replicas, full precision
  ring_lp            B buckets               ring averaging with u8-compressed differences
  sign_compress      8 workers x B buckets   1-bit sign + per-chunk scale with error state
  drr_sign           B buckets               the server step with the sign codec

Inputs are generated on the GPU before the timed region and stay resident in HBM.  Prints ONE JSON
line (see README for the fields).  `--gpus N` with N > 1 is refused: this build is the
single-GPU share of the path.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
K_WORKERS = 8
CHUNK = 4096
SIGN_CHUNK = 2048
GRAD_SETS = 3      # the three iterations of the configuration use fresh gradients; the sets are rotated

# algorithmic HBM bytes per element (per worker / per peer where applicable)
BYTES = {
    "flatten": 8.0,
    "compress_minmax": 13.0 + 8.0 / CHUNK,
    "drr_minmax": K_WORKERS + 13.0 + 8.0 * (K_WORKERS + 1) / CHUNK,
    "ring_fp": 8.0,
    "ring_lp": 17.0 + 8.0 / CHUNK,
    "sign_compress": 12.125 + 4.0 / SIGN_CHUNK,
    "drr_sign": K_WORKERS / 8.0 + 12.125 + 4.0 * (K_WORKERS + 1) / SIGN_CHUNK,
}
PRIMS = list(BYTES)
KERNEL_OF = {
    "flatten": "k_flatten", "compress_minmax": "k_compress_minmax<2,true>", "drr_minmax": "k_drr_minmax<2,true,true>",
    "ring_fp": "k_ring_avg_fp<8>", "ring_lp": "k_ring_avg_lp<8,2>", "sign_compress": "k_sign_compress<2,true>",
    "drr_sign": "k_drr_sign<4,true,true>",
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--only", default="", help="comma list of primitives to run in the step (profiling aid)")
    ap.add_argument("--per-bucket-launch", action="store_true",
                    help="one launch per 25 MiB bucket instead of one per worker covering all its buckets")
    return ap.parse_args()


class Workload:
    """ResNet-50-shaped gradients for K workers, greedy 25 MiB buckets, all state resident on the GPU.

    Each worker's buckets sit back to back in one flat allocation (every bucket is padded to a multiple of
    k*chunk, so chunk and ScatterReduce-partition boundaries coincide with bucket boundaries).  A launch covers
    either all buckets of one worker (`per_bucket=False`, the default: one launch per worker and primitive) or a
    single bucket; the results are bit-identical because chunks are independent.
    """

    def __init__(self, torch, bg, per_bucket=False):
        from bagua_workloads import resnet50_shapes, pack_buckets, draw, seed_for, layer_sigmas
        from bagua_workloads.shapes import numel
        from bagua_workloads.generators import SHARED
        self.torch, self.bg = torch, bg
        dev = torch.device("cuda:0")
        k = K_WORKERS
        shapes = resnet50_shapes()
        self.sizes = [numel(s) for _, s in shapes]
        self.total = sum(self.sizes)
        self.buckets = pack_buckets(shapes, k, CHUNK)
        self.bases = [0]
        for bk in self.buckets:
            self.bases.append(self.bases[-1] + bk.n_pad)
        n = self.n_elems = self.bases[-1]
        sig = layer_sigmas(len(shapes), seed_for(1, 0, SHARED))
        starts = [0]
        for sz in self.sizes:
            starts.append(starts[-1] + sz)
        # layer tensors: one arena per (gradient set, worker); views per layer (all layer sizes are multiples of 4)
        self.layers = []
        for it in range(GRAD_SETS):
            per_worker = []
            for j in range(k):
                arena = draw("normal", self.total, seed_for(1, it, j), dev, 1.0)
                views = []
                for t, sz in enumerate(self.sizes):
                    v = arena[starts[t]:starts[t + 1]]
                    v.mul_(sig[t])
                    views.append(v)
                per_worker.append(views)
            self.layers.append(per_worker)
        # launch units: (first element, length, tensor ids, destination offsets relative to the unit)
        if per_bucket:
            self.units = [(self.bases[b], bk.n_pad, list(bk.tensors), list(bk.offsets)) for b, bk in enumerate(self.buckets)]
        else:
            ids, offs = [], []
            for b, bk in enumerate(self.buckets):
                ids += list(bk.tensors)
                offs += [self.bases[b] + o for o in bk.offsets]
            self.units = [(0, n, ids, offs)]
        U = len(self.units)
        f32 = dict(dtype=torch.float32, device=dev)
        u8 = dict(dtype=torch.uint8, device=dev)
        i32 = dict(dtype=torch.int32, device=dev)

        def views(t, div=1, mul=1):
            """Per-unit views of a flat tensor whose index is element_index * mul / div."""
            return [t[lo * mul // div:(lo + ln) * mul // div] for lo, ln, _, _ in self.units]

        self.plans = [[[None] * U for _ in range(k)] for _ in range(GRAD_SETS)]
        for it in range(GRAD_SETS):
            for j in range(k):
                for u, (lo, ln, ids, offs) in enumerate(self.units):
                    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(ids), ln), **u8)
                    bg.bagua_flatten_plan([self.layers[it][j][t] for t in ids], offs, ln, ws)
                    self.plans[it][j][u] = ws
        nc, ncs = n // CHUNK, n // SIGN_CHUNK
        z = lambda m, **kw: torch.zeros(m, **kw)
        self.bucket = [views(z(n, **f32)) for _ in range(k)]
        self.delta = [views(z(n, **f32)) for _ in range(k)]
        self.codes = [views(z(n, **u8)) for _ in range(k)]
        self.minmax = [views(z(2 * nc, **f32), CHUNK, 2) for _ in range(k)]
        self.eps = views(z(n, **f32))
        self.codes_out = views(z(n, **u8))
        self.minmax_out = views(z(2 * nc, **f32), CHUNK, 2)
        self.out = views(z(n, **f32))
        # sign codec state
        self.sdelta = [views(z(n, **f32)) for _ in range(k)]
        self.bits = [views(z(n // 32, **i32), 32) for _ in range(k)]
        self.scale = [views(z(ncs, **f32), SIGN_CHUNK) for _ in range(k)]
        self.seps = views(z(n, **f32))
        self.bits_out = views(z(n // 32, **i32), 32)
        self.scale_out = views(z(ncs, **f32), SIGN_CHUNK)
        self.sout = views(z(n, **f32))
        # decentralised replicas: shared base + per-peer drift; two ping-pong sets per mode
        base = draw("normal", n, seed_for(3, 0, SHARED), dev, 0.02)
        self.rep_fp = [[None] * k for _ in range(2)]
        self.rep_lp = [[None] * k for _ in range(2)]
        self.xhat = [None] * k
        for i in range(k):
            x = base + draw("normal", n, seed_for(3, 0, i), dev, 1e-3)
            self.rep_fp[0][i] = views(x)
            self.rep_fp[1][i] = views(torch.empty_like(x))
            self.rep_lp[0][i] = views(x.clone())
            self.rep_lp[1][i] = views(torch.empty_like(x))
            self.xhat[i] = views(base.clone())
        self.lp_codes = [views(z(n, **u8)) for _ in range(k)]
        self.lp_minmax = [views(z(2 * nc, **f32), CHUNK, 2) for _ in range(k)]
        self.step_no = 0
        torch.cuda.synchronize()

    # gradient bytes one step consumes, per primitive (4 B x fp32 elements the primitive consumes or represents)
    def grad_bytes(self):
        n, k = self.n_elems, K_WORKERS
        return {p: 4.0 * n * k for p in PRIMS}

    def algo_bytes(self):
        n, k = self.n_elems, K_WORKERS
        per_unit = {"flatten": n * k, "compress_minmax": n * k, "drr_minmax": n, "ring_fp": n * k, "ring_lp": n * k,
                    "sign_compress": n * k, "drr_sign": n}
        return {p: BYTES[p] * per_unit[p] for p in PRIMS}

    def launches(self):
        U, k = len(self.units), K_WORKERS
        return {"flatten": U * k, "compress_minmax": U * k, "drr_minmax": U, "ring_fp": U, "ring_lp": U,
                "sign_compress": U * k, "drr_sign": U}

    def step(self, only=None, marks=None):
        """Enqueue one pass of the hot path.  marks (optional): list receiving (name, event) boundaries."""
        torch, bg = self.torch, self.bg
        k, U = K_WORKERS, len(self.units)
        it = self.step_no % GRAD_SETS
        src, dst = self.step_no % 2, (self.step_no + 1) % 2

        def mark(name):
            if marks is not None:
                ev = torch.cuda.Event(enable_timing=True)
                ev.record()
                marks.append((name, ev))

        run = (lambda p: True) if not only else (lambda p: p in only)
        mark("start")
        if run("flatten"):
            for j in range(k):
                for u in range(U):
                    bg.bagua_bucket_flatten_run(self.plans[it][j][u], len(self.units[u][2]), self.bucket[j][u])
        mark("flatten")
        if run("compress_minmax"):
            for j in range(k):
                for u in range(U):
                    bg.bagua_compress_minmax_u8(self.bucket[j][u], self.delta[j][u], CHUNK, self.codes[j][u], self.minmax[j][u])
        mark("compress_minmax")
        if run("drr_minmax"):
            for u in range(U):
                bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, [self.codes[j][u] for j in range(k)],
                                                      [self.minmax[j][u] for j in range(k)], self.eps[u],
                                                      self.units[u][1], CHUNK, self.codes_out[u], self.minmax_out[u],
                                                      self.out[u])
        mark("drr_minmax")
        if run("ring_fp"):
            for u in range(U):
                bg.bagua_decentralized_avg(bg.AVG_FP, [self.rep_fp[src][i][u] for i in range(k)],
                                           [self.rep_fp[dst][i][u] for i in range(k)])
        mark("ring_fp")
        if run("ring_lp"):
            for u in range(U):
                bg.bagua_decentralized_avg(bg.AVG_LP_MINMAX_U8, [self.rep_lp[src][i][u] for i in range(k)],
                                           [self.rep_lp[dst][i][u] for i in range(k)], [self.xhat[i][u] for i in range(k)],
                                           [self.lp_codes[i][u] for i in range(k)], [self.lp_minmax[i][u] for i in range(k)], CHUNK)
        mark("ring_lp")
        if run("sign_compress"):
            for j in range(k):
                for u in range(U):
                    bg.bagua_sign_compress_ef(self.bucket[j][u], self.sdelta[j][u], SIGN_CHUNK, self.bits[j][u], self.scale[j][u])
        mark("sign_compress")
        if run("drr_sign"):
            for u in range(U):
                bg.bagua_decompress_reduce_recompress(bg.CODEC_SIGN1, [self.bits[j][u] for j in range(k)],
                                                      [self.scale[j][u] for j in range(k)], self.seps[u],
                                                      self.units[u][1], SIGN_CHUNK, self.bits_out[u], self.scale_out[u],
                                                      self.sout[u])
        mark("drr_sign")
        self.step_no += 1


def cpu_baseline(wl, torch):
    """The oracle, as it stands, on the host cores: one step (all seven primitives, every bucket, all 8 workers)
    of the same workload, timed once.  Returns the dict for the JSON line."""
    import numpy as np
    import oracle
    threads = max(1, min(16, oracle.max_threads(), os.cpu_count() or 1))
    oracle.set_threads(threads)
    k = K_WORKERS
    dt = 0.0
    for b, bk in enumerate(wl.buckets):
        n, lo = bk.n_pad, wl.bases[b]
        srcs = [[wl.layers[0][j][t].cpu().numpy() for t in bk.tensors] for j in range(k)]
        full = [wl.rep_fp[wl.step_no % 2][i] for i in range(k)]
        reps = [torch.cat(full[i])[lo:lo + n].cpu().numpy() for i in range(k)]
        hats = [torch.cat(wl.xhat[i])[lo:lo + n].cpu().numpy().copy() for i in range(k)]
        t0 = time.perf_counter()
        flats = [oracle.bucket_flatten(srcs[j], bk.offsets, n) for j in range(k)]
        deltas = [np.zeros(n, np.float32) for _ in range(k)]
        enc = [oracle.compress_minmax_u8(flats[j], deltas[j], CHUNK) for j in range(k)]
        oracle.drr_minmax_u8([e[0] for e in enc], [e[1] for e in enc], np.zeros(n, np.float32), CHUNK)
        oracle.ring_avg_fp(reps)
        oracle.ring_avg_lp(reps, hats, CHUNK)
        sd = [np.zeros(n, np.float32) for _ in range(k)]
        senc = [oracle.sign_compress_ef(flats[j], sd[j], SIGN_CHUNK) for j in range(k)]
        oracle.drr_sign([e[0] for e in senc], [e[1] for e in senc], np.zeros(n, np.float32), n, SIGN_CHUNK)
        dt += time.perf_counter() - t0
    grad_bytes = 4.0 * wl.n_elems * k * len(PRIMS)
    return {"value": round(grad_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "one full step of the same workload (%d elements x %d workers, all seven primitives), "
                      "%.1f s wall on %d threads" % (wl.n_elems, k, dt, threads)}


def read_traffic():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", "compress_minmax_resnet50_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build is the single-GPU share of the path (the k workers are k buffers in one GPU's "
              "HBM); --gpus %d is not supported, run with --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2107_01499_amd as bg     # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    only = set(p for p in args.only.split(",") if p) or None
    wl = Workload(torch, bg, per_bucket=args.per_bucket_launch)

    for _ in range(args.warmup):
        wl.step(only)
    torch.cuda.synchronize()
    all_marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        marks = []
        wl.step(only, marks)
        all_marks.append(marks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # per-primitive GPU time from the events recorded on the launch stream inside the timed region
    prim_ms = {p: 0.0 for p in PRIMS}
    for marks in all_marks:
        for (_, e0), (name, e1) in zip(marks[:-1], marks[1:]):
            prim_ms[name] += e0.elapsed_time(e1)
    gpu_ms = sum(m[0][1].elapsed_time(m[-1][1]) for m in all_marks)
    for p in PRIMS:
        prim_ms[p] /= args.steps
    ms_per_step = wall * 1e3 / args.steps

    gb, ab, nl = wl.grad_bytes(), wl.algo_bytes(), wl.launches()
    active = [p for p in PRIMS if (only is None or p in only)]
    total_grad = sum(gb[p] for p in active)
    per_prim = {}
    for p in active:
        t = prim_ms[p] * 1e-3
        per_prim[p] = {"ms": round(prim_ms[p], 4), "launches": nl[p], "gradient_GBps": round(gb[p] / t / 1e9, 1),
                       "hbm_GBps": round(ab[p] / t / 1e9, 1), "frac_of_peak": round(ab[p] / t / 1e9 / HBM_PEAK_GBS, 4)}
    dom = "compress_minmax" if "compress_minmax" in active else max(active, key=lambda p: prim_ms[p])
    dom_t = prim_ms[dom] * 1e-3 / nl[dom]
    achieved = ab[dom] / nl[dom] / dom_t / 1e9
    traffic = read_traffic() if dom == "compress_minmax" else None
    result = {
        "metric": "gradient GB/s processed per primitive on 1 MI355X; % of HBM roofline",
        "value": round(total_grad / (wall / args.steps) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs[1]: ResNet-50-shaped gradients, 25,557,032 fp32 per worker in %d greedy 25 MiB "
                               "buckets (%d padded elements), 8 simulated workers, chunk %d (sign codec %d), error "
                               "state carried across steps, all seven primitives per step" %
                               (len(wl.buckets), wl.n_elems, CHUNK, SIGN_CHUNK),
                   "workers": K_WORKERS, "chunk": CHUNK, "sign_chunk": SIGN_CHUNK, "buckets": len(wl.buckets),
                   "launch": "per bucket" if args.per_bucket_launch else "per worker (all buckets of a worker in one launch)",
                   "elements_per_worker": wl.n_elems},
        "gpu_ms_per_step": round(gpu_ms / args.steps, 4),
        "per_primitive": per_prim,
        "roofline": {"bound": "hbm", "kernel": KERNEL_OF[dom], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "avg_launch_us": round(dom_t * 1e6, 3), "algorithmic_bytes_per_launch": ab[dom] / nl[dom]},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, torch)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
