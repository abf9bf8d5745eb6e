#!/usr/bin/env python3
"""Benchmark of the compression hot path on one MI355X.

Default run (`python bench.py`): every primitive is timed at the LARGEST benchmark configuration that names it,
one configuration after another (buffers freed in between), each with --warmup untimed and --steps timed steps:

  configs[2]  BERT-large-shaped gradients, 16 workers, C = 8192     flatten, compress_minmax, drr_minmax
  configs[3]  8 peers x BERT-base-shaped replicas on a ring           ring_fp, ring_lp
  configs[4]  1.5e9 elements x 8 workers, 1-bit sign codec, C = 2048  sign_compress, drr_sign (one launch per worker)

One "step" is one pass of the whole hot path: all seven primitives, each over its configuration's batch.  The
headline `value` is 4 B x fp32 gradient elements consumed, summed over the seven primitives, over the summed wall time
of one step of each of the three blocks.  Reported in addition (own timing, not part of `value`): configs[4] as 229
separately allocated buckets per worker through the batched entry points, configs[1] (ResNet-50 shapes, all seven
primitives) and configs[0] replicated 32 times (plus the latency of one cache-resident instance).

Per primitive: ms, launches, gradient GB/s, algorithmic HBM GB/s, fraction of the 8 TB/s peak and of the measured copy
ceiling.  `roofline` is the kernel with the largest share of the timed GPU time; `roofline_per_config` has the dominant
kernel of every block.  `cpu_baseline` times the CPU oracle on a bounded sample (>= 1 GiB of fp32 input where the
configuration is that large) of every block on the host cores; `parity` compares the HIP path with the oracle's
outputs on those same samples, all primitives, word for word.  Inputs are generated on the GPU before the timed
region and stay resident in HBM.  Prints ONE JSON line.

--workload W runs one block only (resnet50, bert_large, bert_base_ring, onebit, single_bucket_x32); --layout chooses
how a worker's buckets are launched: flat (default: back to back in one allocation, one launch per worker; every bucket
is padded to a multiple of k*chunk, so results equal bucket-by-bucket launches bit for bit), per_bucket (one launch per
bucket) or buckets (separately allocated buckets, one batched launch per worker).  --verify-all streams EVERY element
of configs[2], [3] (5 rounds) and [4] through the oracle instead of timing.  --gpus N with N > 1 is refused.
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
ALL_PRIMS = ["flatten", "compress_minmax", "drr_minmax", "ring_fp", "ring_lp", "sign_compress", "drr_sign"]

WORKLOADS = {
    # name: cfg id for seeds, k, chunk, sign chunk, value distribution, gradient sets rotated, primitives
    "resnet50": dict(cfg=1, k=8, chunk=4096, sign_chunk=2048, dist="normal_layer", sets=3, prims=ALL_PRIMS,
                     placement="spread", mean_gap_gib=1.0,
                     label="configs[1]: ResNet-50-shaped gradients, 25,557,032 fp32 per worker"),
    "bert_large": dict(cfg=2, k=16, chunk=8192, sign_chunk=2048, dist="student_t3", sets=1,
                       placement="spread", mean_gap_gib=1.3,
                       prims=["flatten", "compress_minmax", "drr_minmax"],
                       label="configs[2]: BERT-large-shaped gradients, 335,141,888 fp32 per worker, Student-t(3)"),
    "bert_base_ring": dict(cfg=3, k=8, chunk=4096, sign_chunk=2048, dist="normal", sets=1, prims=["ring_fp", "ring_lp"],
                           placement="spread", mean_gap_gib=3.0,
                           label="configs[3]: 8 peers x BERT-base-shaped replicas (109,482,240 fp32), base + drift"),
    "onebit": dict(cfg=4, k=8, chunk=4096, sign_chunk=2048, dist="laplace", sets=1, prims=["sign_compress", "drr_sign"],
                   placement="spread", mean_gap_gib=2.0,
                   label="configs[4]: 1.5e9 fp32 per worker, Laplace(0,1e-3), 1-bit sign codec"),
    "single_bucket_x32": dict(cfg=0, k=4, chunk=4096, sign_chunk=2048, dist="normal", sets=3,
                              placement="spread", mean_gap_gib=4.0,
                              prims=["compress_minmax", "drr_minmax"],
                              label="configs[0] x 32 independent instances: 1,048,576 fp32 per worker and instance, N(0,1e-3)"),
}
SPREAD_GIB = 200            # size of the reservation of the "spread" placement
ONEBIT_N = 1500000000
INSTANCES = 32
# the default run: (workload, layout, counts towards the headline)
DEFAULT_PLAN = [("bert_large", "flat", True), ("bert_base_ring", "flat", True), ("onebit", "flat", True),
                ("onebit", "buckets", False), ("resnet50", "flat", False), ("single_bucket_x32", "flat", False)]


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="all", choices=["all"] + sorted(WORKLOADS))
    ap.add_argument("--layout", default="flat", choices=["flat", "per_bucket", "buckets"],
                    help="with --workload: flat = one launch per worker over its contiguous buckets; per_bucket = one "
                         "launch per bucket; buckets = separately allocated buckets, one batched launch per worker")
    ap.add_argument("--placement", default=None, choices=["spread", "packed"],
                    help="where the resident buffers lie in HBM (default: per workload; see Workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing and parity leg")
    ap.add_argument("--only", default="", help="comma list of primitives to run in the step (profiling aid)")
    ap.add_argument("--extras", default="", help="comma list of additional primitives appended to the step: sgd_step "
                    "(decode of the server's codes fused into an SGD-momentum update of every worker's replica), "
                    "adam_step (the same decode fused into an Adam update), onebit_adam (compression stage of 1-bit Adam: momentum "
                    "sign compression on every worker and the decode + frozen-variance update), "
                    "lp_shares (D_LP_S on a ring as the k single-peer shares a sharded run would execute: encode, then apply + mix), "
                    "peer_fp / peer_lp (full- / low-precision averaging with one chosen peer per worker), reduce_compress (intra-node "
                    "stage of hierarchical C_LP_S: 4 local workers averaged uncompressed, leader compresses), topk (C_LP_S with "
                    "the per-chunk top-K codec, keep = chunk/32: worker side and server side), unflatten (the server's codes decoded "
                    "straight into every worker's layer tensors), flatten_sign (gather fused into the sign compression)")
    ap.add_argument("--fused-flatten", action="store_true",
                    help="replace flatten + compress_minmax by the fused bagua_flatten_compress_minmax_u8")
    ap.add_argument("--per-bucket-launch", action="store_true", help="same as --layout per_bucket")
    ap.add_argument("--verify-all", action="store_true",
                    help="no timing: compare EVERY element of configs[2], configs[3] (5 rounds) and configs[4] with the oracle")
    return ap.parse_args()


class Placer:
    """Places tensors in one large reservation with a seeded pseudo-random gap after each, so that a set of buffers is
    scattered over `gib` GiB of HBM (2 MiB-aligned starts).  Measured on MI355X: kernels that stream 16-40 buffers at
    once run 15-20 % faster when those buffers span more than ~48 GiB of the address space than when they sit back
    to back; kernels with up to ~5 streams do not care."""

    def __init__(self, torch, gib, seed, mean_gap_gib):
        import random
        self.arena = torch.empty(gib << 30, dtype=torch.uint8, device="cuda:0")
        self.rng = random.Random(seed)
        self.mean_gap = int(mean_gap_gib * (1 << 30))
        self.bump = 0
        self.overflow = 0       # tensors that no longer fitted into the reservation

    def place(self, t):
        nbytes = t.numel() * t.element_size()
        start = (self.bump + (1 << 21) - 1) >> 21 << 21
        if start + nbytes > self.arena.numel():      # reservation exhausted: this tensor stays where the allocator put it
            self.overflow += 1
            return t
        out = self.arena[start:start + nbytes].view(t.dtype)
        out.copy_(t)
        self.bump = start + nbytes + self.rng.randrange(0, 2 * self.mean_gap)
        return out


class Workload:
    """Synthetic gradients / replicas of one benchmark configuration, all state resident on the GPU."""

    def __init__(self, torch, bg, name, layout="flat", only=None, fused=False, extras=(), placement=None):
        from bagua_workloads import resnet50_shapes, bert_shapes, pack_buckets, draw, seed_for, layer_sigmas
        from bagua_workloads.shapes import numel
        from bagua_workloads.generators import SHARED
        self.torch, self.bg, self.name, self.layout = torch, bg, name, layout
        # Where the resident buffers lie in HBM.  "spread": every buffer is placed in one large reservation with a seeded
        # pseudo-random gap after it, so the workload's buffers are scattered over SPREAD_GIB of HBM, as they are in a
        # training process whose HBM is mostly in use; "packed": plain allocations, back to back in a fresh process.
        # Every flat block of the default run is spread (also the two big ones: the buffers one server-step launch
        # streams, k code arrays + error state + output, lie within 14 GB of each other when packed); the layout of
        # separately allocated buckets is what the allocator makes of it.
        self.placement = placement or ("packed" if layout == "buckets" else WORKLOADS[name].get("placement", "packed"))
        self._placer = None
        if self.placement == "spread":
            try:
                # separately allocated buckets are thousands of small buffers: a small gap after each
                gap = 0.008 if layout == "buckets" else WORKLOADS[name].get("mean_gap_gib", 1.0)
                self._placer = Placer(torch, SPREAD_GIB, WORKLOADS[name]["cfg"], gap)
            except RuntimeError as e:       # not enough free HBM for the reservation: say so and run packed
                print("bench: %d GiB reservation failed (%s); placement packed" % (SPREAD_GIB, str(e).splitlines()[0]),
                      file=sys.stderr, flush=True)
                self.placement = "packed (the %d GiB reservation of the spread placement could not be allocated)" % SPREAD_GIB
        per_bucket = layout in ("per_bucket", "buckets")
        self.batched = layout == "buckets"
        w = WORKLOADS[name]
        self.w = w
        self.k, self.C, self.SC = w["k"], w["chunk"], w["sign_chunk"]
        self.prims = [p for p in w["prims"] if (only is None or p in only)]
        if fused and "flatten" in self.prims and "compress_minmax" in self.prims:
            self.prims = ["flatten_compress" if p == "flatten" else p for p in self.prims if p != "compress_minmax"]
        if "sgd_step" in extras and "drr_minmax" in self.prims:
            self.prims = self.prims + ["sgd_step"]
        if "adam_step" in extras and "drr_minmax" in self.prims:
            self.prims = self.prims + ["adam_step"]
        if "onebit_adam" in extras and "drr_sign" in self.prims and "sign_compress" in self.prims:
            self.prims = self.prims + ["momentum_sign", "adam_frozen_step"]
        if "reduce_compress" in extras and ("flatten" in self.prims or "flatten_compress" in self.prims):
            self.prims = self.prims + ["reduce_compress"]
        if "topk" in extras and ("flatten" in self.prims or "flatten_compress" in self.prims):
            self.prims = self.prims + ["compress_topk", "drr_topk"]
        if "unflatten" in extras and "drr_minmax" in self.prims and "flatten" in self.prims:
            self.prims = self.prims + ["decompress_unflatten"]
        if "flatten_sign" in extras and "flatten" in self.prims:
            self.prims = self.prims + ["flatten_sign_compress"]
        if "peer_fp" in extras and "ring_fp" in self.prims:
            self.prims = self.prims + ["peer_fp"]
        if "peer_lp" in extras and "ring_lp" in self.prims:
            self.prims = self.prims + ["peer_lp"]
        if "lp_shares" in extras and "ring_lp" in self.prims:
            self.prims = self.prims + ["lp_encode", "lp_apply_mix"]
        k, C, SC, cfg = self.k, self.C, self.SC, w["cfg"]
        dev = torch.device("cuda:0")
        f32 = dict(dtype=torch.float32, device=dev)
        u8 = dict(dtype=torch.uint8, device=dev)
        i32 = dict(dtype=torch.int32, device=dev)
        z = lambda m, **kw: torch.zeros(m, **kw)
        has = lambda *ps: any(p in self.prims for p in ps)

        # ---- shapes, buckets, launch units
        if name == "onebit":
            shapes = [("momentum", (ONEBIT_N,))]
            n = ONEBIT_N
            self.buckets, self.bases = [], [0, n]
            if per_bucket:      # 229 buckets of 25 MiB, the last one short
                from bagua_workloads import BUCKET_ELEMS
                self.units = [(lo, min(BUCKET_ELEMS, n - lo), [0], [0]) for lo in range(0, n, BUCKET_ELEMS)]
            else:
                self.units = [(0, n, [0], [0])]
        else:
            if name == "single_bucket_x32":
                shapes = [("instance%d" % i, (1048576,)) for i in range(INSTANCES)]
                self.buckets = pack_buckets(shapes, k, C, cap=1048576)
            else:
                shapes = {"resnet50": resnet50_shapes, "bert_large": lambda: bert_shapes(24, 1024, 4096),
                          "bert_base_ring": lambda: bert_shapes(12, 768, 3072)}[name]()
                self.buckets = pack_buckets(shapes, k, C)
            self.bases = [0]
            for bk in self.buckets:
                self.bases.append(self.bases[-1] + bk.n_pad)
            n = self.bases[-1]
            if per_bucket:
                self.units = [(self.bases[b], bk.n_pad, list(bk.tensors), list(bk.offsets)) for b, bk in enumerate(self.buckets)]
            else:
                ids, offs = [], []
                for b, bk in enumerate(self.buckets):
                    ids += list(bk.tensors)
                    offs += [self.bases[b] + o for o in bk.offsets]
                self.units = [(0, n, ids, offs)]
        self.n_elems = n
        self.sizes = [numel(s) for _, s in shapes]
        self.total = sum(self.sizes)
        U = len(self.units)
        nc, ncs = (n + C - 1) // C, (n + SC - 1) // SC

        def place(t):
            """The tensor itself ("packed") or a copy of it at the next place of the reservation ("spread")."""
            return t if self._placer is None else self._placer.place(t)

        def views(t, div=1, mul=1):
            """Per-unit views of a flat tensor whose index is element_index * mul / div; in the "buckets" layout every
            unit gets an allocation of its own instead (the flat tensor is dropped by the caller)."""
            if self.batched:        # every unit an allocation (or, spread, a place in the reservation) of its own
                vs = [t[lo * mul // div:-(-(lo + ln) * mul // div)] for lo, ln, _, _ in self.units]
                out = []
                for v in vs:
                    pv = place(v)
                    out.append(v.clone() if pv is v else pv)      # packed, or the reservation is exhausted
                return out
            t = place(t)
            return [t[lo * mul // div:-(-(lo + ln) * mul // div)] for lo, ln, _, _ in self.units]

        # ---- gradients: layer tensors (when flatten runs) or ready-made flat buckets
        self.sets = w["sets"]
        scale = 1e-3
        self.layers, self.plans = [], []
        self.bucket = None
        if has("flatten", "flatten_compress"):
            sig = layer_sigmas(len(shapes), seed_for(cfg, 0, SHARED)) if w["dist"] == "normal_layer" else None
            starts = [0]
            for sz in self.sizes:
                starts.append(starts[-1] + sz)
            for it in range(self.sets):
                per_worker = []
                for j in range(k):
                    if sig is None:
                        arena = draw(w["dist"], self.total, seed_for(cfg, it, j), dev, scale)
                    else:
                        arena = draw("normal", self.total, seed_for(cfg, it, j), dev, 1.0)
                    arena = place(arena)
                    vs = []
                    for t, sz in enumerate(self.sizes):
                        v = arena[starts[t]:starts[t + 1]]
                        if sig is not None:
                            v.mul_(sig[t])
                        vs.append(v)
                    per_worker.append(vs)
                self.layers.append(per_worker)
            self.plans = [[[None] * U for _ in range(k)] for _ in range(self.sets)]
            for it in range(self.sets):
                for j in range(k):
                    for u, (lo, ln, ids, offs) in enumerate(self.units):
                        ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(ids), ln), **u8)
                        bg.bagua_flatten_plan([self.layers[it][j][t] for t in ids], offs, ln, ws)
                        self.plans[it][j][u] = ws
            self.bucket = [views(z(n, **f32)) for _ in range(k)]
        elif has("compress_minmax", "sign_compress"):
            dist = "normal" if w["dist"] == "normal_layer" else w["dist"]
            self.bucket = [views(draw(dist, n, seed_for(cfg, 0, j), dev, scale)) for j in range(k)]
        if has("compress_minmax", "drr_minmax", "flatten_compress"):
            self.delta = [views(z(n, **f32)) for _ in range(k)]
            self.codes = [views(z(n, **u8)) for _ in range(k)]
            self.minmax = [views(z(2 * nc, **f32), C, 2) for _ in range(k)]
        if has("drr_minmax"):
            if not has("compress_minmax", "flatten_compress"):
                for j in range(k):
                    for u in range(U):
                        bg.bagua_compress_minmax_u8(self.bucket[j][u], None, C, self.codes[j][u], self.minmax[j][u])
            self.eps = views(z(n, **f32))
            self.codes_out = views(z(n, **u8))
            self.minmax_out = views(z(2 * nc, **f32), C, 2)
            self.out = views(z(n, **f32))
        if has("flatten_sign_compress"):
            self.fsdelta = [views(z(n, **f32)) for _ in range(k)]
            self.fsbits = [views(z((n + 31) // 32, **i32), 32) for _ in range(k)]
            self.fsscale = [views(z(ncs, **f32), SC) for _ in range(k)]
        if has("reduce_compress"):      # hierarchical C_LP_S: nodes of 4 local workers, one leader each
            self.kl = 4
            self.hdelta = [views(z(n, **f32)) for _ in range(k // self.kl)]
            self.hcodes = [views(z(n, **u8)) for _ in range(k // self.kl)]
            self.hminmax = [views(z(2 * nc, **f32), C, 2) for _ in range(k // self.kl)]
        if has("compress_topk"):        # top-K codec: keep chunk/32 entries per chunk
            self.keep = C // 32
            self.tdelta = [views(z(n, **f32)) for _ in range(k)]
            self.tidx = [views(z(nc * self.keep, dtype=torch.int16, device=dev), C, self.keep) for _ in range(k)]
            self.tval = [views(z(nc * self.keep, **f32), C, self.keep) for _ in range(k)]
            self.teps = views(z(n, **f32))
            self.tidx_out = views(z(nc * self.keep, dtype=torch.int16, device=dev), C, self.keep)
            self.tval_out = views(z(nc * self.keep, **f32), C, self.keep)
            self.tout = views(z(n, **f32))
        if has("sgd_step", "adam_step", "adam_frozen_step"):
            self.param = [views(draw("normal", n, seed_for(cfg, 50, j), dev, 0.02)) for j in range(k)]
            self.mbuf = [views(z(n, **f32)) for _ in range(k)]
        if has("adam_step"):
            self.vbuf = [views(z(n, **f32)) for _ in range(k)]
        if has("momentum_sign"):
            self.shared_m = views(draw("normal", n, seed_for(cfg, 51, SHARED), dev, scale))
            self.frozen_v = views(draw("normal", n, seed_for(cfg, 52, SHARED), dev, scale).square_())
            self.msdelta = [views(z(n, **f32)) for _ in range(k)]
            self.mbits = [views(z((n + 31) // 32, **i32), 32) for _ in range(k)]
            self.mscale = [views(z(ncs, **f32), SC) for _ in range(k)]
        if has("sign_compress", "drr_sign"):
            self.sdelta = [views(z(n, **f32)) for _ in range(k)]
            self.bits = [views(z((n + 31) // 32, **i32), 32) for _ in range(k)]
            self.scale = [views(z(ncs, **f32), SC) for _ in range(k)]
        if has("drr_sign"):
            if not has("sign_compress"):
                for j in range(k):
                    for u in range(U):
                        bg.bagua_sign_compress_ef(self.bucket[j][u], None, SC, self.bits[j][u], self.scale[j][u])
            self.seps = views(z(n, **f32))
            self.bits_out = views(z((n + 31) // 32, **i32), 32)
            self.scale_out = views(z(ncs, **f32), SC)
            self.sout = views(z(n, **f32))
        # ---- decentralised replicas: shared base + per-peer drift; ping-pong sets
        if has("ring_fp", "ring_lp"):
            base = draw("normal", n, seed_for(3, 0, SHARED), dev, 0.02)
            self.rep_fp = [[None] * k for _ in range(2)]
            self.rep_lp = [[None] * k for _ in range(2)]
            self.xhat = [None] * k
            for i in range(k):
                x = base + draw("normal", n, seed_for(3, 0, i), dev, 1e-3)
                if has("ring_fp"):
                    self.rep_fp[0][i] = views(x)
                    self.rep_fp[1][i] = views(torch.empty_like(x))
                if has("ring_lp"):
                    self.rep_lp[0][i] = views(x.clone())
                    self.rep_lp[1][i] = views(torch.empty_like(x))
                    self.xhat[i] = views(base.clone())
            if has("ring_lp"):
                self.lp_codes = [views(z(n, **u8)) for _ in range(k)]
                self.lp_minmax = [views(z(2 * nc, **f32), C, 2) for _ in range(k)]
            if has("lp_encode"):       # every peer's own copies of its two neighbours' public replicas
                self.nb_left = [views(base.clone()) for _ in range(k)]
                self.nb_right = [views(base.clone()) for _ in range(k)]
                self.sh_hat = [views(base.clone()) for _ in range(k)]
        if self.batched:
            self.bws = torch.empty(bg.bagua_batch_workspace_bytes(U, 0), **u8)
            self.bws_k = torch.empty(bg.bagua_batch_workspace_bytes(U, k), **u8)
            self.unit_n = [ln for _, ln, _, _ in self.units]
        self.step_no = 0
        torch.cuda.synchronize()

    # ---- accounting --------------------------------------------------------------------------------
    def bytes_per_element(self):
        k, C, SC = self.k, self.C, self.SC
        keep = getattr(self, "keep", 0)
        wb = 4.0 if "sign_compress" in self.prims else 0.0   # the fused call also writes the bucket if it is needed later
        return {"flatten": 8.0, "flatten_compress": 13.0 + wb + 8.0 / C, "compress_minmax": 13.0 + 8.0 / C, "drr_minmax": k + 13.0 + 8.0 * (k + 1) / C,
                "decompress_unflatten": 5.0 + 8.0 / C, "flatten_sign_compress": 12.125 + 4.0 / SC,
                "compress_topk": 12.0 + 6.0 * keep / C, "drr_topk": 12.0 + 6.0 * (k + 1) * keep / C,
                "sgd_step": 17.0 + 8.0 / C, "adam_step": 25.0 + 8.0 / C, "momentum_sign": 16.125 + 4.0 / SC,
                "adam_frozen_step": 16.125 + 4.0 / SC, "reduce_compress": 4.0 * 4 + 9.0 + 8.0 / C, "peer_fp": 8.0, "peer_lp": 17.0 + 8.0 / C, "lp_encode": 13.0 + 8.0 / C, "lp_apply_mix": 30.0 + 16.0 / C, "ring_fp": 8.0, "ring_lp": 17.0 + 8.0 / C, "sign_compress": 12.125 + 4.0 / SC,
                "drr_sign": k / 8.0 + 12.125 + 4.0 * (k + 1) / SC}

    def grad_bytes(self):
        """4 B x fp32 elements each primitive consumes (or, for the server step, represents)."""
        return {p: 4.0 * self.n_elems * self.k for p in self.prims}

    def algo_bytes(self):
        n, k = self.n_elems, self.k
        units = {"flatten": n * k, "flatten_compress": n * k, "compress_minmax": n * k, "drr_minmax": n, "ring_fp": n * k, "ring_lp": n * k,
                 "sign_compress": n * k, "drr_sign": n, "sgd_step": n * k, "adam_step": n * k, "momentum_sign": n * k, "adam_frozen_step": n * k, "peer_fp": n * k, "peer_lp": n * k, "lp_encode": n * k, "lp_apply_mix": n * k, "reduce_compress": n * (k // 4),
                 "compress_topk": n * k, "drr_topk": n, "decompress_unflatten": n * k, "flatten_sign_compress": n * k}
        bpe = self.bytes_per_element()
        return {p: bpe[p] * units[p] for p in self.prims}

    def launches(self):
        U, k = (1 if self.batched else len(self.units)), self.k
        per = {"flatten": U * k, "flatten_compress": U * k, "compress_minmax": U * k, "drr_minmax": U, "ring_fp": U, "ring_lp": U,
               "sign_compress": U * k, "drr_sign": U, "sgd_step": U * k, "adam_step": U * k, "momentum_sign": U * k, "adam_frozen_step": U * k, "peer_fp": U, "peer_lp": U, "lp_encode": U * k, "lp_apply_mix": U * k, "reduce_compress": U * (k // 4),
               "compress_topk": U * k, "drr_topk": U, "decompress_unflatten": U * k, "flatten_sign_compress": U * k}
        return {p: per[p] for p in self.prims}

    @staticmethod
    def _rpw_worker(chunk):
        """Rows per wave the library picks for an unbatched worker-side launch (pick_rpw_worker in csrc/common.hpp)."""
        rows = chunk // 256
        rpw = 1 if 6 <= rows <= 8 else 2
        while rpw < 8 and (rows + rpw - 1) // rpw > 16:
            rpw *= 2
        return rpw

    def placement_note(self):
        over = self._placer.overflow if self._placer is not None else 0
        return self.placement + (" (%d tensors did not fit into the reservation and lie where the allocator put them)" % over if over else "")

    def kernel_name(self, p):
        if self.batched and p in ("flatten", "compress_minmax", "drr_minmax", "sign_compress", "drr_sign"):
            return {"flatten": "k_flatten_batched", "compress_minmax": "k_compress_minmax_batched<2,true>",
                    "drr_minmax": "k_drr_minmax_batched<4,true,true>", "sign_compress": "k_sign_compress_batched<2,true>",
                    "drr_sign": "k_drr_sign_batched<2,true,true>"}[p]
        return {"flatten": "k_flatten", "flatten_compress": "k_flatten_compress_minmax<2,true,%s>" %
                ("true" if "sign_compress" in self.prims else "false"), "compress_minmax": "k_compress_minmax<%d,true>" % self._rpw_worker(self.C),
                "drr_minmax": "k_drr_minmax<4,true,true>", "ring_fp": "k_ring_avg_fp<%d>" % self.k,
                "ring_lp": "k_ring_avg_lp<%d,2>" % self.k, "sign_compress": "k_sign_compress<%d,true,false>" % self._rpw_worker(self.SC),
                "drr_sign": "k_drr_sign<2,true,true>", "sgd_step": "k_decompress_sgd<0,true,false>",
                "adam_step": "k_decompress_adam<0,false,false>", "momentum_sign": "k_sign_compress<%d,true,true>" % self._rpw_worker(self.SC),
                "adam_frozen_step": "k_decompress_adam<1,true,false>",
                "peer_fp": "k_peer_avg_fp", "peer_lp": "k_peer_avg_lp<2>", "lp_encode": "k_lp_encode<2>", "lp_apply_mix": "k_lp_apply_mix<true,true,false>", "reduce_compress": "k_reduce_compress_minmax<2,true>",
                "compress_topk": "k_compress_topk<4,true>", "drr_topk": "k_drr_topk<4,true,true>",
                "decompress_unflatten": "k_decompress_unflatten<0>", "flatten_sign_compress": "k_flatten_sign_compress<2,true,false>"}[p]

    # ---- one pass of the hot path ------------------------------------------------------------------
    def step(self, marks=None):
        """Enqueue one pass.  marks (optional): list receiving (name, event) boundaries on the launch stream."""
        torch, bg = self.torch, self.bg
        k, U, C, SC = self.k, len(self.units), self.C, self.SC
        it = self.step_no % self.sets
        src, dst = self.step_no % 2, (self.step_no + 1) % 2

        def mark(name):
            if marks is not None:
                ev = torch.cuda.Event(enable_timing=True)
                ev.record()
                marks.append((name, ev))

        mark("start")
        for p in self.prims:
            if self.batched and p in ("flatten", "compress_minmax", "drr_minmax", "sign_compress", "drr_sign"):
                self.step_batched(p, it)
            elif p == "flatten":
                for j in range(k):
                    for u in range(U):
                        bg.bagua_bucket_flatten_run(self.plans[it][j][u], len(self.units[u][2]), self.bucket[j][u])
            elif p == "flatten_compress":
                keep = "sign_compress" in self.prims
                for j in range(k):
                    for u in range(U):
                        bg.bagua_flatten_compress_minmax_u8(self.plans[it][j][u], len(self.units[u][2]), self.delta[j][u],
                                                            self.units[u][1], C, self.codes[j][u], self.minmax[j][u],
                                                            self.bucket[j][u] if keep else None)
            elif p == "compress_minmax":
                for j in range(k):
                    for u in range(U):
                        bg.bagua_compress_minmax_u8(self.bucket[j][u], self.delta[j][u], C, self.codes[j][u], self.minmax[j][u])
            elif p == "drr_minmax":
                for u in range(U):
                    bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, [self.codes[j][u] for j in range(k)],
                                                          [self.minmax[j][u] for j in range(k)], self.eps[u],
                                                          self.units[u][1], C, self.codes_out[u], self.minmax_out[u],
                                                          self.out[u])
            elif p == "decompress_unflatten":   # every worker decodes the server's codes straight into its layer tensors
                for j in range(k):
                    for u in range(U):
                        bg.bagua_decompress_unflatten(bg.CODEC_MINMAX_U8, self.codes_out[u], self.minmax_out[u],
                                                      self.units[u][1], C, self.plans[it][j][u], len(self.units[u][2]))
            elif p == "flatten_sign_compress":
                for j in range(k):
                    for u in range(U):
                        bg.bagua_flatten_sign_compress_ef(self.plans[it][j][u], len(self.units[u][2]), self.fsdelta[j][u],
                                                          self.units[u][1], SC, self.fsbits[j][u], self.fsscale[j][u], None)
            elif p == "sgd_step":
                for j in range(k):
                    for u in range(U):
                        bg.bagua_decompress_sgd_step(bg.CODEC_MINMAX_U8, self.codes_out[u], self.minmax_out[u],
                                                     self.units[u][1], C, self.param[j][u], self.mbuf[j][u], 0.01, 0.9, 0.0)
            elif p == "adam_step":
                for j in range(k):
                    for u in range(U):
                        bg.bagua_decompress_adam_step(bg.CODEC_MINMAX_U8, self.codes_out[u], self.minmax_out[u],
                                                      self.units[u][1], C, self.param[j][u], self.mbuf[j][u],
                                                      self.vbuf[j][u], 1e-3, 0.9, 0.999, 1e-8, 0.0, False)
            elif p == "momentum_sign":
                for j in range(k):
                    for u in range(U):
                        bg.bagua_momentum_sign_compress_ef(self.bucket[j][u], self.shared_m[u], 0.9, self.msdelta[j][u],
                                                           SC, self.mbits[j][u], self.mscale[j][u])
            elif p == "adam_frozen_step":
                for j in range(k):
                    for u in range(U):
                        bg.bagua_decompress_adam_step(bg.CODEC_SIGN1, self.bits_out[u], self.scale_out[u],
                                                      self.units[u][1], SC, self.param[j][u], self.mbuf[j][u],
                                                      self.frozen_v[u], 1e-3, 0.9, 0.999, 1e-8, 0.0, True)
            elif p == "compress_topk":
                for j in range(k):
                    for u in range(U):
                        bg.bagua_compress_topk_ef(self.bucket[j][u], self.tdelta[j][u], C, self.keep, self.tidx[j][u],
                                                  self.tval[j][u])
            elif p == "drr_topk":
                for u in range(U):
                    bg.bagua_decompress_reduce_recompress_topk([self.tidx[j][u] for j in range(k)],
                                                               [self.tval[j][u] for j in range(k)], self.keep, self.teps[u],
                                                               self.units[u][1], C, self.tidx_out[u], self.tval_out[u],
                                                               self.tout[u])
            elif p == "reduce_compress":
                for a in range(k // self.kl):
                    for u in range(U):
                        bg.bagua_reduce_compress_minmax_u8([self.bucket[a * self.kl + b][u] for b in range(self.kl)],
                                                           self.hdelta[a][u], C, self.hcodes[a][u], self.hminmax[a][u])
            elif p == "peer_fp":
                for u in range(U):     # a fixed perfect matching (0,1)(2,3)...; reads what ring_fp just wrote
                    bg.bagua_decentralized_avg_peers([self.rep_fp[dst][i][u] for i in range(k)],
                                                     [self.rep_fp[src][i][u] for i in range(k)], [i ^ 1 for i in range(k)])
            elif p == "peer_lp":
                for u in range(U):     # same matching, low precision; continues from what ring_lp just wrote
                    bg.bagua_decentralized_avg_peers_lp([self.rep_lp[dst][i][u] for i in range(k)],
                                                        [self.rep_lp[src][i][u] for i in range(k)],
                                                        [self.xhat[i][u] for i in range(k)],
                                                        [self.lp_codes[i][u] for i in range(k)],
                                                        [self.lp_minmax[i][u] for i in range(k)],
                                                        [i ^ 1 for i in range(k)], C)
            elif p == "lp_encode":
                for i in range(k):
                    for u in range(U):
                        bg.bagua_lp_encode(self.rep_lp[dst][i][u], self.sh_hat[i][u], C, self.lp_codes[i][u], self.lp_minmax[i][u])
            elif p == "lp_apply_mix":
                for i in range(k):
                    le, ri = (i - 1) % k, (i + 1) % k
                    for u in range(U):
                        bg.bagua_lp_apply_mix(self.rep_lp[dst][i][u], self.sh_hat[i][u], self.nb_left[i][u], self.nb_right[i][u],
                                              self.lp_codes[le][u], self.lp_minmax[le][u], self.lp_codes[ri][u],
                                              self.lp_minmax[ri][u], C, self.rep_lp[src][i][u])
            elif p == "ring_fp":
                for u in range(U):
                    bg.bagua_decentralized_avg(bg.AVG_FP, [self.rep_fp[src][i][u] for i in range(k)],
                                               [self.rep_fp[dst][i][u] for i in range(k)])
            elif p == "ring_lp":
                for u in range(U):
                    bg.bagua_decentralized_avg(bg.AVG_LP_MINMAX_U8, [self.rep_lp[src][i][u] for i in range(k)],
                                               [self.rep_lp[dst][i][u] for i in range(k)],
                                               [self.xhat[i][u] for i in range(k)], [self.lp_codes[i][u] for i in range(k)],
                                               [self.lp_minmax[i][u] for i in range(k)], C)
            elif p == "sign_compress":
                for j in range(k):
                    for u in range(U):
                        bg.bagua_sign_compress_ef(self.bucket[j][u], self.sdelta[j][u], SC, self.bits[j][u], self.scale[j][u])
            elif p == "drr_sign":
                for u in range(U):
                    bg.bagua_decompress_reduce_recompress(bg.CODEC_SIGN1, [self.bits[j][u] for j in range(k)],
                                                          [self.scale[j][u] for j in range(k)], self.seps[u],
                                                          self.units[u][1], SC, self.bits_out[u], self.scale_out[u],
                                                          self.sout[u])
            mark(p)
        self.step_no += 1


    def step_batched(self, p, it):
        """One primitive over all separately allocated buckets: one batched launch per worker (or one in all).  The
        pointer arrays are marshalled once (PreparedCall), as a trainer with fixed buckets would: a step is the C calls."""
        bg, k, U, C, SC = self.bg, self.k, len(self.units), self.C, self.SC
        if not hasattr(self, "_prepared"):
            self._prepared = {}
        key = (p, it if p == "flatten" else 0)
        if key not in self._prepared:
            if p == "flatten":
                calls = [bg.bagua_bucket_flatten_batched_run(self.plans[it][j], [len(u[2]) for u in self.units], self.bucket[j],
                                                             self.bws, prepare=True) for j in range(k)]
            elif p == "compress_minmax":
                calls = [bg.bagua_compress_minmax_u8_batched(self.bucket[j], self.delta[j], C, self.codes[j], self.minmax[j],
                                                             self.bws, prepare=True) for j in range(k)]
            elif p == "sign_compress":
                calls = [bg.bagua_sign_compress_ef_batched(self.bucket[j], self.sdelta[j], SC, self.bits[j], self.scale[j],
                                                           self.bws, prepare=True) for j in range(k)]
            elif p == "drr_minmax":
                calls = [bg.bagua_decompress_reduce_recompress_batched(
                    bg.CODEC_MINMAX_U8, [[self.codes[j][u] for j in range(k)] for u in range(U)],
                    [[self.minmax[j][u] for j in range(k)] for u in range(U)], self.eps, self.unit_n, C, self.codes_out,
                    self.minmax_out, self.out, self.bws_k, prepare=True)]
            else:
                calls = [bg.bagua_decompress_reduce_recompress_batched(
                    bg.CODEC_SIGN1, [[self.bits[j][u] for j in range(k)] for u in range(U)],
                    [[self.scale[j][u] for j in range(k)] for u in range(U)], self.seps, self.unit_n, SC, self.bits_out,
                    self.scale_out, self.sout, self.bws_k, prepare=True)]
            self._prepared[key] = calls
        for call in self._prepared[key]:
            call()


GIB = 1 << 30


class Counts:
    """Word-for-word comparison of HIP outputs with oracle outputs: integer words must be equal; fp32 words are
    counted twice: not bit-identical, and outside 1e-6 relative + 1e-7 absolute."""

    def __init__(self):
        self.c = {"int_words": 0, "int_mismatch": 0, "fp32_words": 0, "fp32_not_bit_exact": 0, "fp32_out_of_tolerance": 0}

    def ints(self, t, ref):
        import numpy as np
        a = t.cpu().numpy().view(ref.dtype).reshape(-1)
        self.c["int_words"] += a.size
        self.c["int_mismatch"] += int(np.count_nonzero(a != ref.reshape(-1)))

    def floats(self, t, ref):
        import numpy as np
        a = t.cpu().numpy().reshape(-1)
        ref = ref.reshape(-1)
        self.c["fp32_words"] += a.size
        nb = int(np.count_nonzero(a.view(np.uint32) != ref.view(np.uint32)))
        self.c["fp32_not_bit_exact"] += nb
        if nb:
            err = np.abs(a.astype(np.float64) - ref.astype(np.float64))
            self.c["fp32_out_of_tolerance"] += int(np.count_nonzero(~(err <= 1e-6 * np.abs(ref.astype(np.float64)) + 1e-7)))

    def add(self, other):
        for k_ in self.c:
            self.c[k_] += other.c[k_]

    def clean(self):
        return self.c["int_mismatch"] == 0 and self.c["fp32_not_bit_exact"] == 0


def c_lp_s_sample(torch, bg, oracle, xs, C, SC, want_minmax, want_sign, cnt, layers=None):
    """Oracle and HIP path on one sample (k flat buckets xs, zero initial error states): MinMax C_LP_S (worker + server)
    and / or sign C_LP_S.  layers = (per-worker tensor lists, offsets): the buckets are first assembled by the flatten on
    both sides.  Returns the oracle's wall time; comparison counts go to cnt."""
    import numpy as np
    k = len(xs)
    n = xs[0].numel()
    dev = xs[0].device
    nc, ncs = (n + C - 1) // C, (n + SC - 1) // SC
    f32 = dict(dtype=torch.float32, device=dev)
    xh = [x.cpu().numpy() for x in xs]
    dt = 0.0
    if layers is not None:
        per_worker, offs = layers
        lay_h = [[t.cpu().numpy() for t in per_worker[j]] for j in range(k)]
        t0 = time.perf_counter()
        flats = [oracle.bucket_flatten(lay_h[j], offs, n) for j in range(k)]
        dt += time.perf_counter() - t0
        ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(offs), n), dtype=torch.uint8, device=dev)
        for j in range(k):
            got = torch.full((n,), float("nan"), **f32)
            bg.bagua_bucket_flatten(per_worker[j], offs, got, ws)
            cnt.ints(got.view(torch.int32), flats[j].view(np.int32))     # a copy: compared as words
            cnt.ints(xs[j].view(torch.int32), flats[j].view(np.int32))   # the resident bucket the timed flatten wrote
        xh = flats
    if want_minmax:
        d_o = [np.zeros(n, np.float32) for _ in range(k)]
        eps_o = np.zeros(n, np.float32)
        t0 = time.perf_counter()
        enc = [oracle.compress_minmax_u8(xh[j], d_o[j], C) for j in range(k)]
        drr = oracle.drr_minmax_u8([e[0] for e in enc], [e[1] for e in enc], eps_o, C)
        dt += time.perf_counter() - t0
        codes = [torch.empty(n, dtype=torch.uint8, device=dev) for _ in range(k)]
        mm = [torch.empty(2 * nc, **f32) for _ in range(k)]
        delta = [torch.zeros(n, **f32) for _ in range(k)]
        for j in range(k):
            bg.bagua_compress_minmax_u8(xs[j], delta[j], C, codes[j], mm[j])
        eps = torch.zeros(n, **f32)
        c2, m2, o2 = torch.empty(n, dtype=torch.uint8, device=dev), torch.empty(2 * nc, **f32), torch.empty(n, **f32)
        bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, codes, mm, eps, n, C, c2, m2, o2)
        for j in range(k):
            cnt.ints(codes[j], enc[j][0]); cnt.floats(mm[j], enc[j][1]); cnt.floats(delta[j], d_o[j])
        cnt.ints(c2, drr[0]); cnt.floats(m2, drr[1]); cnt.floats(o2, drr[2]); cnt.floats(eps, eps_o)
        del codes, mm, delta, eps, c2, m2, o2, enc, drr, d_o
    if want_sign:
        sd_o = [np.zeros(n, np.float32) for _ in range(k)]
        seps_o = np.zeros(n, np.float32)
        t0 = time.perf_counter()
        senc = [oracle.sign_compress_ef(xh[j], sd_o[j], SC) for j in range(k)]
        sdrr = oracle.drr_sign([e[0] for e in senc], [e[1] for e in senc], seps_o, n, SC)
        dt += time.perf_counter() - t0
        bits = [torch.empty((n + 31) // 32, dtype=torch.int32, device=dev) for _ in range(k)]
        scale = [torch.empty(ncs, **f32) for _ in range(k)]
        sdelta = [torch.zeros(n, **f32) for _ in range(k)]
        for j in range(k):
            bg.bagua_sign_compress_ef(xs[j], sdelta[j], SC, bits[j], scale[j])
        seps = torch.zeros(n, **f32)
        b2, s2, so2 = torch.empty((n + 31) // 32, dtype=torch.int32, device=dev), torch.empty(ncs, **f32), torch.empty(n, **f32)
        bg.bagua_decompress_reduce_recompress(bg.CODEC_SIGN1, bits, scale, seps, n, SC, b2, s2, so2)
        for j in range(k):
            cnt.ints(bits[j], senc[j][0]); cnt.floats(scale[j], senc[j][1]); cnt.floats(sdelta[j], sd_o[j])
        cnt.ints(b2, sdrr[0]); cnt.floats(s2, sdrr[1]); cnt.floats(so2, sdrr[2]); cnt.floats(seps, seps_o)
    return dt


def ring_sample(torch, bg, oracle, reps, hats, C, want_fp, want_lp, cnt):
    """One ring round in full and / or low precision on k replica slices, oracle and HIP path; returns oracle time."""
    import numpy as np
    k, n = len(reps), reps[0].numel()
    dev = reps[0].device
    nc = (n + C - 1) // C
    rh = [r.cpu().numpy() for r in reps]
    dt = 0.0
    if want_fp:
        t0 = time.perf_counter()
        ref = oracle.ring_avg_fp(rh)
        dt += time.perf_counter() - t0
        outs = [torch.empty(n, device=dev) for _ in range(k)]
        bg.bagua_decentralized_avg(bg.AVG_FP, reps, outs)
        for i in range(k):
            cnt.floats(outs[i], ref[i])
        del outs, ref
    if want_lp:
        hh = [h.cpu().numpy().copy() for h in hats]
        t0 = time.perf_counter()
        ro, rc, rm = oracle.ring_avg_lp(rh, hh, C)
        dt += time.perf_counter() - t0
        hg = [h.clone() for h in hats]
        outs = [torch.empty(n, device=dev) for _ in range(k)]
        codes = [torch.empty(n, dtype=torch.uint8, device=dev) for _ in range(k)]
        mm = [torch.empty(2 * nc, device=dev) for _ in range(k)]
        bg.bagua_decentralized_avg(bg.AVG_LP_MINMAX_U8, reps, outs, hg, codes, mm, C)
        for i in range(k):
            cnt.floats(outs[i], ro[i]); cnt.ints(codes[i], rc[i]); cnt.floats(mm[i], rm[i]); cnt.floats(hg[i], hh[i])
    return dt


def cpu_baseline(wl, torch):
    """The oracle, as it stands, on the host cores, on a bounded sample of the block's own resident inputs (at least
    1 GiB of fp32 input where the block is that large), and the HIP path compared with the oracle's outputs on that
    same sample (every primitive of the block, zero initial error states).  Flat layout only."""
    import oracle
    bg = wl.bg
    threads = max(1, min(16, oracle.max_threads(), os.cpu_count() or 1))
    oracle.set_threads(threads)
    k, C, SC = wl.k, wl.C, wl.SC
    cnt = Counts()
    has = lambda *ps: any(p in wl.prims for p in ps)
    dt, elems, nprims, what = 0.0, 0, 0, ""
    if has("flatten", "compress_minmax", "drr_minmax", "sign_compress", "drr_sign"):
        if wl.buckets:      # whole buckets from the front until the sample holds >= 1 GiB of input (or everything)
            nb = 0
            while nb < len(wl.buckets) and 4 * k * wl.bases[nb] < GIB:
                nb += 1
            m = wl.bases[nb]
            what = "the first %d of %d buckets" % (nb, len(wl.buckets))
        else:
            m = min(wl.n_elems, -(-GIB // (4 * k)) // SC * SC)
            what = "the first %d elements of every worker" % m
        xs = [wl.bucket[j][0][:m] for j in range(k)]
        layers = None
        if has("flatten"):
            ids = [t for bk in wl.buckets[:nb] for t in bk.tensors]
            offs = [wl.bases[b] + o for b, bk in enumerate(wl.buckets[:nb]) for o in bk.offsets]
            # the resident buckets hold what the LAST timed flatten wrote: gradient set (step_no - 1) % sets
            it = (wl.step_no - 1) % wl.sets
            layers = ([[wl.layers[it][j][t] for t in ids] for j in range(k)], offs)
        mm_p, sg_p = has("compress_minmax", "drr_minmax"), has("sign_compress", "drr_sign")
        dt += c_lp_s_sample(torch, bg, oracle, xs, C, SC, mm_p, sg_p, cnt, layers)
        nprims += (1 if layers else 0) + (2 if mm_p else 0) + (2 if sg_p else 0)
        elems = m
    if has("ring_fp", "ring_lp"):
        m = min(wl.n_elems, -(-GIB // (4 * k)) // C * C)
        src = wl.step_no % 2
        which = wl.rep_fp if has("ring_fp") else wl.rep_lp
        reps = [which[src][i][0][:m] for i in range(k)]
        hats = [wl.xhat[i][0][:m] for i in range(k)] if has("ring_lp") else None
        dt += ring_sample(torch, bg, oracle, reps, hats, C, has("ring_fp"), has("ring_lp"), cnt)
        nprims += int(has("ring_fp")) + int(has("ring_lp"))
        what = (what + "; " if what else "") + "the first %d elements of every replica" % m
        elems = max(elems, m)
    torch.cuda.synchronize()
    grad_bytes = 4.0 * elems * k * nprims
    base = {"value": round(grad_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "seconds": round(dt, 4), "gradient_bytes": grad_bytes,
            "sample": "%s (%d elements x %d workers, %.2f GiB of fp32 input), %d primitives, %.1f s on %d threads" %
                      (what, elems, k, 4.0 * elems * k / GIB, nprims, dt, threads)}
    par = dict(cnt.c)
    par["sample"] = "every primitive of the block on " + what + ", HIP path against the oracle"
    return base, par


def time_fn(torch, fn, reps):
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for i in range(3):
        fn(i)
    ev[0].record()
    for i in range(reps):
        fn(i + 3)
    ev[1].record()
    torch.cuda.synchronize()
    return ev[0].elapsed_time(ev[1]) * 1e-3 / reps


def ceilings(torch, bg):
    """What the memory system of this GPU delivers for plain access patterns, GB/s: a 128-bit copy
    (bagua_bucket_flatten_run with one tensor covering the bucket), a read-only reduction, and stream mixes of the
    ring kernels' traffic shape (one wave per row: 8 reads + 8 writes; the 2 reads + 2 writes + 1 byte stream of one
    ring-LP peer; the same for 8 peers one after another in every wave), the mixes with their 32 buffers back to back
    ("packed") and scattered over a SPREAD_GIB reservation ("spread", see Placer)."""
    n = 128 * 1024 * 1024
    bufs = [(torch.zeros(n, device="cuda"), torch.empty(n, device="cuda")) for _ in range(2)]   # 2 GiB rotated
    plans = []
    for src, dst in bufs:
        ws = torch.empty(bg.bagua_flatten_workspace_bytes(1, n), dtype=torch.uint8, device="cuda")
        bg.bagua_flatten_plan([src], [0], n, ws)
        plans.append(ws)
    out = {}
    t = time_fn(torch, lambda i: bg.bagua_bucket_flatten_run(plans[i % 2], 1, bufs[i % 2][1]), 20)
    out["copy_kernel_GBps"] = round(8.0 * n / t / 1e9, 1)
    sums = torch.empty(n // 4096, device="cuda")
    t = time_fn(torch, lambda i: bg.bagua_probe_read(bufs[i % 2][i % 2], sums), 20)
    out["read_kernel_GBps"] = round(4.0 * n / t / 1e9, 1)
    # the worker-side kernels' traffic without their arithmetic or their barrier: x and the error state read, the error
    # state written in place, one byte stream written (13 B per element; the sign codec writes 1/8 B instead of 1)
    codes = torch.empty(n, dtype=torch.uint8, device="cuda")
    t = time_fn(torch, lambda i: bg.bagua_probe_streams([bufs[i % 2][0], bufs[i % 2][1]], [bufs[i % 2][1]], [codes], 2, 1, 1, 1, n), 20)
    out["mix_2R1W1B_in_place_GBps"] = round(13.0 * n / t / 1e9, 1)
    del bufs, plans, codes
    m = 32 * 1024 * 1024          # 8 peers x (x, xhat, out fp32 + codes u8) = 3.6 GB per launch
    for tag in ("packed", "spread"):
        pl = Placer(torch, SPREAD_GIB, 7, 3.0) if tag == "spread" else None
        put = (lambda t: pl.place(t)) if pl else (lambda t: t)
        x = [put(torch.zeros(m, device="cuda")) for _ in range(8)]
        h = [put(torch.zeros(m, device="cuda")) for _ in range(8)]
        o = [put(torch.zeros(m, device="cuda")) for _ in range(8)]
        c = [put(torch.zeros(m, dtype=torch.uint8, device="cuda")) for _ in range(8)]
        t = time_fn(torch, lambda i: bg.bagua_probe_streams(x, o, [], 8, 8, 0, 1, m), 10)
        out["mix_8R8W_%s_GBps" % tag] = round(64.0 * m / t / 1e9, 1)

        def one_peer_at_a_time(i):
            for p in range(8):
                bg.bagua_probe_streams([x[p], h[p]], [h[p], o[p]], [c[p]], 2, 2, 1, 1, m)
        t = time_fn(torch, one_peer_at_a_time, 10)
        out["mix_2R2W1B_one_peer_per_wave_%s_GBps" % tag] = round(17.0 * 8 * m / t / 1e9, 1)
        ins = [t_ for p in range(8) for t_ in (x[p], h[p])]
        outs = [t_ for p in range(8) for t_ in (h[p], o[p])]
        t = time_fn(torch, lambda i: bg.bagua_probe_streams(ins, outs, c, 2, 2, 1, 8, m), 10)
        out["mix_2R2W1B_eight_peers_per_wave_%s_GBps" % tag] = round(17.0 * 8 * m / t / 1e9, 1)
        del x, h, o, c, ins, outs, pl
        torch.cuda.empty_cache()
    return out


def read_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary of this workload, if there is
    one: profiles/traffic_<workload>.txt, lines `traffic_bytes_per_launch <kernel> <bytes>`."""
    path = os.path.join(ROOT, "profiles", "traffic_%s.txt" % workload)
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel:
                return float(f[2])
    except OSError:
        pass
    return None


def source_hash():
    """sha256 (16 hex digits) over the library's sources: which code the loaded .so was checked against by ensure_built."""
    import glob
    import hashlib
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "paper_2107_01499_amd", "csrc", "*")) + glob.glob(os.path.join(ROOT, "include", "*.h")))
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def run_block(torch, bg, args, name, layout, only, extras):
    """Build one workload, time --warmup + --steps steps of it, then (flat layout) the oracle sample and parity."""
    wl = Workload(torch, bg, name, layout=layout, only=only, fused=args.fused_flatten, extras=extras,
                  placement=getattr(args, "placement", None))
    prims = wl.prims
    for _ in range(args.warmup):
        wl.step()
    torch.cuda.synchronize()
    all_marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        marks = []
        wl.step(marks)
        all_marks.append(marks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # per-primitive GPU time from the events recorded on the launch stream inside the timed region
    prim_ms = {p: 0.0 for p in prims}
    for marks in all_marks:
        for (_, e0), (pname, e1) in zip(marks[:-1], marks[1:]):
            prim_ms[pname] += e0.elapsed_time(e1)
    gpu_ms = sum(m[0][1].elapsed_time(m[-1][1]) for m in all_marks)
    for p in prims:
        prim_ms[p] /= args.steps
    gb, ab, nl = wl.grad_bytes(), wl.algo_bytes(), wl.launches()
    per_prim = {}
    for p in prims:
        t = prim_ms[p] * 1e-3
        per_prim[p] = {"ms": round(prim_ms[p], 4), "launches": nl[p], "gradient_GBps": round(gb[p] / t / 1e9, 1),
                       "hbm_GBps": round(ab[p] / t / 1e9, 1), "frac_of_peak": round(ab[p] / t / 1e9 / HBM_PEAK_GBS, 4),
                       "kernel": wl.kernel_name(p), "gradient_bytes": gb[p], "algorithmic_bytes": ab[p]}
        if p in ("drr_minmax", "drr_sign", "drr_topk"):
            per_prim[p]["note"] = ("gradient_GBps counts the 4*k*n bytes of fp32 gradient the k compressed inputs "
                                   "represent, not bytes moved; hbm_GBps is the bandwidth figure")
    dom = max(prims, key=lambda p: prim_ms[p])
    dom_t = prim_ms[dom] * 1e-3 / nl[dom]
    achieved = ab[dom] / nl[dom] / dom_t / 1e9
    traffic = read_traffic(name, wl.kernel_name(dom)) if layout == "flat" else None
    roof = {"bound": "hbm", "kernel": wl.kernel_name(dom), "primitive": dom, "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
            "avg_launch_us": round(dom_t * 1e6, 3), "algorithmic_bytes_per_launch": ab[dom] / nl[dom]}
    if traffic is not None:
        roof["traffic_source"] = ("profiles/traffic_%s.txt: rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this "
                                  "workload, scaled by what the same counters read for k_flatten (a copy of known size)" % name)
    launch = {"flat": "one launch per worker over all its buckets (contiguous)", "per_bucket": "one launch per bucket",
              "buckets": "separately allocated buckets, one batched launch per worker"}[layout]
    block = {"workload": "%s; %d buckets, %d padded elements per worker, %d simulated workers, chunk %d (sign codec %d); "
                         "primitives per step: %s" % (wl.w["label"], len(wl.units) if layout != "flat" else max(1, len(wl.buckets)),
                                                      wl.n_elems, wl.k, wl.C, wl.SC, ", ".join(prims)),
             "launch": launch, "placement": wl.placement_note(), "ms_per_step": round(wall * 1e3 / args.steps, 4), "gpu_ms_per_step": round(gpu_ms / args.steps, 4),
             "per_primitive": per_prim, "roofline": roof}
    if name == "single_bucket_x32":
        block["single_instance_latency_us"] = single_instance_latency(torch, bg, wl)      # three ways of launching it
    if not args.no_cpu_baseline and layout == "flat" and only is None and not args.fused_flatten and not extras:
        block["cpu_baseline"], block["parity"] = cpu_baseline(wl, torch)
    if "flatten" in prims and layout == "flat" and only is None:      # last: it overwrites the resident buckets
        block["flatten_misaligned"] = misaligned_flatten(torch, bg, wl)
    if layout == "flat" and only is None and not extras and not args.fused_flatten:      # very last: overwrites error states
        probe = same_traffic_probe(torch, bg, wl, dom)
        if probe is not None:
            probe["kernel_vs_probe"] = round(achieved / probe["GBps"], 4)
            roof["same_traffic_probe"] = probe
    del wl
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    return block, wall / args.steps


def same_traffic_probe(torch, bg, wl, dom, reps=3):
    """What the memory system delivers for the dominant kernel's traffic shape on the block's OWN resident buffers, at
    their full size: bagua_probe_streams (one row per wave, loads then stores, no arithmetic, no barrier) over the same
    arrays the kernel streams.  Run last: it overwrites them.  None for shapes the probe does not have."""
    k, U = wl.k, len(wl.units)
    ns = [wl.units[u][1] for u in range(U)]
    if any(m % 256 for m in ns):
        return None
    if dom == "compress_minmax":
        def once(i):
            for j in range(k):
                for u in range(U):
                    bg.bagua_probe_streams([wl.bucket[j][u], wl.delta[j][u]], [wl.delta[j][u]], [wl.codes[j][u]], 2, 1, 1, 1, ns[u])
        bpe, what = 13.0, "x and the error state read, the error state written in place, one byte per element written"
    elif dom == "sign_compress":
        def once(i):
            for j in range(k):
                for u in range(U):
                    bg.bagua_probe_streams([wl.bucket[j][u], wl.sdelta[j][u]], [wl.sdelta[j][u]], [], 2, 1, 0, 1, ns[u])
        bpe, what = 12.0, "x and the error state read, the error state written in place (the kernel's 1/8 B of sign bits left out)"
    elif dom == "ring_lp" and k == 8:
        def once(i):
            for u in range(U):
                ins = [t for p_ in range(k) for t in (wl.rep_lp[0][p_][u], wl.xhat[p_][u])]
                outs = [t for p_ in range(k) for t in (wl.xhat[p_][u], wl.rep_lp[1][p_][u])]
                bg.bagua_probe_streams(ins, outs, [wl.lp_codes[p_][u] for p_ in range(k)], 2, 2, 1, k, ns[u])
        bpe, what = 17.0, "per peer x and the public replica read, the public replica and the new x written, one byte per element written; the 8 peers one after another in every wave"
    elif dom == "ring_fp" and k == 8:
        def once(i):
            for u in range(U):
                bg.bagua_probe_streams([wl.rep_fp[0][p_][u] for p_ in range(k)], [wl.rep_fp[1][p_][u] for p_ in range(k)], [], 8, 8, 0, 1, ns[u])
        bpe, what = 8.0, "8 replicas read, 8 written"
    else:
        return None
    t = time_fn(torch, once, reps)
    rate = bpe * wl.n_elems * k / t / 1e9
    return {"GBps": round(rate, 1), "frac_of_peak": round(rate / HBM_PEAK_GBS, 4), "bytes_per_element": bpe, "streams": what,
            "note": "bagua_probe_streams on this block's own buffers at full size, same launches per step as the kernel; "
                    "the `ceilings` block measures the same probes on 0.1-0.5 GiB buffers"}


def misaligned_flatten(torch, bg, wl, reps=5):
    """The flatten of the block's layout with every layer tensor at a source address that is only 4-byte aligned (one
    element past its 16-byte aligned place), so the copy cannot pair 128-bit loads with 128-bit stores directly.  Same
    launches as the timed flatten.  Returns the per_primitive-style entry."""
    k, U = wl.k, len(wl.units)
    starts, pos = [], 1
    for sz in wl.sizes:
        starts.append(pos)
        pos += (sz + 3) // 4 * 4 + 4            # next tensor again at 16-byte boundary + 4 bytes
    plans = []
    for j in range(k):                           # every worker reads its own tensors, as in the timed flatten
        arena = torch.zeros(pos + 8, device="cuda")
        srcs = [arena[starts[t]:starts[t] + sz] for t, sz in enumerate(wl.sizes)]
        per_unit = []
        for u, (lo, ln, ids, offs) in enumerate(wl.units):
            ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(ids), ln), dtype=torch.uint8, device="cuda")
            bg.bagua_flatten_plan([srcs[t] for t in ids], offs, ln, ws)
            per_unit.append((ws, arena))
        plans.append(per_unit)

    def once(i):
        for j in range(k):
            for u in range(U):
                bg.bagua_bucket_flatten_run(plans[j][u][0], len(wl.units[u][2]), wl.bucket[j][u])
    t = time_fn(torch, once, reps)
    ab = 8.0 * wl.n_elems * k
    return {"ms": round(t * 1e3, 4), "launches": U * k, "hbm_GBps": round(ab / t / 1e9, 1),
            "frac_of_peak": round(ab / t / 1e9 / HBM_PEAK_GBS, 4), "kernel": "k_flatten", "algorithmic_bytes": ab,
            "note": "every source tensor 4 bytes past a 16-byte boundary; timed after the step, not part of value"}


def single_instance_latency(torch, bg, wl):
    """configs[0] as it stands (one 1,048,576-element bucket, 4 workers): 4 compress launches + the server step, data
    resident in the caches; microseconds per pass, launch gaps included: launched call by call, with the compressions
    batched into one launch, and as a HIP graph."""
    n, k, C = 1048576, wl.k, wl.C
    nc = n // C
    xs = [wl.bucket[j][0][:n] for j in range(k)]
    delta = [torch.zeros(n, device="cuda") for _ in range(k)]
    codes = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(k)]
    mm = [torch.empty(2 * nc, device="cuda") for _ in range(k)]
    eps, out = torch.zeros(n, device="cuda"), torch.empty(n, device="cuda")
    c2, m2 = torch.empty(n, dtype=torch.uint8, device="cuda"), torch.empty(2 * nc, device="cuda")

    def once(i):
        for j in range(k):
            bg.bagua_compress_minmax_u8(xs[j], delta[j], C, codes[j], mm[j])
        bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, codes, mm, eps, n, C, c2, m2, out)
    res = {"launch_per_worker": round(time_fn(torch, once, 50) * 1e6, 2)}

    # the k workers' compressions as ONE batched launch (plus the launch that writes its bucket table)
    ws = torch.empty(bg.bagua_batch_workspace_bytes(k, 0), dtype=torch.uint8, device="cuda")

    batched = bg.bagua_compress_minmax_u8_batched(xs, delta, C, codes, mm, ws, prepare=True)

    def once_batched(i):
        batched()
        bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, codes, mm, eps, n, C, c2, m2, out)
    res["batched_compress"] = round(time_fn(torch, once_batched, 50) * 1e6, 2)

    # the per-worker launches recorded into a HIP graph: one graph launch per pass
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        once(0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        once(0)
    res["hip_graph_of_the_per_worker_launches"] = round(time_fn(torch, lambda i: g.replay(), 50) * 1e6, 2)
    del g
    return res


def _verify_setup():
    import oracle
    oracle.set_threads(max(1, min(16, oracle.max_threads(), os.cpu_count() or 1)))
    return oracle


def _say(msg):
    print("verify-all: " + msg, file=sys.stderr, flush=True)


def verify_config2(torch, bg):
    """configs[2] at full size: flatten, compress, server step from zero error states; every bucket of every worker
    against the oracle.  Returns the comparison counts (stops at the first bucket that differs)."""
    import numpy as np
    oracle = _verify_setup()
    wl = Workload(torch, bg, "bert_large")
    wl.step()
    torch.cuda.synchronize()
    k, C = wl.k, wl.C
    cnt = Counts()
    for b, bk in enumerate(wl.buckets):
        lo, hi = wl.bases[b], wl.bases[b + 1]
        enc = []
        for j in range(k):
            lay = [wl.layers[0][j][t].cpu().numpy() for t in bk.tensors]
            f = oracle.bucket_flatten(lay, list(bk.offsets), bk.n_pad)
            cnt.ints(wl.bucket[j][0][lo:hi].view(torch.int32), f.view(np.int32))
            d = np.zeros(bk.n_pad, np.float32)
            c, m = oracle.compress_minmax_u8(f, d, C)
            cnt.ints(wl.codes[j][0][lo:hi], c)
            cnt.floats(wl.minmax[j][0][2 * lo // C:2 * hi // C], m)
            cnt.floats(wl.delta[j][0][lo:hi], d)
            enc.append((c, m))
        e = np.zeros(bk.n_pad, np.float32)
        c2, m2, o2 = oracle.drr_minmax_u8([x[0] for x in enc], [x[1] for x in enc], e, C)
        cnt.ints(wl.codes_out[0][lo:hi], c2)
        cnt.floats(wl.minmax_out[0][2 * lo // C:2 * hi // C], m2)
        cnt.floats(wl.out[0][lo:hi], o2)
        cnt.floats(wl.eps[0][lo:hi], e)
        _say("configs[2] bucket %d/%d (%d elements x %d workers) %s" %
             (b + 1, len(wl.buckets), bk.n_pad, k, "ok" if cnt.clean() else "MISMATCH"))
        if not cnt.clean():
            break
    del wl
    torch.cuda.empty_cache()
    return cnt


def verify_config3(torch, bg, rounds=5):
    """configs[3] at full size: `rounds` ring rounds in full and in low precision, the oracle's state carried on the
    host from round to round; every output of every round compared."""
    oracle = _verify_setup()
    wl = Workload(torch, bg, "bert_base_ring")
    k, C, n = wl.k, wl.C, wl.n_elems
    cnt = Counts()
    x_fp = [wl.rep_fp[0][i][0].cpu().numpy() for i in range(k)]
    x_lp = [wl.rep_lp[0][i][0].cpu().numpy() for i in range(k)]
    hat = [wl.xhat[i][0].cpu().numpy().copy() for i in range(k)]
    for rnd in range(rounds):
        dst = (wl.step_no + 1) % 2
        wl.step()
        torch.cuda.synchronize()
        x_fp = oracle.ring_avg_fp(x_fp)
        x_lp, codes, mm = oracle.ring_avg_lp(x_lp, hat, C)
        for i in range(k):
            cnt.floats(wl.rep_fp[dst][i][0], x_fp[i])
            cnt.floats(wl.rep_lp[dst][i][0], x_lp[i])
            cnt.floats(wl.xhat[i][0], hat[i])
            cnt.ints(wl.lp_codes[i][0], codes[i])
            cnt.floats(wl.lp_minmax[i][0], mm[i])
        _say("configs[3] round %d/%d (%d elements x %d peers, FP and LP) %s" %
             (rnd + 1, rounds, n, k, "ok" if cnt.clean() else "MISMATCH"))
        if not cnt.clean():
            break
    del wl
    torch.cuda.empty_cache()
    return cnt


def verify_config4(torch, bg):
    """configs[4] at full size: sign compression of every worker and the server step from zero error states, the
    oracle streamed over spans of 64 Mi elements."""
    import numpy as np
    oracle = _verify_setup()
    wl = Workload(torch, bg, "onebit")
    wl.step()
    torch.cuda.synchronize()
    k, SC, n = wl.k, wl.SC, wl.n_elems
    cnt = Counts()
    span = 64 * 1024 * 1024
    for lo in range(0, n, span):
        hi = min(n, lo + span)
        m = hi - lo
        enc = []
        for j in range(k):
            x = wl.bucket[j][0][lo:hi].cpu().numpy()
            d = np.zeros(m, np.float32)
            bts, sc = oracle.sign_compress_ef(x, d, SC)
            cnt.ints(wl.bits[j][0][lo // 32:(hi + 31) // 32], bts)
            cnt.floats(wl.scale[j][0][lo // SC:(hi + SC - 1) // SC], sc)
            cnt.floats(wl.sdelta[j][0][lo:hi], d)
            enc.append((bts, sc))
        e = np.zeros(m, np.float32)
        b2, s2, o2 = oracle.drr_sign([x[0] for x in enc], [x[1] for x in enc], e, m, SC)
        cnt.ints(wl.bits_out[0][lo // 32:(hi + 31) // 32], b2)
        cnt.floats(wl.scale_out[0][lo // SC:(hi + SC - 1) // SC], s2)
        cnt.floats(wl.sout[0][lo:hi], o2)
        cnt.floats(wl.seps[0][lo:hi], e)
        _say("configs[4] elements [%d, %d) x %d workers %s" % (lo, hi, k, "ok" if cnt.clean() else "MISMATCH"))
        if not cnt.clean():
            break
    del wl
    torch.cuda.empty_cache()
    return cnt


def verify_all(torch, bg):
    """Every element of configs[2], configs[3] (5 rounds, full and low precision) and configs[4]: the HIP path at full
    size in the launch configuration the benchmark times, against the oracle streamed over the same bits.  Stops at
    the first configuration that differs.  Prints one JSON line with the three counts per configuration."""
    report, ok = {}, True
    for name, fn in (("configs[2]", verify_config2), ("configs[3]", verify_config3), ("configs[4]", verify_config4)):
        t0 = time.perf_counter()
        cnt = fn(torch, bg)
        report[name] = dict(cnt.c, seconds=round(time.perf_counter() - t0, 1))
        _say("%s %s" % (name, report[name]))
        ok = cnt.clean()
        if not ok:
            break
    report["all_equal"] = bool(ok)
    print(json.dumps({"verify_all": report}))
    return 0 if ok else 1


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build is the single-GPU share of the path (the k workers are k buffers in one GPU's "
              "HBM); --gpus %d is not supported, run with --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import __graft_entry__
    __graft_entry__.ensure_built()        # uses what is built; rebuilds a library that is older than its sources
    import paper_2107_01499_amd as bg     # fails loudly if the HIP library cannot be loaded
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.verify_all:
        sys.exit(verify_all(torch, bg))
    only = set(p for p in args.only.split(",") if p) or None
    extras = tuple(e for e in args.extras.split(",") if e)
    layout = "per_bucket" if args.per_bucket_launch else args.layout
    ceil = ceilings(torch, bg)
    plan = DEFAULT_PLAN if args.workload == "all" else [(args.workload, layout, True)]
    blocks, primary_s = {}, 0.0
    for name, lay, primary in plan:
        key = name if lay == "flat" else "%s_%s" % (name, lay)
        print("bench: block %s" % key, file=sys.stderr, flush=True)
        blocks[key], step_s = run_block(torch, bg, args, name, lay, only, extras)
        blocks[key]["counts_towards_value"] = primary
        if primary:
            primary_s += step_s

    # the seven primitives, each at the largest configuration that names it (the blocks that count towards `value`)
    per_prim, total_grad = {}, 0.0
    for key, b in blocks.items():
        if not b["counts_towards_value"]:
            continue
        for p, v in b["per_primitive"].items():
            e = dict(v)
            e["config"] = key
            e["frac_of_copy_kernel"] = round(v["hbm_GBps"] / ceil["copy_kernel_GBps"], 4)
            per_prim[p] = e
            total_grad += v["gradient_bytes"]
        if "flatten_misaligned" in b:
            e = dict(b["flatten_misaligned"])
            e["config"] = key
            per_prim["flatten_misaligned"] = e
    dom_key = max((k_ for k_ in blocks if blocks[k_]["counts_towards_value"]),
                  key=lambda k_: blocks[k_]["per_primitive"][blocks[k_]["roofline"]["primitive"]]["ms"])
    roof = dict(blocks[dom_key]["roofline"])
    roof["config"] = dom_key
    result = {
        "metric": "gradient GB/s processed per primitive on 1 MI355X; % of HBM roofline",
        "value": round(total_grad / primary_s / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(primary_s * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "; ".join("%s [%s]" % (blocks[k_]["workload"], blocks[k_]["launch"])
                                         for k_ in blocks if blocks[k_]["counts_towards_value"]),
                   "also_timed": [k_ for k_ in blocks if not blocks[k_]["counts_towards_value"]],
                   "step": "one pass of every listed primitive over its configuration's batch; ms_per_step and value "
                           "sum the blocks that count towards the value"},
        "per_primitive": per_prim,
        "roofline": roof,
        "roofline_per_config": {k_: b["roofline"] for k_, b in blocks.items()},
        "ceilings": ceil,
        "copy_kernel_GBps": ceil["copy_kernel_GBps"],
        "read_kernel_GBps": ceil["read_kernel_GBps"],
        "blocks": blocks,
        "library": {"path": os.path.relpath(bg.binding.LIB_PATH, ROOT), "source_sha16": source_hash()},
    }
    base = [(k_, b["cpu_baseline"]) for k_, b in blocks.items() if "cpu_baseline" in b]
    if base:
        main_base = [(k_, c) for k_, c in base if blocks[k_]["counts_towards_value"]] or base
        secs = sum(c["seconds"] for _, c in main_base)
        result["cpu_baseline"] = {
            "value": round(sum(c["gradient_bytes"] for _, c in main_base) / secs / 1e9, 3), "unit": "GB/s",
            "cores": main_base[0][1]["cores"], "kind": "oracle",
            "sample": " | ".join("%s: %s" % (k_, c["sample"]) for k_, c in main_base),
            "per_config": {k_: {"value": c["value"], "seconds": c["seconds"]} for k_, c in base}}
        total = Counts()
        for k_, b in blocks.items():
            if "parity" in b:
                for f in total.c:
                    total.c[f] += b["parity"][f]
        par = dict(total.c)
        par["sample"] = "every primitive of every block on its oracle sample (see blocks[*].parity), HIP path against the oracle"
        result["parity"] = par
    print(json.dumps(result))


if __name__ == "__main__":
    main()
