#!/usr/bin/env python3
"""Benchmark of the compression hot path on one MI355X.

Default workload (the one the headline metric is quoted on): ResNet-50-shaped gradients for 8 simulated
workers (8 sets of buffers in one GPU's HBM) in greedy 25 MiB buckets.  One "step" is one pass of the whole
hot path over one batch of gradients:

  flatten            per worker     layer tensors -> contiguous buckets
  compress_minmax    per worker     MinMax-u8 with the worker error state (delta)
  drr_minmax         once           decode + average the 8 workers + server error state (epsilon) + recompress
                                    + decode to fp32
  ring_fp            once           ring averaging of 8 replicas, full precision
  ring_lp            once           ring averaging with u8-compressed differences
  sign_compress      per worker     1-bit sign + per-chunk scale with error state
  drr_sign           once           the server step with the sign codec

A launch covers all buckets of one worker (they sit back to back in one flat allocation and every bucket is
padded to a multiple of k*chunk, so the result is bit-identical to bucket-by-bucket launches, which
--per-bucket-launch times instead).  Inputs are generated on the GPU before the timed region and stay
resident in HBM.  Prints ONE JSON line.  --workload selects the other benchmark configurations' shapes
(bert_large: k=16, C=8192, Student-t; bert_base_ring: 8 peers x 109.5M; onebit: 1.5e9 Laplace elements, C=2048),
each restricted to the primitives that configuration names.  --gpus N with N > 1 is refused.
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
                     label="configs[1]: ResNet-50-shaped gradients, 25,557,032 fp32 per worker"),
    "bert_large": dict(cfg=2, k=16, chunk=8192, sign_chunk=2048, dist="student_t3", sets=1,
                       prims=["flatten", "compress_minmax", "drr_minmax"],
                       label="configs[2]: BERT-large-shaped gradients, 335,141,888 fp32 per worker, Student-t(3)"),
    "bert_base_ring": dict(cfg=3, k=8, chunk=4096, sign_chunk=2048, dist="normal", sets=1, prims=["ring_fp", "ring_lp"],
                           label="configs[3]: 8 peers x BERT-base-shaped replicas (109,482,240 fp32), base + drift"),
    "onebit": dict(cfg=4, k=8, chunk=4096, sign_chunk=2048, dist="laplace", sets=1, prims=["sign_compress", "drr_sign"],
                   label="configs[4]: 1.5e9 fp32 per worker, Laplace(0,1e-3), 1-bit sign codec"),
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--only", default="", help="comma list of primitives to run in the step (profiling aid)")
    ap.add_argument("--extras", default="", help="comma list of additional primitives appended to the step: sgd_step "
                    "(decode of the server's codes fused into an SGD-momentum update of every worker's replica), "
                    "adam_step (the same decode fused into an Adam update), onebit_adam (compression stage of 1-bit Adam: momentum "
                    "sign compression on every worker and the decode + frozen-variance update), "
                    "lp_shares (D_LP_S on a ring as the k single-peer shares a sharded run would execute: encode, then apply + mix), "
                    "peer_fp / peer_lp (full- / low-precision averaging with one chosen peer per worker), reduce_compress (intra-node "
                    "stage of hierarchical C_LP_S: 4 local workers averaged uncompressed, leader compresses), topk (C_LP_S with "
                    "the per-chunk top-K codec, keep = chunk/32: worker side and server side)")
    ap.add_argument("--fused-flatten", action="store_true",
                    help="replace flatten + compress_minmax by the fused bagua_flatten_compress_minmax_u8")
    ap.add_argument("--per-bucket-launch", action="store_true",
                    help="one launch per 25 MiB bucket instead of one per worker covering all its buckets")
    return ap.parse_args()


class Workload:
    """Synthetic gradients / replicas of one benchmark configuration, all state resident on the GPU."""

    def __init__(self, torch, bg, name, per_bucket=False, only=None, fused=False, extras=()):
        from bagua_workloads import resnet50_shapes, bert_shapes, pack_buckets, draw, seed_for, layer_sigmas
        from bagua_workloads.shapes import numel
        from bagua_workloads.generators import SHARED
        self.torch, self.bg, self.name = torch, bg, name
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
            shapes = [("momentum", (1500000000,))]
            n = 1500000000
            self.buckets, self.bases = [], [0, n]
            self.units = [(0, n, [0], [0])]
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

        def views(t, div=1, mul=1):
            """Per-unit views of a flat tensor whose index is element_index * mul / div."""
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
        self.step_no = 0
        torch.cuda.synchronize()

    # ---- accounting --------------------------------------------------------------------------------
    def bytes_per_element(self):
        k, C, SC = self.k, self.C, self.SC
        keep = getattr(self, "keep", 0)
        wb = 4.0 if "sign_compress" in self.prims else 0.0   # the fused call also writes the bucket if it is needed later
        return {"flatten": 8.0, "flatten_compress": 13.0 + wb + 8.0 / C, "compress_minmax": 13.0 + 8.0 / C, "drr_minmax": k + 13.0 + 8.0 * (k + 1) / C,
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
                 "compress_topk": n * k, "drr_topk": n}
        bpe = self.bytes_per_element()
        return {p: bpe[p] * units[p] for p in self.prims}

    def launches(self):
        U, k = len(self.units), self.k
        per = {"flatten": U * k, "flatten_compress": U * k, "compress_minmax": U * k, "drr_minmax": U, "ring_fp": U, "ring_lp": U,
               "sign_compress": U * k, "drr_sign": U, "sgd_step": U * k, "adam_step": U * k, "momentum_sign": U * k, "adam_frozen_step": U * k, "peer_fp": U, "peer_lp": U, "lp_encode": U * k, "lp_apply_mix": U * k, "reduce_compress": U * (k // 4),
               "compress_topk": U * k, "drr_topk": U}
        return {p: per[p] for p in self.prims}

    def kernel_name(self, p):
        return {"flatten": "k_flatten", "flatten_compress": "k_flatten_compress_minmax<2,true,%s>" %
                ("true" if "sign_compress" in self.prims else "false"), "compress_minmax": "k_compress_minmax<2,true>",
                "drr_minmax": "k_drr_minmax<4,true,true>", "ring_fp": "k_ring_avg_fp<%d>" % self.k,
                "ring_lp": "k_ring_avg_lp<%d,2>" % self.k, "sign_compress": "k_sign_compress<2,true,false>",
                "drr_sign": "k_drr_sign<4,true,true>", "sgd_step": "k_decompress_sgd<0,true,false>",
                "adam_step": "k_decompress_adam<0,false,false>", "momentum_sign": "k_sign_compress<2,true,true>",
                "adam_frozen_step": "k_decompress_adam<1,true,false>",
                "peer_fp": "k_peer_avg_fp", "peer_lp": "k_peer_avg_lp<2>", "lp_encode": "k_lp_encode<2>", "lp_apply_mix": "k_lp_apply_mix<true,true,false>", "reduce_compress": "k_reduce_compress_minmax<2,true>",
                "compress_topk": "k_compress_topk<2,true>", "drr_topk": "k_drr_topk<2,true,true>"}[p]

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
            if p == "flatten":
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


def cpu_baseline(wl, torch):
    """The oracle, as it stands, on the host cores: one step of the default workload (every bucket, all workers,
    the same primitives), timed once.  Returns the cpu_baseline dict for the JSON line and, from the one-core leg's
    outputs, the parity report of the HIP path on the same bucket."""
    import numpy as np
    import oracle
    threads = max(1, min(16, oracle.max_threads(), os.cpu_count() or 1))
    oracle.set_threads(threads)
    k, C, SC = wl.k, wl.C, wl.SC
    dt = 0.0
    for b, bk in enumerate(wl.buckets):
        n, lo = bk.n_pad, wl.bases[b]
        srcs = [[wl.layers[0][j][t].cpu().numpy() for t in bk.tensors] for j in range(k)]
        reps = [torch.cat(wl.rep_fp[wl.step_no % 2][i])[lo:lo + n].cpu().numpy() for i in range(k)]
        hats = [torch.cat(wl.xhat[i])[lo:lo + n].cpu().numpy().copy() for i in range(k)]
        t0 = time.perf_counter()
        flats = [oracle.bucket_flatten(srcs[j], bk.offsets, n) for j in range(k)]
        deltas = [np.zeros(n, np.float32) for _ in range(k)]
        enc = [oracle.compress_minmax_u8(flats[j], deltas[j], C) for j in range(k)]
        oracle.drr_minmax_u8([e[0] for e in enc], [e[1] for e in enc], np.zeros(n, np.float32), C)
        oracle.ring_avg_fp(reps)
        oracle.ring_avg_lp(reps, hats, C)
        sd = [np.zeros(n, np.float32) for _ in range(k)]
        senc = [oracle.sign_compress_ef(flats[j], sd[j], SC) for j in range(k)]
        oracle.drr_sign([e[0] for e in senc], [e[1] for e in senc], np.zeros(n, np.float32), n, SC)
        dt += time.perf_counter() - t0
    grad_bytes = 4.0 * wl.n_elems * k * len(ALL_PRIMS)
    # the same on one core, on the last (smallest) bucket only
    oracle.set_threads(1)
    bk = wl.buckets[-1]
    n1, lo = bk.n_pad, wl.bases[len(wl.buckets) - 1]
    flats_g = [torch.cat(wl.bucket[j])[lo:lo + n1].contiguous() for j in range(k)]
    flats = [f.cpu().numpy() for f in flats_g]
    d_o = [np.zeros(n1, np.float32) for _ in range(k)]
    sd_o = [np.zeros(n1, np.float32) for _ in range(k)]
    eps_o, seps_o = np.zeros(n1, np.float32), np.zeros(n1, np.float32)
    t0 = time.perf_counter()
    enc = [oracle.compress_minmax_u8(flats[j], d_o[j], C) for j in range(k)]
    drr = oracle.drr_minmax_u8([e[0] for e in enc], [e[1] for e in enc], eps_o, C)
    senc = [oracle.sign_compress_ef(flats[j], sd_o[j], SC) for j in range(k)]
    sdrr = oracle.drr_sign([e[0] for e in senc], [e[1] for e in senc], seps_o, n1, SC)
    dt1 = time.perf_counter() - t0
    parity = parity_sample(torch, wl.bg, flats_g, C, SC, enc, d_o, drr, eps_o, senc, sd_o, sdrr, seps_o)
    oracle.set_threads(threads)
    return {"value": round(grad_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "one full step of the same workload (%d elements x %d workers, all seven primitives), "
                      "%.1f s wall on %d threads" % (wl.n_elems, k, dt, threads),
            "one_core_value": round(4.0 * n1 * k * 4 / dt1 / 1e9, 3),
            "one_core_sample": "compress_minmax, drr_minmax, sign_compress, drr_sign on the last bucket "
                               "(%d elements x %d workers), %.1f s on 1 thread" % (n1, k, dt1)}, parity


def parity_sample(torch, bg, xs, C, SC, enc, d_o, drr, eps_o, senc, sd_o, sdrr, seps_o):
    """The HIP path on the buckets the one-core oracle leg just processed (same bits, zero initial error state),
    compared word for word with the oracle's outputs.  Integer outputs must be equal; fp32 outputs are counted twice:
    words that are not bit-identical, and words outside 1e-6 relative + 1e-7 absolute."""
    import numpy as np
    k, n = len(xs), xs[0].numel()
    dev = xs[0].device
    nc, ncs = (n + C - 1) // C, (n + SC - 1) // SC
    f32 = dict(dtype=torch.float32, device=dev)
    cnt = {"int_words": 0, "int_mismatch": 0, "fp32_words": 0, "fp32_not_bit_exact": 0, "fp32_out_of_tolerance": 0}

    def ints(t, ref):
        a = t.cpu().numpy().view(ref.dtype).reshape(-1)
        cnt["int_words"] += a.size
        cnt["int_mismatch"] += int(np.count_nonzero(a != ref.reshape(-1)))

    def floats(t, ref):
        a = t.cpu().numpy()
        cnt["fp32_words"] += a.size
        cnt["fp32_not_bit_exact"] += int(np.count_nonzero(a.view(np.uint32) != ref.view(np.uint32)))
        err = np.abs(a.astype(np.float64) - ref.astype(np.float64))
        cnt["fp32_out_of_tolerance"] += int(np.count_nonzero(~(err <= 1e-6 * np.abs(ref.astype(np.float64)) + 1e-7)))

    codes = [torch.empty(n, dtype=torch.uint8, device=dev) for _ in range(k)]
    mm = [torch.empty(2 * nc, **f32) for _ in range(k)]
    delta = [torch.zeros(n, **f32) for _ in range(k)]
    bits = [torch.empty((n + 31) // 32, dtype=torch.int32, device=dev) for _ in range(k)]
    scale = [torch.empty(ncs, **f32) for _ in range(k)]
    sdelta = [torch.zeros(n, **f32) for _ in range(k)]
    for j in range(k):
        bg.bagua_compress_minmax_u8(xs[j], delta[j], C, codes[j], mm[j])
        bg.bagua_sign_compress_ef(xs[j], sdelta[j], SC, bits[j], scale[j])
    eps, seps = torch.zeros(n, **f32), torch.zeros(n, **f32)
    c2, m2, o2 = torch.empty(n, dtype=torch.uint8, device=dev), torch.empty(2 * nc, **f32), torch.empty(n, **f32)
    b2, s2, so2 = torch.empty((n + 31) // 32, dtype=torch.int32, device=dev), torch.empty(ncs, **f32), torch.empty(n, **f32)
    bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, codes, mm, eps, n, C, c2, m2, o2)
    bg.bagua_decompress_reduce_recompress(bg.CODEC_SIGN1, bits, scale, seps, n, SC, b2, s2, so2)
    torch.cuda.synchronize()
    for j in range(k):
        ints(codes[j], enc[j][0]); floats(mm[j], enc[j][1]); floats(delta[j], d_o[j])
        ints(bits[j], senc[j][0]); floats(scale[j], senc[j][1]); floats(sdelta[j], sd_o[j])
    ints(c2, drr[0]); floats(m2, drr[1]); floats(o2, drr[2]); floats(eps, eps_o)
    ints(b2, sdrr[0]); floats(s2, sdrr[1]); floats(so2, sdrr[2]); floats(seps, seps_o)
    cnt["sample"] = ("compress_minmax, drr_minmax, sign_compress, drr_sign on the last bucket (%d elements x %d workers), "
                     "HIP path against the oracle" % (n, k))
    return cnt


def copy_ceiling(torch, bg):
    """Throughput of a plain 128-bit copy on this GPU, for context next to the roofline: bagua_bucket_flatten_run with
    a single tensor covering the whole bucket is exactly that (read 4 B, write 4 B per element).  GB/s."""
    n = 128 * 1024 * 1024
    bufs = [(torch.zeros(n, device="cuda"), torch.empty(n, device="cuda")) for _ in range(2)]   # 2 GiB rotated
    plans = []
    for src, dst in bufs:
        ws = torch.empty(bg.bagua_flatten_workspace_bytes(1, n), dtype=torch.uint8, device="cuda")
        bg.bagua_flatten_plan([src], [0], n, ws)
        plans.append(ws)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for i in range(4):
        bg.bagua_bucket_flatten_run(plans[i % 2], 1, bufs[i % 2][1])
    ev[0].record()
    reps = 20
    for i in range(reps):
        bg.bagua_bucket_flatten_run(plans[i % 2], 1, bufs[i % 2][1])
    ev[1].record()
    torch.cuda.synchronize()
    return 8.0 * n * reps / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9


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
    import __graft_entry__
    __graft_entry__.ensure_built()        # uses what is built; compiles only if a library is missing altogether
    import paper_2107_01499_amd as bg     # fails loudly if the HIP library cannot be loaded
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    only = set(p for p in args.only.split(",") if p) or None
    ceiling = copy_ceiling(torch, bg)
    wl = Workload(torch, bg, args.workload, per_bucket=args.per_bucket_launch, only=only, fused=args.fused_flatten,
                  extras=tuple(e for e in args.extras.split(",") if e))
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
        for (_, e0), (name, e1) in zip(marks[:-1], marks[1:]):
            prim_ms[name] += e0.elapsed_time(e1)
    gpu_ms = sum(m[0][1].elapsed_time(m[-1][1]) for m in all_marks)
    for p in prims:
        prim_ms[p] /= args.steps
    ms_per_step = wall * 1e3 / args.steps

    gb, ab, nl = wl.grad_bytes(), wl.algo_bytes(), wl.launches()
    total_grad = sum(gb[p] for p in prims)
    per_prim = {}
    for p in prims:
        t = prim_ms[p] * 1e-3
        per_prim[p] = {"ms": round(prim_ms[p], 4), "launches": nl[p], "gradient_GBps": round(gb[p] / t / 1e9, 1),
                       "hbm_GBps": round(ab[p] / t / 1e9, 1), "frac_of_peak": round(ab[p] / t / 1e9 / HBM_PEAK_GBS, 4),
                       "frac_of_copy_kernel": round(ab[p] / t / 1e9 / ceiling, 4)}
    dom = next((p for p in ("compress_minmax", "flatten_compress") if p in prims), None) or max(prims, key=lambda p: prim_ms[p])
    dom_t = prim_ms[dom] * 1e-3 / nl[dom]
    achieved = ab[dom] / nl[dom] / dom_t / 1e9
    traffic = read_traffic() if (dom == "compress_minmax" and args.workload == "resnet50" and not args.per_bucket_launch) else None
    result = {
        "metric": "gradient GB/s processed per primitive on 1 MI355X; % of HBM roofline",
        "value": round(total_grad / (wall / args.steps) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s in %d greedy 25 MiB buckets (%d padded elements per worker), %d simulated workers, "
                               "chunk %d (sign codec %d), error state carried across steps; primitives per step: %s" %
                               (wl.w["label"], len(wl.buckets), wl.n_elems, wl.k, wl.C, wl.SC, ", ".join(prims)),
                   "workers": wl.k, "chunk": wl.C, "sign_chunk": wl.SC, "buckets": len(wl.buckets),
                   "launch": "per bucket" if args.per_bucket_launch else "per worker (all buckets of a worker in one launch)",
                   "elements_per_worker": wl.n_elems},
        "gpu_ms_per_step": round(gpu_ms / args.steps, 4),
        "copy_kernel_GBps": round(ceiling, 1),
        "per_primitive": per_prim,
        "roofline": {"bound": "hbm", "kernel": wl.kernel_name(dom), "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "avg_launch_us": round(dom_t * 1e6, 3), "algorithmic_bytes_per_launch": ab[dom] / nl[dom]},
    }
    if not args.no_cpu_baseline and args.workload == "resnet50" and only is None and not args.fused_flatten and not args.extras:
        result["cpu_baseline"], result["parity"] = cpu_baseline(wl, torch)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
