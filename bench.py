#!/usr/bin/env python3
"""Benchmark of the one-GPU share of the AsyncHZP data-parallel hot path on MI355X.

A step is one pass of the whole path over one rank's share of a model-shaped state:
  1. fused gradient reduction (R bf16 contributions, fp32 sum) + AdamW + bf16 cast on the rank's
     ZeRO-1 shard of every layer bucket            (one hzp_adamw_shard call over the layer range)
  2. level-1 gather: K owners' bf16 outputs -> the ZeRO-3 parameter shard, per bucket
  3. level-3 gather: Z3 parameter shards -> the full padded layer bucket, per bucket
The layout plan is built once before the loop (it is static).  All inputs are synthetic, seeded
and resident in HBM before the timed region starts.  Prints ONE JSON line.

The headline workload is the largest of the five that fits one GPU: the full MoE layer set (24
layers, R = 16, about 200 GB resident).  After it, the same step is timed on the other four
workloads (fewer repetitions, each in a child process `bench.py --config N`) and reported under
"configs": one {fused, gather1, gather3} roofline triple per workload.  `--config N` times one
workload only.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=-1,
                    help="time only workload 0..4 (tiny, dense7b, dense70b, moe, irregular); default: headline on "
                         "moe, then the other four under \"configs\"")
    ap.add_argument("--other-steps", type=int, default=20, help="timed steps of each non-headline workload")
    ap.add_argument("--layers", type=int, default=0, help="use only the first N layers (0 = all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true")
    ap.add_argument("--separate-allocations", action="store_true",
                    help="give every slice its own allocation instead of per-kind arenas (layout experiment)")
    ap.add_argument("--layout", default="arena", choices=["arena", "kinds"],
                    help="arena: the rank's streams in one allocation at the planner's offsets (default); kinds: one "
                         "allocation per stream kind")
    ap.add_argument("--arena-variant", default="tune",
                    help="layout variant of hzp_plan_arena (0..7), or 'tune': hzp_arena_tune picks it at set-up, "
                         "before the buffers are filled (default)")
    ap.add_argument("--gather1-per-layer", action="store_true",
                    help="issue the level-1 gather as one call per layer instead of one call for all layers")
    ap.add_argument("--phases", default="fused,gather1,gather3",
                    help="comma list of the step's phases to run (profiling aid)")
    ap.add_argument("--secondary", default="",
                    help="comma list of secondary rows timed after the step loop: unpack,reduce,accumulate,prereduced,perlayer,freegroups,inplace,notinplace,f32class,graph,overlap")
    return ap.parse_args()


class Workload:
    """Device buffers and pre-marshalled pointer arrays of one rank's share.

    Layout "arena" (default): the rank's persistent streams (replica r's gradient slices, master,
    momentum, variance, bf16 output, received ZeRO-1 pieces, the ZeRO-3 shard, received shards) lie
    in ONE allocation at the offsets the planner gives (hzp_plan_arena / hzp_plan_arena_slice: every
    stream on a 2 MiB boundary, the slices of all layer buckets back to back; the spacing variant is
    chosen by hzp_arena_tune on the empty allocation unless `arena_variant` names one); only the gathered
    layer buckets (and a rotating pool's shards) are allocations of their own.  Layout "kinds": one
    allocation per stream kind, same order inside (the earlier default: 1-4 % slower on average and
    much less repeatable from process to process).  `separate=True` gives every slice its own
    allocation (slower again)."""

    def __init__(self, cfg, n_layers, rank, torch, hzp, hzp_inputs, separate=False, l3_pool=0, layout="arena",
                 arena_variant="tune"):
        """l3_pool > 0: the level-3 gather streams through a rotating pool (the cyclic buffers of
        Section 4.2): the received ZeRO-3 shards of only `l3_pool` layers and two destination buckets
        are resident, layer l using slot l % l3_pool and bucket l % 2.  For layer streams whose full
        buckets (2 bytes x P x layers) do not fit beside the rest."""
        self.cfg, self.rank = cfg, rank
        self.l3_pool = l3_pool
        dev = "cuda:0"
        tpl = cfg["tensors_per_layer"][:n_layers]
        numel = cfg["tensor_numel"][:sum(tpl)]
        self.plan = hzp.hzp_plan(tpl, numel, cfg["align"], cfg["z3"], cfg["z1"])
        info = self.plan.info()
        self.n_layers, self.R, self.K, self.z3 = n_layers, cfg["R"], info.k, info.z3
        self.buckets = [self.plan.bucket(l, 0) for l in range(n_layers)]
        self.s1_total = sum(b.s1 for b in self.buckets)
        self.s3_total = sum(b.s3 for b in self.buckets)
        self.p_total = sum(b.padded for b in self.buckets)
        assert self.p_total == info.total_padded
        j, k, i = self.plan.rank(rank)
        bf16, f32 = torch.bfloat16, torch.float32
        arenas = {}
        self.layout = "separate" if separate else layout
        big, big_off = None, 0
        if self.layout == "arena":
            A = hzp.HZP_ARENA_ALIGN
            tune = arena_variant == "tune"
            variants = range(hzp.HZP_ARENA_VARIANTS) if tune else [int(arena_variant)]
            nbytes = max(self.plan.arena(0, self.R, variant=v) for v in variants)
            whole = torch.empty(nbytes + A, dtype=torch.uint8, device=dev)
            big_off = (-whole.data_ptr()) % A          # the arena starts on a multiple of HZP_ARENA_ALIGN
            big = self.arena_buffer = whole
            self.arena_variant, self.arena_tune_seconds = (0 if tune else int(arena_variant)), None
            if tune:                                   # set-up time: the allocation is still empty
                self.plan.prepare()
                self.arena_variant, self.arena_tune_seconds = self.plan.arena_tune(
                    0, rank, self.R, whole.data_ptr() + big_off, nbytes)

        def stream_of(name):
            """(hzp stream, index) of an arena name, or None for buffers outside the planner's arena."""
            if name[0] == "g" and name[1:].isdigit():
                return hzp.HZP_STREAM_GRAD, int(name[1:])
            if name in ("p", "m", "v", "o", "s3"):
                return {"p": hzp.HZP_STREAM_MASTER, "m": hzp.HZP_STREAM_M, "v": hzp.HZP_STREAM_V,
                        "o": hzp.HZP_STREAM_PARAM_OUT, "s3": hzp.HZP_STREAM_SHARD3}[name], 0
            if name.startswith("recv1_"):
                kk = int(name[6:])
                return hzp.HZP_STREAM_RECV1, kk if kk < k else kk - 1      # the K-1 owners other than this rank
            if name.startswith("recv3_") and not l3_pool:
                jj = int(name[6:])
                return hzp.HZP_STREAM_RECV3, jj if jj < j else jj - 1
            return None

        def arena(name, total, dtype):
            if name not in arenas:
                arenas[name] = torch.empty(total, dtype=dtype, device=dev)
            return arenas[name]

        def pack(specs):
            """Places the stream kinds `specs` = [(name, elements, dtype)] in ONE allocation, each on a 2 MiB
            boundary an odd number of 2 MiB units after the one before (the default spacing of the planner's
            arena), instead of one allocation per kind: for the secondary rows' many-stream kernels."""
            if separate or self.layout != "arena":
                return
            A = hzp.HZP_ARENA_ALIGN
            starts, pos, prev = [], 0, None
            for name, total, dtype in specs:
                pos = -(-pos // A) * A
                if prev is not None and ((pos - prev) // A) % 2 == 0:
                    pos += A
                starts.append(pos)
                prev = pos
                pos += total * torch.empty(0, dtype=dtype).element_size()
            whole = torch.empty(pos + A, dtype=torch.uint8, device=dev)
            off = (-whole.data_ptr()) % A
            for (name, total, dtype), st in zip(specs, starts):
                nbytes = total * torch.empty(0, dtype=dtype).element_size()
                arenas[name] = whole[off + st:off + st + nbytes].view(dtype)

        def piece(name, total, dtype, begin, n, fill=None, layer=None):
            """Slice [begin, begin+n) of the arena `name`, or an allocation of its own."""
            st = stream_of(name) if (big is not None and layer is not None) else None
            if separate:
                t = torch.empty(n, dtype=dtype, device=dev)
            elif st is not None:
                off, nbytes = self.plan.arena_slice(0, self.R, st[0], st[1], layer, variant=self.arena_variant)
                t = big[big_off + off:big_off + off + nbytes].view(dtype)
                assert t.numel() == n
                arenas.setdefault(name, t)
            else:
                t = arena(name, total, dtype)[begin:begin + n]
            if fill is not None:
                t.copy_(fill)
            return t

        self.keep = []
        self.payload_params = 0           # tensor elements; the rest of p_total is padding
        g_ptrs, p_ptrs, m_ptrs, v_ptrs, o_ptrs = [], [], [], [], []
        self.l1_args, self.l3_args = [], []
        l1_src, l1_dst = [], []
        tid = 0
        for l, b in enumerate(self.buckets):
            ranges = []
            for _ in range(b.n_tensors):
                t = self.plan.tensor(tid)
                ranges.append((t.offset, t.numel))
                self.payload_params += t.numel
                tid += 1
            beg, n = self.plan.shard(l, 0, 1, rank)
            o1, o3 = b.base // cfg["z1"], b.base // cfg["z3"]       # arena offsets of this bucket's slices
            pad = None if b.payload_end == b.padded else ranges
            grads = [piece("g%d" % r, self.s1_total, bf16, o1, n,
                           hzp_inputs.device_normal(n, cfg["sigma"], 1000003 * l + 17 * r + 1, dev, bf16, pad, beg), layer=l)
                     for r in range(self.R)]
            p = piece("p", self.s1_total, f32, o1, n,
                      hzp_inputs.device_normal(n, 0.02, 1000003 * l + 7919, dev, f32, pad, beg), layer=l)
            m = piece("m", self.s1_total, f32, o1, n, layer=l).zero_()
            v = piece("v", self.s1_total, f32, o1, n, layer=l).zero_()
            out = piece("o", self.s1_total, bf16, o1, n, layer=l).zero_()
            # level 1: this rank's output is owner k; the other K-1 owners' pieces are "received"
            owners = [out if kk == k else piece("recv1_%d" % kk, self.s1_total, bf16, o1, n, layer=l).normal_()
                      for kk in range(self.K)]
            shard3 = piece("s3", self.s3_total, bf16, o3, b.s3, layer=l).zero_()
            # level 3: this rank's shard is j; the other Z3-1 shards are "received"
            if l3_pool:
                slot = l % l3_pool
                s3_max, p_max = max(x.s3 for x in self.buckets), max(x.padded for x in self.buckets)
                fresh = l < l3_pool
                shards = [shard3 if jj == j else piece("recv3_%d" % jj, l3_pool * s3_max, bf16, slot * s3_max, b.s3)
                          for jj in range(self.z3)]
                if fresh:
                    for jj in range(self.z3):
                        if jj != j:
                            shards[jj].normal_()
                bucket = piece("bucket", 2 * p_max, bf16, (l % 2) * p_max, b.padded)
            else:
                shards = [shard3 if jj == j else piece("recv3_%d" % jj, self.s3_total, bf16, o3, b.s3, layer=l).normal_()
                          for jj in range(self.z3)]
                bucket = piece("bucket", self.p_total, bf16, b.base, b.padded)
            self.keep.append((grads, p, m, v, out, owners, shard3, shards, bucket))
            if (l + 1) % 8 == 0:        # a sign of life on stderr: building takes minutes under a counter-collecting profiler
                print("bench: %s: buffers of %d of %d layers filled" % (cfg["name"], l + 1, n_layers), file=sys.stderr, flush=True)
            g_ptrs += grads
            p_ptrs.append(p); m_ptrs.append(m); v_ptrs.append(v); o_ptrs.append(out)
            self.l1_args.append((l, hzp.ptr_array(owners), shard3.data_ptr()))
            l1_src += owners
            l1_dst.append(shard3)
            self.l3_args.append((l, hzp.ptr_array(shards), bucket.data_ptr()))
        self.l1_all = (hzp.ptr_array(l1_src), hzp.ptr_array(l1_dst))       # the post-step gather of all layers in one call
        self.arenas = arenas
        self._piece, self._pack, self._torch, self._hzp, self._dev = piece, pack, torch, hzp, dev
        self.unpack_args, self.reduce_args = None, None
        self.l1_per_layer = False
        self.g_arr, self.p_arr = hzp.ptr_array(g_ptrs), hzp.ptr_array(p_ptrs)
        self.m_arr, self.v_arr, self.o_arr = hzp.ptr_array(m_ptrs), hzp.ptr_array(v_ptrs), hzp.ptr_array(o_ptrs)
        # the same update as one call per layer (the secondary row "perlayer")
        self.layer_args = [(l, hzp.ptr_array(g_ptrs[l * self.R:(l + 1) * self.R]), hzp.ptr_array([p_ptrs[l]]),
                            hzp.ptr_array([m_ptrs[l]]), hzp.ptr_array([v_ptrs[l]]), hzp.ptr_array([o_ptrs[l]]))
                           for l in range(n_layers)]


def add_inplace_arrays(w):
    hzp = w._hzp
    k = w.plan.rank(w.rank)[1]
    own, srcs = [], []
    for l, kept in enumerate(w.keep):
        owners, shard3 = kept[5], kept[6]
        s1 = w.buckets[l].s1
        piece = shard3[k * s1:(k + 1) * s1]
        own.append(piece)
        srcs += [piece if kk == k else owners[kk] for kk in range(w.K)]
    w.inplace_keep = own
    w.inplace_o, w.inplace_l1 = hzp.ptr_array(own), hzp.ptr_array(srcs)


def add_secondary_buffers(w, phases):
    """Buffers of the secondary rows (allocated only when those phases are asked for):
    `unpack`: level-3 gather into unpadded per-tensor buffers; `reduce`: standalone fp32
    reduction of the R bf16 contributions on the rank's ZeRO-3 gradient slice."""
    torch, hzp, bf16 = w._torch, w._hzp, w._torch.bfloat16
    if "unpack" in phases and w.unpack_args is None:
        w.unpack_args, w.payload_total, tid = [], 0, 0
        for l, b in enumerate(w.buckets):
            recs = [w.plan.tensor(tid + t) for t in range(b.n_tensors)]
            tid += b.n_tensors
            total = sum(r.numel for r in recs)
            pool = w._piece("tensors", w.p_total, bf16, b.base, total)
            views, pos = [], 0
            for r in recs:
                views.append(pool[pos:pos + r.numel])
                pos += r.numel
            w.payload_total += total
            w.unpack_args.append((l, w.l3_args[l][1], hzp.ptr_array(views), views))
    if "accumulate" in phases and getattr(w, "accum_args", None) is None:
        # fp32 contributions accumulated into a resident fp32 gradient shard (one micro-batch)
        w.accum_args = []
        w._pack([("ag%d" % r, w.s3_total, torch.float32) for r in range(w.R)] + [("acc", w.s3_total, torch.float32)])
        for l, b in enumerate(w.buckets):
            o3 = b.base // w.cfg["z3"]
            slices = [w._piece("ag%d" % r, w.s3_total, torch.float32, o3, b.s3).normal_(0.0, w.cfg["sigma"])
                      for r in range(w.R)]
            acc = w._piece("acc", w.s3_total, torch.float32, o3, b.s3).zero_()
            w.accum_args.append((l, hzp.ptr_array(slices), acc, slices))
    if "prereduced" in phases and getattr(w, "pre_arr", None) is None:
        # the update from an already reduced fp32 gradient shard (R == 0 form): 30 B per parameter
        w.pre_keep = [w._piece("gpre", w.s1_total, torch.float32, b.base // w.cfg["z1"], b.s1).normal_(0.0, w.cfg["sigma"])
                      for b in w.buckets]
        w.pre_arr = hzp.ptr_array(w.pre_keep)
    if "freegroups" in phases and getattr(w, "free_args", None) is None:
        # the same layers under group sizes that do not nest (Z1 = 3*Z3/2): ZeRO-3 shard 1 of every
        # layer is rebuilt from one partial and one whole ZeRO-1 shard
        cfg = w.cfg
        tpl = cfg["tensors_per_layer"][:w.n_layers]
        w.free_z1 = max(3, 3 * cfg["z3"] // 2)
        w.free_plan = hzp.hzp_plan(tpl, cfg["tensor_numel"][:sum(tpl)], cfg["align"], cfg["z3"], w.free_z1)
        fb = [w.free_plan.bucket(l, 0) for l in range(w.n_layers)]
        w.free_s3_total = sum(b.s3 for b in fb)
        s1_total = sum(b.s1 for b in fb)
        w.free_args, off1, off3 = [], 0, 0
        for l, b in enumerate(fb):
            first, n = w.free_plan.cover(l, 0, 1)
            owners = [w._piece("fo%d" % q, s1_total, bf16, off1, b.s1).normal_() for q in range(n)]
            dst = w._piece("fs3", w.free_s3_total, bf16, off3, b.s3)
            w.free_args.append((l, hzp.ptr_array(owners), dst, owners))
            off1, off3 = off1 + b.s1, off3 + b.s3
    if "f32class" in phases and getattr(w, "f32_args", None) is None:
        # the same layers with every tensor of class F32 (fp32 gradients in, fp32 parameters out: 28 + 4R bytes
        # per parameter), laid out in an arena of its own with the variant the tuner picks
        cfg = w.cfg
        tpl = cfg["tensors_per_layer"][:w.n_layers]
        nt = sum(tpl)
        w.f32_plan = hzp.hzp_plan(tpl, cfg["tensor_numel"][:nt], cfg["align"], cfg["z3"], cfg["z1"], tensor_class=[1] * nt)
        w.f32_plan.prepare()
        A = hzp.HZP_ARENA_ALIGN
        nbytes = max(w.f32_plan.arena(1, w.R, variant=v) for v in range(hzp.HZP_ARENA_VARIANTS))
        whole = torch.empty(nbytes + A, dtype=torch.uint8, device=w._dev)
        off0 = (-whole.data_ptr()) % A
        variant, secs = w.f32_plan.arena_tune(1, w.rank, w.R, whole.data_ptr() + off0, nbytes)
        def view(kind, index, layer):
            off, n = w.f32_plan.arena_slice(1, w.R, kind, index, layer, variant=variant)
            return whole[off0 + off:off0 + off + n].view(torch.float32)
        g, p, m, v, o = [], [], [], [], []
        for l in range(w.n_layers):
            g += [view(hzp.HZP_STREAM_GRAD, r, l).normal_(0.0, cfg["sigma"]) for r in range(w.R)]
            p.append(view(hzp.HZP_STREAM_MASTER, 0, l).normal_(0.0, 0.02))
            m.append(view(hzp.HZP_STREAM_M, 0, l)); v.append(view(hzp.HZP_STREAM_V, 0, l))
            o.append(view(hzp.HZP_STREAM_PARAM_OUT, 0, l))
        w.f32_keep = (whole, g, p, m, v, o)
        w.f32_variant = variant
        w.f32_args = tuple(hzp.ptr_array(x) for x in (g, p, m, v, o))
    if "reduce" in phases and w.reduce_args is None:
        w.reduce_args = []
        w._pack([("rg%d" % r, w.s3_total, bf16) for r in range(w.R)] + [("rout", w.s3_total, torch.float32)])
        for l, b in enumerate(w.buckets):
            o3 = b.base // w.cfg["z3"]
            slices = [w._piece("rg%d" % r, w.s3_total, bf16, o3, b.s3).normal_(0.0, w.cfg["sigma"])
                      for r in range(w.R)]
            out = w._piece("rout", w.s3_total, torch.float32, o3, b.s3)
            w.reduce_args.append((l, hzp.ptr_array(slices), out, slices))


def run_secondary(w, hzp, stream, phase):
    s = stream.cuda_stream
    if phase in ("inplace", "notinplace"):
        # the update and the post-step gather, the update writing the rank's bf16 parameters straight into
        # piece k of its ZeRO-3 shard (that piece is then not copied by the gather) -- or not
        a = w.cfg["adamw"]
        hy = hzp.adamw_hyper(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"], w.cfg["grad_scale"], 1)
        o_arr, l1_src = (w.inplace_o, w.inplace_l1) if phase == "inplace" else (w.o_arr, w.l1_all[0])
        hzp.hzp_adamw_shard(w.plan, 0, w.n_layers, 0, w.rank, hy, w.g_arr, w.R, w.p_arr, w.m_arr, w.v_arr, o_arr, stream=s)
        hzp.hzp_gather_layers(w.plan, 0, w.n_layers, 0, 1, l1_src, w.K, w.l1_all[1], stream=s)
    elif phase == "f32class":
        a = w.cfg["adamw"]
        hy = hzp.adamw_hyper(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"], w.cfg["grad_scale"], 1)
        g, p, m, v, o = w.f32_args
        hzp.hzp_adamw_shard(w.f32_plan, 0, w.n_layers, 1, w.rank, hy, g, w.R, p, m, v, o, stream=s)
    elif phase == "perlayer":
        a = w.cfg["adamw"]
        hy = hzp.adamw_hyper(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"], w.cfg["grad_scale"], 1)
        for l, g, p, m, v, o in w.layer_args:
            hzp.hzp_adamw_shard(w.plan, l, l + 1, 0, w.rank, hy, g, w.R, p, m, v, o, stream=s)
    elif phase == "prereduced":
        a = w.cfg["adamw"]
        hy = hzp.adamw_hyper(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"], 1.0, 1)
        hzp.hzp_adamw_shard(w.plan, 0, w.n_layers, 0, w.rank, hy, w.pre_arr, 0, w.p_arr, w.m_arr, w.v_arr, w.o_arr,
                            stream=s)
    elif phase == "freegroups":
        for l, owners, dst, _ in w.free_args:
            hzp.hzp_gather_shard(w.free_plan, l, 0, 1, owners, dst, stream=s)
    elif phase == "unpack":
        for l, shards, tensors, _ in w.unpack_args:
            hzp.hzp_gather_layer(w.plan, l, 0, 3, shards, None, tensors, stream=s)
    elif phase == "accumulate":
        for l, slices, acc, _ in w.accum_args:
            hzp.hzp_reduce_shard(w.plan, l, 0, 3, w.rank, slices, w.cfg["grad_scale"], True, acc, stream=s, R=w.R,
                                 grad_dtype=hzp.HZP_GRAD_F32)
    elif phase == "reduce":
        for l, slices, out, _ in w.reduce_args:
            hzp.hzp_reduce_shard(w.plan, l, 0, 3, w.rank, slices, w.cfg["grad_scale"], False, out, stream=s, R=w.R)


def time_secondary(w, hzp, torch, stream, phase, steps, warmup):
    for _ in range(warmup):
        run_secondary(w, hzp, stream, phase)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(steps):
        run_secondary(w, hzp, stream, phase)
    e1.record(stream)
    stream.synchronize()
    return e0.elapsed_time(e1) / steps


def graph_probe(w, hzp, torch, stream, phases, steps, warmup):
    """Secondary row: the whole step captured once into a HIP graph and replayed, against the same step
    issued call by call -- what the launch-bound workloads (many small launches per step) gain.  The plan's
    device tables exist (hzp_plan_prepare), so no call of the step allocates or copies."""
    w.plan.prepare()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        run_step(w, hzp, 1, torch.cuda.current_stream(), phases)
    torch.cuda.synchronize()
    out = {}
    for name, fn in (("eager", lambda: run_step(w, hzp, 1, stream, phases)), ("graph", g.replay)):
        with torch.cuda.stream(stream):
            for _ in range(warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(steps):
                fn()
            e1.record(stream)
        stream.synchronize()
        out[name + "_ms_per_step"] = round(e0.elapsed_time(e1) / steps, 4)
    return out


def overlap_probe(w, hzp, torch, stream, depth=2, rounds=5, compute_ratio=4.0):
    """Secondary row for the asynchronous scheduler (Section 4.2): per-layer parameter gathers
    prefetched `depth` layers ahead from the background thread into the cyclic pool, while the
    main stream runs a synthetic compute kernel per layer sized to `compute_ratio` times a layer's
    gather.  Compared with issuing the same gathers on the main stream in front of each layer's
    compute.  Two kinds of compute: `spin` (one workgroup that only waits: no contention, shows
    what the dispatch machinery itself hides) and `gemm` (bf16 4096^3 matmuls: a register-file
    saturating MFMA kernel, beside which no other kernel can be resident on a CU)."""
    import time as _time
    n = w.n_layers
    a = torch.randn(4096, 4096, device="cuda:0", dtype=torch.bfloat16)
    b = torch.randn(4096, 4096, device="cuda:0", dtype=torch.bfloat16)
    c = torch.empty(4096, 4096, device="cuda:0", dtype=torch.bfloat16)
    s = stream.cuda_stream

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = _time.perf_counter()
        for _ in range(rounds):
            fn()
        torch.cuda.synchronize()
        return (_time.perf_counter() - t0) * 1e3 / rounds

    def gathers_only():
        for l, arr, dst in w.l3_args:
            hzp.hzp_gather_layer(w.plan, l, 0, 3, arr, dst, None, stream=s)

    def one_matmul():
        with torch.cuda.stream(stream):
            torch.matmul(a, b, out=c)

    a_half, c_half = a[:2048], c[:2048]

    def one_half_matmul():
        with torch.cuda.stream(stream):
            torch.matmul(a_half, b, out=c_half)

    def one_spin():
        with torch.cuda.stream(stream):
            torch.cuda._sleep(1000000)

    t_gather = timed(gathers_only)
    per_layer = compute_ratio * t_gather / n
    reps = max(1, int(round(per_layer / timed(one_matmul))))
    reps_half = max(1, int(round(per_layer / timed(one_half_matmul))))
    cycles = int(1000000 * per_layer / timed(one_spin))

    def make_compute(kind):
        def compute(l):
            with torch.cuda.stream(stream):
                if kind == "gemm":
                    for _ in range(reps):
                        torch.matmul(a, b, out=c)
                elif kind == "gemm_half":          # 2048 x 4096 x 4096: tiles for about half of the CUs
                    for _ in range(reps_half):
                        torch.matmul(a_half, b, out=c_half)
                else:
                    torch.cuda._sleep(cycles)
        return compute

    out = {"layers": n, "prefetch_depth": depth, "gather_only_ms": round(t_gather, 3), "cases": []}
    for kind in ("spin", "gemm", "gemm_half"):
        compute = make_compute(kind)

        def compute_only():
            for l in range(n):
                compute(l)

        def serial():
            for l, arr, dst in w.l3_args:
                hzp.hzp_gather_layer(w.plan, l, 0, 3, arr, dst, None, stream=s)
                compute(l)

        sched = hzp.Sched(w.plan, gather_slots=depth, queue_capacity=2 * depth + 4)

        def overlapped():
            for l in range(min(depth, n)):
                sched.prefetch(l, w.l3_args[l][1], s)
            for l in range(n):
                sched.acquire(l, s)
                compute(l)
                sched.release(l, s)
                if l + depth < n:
                    sched.prefetch(l + depth, w.l3_args[l + depth][1], s)
            sched.join(s)

        t_compute, t_serial, t_async = timed(compute_only), timed(serial), timed(overlapped)
        sched.drain()
        st = sched.stats()
        out["cases"].append({
            "compute": kind,
            "compute_only_ms": round(t_compute, 3),
            "serial_ms": round(t_serial, 3), "scheduled_ms": round(t_async, 3),
            "gather_time_hidden": round((t_serial - t_async) / t_gather, 3),
            "acquire_host_wait_us_per_layer": round(st.acquire_host_wait_us / max(1, st.gathers_issued), 2)})
        out.update(pool_bytes=st.pool_bytes, peak_live_bytes=st.peak_live_bytes,
                   pool_unused_fraction_at_peak=round(1.0 - st.peak_live_bytes / st.pool_bytes, 4))
        sched.destroy()

    # The same pipeline at the granularity Section 4.2 prefers: one gather per parameter, a layer's
    # parameters acquired before its compute, the ring sized for two layers' worth of parameters.
    first = [0]
    for l in range(n):
        first.append(first[-1] + w.buckets[l].n_tensors)
    needed = []
    for l in range(n):
        shards = w.keep[l][7]
        for t in range(first[l], first[l + 1]):
            rec = w.plan.tensor(t)
            j0, j1 = rec.offset // w.buckets[l].s3, (rec.offset + rec.numel - 1) // w.buckets[l].s3
            needed.append(hzp.ptr_array([shards[j] if j0 <= j <= j1 else None for j in range(w.z3)]))
    per_layer_t = max(b.n_tensors for b in w.buckets)
    layer_bytes = max(2 * b.padded + 256 * b.n_tensors for b in w.buckets)
    sched = hzp.Sched(w.plan, gather_slots=depth * per_layer_t, queue_capacity=2 * depth * per_layer_t + 4,
                      pool_bytes=(depth + 1) * ((layer_bytes + 255) // 256 * 256))
    compute = make_compute("spin")

    def by_parameter():
        for l in range(min(depth, n)):
            for t in range(first[l], first[l + 1]):
                sched.prefetch_tensor(t, needed[t], s)
        for l in range(n):
            for t in range(first[l], first[l + 1]):
                sched.acquire_tensor(t, s)
            compute(l)
            for t in range(first[l], first[l + 1]):
                sched.release_tensor(t, s)
            if l + depth < n:
                for t in range(first[l + depth], first[l + depth + 1]):
                    sched.prefetch_tensor(t, needed[t], s)
        sched.join(s)

    def by_parameter_one_call_per_layer():
        # the same gathers and pool regions, a layer's parameters submitted, acquired and released together
        for l in range(min(depth, n)):
            sched.prefetch_params(l, w.l3_args[l][1], s)
        for l in range(n):
            sched.acquire_params(l, w.buckets[l].n_tensors, s)
            compute(l)
            sched.release_params(l, s)
            if l + depth < n:
                sched.prefetch_params(l + depth, w.l3_args[l + depth][1], s)
        sched.join(s)

    t_param = timed(by_parameter)
    sched.drain()
    st = sched.stats()
    spin = out["cases"][0]
    out["per_parameter"] = {"compute": "spin", "gathers_per_pass": first[-1], "scheduled_ms": round(t_param, 3),
                            "gather_time_hidden": round((spin["serial_ms"] - t_param) / t_gather, 3),
                            "pool_bytes": st.pool_bytes, "peak_live_bytes": st.peak_live_bytes,
                            "wrap_skipped_bytes_per_pass": st.wrap_skipped_bytes // (rounds + 1)}
    t_layer = timed(by_parameter_one_call_per_layer)
    sched.drain()
    out["per_parameter_one_call_per_layer"] = {
        "compute": "spin", "gathers_per_pass": first[-1], "scheduled_ms": round(t_layer, 3),
        "gather_time_hidden": round((spin["serial_ms"] - t_layer) / t_gather, 3)}
    sched.destroy()

    # Backward pass: each layer's gradient contributions are reduced as soon as its compute has produced
    # them ("hungrily", Section 4.2): from the background thread on the scheduler's reduction stream, against
    # the same reductions issued on the compute stream behind each layer's compute.
    add_secondary_buffers(w, ["reduce"])
    torch.cuda.synchronize()

    def reduces_only():
        for l, slices, dst, _ in w.reduce_args:
            hzp.hzp_reduce_shard(w.plan, l, 0, 3, w.rank, slices, w.cfg["grad_scale"], False, dst, stream=s, R=w.R)

    t_reduce = timed(reduces_only)

    def serial_backward():
        for l, slices, dst, _ in reversed(w.reduce_args):
            compute(l)
            hzp.hzp_reduce_shard(w.plan, l, 0, 3, w.rank, slices, w.cfg["grad_scale"], False, dst, stream=s, R=w.R)

    sched = hzp.Sched(w.plan, gather_slots=1, queue_capacity=2 * n + 4)

    def hungry_backward():
        for l, slices, dst, _ in reversed(w.reduce_args):
            compute(l)
            sched.reduce(l, 3, w.rank, slices, w.cfg["grad_scale"], False, dst, s)
        sched.join(s)

    t_serial_b, t_hungry = timed(serial_backward), timed(hungry_backward)
    sched.drain()
    out["hungry_reduce"] = {"compute": "spin", "reduce_only_ms": round(t_reduce, 3), "serial_ms": round(t_serial_b, 3),
                            "scheduled_ms": round(t_hungry, 3),
                            "reduce_time_hidden": round((t_serial_b - t_hungry) / t_reduce, 3)}
    sched.destroy()
    return out


def run_step(w, hzp, step, stream, phases, events=None):
    a = w.cfg["adamw"]
    hy = hzp.adamw_hyper(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"],
                         w.cfg["grad_scale"], step)
    s = stream.cuda_stream
    if events:
        events[0].record(stream)
    if "fused" in phases:
        hzp.hzp_adamw_shard(w.plan, 0, w.n_layers, 0, w.rank, hy, w.g_arr, w.R, w.p_arr, w.m_arr,
                            w.v_arr, w.o_arr, stream=s)
    if events:
        events[1].record(stream)
    if "gather1" in phases:
        if w.l1_per_layer:
            for l, arr, dst in w.l1_args:
                hzp.hzp_gather_layer(w.plan, l, 0, 1, arr, dst, None, stream=s)
        else:       # the post-step gather runs for every layer at once (Section 4.1.2, Optimizer Step)
            hzp.hzp_gather_layers(w.plan, 0, w.n_layers, 0, 1, w.l1_all[0], w.K, w.l1_all[1], stream=s)
    if events:
        events[2].record(stream)
    if "gather3" in phases:
        for l, arr, dst in w.l3_args:
            hzp.hzp_gather_layer(w.plan, l, 0, 3, arr, dst, None, stream=s)
    if events:
        events[3].record(stream)


def copy_probe(torch, hzp, stream):
    """Achievable-bandwidth context: a copy and a triad of 1 GiB arrays, each with the library's
    own kernel (concat with Z3 = 1; reduction of two fp32 contributions) and with torch."""
    n = 1 << 29     # bf16 elements = 1 GiB
    plan = hzp.hzp_plan([1], [n], 8, 1, 1)
    src = torch.empty(n, dtype=torch.bfloat16, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    out = {}
    for name, fn in (("hzp_concat_copy", lambda: hzp.hzp_gather_layer(plan, 0, 0, 3, [src], dst, None,
                                                                        stream=stream.cuda_stream)),
                     ("torch_copy", lambda: dst.copy_(src))):
        with torch.cuda.stream(stream):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                fn()
            e1.record(stream)
        stream.synchronize()
        out[name + "_GBps"] = round(2 * n * 2 * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    del src, dst
    # triad (two reads, one write per element: the read/write mix of the fused update): the
    # library's reduction of two fp32 contributions, a = s*(b + c), and torch's a = b + s*c
    nt = 1 << 28     # fp32 elements = 1 GiB per array
    plan_t = hzp.hzp_plan([1], [nt], 8, 1, 1)
    b = torch.empty(nt, dtype=torch.float32, device="cuda:0").normal_()
    c = torch.empty_like(b).normal_()
    a = torch.empty_like(b)
    bc = hzp.ptr_array([b, c])
    for name, fn in (("hzp_reduce_triad", lambda: hzp.hzp_reduce_shard(plan_t, 0, 0, 1, 0, bc, 0.5, False, a,
                                                                        stream=stream.cuda_stream, R=2,
                                                                        grad_dtype=hzp.HZP_GRAD_F32)),
                     ("torch_triad", lambda: torch.add(b, c, alpha=0.5, out=a))):
        with torch.cuda.stream(stream):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                fn()
            e1.record(stream)
        stream.synchronize()
        out[name + "_GBps"] = round(3 * nt * 4 * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    return out


def cpu_baseline(w, torch, np):
    """The oracle, as it stands, on one layer's share of the same workload: reduce + AdamW on
    the S1 shard, then both gathers for that layer; repeated for roughly 12 s."""
    from oracle import numeric as on
    grads, p, m, v, out, owners, shard3, shards, bucket = w.keep[0]
    a = w.cfg["adamw"]

    def host16(t):
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    g_h = [host16(g) for g in grads]
    p_h, m_h, v_h = p.cpu().numpy().copy(), m.cpu().numpy().copy(), v.cpu().numpy().copy()
    owners_h = [host16(o) for o in owners]
    shards_h = [host16(s) for s in shards]
    n = p_h.size

    def one_pass(step):
        g = on.reduce(g_h, scale=w.cfg["grad_scale"])
        o16 = on.adamw(g, p_h, m_h, v_h, step=step, **a)
        k = w.plan.rank(w.rank)[1]
        j = w.plan.rank(w.rank)[0]
        s3 = on.gather_concat([o16 if kk == k else owners_h[kk] for kk in range(w.K)])
        on.gather_concat([s3 if jj == j else shards_h[jj] for jj in range(w.z3)])

    t0 = time.perf_counter()
    one_pass(1)
    first = time.perf_counter() - t0
    reps = max(1, min(200, int(12.0 / max(first, 1e-3))))
    t0 = time.perf_counter()
    for r in range(reps):
        one_pass(2 + r)
    dt = (time.perf_counter() - t0) / reps
    return {"value": n / dt, "unit": "params/s", "cores": on.threads(), "kind": "oracle",
            "sample": "layer 0 of the same workload: fp32 reduce of R=%d bf16 slices + fp64 AdamW on its "
                      "S1=%d shard, level-1 and level-3 gather of that layer; %d passes, %.2f s each"
                      % (w.R, n, reps, dt)}


def read_traffic(kernel_key):
    """HBM bytes per launch of a kernel as measured with rocprofv3 counters: the committed summary
    profiles/traffic_bytes_per_launch.txt, written from the FETCH_SIZE / WRITE_SIZE runs named there.
    Returns None when the file has no line for the key (the key is printed beside it either way)."""
    path = os.path.join(ROOT, "profiles", "traffic_bytes_per_launch.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split("#")[0].split()
                if len(parts) >= 2 and parts[0] == kernel_key:
                    return float(parts[1])
    except OSError:
        pass
    return None


FUSED_MAX_GROUPS = 300000       # groups of 512 elements one launch of the fused update covers at most


def fused_launch_count(w):
    """Launches one hzp_adamw_shard call over all buckets makes: a launch takes whole runs (a bucket's
    shard, cut at FUSED_MAX_GROUPS groups) while they fit FUSED_MAX_GROUPS groups and the kernel's
    segment table (34 segments, 408 pointers of R + 4 per segment)."""
    cap = min(34, 408 // (w.R + 4))
    runs = []
    for b in w.buckets:
        groups = -(-b.s1 // 512)
        while groups > 0:
            runs.append(min(groups, FUSED_MAX_GROUPS))
            groups -= runs[-1]
    launches, cnt, blocks = 0, 0, 0
    for g in runs:
        if cnt == cap or (cnt > 0 and blocks + g > FUSED_MAX_GROUPS):
            launches, cnt, blocks = launches + 1, 0, 0
        cnt, blocks = cnt + 1, blocks + g
    return launches + (1 if cnt else 0)


def roofline_entry(np, kernel, algo_bytes, ms, launches, key, step_kernel_ms=None, per_step=None):
    """One kernel's roofline object: `ms` is the average time of its `launches` launches in a step (or
    secondary pass), `algo_bytes` what they move together; `per_step` the same time for each timed step."""
    per_launch_ms = ms / launches
    ach = algo_bytes / launches / (per_launch_ms * 1e-3) / 1e9 if ms > 0 else 0.0
    out = {"kernel": kernel, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS,
           "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": read_traffic(key),
           "traffic_key": key, "launches_per_step": launches, "avg_launch_us": round(per_launch_ms * 1e3, 2),
           "algorithmic_bytes_per_launch": algo_bytes / launches}
    if step_kernel_ms is not None:
        out["share_of_step_time"] = round(ms / max(step_kernel_ms, 1e-9), 3)
    if per_step is not None:        # over the timed steps (each step's launches of the kernel bracketed by one event pair)
        out["median_launch_us"] = round(float(np.median(per_step)) / launches * 1e3, 2)
        out["min_launch_us"] = round(float(per_step.min()) / launches * 1e3, 2)
    return out


def time_workload(idx, args, torch, np, hzp, hzp_inputs, steps, warmup, keep=False):
    """Builds workload `idx`, runs warmup + steps of the whole step and returns its figures."""
    cfg = hzp_inputs.config(idx)
    total_layers = len(cfg["tensors_per_layer"])
    n_layers = total_layers if args.layers <= 0 else min(args.layers, total_layers)
    rank = cfg["z3"] + 1 if cfg["z1"] > cfg["z3"] + 1 else 0      # a rank with j = 1, k = 1
    # the 70B-class layer stream does not fit with every layer's full bucket resident: its level-3
    # gather runs through a rotating pool of 8 layers of received shards and 2 destination buckets
    pool = 8 if cfg["name"] == "dense70b" and n_layers > 8 and not args.separate_allocations else 0
    w = Workload(cfg, n_layers, rank, torch, hzp, hzp_inputs, separate=args.separate_allocations, l3_pool=pool,
                 layout=args.layout, arena_variant=args.arena_variant)
    w.l1_per_layer = args.gather1_per_layer
    phases = set(args.phases.split(","))
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()

    step = 0
    for _ in range(warmup):
        step += 1
        run_step(w, hzp, step, stream, phases)
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step += 1
        run_step(w, hzp, step, stream, phases, evs[k])       # events are recorded on `stream`, where the kernels run
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / steps
    ph = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in evs])     # ms
    fused_ms, g1_ms, g3_ms = (float(x) for x in ph.mean(axis=0))
    R = w.R
    fused_bytes = (26 + 2 * R) * w.s1_total
    g1_bytes, g3_bytes = 4 * w.s3_total, 4 * w.p_total

    def roof(kernel, algo_bytes, ms, launches, key, per_step):
        return roofline_entry(np, kernel, algo_bytes, ms, launches, key, fused_ms + g1_ms + g3_ms, per_step)

    fused_launches = fused_launch_count(w)
    rooflines = {}
    if "fused" in phases:
        rooflines["fused_adamw"] = roof("fused_adamw_kernel<R=%d,bf16>" % R, fused_bytes, fused_ms,
                                        fused_launches, "fused_adamw_%s" % cfg["name"], ph[:, 0])
        # context, outside the timed steps: the update alone, call after call (inside the step it starts behind
        # the level-3 gather's trailing writes)
        alone = 10
        for _ in range(2):
            run_step(w, hzp, step, stream, {"fused"})
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(alone):
            run_step(w, hzp, step, stream, {"fused"})
        e1.record(stream)
        stream.synchronize()
        alone_ms = e0.elapsed_time(e1) / alone
        rooflines["fused_adamw"]["alone_back_to_back"] = {
            "achieved": round(fused_bytes / (alone_ms * 1e-3) / 1e9, 1) if alone_ms > 0 else 0.0,
            "frac": round(fused_bytes / (alone_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4) if alone_ms > 0 else 0.0,
            "avg_launch_us": round(alone_ms / fused_launches * 1e3, 2), "calls": alone}
    if "gather1" in phases:
        if w.l1_per_layer:
            rooflines["gather_level1"] = roof("concat_kernel (K=%d x S1 -> S3)" % w.K, g1_bytes, g1_ms,
                                              w.n_layers, "concat_l1_%s" % cfg["name"], ph[:, 1])
        else:
            pieces = w.n_layers * w.K               # one launch of the layer-range gather holds 192 pieces
            rooflines["gather_level1"] = roof("concat_layers_kernel (all layers, K=%d x S1 -> S3)" % w.K, g1_bytes,
                                              g1_ms, -(-pieces // 192), "concat_layers_l1_%s" % cfg["name"], ph[:, 1])
    if "gather3" in phases:
        rooflines["gather_level3"] = roof("concat_kernel (Z3=%d x S3 -> P)" % w.z3, g3_bytes, g3_ms,
                                          w.n_layers, "concat_l3_%s" % cfg["name"], ph[:, 2])
    # the launch-bound workloads also as one captured step replayed (context; the timed steps are issued call by call)
    graph = None
    if cfg["name"] in ("tiny", "irregular") and phases == {"fused", "gather1", "gather3"} and steps >= 10:
        graph = graph_probe(w, hzp, torch, stream, phases, max(steps, 20), warmup)
    out = {
        "graph_replay": graph,
        "cfg": cfg, "w": w if keep else None, "stream": stream if keep else None, "rank": rank, "phases": phases,
        "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "rooflines": rooflines,
        "fused_ms": fused_ms, "g1_ms": g1_ms, "g3_ms": g3_ms, "fused_bytes": fused_bytes,
        "fused_launches": fused_launches, "s1_total": w.s1_total, "p_total": w.p_total,
        "payload_params": w.payload_params, "n_layers": w.n_layers, "R": R, "z3": w.z3, "K": w.K,
        "l1_per_layer": w.l1_per_layer, "l3_pool": pool, "layout": w.layout,
        "arena_variant": getattr(w, "arena_variant", None),
        "arena_tune_GBps": ([round(fused_bytes / s / 1e9, 1) if s > 0 else None for s in w.arena_tune_seconds]
                            if getattr(w, "arena_tune_seconds", None) else None),
    }
    return out


def workload_text(t):
    cfg = t["cfg"]
    where = {"arena": "the rank's streams in one allocation at the planner's offsets (hzp_plan_arena)",
             "kinds": "one allocation per stream kind", "separate": "one allocation per slice"}[t["layout"]]
    if t["layout"] == "arena":
        where += ", layout variant %d%s" % (t["arena_variant"], " chosen by hzp_arena_tune at set-up" if t["arena_tune_GBps"] else "")
    return ("%s: %d layer buckets, R=%d, Z3=%d, Z1=%d, A=%d, rank %d, %s; step = fused reduce+AdamW on the S1 shards "
            "(%d launches) + level-1 gather (%s) + level-3 gather per layer%s; `value` is shard parameters per second of "
            "the whole step, `fused_update` the metric's own kernel"
            % (cfg["name"], t["n_layers"], t["R"], t["z3"], cfg["z1"], cfg["align"], t["rank"], where, t["fused_launches"],
               "one call per layer" if t["l1_per_layer"] else "all layers in one call",
               " through a rotating pool of %d layers of received shards and 2 buckets" % t["l3_pool"] if t["l3_pool"] else ""))


def triple(t):
    """The {fused, gather1, gather3} rooflines of a timed workload, for the per-workload map."""
    r = t["rooflines"]
    short = lambda x: None if x is None else {k: x[k] for k in x if k in ("kernel", "achieved", "frac", "avg_launch_us", "median_launch_us", "min_launch_us", "alone_back_to_back",
                                                               "launches_per_step", "algorithmic_bytes_per_launch",
                                                               "traffic", "traffic_key")}
    return {"workload": workload_text(t), "steps": t["steps"], "ms_per_step": round(t["ms_per_step"], 4),
            "shard_params_per_step": t["s1_total"],
            "arena_variant": t["arena_variant"], "arena_tune_GBps": t["arena_tune_GBps"],
            "graph_replay": t["graph_replay"],
            "fused_update_params_per_s": t["s1_total"] / (t["fused_ms"] * 1e-3) if t["fused_ms"] > 0 else None,
            "fused": short(r.get("fused_adamw")), "gather1": short(r.get("gather_level1")),
            "gather3": short(r.get("gather_level3"))}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers the one-GPU share of the path only; replicas are buffers in one "
              "GPU's HBM and no collective is issued, so --gpus must be 1 (got %d)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import gc

    import numpy as np
    import torch

    import hzp_inputs
    import paper_2510_20111_amd as hzp

    torch.cuda.set_device(0)
    HEADLINE = 3            # the MoE layer set: the largest workload that fits one GPU
    head_idx = HEADLINE if args.config < 0 else args.config
    t = time_workload(head_idx, args, torch, np, hzp, hzp_inputs, args.steps, args.warmup, keep=True)
    w, stream, cfg, rooflines = t["w"], t["stream"], t["cfg"], t["rooflines"]
    R, fused_ms = t["R"], t["fused_ms"]
    dominant = max(rooflines.values(), key=lambda r: r["share_of_step_time"])
    fused_pps = w.s1_total / (fused_ms * 1e-3) if fused_ms > 0 else None

    result = {
        "metric": "fused reduce+AdamW shard update: params/sec and achieved HBM GB/s (% of peak)",
        "value": w.s1_total / (t["ms_per_step"] * 1e-3),
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload_text(t),
                   "shard_params_per_step": w.s1_total, "padded_params": w.p_total,
                   "payload_params": w.payload_params, "padding_params": w.p_total - w.payload_params,
                   "phases": sorted(t["phases"]), "arena_variant": t["arena_variant"],
                   "arena_tune_GBps": t["arena_tune_GBps"]},
        "fused_update_params_per_s": fused_pps,
        "fused_update_GBps": rooflines.get("fused_adamw", {}).get("achieved"),
        "roofline": dominant,
        "rooflines": rooflines,
        "fused_update": {"params_per_s": fused_pps,
                         "GBps": rooflines.get("fused_adamw", {}).get("achieved"),
                         "bytes_per_param": 26 + 2 * R, "ms": round(fused_ms, 4)},
        "phase_ms": {"fused": round(fused_ms, 4), "gather_level1": round(t["g1_ms"], 4),
                     "gather_level3": round(t["g3_ms"], 4)},
        "workload_name": cfg["name"], "triple": triple(t),
    }
    fused_bytes, fused_launches = t["fused_bytes"], t["fused_launches"]

    def roof(kernel, algo_bytes, ms, launches, key):
        return roofline_entry(np, kernel, algo_bytes, ms, launches, key)

    secondary = [x for x in args.secondary.split(",") if x]
    if "overlap" in secondary:
        secondary.remove("overlap")
        result["scheduler_overlap"] = overlap_probe(w, hzp, torch, stream)
    if "graph" in secondary:
        secondary.remove("graph")
        result["graph_replay"] = graph_probe(w, hzp, torch, stream, t["phases"], max(args.steps, 20), args.warmup)
    if secondary:
        add_secondary_buffers(w, secondary)
        if "inplace" in secondary:
            add_inplace_arrays(w)
        torch.cuda.synchronize()        # the new buffers were filled on the default stream
        result["secondary"] = {}
        for phase in secondary:
            ms = time_secondary(w, hzp, torch, stream, phase, args.steps, args.warmup)
            nbytes = {"unpack": lambda: 4 * w.payload_total, "reduce": lambda: (2 * R + 4) * w.s3_total,
                      "accumulate": lambda: (4 * R + 8) * w.s3_total,
                      "inplace": lambda: fused_bytes + 4 * w.s1_total * (w.K - 1),
                      "notinplace": lambda: fused_bytes + 4 * w.s1_total * w.K,
                      "f32class": lambda: (28 + 4 * R) * w.s1_total,
                      "perlayer": lambda: fused_bytes, "freegroups": lambda: 4 * w.free_s3_total,
                      "prereduced": lambda: 30 * w.s1_total}[phase]()
            kname = {"unpack": "unpack_kernel<2>", "reduce": "reduce_kernel<bf16,R=%d>" % R,
                     "accumulate": "reduce_kernel<f32,R=%d,accumulate>" % R,
                     "inplace": "fused update writing into the ZeRO-3 shard + level-1 gather of the other %d pieces" % (w.K - 1),
                     "notinplace": "fused update + level-1 gather of all %d pieces" % w.K,
                     "f32class": "fused_adamw_kernel<R=%d, fp32 gradients, fp32 output> (class F32 on the same shapes)" % R,
                     "perlayer": "fused_adamw_kernel<R=%d,bf16>, one call per layer" % R,
                     "prereduced": "fused_adamw_kernel<R=1,f32 gradient> (update from a reduced fp32 shard)",
                     "freegroups": "concat_ranges_kernel (Z1=%d over Z3=%d: ZeRO-3 shard from partial owners)"
                                   % (getattr(w, "free_z1", 0), w.z3)}[phase]
            launches = fused_launches if phase in ("prereduced", "f32class") else 1 if phase in ("inplace", "notinplace") else w.n_layers
            result["secondary"][phase] = roof(kname, nbytes, ms, launches, "%s_%s" % (phase, cfg["name"]))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, torch, np)
    # The other workloads, each in a child process of its own (`bench.py --config N`): where a process's
    # buffers lie moves the many-stream kernels by a few per cent, and a workload built after the 200 GB
    # of the headline one were freed lies worse than in a fresh process.
    if args.config < 0 and args.layers <= 0:
        import subprocess
        configs = {cfg["name"]: triple(t)}
        t["w"] = t["stream"] = None
        del w, stream
        gc.collect()
        torch.cuda.empty_cache()
        for idx in (0, 1, 2, 4):
            cmd = [sys.executable, os.path.abspath(__file__), "--config", str(idx), "--steps", str(args.other_steps),
                   "--warmup", str(min(args.warmup, 3)), "--no-cpu-baseline", "--no-probe", "--phases", args.phases]
            if args.gather1_per_layer:
                cmd.append("--gather1-per-layer")
            if args.separate_allocations:
                cmd.append("--separate-allocations")
            cmd += ["--layout", args.layout, "--arena-variant", args.arena_variant]
            res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
            if res.returncode != 0:
                print(res.stderr[-2000:], file=sys.stderr)
                raise RuntimeError("bench.py --config %d failed" % idx)
            child = json.loads([l for l in res.stdout.splitlines() if l.startswith("{")][-1])
            configs[child["workload_name"]] = child["triple"]
        result["configs"] = {k: configs[k] for k in ("tiny", "dense7b", "dense70b", "moe", "irregular")}
    if not args.no_probe:
        result["hbm_probe"] = copy_probe(torch, hzp, torch.cuda.Stream())
    print(json.dumps(result))


if __name__ == "__main__":
    main()
