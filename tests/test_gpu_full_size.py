"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times
(its Workload arenas and its run_step): sampled elements are recomputed one by one by the oracle,
and whole outputs are checked through properties that hold at any size."""
import gc

import numpy as np
import pytest
import torch

import bench
import hzp_inputs
import paper_2510_20111_amd as hzp
from oracle import numeric as on
from oracle import planner as op

from gpu_util import (DEV, assert_cast_of, assert_close_f32, oracle_plan, to_dev, to_host)
from test_gpu_parity import Sim, say

pytestmark = pytest.mark.gpu


def _bits16(t):
    return t.view(torch.int16)


def _sample_indices(n, rng, count=4096, edge=1024):
    edge = min(edge, n // 2)
    idx = np.concatenate([np.arange(edge), np.arange(n - edge, n), rng.integers(0, n, size=count)])
    return np.unique(idx)


def _fused_sampled_parity(cfg_idx, n_layers, steps=2):
    cfg = hzp_inputs.config(cfg_idx)
    rank = cfg["z3"] + 1
    gc.collect()                        # an earlier test's workload holds its arenas through reference cycles
    torch.cuda.empty_cache()            # the larger shares need most of the card in a few allocations
    w = bench.Workload(cfg, n_layers, rank, torch, hzp, hzp_inputs)
    stream = torch.cuda.Stream()
    rng = np.random.default_rng(100 + cfg_idx)
    a = cfg["adamw"]
    samples = []
    for l, (grads, p, m, v, out, owners, shard3, shards, bucket) in enumerate(w.keep):
        idx = _sample_indices(p.numel(), rng)
        ti = torch.from_numpy(idx).to(DEV)
        samples.append(dict(idx=idx, ti=ti,
                            g=[to_host(_bits16(g)[ti], np.uint16) for g in grads],
                            p=to_host(p[ti], np.float32).copy(), m=to_host(m[ti], np.float32).copy(),
                            v=to_host(v[ti], np.float32).copy()))
    torch.cuda.synchronize()
    for step in range(1, steps + 1):
        say("workload %s: step %d over %d buckets, %d shard elements" % (cfg["name"], step, n_layers, w.s1_total))
        bench.run_step(w, hzp, step, stream, {"fused", "gather1", "gather3"})
        stream.synchronize()
        for l, s in enumerate(samples):
            grads, p, m, v, out, owners, shard3, shards, bucket = w.keep[l]
            g = on.reduce(s["g"], scale=cfg["grad_scale"])
            want16 = on.adamw(g, s["p"], s["m"], s["v"], step=step, **a)
            tag = "%s bucket %d step %d" % (cfg["name"], l, step)
            for key, t in (("p", p), ("m", m), ("v", v)):
                assert_close_f32(to_host(t[s["ti"]], np.float32), s[key], tag + " " + key, key)
            assert_cast_of(to_host(_bits16(out)[s["ti"]], np.uint16), to_host(p[s["ti"]], np.float32), tag + " bf16")
    # gathers: whole-output properties on the device, plus oracle-computed windows at every seam
    j, k, _ = w.plan.rank(rank)
    for l, (grads, p, m, v, out, owners, shard3, shards, bucket) in enumerate(w.keep):
        b = w.buckets[l]
        assert torch.equal(_bits16(shard3), torch.cat([_bits16(o) for o in owners])), "level 1, bucket %d" % l
        assert torch.equal(_bits16(bucket), torch.cat([_bits16(s) for s in shards])), "level 3, bucket %d" % l
        for pieces, dst, ln in ((owners, shard3, b.s1), (shards, bucket, b.s3)):
            win = min(64, ln)
            for q in range(1, len(pieces)):
                tail = to_host(_bits16(pieces[q - 1])[ln - win:], np.uint16).copy()
                head = to_host(_bits16(pieces[q])[:win], np.uint16).copy()
                want = on.gather_concat([tail, head])
                got = to_host(_bits16(dst)[q * ln - win:q * ln + win], np.uint16)
                assert np.array_equal(got, want), "seam %d of bucket %d" % (q, l)
    return w


def test_dense7b_rank_share_as_benchmarked():
    """The workload bench.py times: 34 buckets in one fused launch, both gather levels."""
    w = _fused_sampled_parity(1, 34)
    assert w.s1_total == 32 * 3162240 + 2048000 + 2048128


def test_dense70b_layer_stream_sampled():
    """36 of the 80 layers in one call: more than one launch holds (a launch takes at most 300,000
    groups of 512 elements, 22 of these layers), two steps."""
    w = _fused_sampled_parity(2, 36)
    assert w.buckets[0].s1 == 6684800 and w.buckets[0].padded == 855654400
    assert 22 * (6684800 // 512) <= 300000 < 23 * (6684800 // 512)


def test_moe_layer_set_sampled_over_many_launches():
    """21 of the 24 MoE layers at R = 16 in one call, two steps: eleven launches of two layers each."""
    w = _fused_sampled_parity(3, 21)
    assert w.buckets[0].s1 == 71385088 and w.s1_total == 21 * 71385088


def test_one_shard_longer_than_a_launch():
    """A single ZeRO-1 shard of 160 M elements: the update cuts it into runs of at most 300,000 groups
    of 512 elements, one launch each.  Sampled against the oracle at both ends, on both sides of the
    cut (element 153,600,000) and at random positions; decay multipliers are looked up per tensor, so
    the second run must see bucket positions that continue the first."""
    n_a, n_b = 153_600_000 - 4096, 6_400_000 + 4096 + 24
    say("one shard of %d elements across two launches" % (n_a + n_b))
    wd = [1.0, 0.0]
    plan = hzp.hzp_plan([2], [n_a, n_b], 8, 1, 1, tensor_wd_mult=wd)
    b = plan.bucket(0, 0)
    n = int(b.s1)
    assert n > 300000 * 512 and plan.tensor(1).offset == n_a
    R = 2
    bf16, f32 = torch.bfloat16, torch.float32
    g = [hzp_inputs.device_normal(n, 1e-3, 31 + r, DEV, bf16, None, 0) for r in range(R)]
    p = hzp_inputs.device_normal(n, 0.02, 77, DEV, f32, None, 0)
    m, v = torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    out = torch.zeros(n, dtype=bf16, device=DEV)
    cut = 300000 * 512
    rng = np.random.default_rng(5)
    idx = np.unique(np.concatenate([np.arange(1024), np.arange(n - 1024, n), np.arange(cut - 1024, cut + 1024),
                                    np.arange(n_a - 512, n_a + 512), rng.integers(0, n, size=8192)]))
    ti = torch.from_numpy(idx).to(DEV)
    s = dict(g=[to_host(_bits16(x)[ti], np.uint16) for x in g], p=to_host(p[ti], np.float32).copy(),
             m=np.zeros(idx.size, np.float32), v=np.zeros(idx.size, np.float32))
    wd_arr = np.where(idx < n_a, 1.0, 0.0).astype(np.float32)
    a = hzp_inputs.ADAMW
    for step in (1, 2):
        hy = hzp.adamw_hyper(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"], 1.0 / R, step)
        hzp.hzp_adamw_shard(plan, 0, 1, 0, 0, hy, g, R, [p], [m], [v], [out])
        torch.cuda.synchronize()
        on.adamw(on.reduce(s["g"], scale=1.0 / R), s["p"], s["m"], s["v"], step=step, wd_mult=wd_arr, **a)
        for key, t in (("p", p), ("m", m), ("v", v)):
            assert_close_f32(to_host(t[ti], np.float32), s[key], "step %d %s" % (step, key), key)
        assert_cast_of(to_host(_bits16(out)[ti], np.uint16), to_host(p[ti], np.float32), "step %d bf16" % step)
    # every element was updated exactly twice: no element of m is still zero except where all gradients are
    assert int((m == 0).sum().item()) <= int(((g[0].float() + g[1].float()) == 0).sum().item())


def test_the_longest_shard_the_entry_points_accept():
    """2^30 - 512 elements, the longest slice below the 2^30 limit of the kernels' 32-bit byte offsets (the
    last fp32 quad lies 2 KiB below 4 GiB): update (seven launches), stand-alone reduction and a two-shard
    gather into a 4 GiB bucket, sampled against the oracle at both ends, around every launch cut and every
    power-of-two byte offset, and at random; whole outputs through device-side comparisons."""
    n = (1 << 30) - 512
    say("one shard of %d elements" % n)
    gc.collect()
    torch.cuda.empty_cache()
    plan = hzp.hzp_plan([1], [n], 8, 1, 1)
    assert plan.bucket(0, 0).s1 == n
    bf16, f32 = torch.bfloat16, torch.float32
    g = hzp_inputs.device_normal(n, 1e-3, 41, DEV, bf16, None, 0)
    p = hzp_inputs.device_normal(n, 0.02, 43, DEV, f32, None, 0)
    m, v = torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    out = torch.zeros(n, dtype=bf16, device=DEV)
    rng = np.random.default_rng(9)
    marks = [k * 300000 * 512 for k in range(1, 7)] + [1 << 26, 1 << 27, 1 << 28, 1 << 29, 3 << 28]
    idx = np.unique(np.concatenate([np.arange(1024), np.arange(n - 1024, n), rng.integers(0, n, size=8192)] +
                                   [np.arange(c - 600, c + 600) for c in marks]))
    ti = torch.from_numpy(idx).to(DEV)
    s = dict(g=to_host(_bits16(g)[ti], np.uint16), p=to_host(p[ti], np.float32).copy(),
             m=np.zeros(idx.size, np.float32), v=np.zeros(idx.size, np.float32))
    a = hzp_inputs.ADAMW
    hy = hzp.adamw_hyper(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"], 1.0, 1)
    hzp.hzp_adamw_shard(plan, 0, 1, 0, 0, hy, [g], 1, [p], [m], [v], [out])
    torch.cuda.synchronize()
    on.adamw(on.reduce([s["g"]], scale=1.0), s["p"], s["m"], s["v"], step=1, **a)
    for key, t in (("p", p), ("m", m), ("v", v)):
        assert_close_f32(to_host(t[ti], np.float32), s[key], "longest shard " + key, key)
    assert_cast_of(to_host(_bits16(out)[ti], np.uint16), to_host(p[ti], np.float32), "longest shard bf16")
    # every element was updated: m = 0.1 g exactly where g is finite, so m is zero only where g is
    assert int((m == 0).sum().item()) == int((g == 0).sum().item())
    # stand-alone reduction of two slices of that length into v's buffer, bit for bit on the samples;
    # the whole output against the same sum formed by the library of the tensors' operations
    hzp.hzp_reduce_shard(plan, 0, 0, 1, 0, [g, out], 0.5, False, v)
    torch.cuda.synchronize()
    want = on.reduce([s["g"], to_host(_bits16(out)[ti], np.uint16)], scale=0.5)
    assert np.array_equal(to_host(v[ti], np.uint32), want.view(np.uint32))
    m.copy_(g)                              # exact in fp32: bf16 values and their sum of two, then one rounding by 0.5
    m.add_(out)
    m.mul_(0.5)
    assert torch.equal(v, m)
    del m, p
    # two shards of that length gathered into one bucket of 2^31 - 1024 elements
    plan2 = hzp.hzp_plan([1], [2 * n], 8, 2, 2)
    assert plan2.bucket(0, 0).s3 == n
    bucket = torch.empty(2 * n, dtype=torch.int16, device=DEV)
    hzp.hzp_gather_layer(plan2, 0, 0, 3, [g, out], bucket, None)
    torch.cuda.synchronize()
    assert torch.equal(bucket[:n], _bits16(g)) and torch.equal(bucket[n:], _bits16(out))
    tail, head = to_host(_bits16(g)[n - 64:], np.uint16).copy(), to_host(_bits16(out)[:64], np.uint16).copy()
    assert np.array_equal(to_host(bucket[n - 64:n + 64], np.uint16), on.gather_concat([tail, head]))


@pytest.mark.parametrize("R", [4, 16])
def test_fp32_class_at_size_over_several_launches(R):
    """Buckets of class F32 (fp32 gradients in, fp32 parameters out) at large shapes: three layers of
    40, 70 and 170 M elements in one call (the last one longer than a launch), per-tensor decay
    multipliers, two steps; sampled against the oracle at the ends, around the cuts and at random."""
    sizes = [40_000_000 + 8, 70_000_000 + 24, 170_000_000]
    say("fp32 class at size, R=%d" % R)
    gc.collect()
    torch.cuda.empty_cache()
    plan = hzp.hzp_plan([1, 1, 1], sizes, 8, 1, 1, tensor_class=[1, 1, 1], tensor_wd_mult=[1.0, 0.0, 0.5])
    f32 = torch.float32
    rng = np.random.default_rng(17 + R)
    a = hzp_inputs.ADAMW
    g, p, m, v, out, samples = [], [], [], [], [], []
    for l, n in enumerate(sizes):
        assert plan.bucket(l, 1).s1 == n
        gl = [hzp_inputs.device_normal(n, 1e-3, 500 + 31 * l + r, DEV, f32, None, 0) for r in range(R)]
        g += gl
        p.append(hzp_inputs.device_normal(n, 0.02, 900 + l, DEV, f32, None, 0))
        m.append(torch.zeros(n, device=DEV)); v.append(torch.zeros(n, device=DEV)); out.append(torch.zeros(n, device=DEV))
        cuts = [c for c in (300000 * 512,) if c < n]
        idx = np.unique(np.concatenate([np.arange(1024), np.arange(n - 1024, n), rng.integers(0, n, size=6000)] +
                                       [np.arange(c - 600, c + 600) for c in cuts]))
        ti = torch.from_numpy(idx).to(DEV)
        samples.append(dict(ti=ti, g=[to_host(x[ti], np.float32).copy() for x in gl], p=to_host(p[l][ti], np.float32).copy(),
                            m=np.zeros(idx.size, np.float32), v=np.zeros(idx.size, np.float32),
                            wd=np.full(idx.size, [1.0, 0.0, 0.5][l], np.float32)))
    for step in (1, 2):
        hy = hzp.adamw_hyper(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"], 1.0 / R, step)
        hzp.hzp_adamw_shard(plan, 0, 3, 1, 0, hy, g, R, p, m, v, out)
        torch.cuda.synchronize()
        for l, s in enumerate(samples):
            on.adamw(on.reduce(s["g"], scale=1.0 / R), s["p"], s["m"], s["v"], step=step, wd_mult=s["wd"], out_bf16=False, **a)
            for key, t in (("p", p[l]), ("m", m[l]), ("v", v[l])):
                assert_close_f32(to_host(t[s["ti"]], np.float32), s[key], "fp32 class layer %d step %d %s" % (l, step, key), key)
            assert torch.equal(out[l], p[l]), "fp32 output is the parameters themselves"


def test_accumulation_flow_at_size():
    """fp32 contributions of two micro-batches accumulated into resident fp32 gradient shards of 100 and
    170 M elements (R = 8 per micro-batch), then the update from those shards (the R == 0 form) over
    several launches; accumulator sampled bit for bit, update sampled within tolerance."""
    sizes = [100_000_000 + 40, 170_000_000]
    R, M = 8, 2
    say("accumulation flow at size")
    gc.collect()
    torch.cuda.empty_cache()
    plan = hzp.hzp_plan([1, 1], sizes, 8, 1, 1)
    f32 = torch.float32
    rng = np.random.default_rng(23)
    a = hzp_inputs.ADAMW
    acc, p, m, v, out, samples = [], [], [], [], [], []
    for l, n in enumerate(sizes):
        acc.append(torch.full((n,), 3.0, device=DEV))
        p.append(hzp_inputs.device_normal(n, 0.02, 700 + l, DEV, f32, None, 0))
        m.append(torch.zeros(n, device=DEV)); v.append(torch.zeros(n, device=DEV))
        out.append(torch.zeros(n, dtype=torch.int16, device=DEV))
        cuts = [c for c in (300000 * 512,) if c < n]
        idx = np.unique(np.concatenate([np.arange(1024), np.arange(n - 1024, n), rng.integers(0, n, size=6000)] +
                                       [np.arange(c - 600, c + 600) for c in cuts]))
        samples.append(dict(ti=torch.from_numpy(idx).to(DEV), acc=np.zeros(idx.size, np.float32),
                            p=to_host(p[l][torch.from_numpy(idx).to(DEV)], np.float32).copy(),
                            m=np.zeros(idx.size, np.float32), v=np.zeros(idx.size, np.float32)))
    for mb in range(M):
        for l, n in enumerate(sizes):
            g = [hzp_inputs.device_normal(n, 1e-3, 3000 + 100 * mb + 10 * l + r, DEV, f32, None, 0) for r in range(R)]
            hzp.hzp_reduce_shard(plan, l, 0, 1, 0, g, 1.0 / R, mb > 0, acc[l], grad_dtype=hzp.HZP_GRAD_F32)
            torch.cuda.synchronize()
            s = samples[l]
            on.reduce([to_host(x[s["ti"]], np.float32).copy() for x in g], scale=1.0 / R, accumulate=(mb > 0), out=s["acc"])
            assert np.array_equal(to_host(acc[l][s["ti"]], np.uint32), s["acc"].view(np.uint32)), (mb, l)
            del g
    hy = hzp.adamw_hyper(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"], 1.0 / M, 1)
    hzp.hzp_adamw_shard(plan, 0, 2, 0, 0, hy, acc, 0, p, m, v, out)
    torch.cuda.synchronize()
    for l, s in enumerate(samples):
        on.adamw(on.reduce([s["acc"]], scale=1.0 / M), s["p"], s["m"], s["v"], step=1, **a)
        for key, t in (("p", p[l]), ("m", m[l]), ("v", v[l])):
            assert_close_f32(to_host(t[s["ti"]], np.float32), s[key], "accumulated layer %d %s" % (l, key), key)
        assert_cast_of(to_host(out[l][s["ti"]], np.uint16), to_host(p[l][s["ti"]], np.float32), "accumulated layer %d bf16" % l)


def test_scheduler_at_layer_size():
    """Ten 7B-class layers (405 MB buckets) through a three-slot pool, prefetched two ahead from the
    background thread; then the same at parameter granularity (9 regions per layer) with one call per
    layer.  Every gathered bucket and tensor is compared on the device with the shards it came from."""
    say("scheduler at layer size")
    cfg = hzp_inputs.config(1)
    gc.collect()
    torch.cuda.empty_cache()
    n = 10
    w = bench.Workload(cfg, n, cfg["z3"] + 1, torch, hzp, hzp_inputs, arena_variant="0")
    consumer = torch.cuda.Stream()
    torch.cuda.synchronize()
    whole = [torch.cat([_bits16(x) for x in w.keep[l][7]]) for l in range(n)]        # what each bucket must hold

    class View:
        def __init__(self, ptr, count):
            self.__cuda_array_interface__ = {"shape": (count,), "typestr": "<i2", "data": (ptr, False), "version": 3}

    ok = torch.ones((), dtype=torch.bool, device=DEV)
    sched = hzp.Sched(w.plan, gather_slots=3, queue_capacity=8)
    for l in range(2):
        sched.prefetch(l, w.l3_args[l][1], consumer.cuda_stream)
    for l in range(n):
        ptr = sched.acquire(l, consumer.cuda_stream)
        with torch.cuda.stream(consumer):
            ok &= torch.equal(torch.as_tensor(View(ptr, whole[l].numel()), device=DEV), whole[l])
        sched.release(l, consumer.cuda_stream)
        if l + 2 < n:
            sched.prefetch(l + 2, w.l3_args[l + 2][1], consumer.cuda_stream)
    consumer.synchronize()
    sched.drain()
    assert bool(ok.item()) and sched.stats().gathers_issued == n
    sched.destroy()
    # parameter granularity, one call per layer
    per_layer = max(b.n_tensors for b in w.buckets)
    layer_bytes = max(2 * b.padded + 256 * b.n_tensors for b in w.buckets)
    sched = hzp.Sched(w.plan, gather_slots=3 * per_layer, queue_capacity=6 * per_layer + 4, pool_bytes=3 * ((layer_bytes + 255) // 256 * 256))
    first = [0]
    for b in w.buckets:
        first.append(first[-1] + b.n_tensors)
    for l in range(2):
        sched.prefetch_params(l, w.l3_args[l][1], consumer.cuda_stream)
    for l in range(n):
        ptrs = sched.acquire_params(l, w.buckets[l].n_tensors, consumer.cuda_stream)
        with torch.cuda.stream(consumer):
            for t, ptr in zip(range(first[l], first[l + 1]), ptrs):
                rec = w.plan.tensor(t)
                ok &= torch.equal(torch.as_tensor(View(ptr, rec.numel), device=DEV), whole[l][rec.offset:rec.offset + rec.numel])
        sched.release_params(l, consumer.cuda_stream)
        if l + 2 < n:
            sched.prefetch_params(l + 2, w.l3_args[l + 2][1], consumer.cuda_stream)
    consumer.synchronize()
    sched.drain()
    assert bool(ok.item()) and sched.stats().gathers_issued == first[n]
    sched.destroy()


def test_moe_layer_sampled_and_unpacked():
    """One MoE layer: S1 = 71.4M elements at R = 16, then unpack into its 199 tensors."""
    w = _fused_sampled_parity(3, 1, steps=1)
    b = w.buckets[0]
    assert b.s1 == 71385088 and b.n_tensors == 199
    grads, p, m, v, out, owners, shard3, shards, bucket = w.keep[0]
    pool = torch.zeros(int(b.payload_end) + 8, dtype=torch.int16, device=DEV)
    views, pos = [], 3                      # element-aligned only
    recs = [w.plan.tensor(t) for t in range(199)]
    for rec in recs:
        views.append(pool[pos:pos + rec.numel])
        pos += rec.numel
    hzp.hzp_gather_layer(w.plan, 0, 0, 3, shards, None, views)
    torch.cuda.synchronize()
    bb = _bits16(bucket)
    for rec, view in zip(recs, views):
        assert torch.equal(view, bb[rec.offset:rec.offset + rec.numel]), rec.offset
    # oracle on sampled windows of three tensors (first, one that straddles a shard seam, last)
    s3 = int(b.s3)
    host_shards = [to_host(_bits16(s), np.uint16) for s in shards]
    straddlers = [r for r in recs if r.offset // s3 != (r.offset + r.numel - 1) // s3]
    assert straddlers
    for rec in [recs[0], straddlers[0], recs[-1]]:
        tid = recs.index(rec)
        seam = (rec.offset // s3 + 1) * s3 - rec.offset - 40       # 40 elements before a shard seam
        for start in (0, seam, rec.numel - 80):
            start = int(min(max(start, 0), rec.numel - 80))
            want = on.unpack_tensor(host_shards, int(rec.offset) + start, 80)
            got = to_host(views[tid][start:start + 80], np.uint16)
            assert np.array_equal(got, want), (tid, start)
    assert not to_host(pool[:3], np.uint16).any() and not to_host(pool[pos:], np.uint16).any()


def test_irregular_4096_tensors_full():
    """The irregular stress workload in full: 64 groups x (bf16 + fp32 bucket), per-tensor decay
    multipliers, R = 16, one rank, two steps, every element compared; then all 4096 tensors are
    unpacked to element-aligned buffers and compared with the oracle bit for bit."""
    cfg = hzp_inputs.config(4)
    say("irregular workload: building both sides")
    sim = Sim(cfg, cfg["align"], cfg["z3"], cfg["z1"], cfg["R"], cfg["sigma"], seed=0, ranks=[cfg["z3"] + 1])
    assert len(sim.oplan["buckets"]) == 128
    for t in (1, 2):
        say("irregular workload step", t)
        sim.step(t)
        sim.compare("irregular step %d" % t)
    oplan, plan = sim.oplan, sim.plan
    rng = np.random.default_rng(15)
    for bi, b in enumerate(oplan["buckets"]):
        np_dt, t_dt = (np.uint32, torch.int32) if b["cls"] == 1 else (np.uint16, torch.int16)
        hi = 1 << (8 * np.dtype(np_dt).itemsize)
        bucket = rng.integers(0, hi, size=b["P"], dtype=np.uint64).astype(np_dt)
        S3 = b["S3"]
        shards = [np.ascontiguousarray(bucket[jj * S3:(jj + 1) * S3]) for jj in range(oplan["z3"])]
        total = sum(oplan["tensors"][t]["numel"] for t in b["tensor_ids"])
        pool = torch.zeros(total + 2, dtype=t_dt, device=DEV)
        views, pos = [], 1
        for t in b["tensor_ids"]:
            n = oplan["tensors"][t]["numel"]
            views.append(pool[pos:pos + n])
            pos += n
        full = torch.empty(b["P"], dtype=t_dt, device=DEV)
        hzp.hzp_gather_layer(plan, b["layer"], b["cls"], 3, [to_dev(s) for s in shards], full, views)
        torch.cuda.synchronize()
        want = np.concatenate([on.unpack_tensor(shards, oplan["tensors"][t]["offset"], oplan["tensors"][t]["numel"])
                               for t in b["tensor_ids"]])
        got = to_host(pool, np_dt)
        assert np.array_equal(got[1:1 + total], want), bi
        assert got[0] == 0 and got[1 + total] == 0
        assert np.array_equal(to_host(full, np_dt), on.gather_concat(shards)), bi


def test_free_group_gather_at_dense7b_size_as_benchmarked():
    """`bench.py --secondary freegroups`: the dense7b layers under Z1 = 12, Z3 = 8, ZeRO-3 shard 1 of
    every layer rebuilt from one partial and one whole ZeRO-1 shard.  Whole output against the
    device's own slices; oracle-computed windows at both ends and at the seam between the owners."""
    cfg = hzp_inputs.config(1)
    n_layers = 4
    w = bench.Workload(cfg, n_layers, cfg["z3"] + 1, torch, hzp, hzp_inputs)
    bench.add_secondary_buffers(w, ["freegroups"])
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()            # the buffers were filled on the default stream
    say("free-group gather at dense7b size, Z1=%d" % w.free_z1)
    bench.run_secondary(w, hzp, stream, "freegroups")
    stream.synchronize()
    tpl = cfg["tensors_per_layer"][:n_layers]
    oplan = op.make_plan(tpl, cfg["tensor_numel"][:sum(tpl)], cfg["align"], cfg["z3"], w.free_z1)
    for (l, _, dst, owners), ob in zip(w.free_args, oplan["buckets"]):
        cover = op.cover(oplan, ob, 1)
        assert len(cover) == len(owners) == 2 and w.free_plan.cover(l, 0, 1) == (cover[0][0], 2)
        parts = [_bits16(o)[src:src + n] for o, (_, src, _, n) in zip(owners, cover)]
        assert torch.equal(_bits16(dst), torch.cat(parts)), l
        S1, S3 = ob["S1"], ob["S3"]
        first = cover[0][0]
        for x0 in (0, cover[1][2] - 40, S3 - 80):                         # start, owner seam, end
            want = [0] * 80
            for x in range(x0, x0 + 80):                                   # the definition, element by element
                pos = S3 + x
                i = pos // S1
                want[x - x0] = int(to_host(_bits16(owners[i - first])[pos - i * S1:pos - i * S1 + 1], np.uint16)[0])
            got = to_host(_bits16(dst)[x0:x0 + 80], np.uint16)
            assert got.tolist() == want, (l, x0)


def test_single_parameter_gather_at_dense7b_size():
    """One 11008 x 4096 projection that straddles ZeRO-3 shards, gathered on its own."""
    cfg = hzp_inputs.config(1)
    w = bench.Workload(cfg, 3, cfg["z3"] + 1, torch, hzp, hzp_inputs)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()            # the buffers were filled on the default stream
    bench.run_step(w, hzp, 1, stream, {"gather3"})         # fills the layer buckets from the same shards
    layer = 1
    grads, p, m, v, out, owners, shard3, shards, bucket = w.keep[layer]
    b = w.buckets[layer]
    first_tid = sum(cfg["tensors_per_layer"][:layer])
    recs = [w.plan.tensor(first_tid + t) for t in range(b.n_tensors)]
    big = [r for r in recs if r.numel == 11008 * 4096 and r.offset // b.s3 != (r.offset + r.numel - 1) // b.s3]
    assert big
    rec = big[0]
    tid = first_tid + recs.index(rec)
    say("gather_tensor at full size: tensor %d, %d elements" % (tid, rec.numel))
    j0, j1 = rec.offset // b.s3, (rec.offset + rec.numel - 1) // b.s3
    ptrs = [shards[j] if j0 <= j <= j1 else None for j in range(w.z3)]
    pool = torch.zeros(rec.numel + 9, dtype=torch.int16, device=DEV)
    view = pool[5:5 + rec.numel]
    torch.cuda.synchronize()            # pool was cleared on the default stream
    hzp.hzp_gather_tensor(w.plan, tid, ptrs, view, stream=stream.cuda_stream)
    stream.synchronize()
    assert torch.equal(view, _bits16(bucket)[rec.offset:rec.offset + rec.numel])
    host_shards = [to_host(_bits16(s), np.uint16) for s in shards]
    seam = (j0 + 1) * b.s3 - rec.offset
    for start in (0, seam - 40, rec.numel - 80):
        want = on.unpack_tensor(host_shards, int(rec.offset) + int(start), 80)
        assert np.array_equal(to_host(view[start:start + 80], np.uint16), want), start
    assert not to_host(pool[:5], np.uint16).any() and not to_host(pool[5 + rec.numel:], np.uint16).any()
