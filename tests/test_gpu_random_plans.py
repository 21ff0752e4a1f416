"""GPU parity on many small random plans (free group sizes, both classes, decay multipliers, tensors
from 1 element up): every kernel entry point against the oracle, with guard bands around every
output.  Seeded; the descriptors are drawn on the host."""
import numpy as np
import pytest
import torch

import hzp_inputs
import paper_2510_20111_amd as hzp
from oracle import numeric as on
from oracle import planner as op

from gpu_util import (DEV, assert_cast_of, assert_close_f32, guarded, guards_intact, payload_ranges,
                      to_dev, to_host, wd_mult_array)
from test_gpu_parity import say

pytestmark = pytest.mark.gpu
HP = hzp_inputs.ADAMW


def _draw(rng):
    n_layers = int(rng.integers(1, 4))
    tpl = [int(rng.integers(1, 6)) for _ in range(n_layers)]
    n = sum(tpl)
    kind = rng.integers(0, 3, size=n)
    numel = [int(rng.integers(1, 9)) if k == 0 else int(rng.integers(9, 700)) if k == 1 else int(rng.integers(700, 9000))
             for k in kind]
    return dict(tensors_per_layer=tpl, tensor_numel=numel,
                tensor_class=[int(x) for x in rng.integers(0, 2, size=n)] if rng.integers(0, 2) else None,
                tensor_wd_mult=[float(x) for x in rng.choice([0.0, 0.5, 1.0], size=n)] if rng.integers(0, 2) else None,
                align=int(rng.choice([8, 16, 64])), z1=int(rng.integers(1, 10)), z2=int(rng.integers(1, 7)),
                z3=int(rng.integers(1, 7)))


@pytest.mark.parametrize("seed", range(60))
def test_random_plan(seed):
    rng = np.random.default_rng(900 + seed)
    d = _draw(rng)
    say("random plan %d: %s" % (seed, {k: d[k] for k in ("tensors_per_layer", "align", "z1", "z2", "z3")}))
    args = (d["tensors_per_layer"], d["tensor_numel"], d["align"], d["z3"], d["z1"], d["z2"])
    kw = dict(tensor_class=d["tensor_class"], tensor_wd_mult=d["tensor_wd_mult"])
    oplan, plan = op.make_plan(*args, **kw), hzp.hzp_plan(*args, **kw)
    z1, z3, W = oplan["z1"], oplan["z3"], oplan["world"]
    R = int(rng.choice([1, 2, 3, 4, 5, 8]))
    rank = int(rng.integers(0, W))
    step = int(rng.integers(1, 4))
    hy = hzp.adamw_hyper(HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], 1.0 / R, step)
    for b in oplan["buckets"]:
        layer, cls, P = b["layer"], b["cls"], b["P"]
        ranges = payload_ranges(oplan, b)
        ndt, tdt = (np.uint32, torch.int32) if cls == 1 else (np.uint16, torch.int16)
        grads = [hzp_inputs.grad_bucket(seed, step, layer, r, P, ranges, 1e-3, cls) for r in range(R)]
        # reduce on every level
        for level in (1, 2, 3):
            beg, n = op.shard_range(oplan, b, level, rank)
            assert plan.shard(layer, cls, level, rank) == (beg, n)
            sl = [np.ascontiguousarray(g[beg:beg + n]) for g in grads]
            whole, out = guarded(n, torch.float32)
            hzp.hzp_reduce_shard(plan, layer, cls, level, rank, [to_dev(s) for s in sl], 1.0 / R, False, out)
            torch.cuda.synchronize()
            assert np.array_equal(to_host(out, np.uint32), on.reduce(sl, scale=1.0 / R).view(np.uint32)), (layer, level)
            assert guards_intact(whole, n)
        # fused update of the rank's ZeRO-1 shard
        beg, n = op.shard_range(oplan, b, 1, rank)
        p0 = np.ascontiguousarray(hzp_inputs.master_bucket(seed, layer, P, ranges, cls)[beg:beg + n])
        mask = hzp_inputs._payload_mask(n, ranges, beg)
        m0 = np.where(mask, rng.standard_normal(n) * 1e-3, 0).astype(np.float32)
        v0 = np.where(mask, rng.random(n) * 1e-6, 0).astype(np.float32)
        dev = {}
        for key, init in (("p", p0), ("m", m0), ("v", v0)):
            dev[key] = guarded(n, torch.float32)
            dev[key][1].copy_(to_dev(init))
        dev["out"] = guarded(n, torch.float32 if cls == 1 else torch.int16)
        sl = [np.ascontiguousarray(g[beg:beg + n]) for g in grads]
        hzp.hzp_adamw_shard(plan, layer, layer + 1, cls, rank, hy, [to_dev(s) for s in sl], R,
                            [dev["p"][1]], [dev["m"][1]], [dev["v"][1]], [dev["out"][1]])
        torch.cuda.synchronize()
        wd = wd_mult_array(oplan, b, beg, n) if d["tensor_wd_mult"] else None
        po, mo, vo = p0.copy(), m0.copy(), v0.copy()
        want_out = on.adamw(on.reduce(sl, scale=1.0 / R), po, mo, vo, step=step, wd_mult=wd, out_bf16=(cls == 0), **HP)
        for key, want in (("p", po), ("m", mo), ("v", vo)):
            assert_close_f32(to_host(dev[key][1], np.float32), want, "seed %d layer %d %s" % (seed, layer, key), key)
            assert guards_intact(dev[key][0], n)
        if cls == 0:
            assert_cast_of(to_host(dev["out"][1], np.uint16), to_host(dev["p"][1], np.float32), "seed %d layer %d bf16" % (seed, layer))
        else:
            assert np.array_equal(to_host(dev["out"][1], np.uint32), to_host(dev["p"][1], np.uint32))
        assert guards_intact(dev["out"][0], n)
        # gathers: ZeRO-1 pieces -> every ZeRO-3 shard -> bucket and tensors; one tensor alone
        pieces = [rng.integers(0, np.iinfo(ndt).max, size=b["S1"], dtype=np.uint64).astype(ndt) for _ in range(z1)]
        dpieces = [to_dev(x) for x in pieces]
        shards, dshards = [], []
        for j in range(z3):
            first, cnt = plan.cover(layer, cls, j)
            whole, out = guarded(b["S3"], tdt)
            hzp.hzp_gather_shard(plan, layer, cls, j, dpieces[first:first + cnt], out)
            torch.cuda.synchronize()
            want = on.gather_shard(pieces, j, z3)
            assert np.array_equal(to_host(out, ndt), want), (layer, j)
            assert guards_intact(whole, b["S3"])
            shards.append(want)
            dshards.append(out)
        wholeb, full = guarded(P, tdt)
        touts = [guarded(oplan["tensors"][t]["numel"], tdt, guard=8 + t % 3) for t in b["tensor_ids"]]
        hzp.hzp_gather_layer(plan, layer, cls, 3, dshards, full, [v for _, v in touts])
        torch.cuda.synchronize()
        assert np.array_equal(to_host(full, ndt), on.gather_concat(shards)) and guards_intact(wholeb, P)
        for t, (whole, view) in zip(b["tensor_ids"], touts):
            rec = oplan["tensors"][t]
            want = on.unpack_tensor(shards, rec["offset"], rec["numel"])
            assert np.array_equal(to_host(view, ndt), want), t
            assert guards_intact(whole, rec["numel"], guard=8 + t % 3)
            view.zero_()
            hzp.hzp_gather_tensor(plan, t, dshards, view)
            torch.cuda.synchronize()
            assert np.array_equal(to_host(view, ndt), want) and guards_intact(whole, rec["numel"], guard=8 + t % 3), t
