"""GPU parity for group sizes that do not nest (Section 4.1.1 leaves Z1, Z2, Z3 free): the
gradient-level reduction, the fused update on a ZeRO-1 shard that straddles ZeRO-3 shards, and the
post-step parameter gather from whole and partial ZeRO-1 shards, against the CPU oracle."""
import numpy as np
import pytest
import torch

import hzp_inputs
import paper_2510_20111_amd as hzp
from oracle import numeric as on
from oracle import planner as op

from gpu_util import (DEV, assert_cast_of, guarded, guards_intact, oracle_plan, payload_ranges,
                      to_dev, to_host)
from test_gpu_parity import Sim, lib_plan, op_rank_of_shard, say

pytestmark = pytest.mark.gpu

GROUPS = [(6, 2, 4), (2, 4, 4), (5, 3, 2), (8, 4, 2), (3, 3, 7), (12, 6, 8), (6, 2, 2)]


@pytest.mark.parametrize("z1,z2,z3", GROUPS)
def test_gather_shard_bit_exact(z1, z2, z3):
    say("gather_shard z1=%d z2=%d z3=%d" % (z1, z2, z3))
    desc = hzp_inputs.irregular_desc(12, seed=60 + z1, max_numel=120000, tensors_per_layer=6)
    oplan, plan = oracle_plan(desc, 8, z3, z1, z2), lib_plan(desc, 8, z3, z1, z2)
    rng = np.random.default_rng(61)
    assert max(b["S3"] for b in oplan["buckets"]) > 4 * 512          # several 64-lane tiles per piece
    for b in oplan["buckets"]:
        cls, S1, S3 = b["cls"], b["S1"], b["S3"]
        ndt, tdt = (np.uint32, torch.int32) if cls == 1 else (np.uint16, torch.int16)
        pieces = [rng.integers(0, np.iinfo(ndt).max, size=S1, dtype=np.uint64).astype(ndt) for _ in range(z1)]
        dpieces = [to_dev(x) for x in pieces]
        for j in range(z3):
            first, n = plan.cover(b["layer"], cls, j)
            cover = op.cover(oplan, b, j)
            assert (first, n) == (cover[0][0], len(cover))
            whole, out = guarded(S3, tdt)
            hzp.hzp_gather_shard(plan, b["layer"], cls, j, dpieces[first:first + n], out)
            torch.cuda.synchronize()
            want = on.gather_shard(pieces, j, z3)
            assert np.array_equal(to_host(out, ndt), want), (b["layer"], cls, j)
            assert guards_intact(whole, S3)


@pytest.mark.parametrize("z1,z2,z3", [(8, 4, 2), (6, 2, 4), (5, 3, 2)])
def test_reduce_on_the_gradient_shard(z1, z2, z3):
    say("reduce level 2, z1=%d z2=%d z3=%d" % (z1, z2, z3))
    desc = hzp_inputs.irregular_desc(6, seed=62, max_numel=40000, tensors_per_layer=3)
    oplan, plan = oracle_plan(desc, 8, z3, z1, z2), lib_plan(desc, 8, z3, z1, z2)
    R = 4
    for b in oplan["buckets"]:
        ranges = payload_ranges(oplan, b)
        full = [hzp_inputs.grad_bucket(7, 0, b["layer"], r, b["P"], ranges, 1e-3, b["cls"]) for r in range(R)]
        for rank in (0, oplan["world"] - 1, oplan["world"] // 2):
            beg, n = op.shard_range(oplan, b, 2, rank)
            assert n == b["S2"] and plan.shard(b["layer"], b["cls"], 2, rank) == (beg, n)
            slices = [np.ascontiguousarray(g[beg:beg + n]) for g in full]
            want = on.reduce(slices, scale=0.25)
            whole, out = guarded(n, torch.float32)
            hzp.hzp_reduce_shard(plan, b["layer"], b["cls"], 2, rank, [to_dev(s) for s in slices], 0.25, False, out)
            torch.cuda.synchronize()
            assert np.array_equal(to_host(out, np.uint32), want.view(np.uint32)), (b["layer"], rank)
            assert guards_intact(whole, n)


@pytest.mark.parametrize("z1,z2,z3", [(6, 2, 4), (5, 3, 2), (2, 4, 4)])
def test_update_then_regather_when_levels_do_not_nest(z1, z2, z3):
    """Every rank updates its ZeRO-1 shard (per-tensor decay multipliers, both classes), then each
    ZeRO-3 shard is rebuilt from the owners that meet it and the layer from the ZeRO-3 shards."""
    say("fused + regather z1=%d z2=%d z3=%d" % (z1, z2, z3))
    desc = hzp_inputs.irregular_desc(10, seed=63, max_numel=60000, tensors_per_layer=5)
    sim = Sim(desc, 8, z3, z1, 4, 1e-3, seed=9, z2=z2)
    for t in (1, 2):
        sim.step(t)
        sim.compare("free groups step %d" % t)
    oplan, plan = sim.oplan, sim.plan
    for bi, b in enumerate(oplan["buckets"]):
        cls = b["cls"]
        ndt, tdt = (np.uint32, torch.int32) if cls == 1 else (np.uint16, torch.int16)
        owner_out = [sim.d[bi, op_rank_of_shard(oplan, i)]["out"][1] for i in range(z1)]
        shards3 = []
        for j in range(z3):
            first, n = plan.cover(b["layer"], cls, j)
            dst = torch.empty(b["S3"], dtype=tdt, device=DEV)
            hzp.hzp_gather_shard(plan, b["layer"], cls, j, owner_out[first:first + n], dst)
            shards3.append(dst)
        full = torch.empty(b["P"], dtype=tdt, device=DEV)
        hzp.hzp_gather_layer(plan, b["layer"], cls, 3, shards3, full)
        torch.cuda.synchronize()
        got = to_host(full, ndt)
        assert np.array_equal(got, np.concatenate([to_host(o, ndt) for o in owner_out])), bi    # bit copies
        if cls == 0:        # the cast of the shards' fp32 parameters (checked against the oracle by sim.compare)
            p_all = np.concatenate([to_host(sim.d[bi, op_rank_of_shard(oplan, i)]["p"][1], np.float32) for i in range(z1)])
            assert_cast_of(got, p_all, "regathered bucket %d" % bi)
