"""The entry point that allocates nothing (hzp_gather_layer_static) against hzp_gather_layer.

Called through the C ABI on two buckets in a row, the second smaller than the first: the fixed
device array keeps the first call's table, and the second call must not be misled by what is
left of it.  Outputs are compared bit for bit with hzp_gather_layer's (whose table lives in
per-plan device memory) and with the oracle's unpack.
"""
import numpy as np
import pytest
import torch

import hzp_inputs
import paper_2510_20111_amd as hzp
from oracle import numeric as on
from gpu_util import DEV, oracle_plan, to_dev, to_host

pytestmark = pytest.mark.gpu


def say(msg):
    print("[no_alloc] " + msg, flush=True)


def _run_bucket(plan, oplan, b, rng, entry):
    """Unpack bucket `b` with `entry`; returns (outputs with guard bands, oracle's tensors)."""
    np_dt, t_dt = (np.uint32, torch.int32) if b["cls"] == 1 else (np.uint16, torch.int16)
    hi = 1 << (8 * np.dtype(np_dt).itemsize)
    z3 = oplan["z3"]
    bucket = rng.integers(0, hi, size=b["P"], dtype=np.uint64).astype(np_dt)
    shards = [np.ascontiguousarray(bucket[j * b["S3"]:(j + 1) * b["S3"]]) for j in range(z3)]
    dshards = [to_dev(s) for s in shards]
    outs = []
    for idx, t in enumerate(b["tensor_ids"]):
        numel = oplan["tensors"][t]["numel"]
        guard = 64 + (idx * 3) % 8          # element-aligned only
        w = torch.empty(numel + 2 * guard, dtype=t_dt, device=DEV)
        w.fill_(0x7FC1)
        outs.append((w, w[guard:guard + numel], guard))
    entry(plan, b["layer"], b["cls"], dshards, [o[1] for o in outs])
    torch.cuda.synchronize()
    want = [on.unpack_tensor(shards, oplan["tensors"][t]["offset"], oplan["tensors"][t]["numel"])
            for t in b["tensor_ids"]]
    got = [to_host(o[0], np_dt) for o in outs]
    return got, want, [o[2] for o in outs]


def _static(plan, layer, cls, shards, touts):
    hzp.hzp_gather_layer_static(plan, layer, cls, shards, touts)


def _dynamic(plan, layer, cls, shards, touts):
    hzp.hzp_gather_layer(plan, layer, cls, 3, shards, None, touts)


def _check_pair(plan, oplan, b, seed):
    got_s, want, guards = _run_bucket(plan, oplan, b, np.random.default_rng(seed), _static)
    got_d, want_d, _ = _run_bucket(plan, oplan, b, np.random.default_rng(seed), _dynamic)
    for t, (gs, gd, w, guard) in enumerate(zip(got_s, got_d, want, guards)):
        assert np.array_equal(gs, gd), "bucket layer %d: tensor %d differs from hzp_gather_layer" % (b["layer"], t)
        assert np.array_equal(gs[guard:guard + w.size], w), "bucket layer %d: tensor %d differs from the oracle" % (b["layer"], t)
        assert (gs[:guard] == 0x7FC1).all() and (gs[guard + w.size:] == 0x7FC1).all(), "guard band touched"


def test_static_table_entry_point_matches_gather_layer_on_two_calls_in_a_row():
    # first call: a bucket of 700 tensors (several argument-block launches of the table writer and two
    # of the unpack kernel); second call: a bucket of 5 tensors on another plan
    rng = np.random.default_rng(77)
    numel = [int(x) for x in rng.integers(1, 3000, size=700)]
    desc_big = dict(tensors_per_layer=[700], tensor_numel=numel)
    say("700 tensors, z3=4")
    oplan, plan = oracle_plan(desc_big, 8, 4, 8), hzp.hzp_plan(desc_big["tensors_per_layer"], numel, 8, 4, 8)
    _check_pair(plan, oplan, oplan["buckets"][0], 1)
    say("5 tensors, z3=2 (after the larger call)")
    desc_small = hzp_inputs.irregular_desc(5, seed=3, max_numel=9000, tensors_per_layer=5, f32_every=0)
    oplan2 = oracle_plan(desc_small, 16, 2, 4)
    plan2 = hzp.hzp_plan(desc_small["tensors_per_layer"], desc_small["tensor_numel"], 16, 2, 4)
    _check_pair(plan2, oplan2, oplan2["buckets"][0], 2)
    say("fp32-class bucket, then the first plan again")
    desc_f = hzp_inputs.irregular_desc(9, seed=5, max_numel=4000, tensors_per_layer=9, f32_every=2)
    oplan3 = oracle_plan(desc_f, 8, 2, 2)
    plan3 = hzp.hzp_plan(desc_f["tensors_per_layer"], desc_f["tensor_numel"], 8, 2, 2,
                         tensor_class=desc_f["tensor_class"], tensor_wd_mult=desc_f["tensor_wd_mult"])
    for b in oplan3["buckets"]:
        _check_pair(plan3, oplan3, b, 10 + b["cls"])
    _check_pair(plan, oplan, oplan["buckets"][0], 4)


def test_static_table_entry_point_refuses_more_pieces_than_the_table_holds():
    say("refusal above the fixed table's size")
    n = 4097
    plan = hzp.hzp_plan([n], [8] * n, 8, 1, 1)
    src = torch.zeros(8 * n, dtype=torch.int16, device=DEV)
    dst = torch.zeros(8 * n, dtype=torch.int16, device=DEV)
    with pytest.raises(hzp.HzpError) as ei:
        hzp.hzp_gather_layer_static(plan, 0, 0, [src], [dst[8 * t:8 * t + 8] for t in range(n)])
    assert ei.value.status == hzp.HZP_ERR_UNSUPPORTED and "4096" in str(ei.value)
    torch.cuda.synchronize()
    assert not dst.any()
    # exactly at the limit it runs
    n = 4096
    plan = hzp.hzp_plan([n], [8] * n, 8, 1, 1)
    src = torch.arange(8 * n, dtype=torch.int16, device=DEV)
    hzp.hzp_gather_layer_static(plan, 0, 0, [src], [dst[8 * t:8 * t + 8] for t in range(n)])
    torch.cuda.synchronize()
    assert torch.equal(dst[:8 * n], src)
