"""Kernels beside a busy second stream, and calls that must not allocate.

Every kernel of the library stores through one hand-written 16-byte write-through store whose
data-register hazard the compiler cannot see.  A too-short wait after it once corrupted stores,
and only while another kernel kept the store pipeline backed up.  These tests run the fused
update, the layer-range gather and the unpack beside a stream that is kept busy with large copies
and compare with the oracle exactly as the quiet parity tests do.
"""
import threading

import numpy as np
import pytest
import torch

import hzp_inputs
import paper_2510_20111_amd as hzp
from oracle import numeric as on
from oracle import planner as op

from gpu_util import DEV, assert_cast_of, assert_close_f32, oracle_plan, to_dev, to_host
from test_gpu_parity import HP, lib_plan, say

pytestmark = pytest.mark.gpu


class Busy:
    """A second stream kept full of 256 MiB copies (store traffic) until stop()."""

    def __init__(self):
        self.stream = torch.cuda.Stream()
        self.a = torch.empty(64 << 20, dtype=torch.float32, device=DEV).normal_()
        self.b = torch.empty_like(self.a)
        self._stop = False
        torch.cuda.synchronize()
        self.thread = threading.Thread(target=self._run)
        self.thread.start()

    def _run(self):
        with torch.cuda.stream(self.stream):
            while not self._stop:
                for _ in range(8):
                    self.b.copy_(self.a)
                self.stream.synchronize()       # bounded queue: at most 8 copies ahead

    def stop(self):
        self._stop = True
        self.thread.join()
        self.stream.synchronize()


@pytest.fixture
def busy():
    b = Busy()
    yield b
    b.stop()


def test_fused_update_beside_a_busy_stream(busy):
    say("fused update under load")
    R, rounds = 8, 6
    desc = dict(tensors_per_layer=[1] * 6, tensor_numel=[400000 + 8 * 517 * l for l in range(6)])
    oplan, plan = oracle_plan(desc, 8, 1, 1), lib_plan(desc, 8, 1, 1)
    rng = np.random.default_rng(80)
    host, dev = [], []
    for b in oplan["buckets"]:
        n = b["S1"]
        h = dict(g=[hzp_inputs.to_bf16_bits((rng.standard_normal(n) * 1e-3).astype(np.float32)) for _ in range(R)],
                 p=(rng.standard_normal(n) * 0.02).astype(np.float32), m=np.zeros(n, np.float32), v=np.zeros(n, np.float32))
        host.append(h)
        dev.append(dict(g=[to_dev(x) for x in h["g"]], p=to_dev(h["p"]), m=to_dev(h["m"]), v=to_dev(h["v"]),
                        out=torch.zeros(n, dtype=torch.int16, device=DEV)))
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    for step in range(1, rounds + 1):
        hy = hzp.adamw_hyper(HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], 1.0 / R, step)
        hzp.hzp_adamw_shard(plan, 0, 6, 0, 0, hy, [x for d in dev for x in d["g"]], R, [d["p"] for d in dev],
                            [d["m"] for d in dev], [d["v"] for d in dev], [d["out"] for d in dev], stream=side)
        side.synchronize()
        for layer, (h, d) in enumerate(zip(host, dev)):
            on.adamw(on.reduce(h["g"], scale=1.0 / R), h["p"], h["m"], h["v"], step=step, **HP)
            for key in ("p", "m", "v"):
                assert_close_f32(to_host(d[key], np.float32), h[key], "step %d layer %d %s" % (step, layer, key), key)
            assert_cast_of(to_host(d["out"], np.uint16), to_host(d["p"], np.float32), "step %d layer %d bf16" % (step, layer))


def test_gathers_and_unpack_beside_a_busy_stream(busy):
    say("layer-range gather, unpack and single-parameter gather under load")
    z3, K = 4, 2
    desc = hzp_inputs.irregular_desc(40, seed=81, max_numel=120000, tensors_per_layer=8, f32_every=0)
    desc = dict(desc, tensor_class=None, tensor_wd_mult=None)
    oplan, plan = oracle_plan(desc, 8, z3, z3 * K), lib_plan(desc, 8, z3, z3 * K)
    plan.prepare()
    rng = np.random.default_rng(82)
    side = torch.cuda.Stream()
    n_layers = len(oplan["buckets"])
    buckets = [rng.integers(0, 1 << 16, size=b["P"], dtype=np.uint64).astype(np.uint16) for b in oplan["buckets"]]
    # level 1 for all layers in one launch: ZeRO-3 shard 1 of every layer from its K owners
    owners = [[np.ascontiguousarray(bk[(1 * K + k) * b["S1"]:(1 * K + k + 1) * b["S1"]]) for k in range(K)]
              for bk, b in zip(buckets, oplan["buckets"])]
    downers = [[to_dev(o) for o in layer] for layer in owners]
    dshard1 = [torch.zeros(b["S3"], dtype=torch.int16, device=DEV) for b in oplan["buckets"]]
    shards = [[np.ascontiguousarray(bk[j * b["S3"]:(j + 1) * b["S3"]]) for j in range(z3)] for bk, b in zip(buckets, oplan["buckets"])]
    dshards = [[to_dev(s) for s in layer] for layer in shards]
    touts = [[torch.zeros(oplan["tensors"][t]["numel"] + 3, dtype=torch.int16, device=DEV) for t in b["tensor_ids"]]
             for b in oplan["buckets"]]
    torch.cuda.synchronize()
    for rnd in range(4):
        hzp.hzp_gather_layers(plan, 0, n_layers, 0, 1, [x for layer in downers for x in layer], K, dshard1, stream=side)
        for l in range(n_layers):
            hzp.hzp_gather_layer(plan, l, 0, 3, dshards[l], None, [t[1:1 + t.numel() - 3] for t in touts[l]], stream=side)
        side.synchronize()
        for l, b in enumerate(oplan["buckets"]):
            assert np.array_equal(to_host(dshard1[l], np.uint16), on.gather_concat(owners[l])), (rnd, l)
            assert np.array_equal(to_host(dshard1[l], np.uint16), shards[l][1])
            for t, tout in zip(b["tensor_ids"], touts[l]):
                rec = oplan["tensors"][t]
                got = to_host(tout, np.uint16)
                assert np.array_equal(got[1:1 + rec["numel"]], on.unpack_tensor(shards[l], rec["offset"], rec["numel"])), (rnd, t)
                assert got[0] == 0 and not got[1 + rec["numel"]:].any()
        for l in range(n_layers):
            dshard1[l].zero_()
            for t in touts[l]:
                t.zero_()
        torch.cuda.synchronize()


def test_after_prepare_no_call_allocates(busy):
    """hzp_plan_prepare creates the device tables; afterwards the calls that read them (unpacking
    gathers, the update with per-tensor decay multipliers) take no device memory, also while another
    stream is busy.  Without it the first such call does."""
    say("hzp_plan_prepare")
    # many tensors, so that the tables are several MiB and show in the device's free memory (the
    # runtime serves small allocations from chunks it already holds)
    desc = hzp_inputs.irregular_desc(400000, seed=83, max_numel=40, tensors_per_layer=200000)
    args = (desc["tensors_per_layer"], desc["tensor_numel"], 8, 2, 2)
    kw = dict(tensor_class=desc["tensor_class"], tensor_wd_mult=desc["tensor_wd_mult"])
    oplan = oracle_plan(desc, 8, 2, 2)
    b = oplan["buckets"][0]
    rng = np.random.default_rng(84)
    bucket = rng.integers(0, 1 << 16, size=b["P"], dtype=np.uint64).astype(np.uint16)
    shards = [np.ascontiguousarray(bucket[j * b["S3"]:(j + 1) * b["S3"]]) for j in range(2)]
    dsh = [to_dev(s) for s in shards]
    t0 = b["tensor_ids"][0]
    rec = oplan["tensors"][t0]
    out = torch.zeros(rec["numel"], dtype=torch.int16, device=DEV)
    n = b["S1"]
    g = [torch.zeros(n, dtype=torch.int16, device=DEV)]
    p, m, v = (torch.zeros(n, device=DEV) for _ in range(3))
    po = torch.zeros(n, dtype=torch.int16, device=DEV)
    hy = hzp.adamw_hyper(HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], 1.0, 1)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()

    def free_bytes():
        return torch.cuda.mem_get_info()[0]

    def calls(plan):
        hzp.hzp_gather_tensor(plan, t0, dsh, out, stream=side)
        hzp.hzp_adamw_shard(plan, 0, 1, 0, 0, hy, g, 1, [p], [m], [v], [po], stream=side)

    plan = hzp.hzp_plan(*args, **kw)
    before = free_bytes()
    plan.prepare(side)
    after_prepare = free_bytes()
    assert after_prepare <= before - (8 << 20)         # the tables (about 25 MiB) were created here
    calls(plan)
    calls(plan)
    assert free_bytes() == after_prepare               # and nothing since
    side.synchronize()
    assert np.array_equal(to_host(out, np.uint16), on.unpack_tensor(shards, rec["offset"], rec["numel"]))
    plan.prepare(side)                                 # again: no effect
    assert free_bytes() == after_prepare
    # without prepare the first call creates them
    plan2 = hzp.hzp_plan(*args, **kw)
    before = free_bytes()
    calls(plan2)
    assert free_bytes() <= before - (8 << 20)
    side.synchronize()
