"""A whole step of the path (fused update of all layers, post-step gather, per-layer gather with
unpack) captured into a HIP graph and replayed: every replay must leave exactly what the same calls
issued eagerly leave, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import hzp_inputs
import paper_2510_20111_amd as hzp
from oracle import numeric as on
from oracle import planner as op

from gpu_util import DEV, assert_cast_of, assert_close_f32, oracle_plan, payload_ranges, to_dev, to_host, wd_mult_array

pytestmark = pytest.mark.gpu

HP = hzp_inputs.ADAMW


def say(*a):
    print(*a, flush=True)


class Rank:
    """One rank's buffers of a small plan with per-tensor decay multipliers (so that the update reads
    the plan's device tables) and the argument lists of a step."""

    def __init__(self, desc, oplan, plan, rank, R, seed):
        self.plan, self.oplan, self.rank, self.R = plan, oplan, rank, R
        j, k, i = op.rank_to_indices(oplan, rank)
        z3, K = oplan["z3"], oplan["K"]
        self.n_layers = oplan["n_layers"]
        rng = np.random.default_rng(seed)
        self.g, self.p, self.m, self.v, self.shard3, self.l1_src, self.l3 = [], [], [], [], [], [], []
        self.host = []
        for layer in range(self.n_layers):
            b = op.find_bucket(oplan, layer, 0)
            beg, n = op.shard_range(oplan, b, 1, rank)
            ranges = payload_ranges(oplan, b)
            p0 = np.ascontiguousarray(hzp_inputs.master_bucket(seed, layer, b["P"], ranges, 0)[beg:beg + n])
            gs = [np.ascontiguousarray(hzp_inputs.grad_bucket(seed, 1, layer, r, b["P"], ranges, 1e-3, 0)[beg:beg + n])
                  for r in range(R)]
            self.host.append(dict(p=p0, g=gs, wd=wd_mult_array(oplan, b, beg, n), n=n))
            self.g += [to_dev(x) for x in gs]
            self.p.append(to_dev(p0))
            self.m.append(torch.zeros(n, device=DEV))
            self.v.append(torch.zeros(n, device=DEV))
            shard3 = to_dev(rng.integers(0, 65536, b["S3"], dtype=np.uint16))
            self.shard3.append(shard3)
            own = shard3[k * n:(k + 1) * n]                       # the update writes here; the gather leaves it
            self.l1_src += [own if kk == k else to_dev(rng.integers(0, 65536, n, dtype=np.uint16)) for kk in range(K)]
            shards = [shard3 if jj == j else to_dev(rng.integers(0, 65536, b["S3"], dtype=np.uint16)) for jj in range(z3)]
            bucket = torch.zeros(b["P"], dtype=torch.int16, device=DEV)
            tensors = [torch.zeros(oplan["tensors"][t]["numel"], dtype=torch.int16, device=DEV) for t in b["tensor_ids"]]
            self.l3.append((layer, shards, bucket, tensors))
        self.k, self.K = k, K
        self.out = [self.shard3[l][k * self.host[l]["n"]:(k + 1) * self.host[l]["n"]] for l in range(self.n_layers)]
        self.hy = hzp.adamw_hyper(HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], 1.0 / R, 1)

    def step(self, stream):
        s = stream.cuda_stream
        hzp.hzp_adamw_shard(self.plan, 0, self.n_layers, 0, self.rank, self.hy, self.g, self.R, self.p, self.m, self.v,
                            self.out, stream=s)
        hzp.hzp_gather_layers(self.plan, 0, self.n_layers, 0, 1, self.l1_src, self.K, self.shard3, stream=s)
        for layer, shards, bucket, tensors in self.l3:
            hzp.hzp_gather_layer(self.plan, layer, 0, 3, shards, bucket, tensors, stream=s)

    def state(self):
        """Everything a step writes, as raw bits."""
        out = []
        for l in range(self.n_layers):
            out += [to_host(self.p[l], np.uint32), to_host(self.m[l], np.uint32), to_host(self.v[l], np.uint32),
                    to_host(self.shard3[l], np.uint16), to_host(self.l3[l][2], np.uint16)]
            out += [to_host(t, np.uint16) for t in self.l3[l][3]]
        return out


def test_a_captured_step_replays_to_the_eager_result():
    say("graph capture of a whole step")
    desc = hzp_inputs.irregular_desc(18, seed=404, max_numel=120000, tensors_per_layer=3, f32_every=0)
    desc = dict(desc, tensor_class=None, tensor_wd_mult=[(0.0, 1.0, 0.5)[i % 3] for i in range(18)])
    oplan = oracle_plan(desc, 8, 2, 8)
    plan = hzp.hzp_plan(desc["tensors_per_layer"], desc["tensor_numel"], 8, 2, 8, tensor_wd_mult=desc["tensor_wd_mult"])
    plan.prepare()                                  # device tables exist before the capture: no call allocates
    rank, R = 5, 3
    eager, graphed = Rank(desc, oplan, plan, rank, R, 12), Rank(desc, oplan, plan, rank, R, 12)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        graphed.step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    scratch = torch.empty(1 << 22, device=DEV)
    for replay in range(1, 4):
        eager.step(side)
        side.synchronize()
        scratch.normal_()                           # eager work of the program between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager.state(), graphed.state()):
            assert np.array_equal(a, b), "replay %d differs from the eager step" % replay
        if replay == 1:                              # and the first one against the oracle
            for l in range(eager.n_layers):
                h = eager.host[l]
                po, mo, vo = h["p"].copy(), np.zeros(h["n"], np.float32), np.zeros(h["n"], np.float32)
                on.adamw(on.reduce(h["g"], scale=1.0 / R), po, mo, vo, step=1, wd_mult=h["wd"], out_bf16=True, **HP)
                assert_close_f32(to_host(graphed.p[l], np.float32), po, "graph p layer %d" % l, "p")
                assert_close_f32(to_host(graphed.m[l], np.float32), mo, "graph m layer %d" % l, "m")
                assert_close_f32(to_host(graphed.v[l], np.float32), vo, "graph v layer %d" % l, "v")
                assert_cast_of(to_host(graphed.out[l], np.uint16), to_host(graphed.p[l], np.float32), "graph bf16 %d" % l)


def test_device_scalars_form_equals_the_host_form_bit_for_bit():
    """hzp_adamw_shard_dev reads the step's scalars from device memory; with the block hzp_adamw_scalars
    derives from the same hyper-parameters it must leave exactly what hzp_adamw_shard leaves: compile-time
    and run-time R, both classes, per-tensor decay, the pre-reduced form."""
    say("update with the scalars in device memory")
    desc = hzp_inputs.irregular_desc(20, seed=505, max_numel=50000, tensors_per_layer=5)
    oplan = oracle_plan(desc, 8, 2, 4)
    plan = hzp.hzp_plan(desc["tensors_per_layer"], desc["tensor_numel"], 8, 2, 4, tensor_class=desc["tensor_class"],
                        tensor_wd_mult=desc["tensor_wd_mult"])
    n_layers = oplan["n_layers"]
    rank = 3
    rng = np.random.default_rng(3)
    for cls in (0, 1):
        for R in (0, 1, 3, 4, 8, 16):
            if R == 0 and cls == 1:
                continue
            g32 = cls == 1 or R == 0
            state = {}
            for tag in ("host", "dev"):
                state[tag] = dict(g=[], p=[], m=[], v=[], o=[])
            for layer in range(n_layers):
                b = op.find_bucket(oplan, layer, cls)
                if b is None:
                    for tag in state:
                        state[tag]["g"] += [0] * max(R, 1)
                        for k in ("p", "m", "v", "o"):
                            state[tag][k].append(0)
                    continue
                _, n = op.shard_range(oplan, b, 1, rank)
                gs = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(max(R, 1))]
                if not g32:
                    gs = [hzp_inputs.to_bf16_bits(x) for x in gs]
                p0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
                m0 = (rng.standard_normal(n) * 1e-4).astype(np.float32)
                v0 = (rng.random(n) * 1e-7).astype(np.float32)
                for tag in state:
                    state[tag]["g"] += [to_dev(x) for x in gs]
                    state[tag]["p"].append(to_dev(p0)); state[tag]["m"].append(to_dev(m0)); state[tag]["v"].append(to_dev(v0))
                    state[tag]["o"].append(torch.zeros(n, dtype=torch.float32 if cls == 1 else torch.int16, device=DEV))
            for step in (1, 7):
                hy = hzp.adamw_hyper(HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], 0.25, step)
                scal = torch.tensor(hzp.hzp_adamw_scalars(hy), dtype=torch.float32, device=DEV)
                h, d = state["host"], state["dev"]
                hzp.hzp_adamw_shard(plan, 0, n_layers, cls, rank, hy, h["g"], R, h["p"], h["m"], h["v"], h["o"])
                hzp.hzp_adamw_shard_dev(plan, 0, n_layers, cls, rank, scal, d["g"], R, d["p"], d["m"], d["v"], d["o"])
                torch.cuda.synchronize()
                for k in ("p", "m", "v", "o"):
                    for a, b_ in zip(h[k], d[k]):
                        if not isinstance(a, int):
                            assert torch.equal(a.view(torch.int16), b_.view(torch.int16)), (cls, R, step, k)


def test_one_captured_step_replayed_as_successive_training_steps():
    """The step captured once with hzp_adamw_shard_dev; before each replay the next step's scalars are copied
    into the device block.  Three replays must equal three eager steps of hzp_adamw_shard with step = 1, 2, 3
    bit for bit (and the last one the oracle's three steps within tolerance)."""
    say("graph replays as successive steps")
    desc = hzp_inputs.irregular_desc(18, seed=404, max_numel=120000, tensors_per_layer=3, f32_every=0)
    desc = dict(desc, tensor_class=None, tensor_wd_mult=[(0.0, 1.0, 0.5)[i % 3] for i in range(18)])
    oplan = oracle_plan(desc, 8, 2, 8)
    plan = hzp.hzp_plan(desc["tensors_per_layer"], desc["tensor_numel"], 8, 2, 8, tensor_wd_mult=desc["tensor_wd_mult"])
    plan.prepare()
    rank, R = 5, 3
    eager, graphed = Rank(desc, oplan, plan, rank, R, 12), Rank(desc, oplan, plan, rank, R, 12)
    side = torch.cuda.Stream()
    scal = torch.zeros(12, dtype=torch.float32, device=DEV)
    staging = torch.zeros(12, dtype=torch.float32).pin_memory()

    def step_dev(r, stream):
        s = stream.cuda_stream
        hzp.hzp_adamw_shard_dev(r.plan, 0, r.n_layers, 0, r.rank, scal, r.g, r.R, r.p, r.m, r.v, r.out, stream=s)
        hzp.hzp_gather_layers(r.plan, 0, r.n_layers, 0, 1, r.l1_src, r.K, r.shard3, stream=s)
        for layer, shards, bucket, tensors in r.l3:
            hzp.hzp_gather_layer(r.plan, layer, 0, 3, shards, bucket, tensors, stream=s)

    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step_dev(graphed, torch.cuda.current_stream())
    torch.cuda.synchronize()
    host = [dict(p=h["p"].copy(), m=np.zeros(h["n"], np.float32), v=np.zeros(h["n"], np.float32)) for h in eager.host]
    for step in (1, 2, 3):
        hy = hzp.adamw_hyper(HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], 1.0 / R, step)
        eager.hy = hy
        eager.step(side)
        side.synchronize()
        staging.copy_(torch.tensor(hzp.hzp_adamw_scalars(hy), dtype=torch.float32))
        scal.copy_(staging, non_blocking=True)          # on the current stream; the replay below follows it there
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager.state(), graphed.state()):
            assert np.array_equal(a, b), "replay as step %d differs from the eager step" % step
        for l, h in enumerate(eager.host):
            on.adamw(on.reduce(h["g"], scale=1.0 / R), host[l]["p"], host[l]["m"], host[l]["v"], step=step, wd_mult=h["wd"],
                     out_bf16=True, **HP)
    for l in range(eager.n_layers):
        assert_close_f32(to_host(graphed.p[l], np.float32), host[l]["p"], "third replay p layer %d" % l, "p")
        assert_close_f32(to_host(graphed.m[l], np.float32), host[l]["m"], "third replay m layer %d" % l, "m")
        assert_close_f32(to_host(graphed.v[l], np.float32), host[l]["v"], "third replay v layer %d" % l, "v")
