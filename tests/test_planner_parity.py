"""The library's planner against the layout oracle, bit for bit (runs without a GPU)."""
import pytest
from hypothesis import given, settings, strategies as st

import hzp_inputs
import paper_2510_20111_amd as hzp
from oracle import planner as op


def _compare(d):
    want = op.make_plan(d["tensors_per_layer"], d["tensor_numel"], d["align"], d["z3"], d["z1"], d.get("z2", 0),
                        tensor_class=d.get("tensor_class"), tensor_wd_mult=d.get("tensor_wd_mult"))
    got = hzp.hzp_plan(d["tensors_per_layer"], d["tensor_numel"], d["align"], d["z3"], d["z1"], d.get("z2", 0),
                       tensor_class=d.get("tensor_class"), tensor_wd_mult=d.get("tensor_wd_mult"))
    info = got.info()
    assert (info.n_layers, info.n_buckets, info.n_tensors) == (
        want["n_layers"], len(want["buckets"]), len(want["tensors"]))
    assert (info.align_elems, info.z3, info.z2, info.z1, info.k, info.world, info.total_padded) == (
        want["align"], want["z3"], want["z2"], want["z1"], want["K"], want["world"], want["total_padded"])
    for layer in range(want["n_layers"]):
        for cls in (0, 1):
            wb = op.find_bucket(want, layer, cls)
            assert got.has_bucket(layer, cls) == (wb is not None)
    for idx, wb in enumerate(want["buckets"]):
        gb = got.bucket(wb["layer"], wb["cls"])
        assert (gb.layer, gb.cls, gb.n_tensors, gb.bucket_index, gb.payload_end, gb.padded, gb.s3,
                gb.s2, gb.s1, gb.base) == (wb["layer"], wb["cls"], len(wb["tensor_ids"]), idx,
                                           wb["payload_end"], wb["P"], wb["S3"], wb["S2"], wb["S1"], wb["base"])
        W = want["world"]
        ranks = range(W) if W <= 16 else [0, 1, want["z3"], want["z1"] - 1, W - 1]
        for rank in ranks:
            for level in (1, 2, 3):
                assert got.shard(wb["layer"], wb["cls"], level, rank) == \
                    op.shard_range(want, wb, level, rank)
        shards3 = range(want["z3"]) if want["z3"] <= 16 else [0, 1, want["z3"] - 1]
        for j in shards3:
            cover = op.cover(want, wb, j)
            assert got.cover(wb["layer"], wb["cls"], j) == (cover[0][0], len(cover))
            assert [c[0] for c in cover] == list(range(cover[0][0], cover[0][0] + len(cover)))
    W = want["world"]
    ranks = range(W) if W <= 64 else [0, 1, 7, 8, want["z1"] - 1, W - 1]
    for rank in ranks:
        assert got.rank(rank) == op.rank_to_indices(want, rank)
        for level in (1, 2, 3):
            assert got.index(level, rank) == op.level_index(want, level, rank)
    tensor_ids = range(len(want["tensors"])) if len(want["tensors"]) <= 300 else \
        list(range(0, len(want["tensors"]), 37)) + [len(want["tensors"]) - 1]
    for t in tensor_ids:
        wt, gt = want["tensors"][t], got.tensor(t)
        assert (gt.layer, gt.cls, gt.bucket_index, gt.offset, gt.numel, gt.wd_mult) == (
            wt["layer"], wt["cls"], wt["bucket"], wt["offset"], wt["numel"], wt["wd_mult"])
        assert want["buckets"][wt["bucket"]]["tensor_ids"][gt.index_in_bucket] == t
    assert got.bytes() == op.per_rank_bytes(want)


@st.composite
def descriptors(draw):
    n_layers = draw(st.integers(1, 5))
    tpl = [draw(st.integers(1, 6)) for _ in range(n_layers)]
    n = sum(tpl)
    numel = [draw(st.one_of(st.integers(1, 400), st.integers(1, 100000))) for _ in range(n)]
    cls = draw(st.one_of(st.none(), st.lists(st.integers(0, 1), min_size=n, max_size=n)))
    wd = draw(st.one_of(st.none(), st.lists(st.sampled_from([0.0, 1.0, 0.5]), min_size=n, max_size=n)))
    align = draw(st.sampled_from([8, 16, 64, 128, 256]))
    z3 = draw(st.sampled_from([1, 2, 3, 4, 8]))
    K = draw(st.sampled_from([1, 2, 4, 5, 16]))
    return dict(tensors_per_layer=tpl, tensor_numel=numel, tensor_class=cls, tensor_wd_mult=wd,
                align=align, z3=z3, z1=z3 * K)


@settings(max_examples=150, deadline=None)
@given(descriptors())
def test_random_descriptors(d):
    _compare(d)


@settings(max_examples=150, deadline=None)
@given(descriptors(), st.integers(1, 12), st.integers(1, 12), st.integers(1, 12))
def test_random_descriptors_with_free_group_sizes(d, z1, z2, z3):
    _compare(dict(d, z1=z1, z2=z2, z3=z3))


def test_group_sizes_whose_lcm_exceeds_32_bits_are_refused():
    import pytest
    with pytest.raises(hzp.HzpError) as e:
        hzp.hzp_plan([1], [8], 8, 65537, 65536, 65539)
    assert e.value.status == hzp.HZP_ERR_UNSUPPORTED
    hzp.hzp_plan([1], [8], 8, 1 << 20, 1 << 30, 1 << 10)         # lcm = 2^30 is fine


def test_the_five_workloads():
    for idx in range(5):
        _compare(hzp_inputs.config(idx))


def test_paper_group_sizes():
    """Z1 = 64 and 256 with Z2 = Z3 = 8, the settings of the paper's experiments (Tables 2-5)."""
    c = hzp_inputs.config(1)
    for z1 in (64, 256):
        _compare(dict(c, z1=z1, tensors_per_layer=c["tensors_per_layer"][:3],
                      tensor_numel=c["tensor_numel"][:27]))


def test_memory_model_matches_closed_form():
    """hzp_memory_model against the oracle's exact fraction and the hand-worked golden values."""
    import math
    import os
    from fractions import Fraction
    golden = os.path.join(os.path.dirname(__file__), "golden", "memory_model.txt")
    for line in open(golden):
        line = line.split("#")[0].split()
        if line:
            N, z1, z2, z3, want = (int(x) for x in line)
            assert hzp.hzp_memory_model(N, z1, z2, z3) == want
    for N, z1, z2, z3 in [(7, 3, 5, 2), (10 ** 12 + 1, 64, 8, 8), (1, 1, 1, 1), (0, 4, 4, 4),
                          (2 ** 60, 2 ** 31, 3, 7), (123456789, 256, 8, 8)]:
        assert hzp.hzp_memory_model(N, z1, z2, z3) == math.ceil(op.hzp_memory_bytes(N, z1, z2, z3))
    # the plan's per-rank bytes are the same model with N -> padded length
    c = hzp_inputs.config(1)
    plan = hzp.hzp_plan(c["tensors_per_layer"], c["tensor_numel"], c["align"], c["z3"], c["z1"])
    assert sum(plan.bytes()) == hzp.hzp_memory_model(plan.info().total_padded, c["z1"], c["z3"], c["z3"])
    import pytest
    with pytest.raises(hzp.HzpError):
        hzp.hzp_memory_model(5, 0, 1, 1)
    with pytest.raises(hzp.HzpError):
        hzp.hzp_memory_model(2 ** 63, 1, 1, 1)


def test_choose_groups_matches_the_oracle():
    import os
    import pytest
    golden = os.path.join(os.path.dirname(__file__), "golden", "choose_groups.txt")
    cases = []
    with open(golden) as f:
        for line in f:
            row = line.split("#")[0].split()
            if row:
                cases.append(tuple(int(x) for x in row[:4]))
    cases += [(12345, 48, 8, b) for b in range(0, 230000, 7919)]
    cases += [(10 ** 12, 4096, 8, b * 10 ** 9) for b in (1, 50, 800, 1600, 20000)]
    cases += [(999, 36, 6, b) for b in range(500, 19000, 613)] + [(0, 8, 8, 0), (5, 1, 8, 90), (5, 1, 8, 89)]
    for N, dp, node, budget in cases:
        want = op.choose_groups(N, dp, node, budget)
        if want is None:
            with pytest.raises(hzp.HzpError) as e:
                hzp.hzp_choose_groups(N, dp, node, budget)
            assert e.value.status == hzp.HZP_ERR_NOMEM
        else:
            assert hzp.hzp_choose_groups(N, dp, node, budget) == want, (N, dp, node, budget)
    for bad in [(5, 0, 8, 1), (5, 8, 0, 1)]:
        with pytest.raises(hzp.HzpError) as e:
            hzp.hzp_choose_groups(*bad)
        assert e.value.status == hzp.HZP_ERR_INVALID_ARG


# ------------------------------------------------------------------ arena layout

@given(desc=descriptors(), R=st.integers(0, 32), gd=st.sampled_from([0, 1, 2]),
       variant=st.integers(0, hzp.HZP_ARENA_VARIANTS - 1))
@settings(max_examples=160, deadline=None)
def test_arena_layout_matches_the_oracle(desc, R, gd, variant):
    oplan = op.make_plan(**desc)
    plan = hzp.hzp_plan(**desc)
    for cls in (0, 1):
        buckets = [b for b in oplan["buckets"] if b["cls"] == cls]
        if not buckets:
            with pytest.raises(hzp.HzpError) as e:
                plan.arena(cls, R, gd)
            assert e.value.status == hzp.HZP_ERR_RANGE
            continue
        gb = (4 if cls == 1 else 2) if gd == 0 else (4 if gd == 2 else 2)
        total, slices = op.arena_layout(oplan, cls, R, gb, variant)
        assert plan.arena(cls, R, gd, variant) == total
        for (kind, index, layer), want in slices.items():
            assert plan.arena_slice(cls, R, kind, index, layer, gd, variant) == want, (kind, index, layer)
        # indices one past the end of each stream are refused
        for kind, count in ((hzp.HZP_STREAM_GRAD, R), (hzp.HZP_STREAM_MASTER, 1), (hzp.HZP_STREAM_RECV3, oplan["z3"] - 1)):
            with pytest.raises(hzp.HzpError) as e:
                plan.arena_slice(cls, R, kind, count, buckets[0]["layer"], gd)
            assert e.value.status == hzp.HZP_ERR_RANGE
        if oplan["K"]:
            with pytest.raises(hzp.HzpError) as e:
                plan.arena_slice(cls, R, hzp.HZP_STREAM_RECV1, oplan["K"] - 1, buckets[0]["layer"], gd)
            assert e.value.status == hzp.HZP_ERR_RANGE
        else:
            with pytest.raises(hzp.HzpError) as e:
                plan.arena_slice(cls, R, hzp.HZP_STREAM_RECV1, 0, buckets[0]["layer"], gd)
            assert e.value.status == hzp.HZP_ERR_UNSUPPORTED


def test_arena_argument_errors():
    plan = hzp.hzp_plan([2, 1], [100, 40, 9], align=8, z3=2, z1=4, tensor_class=[0, 1, 0])
    def status(fn, *a):
        with pytest.raises(hzp.HzpError) as e:
            fn(*a)
        return e.value.status
    assert status(plan.arena, 2, 1) == hzp.HZP_ERR_RANGE
    assert status(plan.arena, 0, 33) == hzp.HZP_ERR_UNSUPPORTED
    assert status(plan.arena, 0, 1, 3) == hzp.HZP_ERR_INVALID_ARG
    assert status(plan.arena_slice, 0, 1, 8, 0, 0) == hzp.HZP_ERR_RANGE          # unknown stream
    assert status(plan.arena_slice, 1, 1, 0, 0, 1) == hzp.HZP_ERR_RANGE          # layer 1 has no fp32 bucket
    assert status(plan.arena_slice, 0, 1, 0, 0, 2) == hzp.HZP_ERR_RANGE          # no layer 2
    assert len(op.ARENA_RULES) == hzp.HZP_ARENA_VARIANTS
    assert status(plan.arena, 0, 1, 0, hzp.HZP_ARENA_VARIANTS) == hzp.HZP_ERR_RANGE
    assert status(plan.arena_slice, 0, 1, 0, 0, 0, 0, hzp.HZP_ARENA_VARIANTS) == hzp.HZP_ERR_RANGE
    huge = hzp.hzp_plan([1] * 60000, [1 << 40] * 60000, align=8, z3=1, z1=1)   # 6.6e16 elements in all
    assert status(huge.arena, 0, 32) == hzp.HZP_ERR_UNSUPPORTED                # 37 streams of 4 bytes each pass 2^63
    # 5 streams (master, m, v, cast parameters, ZeRO-3 shard), each an even number of 2 MiB units long: one more
    # unit between consecutive streams
    assert huge.arena(0, 0) == 60000 * (1 << 40) * (4 * 3 + 2 + 2) + 4 * hzp.HZP_ARENA_ALIGN
    assert huge.arena(0, 0, variant=1) == 60000 * (1 << 40) * (4 * 3 + 2 + 2)   # variant 1 adds no spacing
    # variant 7: spacings congruent 59 modulo 64 units; the streams are multiples of 64 units long
    assert huge.arena(0, 0, variant=7) == 60000 * (1 << 40) * (4 * 3 + 2 + 2) + 4 * 59 * hzp.HZP_ARENA_ALIGN
