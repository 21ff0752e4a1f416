"""Pins for the layout oracle: brute-force ownership enumeration, invariants on random
descriptors, the paper's closed-form memory model, special cases and hand-worked values."""
import os
from fractions import Fraction

import pytest
from hypothesis import given, settings, strategies as st

import hzp_inputs
from oracle import planner as op

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line.split()


@st.composite
def descriptors(draw, max_numel=300):
    n_layers = draw(st.integers(1, 4))
    tpl = [draw(st.integers(1, 5)) for _ in range(n_layers)]
    n = sum(tpl)
    numel = [draw(st.integers(1, max_numel)) for _ in range(n)]
    cls = draw(st.one_of(st.none(), st.lists(st.integers(0, 1), min_size=n, max_size=n)))
    align = draw(st.sampled_from([8, 16, 32, 128]))
    z3 = draw(st.sampled_from([1, 2, 3, 4, 8]))
    K = draw(st.sampled_from([1, 2, 4, 5]))
    return dict(tensors_per_layer=tpl, tensor_numel=numel, tensor_class=cls,
                align=align, z3=z3, z1=z3 * K)


# ------------------------------------------------------------------ brute force ownership

@settings(max_examples=60, deadline=None)
@given(descriptors())
def test_every_element_owned_exactly_once(d):
    """Enumerate every bucket position; count the shards that contain it at each level."""
    plan = op.make_plan(**d)
    z3, z1, K = plan["z3"], plan["z1"], plan["K"]
    seen_i = set()
    for rank in range(z1):
        j, k, i = op.rank_to_indices(plan, rank)
        assert 0 <= j < z3 and 0 <= k < K and 0 <= i < z1
        seen_i.add(i)
    assert seen_i == set(range(z1))                       # rank -> ZeRO-1 shard is a bijection
    for b in plan["buckets"]:
        own3 = [0] * b["P"]
        own1 = [0] * b["P"]
        for rank in range(z1):
            j, k, i = op.rank_to_indices(plan, rank)
            b3, l3 = op.shard_range(plan, b, 3, rank)
            b1, l1 = op.shard_range(plan, b, 1, rank)
            assert b3 <= b1 and b1 + l1 <= b3 + l3          # ZeRO-1 shard nests in the ZeRO-3 shard
            assert i // K == j
            for x in range(b1, b1 + l1):
                own1[x] += 1
            if k == 0:                                      # one representative per ZeRO-3 shard
                for x in range(b3, b3 + l3):
                    own3[x] += 1
        assert own1 == [1] * b["P"]
        assert own3 == [1] * b["P"]
        # the K ranks sharing ZeRO-3 index j tile that shard, in k order
        for j in range(z3):
            pieces = sorted(op.shard_range(plan, b, 1, j + z3 * k)[0] for k in range(K))
            assert pieces == [j * b["S3"] + k * b["S1"] for k in range(K)]


@settings(max_examples=100, deadline=None)
@given(descriptors(max_numel=5000))
def test_layout_invariants(d):
    plan = op.make_plan(**d)
    A, z3, z1 = plan["align"], plan["z3"], plan["z1"]
    base = 0
    n_seen = 0
    for b in plan["buckets"]:
        assert b["base"] == base
        base += b["P"]
        prev_end = 0
        for t in b["tensor_ids"]:
            rec = plan["tensors"][t]
            assert rec["offset"] % A == 0
            assert rec["offset"] >= prev_end                 # disjoint, in the given order
            assert rec["offset"] - prev_end < A              # no more than alignment padding
            prev_end = rec["offset"] + rec["numel"]
            assert rec["layer"] == b["layer"] and rec["cls"] == b["cls"]
            n_seen += 1
        assert b["tensor_ids"] == sorted(b["tensor_ids"])
        assert b["payload_end"] == prev_end
        assert b["payload_end"] <= b["P"] < b["payload_end"] + A * z1
        assert b["P"] % (A * z1) == 0
        assert b["S1"] * z1 == b["P"] == b["S3"] * z3
        assert b["S1"] % A == 0 and b["S3"] % A == 0
        # every A-block meets at most one tensor
        for blk in range(b["P"] // A):
            owners = {op.owner_tensor(plan, b, x) for x in range(blk * A, (blk + 1) * A)} - {-1}
            assert len(owners) <= 1
    assert n_seen == len(plan["tensors"])
    assert plan["total_padded"] == base
    order = [(b["layer"], b["cls"]) for b in plan["buckets"]]
    assert order == sorted(order) and len(set(order)) == len(order)


# ------------------------------------------------------------------ closed-form memory model

def test_memory_closed_form_golden():
    """M_hzp of Section 4.1.1 at the paper's group sizes, values worked by hand."""
    for N, z1, z2, z3, want in _rows("memory_model.txt"):
        got = op.hzp_memory_bytes(int(N), int(z1), int(z2), int(z3))
        assert got == Fraction(int(want)), (N, z1, z2, z3)


@settings(max_examples=60, deadline=None)
@given(descriptors(max_numel=2000))
def test_per_rank_bytes_match_memory_model(d):
    d = dict(d, tensor_class=None)                           # the paper's table: bf16 parameters
    plan = op.make_plan(**d)
    opt, grad, par = op.per_rank_bytes(plan)
    Ptot = plan["total_padded"]
    z1, z3 = plan["z1"], plan["z3"]
    assert Fraction(opt + grad + par) == (Fraction(12 * Ptot, z1) + Fraction(4 * Ptot, z3)
                                          + Fraction(2 * Ptot, z3))
    assert opt + grad + par == op.hzp_memory_bytes(Ptot, z1, z3, z3)
    assert opt == 12 * Ptot // z1 and grad == 4 * Ptot // z3 and par == 2 * Ptot // z3
    if z1 == z3:                                             # collapses to 18N/Z (ZP) ...
        assert opt + grad + par == 18 * Ptot // z1


def test_vanilla_zero3_special_case():
    plan = op.make_plan([2], [1000, 24], align=8, z3=16, z1=16)    # ... and to 18N/DP
    assert sum(op.per_rank_bytes(plan)) * 16 == 18 * plan["total_padded"]


# ------------------------------------------------------------------ special cases

def test_group_size_one_is_whole_bucket():
    plan = op.make_plan([3], [5, 17, 100], align=8, z3=1, z1=1)
    b = plan["buckets"][0]
    assert op.shard_range(plan, b, 1, 0) == (0, b["P"])
    assert op.shard_range(plan, b, 3, 0) == (0, b["P"])
    assert [plan["tensors"][t]["offset"] for t in range(3)] == [0, 8, 32]
    assert b["payload_end"] == 132 and b["P"] == 136


def test_exact_multiple_needs_no_padding():
    plan = op.make_plan([1], [16 * 8 * 5], align=16, z3=2, z1=8)
    b = plan["buckets"][0]
    assert b["P"] == b["payload_end"] == 640 and b["S1"] == 80 and b["S3"] == 320


def test_classes_split_buckets():
    plan = op.make_plan([4, 1], [10, 20, 30, 40, 7], align=8, z3=2, z1=2,
                        tensor_class=[0, 1, 0, 1, 1])
    assert [(b["layer"], b["cls"], b["tensor_ids"]) for b in plan["buckets"]] == [
        (0, 0, [0, 2]), (0, 1, [1, 3]), (1, 1, [4])]
    assert op.find_bucket(plan, 1, 0) is None
    assert [plan["tensors"][t]["offset"] for t in range(5)] == [0, 0, 16, 24, 0]
    # P: bucket0 payload 46 -> 48; bucket1 payload 64 -> 64; bucket2 payload 7 -> 16
    assert [b["P"] for b in plan["buckets"]] == [48, 64, 16]
    assert [b["base"] for b in plan["buckets"]] == [0, 48, 112]
    opt, grad, par = op.per_rank_bytes(plan)
    assert (opt, grad, par) == (12 * 128 // 2, 4 * 128 // 2, (2 * 48 + 4 * 64 + 4 * 16) // 2)


def test_rank_map_example():
    # Z3 = 2, Z1 = 6, K = 3: ranks 0..5 -> (j, k, i)
    plan = op.make_plan([1], [96], align=8, z3=2, z1=6)
    got = [op.rank_to_indices(plan, r) for r in range(6)]
    assert got == [(0, 0, 0), (1, 0, 3), (0, 1, 1), (1, 1, 4), (0, 2, 2), (1, 2, 5)]
    b = plan["buckets"][0]
    assert (b["P"], b["S3"], b["S1"]) == (96, 48, 16)
    assert op.shard_range(plan, b, 1, 3) == (64, 16)
    assert op.shard_range(plan, b, 3, 3) == (48, 48)


@pytest.mark.parametrize("bad", [
    dict(align=12), dict(align=4), dict(z3=0), dict(z1=0), dict(z2=-1),
    dict(tensor_numel=[0, 5]), dict(tensors_per_layer=[0, 2]), dict(tensor_class=[0, 2]),
])
def test_rejects_bad_descriptors(bad):
    d = dict(tensors_per_layer=[2], tensor_numel=[3, 5], align=8, z3=2, z1=8)
    d.update(bad)
    with pytest.raises(op.PlanError):
        op.make_plan(**d)


# ------------------------------------------------------------------ free group sizes

@st.composite
def free_descriptors(draw, max_numel=400):
    n_layers = draw(st.integers(1, 3))
    tpl = [draw(st.integers(1, 4)) for _ in range(n_layers)]
    n = sum(tpl)
    z = st.integers(1, 9)
    return dict(tensors_per_layer=tpl, tensor_numel=[draw(st.integers(1, max_numel)) for _ in range(n)],
                align=draw(st.sampled_from([8, 16])), z3=draw(z), z2=draw(z), z1=draw(z))


def test_free_group_sizes_hand_values():
    for row in _rows("general_groups_hand_values.txt"):
        kind, v = row[0], [int(x) for x in row[1:]]
        if kind == "layout":
            A, z1, z2, z3, payload, P, S1, S2, S3 = v
            b = op.make_plan([1], [payload], A, z3, z1, z2)["buckets"][0]
            assert (b["P"], b["S1"], b["S2"], b["S3"]) == (P, S1, S2, S3), row
        elif kind == "rank":
            z1, z2, z3, rho, j3, j2, i = v
            plan = op.make_plan([1], [8], 8, z3, z1, z2)
            assert [op.level_index(plan, l, rho) for l in (3, 2, 1)] == [j3, j2, i], row
        else:
            A, z1, z2, z3, payload, j = v[:6]
            plan = op.make_plan([1], [payload], A, z3, z1, z2)
            want = [tuple(v[6 + 4 * q:10 + 4 * q]) for q in range((len(v) - 6) // 4)]
            assert op.cover(plan, plan["buckets"][0], j) == want, row


@settings(max_examples=150, deadline=None)
@given(free_descriptors())
def test_free_group_sizes_ownership_by_enumeration(d):
    """Every level: each aligned window of Z consecutive ranks owns every element exactly once;
    shards nest where the group sizes divide; the cover equals element-by-element ownership."""
    plan = op.make_plan(**d)
    A = plan["align"]
    Z = {1: plan["z1"], 2: plan["z2"], 3: plan["z3"]}
    W = plan["world"]
    assert all(W % z == 0 for z in Z.values()) and not any(
        all(w % z == 0 for z in Z.values()) for w in range(1, W))          # least common multiple
    for level, z in Z.items():
        idx = [op.level_index(plan, level, r) for r in range(W)]
        assert all(idx[r] == idx[r % z] for r in range(W))                 # depends on rank mod Z only
        assert sorted(idx[:z]) == list(range(z))                           # one-to-one inside a group
    for b in plan["buckets"]:
        P = b["P"]
        assert b["payload_end"] <= P < b["payload_end"] + A * W and P % (A * W) == 0
        for level, z in Z.items():
            S = b["S%d" % level]
            assert S * z == P and S % A == 0
            count = [0] * P
            for r in range(z):                                             # one aligned window
                beg, n = op.shard_range(plan, b, level, r)
                assert n == S
                for x in range(beg, beg + n):
                    count[x] += 1
            assert count == [1] * P

        def inside(r, inner, outer):
            bi, ni = op.shard_range(plan, b, inner, r)
            bo, no = op.shard_range(plan, b, outer, r)
            return bo <= bi and bi + ni <= bo + no
        for r in range(W):
            if Z[2] % Z[3] == 0:
                assert inside(r, 2, 3)
            if Z[1] % Z[3] == 0:
                assert inside(r, 1, 3)
            if Z[1] % Z[2] == 0 and (Z[2] % Z[3] == 0 or Z[1] % Z[3] != 0):
                assert inside(r, 1, 2)
        for j in range(Z[3]):
            owner = {}
            for x in range(j * b["S3"], (j + 1) * b["S3"]):                # element by element
                owner.setdefault(x // b["S1"], []).append(x)
            want = [(i, xs[0] - i * b["S1"], xs[0] - j * b["S3"], len(xs)) for i, xs in sorted(owner.items())]
            assert op.cover(plan, b, j) == want
    opt, grad, par = op.per_rank_bytes(plan)
    if all(c == 0 for c in [plan["tensors"][t]["cls"] for t in range(len(plan["tensors"]))]):
        assert opt + grad + par == op.hzp_memory_bytes(plan["total_padded"], Z[1], Z[2], Z[3])


def test_free_group_sizes_reduce_to_the_nested_map():
    """With Z2 = Z3 | Z1 the general rule is the nested one: j = r mod Z3, i = j*K + r div Z3."""
    for z3, K in [(1, 1), (2, 3), (8, 8), (4, 4), (3, 5)]:
        plan = op.make_plan([1], [64], 8, z3, z3 * K)
        assert plan["world"] == z3 * K and plan["K"] == K and plan["z2"] == z3
        for r in range(z3 * K):
            assert op.level_index(plan, 3, r) == r % z3 == op.level_index(plan, 2, r)
            assert op.level_index(plan, 1, r) == (r % z3) * K + r // z3
            assert op.rank_to_indices(plan, r) == (r % z3, r // z3, (r % z3) * K + r // z3)


def test_choose_groups_hand_values_and_optimality():
    for row in _rows("choose_groups.txt"):
        N, dp, node, budget = (int(x) for x in row[:4])
        want = None if row[4] == "none" else tuple(int(x) for x in row[4:7])
        assert op.choose_groups(N, dp, node, budget) == want, row
    # whatever is chosen fits, and no admissible candidate with a smaller (Z3, Z1) does
    for N, dp, node, budget in [(12345, 48, 8, 30000), (10 ** 9, 256, 8, 3 * 10 ** 9), (999, 36, 6, 4000)]:
        z1, z2, z3 = op.choose_groups(N, dp, node, budget)
        assert z2 == z3 and node % z3 == 0 and z1 % z3 == 0 and dp % z1 == 0
        assert 12 * N * z3 + 6 * N * z1 <= budget * z1 * z3                       # M_hzp <= budget, in integers
        for c3 in range(1, node + 1):
            for c1 in range(1, dp + 1):
                admissible = node % c3 == 0 and c1 % c3 == 0 and dp % c1 == 0
                if admissible and (c3, c1) < (z3, z1):
                    assert 12 * N * c3 + 6 * N * c1 > budget * c1 * c3, (c3, c1)


# ------------------------------------------------------------------ hand-worked model shapes

def _first_bucket_named(cfg, plan, layer_name):
    return op.find_bucket(plan, cfg["layer_names"].index(layer_name), op.CLASS_BF16)


def test_model_shaped_hand_values():
    want = {r[0]: [int(x) for x in r[1:]] for r in _rows("layout_hand_values.txt")}
    where = {"dense7b_layer": (1, "layer5"), "dense7b_head": (1, "head"),
             "dense70b_layer": (2, "layer79"), "moe_layer": (3, "layer0"),
             "tiny_embed": (0, "embed"), "tiny_layer": (0, "layer1")}
    for key, (idx, lname) in where.items():
        cfg = hzp_inputs.config(idx)
        plan = op.make_plan(cfg["tensors_per_layer"], cfg["tensor_numel"], cfg["align"],
                            cfg["z3"], cfg["z1"])
        b = _first_bucket_named(cfg, plan, lname)
        A, z3, z1, payload_end, P, S3, S1 = want[key]
        assert (plan["align"], plan["z3"], plan["z1"]) == (A, z3, z1)
        assert (b["payload_end"], b["P"], b["S3"], b["S1"]) == (payload_end, P, S3, S1), key


def test_workload_shapes():
    c0 = hzp_inputs.config(0)
    assert len(c0["tensor_numel"]) == 16 and sum(c0["tensor_numel"]) == 1838336
    c3 = hzp_inputs.config(3)
    assert c3["tensors_per_layer"] == [199] * 24
    c4 = hzp_inputs.config(4)
    assert len(c4["tensor_numel"]) == 4096 and c4["tensors_per_layer"] == [64] * 64
    assert min(c4["tensor_numel"]) >= 1 and max(c4["tensor_numel"]) <= 65536
    plan = op.make_plan(c4["tensors_per_layer"], c4["tensor_numel"], c4["align"], c4["z3"],
                        c4["z1"], tensor_class=c4["tensor_class"])
    assert len(plan["buckets"]) == 128                       # a bf16 and an fp32 bucket per group


# ------------------------------------------------------------------ one arena per rank and class

def test_arena_layout_invariants_and_hand_values():
    """Streams follow one another on 2 MiB boundaries, slices of a stream lie back to back in bucket
    order, nothing overlaps, every slice has the length of the shard it holds."""
    plan = op.make_plan([2, 1, 2], [1000, 77, 4096, 300000, 9], 16, 4, 8, tensor_class=[0, 1, 0, 0, 1])
    for cls, R, gb in ((0, 3, 2), (0, 2, 4), (1, 5, 4)):
        total, sl = op.arena_layout(plan, cls, R, gb)
        buckets = [b for b in plan["buckets"] if b["cls"] == cls]
        streams = op.arena_streams(plan, cls, R, gb)
        assert len(streams) == R + 4 + (plan["K"] - 1) + 1 + (plan["z3"] - 1)
        assert len(sl) == len(streams) * len(buckets)
        spans = sorted((off, off + n) for off, n in sl.values())
        assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))            # pairwise disjoint
        assert spans[-1][1] == total
        starts = [sl[kind, index, buckets[0]["layer"]][0] for kind, index, level, eb in streams]
        for a, b, (kind, index, level, eb) in zip(starts, starts[1:], streams):
            size = eb * sum(x["S1"] if level == 1 else x["S3"] for x in buckets)
            units = (b - a) // op.ARENA_ALIGN
            assert units % 2 == 1 and a + size <= b < a + size + 2 * op.ARENA_ALIGN   # odd spacing, no more than needed
        for kind, index, level, eb in streams:
            first = sl[kind, index, buckets[0]["layer"]][0]
            assert first % op.ARENA_ALIGN == 0
            pos = first
            for b in buckets:
                off, n = sl[kind, index, b["layer"]]
                assert off == pos and n == eb * (b["S1"] if level == 1 else b["S3"])
                assert off % 16 == 0                                            # shards are multiples of A >= 8 elements
                pos += n
    # hand values: one bf16 bucket of P = 2^20 elements, Z3 = 2, Z1 = 4, R = 2 bf16 contributions:
    # S1 = 262144 (512 KiB in bf16, 1 MiB in fp32), S3 = 524288 (1 MiB); every stream fits 2 MiB
    plan = op.make_plan([1], [1 << 20], 8, 2, 4)
    total, sl = op.arena_layout(plan, 0, 2, 2)
    M = 2 << 20
    assert sl[op.STREAM_GRAD, 0, 0] == (0, 524288) and sl[op.STREAM_GRAD, 1, 0] == (M, 524288)
    assert sl[op.STREAM_MASTER, 0, 0] == (2 * M, 1048576) and sl[op.STREAM_V, 0, 0] == (4 * M, 1048576)
    assert sl[op.STREAM_PARAM_OUT, 0, 0] == (5 * M, 524288)
    assert sl[op.STREAM_RECV1, 0, 0] == (6 * M, 524288)                         # K - 1 = 1 other owner
    assert sl[op.STREAM_SHARD3, 0, 0] == (7 * M, 1048576)
    assert sl[op.STREAM_RECV3, 0, 0] == (8 * M, 1048576) and total == 8 * M + 1048576
    with pytest.raises(op.PlanError):
        op.arena_layout(plan, 1, 2, 4)                                          # no fp32 bucket
    # streams of an even number of 2 MiB units get one more unit of spacing: P = 2^23, Z1 = Z3 = 1, R = 1:
    # 16 MiB of bf16 (8 units -> spacing 9), 32 MiB of fp32 (16 units -> spacing 17)
    plan = op.make_plan([1], [1 << 23], 8, 1, 1)
    total, sl = op.arena_layout(plan, 0, 1, 2)
    assert sl[op.STREAM_GRAD, 0, 0] == (0, 16 * M // 2) and sl[op.STREAM_MASTER, 0, 0] == (9 * M, 16 * M)
    assert sl[op.STREAM_M, 0, 0] == (26 * M, 16 * M) and sl[op.STREAM_V, 0, 0] == (43 * M, 16 * M)
    assert sl[op.STREAM_PARAM_OUT, 0, 0] == (60 * M, 8 * M) and sl[op.STREAM_SHARD3, 0, 0] == (69 * M, 8 * M)
    assert total == 77 * M
    # the other variants: same streams and slices, only the spacing rule differs.  Hand values for the
    # plan above (streams of 8 and 16 units): variant 1 packs them (8, 16, 16, 16, 8 -> starts 0, 8, 24, 40, 56, 64),
    # variant 2 keeps even spacings as they are, variant 3 takes the next spacing congruent 3 modulo 16
    # (8 -> 19, 16 -> 19), variant 7 the next congruent 59 modulo 64 (59 for both lengths)
    def starts(variant):
        tot, x = op.arena_layout(plan, 0, 1, 2, variant)
        return [x[k, 0, 0][0] // M for k in (op.STREAM_GRAD, op.STREAM_MASTER, op.STREAM_M, op.STREAM_V,
                                              op.STREAM_PARAM_OUT, op.STREAM_SHARD3)], tot
    assert starts(1) == ([0, 8, 24, 40, 56, 64], 72 * M)
    assert starts(2) == starts(1)
    assert starts(3) == ([0, 19, 38, 57, 76, 95], 103 * M)
    assert starts(7) == ([0, 59, 118, 177, 236, 295], 303 * M)
    assert op.ARENA_RULES[0] == (2, 1)
    for variant, (modulus, residue) in enumerate(op.ARENA_RULES):
        st, tot = starts(variant)
        sizes = [8, 16, 16, 16, 8, 8]
        for a, b, n in zip(st, st[1:], sizes):
            assert (b - a) % modulus == residue and n <= b - a < n + modulus      # the least spacing that fits the rule
        assert tot == st[-1] * M + 8 * M
