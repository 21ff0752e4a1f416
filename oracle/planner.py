"""Layout oracle for hierarchical ZeRO sharding (test infrastructure, not product).

Plain Python integers, no numpy, no blocking: every quantity is written out the
way the method defines it so it can be checked by eye.

What the paper fixes (Section 4.1.1, Table 1 and the M_hzp equation):
  * five per-parameter arrays: bf16 parameters (2 B), fp32 gradients (4 B),
    fp32 master copy, momentum and variance (4 B each, 12 B together);
  * three independent sharding-group sizes.  The M_hzp equation divides the
    12 B of optimizer state by Z1, the 4 B gradient by Z2 and the 2 B
    parameter by Z3, and the experiments use Z1=64, Z2=Z3=8 (Table 2), so
    Z_k is the group of ZeRO *stage* k: Z1 optimizer states, Z2 gradients,
    Z3 parameters.  (The sentence introducing the symbols lists them in the
    opposite order; the equation, Figure 1 and the experiments agree with the
    reading used here.)
  * parameters and gradients are sharded inside a small (intra-node) group and
    optimizer states inside a larger one (Section 3.1, Figure 1).

What the paper leaves open and this oracle fixes (each is a stated reading):
  * one flat bucket per (layer, dtype class); every tensor starts on a multiple
    of A elements; the bucket is zero-padded to a multiple of A*lcm(Z1,Z2,Z3),
    so that the shards of every level are whole multiples of A;
  * the three group sizes are free (Section 4.1.1: they "can be arbitrarily
    specified").  Every configuration the paper reports has Z2 = Z3 and
    Z3 | Z1; then lcm = Z1, K = Z1 / Z3 and, for rank rho in [0, Z1):
    ZeRO-3 index j = rho mod Z3 (consecutive ranks form the parameter group,
    i.e. it sits inside a node), outer index k = rho div Z3, ZeRO-1 shard
    i = j*K + k, so ZeRO-1 shard i lies inside ZeRO-3 shard j and the post-step
    gather (Section 4.1.2, "Optimizer Step") is a contiguous concatenation;
  * in general a rank rho in [0, lcm) owns one shard per level, chosen so that
    every window of Z consecutive ranks holds each shard of that level once and
    shards nest wherever one group size divides the next (see level_index).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this.
"""

CLASS_BF16 = 0
CLASS_F32 = 1
_ELEM_BYTES = {CLASS_BF16: 2, CLASS_F32: 4}


def round_up(x, q):
    return ((x + q - 1) // q) * q


def is_pow2(x):
    return x >= 1 and (x & (x - 1)) == 0


class PlanError(ValueError):
    pass


def make_plan(tensors_per_layer, tensor_numel, align, z3, z1, z2=0,
              tensor_class=None, tensor_wd_mult=None):
    """Return the layout as a dict of plain lists/ints.

    tensors_per_layer : list of ints, one per layer, each >= 1
    tensor_numel      : flat list of element counts, layer after layer, each >= 1
    tensor_class      : None (all bf16) or flat list of 0/1
    tensor_wd_mult    : None (all 1.0) or flat list of floats
    """
    n_layers = len(tensors_per_layer)
    n_tensors = sum(tensors_per_layer)
    if n_layers < 1 or any(t < 1 for t in tensors_per_layer):
        raise PlanError("every layer needs at least one tensor")
    if len(tensor_numel) != n_tensors or any(n < 1 for n in tensor_numel):
        raise PlanError("tensor_numel must hold one positive count per tensor")
    if not is_pow2(align) or align < 8:
        raise PlanError("alignment must be a power of two >= 8")
    if z3 < 1 or z1 < 1 or z2 < 0:
        raise PlanError("group sizes must be positive (Z2 = 0 means: same as Z3)")
    if z2 == 0:
        z2 = z3
    if tensor_class is None:
        tensor_class = [CLASS_BF16] * n_tensors
    if tensor_wd_mult is None:
        tensor_wd_mult = [1.0] * n_tensors
    if any(c not in (CLASS_BF16, CLASS_F32) for c in tensor_class):
        raise PlanError("unknown tensor class")

    K = z1 // z3 if z1 % z3 == 0 else 0     # only defined when ZeRO-1 shards nest in ZeRO-3 shards
    world = lcm3(z1, z2, z3)                # number of ranks after which the ownership pattern repeats
    buckets = []          # in (layer, class) order
    tensors = [None] * n_tensors
    base = 0
    tid0 = 0
    for layer in range(n_layers):
        ids = list(range(tid0, tid0 + tensors_per_layer[layer]))
        tid0 += tensors_per_layer[layer]
        for cls in (CLASS_BF16, CLASS_F32):
            members = [t for t in ids if tensor_class[t] == cls]
            if not members:
                continue                       # a bucket with no tensor does not exist
            off = 0
            payload_end = 0
            for t in members:                  # given order, each start A-aligned
                tensors[t] = dict(id=t, layer=layer, cls=cls, offset=off,
                                  numel=tensor_numel[t], wd_mult=tensor_wd_mult[t],
                                  bucket=len(buckets))
                payload_end = off + tensor_numel[t]
                off = round_up(payload_end, align)
            P = round_up(payload_end, align * world)
            buckets.append(dict(layer=layer, cls=cls, tensor_ids=members,
                                payload_end=payload_end, P=P,
                                S3=P // z3, S2=P // z2, S1=P // z1, base=base))
            base += P
    return dict(align=align, z3=z3, z2=z2, z1=z1, K=K, world=world, n_layers=n_layers,
                buckets=buckets, tensors=tensors, total_padded=base)


def lcm3(a, b, c):
    from math import gcd
    ab = a * b // gcd(a, b)
    return ab * c // gcd(ab, c)


def find_bucket(plan, layer, cls):
    for b in plan["buckets"]:
        if b["layer"] == layer and b["cls"] == cls:
            return b
    return None


def level_index(plan, level, rank):
    """Index of the shard that `rank` owns at `level` (3 parameters, 2 gradients, 1 optimizer states).

    The index depends on rank mod Z_level only, one-to-one.  Where a smaller group size divides
    this level's, the shard is placed inside the rank's shard of that smaller group (mixed radix:
    parent index first, then the rank's position among the parent's co-owners):
        level 3:  j3 = rho mod Z3
        level 2:  Z3 | Z2:  j2 = j3*(Z2/Z3) + (rho div Z3) mod (Z2/Z3)      else  j2 = rho mod Z2
        level 1:  Z3 | Z2 | Z1:  i = j2*(Z1/Z2) + (rho div Z2) mod (Z1/Z2)
                  else Z3 | Z1:  i = j3*(Z1/Z3) + (rho div Z3) mod (Z1/Z3)
                  else Z2 | Z1:  i = j2*(Z1/Z2) + (rho div Z2) mod (Z1/Z2)
                  else           i = rho mod Z1
    """
    z1, z2, z3 = plan["z1"], plan["z2"], plan["z3"]
    if not (0 <= rank < plan["world"]):
        raise PlanError("rank out of range")
    j3 = rank % z3
    if level == 3:
        return j3
    chain32 = z2 % z3 == 0
    j2 = j3 * (z2 // z3) + (rank // z3) % (z2 // z3) if chain32 else rank % z2
    if level == 2:
        return j2
    if level != 1:
        raise PlanError("level must be 1, 2 or 3")
    if z1 % z3 == 0 and not (chain32 and z1 % z2 == 0):
        return j3 * (z1 // z3) + (rank // z3) % (z1 // z3)
    if z1 % z2 == 0:
        return j2 * (z1 // z2) + (rank // z2) % (z1 // z2)
    return rank % z1


def rank_to_indices(plan, rank):
    """rank -> (j, k, i): ZeRO-3 index, outer index, ZeRO-1 shard index (k is 0 when Z3 does not divide Z1)."""
    j, i = level_index(plan, 3, rank), level_index(plan, 1, rank)
    k = i - j * plan["K"] if plan["K"] else 0
    return j, k, i


def shard_range(plan, bucket, level, rank):
    """(begin, length) in bucket-relative elements of the rank's shard.

    level 3: the parameter shard (group size Z3); level 2: the gradient shard (Z2);
    level 1: the optimizer-state shard (Z1).
    """
    if level not in (1, 2, 3):
        raise PlanError("level must be 1, 2 or 3")
    length = bucket["S%d" % level]
    return level_index(plan, level, rank) * length, length


def cover(plan, bucket, j):
    """ZeRO-1 shards that meet ZeRO-3 shard j, in order: [(i, src_off, dst_off, length)].

    src_off is relative to ZeRO-1 shard i, dst_off to ZeRO-3 shard j.  This is what the post-step
    parameter gather (Section 4.1.2, "Optimizer Step") has to place when the two levels do not
    nest; with Z3 | Z1 it is the K whole shards j*K .. j*K+K-1.
    """
    S1, S3 = bucket["S1"], bucket["S3"]
    lo3, hi3 = j * S3, (j + 1) * S3
    out = []
    for i in range(plan["z1"]):
        lo, hi = max(lo3, i * S1), min(hi3, (i + 1) * S1)
        if lo < hi:
            out.append((i, lo - i * S1, lo - lo3, hi - lo))
    return out


def per_rank_bytes(plan):
    """(optimizer, gradient, parameter) bytes one rank holds.

    Table 1 with N replaced by the padded length of each bucket: 12 B of
    fp32 master/momentum/variance per ZeRO-1 element, a 4 B fp32 gradient per
    gradient-shard element, and the parameter itself (2 B bf16; 4 B for the
    fp32 class) per ZeRO-3 element.
    """
    opt = grad = par = 0
    for b in plan["buckets"]:
        opt += 12 * b["S1"]
        grad += 4 * (b["P"] // plan["z2"])
        par += _ELEM_BYTES[b["cls"]] * b["S3"]
    return opt, grad, par


def hzp_memory_bytes(N, z1, z2, z3):
    """M_hzp of Section 4.1.1 as an exact fraction (numerator, denominator)."""
    from fractions import Fraction
    return Fraction(12 * N, z1) + Fraction(4 * N, z2) + Fraction(2 * N, z3)


def owner_tensor(plan, bucket, pos):
    """Tensor id that owns bucket element `pos`, or -1 for padding (linear scan)."""
    for t in bucket["tensor_ids"]:
        rec = plan["tensors"][t]
        if rec["offset"] <= pos < rec["offset"] + rec["numel"]:
            return t
    return -1


def choose_groups(N, dp, node, budget_bytes):
    """Least sharding whose static memory M_hzp fits `budget_bytes`: (z1, z2, z3) or None.

    The paper sets the group sizes "according to the available device memory" and keeps parameters
    and gradients inside a node (Section 3.1, Section 4.1.1) but gives no procedure; this is the
    reading used here.  Candidates: Z3 divides `node` (parameter groups tile a node) and Z2 = Z3;
    Z3 | Z1 | dp.  Among the candidates with 12N/Z1 + 4N/Z2 + 2N/Z3 <= budget the one with the
    smallest Z3 wins (least parameter all-gather per layer), then the smallest Z1.
    """
    best = None
    for z3 in range(1, node + 1):
        if node % z3 or dp % z3:
            continue
        for z1 in range(z3, dp + 1, z3):
            if dp % z1:
                continue
            if hzp_memory_bytes(N, z1, z3, z3) <= budget_bytes and (best is None or (z3, z1) < best):
                best = (z3, z1)
    return None if best is None else (best[1], best[0], best[0])


# ---------------------------------------------------------------------------------------------
# One arena for a rank's persistent buffers of one class.
#
# Section 4.2 keeps communication buffers in pre-allocated, contiguous memory; the paper gives no
# layout.  The reading used here: a rank's buffers of one class are streams (R gradient
# contributions, master, momentum, variance, cast parameters, the received ZeRO-1 pieces of the
# other owners, the rank's ZeRO-3 shard, the received ZeRO-3 shards), each stream holds the slices
# of all buckets of the class back to back in bucket order, and the streams follow one another
# inside one allocation, each starting on a multiple of ARENA_ALIGN bytes.  The distance between the
# starts of consecutive streams, in ARENA_ALIGN units, is the smallest that holds the earlier stream
# and is congruent to r modulo M; (M, r) = ARENA_RULES[variant].  Variant 0 is "an odd number of
# units" (streams that are read at the same relative position should not lie a large power of two
# apart); the others exist because the best spacing depends on sizes and placement and is chosen by
# measurement.  The table is part of the interface and therefore the same on both sides.
# ---------------------------------------------------------------------------------------------
ARENA_ALIGN = 2 << 20
ARENA_RULES = ((2, 1), (1, 0), (2, 0), (16, 3), (16, 13), (64, 21), (64, 35), (64, 59))
STREAM_GRAD, STREAM_MASTER, STREAM_M, STREAM_V, STREAM_PARAM_OUT, STREAM_RECV1, STREAM_SHARD3, STREAM_RECV3 = range(8)


def arena_streams(plan, cls, R, grad_bytes):
    """[(kind, index, level, element_bytes)] in arena order.  level 1: ZeRO-1 slices, 3: ZeRO-3."""
    eb = _ELEM_BYTES[cls]
    out = [(STREAM_GRAD, r, 1, grad_bytes) for r in range(R)]
    out += [(STREAM_MASTER, 0, 1, 4), (STREAM_M, 0, 1, 4), (STREAM_V, 0, 1, 4), (STREAM_PARAM_OUT, 0, 1, eb)]
    if plan["K"]:                                      # the K-1 other owners of the rank's ZeRO-3 shard
        out += [(STREAM_RECV1, k, 1, eb) for k in range(plan["K"] - 1)]
    out += [(STREAM_SHARD3, 0, 3, eb)]
    out += [(STREAM_RECV3, j, 3, eb) for j in range(plan["z3"] - 1)]
    return out


def arena_layout(plan, cls, R, grad_bytes, variant=0):
    """(total_bytes, {(kind, index, layer): (byte_offset, bytes)}) for the class's buckets."""
    modulus, residue = ARENA_RULES[variant]
    buckets = [b for b in plan["buckets"] if b["cls"] == cls]
    if not buckets:
        raise PlanError("the plan has no bucket of that class")
    slices = {}
    pos = 0
    prev_start = None
    for kind, index, level, eb in arena_streams(plan, cls, R, grad_bytes):
        pos = round_up(pos, ARENA_ALIGN)
        while prev_start is not None and ((pos - prev_start) // ARENA_ALIGN) % modulus != residue:
            pos += ARENA_ALIGN                      # next spacing that satisfies the variant's rule
        prev_start = pos
        for b in buckets:
            n = b["S1"] if level == 1 else b["S3"]
            slices[kind, index, b["layer"]] = (pos, n * eb)
            pos += n * eb
    return pos, slices
