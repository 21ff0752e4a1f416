"""Pins for the numeric oracle: hand-worked roundings and sums, closed-form AdamW
trajectories, library routines (torch's bf16 cast, torch.optim.AdamW) and brute force."""
import math

import numpy as np
import pytest
import torch

import hzp_inputs
from oracle import numeric as on
from oracle import planner as op

HP = dict(lr=1e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def f32(x):
    return np.float32(x)


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


# ------------------------------------------------------------------ bf16 <-> fp32

def test_bf16_hand_values():
    def enc(u32):
        return int(on.f32_to_bf16(np.array([u32], dtype=np.uint32).view(np.float32))[0])
    assert enc(0x3F800000) == 0x3F80          # 1.0
    assert enc(0x3F808000) == 0x3F80          # 1 + 2^-8: tie, kept half even -> down
    assert enc(0x3F808001) == 0x3F81          # just above the tie -> up
    assert enc(0x3F818000) == 0x3F82          # tie, kept half odd -> up to even
    assert enc(0x3F817FFF) == 0x3F81          # just below the tie -> down
    assert enc(0x3FFF8000) == 0x4000          # carry runs through the mantissa into the exponent
    assert enc(0x7F7FFFFF) == 0x7F80          # largest finite fp32 rounds to +inf
    assert enc(0xFF7FFFFF) == 0xFF80
    assert enc(0x7F800000) == 0x7F80          # inf stays inf
    assert enc(0x80000000) == 0x8000          # -0 stays -0
    assert enc(0x00008000) == 0x0000          # subnormal tie to even (zero)
    assert enc(0x00018000) == 0x0002          # subnormal tie, odd -> up
    nan = enc(0x7F800001)
    assert (nan & 0x7F80) == 0x7F80 and (nan & 0x007F) != 0     # a NaN stays a NaN
    assert float(on.bf16_to_f32(0x3F80)) == 1.0
    assert float(on.bf16_to_f32(0xC000)) == -2.0
    assert float(on.bf16_to_f32(0x0001)) == 2.0 ** -133


def test_bf16_cast_exhaustive_vs_library():
    """All 2^16 high halves x several low halves against torch's fp32->bf16 cast."""
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    for low in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x1234):
        u = hi | np.uint32(low)
        x = u.view(np.float32)
        got = on.f32_to_bf16(x)
        want = (torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16)
                .numpy().view(np.uint16))
        finite_or_inf = ~np.isnan(x)
        assert np.array_equal(got[finite_or_inf], want[finite_or_inf]), hex(low)
        nan_out = got[~finite_or_inf]
        assert np.all((nan_out & 0x7F80) == 0x7F80) and np.all((nan_out & 0x007F) != 0)


def test_bf16_roundtrip_exact():
    h = np.arange(1 << 16, dtype=np.uint16)
    x = on.bf16_to_f32(h)
    keep = ~np.isnan(x)               # (a signalling NaN is quieted on its way through Python)
    assert np.array_equal(x.view(np.uint32)[keep], (h.astype(np.uint32) << 16)[keep])
    assert np.array_equal(on.f32_to_bf16(x)[keep], h[keep])
    want = torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    assert np.array_equal(x.view(np.uint32)[keep], want.view(np.uint32)[keep])


# ------------------------------------------------------------------ reduce

def bf(x):
    return hzp_inputs.to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_reduce_single_replica_is_exact_widening():
    rng = np.random.default_rng(1)
    h = rng.integers(0, 1 << 16, size=4096, dtype=np.uint16)
    h = h[(h & 0x7F80) != 0x7F80]                      # finite only
    out = on.reduce([np.ascontiguousarray(h)])
    assert np.array_equal(out.view(np.uint32), h.astype(np.uint32) << 16)


def test_reduce_order_is_left_to_right():
    """(1 + 2^-24) + 2^-24 = 1 in fp32 (two ties to even), but 2^-24 + 2^-24 + 1 = 1 + 2^-23."""
    t = 2.0 ** -24
    fwd = on.reduce([bf([1.0]), bf([t]), bf([t])])
    rev = on.reduce([bf([t]), bf([t]), bf([1.0])])
    assert fwd[0] == np.float32(1.0)
    assert rev[0] == np.float32(1.0 + 2.0 ** -23)
    # a tree (pairwise) order would give (1 + t) + (t + t) = 1 + 2^-23 for 4 inputs; the
    # running order gives ((1 + t) + t) + t = 1
    assert on.reduce([bf([1.0]), bf([t]), bf([t]), bf([t])])[0] == np.float32(1.0)


def test_reduce_small_integers_exact_with_scale():
    rng = np.random.default_rng(2)
    R, n = 16, 1000
    ints = rng.integers(-100, 101, size=(R, n))
    out = on.reduce([bf(ints[r]) for r in range(R)], scale=1.0 / R)
    assert np.array_equal(out.astype(np.float64), ints.sum(axis=0) / R)
    # index check: element x of the output only sees element x of every slice
    ints2 = np.zeros((3, 5), dtype=np.int64)
    ints2[0, 1], ints2[1, 3], ints2[2, 4] = 7, 11, 13
    assert on.reduce([bf(r) for r in ints2]).tolist() == [0, 7, 0, 11, 13]


def test_reduce_accumulate_semantics():
    g = [bf([1.0, 2.0, -3.0]), bf([4.0, 5.0, 6.0])]
    out = np.array([10.0, 20.0, 30.0], dtype=np.float32)
    on.reduce(g, scale=0.5, accumulate=True, out=out)         # out + scale * sum
    assert out.tolist() == [12.5, 23.5, 31.5]
    # scale multiplies the new sum only, after the sum, with one rounding
    s = np.float32(1.0 + 2.0 ** -7)                           # bf16-representable
    o = on.reduce([bf([s]), bf([s]), bf([s])], scale=1.0 / 3.0)
    want = np.float32(np.float32(1.0 / 3.0) * np.float32(np.float32(s + s) + s))
    assert o[0] == want


def test_reduce_fp32_inputs_and_error_bound():
    rng = np.random.default_rng(3)
    R, n = 8, 5000
    g = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(R)]
    out = on.reduce(g)
    exact = np.sum(np.stack(g).astype(np.float64), axis=0)
    bound = (R - 1) * 2.0 ** -24 * np.sum(np.abs(np.stack(g).astype(np.float64)), axis=0)
    assert np.all(np.abs(out.astype(np.float64) - exact) <= bound * 1.0001)
    # same chain written with numpy's own fp32 adds (a second implementation of IEEE add)
    acc = g[0].copy()
    for r in range(1, R):
        acc = acc + g[r]
    assert np.array_equal(out, acc)
    gb = [hzp_inputs.to_bf16_bits(x) for x in g]
    acc = on.bf16_to_f32(gb[0])
    for r in range(1, R):
        acc = acc + on.bf16_to_f32(gb[r])
    assert np.array_equal(on.reduce(gb), acc)


# ------------------------------------------------------------------ AdamW closed forms

def _run(g, p, m, v, step, hp, **kw):
    g, p, m, v = (np.array(a, dtype=np.float32) for a in (g, p, m, v))
    out = on.adamw(g, p, m, v, step=step, **hp, **kw)
    return p, m, v, out


@pytest.mark.parametrize("precision", ["f64", "f32"])
def test_adamw_first_step_closed_form(precision):
    """From m = v = 0: m1 = (1-b1) g, v1 = (1-b2) g^2, p1 = p0 - lr (g/(|g|+eps) + wd p0)."""
    hp = dict(lr=0.125, beta1=0.75, beta2=0.5, eps=0.25, weight_decay=0.5)
    g = [0.25, -0.75, 0.0, 2.0]
    p0 = [1.0, -2.0, 4.0, 0.5]
    p, m, v, p16 = _run(g, p0, [0] * 4, [0] * 4, 1, hp, precision=precision)
    # every number below is exact in binary, worked by hand
    assert m.tolist() == [0.0625, -0.1875, 0.0, 0.5]
    assert v.tolist() == [0.03125, 0.28125, 0.0, 2.0]
    # u = g/(|g|+eps) = 0.5, -0.75, 0, 8/9 ; p1 = p0 - 0.125*(u + 0.5*p0)
    want = [1.0 - 0.125 * (0.5 + 0.5), -2.0 - 0.125 * (-0.75 - 1.0), 4.0 - 0.125 * 2.0,
            0.5 - 0.125 * (2.0 / 2.25 + 0.25)]
    assert np.allclose(p, want, rtol=3e-7, atol=0)
    assert p.tolist()[:3] == want[:3]
    assert np.array_equal(p16, on.f32_to_bf16(p))


def test_adamw_eps_sits_outside_the_square_root():
    hp = dict(lr=1.0, beta1=0.0, beta2=0.0, eps=3.0, weight_decay=0.0)
    p, m, v, _ = _run([4.0], [0.0], [0.0], [0.0], 1, hp)
    assert p[0] == np.float32(-4.0 / 7.0)                 # 4/(sqrt(16)+3), not 4/sqrt(16+3)


def test_adamw_constant_gradient_closed_form():
    """g constant: bias-corrected m and v equal g and g^2 at every step, so with
    a = 1 - lr*wd and u = g/(|g|+eps):  p_t = a^t p0 - lr*u*(1-a^t)/(1-a)."""
    hp = dict(lr=0.01, beta1=0.9, beta2=0.95, eps=1e-3, weight_decay=0.1)
    g = np.array([3e-3, -1e-3, 2e-2], dtype=np.float32)
    p0 = np.array([0.5, -0.25, 1.5], dtype=np.float32)
    p, m, v = p0.copy(), np.zeros(3, np.float32), np.zeros(3, np.float32)
    lr, wd, eps = (float(f32(hp[k])) for k in ("lr", "weight_decay", "eps"))
    b1, b2 = float(f32(hp["beta1"])), float(f32(hp["beta2"]))
    a = 1.0 - lr * wd
    gd = g.astype(np.float64)
    u = gd / (np.abs(gd) + eps)
    for t in range(1, 41):
        on.adamw(g, p, m, v, step=t, **hp)
        want_p = a ** t * p0.astype(np.float64) - lr * u * (1 - a ** t) / (1 - a)
        assert np.allclose(p, want_p, rtol=1e-6, atol=0), t
        assert np.allclose(m, gd * (1 - b1 ** t), rtol=1e-6, atol=0)
        assert np.allclose(v, gd * gd * (1 - b2 ** t), rtol=1e-6, atol=0)


def test_adamw_zero_gradient_is_pure_decay():
    hp = dict(HP, lr=0.05)
    p0 = np.array([1.0, -3.0, 0.0], dtype=np.float32)
    p, m, v = p0.copy(), np.zeros(3, np.float32), np.zeros(3, np.float32)
    g = np.zeros(3, np.float32)
    a = 1.0 - float(f32(hp["lr"])) * float(f32(hp["weight_decay"]))
    for t in range(1, 11):
        on.adamw(g, p, m, v, step=t, **hp)
        assert np.allclose(p, a ** t * p0.astype(np.float64), rtol=5e-7, atol=0)
        assert not m.any() and not v.any()
    assert p[2] == 0.0 and bits(p)[2] == 0                 # padding stays +0.0


def test_adamw_step_size_is_lr_without_decay():
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-30, weight_decay=0.0)
    g = np.array([5.0, -1e-4, 3e-2], dtype=np.float32)
    p, m, v, _ = _run(g, [1.0, 1.0, 1.0], [0] * 3, [0] * 3, 1, hp)
    assert np.allclose(1.0 - p.astype(np.float64), 1e-3 * np.sign(g), rtol=2e-4)


def test_adamw_wd_multiplier_and_outputs():
    hp = dict(lr=0.5, beta1=0.0, beta2=0.0, eps=1.0, weight_decay=0.5)
    g = np.zeros(2, np.float32)
    mult = np.array([1.0, 0.0], dtype=np.float32)
    p, m, v, out = _run(g, [2.0, 2.0], [0, 0], [0, 0], 1, hp, wd_mult=mult, out_bf16=False)
    assert p.tolist() == [1.5, 2.0] and out.dtype == np.float32 and out.tolist() == [1.5, 2.0]


def _tol_ok(a, b, rel=2e-6):
    """|a-b| <= rel * max(|a|, |b|, rms(b)): relative, with elements below the array's RMS
    judged against the RMS (beta1*m + (1-beta1)*g cancels, so its rounding error scales with
    the operands, not with the result)."""
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    rms = math.sqrt(float(np.mean(b64 * b64)))
    scale = np.maximum(np.maximum(np.abs(a64), np.abs(b64)), rms)
    return np.all(np.abs(a64 - b64) <= rel * scale)


def test_adamw_fp32_evaluation_is_within_tolerance_of_fp64():
    rng = np.random.default_rng(5)
    n = 50000
    p64 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m64, v64 = np.zeros(n, np.float32), np.zeros(n, np.float32)
    p32, m32, v32 = p64.copy(), m64.copy(), v64.copy()
    for t in range(1, 11):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        a = on.adamw(g, p64, m64, v64, step=t, precision="f64", **HP)
        b = on.adamw(g, p32, m32, v32, step=t, precision="f32", **HP)
        assert _tol_ok(p32, p64) and _tol_ok(m32, m64) and _tol_ok(v32, v64)
        d = np.abs(a.astype(np.int32) - b.astype(np.int32))
        assert d.max() <= 1


@pytest.mark.parametrize("hp", [HP, dict(lr=1e-2, beta1=0.8, beta2=0.9, eps=1e-4, weight_decay=0.3)])
def test_adamw_matches_library_optimizer(hp):
    """torch.optim.AdamW in float64 on the tiny workload's first bucket, 10 steps."""
    cfg = hzp_inputs.config(0)
    plan = op.make_plan(cfg["tensors_per_layer"], cfg["tensor_numel"], cfg["align"], cfg["z3"],
                        cfg["z1"])
    b = plan["buckets"][0]
    ranges = [(plan["tensors"][t]["offset"], plan["tensors"][t]["numel"]) for t in b["tensor_ids"]]
    p = hzp_inputs.master_bucket(0, 0, b["P"], ranges)
    m, v = np.zeros_like(p), np.zeros_like(p)
    ref = torch.nn.Parameter(torch.from_numpy(p.copy()).double())
    opt = torch.optim.AdamW([ref], lr=float(f32(hp["lr"])),
                            betas=(float(f32(hp["beta1"])), float(f32(hp["beta2"]))),
                            eps=float(f32(hp["eps"])), weight_decay=float(f32(hp["weight_decay"])))
    for t in range(1, 11):
        slices = [hzp_inputs.grad_bucket(0, t, 0, r, b["P"], ranges, cfg["sigma"]) for r in range(4)]
        g = on.reduce(slices, scale=0.25)
        ref.grad = torch.from_numpy(g.copy()).double()
        before = p.astype(np.float64)
        want_before = ref.detach().numpy().copy()
        opt.step()
        on.adamw(g, p, m, v, step=t, **hp)
        want = ref.detach().numpy()
        assert _tol_ok(p, want, rel=1e-6), t
        st = opt.state[ref]
        assert _tol_ok(m, st["exp_avg"].numpy(), rel=1e-6)
        assert _tol_ok(v, st["exp_avg_sq"].numpy(), rel=1e-6)
        # the step itself (p barely moves, so compare the move): fp32 storage of p limits
        # the agreement to about one rounding of p
        move, want_move = p.astype(np.float64) - before, want - want_before
        assert np.all(np.abs(move - want_move) <= 1e-3 * np.abs(want_move)
                      + 2.0 ** -23 * np.abs(want) + 1e-6 * hp["lr"])
    pay = hzp_inputs._payload_mask(b["P"], ranges)
    assert not p[~pay].any() and not m[~pay].any() and not v[~pay].any()


def test_adamw_update_term_matches_library_where_eps_matters():
    """Tiny gradients (|g| ~ eps) make the update sensitive to where eps and the bias
    corrections enter; compare the update, not the parameter."""
    hp = dict(lr=1.0, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0)
    rng = np.random.default_rng(9)
    n = 2000
    p = np.zeros(n, np.float32)
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    ref = torch.nn.Parameter(torch.zeros(n, dtype=torch.float64))
    opt = torch.optim.AdamW([ref], lr=1.0, betas=(float(f32(0.9)), float(f32(0.95))),
                            eps=float(f32(1e-8)), weight_decay=0.0)
    for t in range(1, 6):
        g = (rng.standard_normal(n) * 2e-8).astype(np.float32)
        ref.grad = torch.from_numpy(g.copy()).double()
        opt.step()
        on.adamw(g, p, m, v, step=t, **hp)
        assert np.allclose(p, ref.detach().numpy(), rtol=2e-6, atol=5e-7), t   # p is O(1): fp32 storage


def test_sharded_update_equals_unsharded_update():
    """Updating every ZeRO-1 shard separately and concatenating equals updating the whole
    bucket (the method computes what full-parameter training computes, Section 4.2)."""
    d = hzp_inputs.irregular_desc(12, seed=3, f32_every=0)
    plan = op.make_plan(d["tensors_per_layer"], d["tensor_numel"], 8, 2, 8)
    b = plan["buckets"][1]
    ranges = [(plan["tensors"][t]["offset"], plan["tensors"][t]["numel"]) for t in b["tensor_ids"]]
    P = b["P"]
    slices = [hzp_inputs.grad_bucket(7, 1, 1, r, P, ranges, 1e-3) for r in range(4)]
    p0 = hzp_inputs.master_bucket(7, 1, P, ranges)
    g = on.reduce(slices, scale=0.25)
    pw, mw, vw = p0.copy(), np.zeros(P, np.float32), np.zeros(P, np.float32)
    outw = on.adamw(g, pw, mw, vw, step=1, **HP)
    parts = {}
    for rank in range(plan["z1"]):
        beg, ln = op.shard_range(plan, b, 1, rank)
        gs = on.reduce([np.ascontiguousarray(s[beg:beg + ln]) for s in slices], scale=0.25)
        ps = np.ascontiguousarray(p0[beg:beg + ln])
        ms, vs = np.zeros(ln, np.float32), np.zeros(ln, np.float32)
        outs = on.adamw(gs, ps, ms, vs, step=1, **HP)
        assert np.array_equal(ps, pw[beg:beg + ln]) and np.array_equal(ms, mw[beg:beg + ln])
        assert np.array_equal(vs, vw[beg:beg + ln])
        parts[rank] = outs
    # level-1 gather for each ZeRO-3 index j, then level-3 gather, rebuilds the bucket
    z3, K = plan["z3"], plan["K"]
    shards3 = [on.gather_concat([parts[j + z3 * k] for k in range(K)]) for j in range(z3)]
    assert np.array_equal(on.gather_concat(shards3), outw)


# ------------------------------------------------------------------ gather

def test_gather_concat_brute_force():
    rng = np.random.default_rng(11)
    for dt in (np.uint16, np.float32):
        srcs = [rng.integers(0, 60000, size=7).astype(dt) for _ in range(5)]
        got = on.gather_concat(srcs)
        want = [srcs[s][x] for s in range(5) for x in range(7)]
        assert got.dtype == dt and got.tolist() == want
        assert np.array_equal(got, np.concatenate(srcs))


def test_gather_of_shards_is_identity_and_unpack_inverts_pack():
    d = hzp_inputs.irregular_desc(9, seed=5, max_numel=700, tensors_per_layer=9, f32_every=0)
    plan = op.make_plan(d["tensors_per_layer"], d["tensor_numel"], 16, 4, 8)
    b = plan["buckets"][0]
    rng = np.random.default_rng(12)
    tensors = [rng.integers(1, 1 << 16, size=n).astype(np.uint16) for n in d["tensor_numel"]]
    bucket = np.zeros(b["P"], dtype=np.uint16)              # pack by the plan's offsets
    for t, vals in enumerate(tensors):
        off = plan["tensors"][t]["offset"]
        bucket[off:off + vals.size] = vals
    S3, S1 = b["S3"], b["S1"]
    shards3 = [np.ascontiguousarray(bucket[j * S3:(j + 1) * S3]) for j in range(plan["z3"])]
    assert np.array_equal(on.gather_concat(shards3), bucket)
    shards1 = [np.ascontiguousarray(bucket[i * S1:(i + 1) * S1]) for i in range(plan["z1"])]
    K = plan["K"]
    rebuilt3 = [on.gather_concat(shards1[j * K:(j + 1) * K]) for j in range(plan["z3"])]
    for j in range(plan["z3"]):
        assert np.array_equal(rebuilt3[j], shards3[j])
    for t, vals in enumerate(tensors):
        rec = plan["tensors"][t]
        got = on.unpack_tensor(shards3, rec["offset"], rec["numel"])
        assert np.array_equal(got, vals)
        # brute force: walk the bucket positions one by one
        want = [int(shards3[(rec["offset"] + y) // S3][(rec["offset"] + y) % S3])
                for y in range(rec["numel"])]
        assert got.tolist() == want
    with pytest.raises(ValueError):
        on.unpack_tensor(shards3, b["P"] - 3, 4)


def test_gather_shard_free_group_sizes_brute_force():
    """Shard j rebuilt from all ZeRO-1 pieces equals the element-by-element walk
    bucket[j*S3 + x] = piece[(j*S3 + x) // S1][(j*S3 + x) % S1], and equals placing the
    pieces the planner's cover lists -- for group sizes that do not nest."""
    rng = np.random.default_rng(13)
    for z1, z2, z3 in [(6, 2, 4), (2, 4, 4), (5, 3, 2), (8, 4, 2), (3, 3, 7)]:
        plan = op.make_plan([2], [37, 150], 8, z3, z1, z2)
        b = plan["buckets"][0]
        S1, S3 = b["S1"], b["S3"]
        pieces = [rng.integers(0, 1 << 16, size=S1).astype(np.uint16) for _ in range(z1)]
        for j in range(z3):
            got = on.gather_shard(pieces, j, z3)
            want = [int(pieces[(j * S3 + x) // S1][(j * S3 + x) % S1]) for x in range(S3)]
            assert got.tolist() == want
            placed = np.zeros(S3, dtype=np.uint16)
            for i, src, dst, n in op.cover(plan, b, j):
                placed[dst:dst + n] = pieces[i][src:src + n]
            assert np.array_equal(placed, got)
