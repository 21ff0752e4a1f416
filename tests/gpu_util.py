"""Helpers of the GPU parity tests: host<->device moves, tolerances, oracle drivers."""
import math

import numpy as np
import torch

import hzp_inputs
from oracle import numeric as on
from oracle import planner as op

DEV = "cuda:0"
REL_TOL = 2e-6          # fp32 master / momentum / variance against the fp64 evaluation
POISON16 = 0x7FC1       # a NaN pattern used for guard bands (positive as int16)
POISON32 = 0x7FC12345


def to_dev(a):
    """numpy array (uint16 / float32 / uint32) -> device tensor with the same bits."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def to_host(t, dtype):
    """device tensor -> numpy array reinterpreted as `dtype`."""
    a = t.detach().cpu().contiguous()
    if a.dtype == torch.bfloat16:
        a = a.view(torch.int16)
    return a.numpy().view(dtype)


# Additive floors, as multiples of the array's RMS, on top of the 2e-6 relative bound.  An element
# far below the RMS of its array cannot meet a purely relative bound in fp32: beta1*m + (1-beta1)*g
# and p - lr*(...) cancel, and their rounding error (a few 2^-24 of the operands) is proportional to
# the operands.  Measured on 2e7 samples of the tiny workload, the oracle's own fp32 evaluation needs
# 4.4e-7*rms for m and 6e-9*rms for p against its fp64 evaluation, and nothing for v (a sum of
# positive terms).  The floors below leave a factor of 2-3 over that.
RMS_FLOOR = {"p": 2e-8, "m": 1e-6, "v": 0.0}
TINY = 1e-37            # below the normal range an fp32 value has no relative precision
# The step lr*u enters p with the error of u: the kernel's hardware reciprocal and square root (1 ulp
# each) and two multiplications leave u good to about 2.5e-7 relative, and |u| stays below about 2.
U_ERR = 5e-7


def assert_close_f32(got, want, what, kind, rel=REL_TOL, lr=hzp_inputs.ADAMW["lr"]):
    """|got-want| <= rel * max(|got|, |want|) + RMS_FLOOR[kind] * rms(want) (+ U_ERR * lr for p),
    element by element (kind: "p", "m" or "v").  Non-finite values must match in kind at the same
    index."""
    g64, w64 = got.astype(np.float64), want.astype(np.float64)
    fin = np.isfinite(w64)
    assert np.array_equal(np.isfinite(g64), fin), what + ": non-finite pattern differs"
    if not fin.all():
        assert np.array_equal(np.isnan(g64), np.isnan(w64)), what + ": NaN pattern differs"
        g64, w64 = g64[fin], w64[fin]
    if w64.size == 0:
        return
    rms = math.sqrt(float(np.mean(w64 * w64)))
    bound = rel * np.maximum(np.abs(g64), np.abs(w64)) + RMS_FLOOR[kind] * rms + TINY
    if kind == "p":
        bound = bound + U_ERR * lr
    err = np.abs(g64 - w64)
    bad = err > bound
    assert not bad.any(), "%s: %d of %d outside the bound (worst %g of it)" % (
        what, int(bad.sum()), bad.size, float(np.max(err / bound)))


def bf16_ulp_distance(a, b):
    """Distance in units of the last place between bf16 patterns of equal sign (NaN excluded)."""
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a) - key(b))


def assert_cast_of(got16, p_gpu, what):
    """Cast parameters: param_out must be the round-to-nearest-even bf16 cast of the fp32 parameters
    the GPU itself produced, bit for bit (the oracle's cast applied to the GPU's p; NaN matches any
    NaN).  Together with the fp32 check of p against the oracle this bounds param_out to one bf16
    ulp of the oracle's cast wherever a bf16 ulp is wider than the fp32 tolerance."""
    want = on.f32_to_bf16_array(np.ascontiguousarray(p_gpu, dtype=np.float32))
    nan_w = (want & 0x7F80 == 0x7F80) & (want & 0x007F != 0)
    nan_g = (got16 & 0x7F80 == 0x7F80) & (got16 & 0x007F != 0)
    assert np.array_equal(nan_g, nan_w), what + ": NaN pattern differs"
    bad = (got16 != want) & ~nan_w
    assert not bad.any(), "%s: %d of %d cast parameters are not bf16(p) (first at %d: %#x vs %#x)" % (
        what, int(bad.sum()), bad.size, int(np.argmax(bad)), int(got16[np.argmax(bad)]), int(want[np.argmax(bad)]))


def assert_bf16_within_one_ulp(got, want, what):
    """bf16 patterns at most one unit in the last place apart (NaN must meet NaN)."""
    nan_w = (want & 0x7F80 == 0x7F80) & (want & 0x007F != 0)
    nan_g = (got & 0x7F80 == 0x7F80) & (got & 0x007F != 0)
    assert np.array_equal(nan_g, nan_w), what + ": NaN pattern differs"
    d = bf16_ulp_distance(got, want)
    d[nan_w] = 0
    assert not (d > 1).any(), "%s: %d elements more than one bf16 ulp away (worst %d)" % (
        what, int((d > 1).sum()), int(d.max()))


def payload_ranges(oplan, bucket):
    return [(oplan["tensors"][t]["offset"], oplan["tensors"][t]["numel"]) for t in bucket["tensor_ids"]]


def wd_mult_array(oplan, bucket, begin, n):
    """Per-element weight-decay multiplier of bucket positions [begin, begin+n) for the oracle:
    the multiplier of the tensor that owns the position (padding: of the tensor before it)."""
    out = np.ones(n, dtype=np.float32)
    recs = [oplan["tensors"][t] for t in bucket["tensor_ids"]]
    for idx, rec in enumerate(recs):
        lo = rec["offset"]
        hi = recs[idx + 1]["offset"] if idx + 1 < len(recs) else bucket["P"]
        lo, hi = max(lo, begin), min(hi, begin + n)
        if lo < hi:
            out[lo - begin:hi - begin] = rec["wd_mult"]
    return out


def oracle_plan(desc, align, z3, z1, z2=0):
    return op.make_plan(desc["tensors_per_layer"], desc["tensor_numel"], align, z3, z1, z2,
                        tensor_class=desc.get("tensor_class"),
                        tensor_wd_mult=desc.get("tensor_wd_mult"))


def guarded(n, torch_dtype, guard=64):
    """Device buffer of n elements with poison-filled guard bands on both sides.
    Returns (whole, view): `view` is 16-byte aligned when guard*itemsize is a multiple of 16."""
    whole = torch.empty(n + 2 * guard, dtype=torch_dtype, device=DEV)
    if whole.element_size() == 2:
        whole.view(torch.int16).fill_(POISON16)
    else:
        whole.view(torch.int32).fill_(POISON32)
    return whole, whole[guard:guard + n]


def guards_intact(whole, n, guard=64):
    it = torch.int16 if whole.element_size() == 2 else torch.int32
    w = whole.view(it)
    want = POISON16 if whole.element_size() == 2 else POISON32
    return bool((w[:guard] == want).all().item()) and bool((w[guard + n:] == want).all().item())
