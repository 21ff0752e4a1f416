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


def assert_close_f32(got, want, what, rel=REL_TOL):
    """|got-want| <= rel * max(|got|, |want|, rms(want)), element by element.

    The relative bound is 2e-6; elements smaller than the array's RMS are judged against the
    RMS, because beta1*m + (1-beta1)*g and p - lr*(...) cancel and leave a rounding error
    proportional to the operands rather than to the result.  Non-finite values must match in
    kind at the same index.
    """
    g64, w64 = got.astype(np.float64), want.astype(np.float64)
    fin = np.isfinite(w64)
    assert np.array_equal(np.isfinite(g64), fin), what + ": non-finite pattern differs"
    if not fin.all():
        assert np.array_equal(np.isnan(g64), np.isnan(w64)), what + ": NaN pattern differs"
        g64, w64 = g64[fin], w64[fin]
    if w64.size == 0:
        return
    rms = math.sqrt(float(np.mean(w64 * w64)))
    scale = np.maximum(np.maximum(np.abs(g64), np.abs(w64)), rms)
    err = np.abs(g64 - w64)
    bad = err > rel * scale
    assert not bad.any(), "%s: %d of %d outside %g (worst %g relative)" % (
        what, int(bad.sum()), bad.size, rel, float(np.max(err / np.maximum(scale, 1e-300))))


def bf16_ulp_distance(a, b):
    """Distance in units of the last place between bf16 patterns of equal sign (NaN excluded)."""
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a) - key(b))


def assert_bf16_within_one_ulp(got, want, what, p_ref=None):
    """Cast parameters: at most one bf16 ulp from the oracle's cast parameters.

    An element far below the array's RMS is judged like the fp32 parameter it is the cast of:
    there the fp32 tolerance (REL_TOL * rms, see assert_close_f32) is wider than a bf16 ulp of the
    element, so two correct fp32 values may round to bf16 values several ulps apart.  With
    `p_ref` (the oracle's fp32 parameters) such an element passes if its value is within one
    bf16 ulp plus that fp32 tolerance of the oracle's."""
    nan_w = (want & 0x7F80 == 0x7F80) & (want & 0x007F != 0)
    nan_g = (got & 0x7F80 == 0x7F80) & (got & 0x007F != 0)
    assert np.array_equal(nan_g, nan_w), what + ": NaN pattern differs"
    d = bf16_ulp_distance(got, want)
    d[nan_w] = 0
    bad = d > 1
    if bad.any() and p_ref is not None:
        p64 = p_ref.astype(np.float64)
        p64 = p64[np.isfinite(p64)]
        floor = REL_TOL * math.sqrt(float(np.mean(p64 * p64))) if p64.size else 0.0
        val = lambda u: (u.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        w = want[bad]
        ulp = np.abs(val(w + np.uint16(1)) - val(w))
        bad[bad] = np.abs(val(got[bad]) - val(w)) > ulp + floor
    assert not bad.any(), "%s: %d elements more than one bf16 ulp away (worst %d)" % (
        what, int(bad.sum()), int(d[bad].max()))


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
