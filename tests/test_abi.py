"""The C-ABI library loads without a GPU and exports every symbol the header declares;
argument validation returns status codes before any kernel launch."""
import ctypes
import os
import re

import pytest

import paper_2510_20111_amd as hzp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "hzp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hzp_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared_functions()
    assert sorted(names) == sorted(hzp.EXPORTS)
    lib = ctypes.CDLL(hzp.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_header_is_plain_c_and_struct_layouts_match_the_binding(tmp_path):
    """hzp.h compiles as C99 with no other include, and a C program's sizeof/offsetof of every
    struct the binding mirrors agree with the ctypes declarations."""
    import subprocess
    from paper_2510_20111_amd import binding as bd
    pairs = [("hzp_plan_desc_t", bd.PlanDesc), ("hzp_plan_info_t", bd.PlanInfo), ("hzp_bucket_info_t", bd.BucketInfo),
             ("hzp_tensor_info_t", bd.TensorInfo), ("hzp_adamw_t", bd.AdamW), ("hzp_sched_desc_t", bd.SchedDesc),
             ("hzp_sched_stats_t", bd.SchedStats)]
    lines = ['#include "hzp.h"', "#include <stdio.h>", "#include <stddef.h>", "int main(void) {"]
    for cname, ct in pairs:
        lines.append('printf("%s %%zu", sizeof(%s));' % (cname, cname))
        for fname, _ in ct._fields_:
            lines.append('printf(" %%zu", offsetof(%s, %s));' % (cname, fname))
        lines.append('printf("\\n");')
    lines.append("return 0; }")
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    for (cname, ct), line in zip(pairs, out):
        got = line.split()
        want = [cname, str(ctypes.sizeof(ct))] + [str(getattr(ct, f).offset) for f, _ in ct._fields_]
        assert got == want, cname


def test_binding_has_the_same_names():
    for n in ("hzp_plan", "hzp_plan_free", "hzp_reduce_shard", "hzp_adamw_shard",
              "hzp_gather_layer", "hzp_last_error"):
        assert callable(getattr(hzp, n))


def _plan():
    return hzp.hzp_plan([2, 1], [100, 40, 9], align=8, z3=2, z1=4, tensor_class=[0, 1, 0])


def _status(fn, *a, **k):
    with pytest.raises(hzp.HzpError) as e:
        fn(*a, **k)
    assert hzp.hzp_last_error() != ""
    return e.value.status


FAKE = 0x10000      # a non-null, 16-byte aligned address that is never dereferenced on these paths


@pytest.mark.parametrize("kw,want", [
    (dict(align=12), hzp.HZP_ERR_INVALID_ARG),
    (dict(align=4), hzp.HZP_ERR_INVALID_ARG),
    (dict(z3=0), hzp.HZP_ERR_INVALID_ARG),
    (dict(z1=0), hzp.HZP_ERR_INVALID_ARG),
    (dict(z3=65537, z1=65536, z2=65539), hzp.HZP_ERR_UNSUPPORTED),      # lcm exceeds 32 bits
    (dict(tensor_numel=[0, 5]), hzp.HZP_ERR_INVALID_ARG),
    (dict(tensors_per_layer=[0, 2]), hzp.HZP_ERR_INVALID_ARG),
    (dict(tensor_class=[0, 2]), hzp.HZP_ERR_INVALID_ARG),
    (dict(tensor_numel=[2 ** 63, 2 ** 63]), hzp.HZP_ERR_INVALID_ARG),
])
def test_plan_errors(kw, want):
    d = dict(tensors_per_layer=[2], tensor_numel=[3, 5], align=8, z3=2, z1=8)
    d.update(kw)
    assert _status(hzp.hzp_plan, **d) == want


def test_plan_query_errors():
    p = _plan()
    assert _status(p.bucket, 2, 0) == hzp.HZP_ERR_RANGE
    assert _status(p.bucket, 1, 1) == hzp.HZP_ERR_RANGE          # layer 1 has no fp32 tensor
    assert _status(p.tensor, 3) == hzp.HZP_ERR_RANGE
    assert _status(p.rank, 4) == hzp.HZP_ERR_RANGE
    assert _status(p.shard, 0, 0, 0, 0) == hzp.HZP_ERR_RANGE
    assert _status(p.shard, 0, 0, 4, 0) == hzp.HZP_ERR_RANGE
    assert _status(p.shard, 0, 0, 1, 4) == hzp.HZP_ERR_RANGE
    assert _status(p.index, 4, 0) == hzp.HZP_ERR_RANGE
    assert _status(p.index, 1, 4) == hzp.HZP_ERR_RANGE
    assert _status(p.cover, 0, 0, 2) == hzp.HZP_ERR_RANGE
    assert _status(p.cover, 1, 1, 0) == hzp.HZP_ERR_RANGE


def test_reduce_argument_errors():
    p = _plan()
    f = hzp.hzp_reduce_shard
    assert _status(f, p, 0, 0, 1, 0, [FAKE] * 33, 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_UNSUPPORTED
    assert _status(f, p, 0, 0, 1, 0, [], 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 0, 1, 0, [FAKE, 0], 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 0, 1, 0, [FAKE, FAKE + 2], 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 0, 1, 0, [FAKE], 1.0, 0, FAKE + 4, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 0, 1, 0, [FAKE], 1.0, 0, 0, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 5, 0, 1, 0, [FAKE], 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 0, 0, 0, [FAKE], 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 0, 4, 0, [FAKE], 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 0, 1, 9, [FAKE], 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_RANGE


def test_adamw_argument_errors():
    p = _plan()
    f = hzp.hzp_adamw_shard
    hy = hzp.adamw_hyper(1e-4, 0.9, 0.95, 1e-8, 0.1, 0.5, 1)
    one = [FAKE]
    assert _status(f, p, 0, 0, 0, 0, hy, one, 1, one, one, one, one, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 3, 0, 0, hy, one * 3, 1, one * 3, one * 3, one * 3, None, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 1, 2, 0, hy, one, 1, one, one, one, one, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 1, 0, 7, hy, one, 1, one, one, one, one, stream=0) == hzp.HZP_ERR_RANGE
    hy0 = hzp.adamw_hyper(1e-4, 0.9, 0.95, 1e-8, 0.1, 0.5, 0)
    assert _status(f, p, 0, 1, 0, 0, hy0, one, 1, one, one, one, one, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 1, 0, 0, hy, one * 33, 33, one, one, one, one, stream=0) == hzp.HZP_ERR_UNSUPPORTED
    assert _status(f, p, 0, 1, 0, 0, hy, one, 1, [0], one, one, one, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 1, 0, 0, hy, one, 1, one, [FAKE + 8], one, one, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 1, 0, 0, hy, [FAKE + 2], 1, one, one, one, one, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 1, 0, 0, hy, one, 1, one, one, one, [0], stream=0) == hzp.HZP_ERR_INVALID_ARG


def test_adamw_scalars_and_the_device_form_argument_errors():
    import numpy as np
    hy = hzp.adamw_hyper(1e-4, 0.9, 0.95, 1e-8, 0.1, 0.125, 3)
    f = np.array(hzp.hzp_adamw_scalars(hy), np.float32)
    f32 = np.float32
    b1, b2 = f32(0.9), f32(0.95)
    want = [f32(1e-4), b1, b2, f32(1) - b1, f32(1) - b2, f32(1e-8), f32(0.1), f32(0.125),
            f32(1.0 / (1.0 - float(b1) ** 3)), f32(1.0 / (1.0 - float(b2) ** 3)), f32(0), f32(0)]
    assert np.array_equal(f.view(np.uint32), np.array(want, np.float32).view(np.uint32))
    assert abs(float(f[8]) - 1.0 / 0.271) < 1e-5 and abs(float(f[9]) - 1.0 / 0.142625) < 1e-5   # closed forms at step 3
    assert _status(hzp.hzp_adamw_scalars, hzp.adamw_hyper(1e-4, 0.9, 0.95, 1e-8, 0.1, 0.5, 0)) == hzp.HZP_ERR_INVALID_ARG
    assert _status(hzp.hzp_adamw_scalars, None) == hzp.HZP_ERR_INVALID_ARG
    p = _plan()
    g = hzp.hzp_adamw_shard_dev
    one = [FAKE]
    assert _status(g, p, 0, 1, 0, 0, 0, one, 1, one, one, one, one, stream=0) == hzp.HZP_ERR_INVALID_ARG      # NULL scalars
    assert _status(g, p, 0, 1, 0, 0, FAKE + 4, one, 1, one, one, one, one, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(g, p, 0, 0, 0, 0, FAKE, one, 1, one, one, one, one, stream=0) == hzp.HZP_ERR_INVALID_ARG   # empty range
    assert _status(g, p, 0, 1, 0, 0, FAKE, one, 1, [0], one, one, one, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(g, p, 0, 1, 0, 0, FAKE, one * 33, 33, one, one, one, one, stream=0) == hzp.HZP_ERR_UNSUPPORTED


def test_arena_tune_argument_errors_before_any_gpu_call():
    p = _plan()
    f = p.arena_tune
    big = 1 << 30
    base = hzp.HZP_ARENA_ALIGN * 16
    assert _status(f, 0, 0, 1, 0, big, stream=0) == hzp.HZP_ERR_INVALID_ARG            # NULL arena
    assert _status(f, 2, 0, 1, base, big, stream=0) == hzp.HZP_ERR_RANGE               # class
    assert _status(f, 0, 99, 1, base, big, stream=0) == hzp.HZP_ERR_RANGE              # rank
    assert _status(f, 0, 0, 0, base, big, stream=0) == hzp.HZP_ERR_INVALID_ARG         # R == 0
    assert _status(f, 0, 0, 33, base, big, stream=0) == hzp.HZP_ERR_UNSUPPORTED
    assert _status(f, 0, 0, 1, base + 4096, big, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, 0, 0, 1, base, p.arena(0, 1) - 1, stream=0) == hzp.HZP_ERR_INVALID_ARG   # variant 0 does not fit


def test_gather_argument_errors():
    p = _plan()
    f = hzp.hzp_gather_layer
    assert _status(f, p, 0, 0, 3, [FAKE], FAKE, None, stream=0) == hzp.HZP_ERR_INVALID_ARG      # needs Z3=2 shards
    assert _status(f, p, 0, 0, 1, [FAKE] * 3, FAKE, None, stream=0) == hzp.HZP_ERR_INVALID_ARG  # needs K=2
    assert _status(f, p, 0, 0, 3, [FAKE] * 2, None, None, stream=0) == hzp.HZP_ERR_INVALID_ARG  # no output
    assert _status(f, p, 0, 0, 1, [FAKE] * 2, FAKE, [FAKE], stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 0, 3, [FAKE, FAKE + 8], FAKE, None, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 0, 3, [FAKE] * 2, FAKE + 2, None, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 0, 3, [FAKE] * 2, None, [FAKE + 1], stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 0, 3, [FAKE] * 2, None, [0], stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 0, 2, [FAKE] * 2, FAKE, None, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 1, 1, 3, [FAKE] * 2, FAKE, None, stream=0) == hzp.HZP_ERR_RANGE
    big = hzp.hzp_plan([1], [8 * 128], align=8, z3=128, z1=128)
    assert _status(f, big, 0, 0, 3, [FAKE] * 128, FAKE, None, stream=0) == hzp.HZP_ERR_UNSUPPORTED
    loose = hzp.hzp_plan([1], [100], align=8, z3=4, z1=6, z2=2)      # Z3 does not divide Z1
    assert _status(f, loose, 0, 0, 1, [FAKE] * 2, FAKE, None, stream=0) == hzp.HZP_ERR_UNSUPPORTED


def test_gather_layers_argument_errors():
    p = _plan()                      # 2 layers; z3 = 2, K = 2; layer 1 has no fp32 bucket
    f = hzp.hzp_gather_layers
    two = [FAKE] * 4
    assert _status(f, p, 0, 0, 0, 3, two, 2, [FAKE] * 2, stream=0) == hzp.HZP_ERR_INVALID_ARG      # empty range
    assert _status(f, p, 0, 3, 0, 3, two, 2, [FAKE] * 2, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 2, 2, 3, two, 2, [FAKE] * 2, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 2, 0, 2, two, 2, [FAKE] * 2, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 2, 0, 3, two, 3, [FAKE] * 2, stream=0) == hzp.HZP_ERR_INVALID_ARG      # Z3 = 2 per layer
    assert _status(f, p, 0, 2, 0, 3, [FAKE, FAKE, FAKE, 0], 2, [FAKE] * 2, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 2, 0, 3, [FAKE, FAKE + 4, FAKE, FAKE], 2, [FAKE] * 2, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 2, 0, 3, two, 2, [FAKE, 0], stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 2, 0, 1, two, 2, [FAKE, FAKE + 2], stream=0) == hzp.HZP_ERR_ALIGN
    loose = hzp.hzp_plan([1], [100], align=8, z3=4, z1=6, z2=2)
    assert _status(f, loose, 0, 1, 0, 1, [FAKE] * 2, 2, [FAKE], stream=0) == hzp.HZP_ERR_UNSUPPORTED


def test_gather_tensor_argument_errors():
    p = _plan()
    f = hzp.hzp_gather_tensor
    assert _status(f, p, 3, [FAKE] * 2, FAKE, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, [FAKE], FAKE, stream=0) == hzp.HZP_ERR_INVALID_ARG           # needs Z3 = 2 entries
    assert _status(f, p, 0, [FAKE] * 2, 0, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, [0, 0], FAKE, stream=0) == hzp.HZP_ERR_INVALID_ARG            # the shard it lies in
    assert _status(f, p, 0, [FAKE + 8, FAKE], FAKE, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, [FAKE] * 2, FAKE + 1, stream=0) == hzp.HZP_ERR_ALIGN          # bf16 needs 2-byte alignment


def test_gather_layer_static_argument_errors():
    p = _plan()
    f = hzp.hzp_gather_layer_static
    assert _status(f, p, 0, 0, [FAKE], [FAKE], stream=0) == hzp.HZP_ERR_INVALID_ARG               # needs Z3 = 2 shards
    assert _status(f, p, 0, 0, [FAKE] * 2, None, stream=0) == hzp.HZP_ERR_INVALID_ARG            # tensor_out is required
    assert _status(f, p, 0, 0, [FAKE, 0], [FAKE], stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 0, [FAKE, FAKE + 8], [FAKE], stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 0, [FAKE] * 2, [FAKE + 1], stream=0) == hzp.HZP_ERR_ALIGN            # bf16: 2-byte aligned
    assert _status(f, p, 0, 1, [FAKE] * 2, [FAKE + 2], stream=0) == hzp.HZP_ERR_ALIGN            # fp32: 4-byte aligned
    assert _status(f, p, 0, 0, [FAKE] * 2, [0], stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 2, 0, [FAKE] * 2, [FAKE], stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 1, 1, [FAKE] * 2, [FAKE], stream=0) == hzp.HZP_ERR_RANGE                # no fp32 bucket in layer 1
    many = hzp.hzp_plan([4097], [8] * 4097, align=8, z3=1, z1=1)     # one piece per tensor: 4097 > 4096
    assert _status(f, many, 0, 0, [FAKE], [FAKE] * 4097, stream=0) == hzp.HZP_ERR_UNSUPPORTED
    assert "4096" in hzp.hzp_last_error()
    big = hzp.hzp_plan([1], [8 * 128], align=8, z3=128, z1=128)
    assert _status(f, big, 0, 0, [FAKE] * 128, [FAKE], stream=0) == hzp.HZP_ERR_UNSUPPORTED


def test_gather_shard_argument_errors():
    p = hzp.hzp_plan([1], [100], align=8, z3=4, z1=6, z2=2)          # S1 = 32, S3 = 48: two owners per shard
    f = hzp.hzp_gather_shard
    assert p.cover(0, 0, 1) == (1, 2)
    assert _status(f, p, 0, 0, 1, [FAKE], FAKE, stream=0) == hzp.HZP_ERR_INVALID_ARG            # cover has 2
    assert _status(f, p, 0, 0, 1, [FAKE] * 3, FAKE, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 0, 4, [FAKE] * 2, FAKE, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 1, 0, 0, [FAKE] * 2, FAKE, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 1, 0, [FAKE] * 2, FAKE, stream=0) == hzp.HZP_ERR_RANGE
    assert _status(f, p, 0, 0, 1, [FAKE, 0], FAKE, stream=0) == hzp.HZP_ERR_INVALID_ARG
    assert _status(f, p, 0, 0, 1, [FAKE, FAKE + 4], FAKE, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 0, 1, [FAKE] * 2, FAKE + 8, stream=0) == hzp.HZP_ERR_ALIGN
    assert _status(f, p, 0, 0, 1, [FAKE] * 2, 0, stream=0) == hzp.HZP_ERR_INVALID_ARG
    wide = hzp.hzp_plan([1], [8], align=8, z3=1, z1=65)              # 65 owners for the one shard
    assert _status(f, wide, 0, 0, 0, [FAKE] * 65, FAKE, stream=0) == hzp.HZP_ERR_UNSUPPORTED


def test_scheduler_argument_errors_before_any_gpu_call():
    p = _plan()
    for kw, want in [(dict(gather_slots=0), hzp.HZP_ERR_INVALID_ARG),
                     (dict(queue_capacity=0), hzp.HZP_ERR_INVALID_ARG),
                     (dict(cls=2), hzp.HZP_ERR_RANGE)]:
        with pytest.raises(hzp.HzpError) as e:
            hzp.Sched(p, **kw)
        assert e.value.status == want
    only_bf16 = hzp.hzp_plan([1], [64], align=8, z3=1, z1=1)
    with pytest.raises(hzp.HzpError) as e:
        hzp.Sched(only_bf16, cls=hzp.HZP_CLASS_F32)
    assert e.value.status == hzp.HZP_ERR_RANGE
    # every scheduler call refuses a NULL scheduler before touching anything
    import ctypes
    L = ctypes.CDLL(hzp.LIB_PATH)
    for name, args in [("hzp_sched_prefetch_params", (None, 0, None, 0, None)),
                       ("hzp_sched_acquire_params", (None, 0, None, None)),
                       ("hzp_sched_release_params", (None, 0, None)),
                       ("hzp_sched_release_tensor", (None, 0, None)),
                       ("hzp_sched_join", (None, None)), ("hzp_sched_drain", (None,))]:
        fn = getattr(L, name)
        fn.restype = ctypes.c_int
        assert fn(*args) == hzp.HZP_ERR_INVALID_ARG, name


def test_shards_of_2_to_the_30_elements_are_refused_before_any_launch():
    """Kernels address a slice with a 32-bit byte offset; the entry points refuse longer slices."""
    big = hzp.hzp_plan([1], [1 << 31], align=8, z3=1, z1=2)          # S1 = 2^30, S3 = 2^31
    hy = hzp.adamw_hyper(1e-4, 0.9, 0.95, 1e-8, 0.1, 1.0, 1)
    one = [FAKE]
    assert _status(hzp.hzp_reduce_shard, big, 0, 0, 1, 0, one, 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_UNSUPPORTED
    assert _status(hzp.hzp_reduce_shard, big, 0, 0, 3, 0, one, 1.0, 0, FAKE, stream=0) == hzp.HZP_ERR_UNSUPPORTED
    assert _status(hzp.hzp_adamw_shard, big, 0, 1, 0, 0, hy, one, 1, one, one, one, one, stream=0) == hzp.HZP_ERR_UNSUPPORTED
    ok = hzp.hzp_plan([1], [1 << 31], align=8, z3=1, z1=4)           # S1 = 2^29 passes the size check
    assert ok.bucket(0).s1 == 1 << 29


def test_a_plain_c_program_can_plan_through_the_library(tmp_path):
    """hzp.h + libhzp.so used from C without Python in between: plan, read-back, memory model."""
    import subprocess
    from oracle import planner as op
    src = tmp_path / "plan.c"
    src.write_text(r"""
#include <stdio.h>
#include "hzp.h"
int main(void) {
    const uint32_t per_layer[2] = {2, 1};
    const uint64_t numel[3] = {1000, 77, 4096};
    hzp_plan_desc_t d = {2, per_layer, numel, NULL, NULL, 16, 4, 2, 6};      /* A=16, Z3=4, Z2=2, Z1=6 */
    hzp_plan_t *plan = NULL;
    if (hzp_plan(&d, &plan) != HZP_OK) { printf("error: %s\n", hzp_last_error()); return 1; }
    hzp_plan_info_t info;
    hzp_plan_info(plan, &info);
    printf("%u %u %llu\n", info.world, info.k, (unsigned long long)info.total_padded);
    for (uint32_t l = 0; l < 2; ++l) {
        hzp_bucket_info_t b;
        hzp_plan_bucket(plan, l, HZP_CLASS_BF16, &b);
        printf("%llu %llu %llu %llu %llu\n", (unsigned long long)b.payload_end, (unsigned long long)b.padded,
               (unsigned long long)b.s1, (unsigned long long)b.s2, (unsigned long long)b.s3);
    }
    uint32_t first, n;
    hzp_plan_cover(plan, 0, HZP_CLASS_BF16, 1, &first, &n);
    uint64_t bytes;
    hzp_memory_model(7000000000ull, 64, 8, 8, &bytes);
    uint32_t z1, z2, z3;
    hzp_status_t st = hzp_choose_groups(7000000000ull, 64, 8, 22000000000ull, &z1, &z2, &z3);
    printf("%u %u %llu %d %u %u %u\n", first, n, (unsigned long long)bytes, (int)st, z1, z2, z3);
    d.align_elems = 12;
    printf("%d\n", (int)hzp_plan(&d, &plan));                                 /* refused: not a power of two */
    hzp_plan_free(plan);
    return 0;
}
""")
    exe = tmp_path / "plan"
    libdir = os.path.dirname(hzp.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-l:" + os.path.basename(hzp.LIB_PATH), "-Wl,-rpath," + libdir,
                    "-Wl,--allow-shlib-undefined"], check=True)
    import torch
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = os.pathsep.join([os.path.join(os.path.dirname(torch.__file__), "lib"), "/opt/rocm/lib",
                                              env.get("LD_LIBRARY_PATH", "")])
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, env=env).stdout.split("\n")
    want = op.make_plan([2, 1], [1000, 77, 4096], 16, 4, 6, 2)
    assert out[0].split() == [str(want["world"]), str(want["K"]), str(want["total_padded"])]
    for l in range(2):
        b = want["buckets"][l]
        assert [int(x) for x in out[1 + l].split()] == [b["payload_end"], b["P"], b["S1"], b["S2"], b["S3"]]
    cover = op.cover(want, want["buckets"][0], 1)
    mem = op.hzp_memory_bytes(7000000000, 64, 8, 8)
    assert out[3].split() == [str(cover[0][0]), str(len(cover)), str(-(-mem.numerator // mem.denominator)), "0", "8", "4", "4"]
    assert out[4].split() == [str(hzp.HZP_ERR_INVALID_ARG)]
