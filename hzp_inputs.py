"""Seeded synthetic workloads shared by the tests, the smoke check and the benchmark.

This module holds shapes and random values only.  It contains none of the
method's arithmetic: no layout rule, no reduction, no optimizer step.  Where a
generator needs to know which bucket positions are payload and which are
padding, the caller passes the (offset, numel) ranges it obtained from
whichever planner it is exercising.

The paper's workloads (dense Seed-OSS models and a DeepSeek-V3-like MoE,
Section 5.1, all run with Z1 >> Z2 = Z3 = 8) are characterised only by name;
the five model-shaped tensor lists below stand in for them: dense transformer
layers, an MoE expert set, and an irregular multi-tensor stress case.
Values: gradients N(0, sigma) rounded to bf16 (library cast), master weights
N(0, 0.02) in fp32, momentum and variance zero, padding zero everywhere.
"""
import math

import numpy as np

CLASS_BF16 = 0
CLASS_F32 = 1

ADAMW = dict(lr=1e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def _dense_layer(hidden, ffn, q_out=None, kv_out=None):
    q_out = hidden if q_out is None else q_out
    kv_out = hidden if kv_out is None else kv_out
    names = ["attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"]
    sizes = [hidden, q_out * hidden, kv_out * hidden, kv_out * hidden, hidden * q_out,
             hidden, ffn * hidden, ffn * hidden, hidden * ffn]
    return names, sizes


def config(idx):
    """Workload `idx` (0..4) as plain lists: tiny, dense7b, dense70b, moe, irregular."""
    if idx == 0:      # tiny 2-layer transformer state, 16 tensors
        layers = [("embed", ["tok_embed", "final_norm"], [1024 * 256, 256])]
        for l in range(2):
            layers.append(("layer%d" % l,
                           ["ln1", "wqkv", "wo", "ln2", "w_up", "b_up", "w_down"],
                           [256, 768 * 256, 256 * 256, 256, 1024 * 256, 1024, 256 * 1024]))
        cfg = dict(name="tiny", align=128, z3=2, z1=4, R=4, sigma=1e-3)
    elif idx == 1:    # 7B-class dense rank share
        names, sizes = _dense_layer(4096, 11008)
        layers = [("layer%d" % l, names, sizes) for l in range(32)]
        layers.append(("embed", ["tok_embed"], [32000 * 4096]))
        layers.append(("head", ["lm_head", "final_norm"], [32000 * 4096, 4096]))
        cfg = dict(name="dense7b", align=128, z3=8, z1=64, R=8, sigma=1e-3)
    elif idx == 2:    # 70B-class dense layer stream, GQA 64 query / 8 KV heads, head dim 128
        names, sizes = _dense_layer(8192, 28672, q_out=64 * 128, kv_out=8 * 128)
        layers = [("layer%d" % l, names, sizes) for l in range(80)]
        cfg = dict(name="dense70b", align=128, z3=8, z1=128, R=8, sigma=5e-4)
    elif idx == 3:    # MoE layer set: router + 64 experts + 2 shared experts, 3 matrices each
        names, sizes = ["router"], [4096 * 64]
        for e in range(66):
            tag = "expert%d" % e if e < 64 else "shared%d" % (e - 64)
            names += [tag + ".w_gate", tag + ".w_up", tag + ".w_down"]
            sizes += [1408 * 4096, 1408 * 4096, 4096 * 1408]
        layers = [("layer%d" % l, names, sizes) for l in range(24)]
        cfg = dict(name="moe", align=128, z3=4, z1=16, R=16, sigma=1e-3)
    elif idx == 4:    # irregular multi-tensor stress, 4096 tensors log-uniform in [1, 65536]
        rng = np.random.default_rng(0)
        draw = np.floor(np.exp(rng.uniform(0.0, math.log(65536.0), size=4096))).astype(np.int64)
        draw = np.clip(draw, 1, 65536)
        layers = []
        for l in range(64):
            ids = range(64 * l, 64 * l + 64)
            layers.append(("group%d" % l, ["t%d" % i for i in ids], [int(draw[i]) for i in ids]))
        cfg = dict(name="irregular", align=256, z3=2, z1=32, R=16, sigma=1e-3)
    else:
        raise ValueError("config index 0..4")
    tensors_per_layer = [len(s) for _, _, s in layers]
    tensor_numel = [n for _, _, s in layers for n in s]
    tensor_names = [ln + "." + tn for ln, ns, _ in layers for tn in ns]
    n = len(tensor_numel)
    if idx == 4:      # every fourth tensor is an fp32 1-D state without weight decay
        tensor_class = [CLASS_F32 if i % 4 == 3 else CLASS_BF16 for i in range(n)]
        tensor_wd_mult = [0.0 if i % 4 == 3 else 1.0 for i in range(n)]
    else:
        tensor_class = None
        tensor_wd_mult = None
    cfg.update(layer_names=[ln for ln, _, _ in layers], tensors_per_layer=tensors_per_layer,
               tensor_numel=tensor_numel, tensor_names=tensor_names,
               tensor_class=tensor_class, tensor_wd_mult=tensor_wd_mult,
               grad_scale=1.0 / cfg["R"], adamw=dict(ADAMW))
    return cfg


def irregular_desc(n_tensors, seed, max_numel=5000, tensors_per_layer=4, f32_every=3):
    """A small random descriptor with ragged sizes for parity tests."""
    rng = np.random.default_rng(seed)
    numel = [int(x) for x in
             np.clip(np.floor(np.exp(rng.uniform(0.0, math.log(max_numel), size=n_tensors))),
                     1, max_numel)]
    tpl = []
    left = n_tensors
    while left > 0:
        tpl.append(min(tensors_per_layer, left))
        left -= tpl[-1]
    cls = [CLASS_F32 if (f32_every and i % f32_every == f32_every - 1) else CLASS_BF16
           for i in range(n_tensors)]
    wd = [0.0 if c == CLASS_F32 else 1.0 for c in cls]
    return dict(tensors_per_layer=tpl, tensor_numel=numel, tensor_class=cls, tensor_wd_mult=wd)


# --------------------------------------------------------------------------- values

def _rng(*key):
    return np.random.default_rng([int(k) for k in key])


def _payload_mask(n, ranges, begin=0):
    """Boolean mask over bucket positions [begin, begin+n): True inside a payload range."""
    mask = np.zeros(n, dtype=bool)
    for off, numel in ranges:
        lo, hi = max(off, begin), min(off + numel, begin + n)
        if lo < hi:
            mask[lo - begin:hi - begin] = True
    return mask


def to_bf16_bits(x_f32):
    """Round float32 values to bf16 with the library cast; return uint16 bit patterns."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x_f32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def grad_bucket(seed, step, layer, replica, P, ranges, sigma, cls=CLASS_BF16):
    """One replica's gradient for a whole padded bucket (padding positions are zero)."""
    g = (_rng(seed, 1, step, layer, replica, cls).standard_normal(P, dtype=np.float32)
         * np.float32(sigma))
    g[~_payload_mask(P, ranges)] = 0.0
    return g if cls == CLASS_F32 else to_bf16_bits(g)


def master_bucket(seed, layer, P, ranges, cls=CLASS_BF16, std=0.02):
    """Initial fp32 master weights for a whole padded bucket (padding positions are zero)."""
    p = _rng(seed, 2, layer, cls).standard_normal(P, dtype=np.float32) * np.float32(std)
    p[~_payload_mask(P, ranges)] = 0.0
    return p


def device_normal(n, std, seed, device, dtype, ranges=None, begin=0):
    """N(0, std) values generated on `device` with torch's seeded generator.

    Used for the full-size workloads, where host generation would take minutes.
    `ranges` (bucket-relative payload ranges) and `begin` (bucket position of
    element 0) zero the padding part of the slice, if any.
    """
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    x = torch.empty(n, dtype=torch.float32, device=device)
    x.normal_(0.0, std, generator=gen)
    if ranges is not None:
        covered = 0
        keep = torch.zeros(n, dtype=torch.bool, device=device)
        for off, numel in ranges:
            lo, hi = max(off, begin), min(off + numel, begin + n)
            if lo < hi:
                keep[lo - begin:hi - begin] = True
                covered += hi - lo
        if covered < n:
            x.mul_(keep)
    return x.to(dtype)
