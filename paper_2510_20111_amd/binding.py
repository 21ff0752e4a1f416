"""ctypes binding of libhzp: argument marshalling only, every step runs in the library.

Function names and argument order follow ``include/hzp.h``.  Device buffers may be given as
torch tensors (their ``data_ptr()`` is taken) or as integer addresses; a stream may be a
``torch.cuda.Stream``, an integer ``hipStream_t`` or None (torch's current stream).
There is no fallback: if ``libhzp.so`` has not been built, importing this module fails.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# HZP_LIBRARY names another build of the same library (the host-only sanitizer build of the tests)
LIB_PATH = os.environ.get("HZP_LIBRARY") or os.path.join(_HERE, "libhzp.so")

HZP_OK, HZP_ERR_INVALID_ARG, HZP_ERR_RANGE, HZP_ERR_UNSUPPORTED, HZP_ERR_ALIGN, HZP_ERR_NOMEM, \
    HZP_ERR_HIP = range(7)
HZP_CLASS_BF16, HZP_CLASS_F32 = 0, 1
HZP_GRAD_DEFAULT, HZP_GRAD_BF16, HZP_GRAD_F32 = 0, 1, 2
HZP_MAX_REPLICAS, HZP_MAX_GROUP = 32, 64
HZP_ARENA_ALIGN = 2 << 20
HZP_ARENA_VARIANTS = 8
(HZP_STREAM_GRAD, HZP_STREAM_MASTER, HZP_STREAM_M, HZP_STREAM_V, HZP_STREAM_PARAM_OUT, HZP_STREAM_RECV1,
 HZP_STREAM_SHARD3, HZP_STREAM_RECV3) = range(8)
_STATUS_NAMES = ["HZP_OK", "HZP_ERR_INVALID_ARG", "HZP_ERR_RANGE", "HZP_ERR_UNSUPPORTED",
                 "HZP_ERR_ALIGN", "HZP_ERR_NOMEM", "HZP_ERR_HIP"]

EXPORTS = ["hzp_plan", "hzp_plan_free", "hzp_plan_prepare", "hzp_plan_info", "hzp_plan_bucket", "hzp_plan_tensor",
           "hzp_plan_rank", "hzp_plan_index", "hzp_plan_cover", "hzp_plan_shard", "hzp_plan_bytes",
           "hzp_plan_arena", "hzp_plan_arena_slice", "hzp_arena_tune", "hzp_adamw_scalars", "hzp_adamw_shard_dev",
           "hzp_reduce_shard", "hzp_adamw_shard", "hzp_gather_layer", "hzp_gather_layer_static", "hzp_gather_layers", "hzp_gather_shard", "hzp_gather_tensor", "hzp_last_error",
           "hzp_memory_model", "hzp_choose_groups",
           "hzp_sched_create", "hzp_sched_destroy", "hzp_sched_prefetch", "hzp_sched_prefetch_ahead", "hzp_sched_acquire",
           "hzp_sched_release", "hzp_sched_prefetch_tensor", "hzp_sched_acquire_tensor",
           "hzp_sched_release_tensor", "hzp_sched_prefetch_params", "hzp_sched_acquire_params",
           "hzp_sched_release_params", "hzp_sched_reduce", "hzp_sched_join", "hzp_sched_drain", "hzp_sched_stats"]


class HzpError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("%s: %s" % (_STATUS_NAMES[status] if 0 <= status < 7 else status, text))
        self.status = status


class PlanDesc(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_uint32),
                ("tensors_per_layer", ctypes.POINTER(ctypes.c_uint32)),
                ("tensor_numel", ctypes.POINTER(ctypes.c_uint64)),
                ("tensor_class", ctypes.POINTER(ctypes.c_uint8)),
                ("tensor_wd_mult", ctypes.POINTER(ctypes.c_float)),
                ("align_elems", ctypes.c_uint32),
                ("z3", ctypes.c_uint32), ("z2", ctypes.c_uint32), ("z1", ctypes.c_uint32)]


class PlanInfo(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_uint32), ("n_buckets", ctypes.c_uint32),
                ("n_tensors", ctypes.c_uint32), ("align_elems", ctypes.c_uint32),
                ("z3", ctypes.c_uint32), ("z2", ctypes.c_uint32), ("z1", ctypes.c_uint32),
                ("k", ctypes.c_uint32), ("world", ctypes.c_uint32), ("total_padded", ctypes.c_uint64)]


class BucketInfo(ctypes.Structure):
    _fields_ = [("layer", ctypes.c_uint32), ("cls", ctypes.c_uint32),
                ("n_tensors", ctypes.c_uint32), ("bucket_index", ctypes.c_uint32),
                ("payload_end", ctypes.c_uint64), ("padded", ctypes.c_uint64),
                ("s3", ctypes.c_uint64), ("s1", ctypes.c_uint64), ("base", ctypes.c_uint64),
                ("s2", ctypes.c_uint64)]


class TensorInfo(ctypes.Structure):
    _fields_ = [("layer", ctypes.c_uint32), ("cls", ctypes.c_uint32),
                ("bucket_index", ctypes.c_uint32), ("index_in_bucket", ctypes.c_uint32),
                ("offset", ctypes.c_uint64), ("numel", ctypes.c_uint64),
                ("wd_mult", ctypes.c_float)]


class SchedDesc(ctypes.Structure):
    _fields_ = [("cls", ctypes.c_uint32), ("gather_slots", ctypes.c_uint32),
                ("queue_capacity", ctypes.c_uint32), ("reserved_", ctypes.c_uint32),
                ("pool_bytes", ctypes.c_uint64)]


class SchedStats(ctypes.Structure):
    _fields_ = [("pool_bytes", ctypes.c_uint64), ("slot_bytes", ctypes.c_uint64),
                ("peak_live_bytes", ctypes.c_uint64), ("peak_live_slots", ctypes.c_uint32),
                ("reserved_", ctypes.c_uint32), ("gathers_issued", ctypes.c_uint64),
                ("reduces_issued", ctypes.c_uint64), ("acquire_host_wait_us", ctypes.c_uint64),
                ("wrap_skipped_bytes", ctypes.c_uint64)]


class AdamW(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("grad_scale", ctypes.c_float), ("step", ctypes.c_uint32)]


class AdamWScalars(ctypes.Structure):
    _fields_ = [("f", ctypes.c_float * 12)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libhzp.so is not built: run `python paper_2510_20111_amd/build.py` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    # torch ships its own HIP runtime (same soname as the system one).  Loading torch first
    # makes libhzp bind to that copy, so both share one runtime, one device context and the
    # same streams; two runtimes in one process cannot both open the GPU.
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, u32, u64p = ctypes.c_void_p, ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint64)
    u32p = ctypes.POINTER(ctypes.c_uint32)
    L.hzp_plan.restype = ctypes.c_int
    L.hzp_plan.argtypes = [ctypes.POINTER(PlanDesc), ctypes.POINTER(vp)]
    L.hzp_plan_free.restype = None
    L.hzp_plan_free.argtypes = [vp]
    L.hzp_plan_prepare.restype = ctypes.c_int
    L.hzp_plan_prepare.argtypes = [vp, vp]
    L.hzp_plan_info.restype = ctypes.c_int
    L.hzp_plan_info.argtypes = [vp, ctypes.POINTER(PlanInfo)]
    L.hzp_plan_bucket.restype = ctypes.c_int
    L.hzp_plan_bucket.argtypes = [vp, u32, u32, ctypes.POINTER(BucketInfo)]
    L.hzp_plan_tensor.restype = ctypes.c_int
    L.hzp_plan_tensor.argtypes = [vp, u32, ctypes.POINTER(TensorInfo)]
    L.hzp_plan_rank.restype = ctypes.c_int
    L.hzp_plan_rank.argtypes = [vp, u32, u32p, u32p, u32p]
    L.hzp_plan_index.restype = ctypes.c_int
    L.hzp_plan_index.argtypes = [vp, ctypes.c_int, u32, u32p]
    L.hzp_plan_cover.restype = ctypes.c_int
    L.hzp_plan_cover.argtypes = [vp, u32, u32, u32, u32p, u32p]
    L.hzp_gather_shard.restype = ctypes.c_int
    L.hzp_gather_shard.argtypes = [vp, u32, u32, u32, vp, u32, vp, vp]
    L.hzp_gather_layers.restype = ctypes.c_int
    L.hzp_gather_layers.argtypes = [vp, u32, u32, u32, ctypes.c_int, vp, u32, vp, vp]
    L.hzp_gather_tensor.restype = ctypes.c_int
    L.hzp_gather_tensor.argtypes = [vp, u32, vp, u32, vp, vp]
    L.hzp_plan_shard.restype = ctypes.c_int
    L.hzp_plan_shard.argtypes = [vp, u32, u32, ctypes.c_int, u32, u64p, u64p]
    L.hzp_plan_arena.restype = ctypes.c_int
    L.hzp_plan_arena.argtypes = [vp, u32, u32, u32, u32, u64p]
    L.hzp_plan_arena_slice.restype = ctypes.c_int
    L.hzp_plan_arena_slice.argtypes = [vp, u32, u32, u32, u32, u32, u32, u32, u64p, u64p]
    L.hzp_arena_tune.restype = ctypes.c_int
    L.hzp_arena_tune.argtypes = [vp, u32, u32, u32, vp, ctypes.c_uint64, vp, ctypes.POINTER(u32), ctypes.POINTER(ctypes.c_double)]
    L.hzp_plan_bytes.restype = ctypes.c_int
    L.hzp_plan_bytes.argtypes = [vp, u64p, u64p, u64p]
    L.hzp_reduce_shard.restype = ctypes.c_int
    L.hzp_reduce_shard.argtypes = [vp, u32, u32, ctypes.c_int, u32, vp, u32, u32, ctypes.c_float,
                                   ctypes.c_int, vp, vp]
    L.hzp_adamw_shard.restype = ctypes.c_int
    L.hzp_adamw_shard.argtypes = [vp, u32, u32, u32, u32, ctypes.POINTER(AdamW), vp, u32,
                                  vp, vp, vp, vp, vp]
    L.hzp_adamw_scalars.restype = ctypes.c_int
    L.hzp_adamw_scalars.argtypes = [ctypes.POINTER(AdamW), ctypes.POINTER(AdamWScalars)]
    L.hzp_adamw_shard_dev.restype = ctypes.c_int
    L.hzp_adamw_shard_dev.argtypes = [vp, u32, u32, u32, u32, vp, vp, u32, vp, vp, vp, vp, vp]
    L.hzp_gather_layer.restype = ctypes.c_int
    L.hzp_gather_layer.argtypes = [vp, u32, u32, ctypes.c_int, vp, u32, vp, vp, vp]
    L.hzp_gather_layer_static.restype = ctypes.c_int
    L.hzp_gather_layer_static.argtypes = [vp, u32, u32, vp, u32, vp, vp]
    L.hzp_memory_model.restype = ctypes.c_int
    L.hzp_memory_model.argtypes = [ctypes.c_uint64, u32, u32, u32, u64p]
    L.hzp_choose_groups.restype = ctypes.c_int
    L.hzp_choose_groups.argtypes = [ctypes.c_uint64, u32, u32, ctypes.c_uint64, u32p, u32p, u32p]
    L.hzp_sched_create.restype = ctypes.c_int
    L.hzp_sched_create.argtypes = [vp, ctypes.POINTER(SchedDesc), ctypes.POINTER(vp)]
    L.hzp_sched_destroy.restype = None
    L.hzp_sched_destroy.argtypes = [vp]
    L.hzp_sched_prefetch.restype = ctypes.c_int
    L.hzp_sched_prefetch.argtypes = [vp, u32, vp, u32, vp]
    L.hzp_sched_prefetch_ahead.restype = ctypes.c_int
    L.hzp_sched_prefetch_ahead.argtypes = [vp, u32, u32, vp, u32, vp, u32p]
    L.hzp_sched_acquire.restype = ctypes.c_int
    L.hzp_sched_acquire.argtypes = [vp, u32, vp, ctypes.POINTER(vp)]
    L.hzp_sched_release.restype = ctypes.c_int
    L.hzp_sched_release.argtypes = [vp, u32, vp]
    L.hzp_sched_prefetch_tensor.restype = ctypes.c_int
    L.hzp_sched_prefetch_tensor.argtypes = [vp, u32, vp, u32, vp]
    L.hzp_sched_acquire_tensor.restype = ctypes.c_int
    L.hzp_sched_acquire_tensor.argtypes = [vp, u32, vp, ctypes.POINTER(vp)]
    L.hzp_sched_release_tensor.restype = ctypes.c_int
    L.hzp_sched_release_tensor.argtypes = [vp, u32, vp]
    L.hzp_sched_prefetch_params.restype = ctypes.c_int
    L.hzp_sched_prefetch_params.argtypes = [vp, u32, vp, u32, vp]
    L.hzp_sched_acquire_params.restype = ctypes.c_int
    L.hzp_sched_acquire_params.argtypes = [vp, u32, vp, ctypes.POINTER(ctypes.c_void_p)]
    L.hzp_sched_release_params.restype = ctypes.c_int
    L.hzp_sched_release_params.argtypes = [vp, u32, vp]
    L.hzp_sched_reduce.restype = ctypes.c_int
    L.hzp_sched_reduce.argtypes = [vp, u32, ctypes.c_int, u32, vp, u32, u32, ctypes.c_float, ctypes.c_int, vp, vp]
    L.hzp_sched_join.restype = ctypes.c_int
    L.hzp_sched_join.argtypes = [vp, vp]
    L.hzp_sched_drain.restype = ctypes.c_int
    L.hzp_sched_drain.argtypes = [vp]
    L.hzp_sched_stats.restype = ctypes.c_int
    L.hzp_sched_stats.argtypes = [vp, ctypes.POINTER(SchedStats)]
    L.hzp_last_error.restype = ctypes.c_char_p
    L.hzp_last_error.argtypes = []
    return L


_L = _load()


def _check(status):
    if status != HZP_OK:
        raise HzpError(status, hzp_last_error())


def hzp_last_error():
    return _L.hzp_last_error().decode("utf-8", "replace")


def _addr(x):
    """Device address of a torch tensor, or the integer itself."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return x.data_ptr()


def ptr_array(items):
    """Host array of device pointers (void*[]) from tensors / integer addresses."""
    if isinstance(items, ctypes.Array):
        return items
    return (ctypes.c_void_p * len(items))(*[_addr(x) for x in items])


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Plan:
    """Owner of an ``hzp_plan_t*``; freed when the object dies."""

    def __init__(self, handle, keep):
        self.handle = handle
        self._keep = keep

    def __del__(self):
        if getattr(self, "handle", None):
            _L.hzp_plan_free(self.handle)
            self.handle = None

    def prepare(self, stream=None):
        _check(_L.hzp_plan_prepare(self.handle, _stream(stream)))

    def info(self):
        out = PlanInfo()
        _check(_L.hzp_plan_info(self.handle, ctypes.byref(out)))
        return out

    def bucket(self, layer, cls=HZP_CLASS_BF16):
        out = BucketInfo()
        _check(_L.hzp_plan_bucket(self.handle, layer, cls, ctypes.byref(out)))
        return out

    def has_bucket(self, layer, cls):
        out = BucketInfo()
        return _L.hzp_plan_bucket(self.handle, layer, cls, ctypes.byref(out)) == HZP_OK

    def tensor(self, tensor_id):
        out = TensorInfo()
        _check(_L.hzp_plan_tensor(self.handle, tensor_id, ctypes.byref(out)))
        return out

    def rank(self, rank):
        j, k, i = ctypes.c_uint32(), ctypes.c_uint32(), ctypes.c_uint32()
        _check(_L.hzp_plan_rank(self.handle, rank, ctypes.byref(j), ctypes.byref(k), ctypes.byref(i)))
        return j.value, k.value, i.value

    def index(self, level, rank):
        out = ctypes.c_uint32()
        _check(_L.hzp_plan_index(self.handle, level, rank, ctypes.byref(out)))
        return out.value

    def cover(self, layer, cls, j):
        first, n = ctypes.c_uint32(), ctypes.c_uint32()
        _check(_L.hzp_plan_cover(self.handle, layer, cls, j, ctypes.byref(first), ctypes.byref(n)))
        return first.value, n.value

    def shard(self, layer, cls, level, rank):
        b, n = ctypes.c_uint64(), ctypes.c_uint64()
        _check(_L.hzp_plan_shard(self.handle, layer, cls, level, rank, ctypes.byref(b), ctypes.byref(n)))
        return b.value, n.value

    def arena(self, cls, R, grad_dtype=HZP_GRAD_DEFAULT, variant=0):
        """Bytes of the one allocation that holds the rank's streams of class `cls`."""
        out = ctypes.c_uint64()
        _check(_L.hzp_plan_arena(self.handle, cls, R, grad_dtype, variant, ctypes.byref(out)))
        return out.value

    def arena_slice(self, cls, R, stream, index, layer, grad_dtype=HZP_GRAD_DEFAULT, variant=0):
        """(byte_offset, bytes) of bucket (layer, cls)'s slice of a stream inside the arena."""
        off, n = ctypes.c_uint64(), ctypes.c_uint64()
        _check(_L.hzp_plan_arena_slice(self.handle, cls, R, grad_dtype, variant, stream, index, layer,
                                       ctypes.byref(off), ctypes.byref(n)))
        return off.value, n.value

    def arena_tune(self, cls, rank, R, arena, arena_bytes, stream=None):
        """(best variant, [seconds per update of each variant, 0 where it does not fit]); `arena` is
        a device pointer or a tensor.  Clears the arena."""
        best = ctypes.c_uint32()
        secs = (ctypes.c_double * HZP_ARENA_VARIANTS)()
        _check(_L.hzp_arena_tune(self.handle, cls, rank, R, _addr(arena), arena_bytes, _stream(stream),
                                 ctypes.byref(best), secs))
        return best.value, list(secs)

    def bytes(self):
        o, g, p = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
        _check(_L.hzp_plan_bytes(self.handle, ctypes.byref(o), ctypes.byref(g), ctypes.byref(p)))
        return o.value, g.value, p.value


def hzp_plan(tensors_per_layer, tensor_numel, align, z3, z1, z2=0, tensor_class=None,
             tensor_wd_mult=None):
    n_layers, n = len(tensors_per_layer), len(tensor_numel)
    tpl = (ctypes.c_uint32 * n_layers)(*tensors_per_layer)
    numel = (ctypes.c_uint64 * n)(*tensor_numel)
    cls = (ctypes.c_uint8 * n)(*tensor_class) if tensor_class is not None else None
    wd = (ctypes.c_float * n)(*tensor_wd_mult) if tensor_wd_mult is not None else None
    desc = PlanDesc(n_layers, tpl, numel, cls, wd, align, z3, z2, z1)
    handle = ctypes.c_void_p()
    _check(_L.hzp_plan(ctypes.byref(desc), ctypes.byref(handle)))
    return Plan(handle, None)


def hzp_memory_model(n_params, z1, z2, z3):
    out = ctypes.c_uint64()
    _check(_L.hzp_memory_model(n_params, z1, z2, z3, ctypes.byref(out)))
    return out.value


def hzp_choose_groups(n_params, dp, node, budget_bytes):
    """(z1, z2, z3) of the least sharding that fits; raises HzpError(HZP_ERR_NOMEM) if none does."""
    z1, z2, z3 = ctypes.c_uint32(), ctypes.c_uint32(), ctypes.c_uint32()
    _check(_L.hzp_choose_groups(n_params, dp, node, budget_bytes, ctypes.byref(z1), ctypes.byref(z2),
                                ctypes.byref(z3)))
    return z1.value, z2.value, z3.value


def hzp_plan_free(plan):
    plan.__del__()


def hzp_reduce_shard(plan, layer, cls, level, rank, grad_slices, scale, accumulate, out_f32,
                     stream=None, R=None, grad_dtype=HZP_GRAD_DEFAULT):
    arr = ptr_array(grad_slices)
    _check(_L.hzp_reduce_shard(plan.handle, layer, cls, level, rank, arr,
                               len(arr) if R is None else R, grad_dtype, scale, int(bool(accumulate)),
                               _addr(out_f32), _stream(stream)))


def adamw_hyper(lr, beta1, beta2, eps, weight_decay, grad_scale, step):
    return AdamW(lr, beta1, beta2, eps, weight_decay, grad_scale, step)


def hzp_adamw_shard(plan, layer_begin, layer_end, cls, rank, hyper, grad_slices, R, master, m, v,
                    param_out, stream=None):
    """grad_slices: flat sequence, entry (layer-layer_begin)*max(R,1) + r."""
    _check(_L.hzp_adamw_shard(plan.handle, layer_begin, layer_end, cls, rank, ctypes.byref(hyper),
                              ptr_array(grad_slices), R, ptr_array(master), ptr_array(m),
                              ptr_array(v), ptr_array(param_out) if param_out is not None else None,
                              _stream(stream)))


def hzp_adamw_scalars(hyper):
    """The 48-byte block hzp_adamw_shard_dev reads from device memory, as 12 floats (a list)."""
    out = AdamWScalars()
    _check(_L.hzp_adamw_scalars(ctypes.byref(hyper) if hyper is not None else None, ctypes.byref(out)))
    return list(out.f)


def hzp_adamw_shard_dev(plan, layer_begin, layer_end, cls, rank, scalars, grad_slices, R, master, m, v,
                        param_out, stream=None):
    """`scalars`: device tensor (or address) holding hzp_adamw_scalars' 12 floats."""
    _check(_L.hzp_adamw_shard_dev(plan.handle, layer_begin, layer_end, cls, rank, _addr(scalars),
                                  ptr_array(grad_slices), R, ptr_array(master), ptr_array(m),
                                  ptr_array(v), ptr_array(param_out) if param_out is not None else None,
                                  _stream(stream)))


def hzp_gather_layer(plan, layer, cls, level, shard_ptrs, bucket_out=None, tensor_out=None,
                     stream=None, n_shards=None):
    arr = ptr_array(shard_ptrs)
    _check(_L.hzp_gather_layer(plan.handle, layer, cls, level, arr,
                               len(arr) if n_shards is None else n_shards, _addr(bucket_out),
                               ptr_array(tensor_out) if tensor_out is not None else None,
                               _stream(stream)))


def hzp_gather_layer_static(plan, layer, cls, shard_ptrs, tensor_out, stream=None, n_shards=None):
    arr = ptr_array(shard_ptrs)
    _check(_L.hzp_gather_layer_static(plan.handle, layer, cls, arr, len(arr) if n_shards is None else n_shards,
                                      ptr_array(tensor_out) if tensor_out is not None else None, _stream(stream)))


def hzp_gather_shard(plan, layer, cls, j, owner_ptrs, shard_out, stream=None, n_owners=None):
    arr = ptr_array(owner_ptrs)
    _check(_L.hzp_gather_shard(plan.handle, layer, cls, j, arr, len(arr) if n_owners is None else n_owners,
                               _addr(shard_out), _stream(stream)))


def hzp_gather_layers(plan, layer_begin, layer_end, cls, level, shard_ptrs, n_shards, bucket_out, stream=None):
    _check(_L.hzp_gather_layers(plan.handle, layer_begin, layer_end, cls, level, ptr_array(shard_ptrs), n_shards,
                                ptr_array(bucket_out), _stream(stream)))


def hzp_gather_tensor(plan, tensor_id, shard_ptrs, tensor_out, stream=None, n_shards=None):
    arr = ptr_array(shard_ptrs)
    _check(_L.hzp_gather_tensor(plan.handle, tensor_id, arr, len(arr) if n_shards is None else n_shards,
                                _addr(tensor_out), _stream(stream)))


class Sched:
    """Owner of an ``hzp_sched_t*`` (hzp_sched_create ... hzp_sched_destroy)."""

    def __init__(self, plan, cls=HZP_CLASS_BF16, gather_slots=2, queue_capacity=64, pool_bytes=0):
        self.plan = plan                      # keeps the plan alive
        desc = SchedDesc(cls, gather_slots, queue_capacity, 0, pool_bytes)
        self.handle = ctypes.c_void_p()
        _check(_L.hzp_sched_create(plan.handle, ctypes.byref(desc), ctypes.byref(self.handle)))

    def destroy(self):
        if getattr(self, "handle", None):
            _L.hzp_sched_destroy(self.handle)
            self.handle = None

    __del__ = destroy

    def prefetch(self, layer, shard_ptrs, producer=None):
        arr = ptr_array(shard_ptrs)
        _check(_L.hzp_sched_prefetch(self.handle, layer, arr, len(arr), _stream(producer)))

    def prefetch_ahead(self, first_layer, n_layers, shard_ptrs, n_shards, producer=None):
        """Queues layers first_layer.. as far as the pool allows; returns how many were dealt with."""
        issued = ctypes.c_uint32()
        _check(_L.hzp_sched_prefetch_ahead(self.handle, first_layer, n_layers, ptr_array(shard_ptrs), n_shards,
                                           _stream(producer), ctypes.byref(issued)))
        return issued.value

    def acquire(self, layer, consumer=None):
        out = ctypes.c_void_p()
        _check(_L.hzp_sched_acquire(self.handle, layer, _stream(consumer), ctypes.byref(out)))
        return out.value

    def release(self, layer, consumer=None):
        _check(_L.hzp_sched_release(self.handle, layer, _stream(consumer)))

    def prefetch_tensor(self, tensor_id, shard_ptrs, producer=None):
        arr = ptr_array(shard_ptrs)
        _check(_L.hzp_sched_prefetch_tensor(self.handle, tensor_id, arr, len(arr), _stream(producer)))

    def acquire_tensor(self, tensor_id, consumer=None):
        out = ctypes.c_void_p()
        _check(_L.hzp_sched_acquire_tensor(self.handle, tensor_id, _stream(consumer), ctypes.byref(out)))
        return out.value

    def release_tensor(self, tensor_id, consumer=None):
        _check(_L.hzp_sched_release_tensor(self.handle, tensor_id, _stream(consumer)))

    def prefetch_params(self, layer, shard_ptrs, producer=None):
        arr = ptr_array(shard_ptrs)
        _check(_L.hzp_sched_prefetch_params(self.handle, layer, arr, len(arr), _stream(producer)))

    def acquire_params(self, layer, n_tensors, consumer=None):
        """Device addresses of the layer's tensors in the pool, in bucket order."""
        out = (ctypes.c_void_p * n_tensors)()
        _check(_L.hzp_sched_acquire_params(self.handle, layer, _stream(consumer), out))
        return [int(x or 0) for x in out]

    def release_params(self, layer, consumer=None):
        _check(_L.hzp_sched_release_params(self.handle, layer, _stream(consumer)))

    def reduce(self, layer, level, rank, grad_slices, scale, accumulate, out_f32, producer=None,
               grad_dtype=HZP_GRAD_DEFAULT):
        arr = ptr_array(grad_slices)
        _check(_L.hzp_sched_reduce(self.handle, layer, level, rank, arr, len(arr), grad_dtype, scale,
                                   int(bool(accumulate)), _addr(out_f32), _stream(producer)))

    def join(self, consumer=None):
        _check(_L.hzp_sched_join(self.handle, _stream(consumer)))

    def drain(self):
        _check(_L.hzp_sched_drain(self.handle))

    def stats(self):
        out = SchedStats()
        _check(_L.hzp_sched_stats(self.handle, ctypes.byref(out)))
        return out
