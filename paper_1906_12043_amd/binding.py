"""ctypes binding of libcocod.so: same names as include/cocod.h, argument marshalling only.

Device buffers are passed as integer addresses (`tensor.data_ptr()`), streams as the raw
hipStream_t (`torch.cuda.Stream().cuda_stream`); anything with a `data_ptr` / `cuda_stream`
attribute is unwrapped.  There is no fallback: a missing library is an error.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))

OK, ERR_INVALID, ERR_STATE, ERR_HIP, ERR_NOMEM, ERR_UNSUPPORTED = 0, -1, -2, -3, -4, -5
GRAD_QUADRATIC, GRAD_MLP, GRAD_EXTERNAL = 0, 1, 2
SCHED_OVERLAP, SCHED_SERIAL, SCHED_FUSED, SCHED_HEAD = 0, 1, 2, 3
FLAG_DRY_RUN = 1


class Config(C.Structure):
    """Mirror of struct cocod_config."""
    _fields_ = [
        ("struct_size", C.c_uint32), ("W", C.c_uint32), ("d", C.c_uint64),
        ("n_tensors", C.c_uint32), ("grad", C.c_uint32),
        ("tensor_numel", C.POINTER(C.c_uint64)), ("bucket_bytes", C.c_uint64),
        ("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float), ("noise_sigma", C.c_float),
        ("seed", C.c_uint64), ("weights", C.POINTER(C.c_float)), ("noise_sigma_w", C.POINTER(C.c_float)),
        ("xA", C.c_void_p), ("xB", C.c_void_p), ("v", C.c_void_p), ("mean", C.c_void_p),
        ("h", C.c_void_p), ("c", C.c_void_p), ("stride", C.c_uint64),
        ("compute_stream", C.c_void_p), ("avg_stream", C.c_void_p),
        ("mlp_in", C.c_uint32), ("mlp_hidden", C.c_uint32), ("mlp_out", C.c_uint32), ("mlp_batch", C.c_uint32),
        ("flags", C.c_uint32),
    ]


class CocodError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("cocod status %d: %s" % (status, message))
        self.status = status


def lib_path():
    return os.path.join(HERE, "libcocod.so")


_lib = None


def lib():
    """The loaded library; raises if it has not been built (there is no other code path)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError("libcocod.so is missing: run `python -m paper_1906_12043_amd.build`")
        L = C.CDLL(path)
        vp, u64, u32, i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int
        P = C.POINTER
        sigs = {
            "cocod_version": ([], i32),
            "cocod_last_error": ([vp], C.c_char_p),
            "cocod_plan_layout": ([u64, u32, P(u64), u64, P(u64), P(u64), P(u32), P(u64)], i32),
            "cocod_create": ([P(Config), P(vp)], i32),
            "cocod_destroy": ([vp], i32),
            "cocod_sync": ([vp], i32),
            "cocod_local_steps": ([vp, i32], i32),
            "cocod_local_steps_end_apply": ([vp, i32], i32),
            "cocod_external_step": ([vp, vp, i32], i32),
            "cocod_external_step_bf16": ([vp, vp, i32], i32),
            "cocod_graph_round": ([vp, i32, i32], i32),
            "cocod_average_begin": ([vp], i32),
            "cocod_average_end_apply": ([vp], i32),
            "cocod_average_apply_fused": ([vp], i32),
            "cocod_set_schedule": ([vp, i32], i32),
            "cocod_set_lr": ([vp, C.c_float], i32),
            "cocod_get_step": ([vp, P(u64)], i32),
            "cocod_set_step": ([vp, u64], i32),
            "cocod_live_model": ([vp, P(vp)], i32),
            "cocod_is_averaging": ([vp], i32),
            "cocod_get_plan": ([vp, P(u64), P(u32), P(u32)], i32),
            "cocod_consensus_distance": ([vp, P(C.c_double)], i32),
            "cocod_consensus_distance_noalloc": ([vp, vp], i32),
            "cocod_quadratic_objective": ([vp, P(C.c_double), P(C.c_double)], i32),
            "cocod_fill_quadratic": ([vp], i32),
            "cocod_mlp_workspace": ([vp, P(vp), P(vp), P(vp), P(vp), P(vp), P(u32)], i32),
            "cocod_step_timing": ([vp, i32], i32),
            "cocod_step_timing_read": ([vp, P(C.c_double), P(u32)], i32),
            "cocod_debug_copy": ([vp, vp, vp, u64], i32),
            "cocod_debug_normals": ([vp, u64, u32, u32, u32, u64, u64, i32, vp], i32),
        }
        for name, (args, res) in sigs.items():
            fn = getattr(L, name)
            fn.argtypes, fn.restype = args, res
        _lib = L
    return _lib


def _addr(obj):
    if obj is None:
        return None
    if hasattr(obj, "data_ptr"):
        return obj.data_ptr()
    if hasattr(obj, "cuda_stream"):
        return obj.cuda_stream
    return int(obj)


def _check(status, ctx=None):
    if status < 0:
        raise CocodError(status, lib().cocod_last_error(ctx).decode())
    return status


def plan_layout(d, tensor_numel=None, bucket_bytes=0):
    """(padded_d, tensor_offsets, bucket_begin) of a parameter list; pure host arithmetic."""
    n = len(tensor_numel) if tensor_numel else 0
    arr = (C.c_uint64 * max(n, 1))(*(tensor_numel or [d]))
    padded = C.c_uint64()
    offsets = (C.c_uint64 * max(n, 1))()
    n_buckets = C.c_uint32()
    begins = (C.c_uint64 * (max(n, 1) + 1))()
    _check(lib().cocod_plan_layout(d, n, arr if n else None, bucket_bytes, C.byref(padded), offsets,
                                   C.byref(n_buckets), begins))
    return padded.value, list(offsets)[:max(n, 1)], list(begins)[:n_buckets.value + 1]


def debug_normals(stream, seed, tag, worker, step, j0, n, fast, out):
    _check(lib().cocod_debug_normals(_addr(stream), seed, tag, worker, step, j0, n, int(fast), _addr(out)))


def debug_copy(stream, src, dst, n):
    _check(lib().cocod_debug_copy(_addr(stream), _addr(src), _addr(dst), n))


# ---- the five entry points of the round, by their C names -----------------------------------

def cocod_create(*, W, d, xA, xB, mean, stride, v=None, h=None, c=None, lr, momentum=0.0, weight_decay=0.0,
                 noise_sigma=0.0, seed=0, tensor_numel=None, bucket_bytes=0, weights=None, noise_sigma_w=None,
                 compute_stream=None, avg_stream=None, grad=GRAD_QUADRATIC, mlp=(0, 0, 0, 0), flags=0):
    """Returns an opaque context handle (int)."""
    cfg = Config()
    cfg.struct_size = C.sizeof(Config)
    cfg.W, cfg.d, cfg.grad = W, d, grad
    keep = []
    if tensor_numel:
        arr = (C.c_uint64 * len(tensor_numel))(*tensor_numel)
        keep.append(arr)
        cfg.n_tensors, cfg.tensor_numel = len(tensor_numel), arr
    cfg.bucket_bytes = bucket_bytes
    cfg.lr, cfg.momentum, cfg.weight_decay, cfg.noise_sigma = lr, momentum, weight_decay, noise_sigma
    cfg.seed = seed
    if weights is not None:
        warr = (C.c_float * len(weights))(*weights)
        keep.append(warr)
        cfg.weights = warr
    if noise_sigma_w is not None:
        sarr = (C.c_float * len(noise_sigma_w))(*noise_sigma_w)
        keep.append(sarr)
        cfg.noise_sigma_w = sarr
    cfg.xA, cfg.xB, cfg.v, cfg.mean = _addr(xA), _addr(xB), _addr(v), _addr(mean)
    cfg.h, cfg.c, cfg.stride = _addr(h), _addr(c), stride
    cfg.compute_stream, cfg.avg_stream = _addr(compute_stream), _addr(avg_stream)
    cfg.mlp_in, cfg.mlp_hidden, cfg.mlp_out, cfg.mlp_batch = mlp
    cfg.flags = flags
    handle = C.c_void_p()
    _check(lib().cocod_create(C.byref(cfg), C.byref(handle)))
    return handle.value


def cocod_destroy(ctx):
    return _check(lib().cocod_destroy(ctx))


def cocod_local_steps(ctx, k):
    return _check(lib().cocod_local_steps(ctx, k), ctx)


def cocod_average_begin(ctx):
    return _check(lib().cocod_average_begin(ctx), ctx)


def cocod_average_end_apply(ctx):
    return _check(lib().cocod_average_end_apply(ctx), ctx)


class Context:
    """Owns a context handle; methods are the C calls without the prefix."""

    def __init__(self, **kw):
        self.handle = cocod_create(**kw)

    def close(self):
        if self.handle:
            handle, self.handle = self.handle, None
            cocod_destroy(handle)

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def local_steps(self, k):
        return cocod_local_steps(self.handle, k)

    def average_begin(self):
        return cocod_average_begin(self.handle)

    def average_end_apply(self):
        return cocod_average_end_apply(self.handle)

    def average_apply_fused(self):
        return _check(lib().cocod_average_apply_fused(self.handle), self.handle)

    def local_steps_end_apply(self, k):
        return _check(lib().cocod_local_steps_end_apply(self.handle, k), self.handle)

    def external_step(self, g, close_round=False):
        return _check(lib().cocod_external_step(self.handle, _addr(g), int(close_round)), self.handle)

    def external_step_bf16(self, g, close_round=False):
        return _check(lib().cocod_external_step_bf16(self.handle, _addr(g), int(close_round)), self.handle)

    def round_fused_tail(self, k):
        """One round with line 6 applied inside the last local step."""
        self.average_begin()
        self.local_steps_end_apply(k)

    def graph_round(self, k, fused_tail=True):
        """One round replayed from a HIP graph (recorded on first use)."""
        return _check(lib().cocod_graph_round(self.handle, k, int(fused_tail)), self.handle)

    def round(self, k):
        """One pass of the while-loop body of Algorithm 1."""
        self.average_begin()
        self.local_steps(k)
        self.average_end_apply()

    def sync(self):
        return _check(lib().cocod_sync(self.handle), self.handle)

    def set_schedule(self, schedule):
        return _check(lib().cocod_set_schedule(self.handle, schedule), self.handle)

    def set_lr(self, lr):
        return _check(lib().cocod_set_lr(self.handle, lr), self.handle)

    def get_step(self):
        out = C.c_uint64()
        _check(lib().cocod_get_step(self.handle, C.byref(out)), self.handle)
        return out.value

    def set_step(self, step):
        return _check(lib().cocod_set_step(self.handle, step), self.handle)

    def live_model(self):
        out = C.c_void_p()
        _check(lib().cocod_live_model(self.handle, C.byref(out)), self.handle)
        return out.value

    def is_averaging(self):
        return bool(_check(lib().cocod_is_averaging(self.handle), self.handle))

    def get_plan(self):
        padded, chunks, buckets = C.c_uint64(), C.c_uint32(), C.c_uint32()
        _check(lib().cocod_get_plan(self.handle, C.byref(padded), C.byref(chunks), C.byref(buckets)), self.handle)
        return padded.value, chunks.value, buckets.value

    def step_timing(self, max_launches):
        return _check(lib().cocod_step_timing(self.handle, max_launches), self.handle)

    def step_timing_read(self):
        """[(summed kernel milliseconds, launches)] for plain steps, for steps carrying line 6 and for
        first steps of a round that also form the mean."""
        total, n = (C.c_double * 3)(), (C.c_uint32 * 3)()
        _check(lib().cocod_step_timing_read(self.handle, total, n), self.handle)
        return [(total[i], n[i]) for i in range(3)]

    def consensus_distance(self):
        out = C.c_double()
        _check(lib().cocod_consensus_distance(self.handle, C.byref(out)), self.handle)
        return out.value

    def consensus_distance_noalloc(self, result_device):
        """Enqueue the reduction; the scalar lands in the caller's device double."""
        return _check(lib().cocod_consensus_distance_noalloc(self.handle, _addr(result_device)), self.handle)

    def quadratic_objective(self):
        """(f(x^), ||grad f(x^)||^2) at the weighted mean of the live models."""
        f, g = C.c_double(), C.c_double()
        _check(lib().cocod_quadratic_objective(self.handle, C.byref(f), C.byref(g)), self.handle)
        return f.value, g.value

    def mlp_workspace(self):
        """Device addresses {X, H, dA, dZ, y} of the MLP work space and the row pitch of dZ."""
        ptrs = [C.c_void_p() for _ in range(5)]
        pitch = C.c_uint32()
        _check(lib().cocod_mlp_workspace(self.handle, *[C.byref(q) for q in ptrs], C.byref(pitch)), self.handle)
        return dict(zip(("X", "H", "dA", "dZ", "y"), [q.value for q in ptrs])), pitch.value

    def fill_quadratic(self):
        return _check(lib().cocod_fill_quadratic(self.handle), self.handle)
