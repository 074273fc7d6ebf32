"""ctypes binding of include/recover.h: the same names, argument marshalling only.

Every function takes plain integers for device pointers (`tensor.data_ptr()`) and streams
(`torch.cuda.current_stream().cuda_stream`) and returns the library's int code; `check`
turns a negative code into `RecoverError`.  `Shard` is a convenience holder that allocates
the buffers of one context with PyTorch (device memory and streams only) and forwards to
the same calls.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librecover.so")

OK, SKIPPED = 0, 1
ERR_ARG, ERR_STATE, ERR_NO_SURVIVOR, ERR_HIP, ERR_ALIGN, ERR_NO_SNAPSHOT = -1, -2, -3, -4, -5, -6
F32, BF16 = 0, 1
ROLE_MAJOR, ROLE_MINOR, ROLE_MAJOR_SPARE, ROLE_MINOR_SPARE, ROLE_DEAD = 0, 1, 2, 3, 4
RESTORE_SKIP, RESTORE_BLOCKING, RESTORE_NONBLOCKING = 0, 1, 2
FLAG_ADAPTIVE, FLAG_ANY_ORDER, FLAG_HOST_ONLY = 1, 2, 4
REDUCE_INPLACE = 1
MAX_REPLICAS = 64
STATIC_STEP_SLOTS = 64

FUSED_WRITE_GRAD = 1
(KERNEL_ACCUMULATE_FIRST_F32, KERNEL_ACCUMULATE_RMW_F32, KERNEL_ACCUMULATE_FIRST_BF16, KERNEL_ACCUMULATE_RMW_BF16,
 KERNEL_COPY, KERNEL_REDUCE, KERNEL_ADAMW, KERNEL_REDUCE_ADAMW, KERNEL_ACCUMULATE_SNAPSHOT_F32,
 KERNEL_ACCUMULATE_SNAPSHOT_BF16, KERNEL_CLASSES) = range(11)
TUNE_NONTEMPORAL, TUNE_ONE_PASS_MAX, TUNE_THREADS, TUNE_VECS, TUNE_WAVES, TUNE_DEPTH = 1, 2, 7, 16, 32, 48

EXPORTS = ["recover_init", "recover_destroy", "recover_accumulate", "recover_accumulate_many",
           "recover_accumulate_snapshot",
           "recover_reduce_adamw_step", "recover_snapshot", "recover_restore",
           "recover_policy_adjust", "recover_reduce", "recover_adamw_step", "recover_query",
           "recover_committed_ids", "recover_compare", "recover_last_error", "recover_set_tuning",
           "recover_get_tuning", "recover_adamw_step_static", "recover_device_alloc", "recover_device_free"]


class RecoverError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("recover error %d: %s" % (code, msg))
        self.code = code


class Config(C.Structure):
    _fields_ = [("W_init", C.c_int32), ("G_init", C.c_int32), ("n_elems", C.c_int64), ("n_tensors", C.c_int32),
                ("tensor_offsets", C.POINTER(C.c_int64)), ("acc", C.POINTER(C.c_void_p)),
                ("snap", C.POINTER(C.c_void_p)), ("grad_out", C.c_void_p), ("param", C.c_void_p),
                ("exp_avg", C.c_void_p), ("exp_avg_sq", C.c_void_p), ("param_bf16", C.c_void_p),
                ("flags", C.c_uint32), ("step_state", C.c_void_p)]


class Decision(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("at_boundary", "restore_mode", "epoch", "W_cur", "C_cur", "G_ext", "n_bdry",
                                         "G_cur", "R_cur", "loop_bound", "n_maj", "n_min", "n_ms", "n_mi", "n_bm")] + \
               [(k, C.POINTER(C.c_int32)) for k in ("role", "target", "contributed", "is_boundary_minor")]


_lib = None


def lib():
    """The loaded shared library.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("librecover.so is not built; run `python -m paper_2605_11215_amd.build` "
                               "(there is no CPU implementation of this library)")
        # PyTorch ships its own HIP runtime; it has to be in the process first so that this library
        # binds to the same runtime instead of loading a second one (device pointers and streams
        # are shared between the two).
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        P, I, U32, F, VP = C.c_void_p, C.c_int, C.c_uint32, C.c_float, C.c_void_p
        L.recover_init.argtypes = [C.POINTER(Config), C.POINTER(P)]
        L.recover_destroy.argtypes = [P]
        L.recover_accumulate.argtypes = [P, I, U32, VP, I, I, I, VP]
        L.recover_accumulate_snapshot.argtypes = [P, I, U32, VP, I, I, I, VP]
        L.recover_accumulate_many.argtypes = [P, I, C.POINTER(C.c_int32), C.POINTER(U32), C.POINTER(VP), I,
                                              C.POINTER(C.c_int32), VP]
        L.recover_reduce_adamw_step.argtypes = [P, F, F, F, F, F, U32, VP]
        L.recover_snapshot.argtypes = [P, I, I, I, VP]
        L.recover_restore.argtypes = [P, I, I, VP]
        L.recover_policy_adjust.argtypes = [P, C.POINTER(C.c_int32), I, C.POINTER(Decision)]
        L.recover_reduce.argtypes = [P, I, I, U32, VP]
        L.recover_adamw_step.argtypes = [P, F, F, F, F, F, VP]
        L.recover_adamw_step_static.argtypes = [P, I, I, F, F, F, F, F, VP]
        L.recover_query.argtypes = [P, C.POINTER(Decision)]
        L.recover_committed_ids.argtypes = [P, I, C.POINTER(U32), I]
        L.recover_compare.argtypes = [VP, VP, C.c_int64, VP, VP]
        L.recover_last_error.argtypes = [P]
        L.recover_last_error.restype = C.c_char_p
        L.recover_set_tuning.argtypes = [I, I]
        L.recover_device_alloc.argtypes = [C.c_uint64, I, C.POINTER(VP)]
        L.recover_device_free.argtypes = [VP]
        L.recover_get_tuning.argtypes = [I, C.POINTER(C.c_int)]
        for name in EXPORTS:
            if name != "recover_last_error":
                getattr(L, name).restype = I
        _lib = L
    return _lib


def recover_last_error(ctx):
    return lib().recover_last_error(ctx).decode()


def check(code, ctx=None):
    if code < 0:
        raise RecoverError(code, recover_last_error(ctx))
    return code


def recover_init(W_init, G_init, tensor_offsets, acc, snap, grad_out, param, exp_avg, exp_avg_sq, param_bf16=0,
                 flags=0, step_state=0):
    """acc / snap: sequences of W_init device addresses (snap may be None).  Returns (code, ctx)."""
    T = len(tensor_offsets) - 1
    off = (C.c_int64 * (T + 1))(*tensor_offsets)
    cfg = Config()
    cfg.W_init, cfg.G_init, cfg.n_elems, cfg.n_tensors = W_init, G_init, tensor_offsets[-1], T
    cfg.tensor_offsets = off
    keep = [off]
    if acc is not None:
        a = (C.c_void_p * len(acc))(*acc)
        cfg.acc = a
        keep.append(a)
    if snap is not None:
        s = (C.c_void_p * len(snap))(*snap)
        cfg.snap = s
        keep.append(s)
    cfg.grad_out, cfg.param, cfg.exp_avg, cfg.exp_avg_sq = grad_out or None, param or None, exp_avg or None, exp_avg_sq or None
    cfg.param_bf16 = param_bf16 or None
    cfg.flags = flags
    cfg.step_state = step_state or None
    ctx = C.c_void_p()
    code = lib().recover_init(C.byref(cfg), C.byref(ctx))
    return code, ctx


def recover_destroy(ctx):
    return lib().recover_destroy(ctx)


def recover_accumulate(ctx, replica, global_mb_id, grad, dtype, tensor_begin, tensor_end, stream=0):
    return lib().recover_accumulate(ctx, replica, global_mb_id, grad or None, dtype, tensor_begin, tensor_end,
                                    stream or None)


def recover_accumulate_many(ctx, replicas, ids, grads, dtype, stream=0):
    """Returns (code, per-pair status list)."""
    n = len(replicas)
    r = (C.c_int32 * n)(*replicas)
    i = (C.c_uint32 * n)(*ids)
    g = (C.c_void_p * n)(*[p or None for p in grads])
    st = (C.c_int32 * n)()
    code = lib().recover_accumulate_many(ctx, n, r, i, g, dtype, st, stream or None)
    return code, list(st)


def recover_accumulate_snapshot(ctx, replica, global_mb_id, grad, dtype, tensor_begin, tensor_end, stream=0):
    return lib().recover_accumulate_snapshot(ctx, replica, global_mb_id, grad or None, dtype, tensor_begin,
                                             tensor_end, stream or None)


def recover_reduce_adamw_step(ctx, lr, beta1, beta2, eps, weight_decay, flags=0, stream=0):
    return lib().recover_reduce_adamw_step(ctx, lr, beta1, beta2, eps, weight_decay, flags, stream or None)


def recover_snapshot(ctx, replica, tensor_begin, tensor_end, stream=0):
    return lib().recover_snapshot(ctx, replica, tensor_begin, tensor_end, stream or None)


def recover_restore(ctx, replica, stale_only, stream=0):
    return lib().recover_restore(ctx, replica, int(stale_only), stream or None)


def _decision(W):
    d = Decision()
    arrs = [(C.c_int32 * W)() for _ in range(4)]
    d.role, d.target, d.contributed, d.is_boundary_minor = [C.cast(a, C.POINTER(C.c_int32)) for a in arrs]
    return d, arrs


def _decision_dict(d, arrs):
    out = {k: getattr(d, k) for k, _ in Decision._fields_[:15]}
    for k, a in zip(("role", "target", "contributed", "is_boundary_minor"), arrs):
        out[k] = list(a)
    return out


def recover_policy_adjust(ctx, failed, W_init):
    """Returns (code, decision dict)."""
    d, arrs = _decision(W_init)
    f = (C.c_int32 * max(1, len(failed)))(*failed)
    code = lib().recover_policy_adjust(ctx, f, len(failed), C.byref(d))
    return code, _decision_dict(d, arrs)


def recover_reduce(ctx, tensor_begin, tensor_end, flags=0, stream=0):
    return lib().recover_reduce(ctx, tensor_begin, tensor_end, flags, stream or None)


def recover_adamw_step(ctx, lr, beta1, beta2, eps, weight_decay, stream=0):
    return lib().recover_adamw_step(ctx, lr, beta1, beta2, eps, weight_decay, stream or None)


def recover_adamw_step_static(ctx, slot, restart, lr, beta1, beta2, eps, weight_decay, stream=0):
    return lib().recover_adamw_step_static(ctx, slot, int(restart), lr, beta1, beta2, eps, weight_decay, stream or None)


def recover_query(ctx, W_init):
    d, arrs = _decision(W_init)
    code = lib().recover_query(ctx, C.byref(d))
    return code, _decision_dict(d, arrs)


def recover_committed_ids(ctx, replica, cap=64):
    """Returns (count or negative code, all ids): asks again with a larger array when the count exceeds it."""
    while True:
        buf = (C.c_uint32 * max(1, cap))()
        n = lib().recover_committed_ids(ctx, replica, buf, cap)
        if n <= cap:
            return n, list(buf[:max(0, n)])
        cap = n


class CompareResult(C.Structure):
    _fields_ = [("n_mismatch", C.c_uint64), ("n_nan", C.c_uint64), ("checksum_x", C.c_uint64),
                ("checksum_ref", C.c_uint64), ("max_abs_diff", C.c_float), ("max_abs_ref", C.c_float)]


def recover_compare(x, ref, n, out_device, stream=0):
    return lib().recover_compare(x, ref, n, out_device, stream or None)


def compare_tensors(x, ref, n=None):
    """Compare two float32 device tensors on the GPU through recover_compare; returns a dict."""
    import torch
    n = min(x.numel(), ref.numel()) if n is None else n
    out = torch.empty(5, dtype=torch.int64, device=x.device)
    check(recover_compare(x.data_ptr(), ref.data_ptr(), n, out.data_ptr(), torch.cuda.current_stream().cuda_stream))
    raw = out.cpu().numpy().tobytes()
    r = CompareResult.from_buffer_copy(raw)
    return {k: getattr(r, k) for k, _ in CompareResult._fields_}


def recover_set_tuning(key, value):
    return lib().recover_set_tuning(key, value)


def recover_get_tuning(key):
    """Returns (code, value)."""
    v = C.c_int(0)
    code = lib().recover_get_tuning(key, C.byref(v))
    return code, v.value


class DeviceSlab:
    """Device memory from recover_device_alloc, visible to torch through __cuda_array_interface__."""

    def __init__(self, nbytes, contiguous):
        p = C.c_void_p()
        code = lib().recover_device_alloc(nbytes, int(contiguous), C.byref(p))
        if code < 0:
            raise RecoverError(code, recover_last_error(None))
        self.ptr, self.nbytes = p.value, nbytes
        self.__cuda_array_interface__ = dict(shape=(nbytes,), typestr="|u1", data=(self.ptr, False), version=2, strides=None)

    def data_ptr(self):
        return self.ptr

    def free(self):
        if self.ptr:
            check(lib().recover_device_free(self.ptr))
            self.ptr = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def alloc_slab(specs, device="cuda:0", pad_bytes=4 << 20, align=2 << 20, contiguous=False, groups=None, window=0):
    """One device allocation carved into zero-filled flat tensors: specs = [(torch dtype, numel), ...].  Every
    tensor starts `align`-aligned inside the slab and is followed by `pad_bytes` of padding.  A single
    allocation gives the buffers of a context fixed relative placement (separate allocations land wherever
    the driver puts them, and HBM efficiency of the multi-stream kernels then differs from run to run).
    contiguous: ask the driver for physically contiguous memory first (recover_device_alloc) and fall back to an
    ordinary torch allocation if it cannot provide it.
    groups, window: groups = lists of indices into specs, in address order (every index once); a group that fits into
    `window` bytes is not laid across a multiple of `window` from the start of the slab, it starts at the next multiple
    instead.  Measured on MI355X: a large physically contiguous allocation falls into zones at multiples of 32 GiB, and
    two streams of one kernel launch run 7 % slower together when they come from different zones.
    Returns (owner of the memory, tensors in the order of specs); the owner must outlive the tensors."""
    import torch
    sizes = [n * torch.empty(0, dtype=dt).element_size() for dt, n in specs]
    room = [(b + align - 1) // align * align + pad_bytes for b in sizes]
    if groups is None:
        groups = [list(range(len(specs)))]
        window = 0
    assert sorted(i for g in groups for i in g) == list(range(len(specs)))
    offs, total = [0] * len(specs), 0
    for g in groups:
        need = sum(room[i] for i in g)
        if window and need <= window and total % window + need > window:
            total = (total // window + 1) * window
        for i in g:
            offs[i] = total
            total += room[i]
    owner, flat = None, None
    if contiguous and str(device).startswith("cuda"):
        try:
            with torch.cuda.device(device):
                owner = DeviceSlab(total + align, True)
            flat = torch.as_tensor(owner, device=device)
            flat.zero_()
        except RecoverError:
            owner = None
    if flat is None:
        owner = flat = torch.zeros(total + align, dtype=torch.uint8, device=device)
    base = (-flat.data_ptr()) % align
    out = []
    for (dt, n), o, b in zip(specs, offs, sizes):
        out.append(flat[base + o: base + o + b].view(dt))
    return owner, out


def stream_groups(W, n_extra, snapshots, param_bf16):
    """Index groups for alloc_slab of the buffers [extra..., acc[0..W), grad_out, param, exp_avg, exp_avg_sq, (param_bf16),
    (snap[0..W))]: buffers that one kernel launch streams together.  With n_extra dividing W the replicas are cut into n_extra
    runs and extra buffer c (the microbatch gradients of run c) goes with the accumulators of run c; otherwise all extra
    buffers and accumulators form one group.  Then the reduced gradient with the optimiser state; then the snapshots, cut
    like the accumulators."""
    e0, a0 = 0, n_extra
    st0 = a0 + W
    n_state = 4 + (1 if param_bf16 else 0)
    sn0 = st0 + n_state
    if n_extra and W % n_extra == 0:
        per = W // n_extra
        runs = [list(range(c * per, (c + 1) * per)) for c in range(n_extra)]
        groups = [[e0 + c] + [a0 + r for r in runs[c]] for c in range(n_extra)]
    else:
        runs = [list(range(W))]
        groups = [list(range(e0, e0 + n_extra)) + [a0 + r for r in range(W)]]
    groups.append(list(range(st0, st0 + n_state)))
    if snapshots:
        groups += [[sn0 + r for r in run] for run in runs]
    return groups


class Shard:
    """Buffers of one context allocated with PyTorch on `device`, plus the calls on it.

    Holds: acc[r], snap[r] (optional), grad_out, param, exp_avg, exp_avg_sq (all fp32, flat).
    Methods mirror the C calls, raise RecoverError on negative codes, and use torch's
    current stream."""

    def __init__(self, W_init, G_init, tensor_offsets, device="cuda:0", snapshots=True, flags=0, param_bf16=False,
                 host_only=False, device_step=False, slab=False, slab_pad=4 << 20, extra=(), contiguous=False,
                 slab_window=32 << 30):
        """slab: all buffers (and the `extra` = [(dtype, numel), ...] tensors, returned in self.extra) are carved
        from one allocation, see alloc_slab (contiguous: physically contiguous if the driver can; slab_window: groups of
        buffers that stream together stay inside one window of this many bytes, see stream_groups; 0 = plain sequence).
        With len(extra) dividing W_init, extra[c] is meant as the gradient buffer of replicas c W/len .. (c+1) W/len - 1."""
        import torch
        self.torch = torch
        self.W, self.G = W_init, G_init
        self.off = [int(x) for x in tensor_offsets]
        self.N, self.T = self.off[-1], len(self.off) - 1
        self.host_only = host_only
        if host_only:
            flags |= FLAG_HOST_ONLY
            # no device memory at all; the presence of the snap array alone says "with snapshots"
            code, self.ctx = recover_init(W_init, G_init, self.off, None, [0] * W_init if snapshots else None,
                                          0, 0, 0, 0, 0, flags)
        else:
            n = max(self.N, 4)
            if slab:
                # Address order inside the slab: the caller's extra buffers (the microbatch gradients) with the accumulators
                # they are added to, the reduced gradient and the optimiser state, the snapshots.  Buffers that one launch
                # streams together are neighbours and, where they fit, inside one 32 GiB window of the slab.
                specs = list(extra) + [(torch.float32, n)] * (W_init + 4) + ([(torch.bfloat16, n)] if param_bf16 else []) + \
                    ([(torch.float32, n)] * W_init if snapshots else [])
                groups = stream_groups(W_init, len(extra), snapshots, param_bf16)
                self._slab, bufs = alloc_slab(specs, device, slab_pad, contiguous=contiguous, groups=groups, window=slab_window)
                self.contiguous = isinstance(self._slab, DeviceSlab)
                z = lambda dt=torch.float32: bufs.pop(0)
                self.extra = [z() for _ in extra]
                self.acc = [z() for _ in range(W_init)]
                self.grad_out, self.param, self.exp_avg, self.exp_avg_sq = z(), z(), z(), z()
                self.param_bf16 = z() if param_bf16 else None
                self.snap = [z() for _ in range(W_init)] if snapshots else None
            else:
                z = lambda dt=torch.float32: torch.zeros(n, dtype=dt, device=device)
                self.acc = [z() for _ in range(W_init)]
                self.snap = [z() for _ in range(W_init)] if snapshots else None
                self.grad_out, self.param, self.exp_avg, self.exp_avg_sq = z(), z(), z(), z()
                self.param_bf16 = z(torch.bfloat16) if param_bf16 else None
                self.extra = [torch.zeros(k, dtype=dt, device=device) for dt, k in extra]
            self.step_state = torch.zeros(8, dtype=torch.int64, device=device) if device_step else None
            code, self.ctx = recover_init(
                W_init, G_init, self.off, [t.data_ptr() for t in self.acc],
                [t.data_ptr() for t in self.snap] if snapshots else None, self.grad_out.data_ptr(),
                self.param.data_ptr(), self.exp_avg.data_ptr(), self.exp_avg_sq.data_ptr(),
                self.param_bf16.data_ptr() if param_bf16 else 0, flags,
                self.step_state.data_ptr() if device_step else 0)
        if code < 0:
            raise RecoverError(code, recover_last_error(None))

    def close(self):
        if self.ctx:
            recover_destroy(self.ctx)
            self.ctx = None
        slab = getattr(self, "_slab", None)
        if isinstance(slab, DeviceSlab):          # the views go first, then the memory they look at
            self.torch.cuda.synchronize()
            self.acc = self.snap = self.extra = None
            self.grad_out = self.param = self.exp_avg = self.exp_avg_sq = self.param_bf16 = None
            slab.free()
        self._slab = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self):
        return 0 if self.host_only else self.torch.cuda.current_stream().cuda_stream

    def accumulate(self, r, mb_id, g, tb=0, te=None, snapshot=False):
        """g: a flat torch tensor on the device (float32 or bfloat16), or None on a host-only context.
        snapshot=True takes the fused accumulate+snapshot call.  Returns False if the quota was already met."""
        te = self.T if te is None else te
        if self.host_only:
            ptr, dt = 0, F32
        else:
            dt = BF16 if g.dtype == self.torch.bfloat16 else F32
            assert g.is_contiguous() and g.numel() >= self.N
            ptr = g.data_ptr()
        f = recover_accumulate_snapshot if snapshot else recover_accumulate
        return check(f(self.ctx, r, mb_id, ptr, dt, tb, te, self._stream()), self.ctx) == OK

    def accumulate_many(self, replicas, ids, grads):
        """One launch for several replicas.  Returns the per-pair list of True (accumulated) / False (skipped)."""
        if self.host_only:
            ptrs, dt = [0] * len(replicas), F32
        else:
            dt = BF16 if grads[0].dtype == self.torch.bfloat16 else F32
            ptrs = [g.data_ptr() for g in grads]
        code, st = recover_accumulate_many(self.ctx, list(replicas), list(ids), ptrs, dt, self._stream())
        check(code, self.ctx)
        return [x == OK for x in st]

    def snapshot(self, r=None, tb=0, te=None):
        te = self.T if te is None else te
        check(recover_snapshot(self.ctx, -1 if r is None else r, tb, te, self._stream()), self.ctx)

    def restore(self, r=None, stale_only=True):
        check(recover_restore(self.ctx, -1 if r is None else r, stale_only, self._stream()), self.ctx)

    def on_failure(self, failed):
        code, d = recover_policy_adjust(self.ctx, list(failed), self.W)
        check(code, self.ctx)
        return d

    def advance(self):
        code, d = recover_policy_adjust(self.ctx, [], self.W)
        check(code, self.ctx)
        return d

    def reduce(self, tb=0, te=None, inplace=False):
        te = self.T if te is None else te
        return check(recover_reduce(self.ctx, tb, te, REDUCE_INPLACE if inplace else 0, self._stream()), self.ctx) == OK

    def adamw_step(self, lr, beta1, beta2, eps, weight_decay):
        check(recover_adamw_step(self.ctx, lr, beta1, beta2, eps, weight_decay, self._stream()), self.ctx)

    def reduce_adamw_step(self, lr, beta1, beta2, eps, weight_decay, write_grad=False):
        check(recover_reduce_adamw_step(self.ctx, lr, beta1, beta2, eps, weight_decay,
                                        FUSED_WRITE_GRAD if write_grad else 0, self._stream()), self.ctx)

    def query(self):
        code, d = recover_query(self.ctx, self.W)
        check(code, self.ctx)
        return d

    def committed_ids_by_replica(self):
        q = self.query()
        out = {}
        for r in range(self.W):
            if q["role"][r] in (ROLE_MAJOR, ROLE_MINOR):
                n, ids = recover_committed_ids(self.ctx, r)
                out[r] = ids
        return out
