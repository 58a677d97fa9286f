"""ctypes binding of the kvb C ABI (include/kvb.h): argument marshalling only.

Every step of the path runs in the HIP kernels of libkvb.so; nothing here
computes.  PyTorch supplies device memory (``tensor.data_ptr()``) and the stream.
The library must have been built (``python -m paper_2605_19049_amd.build``);
there is no fallback.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvb.so")

OK, EINVAL, EUNSUPPORTED, EHIP = 0, -1, -2, -3
F32, BF16, F16 = 0, 1, 2
MAX_CAP, MAX_DRAFTS, MAX_DIRECT_LEN = 128, 8, 128
STATUS_OVERFLOW = 1
STATUS_BADPATH = 2
STORE_STREAM, STORE_RESIDENT = 1, 2

EXPORTS = ("kvb_decode", "kvb_decode_flush", "kvb_flush", "kvb_verify", "kvb_verify_tree", "kvb_compact", "kvb_direct",
           "kvb_timer_create", "kvb_timer_arm", "kvb_timer_read", "kvb_timer_destroy",
           "kvb_strerror", "kvb_version")


class KvbShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hk", ctypes.c_int32), ("Hv", ctypes.c_int32),
                ("dk", ctypes.c_int32), ("dv", ctypes.c_int32), ("cap", ctypes.c_int32),
                ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32), ("rec_dtype", ctypes.c_int32),
                ("scale", ctypes.c_float)]


class KvbStore(ctypes.Structure):
    _fields_ = [("state", ctypes.c_void_p), ("buf_k", ctypes.c_void_p), ("buf_u", ctypes.c_void_p),
                ("buf_G", ctypes.c_void_p), ("fill", ctypes.c_void_p), ("status", ctypes.c_void_p),
                ("n_slots", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("block_table", ctypes.c_void_p), ("block_size", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("n_blocks", ctypes.c_int32)]


class KvbError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, strerror(code), code))


_lib = None


def lib():
    """The loaded libkvb.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libkvb.so is missing: build it with `python -m paper_2605_19049_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        sp, tp = ctypes.POINTER(KvbShape), ctypes.POINTER(KvbStore)
        L.kvb_decode.argtypes = [sp, tp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.kvb_decode_flush.argtypes = [sp, tp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.kvb_flush.argtypes = [sp, tp, vp, vp, i32, vp]
        L.kvb_timer_create.argtypes = [ctypes.POINTER(vp)]
        L.kvb_timer_arm.argtypes = [vp]
        L.kvb_timer_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
        L.kvb_timer_destroy.argtypes = [vp]
        L.kvb_timer_destroy.restype = None
        L.kvb_verify.argtypes = [sp, tp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.kvb_verify_tree.argtypes = [sp, tp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.kvb_compact.argtypes = [sp, tp, vp, i32, vp, vp, vp]
        L.kvb_direct.argtypes = [sp, tp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        for name in ("kvb_decode", "kvb_decode_flush", "kvb_flush", "kvb_verify", "kvb_verify_tree", "kvb_compact",
                     "kvb_direct", "kvb_version",
                     "kvb_timer_create", "kvb_timer_arm", "kvb_timer_read"):
            getattr(L, name).restype = ctypes.c_int
        L.kvb_strerror.argtypes = [ctypes.c_int]
        L.kvb_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _ptr(x):
    """Device address of a torch tensor, or an int / None passed through."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def shape(B, Hk, Hv, dk, dv, cap, in_dtype, scale=1.0, out_dtype=F32, rec_dtype=F32):
    return KvbShape(B, Hk, Hv, dk, dv, cap, in_dtype, out_dtype, rec_dtype, scale)


def torch_dtype(code):
    """The torch element type of a KVB_* type code (memory plumbing)."""
    import torch
    return {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16}[code]


def store(state, buf_k, buf_u, buf_G, fill, status, n_slots, flags=0, block_table=None, block_size=0,
          max_blocks=0, n_blocks=0):
    return KvbStore(_ptr(state), _ptr(buf_k), _ptr(buf_u), _ptr(buf_G), _ptr(fill), _ptr(status), n_slots, flags,
                    _ptr(block_table), block_size, max_blocks, n_blocks)


def strerror(code):
    return lib().kvb_strerror(code).decode()


def version():
    return lib().kvb_version()


def _check(rc, where, check):
    if check and rc != OK:
        raise KvbError(rc, where)
    return rc


def kvb_decode(sh, st, slot, q, k, v, g, beta, out, stream=None, check=True):
    rc = lib().kvb_decode(ctypes.byref(sh), ctypes.byref(st), _ptr(slot), _ptr(q), _ptr(k), _ptr(v),
                          _ptr(g), _ptr(beta), _ptr(out), _stream(stream))
    return _check(rc, "kvb_decode", check)


def kvb_decode_flush(sh, st, slot, q, k, v, g, beta, out, threshold, stream=None, check=True):
    rc = lib().kvb_decode_flush(ctypes.byref(sh), ctypes.byref(st), _ptr(slot), _ptr(q), _ptr(k), _ptr(v),
                                _ptr(g), _ptr(beta), _ptr(out), threshold, _stream(stream))
    return _check(rc, "kvb_decode_flush", check)


class Timer:
    """A kvb_timer: arm() before a call, us() after it to get that call's kernel duration."""

    def __init__(self):
        self._h = ctypes.c_void_p()
        _check(lib().kvb_timer_create(ctypes.byref(self._h)), "kvb_timer_create", True)

    def arm(self):
        lib().kvb_timer_arm(self._h)

    def us(self):
        out = ctypes.c_float()
        _check(lib().kvb_timer_read(self._h, ctypes.byref(out)), "kvb_timer_read", True)
        return out.value

    def close(self):
        if self._h:
            lib().kvb_timer_destroy(self._h)
            self._h = ctypes.c_void_p()


def kvb_flush(sh, st, slot, accepted, threshold, stream=None, check=True):
    rc = lib().kvb_flush(ctypes.byref(sh), ctypes.byref(st), _ptr(slot), _ptr(accepted), threshold,
                         _stream(stream))
    return _check(rc, "kvb_flush", check)


def kvb_verify(sh, st, slot, T, q, k, v, g, beta, out, stream=None, check=True):
    rc = lib().kvb_verify(ctypes.byref(sh), ctypes.byref(st), _ptr(slot), T, _ptr(q), _ptr(k), _ptr(v),
                          _ptr(g), _ptr(beta), _ptr(out), _stream(stream))
    return _check(rc, "kvb_verify", check)


def kvb_verify_tree(sh, st, slot, T, parent, q, k, v, g, beta, out, stream=None, check=True):
    rc = lib().kvb_verify_tree(ctypes.byref(sh), ctypes.byref(st), _ptr(slot), T, _ptr(parent), _ptr(q), _ptr(k),
                               _ptr(v), _ptr(g), _ptr(beta), _ptr(out), _stream(stream))
    return _check(rc, "kvb_verify_tree", check)


def kvb_compact(sh, st, slot, T, path, path_len, stream=None, check=True):
    rc = lib().kvb_compact(ctypes.byref(sh), ctypes.byref(st), _ptr(slot), T, _ptr(path), _ptr(path_len),
                           _stream(stream))
    return _check(rc, "kvb_compact", check)


def kvb_direct(sh, st, slot, lens, Lmax, q, k, v, g, beta, out, stream=None, check=True):
    rc = lib().kvb_direct(ctypes.byref(sh), ctypes.byref(st), _ptr(slot), _ptr(lens), Lmax, _ptr(q),
                          _ptr(k), _ptr(v), _ptr(g), _ptr(beta), _ptr(out), _stream(stream))
    return _check(rc, "kvb_direct", check)


def bind(fn_name, *args):
    """Pre-marshal one call: returns a zero-argument callable that re-issues it with the
    same pointers (for serving loops, where per-call marshalling would rival a 20 us
    kernel).  `args` are exactly the C arguments; tensors, structs and ints are converted
    once.  The caller keeps the tensors and structs alive."""
    fn = getattr(lib(), fn_name)
    conv = []
    for a, t in zip(args, fn.argtypes):
        if isinstance(a, ctypes.Structure):
            conv.append(ctypes.byref(a))
        elif t is ctypes.c_void_p:
            conv.append(ctypes.c_void_p(_ptr(a)))
        else:
            conv.append(t(a))
    assert len(conv) == len(fn.argtypes), fn_name

    def call():
        rc = fn(*conv)
        if rc != OK:
            raise KvbError(rc, fn_name)
    return call


class DeviceStore:
    """Caller-side holder of the device arrays of include/kvb.h's kvb_store, allocated
    with PyTorch (memory plumbing only)."""

    def __init__(self, n_slots, Hk, Hv, dk, dv, cap, in_dtype, device="cuda", with_state=True,
                 block_size=None, n_blocks=None, block_table=None, rec_dtype=F32):
        """block_size given: paged record buffers, pools of n_blocks blocks and a block table
        [n_slots, ceil(cap / block_size)] (block_table: an int array of that shape; default
        slot s takes the blocks s*mb .. s*mb+mb-1)."""
        import torch
        kd = torch_dtype(in_dtype)
        self.rec_dtype = rec_dtype
        self.n_slots, self.Hk, self.Hv, self.dk, self.dv, self.cap = n_slots, Hk, Hv, dk, dv, cap
        self.in_dtype = in_dtype
        self.state = torch.zeros((n_slots, Hv, dk, dv), dtype=torch.float32, device=device) \
            if with_state else None
        self.block_size = block_size
        if block_size:
            self.max_blocks = -(-cap // block_size)
            self.n_blocks = n_blocks if n_blocks else n_slots * self.max_blocks
            if block_table is None:
                block_table = torch.arange(n_slots * self.max_blocks).reshape(n_slots, self.max_blocks)
            self.block_table = torch.as_tensor(block_table).to(dtype=torch.int32, device=device).contiguous()
            assert tuple(self.block_table.shape) == (n_slots, self.max_blocks)
            nb, per = self.n_blocks, block_size
        else:
            self.block_table, self.max_blocks, self.n_blocks = None, 0, 0
            nb, per = n_slots, cap
        self.buf_k = torch.zeros((nb, Hk, per, dk), dtype=kd, device=device)
        self.buf_u = torch.zeros((nb, Hv, per, dv), dtype=torch_dtype(rec_dtype), device=device)
        self.buf_G = torch.zeros((nb, Hv, per), dtype=torch.float32, device=device)
        self.fill = torch.zeros((n_slots,), dtype=torch.int32, device=device)
        self.status = torch.zeros((n_slots,), dtype=torch.int32, device=device)

    def c(self, with_state=True, flags=0):
        return store(self.state if with_state else None, self.buf_k, self.buf_u, self.buf_G, self.fill,
                     self.status, self.n_slots, flags, self.block_table, self.block_size or 0,
                     self.max_blocks, self.n_blocks)

    def records(self, slot, lo, hi):
        """(k [Hk,n,dk], u [Hv,n,dv], G [Hv,n]) of records lo..hi-1 of a slot, through the block
        table if there is one (test and debugging aid; copies)."""
        import torch
        if not self.block_size:
            return self.buf_k[slot, :, lo:hi], self.buf_u[slot, :, lo:hi], self.buf_G[slot, :, lo:hi]
        ls = torch.arange(lo, hi, device=self.fill.device)
        blk = self.block_table[slot, ls // self.block_size].long()
        off = ls % self.block_size
        return self.buf_k[blk, :, off].transpose(0, 1), self.buf_u[blk, :, off].transpose(0, 1), \
            self.buf_G[blk, :, off].transpose(0, 1)
