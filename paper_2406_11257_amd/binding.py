"""ctypes binding of include/excp.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))

EXCP_OK, EXCP_E_ARG, EXCP_E_CAP, EXCP_E_NONFINITE = 0, -1, -2, -3
EXCP_E_BLOB, EXCP_E_HIP, EXCP_E_STATE, EXCP_E_INTERNAL = -4, -5, -6, -7
EXCP_FLAG_MEDIAN_OF_WEIGHTS, EXCP_FLAG_NO_M2W, EXCP_FLAG_NO_QUANT, EXCP_FLAG_NO_W2M = 1, 2, 4, 8
EXCP_FLAG_W_F16, EXCP_FLAG_W_BF16 = 16, 32
EXCP_PARAM_WIDE_ELEMS, EXCP_PARAM_CAND_LIST_ELEMS = 1, 2


class ExcpTensor(C.Structure):
    _fields_ = [("W_prev_recon", C.c_void_p), ("W_t", C.c_void_p), ("m_t", C.c_void_p),
                ("v_t", C.c_void_p), ("n", C.c_uint64), ("blob", C.c_void_p),
                ("blob_cap", C.c_uint64), ("W_recon_out", C.c_void_p)]


class ExcpChain(C.Structure):
    _fields_ = [("W0", C.c_void_p), ("n", C.c_uint64), ("steps", C.c_int),
                ("blobs", C.POINTER(C.c_void_p)), ("blob_bytes", C.POINTER(C.c_uint64)),
                ("W_out", C.c_void_p), ("m_out", C.c_void_p), ("v_out", C.c_void_p),
                ("flags", C.c_uint32), ("reserved", C.c_uint32)]


class ExcpBlob(C.Structure):
    _fields_ = [("W_prev_recon", C.c_void_p), ("blob", C.c_void_p), ("blob_bytes", C.c_uint64),
                ("n", C.c_uint64), ("W_recon_out", C.c_void_p), ("m_out", C.c_void_p),
                ("v_out", C.c_void_p), ("flags", C.c_uint32), ("reserved", C.c_uint32)]


class ExcpDenseExport(C.Structure):
    _fields_ = [("blob", C.c_void_p), ("blob_bytes", C.c_uint64), ("n", C.c_uint64), ("head", C.c_void_p),
                ("codes_w", C.c_void_p), ("codes_m", C.c_void_p), ("codes_v", C.c_void_p)]


class ExcpDenseBlob(C.Structure):
    _fields_ = [("W_prev_recon", C.c_void_p), ("head", C.c_void_p), ("head_bytes", C.c_uint64),
                ("n", C.c_uint64), ("codes_w", C.c_void_p), ("codes_m", C.c_void_p), ("codes_v", C.c_void_p),
                ("W_recon_out", C.c_void_p), ("m_out", C.c_void_p), ("v_out", C.c_void_p),
                ("flags", C.c_uint32), ("reserved", C.c_uint32)]


class ExcpStats(C.Structure):
    _fields_ = [("n", C.c_uint64), ("n_w", C.c_uint64), ("n_o", C.c_uint64),
                ("blob_bytes", C.c_uint64), ("nonfinite", C.c_uint64),
                ("abs_sum_m", C.c_double), ("obj_w", C.c_double), ("obj_m", C.c_double),
                ("obj_v", C.c_double), ("median_abs_dw", C.c_float), ("mean_abs_m", C.c_float),
                ("t_w", C.c_float), ("r_o", C.c_float), ("status", C.c_int32), ("reserved", C.c_int32)]


class ExcpError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {excp_strerror(code)} ({code})")


SYMBOLS = {
    "excp_create": (C.c_int, [C.POINTER(C.c_void_p), C.c_int, C.c_void_p, C.c_uint64, C.c_uint64]),
    "excp_destroy": (None, [C.c_void_p]),
    "excp_reconstruct_chain": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p]),
    "excp_blob_bound": (C.c_uint64, [C.c_uint64, C.c_int]),
    "excp_blob_size": (C.c_uint64, [C.c_uint64, C.c_uint64, C.c_uint64, C.c_int]),
    "excp_blob_size_ex": (C.c_uint64, [C.c_uint64, C.c_uint64, C.c_uint64, C.c_int, C.c_uint32]),
    "excp_compress_tensors": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(ExcpTensor), C.c_float, C.c_float,
                                        C.c_int, C.c_int, C.c_uint32]),
    "excp_decompress_tensors": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(ExcpBlob)]),
    "excp_dense_bytes": (C.c_uint64, [C.c_uint64, C.c_int]),
    "excp_head_bytes": (C.c_uint64, [C.c_int]),
    "excp_export_dense": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(ExcpDenseExport)]),
    "excp_decompress_dense": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(ExcpDenseBlob)]),
    "excp_collect": (C.c_int, [C.c_void_p, C.POINTER(ExcpStats)]),
    "excp_compress_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64,
                                     C.c_float, C.c_float, C.c_int, C.c_int, C.c_uint32, C.c_void_p,
                                     C.c_uint64, C.POINTER(C.c_uint64), C.c_void_p, C.POINTER(ExcpStats)]),
    "excp_decompress_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32]),
    "excp_decompress_step_static": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32]),
    "excp_set_profiling": (C.c_int, [C.c_void_p, C.c_int]),
    "excp_set_param": (C.c_int, [C.c_void_p, C.c_int, C.c_uint64]),
    "excp_stage_count": (C.c_int, []),
    "excp_stage_name": (C.c_char_p, [C.c_int]),
    "excp_stage_ms": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int)]),
    "excp_workspace_bytes": (C.c_uint64, [C.c_void_p]),
    "excp_copy_probe": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64]),
    "excp_strerror": (C.c_char_p, [C.c_int]),
}

_lib = None


def lib_path() -> str:
    return os.path.join(HERE, "libexcp.so")


def lib():
    """The loaded library.  Raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -m paper_2406_11257_amd.build` "
                              "(or __graft_entry__.build()) first")
        L = C.CDLL(path)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def excp_strerror(code: int) -> str:
    return lib().excp_strerror(code).decode()


def excp_blob_bound(n: int, nbits: int) -> int:
    return int(lib().excp_blob_bound(n, nbits))


def excp_blob_size(n: int, n_w: int, n_o: int, nbits: int) -> int:
    return int(lib().excp_blob_size(n, n_w, n_o, nbits))


def excp_blob_size_ex(n: int, n_w: int, n_o: int, nbits: int, flags: int) -> int:
    return int(lib().excp_blob_size_ex(n, n_w, n_o, nbits, flags))


def excp_dense_bytes(n: int, nbits: int) -> int:
    return int(lib().excp_dense_bytes(n, nbits))


def excp_head_bytes(nbits: int) -> int:
    return int(lib().excp_head_bytes(nbits))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


_WEIGHT_NAMES = ("W_prev_recon", "W_t", "W_recon_out", "W0", "W_out")


def _check_f32(t, name, device, flags=None):
    """Moments are float32.  Weight tensors are float32, or float16 / bfloat16 with EXCP_FLAG_W_F16 /
    EXCP_FLAG_W_BF16; where no flags are at hand (reading a blob) the blob's header names the storage
    and the caller passes tensors of that type."""
    import torch
    allowed = (torch.float32,)
    if name in _WEIGHT_NAMES:
        if flags is None:
            allowed = (torch.float32, torch.float16, torch.bfloat16)
        elif flags & EXCP_FLAG_W_F16:
            allowed = (torch.float16,)
        elif flags & EXCP_FLAG_W_BF16:
            allowed = (torch.bfloat16,)
    if t.dtype not in allowed or not t.is_contiguous() or t.device != device:
        raise TypeError(f"{name} must be a contiguous tensor on {device} of type {' / '.join(str(a) for a in allowed)}")


def _wflags(*tensors) -> int:
    """The storage flag that says what the given weight tensors hold (they must agree)."""
    import torch
    kinds = {t.dtype for t in tensors if t is not None}
    if len(kinds) > 1:
        raise TypeError("the weight tensors of one item differ in type")
    kind = kinds.pop() if kinds else torch.float32
    return {torch.float32: 0, torch.float16: EXCP_FLAG_W_F16, torch.bfloat16: EXCP_FLAG_W_BF16}[kind]


EXCP_STATIC_MAX_ELEMS = 1 << 28


def excp_decompress_step_static(Wp, blob, blob_bytes, W_recon_out=None, m_out=None, v_out=None, stream=None, check=True):
    """Alg. 2 for one tensor through the entry point that allocates nothing (no context)."""
    import torch
    device = Wp.device
    _check_f32(Wp, "W_prev_recon", device)
    n = Wp.numel()
    for t, nm in ((W_recon_out, "W_recon_out"), (m_out, "m_out"), (v_out, "v_out")):
        if t is not None:
            _check_f32(t, nm, device)
            if t.numel() != n:
                raise ValueError(nm + " length differs")
    st = torch.cuda.current_stream(device) if stream is None else stream
    rc = lib().excp_decompress_step_static(device.index, C.c_void_p(st.cuda_stream), _ptr(Wp), _ptr(blob), blob_bytes, n,
                                           _ptr(W_recon_out), _ptr(m_out), _ptr(v_out), _wflags(Wp, W_recon_out))
    if check and rc != EXCP_OK:
        raise ExcpError(rc, "excp_decompress_step_static")
    return rc


class PreparedBatch:
    """A marshalled batch (Context.prepare_*): the argument array of one of the batched calls and the
    tensors it points into, kept alive with it.  A job that passes the same tensors again and again
    builds the array once, as a C caller would, and hands it to the call in place of the sequence."""

    def __init__(self, kind, arr, count, keep, wflags=0):
        self.kind, self.arr, self.count, self.keep, self.wflags = kind, arr, count, keep, wflags


class Context:
    """Owns one excp_ctx.  Tensors are torch CUDA tensors; blobs are uint8 CUDA tensors."""

    def __init__(self, max_tensor_elems: int, max_group_elems: int | None = None, device=None, stream=None):
        import torch
        self.device = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
        if self.device.index is None:
            self.device = torch.device("cuda", torch.cuda.current_device())
        self._stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        handle = C.c_void_p()
        group = max_tensor_elems if max_group_elems is None else max_group_elems
        rc = lib().excp_create(C.byref(handle), self.device.index, C.c_void_p(self._stream.cuda_stream),
                               max_tensor_elems, group)
        if rc != EXCP_OK:
            raise ExcpError(rc, "excp_create")
        self._h = handle
        self._keep = None
        self._count = 0

    def close(self):
        if getattr(self, "_h", None):
            lib().excp_destroy(self._h)
            self._h = None

    __del__ = close

    @property
    def workspace_bytes(self) -> int:
        return int(lib().excp_workspace_bytes(self._h))

    # -- batched -----------------------------------------------------------------
    def _batch(self, items, kind, make):
        if not isinstance(items, PreparedBatch):
            return make()
        if items.kind != kind:
            raise TypeError(f"a batch prepared for {items.kind} was passed to a {kind} call")
        return items

    def _submit(self, fn, name, batch):
        rc = fn(self._h, batch.count, batch.arr)
        if rc != EXCP_OK:
            raise ExcpError(rc, name)
        self._keep = batch
        self._count = batch.count

    def prepare_compress(self, tensors, flags=0):
        """Marshals a compress batch once: sequence of (W_prev_recon, W_t, m_t, v_t, blob,
        W_recon_out-or-None) -> a PreparedBatch that excp_compress_tensors accepts in place of the
        sequence, as often as wanted (a job that checkpoints the same tensors again and again builds
        its argument array once, as a C caller would).  `flags` names the weight storage."""
        arr = (ExcpTensor * max(len(tensors), 1))()
        for i, (Wp, W, m, v, blob, Wout) in enumerate(tensors):
            for t, nm in ((Wp, "W_prev_recon"), (W, "W_t"), (m, "m_t"), (v, "v_t")):
                _check_f32(t, nm, self.device, flags)
            n = W.numel()
            if not (Wp.numel() == n == m.numel() == v.numel()):
                raise ValueError("tensor lengths differ")
            if Wout is not None:
                _check_f32(Wout, "W_recon_out", self.device, flags)
                if Wout.numel() != n:
                    raise ValueError("W_recon_out length differs")
            arr[i] = ExcpTensor(Wp.data_ptr(), W.data_ptr(), m.data_ptr(), v.data_ptr(), n,
                                blob.data_ptr(), blob.numel() * blob.element_size(),
                                0 if Wout is None else Wout.data_ptr())
        return PreparedBatch("compress", arr, len(tensors), tensors, flags & (EXCP_FLAG_W_F16 | EXCP_FLAG_W_BF16))

    def excp_compress_tensors(self, tensors, alpha=5e-5, beta=2.0, nbits=4, lloyd_iters=10, flags=0):
        """tensors: sequence of (W_prev_recon, W_t, m_t, v_t, blob, W_recon_out-or-None), or the
        PreparedBatch that prepare_compress made of one."""
        batch = self._batch(tensors, "compress", lambda: self.prepare_compress(tensors, flags))
        if batch.wflags != flags & (EXCP_FLAG_W_F16 | EXCP_FLAG_W_BF16):
            raise TypeError("the batch was prepared for another weight storage")
        rc = lib().excp_compress_tensors(self._h, batch.count, batch.arr, alpha, beta, nbits, lloyd_iters, flags)
        if rc != EXCP_OK:
            raise ExcpError(rc, "excp_compress_tensors")
        self._keep = batch
        self._count = batch.count

    def excp_decompress_tensors(self, blobs):
        """blobs: sequence of (W_prev_recon, blob, blob_bytes, n, W_recon_out, m_out, v_out), or the
        PreparedBatch that prepare_decompress made of one."""
        self._submit(lib().excp_decompress_tensors, "excp_decompress_tensors",
                     self._batch(blobs, "decompress", lambda: self.prepare_decompress(blobs)))

    def prepare_decompress(self, blobs):
        """Marshals a decompress batch once (see prepare_compress)."""
        arr = (ExcpBlob * max(len(blobs), 1))()
        for i, (Wp, blob, nbytes, n, Wout, mout, vout) in enumerate(blobs):
            _check_f32(Wp, "W_prev_recon", self.device)
            for t, nm in ((Wout, "W_recon_out"), (mout, "m_out"), (vout, "v_out")):
                if t is not None:
                    _check_f32(t, nm, self.device)
                    if t.numel() != n:
                        raise ValueError(nm + " length differs")
            if Wp.numel() != n:
                raise ValueError("W_prev_recon length differs")
            if nbytes > blob.numel() * blob.element_size():
                raise ValueError("blob_bytes exceeds the blob tensor")
            arr[i] = ExcpBlob(Wp.data_ptr(), blob.data_ptr(), nbytes, n,
                              0 if Wout is None else Wout.data_ptr(),
                              0 if mout is None else mout.data_ptr(),
                              0 if vout is None else vout.data_ptr(), _wflags(Wp, Wout), 0)
        return PreparedBatch("decompress", arr, len(blobs), blobs)

    def excp_export_dense(self, items):
        """items: sequence of (blob, blob_bytes, n, head, codes_w, codes_m, codes_v); the last four are
        uint8 device tensors or None; or the PreparedBatch that prepare_export_dense made of one."""
        self._submit(lib().excp_export_dense, "excp_export_dense",
                     self._batch(items, "export_dense", lambda: self.prepare_export_dense(items)))

    def prepare_export_dense(self, items):
        """Marshals an export batch once (see prepare_compress)."""
        arr = (ExcpDenseExport * max(len(items), 1))()
        for i, (blob, nbytes, n, head, cw, cm, cv) in enumerate(items):
            if nbytes > blob.numel() * blob.element_size():
                raise ValueError("blob_bytes exceeds the blob tensor")
            arr[i] = ExcpDenseExport(blob.data_ptr(), nbytes, n, *[0 if t is None else t.data_ptr()
                                                                     for t in (head, cw, cm, cv)])
        return PreparedBatch("export_dense", arr, len(items), items)

    def excp_decompress_dense(self, items):
        """items: sequence of (W_prev_recon, head, head_bytes, n, codes_w, codes_m, codes_v,
        W_recon_out, m_out, v_out), or the PreparedBatch that prepare_decompress_dense made of one."""
        self._submit(lib().excp_decompress_dense, "excp_decompress_dense",
                     self._batch(items, "decompress_dense", lambda: self.prepare_decompress_dense(items)))

    def prepare_decompress_dense(self, items):
        """Marshals a batch of reconstructions from the stored layout once (see prepare_compress)."""
        arr = (ExcpDenseBlob * max(len(items), 1))()
        for i, (Wp, head, hbytes, n, cw, cm, cv, Wout, mout, vout) in enumerate(items):
            if Wp is not None:
                _check_f32(Wp, "W_prev_recon", self.device)
                if Wp.numel() != n:
                    raise ValueError("W_prev_recon length differs")
            for t, nm in ((Wout, "W_recon_out"), (mout, "m_out"), (vout, "v_out")):
                if t is not None:
                    _check_f32(t, nm, self.device)
                    if t.numel() != n:
                        raise ValueError(nm + " length differs")
            if hbytes > head.numel() * head.element_size():
                raise ValueError("head_bytes exceeds the head tensor")
            arr[i] = ExcpDenseBlob(0 if Wp is None else Wp.data_ptr(), head.data_ptr(), hbytes, n,
                                   *[0 if t is None else t.data_ptr() for t in (cw, cm, cv, Wout, mout, vout)],
                                   _wflags(Wp, Wout), 0)
        return PreparedBatch("decompress_dense", arr, len(items), items)

    def excp_reconstruct_chain(self, chains):
        """chains: sequence of (W0, [blob tensors, oldest first], [blob_bytes], W_out, m_out, v_out), or
        the PreparedBatch that prepare_chain made of one."""
        self._submit(lib().excp_reconstruct_chain, "excp_reconstruct_chain",
                     self._batch(chains, "chain", lambda: self.prepare_chain(chains)))

    def prepare_chain(self, chains):
        """Marshals a batch of chains once (see prepare_compress)."""
        arr = (ExcpChain * max(len(chains), 1))()
        keep = []
        for i, (W0, blobs, sizes, Wout, mout, vout) in enumerate(chains):
            _check_f32(W0, "W0", self.device)
            n = W0.numel()
            for t, nm in ((Wout, "W_out"), (mout, "m_out"), (vout, "v_out")):
                if t is not None:
                    _check_f32(t, nm, self.device)
                    if t.numel() != n:
                        raise ValueError(nm + " length differs")
            if len(blobs) != len(sizes):
                raise ValueError("blobs and blob_bytes differ in length")
            for b, nb in zip(blobs, sizes):
                if nb > b.numel() * b.element_size():
                    raise ValueError("blob_bytes exceeds the blob tensor")
            ptrs = (C.c_void_p * max(len(blobs), 1))(*[b.data_ptr() for b in blobs])
            nbs = (C.c_uint64 * max(len(blobs), 1))(*[int(x) for x in sizes])
            keep.append((ptrs, nbs))
            arr[i] = ExcpChain(W0.data_ptr(), n, len(blobs), C.cast(ptrs, C.POINTER(C.c_void_p)),
                               C.cast(nbs, C.POINTER(C.c_uint64)),
                               0 if Wout is None else Wout.data_ptr(),
                               0 if mout is None else mout.data_ptr(),
                               0 if vout is None else vout.data_ptr(), _wflags(W0, Wout), 0)
        return PreparedBatch("chain", arr, len(chains), (chains, keep))

    def excp_collect(self, check=True):
        stats = (ExcpStats * max(self._count, 1))()
        rc = lib().excp_collect(self._h, stats)
        self._keep = None
        out = [stats[i] for i in range(self._count)]
        if check and rc != EXCP_OK:
            raise ExcpError(rc, "excp_collect")
        return rc, out

    # -- single tensor -------------------------------------------------------------
    def excp_compress_step(self, Wp, W, m, v, blob, alpha=5e-5, beta=2.0, nbits=4, lloyd_iters=10,
                           flags=0, W_recon_out=None, check=True):
        for t, nm in ((Wp, "W_prev_recon"), (W, "W_t"), (m, "m_t"), (v, "v_t")):
            _check_f32(t, nm, self.device, flags)
        n = W.numel()
        if not (Wp.numel() == n == m.numel() == v.numel()):
            raise ValueError("tensor lengths differ")
        if W_recon_out is not None:
            _check_f32(W_recon_out, "W_recon_out", self.device, flags)
        nbytes = C.c_uint64(0)
        st = ExcpStats()
        rc = lib().excp_compress_step(self._h, _ptr(Wp), _ptr(W), _ptr(m), _ptr(v), n, alpha, beta, nbits,
                                      lloyd_iters, flags, _ptr(blob), blob.numel() * blob.element_size(),
                                      C.byref(nbytes), _ptr(W_recon_out), C.byref(st))
        if check and rc != EXCP_OK:
            raise ExcpError(rc, "excp_compress_step")
        return rc, int(nbytes.value), st

    def excp_decompress_step(self, Wp, blob, blob_bytes, W_recon_out=None, m_out=None, v_out=None, check=True):
        _check_f32(Wp, "W_prev_recon", self.device)
        n = Wp.numel()
        for t, nm in ((W_recon_out, "W_recon_out"), (m_out, "m_out"), (v_out, "v_out")):
            if t is not None:
                _check_f32(t, nm, self.device)
                if t.numel() != n:
                    raise ValueError(nm + " length differs")
        rc = lib().excp_decompress_step(self._h, _ptr(Wp), _ptr(blob), blob_bytes, n, _ptr(W_recon_out),
                                        _ptr(m_out), _ptr(v_out), _wflags(Wp, W_recon_out))
        if check and rc != EXCP_OK:
            raise ExcpError(rc, "excp_decompress_step")
        return rc

    def excp_copy_probe(self, dst, src, nbytes: int):
        rc = lib().excp_copy_probe(self._h, _ptr(dst), _ptr(src), nbytes)
        if rc != EXCP_OK:
            raise ExcpError(rc, "excp_copy_probe")

    def excp_set_param(self, param: int, value: int):
        rc = lib().excp_set_param(self._h, param, value)
        if rc != EXCP_OK:
            raise ExcpError(rc, "excp_set_param")

    # -- timing ----------------------------------------------------------------------
    def excp_set_profiling(self, enabled: bool):
        rc = lib().excp_set_profiling(self._h, int(enabled))
        if rc != EXCP_OK:
            raise ExcpError(rc, "excp_set_profiling")

    def stage_times(self) -> dict:
        out = {}
        for i in range(lib().excp_stage_count()):
            ms, launches = C.c_double(0), C.c_int(0)
            lib().excp_stage_ms(self._h, i, C.byref(ms), C.byref(launches))
            out[lib().excp_stage_name(i).decode()] = (ms.value, launches.value)
        return out
