"""ctypes binding of the IST C ABI (include/ist.h): argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the
hot path runs in the HIP kernels of libist.so.  There is no CPU fallback: if the
library has not been built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch  # loads the HIP runtime the library resolves against

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libist.so")

IST_OK = 0
STATUS = {0: "IST_OK", -1: "IST_EINVAL", -2: "IST_ESHAPE", -3: "IST_EPERM", -4: "IST_ENOMEM",
          -5: "IST_EHIP", -6: "IST_ESTATE", -7: "IST_EUNSUPPORTED"}
IST_F32, IST_BF16 = 0, 1
IST_DENSE, IST_CSR = 0, 1

EXPORTS = ["ist_create", "ist_destroy", "ist_subnets_bytes", "ist_workspace_bytes", "ist_bind",
           "ist_set_checked", "ist_partition", "ist_subnet_steps", "ist_merge", "ist_subnet_export",
           "ist_subnet_shape", "ist_last_error", "ist_version", "ist_profile_enable",
           "ist_profile_reset", "ist_profile_read", "ist_profile_classes", "ist_profile_class_name",
           "ist_profile_kernel_count", "ist_profile_kernel", "ist_bind_spare", "ist_resample",
           "ist_forward_full", "ist_forward_full_static", "ist_subnet_shape_of"]


class ISTError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status


class _ModelDesc(C.Structure):
    _fields_ = [("t", C.c_int32), ("dims", C.POINTER(C.c_int64)), ("S", C.c_int32),
                ("dtype", C.c_int32), ("input", C.c_int32), ("has_bias", C.c_int32),
                ("normalize", C.c_int32), ("norm_eps", C.c_float),
                ("layer_scale", C.POINTER(C.c_float))]


class _Params(C.Structure):
    _fields_ = [("W", C.POINTER(C.c_void_p)), ("b", C.POINTER(C.c_void_p))]


class _Batch(C.Structure):
    _fields_ = [("x", C.c_void_p), ("rowptr", C.c_void_p), ("colidx", C.c_void_p),
                ("vals", C.c_void_p), ("nnz", C.c_int64), ("y", C.c_void_p),
                ("stride_s", C.c_int64), ("stride_k", C.c_int64), ("B", C.c_int32)]


_lib = None


def load_library() -> C.CDLL:
    """Load libist.so (built by paper_1910_02120_amd/build.py).  Fails loudly."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_1910_02120_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    p = C.c_void_p
    lib.ist_create.argtypes = [C.POINTER(_ModelDesc), C.c_int32, C.POINTER(p)]
    lib.ist_destroy.argtypes = [p]
    lib.ist_subnets_bytes.argtypes = [p, C.POINTER(C.c_size_t)]
    lib.ist_workspace_bytes.argtypes = [p, C.POINTER(C.c_size_t)]
    lib.ist_bind.argtypes = [p, p, C.c_size_t, p, C.c_size_t]
    lib.ist_set_checked.argtypes = [p, C.c_int32]
    lib.ist_partition.argtypes = [p, C.POINTER(_Params), C.POINTER(p), p]
    lib.ist_subnet_steps.argtypes = [p, C.POINTER(_Batch), C.c_float, C.c_int32, p, p]
    lib.ist_merge.argtypes = [p, C.POINTER(_Params), p]
    lib.ist_forward_full.argtypes = [p, C.POINTER(_Params), C.POINTER(_Batch), p, p]
    lib.ist_forward_full_static.argtypes = [p, C.POINTER(_Params), C.POINTER(_Batch), p, p]
    lib.ist_bind_spare.argtypes = [p, p, C.c_size_t]
    lib.ist_resample.argtypes = [p, C.POINTER(_Params), C.POINTER(p), p]
    lib.ist_subnet_export.argtypes = [p, C.c_int32, C.c_int32, p, p, p]
    lib.ist_subnet_shape.argtypes = [p, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.ist_subnet_shape_of.argtypes = [p, C.c_int32, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.ist_profile_enable.argtypes = [p, C.c_int32]
    lib.ist_profile_reset.argtypes = [p]
    lib.ist_profile_read.argtypes = [p, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.ist_profile_kernel_count.argtypes = [p, C.POINTER(C.c_int32)]
    lib.ist_profile_kernel.argtypes = [p, C.c_int32, C.c_char_p, C.c_size_t, C.POINTER(C.c_int32),
                                       C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                       C.POINTER(C.c_double)]
    lib.ist_profile_classes.argtypes = []
    lib.ist_profile_class_name.argtypes = [C.c_int32]
    for name in EXPORTS:
        getattr(lib, name).restype = C.c_int32
    lib.ist_profile_class_name.restype = C.c_char_p
    lib.ist_last_error.argtypes = [p]
    lib.ist_last_error.restype = C.c_char_p
    lib.ist_version.argtypes = []
    lib.ist_version.restype = C.c_char_p
    _lib = lib
    return lib


def _torch_dtype(dtype: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


class ISTContext:
    """One network shape split into S subnets; owns the two device buffers the
    library asks for (allocated through torch) and the opaque ist_ctx."""

    def __init__(self, dims: Sequence[int], S: int, dtype: str = "f32", input: str = "dense",
                 has_bias: bool = True, max_B: int = 128, device: str = "cuda:0",
                 bind: bool = True, normalize: bool = False, norm_eps: float = 0.0,
                 layer_scale: Optional[Sequence[float]] = None):
        self.lib = load_library()
        self.dims = [int(d) for d in dims]
        self.t = len(self.dims) - 1
        self.S, self.dtype, self.input, self.has_bias = int(S), dtype, input, bool(has_bias)
        self.device = torch.device(device)
        self._dims_arr = (C.c_int64 * len(self.dims))(*self.dims)
        desc = _ModelDesc(self.t, self._dims_arr, self.S, IST_BF16 if dtype == "bf16" else IST_F32,
                          IST_CSR if input == "csr" else IST_DENSE, 1 if has_bias else 0,
                          1 if normalize else 0, float(norm_eps))
        if layer_scale is not None:
            assert len(layer_scale) == self.t
            self._scale_arr = (C.c_float * self.t)(*[float(v) for v in layer_scale])
            desc.layer_scale = self._scale_arr
        self.normalize = bool(normalize)
        self._ctx = C.c_void_p()
        st = self.lib.ist_create(C.byref(desc), int(max_B), C.byref(self._ctx))
        if st != IST_OK:
            self._ctx = C.c_void_p()
            raise ISTError(st, "ist_create rejected the model description")
        self.max_B = int(max_B)
        self.subnets = self.workspace = None
        if bind:
            self.bind()

    # -- helpers ---------------------------------------------------------
    def _check(self, st: int):
        if st != IST_OK:
            raise ISTError(st, (self.lib.ist_last_error(self._ctx) or b"").decode())

    def subnets_bytes(self) -> int:
        n = C.c_size_t()
        self._check(self.lib.ist_subnets_bytes(self._ctx, C.byref(n)))
        return n.value

    def workspace_bytes(self) -> int:
        n = C.c_size_t()
        self._check(self.lib.ist_workspace_bytes(self._ctx, C.byref(n)))
        return n.value

    def bind(self):
        self.subnets = torch.empty(self.subnets_bytes(), dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(self.workspace_bytes(), dtype=torch.uint8, device=self.device)
        self._check(self.lib.ist_bind(self._ctx, self.subnets.data_ptr(), self.subnets.numel(),
                                      self.workspace.data_ptr(), self.workspace.numel()))

    def set_checked(self, checked: bool):
        self._check(self.lib.ist_set_checked(self._ctx, 1 if checked else 0))

    def _params(self, Ws, bs):
        assert len(Ws) == self.t
        td = _torch_dtype(self.dtype)
        for l, w in enumerate(Ws, 1):
            assert w.is_cuda and w.is_contiguous() and w.dtype == td
            assert tuple(w.shape) == (self.dims[l], self.dims[l - 1])
        Wp = (C.c_void_p * self.t)(*[w.data_ptr() for w in Ws])
        if self.has_bias:
            for l, b in enumerate(bs, 1):
                assert b.is_cuda and b.is_contiguous() and b.dtype == td and b.numel() == self.dims[l]
            bp = (C.c_void_p * self.t)(*[b.data_ptr() for b in bs])
        else:
            bp = None
        pr = _Params(Wp, bp)
        pr._keep = (Wp, bp)
        return pr

    # -- the three calls of one IST round -----------------------------------
    def partition(self, Ws: List[torch.Tensor], bs: Optional[List[torch.Tensor]],
                  perms: List[torch.Tensor], stream=None):
        assert len(perms) == self.t - 1
        for l, p in enumerate(perms, 1):
            assert p.is_cuda and p.dtype == torch.int32 and p.is_contiguous()
            assert p.numel() == self.dims[l]
        pp = (C.c_void_p * max(1, self.t - 1))(*[p.data_ptr() for p in perms])
        pr = self._params(Ws, bs)
        self._check(self.lib.ist_partition(self._ctx, C.byref(pr), pp, _stream_ptr(stream)))

    def subnet_steps(self, y: torch.Tensor, lr: float, k: int, B: int, X: torch.Tensor = None,
                     csr=None, stride_s: Optional[int] = None, stride_k: Optional[int] = None,
                     loss_out: Optional[torch.Tensor] = None, stream=None):
        """X: rows of N_0 values ([S][k][B][N_0] contiguous by default) or
        csr = (rowptr, colidx, vals) device tensors; y int32 class ids per row."""
        assert y.is_cuda and y.dtype == torch.int32 and y.is_contiguous()
        stride_k = B if stride_k is None else int(stride_k)
        stride_s = k * B if stride_s is None else int(stride_s)
        rows_needed = (self.S - 1) * stride_s + (k - 1) * stride_k + B if k > 0 else 0
        assert y.numel() >= rows_needed
        bt = _Batch()
        td = _torch_dtype(self.dtype)
        if self.input == "csr":
            rp, ci, va = csr
            assert rp.dtype == torch.int32 and ci.dtype == torch.int32 and va.dtype == td
            assert rp.is_cuda and ci.is_cuda and va.is_cuda
            assert rp.numel() >= rows_needed + 1 and ci.numel() == va.numel()
            bt.rowptr, bt.colidx, bt.vals, bt.nnz = rp.data_ptr(), ci.data_ptr(), va.data_ptr(), ci.numel()
        else:
            assert X.is_cuda and X.is_contiguous() and X.dtype == td
            assert X.numel() >= rows_needed * self.dims[0]
            bt.x = X.data_ptr()
        bt.y, bt.stride_s, bt.stride_k, bt.B = y.data_ptr(), stride_s, stride_k, int(B)
        lp = None
        if loss_out is not None:
            assert loss_out.is_cuda and loss_out.dtype == torch.float32 and loss_out.numel() >= self.S * k
            lp = loss_out.data_ptr()
        self._check(self.lib.ist_subnet_steps(self._ctx, C.byref(bt), float(lr), int(k), lp,
                                              _stream_ptr(stream)))

    def merge(self, Ws, bs, stream=None):
        pr = self._params(Ws, bs)
        self._check(self.lib.ist_merge(self._ctx, C.byref(pr), _stream_ptr(stream)))

    def forward_full(self, Ws, bs, B: int, X: torch.Tensor = None, csr=None,
                     logits: Optional[torch.Tensor] = None, stream=None, static: bool = False) -> torch.Tensor:
        """Logits [B][N_t] (float32) of the full network on samples 0..B-1 of X (rows of N_0
        values) or of csr = (rowptr, colidx, vals).  static: ist_forward_full_static (the library's own
        scratch array instead of the bound workspace; `logits` must then be given: nothing is allocated)."""
        pr = self._params(Ws, bs)
        bt = _Batch()
        td = _torch_dtype(self.dtype)
        if self.input == "csr":
            rp, ci, va = csr
            assert rp.dtype == torch.int32 and ci.dtype == torch.int32 and va.dtype == td
            assert rp.is_cuda and ci.is_cuda and va.is_cuda
            assert rp.numel() >= B + 1 and ci.numel() == va.numel()
            bt.rowptr, bt.colidx, bt.vals, bt.nnz = rp.data_ptr(), ci.data_ptr(), va.data_ptr(), ci.numel()
        else:
            assert X.is_cuda and X.is_contiguous() and X.dtype == td
            assert X.numel() >= B * self.dims[0]
            bt.x = X.data_ptr()
        bt.B = int(B)
        if logits is None:
            assert not static, "ist_forward_full_static: pass the logits buffer"
            logits = torch.empty((B, self.dims[-1]), dtype=torch.float32, device=self.device)
        assert logits.is_cuda and logits.is_contiguous() and logits.dtype == torch.float32
        assert logits.numel() >= B * self.dims[-1]
        fn = self.lib.ist_forward_full_static if static else self.lib.ist_forward_full
        self._check(fn(self._ctx, C.byref(pr), C.byref(bt), logits.data_ptr(), _stream_ptr(stream)))
        return logits

    def resample(self, Ws, bs, perms: List[torch.Tensor], stream=None):
        """merge(Ws, bs) followed by partition(Ws, bs, perms), in one pass over the weights.
        The second subnet buffer it needs is allocated at the first call."""
        if getattr(self, "spare", None) is None:
            self.spare = torch.empty(self.subnets_bytes(), dtype=torch.uint8, device=self.device)
            self._check(self.lib.ist_bind_spare(self._ctx, self.spare.data_ptr(), self.spare.numel()))
        assert len(perms) == self.t - 1
        for l, p in enumerate(perms, 1):
            assert p.is_cuda and p.dtype == torch.int32 and p.is_contiguous() and p.numel() == self.dims[l]
        pp = (C.c_void_p * max(1, self.t - 1))(*[p.data_ptr() for p in perms])
        pr = self._params(Ws, bs)
        self._check(self.lib.ist_resample(self._ctx, C.byref(pr), pp, _stream_ptr(stream)))

    # -- inspection ---------------------------------------------------------
    def subnet_shape(self, l: int, s: Optional[int] = None):
        """(rows, cols) of layer l of subnet s; of the widest subnet when s is None."""
        r, c = C.c_int64(), C.c_int64()
        if s is None:
            self._check(self.lib.ist_subnet_shape(self._ctx, l, C.byref(r), C.byref(c)))
        else:
            self._check(self.lib.ist_subnet_shape_of(self._ctx, s, l, C.byref(r), C.byref(c)))
        return r.value, c.value

    def subnet_export(self, s: int, l: int, stream=None):
        """(W_l^s [rows][cols], b_l^s [rows] or None) in permutation-block order."""
        r, c = self.subnet_shape(l, s)
        td = _torch_dtype(self.dtype)
        W = torch.empty((r, c), dtype=td, device=self.device)
        b = torch.empty((r,), dtype=td, device=self.device) if self.has_bias else None
        self._check(self.lib.ist_subnet_export(self._ctx, s, l, W.data_ptr(),
                                               b.data_ptr() if b is not None else None,
                                               _stream_ptr(stream)))
        return W, b

    # -- measurement ------------------------------------------------------
    def profile_enable(self, on: bool):
        self._check(self.lib.ist_profile_enable(self._ctx, 1 if on else 0))

    def profile_reset(self):
        self._check(self.lib.ist_profile_reset(self._ctx))

    def profile_read(self):
        """{kernel class: (total_ms, launches)} since the last reset (synchronises)."""
        out = {}
        for c in range(self.lib.ist_profile_classes()):
            ms, n = C.c_double(), C.c_int64()
            self._check(self.lib.ist_profile_read(self._ctx, c, C.byref(ms), C.byref(n)))
            if n.value:
                out[self.lib.ist_profile_class_name(c).decode()] = (ms.value, n.value)
        return out

    def profile_kernels(self):
        """[{label, kernel_class, ms, launches, flops, bytes}] per kernel label since the last reset."""
        n = C.c_int32()
        self._check(self.lib.ist_profile_kernel_count(self._ctx, C.byref(n)))
        out = []
        buf = C.create_string_buffer(96)
        for i in range(n.value):
            cls, ms, cnt, fl, by = C.c_int32(), C.c_double(), C.c_int64(), C.c_double(), C.c_double()
            self._check(self.lib.ist_profile_kernel(self._ctx, i, buf, len(buf), C.byref(cls), C.byref(ms),
                                                    C.byref(cnt), C.byref(fl), C.byref(by)))
            out.append(dict(label=buf.value.decode(), kernel_class=self.lib.ist_profile_class_name(cls.value).decode(),
                            ms=ms.value, launches=cnt.value, flops=fl.value, bytes=by.value))
        return out

    def close(self):
        if getattr(self, "_ctx", None) and self._ctx.value:
            self.lib.ist_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def version() -> str:
    return load_library().ist_version().decode()
