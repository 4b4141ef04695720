"""Thin ctypes binding of the C ABI in ``include/intattn.h``.

Argument marshalling only: torch supplies device memory and the stream, every step of the
attention path runs inside ``libintattn.so``.  There is no fallback: if the library has not
been built (``python -m paper_2511_21513_amd.build`` or ``__graft_entry__.build()``), loading
raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libintattn.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_HIP, ERR_NOMEM = 0, -1, -2, -3, -4

SYMBOLS = (
    "intattn_create",
    "intattn_forward",
    "intattn_forward_noalloc",
    "intattn_reserve",
    "intattn_forward_stage",
    "intattn_forward_dynamic",
    "intattn_dynamic_status",
    "intattn_forward_quantonly",
    "intattn_quantize",
    "intattn_quantize_batch",
    "intattn_index_softmax",
    "intattn_derive_params",
    "intattn_derive_index_map",
    "intattn_get_lut",
    "intattn_last_error",
    "intattn_destroy",
)


class IntAttnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"intattn error {code}: {text}")
        self.code = code


class Config(ctypes.Structure):
    _fields_ = [
        ("device", ctypes.c_int32),
        ("lut_bits", ctypes.c_int32),
        ("clip", ctypes.c_double),
        ("variant", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
    ]


class Args(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("L", ctypes.c_int32), ("d", ctypes.c_int32), ("causal", ctypes.c_int32),
        ("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("out", ctypes.c_void_p),
        ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3),
        ("v_stride", ctypes.c_int64 * 3), ("out_stride", ctypes.c_int64 * 3),
        ("scale_mode", ctypes.c_int32), ("Lkv", ctypes.c_int32),
        ("scale_q", ctypes.c_void_p), ("scale_k", ctypes.c_void_p),
        ("scale_v", ctypes.c_void_p), ("scale_out", ctypes.c_void_p),
        ("dbg_row_max", ctypes.c_void_p), ("dbg_row_sum", ctypes.c_void_p), ("dbg_acc", ctypes.c_void_p),
        ("q_block", ctypes.c_int32), ("k_block", ctypes.c_int32),
    ]


class SoftmaxArgs(ctypes.Structure):
    _fields_ = [
        ("rows", ctypes.c_int64), ("cols", ctypes.c_int32), ("c_int", ctypes.c_int32),
        ("logits", ctypes.c_void_p), ("prob", ctypes.c_void_p),
        ("logits_stride", ctypes.c_int64), ("prob_stride", ctypes.c_int64),
        ("causal", ctypes.c_int32), ("rows_per_matrix", ctypes.c_int32),
    ]


class QuantArgs(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32), ("d", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("scale_mode", ctypes.c_int32),
        ("src", ctypes.c_void_p), ("dst", ctypes.c_void_p),
        ("src_stride", ctypes.c_int64 * 3), ("dst_stride", ctypes.c_int64 * 3),
        ("scales", ctypes.c_void_p),
        ("q_block", ctypes.c_int32), ("reserved", ctypes.c_int32),
    ]


_lib = None


def load() -> ctypes.CDLL:
    """Loads libintattn.so (raises if it is not built) and declares the prototypes."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2511_21513_amd.build` "
                "(there is no fallback path)"
            )
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.intattn_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(Config)]
        lib.intattn_create.restype = i32
        lib.intattn_forward.argtypes = [vp, ctypes.POINTER(Args), vp]
        lib.intattn_forward.restype = i32
        lib.intattn_forward_noalloc.argtypes = [vp, ctypes.POINTER(Args), vp]
        lib.intattn_forward_noalloc.restype = i32
        lib.intattn_reserve.argtypes = [vp, ctypes.POINTER(Args), i32]
        lib.intattn_reserve.restype = i32
        lib.intattn_forward_stage.argtypes = [vp, ctypes.POINTER(Args), vp, i32]
        lib.intattn_forward_stage.restype = i32
        lib.intattn_forward_dynamic.argtypes = [vp, ctypes.POINTER(Args), vp]
        lib.intattn_forward_dynamic.restype = ctypes.c_int
        lib.intattn_dynamic_status.argtypes = [vp, ctypes.POINTER(i32)]
        lib.intattn_dynamic_status.restype = ctypes.c_int
        lib.intattn_index_softmax.argtypes = [vp, ctypes.POINTER(SoftmaxArgs), vp]
        lib.intattn_index_softmax.restype = ctypes.c_int
        lib.intattn_quantize.argtypes = [vp, ctypes.POINTER(QuantArgs), vp]
        lib.intattn_quantize.restype = i32
        lib.intattn_quantize_batch.argtypes = [vp, ctypes.POINTER(QuantArgs), i32, vp]
        lib.intattn_quantize_batch.restype = i32
        lib.intattn_forward_quantonly.argtypes = [vp, ctypes.POINTER(Args), vp]
        lib.intattn_forward_quantonly.restype = i32
        lib.intattn_derive_params.argtypes = [
            vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float, i32,
            ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(i32), ctypes.POINTER(i32),
        ]
        lib.intattn_derive_params.restype = i32
        lib.intattn_derive_index_map.argtypes = [
            vp, ctypes.c_int64, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_uint32),
            ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(i32),
        ]
        lib.intattn_derive_index_map.restype = i32
        lib.intattn_get_lut.argtypes = [vp, vp, i32]
        lib.intattn_get_lut.restype = i32
        lib.intattn_last_error.argtypes = [vp]
        lib.intattn_last_error.restype = ctypes.c_char_p
        lib.intattn_destroy.argtypes = [vp]
        lib.intattn_destroy.restype = None
        _lib = lib
    return _lib


def _host_f32(x):
    if x is None:
        return None
    return np.ascontiguousarray(np.atleast_1d(np.asarray(x, dtype=np.float32)))


class IntAttn:
    """One library context (``intattn_create`` .. ``intattn_destroy``)."""

    def __init__(self, device: int = 0, lut_bits: int = 5, clip: float = 6.6, variant: int = 0):
        self._lib = load()
        self._ctx = ctypes.c_void_p()
        cfg = Config(device, lut_bits, clip, variant, 0)
        rc = self._lib.intattn_create(ctypes.byref(self._ctx), ctypes.byref(cfg))
        if rc != OK:
            raise IntAttnError(rc, (self._lib.intattn_last_error(None) or b"").decode())
        self.device = device

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self._lib.intattn_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return (self._lib.intattn_last_error(self._ctx) or b"").decode()

    def lut(self) -> np.ndarray:
        buf = np.zeros(64, dtype=np.uint8)
        n = self._lib.intattn_get_lut(self._ctx, buf.ctypes.data_as(ctypes.c_void_p), 64)
        if n < 0:
            raise IntAttnError(n, "intattn_get_lut")
        return buf[:n].copy()

    def derive_params(self, s_q, s_k, s_v, s_o, d):
        c, m, sh = ctypes.c_int64(0), ctypes.c_int32(0), ctypes.c_int32(0)
        rc = self._lib.intattn_derive_params(
            self._ctx, float(np.float32(s_q)), float(np.float32(s_k)), float(np.float32(s_v)),
            float(np.float32(s_o)), d, ctypes.byref(c), ctypes.byref(m), ctypes.byref(sh),
        )
        if rc != OK:
            raise IntAttnError(rc, "intattn_derive_params")
        return int(c.value), int(m.value), int(sh.value)

    def derive_index_map(self, c_int: int, mode: int = 2):
        mode, sh = ctypes.c_int32(mode), ctypes.c_int32(0)
        mul, add = ctypes.c_uint32(0), ctypes.c_uint32(0)
        rc = self._lib.intattn_derive_index_map(
            self._ctx, c_int, ctypes.byref(mode), ctypes.byref(mul), ctypes.byref(add), ctypes.byref(sh)
        )
        if rc != OK:
            raise IntAttnError(rc, "intattn_derive_index_map")
        return int(mode.value), int(mul.value), int(add.value), int(sh.value)

    def make_args(self, q, k, v, out, s_q, s_k, s_v, s_o=None, *, causal=False, per_head=False,
                  row_max=None, row_sum=None, acc=None, device_scales=False, q_block=0, k_block=0):
        """Marshals torch int8 tensors [B,H,L,d] (last dim contiguous) into an ``Args``.  Returns
        (args, keepalive): keepalive holds the scale arrays the struct points at: host arrays, or
        with ``device_scales`` the float32 device tensors given (for ``forward_dynamic_args``).
        ``q_block`` > 0 (device scales only): scale mode 2, s_q and s_o hold one value per block of
        ``q_block`` query rows of every (batch, head), s_k and s_v one per KV head.  ``k_block`` > 0 as
        well: scale mode 3, s_k holds one value per block of ``k_block`` keys of every (batch, KV head)."""
        B, Hq, L, d = q.shape
        Hkv = k.shape[1]
        if k.shape != v.shape or k.shape[0] != B or k.shape[3] != d or out.shape != q.shape:
            raise ValueError("q, out must be [B,Hq,L,d] and k, v [B,Hkv,Lkv,d]")
        for t in (q, k, v, out):
            if t.stride(-1) != 1:
                raise ValueError("the head dimension must be contiguous")
        a = Args()
        a.B, a.Hq, a.Hkv, a.L, a.d, a.causal = B, Hq, Hkv, L, d, int(bool(causal))
        a.q, a.k, a.v, a.out = q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr()
        a.q_stride = (ctypes.c_int64 * 3)(*q.stride()[:3])
        a.k_stride = (ctypes.c_int64 * 3)(*k.stride()[:3])
        a.v_stride = (ctypes.c_int64 * 3)(*v.stride()[:3])
        a.out_stride = (ctypes.c_int64 * 3)(*out.stride()[:3])
        a.scale_mode = int(bool(per_head))
        a.Lkv = k.shape[2]
        if device_scales:
            import torch

            keep = [s_q, s_k, s_v, s_o]
            for t in keep:
                if t is not None and (t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous()):
                    raise ValueError("device scales must be contiguous float32 tensors on the GPU")
            sizes = [t.numel() if t is not None else None for t in keep]
            ptr = lambda t: t.data_ptr()  # noqa: E731
        else:
            keep = [_host_f32(s_q), _host_f32(s_k), _host_f32(s_v), _host_f32(s_o)]
            sizes = [t.size if t is not None else None for t in keep]
            ptr = lambda t: t.ctypes.data  # noqa: E731
        if q_block:
            if not device_scales:
                raise ValueError("q_block needs device_scales")
            n_grp = B * Hq * ((L + q_block - 1) // q_block)
            a.scale_mode, a.q_block = 2, int(q_block)
            want = [n_grp, Hkv, Hkv, n_grp]
            if k_block:
                a.scale_mode, a.k_block = 3, int(k_block)
                want[1] = B * Hkv * ((k.shape[2] + k_block - 1) // k_block)
        elif k_block:
            raise ValueError("k_block needs q_block (use q_block = L for one query scale per head)")
        else:
            want = [Hq, Hkv, Hkv, Hq] if per_head else [1, 1, 1, 1]
        for have, need in zip(sizes, want):
            if have is not None and (have != need if (per_head or q_block) else have < 1):
                raise ValueError("scale arrays do not have the number of entries the scale mode needs")
        a.scale_q, a.scale_k, a.scale_v = (ptr(x) for x in keep[:3])
        a.scale_out = ptr(keep[3]) if keep[3] is not None else None
        a.dbg_row_max = row_max.data_ptr() if row_max is not None else None
        a.dbg_row_sum = row_sum.data_ptr() if row_sum is not None else None
        a.dbg_acc = acc.data_ptr() if acc is not None else None
        return a, keep

    def forward_args(self, args: Args, stream: int = 0, quantonly: bool = False):
        fn = self._lib.intattn_forward_quantonly if quantonly else self._lib.intattn_forward
        rc = fn(self._ctx, ctypes.byref(args), ctypes.c_void_p(stream))
        if rc != OK:
            raise IntAttnError(rc, self.last_error())

    def forward_noalloc_args(self, args: Args, stream: int = 0):
        """intattn_forward_noalloc: the forward with its workspace in the library's static device array."""
        rc = self._lib.intattn_forward_noalloc(self._ctx, ctypes.byref(args), ctypes.c_void_p(stream))
        if rc != OK:
            raise IntAttnError(rc, self.last_error())

    def reserve(self, args: Args, dynamic: bool = False):
        """intattn_reserve: pre-size the context's device memory for problems up to this one."""
        rc = self._lib.intattn_reserve(self._ctx, ctypes.byref(args), int(bool(dynamic)))
        if rc != OK:
            raise IntAttnError(rc, self.last_error())

    def forward_dynamic_args(self, args: Args, stream: int = 0):
        """intattn_forward_dynamic: ``args`` built with ``device_scales=True``."""
        rc = self._lib.intattn_forward_dynamic(self._ctx, ctypes.byref(args), ctypes.c_void_p(stream))
        if rc != OK:
            raise IntAttnError(rc, self.last_error())

    def dynamic_status(self) -> int:
        st = ctypes.c_int32(0)
        rc = self._lib.intattn_dynamic_status(self._ctx, ctypes.byref(st))
        if rc != OK:
            raise IntAttnError(rc, self.last_error())
        return int(st.value)

    def index_softmax(self, logits, c_int: int, *, causal: bool = False, rows_per_matrix: int = 0, out=None, stream=None):
        """intattn_index_softmax on a torch int32 tensor [..., cols] (rows contiguous, all leading
        axes collapsible to one row stride): uint8 probabilities of the same shape."""
        import torch

        cols = logits.shape[-1]
        flat = logits.reshape(-1, cols)  # a view, or torch raises on a copy below
        if flat.data_ptr() != logits.data_ptr() or flat.stride(-1) != 1:
            raise ValueError("logits must be viewable as [rows, cols] with contiguous rows")
        if out is None:
            out = torch.empty(logits.shape, dtype=torch.uint8, device=logits.device)
        oflat = out.reshape(-1, cols)
        if oflat.data_ptr() != out.data_ptr() or oflat.stride(-1) != 1 or oflat.shape[0] != flat.shape[0]:
            raise ValueError("out must be viewable as [rows, cols] with contiguous rows")
        a = SoftmaxArgs()
        a.rows, a.cols, a.c_int = flat.shape[0], cols, int(c_int)
        a.logits, a.prob = flat.data_ptr(), oflat.data_ptr()
        a.logits_stride = (flat.stride(0) if flat.shape[0] > 1 else cols) * 4
        a.prob_stride = oflat.stride(0) if oflat.shape[0] > 1 else cols
        a.causal, a.rows_per_matrix = int(bool(causal)), int(rows_per_matrix)
        if stream is None:
            stream = torch.cuda.current_stream(logits.device).cuda_stream
        rc = self._lib.intattn_index_softmax(self._ctx, ctypes.byref(a), ctypes.c_void_p(stream))
        if rc != OK:
            raise IntAttnError(rc, self.last_error())
        return out

    def quantize(self, x, per_head: bool = False, out=None, scales=None, stream=None, q_block: int = 0):
        """intattn_quantize on a [B, H, L, d] device tensor (torch float32 / float16 / bfloat16,
        last dimension contiguous): returns (int8 tensor, float32 device tensor of 1 or H scales;
        with ``q_block`` > 0 one scale per block of ``q_block`` rows, [B, H, ceil(L / q_block)]).
        Argument marshalling only."""
        import torch

        dtypes = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}
        if x.dim() != 4 or x.dtype not in dtypes or x.stride(3) != 1:
            raise ValueError("expected a [B, H, L, d] float32/float16/bfloat16 tensor with contiguous last dimension")
        B, H, L, d = x.shape
        if out is None:
            out = torch.empty((B, H, L, d), dtype=torch.int8, device=x.device)
        if scales is None:
            shape = (B, H, (L + q_block - 1) // q_block) if q_block else (H if per_head else 1,)
            scales = torch.empty(shape, dtype=torch.float32, device=x.device)
        a = QuantArgs()
        a.B, a.H, a.L, a.d = B, H, L, d
        a.dtype, a.scale_mode = dtypes[x.dtype], 2 if q_block else int(per_head)
        a.q_block = int(q_block)
        a.src, a.dst, a.scales = x.data_ptr(), out.data_ptr(), scales.data_ptr()
        es = x.element_size()
        for i in range(3):
            a.src_stride[i] = x.stride(i) * es
            a.dst_stride[i] = out.stride(i)
        st = torch.cuda.current_stream(x.device).cuda_stream if stream is None else stream
        rc = self._lib.intattn_quantize(self._ctx, ctypes.byref(a), ctypes.c_void_p(st))
        if rc != OK:
            raise IntAttnError(rc, self.last_error())
        return out, scales

    def quant_args(self, x, out, scales, per_head: bool = False, q_block: int = 0) -> "QuantArgs":
        """Marshals one tensor of a quantizer call (see ``quantize``)."""
        import torch

        dtypes = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}
        if x.dim() != 4 or x.dtype not in dtypes or x.stride(3) != 1:
            raise ValueError("expected a [B, H, L, d] float32/float16/bfloat16 tensor with contiguous last dimension")
        a = QuantArgs()
        a.B, a.H, a.L, a.d = x.shape
        a.dtype, a.scale_mode = dtypes[x.dtype], 2 if q_block else int(per_head)
        a.q_block = int(q_block)
        a.src, a.dst, a.scales = x.data_ptr(), out.data_ptr(), scales.data_ptr()
        es = x.element_size()
        for i in range(3):
            a.src_stride[i] = x.stride(i) * es
            a.dst_stride[i] = out.stride(i)
        return a

    def quantize_batch(self, xs, per_head=False, outs=None, scales=None, stream=None):
        """intattn_quantize_batch: up to four [B, H, L, d] device tensors in one pair of launches.
        ``per_head``: one flag, or one per tensor.  Returns (list of int8 tensors, list of scale tensors)."""
        import torch

        n = len(xs)
        flags = list(per_head) if isinstance(per_head, (list, tuple)) else [per_head] * n
        if outs is None:
            outs = [torch.empty(x.shape, dtype=torch.int8, device=x.device) for x in xs]
        if scales is None:
            scales = [torch.empty(x.shape[1] if f else 1, dtype=torch.float32, device=x.device) for x, f in zip(xs, flags)]
        arr = (QuantArgs * n)(*[self.quant_args(x, o, s, f) for x, o, s, f in zip(xs, outs, scales, flags)])
        st = torch.cuda.current_stream(xs[0].device).cuda_stream if stream is None else stream
        rc = self._lib.intattn_quantize_batch(self._ctx, arr, n, ctypes.c_void_p(st))
        if rc != OK:
            raise IntAttnError(rc, self.last_error())
        return outs, scales

    def forward_stage(self, args: Args, stage: int, stream: int = 0):
        """intattn_forward_stage: 0 = everything, 1 = column sums and sweeps A+B, 2 = sweep C."""
        rc = self._lib.intattn_forward_stage(self._ctx, ctypes.byref(args), ctypes.c_void_p(stream), stage)
        if rc != OK:
            raise IntAttnError(rc, self.last_error())

    def forward(self, q, k, v, s_q, s_k, s_v, s_o=None, *, causal=False, per_head=False, out=None,
                taps=False, stream=None, quantonly=False):
        """intattn_forward on torch tensors.  Returns ``out`` (int8 [B,Hq,L,d]); with ``taps`` a
        dict with out, row_max, row_sum, acc.  Enqueued on torch's current stream unless given."""
        import torch

        if out is None:
            out = torch.empty_like(q)
        extra = {}
        if taps:
            B, Hq, L, d = q.shape
            extra = {
                "row_max": torch.zeros((B, Hq, L), dtype=torch.int32, device=q.device),
                "row_sum": torch.zeros((B, Hq, L), dtype=torch.int32, device=q.device),
                "acc": torch.zeros((B, Hq, L, d), dtype=torch.int32, device=q.device),
            }
        args, keep = self.make_args(q, k, v, out, s_q, s_k, s_v, s_o, causal=causal, per_head=per_head, **extra)
        if stream is None:
            stream = torch.cuda.current_stream(q.device).cuda_stream
        self.forward_args(args, stream, quantonly)
        del keep
        if taps:
            extra["out"] = out
            return extra
        return out
