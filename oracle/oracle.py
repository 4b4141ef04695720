"""ctypes front end of ``intattn_oracle.c`` -- TEST INFRASTRUCTURE ONLY.

Argument marshalling and a thread fan-out over heads; all arithmetic of the
method lives in the C file.  numpy arrays in, numpy arrays out.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "intattn_oracle.c")
_LIB = os.path.join(_HERE, "libintattn_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            build()
            lib = ctypes.CDLL(_LIB)
            i32, i64, dbl, f32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_float
            vp = ctypes.c_void_p
            lib.intattn_oracle_lut.argtypes = [i32, dbl, vp]
            lib.intattn_oracle_lut.restype = i32
            lib.intattn_oracle_c_int.argtypes = [dbl, f32, f32, i32]
            lib.intattn_oracle_c_int.restype = i64
            lib.intattn_oracle_requant_params.argtypes = [f32, f32, ctypes.POINTER(i64), ctypes.POINTER(i32)]
            lib.intattn_oracle_requant_params.restype = i32
            lib.intattn_oracle_index.argtypes = [i64, i64, i32]
            lib.intattn_oracle_index.restype = i64
            lib.intattn_oracle_prob.argtypes = [i64, i64]
            lib.intattn_oracle_prob.restype = i64
            lib.intattn_oracle_forward.argtypes = (
                [i32] * 7 + [vp] * 3 + [i32] + [vp] * 4 + [i32, dbl] + [i32] * 4 + [vp] * 5
            )
            lib.intattn_oracle_forward.restype = i32
            lib.intattn_oracle_rows.argtypes = (
                [i32] * 7 + [vp] * 3 + [i32] + [vp] * 4 + [i32, dbl] + [i32] * 3 + [vp] * 5
            )
            lib.intattn_oracle_rows.restype = i32
            lib.intattn_oracle_index_softmax.argtypes = [i64, i64, vp, i64, i32, dbl, i64, i32, vp]
            lib.intattn_oracle_index_softmax.restype = i32
            lib.intattn_oracle_forward_groups.argtypes = [i32] * 7 + [vp] * 3 + [i32, i32] + [vp] * 4 + [i32, dbl] + [vp] * 5
            lib.intattn_oracle_forward_groups.restype = i32
            lib.intattn_oracle_quantize.argtypes = [i32] * 4 + [vp, i32, vp, vp]
            lib.intattn_oracle_quantize.restype = i32
            _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(x):
    return None if x is None else np.ascontiguousarray(np.atleast_1d(np.asarray(x, dtype=np.float32)))


def lut(lut_bits: int = 5, clip: float = 6.6) -> np.ndarray:
    out = np.zeros(1 << lut_bits, dtype=np.uint8)
    rc = _load().intattn_oracle_lut(lut_bits, clip, _ptr(out))
    if rc:
        raise ValueError(f"intattn_oracle_lut rc={rc}")
    return out


def c_int(clip: float, s_q: float, s_k: float, d: int) -> int:
    return int(_load().intattn_oracle_c_int(clip, float(np.float32(s_q)), float(np.float32(s_k)), d))


def requant_params(s_v: float, s_o: float):
    m, sh = ctypes.c_int64(0), ctypes.c_int32(0)
    rc = _load().intattn_oracle_requant_params(
        float(np.float32(s_v)), float(np.float32(s_o)), ctypes.byref(m), ctypes.byref(sh)
    )
    if rc:
        raise ValueError(f"intattn_oracle_requant_params rc={rc}")
    return int(m.value), int(sh.value)


def index_map(delta_clipped: int, c_int_: int, lut_bits: int = 5) -> int:
    return int(_load().intattn_oracle_index(delta_clipped, c_int_, lut_bits))


def prob(e: int, row_sum: int) -> int:
    return int(_load().intattn_oracle_prob(e, row_sum))


def _check_inputs(q, k, v):
    for name, a in (("q", q), ("k", k), ("v", v)):
        if a.dtype != np.int8 or a.ndim != 4 or not a.flags.c_contiguous:
            raise ValueError(f"{name} must be a C-contiguous int8 [B,H,L,d] array")
    B, Hq, L, d = q.shape
    Bk, Hkv, Lk, dk = k.shape
    if (Bk, dk) != (B, d) or v.shape != k.shape:
        raise ValueError("shape mismatch between q, k, v")
    return B, Hq, Hkv, L, Lk, d


def forward(q, k, v, s_q, s_k, s_v, s_o=None, *, causal=False, per_head=False, lut_bits=5, clip=6.6,
            taps=False, want_prob=False, threads=1, rows_range=None):
    """Run the oracle over all (b, h).  Returns a dict with ``out`` (int8 [B,Hq,L,d]) and,
    with ``taps``, ``row_max``/``row_sum`` (int32 [B,Hq,L]) and ``acc`` (int32 [B,Hq,L,d]);
    with ``want_prob``, ``prob`` (uint8 [B,Hq,L,Lk]).  k and v may hold Lk != L keys (then a causal
    mask is aligned to the end: row i sees keys j <= i + Lk - L).  ``threads`` fans heads over host threads
    (the C call releases the GIL); each thread runs the same single-threaded row routine."""
    lib = _load()
    B, Hq, Hkv, L, Lk, d = _check_inputs(q, k, v)
    sq, sk, sv, so = _f32(s_q), _f32(s_k), _f32(s_v), _f32(s_o)
    if per_head:
        if sq.size != Hq or sk.size != Hkv or sv.size != Hkv or (so is not None and so.size != Hq):
            raise ValueError("per-head scales must have Hq (q, out) / Hkv (k, v) entries")
    out = np.zeros((B, Hq, L, d), dtype=np.int8)
    res = {"out": out}
    if taps:
        res["row_max"] = np.zeros((B, Hq, L), dtype=np.int32)
        res["row_sum"] = np.zeros((B, Hq, L), dtype=np.int32)
        res["acc"] = np.zeros((B, Hq, L, d), dtype=np.int32)
    if want_prob:
        res["prob"] = np.zeros((B, Hq, L, Lk), dtype=np.uint8)
    r0, r1 = (0, L) if rows_range is None else rows_range

    def run(bh0, bh1):
        rc = lib.intattn_oracle_forward(
            B, Hq, Hkv, L, Lk, d, int(bool(causal)), _ptr(q), _ptr(k), _ptr(v), int(bool(per_head)),
            _ptr(sq), _ptr(sk), _ptr(sv), _ptr(so), lut_bits, clip, bh0, bh1, r0, r1, _ptr(out),
            _ptr(res.get("row_max")), _ptr(res.get("row_sum")), _ptr(res.get("acc")), _ptr(res.get("prob")),
        )
        if rc:
            raise ValueError(f"intattn_oracle_forward rc={rc}")

    nbh = B * Hq
    threads = max(1, min(int(threads), nbh))
    if threads == 1:
        run(0, nbh)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            futs = [ex.submit(run, bh, bh + 1) for bh in range(nbh)]
            for f in futs:
                f.result()
    return res


def rows(q, k, v, s_q, s_k, s_v, s_o=None, *, b, hq, rows, causal=False, per_head=False, lut_bits=5,
         clip=6.6):
    """Selected query rows of one (b, hq).  Returns dict: out [n,d] int8, row_max/row_sum [n] int32,
    acc [n,d] int32."""
    lib = _load()
    B, Hq, Hkv, L, Lk, d = _check_inputs(q, k, v)
    sq, sk, sv, so = _f32(s_q), _f32(s_k), _f32(s_v), _f32(s_o)
    idx = np.ascontiguousarray(np.asarray(rows, dtype=np.int32))
    n = idx.size
    res = {
        "out": np.zeros((n, d), dtype=np.int8),
        "row_max": np.zeros(n, dtype=np.int32),
        "row_sum": np.zeros(n, dtype=np.int32),
        "acc": np.zeros((n, d), dtype=np.int32),
    }
    rc = lib.intattn_oracle_rows(
        B, Hq, Hkv, L, Lk, d, int(bool(causal)), _ptr(q), _ptr(k), _ptr(v), int(bool(per_head)), _ptr(sq),
        _ptr(sk), _ptr(sv), _ptr(so), lut_bits, clip, b, hq, n, _ptr(idx), _ptr(res["out"]),
        _ptr(res["row_max"]), _ptr(res["row_sum"]), _ptr(res["acc"]),
    )
    if rc:
        raise ValueError(f"intattn_oracle_rows rc={rc}")
    return res


def forward_row_groups(q, k, v, s_q, s_k, s_v, s_o=None, *, q_block, causal=False, lut_bits=5, clip=6.6, taps=False):
    """Finer quantization groups over the QUERY rows (Sec. 3.3 with groups = blocks of ``q_block``
    consecutive query rows of one (batch, head); ``q_block`` = 1 is per-token quantization of Q):
    ``s_q`` (and ``s_o`` if given) hold one scale per group, [B, Hq, ceil(L / q_block)]; ``s_k``,
    ``s_v`` one per KV head.  Rows never interact, so the definition is the per-tensor pipeline run
    on each group's rows with that group's scales -- which is literally what this does."""
    B, Hq, Hkv, L, Lk, d = _check_inputs(q, k, v)
    nblk = (L + q_block - 1) // q_block
    sq = np.asarray(s_q, dtype=np.float32).reshape(B, Hq, nblk)
    so = None if s_o is None else np.asarray(s_o, dtype=np.float32).reshape(B, Hq, nblk)
    sk, sv = _f32(s_k), _f32(s_v)
    g = Hq // Hkv
    res = {"out": np.zeros((B, Hq, L, d), dtype=np.int8)}
    if taps:
        res["row_max"] = np.zeros((B, Hq, L), dtype=np.int32)
        res["row_sum"] = np.zeros((B, Hq, L), dtype=np.int32)
        res["acc"] = np.zeros((B, Hq, L, d), dtype=np.int32)
    for b in range(B):
        for h in range(Hq):
            kv = h // g
            for blk in range(nblk):
                r0, r1 = blk * q_block, min(L, (blk + 1) * q_block)
                part = rows(q, k, v, sq[b, h, blk:blk + 1], sk[kv:kv + 1], sv[kv:kv + 1],
                            None if so is None else so[b, h, blk:blk + 1], b=b, hq=h, rows=np.arange(r0, r1),
                            causal=causal, per_head=False, lut_bits=lut_bits, clip=clip)
                for key in res:
                    res[key][b, h, r0:r1] = part[key]
    return res


def forward_groups(q, k, v, s_q, s_k, s_v, s_o=None, *, q_block, k_block, causal=False, lut_bits=5, clip=6.6,
                   taps=False, want_prob=False):
    """Finer quantization groups over both axes (Sec. 3.3): ``s_q`` (and ``s_o`` if given) hold one
    scale per block of ``q_block`` query rows of every (batch, head), [B, Hq, ceil(L / q_block)];
    ``s_k`` one per block of ``k_block`` keys of every (batch, KV head), [B, Hkv, ceil(Lk / k_block)]
    (``k_block`` = 1: per key); ``s_v`` one per KV head.  Returns ``out`` and, with ``taps``,
    ``row_max_real`` (fp64 maximum of the dequantized logits), ``row_sum``, ``acc``; with
    ``want_prob``, ``prob``."""
    B, Hq, Hkv, L, Lk, d = _check_inputs(q, k, v)
    if q_block < 1 or k_block < 1:
        raise ValueError("q_block and k_block must be >= 1")
    nqb, nkb = (L + q_block - 1) // q_block, (Lk + k_block - 1) // k_block
    sq = np.ascontiguousarray(np.asarray(s_q, dtype=np.float32).reshape(B, Hq, nqb))
    so = None if s_o is None else np.ascontiguousarray(np.asarray(s_o, dtype=np.float32).reshape(B, Hq, nqb))
    sk = np.ascontiguousarray(np.asarray(s_k, dtype=np.float32).reshape(B, Hkv, nkb))
    sv = _f32(s_v)
    if sv.size != Hkv:
        raise ValueError("s_v holds one scale per KV head")
    res = {"out": np.zeros((B, Hq, L, d), dtype=np.int8)}
    if taps:
        res["row_max_real"] = np.zeros((B, Hq, L), dtype=np.float64)
        res["row_sum"] = np.zeros((B, Hq, L), dtype=np.int32)
        res["acc"] = np.zeros((B, Hq, L, d), dtype=np.int32)
    if want_prob:
        res["prob"] = np.zeros((B, Hq, L, Lk), dtype=np.uint8)
    rc = _load().intattn_oracle_forward_groups(
        B, Hq, Hkv, L, Lk, d, int(bool(causal)), _ptr(q), _ptr(k), _ptr(v), int(q_block), int(k_block),
        _ptr(sq), _ptr(sk), _ptr(sv), _ptr(so), lut_bits, clip, _ptr(res["out"]), _ptr(res.get("row_max_real")),
        _ptr(res.get("row_sum")), _ptr(res.get("acc")), _ptr(res.get("prob")))
    if rc:
        raise ValueError(f"intattn_oracle_forward_groups rc={rc}")
    return res


def quantize_row_groups(x, q_block: int):
    """Eq. quant with one scale per block of ``q_block`` consecutive rows of every (b, h) slice of
    x [B, H, L, d] (``q_block`` = 1: per token): the per-tensor quantizer applied to each block.
    Returns (int8 array, float32 scales [B, H, ceil(L / q_block)])."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    B, H, L, d = a.shape
    nblk = (L + q_block - 1) // q_block
    xq = np.zeros(a.shape, dtype=np.int8)
    scales = np.zeros((B, H, nblk), dtype=np.float32)
    for b in range(B):
        for h in range(H):
            for blk in range(nblk):
                r0, r1 = blk * q_block, min(L, (blk + 1) * q_block)
                part, sc = quantize(a[b:b + 1, h:h + 1, r0:r1], per_head=False)
                xq[b, h, r0:r1] = part[0, 0]
                scales[b, h, blk] = sc[0]
    return xq, scales


def index_softmax(logits, c_int_: int, *, lut_bits=5, clip=6.6, rows_per_matrix=0, causal=False):
    """IndexSoftmax on int32 logits [..., cols] (rows are everything before the last axis): uint8
    probabilities of the same shape.  ``causal`` with ``rows_per_matrix``: the attention path's mask
    on stacked [rows_per_matrix, cols] matrices."""
    lib = _load()
    a = np.ascontiguousarray(logits, dtype=np.int32)
    cols = a.shape[-1]
    rows = a.size // cols
    out = np.zeros(a.shape, dtype=np.uint8)
    rc = lib.intattn_oracle_index_softmax(rows, cols, _ptr(a), int(c_int_), lut_bits, clip, int(rows_per_matrix),
                                          int(bool(causal)), _ptr(out))
    if rc:
        raise ValueError(f"intattn_oracle_index_softmax rc={rc}")
    return out


def quantize(x, per_head: bool = False):
    """Eq. quant on a [B, H, L, d] tensor (fp32, or fp16 widened exactly): returns (int8 tensor,
    fp32 scales of shape [1] or [H])."""
    x = np.ascontiguousarray(np.asarray(x).astype(np.float32))
    if x.ndim != 4:
        raise ValueError("expected a [B, H, L, d] tensor")
    B, H, L, d = x.shape
    xq = np.empty(x.shape, dtype=np.int8)
    scales = np.empty(H if per_head else 1, dtype=np.float32)
    rc = _load().intattn_oracle_quantize(B, H, L, d, _ptr(x), int(per_head), _ptr(xq), _ptr(scales))
    if rc != 0:
        raise ValueError(f"intattn_oracle_quantize failed with {rc}")
    return xq, scales
