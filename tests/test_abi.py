"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
its structs have the layout the binding assumes, its argument checks reject bad calls
without touching a GPU, and its host-side parameter derivation (which shares no code with
the oracle) agrees with the oracle's."""
import ctypes
import os
import re
import subprocess
import tempfile

import numpy as np
import pytest

from paper_2511_21513_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "intattn.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_21513_amd import build

        build.build()
    return binding.load()


def declared_symbols():
    text = open(HEADER).read()
    return re.findall(r"INTATTN_API\s+[\w\s\*]+?\b(intattn_\w+)\s*\(", text)


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert len(names) >= 8
    assert set(names) == set(binding.SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layout_matches_header(lib):
    """Compile a probe against the real header with gcc and compare sizeof/offsetof with the
    ctypes mirrors."""
    fields_cfg = [f[0] for f in binding.Config._fields_]
    fields_arg = [f[0] for f in binding.Args._fields_]
    fields_qnt = [f[0] for f in binding.QuantArgs._fields_]
    fields_smx = [f[0] for f in binding.SoftmaxArgs._fields_]
    src = ['#include <stdio.h>', '#include <stddef.h>', f'#include "{HEADER}"', "int main(void){"]
    src.append('printf("%zu\\n", sizeof(intattn_config));')
    src += [f'printf("%zu\\n", offsetof(intattn_config, {f}));' for f in fields_cfg]
    src.append('printf("%zu\\n", sizeof(intattn_args));')
    src += [f'printf("%zu\\n", offsetof(intattn_args, {f}));' for f in fields_arg]
    src.append('printf("%zu\\n", sizeof(intattn_quant_args));')
    src += [f'printf("%zu\\n", offsetof(intattn_quant_args, {f}));' for f in fields_qnt]
    src.append('printf("%zu\\n", sizeof(intattn_softmax_args));')
    src += [f'printf("%zu\\n", offsetof(intattn_softmax_args, {f}));' for f in fields_smx]
    src.append("return 0;}")
    with tempfile.TemporaryDirectory() as td:
        c = os.path.join(td, "probe.c")
        open(c, "w").write("\n".join(src))
        exe = os.path.join(td, "probe")
        subprocess.run(["gcc", "-std=c11", "-o", exe, c], check=True)
        vals = [int(x) for x in subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()]
    want = [ctypes.sizeof(binding.Config)] + [getattr(binding.Config, f).offset for f in fields_cfg]
    want += [ctypes.sizeof(binding.Args)] + [getattr(binding.Args, f).offset for f in fields_arg]
    want += [ctypes.sizeof(binding.QuantArgs)] + [getattr(binding.QuantArgs, f).offset for f in fields_qnt]
    want += [ctypes.sizeof(binding.SoftmaxArgs)] + [getattr(binding.SoftmaxArgs, f).offset for f in fields_smx]
    assert vals == want


def test_create_rejects_bad_config(lib):
    ctx = ctypes.c_void_p()
    assert lib.intattn_create(None, None) == binding.ERR_INVALID_ARG
    for cfg in (binding.Config(-1, 0, 6.6, 0, 0), binding.Config(-1, 7, 6.6, 0, 0)):
        assert lib.intattn_create(ctypes.byref(ctx), ctypes.byref(cfg)) == binding.ERR_UNSUPPORTED
    for cfg in (binding.Config(-1, 5, 0.0, 0, 0), binding.Config(-1, 5, float("nan"), 0, 0),
                binding.Config(-1, 5, 6.6, 0, 7), binding.Config(-5, 5, 6.6, 0, 0),
                binding.Config(-1, 5, 6.6, 11, 0), binding.Config(-1, 5, 6.6, -1, 0)):  # unknown kernel variants
        assert lib.intattn_create(ctypes.byref(ctx), ctypes.byref(cfg)) == binding.ERR_INVALID_ARG
        assert lib.intattn_last_error(None)
    lib.intattn_destroy(None)  # allowed


@pytest.fixture()
def host_ctx(lib):
    ia = binding.IntAttn(device=-1)
    yield ia
    ia.close()


def test_host_only_context_lut_and_params_agree_with_oracle(host_ctx, oracle):
    np.testing.assert_array_equal(host_ctx.lut(), oracle.lut(5, 6.6))
    rng = np.random.default_rng(0)
    for _ in range(300):
        sq, sk = np.float32(rng.uniform(0.002, 0.5)), np.float32(rng.uniform(0.002, 0.5))
        sv, so = np.float32(rng.uniform(0.002, 0.5)), np.float32(rng.uniform(0.0005, 0.5))
        d = int(rng.choice([64, 128]))
        c, m, sh = host_ctx.derive_params(sq, sk, sv, so, d)
        assert c == oracle.c_int(6.6, sq, sk, d)
        assert (m, sh) == oracle.requant_params(sv, so)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 6])
def test_other_table_sizes_agree_with_oracle(lib, oracle, bits):
    for clip in (5.5, 6.6, 7.7):
        ia = binding.IntAttn(device=-1, lut_bits=bits, clip=clip)
        assert ia.lut().size == 1 << bits
        np.testing.assert_array_equal(ia.lut(), oracle.lut(bits, clip))
        ia.close()


def test_table_sizes_beyond_six_bits_are_rejected(lib):
    for bits in (0, 7, 8):
        with pytest.raises(binding.IntAttnError):
            binding.IntAttn(device=-1, lut_bits=bits)


def apply_index_map(mode, mul, add, sh, x):
    x = x.astype(np.uint64)
    if mode in (1, 6):
        return (x * np.uint64(mul) + np.uint64(add)) >> np.uint64(sh)
    if mode == 3:
        r = np.array([mul], dtype=np.uint32).view(np.float32)[0]
        # fp32 fma emulated exactly: the product of two fp32 values and 0.5 fit fp64 without rounding
        y = (x.astype(np.float32).astype(np.float64) * np.float64(r) + 0.5).astype(np.float32)
        return np.trunc(y).astype(np.uint64)
    return (((x << np.uint64(sh)) + np.uint64(add)) * np.uint64(mul)) >> np.uint64(32)


@pytest.mark.parametrize("mode", [1, 2, 3])
def test_index_map_constants_are_exact(host_ctx, oracle, mode):
    """The multiply-shift the kernels use instead of a division must equal the exact rounded
    quotient for every clipped distance; checked exhaustively for a spread of thresholds, and
    spot-checked against the oracle's own index map."""
    rng = np.random.default_rng(mode)
    cs = [1, 2, 3, 30, 31, 32, 61, 62, 63, 445, 1462, 5203, 6274, 8191, 8192, 28794, 55064, 100000]
    cs += [int(x) for x in rng.integers(1, 9000, 30)] + [int(x) for x in rng.integers(9000, 130000, 10)]
    n_fast = 0
    for c in cs:
        got_mode, mul, add, sh = host_ctx.derive_index_map(c, mode)
        if got_mode == 0:
            continue
        assert got_mode == mode
        n_fast += 1
        if mode == 1:
            assert mul < 2**23 and c * mul + add < 2**31
        elif mode == 2:
            assert mul < 2**23 and (c << sh) + add < 2**23
        x = np.arange(c + 1, dtype=np.uint64)
        want = (2 * 31 * x + c) // (2 * c)
        np.testing.assert_array_equal(apply_index_map(mode, mul, add, sh, x), want)
        for xi in (0, c // 3, c):
            assert int(want[xi]) == oracle.index_map(int(xi), c, 5)
    if mode == 3:
        assert n_fast == len(cs)  # the fp32 scheme covers every threshold of the list
    else:
        assert n_fast >= 35
    # far beyond the schemes' precision the library must say so (mode 0), never return wrong constants
    for c in (10**6, 2**24 + 1, 2**30):
        got_mode, mul, add, sh = host_ctx.derive_index_map(c, mode)
        if got_mode:
            x = np.unique(np.concatenate([np.arange(0, 70001), rng.integers(0, c + 1, 50000)])).astype(np.uint64)
            np.testing.assert_array_equal(apply_index_map(got_mode, mul, add, sh, x), (2 * 31 * x + c) // (2 * c))


@pytest.mark.parametrize("bits", [2, 5, 6])
def test_top_byte_index_map_and_wider_tables(lib, oracle, bits):
    """Scheme 6 (the index is the top byte of a 24-bit multiply-add) for 2^bits-entry tables, and
    schemes 1 and 2 for the 64-entry table: exhaustively equal to the exact rounded quotient over
    [0, c_int] wherever the library reports constants, and within the 24-bit operand range."""
    ia = binding.IntAttn(device=-1, lut_bits=bits)
    top = (1 << bits) - 1
    rng = np.random.default_rng(bits)
    cs = [1, 2, 3, 2 * top - 1, 2 * top, 2 * top + 1, 126, 127, 128, 445, 1462, 5203, 6274, 8191, 8192, 28794, 55064]
    cs += [int(x) for x in rng.integers(1, 9000, 30)] + [int(x) for x in rng.integers(9000, 130000, 10)]
    found = {1: 0, 2: 0, 6: 0}
    for mode in (6, 1, 2):
        for c in cs:
            got_mode, mul, add, sh = ia.derive_index_map(c, mode)
            if got_mode == 0:
                continue
            assert got_mode == mode
            found[mode] += 1
            if mode == 6:
                assert sh == 24 and 0 < mul < 2**23 and c * mul + add < 2**31
            x = np.arange(c + 1, dtype=np.uint64)
            want = (2 * top * x + c) // (2 * c)
            np.testing.assert_array_equal(apply_index_map(mode, mul, add, sh, x), want)
            for xi in (0, c // 3, c):
                assert int(want[xi]) == oracle.index_map(int(xi), c, bits)
    assert found[6] >= 30 and found[1] >= 30, found
    ia.close()


def test_fp64_index_map_is_exact_for_every_threshold(host_ctx):
    """Scheme 0, the one without a search: trunc(fma(x, r, 0.5)) in IEEE double with r the double
    after 31 / c_int.  The fma is emulated in exact rationals and rounded once; checked on both
    sides of every index step (ties included: c_int even makes x = c_int / 2 one), at the ends of
    the range and at random points, for thresholds up to the cap of 2^30."""
    from fractions import Fraction

    rng = np.random.default_rng(64)
    cs = [1, 2, 3, 31, 62, 63, 5203, 55064, 390001, 10**6, 2**24 - 1, 2**24, 2**24 + 1, 31 * 2**20, 62 * 2**22,
          2**30 - 1, 2**30]
    cs += [int(c) for c in rng.integers(1, 2**30, 40)] + [2 * int(c) for c in rng.integers(1, 2**29, 20)]
    for c in cs:
        got_mode, lo, hi, sh = host_ctx.derive_index_map(c, 0)
        assert got_mode == 0 and sh == 0
        r = float(np.array([lo | (hi << 32)], dtype=np.uint64).view(np.float64)[0])
        assert r == np.nextafter(31.0 / c, np.inf)
        xs = {0, c, c // 2, (c + 1) // 2}
        for k in range(1, 32):  # first x with index >= k is ceil((2k - 1) c / 62)
            t = -((-(2 * k - 1) * c) // 62)
            xs.update(x for x in (t - 1, t, t + 1) if 0 <= x <= c)
        xs.update(int(x) for x in rng.integers(0, c + 1, 200))
        for x in xs:
            y = float(Fraction(x) * Fraction(r) + Fraction(1, 2))  # one rounding to nearest, as the fma does
            assert int(y) == (62 * x + c) // (2 * c), (c, x)


def test_forward_rejects_bad_arguments_without_a_gpu(host_ctx, lib):
    buf = np.zeros(1 << 14, dtype=np.int8)
    base = buf.ctypes.data
    base += (-base) % 16
    s = np.asarray([0.05], dtype=np.float32)

    def mk(**kw):
        a = binding.Args()
        a.B, a.Hq, a.Hkv, a.L, a.d, a.causal = 1, 2, 1, 8, 64, 0
        a.q, a.k, a.v, a.out = base, base + 2048, base + 4096, base + 8192
        for name in ("q_stride", "k_stride", "v_stride", "out_stride"):
            setattr(a, name, (ctypes.c_int64 * 3)(1024, 512, 64))
        a.scale_mode = 0
        a.scale_q = a.scale_k = a.scale_v = s.ctypes.data
        for k_, v_ in kw.items():
            setattr(a, k_, v_)
        return a

    def call(a):
        return lib.intattn_forward(host_ctx._ctx, ctypes.byref(a), None)

    assert call(mk()) == binding.ERR_INVALID_ARG and "host-only" in host_ctx.last_error()
    assert call(mk(d=96)) == binding.ERR_UNSUPPORTED
    for bad in (dict(L=0), dict(Hq=3, Hkv=2), dict(L=200000), dict(causal=2), dict(scale_mode=3), dict(q=None),
                dict(Lkv=-1), dict(Lkv=200000), dict(Lkv=4, causal=1), dict(scale_mode=2), dict(scale_mode=4), dict(k_block=1), dict(scale_mode=3, q_block=1),
                dict(scale_k=None), dict(out=base), dict(k=base + 2049),
                dict(v_stride=(ctypes.c_int64 * 3)(1024, 512, 60)), dict(q_stride=(ctypes.c_int64 * 3)(1024, 512, 32))):
        assert call(mk(**bad)) == binding.ERR_INVALID_ARG, bad
        assert host_ctx.last_error()
    assert lib.intattn_forward(None, ctypes.byref(mk()), None) == binding.ERR_INVALID_ARG
    assert lib.intattn_forward(host_ctx._ctx, None, None) == binding.ERR_INVALID_ARG
    zero = np.asarray([0.0], dtype=np.float32)
    # scale checks come after the host-only rejection on this context, so only the struct checks are reachable here
    assert call(mk(scale_q=zero.ctypes.data)) == binding.ERR_INVALID_ARG


def test_quantize_rejects_bad_arguments_without_a_gpu(host_ctx, lib):
    a = binding.QuantArgs()
    a.B, a.H, a.L, a.d, a.dtype, a.scale_mode = 1, 2, 16, 64, 1, 0
    a.src, a.dst, a.scales = 0x1000, 0x2000, 0x3000
    for i, st in enumerate((2 * 16 * 128, 16 * 128, 128)):
        a.src_stride[i] = st
        a.dst_stride[i] = st // 2
    ctx = host_ctx._ctx
    # a host-only context has no device to run on; everything else is refused before that matters
    assert lib.intattn_quantize(ctx, None, None) == binding.ERR_INVALID_ARG
    assert lib.intattn_quantize(ctx, ctypes.byref(a), None) == binding.ERR_UNSUPPORTED
    assert lib.intattn_quantize(None, ctypes.byref(a), None) == binding.ERR_INVALID_ARG


def test_dynamic_forward_needs_a_device(host_ctx, lib):
    """The device-scale entry validates like the plain forward and refuses a host-only context;
    the status word of a context that never ran it reads 0."""
    a = binding.Args()
    assert lib.intattn_forward_dynamic(host_ctx._ctx, None, None) == binding.ERR_INVALID_ARG
    assert lib.intattn_forward_dynamic(host_ctx._ctx, ctypes.byref(a), None) == binding.ERR_INVALID_ARG
    assert host_ctx.dynamic_status() == 0
    assert lib.intattn_dynamic_status(host_ctx._ctx, None) == binding.ERR_INVALID_ARG


def test_index_softmax_rejects_bad_arguments_without_a_gpu(host_ctx, lib):
    a = binding.SoftmaxArgs()
    assert lib.intattn_index_softmax(host_ctx._ctx, None, None) == binding.ERR_INVALID_ARG
    assert lib.intattn_index_softmax(host_ctx._ctx, ctypes.byref(a), None) == binding.ERR_UNSUPPORTED  # host-only context
