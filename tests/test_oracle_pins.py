"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests needs a GPU or the HIP library.  Each one checks the oracle against
something other than itself: a closed form evaluated independently, an invariant of the
definitions, a special case whose answer is known a priori, exact rational arithmetic
(``fractions``), or fp64 softmax attention within a stated bound.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import workloads as inputs

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
CLIP, BITS = 6.6, 5


def round_half_up(fr: Fraction) -> int:
    return math.floor(fr + Fraction(1, 2))


# ----------------------------------------------------------------------------- LUT
def test_lut_matches_paper_closed_form(oracle):
    """Sec. 3.1 Eq. lut_re + Sec. 3.2 Eq. lut16 at (b, c) = (5, 6.6): golden values written by
    tests/golden/make_lut_golden.py with 50-digit arithmetic."""
    with open(os.path.join(GOLDEN, "lut_b5_c6p6.txt")) as f:
        rows = [ln for ln in f if not ln.startswith("#")]
    golden = np.array([int(t) for t in rows[0].split()], dtype=np.uint8)
    lut = oracle.lut(5, 6.6)
    assert lut.dtype == np.uint8 and lut.size == 32  # 32 entries, 32 bytes (Sec. 4.3)
    np.testing.assert_array_equal(lut, golden)


@pytest.mark.parametrize("b,c", [(2, 5.5), (3, 6.6), (4, 6.6), (5, 5.5), (5, 7.7), (6, 6.6), (8, 7.0)])
def test_lut_against_exp_at_index_points(oracle, b, c):
    """LUT entries against exp at the paper's index points x_i = c*i/(2^b-1)."""
    lut = oracle.lut(b, c)
    n = 1 << b
    assert lut[0] == 255 and lut[n - 1] == 0
    assert np.all(np.diff(lut.astype(int)) <= 0)
    for i in range(n - 1):
        x = 255.0 * math.exp(-c * i / (n - 1))
        assert abs(int(lut[i]) - x) <= 0.5 + 1e-9


# ----------------------------------------------------------------------------- c_int
def test_c_int_closed_form(oracle):
    """Eq. clipping_thr: c_int = round(c*sqrt(d)/(s_Q*s_K)); hence |c_int*alpha - c| <= alpha/2."""
    rng = np.random.default_rng(11)
    for _ in range(200):
        sq = np.float32(rng.uniform(0.005, 0.3))
        sk = np.float32(rng.uniform(0.005, 0.3))
        d = int(rng.choice([16, 64, 128]))
        ci = oracle.c_int(CLIP, sq, sk, d)
        alpha = float(sq) * float(sk) / math.sqrt(d)
        assert abs(ci * alpha - CLIP) <= alpha / 2 * (1 + 1e-9)
    # exact-arithmetic instance: s_Q*s_K = 1/4, d = 64 -> c/alpha = 6.6*8*4 = 211.2 -> 211
    assert oracle.c_int(6.6, 0.5, 0.5, 64) == 211
    # tie rounds up: c/alpha = 2.5 -> 3
    assert oracle.c_int(2.5, 1.0, 1.0, 1) == 3
    # degenerate: threshold below one is raised to one
    assert oracle.c_int(6.6, 100.0, 100.0, 1) == 1


# ----------------------------------------------------------------------------- index map
@pytest.mark.parametrize("c_int", [1, 2, 3, 31, 62, 63, 100, 445, 1462, 6274])
def test_index_map_exact_rational(oracle, c_int):
    """idx = round(delta' * (2^b-1)/c_int) for every delta' in [0, c_int], against exact
    rational arithmetic; plus the invariants the definition implies."""
    prev = -1
    for dl in range(c_int + 1):
        got = oracle.index_map(dl, c_int, BITS)
        fr = Fraction(dl * 31, c_int)
        assert got == round_half_up(fr)
        assert abs(Fraction(got) - fr) <= Fraction(1, 2)
        assert got >= prev
        prev = got
    assert oracle.index_map(0, c_int, BITS) == 0
    assert oracle.index_map(c_int, c_int, BITS) == 31


def test_prob_exact_rational(oracle):
    """Eq. uint8-prob element-wise against exact rational arithmetic, including a tie."""
    lut = oracle.lut(5, 6.6)
    rng = np.random.default_rng(5)
    for _ in range(2000):
        e = int(lut[rng.integers(32)])
        s = int(rng.integers(max(e, 255), 255 * 64))
        assert oracle.prob(e, s) == round_half_up(Fraction(255 * e, s))
    assert oracle.prob(255, 510) == 128  # 127.5 rounds up
    assert oracle.prob(255, 255) == 255
    assert oracle.prob(0, 255) == 0


# ----------------------------------------------------------------------------- requant
def test_requant_default_scale_is_round_of_acc_over_255(oracle):
    """With s_O = s_V the multiplier encodes 1/255, and 255 is odd, so acc/255 never hits a
    tie: the fixed-point result must equal round(acc/255) for every accumulator in range."""
    m, sh = oracle.requant_params(0.037, 0.037)
    assert 2**30 <= m < 2**31 and 1 <= sh <= 62
    assert abs(m / 2.0**sh - 1.0 / 255.0) < 2.0**-38
    for acc in list(range(-40000, 40000, 7)) + [-(2**22), 2**22 - 1, 127 * 255, -127 * 255, 128 * 255]:
        got = (acc * m + (1 << (sh - 1))) >> sh  # python's >> floors
        assert got == round_half_up(Fraction(acc, 255))


def test_requant_general_scale_close_to_ratio(oracle):
    rng = np.random.default_rng(2)
    for _ in range(200):
        sv = np.float32(rng.uniform(0.001, 0.2))
        so = np.float32(rng.uniform(0.0001, 0.2))
        m, sh = oracle.requant_params(sv, so)
        r = float(sv) / (255.0 * float(so))
        assert 2**30 <= m < 2**31
        assert abs(m / 2.0**sh - r) <= r * 2.0**-30


# ----------------------------------------------------------------------------- helpers
def run(oracle, p, s_o=None, **kw):
    return oracle.forward(p.q, p.k, p.v, p.s_q, p.s_k, p.s_v, s_o, causal=p.causal,
                          per_head=p.per_head, **kw)


def python_reference_row(qrow, K, V, n_vis, c_int, lut, rq):
    """Exact-rational restatement of one row (cross-check of the C code's indexing and
    integer widths; the pins proper are the tests further down)."""
    a = [int(np.dot(qrow.astype(np.int64), K[j].astype(np.int64))) for j in range(n_vis)]
    m = max(a)
    e = [int(lut[round_half_up(Fraction(min(m - x, c_int) * 31, c_int))]) for x in a]
    s = sum(e)
    p = [round_half_up(Fraction(255 * x, s)) for x in e]
    acc = [sum(p[j] * int(V[j, c]) for j in range(n_vis)) for c in range(V.shape[1])]
    mlt, sh = rq
    out = [max(-127, min(127, (x * mlt + (1 << (sh - 1))) >> sh)) for x in acc]
    return m, s, p, acc, out


# ----------------------------------------------------------------------------- whole pipeline
@pytest.mark.parametrize("causal", [False, True])
def test_pipeline_against_rational_python(oracle, causal):
    p = inputs.random_problem(3, 1, 2, 1, 19, 8, causal)
    r = run(oracle, p, taps=True, want_prob=True)
    lut = oracle.lut()
    ci = oracle.c_int(CLIP, p.s_q[0], p.s_k[0], p.d)
    rq = oracle.requant_params(p.s_v[0], p.s_v[0])
    for h in range(p.Hq):
        for i in range(p.L):
            n_vis = i + 1 if causal else p.L
            m, s, pr, acc, out = python_reference_row(p.q[0, h, i], p.k[0, 0], p.v[0, 0], n_vis, ci, lut, rq)
            assert r["row_max"][0, h, i] == m and r["row_sum"][0, h, i] == s
            assert list(r["prob"][0, h, i, :n_vis]) == pr
            assert not r["prob"][0, h, i, n_vis:].any()
            assert list(r["acc"][0, h, i]) == acc
            assert list(r["out"][0, h, i]) == out


def test_lut_grid_rows_reproduce_exp_through_the_pipeline(oracle):
    """d = 1, logits placed exactly on the table's grid: with c_int = 31*t and key values
    chosen so that delta_j = t*i_j, the index map returns i_j exactly, so E_j must be
    round(255*exp(-c*i_j/31)) (computed here with math.exp) and the probabilities follow.
    A wrong sign of delta, a reversed table or an off-by-one gather fails this."""
    t = 4
    c_int = 31 * t
    s_q = np.float32(1.0)
    s_k = np.float32(CLIP / c_int)  # alpha = s_k -> c/alpha = c_int up to fp rounding
    assert oracle.c_int(CLIP, s_q, s_k, 1) == c_int
    steps = np.array([0, 1, 2, 5, 9, 17, 30, 31, 3, 0], dtype=np.int64)
    kvals = (124 - t * steps).astype(np.int8)  # q = 1 -> a_j = k_j, max = 124 at step 0
    L = steps.size
    q = np.ones((1, 1, L, 1), dtype=np.int8)
    k = kvals.reshape(1, 1, L, 1).copy()
    v = np.arange(1, L + 1, dtype=np.int8).reshape(1, 1, L, 1).copy()
    r = oracle.forward(q, k, v, [s_q], [s_k], [1.0], None, taps=True, want_prob=True)
    e = [0 if i == 31 else math.floor(255 * math.exp(-CLIP * i / 31) + 0.5) for i in steps]
    s = sum(e)
    assert r["row_max"][0, 0, 0] == 124
    assert r["row_sum"][0, 0, 0] == s
    pr = [math.floor(255 * x / s + 0.5) for x in e]
    assert list(r["prob"][0, 0, 0]) == pr
    acc = sum(pj * (j + 1) for j, pj in enumerate(pr))
    assert r["acc"][0, 0, 0, 0] == acc


def test_causal_first_row_and_single_key_copy_v(oracle):
    """One visible key: P = 255, and with s_O = s_V the output is V_hat[0] exactly."""
    p = inputs.random_problem(7, 2, 3, 3, 9, 16, True)
    r = run(oracle, p, taps=True)
    np.testing.assert_array_equal(r["out"][:, :, 0, :], p.v[:, :, 0, :])
    assert (r["row_sum"][:, :, 0] == 255).all()
    p1 = inputs.random_problem(8, 1, 2, 2, 1, 16, False)
    np.testing.assert_array_equal(run(oracle, p1)["out"], p1.v)


def test_dominant_key_gives_one_hot(oracle):
    """A key whose logit leads every other by at least c_int: every other key lands on the last
    table entry (zero), P is one-hot, out = V_hat[j*]."""
    rng = np.random.default_rng(21)
    L, d, jstar = 12, 16, 5
    q = np.full((1, 1, L, d), 100, dtype=np.int8)
    k = rng.integers(-3, 4, size=(1, 1, L, d)).astype(np.int8)
    k[0, 0, jstar] = 120
    v = rng.integers(-127, 128, size=(1, 1, L, d)).astype(np.int8)
    s = np.float32(0.5)  # c_int = round(6.6*4/0.25) = 106, gap >= 100*16*(120-3) >> 106
    r = oracle.forward(q, k, v, [s], [s], [0.1], None, taps=True, want_prob=True)
    assert oracle.c_int(CLIP, s, s, d) == 106
    assert (r["prob"][0, 0, :, jstar] == 255).all()
    assert r["prob"][0, 0].sum() == 255 * L
    np.testing.assert_array_equal(r["out"][0, 0], np.broadcast_to(v[0, 0, jstar], (L, d)))


@pytest.mark.parametrize("n", [1, 2, 3, 7, 100, 510, 511, 600])
def test_equal_logits_uniform_probabilities(oracle, n):
    """A zero query row makes all n logits equal: E = 255 each, P = round(255/n),
    acc = P * sum_j V_hat[j]; beyond n = 510 the row rounds to all-zero (a property of
    Eq. uint8-prob, not a defect)."""
    rng = np.random.default_rng(n)
    d = 8
    q = np.zeros((1, 1, n, d), dtype=np.int8)
    k = rng.integers(-127, 128, size=(1, 1, n, d)).astype(np.int8)
    v = rng.integers(-127, 128, size=(1, 1, n, d)).astype(np.int8)
    r = oracle.forward(q, k, v, [0.1], [0.1], [0.1], None, taps=True)
    pexp = math.floor(Fraction(255, n) + Fraction(1, 2))
    assert (r["row_sum"] == 255 * n).all()
    acc = pexp * v[0, 0].astype(np.int64).sum(axis=0)
    np.testing.assert_array_equal(r["acc"][0, 0, 0], acc)
    if n > 510:
        assert pexp == 0 and not r["out"].any()


def test_key_permutation_invariance(oracle):
    p = inputs.random_problem(13, 1, 2, 2, 37, 16, False)
    r0 = run(oracle, p)["out"]
    perm = np.random.default_rng(1).permutation(p.L)
    k2 = np.ascontiguousarray(p.k[:, :, perm])
    v2 = np.ascontiguousarray(p.v[:, :, perm])
    r1 = oracle.forward(p.q, k2, v2, p.s_q, p.s_k, p.s_v)["out"]
    np.testing.assert_array_equal(r0, r1)


def test_negating_q_and_k_changes_nothing(oracle):
    p = inputs.random_problem(14, 1, 2, 2, 23, 16, True)
    r0 = run(oracle, p, taps=True)
    r1 = oracle.forward(-p.q, -p.k, p.v, p.s_q, p.s_k, p.s_v, causal=True, taps=True)
    for key in ("out", "row_max", "row_sum", "acc"):
        np.testing.assert_array_equal(r0[key], r1[key])


def test_causal_row_equals_noncausal_prefix(oracle):
    """Row i under the causal mask is the non-causal problem over keys 0..i."""
    p = inputs.random_problem(15, 1, 1, 1, 21, 8, True)
    rc = run(oracle, p, taps=True)
    for i in (0, 4, 20):
        q = np.ascontiguousarray(p.q[:, :, : i + 1])
        k = np.ascontiguousarray(p.k[:, :, : i + 1])
        v = np.ascontiguousarray(p.v[:, :, : i + 1])
        rn = oracle.forward(q, k, v, p.s_q, p.s_k, p.s_v, taps=True)
        np.testing.assert_array_equal(rc["out"][0, 0, i], rn["out"][0, 0, i])
        assert rc["row_sum"][0, 0, i] == rn["row_sum"][0, 0, i]


def test_gqa_maps_query_head_to_kv_head(oracle):
    """Hq = 4, Hkv = 2: the result must equal plain multi-head attention with each KV head
    repeated for its group."""
    p = inputs.random_problem(16, 2, 4, 2, 17, 8, True)
    r0 = run(oracle, p)["out"]
    k_rep = np.ascontiguousarray(np.repeat(p.k, 2, axis=1))
    v_rep = np.ascontiguousarray(np.repeat(p.v, 2, axis=1))
    r1 = oracle.forward(p.q, k_rep, v_rep, p.s_q, p.s_k, p.s_v, causal=True)["out"]
    np.testing.assert_array_equal(r0, r1)


def test_per_head_scales_equal_per_tensor_runs_head_by_head(oracle):
    """Sec. 3.3 with one group per head: each head must behave as a per-tensor problem with
    that head's scales."""
    p = inputs.random_problem(17, 1, 4, 2, 15, 8, False, per_head=True)
    assert len(set(p.s_q.tolist())) > 1
    s_o = np.array([0.02, 0.03, 0.04, 0.05], dtype=np.float32)
    r = run(oracle, p, s_o)["out"]
    for h in range(4):
        kv = h // 2
        r1 = oracle.forward(np.ascontiguousarray(p.q[:, h:h + 1]), np.ascontiguousarray(p.k[:, kv:kv + 1]),
                            np.ascontiguousarray(p.v[:, kv:kv + 1]), [p.s_q[h]], [p.s_k[kv]], [p.s_v[kv]],
                            [s_o[h]])["out"]
        np.testing.assert_array_equal(r[:, h], r1[:, 0])


def test_probability_row_invariants(oracle):
    """Rows are non-negative, monotone in the logits, bounded per element by the exact
    quotient +-1/2, and sum to 255 within n_nonzero/2 (what 'within rounding' means for
    Eq. uint8-prob); the row sum equals the histogram-weighted table sum."""
    p = inputs.make_problem("c2_vit_b16", B=1, Hq=2, Hkv=2, L=197)
    r = run(oracle, p, taps=True, want_prob=True)
    lut = oracle.lut().astype(np.int64)
    ci = oracle.c_int(CLIP, p.s_q[0], p.s_k[0], p.d)
    a = np.einsum("hid,hjd->hij", p.q[0].astype(np.int64), p.k[0].astype(np.int64))
    for h in range(2):
        for i in range(0, p.L, 9):
            row, pr = a[h, i], r["prob"][0, h, i].astype(np.int64)
            assert row.max() == r["row_max"][0, h, i]
            dl = np.minimum(row.max() - row, ci)
            idx = (2 * 31 * dl + ci) // (2 * ci)
            hist = np.bincount(idx, minlength=32)
            s = int((hist * lut).sum())
            assert s == r["row_sum"][0, h, i] and 255 <= s <= 255 * p.L
            order = np.argsort(row, kind="stable")
            assert np.all(np.diff(pr[order]) >= 0)  # monotone in the logit
            assert pr.min() >= 0 and pr.max() <= 255
            e = lut[idx]
            assert np.all(np.abs(pr * 2 * s - 2 * 255 * e) <= s)  # |P - 255E/S| <= 1/2
            n_nz = int((e > 0).sum())
            assert abs(int(pr.sum()) - 255) <= n_nz / 2
            assert pr[row.argmax()] == (2 * 255 * 255 + s) // (2 * s)


def fp64_attention(p, s_o):
    g = p.Hq // p.Hkv
    out = np.zeros((p.B, p.Hq, p.L, p.d))
    prob = np.zeros((p.B, p.Hq, p.L, p.L))
    for b in range(p.B):
        for h in range(p.Hq):
            kv = h // g
            a = (p.q[b, h].astype(np.float64) * p.s_q[0]) @ (p.k[b, kv].astype(np.float64) * p.s_k[0]).T
            a /= math.sqrt(p.d)
            if p.causal:
                a = np.where(np.tril(np.ones((p.L, p.L), dtype=bool)), a, -np.inf)
            a -= a.max(axis=1, keepdims=True)
            w = np.exp(a)
            w /= w.sum(axis=1, keepdims=True)
            prob[b, h] = w
            out[b, h] = w @ (p.v[b, kv].astype(np.float64) * p.s_v[0]) / s_o
    return prob, out


@pytest.mark.parametrize("causal,spread", [(False, 1.0), (True, 1.0), (False, 2.5), (True, 2.5)])
def test_fidelity_against_fp64_softmax_attention(oracle, causal, spread):
    """Brute force on tiny inputs (L <= 32, d = 16): the integer pipeline against fp64
    softmax attention of the same dequantized INT8 inputs (Eq. attention_re).

    Bound used.  The table step is c/31, so E/255 is exp(-alpha*delta) up to a factor
    e^{+-c/62} (index rounding) and +-1/510 (table rounding); entries past the clip are
    dropped (each below exp(-c*61/62) < 0.0016).  Normalizing gives probabilities within
    a factor e^{+-c/31} of softmax, i.e. an L1 distance below e^{c/31} - 1 = 0.2373, plus
    n*(1/510 + 0.0016 + 1/510) for table rounding, the tail cut and Eq. uint8-prob's own
    rounding: ||P_hat/255 - p||_1 <= 0.2373 + 0.0056*n.  The output then differs from the
    fp64 output (in units of s_O = s_V) by at most 127 * that distance + 1/2.
    Typical values are 5-10x smaller; a looser sanity check on the mean is added."""
    p = inputs.random_problem(31, 1, 2, 2, 32, 16, causal, spread=spread)
    r = run(oracle, p, want_prob=True)
    ref_p, ref_o = fp64_attention(p, float(p.s_v[0]))
    l1 = np.abs(r["prob"].astype(np.float64) / 255.0 - ref_p).sum(axis=-1)
    n = np.arange(1, p.L + 1)[None, None, :] if causal else p.L
    assert np.all(l1 <= 0.2373 + 0.0056 * n)
    assert l1.mean() <= 0.10
    err = np.abs(r["out"].astype(np.float64) - ref_o)
    assert np.all(err.max(axis=-1) <= 127 * (0.2373 + 0.0056 * n) + 0.5)
    assert err.mean() <= 2.0


def test_rows_entry_matches_forward(oracle):
    p = inputs.random_problem(41, 2, 4, 2, 50, 16, True, per_head=True)
    full = run(oracle, p, taps=True)
    sel = [0, 7, 49]
    r = oracle.rows(p.q, p.k, p.v, p.s_q, p.s_k, p.s_v, None, b=1, hq=3, rows=sel, causal=True, per_head=True)
    np.testing.assert_array_equal(r["out"], full["out"][1, 3, sel])
    np.testing.assert_array_equal(r["acc"], full["acc"][1, 3, sel])
    np.testing.assert_array_equal(r["row_max"], full["row_max"][1, 3, sel])
    np.testing.assert_array_equal(r["row_sum"], full["row_sum"][1, 3, sel])


def test_threaded_fanout_matches_single_thread(oracle):
    p = inputs.random_problem(42, 2, 4, 4, 33, 16, False)
    a = run(oracle, p, threads=1)["out"]
    b = run(oracle, p, threads=4)["out"]
    np.testing.assert_array_equal(a, b)


def test_output_saturates_symmetrically(oracle):
    """Eq. quant's range is [-127, 127]; a small s_O must saturate there, never at -128."""
    L, d = 4, 8
    q = np.zeros((1, 1, L, d), dtype=np.int8)
    k = np.zeros((1, 1, L, d), dtype=np.int8)
    v = np.empty((1, 1, L, d), dtype=np.int8)
    v[..., ::2], v[..., 1::2] = -127, 127
    r = oracle.forward(q, k, v, [0.1], [0.1], [0.1], [0.01])["out"]
    assert (r[..., ::2] == -127).all() and (r[..., 1::2] == 127).all()


# ------------------------------------------------------------------ dynamic quantizer (Sec. 2.1, Eq. quant)

def test_quantizer_grid_points_come_back_exactly(oracle):
    """A tensor whose values are integers k in [-127, 127] times a power of two has
    s = 2^e exactly (max|x| = 127 * 2^e) and must quantize to exactly those integers."""
    rng = np.random.default_rng(50)
    k = rng.integers(-127, 128, size=(2, 3, 17, 8)).astype(np.int32)
    k[0, 0, 0, 0] = 127
    for e in (-9, 0, 5):
        x = (k.astype(np.float32) * np.float32(2.0 ** e))
        xq, s = oracle.quantize(x)
        assert s.shape == (1,) and s[0] == np.float32(2.0 ** e)
        np.testing.assert_array_equal(xq.astype(np.int32), k)


def test_quantizer_scale_is_one_fp32_division_and_max_maps_to_127(oracle):
    rng = np.random.default_rng(51)
    x = rng.standard_normal((1, 4, 33, 16)).astype(np.float32) * np.float32(3.7)
    xq, s = oracle.quantize(x)
    amax = np.abs(x).max()
    assert s[0] == np.float32(amax) / np.float32(127.0)
    i = np.unravel_index(np.abs(x).argmax(), x.shape)
    assert abs(int(xq[i])) == 127 and np.sign(xq[i]) == np.sign(x[i])
    assert xq.min() >= -127  # symmetric range: -128 is never produced
    # reconstruction error at most half a step (plus the rounding of the fp32 quotient)
    err = np.abs(xq.astype(np.float64) * float(s[0]) - x.astype(np.float64))
    assert err.max() <= 0.5 * float(s[0]) * (1 + 1e-6)


def test_quantizer_ties_go_to_even(oracle):
    """With max|x| = 127 the scale is exactly 1, so x/s = x: halves are exact ties."""
    x = np.zeros((1, 1, 1, 8), dtype=np.float32)
    x[0, 0, 0] = [127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5]
    xq, s = oracle.quantize(x)
    assert s[0] == np.float32(1.0)
    np.testing.assert_array_equal(xq[0, 0, 0], [127, 0, 2, 2, 0, -2, -2, 126])


def test_quantizer_exact_rational_restatement(oracle):
    """Element by element with exact rationals: the fp32 quotient x/s is the fp32 value nearest
    to the rational x/s (checked through fp64, which holds the quotient of two fp32 values to
    well below half an fp32 ulp except at exact fp32 ties, which the fp64 quotient reproduces),
    then nearest integer, ties to even."""
    rng = np.random.default_rng(52)
    x = (rng.standard_t(4, size=(1, 2, 9, 8)) * 0.3).astype(np.float32)
    xq, s = oracle.quantize(x, per_head=True)
    for h in range(2):
        sh = np.float32(np.abs(x[:, h]).max()) / np.float32(127.0)
        assert s[h] == sh
        for xv, qv in zip(x[0, h].ravel(), xq[0, h].ravel()):
            y = np.float32(np.float64(xv) / np.float64(sh))  # correctly rounded fp32 quotient
            fr = Fraction(float(y))
            fl = fr.numerator // fr.denominator
            rem = fr - fl
            want = fl + (1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1) else 0)
            assert int(qv) == max(-127, min(127, want))


def test_quantizer_zero_tensor_and_per_head_groups(oracle):
    z, s = oracle.quantize(np.zeros((1, 2, 3, 8), dtype=np.float32), per_head=True)
    assert not z.any() and (s == np.float32(1e-12) / np.float32(127.0)).all()
    rng = np.random.default_rng(53)
    x = rng.standard_normal((3, 4, 11, 8)).astype(np.float32)
    x[:, 2] *= 50.0  # one loud head must not change the others' scales
    xq, s = oracle.quantize(x, per_head=True)
    for h in range(4):
        one, s1 = oracle.quantize(np.ascontiguousarray(x[:, h:h + 1]))
        assert s1[0] == s[h]
        np.testing.assert_array_equal(one[:, 0], xq[:, h])
    # per tensor: the loud head sets the only scale
    _, st = oracle.quantize(x)
    assert st[0] == s[2] == s.max()


def test_workload_generator_quantizes_as_eq_quant(oracle):
    """A test OF THE GENERATOR, not a pin of the oracle: the seeded workload generator turns its
    fp32 draws into INT8 with numpy (max, divide, rint, clip).  The oracle's quantizer is pinned
    by the exact-rational and grid-point tests above; here it serves as the reference that the
    generator's recipe must agree with, so that the INT8 workloads are what Eq. quant yields."""
    rng = np.random.default_rng(54)
    x = rng.standard_normal((2, 3, 40, 16), dtype=np.float32)
    for per_head in (False, True):
        a, sa = oracle.quantize(x, per_head)
        b, sb = inputs.quantize(x, per_head)
        np.testing.assert_array_equal(a, b)
        np.testing.assert_array_equal(sa, sb)


# ----------------------------------------------------------------------------- rectangular shapes (Lq != Lk)
# The paper states the method for square self-attention only; a chunk of queries or one decoded
# token against a longer key/value sequence is this build's reading: nothing changes per row, and
# a causal mask is aligned to the end (the last query sees every key).  Pinned to the square case.
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("lq", [1, 5, 22])
def test_rectangular_is_the_tail_of_the_square_problem(oracle, causal, lq):
    """Queries = the last lq rows of a square problem over the same keys: identical rows."""
    p = inputs.random_problem(51, 2, 4, 2, 37, 8, causal, per_head=True)
    sq = run(oracle, p, taps=True, want_prob=True)
    q_tail = np.ascontiguousarray(p.q[:, :, p.L - lq:])
    r = oracle.forward(q_tail, p.k, p.v, p.s_q, p.s_k, p.s_v, causal=causal, per_head=True, taps=True, want_prob=True)
    for key in ("out", "row_max", "row_sum", "acc", "prob"):
        np.testing.assert_array_equal(r[key], sq[key][:, :, p.L - lq:])


def test_rectangular_against_rational_python(oracle):
    """More queries than keys (no mask) and fewer (mask aligned to the end), row by row in exact rationals."""
    lut = oracle.lut()
    for (lq, lk, causal) in ((9, 4, False), (3, 11, True), (1, 6, True)):
        base = inputs.random_problem(60 + lq, 1, 1, 1, max(lq, lk), 8, causal)
        q = np.ascontiguousarray(base.q[:, :, :lq])
        k = np.ascontiguousarray(base.k[:, :, :lk])
        v = np.ascontiguousarray(base.v[:, :, :lk])
        r = oracle.forward(q, k, v, base.s_q, base.s_k, base.s_v, causal=causal, taps=True, want_prob=True)
        ci = oracle.c_int(CLIP, base.s_q[0], base.s_k[0], 8)
        rq = oracle.requant_params(base.s_v[0], base.s_v[0])
        assert r["prob"].shape == (1, 1, lq, lk)
        for i in range(lq):
            n_vis = i + (lk - lq) + 1 if causal else lk
            m, s, pr, acc, out = python_reference_row(q[0, 0, i], k[0, 0], v[0, 0], n_vis, ci, lut, rq)
            assert r["row_max"][0, 0, i] == m and r["row_sum"][0, 0, i] == s
            assert list(r["prob"][0, 0, i, :n_vis]) == pr and not r["prob"][0, 0, i, n_vis:].any()
            assert list(r["acc"][0, 0, i]) == acc and list(r["out"][0, 0, i]) == out


def test_rectangular_rows_entry_and_bad_shapes(oracle):
    p = inputs.random_problem(53, 1, 2, 1, 40, 8, True)
    q = np.ascontiguousarray(p.q[:, :, 25:])
    full = oracle.forward(q, p.k, p.v, p.s_q, p.s_k, p.s_v, causal=True, taps=True)
    some = oracle.rows(q, p.k, p.v, p.s_q, p.s_k, p.s_v, b=0, hq=1, rows=[0, 7, 14], causal=True)
    np.testing.assert_array_equal(some["out"], full["out"][0, 1, [0, 7, 14]])
    np.testing.assert_array_equal(some["row_sum"], full["row_sum"][0, 1, [0, 7, 14]])
    # a causal row without a visible key has no softmax: more queries than keys is refused
    with pytest.raises(ValueError):
        oracle.forward(p.q, np.ascontiguousarray(p.k[:, :, :30]), np.ascontiguousarray(p.v[:, :, :30]),
                       p.s_q, p.s_k, p.s_v, causal=True)


# ----------------------------------------------------------------------------- IndexSoftmax as an operator
@pytest.mark.parametrize("causal", [False, True])
def test_index_softmax_operator_equals_the_pipeline_tap(oracle, causal):
    """Fed with Q.K^T computed by numpy, the operator returns the probabilities the (pinned)
    attention pipeline produces, square and rectangular, with and without mask."""
    for (lq, lk) in ((23, 23), (7, 31)):
        base = inputs.random_problem(70 + lq, 2, 2, 1, max(lq, lk), 8, causal)
        q = np.ascontiguousarray(base.q[:, :, :lq])
        k = np.ascontiguousarray(base.k[:, :, :lk])
        v = np.ascontiguousarray(base.v[:, :, :lk])
        want = oracle.forward(q, k, v, base.s_q, base.s_k, base.s_v, causal=causal, want_prob=True)["prob"]
        logits = np.einsum("bhid,bjd->bhij", q.astype(np.int64), k[:, 0].astype(np.int64)).astype(np.int32)
        ci = oracle.c_int(CLIP, base.s_q[0], base.s_k[0], 8)
        got = oracle.index_softmax(logits, ci, rows_per_matrix=lq, causal=causal)
        np.testing.assert_array_equal(got, want)


def test_index_softmax_operator_exact_rational_and_invariants(oracle):
    rng = np.random.default_rng(5)
    lut = oracle.lut()
    a = rng.integers(-40000, 40000, size=(6, 50)).astype(np.int32)
    a[1] = 7                       # equal logits: uniform
    a[2, 3] = 2**31 - 1            # extreme values: the distance needs more than 32 bits
    a[2, 4] = -2**31
    for ci in (1, 37, 5203, 2**30):
        p = oracle.index_softmax(a, ci)
        for r in range(a.shape[0]):
            row = [int(x) for x in a[r]]
            m = max(row)
            e = [int(lut[round_half_up(Fraction(min(m - x, ci) * 31, ci))]) for x in row]
            s = sum(e)
            assert list(p[r]) == [round_half_up(Fraction(255 * x, s)) for x in e]
        assert (p[1] == round_half_up(Fraction(255, 50))).all()
        assert p[2, 3] == 255 or ci == 2**30  # the dominant logit takes everything unless nothing is clipped away
    with pytest.raises(ValueError):
        oracle.index_softmax(a, 0)
    with pytest.raises(ValueError):
        oracle.index_softmax(a, 5, rows_per_matrix=4, causal=True)  # 6 rows are not stacked 4-row matrices


# ----------------------------------------------------------------------------- finer groups over query rows
def test_row_groups_reduce_to_per_head_and_follow_each_groups_scale(oracle):
    """Sec. 3.3 with groups = blocks of query rows: equal group scales give the per-head result;
    with distinct scales every row follows the exact-rational pipeline with ITS group's c_int."""
    p = inputs.random_problem(81, 2, 4, 2, 29, 8, True, per_head=True)
    qb = 4
    nblk = (p.L + qb - 1) // qb
    same = np.broadcast_to(p.s_q[None, :, None], (2, 4, nblk)).copy()
    a = oracle.forward_row_groups(p.q, p.k, p.v, same, p.s_k, p.s_v, q_block=qb, causal=True, taps=True)
    b = oracle.forward(p.q, p.k, p.v, p.s_q, p.s_k, p.s_v, causal=True, per_head=True, taps=True)
    for key in ("out", "row_max", "row_sum", "acc"):
        np.testing.assert_array_equal(a[key], b[key])
    rng = np.random.default_rng(2)
    s_q = (same * rng.uniform(0.2, 3.0, size=same.shape)).astype(np.float32)
    r = oracle.forward_row_groups(p.q, p.k, p.v, s_q, p.s_k, p.s_v, q_block=qb, causal=True, taps=True)
    lut = oracle.lut()
    for (bb, h, i) in ((0, 0, 0), (0, 1, 7), (1, 3, 28), (1, 2, 16)):
        kv = h // 2
        ci = oracle.c_int(CLIP, s_q[bb, h, i // qb], p.s_k[kv], 8)
        rq = oracle.requant_params(p.s_v[kv], p.s_v[kv])
        m, s, pr, acc, out = python_reference_row(p.q[bb, h, i], p.k[bb, kv], p.v[bb, kv], i + 1, ci, lut, rq)
        assert r["row_max"][bb, h, i] == m and r["row_sum"][bb, h, i] == s
        assert list(r["acc"][bb, h, i]) == acc and list(r["out"][bb, h, i]) == out
    assert (r["row_sum"] != b["row_sum"]).any()  # the group scales do change the result


def test_row_group_quantizer_is_the_per_tensor_quantizer_per_block(oracle):
    rng = np.random.default_rng(9)
    x = (rng.standard_normal((2, 2, 11, 8)) * rng.uniform(0.1, 9.0, size=(2, 2, 11, 1))).astype(np.float32)
    xq, sc = oracle.quantize_row_groups(x, 1)
    assert sc.shape == (2, 2, 11)
    amax = np.abs(x).max(axis=-1)
    np.testing.assert_array_equal(sc, (amax / np.float32(127.0)).astype(np.float32))
    assert (np.abs(xq).max(axis=-1) == 127).all()  # every token's largest element maps to +-127
    xq4, sc4 = oracle.quantize_row_groups(x, 4)
    assert sc4.shape == (2, 2, 3)
    np.testing.assert_array_equal(sc4[:, :, 2], (np.abs(x[:, :, 8:]).max(axis=(-1, -2)) / np.float32(127.0)).astype(np.float32))
    whole, s1 = oracle.quantize_row_groups(x[:1, :1], 11)
    ref, s0 = oracle.quantize(x[:1, :1])
    np.testing.assert_array_equal(whole, ref)
    assert s1[0, 0, 0] == s0[0]


# ----------------------------------------------------------------------------- finer groups over the key axis
def grouped_problem(seed, B, Hq, Hkv, L, Lk, d, q_block, k_block, spread_blocks=(0.2, 5.0)):
    """fp32 Q, K, V whose key blocks (and query blocks) differ in range, quantized per block by the
    oracle's own per-block quantizer (pinned above): int8 tensors and the scale arrays."""
    import oracle as orc

    rng = np.random.default_rng(seed)
    nqb, nkb = -(-L // q_block), -(-Lk // k_block)
    q = rng.standard_normal((B, Hq, L, d)).astype(np.float32)
    k = rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32)
    v = rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32)
    lo, hi = spread_blocks
    fq = np.exp(rng.uniform(math.log(lo), math.log(hi), size=(B, Hq, nqb))).astype(np.float32)
    fk = np.exp(rng.uniform(math.log(lo), math.log(hi), size=(B, Hkv, nkb))).astype(np.float32)
    q *= np.repeat(fq, q_block, axis=2)[:, :, :L, None]
    k *= np.repeat(fk, k_block, axis=2)[:, :, :Lk, None]
    q8, sq = orc.quantize_row_groups(q, q_block)
    k8, sk = orc.quantize_row_groups(k, k_block)
    sv = np.zeros(Hkv, dtype=np.float32)
    v8 = np.zeros((B, Hkv, Lk, d), dtype=np.int8)
    for h in range(Hkv):  # V per KV head, shared over the batch
        part, s = orc.quantize(v[:, h:h + 1], per_head=False)
        v8[:, h:h + 1] = part
        sv[h] = s[0]
    return q8, k8, v8, sq, sk, sv


def test_key_groups_with_equal_scales_are_the_per_head_pipeline(oracle):
    """Sec. 3.3 must collapse to Sec. 3.1-3.2 when every group carries the same scale: every byte
    and tap of the per-head oracle, for blocks of keys and for one scale per key; the real row
    maximum is then alpha times the integer one."""
    p = inputs.random_problem(91, 2, 4, 2, 37, 16, True, per_head=True, spread=1.5)
    ref = oracle.forward(p.q, p.k, p.v, p.s_q, p.s_k, p.s_v, causal=True, per_head=True, taps=True, want_prob=True)
    for qb, kb in ((5, 8), (1, 1), (37, 37), (64, 3)):
        nqb, nkb = -(-p.L // qb), -(-p.L // kb)
        sq = np.broadcast_to(p.s_q[None, :, None], (2, 4, nqb)).copy()
        sk = np.broadcast_to(p.s_k[None, :, None], (2, 2, nkb)).copy()
        r = oracle.forward_groups(p.q, p.k, p.v, sq, sk, p.s_v, q_block=qb, k_block=kb, causal=True, taps=True,
                                  want_prob=True)
        for key in ("out", "row_sum", "acc", "prob"):
            np.testing.assert_array_equal(r[key], ref[key], err_msg=f"{key} q_block {qb} k_block {kb}")
        alpha = (p.s_q.astype(np.float64)[:, None] * np.repeat(p.s_k.astype(np.float64), 2)[:, None]) / math.sqrt(16)
        np.testing.assert_array_equal(r["row_max_real"], alpha[None] * ref["row_max"])


@pytest.mark.parametrize("causal,kb", [(False, 4), (True, 4), (True, 1), (False, 32)])
def test_key_groups_are_softmax_of_the_dequantized_logits(oracle, causal, kb):
    """Brute force: with key blocks (and query blocks) whose scales differ by up to 25x, the
    probabilities stay within the per-tensor pipeline's distance of fp64 softmax of the DEQUANTIZED
    logits alpha^(g) A_hat -- plus a factor e^{alpha} for rounding the row maximum into each group's
    integer units.  Two plausible wrong readings (row maximum over raw integers across groups; each
    group normalized to its own maximum) are evaluated beside it and must break the same bound, so
    the bound does discriminate."""
    B, Hq, Hkv, L, d, qb = 1, 2, 1, 32, 16, 8
    q8, k8, v8, sq, sk, sv = grouped_problem(5 + kb, B, Hq, Hkv, L, L, d, qb, kb)
    r = oracle.forward_groups(q8, k8, v8, sq, sk, sv, q_block=qb, k_block=kb, causal=causal, want_prob=True, taps=True)
    lut = oracle.lut().astype(np.int64)
    worst_right, worst_intmax, worst_local = 0.0, 0.0, 0.0
    for h in range(Hq):
        alpha = (np.repeat(sq[0, h].astype(np.float64), qb)[:L, None] *
                 np.repeat(sk[0, 0].astype(np.float64), kb)[None, :L]) / math.sqrt(d)
        a_int = q8[0, h].astype(np.int64) @ k8[0, 0].astype(np.int64).T
        a = alpha * a_int
        vis = np.tril(np.ones((L, L), dtype=bool)) if causal else np.ones((L, L), dtype=bool)
        a_m = np.where(vis, a, -np.inf)
        w = np.exp(a_m - a_m.max(axis=1, keepdims=True))
        w /= w.sum(axis=1, keepdims=True)
        n = vis.sum(axis=1)
        bound = (np.exp(CLIP / 31 + alpha.max()) - 1.0) + 0.0056 * n
        l1 = np.abs(r["prob"][0, h].astype(np.float64) / 255.0 - w).sum(axis=1)
        assert np.all(l1 <= bound), (h, float((l1 - bound).max()))
        np.testing.assert_allclose(r["row_max_real"][0, h], a_m.max(axis=1), rtol=1e-15)
        worst_right = max(worst_right, float((l1 / bound).max()))
        # wrong reading 1: Delta from the maximum of the raw integers of the whole row
        c_int = np.maximum(1, np.floor(CLIP / alpha + 0.5)).astype(np.int64)
        for name in ("intmax", "local"):
            if name == "intmax":
                m = np.where(vis, a_int, -10**9).max(axis=1, keepdims=True) * np.ones_like(a_int)
            else:  # wrong reading 2: every key block measured from its own maximum
                m = np.zeros_like(a_int)
                for g0 in range(0, L, kb):
                    blk = np.where(vis[:, g0:g0 + kb], a_int[:, g0:g0 + kb], -10**9).max(axis=1, keepdims=True)
                    m[:, g0:g0 + kb] = blk
            dl = np.clip(m - a_int, 0, c_int)
            idx = (2 * 31 * dl + c_int) // (2 * c_int)
            e = np.where(vis, lut[idx], 0)
            pw = e / e.sum(axis=1, keepdims=True)
            bad = float((np.abs(pw - w).sum(axis=1) / bound).max())
            if name == "intmax":
                worst_intmax = max(worst_intmax, bad)
            else:
                worst_local = max(worst_local, bad)
    assert worst_right <= 1.0
    if kb < L:  # with a single key block both wrong readings coincide with the right one
        assert worst_intmax > 1.5 and worst_local > 1.5, (worst_intmax, worst_local)


def test_key_groups_follow_each_logits_own_scale_exactly(oracle):
    """Dyadic scales and c = 6.5 make every quantity of Sec. 3.3 exact (alpha^(g) a power of two,
    c_int^(g) = 6.5 / alpha^(g) an integer): doubling the INT8 values of one key block while
    halving its scale leaves every dequantized logit, and therefore every probability and output
    byte, unchanged -- and the rows must equal an exact-rational evaluation of the reading."""
    rng = np.random.default_rng(17)
    B, Hq, Hkv, L, d, qb, kb = 1, 2, 2, 24, 16, 6, 4
    q8 = rng.integers(-127, 128, (B, Hq, L, d), dtype=np.int8)
    k8 = rng.integers(-60, 61, (B, Hkv, L, d), dtype=np.int8)
    v8 = rng.integers(-127, 128, (B, Hkv, L, d), dtype=np.int8)
    sq = (2.0 ** -rng.integers(3, 6, (B, Hq, L // qb))).astype(np.float32)
    sk = (2.0 ** -rng.integers(2, 6, (B, Hkv, L // kb))).astype(np.float32)
    sv = np.asarray([0.01, 0.02], dtype=np.float32)
    kw = dict(q_block=qb, k_block=kb, causal=True, clip=6.5, taps=True, want_prob=True)
    base = oracle.forward_groups(q8, k8, v8, sq, sk, sv, **kw)
    k2, sk2 = k8.copy(), sk.copy()
    for (h, g) in ((0, 1), (0, 4), (1, 0), (1, 5)):
        k2[0, h, g * kb:(g + 1) * kb] *= 2
        sk2[0, h, g] /= 2
    other = oracle.forward_groups(q8, k2, v8, sq, sk2, sv, **kw)
    # V is untouched and P must be: the accumulators and bytes agree, although the integers differ
    for key in ("prob", "row_sum", "acc", "out", "row_max_real"):
        np.testing.assert_array_equal(base[key], other[key], err_msg=key)
    assert (k2 != k8).any()
    # exact rationals (every float here is a dyadic rational, so Fraction(float) is exact and no
    # floating-point rounding enters anywhere)
    lut = oracle.lut(5, 6.5)
    for (h, i) in ((0, 0), (0, 13), (1, 23), (1, 7)):
        n_vis = i + 1
        al = [Fraction(float(sq[0, h, i // qb])) * Fraction(float(sk2[0, h, j // kb])) / 4 for j in range(n_vis)]
        a = [int(np.dot(q8[0, h, i].astype(np.int64), k2[0, h, j].astype(np.int64))) for j in range(n_vis)]
        M = max(x * y for x, y in zip(al, a))
        e = []
        for j in range(n_vis):
            ci = round_half_up(Fraction(13, 2) / al[j])
            dl = min(max(round_half_up(M / al[j]) - a[j], 0), ci)
            e.append(int(lut[round_half_up(Fraction(dl * 31, ci))]))
        s = sum(e)
        pr = [round_half_up(Fraction(255 * x, s)) for x in e]
        assert other["row_sum"][0, h, i] == s
        assert list(other["prob"][0, h, i, :n_vis]) == pr and not other["prob"][0, h, i, n_vis:].any()
        assert float(M) == other["row_max_real"][0, h, i]
        acc = [sum(pr[j] * int(v8[0, h, j, c]) for j in range(n_vis)) for c in range(d)]
        assert list(other["acc"][0, h, i]) == acc
        mlt, sh = oracle.requant_params(sv[h], sv[h])
        assert list(other["out"][0, h, i]) == [max(-127, min(127, (x * mlt + (1 << (sh - 1))) >> sh)) for x in acc]


def test_key_groups_reject_unusable_scales(oracle):
    q8, k8, v8, sq, sk, sv = grouped_problem(3, 1, 2, 1, 8, 8, 8, 4, 2)
    for bad in (0.0, -1.0, np.inf, np.nan):
        s2 = sk.copy()
        s2[0, 0, 1] = bad
        with pytest.raises(ValueError):
            oracle.forward_groups(q8, k8, v8, sq, s2, sv, q_block=4, k_block=2)
    with pytest.raises(ValueError):
        oracle.forward_groups(q8, k8, v8, sq, sk, sv, q_block=4, k_block=0)
