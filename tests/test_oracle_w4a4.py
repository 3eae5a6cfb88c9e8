"""Pins for the W4A4 half of the CPU oracle (signed 4-bit weights per output
channel, unsigned 4-bit activations per tensor, exact integer conv-as-GEMM,
requantisation): invariants, closed forms, textbook special cases, brute force."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import qail_oracle as O
from paper_2412_01034_amd import synth


def _tiny(B=1, H=4, W=4, Cin=8, Cout=3, KH=3, KW=3, stride=1, pad=1, name="t"):
    return synth.ConvShape(name, B, H, W, Cin, Cout, KH, KW, stride, pad)


def _codes(shape, seed):
    a = synth.random_codes((shape.B, shape.H, shape.W, shape.Cin), 0, 15, seed).astype(np.uint8)
    w = synth.random_codes((shape.Cout, shape.KH, shape.KW, shape.Cin), -8, 7, seed + 1)
    return a, w


def _acc(shape, a, w, **kw):
    return O.w4a4_conv_acc(O.pack_nibbles(a), O.pack_nibbles(w.reshape(shape.Cout, -1)),
                           shape.B, shape.H, shape.W, shape.Cin, shape.Cout, shape.KH, shape.KW,
                           shape.stride, shape.pad, **kw)


# ---- quantisers -------------------------------------------------------------

def test_weight_codes_range_error_bound_and_extremes():
    sh = _tiny(Cin=16, Cout=12)
    w = synth.conv_weight(sh, 3)
    q, s = O.quantize_w4_sym_channel(w)
    assert q.dtype == np.int8 and q.min() >= -7 and q.max() <= 7      # absmax/7 never emits -8
    flat = w.reshape(12, -1).astype(np.float64)
    err = np.abs(flat - q.reshape(12, -1) * s.astype(np.float64)[:, None])
    assert np.all(err <= s.astype(np.float64)[:, None] * (0.5 + 2.0 ** -20))
    assert np.all(np.abs(q.reshape(12, -1)).max(axis=1) == 7)          # the absmax element maps to +-7
    # per-tensor quantisation = every channel sharing one absmax
    w2 = w.copy()
    w2[:, 0, 0, 0] = np.abs(w).max()
    _, s2 = O.quantize_w4_sym_channel(w2)
    assert np.all(s2 == s2[0])
    # exact cases, ties to even, sign symmetry
    wq = np.array([[7, -7, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5]], np.float32)
    q3, s3 = O.quantize_w4_sym_channel(wq)
    assert float(s3[0]) == 1.0 and q3[0].tolist() == [7, -7, 0, 2, 2, 0, -2, -2]
    q4, s4 = O.quantize_w4_sym_channel(np.zeros((2, 8), np.float32))
    assert np.all(q4 == 0) and s4.tolist() == [1.0, 1.0]


def test_activation_codes_range_bound_and_skew():
    sh = _tiny(B=2, H=16, W=16, Cin=64)
    a = synth.conv_activation(sh, 5)
    s_a = O.act_scale_u4(a)
    q = O.quantize_act_u4(a, s_a)
    assert q.dtype == np.uint8 and q.max() == 15 and q.min() == 0
    err = np.abs(a.astype(np.float64) - q * float(s_a))
    assert np.all(err <= float(s_a) * (0.5 + 2.0 ** -20))
    assert (q == 0).mean() > 0.5                       # ReLU input: at least half the codes are 0
    # exact cases with s_a = 1: range, clamp below 0 and above 15, ties to even
    v = np.array([0, 15, 0.5, 1.5, 2.5, -3.0, 14.5, 99.0], np.float32)
    assert O.quantize_act_u4(v, 1.0).tolist() == [0, 15, 0, 2, 2, 0, 14, 15]
    assert float(O.act_scale_u4(np.array([0, 30, 7.5], np.float32))) == 2.0
    assert float(O.act_scale_u4(np.zeros(4, np.float32))) == 1.0


# ---- integer conv-as-GEMM ---------------------------------------------------

def _brute(shape, a, w):
    OH, OW = shape.OH, shape.OW
    out = np.zeros((shape.B * OH * OW, shape.Cout), dtype=np.int64)
    for b in range(shape.B):
        for oh in range(OH):
            for ow in range(OW):
                for n in range(shape.Cout):
                    t = 0
                    for kh in range(shape.KH):
                        for kw in range(shape.KW):
                            ih = oh * shape.stride + kh - shape.pad
                            iw = ow * shape.stride + kw - shape.pad
                            if 0 <= ih < shape.H and 0 <= iw < shape.W:
                                for c in range(shape.Cin):
                                    t += int(a[b, ih, iw, c]) * int(w[n, kh, kw, c])
                    out[(b * OH + oh) * OW + ow, n] = t
    return out


@pytest.mark.parametrize("shape", [
    _tiny(),
    _tiny(B=2, H=5, W=6, Cin=8, Cout=4, stride=2, pad=1),
    _tiny(B=1, H=6, W=6, Cin=16, Cout=2, KH=1, KW=1, stride=2, pad=0),
    _tiny(B=1, H=7, W=5, Cin=8, Cout=2, KH=3, KW=3, stride=2, pad=1),
])
def test_conv_matches_nested_loop_definition(shape):
    a, w = _codes(shape, 7)
    ref = _brute(shape, a, w)
    assert np.array_equal(_acc(shape, a, w), ref)
    assert np.array_equal(_acc(shape, a, w, use_blas=True), ref)


@pytest.mark.parametrize("shape", [
    _tiny(),
    _tiny(B=2, H=5, W=6, Cin=8, Cout=4, stride=2, pad=1),
    _tiny(B=3, H=6, W=6, Cin=16, Cout=2, KH=1, KW=1, stride=2, pad=0),
    _tiny(B=2, H=7, W=5, Cin=8, Cout=2, KH=3, KW=3, stride=2, pad=1),
])
def test_selected_rows_match_nested_loop_definition(shape):
    # the row-sampling form used on tensors too large to recompute whole: every row, in a shuffled
    # order with repeats, against the brute-force definition (not against the oracle's own full form)
    a, w = _codes(shape, 27)
    ref = _brute(shape, a, w)
    rows = np.random.default_rng(5).permutation(np.r_[np.arange(shape.M), [0, shape.M - 1]])
    got = O.w4a4_conv_acc_rows(O.pack_nibbles(a), O.pack_nibbles(w.reshape(shape.Cout, -1)),
                               shape.B, shape.H, shape.W, shape.Cin, shape.Cout, shape.KH, shape.KW,
                               shape.stride, shape.pad, rows)
    assert np.array_equal(got, ref[rows])
    cols = O.im2col_rows_nhwc(a.astype(np.int64), shape.KH, shape.KW, shape.stride, shape.pad, rows)
    assert np.array_equal(cols, O.im2col_nhwc(a.astype(np.int64), shape.KH, shape.KW, shape.stride, shape.pad)[rows])
    assert O.w4a4_conv_acc_rows(O.pack_nibbles(a), O.pack_nibbles(w.reshape(shape.Cout, -1)),
                                shape.B, shape.H, shape.W, shape.Cin, shape.Cout, shape.KH, shape.KW,
                                shape.stride, shape.pad, np.zeros(0, np.int64)).shape == (0, shape.Cout)


def test_1x1_conv_is_plain_gemm():
    sh = _tiny(B=2, H=3, W=5, Cin=24, Cout=7, KH=1, KW=1, stride=1, pad=0)
    a, w = _codes(sh, 9)
    ref = a.reshape(-1, 24).astype(np.int64) @ w.reshape(7, 24).astype(np.int64).T
    assert np.array_equal(_acc(sh, a, w), ref)


def test_centre_tap_identity_and_shifted_tap():
    sh = _tiny(B=1, H=5, W=6, Cin=8, Cout=8)
    a, _ = _codes(sh, 13)
    w = np.zeros((8, 3, 3, 8), np.int8)
    for c in range(8):
        w[c, 1, 1, c] = 1
    assert np.array_equal(_acc(sh, a, w).reshape(1, 5, 6, 8), a.astype(np.int32))
    # tap (kh=0, kw=2): out[oh, ow] = in[oh-1, ow+1], zero outside the image
    w = np.zeros((8, 3, 3, 8), np.int8)
    for c in range(8):
        w[c, 0, 2, c] = -3
    exp = np.zeros((1, 5, 6, 8), np.int64)
    exp[:, 1:, :-1, :] = a[:, :-1, 1:, :]
    assert np.array_equal(_acc(sh, a, w).reshape(1, 5, 6, 8), -3 * exp)


def test_extreme_codes_closed_form_and_bound():
    for K_ch in (8, 64, 512):
        sh = _tiny(B=1, H=3, W=3, Cin=K_ch, Cout=2, KH=3, KW=3, stride=1, pad=1)
        a = np.full((1, 3, 3, K_ch), 15, np.uint8)
        w = np.empty((2, 3, 3, K_ch), np.int8)
        w[0], w[1] = -8, 7
        acc = _acc(sh, a, w).reshape(3, 3, 2)
        # the centre pixel sees all 9 taps; a corner sees 4
        assert acc[1, 1].tolist() == [-120 * 9 * K_ch, 105 * 9 * K_ch]
        assert acc[0, 0].tolist() == [-120 * 4 * K_ch, 105 * 4 * K_ch]
    assert 8 * 15 * 4608 == 552960 < 2 ** 31


def test_im2col_column_order_is_kh_kw_c():
    sh = _tiny(B=1, H=3, W=3, Cin=8, Cout=1)
    a = np.arange(72, dtype=np.int64).reshape(1, 3, 3, 8)
    cols = O.im2col_nhwc(a, 3, 3, 1, 1)
    assert cols.shape == (9, 72)
    centre = cols[4].reshape(3, 3, 8)
    assert np.array_equal(centre, a[0])
    corner = cols[0].reshape(3, 3, 8)
    assert np.all(corner[0] == 0) and np.all(corner[:, 0] == 0) and np.array_equal(corner[1:, 1:], a[0, :2, :2])


# ---- requantisation ---------------------------------------------------------

def test_requant_closed_form():
    acc = np.array([[3, -4], [0, 100]], np.int32)
    scale = np.array([0.5, 0.25], np.float32)
    bias = np.array([1.0, -2.0], np.float32)
    assert O.requant(acc, scale, bias).tolist() == [[2.5, -3.0], [1.0, 23.0]]
    s = O.requant_scale(np.float32(0.1), np.array([0.3, 2.0], np.float32))
    assert s.dtype == np.float32
    for i, sw in enumerate((0.3, 2.0)):
        exact = Fraction(float(np.float32(0.1))) * Fraction(float(np.float32(sw)))
        assert abs(Fraction(float(s[i])) - exact) <= abs(exact) * Fraction(1, 2 ** 24)


def _round_to_f32(v: Fraction) -> np.float32:
    """Nearest float32 of an exact rational, ties to even, by comparing exact distances."""
    c = np.float32(float(v))
    cands = [np.nextafter(c, np.float32(-np.inf)), c, np.nextafter(c, np.float32(np.inf))]
    best = min(cands, key=lambda f: (abs(Fraction(float(f)) - v), int(np.float32(f).view(np.uint32)) & 1))
    return np.float32(best)


def test_requant_f32_is_one_correctly_rounded_fma():
    # hand cases: exact results, and a sum that needs the single rounding
    acc = np.array([[3, -4], [0, 100]], np.int32)
    scale = np.array([0.5, 0.25], np.float32)
    bias = np.array([1.0, -2.0], np.float32)
    got = O.requant_f32(acc, scale, bias)
    assert got.dtype == np.float32 and got.tolist() == [[2.5, -3.0], [1.0, 23.0]]
    # 1 + 2^-24 + 2^-47 lies just above the midpoint of 1 and 1 + 2^-23: a multiply rounded on its
    # own (2^-24 exactly) followed by an add would tie to even (1.0); the single rounding gives 1 + 2^-23
    sc = np.array([np.float32(2.0 ** -24) * (np.float32(1) + np.float32(2.0 ** -23))], np.float32)
    assert O.requant_f32(np.array([[1]], np.int32), sc, np.array([1.0], np.float32))[0, 0] == np.float32(1 + 2.0 ** -23)
    # a float64 sum that lands on a float32 midpoint although the true sum is below it:
    # p = (2^23 + 1)(1 - 2^-23) = 2^23 - 2^-23, bias = 2^47 + 2^24 (odd significand); the midpoint above
    # the bias is 2^47 + 2^24 + 2^23, float64 resolves 2^-5 there, so the float64 sum is that midpoint and
    # ties-to-even on it would round up, while the true sum rounds down to the bias
    acc2 = np.array([[2 ** 23 + 1]], np.int32)
    sc2 = np.array([1 - 2.0 ** -23], np.float32)
    b2 = np.array([2.0 ** 47 + 2.0 ** 24], np.float32)
    exact = Fraction(2 ** 23 + 1) * Fraction(float(sc2[0])) + Fraction(float(b2[0]))
    assert exact == Fraction(2 ** 47 + 2 ** 24 + 2 ** 23) - Fraction(1, 2 ** 23)
    naive = (acc2.astype(np.float64) * sc2.astype(np.float64) + b2.astype(np.float64)).astype(np.float32)
    assert naive[0, 0] == np.float32(2.0 ** 47 + 2.0 ** 25)                  # the double rounding this guards against
    assert O.requant_f32(acc2, sc2, b2)[0, 0] == b2[0] == _round_to_f32(exact)
    # mirrored: true sum just above the midpoint below an even neighbour
    assert O.requant_f32(-acc2, sc2, -b2)[0, 0] == -b2[0]
    # random operands, cancelling and not, against exact rational arithmetic
    rng = np.random.default_rng(77)
    acc = rng.integers(-552960, 552961, size=(40, 6)).astype(np.int32)
    scale = (rng.random(6) * 1e-3 + 1e-6).astype(np.float32)
    bias = np.array([0.0, 0.3, -0.3, 1e-7, -250.0, 3e4], np.float32)
    got = O.requant_f32(acc, scale, bias)
    for m in range(40):
        for n in range(6):
            v = Fraction(int(acc[m, n])) * Fraction(float(scale[n])) + Fraction(float(bias[n]))
            assert got[m, n] == _round_to_f32(v), (m, n)
    # and it is the float64 definition rounded: never further than half a float32 step from it
    y64 = O.requant(acc, scale, bias)
    assert np.all(np.abs(got.astype(np.float64) - y64) <= np.abs(y64) * 2.0 ** -24 + 1e-45)


def test_end_to_end_quantised_conv_tracks_real_conv():
    # the integer path reproduces the real-valued convolution up to the
    # quantisation step sizes (a dropped scale or transposed operand would not)
    sh = _tiny(B=1, H=8, W=8, Cin=32, Cout=16)
    w = synth.conv_weight(sh, 17)
    a = synth.conv_activation(sh, 18)
    bias = synth.conv_bias(sh, 19)
    qw, s_w = O.quantize_w4_sym_channel(w)
    s_a = O.act_scale_u4(a)
    qa = O.quantize_act_u4(a, s_a)
    acc = _acc(sh, qa, qw)
    y = O.requant(acc, O.requant_scale(s_a, s_w), bias)
    real = O.im2col_nhwc(a.astype(np.float64), 3, 3, 1, 1) @ w.reshape(16, -1).astype(np.float64).T + bias
    rel = np.linalg.norm(y - real) / np.linalg.norm(real)
    assert rel < 0.2
    deq = (O.im2col_nhwc(qa.astype(np.float64) * float(s_a), 3, 3, 1, 1)
           @ (qw.reshape(16, -1) * s_w.astype(np.float64)[:, None]).T + bias)
    assert np.allclose(y, deq, rtol=1e-6, atol=1e-6)


# ------------------------------------------------------------------ fused output epilogue

def _golden_fused():
    rows = []
    path = os.path.join(os.path.dirname(__file__), "golden", "w4a4_fused_epilogue.txt")
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            v = line.split()
            rows.append((int(v[0]), float(v[1]), float(v[2]), int(v[3]), float(v[4]), float(v[5]), int(v[6])))
    return rows


def test_fused_epilogue_hand_worked_cases():
    rows = _golden_fused()
    assert len(rows) >= 10
    for acc, sc, bi, rc, rs, so, want in rows:
        a = np.array([[acc]], np.int32)
        if rc < 0:
            got = O.fused_requant_u4(a, [sc], [bi], so)
        else:
            got = O.fused_requant_u4(a, [sc], [bi], so, res_codes=np.array([[rc]], np.uint8), res_scale=rs)
        assert int(got[0, 0]) == want, (acc, sc, bi, rc, rs, so, int(got[0, 0]), want)


def _fl32(x64):
    return np.asarray(x64, np.float64).astype(np.float32)


def test_fused_epilogue_is_a_chain_of_single_float32_operations():
    # +, * and / of float32 operands carried out in float64 (53 >= 2*24+2 bits) and then
    # rounded to float32 equal the correctly rounded float32 operation, so this re-derivation,
    # which never lets numpy do float32 arithmetic, pins every step: a fused multiply-add,
    # a float64 accumulation or a reciprocal multiply would differ on some element.
    rng = np.random.default_rng(5)
    M, N = 257, 64
    acc = rng.integers(-40000, 40000, size=(M, N)).astype(np.int32)
    scale = (rng.random(N).astype(np.float32) * 1e-3 + 1e-4).astype(np.float32)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float32)
    rc = rng.integers(0, 16, size=(M, N)).astype(np.uint8)
    rs, so = np.float32(0.2371), np.float32(0.3113)
    rf = rng.standard_normal((M, N)).astype(np.float32)
    for kind in ("none", "codes", "f32"):
        t = _fl32(acc.astype(np.float64) * scale.astype(np.float64)[None, :])
        t = _fl32(t.astype(np.float64) + bias.astype(np.float64)[None, :])
        if kind == "codes":
            r = _fl32(np.float64(rs) * rc.astype(np.float64))
            t = _fl32(t.astype(np.float64) + r.astype(np.float64))
            got = O.fused_requant_u4(acc, scale, bias, so, res_codes=rc, res_scale=rs)
        elif kind == "f32":
            t = _fl32(t.astype(np.float64) + rf.astype(np.float64))
            got = O.fused_requant_u4(acc, scale, bias, so, res_f32=rf)
        else:
            got = O.fused_requant_u4(acc, scale, bias, so)
        t = np.maximum(t, np.float32(0))
        q = np.clip(np.rint(_fl32(t.astype(np.float64) / np.float64(so)).astype(np.float64)), 0, 15).astype(np.uint8)
        assert np.array_equal(got, q), kind
        assert got.min() == 0 and got.max() == 15          # the data exercises both clamps


def test_fused_epilogue_agrees_with_the_unfused_chain_away_from_ties():
    # requant (float64, pinned above) -> + shortcut -> ReLU -> quantize_act_u4 (pinned above)
    rng = np.random.default_rng(6)
    M, N = 300, 32
    acc = rng.integers(-3000, 3000, size=(M, N)).astype(np.int32)
    scale = (rng.random(N) * 2e-3 + 5e-4).astype(np.float32)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float32)
    rc = rng.integers(0, 16, size=(M, N)).astype(np.uint8)
    rs, so = np.float32(0.11), np.float32(0.27)
    y64 = O.requant(acc, scale, bias) + np.float64(rs) * rc
    y64 = np.maximum(y64, 0.0)
    frac = y64 / np.float64(so)
    away = np.abs(frac - np.floor(frac) - 0.5) > 1e-4
    ref = O.quantize_act_u4(y64.astype(np.float32), so)
    got = O.fused_requant_u4(acc, scale, bias, so, res_codes=rc, res_scale=rs)
    assert away.mean() > 0.99
    assert np.array_equal(got[away], ref[away])


def test_fused_epilogue_invariants_and_identity_case():
    rng = np.random.default_rng(7)
    N = 16
    scale = (rng.random(N) * 1e-2 + 1e-3).astype(np.float32)
    bias = (rng.standard_normal(N) * 0.05).astype(np.float32)
    accs = np.arange(-500, 2500, dtype=np.int32)[:, None].repeat(N, 1)
    q = O.fused_requant_u4(accs, scale, bias, np.float32(0.4))
    assert q.min() >= 0 and q.max() <= 15
    assert np.all(np.diff(q.astype(int), axis=0) >= 0)              # monotone in acc for scale > 0
    y = O.requant(accs, scale, bias)
    assert np.all(q[y <= 0] == 0)                                   # ReLU
    # scale == s_out, no bias: the code is the accumulator itself, clamped
    a = np.arange(-3, 20, dtype=np.int32)[:, None]
    q = O.fused_requant_u4(a, [0.37], [0.0], 0.37)
    assert np.array_equal(q[:, 0], np.clip(a[:, 0], 0, 15))
    # a shortcut given as codes or as the float32 tensor they stand for is the same thing
    rc = rng.integers(0, 16, size=accs.shape).astype(np.uint8)
    rs = np.float32(0.3)
    qa = O.fused_requant_u4(accs, scale, bias, 0.4, res_codes=rc, res_scale=rs)
    qb = O.fused_requant_u4(accs, scale, bias, 0.4, res_f32=(rs * rc.astype(np.float32)))
    assert np.array_equal(qa, qb)


def test_product_first_quotient_claim_used_by_the_fused_epilogue():
    """The fused epilogue's kernel may take u = t * fl(1 / s) instead of t / s when that provably
    gives the same code: the claim is that, outside a band of 2^-17 around the half-integers (where
    the kernel divides after all), rint(u) and rint(t / s) agree after the clamp at 15, for every
    t >= 0 and every step s whose reciprocal is a normal number.  Checked here in float32 on a few
    million pairs, half of them placed within 40 ulps of a tie, against the last line of the
    oracle's fused epilogue, q = clamp(rint(t / s), 0, 15), written out per pair (the oracle's own
    function takes one step per tensor)."""
    rng = np.random.default_rng(2024)
    n = 1_500_000
    F = np.float32
    s = np.concatenate([
        np.exp(rng.uniform(np.log(1e-30), np.log(1e30), n)).astype(F),          # any magnitude
        rng.uniform(0.01, 2.0, n).astype(F),                                     # the realistic range
    ])
    k = rng.integers(0, 17, size=2 * n).astype(F)
    near_tie = (k + F(0.5)) * s                                                  # t / s lands near k + 0.5
    ulps = rng.integers(-40, 41, size=2 * n)
    near_tie = (near_tie.view(np.int32) + ulps.astype(np.int32)).view(F)
    anywhere = (rng.uniform(0, 17, 2 * n).astype(F) * s).astype(F)
    for t in (near_tie, anywhere):
        t = np.abs(t)
        ok = np.isfinite(t) & np.isfinite(s) & (s > 0)
        t, sv = t[ok], s[ok]
        inv = (F(1) / sv).astype(F)
        normal = np.isfinite(inv) & (np.abs(inv) >= np.finfo(F).tiny)
        t, sv, inv = t[normal], sv[normal], inv[normal]
        with np.errstate(over="ignore", invalid="ignore"):
            u = (t * inv).astype(F)
            q = np.rint(u)
            doubt = ~(np.abs(np.abs(u - q) - F(0.5)) >= F(2.0 ** -17))          # NaN counts as doubt
            quick = np.minimum(q, F(15))
            exact = np.minimum(np.rint((t / sv).astype(F)), F(15))
        sure = ~doubt & np.isfinite(u)
        assert sure.mean() > 0.3                      # the band is narrow: most pairs take the product
        assert np.array_equal(quick[sure], exact[sure])
