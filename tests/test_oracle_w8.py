"""Pins of the 8-bit oracle functions (no GPU)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import qail_oracle as O
from paper_2412_01034_amd import synth


def test_byte_packing_round_trip_and_known_word():
    codes = np.array([[1, -1, 127, -128, 0, 5, -5, 64]], np.int8)
    words = O.pack_bytes(codes)
    assert words.dtype == np.uint32 and words.shape == (1, 2)
    assert int(words[0, 0]) == 0x807FFF01 and int(words[0, 1]) == 0x40FB0500
    assert np.array_equal(O.unpack_bytes_s8(words, 8), codes)
    rng = np.random.default_rng(1)
    w = rng.integers(0, 2 ** 32, size=(7, 5), dtype=np.uint64).astype(np.uint32)
    assert np.array_equal(O.pack_bytes(O.unpack_bytes_s8(w, 20)), w)


def test_w8_channel_quantiser_invariants_and_torch():
    rng = np.random.default_rng(2)
    w = rng.standard_normal((9, 3, 3, 16)).astype(np.float32)
    w[4] = 0
    q, s = O.quantize_w8_sym_channel(w)
    assert q.dtype == np.int8 and np.abs(q.astype(int)).max() == 127 and s[4] == 1 and not q[4].any()
    err = np.abs(w.reshape(9, -1) - q.reshape(9, -1).astype(np.float64) * s.astype(np.float64)[:, None])
    assert np.all(err <= s.astype(np.float64)[:, None] * (0.5 + 2.0 ** -20))
    # each channel's largest magnitude maps to +-127 exactly
    for n in range(9):
        if n != 4:
            assert np.abs(q[n].astype(int)).max() == 127
    # library cross-check at power-of-two scales (there a reciprocal multiply equals the division)
    import torch
    w2 = (rng.integers(-127, 128, size=(6, 32)) * 0.25).astype(np.float32)
    w2[:, 0] = 127 * 0.25
    q2, s2 = O.quantize_w8_sym_channel(w2)
    assert np.all(s2 == 0.25)
    tq = torch.quantize_per_channel(torch.from_numpy(w2), torch.from_numpy(s2.astype(np.float64)),
                                    torch.zeros(6, dtype=torch.int64), 0, torch.qint8).int_repr().numpy()
    assert np.array_equal(tq, q2)


def test_act_s8_quantiser():
    a = np.array([0.0, 1.0, -2.54, 1.27, 0.635, -0.01], np.float32)
    s = O.act_scale_s8(a)
    assert s == np.float32(np.float32(2.54) / np.float32(127))
    q = O.quantize_act_s8(a, s)
    # float32 quotient re-derived through float64 (53 >= 2 * 24 + 2 bits: same rounding), then ties to even
    want = np.clip(np.rint((a.astype(np.float64) / np.float64(s)).astype(np.float32)), -127, 127)
    assert q.tolist() == want.astype(int).tolist() and q[2] == -127 and q[1] == 50 and q[0] == 0
    assert O.act_scale_s8(np.zeros(4, np.float32)) == 1
    # ties to even with an exact step
    assert O.quantize_act_s8(np.array([0.5, 1.5, 2.5, -0.5, -1.5, 200.0], np.float32), 1.0).tolist() == [0, 2, 2, 0, -2, 127]


def test_w8a8_conv_brute_force_and_special_cases():
    rng = np.random.default_rng(3)
    B, H, W, Cin, Cout, KH, KW, stride, pad = 1, 4, 5, 4, 3, 3, 3, 1, 1
    a = rng.integers(-128, 128, size=(B, H, W, Cin)).astype(np.int8)
    w = rng.integers(-128, 128, size=(Cout, KH, KW, Cin)).astype(np.int8)
    got = O.w8a8_conv_acc(O.pack_bytes(a), O.pack_bytes(w.reshape(Cout, -1)), B, H, W, Cin, Cout, KH, KW, stride, pad)
    ref = np.zeros((B * H * W, Cout), np.int64)
    for oh in range(H):
        for ow in range(W):
            for n in range(Cout):
                t = 0
                for kh in range(KH):
                    for kw in range(KW):
                        ih, iw = oh + kh - pad, ow + kw - pad
                        if 0 <= ih < H and 0 <= iw < W:
                            for c in range(Cin):
                                t += int(a[0, ih, iw, c]) * int(w[n, kh, kw, c])
                ref[oh * W + ow, n] = t
    assert np.array_equal(got, ref)
    # the row-sampling form, every row in shuffled order, against the same brute force
    rows = rng.permutation(B * H * W)
    assert np.array_equal(O.w8a8_conv_acc_rows(O.pack_bytes(a), O.pack_bytes(w.reshape(Cout, -1)), B, H, W, Cin, Cout,
                                               KH, KW, stride, pad, rows), ref[rows])
    # 1x1, stride 1: a plain integer matrix product
    a1 = rng.integers(-128, 128, size=(2, 3, 3, 8)).astype(np.int8)
    w1 = rng.integers(-128, 128, size=(5, 8)).astype(np.int8)
    got = O.w8a8_conv_acc(O.pack_bytes(a1), O.pack_bytes(w1), 2, 3, 3, 8, 5, 1, 1, 1, 0)
    assert np.array_equal(got, a1.reshape(18, 8).astype(np.int64) @ w1.astype(np.int64).T)
    # extremes: all -128 x all -128 over K = 16384 * K... fits int32 for K up to 131071
    K = 64
    ae = np.full((1, 1, 1, K), -128, np.int8)
    we = np.full((1, K), -128, np.int8)
    assert O.w8a8_conv_acc(O.pack_bytes(ae), O.pack_bytes(we), 1, 1, 1, K, 1, 1, 1, 1, 0)[0, 0] == 16384 * K


def test_w8_group_quantiser_and_linear():
    w = synth.llm_weight(12, 256, 9, outlier_frac=0.01)
    q, s = O.quantize_w8_sym_group(w, 64)
    assert q.dtype == np.int8 and s.dtype == np.float16 and s.shape == (12, 4)
    wg = w.reshape(12, 4, 64).astype(np.float64)
    sf = s.astype(np.float64)
    # the stored scale is the smallest float16 >= max|w| / 127 (exact rationals)
    for n in range(12):
        for g in range(4):
            amax = Fraction(float(np.abs(w.reshape(12, 4, 64)[n, g]).max()))
            s32 = np.float32(np.float32(amax) / np.float32(127))
            st = Fraction(float(s[n, g]))
            assert st >= Fraction(float(s32))
            below = np.nextafter(s[n, g], np.float16(0))
            assert Fraction(float(below)) < Fraction(float(s32))
    err = np.abs(wg - q.reshape(12, 4, 64) * sf[:, :, None])
    assert np.all(err <= sf[:, :, None] * (0.5 + 2.0 ** -20))
    assert np.abs(q.astype(int)).max() <= 127
    # linear: against a rational dot product on one output, and the integer special case
    xb = synth.llm_activation_bf16(2, 256, 10)
    y = O.w8a16_linear(xb, q, s, 64)
    x = O.bf16_bits_to_f64(xb)
    t = sum(Fraction(float(x[1, k])) * int(q[3, k]) * Fraction(float(s[3, k // 64])) for k in range(256))
    assert abs(Fraction(float(y[1, 3])) - t) <= abs(t) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 12)
    ones = np.ones((12, 4), np.float16)
    xi = synth.f32_to_bf16_bits(np.round(synth.bf16_bits_to_f32(xb) * 4))
    assert np.array_equal(O.w8a16_linear(xi, q, ones, 64),
                          synth.bf16_bits_to_f32(xi).astype(np.int64) @ q.astype(np.int64).T)
    with pytest.raises(ValueError):
        O.quantize_w8_sym_group(np.full((1, 64), 3.0e7, np.float32), 64)
