"""Pins for the W4A16 half of the CPU oracle: none of these re-types the
oracle's formula; each is an invariant, a closed form, a hand-worked value, a
library routine on a case where both must agree exactly, or brute force."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import qail_oracle as O
from paper_2412_01034_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _quant(N, K, g, seed, **kw):
    w = synth.llm_weight(N, K, seed, **kw)
    q, s, z = O.quantize_w4_asym_group(w, g)
    return w, q, s, z


# ---- packing ---------------------------------------------------------------

def test_pack_known_words():
    assert O.pack_nibbles(np.arange(8))[0] == 0x76543210
    assert O.pack_nibbles(np.array([15, 0, 0, 0, 0, 0, 0, 1]))[0] == 0x1000000F
    # signed codes are stored as two's-complement nibbles
    assert O.pack_nibbles(np.array([-8, -1, 7, 0, 0, 0, 0, -2]))[0] == 0xE00007F8
    # ragged tail pads with zero nibbles (86 groups -> 11 words)
    assert O.pack_nibbles(np.full((3, 86), 15)).shape == (3, 11)
    assert O.pack_nibbles(np.full(86, 15))[10] == 0x00FFFFFF


def test_pack_unpack_round_trips():
    rng = np.random.default_rng(1)
    c = rng.integers(0, 16, size=(5, 7, 24), dtype=np.uint8)
    assert np.array_equal(O.unpack_nibbles_u4(O.pack_nibbles(c), 24), c)
    s = rng.integers(-8, 8, size=(4, 40), dtype=np.int8)
    assert np.array_equal(O.unpack_nibbles_s4(O.pack_nibbles(s), 40), s)
    words = rng.integers(0, 2 ** 32, size=(6, 9), dtype=np.uint64).astype(np.uint32)
    assert np.array_equal(O.pack_nibbles(O.unpack_nibbles_u4(words, 72)), words)
    assert np.array_equal(O.pack_nibbles(O.unpack_nibbles_s4(words, 72)), words)
    r = rng.integers(0, 16, size=(2, 13), dtype=np.uint8)     # ragged
    assert np.array_equal(O.unpack_nibbles_u4(O.pack_nibbles(r), 13), r)


# ---- float16 scale rounding -------------------------------------------------

def test_fp16_round_up_is_the_smallest_not_below():
    rng = np.random.default_rng(2)
    v = np.concatenate([
        np.exp(rng.uniform(np.log(1e-6), np.log(6e4), 4000)).astype(np.float32),
        np.array([0.1, 1.0, 65504.0, 2.0 ** -14, 2.0 ** -24, 1.0009765625, 1.00048828125], np.float32)])
    h = O.fp16_round_up(v)
    for vi, hi in zip(v.tolist(), h.tolist()):
        assert Fraction(hi) >= Fraction(vi)
        below = np.nextafter(np.float16(hi), np.float16(-np.inf))
        assert Fraction(float(below)) < Fraction(vi)


# ---- hand-worked example ----------------------------------------------------

def _read_golden(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = v
    return out


def test_worked_group_matches_hand_computation():
    g = _read_golden("w4a16_worked_group.txt")
    w = np.array([[float(v) for v in g["w"]]], dtype=np.float32)
    q, s, z = O.quantize_w4_asym_group(w, 8)
    assert int(s.view(np.uint16)[0, 0]) == int(g["scale_f16_bits"][0], 16)
    assert int(z[0, 0]) == int(g["zero"][0])
    assert q[0].tolist() == [int(v) for v in g["codes"]]
    qw, zw = O.pack_w4a16(q, z)
    assert int(qw[0, 0]) == int(g["word"][0], 16)
    assert int(zw[0, 0]) == int(g["zero"][0])


def test_ties_round_to_even_and_zero_point_sign():
    # range [-3, 12]: s = 1 exactly, z = 3
    w = np.array([[-3, 12, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5]], dtype=np.float32)
    q, s, z = O.quantize_w4_asym_group(w, 8)
    assert float(s[0, 0]) == 1.0 and int(z[0, 0]) == 3
    assert q[0].tolist() == [0, 15, 3, 5, 5, 3, 1, 1]


# ---- invariants -------------------------------------------------------------

@pytest.mark.parametrize("N,K,g,kw", [
    (64, 512, 64, {}),
    (48, 1024, 128, dict(outlier_frac=0.01)),
    (16, 256, 256, {}),                       # channel-wise: one group per row
    (32, 384, 8, dict(std=3.0)),
])
def test_code_range_and_half_step_bound(N, K, g, kw):
    w, q, s, z = _quant(N, K, g, 11, **kw)
    assert q.dtype == np.uint8 and q.max() <= 15
    assert z.dtype == np.uint8 and z.max() <= 15
    assert s.dtype == np.float16 and np.all(s.astype(np.float32) >= 2.0 ** -14)
    w_hat = O.dequantize_w4_asym_group(q, s, z, g)
    step = np.repeat(s.astype(np.float64), g, axis=1)
    err = np.abs(w.astype(np.float64) - w_hat)
    assert np.all(err <= step * (0.5 + 2.0 ** -20))
    # and the bound is not vacuous: some element is near half a step off
    assert (err / step).max() > 0.45


def test_one_sided_groups_keep_zero_in_range():
    rng = np.random.default_rng(5)
    w = np.abs(rng.standard_normal((8, 64)).astype(np.float32)) + 0.5      # all positive
    q, s, z = O.quantize_w4_asym_group(w, 64)
    assert np.all(z == 0)
    q2, s2, z2 = O.quantize_w4_asym_group(-w, 64)                            # all negative
    assert np.all(z2 == 15)
    assert np.array_equal(q2, 15 - q) and np.array_equal(s, s2)


def test_degenerate_and_tiny_groups():
    w = np.zeros((2, 16), dtype=np.float32)
    w[1, 8:] = 1e-9                      # far below the smallest float16 normal
    q, s, z = O.quantize_w4_asym_group(w, 8)
    assert s[0].tolist() == [1.0, 1.0] and np.all(q[0] == 0) and np.all(z[0] == 0)
    assert float(s[1, 1]) == 2.0 ** -14 and np.all(q[1] == 0)
    assert np.all(O.dequantize_w4_asym_group(q, s, z, 8) == 0)
    big = np.zeros((1, 8), dtype=np.float32)
    big[0, 0] = 1e6
    with pytest.raises(ValueError):
        O.quantize_w4_asym_group(big, 8)
    with pytest.raises(ValueError):
        O.quantize_w4_asym_group(np.zeros((1, 12), np.float32), 8)


def test_fixed_scale_idempotence_all_codes_all_zeros():
    # Every (code, zero-point) pair survives dequantise -> quantise when the
    # group spans codes 0 and 15 (so the data-derived scale/zero are unchanged).
    for s_bits in (0x3C00, 0x2E67, 0x1400, 0x5640):          # 1, ~0.1, 2^-10, 100
        s = np.array([s_bits], dtype=np.uint16).view(np.float16)[0]
        for z in range(16):
            codes = np.arange(16, dtype=np.uint8)[None, :]
            sc = np.array([[s]], dtype=np.float16)
            zz = np.array([[z]], dtype=np.uint8)
            w = O.dequantize_w4_asym_group(codes, sc, zz, 16).astype(np.float32)
            q2, s2, z2 = O.quantize_w4_asym_group(w, 16)
            assert s2[0, 0] == s and int(z2[0, 0]) == z
            assert np.array_equal(q2, codes)


def test_requantize_idempotent_on_random_weights():
    w, q, s, z = _quant(32, 512, 64, 21)
    full = (q.reshape(32, 8, 64).min(axis=2) == 0) & (q.reshape(32, 8, 64).max(axis=2) == 15)
    assert full.mean() > 0.5
    w_hat = O.dequantize_w4_asym_group(q, s, z, 64).astype(np.float32)
    q2, s2, z2 = O.quantize_w4_asym_group(w_hat, 64)
    sel = np.repeat(full, 64, axis=1)
    assert np.array_equal(s2[full], s[full]) and np.array_equal(z2[full], z[full])
    assert np.array_equal(q2[sel], q[sel])


def test_channelwise_matches_library_affine_quantizer():
    # group_size == K is per-channel affine quantisation.  With ranges built so
    # that the scale is an exact power of two, multiplying by the reciprocal
    # (the library) and dividing (the oracle) agree bit for bit.
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(8)
    N, K = 12, 96
    w = rng.uniform(-1, 1, size=(N, K)).astype(np.float32)
    for n in range(N):
        p = 2.0 ** (-(n % 5))
        zn = n % 16
        w[n] = np.clip(w[n] * 8 * p, -zn * p, (15 - zn) * p)
        w[n, 0], w[n, 1] = -zn * p, (15 - zn) * p              # pin the range
    q, s, z = O.quantize_w4_asym_group(w, K)
    assert [float(v) for v in s[:, 0]] == [2.0 ** (-(n % 5)) for n in range(N)]
    assert z[:, 0].tolist() == [n % 16 for n in range(N)]
    ref = torch.quantize_per_channel(torch.from_numpy(w), torch.from_numpy(s[:, 0].astype(np.float32)),
                                     torch.from_numpy(z[:, 0].astype(np.int64)), 0, torch.quint8)
    ref_codes = np.minimum(ref.int_repr().numpy(), 15)
    assert np.array_equal(ref_codes, q)
    fq = torch.fake_quantize_per_channel_affine(
        torch.from_numpy(w), torch.from_numpy(s[:, 0].astype(np.float32)),
        torch.from_numpy(z[:, 0].astype(np.int32)), 0, 0, 15).numpy()
    assert np.array_equal(fq.astype(np.float64), O.dequantize_w4_asym_group(q, s, z, K))


# ---- linear layer -----------------------------------------------------------

def _pack(q, z):
    return O.pack_w4a16(q, z)


def test_linear_constant_codes_closed_form():
    K, N = 512, 16
    for c in (1, 7, 15):
        q = np.full((N, K), c, np.uint8)
        s = np.ones((N, K // 64), np.float16)
        z = np.zeros((N, K // 64), np.uint8)
        x = synth.f32_to_bf16_bits(np.ones((1, K), np.float32))
        y = O.w4a16_linear(x, *_pack(q, z)[:1], s, _pack(q, z)[1], 64)
        assert np.all(y == K * c)


def test_linear_one_hot_reads_one_dequantized_weight():
    w, q, s, z = _quant(24, 256, 64, 31)
    qw, zw = _pack(q, z)
    w_hat = O.dequantize_w4_asym_group(q, s, z, 64)
    for k in (0, 1, 7, 8, 63, 64, 200, 255):
        x = np.zeros((1, 256), np.float32)
        x[0, k] = 1.0
        y = O.w4a16_linear(synth.f32_to_bf16_bits(x), qw, s, zw, 64)
        assert np.array_equal(y[0], w_hat[:, k])


def test_linear_integer_case_is_plain_integer_matmul():
    rng = np.random.default_rng(41)
    M, N, K = 5, 9, 128
    q = rng.integers(0, 16, size=(N, K), dtype=np.uint8)
    z = np.full((N, K // 32), 8, np.uint8)
    s = np.ones((N, K // 32), np.float16)
    xi = rng.integers(-20, 21, size=(M, K))
    x = synth.f32_to_bf16_bits(xi.astype(np.float32))
    y = O.w4a16_linear(x, *O.pack_w4a16(q, z)[:1], s, O.pack_w4a16(q, z)[1], 32)
    ref = xi.astype(np.int64) @ (q.astype(np.int64) - 8).T
    assert np.array_equal(y, ref.astype(np.float64))


def test_linear_brute_force_tiny():
    rng = np.random.default_rng(43)
    M, N, K, g = 3, 6, 32, 8
    w = rng.standard_normal((N, K)).astype(np.float32)
    q, s, z = O.quantize_w4_asym_group(w, g)
    qw, zw = O.pack_w4a16(q, z)
    xb = synth.llm_activation_bf16(M, K, 44)
    xf = synth.bf16_bits_to_f32(xb)
    y = O.w4a16_linear(xb, qw, s, zw, g)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                word = int(qw[n, k // 8])
                code = (word >> (4 * (k % 8))) & 15
                zp = (int(zw[n, (k // g) // 8]) >> (4 * ((k // g) % 8))) & 15
                acc += Fraction(float(xf[m, k])) * (code - zp) * Fraction(float(s[n, k // g]))
            assert abs(float(acc) - y[m, n]) <= 1e-12 * max(1.0, abs(float(acc)))


def test_linear_power_of_two_homogeneity_and_shapes():
    w, q, s, z = _quant(16, 128, 64, 51)
    qw, zw = O.pack_w4a16(q, z)
    xb = synth.llm_activation_bf16(4, 128, 52)
    y1 = O.w4a16_linear(xb, qw, s, zw, 64)
    x4 = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(xb) * np.float32(4))
    assert y1.shape == (4, 16)
    assert np.array_equal(O.w4a16_linear(x4, qw, s, zw, 64), 4 * y1)
    nx, nw = O.w4a16_row_norms(xb, qw, s, zw, 64)
    assert nx.shape == (4,) and nw.shape == (16,)
    assert np.all(np.abs(y1) <= nx[:, None] * nw[None, :] * (1 + 1e-12))      # Cauchy-Schwarz


def test_row_norms_equal_closed_forms_and_library_norm():
    # The norms are the denominator of the acceptance error of every W4A16 parity test: an
    # over-estimate would loosen the bar, so they are pinned by equalities, not by a bound.
    N, K, g = 7, 256, 64
    G = K // g
    ones = synth.f32_to_bf16_bits(np.ones((3, K), np.float32))
    # x = 1 everywhere -> ||x|| = sqrt(K); constant code c, z = 0, s = 1 -> ||w_hat|| = c sqrt(K)
    for c in (1, 3, 15):
        qw = O.pack_nibbles(np.full((N, K), c))
        zw = O.pack_nibbles(np.zeros((N, G), np.uint8))
        nx, nw = O.w4a16_row_norms(ones, qw, np.ones((N, G), np.float16), zw, g)
        assert np.array_equal(nx, np.full(3, 16.0)) and np.array_equal(nw, np.full(N, c * 16.0))
    # a zero-point and a scale: every dequantised weight is (5 - 2) * 0.5 = 1.5
    qw = O.pack_nibbles(np.full((N, K), 5))
    zw = O.pack_nibbles(np.full((N, G), 2))
    _, nw = O.w4a16_row_norms(ones, qw, np.full((N, G), 0.5, np.float16), zw, g)
    assert np.array_equal(nw, np.full(N, 1.5 * 16.0))
    # 3-4-5 triangle on one row of x
    x = np.zeros((1, K), np.float32)
    x[0, 3], x[0, 200] = 3.0, -4.0
    nx, _ = O.w4a16_row_norms(synth.f32_to_bf16_bits(x), qw, np.ones((N, G), np.float16), zw, g)
    assert nx[0] == 5.0
    # random case against numpy's norm of a matrix dequantised here, code by code, from the
    # packed words (not through the oracle's unpack / dequantise helpers)
    w, q, s, z = _quant(N, K, g, 61)
    qw, zw = O.pack_w4a16(q, z)
    xb = synth.llm_activation_bf16(4, K, 62)
    w_hat = np.empty((N, K))
    for n in range(N):
        for k in range(K):
            code = (int(qw[n, k // 8]) >> (4 * (k % 8))) & 15
            zp = (int(zw[n, (k // g) // 8]) >> (4 * ((k // g) % 8))) & 15
            w_hat[n, k] = (code - zp) * float(s[n, k // g])
    nx, nw = O.w4a16_row_norms(xb, qw, s, zw, g)
    assert np.allclose(nw, np.linalg.norm(w_hat, axis=1), rtol=1e-14, atol=0)
    assert np.allclose(nx, np.linalg.norm(synth.bf16_bits_to_f32(xb).astype(np.float64), axis=1), rtol=1e-14, atol=0)
    # per row, not per matrix: scaling one weight row changes only its own norm
    s2 = s.copy()
    s2[2] = s2[2] * np.float16(2)
    _, nw2 = O.w4a16_row_norms(xb, qw, s2, zw, g)
    assert np.allclose(nw2[2], 2 * nw[2], rtol=1e-14) and np.array_equal(np.delete(nw2, 2), np.delete(nw, 2))


def test_packed_size_consistent_with_paper_memory_table():
    # Table "Performance Metrics for OpenVLA": BF16 15.2 GB -> INT4 4.0 GB.
    # The 32 x 4 backbone linears at 4 + 16/128 + 4/128 bits per weight must
    # come to a bit under the printed 4.0 GB (embeddings, head and the vision
    # tower stay unquantised), and the bf16 form to a bit under 15.2 GB.
    params = 32 * sum(n * k for _, n, k in synth.LLAMA7B_LINEARS)
    packed = params * (4 + 16 / 128 + 4 / 128) / 8
    assert 3.2e9 < packed < 4.0e9
    assert 12.5e9 < params * 2 < 15.2e9
    assert abs(packed - 3.364e9) < 0.01e9


# ------------------------------------------------------------------ low-rank adapter beside the 4-bit linear

def _lora_case(N=24, K=256, g=64, M=3, r=8, seed=70):
    w = synth.llm_weight(N, K, seed)
    q, s, z = O.quantize_w4_asym_group(w, g)
    qw, zw = O.pack_w4a16(q, z)
    xb = synth.llm_activation_bf16(M, K, seed + 1)
    ab, bb = synth.lora_factors(N, K, r, seed + 2, std_a=0.05, std_b=0.05)
    return q, s, z, qw, zw, xb, ab, bb


def test_lora_equals_the_merged_weight_matrix():
    # (W_hat + scaling * B A) x, the textbook identity, with plain float64 matmuls
    q, s, z, qw, zw, xb, ab, bb = _lora_case()
    scaling = 1.75
    w_hat = O.dequantize_w4_asym_group(q, s, z, 64)
    A, Bm = O.bf16_bits_to_f64(ab), O.bf16_bits_to_f64(bb)
    x = O.bf16_bits_to_f64(xb)
    merged = x @ (w_hat + scaling * (Bm @ A)).T
    got = O.w4a16_linear_lora(xb, qw, s, zw, 64, ab, bb, scaling)
    assert np.allclose(got, merged, rtol=1e-12, atol=1e-12)
    assert np.abs(got - O.w4a16_linear(xb, qw, s, zw, 64)).max() > 1e-3    # the adapter matters in this case


def test_lora_special_cases():
    q, s, z, qw, zw, xb, ab, bb = _lora_case()
    base = O.w4a16_linear(xb, qw, s, zw, 64)
    zero_a, zero_b = np.zeros_like(ab), np.zeros_like(bb)
    assert np.array_equal(O.w4a16_linear_lora(xb, qw, s, zw, 64, zero_a, bb, 2.0), base)
    assert np.array_equal(O.w4a16_linear_lora(xb, qw, s, zw, 64, ab, zero_b, 2.0), base)
    assert np.array_equal(O.w4a16_linear_lora(xb, qw, s, zw, 64, ab, bb, 0.0), base)
    # linear in the scaling
    y1 = O.w4a16_linear_lora(xb, qw, s, zw, 64, ab, bb, 1.0)
    y3 = O.w4a16_linear_lora(xb, qw, s, zw, 64, ab, bb, 3.0)
    assert np.allclose(y3 - base, 3.0 * (y1 - base), rtol=1e-12, atol=1e-15)
    # rank one with A = e_k (row 0) and B = e_n (column 0): only y[:, n] changes, by scaling * x[:, k]
    N, K, r = 24, 256, 8
    a1 = np.zeros((r, K), np.float32); a1[0, 17] = 1.0
    b1 = np.zeros((N, r), np.float32); b1[5, 0] = 1.0
    y = O.w4a16_linear_lora(xb, qw, s, zw, 64, synth.f32_to_bf16_bits(a1), synth.f32_to_bf16_bits(b1), 0.5)
    d = y - base
    x = O.bf16_bits_to_f64(xb)
    assert np.allclose(d[:, 5], 0.5 * x[:, 17]) and np.count_nonzero(np.delete(d, 5, axis=1)) == 0
    # a transposed factor would not even have the right shape; a swapped pair (B A vs A B) fails here:
    assert not np.allclose(O.w4a16_linear_lora(xb, qw, s, zw, 64, ab, bb, 1.0),
                           base + (O.bf16_bits_to_f64(xb) @ O.bf16_bits_to_f64(ab).T[:, ::-1]) @ O.bf16_bits_to_f64(bb).T)
