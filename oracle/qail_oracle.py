"""CPU oracle for the 4-bit quantised linear layer.  TEST INFRASTRUCTURE ONLY.

This file is the plain, slow definition that the GPU library is checked
against.  It is imported by the tests, by the smoke check and by the CPU
baseline leg of the benchmark, never by the product path, and it shares no
code with the HIP kernels or their Python binding.

What it follows in the paper:
  * Sec. 2.1: quantisation is applied to the operands of a GEMM, one operand
    (weight-only, for bandwidth-bound LLM linears) or both (weights and
    activations, for compute-bound convolutions); round-to-nearest (RTN) maps
    real values to a small set of integer states.
  * Sec. 5.1: the VLA policy uses 4-bit weight-only quantisation (AWQ output
    format: asymmetric unsigned 4-bit codes with a scale and an integer
    zero-point); the driving policy uses 4-bit weights and 4-bit activations
    (RTN / LSQ integer format: signed weight codes, unsigned post-ReLU
    activation codes, one real scale each).
  * Appendix "Hyperparameter Setting": granularity.  Channel-wise is the
    special case group_size == K here.

The RTN formula itself is only drawn in a figure of the paper; the affine
min/max reading used here, and every other point where the paper is silent,
is spelled out next to the step that needs it.

Pins (tests/test_oracle_*.py): code ranges, the half-step reconstruction
bound against the stored scale, fixed-(s,z) idempotence, pack/unpack round
trips, closed forms (constant codes, one-hot activations, power-of-two
homogeneity, extreme integer codes), reductions to textbook routines
(per-channel affine quantisation, plain integer matmul, 1x1 convolution as a
GEMM, centre-tap identity, shifted single tap), and pure-Python brute force
on tiny shapes.  No function here is unpinned.

Floating point: the quantiser works in IEEE float32 (the codes depend on the
rounding of a float32 quotient, so float64 would change them at ties); the
linear layer and the requantisation are evaluated in float64.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32

# ---------------------------------------------------------------------------
# nibble packing (8 four-bit codes per 32-bit word, lowest nibble first)
# ---------------------------------------------------------------------------


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """[..., L] integer codes (only the low 4 bits are kept, so signed codes
    are stored as two's-complement nibbles) -> [..., ceil(L/8)] uint32.
    Code j of the last axis goes to bits [4*(j%8), 4*(j%8)+3] of word j//8;
    a ragged tail is padded with zero nibbles."""
    c = np.asarray(codes).astype(np.int64) & 0xF
    L = c.shape[-1]
    pad = (-L) % 8
    if pad:
        c = np.concatenate([c, np.zeros(c.shape[:-1] + (pad,), dtype=np.int64)], axis=-1)
    c = c.reshape(c.shape[:-1] + (-1, 8))
    word = np.zeros(c.shape[:-1], dtype=np.int64)
    for j in range(8):
        word |= c[..., j] << (4 * j)
    return word.astype(np.uint32)


def unpack_nibbles_u4(words: np.ndarray, L: int) -> np.ndarray:
    """Inverse of pack_nibbles for unsigned codes: [..., W] uint32 -> [..., L] uint8."""
    w = np.asarray(words, dtype=np.uint32).astype(np.int64)
    out = np.empty(w.shape + (8,), dtype=np.uint8)
    for j in range(8):
        out[..., j] = (w >> (4 * j)) & 0xF
    out = out.reshape(w.shape[:-1] + (-1,))
    return out[..., :L]


def unpack_nibbles_s4(words: np.ndarray, L: int) -> np.ndarray:
    """Inverse of pack_nibbles for signed codes: nibble v >= 8 means v - 16."""
    u = unpack_nibbles_u4(words, L).astype(np.int8)
    return np.where(u >= 8, u - 16, u).astype(np.int8)


# ---------------------------------------------------------------------------
# W4A16: group-wise asymmetric 4-bit weights (Sec. 2.1 RTN; Sec. 5.1 AWQ format)
# ---------------------------------------------------------------------------


def fp16_round_up(s32: np.ndarray) -> np.ndarray:
    """Smallest float16 that is >= the given float32 (elementwise).
    Rounding the stored scale upwards keeps (hi - lo) / s <= 15, so that the
    half-step error bound holds against the scale that is actually stored."""
    s32 = np.asarray(s32, dtype=F32)
    with np.errstate(over="ignore"):
        h = s32.astype(np.float16)
    low = h.astype(F32) < s32
    with np.errstate(over="ignore"):
        h = np.where(low, np.nextafter(h, np.float16(np.inf)), h)
    return h.astype(np.float16)


def quantize_w4_asym_group(w: np.ndarray, group_size: int):
    """RTN to unsigned 4-bit codes with one float16 scale and one integer
    zero-point per run of `group_size` consecutive input channels of a row.

    w: float32 [N, K], K % group_size == 0.
    Returns (codes uint8 [N, K] in 0..15, scales float16 [N, K/g],
             zeros uint8 [N, K/g] in 0..15).

    Per group, all in float32:
      lo = min(min w, 0), hi = max(max w, 0)      (the range always holds 0,
                                                   so the zero-point is in 0..15)
      s  = fp16_round_up((hi - lo) / 15), at least 2^-14 (no subnormal scale);
           an all-zero group takes s = 1
      z  = clamp(rint(-lo / s), 0, 15)            (rint = ties to even)
      q  = clamp(rint(w / s) + z, 0, 15)
    A group whose range does not fit float16 ((hi - lo)/15 > 65504) is an error.
    """
    w = np.asarray(w, dtype=F32)
    N, K = w.shape
    g = int(group_size)
    if g <= 0 or K % g != 0:
        raise ValueError("K must be a positive multiple of group_size")
    G = K // g
    wg = w.reshape(N, G, g)
    lo = np.minimum(wg.min(axis=2), F32(0))
    hi = np.maximum(wg.max(axis=2), F32(0))
    s32 = ((hi - lo) / F32(15)).astype(F32)
    if np.any(s32 > F32(65504)):
        raise ValueError("group range does not fit a float16 scale")
    s16 = fp16_round_up(s32)
    s16 = np.maximum(s16, np.float16(2.0 ** -14))
    s16 = np.where(hi == lo, np.float16(1.0), s16).astype(np.float16)
    s = s16.astype(F32)
    z = np.clip(np.rint((-lo) / s), F32(0), F32(15)).astype(F32)
    q = np.rint(wg / s[:, :, None]).astype(F32) + z[:, :, None]
    q = np.clip(q, F32(0), F32(15))
    return (q.reshape(N, K).astype(np.uint8), s16, z.astype(np.uint8))


def pack_w4a16(codes: np.ndarray, zeros: np.ndarray):
    """Canonical packed form: qweight uint32 [N, K/8] and zeros uint32
    [N, ceil(G/8)], both lowest-nibble-first along K resp. the group index."""
    return pack_nibbles(codes), pack_nibbles(zeros)


def dequantize_w4_asym_group(codes: np.ndarray, scales: np.ndarray, zeros: np.ndarray,
                             group_size: int) -> np.ndarray:
    """w_hat[n, k] = (q[n, k] - z[n, k // g]) * s[n, k // g], float64 (exact:
    a 5-bit integer times an 11-bit significand)."""
    N, K = codes.shape
    g = int(group_size)
    q = codes.astype(np.float64).reshape(N, K // g, g)
    z = zeros.astype(np.float64)[:, :, None]
    s = scales.astype(np.float64)[:, :, None]
    return ((q - z) * s).reshape(N, K)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exact."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def w4a16_linear(x_bf16_bits: np.ndarray, qweight: np.ndarray, scales: np.ndarray,
                 zeros_packed: np.ndarray, group_size: int) -> np.ndarray:
    """y[m, n] = sum_k x[m, k] * w_hat[n, k] in float64, not rounded.

    Takes the packed form on purpose (quantise -> pack -> unpack -> dequantise
    -> matmul), so that the packing convention is part of what is checked.
    x: bf16 bit patterns [M, K]; qweight uint32 [N, K/8]; scales float16
    [N, G]; zeros_packed uint32 [N, ceil(G/8)]."""
    N = qweight.shape[0]
    K = qweight.shape[1] * 8
    G = K // int(group_size)
    codes = unpack_nibbles_u4(qweight, K)
    zeros = unpack_nibbles_u4(zeros_packed, G)
    w_hat = dequantize_w4_asym_group(codes, np.asarray(scales, dtype=np.float16), zeros, group_size)
    x = bf16_bits_to_f64(x_bf16_bits)
    return x @ w_hat.T


def w4a16_row_norms(x_bf16_bits, qweight, scales, zeros_packed, group_size):
    """(||x[m, :]||_2, ||w_hat[n, :]||_2) in float64: the normalisation of the
    W4A16 acceptance error |y - y_ref| / (||x_m|| * ||w_hat_n||)."""
    K = qweight.shape[1] * 8
    G = K // int(group_size)
    w_hat = dequantize_w4_asym_group(unpack_nibbles_u4(qweight, K),
                                     np.asarray(scales, dtype=np.float16),
                                     unpack_nibbles_u4(zeros_packed, G), group_size)
    x = bf16_bits_to_f64(x_bf16_bits)
    return np.sqrt((x * x).sum(axis=1)), np.sqrt((w_hat * w_hat).sum(axis=1))


def w4a16_linear_lora(x_bf16_bits: np.ndarray, qweight: np.ndarray, scales: np.ndarray,
                      zeros_packed: np.ndarray, group_size: int, a_bf16_bits: np.ndarray,
                      b_bf16_bits: np.ndarray, scaling: float) -> np.ndarray:
    """The 4-bit linear with an unmerged low-rank adapter beside it (Sec. 5.1: the
    4-bit OpenVLA policy is fine-tuned with rank-32 adapters on the quantised
    backbone, which then run next to the packed weights):

        y[m, n] = sum_k x[m, k] w_hat[n, k]  +  scaling * sum_j (sum_k x[m, k] A[j, k]) B[n, j]

    A [r, K] and B [N, r] are bfloat16 bit patterns; everything in float64, not
    rounded."""
    base = w4a16_linear(x_bf16_bits, qweight, scales, zeros_packed, group_size)
    x = bf16_bits_to_f64(x_bf16_bits)
    t = x @ bf16_bits_to_f64(a_bf16_bits).T          # [M, r]
    return base + np.float64(scaling) * (t @ bf16_bits_to_f64(b_bf16_bits).T)


# ---------------------------------------------------------------------------
# W4A4: signed 4-bit weights per output channel, unsigned 4-bit activations
# per tensor (Sec. 5.1 "Autonomous Driving"; appendix granularity)
# ---------------------------------------------------------------------------


def quantize_w4_sym_channel(w: np.ndarray):
    """w: float32 [Cout, ...]; per output channel n, in float32:
      s_w[n] = max |w[n]| / 7   (1 if the channel is all zero)
      q      = clamp(rint(w / s_w[n]), -8, 7)
    Returns (codes int8 same shape, s_w float32 [Cout]).  Per-tensor
    quantisation is the special case of all channels sharing one absmax."""
    w = np.asarray(w, dtype=F32)
    flat = w.reshape(w.shape[0], -1)
    amax = np.abs(flat).max(axis=1).astype(F32)
    s = (amax / F32(7)).astype(F32)
    s = np.where(amax == 0, F32(1), s).astype(F32)
    q = np.clip(np.rint(flat / s[:, None]), F32(-8), F32(7))
    return q.astype(np.int8).reshape(w.shape), s


def act_scale_u4(a: np.ndarray) -> np.float32:
    """One step size for a whole (non-negative) activation tensor:
    s_a = max(a) / 15 in float32, 1 if the maximum is not positive."""
    m = F32(np.max(np.asarray(a, dtype=F32)))
    return F32(m / F32(15)) if m > 0 else F32(1)


def quantize_act_u4(a: np.ndarray, s_a) -> np.ndarray:
    """q = clamp(rint(a / s_a), 0, 15), float32 arithmetic, uint8 codes."""
    a = np.asarray(a, dtype=F32)
    q = np.clip(np.rint(a / F32(s_a)), F32(0), F32(15))
    return q.astype(np.uint8)


def im2col_nhwc(a: np.ndarray, KH: int, KW: int, stride: int, pad: int) -> np.ndarray:
    """[B, H, W, C] -> [B*OH*OW, KH*KW*C] with zero padding; row index
    (b, oh, ow), column index (kh, kw, c)."""
    B, H, W, C = a.shape
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (W + 2 * pad - KW) // stride + 1
    ap = np.zeros((B, H + 2 * pad, W + 2 * pad, C), dtype=a.dtype)
    ap[:, pad:pad + H, pad:pad + W, :] = a
    cols = np.empty((B, OH, OW, KH, KW, C), dtype=a.dtype)
    for kh in range(KH):
        for kw in range(KW):
            cols[:, :, :, kh, kw, :] = ap[:, kh:kh + stride * OH:stride, kw:kw + stride * OW:stride, :]
    return cols.reshape(B * OH * OW, KH * KW * C)


def w4a4_conv_acc(a_words: np.ndarray, w_words: np.ndarray, B: int, H: int, W: int, Cin: int,
                  Cout: int, KH: int, KW: int, stride: int, pad: int,
                  use_blas: bool = False) -> np.ndarray:
    """Exact integer convolution as a GEMM.

    acc[(b, oh, ow), n] = sum_{kh, kw, c} a[b, oh*stride + kh - pad, ow*stride + kw - pad, c]
                                          * w[n, kh, kw, c]
    with zero outside the image.  a_words: packed unsigned codes, uint32
    [B, H, W, Cin/8]; w_words: packed signed codes, uint32 [Cout, KH*KW*Cin/8]
    with K ordered (kh, kw, c).  Summed in int64 (or, with use_blas, in
    float64, which is exact because every partial sum is an integer far below
    2^53), then checked against the bound 8*15*K and returned as int32 [M, Cout].
    """
    a = unpack_nibbles_u4(np.asarray(a_words).reshape(B, H, W, Cin // 8), Cin).astype(np.int64)
    K = KH * KW * Cin
    wq = unpack_nibbles_s4(np.asarray(w_words).reshape(Cout, K // 8), K).astype(np.int64)
    cols = im2col_nhwc(a, KH, KW, stride, pad)
    if use_blas:
        acc = np.rint(cols.astype(np.float64) @ wq.astype(np.float64).T).astype(np.int64)
    else:
        acc = cols @ wq.T
    if acc.size and np.abs(acc).max() > 8 * 15 * K:
        raise AssertionError("accumulator exceeds 8*15*K")
    return acc.astype(np.int32)


def im2col_rows_nhwc(a: np.ndarray, KH: int, KW: int, stride: int, pad: int, rows: np.ndarray) -> np.ndarray:
    """Selected rows of im2col_nhwc(a, ...) without forming the others: row m = (b, oh, ow) with
    m = (b * OH + oh) * OW + ow gathers a[b, oh*stride + kh - pad, ow*stride + kw - pad, :] for
    every tap (kh, kw), zero outside the image.  Returns [len(rows), KH*KW*C]."""
    B, H, W, C = a.shape
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (W + 2 * pad - KW) // stride + 1
    rows = np.asarray(rows, dtype=np.int64)
    b, oh, ow = rows // (OH * OW), (rows // OW) % OH, rows % OW
    out = np.zeros((rows.size, KH, KW, C), dtype=a.dtype)
    for kh in range(KH):
        for kw in range(KW):
            ih = oh * stride + kh - pad
            iw = ow * stride + kw - pad
            ok = (ih >= 0) & (ih < H) & (iw >= 0) & (iw < W)
            out[ok, kh, kw, :] = a[b[ok], ih[ok], iw[ok], :]
    return out.reshape(rows.size, KH * KW * C)


def w4a4_conv_acc_rows(a_words: np.ndarray, w_words: np.ndarray, B: int, H: int, W: int, Cin: int,
                       Cout: int, KH: int, KW: int, stride: int, pad: int, rows: np.ndarray) -> np.ndarray:
    """Rows `rows` of w4a4_conv_acc(...): the same sum for selected output pixels only, so that
    outputs of a tensor too large to recompute whole can be checked one by one.  int32
    [len(rows), Cout]."""
    a = unpack_nibbles_u4(np.asarray(a_words).reshape(B, H, W, Cin // 8), Cin)
    K = KH * KW * Cin
    wq = unpack_nibbles_s4(np.asarray(w_words).reshape(Cout, K // 8), K).astype(np.int64)
    acc = im2col_rows_nhwc(a, KH, KW, stride, pad, rows).astype(np.int64) @ wq.T
    if acc.size and np.abs(acc).max() > 8 * 15 * K:
        raise AssertionError("accumulator exceeds 8*15*K")
    return acc.astype(np.int32)


def requant(acc: np.ndarray, scale: np.ndarray, bias: np.ndarray) -> np.ndarray:
    """y[m, n] = acc[m, n] * scale[n] + bias[n] in float64, where scale[n] is
    the float32 product s_a * s_w[n] and bias a float32 per-channel shift."""
    return (acc.astype(np.float64) * np.asarray(scale, dtype=F32).astype(np.float64)[None, :]
            + np.asarray(bias, dtype=F32).astype(np.float64)[None, :])


def requant_scale(s_a, s_w: np.ndarray) -> np.ndarray:
    """scale[n] = float32(s_a * s_w[n])."""
    return (F32(s_a) * np.asarray(s_w, dtype=F32)).astype(F32)


def requant_f32(acc: np.ndarray, scale: np.ndarray, bias: np.ndarray) -> np.ndarray:
    """The requantised output as the float32 tensor a layer hands on (the projection shortcut
    of a residual block): per element ONE float32 fused multiply-add, i.e. the exact value
    acc * scale[n] + bias[n] rounded once to float32, ties to even.

    float(acc) * scale is exact in float64 (24 x 24 significand bits).  Adding the bias in
    float64 rounds to 53 bits first, and rounding that again to 24 bits goes wrong exactly when
    the float64 sum lands on the midpoint of two neighbouring float32 values although the true
    sum does not; the error of the float64 addition (recovered exactly by the two-sum
    identities) then says on which side of the midpoint the true sum lies."""
    p = acc.astype(np.float64) * np.asarray(scale, dtype=F32).astype(np.float64)[None, :]
    b = np.broadcast_to(np.asarray(bias, dtype=F32).astype(np.float64)[None, :], p.shape)
    s = p + b
    bv = s - p
    err = (p - (s - bv)) + (b - bv)               # true sum = s + err exactly
    r = s.astype(F32)                             # nearest float32 of s, ties to even
    r64 = r.astype(np.float64)
    other = np.where(r64 <= s, np.nextafter(r, F32(np.inf)), np.nextafter(r, F32(-np.inf))).astype(F32)
    o64 = other.astype(np.float64)
    tie = (np.abs(s - r64) == np.abs(o64 - s)) & (s != r64) & np.isfinite(o64)
    # on a tie of s the true sum is nearer to the neighbour on the side err points to
    toward_other = tie & (np.sign(err) == np.sign(o64 - r64)) & (err != 0)
    return np.where(toward_other, other, r).astype(F32)


def fused_requant_u4(acc: np.ndarray, scale: np.ndarray, bias: np.ndarray, s_out,
                     res_codes: np.ndarray = None, res_scale=None, res_f32: np.ndarray = None) -> np.ndarray:
    """Output of a W4A4 layer written directly as the next layer's unsigned 4-bit
    codes (Sec. 5.1 and the appendix's implementation details for autonomous
    driving: every activation tensor is 4-bit with one learned step per tensor, so
    the step s_out of the consumer is a constant known when the producer runs).
    The shortcut of a residual block is added before the ReLU, either as the 4-bit
    codes of the block input with their step, or as a float32 tensor (projection
    shortcut).  Per element, every line one IEEE float32 operation, no fused
    multiply-add:

        t = float32(acc) * scale[n]
        t = t + bias[n]
        t = t + r              r = res_scale * float32(q_r)  or  r = res_f32, if given
        t = max(t, 0)
        q = clamp(rint(t / s_out), 0, 15)          rint: ties to even

    acc int [M, N]; scale, bias float32 [N]; returns uint8 codes [M, N]."""
    t = acc.astype(F32) * np.asarray(scale, dtype=F32)[None, :]
    t = t + np.asarray(bias, dtype=F32)[None, :]
    if res_codes is not None:
        assert res_f32 is None
        t = t + F32(res_scale) * np.asarray(res_codes).astype(F32)
    elif res_f32 is not None:
        t = t + np.asarray(res_f32, dtype=F32)
    t = np.maximum(t, F32(0))
    assert t.dtype == F32
    q = np.rint(t / F32(s_out))
    return np.clip(q, 0, 15).astype(np.uint8)


# ===========================================================================
# 8-bit variants (Sec. 5.4: the driving encoder is also deployed W8A8, the
# backbone also with 8-bit weights only).  The paper names no quantiser for them;
# the readings: symmetric round-to-nearest, weights per output channel (W8A8) or
# per group with a float16 scale (weight-only), activations per tensor, codes in
# [-127, 127] (the accumulating GEMM itself is exact for all of [-128, 127]).
# ===========================================================================

def pack_bytes(codes: np.ndarray) -> np.ndarray:
    """[..., L] integer codes (low 8 bits kept, so signed codes become their
    two's-complement byte), L % 4 == 0 -> uint32 [..., L/4]; code i of a word
    occupies bits [8*(i%4), 8*(i%4)+7]."""
    c = np.asarray(codes)
    assert c.shape[-1] % 4 == 0
    b = (c.astype(np.int64) & 0xFF).astype(np.uint32).reshape(*c.shape[:-1], c.shape[-1] // 4, 4)
    shifts = (8 * np.arange(4, dtype=np.uint32))
    return np.bitwise_or.reduce(b << shifts, axis=-1).astype(np.uint32)


def unpack_bytes_s8(words: np.ndarray, L: int) -> np.ndarray:
    """Inverse of pack_bytes for signed codes: [..., W] uint32 -> [..., L] int8."""
    w = np.asarray(words, dtype=np.uint32)
    shifts = (8 * np.arange(4, dtype=np.uint32))
    b = ((w[..., None] >> shifts) & np.uint32(0xFF)).astype(np.uint8)
    return b.reshape(*w.shape[:-1], -1)[..., :L].view(np.int8)


def quantize_w8_sym_channel(w: np.ndarray):
    """w: float32 [Cout, ...]; per output channel n, in float32:
    s_w[n] = max|w[n]| / 127 (1 if the channel is all zero),
    q = clamp(rint(w / s_w[n]), -127, 127).  Returns (q int8 same shape, s_w float32 [Cout])."""
    w = np.asarray(w, dtype=F32)
    flat = w.reshape(w.shape[0], -1)
    amax = np.abs(flat).max(axis=1)
    s = (amax / F32(127)).astype(F32)
    s = np.where(amax == 0, F32(1), s).astype(F32)
    q = np.clip(np.rint(flat / s[:, None]), -127, 127).astype(np.int8)
    return q.reshape(w.shape), s


def act_scale_s8(a: np.ndarray) -> np.float32:
    """One step for a whole activation tensor: max|a| / 127 in float32 (1 if all zero)."""
    amax = F32(np.abs(np.asarray(a, dtype=F32)).max()) if np.asarray(a).size else F32(0)
    return F32(1) if amax == 0 else F32(amax / F32(127))


def quantize_act_s8(a: np.ndarray, s_a) -> np.ndarray:
    """q = clamp(rint(a / s_a), -127, 127), float32 arithmetic, int8 codes."""
    a = np.asarray(a, dtype=F32)
    return np.clip(np.rint(a / F32(s_a)), -127, 127).astype(np.int8)


def w8a8_conv_acc(a_words: np.ndarray, w_words: np.ndarray, B: int, H: int, W: int, Cin: int,
                  Cout: int, KH: int, KW: int, stride: int, pad: int) -> np.ndarray:
    """The exact integer convolution of w4a4_conv_acc with signed 8-bit codes on both
    sides: a_words uint32 [B, H, W, Cin/4], w_words uint32 [Cout, KH*KW*Cin/4], K ordered
    (kh, kw, c), zero outside the image; summed in int64, checked against 128*128*K,
    returned as int32 [M, Cout]."""
    a = unpack_bytes_s8(np.asarray(a_words).reshape(B, H, W, Cin // 4), Cin).astype(np.int64)
    K = KH * KW * Cin
    wq = unpack_bytes_s8(np.asarray(w_words).reshape(Cout, K // 4), K).astype(np.int64)
    acc = im2col_nhwc(a, KH, KW, stride, pad) @ wq.T
    if acc.size and np.abs(acc).max() > 128 * 128 * K:
        raise AssertionError("accumulator exceeds 128*128*K")
    return acc.astype(np.int32)


def w8a8_conv_acc_rows(a_words: np.ndarray, w_words: np.ndarray, B: int, H: int, W: int, Cin: int,
                       Cout: int, KH: int, KW: int, stride: int, pad: int, rows: np.ndarray) -> np.ndarray:
    """Rows `rows` of w8a8_conv_acc(...), for outputs checked one by one.  int32 [len(rows), Cout]."""
    a = unpack_bytes_s8(np.asarray(a_words).reshape(B, H, W, Cin // 4), Cin)
    K = KH * KW * Cin
    wq = unpack_bytes_s8(np.asarray(w_words).reshape(Cout, K // 4), K).astype(np.int64)
    acc = im2col_rows_nhwc(a, KH, KW, stride, pad, rows).astype(np.int64) @ wq.T
    if acc.size and np.abs(acc).max() > 128 * 128 * K:
        raise AssertionError("accumulator exceeds 128*128*K")
    return acc.astype(np.int32)


def quantize_w8_sym_group(w: np.ndarray, group_size: int):
    """Weight-only 8-bit: per row n and group of g consecutive k, in float32:
    s = float16 round-up of max|w| / 127, at least 2^-14 (1 for an all-zero group;
    raises beyond the float16 range), q = clamp(rint(w / s), -127, 127).
    Returns (q int8 [N, K], s float16 [N, K/g])."""
    w = np.asarray(w, dtype=F32)
    N, K = w.shape
    assert K % group_size == 0
    wg = w.reshape(N, K // group_size, group_size)
    amax = np.abs(wg).max(axis=2)
    s32 = (amax / F32(127)).astype(F32)
    if np.any(s32 > F32(65504)):
        raise ValueError("group range exceeds the float16 scale format")
    s = np.maximum(fp16_round_up(s32), np.float16(2.0 ** -14)).astype(np.float16)
    s = np.where(amax == 0, np.float16(1), s).astype(np.float16)
    q = np.clip(np.rint(wg / s.astype(F32)[:, :, None]), -127, 127).astype(np.int8)
    return q.reshape(N, K), s


def w8a16_linear(x_bf16_bits: np.ndarray, codes: np.ndarray, scales: np.ndarray, group_size: int) -> np.ndarray:
    """y[m, n] = sum_k x[m, k] * q[n, k] * s[n, k // g] in float64, not rounded."""
    x = bf16_bits_to_f64(x_bf16_bits)
    q = np.asarray(codes).astype(np.float64)
    s = np.repeat(np.asarray(scales).astype(np.float64), group_size, axis=1)
    return x @ (q * s).T


# ===========================================================================
# Training-side operators (Sec. 4.1, Algorithm 1: the quantised policy is trained
# through its quantisers with the straight-through estimator; Sec. 4.2, Eq. 3 and the
# appendix's implementation details: the QBC term is the mean L2 distance between
# the final logits of the quantised and the full-precision policy).
# ===========================================================================

def fake_quant_w4_group(w: np.ndarray, group_size: int) -> np.ndarray:
    """Quantise-dequantise of a weight matrix with the 4-bit group quantiser above:
    what the forward pass of quantisation-aware training sees.  float32 [N, K]; the
    products (q - z) * s are exact in float32 (5-bit integer times 11-bit significand).
    Its straight-through backward is the identity (Algorithm 1), so it has no code."""
    q, s, z = quantize_w4_asym_group(w, group_size)
    return dequantize_w4_asym_group(q, s, z, group_size).astype(F32)


def lsq_fake_quant_fwd(v: np.ndarray, s, qn: int, qp: int) -> np.ndarray:
    """Learned-step quantiser named in Sec. 5.1 for weights and activations:
    v_hat = clamp(rint(v / s), qn, qp) * s, every operation in float32."""
    v = np.asarray(v, dtype=F32)
    return (np.clip(np.rint(v / F32(s)), qn, qp).astype(F32) * F32(s)).astype(F32)


def lsq_fake_quant_bwd(v: np.ndarray, s, qn: int, qp: int, dout: np.ndarray, grad_scale: float):
    """Straight-through backward of lsq_fake_quant_fwd (rint treated as the identity when
    differentiating, clamp as it is):
        dv = dout                         where qn <= v / s <= qp, else 0
        ds = grad_scale * sum dout * t,   t = rint(v/s) - v/s inside, qn below, qp above.
    The ratio v / s is the float32 one of the forward; the sum is in float64.
    Returns (dv float32, ds float64 scalar)."""
    v = np.asarray(v, dtype=F32)
    dout = np.asarray(dout, dtype=F32)
    r = v / F32(s)
    inside = (r >= F32(qn)) & (r <= F32(qp))
    dv = np.where(inside, dout, F32(0)).astype(F32)
    t = np.where(inside, np.rint(r).astype(np.float64) - r.astype(np.float64),
                 np.where(r < F32(qn), np.float64(qn), np.float64(qp)))
    return dv, float(grad_scale) * float((dout.astype(np.float64) * t).sum())


def qbc_loss(logits_q: np.ndarray, logits_fp: np.ndarray):
    """Eq. 3 with the discrepancy the appendix states: the mean over the batch of the L2
    distance between the two policies' final logits.  float64.
    Returns (loss, d loss / d logits_q); rows with zero distance have zero gradient."""
    a = np.asarray(logits_q, dtype=np.float64)
    b = np.asarray(logits_fp, dtype=np.float64)
    diff = a - b
    dist = np.sqrt((diff * diff).sum(axis=1))
    Bn = a.shape[0]
    grad = np.where(dist[:, None] > 0, diff / np.where(dist > 0, dist, 1.0)[:, None], 0.0) / Bn
    return float(dist.mean()), grad
