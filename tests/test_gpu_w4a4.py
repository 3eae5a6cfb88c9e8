"""GPU parity of the W4A4 conv-as-GEMM against the CPU oracle: int32
accumulators bit-exact, requantised output within one fp32 rounding."""
import numpy as np
import pytest

from oracle import qail_oracle as O
from paper_2412_01034_amd import synth
from tests.helpers import dev, ensure_built, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    return ensure_built()


def geom(s):
    return (s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad)


def conv_fields(s):
    return dict(B=s.B, H=s.H, W=s.W, Cin=s.Cin, Cout=s.Cout, KH=s.KH, KW=s.KW, stride=s.stride, pad=s.pad)


def gpu_conv(B, s, a_words, w_words, scale=None, bias=None, want_acc=True):
    import torch
    acc = torch.full((s.M * s.Cout,), 0x55555555, dtype=torch.int32, device="cuda") if want_acc else None
    y = torch.full((s.M * s.Cout,), float("nan"), dtype=torch.float32, device="cuda") if scale is not None else None
    B.qail_w4a4_gemm(*geom(s), dev(a_words), dev(w_words), acc_out=acc,
                     scale=dev(scale) if scale is not None else None,
                     bias=dev(bias) if bias is not None else None, y_out=y)
    torch.cuda.synchronize()
    return (host(acc, np.int32).reshape(s.M, s.Cout) if want_acc else None,
            host(y, np.float32).reshape(s.M, s.Cout) if y is not None else None)


def quantised_inputs(s, seed):
    w = synth.conv_weight(s, seed)
    a = synth.conv_activation(s, seed + 1)
    bias = synth.conv_bias(s, seed + 2)
    qw, s_w = O.quantize_w4_sym_channel(w)
    s_a = O.act_scale_u4(a)
    qa = O.quantize_act_u4(a, s_a)
    return O.pack_nibbles(qa), O.pack_nibbles(qw.reshape(s.Cout, -1)), O.requant_scale(s_a, s_w), bias


def check_requant(y, acc_ref, scale, bias):
    ref = O.requant(acc_ref, scale, bias)
    bound = 2.0 ** -22 * (np.abs(acc_ref.astype(np.float64) * scale.astype(np.float64)[None, :])
                          + np.abs(bias.astype(np.float64))[None, :])
    assert np.all(np.abs(y.astype(np.float64) - ref) <= bound)


TINY = [
    synth.ConvShape("t0", 1, 4, 4, 64, 3, 3, 3, 1, 1),
    synth.ConvShape("t1", 2, 9, 7, 64, 70, 3, 3, 2, 1),       # odd sizes, ragged M and N tiles
    synth.ConvShape("t2", 3, 6, 6, 128, 64, 1, 1, 2, 0),
    synth.ConvShape("t3", 1, 12, 12, 192, 40, 3, 3, 1, 1),
    synth.ConvShape("t4", 2, 5, 5, 8, 6, 3, 3, 1, 1),         # Cin not a multiple of 64: generic kernel
    synth.ConvShape("t5", 1, 7, 7, 24, 9, 1, 1, 1, 0),
    synth.ConvShape("t6", 1, 1, 1, 64, 1, 1, 1, 1, 0),        # a single dot product
    synth.ConvShape("t7", 1, 16, 16, 64, 16, 5, 5, 1, 2),
]


@pytest.mark.parametrize("s", TINY, ids=[s.name for s in TINY])
def test_random_codes_full_range_bit_exact(B, s):
    a = synth.random_codes((s.B, s.H, s.W, s.Cin), 0, 15, 3).astype(np.uint8)
    w = synth.random_codes((s.Cout, s.K), -8, 7, 4)
    aw, ww = O.pack_nibbles(a), O.pack_nibbles(w)
    ref = O.w4a4_conv_acc(aw, ww, *geom(s))
    acc, _ = gpu_conv(B, s, aw, ww)
    assert np.array_equal(acc, ref)
    acc2, _ = gpu_conv(B, s, aw, ww)
    assert np.array_equal(acc, acc2)


def test_extreme_codes(B):
    s = synth.ConvShape("x", 1, 6, 6, 512, 32, 3, 3, 1, 1)        # K = 4608, the deepest layer
    a = np.full((1, 6, 6, 512), 15, np.uint8)
    w = np.empty((32, s.K), np.int8)
    w[0::2], w[1::2] = -8, 7
    acc, _ = gpu_conv(B, s, O.pack_nibbles(a), O.pack_nibbles(w))
    acc = acc.reshape(6, 6, 32)
    assert acc[2, 3, 0] == -120 * 4608 and acc[2, 3, 1] == 105 * 4608
    assert acc[0, 0, 0] == -120 * 4 * 512 and acc[5, 0, 1] == 105 * 4 * 512
    assert np.array_equal(acc.reshape(36, 32), O.w4a4_conv_acc(O.pack_nibbles(a), O.pack_nibbles(w), *geom(s)))


def distinct_resnet_shapes(batch):
    seen, out = set(), []
    for s in synth.resnet34_convs(batch):
        key = (s.H, s.Cin, s.Cout, s.KH, s.stride)
        if key not in seen:
            seen.add(key)
            out.append(s)
    return out


@pytest.mark.parametrize("s", distinct_resnet_shapes(2), ids=lambda s: s.name)
def test_resnet34_shapes_small_batch(B, s):
    aw, ww, scale, bias = quantised_inputs(s, 20)
    ref = O.w4a4_conv_acc(aw, ww, *geom(s), use_blas=True)
    acc, y = gpu_conv(B, s, aw, ww, scale, bias)
    assert np.array_equal(acc, ref)
    check_requant(y, ref, scale, bias)
    _, y_only = gpu_conv(B, s, aw, ww, scale, bias, want_acc=False)
    assert np.array_equal(y_only, y)


def stratified_rows(M, stripe, seed):
    """One output row drawn from every run of `stripe` consecutive rows, plus both ends: the
    convolution's tiles are 64 or 128 rows high with edges on multiples of 64, so every tile of
    every launch has rows in the sample."""
    rng = np.random.default_rng(seed)
    lo = np.arange(0, M, stripe)
    return np.unique(np.r_[0, lo + rng.integers(0, np.minimum(stripe, M - lo)), M - 1])


@pytest.mark.parametrize("s", distinct_resnet_shapes(32), ids=lambda s: s.name)
def test_resnet34_shapes_full_batch_sampled_images(B, s):
    # batch 32 as benchmarked; the oracle recomputes images 0, 13 and 31 whole (images are
    # independent) and, over the whole batch, an output row out of every 32 with all its
    # channels, so that every tile of the launch is covered
    aw, ww, scale, bias = quantised_inputs(s, synth.seed_for(3, 1, 0))
    acc, y = gpu_conv(B, s, aw, ww, scale, bias)
    per = s.OH * s.OW
    for b in (0, 13, 31):
        one = (1,) + geom(s)[1:]
        ref = O.w4a4_conv_acc(aw[b:b + 1], ww, *one, use_blas=True)
        assert np.array_equal(acc[b * per:(b + 1) * per], ref)
        check_requant(y[b * per:(b + 1) * per], ref, scale, bias)
    rows = stratified_rows(s.M, 32, s.M)
    ref = O.w4a4_conv_acc_rows(aw, ww, *geom(s), rows)
    assert np.array_equal(acc[rows], ref)
    check_requant(y[rows], ref, scale, bias)


# ------------------------------------------------------------------ fused 4-bit output

FUSED = [
    synth.ConvShape("f0", 1, 8, 8, 64, 64, 3, 3, 1, 1),
    synth.ConvShape("f1", 2, 9, 7, 64, 72, 3, 3, 2, 1),       # ragged M and N tiles
    synth.ConvShape("f2", 3, 14, 14, 128, 128, 3, 3, 1, 1),   # 128-wide tile, several row tiles
    synth.ConvShape("f3", 2, 12, 12, 64, 128, 1, 1, 2, 0),    # projection geometry
    synth.ConvShape("f4", 2, 5, 5, 8, 16, 3, 3, 1, 1),        # generic kernel
    synth.ConvShape("f5", 4, 28, 28, 128, 256, 3, 3, 2, 1),   # 128 x 128 tiles over many blocks
]


def gpu_conv_u4(B, s, aw, ww, scale, bias, s_out, res_codes=None, res_scale=0.0, res_f32=None):
    import torch
    out = torch.full((s.M * s.Cout // 8,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    B.qail_w4a4_conv_u4(*geom(s), dev(aw), dev(ww), dev(scale), dev(bias), float(s_out), out,
                        res_u4=dev(O.pack_nibbles(res_codes)) if res_codes is not None else None,
                        res_scale=float(res_scale),
                        res_f32=dev(res_f32) if res_f32 is not None else None)
    torch.cuda.synchronize()
    return host(out, np.uint32).reshape(s.M, s.Cout // 8)


@pytest.mark.parametrize("kind", ["none", "codes", "f32"])
@pytest.mark.parametrize("s", FUSED, ids=[s.name for s in FUSED])
def test_fused_u4_output_bit_exact(B, s, kind):
    aw, ww, scale, bias = quantised_inputs(s, 500 + s.Cout)
    acc_ref = O.w4a4_conv_acc(aw, ww, *geom(s))
    y = O.requant(acc_ref, scale, bias)
    s_out = np.float32(max(float(y.max()), 1e-3) / 20.0)      # the largest outputs clamp at 15
    rng = np.random.default_rng(s.M)
    rc = rs = rf = None
    if kind == "codes":
        rc, rs = rng.integers(0, 16, size=(s.M, s.Cout)).astype(np.uint8), np.float32(s_out * 0.8)
    elif kind == "f32":
        rf = (rng.standard_normal((s.M, s.Cout)) * float(s_out) * 3).astype(np.float32)
    ref = O.fused_requant_u4(acc_ref, scale, bias, s_out, res_codes=rc, res_scale=rs, res_f32=rf)
    assert ref.max() == 15 and ref.min() == 0
    got = gpu_conv_u4(B, s, aw, ww, scale, bias, s_out, rc, rs if rs is not None else 0.0, rf)
    assert np.array_equal(got, O.pack_nibbles(ref))


def test_fused_u4_ties_and_clamps(B):
    # operands exact in binary so that t / s_out lands on k + 0.5 for many elements: the kernel
    # must round those to even and must not fuse the multiply into the add
    s = synth.ConvShape("tie", 1, 6, 6, 64, 64, 1, 1, 1, 0)
    a = synth.random_codes((s.B, s.H, s.W, s.Cin), 0, 3, 21).astype(np.uint8)
    w = synth.random_codes((s.Cout, s.K), -2, 2, 22)
    aw, ww = O.pack_nibbles(a), O.pack_nibbles(w)
    acc_ref = O.w4a4_conv_acc(aw, ww, *geom(s))
    scale = np.full(s.Cout, 0.25, np.float32)
    bias = np.full(s.Cout, 0.125, np.float32)
    ref = O.fused_requant_u4(acc_ref, scale, bias, np.float32(0.25))
    t = acc_ref * 0.25 + 0.125
    assert np.any((t > 0) & (t / 0.25 % 1 == 0.5))               # ties are present
    got = gpu_conv_u4(B, s, aw, ww, scale, bias, 0.25)
    assert np.array_equal(got, O.pack_nibbles(ref))


@pytest.mark.parametrize("s_out", [0.3, 0.0123, 1.1754944e-38, 1e-39, 3e38])
def test_fused_u4_quotient_paths(B, s_out):
    # The kernel may replace t / s_out by a product when that provably gives the same code and
    # divides otherwise.  scale = s_out / 2 (exact) puts t / s_out within an ulp of a multiple of
    # 1/2 for every element, a step that is not a power of two makes the quotient inexact, and
    # steps at the ends of the range (smallest normal, denormal, near the largest float) take
    # the division throughout.
    s = synth.ConvShape("quot", 2, 5, 5, 64, 64, 3, 3, 1, 1)
    a = synth.random_codes((s.B, s.H, s.W, s.Cin), 0, 3, 31).astype(np.uint8)
    w = synth.random_codes((s.Cout, s.K), -1, 1, 32)
    aw, ww = O.pack_nibbles(a), O.pack_nibbles(w)
    acc_ref = O.w4a4_conv_acc(aw, ww, *geom(s))
    so = np.float32(s_out)
    scale = np.full(s.Cout, so / np.float32(2), np.float32)
    bias = np.zeros(s.Cout, np.float32)
    with np.errstate(over="ignore"):                          # the largest step overflows to inf: code 15
        ref = O.fused_requant_u4(acc_ref, scale, bias, so)
    if 1e-30 < s_out < 1e30:
        assert len(np.unique(ref)) >= 8                       # codes spread over the range
        assert np.any((acc_ref > 0) & (acc_ref < 31) & (acc_ref % 2 == 1))   # near-ties below the clamp
    got = gpu_conv_u4(B, s, aw, ww, scale, bias, so)
    assert np.array_equal(got, O.pack_nibbles(ref))


def test_fused_output_feeds_the_next_layer(B):
    # conv1 (fused) -> conv2 (int32): the codes written by the first call are the a_u4 of the second
    import torch
    s1 = synth.ConvShape("c1", 2, 10, 10, 64, 64, 3, 3, 1, 1)
    s2 = synth.ConvShape("c2", 2, 10, 10, 64, 128, 3, 3, 2, 1)
    aw, w1, scale1, bias1 = quantised_inputs(s1, 901)
    _, w2, _, _ = quantised_inputs(s2, 902)
    acc1 = O.w4a4_conv_acc(aw, w1, *geom(s1))
    s_mid = np.float32(float(O.requant(acc1, scale1, bias1).max()) / 15.0)
    res = O.unpack_nibbles_u4(aw.reshape(s1.M, s1.Cin // 8), s1.Cin)        # identity shortcut: the block input
    mid_ref = O.fused_requant_u4(acc1, scale1, bias1, s_mid, res_codes=res, res_scale=np.float32(0.05))
    mid = torch.zeros(s1.M * s1.Cout // 8, dtype=torch.int32, device="cuda")
    B.qail_w4a4_conv_u4(*geom(s1), dev(aw), dev(w1), dev(scale1), dev(bias1), float(s_mid), mid,
                        res_u4=dev(aw), res_scale=0.05)
    acc2 = torch.zeros(s2.M * s2.Cout, dtype=torch.int32, device="cuda")
    B.qail_w4a4_gemm(*geom(s2), mid, dev(w2), acc_out=acc2)
    torch.cuda.synchronize()
    assert np.array_equal(host(mid, np.uint32).reshape(s1.M, -1), O.pack_nibbles(mid_ref))
    ref2 = O.w4a4_conv_acc(O.pack_nibbles(mid_ref).reshape(s1.B, s1.H, s1.W, -1), w2, *geom(s2))
    assert np.array_equal(host(acc2, np.int32).reshape(s2.M, s2.Cout), ref2)


@pytest.mark.parametrize("paired", [False, True])
def test_chained_resnet34_body_bit_exact(B, paired):
    """The whole ResNet-34 body (16 residual blocks, 32 3x3 convolutions and the 3 projection
    shortcuts) chained on the 4-bit path at a small image: every convolution but the projections
    writes the next layer's packed codes, identity shortcuts come in as the block input's codes,
    projection shortcuts as fp32.  Every step of every tensor is fixed by the oracle's own chain
    (the largest pre-quantisation value / 15), so the GPU chain must reproduce the oracle's codes
    bit for bit down to the last layer.  `paired`: the two convolutions that open a down-sampling
    block (3x3 stride 2 with fused output, 1x1 projection with fp32 output; both read the block
    input) go out as one qail_w4a4_conv_batch launch instead of two calls."""
    import torch
    Bn, H = 2, 16
    stages = [(64, 3), (128, 4), (256, 6), (512, 3)]
    seed = [7000]

    def layer(shape):
        seed[0] += 3
        w = synth.conv_weight(shape, seed[0])
        qw, s_w = O.quantize_w4_sym_channel(w)
        return O.pack_nibbles(qw.reshape(shape.Cout, -1)), s_w, synth.conv_bias(shape, seed[0] + 1)

    def step_of(acc, scale, bias, r=None):
        t = acc.astype(np.float32) * scale[None, :] + bias[None, :]
        if r is not None:
            t = t + r
        return np.float32(max(float(np.maximum(t, 0).max()), 1e-3) / 15.0)

    s0 = synth.ConvShape("in", Bn, H, H, 64, 64, 3, 3, 1, 1)
    a = synth.conv_activation(s0, 6999)
    s_in = O.act_scale_u4(a)
    codes = O.quantize_act_u4(a, s_in).reshape(Bn * H * H, 64)       # oracle chain: codes [M, C] and their step
    g_codes = dev(O.pack_nibbles(codes))                              # GPU chain: packed words
    Cin = 64
    for si, (C, nblocks) in enumerate(stages):
        for bi in range(nblocks):
            stride = 2 if (si > 0 and bi == 0) else 1
            c1 = synth.ConvShape(f"s{si}b{bi}c1", Bn, H, H, Cin, C, 3, 3, stride, 1)
            Ho = c1.OH
            c2 = synth.ConvShape(f"s{si}b{bi}c2", Bn, Ho, Ho, C, C, 3, 3, 1, 1)
            w1, sw1, b1 = layer(c1)
            w2, sw2, b2 = layer(c2)
            a_words = O.pack_nibbles(codes).reshape(Bn, H, H, Cin // 8)
            # ---- oracle: conv1 + ReLU -> codes
            acc1 = O.w4a4_conv_acc(a_words, w1, *geom(c1))
            sc1 = O.requant_scale(s_in, sw1)
            s_mid = step_of(acc1, sc1, b1)
            mid = O.fused_requant_u4(acc1, sc1, b1, s_mid)
            # ---- oracle: shortcut
            res_codes = res_f32 = None
            if stride == 2:
                cd = synth.ConvShape(f"s{si}b{bi}d", Bn, H, H, Cin, C, 1, 1, 2, 0)
                wd, swd, bd = layer(cd)
                accd = O.w4a4_conv_acc(a_words, wd, *geom(cd))
                scd = O.requant_scale(s_in, swd)
                res_f32 = O.requant_f32(accd, scd, bd)
            else:
                res_codes = codes
            # ---- oracle: conv2 + shortcut + ReLU -> codes
            acc2 = O.w4a4_conv_acc(O.pack_nibbles(mid).reshape(Bn, Ho, Ho, C // 8), w2, *geom(c2))
            sc2 = O.requant_scale(s_mid, sw2)
            r = res_f32 if res_f32 is not None else np.float32(s_in) * res_codes.astype(np.float32)
            s_out = step_of(acc2, sc2, b2, r)
            out = O.fused_requant_u4(acc2, sc2, b2, s_out, res_codes=res_codes,
                                     res_scale=np.float32(s_in) if res_codes is not None else None, res_f32=res_f32)
            # ---- GPU: the same three or two calls
            g_mid = torch.zeros(c1.M * C // 8, dtype=torch.int32, device="cuda")
            g_out = torch.zeros(c2.M * C // 8, dtype=torch.int32, device="cuda")
            if stride == 2 and paired:
                g_res = torch.zeros(cd.M * C, dtype=torch.float32, device="cuda")
                keep = [dev(w1), dev(sc1), dev(b1), dev(wd), dev(scd), dev(bd)]
                items = B.make_conv_items([
                    dict(conv_fields(c1), a_u4=g_codes, w_s4=keep[0], scale=keep[1], bias=keep[2], out_u4=g_mid,
                         s_out=float(s_mid)),
                    dict(conv_fields(cd), a_u4=g_codes, w_s4=keep[3], scale=keep[4], bias=keep[5], y_out=g_res)])
                B.qail_w4a4_conv_batch(items, 2)
            else:
                B.qail_w4a4_conv_u4(*geom(c1), g_codes, dev(w1), dev(sc1), dev(b1), float(s_mid), g_mid)
            if stride == 2:
                if not paired:
                    g_res = torch.zeros(cd.M * C, dtype=torch.float32, device="cuda")
                    B.qail_w4a4_gemm(*geom(cd), g_codes, dev(wd), scale=dev(scd), bias=dev(bd), y_out=g_res)
                B.qail_w4a4_conv_u4(*geom(c2), g_mid, dev(w2), dev(sc2), dev(b2), float(s_out), g_out, res_f32=g_res)
            else:
                B.qail_w4a4_conv_u4(*geom(c2), g_mid, dev(w2), dev(sc2), dev(b2), float(s_out), g_out,
                                    res_u4=g_codes, res_scale=float(s_in))
            torch.cuda.synchronize()
            assert np.array_equal(host(g_mid, np.uint32).reshape(c1.M, -1), O.pack_nibbles(mid)), c1.name
            assert np.array_equal(host(g_out, np.uint32).reshape(c2.M, -1), O.pack_nibbles(out)), c2.name
            assert out.max() == 15 and mid.max() == 15       # the steps use the full code range
            codes, s_in, g_codes, Cin, H = out, s_out, g_out, C, Ho
    assert H == 2 and Cin == 512 and codes.any()


BATCHES = [
    # the two convolutions that open a down-sampling block (same input, same M and Cout)
    [("u4", synth.ConvShape("p1", 2, 14, 14, 128, 256, 3, 3, 2, 1)), ("y", synth.ConvShape("p1d", 2, 14, 14, 128, 256, 1, 1, 2, 0))],
    # different widths (the grid is as wide as the widest), different M, a ragged last tile, all three outputs
    [("y", synth.ConvShape("q0", 1, 9, 9, 64, 200, 3, 3, 1, 1)), ("acc", synth.ConvShape("q1", 3, 6, 6, 128, 64, 1, 1, 2, 0)),
     ("u4", synth.ConvShape("q2", 2, 12, 12, 192, 40, 3, 3, 1, 1)), ("res", synth.ConvShape("q3", 1, 8, 8, 64, 64, 3, 3, 1, 1))],
    # more items than one launch takes, one of them a shape only the one-thread-per-output kernel runs
    [("acc", synth.ConvShape("r0", 1, 6, 6, 64, 32, 3, 3, 1, 1)), ("y", synth.ConvShape("r1", 2, 5, 5, 8, 6, 3, 3, 1, 1)),
     ("u4", synth.ConvShape("r2", 1, 6, 6, 64, 64, 3, 3, 2, 1)), ("acc", synth.ConvShape("r3", 1, 4, 4, 256, 512, 3, 3, 1, 1)),
     ("y", synth.ConvShape("r4", 1, 7, 7, 512, 24, 1, 1, 1, 0)), ("u4", synth.ConvShape("r5", 2, 4, 4, 64, 8, 1, 1, 1, 0))],
]


@pytest.mark.parametrize("case", range(len(BATCHES)))
def test_conv_batch_equals_single_calls(B, case):
    """qail_w4a4_conv_batch: every item's result equals the single call's bit for bit (and the oracle's
    accumulators), whatever shares the launch with it."""
    import torch
    entries, singles, keep = [], [], []
    for i, (kind, s) in enumerate(BATCHES[case]):
        aw, ww, scale, bias = quantised_inputs(s, 1300 + 10 * case + i)
        t = dict(a=dev(aw), w=dev(ww), scale=dev(scale), bias=dev(bias))
        keep.append(t)
        e = dict(conv_fields(s), a_u4=t["a"], w_s4=t["w"])
        if kind == "acc":
            outs = [torch.full((s.M * s.Cout,), 0x55555555, dtype=torch.int32, device="cuda") for _ in range(2)]
            e.update(acc_out=outs[0])
            B.qail_w4a4_gemm(*geom(s), t["a"], t["w"], acc_out=outs[1])
        elif kind == "y":
            outs = [torch.full((s.M * s.Cout,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(2)]
            e.update(scale=t["scale"], bias=t["bias"], y_out=outs[0])
            B.qail_w4a4_gemm(*geom(s), t["a"], t["w"], scale=t["scale"], bias=t["bias"], y_out=outs[1])
        else:
            outs = [torch.full((s.M * s.Cout // 8,), 0x55555555, dtype=torch.int32, device="cuda") for _ in range(2)]
            res = t["a"] if kind == "res" else None   # identity shortcut: Cin == Cout, stride 1
            e.update(scale=t["scale"], bias=t["bias"], out_u4=outs[0], s_out=0.21, res_u4=res, res_scale=0.07)
            B.qail_w4a4_conv_u4(*geom(s), t["a"], t["w"], t["scale"], t["bias"], 0.21, outs[1], res_u4=res, res_scale=0.07)
        entries.append(e)
        singles.append((kind, s, outs, aw, ww))
    items = B.make_conv_items(entries)
    B.qail_w4a4_conv_batch(items, len(entries))
    torch.cuda.synchronize()
    for kind, s, outs, aw, ww in singles:
        got, ref = host(outs[0], np.uint32), host(outs[1], np.uint32)
        assert np.array_equal(got, ref), (kind, s.name)
        if kind == "acc":
            assert np.array_equal(got.view(np.int32).reshape(s.M, s.Cout), O.w4a4_conv_acc(aw, ww, *geom(s))), s.name


@pytest.mark.parametrize("batch", [32, 256])
def test_fused_u4_full_batch_sampled_images(B, batch):
    """The fused-output calls as the benchmark issues them (batch 32: all ten shapes; batch 256: the
    largest, a middle and the deepest one), identity shortcut where the block has one; the oracle
    recomputes three images of each (images are independent)."""
    import torch
    shapes = distinct_resnet_shapes(batch)
    if batch == 256:
        shapes = [shapes[0], shapes[len(shapes) // 2], shapes[-1]]
    for n, s in enumerate(shapes):
        rng = np.random.default_rng(8100 + n)
        a_words = rng.integers(0, 2 ** 32, size=(s.B, s.H, s.W, s.Cin // 8), dtype=np.uint64).astype(np.uint32)
        one = synth.ConvShape(s.name, 1, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad)
        _, ww, scale, bias = quantised_inputs(one, 8200 + n)
        identity = s.Cin == s.Cout and s.stride == 1
        rs = np.float32(0.05)
        acc0 = O.w4a4_conv_acc(a_words[:1], ww, *geom(one), use_blas=True)
        s_out = np.float32(max(float(O.requant(acc0, scale, bias).max()), 1e-3) / 15.0)
        out = torch.full((s.M * s.Cout // 8,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
        a_dev = dev(a_words)
        B.qail_w4a4_conv_u4(*geom(s), a_dev, dev(ww), dev(scale), dev(bias), float(s_out), out,
                            res_u4=a_dev if identity else None, res_scale=float(rs) if identity else 0.0)
        torch.cuda.synchronize()
        got = host(out, np.uint32).reshape(s.M, s.Cout // 8)
        per = s.OH * s.OW
        for b in (0, s.B // 2 - 3, s.B - 1):
            acc = O.w4a4_conv_acc(a_words[b:b + 1], ww, *geom(one), use_blas=True)
            res = O.unpack_nibbles_u4(a_words[b].reshape(per, s.Cin // 8), s.Cin) if identity else None
            ref = O.fused_requant_u4(acc, scale, bias, s_out, res_codes=res, res_scale=rs if identity else None)
            assert np.array_equal(got[b * per:(b + 1) * per], O.pack_nibbles(ref)), (s.name, b)
        # over the whole batch: an output row out of every 32 (every tile of the launch), all channels
        rows = stratified_rows(s.M, 32, 8400 + n)
        acc = O.w4a4_conv_acc_rows(a_words, ww, *geom(s), rows)
        res = O.unpack_nibbles_u4(a_words.reshape(s.M, s.Cin // 8)[rows], s.Cin) if identity else None
        ref = O.fused_requant_u4(acc, scale, bias, s_out, res_codes=res, res_scale=rs if identity else None)
        assert np.array_equal(got[rows], O.pack_nibbles(ref)), s.name
        del out, a_dev
