"""GPU parity of the 8-bit variants against the CPU oracle: codes, scales and int32
accumulators bit-exact, the weight-only linear within the W4A16 bar."""
import numpy as np
import pytest

from oracle import qail_oracle as O
from paper_2412_01034_amd import synth
from tests.helpers import dev, ensure_built, host, w4a16_norm_err

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def B():
    return ensure_built()


def geom(s):
    return (s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad)


def test_weight_quantisers_bit_exact(B):
    import torch
    # per channel (the W8A8 encoder): a conv filter bank
    s = synth.ConvShape("q", 1, 8, 8, 64, 40, 3, 3, 1, 1)
    w = synth.conv_weight(s, 11)
    w[7] = 0
    q_ref, s_ref = O.quantize_w8_sym_channel(w)
    qw = torch.zeros(s.Cout * s.K // 4, dtype=torch.int32, device="cuda")
    sc = torch.zeros(s.Cout, dtype=torch.float32, device="cuda")
    B.qail_quantize_weights(dev(w.reshape(s.Cout, -1)), s.K, B.QAIL_W8_SYM_CHANNEL, qw, sc, None)
    torch.cuda.synchronize()
    assert np.array_equal(host(qw, np.uint32).reshape(s.Cout, -1), O.pack_bytes(q_ref.reshape(s.Cout, -1)))
    assert np.array_equal(host(sc, np.float32), s_ref)
    # per group (weight-only), with outlier columns and an all-zero group
    N, K, g = 96, 1024, 128
    w = synth.llm_weight(N, K, 12, outlier_frac=0.01)
    w[3, 128:256] = 0
    q_ref, s_ref = O.quantize_w8_sym_group(w, g)
    qw = torch.zeros(N * K // 4, dtype=torch.int32, device="cuda")
    sc = torch.zeros(N * K // g, dtype=torch.int16, device="cuda")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.qail_quantize_weights(dev(w), g, B.QAIL_W8_SYM_GROUP, qw, sc, None, err)
    torch.cuda.synchronize()
    assert np.array_equal(host(qw, np.uint32).reshape(N, -1), O.pack_bytes(q_ref))
    assert np.array_equal(host(sc, np.uint16).reshape(N, -1), s_ref.view(np.uint16))
    assert int(err.item()) == 0
    assert B.qail_packed_sizes(N, K, g, B.QAIL_W8_SYM_GROUP) == (N * K, N * (K // g) * 2, 0)
    assert B.qail_packed_sizes(N, K, g, B.QAIL_W8_SYM_CHANNEL) == (N * K, N * 4, 0)


def test_activation_quantiser_bit_exact(B):
    import torch
    rng = np.random.default_rng(13)
    a = (rng.standard_normal(50000) * 3).astype(np.float32)
    a[:4] = [0.0, -0.0, 1e-30, -7.5]
    sa = torch.zeros(1, dtype=torch.float32, device="cuda")
    ad = dev(a)
    B.qail_act_scale_s8(ad, sa)
    out = torch.zeros(a.size // 4, dtype=torch.int32, device="cuda")
    B.qail_quantize_act_s8(ad, sa, out)
    torch.cuda.synchronize()
    s_ref = O.act_scale_s8(a)
    assert host(sa, np.float32)[0] == s_ref
    assert np.array_equal(host(out, np.uint32), O.pack_bytes(O.quantize_act_s8(a, s_ref)))
    z = torch.zeros(64, dtype=torch.float32, device="cuda")
    B.qail_act_scale_s8(z, sa)
    torch.cuda.synchronize()
    assert host(sa, np.float32)[0] == 1.0


SHAPES = [
    synth.ConvShape("e0", 1, 4, 4, 64, 3, 3, 3, 1, 1),
    synth.ConvShape("e1", 2, 9, 7, 64, 70, 3, 3, 2, 1),        # ragged M and N tiles
    synth.ConvShape("e2", 3, 6, 6, 128, 64, 1, 1, 2, 0),
    synth.ConvShape("e3", 1, 12, 12, 192, 40, 3, 3, 1, 1),     # K split over two wave groups
    synth.ConvShape("e4", 2, 5, 5, 4, 6, 3, 3, 1, 1),          # Cin = 4: generic kernel
    synth.ConvShape("e5", 1, 6, 6, 512, 32, 3, 3, 1, 1),       # K = 4608: four wave groups
    synth.ConvShape("e6", 4, 28, 28, 128, 256, 3, 3, 2, 1),    # 128 x 128 tiles
    synth.ConvShape("e7", 2, 20, 20, 64, 64, 3, 3, 1, 1),      # 128 x 64 / 64 x 64 tiles, several blocks
]


@pytest.mark.parametrize("s", SHAPES, ids=[s.name for s in SHAPES])
def test_w8a8_conv_bit_exact(B, s):
    import torch
    a = synth.random_codes((s.B, s.H, s.W, s.Cin), -128, 127, 31).astype(np.int8)
    w = synth.random_codes((s.Cout, s.K), -128, 127, 32).astype(np.int8)
    aw, ww = O.pack_bytes(a), O.pack_bytes(w)
    ref = O.w8a8_conv_acc(aw, ww, *geom(s))
    scale = (np.random.default_rng(33).random(s.Cout) * 1e-3 + 1e-4).astype(np.float32)
    bias = synth.conv_bias(s, 34)
    acc = torch.full((s.M * s.Cout,), 0x55555555, dtype=torch.int32, device="cuda")
    y = torch.full((s.M * s.Cout,), float("nan"), dtype=torch.float32, device="cuda")
    B.qail_w8a8_gemm(*geom(s), dev(aw), dev(ww), acc_out=acc, scale=dev(scale), bias=dev(bias), y_out=y)
    torch.cuda.synchronize()
    assert np.array_equal(host(acc, np.int32).reshape(s.M, s.Cout), ref)
    yref = O.requant(ref, scale, bias)
    bound = 2.0 ** -22 * (np.abs(ref.astype(np.float64) * scale.astype(np.float64)[None, :])
                          + np.abs(bias.astype(np.float64))[None, :])
    assert np.all(np.abs(host(y, np.float32).reshape(s.M, s.Cout).astype(np.float64) - yref) <= bound)


def test_w8a8_resnet34_shapes_full_batch_sampled_images(B):
    """The ten distinct ResNet-34 body shapes at batch 32, as the benchmark's W8A8 line issues them;
    the oracle recomputes images 0, 13 and 31 (images are independent)."""
    import torch
    seen, shapes = set(), []
    for s in synth.resnet34_convs(32):
        key = (s.H, s.Cin, s.Cout, s.KH, s.stride)
        if key not in seen:
            seen.add(key)
            shapes.append(s)
    for n, s in enumerate(shapes):
        rng = np.random.default_rng(8300 + n)
        aw = rng.integers(0, 2 ** 32, size=(s.B, s.H, s.W, s.Cin // 4), dtype=np.uint64).astype(np.uint32)
        ww = rng.integers(0, 2 ** 32, size=(s.Cout, s.K // 4), dtype=np.uint64).astype(np.uint32)
        acc = torch.full((s.M * s.Cout,), 0x55555555, dtype=torch.int32, device="cuda")
        B.qail_w8a8_gemm(*geom(s), dev(aw), dev(ww), acc_out=acc)
        torch.cuda.synchronize()
        got = host(acc, np.int32).reshape(s.M, s.Cout)
        per = s.OH * s.OW
        for b in (0, 13, 31):
            ref = O.w8a8_conv_acc(aw[b:b + 1], ww, 1, *geom(s)[1:])
            assert np.array_equal(got[b * per:(b + 1) * per], ref), (s.name, b)
        # over the whole batch: an output row out of every 32 (every tile of the launch), all channels
        lo = np.arange(0, s.M, 32)
        rows = np.unique(np.r_[0, lo + rng.integers(0, np.minimum(32, s.M - lo)), s.M - 1])
        assert np.array_equal(got[rows], O.w8a8_conv_acc_rows(aw, ww, *geom(s), rows)), s.name
        del acc


def test_w8a8_extremes(B):
    import torch
    s = synth.ConvShape("x", 1, 6, 6, 512, 32, 3, 3, 1, 1)
    a = np.full((1, 6, 6, 512), -128, np.int8)
    w = np.empty((32, s.K), np.int8)
    w[0::2], w[1::2] = -128, 127
    acc = torch.zeros(s.M * s.Cout, dtype=torch.int32, device="cuda")
    B.qail_w8a8_gemm(*geom(s), dev(O.pack_bytes(a)), dev(O.pack_bytes(w)), acc_out=acc)
    torch.cuda.synchronize()
    got = host(acc, np.int32).reshape(s.M, s.Cout)
    centre = 2 * 6 + 2                                  # an interior pixel sees all 9 taps
    assert got[centre, 0] == 128 * 128 * s.K and got[centre, 1] == -128 * 127 * s.K


def w8_ws(B, N, K, g, M):
    import torch
    n = B.qail_w8a16_workspace(N, K, g, M)
    return torch.empty(n, dtype=torch.uint8, device="cuda") if n else None


@pytest.mark.parametrize("M", [1, 5, 16, 40])
@pytest.mark.parametrize("N,K,g", [(300, 4096, 128), (64, 11008, 128), (33, 256, 32), (7, 40, 8),
                                   (5, 16, 16),            # one stretch of one chunk
                                   (40, 4096, 1024),       # a group is a chunk
                                   (24, 8192, 2048),       # a group is two chunks
                                   (18, 12288, 64),        # the longest K of the streaming kernel
                                   (20, 12304, 16),        # just beyond it: row-wise kernel
                                   (300000, 16, 16)])      # more rows than 256 blocks x 16 waves x 64 hold: extra blocks
def test_w8a16_linear(B, M, N, K, g):
    import torch
    w = synth.llm_weight(N, K, 50 + N, outlier_frac=0.01)
    xb = synth.llm_activation_bf16(M, K, 51 + N)
    q, s = O.quantize_w8_sym_group(w, g)
    y = torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")
    B.qail_w8a16_linear(N, K, g, dev(O.pack_bytes(q)), dev(s.view(np.uint16)), dev(xb), y, M, w8_ws(B, N, K, g, M))
    torch.cuda.synchronize()
    ref = O.w8a16_linear(xb, q, s, g)
    nx = np.sqrt((O.bf16_bits_to_f64(xb) ** 2).sum(axis=1))
    wh = q.astype(np.float64) * np.repeat(s.astype(np.float64), g, axis=1)
    nw = np.sqrt((wh ** 2).sum(axis=1))
    tol = TOL if K >= 512 else 2.0 ** -8 * 1.01
    assert w4a16_norm_err(host(y, np.uint16).reshape(M, N), ref, nx, nw) <= tol


def test_w8a16_batch_equals_single_calls(B):
    """Up to 8 linears share a launch at M = 1, each on its own run of blocks; more than 8 and
    shapes the streaming kernel does not take (K beyond its range) go out on their own.  Rows are
    summed in the same order either way: bit for bit the single calls' results."""
    import torch
    M = 1
    shapes = [(300, 4096, 128), (64, 11008, 128), (33, 256, 32), (20, 12304, 16), (1000, 2048, 64), (5, 16, 16),
              (40, 4096, 1024), (700, 1024, 128), (18, 12288, 64), (129, 512, 16), (257, 8192, 2048)]
    ents, singles = [], []
    for i, (N, K, g) in enumerate(shapes):
        w = synth.llm_weight(N, K, 600 + i, outlier_frac=0.01)
        xb = synth.llm_activation_bf16(M, K, 700 + i)
        q, s = O.quantize_w8_sym_group(w, g)
        e = dict(N=N, K=K, group_size=g, qweight=dev(O.pack_bytes(q)), scales=dev(s.view(np.uint16)), x=dev(xb),
                 y=torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda"))
        y1 = torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")
        B.qail_w8a16_linear(N, K, g, e["qweight"], e["scales"], e["x"], y1, M)
        ents.append(e)
        singles.append(y1)
    items = B.make_w8a16_items(ents, M)
    assert B.qail_w8a16_batch_workspace(items, len(ents), M) == 0
    B.qail_w8a16_linear_batch(items, len(ents), M)
    B.qail_w8a16_linear_batch(items, 0, M)     # a no-op
    torch.cuda.synchronize()
    for e, y1 in zip(ents, singles):
        assert np.array_equal(host(e["y"], np.uint16), host(y1, np.uint16))


def _w8_norms(xb, q, s, g):
    nx = np.sqrt((O.bf16_bits_to_f64(xb) ** 2).sum(axis=1))
    wh = q.astype(np.float64) * np.repeat(s.astype(np.float64), g, axis=1)
    return nx, np.sqrt((wh ** 2).sum(axis=1))


@pytest.mark.parametrize("M", [3, 17, 130])
def test_w8a16_batch_on_the_matrix_cores(B, M):
    """M > 1: linears the matrix-core kernel takes share launches (each on a share of the blocks, K
    dealt in steps), the others (odd scale counts, K not a multiple of 64) go out on their own;
    all against the oracle."""
    import torch
    shapes = [(300, 4096, 128), (64, 11008, 128), (1000, 2048, 64), (96, 1024, 256), (257, 8192, 2048), (520, 192, 64),
              (33, 256, 32), (20, 12304, 16), (301, 192, 64), (2100, 1024, 128), (40, 8256, 64)]
    ents, keep = [], []
    for i, (N, K, g) in enumerate(shapes):
        w = synth.llm_weight(N, K, 640 + i, outlier_frac=0.01)
        xb = synth.llm_activation_bf16(M, K, 740 + i, outlier_frac=0.005)
        q, s = O.quantize_w8_sym_group(w, g)
        ents.append(dict(N=N, K=K, group_size=g, qweight=dev(O.pack_bytes(q)), scales=dev(s.view(np.uint16)), x=dev(xb),
                         y=torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")))
        keep.append((xb, q, s))
    items = B.make_w8a16_items(ents, M)
    nws = B.qail_w8a16_batch_workspace(items, len(ents), M)
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    for _ in range(2):     # run-to-run identical
        B.qail_w8a16_linear_batch(items, len(ents), M, ws)
        torch.cuda.synchronize()
        got = [host(e["y"], np.uint16).copy() for e in ents]
        if _ == 0:
            first = got
    for e, (xb, q, s), y, y0 in zip(ents, keep, got, first):
        assert np.array_equal(y, y0)
        ref = O.w8a16_linear(xb, q, s, e["group_size"])
        nx, nw = _w8_norms(xb, q, s, e["group_size"])
        tol = TOL if e["K"] >= 512 else 2.0 ** -8 * 1.01
        assert w4a16_norm_err(y.reshape(M, e["N"]), ref, nx, nw) <= tol, (e["N"], e["K"])


def test_w8a16_closed_forms_on_the_matrix_cores(B):
    # all codes c, s = 1, x = 1 -> y = K * c exactly (K * 127 = 130048 = 127 * 2^10 is a bf16 number);
    # one-hot x reads single weights: q * s rounded to fp16 (exact here: 8-bit q, s a power of two)
    import torch
    N, K, g, M = 96, 1024, 128, 40
    for c in (-128, -1, 1, 127):
        q = np.full((N, K), c, np.int8)
        s = np.ones((N, K // g), np.float16)
        xb = synth.f32_to_bf16_bits(np.ones((M, K), np.float32))
        y = torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")
        B.qail_w8a16_linear(N, K, g, dev(O.pack_bytes(q)), dev(s.view(np.uint16)), dev(xb), y, M, w8_ws(B, N, K, g, M))
        torch.cuda.synchronize()
        assert np.all(host(y, np.uint16) == synth.f32_to_bf16_bits(np.float32([K * c]))[0]), c
    rng = np.random.default_rng(5)
    q = rng.integers(-128, 128, size=(N, K)).astype(np.int8)
    s = (2.0 ** rng.integers(-6, 3, size=(N, K // g))).astype(np.float16)
    for k in (0, 5, 63, 64, 127, 128, 1023):
        x = np.zeros((M, K), np.float32)
        x[:, k] = 1.0
        x[M - 1, k] = -2.0
        y = torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")
        B.qail_w8a16_linear(N, K, g, dev(O.pack_bytes(q)), dev(s.view(np.uint16)), dev(synth.f32_to_bf16_bits(x)), y, M,
                            w8_ws(B, N, K, g, M))
        torch.cuda.synchronize()
        exp = np.repeat((q[:, k].astype(np.float32) * s[:, k // g].astype(np.float32))[None, :], M, axis=0)
        exp[M - 1] *= -2.0
        assert np.array_equal(synth.bf16_bits_to_f32(host(y, np.uint16).reshape(M, N)),
                              synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(exp))), k


@pytest.mark.parametrize("M", [2, 3, 4, 7, 8, 13, 16, 17, 25, 32])
def test_w8a16_small_batch_kernel(B, M):
    """2 <= M <= 32 (two blocks of 16 rows of x above 16) at group size 128 with an even number of groups: the small-batch streaming kernel with
    byte weights (a byte as two nibbles against the same x).  Shapes with one tile, a ragged last
    tile, more than 32 tiles per block's worth, K in one, two and three passes of the staging, K
    parts of a tile (few rows, long K); shapes it does not take (odd group count, other group
    sizes) ride along on the other paths.  Against the oracle and run to run identical; single
    calls of the first shapes against the oracle as well (the division of K among a tile's waves
    depends on the blocks an item gets, so they need not equal the batched call bit for bit)."""
    import torch
    shapes = [(16, 256, 128), (7, 256, 128), (300, 4096, 128), (64, 11008, 128), (2100, 1024, 128), (4100, 2048, 128),
              (33, 8192, 128), (8200, 512, 128), (40, 12288, 128), (300, 384, 128), (96, 1024, 256), (33, 256, 32)]
    ents, keep = [], []
    for i, (N, K, g) in enumerate(shapes):
        w = synth.llm_weight(N, K, 1640 + i, outlier_frac=0.01)
        xb = synth.llm_activation_bf16(M, K, 1740 + i, outlier_frac=0.005)
        q, s = O.quantize_w8_sym_group(w, g)
        ents.append(dict(N=N, K=K, group_size=g, qweight=dev(O.pack_bytes(q)), scales=dev(s.view(np.uint16)), x=dev(xb),
                         y=torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")))
        keep.append((xb, q, s))
    items = B.make_w8a16_items(ents, M)
    nws = B.qail_w8a16_batch_workspace(items, len(ents), M)
    ws = torch.empty(max(nws, 256), dtype=torch.uint8, device="cuda")
    for rep in range(2):
        for e in ents:
            e["y"].fill_(0x7FC0)
        B.qail_w8a16_linear_batch(items, len(ents), M, ws)
        torch.cuda.synchronize()
        got = [host(e["y"], np.uint16).copy() for e in ents]
        if rep == 0:
            first = got
    for e, (xb, q, s), y, y0 in zip(ents, keep, got, first):
        assert np.array_equal(y, y0), (e["N"], e["K"])
        ref = O.w8a16_linear(xb, q, s, e["group_size"])
        nx, nw = _w8_norms(xb, q, s, e["group_size"])
        tol = TOL if e["K"] >= 512 else 2.0 ** -8 * 1.01
        assert w4a16_norm_err(y.reshape(M, e["N"]), ref, nx, nw) <= tol, (e["N"], e["K"])
    # single calls of the shapes the kernel takes: the same sums in a different division, within the tolerance
    for e, (xb, q, s) in list(zip(ents, keep))[:4]:
        y1 = torch.full((M * e["N"],), 0x7FC0, dtype=torch.int16, device="cuda")
        B.qail_w8a16_linear(e["N"], e["K"], e["group_size"], e["qweight"], e["scales"], e["x"], y1, M,
                            w8_ws(B, e["N"], e["K"], e["group_size"], M))
        torch.cuda.synchronize()
        ref = O.w8a16_linear(xb, q, s, e["group_size"])
        nx, nw = _w8_norms(xb, q, s, e["group_size"])
        tol = TOL if e["K"] >= 512 else 2.0 ** -8 * 1.01
        assert w4a16_norm_err(host(y1, np.uint16).reshape(M, e["N"]), ref, nx, nw) <= tol, (e["N"], e["K"])


@pytest.mark.parametrize("M", [5, 29])
def test_w8a16_small_batch_kernel_closed_forms(B, M):
    """All codes c, s = 1, x = 1 -> y = K * c exactly (every partial sum is an integer below 2^24, K * c a
    bf16 number for these c); one-hot x reads single weights, q * s exactly (nothing is rounded
    before the accumulation), at the first and last k of a load, a group, a turn of the ring, a pass."""
    import torch
    N, K, g = 96, 2048, 128
    for c in (-128, -1, 1, 127):
        q = np.full((N, K), c, np.int8)
        s = np.ones((N, K // g), np.float16)
        xb = synth.f32_to_bf16_bits(np.ones((M, K), np.float32))
        y = torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")
        B.qail_w8a16_linear(N, K, g, dev(O.pack_bytes(q)), dev(s.view(np.uint16)), dev(xb), y, M, w8_ws(B, N, K, g, M))
        torch.cuda.synchronize()
        assert np.all(host(y, np.uint16) == synth.f32_to_bf16_bits(np.float32([K * c]))[0]), c
    rng = np.random.default_rng(6)
    q = rng.integers(-128, 128, size=(N, K)).astype(np.int8)
    s = (2.0 ** rng.integers(-6, 3, size=(N, K // g))).astype(np.float16)
    for k in (0, 1, 7, 8, 15, 16, 63, 64, 127, 128, 511, 512, 1023, 1024, 2047):
        x = np.zeros((M, K), np.float32)
        x[:, k] = 1.0
        x[M - 1, k] = -2.0
        y = torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")
        B.qail_w8a16_linear(N, K, g, dev(O.pack_bytes(q)), dev(s.view(np.uint16)), dev(synth.f32_to_bf16_bits(x)), y, M,
                            w8_ws(B, N, K, g, M))
        torch.cuda.synchronize()
        exp = np.repeat((q[:, k].astype(np.float32) * s[:, k // g].astype(np.float32))[None, :], M, axis=0)
        exp[M - 1] *= -2.0
        assert np.array_equal(synth.bf16_bits_to_f32(host(y, np.uint16).reshape(M, N)),
                              synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(exp))), k


@pytest.mark.parametrize("M", [1, 4, 16, 288, 1024])
def test_w8a16_full_size_layer_batched_sampled(B, M):
    """The four Llama-2-7B linears at full size with 8-bit weights through the batched call (M = 1:
    the decode launch the benchmark times; 288 and 1024: its prefill lines): the GPU quantises the
    full matrices, the oracle re-derives a weight row out of every 16 and checks them against a
    row of x out of every 16 (every tile of the launch has outputs in the sample)."""
    import torch
    rng = np.random.default_rng(88)

    def strat(n):
        lo = np.arange(0, n, 16)
        return np.unique(np.r_[0, lo + rng.integers(0, np.minimum(16, n - lo)), n - 1])

    ents, keep = [], []
    for i, (name, N, K) in enumerate(synth.LLAMA7B_LINEARS):
        w = synth.llm_weight(N, K, synth.seed_for(1, i, 0), outlier_frac=0.01)
        xb = synth.llm_activation_bf16(M, K, synth.seed_for(1, i, 1), **({} if M <= 16 else dict(outlier_frac=0.005)))
        qw = torch.zeros(N * K // 4, dtype=torch.int32, device="cuda")
        sc = torch.zeros(N * (K // 128), dtype=torch.int16, device="cuda")
        wd = dev(w)
        B.qail_quantize_weights(wd, 128, B.QAIL_W8_SYM_GROUP, qw, sc, None)
        torch.cuda.synchronize()
        del wd
        rows = strat(N)
        ents.append(dict(N=N, K=K, group_size=128, qweight=qw, scales=sc, x=dev(xb),
                         y=torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")))
        keep.append((w[rows], xb, rows))
        del w
    items = B.make_w8a16_items(ents, M)
    nws = B.qail_w8a16_batch_workspace(items, len(ents), M)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
    B.qail_w8a16_linear_batch(items, len(ents), M, ws)
    torch.cuda.synchronize()
    ms = strat(M)
    worst = 0.0
    for e, (w_rows, xb, rows) in zip(ents, keep):
        N, K = e["N"], e["K"]
        q, s = O.quantize_w8_sym_group(w_rows, 128)
        assert np.array_equal(host(e["qweight"], np.uint32).reshape(N, K // 4)[rows], O.pack_bytes(q))
        assert np.array_equal(host(e["scales"], np.uint16).reshape(N, K // 128)[rows], s.view(np.uint16))
        y = host(e["y"], np.uint16).reshape(M, N)[np.ix_(ms, rows)]
        ref = O.w8a16_linear(xb[ms], q, s, 128)
        nx, nw = _w8_norms(xb[ms], q, s, 128)
        worst = max(worst, w4a16_norm_err(y, ref, nx, nw))
    assert worst <= TOL, worst
