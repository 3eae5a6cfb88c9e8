"""GPU parity of the quantisers and (un)packers against the CPU oracle: bit-exact."""
import numpy as np
import pytest

from oracle import qail_oracle as O
from paper_2412_01034_amd import synth
from tests.helpers import dev, ensure_built, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    return ensure_built()


def gpu_quantize_asym(B, w, g, with_errors=False):
    import torch
    N, K = w.shape
    qb, sb, zb = B.qail_packed_sizes(N, K, g, B.QAIL_W4_ASYM_GROUP)
    qw = torch.full((qb // 4,), -1, dtype=torch.int32, device="cuda")
    sc = torch.full((sb // 2,), -1, dtype=torch.int16, device="cuda")
    zr = torch.full((zb // 4,), -1, dtype=torch.int32, device="cuda")
    err = torch.zeros(4, dtype=torch.int32, device="cuda")
    B.qail_quantize_weights(dev(w), g, B.QAIL_W4_ASYM_GROUP, qw, sc, zr, err if with_errors else None)
    torch.cuda.synchronize()
    G = K // g
    out = (host(qw, np.uint32).reshape(N, K // 8), host(sc, np.float16).reshape(N, G),
           host(zr, np.uint32).reshape(N, (G + 7) // 8))
    return out + (int(err[0].item()),) if with_errors else out


def check_asym(B, w, g):
    q, s, z = O.quantize_w4_asym_group(w, g)
    qw_ref, zw_ref = O.pack_w4a16(q, z)
    qw, sc, zr = gpu_quantize_asym(B, w, g)
    assert np.array_equal(sc.view(np.uint16), s.view(np.uint16))
    assert np.array_equal(zr, zw_ref)
    assert np.array_equal(qw, qw_ref)
    return qw


def test_config0_bit_exact(B):
    # tiny GEMV config: 512 x 512, N(0, 0.02), group 64, seed 0
    w = synth.llm_weight(512, 512, synth.seed_for(0, 0, 0))
    check_asym(B, w, 64)


@pytest.mark.parametrize("N,K,g,kw", [
    (48, 1024, 128, dict(outlier_frac=0.01)),
    (7, 11008, 128, dict(outlier_frac=0.01)),     # 86 groups: last zero-point word half used
    (16, 256, 256, {}),                           # channel-wise
    (5, 4096, 4096, {}),                          # channel-wise, group wider than a wave's reach
    (33, 384, 8, dict(std=3.0)),
    (1, 64, 32, {}),
    (3, 2048, 1024, dict(std=50.0)),
    (9, 1200, 24, {}),                            # group that is not a power of two
])
def test_shapes_bit_exact(B, N, K, g, kw):
    w = synth.llm_weight(N, K, 100 + N, **kw)
    check_asym(B, w, g)


def test_edge_values_bit_exact(B):
    w = np.zeros((6, 64), np.float32)
    w[1, :8] = [-3, 12, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5]          # exact ties, s = 1
    w[2, 8:16] = 1e-9                                               # below the smallest scale
    w[3, :] = 1e-41                                                 # fp32 subnormals
    w[4, :32] = np.linspace(0.1, 3.0, 32, dtype=np.float32)         # one-sided positive
    w[4, 32:] = -np.linspace(0.1, 3.0, 32, dtype=np.float32)        # one-sided negative
    w[5, :] = np.float32(65504.0 * 15 / 2) * np.where(np.arange(64) % 2, 1, -1)   # largest legal range
    check_asym(B, w, 8)
    check_asym(B, w, 32)


def test_range_error_counter(B):
    w = np.zeros((4, 64), np.float32)
    w[1, 3] = 1e6
    w[1, 40] = -1e6
    w[3, 9] = 2e6
    *_, sc, zr, errs = gpu_quantize_asym(B, w, 32, with_errors=True)
    assert errs == 3
    with pytest.raises(ValueError):
        O.quantize_w4_asym_group(w, 32)
    assert sc.view(np.uint16)[1, 0] == 0x7BFF


def test_unpack_matches_oracle(B):
    import torch
    rng = np.random.default_rng(3)
    words = rng.integers(0, 2 ** 32, size=(37, 24), dtype=np.uint64).astype(np.uint32)
    for scheme, ref in ((B.QAIL_W4_ASYM_GROUP, O.unpack_nibbles_u4(words, 192)),
                        (B.QAIL_W4_SYM_CHANNEL, O.unpack_nibbles_s4(words, 192))):
        codes = torch.zeros(37 * 192, dtype=torch.int8, device="cuda")
        B.qail_unpack_weights(37, 192, 64, scheme, dev(words), codes)
        got = host(codes, ref.dtype).reshape(37, 192)
        assert np.array_equal(got, ref)


def test_sym_channel_bit_exact(B):
    import torch
    for shape, seed in ((synth.ConvShape("a", 1, 8, 8, 64, 64, 3, 3, 1, 1), 5),
                        (synth.ConvShape("b", 1, 8, 8, 8, 5, 1, 1, 1, 0), 6),
                        (synth.ConvShape("c", 1, 8, 8, 512, 17, 3, 3, 1, 1), 7)):
        w = synth.conv_weight(shape, seed)
        if shape.name == "b":
            w[2] = 0                                        # all-zero channel
            w[3, 0, 0, :] = [7, -7, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5]
        q, s = O.quantize_w4_sym_channel(w)
        ref = O.pack_nibbles(q.reshape(shape.Cout, -1))
        qb, sb, zb = B.qail_packed_sizes(shape.Cout, shape.K, 0, B.QAIL_W4_SYM_CHANNEL)
        assert zb == 0
        qw = torch.zeros(qb // 4, dtype=torch.int32, device="cuda")
        sc = torch.zeros(sb // 4, dtype=torch.float32, device="cuda")
        B.qail_quantize_weights(dev(w), 0, B.QAIL_W4_SYM_CHANNEL, qw, sc, None)
        assert np.array_equal(host(sc, np.float32).view(np.uint32), s.view(np.uint32))
        assert np.array_equal(host(qw, np.uint32).reshape(ref.shape), ref)


def test_activation_scale_and_codes_bit_exact(B):
    import torch
    shape = synth.ConvShape("a", 2, 28, 28, 128, 128, 3, 3, 1, 1)
    a = synth.conv_activation(shape, 11)
    s_ref = O.act_scale_u4(a)
    ref = O.pack_nibbles(O.quantize_act_u4(a, s_ref))
    s_a = torch.full((1,), -5.0, dtype=torch.float32, device="cuda")
    out = torch.zeros(a.size // 8, dtype=torch.int32, device="cuda")
    B.qail_act_scale_u4(dev(a), s_a)
    B.qail_quantize_act_u4(dev(a), s_a, out)
    assert host(s_a, np.uint32)[0] == np.float32(s_ref).view(np.uint32)
    assert np.array_equal(host(out, np.uint32).reshape(ref.shape), ref)
    # no positive element -> scale 1; empty tensor -> scale 1, nothing written
    neg = -np.abs(a[:1, :2, :2, :8])
    B.qail_act_scale_u4(dev(neg), s_a)
    assert float(s_a.item()) == 1.0
    B.qail_act_scale_u4(torch.zeros(0, dtype=torch.float32, device="cuda"), s_a)
    assert float(s_a.item()) == 1.0
    B.qail_quantize_act_u4(torch.zeros(0, dtype=torch.float32, device="cuda"), s_a, out)
    # ties and clamps with a scale of exactly 1
    v = np.array([0, 15, 0.5, 1.5, 2.5, -3.0, 14.5, 99.0], np.float32)
    one = torch.ones(1, dtype=torch.float32, device="cuda")
    o2 = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.qail_quantize_act_u4(dev(v), one, o2)
    assert host(o2, np.uint32)[0] == O.pack_nibbles(O.quantize_act_u4(v, 1.0))[0]
