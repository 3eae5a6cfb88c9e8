"""GPU parity of the training-side operators against the CPU oracle."""
import numpy as np
import pytest

from oracle import qail_oracle as O
from paper_2412_01034_amd import synth
from tests.helpers import dev, ensure_built, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    return ensure_built()


@pytest.mark.parametrize("N,K,g", [(64, 1024, 128), (33, 256, 64), (5, 4096, 4096), (300, 64, 8), (40, 768, 192),
                                   (16, 2048, 256), (9, 1536, 512),
                                   (3000, 2048, 128)])   # more groups than one sweep of the grid
def test_fake_quant_w4_bit_exact(B, N, K, g):
    import torch
    w = synth.llm_weight(N, K, 7 + N, outlier_frac=0.01)
    w[0, :g] = 0
    out = torch.full((N * K,), float("nan"), dtype=torch.float32, device="cuda")
    B.qail_fake_quant_w4(dev(w), g, out)
    torch.cuda.synchronize()
    assert np.array_equal(host(out, np.float32).reshape(N, K), O.fake_quant_w4_group(w, g))


@pytest.mark.parametrize("qn,qp", [(-8, 7), (0, 15), (-128, 127)])
def test_lsq_forward_and_backward(B, qn, qp):
    import torch
    rng = np.random.default_rng(qp)
    n = 100003      # not a multiple of 4: the last three values take the scalar path
    v = (rng.standard_normal(n) * 2).astype(np.float32)
    v[:6] = [0.0, 0.25, 0.75, -0.25, 1e9, -1e9]           # ties and both clamps with s = 0.5
    dout = rng.standard_normal(n).astype(np.float32)
    for s in (np.float32(0.5), np.float32(0.3137)):
        sd = dev(np.array([s], np.float32))
        vd, dd = dev(v), dev(dout)
        out = torch.empty(n, dtype=torch.float32, device="cuda")
        B.qail_lsq_forward(vd, sd, qn, qp, out)
        dv = torch.empty(n, dtype=torch.float32, device="cuda")
        ds = torch.zeros(1, dtype=torch.float32, device="cuda")
        ws = torch.empty(B.qail_lsq_backward_workspace(), dtype=torch.uint8, device="cuda")
        gs = 1.0 / np.sqrt(n * max(qp, 1))
        B.qail_lsq_backward(vd, dd, sd, qn, qp, gs, dv, ds, ws)
        ds2 = torch.zeros(1, dtype=torch.float32, device="cuda")
        B.qail_lsq_backward(vd, dd, sd, qn, qp, gs, dv, ds2, ws)
        torch.cuda.synchronize()
        assert np.array_equal(host(out, np.float32), O.lsq_fake_quant_fwd(v, s, qn, qp))
        dv_ref, ds_ref = O.lsq_fake_quant_bwd(v, s, qn, qp, dout, gs)
        assert np.array_equal(host(dv, np.float32), dv_ref)
        # fp32 partial sums against the float64 sum: relative to the sum of magnitudes
        r = v / s
        t = np.where((r >= qn) & (r <= qp), np.rint(r) - r, np.clip(r, qn, qp)).astype(np.float64)
        mag = gs * float(np.abs(dout.astype(np.float64) * t).sum())
        assert abs(float(ds.item()) - ds_ref) <= 1e-5 * mag
        assert ds.item() == ds2.item()                       # fixed reduction order


@pytest.mark.parametrize("Bn,D", [(1, 7), (64, 256), (300, 1000), (9, 32000), (5, 32768), (3, 32772), (4, 4098)])
def test_qbc_loss(B, Bn, D):
    import torch
    rng = np.random.default_rng(Bn)
    lq = rng.standard_normal((Bn, D)).astype(np.float32)
    lf = rng.standard_normal((Bn, D)).astype(np.float32)
    if Bn > 1:
        lf[1] = lq[1]                                        # a row with zero distance
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    grad = torch.full((Bn * D,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(Bn, 4), dtype=torch.float32, device="cuda")
    B.qail_qbc_loss(dev(lq), dev(lf), loss, grad.view(Bn, D), ws)
    torch.cuda.synchronize()
    l_ref, g_ref = O.qbc_loss(lq, lf)
    assert abs(float(loss.item()) - l_ref) <= 2e-6 * l_ref + 1e-12
    g = host(grad, np.float32).reshape(Bn, D).astype(np.float64)
    assert np.all(np.abs(g - g_ref) <= 2e-6 * np.abs(g_ref).max() + 1e-12)
    if Bn > 1:
        assert not g[1].any()


def test_training_operators_at_the_benchmark_sizes(B):
    """The sizes bench.py times: fake quantisation of a 12288 x 4096 matrix in groups of 128 (bit for
    bit), the learned-step quantiser over the same 50 M values (forward and masked gradient bit for
    bit, step gradient against the float64 sum), the QBC loss and gradient of 1024 x 32000 logits."""
    import torch
    N, K, g = 12288, 4096, 128
    w = synth.llm_weight(N, K, 4242, outlier_frac=0.01)
    wd = dev(w)
    out = torch.empty(N * K, dtype=torch.float32, device="cuda")
    B.qail_fake_quant_w4(wd, g, out)
    torch.cuda.synchronize()
    assert np.array_equal(host(out, np.float32).reshape(N, K), O.fake_quant_w4_group(w, g))
    # learned-step quantiser on the same values
    s = np.float32(0.004)
    sd = dev(np.array([s], np.float32))
    B.qail_lsq_forward(wd.view(-1), sd, -8, 7, out)
    torch.cuda.synchronize()
    v = w.reshape(-1)
    assert np.array_equal(host(out, np.float32), O.lsq_fake_quant_fwd(v, s, -8, 7))
    rng = np.random.default_rng(4243)
    dout = rng.standard_normal(v.size).astype(np.float32)
    dv = torch.empty(v.size, dtype=torch.float32, device="cuda")
    ds = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(B.qail_lsq_backward_workspace(), dtype=torch.uint8, device="cuda")
    gs = 1.0 / np.sqrt(v.size * 7)
    B.qail_lsq_backward(wd.view(-1), dev(dout), sd, -8, 7, gs, dv, ds, ws)
    torch.cuda.synchronize()
    dv_ref, ds_ref = O.lsq_fake_quant_bwd(v, s, -8, 7, dout, gs)
    assert np.array_equal(host(dv, np.float32), dv_ref)
    r = v / s
    t = np.where((r >= -8) & (r <= 7), np.rint(r) - r, np.clip(r, -8, 7)).astype(np.float64)
    mag = gs * float(np.abs(dout.astype(np.float64) * t).sum())
    assert abs(float(ds.item()) - ds_ref) <= 1e-5 * mag
    del out, dv, wd
    # QBC
    Bn, D = 1024, 32000
    lq = rng.standard_normal((Bn, D)).astype(np.float32)
    lf = (lq + 0.1 * rng.standard_normal((Bn, D))).astype(np.float32)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    grad = torch.empty(Bn * D, dtype=torch.float32, device="cuda")
    wsq = torch.empty(Bn, dtype=torch.float32, device="cuda")
    B.qail_qbc_loss(dev(lq), dev(lf), loss, grad.view(Bn, D), wsq)
    torch.cuda.synchronize()
    l_ref, g_ref = O.qbc_loss(lq, lf)
    assert abs(float(loss.item()) - l_ref) <= 2e-6 * l_ref
    gh = host(grad, np.float32).reshape(Bn, D).astype(np.float64)
    assert np.all(np.abs(gh - g_ref) <= 2e-6 * np.abs(g_ref).max())
