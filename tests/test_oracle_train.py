"""Pins of the training-side oracle functions (no GPU)."""
import numpy as np

from oracle import qail_oracle as O
from paper_2412_01034_amd import synth


def test_fake_quant_w4_is_quantise_then_dequantise_and_idempotent_on_full_range_groups():
    w = synth.llm_weight(8, 256, 3)
    wh = O.fake_quant_w4_group(w, 64)
    q, s, z = O.quantize_w4_asym_group(w, 64)
    assert wh.dtype == np.float32
    assert np.array_equal(wh.astype(np.float64), O.dequantize_w4_asym_group(q, s, z, 64))     # exact in float32
    sf = np.repeat(s.astype(np.float64), 64, axis=1)
    assert np.all(np.abs(w - wh) <= sf * (0.5 + 2.0 ** -20))
    # groups whose codes reach both 0 and 15 keep their scale and zero, so a second pass changes nothing
    full = (q.reshape(8, 4, 64).min(axis=2) == 0) & (q.reshape(8, 4, 64).max(axis=2) == 15)
    wh2 = O.fake_quant_w4_group(wh, 64)
    assert full.any()
    assert np.array_equal(wh2.reshape(8, 4, 64)[full], wh.reshape(8, 4, 64)[full])


def test_lsq_forward_hand_worked_and_matches_the_activation_quantiser():
    v = np.array([0.0, 0.3, 0.5, 0.75, 1.25, -0.6, 10.0, -10.0], np.float32)
    out = O.lsq_fake_quant_fwd(v, 0.5, -8, 7)
    #   v/s  =  0, 0.6, 1, 1.5, 2.5, -1.2, 20, -20  ->  0, 1, 1, 2 (tie, even), 2 (tie, even), -1, 7, -8
    assert out.tolist() == [0.0, 0.5, 0.5, 1.0, 1.0, -0.5, 3.5, -4.0]
    a = np.abs(np.random.default_rng(0).standard_normal(1000)).astype(np.float32)
    s = O.act_scale_u4(a)
    assert np.array_equal(O.lsq_fake_quant_fwd(a, s, 0, 15), O.quantize_act_u4(a, s).astype(np.float32) * s)
    # idempotent: codes times step go back to the same codes
    assert np.array_equal(O.lsq_fake_quant_fwd(out, 0.5, -8, 7), out)


def test_lsq_backward_hand_worked():
    v = np.array([0.3, 0.75, -0.6, 10.0, -10.0, 3.5], np.float32)
    dout = np.array([1.0, 2.0, -1.0, 0.5, 4.0, 3.0], np.float32)
    dv, ds = O.lsq_fake_quant_bwd(v, 0.5, -8, 7, dout, 0.25)
    #   v/s = 0.6, 1.5, -1.2, 20 (above), -20 (below), 7 (inside, on the edge)
    assert dv.tolist() == [1.0, 2.0, -1.0, 0.0, 0.0, 3.0]
    #   t  = 1-0.6, 2-1.5, -1+1.2, 7, -8, 0
    want = 0.25 * (1.0 * 0.4 + 2.0 * 0.5 + (-1.0) * 0.2 + 0.5 * 7 + 4.0 * (-8) + 3.0 * 0.0)
    assert abs(ds - want) < 1e-6
    # the step gradient is the derivative of v_hat with rint frozen: compare with a difference
    # quotient of  clamp(n, qn, qp) * s  at fixed integers n = rint(v/s) ... plus the STE term -v/s
    rng = np.random.default_rng(1)
    v = rng.standard_normal(200).astype(np.float32)
    dout = rng.standard_normal(200).astype(np.float32)
    s = np.float32(0.2)
    _, ds = O.lsq_fake_quant_bwd(v, s, -8, 7, dout, 1.0)
    r = v.astype(np.float64) / np.float64(s)
    inside = (r >= -8) & (r <= 7)
    t = np.where(inside, np.rint(r) - r, np.clip(r, -8, 7))
    assert abs(ds - float((dout * t).sum())) < 1e-4


def test_qbc_loss_closed_form_and_gradient():
    lq = np.array([[3.0, 4.0], [1.0, 1.0], [0.0, 2.0]])
    lf = np.array([[0.0, 0.0], [1.0, 1.0], [0.0, -1.0]])
    loss, grad = O.qbc_loss(lq, lf)
    assert abs(loss - (5.0 + 0.0 + 3.0) / 3.0) < 1e-15          # 3-4-5 triangle, identical rows, one axis
    assert np.allclose(grad, [[0.2, 4.0 / 15.0], [0.0, 0.0], [0.0, 1.0 / 3.0]])
    # central differences on random logits
    rng = np.random.default_rng(2)
    a, b = rng.standard_normal((5, 7)), rng.standard_normal((5, 7))
    _, g = O.qbc_loss(a, b)
    num = np.zeros_like(a)
    h = 1e-6
    for i in range(5):
        for j in range(7):
            ap, am = a.copy(), a.copy()
            ap[i, j] += h
            am[i, j] -= h
            num[i, j] = (O.qbc_loss(ap, b)[0] - O.qbc_loss(am, b)[0]) / (2 * h)
    assert np.allclose(g, num, atol=1e-8)
    assert O.qbc_loss(a, a)[0] == 0.0
