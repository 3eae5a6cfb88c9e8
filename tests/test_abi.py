"""CPU-side checks of the C ABI: the library loads, exports every function the
header declares, and reports argument errors before touching the GPU."""
import ctypes

import pytest

from tests.helpers import ensure_built, header_functions


@pytest.fixture(scope="module")
def B():
    return ensure_built()


def test_exports_match_header(B):
    L = B.lib()
    names = header_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(L, n), n
    assert B.qail_version() >= 100
    assert B.status_string(0) == "ok"
    for s in range(-6, 0):
        assert B.status_string(s) not in ("ok", "unknown status")


def test_packed_sizes(B):
    # K=11008, g=128: 86 groups -> 11 zero-point words per row
    assert B.qail_packed_sizes(4096, 11008, 128, B.QAIL_W4_ASYM_GROUP) == (4096 * 1376 * 4, 4096 * 86 * 2, 4096 * 11 * 4)
    assert B.qail_packed_sizes(512, 512, 64, B.QAIL_W4_ASYM_GROUP) == (512 * 64 * 4, 512 * 8 * 2, 512 * 4)
    assert B.qail_packed_sizes(64, 576, 0, B.QAIL_W4_SYM_CHANNEL) == (64 * 72 * 4, 64 * 4, 0)
    total = 0
    for n, k in ((12288, 4096), (4096, 4096), (22016, 4096), (4096, 11008)):
        total += sum(B.qail_packed_sizes(n, k, 128, B.QAIL_W4_ASYM_GROUP))
    assert abs(total - 105.14e6) < 0.2e6          # one decoder layer
    for bad in ((0, 64, 64), (4, 60, 8), (4, 64, 12), (4, 64, 48), (4, 0, 8)):
        with pytest.raises(B.QailError) as e:
            B.qail_packed_sizes(*bad, B.QAIL_W4_ASYM_GROUP)
        assert e.value.status == B.QAIL_ERR_SHAPE
    with pytest.raises(B.QailError) as e:
        B.qail_packed_sizes(4, 64, 8, 7)
    assert e.value.status == B.QAIL_ERR_UNSUPPORTED


def test_argument_errors_are_reported_without_a_gpu(B):
    L = B.lib()
    d = B.qail_wdesc(16, 64, 32, B.QAIL_W4_ASYM_GROUP)
    ok, odd = 0x10000, 0x10008
    st = L.qail_quantize_weights(ctypes.byref(d), None, ok, ok, ok, None, None)
    assert st == B.QAIL_ERR_NULL
    assert L.qail_quantize_weights(ctypes.byref(d), ok, ok, ok, None, None, None) == B.QAIL_ERR_NULL
    assert L.qail_quantize_weights(ctypes.byref(d), odd, ok, ok, ok, None, None) == B.QAIL_ERR_ALIGN
    assert L.qail_quantize_weights(None, ok, ok, ok, ok, None, None) == B.QAIL_ERR_NULL
    assert L.qail_unpack_weights(ctypes.byref(d), ok, None, None) == B.QAIL_ERR_NULL
    assert L.qail_w4a16_linear(ctypes.byref(d), ok, ok, ok, ok, ok, 0, None, 0, None) == B.QAIL_ERR_SHAPE
    assert L.qail_w4a16_linear(ctypes.byref(d), ok, ok, ok, None, ok, 1, None, 0, None) == B.QAIL_ERR_NULL
    assert L.qail_w4a16_linear(ctypes.byref(d), ok, ok, odd, ok, ok, 1, None, 0, None) == B.QAIL_ERR_ALIGN
    ds = B.qail_wdesc(16, 64, 32, B.QAIL_W4_SYM_CHANNEL)
    assert L.qail_w4a16_linear(ctypes.byref(ds), ok, ok, ok, ok, ok, 1, None, 0, None) == B.QAIL_ERR_UNSUPPORTED
    assert L.qail_w4a16_linear_batch(None, 0, 1, None, 0, None) == B.QAIL_OK
    assert L.qail_w4a16_linear_batch(None, 2, 1, None, 0, None) == B.QAIL_ERR_NULL
    assert L.qail_w4a16_linear_batch(None, -1, 1, None, 0, None) == B.QAIL_ERR_SHAPE
    assert L.qail_quantize_act_u4(ok, 12, ok, ok, None) == B.QAIL_ERR_SHAPE
    assert L.qail_quantize_act_u4(None, 0, None, None, None) == B.QAIL_OK
    assert L.qail_act_scale_u4(ok, 8, None, None) == B.QAIL_ERR_NULL
    c = B.qail_conv_desc(1, 4, 4, 8, 4, 3, 3, 1, 1)
    assert L.qail_w4a4_gemm(ctypes.byref(c), ok, ok, None, None, None, None, None, 0, None) == B.QAIL_ERR_NULL
    assert L.qail_w4a4_gemm(ctypes.byref(c), ok, ok, None, None, ok, ok, None, 0, None) == B.QAIL_ERR_NULL
    assert L.qail_w4a4_gemm(ctypes.byref(c), ok, odd, ok, None, None, None, None, 0, None) == B.QAIL_ERR_ALIGN
    bad = B.qail_conv_desc(1, 4, 4, 12, 4, 3, 3, 1, 1)
    assert L.qail_w4a4_gemm(ctypes.byref(bad), ok, ok, ok, None, None, None, None, 0, None) == B.QAIL_ERR_SHAPE
    bad = B.qail_conv_desc(1, 2, 2, 8, 4, 5, 5, 1, 0)
    assert L.qail_w4a4_gemm(ctypes.byref(bad), ok, ok, ok, None, None, None, None, 0, None) == B.QAIL_ERR_SHAPE
    # fused 4-bit output: argument order (d, a, w, scale, bias, s_out, res_u4, res_scale, res_f32, out, ws, n, stream)
    c8 = B.qail_conv_desc(1, 4, 4, 8, 8, 3, 3, 1, 1)
    f = L.qail_w4a4_conv_u4
    assert f(ctypes.byref(c8), ok, ok, ok, ok, 0.5, None, 0.0, None, None, None, 0, None) == B.QAIL_ERR_NULL
    assert f(ctypes.byref(c8), ok, ok, None, ok, 0.5, None, 0.0, None, ok, None, 0, None) == B.QAIL_ERR_NULL
    assert f(ctypes.byref(c), ok, ok, ok, ok, 0.5, None, 0.0, None, ok, None, 0, None) == B.QAIL_ERR_SHAPE   # Cout = 4
    assert f(ctypes.byref(c8), ok, ok, ok, ok, 0.0, None, 0.0, None, ok, None, 0, None) == B.QAIL_ERR_SHAPE
    assert f(ctypes.byref(c8), ok, ok, ok, ok, float("nan"), None, 0.0, None, ok, None, 0, None) == B.QAIL_ERR_SHAPE
    assert f(ctypes.byref(c8), ok, ok, ok, ok, 0.5, ok, 0.1, ok, ok, None, 0, None) == B.QAIL_ERR_SHAPE    # two shortcuts
    assert f(ctypes.byref(c8), ok, ok, ok, ok, 0.5, ok, -1.0, None, ok, None, 0, None) == B.QAIL_ERR_SHAPE
    assert f(ctypes.byref(c8), ok, ok, ok, ok, 0.5, odd, 0.1, None, ok, None, 0, None) == B.QAIL_ERR_ALIGN
    # several convolutions per launch: each item obeys the rules of the single call of its kind
    f = L.qail_w4a4_conv_batch

    def conv_item(desc, **kw):
        it = B.qail_conv_item()
        it.d = desc
        for k in ("a_u4", "w_s4", "scale", "bias", "acc_out", "y_out", "out_u4", "res_u4", "res_f32"):
            setattr(it, k, kw.get(k))
        it.s_out = kw.get("s_out", 0.0)
        it.res_scale = kw.get("res_scale", 0.0)
        return (B.qail_conv_item * 1)(it)
    assert f(None, 1, None) == B.QAIL_ERR_NULL
    good = conv_item(c8, a_u4=ok, w_s4=ok, scale=ok, bias=ok, out_u4=ok, s_out=0.5)
    assert f(good, 0, None) == B.QAIL_ERR_SHAPE and f(good, 65, None) == B.QAIL_ERR_SHAPE
    assert f(conv_item(c8, a_u4=ok, w_s4=ok), 1, None) == B.QAIL_ERR_NULL                      # no output at all
    assert f(conv_item(c8, a_u4=ok, w_s4=ok, y_out=ok), 1, None) == B.QAIL_ERR_NULL            # y without scale
    assert f(conv_item(c8, a_u4=ok, w_s4=ok, scale=ok, bias=ok, out_u4=ok, acc_out=ok, s_out=0.5), 1, None) == B.QAIL_ERR_SHAPE
    assert f(conv_item(c8, a_u4=ok, w_s4=ok, acc_out=ok, res_u4=ok), 1, None) == B.QAIL_ERR_SHAPE   # shortcut without fused output
    assert f(conv_item(c8, a_u4=ok, w_s4=ok, scale=ok, bias=ok, out_u4=ok, s_out=0.0), 1, None) == B.QAIL_ERR_SHAPE
    assert f(conv_item(c, a_u4=ok, w_s4=ok, scale=ok, bias=ok, out_u4=ok, s_out=0.5), 1, None) == B.QAIL_ERR_SHAPE   # Cout = 4
    assert f(conv_item(c8, a_u4=ok, w_s4=odd, acc_out=ok), 1, None) == B.QAIL_ERR_ALIGN
    assert f(conv_item(bad, a_u4=ok, w_s4=ok, acc_out=ok), 1, None) == B.QAIL_ERR_SHAPE
    # low-rank adapters: rank must be a multiple of 8 in [8, 64], factors present and aligned
    it = B.qail_w4a16_item(d, ok, ok, ok, ok, ok)
    its = (B.qail_w4a16_item * 1)(it)
    f = L.qail_w4a16_linear_lora_batch
    for bad_r in (0, 4, 12, 72):
        lo = (B.qail_lora * 1)(B.qail_lora(ok, ok, bad_r, 1.0))
        assert f(its, lo, 1, 1, ok, 1 << 20, None) == B.QAIL_ERR_SHAPE
    lo = (B.qail_lora * 1)(B.qail_lora(None, ok, 32, 1.0))
    assert f(its, lo, 1, 1, ok, 1 << 20, None) == B.QAIL_ERR_NULL
    lo = (B.qail_lora * 1)(B.qail_lora(ok, odd, 32, 1.0))
    assert f(its, lo, 1, 1, ok, 1 << 20, None) == B.QAIL_ERR_ALIGN
    lo = (B.qail_lora * 1)(B.qail_lora(ok, ok, 32, float("inf")))
    assert f(its, lo, 1, 1, ok, 1 << 20, None) == B.QAIL_ERR_SHAPE
    lo = (B.qail_lora * 1)(B.qail_lora(ok, ok, 32, 1.0))
    assert f(its, lo, 1, 1, None, 0, None) == B.QAIL_ERR_WORKSPACE          # the down-projection needs room
    assert f(its, None, 1, 1, ok, 1 << 20, None) == B.QAIL_ERR_NULL
    assert f(its, lo, 0, 1, None, 0, None) == B.QAIL_OK
    # dependent linears in one launch: a status word, arrival counters and a flag per block (two blocks
    # on each of 256 CUs when no GPU can be asked); every item must be
    # one the M = 1 stream takes
    szc = ctypes.c_size_t(0)
    assert L.qail_w4a16_chain_workspace(its, 1, ctypes.byref(szc)) == B.QAIL_OK and szc.value == (64 + 512) * 4
    its40 = (B.qail_w4a16_item * 40)(*([it] * 40))
    assert L.qail_w4a16_chain_workspace(its40, 40, ctypes.byref(szc)) == B.QAIL_OK and szc.value == (64 + 512) * 4
    assert L.qail_w4a16_chain_workspace(its, 1, None) == B.QAIL_ERR_NULL
    assert L.qail_w4a16_chain_workspace(None, 1, ctypes.byref(szc)) == B.QAIL_ERR_NULL
    assert L.qail_w4a16_linear_chain(its, 0, None, 0, None) == B.QAIL_OK
    assert L.qail_w4a16_linear_chain(its, -1, None, 0, None) == B.QAIL_ERR_SHAPE
    assert L.qail_w4a16_linear_chain(None, 1, ok, 1 << 20, None) == B.QAIL_ERR_NULL
    assert L.qail_w4a16_linear_chain(its, 1, None, 0, None) == B.QAIL_ERR_WORKSPACE
    assert L.qail_w4a16_linear_chain(its, 1, ok, 100, None) == B.QAIL_ERR_WORKSPACE
    assert L.qail_w4a16_linear_chain(its, 1, odd, 1 << 20, None) == B.QAIL_ERR_ALIGN
    dbig = B.qail_wdesc(16, 16384, 128, B.QAIL_W4_ASYM_GROUP)            # K beyond the streaming kernel
    itb = (B.qail_w4a16_item * 1)(B.qail_w4a16_item(dbig, ok, ok, ok, ok, ok))
    assert L.qail_w4a16_linear_chain(itb, 1, ok, 1 << 20, None) == B.QAIL_ERR_UNSUPPORTED
    assert L.qail_w4a16_chain_workspace(itb, 1, ctypes.byref(szc)) == B.QAIL_ERR_UNSUPPORTED
    # 8-bit weight-only linear: M > 1 on the matrix cores needs the workspace its query reports
    d8 = B.qail_wdesc(256, 1024, 128, B.QAIL_W8_SYM_GROUP)
    sz8 = ctypes.c_size_t(99)
    assert L.qail_w8a16_workspace(ctypes.byref(d8), 1, ctypes.byref(sz8)) == B.QAIL_OK and sz8.value == 0
    assert L.qail_w8a16_workspace(ctypes.byref(d8), 40, ctypes.byref(sz8)) == B.QAIL_OK and sz8.value > 0
    assert L.qail_w8a16_workspace(ctypes.byref(d8), 0, ctypes.byref(sz8)) == B.QAIL_ERR_SHAPE
    assert L.qail_w8a16_workspace(ctypes.byref(d8), 40, None) == B.QAIL_ERR_NULL
    assert L.qail_w8a16_workspace(ctypes.byref(d), 40, ctypes.byref(sz8)) == B.QAIL_ERR_UNSUPPORTED   # a 4-bit descriptor
    assert L.qail_w8a16_linear(ctypes.byref(d8), ok, ok, ok, ok, 40, None, 0, None) == B.QAIL_ERR_WORKSPACE
    assert L.qail_w8a16_linear(ctypes.byref(d8), ok, ok, ok, ok, 40, odd, 1 << 30, None) == B.QAIL_ERR_ALIGN
    assert L.qail_w8a16_linear(ctypes.byref(d8), ok, None, ok, ok, 40, ok, 1 << 30, None) == B.QAIL_ERR_NULL
    assert L.qail_w8a16_linear(ctypes.byref(d8), ok, ok, ok, ok, 0, ok, 1 << 30, None) == B.QAIL_ERR_SHAPE
    it8 = (B.qail_w8a16_item * 2)(B.qail_w8a16_item(d8, ok, ok, ok, ok), B.qail_w8a16_item(d8, ok, ok, ok, ok))
    assert L.qail_w8a16_batch_workspace(it8, 2, 40, ctypes.byref(sz8)) == B.QAIL_OK and sz8.value > 0
    assert L.qail_w8a16_batch_workspace(it8, 2, 1, ctypes.byref(sz8)) == B.QAIL_OK and sz8.value == 0
    assert L.qail_w8a16_linear_batch(it8, 2, 40, None, 0, None) == B.QAIL_ERR_WORKSPACE
    assert L.qail_w8a16_linear_batch(it8, 0, 40, None, 0, None) == B.QAIL_OK
    assert L.qail_w8a16_linear_batch(None, 2, 40, ok, 1 << 30, None) == B.QAIL_ERR_NULL
    szl = ctypes.c_size_t(0)
    assert L.qail_w4a16_lora_workspace(its, lo, 1, 3, ctypes.byref(szl)) == B.QAIL_OK and szl.value == 768
    assert L.qail_w4a16_lora_workspace(its, lo, 1, 3, None) == B.QAIL_ERR_NULL
    # the adapter kernels index the rows of x with the grid's y axis: larger batches are refused
    # before anything is launched, by the size query and by the call
    assert L.qail_w4a16_lora_workspace(its, lo, 1, 65536, ctypes.byref(szl)) == B.QAIL_ERR_UNSUPPORTED
    assert f(its, lo, 1, 65536, ok, 1 << 40, None) == B.QAIL_ERR_UNSUPPORTED
    sz = ctypes.c_size_t(99)
    assert L.qail_w4a4_workspace(ctypes.byref(c), ctypes.byref(sz)) == B.QAIL_OK
    assert L.qail_w4a16_workspace(ctypes.byref(d), 1, ctypes.byref(sz)) == B.QAIL_OK
    assert L.qail_w4a16_workspace(ctypes.byref(d), 0, ctypes.byref(sz)) == B.QAIL_ERR_SHAPE
    # the matrix-core GEMM (M > 16) needs a workspace: fp16 copy of x padded to 128 rows and
    # 128 columns, one float per padded row, one per output column, rounded up to 256 bytes;
    # then two tile-shaped fp32 slots (here 32 x 256) per block of the largest grid (one block per
    # CU; 256 CUs on the target, which is also what the library assumes when it sees no device)
    dg = B.qail_wdesc(300, 4096 + 64, 64, B.QAIL_W4_ASYM_GROUP)
    assert L.qail_w4a16_workspace(ctypes.byref(dg), 1, ctypes.byref(sz)) == B.QAIL_OK and sz.value == 0
    d7 = B.qail_wdesc(4096, 4096, 128, B.QAIL_W4_ASYM_GROUP)   # M <= 16 streams without a workspace
    assert L.qail_w4a16_workspace(ctypes.byref(d7), 16, ctypes.byref(sz)) == B.QAIL_OK and sz.value == 0
    assert L.qail_w4a16_workspace(ctypes.byref(dg), 17, ctypes.byref(sz)) == B.QAIL_OK
    want = 128 * 4224 * 2 + 128 * 4 + 320 * 4
    assert sz.value == (want + 255) // 256 * 256 + 2 * 256 * 32 * 256 * 4
    assert L.qail_w4a16_linear(ctypes.byref(dg), ok, ok, ok, ok, ok, 17, None, 0, None) == B.QAIL_ERR_WORKSPACE
    assert L.qail_w4a16_linear(ctypes.byref(dg), ok, ok, ok, ok, ok, 17, ok, sz.value - 1, None) == B.QAIL_ERR_WORKSPACE
    assert L.qail_w4a16_linear(ctypes.byref(dg), ok, ok, ok, ok, ok, 17, ok + 16, sz.value, None) == B.QAIL_ERR_ALIGN


def test_batch_workspace_is_host_arithmetic(B):
    """Linears of the matrix-core path that share launches (up to 8) keep their prepared activations
    side by side and share one pool of slots; runs that other kernels interrupt, and launches after
    the eighth linear, reuse the space.  All of it is computed on the host, no GPU needed."""
    L = B.lib()
    ok = ctypes.c_void_p(0x1000)

    def items(shapes):
        arr = (B.qail_w4a16_item * len(shapes))()
        for i, (N, K, g) in enumerate(shapes):
            arr[i].d = B.qail_wdesc(N, K, g, B.QAIL_W4_ASYM_GROUP)
            arr[i].qweight = arr[i].scales = arr[i].zeros = arr[i].x = arr[i].y = 0x1000
        return arr

    def single(N, K, g, M):
        sz = ctypes.c_size_t(0)
        assert L.qail_w4a16_workspace(ctypes.byref(B.qail_wdesc(N, K, g, B.QAIL_W4_ASYM_GROUP)), M, ctypes.byref(sz)) == B.QAIL_OK
        return sz.value

    def batch(shapes, M):
        sz = ctypes.c_size_t(0)
        assert L.qail_w4a16_batch_workspace(items(shapes), len(shapes), M, ctypes.byref(sz)) == B.QAIL_OK
        return sz.value

    def head(N, K, M):     # fp16 x padded to 128 rows x 128 columns, row scales, per-column powers of two
        return (128 * ((M + 127) // 128) * ((K + 127) // 128 * 128) * 2 + 128 * ((M + 127) // 128) * 4
                + (N + 63) // 64 * 64 * 4 + 255) // 256 * 256

    M = 40                                    # 64-row tiles
    pool = 2 * 256 * 64 * 256 * 4             # two slots of 64 x 256 floats per block of the grid
    a, b_, c = (300, 4096, 128), (1000, 2048, 64), (96, 11008, 128)
    assert single(*a, M) == head(a[0], a[1], M) + pool
    assert batch([a], M) == single(*a, M)
    assert batch([a, b_, c], M) == sum(head(s[0], s[1], M) for s in (a, b_, c)) + pool
    assert batch([(64, 256, 64)], M) == head(64, 256, M) + pool // 2          # N <= 128: narrow slots
    # nine linears: the ninth goes out after the first eight and reuses their space
    assert batch([a] * 9, M) == 8 * head(a[0], a[1], M) + pool
    # a linear the matrix-core path does not take (K not a multiple of 64) splits the run
    odd = (64, 40, 8)
    assert batch([a, odd, b_], M) == max(single(*a, M), single(*b_, M))
    assert batch([a, c], 16) == 0 and batch([a, b_, c], 1) == 0               # streaming kernels need none
    assert batch([a, b_, c], 16) == single(*b_, 16) > 0                       # groups of 64 at M = 16: matrix cores
    assert batch([], 5) == 0
    # the batch call checks against the same figure
    its = items([a, b_])
    need = batch([a, b_], M)
    f = L.qail_w4a16_linear_batch
    assert f(its, 2, M, ok, need - 1, None) == B.QAIL_ERR_WORKSPACE
    assert f(its, 2, M, None, 0, None) == B.QAIL_ERR_WORKSPACE
    assert f(its, 2, M, ctypes.c_void_p(0x1010), need, None) == B.QAIL_ERR_ALIGN


def test_binding_refuses_host_tensors(B):
    import torch
    t = torch.zeros(16, 64)
    with pytest.raises(ValueError):
        B.qail_quantize_weights(t, 32, B.QAIL_W4_ASYM_GROUP, torch.zeros(128, dtype=torch.int32),
                                torch.zeros(32, dtype=torch.float16), torch.zeros(16, dtype=torch.int32))
