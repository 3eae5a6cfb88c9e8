"""The entry point that allocates nothing (qail_w4a16_linear_lora_batch_static): called through
the C ABI with raw pointers, its output must equal that of qail_w4a16_linear_lora_batch bit for
bit (same kernels, the workspace replaced by the library's built-in scratch), on two calls in a
row, the second with a smaller input, so that what the first left in the scratch is there when
the second runs."""
import ctypes

import numpy as np
import pytest

from oracle import qail_oracle as O
from paper_2412_01034_amd import synth
from tests.helpers import dev, ensure_built, host, w4a16_norm_err

pytestmark = pytest.mark.gpu


def _case(B, specs, M, seed):
    """Packed linears with adapters on the device; returns (item array, lora array, entries, host
    copies).  The entries own the device tensors the two arrays point into (the adapters' factors
    are stored with their linear's entry), so they live as long as the caller holds `ents`."""
    import torch
    ents, lents, keep = [], [], []
    for i, (N, K, g, r, scaling) in enumerate(specs):
        w = synth.llm_weight(N, K, seed + 10 * i, outlier_frac=0.01)
        xb = synth.llm_activation_bf16(M, K, seed + 10 * i + 1)
        ab, bb = synth.lora_factors(N, K, r, seed + 10 * i + 2, std_a=0.03, std_b=0.03)
        q, s, z = O.quantize_w4_asym_group(w, g)
        qw, zw = O.pack_w4a16(q, z)
        ents.append(dict(N=N, K=K, group_size=g, qweight=dev(qw), scales=dev(s.view(np.uint16)), zeros=dev(zw),
                         x=dev(xb), y=torch.full((M * N,), 0x7FC0, dtype=torch.int16, device="cuda")))
        lents.append(dict(A=dev(ab), B=dev(bb), r=r, scaling=scaling, N=N, K=K))
        ents[-1]["lora"] = lents[-1]
        keep.append((qw, s, zw, xb, ab, bb))
    return B.make_w4a16_items(ents, M), B.make_loras(lents), ents, keep


def _run_both(B, specs, M, seed):
    import torch
    L = B.lib()
    items, loras, ents, keep = _case(B, specs, M, seed)
    n = len(specs)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # reference: the existing entry point with a caller-owned workspace
    need = ctypes.c_size_t(0)
    assert L.qail_w4a16_lora_workspace(items, loras, n, M, ctypes.byref(need)) == B.QAIL_OK
    ws = torch.empty(max(need.value, 256), dtype=torch.uint8, device="cuda")
    assert L.qail_w4a16_linear_lora_batch(items, loras, n, M, ctypes.c_void_p(ws.data_ptr()), need.value, stream) == B.QAIL_OK
    torch.cuda.synchronize()
    want = [host(e["y"], np.uint16).copy() for e in ents]
    for e in ents:
        e["y"].fill_(0x7FC0)
    torch.cuda.synchronize()
    # the entry point under test: no workspace argument, nothing allocated in between
    before = torch.cuda.memory_allocated()
    assert L.qail_w4a16_linear_lora_batch_static(items, loras, n, M, stream) == B.QAIL_OK
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    got = [host(e["y"], np.uint16) for e in ents]
    for (N, K, g, r, scaling), (qw, s, zw, xb, ab, bb), y_want, y_got in zip(specs, keep, want, got):
        assert np.array_equal(y_got, y_want), (N, K, M)
        # and both are the oracle's result within the W4A16 bar
        ref = O.w4a16_linear_lora(xb, qw, s, zw, g, ab, bb, scaling)
        w_eff = (O.dequantize_w4_asym_group(O.unpack_nibbles_u4(qw, K), s, O.unpack_nibbles_u4(zw, K // g), g)
                 + scaling * (O.bf16_bits_to_f64(bb) @ O.bf16_bits_to_f64(ab)))
        nx = np.sqrt((O.bf16_bits_to_f64(xb) ** 2).sum(axis=1))
        assert w4a16_norm_err(y_got.reshape(M, N), ref, nx, np.sqrt((w_eff ** 2).sum(axis=1))) <= 2e-3


def test_static_scratch_entry_point_two_calls_in_a_row():
    B = ensure_built()
    assert B.qail_static_scratch_bytes() == 1 << 20
    big = [(520, 4096, 128, 32, 2.0), (200, 11008, 128, 64, 1.0), (96, 1024, 128, 8, -0.5), (300, 2048, 256, 16, 1.5)]
    small = [(72, 1024, 128, 8, 1.0), (40, 2048, 128, 32, -2.0)]
    _run_both(B, big, 16, 4100)      # largest decode batch: 4 x 16 x 64 floats of scratch
    _run_both(B, small, 3, 4200)     # fewer, smaller linears, fewer rows: the scratch still holds the first call's sums
    _run_both(B, big, 1, 4300)       # M = 1: the up-projection joins the streaming kernel's final store
    _run_both(B, small, 1, 4400)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    B = ensure_built()
    L = B.lib()
    # 40 rows of x on the matrix-core path need its workspace (megabytes): beyond the built-in scratch
    specs = [(520, 4096, 128, 32, 2.0)]
    items, loras, ents, _ = _case(B, specs, 40, 4500)
    need = ctypes.c_size_t(0)
    assert L.qail_w4a16_lora_workspace(items, loras, 1, 40, ctypes.byref(need)) == B.QAIL_OK
    assert need.value > B.qail_static_scratch_bytes()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.qail_w4a16_linear_lora_batch_static(items, loras, 1, 40, stream) == B.QAIL_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert np.all(host(ents[0]["y"], np.uint16) == 0x7FC0)     # nothing was launched
    assert L.qail_w4a16_linear_lora_batch_static(items, loras, 0, 1, stream) == B.QAIL_OK
    assert L.qail_w4a16_linear_lora_batch_static(None, loras, 1, 1, stream) == B.QAIL_ERR_NULL
