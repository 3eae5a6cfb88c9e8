"""The library under HIP graph capture: every entry point only launches kernels on the caller's
stream (no allocation, no memset, no synchronisation), so a decode step or a whole encoder pass
can be captured once and replayed.  Each replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest

from tests.helpers import dev, ensure_built, host, ws_for
from paper_2412_01034_amd import synth
from oracle import qail_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    return ensure_built()


def _linear_case(B, N, K, g, M, seed):
    import torch
    w = synth.llm_weight(N, K, seed, outlier_frac=0.01)
    xb = synth.llm_activation_bf16(M, K, seed + 1)
    q, s, z = O.quantize_w4_asym_group(w, g)
    qw, zw = O.pack_w4a16(q, z)
    t = dict(N=N, K=K, g=g, M=M, qw=dev(qw), s=dev(s.view(np.uint16)), z=dev(zw), x=dev(xb),
             y=torch.zeros(M * N, dtype=torch.int16, device="cuda"),
             ws=ws_for(B, B.qail_w4a16_workspace(N, K, g, M)))
    return t


def _run_linear(B, t):
    B.qail_w4a16_linear(t["N"], t["K"], t["g"], t["qw"], t["s"], t["z"], t["x"], t["y"], t["M"], t["ws"])


def test_replays_match_eager(B):
    import torch
    # one case per W4A16 kernel: M = 1 stream, four-row stream, small batch (one and two blocks of 16 rows of
    # x, the latter with K in several passes; the kernel for other group sizes), matrix-core GEMM with tiles
    # shared between blocks (K = 8192: 64 steps), and a convolution
    lin = [_linear_case(B, 256, 4096, 128, 1, 11), _linear_case(B, 64, 11008, 128, 4, 12),
           _linear_case(B, 80, 4096, 128, 16, 13), _linear_case(B, 300, 8192, 128, 100, 14),
           _linear_case(B, 100, 11008, 128, 27, 15), _linear_case(B, 72, 2048, 256, 9, 16)]
    s = synth.ConvShape("graph", B=2, H=14, W=14, Cin=64, Cout=64, KH=3, KW=3, stride=1, pad=1)
    rng = np.random.default_rng(5)
    a = dev(rng.integers(0, 2 ** 32, size=s.B * s.H * s.W * s.Cin // 8, dtype=np.uint64).astype(np.uint32))
    ww = dev(rng.integers(0, 2 ** 32, size=s.Cout * s.K // 8, dtype=np.uint64).astype(np.uint32))
    acc = torch.zeros(s.M * s.Cout, dtype=torch.int32, device="cuda")
    # two convolutions on the same input in one launch: a fused 4-bit output and an int32 output
    acc2 = torch.zeros(s.M * s.Cout, dtype=torch.int32, device="cuda")
    u4 = torch.zeros(s.M * s.Cout // 8, dtype=torch.int32, device="cuda")
    cscale = torch.full((s.Cout,), 2e-3, dtype=torch.float32, device="cuda")
    cbias = torch.zeros(s.Cout, dtype=torch.float32, device="cuda")
    cf = dict(B=s.B, H=s.H, W=s.W, Cin=s.Cin, Cout=s.Cout, KH=s.KH, KW=s.KW, stride=s.stride, pad=s.pad)
    citems = B.make_conv_items([dict(cf, a_u4=a, w_s4=ww, scale=cscale, bias=cbias, out_u4=u4, s_out=0.3),
                                dict(cf, a_u4=a, w_s4=ww, acc_out=acc2)])

    # three linears of the matrix-core path in one batched call (they share launches), and an 8-bit batch
    bat = [_linear_case(B, 300, 4096, 128, 40, 21), _linear_case(B, 96, 11008, 128, 40, 22),
           _linear_case(B, 64, 256, 64, 40, 23)]
    bitems = B.make_w4a16_items([dict(N=t["N"], K=t["K"], group_size=t["g"], qweight=t["qw"], scales=t["s"],
                                      zeros=t["z"], x=t["x"], y=t["y"]) for t in bat], 40)
    bws = ws_for(B, B.qail_w4a16_batch_workspace(bitems, 3, 40))
    w8 = []
    for i, (N, K, g) in enumerate([(200, 4096, 128), (64, 1024, 64)]):
        q, s8 = O.quantize_w8_sym_group(synth.llm_weight(N, K, 31 + i), g)
        w8.append(dict(N=N, K=K, group_size=g, qweight=dev(O.pack_bytes(q)), scales=dev(s8.view(np.uint16)),
                       x=dev(synth.llm_activation_bf16(1, K, 41 + i)), y=torch.zeros(N, dtype=torch.int16, device="cuda")))
    w8items = B.make_w8a16_items(w8, 1)
    # 8-bit weights at M = 6 and 20: the small-batch stream with byte weights; the second shape rides on the matrix cores
    w8m = {}
    for M8 in (6, 20):
        ents8 = []
        for i, (N, K, g) in enumerate([(200, 4096, 128), (64, 1024, 64)]):
            q, s8 = O.quantize_w8_sym_group(synth.llm_weight(N, K, 51 + i), g)
            ents8.append(dict(N=N, K=K, group_size=g, qweight=dev(O.pack_bytes(q)), scales=dev(s8.view(np.uint16)),
                              x=dev(synth.llm_activation_bf16(M8, K, 61 + i + M8)),
                              y=torch.zeros(M8 * N, dtype=torch.int16, device="cuda")))
        it8 = B.make_w8a16_items(ents8, M8)
        w8m[M8] = (ents8, it8, ws_for(B, B.qail_w8a16_batch_workspace(it8, 2, M8)))

    def step():
        for t in lin:
            _run_linear(B, t)
        B.qail_w4a16_linear_batch(bitems, 3, 40, bws)
        B.qail_w8a16_linear_batch(w8items, 2, 1)
        for M8, (_, it8, ws8) in w8m.items():
            B.qail_w8a16_linear_batch(it8, 2, M8, ws8)
        B.qail_w4a4_gemm(s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad, a, ww, acc_out=acc)
        B.qail_w4a4_conv_batch(citems, 2)

    def snapshot():
        torch.cuda.synchronize()
        return ([host(t["y"], np.uint16).copy() for t in lin + bat] + [host(e["y"], np.uint16).copy() for e in w8] +
                [host(e["y"], np.uint16).copy() for ents8, _, _ in w8m.values() for e in ents8] + [host(acc, np.int32).copy(), host(acc2, np.int32).copy(), host(u4, np.int32).copy()])

    def clear():
        for t in lin + bat:
            t["y"].fill_(0x7FC0)
        for e in w8 + [e for ents8, _, _ in w8m.values() for e in ents8]:
            e["y"].fill_(0x7FC0)
        acc.fill_(-1)
        acc2.fill_(-1)
        u4.fill_(-1)

    gs = torch.cuda.Stream()
    with torch.cuda.stream(gs):
        clear()
        step()          # eager; also the first call of every kernel (attributes are set here, not under capture)
        want = snapshot()
        clear()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=gs):
            step()
        for _ in range(3):
            clear()                   # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            got = snapshot()
            for g_, w_ in zip(got, want):
                assert np.array_equal(g_, w_)
