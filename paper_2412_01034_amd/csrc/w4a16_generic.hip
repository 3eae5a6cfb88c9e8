// W4A16 linear, any valid shape: y[m][n] = sum_k x[m][k] * (q[n][k] - z[n][k/g]) * s[n][k/g].
//
// Sec. 2.1: weight-only quantised GEMM operand.  This is the fallback for shapes the
// streaming (M <= 16) and matrix-core (M > 16) kernels do not take.
#include "qail_internal.h"

namespace qail {

namespace {

// Any valid shape (K % 8 == 0, g % 8 == 0): one thread per output, fp32
// accumulation in k order.  Slow; only for shapes the tiled kernels do not take.
__global__ __launch_bounds__(256) void w4a16_generic_kernel(
    const uint32_t* __restrict__ qw, const uint16_t* __restrict__ sc, const uint32_t* __restrict__ zr,
    const uint16_t* __restrict__ x, uint16_t* __restrict__ y, int M, int N, int K, int g) {
    const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= (size_t)M * N) return;
    const int m = (int)(o / N), n = (int)(o % N);
    const int G = K / g, zwords = (G + 7) / 8, kw = K / 8;
    float acc = 0.f;
    for (int wi = 0; wi < kw; ++wi) {
        const int grp = (wi * 8) / g;
        const uint32_t w = qw[(size_t)n * kw + wi];
        const float s = f16_bits_to_f32(sc[(size_t)n * G + grp]);
        const int z = (zr[(size_t)n * zwords + grp / 8] >> (4 * (grp & 7))) & 0xF;
        float part = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int q = (w >> (4 * j)) & 0xF;
            part = fmaf(bf16_bits_to_f32(x[(size_t)m * K + wi * 8 + j]), (float)(q - z), part);
        }
        acc = fmaf(part, s, acc);
    }
    y[o] = f32_to_bf16_rne(acc);
}

}  // namespace

hipError_t launch_w4a16_generic(const qail_w4a16_item& it, int M, hipStream_t st) {
    const size_t outs = (size_t)M * it.d.N;
    hipLaunchKernelGGL(w4a16_generic_kernel, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, st,
                       it.qweight, it.scales, it.zeros, it.x, it.y, M, it.d.N, it.d.K, it.d.group_size);
    return hipGetLastError();
}

}  // namespace qail
