// W4A4 convolution as an implicit GEMM with exact int32 accumulation.
//
//   acc[(b,oh,ow)][n] = sum_{kh,kw,c} a[b][oh*s+kh-p][ow*s+kw-p][c] * w[n][kh][kw][c]
//
// Sec. 2.1 / Sec. 5.1: the driving policy's convolutions are compute-bound, so both
// GEMM operands are 4-bit integers.  CDNA4 has no 4-bit integer matrix
// instruction, so nibbles are widened to int8 in registers and fed to
// v_mfma_i32_16x16x64_i8 (int32 accumulate):
//   * unsigned activation codes:  w & 0x0F0F0F0F  and (w >> 4) & 0x0F0F0F0F
//     give the even and the odd codes of a word as bytes;
//   * signed weight codes are moved to the HIGH nibble of each byte,
//     (w << 4) & 0xF0F0F0F0 and w & 0xF0F0F0F0, which is the int8 value 16*code,
//     so no sign extension is needed; the accumulator is 16x the result and an
//     arithmetic shift by 4 restores it exactly.
// The two operands are permuted along k in the same way (even codes, then odd
// codes of each word), which leaves the sum unchanged.
//
// MFMA operand layout (16x16x64 int8, wave64): lane l supplies row (A) / column
// (B) l%16 and the 16 consecutive k starting at 16*(l/16); it receives
// D[4*(l/16)+r][l%16], r = 0..3.  A = activations (rows m), B = weights (columns n).
//
// Zero padding costs nothing: code 0 of the unsigned activations is the value 0.
#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kCBM = 128, kCBN = 64, kCBK = 64;  // block tile; kCBK codes = 8 words of one filter tap
constexpr int kCPitch = 8 + 4;                   // words per LDS row (48 B)

struct ConvGeom {
    int B, H, W, Cin, Cout, KH, KW, stride, pad, OH, OW, M;
};

__global__ __launch_bounds__(256) void w4a4_conv_kernel(
    const ConvGeom gm, const uint32_t* __restrict__ a, const uint32_t* __restrict__ w,
    int32_t* __restrict__ acc_out, const float* __restrict__ scale, const float* __restrict__ bias,
    float* __restrict__ y_out) {
    __shared__ __attribute__((aligned(16))) uint32_t As[kCBM * kCPitch];
    __shared__ __attribute__((aligned(16))) uint32_t Bs[kCBN * kCPitch];

    const int t = threadIdx.x;
    const int lane = t % kWave, wave = t / kWave;
    const int wm = wave / 2, wn = wave % 2;  // 2 x 2 waves, each 64 (m) x 32 (n)
    const int bm = blockIdx.y * kCBM, bn = blockIdx.x * kCBN;
    const int cw = gm.Cin / 8;                 // words per pixel
    const int kwords = gm.KH * gm.KW * cw;     // words per filter

    // this thread's share of the A tile: row t/2, 4 words at (t%2)*4
    const int arow = t >> 1, ahalf = t & 1;
    const int am = bm + arow;
    const bool am_ok = am < gm.M;
    int ab = 0, ih0 = 0, iw0 = 0;
    if (am_ok) {
        ab = am / (gm.OH * gm.OW);
        const int rem = am - ab * (gm.OH * gm.OW);
        const int oh = rem / gm.OW, ow = rem - oh * gm.OW;
        ih0 = oh * gm.stride - gm.pad;
        iw0 = ow * gm.stride - gm.pad;
    }
    // B tile: 64 rows x 8 words; threads 0..127: row t/2, 4 words at (t%2)*4
    const int brow = (t >> 1) & 63;
    const int bnrow = min(bn + brow, gm.Cout - 1);

    i32x4_t acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = i32x4_t{0, 0, 0, 0};

    for (int kh = 0; kh < gm.KH; ++kh) {
        for (int kwi = 0; kwi < gm.KW; ++kwi) {
            const int ih = ih0 + kh, iw = iw0 + kwi;
            const bool in = am_ok && ih >= 0 && ih < gm.H && iw >= 0 && iw < gm.W;
            const uint32_t* ap = a + ((size_t)(ab * gm.H + (in ? ih : 0)) * gm.W + (in ? iw : 0)) * cw;
            const uint32_t* wp = w + (size_t)bnrow * kwords + (size_t)(kh * gm.KW + kwi) * cw;
            for (int c0 = 0; c0 < cw; c0 += 8) {
                uint4 av = make_uint4(0, 0, 0, 0);
                if (in) av = *reinterpret_cast<const uint4*>(ap + c0 + ahalf * 4);
                uint4 bv = make_uint4(0, 0, 0, 0);
                if (t < 128) bv = *reinterpret_cast<const uint4*>(wp + c0 + ahalf * 4);
                __syncthreads();
                *reinterpret_cast<uint4*>(&As[arow * kCPitch + ahalf * 4]) = av;
                if (t < 128) *reinterpret_cast<uint4*>(&Bs[brow * kCPitch + ahalf * 4]) = bv;
                __syncthreads();

                i32x4_t af[4], bf[2];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint2 p = *reinterpret_cast<const uint2*>(
                        &As[(wm * 64 + i * 16 + (lane & 15)) * kCPitch + (lane >> 4) * 2]);
                    af[i] = i32x4_t{(int)(p.x & 0x0F0F0F0Fu), (int)((p.x >> 4) & 0x0F0F0F0Fu),
                                    (int)(p.y & 0x0F0F0F0Fu), (int)((p.y >> 4) & 0x0F0F0F0Fu)};
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const uint2 p = *reinterpret_cast<const uint2*>(
                        &Bs[(wn * 32 + j * 16 + (lane & 15)) * kCPitch + (lane >> 4) * 2]);
                    bf[j] = i32x4_t{(int)((p.x << 4) & 0xF0F0F0F0u), (int)(p.x & 0xF0F0F0F0u),
                                    (int)((p.y << 4) & 0xF0F0F0F0u), (int)(p.y & 0xF0F0F0F0u)};
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
            }
        }
    }

#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = bn + wn * 32 + j * 16 + (lane & 15);
            if (n >= gm.Cout) continue;
            const float sc = y_out ? scale[n] : 0.f;
            const float bi = y_out ? bias[n] : 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = bm + wm * 64 + i * 16 + (lane >> 4) * 4 + r;
                if (m >= gm.M) continue;
                const int v = acc[i][j][r] >> 4;  // exact: the accumulator is 16 * result
                const size_t o = (size_t)m * gm.Cout + n;
                if (acc_out) acc_out[o] = v;
                if (y_out) y_out[o] = fmaf((float)v, sc, bi);
            }
        }
}

// Any Cin % 8 == 0: one thread per output.  Slow; for shapes whose Cin is not a
// multiple of 64.
__global__ __launch_bounds__(256) void w4a4_generic_kernel(
    const ConvGeom gm, const uint32_t* __restrict__ a, const uint32_t* __restrict__ w,
    int32_t* __restrict__ acc_out, const float* __restrict__ scale, const float* __restrict__ bias,
    float* __restrict__ y_out) {
    const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= (size_t)gm.M * gm.Cout) return;
    const int m = (int)(o / gm.Cout), n = (int)(o % gm.Cout);
    const int b = m / (gm.OH * gm.OW);
    const int rem = m - b * (gm.OH * gm.OW);
    const int oh = rem / gm.OW, ow = rem - oh * gm.OW;
    const int cw = gm.Cin / 8;
    int acc = 0;
    for (int kh = 0; kh < gm.KH; ++kh)
        for (int kwi = 0; kwi < gm.KW; ++kwi) {
            const int ih = oh * gm.stride + kh - gm.pad, iw = ow * gm.stride + kwi - gm.pad;
            if (ih < 0 || ih >= gm.H || iw < 0 || iw >= gm.W) continue;
            const uint32_t* ap = a + ((size_t)(b * gm.H + ih) * gm.W + iw) * cw;
            const uint32_t* wp = w + ((size_t)(n * gm.KH + kh) * gm.KW + kwi) * cw;
            for (int c = 0; c < cw; ++c) {
                const uint32_t av = ap[c], wv = wp[c];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int qa = (av >> (4 * j)) & 0xF;
                    const int qw = (int)(((wv >> (4 * j)) & 0xFu) ^ 8u) - 8;
                    acc += qa * qw;
                }
            }
        }
    if (acc_out) acc_out[o] = acc;
    if (y_out) y_out[o] = fmaf((float)acc, scale[n], bias[n]);
}

}  // namespace

hipError_t launch_w4a4_conv(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, int32_t* acc,
                            const float* scale, const float* bias, float* y, hipStream_t st) {
    ConvGeom gm;
    gm.B = d.B; gm.H = d.H; gm.W = d.W; gm.Cin = d.Cin; gm.Cout = d.Cout;
    gm.KH = d.KH; gm.KW = d.KW; gm.stride = d.stride; gm.pad = d.pad;
    gm.OH = (d.H + 2 * d.pad - d.KH) / d.stride + 1;
    gm.OW = (d.W + 2 * d.pad - d.KW) / d.stride + 1;
    gm.M = d.B * gm.OH * gm.OW;
    if (d.Cin % kCBK == 0) {
        dim3 grid((d.Cout + kCBN - 1) / kCBN, (gm.M + kCBM - 1) / kCBM);
        hipLaunchKernelGGL(w4a4_conv_kernel, grid, dim3(256), 0, st, gm, a, w, acc, scale, bias, y);
    } else {
        const size_t outs = (size_t)gm.M * d.Cout;
        hipLaunchKernelGGL(w4a4_generic_kernel, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, st, gm,
                           a, w, acc, scale, bias, y);
    }
    return hipGetLastError();
}

}  // namespace qail
