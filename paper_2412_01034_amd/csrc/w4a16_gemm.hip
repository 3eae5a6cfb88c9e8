// W4A16 linear for M > 1: y[m][n] = sum_k x[m][k] * (q[n][k] - z[n][k/g]) * s[n][k/g].
//
// Appendix "Analysis": prefill is the compute-heavy stage of the backbone.  The
// weights are dequantised to bf16 on their way into LDS and the contraction runs
// on the bf16 matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate).
//
// MFMA operand layout used here (16x16x32, wave64): lane l supplies, for the A
// operand, row l%16 and the 8 consecutive k starting at 8*(l/16); for the B
// operand, column l%16 and the same k; it receives D[4*(l/16)+r][l%16], r=0..3.
// A = activations (rows m), B = weights (columns n), so that a lane's results
// are contiguous along n in y.
#include "qail_internal.h"

namespace qail {

namespace {

typedef __attribute__((ext_vector_type(2))) float f32x2_t;

constexpr int kBN = 128, kBK = 64;
constexpr int kPitch = kBK + 8;  // bf16 elements per LDS row (144 B: 16-byte aligned)

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2_t v = {a, b};
    bf16x2_t r = __builtin_convertvector(v, bf16x2_t);  // nearest even
    return __builtin_bit_cast(uint32_t, r);
}

// 8 codes of one word -> 8 bf16 (q - z) * s, in k order.  The even and the odd codes are
// masked into bytes, converted with the byte-to-float instruction, and q * s - z * s is one
// fused multiply-add (both products are exact, so the result is the exact (q - z) * s).
__device__ __forceinline__ uint4 dequant8(uint32_t w, float s, float nzs) {
    const uint32_t e = w & 0x0F0F0F0Fu, o = (w >> 4) & 0x0F0F0F0Fu;
    float d[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        d[2 * i] = fmaf((float)((e >> (8 * i)) & 0xFFu), s, nzs);
        d[2 * i + 1] = fmaf((float)((o >> (8 * i)) & 0xFFu), s, nzs);
    }
    return make_uint4(pack_bf16(d[0], d[1]), pack_bf16(d[2], d[3]), pack_bf16(d[4], d[5]),
                      pack_bf16(d[6], d[7]));
}

// Block tile (64 * kWM) x 128 with kWM x 2 waves of 64 x 64, K step 64, one LDS buffer.
// The weight tile is dequantised once per block and step, so a taller tile spreads that
// vector-ALU work over more matrix work; the next step's global loads are in flight while
// the current step's MFMAs run.
template <int kWM>
__global__ __launch_bounds__(128 * kWM) void w4a16_gemm_kernel(
    const uint32_t* __restrict__ qw, const uint16_t* __restrict__ sc, const uint32_t* __restrict__ zr,
    const uint16_t* __restrict__ x, uint16_t* __restrict__ y, int M, int N, int K, int g) {
    constexpr int kBM = 64 * kWM;
    constexpr int kThreads = 128 * kWM;
    constexpr int kBT = kThreads < 512 ? kThreads : 512;  // threads that load weights
    constexpr int kBW = 1024 / kBT;                       // packed words per such thread: 8, 4 or 2
    __shared__ __attribute__((aligned(16))) uint16_t As[kBM * kPitch];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[kBN * kPitch];

    const int t = threadIdx.x;
    const int lane = t % kWave, wave = t / kWave;
    const int wm = wave / 2, wn = wave % 2;
    const int bm = blockIdx.y * kBM, bn = blockIdx.x * kBN;
    const int G = K / g, zwords = (G + 7) / 8, kw = K / 8;

    f32x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // weight loader: row t / (8 / kBW), words [kBW * part, kBW * (part + 1)) of the step's 8
    constexpr int kParts = 8 / kBW;
    const bool bact = t < kBT;
    const int brow = (t / kParts) & 127, bpart = t % kParts;
    const int bnrow = min(bn + brow, N - 1);
    const uint32_t* qrow = qw + (size_t)bnrow * kw + bpart * kBW;
    const _Float16* srow = reinterpret_cast<const _Float16*>(sc) + (size_t)bnrow * G;
    const uint32_t* zrow = zr + (size_t)bnrow * zwords;

    // this thread's share of one K step, fetched one step ahead of its use
    uint4 av[4];
    uint32_t qv[kBW];
    _Float16 sh = (_Float16)0.f;  // kept in its loaded type: a widening at the load would wait there
    uint32_t zword = 0;
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = t + kThreads * i;
            const int row = idx >> 3, seg = idx & 7;
            const int m = bm + row;
            av[i] = (m < M) ? *reinterpret_cast<const uint4*>(x + (size_t)m * K + k0 + seg * 8)
                            : make_uint4(0, 0, 0, 0);
        }
        if (bact) {
            const int grp = (k0 + bpart * kBW * 8) / g;
            if (kBW == 2) {
                const uint2 v = *reinterpret_cast<const uint2*>(qrow + k0 / 8);
                qv[0] = v.x; qv[1] = v.y;
            } else {
#pragma unroll
                for (int u = 0; u < kBW; u += 4) {
                    const uint4 v = *reinterpret_cast<const uint4*>(qrow + k0 / 8 + u);
                    qv[u] = v.x; qv[u + 1] = v.y; qv[u + 2] = v.z; qv[u + 3] = v.w;
                }
            }
            sh = srow[grp];
            zword = zrow[grp / 8];
        }
    };
    gload(0);

    for (int k0 = 0; k0 < K; k0 += kBK) {
        __syncthreads();  // previous step's MFMAs have read LDS
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = t + kThreads * i;
            const int row = idx >> 3, seg = idx & 7;
            *reinterpret_cast<uint4*>(&As[row * kPitch + seg * 8]) = av[i];
        }
        if (bact) {
            const int grp = (k0 + bpart * kBW * 8) / g;
            const float s = (float)sh;
            const float nzs = -(float)((zword >> (4 * (grp & 7))) & 0xFu) * s;
            uint4* dst = reinterpret_cast<uint4*>(&Bs[brow * kPitch + bpart * kBW * 8]);
#pragma unroll
            for (int u = 0; u < kBW; ++u) dst[u] = dequant8(qv[u], s, nzs);
        }
        __syncthreads();
        if (k0 + kBK < K) gload(k0 + kBK);  // lands while the MFMAs below run

#pragma unroll
        for (int kk = 0; kk < kBK; kk += 32) {
            bf16x8_t a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                a[i] = *reinterpret_cast<const bf16x8_t*>(
                    &As[(wm * 64 + i * 16 + (lane & 15)) * kPitch + kk + (lane >> 4) * 8]);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                b[j] = *reinterpret_cast<const bf16x8_t*>(
                    &Bs[(wn * 64 + j * 16 + (lane & 15)) * kPitch + kk + (lane >> 4) * 8]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }

#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = bn + wn * 64 + j * 16 + (lane & 15);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = bm + wm * 64 + i * 16 + (lane >> 4) * 4 + r;
                if (m < M && n < N) y[(size_t)m * N + n] = f32_to_bf16_rne(acc[i][j][r]);
            }
        }
}

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

namespace {
template <int kWM>
hipError_t launch_gemm_tile(const qail_w4a16_item& it, int M, hipStream_t st) {
    constexpr int kBM = 64 * kWM;
    dim3 grid((it.d.N + kBN - 1) / kBN, (M + kBM - 1) / kBM);
    hipLaunchKernelGGL(w4a16_gemm_kernel<kWM>, grid, dim3(128 * kWM), 0, st, it.qweight, it.scales, it.zeros,
                       it.x, it.y, M, it.d.N, it.d.K, it.d.group_size);
    return hipGetLastError();
}
}  // namespace

// 64-row tiles for small batches, 128-row tiles otherwise.  (Taller tiles with more waves
// spread the dequantisation further but leave too few blocks for 256 CUs at these shapes:
// measured slower.)
hipError_t launch_w4a16_gemm(const qail_w4a16_item& it, int M, hipStream_t st) {
    if (M <= 64) return launch_gemm_tile<1>(it, M, st);
    return launch_gemm_tile<2>(it, M, st);
}

hipError_t launch_w4a16_generic(const qail_w4a16_item& it, int M, hipStream_t st) {
    const size_t outs = (size_t)M * it.d.N;
    hipLaunchKernelGGL(w4a16_generic_kernel, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, st,
                       it.qweight, it.scales, it.zeros, it.x, it.y, M, it.d.N, it.d.K, it.d.group_size);
    return hipGetLastError();
}

}  // namespace qail
