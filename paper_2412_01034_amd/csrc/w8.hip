// 8-bit variants (Sec. 5.4: the driving encoder is also deployed W8A8, the backbone also with
// 8-bit weights only): symmetric round-to-nearest quantisers and the weight-only linear.  The
// W8A8 convolution itself is the kBits = 8 instantiation of the kernel in w4a4_conv.hip.
//
// Readings (the paper names no 8-bit quantiser): weights per output channel (fp32 step
// max|w| / 127) for W8A8, per group with an fp16 step rounded up for weight-only; activations
// one step per tensor, max|a| / 127; codes clamp(rint(v / s), -127, 127), 4 per word.
#include "qail_internal.h"

namespace qail {

namespace {

__device__ __forceinline__ uint16_t f32_to_f16_bits_up(float v) {
    _Float16 h = (_Float16)v;  // nearest even
    uint16_t b = __builtin_bit_cast(uint16_t, h);
    if ((float)h < v) b += 1;  // positive fp16 patterns are ordered like integers
    return b;
}

__device__ __forceinline__ uint32_t pack4_s8(float4 v, float s) {
    const float q0 = fminf(fmaxf(rintf(v.x / s), -127.f), 127.f), q1 = fminf(fmaxf(rintf(v.y / s), -127.f), 127.f);
    const float q2 = fminf(fmaxf(rintf(v.z / s), -127.f), 127.f), q3 = fminf(fmaxf(rintf(v.w / s), -127.f), 127.f);
    return ((uint32_t)(int)q0 & 0xFFu) | (((uint32_t)(int)q1 & 0xFFu) << 8) | (((uint32_t)(int)q2 & 0xFFu) << 16) |
           (((uint32_t)(int)q3 & 0xFFu) << 24);
}

// One wave per (row, group); g = K gives the per-channel quantiser.  kF16: fp16 step rounded
// up (at least 2^-14, counted in range_errors beyond 65504), else fp32 step.
template <bool kF16>
__global__ __launch_bounds__(256) void quantize_s8_kernel(const float* __restrict__ w, uint32_t* __restrict__ qw,
                                                          void* __restrict__ scales, uint32_t* __restrict__ range_errors,
                                                          long long ngroups, int g) {
    const long long gi = (long long)blockIdx.x * 4 + threadIdx.x / kWave;
    if (gi >= ngroups) return;  // wave-uniform
    const int lane = threadIdx.x % kWave;
    const float4* src = reinterpret_cast<const float4*>(w + gi * g);
    float amax = 0.f;
    for (int i = lane; i < g / 4; i += kWave) {
        const float4 v = src[i];
        amax = fmaxf(fmaxf(amax, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o, kWave));
    float s;
    if (kF16) {
        float s32 = amax / 127.0f;
        const bool over = s32 > 65504.0f;
        if (over) s32 = 65504.0f;
        uint16_t sb = f32_to_f16_bits_up(s32);
        if (sb < 0x0400) sb = 0x0400;
        if (amax == 0.f) sb = 0x3C00;
        s = f16_bits_to_f32(sb);
        if (lane == 0) {
            static_cast<uint16_t*>(scales)[gi] = sb;
            if (over && range_errors) atomicAdd(range_errors, 1u);
        }
    } else {
        s = (amax == 0.f) ? 1.0f : amax / 127.0f;
        if (lane == 0) static_cast<float*>(scales)[gi] = s;
    }
    uint32_t* dst = qw + gi * (g / 4);
    for (int i = lane; i < g / 4; i += kWave) dst[i] = pack4_s8(src[i], s);
}

__global__ void abs_scale_init_kernel(float* s_a) { *reinterpret_cast<uint32_t*>(s_a) = 0u; }

// max |a| through an integer atomic on the bit pattern (order-preserving for non-negative floats)
__global__ __launch_bounds__(256) void abs_scale_reduce_kernel(const float* __restrict__ a, size_t n, float* s_a) {
    float m = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) m = fmaxf(m, fabsf(a[i]));
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) m = fmaxf(m, __shfl_xor(m, o, kWave));
    if (threadIdx.x % kWave == 0) atomicMax(reinterpret_cast<uint32_t*>(s_a), __builtin_bit_cast(uint32_t, m));
}

__global__ void abs_scale_final_kernel(float* s_a) {
    const float m = *s_a;
    *s_a = (m == 0.f) ? 1.0f : m / 127.0f;
}

__global__ __launch_bounds__(256) void act_quant_s8_kernel(const float* __restrict__ a, size_t words,
                                                           const float* __restrict__ s_a, uint32_t* __restrict__ out) {
    const float s = *s_a;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256)
        out[i] = pack4_s8(reinterpret_cast<const float4*>(a)[i], s);
}

// ---------------------------------------------------------------------------------------
// Weight-only 8-bit linear, M = 1: y[n] = sum_k x[k] q[n][k] s[n][k/g], for the shapes the
// streaming kernel (w8a16_gemv.hip) does not take.  One wave per row at a time, 16 codes per lane and
// load; bytes are converted with v_cvt_f32_ubyte after flipping the sign bit (u = q + 128), so
//   sum_k x q = sum_k x u - 128 sum_k x,   with sum_k x per group staged beside x in LDS.
constexpr int kW8Waves = 16;
__global__ __launch_bounds__(kW8Waves* kWave) void w8a16_gemv_kernel(const uint32_t* __restrict__ qw,
                                                                      const uint16_t* __restrict__ sc,
                                                                      const uint16_t* __restrict__ x,
                                                                      uint16_t* __restrict__ y, int N, int K, int g) {
    extern __shared__ float xs[];   // [K] activations as fp32, then [K/g] group sums
    const int G = K / g;
    float* gsum = xs + K;
    for (int k = threadIdx.x; k < K; k += blockDim.x) xs[k] = bf16_bits_to_f32(x[k]);
    __syncthreads();
    for (int gi = threadIdx.x; gi < G; gi += blockDim.x) {
        float t = 0.f;
        for (int k = 0; k < g; ++k) t += xs[gi * g + k];
        gsum[gi] = t;
    }
    __syncthreads();
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int chunks = K / 16;            // 16-code pieces per row
    const int cpg = g / 16;               // pieces per group
    for (int n = blockIdx.x * kW8Waves + wave; n < N; n += gridDim.x * kW8Waves) {
        const uint4* row = reinterpret_cast<const uint4*>(qw + (size_t)n * (K / 4));
        float acc = 0.f;
        // four loads in flight per lane (pieces past the end of the row re-read its last piece and
        // contribute nothing)
        for (int c0 = lane; c0 < chunks; c0 += 4 * kWave) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = row[min(c0 + u * kWave, chunks - 1)];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * kWave;
                if (c >= chunks) continue;
                const uint32_t w[4] = {v[u].x ^ 0x80808080u, v[u].y ^ 0x80808080u, v[u].z ^ 0x80808080u,
                                       v[u].w ^ 0x80808080u};
                const float4* xp = reinterpret_cast<const float4*>(xs + c * 16);
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float4 xv = xp[e];
                    part = fmaf(xv.x, (float)(w[e] & 0xFFu), part);
                    part = fmaf(xv.y, (float)((w[e] >> 8) & 0xFFu), part);
                    part = fmaf(xv.z, (float)((w[e] >> 16) & 0xFFu), part);
                    part = fmaf(xv.w, (float)(w[e] >> 24), part);
                }
                const int grp = c / cpg;
                // the group's -128 sum x goes in with the group's first piece
                if (c - grp * cpg == 0) part = fmaf(-128.f, gsum[grp], part);
                const float s = f16_bits_to_f32(sc[(size_t)n * G + grp]);
                acc = fmaf(s, part, acc);
            }
        }
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) acc += __shfl_xor(acc, o, kWave);
        if (lane == 0) y[n] = f32_to_bf16_rne(acc);
    }
}

// Any M: one thread per output (slow; the 8-bit weight-only path is built for decode).
__global__ __launch_bounds__(256) void w8a16_generic_kernel(const uint32_t* __restrict__ qw, const uint16_t* __restrict__ sc,
                                                            const uint16_t* __restrict__ x, uint16_t* __restrict__ y,
                                                            int M, int N, int K, int g) {
    const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= (size_t)M * N) return;
    const int m = (int)(o / N), n = (int)(o % N);
    const int G = K / g;
    float acc = 0.f;
    for (int gi = 0; gi < G; ++gi) {
        float part = 0.f;
        for (int k = gi * g; k < (gi + 1) * g; k += 4) {
            const uint32_t w = qw[(size_t)n * (K / 4) + k / 4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                part = fmaf(bf16_bits_to_f32(x[(size_t)m * K + k + j]), (float)(int)(int8_t)(w >> (8 * j)), part);
        }
        acc = fmaf(part, f16_bits_to_f32(sc[(size_t)n * G + gi]), acc);
    }
    y[o] = f32_to_bf16_rne(acc);
}

}  // namespace

hipError_t launch_quantize_s8(const qail_wdesc& d, const float* w, uint32_t* qw, void* scales,
                              uint32_t* range_errors, hipStream_t st) {
    const bool group = d.scheme == QAIL_W8_SYM_GROUP;
    const int g = group ? d.group_size : d.K;
    const long long ngroups = (long long)d.N * (d.K / g);
    const unsigned blocks = (unsigned)((ngroups + 3) / 4);
    if (group)
        hipLaunchKernelGGL(quantize_s8_kernel<true>, dim3(blocks), dim3(256), 0, st, w, qw, scales, range_errors, ngroups, g);
    else
        hipLaunchKernelGGL(quantize_s8_kernel<false>, dim3(blocks), dim3(256), 0, st, w, qw, scales, range_errors, ngroups, g);
    return hipGetLastError();
}

hipError_t launch_act_scale_s8(const float* a, size_t n, float* s_a, hipStream_t st) {
    hipLaunchKernelGGL(abs_scale_init_kernel, dim3(1), dim3(1), 0, st, s_a);
    if (n > 0) {
        size_t blocks = (n + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(abs_scale_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a, n, s_a);
    }
    hipLaunchKernelGGL(abs_scale_final_kernel, dim3(1), dim3(1), 0, st, s_a);
    return hipGetLastError();
}

hipError_t launch_act_quant_s8(const float* a, size_t n, const float* s_a, uint32_t* out, hipStream_t st) {
    const size_t words = n / 4;
    size_t blocks = (words + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(act_quant_s8_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a, words, s_a, out);
    return hipGetLastError();
}

hipError_t launch_w8a16_linear(const qail_wdesc& d, const uint32_t* qw, const uint16_t* sc, const uint16_t* x,
                               uint16_t* y, int M, hipStream_t st) {
    if (w8a16_stream_supports(d, M)) return launch_w8a16_stream(d, qw, sc, x, y, st);
    const int G = d.K / d.group_size;
    const size_t lds = ((size_t)d.K + G) * 4;
    if (M == 1 && d.K % 16 == 0 && d.group_size % 16 == 0 && lds <= 64 * 1024) {
        int blocks = (d.N + kW8Waves - 1) / kW8Waves;
        if (blocks > 2048) blocks = 2048;
        hipLaunchKernelGGL(w8a16_gemv_kernel, dim3(blocks), dim3(kW8Waves * kWave), lds, st, qw, sc, x, y, d.N, d.K,
                           d.group_size);
    } else {
        const size_t outs = (size_t)M * d.N;
        hipLaunchKernelGGL(w8a16_generic_kernel, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, st, qw, sc, x, y,
                           M, d.N, d.K, d.group_size);
    }
    return hipGetLastError();
}

}  // namespace qail
